"""GPU parity of the half-precision library (libmolink_stage_f16.so: IEEE half storage, the precision the
paper serves its 7B model in, section 5 "Models") against the CPU oracle on the same seeded inputs drawn as
float16.  The oracle is the same one: it widens its inputs exactly and computes in fp32/fp64.  Same stated
tolerances as the bfloat16 library (rel-L2 1e-2, max-abs 5e-2 scaled by max(1, rms)); slot indexing bit-exact."""
import numpy as np
import pytest
import torch

import oracle
from oracle import w4_oracle
from paper_2507_05043_amd import synth
from paper_2507_05043_amd.stage import load_library
from tests import gpu_harness as H
from tests.helpers import draw_layers, oracle_shape, rel_l2

pytestmark = pytest.mark.gpu

F16 = torch.float16
W4_TINY = synth.StageShape("tiny-w4", 2, 256, 4, 2, 64, 768)
MID = synth.StageShape("mid", 2, 1024, 8, 2, 128, 2816)


def f16_parity(shape, mb, seed, weight_std=None, taps=False, qkv_bias=False, activation_planes=0, group=0):
    print(f"[case] f16 {shape.name} T={mb.num_tokens} S={mb.num_seqs} q={mb.q_lens[:6]} ctx={mb.ctx_lens[:6]} "
          f"std={weight_std} seed={seed} bias={qkv_bias} planes={activation_planes} group={group}", flush=True)
    st = H.make_stage(shape, mb, seed, weight_std, qkv_bias=qkv_bias, activation_planes=activation_planes,
                      weight_group_size=group, dtype=F16)
    assert st.dtype == F16 and st.kv_pool.view(F16).isnan().any()
    before = H.snapshot_pool(st, shape, mb)
    if group:
        stored = [synth.draw_w4_layer(shape, l, seed=seed, group=group, dtype=F16) for l in range(shape.num_layers)]
        layers = [w4_oracle.dequantize_layer(lw, group) for lw in stored]
    else:
        layers = draw_layers(shape, seed, weight_std, qkv_bias=qkv_bias, elem=F16)
    for l, lw in enumerate(layers if not group else stored):     # the GPU stage holds the same bits
        for k, v in lw.items():
            assert torch.equal(st.layers[l][k].cpu().view(torch.int16 if v.dtype == F16 else v.dtype),
                               v.view(torch.int16 if v.dtype == F16 else v.dtype)), (l, k)
    ref, ref_slots, ref_pool, otaps = H.run_oracle(shape, mb, seed, weight_std, want_taps=True, layers=layers, elem=F16)
    out, slots = H.run_gpu(st, shape, mb, seed)
    assert out.dtype == F16
    assert slots == ref_slots                                   # bit-exact slot indexing
    stats = H.check_output(out, ref)
    H.check_pool(st, shape, mb, ref_pool, before, slots)
    if taps:
        hidden = synth.draw_hidden(shape, mb.num_tokens, seed=seed, dtype=F16)
        x_in_gpu = hidden
        for l in range(shape.num_layers):
            H.fill_pool(st, shape, mb, seed)
            out2, _, gt = H.run_gpu(st, shape, mb, seed, taps_layer=l)
            x_in = hidden.double() if l == 0 else otaps[l - 1]["x"]
            errs = H.check_taps(gt, otaps[l], x_in, x_in_gpu, f"f16 {shape.name} layer {l}")
            x_in_gpu = gt["x"]
            assert torch.equal(out2, out), "taps run changed the output"
            print(f"  layer {l} taps rel-L2: " + " ".join(f"{k}={v:.2e}" for k, v in errs.items()), flush=True)
    print(f"  output rel-L2 {stats['rel_l2']:.3e} max-abs {stats['max_abs']:.3e} rms {stats['rms']:.3f}", flush=True)
    st.close()
    return stats


def test_the_two_libraries_report_their_element_types():
    assert load_library(torch.bfloat16).stage_elem_type() == 0
    assert load_library(F16).stage_elem_type() == 1


def test_tiny_mixed_batch_with_taps():
    shape, mb = synth.workload("tiny", seed=0)
    stats = f16_parity(shape, mb, 0, taps=True)
    # three more mantissa bits than bfloat16: the same stage lands well inside the tolerance
    assert stats["rel_l2"] < 2e-3


def test_mid_stage_prefill_with_prefix_bias_and_decode():
    # 130 + 61 prefill rows (the second after a cached prefix), nine decode tokens; fan-in weights; q/k/v bias
    mb = synth.make_microbatch([130, 61, 1, 1, 1, 1, 1, 1, 1, 1, 1], [0, 40] + [20 + 9 * i for i in range(9)], seed=3,
                               max_blocks_per_seq=16)
    f16_parity(MID, mb, 3, "fan_in", taps=True, qkv_bias=True)


@pytest.mark.parametrize("n_decode", [1, 33, 64])
def test_decode_micro_batches_take_the_weight_streaming_kernels(n_decode):
    ctx = [40 + 97 * i % 700 for i in range(n_decode)]      # up to 700 cached keys: several key ranges per sequence
    mb = synth.make_microbatch([1] * n_decode, ctx, seed=5, max_blocks_per_seq=48)
    f16_parity(MID, mb, 5, "fan_in")


def test_more_than_64_rows_of_decode_take_the_tiled_kernels():
    ctx = [11 + 53 * i % 300 for i in range(150)]
    mb = synth.make_microbatch([1] * 150, ctx, seed=6, max_blocks_per_seq=20)
    f16_parity(MID, mb, 6, "fan_in")


def test_two_activation_planes_on_request():
    mb = synth.make_microbatch([40, 1, 1, 1], [0, 30, 5, 66], seed=2, max_blocks_per_seq=8)
    f16_parity(synth.TINY, mb, 2, activation_planes=2, taps=True)


@pytest.mark.parametrize("group", [32, 128])
def test_four_bit_weights_mixed_batch(group):
    mb = synth.make_microbatch([32, 32, 1, 1, 1, 1, 1, 1], [0, 0, 16, 37, 52, 64, 81, 100], seed=0, max_blocks_per_seq=12)
    f16_parity(W4_TINY, mb, 0, group=group)


@pytest.mark.parametrize("n_decode", [7, 20, 40, 64])
def test_four_bit_weights_streamed_in_decode(n_decode):
    ctx = [5 + 17 * i % 120 for i in range(n_decode)]
    mb = synth.make_microbatch([1] * n_decode, ctx, seed=4, max_blocks_per_seq=10)
    st = H.make_stage(MID, mb, 4, weight_group_size=128, dtype=F16)
    st.profile_enable(["dequant", "gemm_down"])
    out1, _ = H.run_gpu(st, MID, mb, 4)
    assert st.profile_read("dequant")[1] == 0          # nothing was expanded: the GEMMs read the codes
    assert st.profile_read("gemm_down")[1] == MID.num_layers
    H.fill_pool(st, MID, mb, 4)
    out2, _ = H.run_gpu(st, MID, mb, 4)
    assert torch.equal(out1, out2)                     # fixed summation order
    st.close()
    f16_parity(MID, mb, 4, group=128)


def test_four_bit_tiles_read_the_stored_form_above_64_rows():
    """A mixed micro-batch of 194 rows: every projection runs on the 4-bit tiles (the element type is half already),
    nothing is expanded in the workspace."""
    mb = synth.make_microbatch([130, 61, 1, 1, 1], [0, 40, 20, 29, 38], seed=3, max_blocks_per_seq=16)
    st = H.make_stage(MID, mb, 6, weight_group_size=128, dtype=F16)
    st.profile_enable(["dequant", "gemm_down"])
    H.run_gpu(st, MID, mb, 6)
    assert st.profile_read("dequant")[1] == 0
    assert st.profile_read("gemm_down")[1] == MID.num_layers
    st.close()
    f16_parity(MID, mb, 6, group=128)


def test_llama2_7b_stage_in_half_precision_sampled_rows_at_full_size():
    """The paper's 7B serving precision at the benchmark workload's real shape: 8 of 64 sequences checked row
    by row against the oracle at full depth (rows of different sequences are independent)."""
    shape, mb = synth.workload("llama2-7b", seed=0)
    print(f"[case] f16 {shape.name} T={mb.num_tokens} blocks={mb.num_kv_blocks}", flush=True)
    st = H.make_stage(shape, mb, 0, dtype=F16)
    out, slots = H.run_gpu(st, shape, mb, 0)
    assert slots == oracle.slot_mapping(mb.q_lens, mb.ctx_lens, mb.block_tables, 16)
    assert torch.isfinite(out.float()).all()
    seqs = list(range(0, 64, 8))
    sub, rows, pool = H.sub_problem(shape, mb, seqs, 0, dtype=torch.float32, draw_device="cuda:0", elem=F16)
    layers = [{k: v.cpu() for k, v in w.items()} for w in draw_layers(shape, 0, device="cuda:0", elem=F16)]
    hidden = synth.draw_hidden(shape, mb.num_tokens, seed=0, dtype=F16)[rows]
    ref, _ = oracle.stage_forward(oracle_shape(shape), layers, hidden, sub.positions, sub.q_lens, sub.ctx_lens,
                                  sub.block_tables, pool, dtype=torch.float32)
    stats = H.check_output(out[rows.cuda()], ref, "f16 llama2-7b sampled rows")
    print(f"  rel-L2 {stats['rel_l2']:.3e} max-abs {stats['max_abs']:.3e} rms {stats['rms']:.3f}", flush=True)
    st.close()


@pytest.mark.timeout(600)
def test_llama3_70b_stage_in_half_precision_keeps_one_activation_plane():
    """20 layers at the real shape, 256 decode tokens, contexts up to 8192.  The half-precision library does not
    change how it carries activations with depth (the bfloat16 one switches to half activations beyond 8
    layers); 4 sequences row by row show that one plane of half stays within the tolerance at this depth."""
    shape, mb = synth.workload("llama3-70b", seed=0)
    print(f"[case] f16 {shape.name} T={mb.num_tokens} blocks={mb.num_kv_blocks}", flush=True)
    from paper_2507_05043_amd.stage import make_config, stage_workspace_bytes
    def ws(planes, elem):
        cfg = make_config(num_layers=shape.num_layers, hidden=shape.hidden, num_q_heads=shape.num_q_heads,
                          num_kv_heads=shape.num_kv_heads, head_dim=shape.head_dim, ffn=shape.ffn, rms_eps=shape.rms_eps,
                          rope_theta=shape.rope_theta, num_kv_blocks=mb.num_kv_blocks, max_tokens=mb.num_tokens,
                          max_seqs=mb.num_seqs, max_blocks_per_seq=mb.max_blocks_per_seq, activation_planes=planes)
        return stage_workspace_bytes(cfg, elem)
    # left to the library (0), the half-precision one lays its workspace out for one plane of its own element
    # type; the bfloat16 one for second planes too (it decides per micro-batch between them and half activations)
    assert ws(0, F16) == ws(1, F16) != ws(2, F16)
    bf = torch.bfloat16
    assert ws(0, bf) > ws(1, bf) and ws(0, bf) >= ws(2, bf) and ws(0, bf) >= ws(3, bf) > ws(1, bf)
    st = H.make_stage(shape, mb, 0, dtype=F16)
    print("  stage ready", flush=True)
    out, slots = H.run_gpu(st, shape, mb, 0)
    assert slots == oracle.slot_mapping(mb.q_lens, mb.ctx_lens, mb.block_tables, 16)
    assert torch.isfinite(out.float()).all()
    seqs = [0, 85, 170, 255]
    sub, rows, pool = H.sub_problem(shape, mb, seqs, 0, dtype=torch.float32, draw_device="cuda:0", elem=F16)
    layers = [{k: v.cpu() for k, v in st.layers[l].items()} for l in range(shape.num_layers)]
    hidden = synth.draw_hidden(shape, mb.num_tokens, seed=0, dtype=F16)[rows]
    print("  oracle inputs ready", flush=True)
    ref, _ = oracle.stage_forward(oracle_shape(shape), layers, hidden, sub.positions, sub.q_lens, sub.ctx_lens,
                                  sub.block_tables, pool, dtype=torch.float32)
    stats = H.check_output(out[rows.cuda()], ref, "f16 llama3-70b sampled rows")
    print(f"  rel-L2 {stats['rel_l2']:.3e} max-abs {stats['max_abs']:.3e} rms {stats['rms']:.3f}", flush=True)
    st.close()
    del st
    torch.cuda.empty_cache()


def test_the_pipeline_ends_in_half_precision():
    shape = synth.TINY
    q_lens = [3, 1, 1, 5, 1, 1, 2]
    t = sum(q_lens)
    mb = synth.make_microbatch(q_lens, [0] * len(q_lens), seed=0, max_blocks_per_seq=2)
    st = H.make_stage(shape, mb, 0, vocab_size=shape.vocab, fill_kv=False, dtype=F16)
    ends = synth.draw_ends_weights(shape, seed=0, device="cuda:0", head_std=0.06, dtype=F16)
    ids = synth.draw_token_ids(shape, t, seed=0)
    emb = st.embed(ends["embed"], ids)
    torch.cuda.synchronize()
    assert emb.dtype == F16 and torch.equal(emb.cpu(), ends["embed"].cpu()[torch.tensor(ids)])   # a gather: bit-exact
    hidden = (synth.draw_hidden(shape, t, seed=0, device="cuda:0", dtype=F16).float() * 3.0).to(F16)
    tokens, logits = st.head(hidden, q_lens, ends["final_norm"], ends["lm_head"])
    torch.cuda.synchronize()
    ref = oracle.head_logits(hidden.cpu(), q_lens, ends["final_norm"].cpu(), ends["lm_head"].cpu(), shape.rms_eps)
    r = rel_l2(logits.cpu().double(), ref)
    assert r <= 1e-2, f"logits rel-L2 {r:.3e}"
    gl = logits.cpu().numpy()
    assert np.array_equal(tokens.cpu().numpy(), gl.argmax(axis=1))
    err = np.abs(gl.astype(np.float64) - ref.numpy()).max()
    srt = np.sort(ref.numpy(), axis=1)
    clear = (srt[:, -1] - srt[:, -2]) > 2 * err
    assert clear.any()
    assert np.array_equal(tokens.cpu().numpy()[clear], oracle.greedy_tokens(ref).numpy()[clear])
    st.close()
