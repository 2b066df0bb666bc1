"""GPU parity of stages with 4-bit group-quantised weights: the HIP library (through its C ABI) against the
CPU oracle run on the matrices the stored form stands for (oracle/w4_oracle.py), same seeded inputs."""
import pytest
import torch

from oracle import w4_oracle
from paper_2507_05043_amd import synth
from tests import gpu_harness as H

pytestmark = pytest.mark.gpu

# the tiny stage with an inner width that every supported group size divides
W4_TINY = synth.StageShape("tiny-w4", 2, 256, 4, 2, 64, 768)


def w4_parity(shape, mb, seed, group, activation_planes=0, check_kv=True):
    print(f"[case] {shape.name} 4-bit group={group} T={mb.num_tokens} S={mb.num_seqs} q={mb.q_lens[:6]} "
          f"ctx={mb.ctx_lens[:6]} seed={seed} planes={activation_planes}", flush=True)
    st = H.make_stage(shape, mb, seed, weight_group_size=group, activation_planes=activation_planes)
    before = H.snapshot_pool(st, shape, mb) if check_kv else None
    stored = [synth.draw_w4_layer(shape, l, seed=seed, group=group) for l in range(shape.num_layers)]
    for l, lw in enumerate(stored):          # the GPU stage was built from the same stored form, bit for bit
        for k, v in lw.items():
            assert torch.equal(st.layers[l][k].cpu().view(torch.int16 if v.dtype == torch.bfloat16 else v.dtype),
                               v.view(torch.int16 if v.dtype == torch.bfloat16 else v.dtype)), (l, k)
    layers = [w4_oracle.dequantize_layer(lw, group) for lw in stored]
    ref, ref_slots, ref_pool, _ = H.run_oracle(shape, mb, seed, layers=layers)
    out, slots = H.run_gpu(st, shape, mb, seed)
    assert slots == ref_slots
    stats = H.check_output(out, ref)
    if check_kv:
        H.check_pool(st, shape, mb, ref_pool, before, slots)
    print(f"  output rel-L2 {stats['rel_l2']:.3e} max-abs {stats['max_abs']:.3e} rms {stats['rms']:.3f}", flush=True)
    st.close()
    return stats


@pytest.mark.parametrize("group", [32, 64, 128])
def test_tiny_mixed_batch(group):
    mb = synth.make_microbatch([32, 32, 1, 1, 1, 1, 1, 1], [0, 0, 16, 37, 52, 64, 81, 100], seed=0, max_blocks_per_seq=12)
    w4_parity(W4_TINY, mb, 0, group)


@pytest.mark.parametrize("n_decode", [1, 7, 64])
def test_decode_micro_batches(n_decode):
    ctx = [17 + 13 * i % 90 for i in range(n_decode)]
    mb = synth.make_microbatch([1] * n_decode, ctx, seed=1, max_blocks_per_seq=8)
    w4_parity(W4_TINY, mb, 1, 128)


@pytest.mark.parametrize("n_decode", [11, 20, 32, 40, 48, 64])
def test_decode_streams_the_stored_form_with_a_ragged_last_slice(n_decode):
    # inner width 2816 = 2.75 slices of 1024: the down projection's last slice is partly empty; 1..4 blocks of rows
    shape = synth.StageShape("w4-mid", 2, 1024, 8, 2, 128, 2816)
    ctx = [5 + 17 * i % 120 for i in range(n_decode)]
    mb = synth.make_microbatch([1] * n_decode, ctx, seed=4, max_blocks_per_seq=10)
    st = H.make_stage(shape, mb, 4, weight_group_size=128)
    st.profile_enable(["dequant", "gemm_qkv", "gemm_down"])
    out1, _ = H.run_gpu(st, shape, mb, 4)
    assert st.profile_read("dequant")[1] == 0          # nothing was expanded: the GEMMs read the codes
    assert st.profile_read("gemm_down")[1] == shape.num_layers
    H.fill_pool(st, shape, mb, 4)
    out2, _ = H.run_gpu(st, shape, mb, 4)
    assert torch.equal(out1, out2)                     # fixed summation order
    st.close()
    w4_parity(shape, mb, 4, 128)


def test_two_activation_planes():
    mb = synth.make_microbatch([40, 1, 1, 1], [0, 30, 5, 66], seed=2, max_blocks_per_seq=8)
    w4_parity(W4_TINY, mb, 2, 128, activation_planes=2)


W4_MID = synth.StageShape("w4-mid", 2, 1024, 8, 2, 128, 2816)


def _mid_batch(kind):
    if kind == "decode-40":
        return synth.make_microbatch([1] * 40, [5 + 17 * i % 120 for i in range(40)], seed=4, max_blocks_per_seq=10)
    if kind == "decode-150":       # more than 64 rows of decode: the tiles, not the streaming kernel
        return synth.make_microbatch([1] * 150, [5 + 17 * i % 120 for i in range(150)], seed=4, max_blocks_per_seq=10)
    if kind == "mixed-194":
        return synth.make_microbatch([130, 61, 1, 1, 1], [0, 40, 20, 29, 38], seed=3, max_blocks_per_seq=16)
    if kind == "mixed-345":        # two rows of 256-row tiles, the second one ragged
        return synth.make_microbatch([280, 61, 1, 1, 1, 1], [0, 40, 20, 29, 38, 7], seed=3, max_blocks_per_seq=24)
    raise ValueError(kind)


@pytest.mark.parametrize("kind", ["decode-40", "decode-150", "mixed-194", "mixed-345"])
def test_half_activations_with_four_bit_weights(kind):
    """What a deep bfloat16 stage with 4-bit weights runs by default: projection inputs as IEEE half.  Every
    projection reads the stored form - a decode batch of at most 64 rows through the streaming kernel, anything
    larger through the 4-bit tiles - with the codes expanded to half in registers; nothing is expanded in memory,
    and the summation order is fixed."""
    shape, mb = W4_MID, _mid_batch(kind)
    st = H.make_stage(shape, mb, 6, weight_group_size=128, activation_planes=3)
    st.profile_enable(["dequant", "gemm_gateup"])
    out1, _ = H.run_gpu(st, shape, mb, 6)
    assert st.profile_read("dequant")[1] == 0
    assert st.profile_read("gemm_gateup")[1] == shape.num_layers
    H.fill_pool(st, shape, mb, 6)
    out2, _ = H.run_gpu(st, shape, mb, 6)
    assert torch.equal(out1, out2)
    st.close()
    w4_parity(shape, mb, 6, 128, activation_planes=3)


def test_inner_widths_the_four_bit_tiles_do_not_take_are_expanded():
    """The tiles need K to be a multiple of 256: with an inner width of 2944 = 23 groups the down projection is
    expanded in the workspace while the other three read the stored form."""
    shape = synth.StageShape("w4-mid-23-groups", 2, 1024, 8, 2, 128, 2944)
    mb = _mid_batch("mixed-194")
    st = H.make_stage(shape, mb, 6, weight_group_size=128, activation_planes=3)
    st.profile_enable(["dequant"])
    H.run_gpu(st, shape, mb, 6)
    assert st.profile_read("dequant")[1] == shape.num_layers
    st.close()
    w4_parity(shape, mb, 6, 128, activation_planes=3)


def test_fractional_zero_points_and_uneven_scales():
    """Zero points that are not integers and scales spread over a factor of 16 (the synthetic draw has integer zero
    points and scales within a factor of 1.7): stored form edited on the host, the same edit on both sides.  The
    factors' mean square is about one, so the stage keeps its scale."""
    from paper_2507_05043_amd.stage import Stage, make_config
    shape, mb, seed = W4_MID, _mid_batch("mixed-194"), 8
    stored = [synth.draw_w4_layer(shape, l, seed=seed, group=128) for l in range(shape.num_layers)]
    for lw in stored:
        for name in ("qkv", "o", "gate", "up", "down"):
            z, s = lw["z" + name], lw["s" + name]
            rows = torch.arange(z.shape[0]).view(-1, 1)
            cols = torch.arange(z.shape[1]).view(1, -1)
            lw["z" + name] = (z.float() + ((rows * 7 + cols * 3) % 16).float() / 16 - 0.5).to(torch.bfloat16)
            lw["s" + name] = (s.float() * torch.pow(2.0, ((rows + cols) % 5 - 3).float())).to(torch.bfloat16)
    cfg = make_config(num_layers=shape.num_layers, hidden=shape.hidden, num_q_heads=shape.num_q_heads,
                      num_kv_heads=shape.num_kv_heads, head_dim=shape.head_dim, ffn=shape.ffn, rms_eps=shape.rms_eps,
                      rope_theta=shape.rope_theta, num_kv_blocks=mb.num_kv_blocks, max_tokens=mb.num_tokens,
                      max_seqs=mb.num_seqs, max_blocks_per_seq=mb.max_blocks_per_seq, activation_planes=3,
                      weight_bits=4, weight_group_size=128)
    st = Stage(cfg, [{k: v.to("cuda:0") for k, v in lw.items()} for lw in stored], device="cuda:0")
    H.fill_pool(st, shape, mb, seed)
    st.profile_enable(["dequant"])
    layers = [w4_oracle.dequantize_layer(lw, 128) for lw in stored]
    ref, ref_slots, _, _ = H.run_oracle(shape, mb, seed, layers=layers)
    out, slots = H.run_gpu(st, shape, mb, seed)
    assert st.profile_read("dequant")[1] == 0
    assert slots == ref_slots
    stats = H.check_output(out, ref)
    print(f"  output rel-L2 {stats['rel_l2']:.3e} max-abs {stats['max_abs']:.3e} rms {stats['rms']:.3f}", flush=True)
    st.close()


@pytest.mark.timeout(600)
def test_four_bit_tiles_at_the_70b_widths():
    """One layer of the Llama-3-70B shape (hidden 8192, inner width 28672, 64 / 8 heads) with 4-bit weights and 256
    decode tokens - the micro-batch of the largest benchmark workload at short contexts: 16 sequences row by row."""
    import oracle
    from tests.helpers import oracle_shape
    shape = synth.StageShape("llama3-70b-w4-1layer", 1, 8192, 64, 8, 128, 28672, rope_theta=5e5)
    ctx = [16 + (37 * i) % 180 for i in range(256)]
    mb = synth.make_microbatch([1] * 256, ctx, seed=5, max_blocks_per_seq=14)
    print(f"[case] {shape.name} 4-bit T={mb.num_tokens} blocks={mb.num_kv_blocks}", flush=True)
    st = H.make_stage(shape, mb, 5, weight_group_size=128, activation_planes=3)
    st.profile_enable(["dequant"])
    out, slots = H.run_gpu(st, shape, mb, 5)
    assert st.profile_read("dequant")[1] == 0
    assert slots == oracle.slot_mapping(mb.q_lens, mb.ctx_lens, mb.block_tables, 16)
    print("  GPU forward done", flush=True)
    stored = {k: v.cpu() for k, v in synth.draw_w4_layer(shape, 0, seed=5, group=128, device="cuda:0").items()}
    for k, v in stored.items():
        assert torch.equal(st.layers[0][k].cpu().view(torch.int16 if v.dtype == torch.bfloat16 else v.dtype),
                           v.view(torch.int16 if v.dtype == torch.bfloat16 else v.dtype)), k
    layers = [w4_oracle.dequantize_layer(stored, 128, dtype=torch.float32)]
    print("  oracle weights ready", flush=True)
    seqs = sorted({round(i * 255 / 15) for i in range(16)})
    sub, rows, pool = H.sub_problem(shape, mb, seqs, 5, dtype=torch.float32, draw_device="cuda:0")
    hidden = synth.draw_hidden(shape, mb.num_tokens, seed=5)[rows]
    ref, _ = oracle.stage_forward(oracle_shape(shape), layers, hidden, sub.positions, sub.q_lens, sub.ctx_lens,
                                  sub.block_tables, pool, dtype=torch.float32)
    stats = H.check_output(out[rows.cuda()], ref, shape.name)
    print(f"  output rel-L2 {stats['rel_l2']:.3e} max-abs {stats['max_abs']:.3e} rms {stats['rms']:.3f}", flush=True)
    st.close()


def test_ragged_rows_and_longer_k():
    # 200 rows (not a multiple of any tile), hidden 1024, inner width 2816 = 22 groups of 128
    shape = synth.StageShape("w4-mid", 2, 1024, 8, 2, 128, 2816)
    mb = synth.make_microbatch([130, 61, 1, 1, 1, 1, 1, 1, 1, 1, 1], [0, 40] + [20 + 9 * i for i in range(9)], seed=3,
                               max_blocks_per_seq=16)
    w4_parity(shape, mb, 3, 128)


def test_missing_scales_are_rejected():
    from paper_2507_05043_amd import StageError
    from paper_2507_05043_amd.stage import Stage, make_config
    mb = synth.make_microbatch([4], [0], seed=0, max_blocks_per_seq=2)
    layers = [synth.draw_w4_layer(W4_TINY, l, seed=0, group=128, device="cuda:0") for l in range(2)]
    cfg = make_config(num_layers=2, hidden=256, num_q_heads=4, num_kv_heads=2, head_dim=64, ffn=768, rms_eps=1e-5,
                      rope_theta=1e4, num_kv_blocks=mb.num_kv_blocks, max_tokens=8, max_seqs=2, max_blocks_per_seq=2,
                      weight_bits=4, weight_group_size=128)
    st = Stage(cfg, layers)
    st.close()
    del layers[1]["zdown"]
    with pytest.raises(KeyError):
        Stage(cfg, layers)
