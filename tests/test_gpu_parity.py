"""GPU parity: the HIP library (through its C ABI) against the CPU oracle on the same seeded inputs."""
import pytest
import torch

import oracle
from paper_2507_05043_amd import StageError, synth
from tests import gpu_harness as H
from tests.helpers import draw_layers, oracle_shape, rel_l2

pytestmark = pytest.mark.gpu


def _shape(name, L, H_, nq, nkv, d, F, theta=1e4):
    return synth.StageShape(name, L, H_, nq, nkv, d, F, rope_theta=theta)


def full_parity(shape, mb, seed, weight_std, taps=True, check_kv=True):
    print(f"[case] {shape.name} T={mb.num_tokens} S={mb.num_seqs} q={mb.q_lens[:6]} ctx={mb.ctx_lens[:6]} "
          f"std={weight_std} seed={seed}", flush=True)
    st = H.make_stage(shape, mb, seed, weight_std)
    before = H.snapshot_pool(st, shape, mb) if check_kv else None
    ref, ref_slots, ref_pool, otaps = H.run_oracle(shape, mb, seed, weight_std, want_taps=True)
    out, slots = H.run_gpu(st, shape, mb, seed)
    assert slots == ref_slots                                   # bit-exact slot indexing
    stats = H.check_output(out, ref)
    if check_kv:
        H.check_pool(st, shape, mb, ref_pool, before, slots)
    if taps:
        hidden = synth.draw_hidden(shape, mb.num_tokens, seed=seed)
        x_in_gpu = hidden
        for l in range(shape.num_layers):
            H.fill_pool(st, shape, mb, seed)
            out2, _, gt = H.run_gpu(st, shape, mb, seed, taps_layer=l)
            x_in = hidden.double() if l == 0 else otaps[l - 1]["x"]
            errs = H.check_taps(gt, otaps[l], x_in, x_in_gpu, f"{shape.name} layer {l}")
            x_in_gpu = gt["x"]
            assert torch.equal(out2, out), "taps run changed the output"
            print(f"  layer {l} taps rel-L2: " + " ".join(f"{k}={v:.2e}" for k, v in errs.items()), flush=True)
    print(f"  output rel-L2 {stats['rel_l2']:.3e} max-abs {stats['max_abs']:.3e} rms {stats['rms']:.3f}", flush=True)
    st.close()
    return stats


def test_generator_same_bits_on_gpu_and_cpu():
    a = synth.draw_normal_bf16(0, 7, 100000, std=0.02, mean=1.0)
    b = synth.draw_normal_bf16(0, 7, 100000, std=0.02, mean=1.0, device="cuda:0").cpu()
    assert torch.equal(a.view(torch.int16), b.view(torch.int16))
    blocks = torch.tensor([5, 0, 33])
    x = synth.draw_kv_blocks(synth.TINY, 35, 1, 1, blocks, seed=0)
    y = synth.draw_kv_blocks(synth.TINY, 35, 1, 1, blocks.cuda(), seed=0).cpu()
    assert torch.equal(x.view(torch.int16), y.view(torch.int16))


@pytest.mark.parametrize("weight_std", [None, "fan_in"])
def test_tiny_stage(weight_std):
    shape, mb = synth.workload("tiny", seed=0)
    full_parity(shape, mb, 0, weight_std)


@pytest.mark.parametrize("case", [
    dict(q=[1], c=[0]),                                   # a single fresh token: one key
    dict(q=[1, 1, 1], c=[15, 16, 31]),                    # block boundaries
    dict(q=[17, 33, 5, 1, 1], c=[0, 15, 100, 0, 31]),     # ragged chunks with and without cached prefix
    dict(q=[64], c=[0]),                                  # exactly two query tiles
    dict(q=[3, 1], c=[700, 1500]),                        # long caches: several key ranges per decode token
])
def test_edge_batches_d64(case):
    shape = _shape("edge-d64-g2", 2, 256, 4, 2, 64, 688)
    mb = synth.make_microbatch(case["q"], case["c"], seed=21)
    full_parity(shape, mb, 21, "fan_in")


@pytest.mark.parametrize("nq,nkv", [(4, 4), (8, 2), (14, 2), (16, 1)])
def test_head_groupings_d128(nq, nkv):
    shape = _shape(f"d128-nq{nq}-nkv{nkv}", 1, 512, nq, nkv, 128, 1096)
    mb = synth.make_microbatch([40, 1, 1, 9, 1], [0, 257, 33, 50, 1200], seed=22)
    full_parity(shape, mb, 22, "fan_in")


def test_large_m_tiles_and_k_tails():
    # T > 64 takes the 128-row GEMM tiles; F = 1096 and H = 520 leave K and N tails in every GEMM
    shape = _shape("gemm-tails", 2, 520, 4, 2, 64, 1096)
    mb = synth.make_microbatch([150, 61, 1, 1], [0, 20, 300, 5], seed=23)
    full_parity(shape, mb, 23, "fan_in")
    full_parity(shape, mb, 23, None, taps=False)


def test_chunked_prefill_equals_unsplit_on_gpu():
    shape = _shape("chunks", 2, 256, 4, 2, 64, 688)
    n = 75
    mb = synth.make_microbatch([n], [0], seed=24)
    st = H.make_stage(shape, mb, 24, "fan_in")
    hidden = synth.draw_hidden(shape, n, seed=24, device="cuda:0")
    full = st.forward(hidden, mb.positions, [n], [0], mb.block_tables).clone()
    H.fill_pool(st, shape, mb, 24)
    outs, done = [], 0
    for c in (5, 11, 16, 42, 1):
        pos = torch.arange(done, done + c, dtype=torch.int32)
        outs.append(st.forward(hidden[done:done + c].contiguous(), pos, [c], [done], mb.block_tables).clone())
        done += c
    torch.cuda.synchronize()
    got = torch.cat(outs).cpu().double()
    ref, _, _, _ = H.run_oracle(shape, mb, 24, "fan_in")
    H.check_output(torch.cat(outs), ref, "chunked output")
    assert rel_l2(got, full.cpu().double()) <= 5e-3
    st.close()


def test_shifted_positions_are_used_for_rope_only():
    shape = _shape("shift", 1, 256, 4, 2, 64, 688)
    mb = synth.make_microbatch([20, 1], [0, 40], seed=25, position_shift=1000)
    full_parity(shape, mb, 25, "fan_in")


def test_two_runs_are_bitwise_identical():
    shape, mb = synth.workload("tiny", seed=0)
    st = H.make_stage(shape, mb, 0, "fan_in")
    out1, _ = H.run_gpu(st, shape, mb, 0)
    out1 = out1.clone()
    H.fill_pool(st, shape, mb, 0)
    out2, _ = H.run_gpu(st, shape, mb, 0)
    assert torch.equal(out1.view(torch.int16), out2.view(torch.int16))
    st.close()


def test_invalid_batches_are_rejected_and_leave_the_pool_untouched():
    shape, mb = synth.workload("tiny", seed=0)
    st = H.make_stage(shape, mb, 0)
    before = st.kv_pool.clone()
    hidden = synth.draw_hidden(shape, mb.num_tokens, seed=0, device="cuda:0")
    bad_table = mb.block_tables.clone()
    bad_table[2, 1] = mb.num_kv_blocks
    cases = [
        (dict(q_lens=[33] + mb.q_lens[1:]), -4),                       # sum(q_lens) != T ... needs a block too
        (dict(ctx_lens=[-1] + mb.ctx_lens[1:]), -4),
        (dict(q_lens=[0] + mb.q_lens[1:]), -4),
        (dict(block_tables=bad_table), -5),
        (dict(ctx_lens=[200] + mb.ctx_lens[1:]), -5),                  # needs more blocks than a row holds
    ]
    for change, code in cases:
        args = dict(positions=mb.positions, q_lens=mb.q_lens, ctx_lens=mb.ctx_lens, block_tables=mb.block_tables)
        args.update(change)
        with pytest.raises(StageError) as ei:
            st.forward(hidden, **args)
        assert ei.value.code in (code, -4, -5)
    with pytest.raises(StageError) as ei:
        st.forward(hidden, mb.positions, mb.q_lens, mb.ctx_lens, mb.block_tables, out=hidden)
    assert ei.value.code == -7
    torch.cuda.synchronize()
    assert torch.equal(before, st.kv_pool)
    st.close()


def test_llama2_7b_stage_sampled_rows_at_full_size():
    """The benchmark workload at its real shape: 8 of 64 sequences checked row by row against the
    oracle at full depth (rows of different sequences are independent, so the sample is exact)."""
    shape, mb = synth.workload("llama2-7b", seed=0)
    print(f"[case] {shape.name} T={mb.num_tokens} blocks={mb.num_kv_blocks}", flush=True)
    st = H.make_stage(shape, mb, 0)
    out, slots = H.run_gpu(st, shape, mb, 0)
    assert slots == oracle.slot_mapping(mb.q_lens, mb.ctx_lens, mb.block_tables, 16)
    assert torch.isfinite(out.float()).all()
    seqs = list(range(0, 64, 8))
    sub, rows, pool = H.sub_problem(shape, mb, seqs, 0, dtype=torch.float32, draw_device="cuda:0")
    layers = draw_layers(shape, 0, device="cuda:0")
    layers = [{k: v.cpu() for k, v in w.items()} for w in layers]
    hidden = synth.draw_hidden(shape, mb.num_tokens, seed=0)[rows]
    ref, _ = oracle.stage_forward(oracle_shape(shape), layers, hidden, sub.positions, sub.q_lens, sub.ctx_lens,
                                  sub.block_tables, pool, dtype=torch.float32)
    stats = H.check_output(out[rows.cuda()], ref, "llama2-7b sampled rows")
    print(f"  rel-L2 {stats['rel_l2']:.3e} max-abs {stats['max_abs']:.3e} rms {stats['rms']:.3f}", flush=True)
    st.close()
