"""The entry point that allocates nothing: stage_forward_static, whose scratch is an array inside the library's
device image, against stage_forward with a caller workspace - same kernels, same launch shapes, so the same bits."""
import ctypes

import pytest
import torch

from paper_2507_05043_amd import StageError, synth
from tests import gpu_harness as H

pytestmark = pytest.mark.gpu


def _shape(name, L, H_, nq, nkv, d, F):
    return synth.StageShape(name, L, H_, nq, nkv, d, F)


def _both(st, shape, mb, seed):
    """stage_forward, then stage_forward_static on the same cache contents, outputs preallocated."""
    hidden = synth.draw_hidden(shape, mb.num_tokens, seed=seed, device="cuda:0")
    tables = torch.full((mb.num_seqs, st.cfg.max_blocks_per_seq), -1, dtype=torch.int32)
    tables[:, : mb.block_tables.shape[1]] = mb.block_tables
    want = torch.empty_like(hidden)
    got = torch.empty_like(hidden)
    st.forward(hidden, mb.positions, mb.q_lens, mb.ctx_lens, tables, out=want)
    torch.cuda.synchronize()
    pool_after = st.kv_pool.clone()
    return hidden, tables, want, got, pool_after


@pytest.mark.parametrize("weight_copies", [1, 0], ids=["no-copies", "weight-copies"])
def test_static_scratch_forward_equals_the_workspace_forward_twice_in_a_row(weight_copies):
    """Without the weights' second copies nothing of the caller's workspace takes part in the call (it is overwritten
    beforehand and must come back untouched); with them, the copies - written once by stage_init - are the one part
    of it that is read."""
    shape = _shape("static-mid", 2, 1024, 8, 2, 128, 2816)
    big = synth.make_microbatch([130, 61, 1, 1, 1, 1, 1, 1, 1], [0, 40] + [20 + 9 * i for i in range(7)], seed=3,
                                max_blocks_per_seq=16)
    small = synth.make_microbatch([1, 1, 17], [33, 5, 8], seed=4, max_blocks_per_seq=16)
    st = H.make_stage(shape, big, 3, "fan_in", weight_copies=weight_copies)
    ws_before = None
    for call, mb in enumerate((big, small)):           # the second call is smaller: stale scratch lies behind it
        print(f"[case] static scratch call {call}: T={mb.num_tokens} S={mb.num_seqs}", flush=True)
        if mb is small:
            # the small batch's cached context, drawn at its own block numbers into the same pool
            st.kv_pool.view(st.dtype).fill_(float("nan"))
            tmp = H.make_stage(shape, small, 4, "fan_in", weight_copies=1)
            blocks = torch.arange(small.num_kv_blocks, device="cuda:0")
            for l in range(shape.num_layers):
                for kv in (0, 1):
                    st.write_kv_blocks(l, kv, blocks, tmp.read_kv_blocks(l, kv, blocks))
            tmp.close()
        pool_before = st.kv_pool.clone()
        hidden, tables, want, got, pool_after = _both(st, shape, mb, 3 + call)
        st.kv_pool.copy_(pool_before)
        if weight_copies == 1:
            st.workspace.fill_(0x5A)                    # the caller workspace must not take part
        ws_before = st.workspace.clone()
        slots = st.forward(hidden, mb.positions, mb.q_lens, mb.ctx_lens, tables, out=got, want_slots=True,
                           static_scratch=True)[1]
        torch.cuda.synchronize()
        assert torch.isfinite(got.float()).all()
        assert torch.equal(got.view(torch.int16), want.view(torch.int16)), f"call {call}: outputs differ"
        assert torch.equal(st.kv_pool, pool_after), f"call {call}: appended keys/values differ"
        assert torch.equal(st.workspace, ws_before), f"call {call}: the caller workspace was written"
        import oracle
        assert slots == oracle.slot_mapping(mb.q_lens, mb.ctx_lens, mb.block_tables, 16)
        if mb is big:
            ref, _, _, _ = H.run_oracle(shape, mb, 3, "fan_in")
            H.check_output(got, ref, "static scratch output")
    st.close()


def test_static_scratch_rejects_what_does_not_fit_and_leaves_the_pool_untouched():
    """A micro-batch whose intermediates exceed the library's scratch array is an error before anything is enqueued."""
    shape = _shape("static-wide", 1, 4096, 32, 32, 128, 11008)
    mb = synth.make_microbatch([2048], [0], seed=5)
    st = H.make_stage(shape, mb, 5)
    hidden = synth.draw_hidden(shape, mb.num_tokens, seed=5, device="cuda:0")
    out = torch.empty_like(hidden)
    before = st.kv_pool.clone()
    with pytest.raises(StageError) as ei:
        st.forward(hidden, mb.positions, mb.q_lens, mb.ctx_lens, mb.block_tables, out=out, static_scratch=True)
    assert ei.value.code == -3
    torch.cuda.synchronize()
    assert torch.equal(before.view(torch.int16), st.kv_pool.view(torch.int16))
    # the same handle still serves the ordinary entry point
    st.forward(hidden, mb.positions, mb.q_lens, mb.ctx_lens, mb.block_tables, out=out)
    torch.cuda.synchronize()
    assert torch.isfinite(out.float()).all()
    st.close()


def test_static_scratch_forward_of_a_parallel_layernorm_block():
    """The blocks that keep more intermediates (the second norm of a parallel block, the ungated MLP's first product)
    carve them from the library's array too: same bits as with the caller's workspace."""
    import dataclasses
    shape = dataclasses.replace(_shape("static-block-kinds", 2, 1024, 8, 2, 128, 2816), norm_kind="layer",
                                mlp_kind="gelu_erf", parallel_block=True)
    mb = synth.make_microbatch([90, 1, 1, 1], [5, 40, 300, 17], seed=6, max_blocks_per_seq=24)
    st = H.make_stage(shape, mb, 6, "fan_in", block_biases=True, alibi=True)
    pool_before = st.kv_pool.clone()
    hidden, tables, want, got, pool_after = _both(st, shape, mb, 6)
    st.kv_pool.copy_(pool_before)
    st.forward(hidden, mb.positions, mb.q_lens, mb.ctx_lens, tables, out=got, static_scratch=True)
    torch.cuda.synchronize()
    assert torch.equal(got.view(torch.int16), want.view(torch.int16))
    assert torch.equal(st.kv_pool, pool_after)
    from tests.helpers import draw_layers
    ref, _, _, _ = H.run_oracle(shape, mb, 6, "fan_in", layers=draw_layers(shape, 6, "fan_in", block_biases=True, alibi=True))
    H.check_output(got, ref, "static scratch, parallel LayerNorm block")
    st.close()
