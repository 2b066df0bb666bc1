"""GPU parity of the pipeline's two ends (stage_embed, stage_head through the C ABI) against the CPU
oracle on the same seeded inputs."""
import dataclasses

import numpy as np
import pytest
import torch

import oracle
from paper_2507_05043_amd import StageError, synth
from tests import gpu_harness as H
from tests.helpers import draw_layers, oracle_shape, rel_l2

pytestmark = pytest.mark.gpu

LOGIT_REL_L2_TOL = 1e-2     # same bar as the hidden states: one bf16 rounding (the norm output) then fp32 sums


def _head_stage(shape, num_seqs, num_tokens, seed):
    """A one-layer stage of the shape's width, sized for the batch, with the output head's scratch."""
    one = dataclasses.replace(shape, num_layers=1)
    mb = synth.make_microbatch([1] * num_seqs, [0] * num_seqs, seed=seed)
    return H.make_stage(one, mb, seed, max_tokens=max(num_tokens, num_seqs), fill_kv=False, vocab_size=shape.vocab)


def _q_lens(num_seqs, seed):
    """A mix of decode rows and a few chunks, so last rows are not simply every row."""
    q = [1] * num_seqs
    for i, extra in zip(range(0, num_seqs, 3), synth.draw_int_uniform(seed, 77, num_seqs, 0, 4)):
        q[i] += extra
    return q


def _check_tokens(tokens, gpu_logits, ref_logits, what):
    """Greedy choice: bit-exact against the GPU's own logits (first maximum); against the oracle, equal
    wherever the oracle's winner leads by more than the logits' error allows, and otherwise a token
    whose oracle logit is within that error of the oracle's maximum."""
    got = tokens.cpu().numpy().astype(np.int64)
    gl = gpu_logits.cpu().numpy()
    assert np.array_equal(got, gl.argmax(axis=1)), f"{what}: argmax of the GPU logits"
    ref = ref_logits.numpy()
    err = np.abs(gl.astype(np.float64) - ref).max()
    ref_tok = oracle.greedy_tokens(ref_logits).numpy()
    srt = np.sort(ref, axis=1)
    margin = srt[:, -1] - srt[:, -2]
    clear = margin > 2 * err
    assert np.array_equal(got[clear], ref_tok[clear]), f"{what}: greedy tokens where the oracle's margin is clear"
    chosen = ref[np.arange(ref.shape[0]), got]
    assert (chosen >= srt[:, -1] - 2 * err).all(), f"{what}: a chosen token is not within the error of the maximum"
    return int(clear.sum())


def _head_case(shape, num_seqs, seed, sample=None, head_std=0.02, norm_bias=False):
    """shape.norm_kind "layer": the LayerNorm head (stage_head_layernorm), with a bias if norm_bias; the hidden rows
    then get a mean of their own."""
    layer = shape.norm_kind == "layer"
    q_lens = _q_lens(num_seqs, seed)
    t = sum(q_lens)
    print(f"[case] head {shape.name} S={num_seqs} T={t} vocab={shape.vocab} seed={seed}", flush=True)
    st = _head_stage(shape, num_seqs, t, seed)
    ends = synth.draw_ends_weights(shape, seed=seed, device="cuda:0", head_std=head_std)
    hidden = (synth.draw_hidden(shape, t, seed=seed, device="cuda:0").float() * 3.0 + (2.0 if layer else 0.0)).to(torch.bfloat16)
    bias = synth.draw_block_biases(shape, 0, seed=seed, device="cuda:0")["norm1_bias"] if norm_bias else None
    tokens, logits = st.head(hidden, q_lens, ends["final_norm"], ends["lm_head"], final_norm_bias=bias)
    tokens2, none = st.head(hidden, q_lens, ends["final_norm"], ends["lm_head"], want_logits=False, final_norm_bias=bias)
    torch.cuda.synchronize()
    assert none is None and torch.equal(tokens, tokens2), "tokens differ when no logits are requested"
    # oracle on the same bf16 inputs; at the largest shape on a sample of sequences (rows are independent)
    seqs = list(range(num_seqs)) if sample is None else sample
    hid_cpu, gain, w = hidden.cpu(), ends["final_norm"].cpu(), ends["lm_head"].cpu()
    ref = oracle.head_logits(hid_cpu, q_lens, gain, w, shape.rms_eps, norm_kind=shape.norm_kind,
                             bias=None if bias is None else bias.cpu())[seqs]
    got = logits[seqs]
    r = rel_l2(got.cpu().double(), ref)
    rms = float(ref.pow(2).mean().sqrt())
    max_abs = float((got.cpu().double() - ref).abs().max())
    assert torch.isfinite(logits).all()
    assert r <= LOGIT_REL_L2_TOL, f"logits rel-L2 {r:.3e}"
    assert max_abs <= H.MAX_ABS_TOL * max(1.0, rms), f"logits max-abs {max_abs:.3e} (rms {rms:.3f})"
    clear = _check_tokens(tokens[seqs], got, ref, shape.name)
    # the argmax kernel on every row, sampled or not
    assert np.array_equal(tokens.cpu().numpy(), logits.cpu().numpy().argmax(axis=1))
    print(f"  logits rel-L2 {r:.3e} max-abs {max_abs:.3e} rms {rms:.3f}; {clear}/{len(seqs)} rows with a clear margin",
          flush=True)
    st.close()


@pytest.mark.parametrize("num_seqs", [1, 5, 64, 65, 130])
def test_head_tiny_shapes_cover_both_gemm_paths_and_ragged_rows(num_seqs):
    _head_case(synth.TINY, num_seqs, seed=num_seqs, head_std=0.06)


def test_head_vocab_and_width_tails():
    # vocab not a multiple of 16 rows, hidden not a multiple of the 1024-wide K slice
    shape = synth.StageShape("tails", 1, 328, 2, 2, 64, 128, vocab=1064)
    _head_case(shape, 7, seed=3, head_std=0.05)
    _head_case(shape, 70, seed=4, head_std=0.05)


@pytest.mark.parametrize("num_seqs,norm_bias", [(5, True), (64, False), (130, True)])
def test_layernorm_head(num_seqs, norm_bias):
    """The head of the families whose blocks use LayerNorms: a LayerNorm, with and without a bias, on rows with a
    mean; both GEMM paths of the vocabulary projection."""
    shape = dataclasses.replace(synth.TINY, norm_kind="layer")
    _head_case(shape, num_seqs, seed=40 + num_seqs, head_std=0.06, norm_bias=norm_bias)


def test_each_head_serves_its_own_norm_kind():
    st = _head_stage(synth.TINY, 4, 4, 0)
    ends = synth.draw_ends_weights(synth.TINY, seed=0, device="cuda:0")
    hidden = synth.draw_hidden(synth.TINY, 4, seed=0, device="cuda:0")
    with pytest.raises(StageError) as ei:                     # a bias asks for the LayerNorm head
        st.head(hidden, [1] * 4, ends["final_norm"], ends["lm_head"], final_norm_bias=ends["final_norm"])
    assert ei.value.code == -2
    st.close()
    layer = dataclasses.replace(synth.TINY, norm_kind="layer")
    st = _head_stage(layer, 4, 4, 0)
    import ctypes
    tokens = torch.empty(4, dtype=torch.int32, device="cuda:0")
    q = (ctypes.c_int32 * 4)(1, 1, 1, 1)
    rc = st._lib.stage_head(st._handle, None, 4, hidden.data_ptr(), 4, q, ends["final_norm"].data_ptr(),
                            ends["lm_head"].data_ptr(), layer.vocab, None, tokens.data_ptr())
    assert rc == -2
    st.close()


def test_head_llama2_7b_full_size():
    _head_case(synth.LLAMA2_7B_STAGE, 64, seed=0)


def test_head_qwen2_7b_full_size():
    _head_case(synth.QWEN2_7B_STAGE, 129, seed=0, sample=list(range(0, 129, 4)))


def test_head_llama3_70b_full_size():
    _head_case(synth.LLAMA3_70B_STAGE, 256, seed=0, sample=list(range(0, 256, 16)))


def test_head_llama3_70b_few_sequences():
    # at most 64 rows on a wide head (K = 8192): planned onto 64-row tiles, the logits written by the GEMM itself
    _head_case(synth.LLAMA3_70B_STAGE, 40, seed=2, sample=list(range(0, 40, 5)))


def test_equal_logits_resolve_to_the_smallest_index():
    shape = synth.TINY
    st = _head_stage(shape, 4, 4, 1)
    ends = synth.draw_ends_weights(shape, seed=1, device="cuda:0", head_std=0.05)
    hidden = synth.draw_hidden(shape, 4, seed=1, device="cuda:0")
    w = ends["lm_head"].clone()
    # rows 17, 400 and 999 become the same strong direction: identical arithmetic, identical logits
    direction = (hidden[2].float() * ends["final_norm"].float()).to(torch.bfloat16)
    for r in (999, 400, 17):
        w[r] = direction
    tokens, logits = st.head(hidden, [1, 1, 1, 1], ends["final_norm"], w)
    torch.cuda.synchronize()
    row = logits[2]
    assert row[17] == row[400] == row[999] and row[17] == row.max()
    assert int(tokens[2]) == 17
    st.close()


@pytest.mark.parametrize("shape,num_tokens", [(synth.TINY, 37), (synth.LLAMA2_7B_STAGE, 300)])
def test_embedding_gather_is_bit_exact(shape, num_tokens):
    st = _head_stage(shape, 1, num_tokens, 0)
    table = synth.draw_ends_weights(shape, seed=0, device="cuda:0")["embed"]
    ids = synth.draw_token_ids(shape, num_tokens, seed=5)
    ids[0], ids[1], ids[2], ids[3] = 0, shape.vocab - 1, ids[4], ids[4]      # both ends of the table, a repeat
    out = st.embed(table, ids)
    torch.cuda.synchronize()
    ref = oracle.embed_tokens(table.cpu(), ids)
    assert torch.equal(out.cpu().double(), ref)
    st.close()


def test_invalid_ends_calls_are_rejected():
    shape = synth.TINY
    st = _head_stage(shape, 4, 8, 0)
    ends = synth.draw_ends_weights(shape, seed=0, device="cuda:0")
    hidden = synth.draw_hidden(shape, 8, seed=0, device="cuda:0")
    out = torch.full((3, shape.hidden), 7.0, dtype=torch.bfloat16, device="cuda:0")
    for bad in ([0, shape.vocab, 1], [0, -1, 1]):
        with pytest.raises(StageError):
            st.embed(ends["embed"], bad, out=out)
    torch.cuda.synchronize()
    assert (out == 7.0).all(), "a rejected embed call wrote its output"
    with pytest.raises(StageError):
        st.head(hidden, [4, 3], ends["final_norm"], ends["lm_head"])            # rows do not add up
    with pytest.raises(StageError):
        st.head(hidden, [8, 0], ends["final_norm"], ends["lm_head"])            # an empty sequence
    with pytest.raises(StageError):
        st.head(hidden, [2] * 4 + [0], ends["final_norm"], ends["lm_head"])     # more sequences than max_seqs... and empty
    with pytest.raises(StageError):
        st.head(hidden, [4, 4], ends["final_norm"], ends["lm_head"][:504].contiguous())   # vocab != config
    st.close()
    no_head = H.make_stage(dataclasses.replace(shape, num_layers=1), synth.make_microbatch([1], [0], seed=0), 0,
                           fill_kv=False)
    with pytest.raises(StageError):
        no_head.head(hidden[:1].contiguous(), [1], ends["final_norm"], ends["lm_head"])
    no_head.close()


def test_token_loop_embed_stage_head_against_the_oracle_chain():
    """Token ids -> embedding -> the stage's layers -> output head, both sides from the same ids."""
    shape, mb = synth.workload("tiny", seed=0)
    seed = 0
    st = H.make_stage(shape, mb, seed, "fan_in", vocab_size=shape.vocab)
    ends = synth.draw_ends_weights(shape, seed=seed, device="cuda:0", head_std=0.06)
    ids = synth.draw_token_ids(shape, mb.num_tokens, seed=seed)
    hidden = st.embed(ends["embed"], ids)
    out = st.forward(hidden, mb.positions, mb.q_lens, mb.ctx_lens, mb.block_tables)
    tokens, logits = st.head(out, mb.q_lens, ends["final_norm"], ends["lm_head"])
    torch.cuda.synchronize()
    layers = draw_layers(shape, seed, "fan_in")
    from tests.helpers import oracle_pool
    pool = oracle_pool(shape, mb, seed)
    o_hidden = oracle.embed_tokens(ends["embed"].cpu(), ids)
    o_out, _ = oracle.stage_forward(oracle_shape(shape), layers, o_hidden, mb.positions, mb.q_lens, mb.ctx_lens,
                                    mb.block_tables, pool)
    o_logits = oracle.head_logits(o_out, mb.q_lens, ends["final_norm"].cpu(), ends["lm_head"].cpu(), shape.rms_eps)
    r = rel_l2(logits.cpu().double(), o_logits)
    print(f"  token loop: logits rel-L2 {r:.3e}", flush=True)
    assert r <= LOGIT_REL_L2_TOL
    _check_tokens(tokens, logits, o_logits, "token loop")
    st.close()
