"""Pins for the CPU oracle: brute force, invariants, closed forms, library cross-checks.

The paper prints no numbers for a stage's forward pass (it leaves the computation to its
engine runtime, section 3.2.2), so the oracle is pinned to the mathematics of the decoder
block instead of to printed values.
"""
import dataclasses
import math

import pytest
import torch

import oracle
from paper_2507_05043_amd import synth
from tests import brute_force
from tests.helpers import draw_layers, oracle_pool, oracle_shape, rel_l2

F64 = torch.float64


def small_shape(**kw):
    base = dict(name="pin", num_layers=2, hidden=24, num_q_heads=4, num_kv_heads=2, head_dim=8, ffn=40,
                rms_eps=1e-5, rope_theta=1e4, kv_block_size=16)
    base.update(kw)
    return synth.StageShape(**base)


def run_oracle(shape, mb, seed=0, weight_std="fan_in", layers=None, hidden=None, pool=None, taps=None,
               kv_store_dtype=None):
    layers = layers if layers is not None else draw_layers(shape, seed, weight_std)
    hidden = hidden if hidden is not None else synth.draw_hidden(shape, mb.num_tokens, seed=seed)
    pool = pool if pool is not None else oracle_pool(shape, mb, seed)
    out, slots = oracle.stage_forward(oracle_shape(shape), layers, hidden, mb.positions, mb.q_lens,
                                      mb.ctx_lens, mb.block_tables, pool, taps=taps, kv_store_dtype=kv_store_dtype)
    return out, slots, pool


# ---------------------------------------------------------------- brute force, whole block

@pytest.mark.parametrize("nq,nkv,bias,qk_norm", [(4, 2, False, False), (3, 3, False, False), (4, 1, False, False),
                                                 (4, 2, True, False), (4, 2, False, True), (4, 1, True, True)])
def test_whole_stage_matches_scalar_loops(nq, nkv, bias, qk_norm):
    shape = small_shape(num_q_heads=nq, num_kv_heads=nkv, hidden=12, ffn=20, head_dim=4, kv_block_size=4)
    q_lens, ctx_lens = [5, 1, 3], [0, 6, 2]
    mb = synth.make_microbatch(q_lens, ctx_lens, seed=3, block=4)
    layers = draw_layers(shape, 3, "fan_in")
    if bias:
        for l, w in enumerate(layers):
            w["bqkv"] = synth.draw_qkv_bias(shape, l, seed=3)
    if qk_norm:
        for l, w in enumerate(layers):
            w.update(synth.draw_qk_norm(shape, l, seed=3))
    hidden = synth.draw_hidden(shape, mb.num_tokens, seed=3)
    pool = oracle_pool(shape, mb, 3)
    pool0 = pool.clone()
    out, _, _ = run_oracle(shape, mb, layers=layers, hidden=hidden, pool=pool)
    # contiguous per-sequence caches for the scalar version, read from the pre-call pool
    got = []
    row0 = 0
    x_rows = hidden.double().tolist()
    for s, (q, c) in enumerate(zip(q_lens, ctx_lens)):
        rows = x_rows[row0:row0 + q]
        for l in range(shape.num_layers):
            w = {k: v.double().tolist() for k, v in layers[l].items()}
            ck, cv = [], []
            for j in range(c):
                blk = int(mb.block_tables[s][j // 4])
                ck.append(pool0[l, 0, blk, j % 4].tolist())
                cv.append(pool0[l, 1, blk, j % 4].tolist())
            pos = list(range(c, c + q))
            rows = brute_force.layer_one_sequence(shape, w, rows, pos, ck, cv)
        got.extend(rows)
        row0 += q
    got = torch.tensor(got, dtype=F64)
    assert torch.allclose(out, got, rtol=1e-10, atol=1e-11), float((out - got).abs().max())


def test_projection_bias_is_added_before_the_rotation():
    """q, k, v of a biased layer are the rotation of (unbiased pre-rotation values + bias); v is not rotated."""
    shape = small_shape(num_layers=1)
    mb = synth.make_microbatch([4, 1], [0, 5], seed=2, block=shape.kv_block_size)
    layers = draw_layers(shape, 2, "fan_in")
    hidden = synth.draw_hidden(shape, mb.num_tokens, seed=2)
    bias = synth.draw_qkv_bias(shape, 0, seed=2).double()
    nq, nkv, d = shape.num_q_heads, shape.num_kv_heads, shape.head_dim
    osh = oracle_shape(shape)
    taps0, taps1 = [], []
    run_oracle(shape, mb, layers=layers, hidden=hidden, taps=taps0)
    biased = [dict(layers[0], bqkv=bias)]
    run_oracle(shape, mb, layers=biased, hidden=hidden, taps=taps1)
    a = taps0[0]["a"]
    assert torch.equal(a, taps1[0]["a"])
    pre = a @ layers[0]["wqkv"].double().T + bias
    pos = torch.as_tensor(mb.positions)
    t = a.shape[0]
    q = oracle.rope_rotate(pre[:, : nq * d].reshape(t, nq, d), pos, osh.rope_theta)
    k = oracle.rope_rotate(pre[:, nq * d: (nq + nkv) * d].reshape(t, nkv, d), pos, osh.rope_theta)
    assert torch.allclose(taps1[0]["q"], q, rtol=1e-12, atol=1e-12)
    assert torch.allclose(taps1[0]["k"], k, rtol=1e-12, atol=1e-12)
    assert torch.allclose(taps1[0]["v"], pre[:, (nq + nkv) * d:].reshape(t, nkv, d), rtol=1e-12, atol=1e-12)
    assert not torch.allclose(taps1[0]["x"], taps0[0]["x"])
    # a zero bias changes nothing, bit for bit
    taps2 = []
    run_oracle(shape, mb, layers=[dict(layers[0], bqkv=torch.zeros_like(bias))], hidden=hidden, taps=taps2)
    assert torch.equal(taps2[0]["x"], taps0[0]["x"])


def test_head_norm_of_queries_and_keys():
    """The per-head norm sits between the bias and the rotation, acts on q and k heads only, makes the
    block blind to the scale of the q and k projection rows, and with unit gains leaves heads of rms 1."""
    shape = small_shape(num_layers=1, rms_eps=1e-12)
    mb = synth.make_microbatch([4, 1], [0, 5], seed=4, block=shape.kv_block_size)
    layers = draw_layers(shape, 4, "fan_in")
    hidden = synth.draw_hidden(shape, mb.num_tokens, seed=4)
    nq, nkv, d = shape.num_q_heads, shape.num_kv_heads, shape.head_dim
    gains = {k: v.double() for k, v in synth.draw_qk_norm(shape, 0, seed=4).items()}
    assert gains["qnorm"].shape == (d,) and not torch.equal(gains["qnorm"], gains["knorm"])
    plain, normed, unit = [], [], []
    run_oracle(shape, mb, seed=4, layers=layers, hidden=hidden, taps=plain)
    run_oracle(shape, mb, seed=4, layers=[dict(layers[0], **gains)], hidden=hidden, taps=normed)
    ones = {"qnorm": torch.ones(d, dtype=F64), "knorm": torch.ones(d, dtype=F64)}
    run_oracle(shape, mb, seed=4, layers=[dict(layers[0], **ones)], hidden=hidden, taps=unit)
    # values untouched; queries and keys = rotation of (pre-rotation head * gain / its rms), retyped here
    assert torch.equal(normed[0]["v"], plain[0]["v"])
    pre = plain[0]["a"] @ layers[0]["wqkv"].double().T
    pos = torch.as_tensor(mb.positions)
    t = pre.shape[0]
    for name, lo, n, gain in (("q", 0, nq, "qnorm"), ("k", nq * d, nkv, "knorm")):
        u = pre[:, lo: lo + n * d].reshape(t, n, d)
        u = u / u.pow(2).mean(dim=-1, keepdim=True).sqrt() * gains[gain]
        want = oracle.rope_rotate(u, pos, shape.rope_theta)
        assert torch.allclose(normed[0][name], want, rtol=1e-9, atol=1e-10), name
        # unit gains: every head has rms 1 (the rotation keeps lengths)
        rms = unit[0][name].pow(2).mean(dim=-1).sqrt()
        assert torch.allclose(rms, torch.ones_like(rms), rtol=1e-9)
    assert not torch.allclose(normed[0]["x"], plain[0]["x"], rtol=1e-3)
    # scaling the q rows by 7 and the k rows by 0.3 changes nothing once heads are normalised ...
    scaled = layers[0]["wqkv"].double().clone()
    scaled[: nq * d] *= 7.0
    scaled[nq * d: (nq + nkv) * d] *= 0.3
    again = []
    run_oracle(shape, mb, seed=4, layers=[dict(layers[0], wqkv=scaled, **gains)], hidden=hidden, taps=again)
    assert torch.allclose(again[0]["x"], normed[0]["x"], rtol=1e-9, atol=1e-10)
    # ... and does change the plain block
    again_plain = []
    run_oracle(shape, mb, seed=4, layers=[dict(layers[0], wqkv=scaled)], hidden=hidden, taps=again_plain)
    assert not torch.allclose(again_plain[0]["x"], plain[0]["x"], rtol=1e-3)


# ---------------------------------------------------------------- attention

def dense_attention_reference(q, keys, vals, ctx):
    """Full score matrix with -inf mask and fp64 softmax on contiguous K/V, per head, no GQA trick."""
    n, nq, d = q.shape
    g = nq // keys.shape[1]
    out = torch.zeros(n, nq, d, dtype=F64)
    for h in range(nq):
        for i in range(n):
            e = torch.full((keys.shape[0],), float("-inf"), dtype=F64)
            for j in range(ctx + i + 1):
                e[j] = torch.dot(q[i, h], keys[j, h // g]) / math.sqrt(d)
            w = torch.softmax(e, dim=0)
            for j in range(ctx + i + 1):
                out[i, h] += w[j] * vals[j, h // g]
    return out


def test_attention_matches_dense_brute_force():
    torch.manual_seed(1)
    for (n, ctx, nq, nkv, d) in [(1, 0, 2, 1, 4), (1, 9, 4, 2, 8), (6, 0, 4, 4, 8), (5, 7, 6, 2, 4)]:
        q = torch.randn(n, nq, d, dtype=F64)
        k = torch.randn(ctx + n, nkv, d, dtype=F64)
        v = torch.randn(ctx + n, nkv, d, dtype=F64)
        got = oracle.attention_rows(q, k, v, ctx)
        assert torch.allclose(got, dense_attention_reference(q, k, v, ctx), rtol=1e-12, atol=1e-13)


def test_attention_matches_library_sdpa():
    torch.manual_seed(2)
    n, ctx, nq, nkv, d = 7, 5, 6, 3, 16
    q = torch.randn(n, nq, d, dtype=F64)
    k = torch.randn(ctx + n, nkv, d, dtype=F64)
    v = torch.randn(ctx + n, nkv, d, dtype=F64)
    mask = torch.arange(ctx + n).view(1, -1) <= (ctx + torch.arange(n)).view(-1, 1)
    kk = k.repeat_interleave(nq // nkv, dim=1)
    vv = v.repeat_interleave(nq // nkv, dim=1)
    ref = torch.nn.functional.scaled_dot_product_attention(
        q.transpose(0, 1)[None], kk.transpose(0, 1)[None], vv.transpose(0, 1)[None], attn_mask=mask)
    assert torch.allclose(oracle.attention_rows(q, k, v, ctx), ref[0].transpose(0, 1), rtol=1e-12, atol=1e-13)


def test_softmax_degenerate_cases():
    torch.manual_seed(3)
    n, ctx, nq, nkv, d = 3, 4, 2, 1, 8
    q = torch.randn(n, nq, d, dtype=F64)
    v = torch.randn(ctx + n, nkv, d, dtype=F64)
    # identical keys -> uniform weights -> running mean of the visible values
    k = torch.randn(1, nkv, d, dtype=F64).expand(ctx + n, nkv, d).contiguous()
    o = oracle.attention_rows(q, k, v, ctx)
    for i in range(n):
        assert torch.allclose(o[i, 0], v[: ctx + i + 1, 0].mean(dim=0), rtol=1e-12, atol=1e-13)
    # identical values -> that value, whatever the scores
    k = torch.randn(ctx + n, nkv, d, dtype=F64)
    v1 = torch.randn(1, nkv, d, dtype=F64).expand(ctx + n, nkv, d).contiguous()
    o = oracle.attention_rows(q, k, v1, ctx)
    assert torch.allclose(o, v1[0, 0].expand_as(o), rtol=1e-12, atol=1e-13)
    # one visible key -> its value
    o = oracle.attention_rows(q[:1], k[:1], v[:1], 0)
    assert torch.allclose(o[0, 1], v[0, 0], rtol=0, atol=1e-15)
    # causal: changing a future key/value does not change an earlier row
    k2, v2 = k.clone(), v.clone()
    k2[-1] += 5.0
    v2[-1] -= 3.0
    o1 = oracle.attention_rows(q, k, v, ctx)
    o2 = oracle.attention_rows(q, k2, v2, ctx)
    assert torch.equal(o1[:-1], o2[:-1]) and not torch.allclose(o1[-1], o2[-1])
    # the 1/sqrt(d) scale: one hot query against two keys gives softmax of (k/sqrt(d))
    qh = torch.zeros(1, 1, 4, dtype=F64)
    qh[0, 0, 0] = 2.0
    kk = torch.zeros(2, 1, 4, dtype=F64)
    kk[1, 0, 0] = 3.0
    vv = torch.tensor([[[1.0, 0, 0, 0]], [[0, 1.0, 0, 0]]], dtype=F64)
    o = oracle.attention_rows(qh, kk, vv, 1)
    p1 = math.exp(3.0) / (1 + math.exp(3.0))       # 2*3/sqrt(4) = 3
    assert torch.allclose(o[0, 0, :2], torch.tensor([1 - p1, p1], dtype=F64), rtol=1e-13, atol=0)


def test_gqa_equals_mha_with_replicated_kv_heads():
    shape = small_shape(num_layers=1)
    g = shape.num_q_heads // shape.num_kv_heads
    mb = synth.make_microbatch([4, 1], [0, 5], seed=1)
    layers = draw_layers(shape, 1, "fan_in")
    out, _, pool = run_oracle(shape, mb, seed=1, layers=layers)
    d, nq, nkv = shape.head_dim, shape.num_q_heads, shape.num_kv_heads
    mha = synth.StageShape("mha", 1, shape.hidden, nq, nq, d, shape.ffn)
    w = dict(layers[0])
    wq, wk, wv = w["wqkv"][: nq * d], w["wqkv"][nq * d:(nq + nkv) * d], w["wqkv"][(nq + nkv) * d:]
    rep = lambda m: m.view(nkv, d, -1).repeat_interleave(g, dim=0).reshape(nq * d, -1)
    w["wqkv"] = torch.cat([wq, rep(wk), rep(wv)], dim=0)
    pool_g = oracle_pool(shape, mb, 1)
    pool_m = pool_g.repeat_interleave(g, dim=4)
    out_m, _ = oracle.stage_forward(oracle_shape(mha), [w], synth.draw_hidden(shape, mb.num_tokens, seed=1),
                                    mb.positions, mb.q_lens, mb.ctx_lens, mb.block_tables, pool_m)
    assert torch.allclose(out, out_m, rtol=1e-12, atol=1e-13)
    # and the mapping is h // g, not h % nkv: replicating the KV heads the other way round (head h takes KV head
    # h % nkv) is a different block
    assert g > 1
    til = lambda m: m.view(nkv, d, -1).repeat(g, 1, 1).reshape(nq * d, -1)
    w_mod = dict(w, wqkv=torch.cat([wq, til(wk), til(wv)], dim=0))
    pool_mod = pool_g.repeat(1, 1, 1, 1, g, 1)
    out_mod, _ = oracle.stage_forward(oracle_shape(mha), [w_mod], synth.draw_hidden(shape, mb.num_tokens, seed=1),
                                      mb.positions, mb.q_lens, mb.ctx_lens, mb.block_tables, pool_mod)
    assert not torch.allclose(out, out_mod, rtol=1e-3, atol=1e-4)


# ---------------------------------------------------------------- paging, chunking, batching

def test_paged_equals_contiguous_bitwise():
    shape = small_shape()
    q_lens, ctx_lens = [7, 1, 1, 20], [0, 33, 5, 11]
    mb_p = synth.make_microbatch(q_lens, ctx_lens, seed=5, paging="permuted")
    mb_c = synth.make_microbatch(q_lens, ctx_lens, seed=5, paging="identity")
    assert not torch.equal(mb_p.block_tables, mb_c.block_tables)
    layers = draw_layers(shape, 5, "fan_in")
    hidden = synth.draw_hidden(shape, mb_p.num_tokens, seed=5)
    # same logical cache contents in both layouts
    torch.manual_seed(0)
    pool_p = oracle.new_pool(oracle_shape(shape), mb_p.num_kv_blocks)
    pool_c = oracle.new_pool(oracle_shape(shape), mb_c.num_kv_blocks)
    for s, c in enumerate(ctx_lens):
        for j in range(c):
            val = torch.randn(shape.num_layers, 2, shape.num_kv_heads, shape.head_dim, dtype=F64)
            pool_p[:, :, int(mb_p.block_tables[s][j // 16]), j % 16] = val
            pool_c[:, :, int(mb_c.block_tables[s][j // 16]), j % 16] = val
    out_p, slots_p, _ = run_oracle(shape, mb_p, layers=layers, hidden=hidden, pool=pool_p)
    out_c, slots_c, _ = run_oracle(shape, mb_c, layers=layers, hidden=hidden, pool=pool_c)
    assert torch.equal(out_p, out_c)
    assert slots_p != slots_c
    # logical cache contents equal after the call
    for s, (q, c) in enumerate(zip(q_lens, ctx_lens)):
        for j in range(c + q):
            a = pool_p[:, :, int(mb_p.block_tables[s][j // 16]), j % 16]
            b = pool_c[:, :, int(mb_c.block_tables[s][j // 16]), j % 16]
            assert torch.equal(a, b)


@pytest.mark.parametrize("chunks", [[5, 11, 16], [31, 1], [1] * 6 + [26]])
def test_chunked_prefill_equals_unsplit(chunks):
    shape = small_shape()
    n = sum(chunks)
    layers = draw_layers(shape, 7, "fan_in")
    hidden = synth.draw_hidden(shape, n, seed=7)
    mb = synth.make_microbatch([n], [0], seed=7)
    full, _, pool_full = run_oracle(shape, mb, layers=layers, hidden=hidden)
    pool = oracle.new_pool(oracle_shape(shape), mb.num_kv_blocks)
    outs, done = [], 0
    for c in chunks:
        pos = torch.arange(done, done + c, dtype=torch.int32)
        o, _ = oracle.stage_forward(oracle_shape(shape), layers, hidden[done:done + c], pos, [c], [done],
                                    mb.block_tables, pool)
        outs.append(o)
        done += c
    got = torch.cat(outs)
    assert torch.allclose(got, full, rtol=1e-11, atol=1e-12)
    used = synth.valid_slot_mask(mb, 16, include_new=True)
    assert torch.allclose(pool[:, :, used], pool_full[:, :, used], rtol=1e-11, atol=1e-12)
    assert torch.isnan(pool[:, :, ~used]).all()


def test_decode_equals_last_prefill_row():
    shape = small_shape()
    n = 19
    layers = draw_layers(shape, 8, "fan_in")
    hidden = synth.draw_hidden(shape, n, seed=8)
    mb = synth.make_microbatch([n], [0], seed=8)
    full, _, _ = run_oracle(shape, mb, layers=layers, hidden=hidden)
    pool = oracle.new_pool(oracle_shape(shape), mb.num_kv_blocks)
    osh = oracle_shape(shape)
    oracle.stage_forward(osh, layers, hidden[: n - 1], torch.arange(n - 1), [n - 1], [0], mb.block_tables, pool)
    last, _ = oracle.stage_forward(osh, layers, hidden[n - 1:], torch.tensor([n - 1]), [1], [n - 1],
                                   mb.block_tables, pool)
    assert torch.allclose(last[0], full[-1], rtol=1e-11, atol=1e-12)


def test_rows_independent_of_batch_composition_and_order():
    shape = small_shape()
    q_lens, ctx_lens = [6, 1, 1, 9], [4, 17, 0, 0]
    mb = synth.make_microbatch(q_lens, ctx_lens, seed=9)
    layers = draw_layers(shape, 9, "fan_in")
    hidden = synth.draw_hidden(shape, mb.num_tokens, seed=9)
    pool = oracle_pool(shape, mb, 9)
    out, _, _ = run_oracle(shape, mb, layers=layers, hidden=hidden, pool=pool.clone())
    # reversed sequence order, same block tables
    order = [3, 2, 1, 0]
    cu = [0, 6, 7, 8, 17]
    rows = torch.cat([torch.arange(cu[s], cu[s + 1]) for s in order])
    mb_r = synth.MicroBatch([q_lens[s] for s in order], [ctx_lens[s] for s in order],
                            mb.block_tables[order], mb.positions[rows], mb.num_kv_blocks)
    out_r, _, _ = run_oracle(shape, mb_r, layers=layers, hidden=hidden[rows], pool=pool.clone())
    assert torch.allclose(out_r, out[rows], rtol=1e-12, atol=1e-13)
    # one sequence alone
    s = 1
    mb_1 = synth.MicroBatch([q_lens[s]], [ctx_lens[s]], mb.block_tables[s:s + 1],
                            mb.positions[cu[s]:cu[s + 1]], mb.num_kv_blocks)
    out_1, _, _ = run_oracle(shape, mb_1, layers=layers, hidden=hidden[cu[s]:cu[s + 1]], pool=pool.clone())
    assert torch.allclose(out_1, out[cu[s]:cu[s + 1]], rtol=1e-12, atol=1e-13)


# ---------------------------------------------------------------- partial rotary

@pytest.mark.parametrize("nq,nkv,rd", [(4, 2, 4), (3, 3, 2), (4, 1, 6)])
def test_partial_rotary_matches_scalar_loops(nq, nkv, rd):
    shape = small_shape(num_q_heads=nq, num_kv_heads=nkv, hidden=12, ffn=20, head_dim=8, kv_block_size=4, rotary_dim=rd)
    q_lens, ctx_lens = [5, 1, 3], [0, 6, 2]
    mb = synth.make_microbatch(q_lens, ctx_lens, seed=3, block=4)
    layers = draw_layers(shape, 3, "fan_in")
    hidden = synth.draw_hidden(shape, mb.num_tokens, seed=3)
    pool = oracle_pool(shape, mb, 3)
    pool0 = pool.clone()
    out, _, _ = run_oracle(shape, mb, layers=layers, hidden=hidden, pool=pool)
    got, row0 = [], 0
    x_rows = hidden.double().tolist()
    for s, (q, c) in enumerate(zip(q_lens, ctx_lens)):
        rows = x_rows[row0:row0 + q]
        for l in range(shape.num_layers):
            w = {k: v.double().tolist() for k, v in layers[l].items()}
            ck, cv = [], []
            for j in range(c):
                blk = int(mb.block_tables[s][j // 4])
                ck.append(pool0[l, 0, blk, j % 4].tolist())
                cv.append(pool0[l, 1, blk, j % 4].tolist())
            rows = brute_force.layer_one_sequence(shape, w, rows, list(range(c, c + q)), ck, cv)
        got.extend(rows)
        row0 += q
    got = torch.tensor(got, dtype=F64)
    assert torch.allclose(out, got, rtol=1e-10, atol=1e-11), float((out - got).abs().max())


def test_partial_rotary_rotates_a_head_of_its_own_size_and_passes_the_rest():
    import dataclasses
    shape = small_shape(num_layers=1, head_dim=16)
    mb = synth.make_microbatch([6, 1], [0, 9], seed=6, block=shape.kv_block_size)
    layers = draw_layers(shape, 6, "fan_in")
    hidden = synth.draw_hidden(shape, mb.num_tokens, seed=6)
    full, whole, part = [], [], []
    run_oracle(shape, mb, seed=6, layers=layers, hidden=hidden, taps=full)
    run_oracle(dataclasses.replace(shape, rotary_dim=16), mb, seed=6, layers=layers, hidden=hidden, taps=whole)
    run_oracle(dataclasses.replace(shape, rotary_dim=8), mb, seed=6, layers=layers, hidden=hidden, taps=part)
    # rotary_dim = head_dim is the default, bit for bit
    assert torch.equal(whole[0]["x"], full[0]["x"]) and torch.equal(whole[0]["q"], full[0]["q"])
    nq, nkv, d = shape.num_q_heads, shape.num_kv_heads, shape.head_dim
    pre = part[0]["a"] @ layers[0]["wqkv"].double().T
    pos = torch.as_tensor(mb.positions)
    t = pre.shape[0]
    for name, lo, n in (("q", 0, nq), ("k", nq * d, nkv)):
        u = pre[:, lo: lo + n * d].reshape(t, n, d)
        got = part[0][name]
        assert torch.equal(got[..., 8:], u[..., 8:])                                    # the rest passes through
        assert torch.equal(got[..., :8], oracle.rope_rotate(u[..., :8].contiguous(), pos, shape.rope_theta))
        # the angle of pair (i, i + 4) is pos * theta**(-2i/8): element 1 of a unit vector at position 3
        ang = 3 * shape.rope_theta ** (-2.0 * 1 / 8)
        e = torch.zeros(1, 1, d, dtype=F64); e[0, 0, 1] = 1.0
        z = oracle.rope_rotate(e, torch.tensor([3]), shape.rope_theta, 8)[0, 0]
        assert math.isclose(float(z[1]), math.cos(ang), rel_tol=1e-14) and math.isclose(float(z[5]), math.sin(ang), rel_tol=1e-14)
        assert float(z.abs().sum()) == pytest.approx(abs(math.cos(ang)) + abs(math.sin(ang)), rel=1e-14)
    assert torch.equal(part[0]["v"], full[0]["v"])
    assert not torch.allclose(part[0]["x"], full[0]["x"], rtol=1e-3)


# ---------------------------------------------------------------- rotation of neighbouring elements

@pytest.mark.parametrize("nq,nkv,rd", [(4, 2, 0), (4, 2, 4), (3, 3, 6)])
def test_neighbour_pairing_matches_scalar_loops(nq, nkv, rd):
    """Whole heads and partial rotary (the GLM / ChatGLM block), two layers, prefill with and without prefix, decode."""
    shape = small_shape(num_q_heads=nq, num_kv_heads=nkv, hidden=12, ffn=20, head_dim=8, kv_block_size=4, rotary_dim=rd,
                        rope_interleaved=True)
    q_lens, ctx_lens = [5, 1, 3], [0, 6, 2]
    mb = synth.make_microbatch(q_lens, ctx_lens, seed=3, block=4)
    layers = draw_layers(shape, 3, "fan_in")
    hidden = synth.draw_hidden(shape, mb.num_tokens, seed=3)
    pool = oracle_pool(shape, mb, 3)
    pool0 = pool.clone()
    out, _, _ = run_oracle(shape, mb, layers=layers, hidden=hidden, pool=pool)
    got, row0 = [], 0
    x_rows = hidden.double().tolist()
    for s, (q, c) in enumerate(zip(q_lens, ctx_lens)):
        rows = x_rows[row0:row0 + q]
        for l in range(shape.num_layers):
            w = {k: v.double().tolist() for k, v in layers[l].items()}
            ck, cv = [], []
            for j in range(c):
                blk = int(mb.block_tables[s][j // 4])
                ck.append(pool0[l, 0, blk, j % 4].tolist())
                cv.append(pool0[l, 1, blk, j % 4].tolist())
            rows = brute_force.layer_one_sequence(shape, w, rows, list(range(c, c + q)), ck, cv)
        got.extend(rows)
        row0 += q
    got = torch.tensor(got, dtype=F64)
    assert torch.allclose(out, got, rtol=1e-10, atol=1e-11), float((out - got).abs().max())
    import dataclasses
    other, _, _ = run_oracle(dataclasses.replace(shape, rope_interleaved=False), mb, layers=layers, hidden=hidden,
                             pool=oracle_pool(shape, mb, 3))
    assert not torch.allclose(out, other, rtol=1e-3)             # the pairing matters


def test_neighbour_pairing_is_the_half_split_rotation_of_the_regrouped_head():
    """Moving a head's even elements to the front and its odd elements to the back turns neighbour pairs into
    half-split pairs with the same index, hence the same angles: rotating the regrouped head the half-split way
    and moving the elements back is the neighbour rotation (bit for bit: the same products and sums).  Also with
    a partial rotary size, and one literal angle."""
    gen = torch.Generator().manual_seed(5)
    u = torch.randn(7, 3, 16, generator=gen, dtype=F64)
    pos = torch.tensor([0, 1, 2, 9, 100, 1000, 4095])
    for rd in (0, 8):
        n = rd or 16
        got = oracle.rope_rotate(u, pos, 1e4, rd, True)
        head = u[..., :n]
        regrouped = torch.cat([head[..., 0::2], head[..., 1::2]], dim=-1)
        rot = oracle.rope_rotate(regrouped, pos, 1e4)
        back = torch.empty_like(head)
        back[..., 0::2] = rot[..., : n // 2]
        back[..., 1::2] = rot[..., n // 2:]
        assert torch.equal(got[..., :n], back)
        assert torch.equal(got[..., n:], u[..., n:])
        norm = lambda x: x.pow(2).sum(-1)
        assert torch.allclose(norm(got), norm(u), rtol=1e-13)    # a rotation keeps the length
    # pair (2, 3) of an 8-element rotary part turns by pos * theta**(-2*1/8): unit vector along element 2 at position 3
    ang = 3 * 1e4 ** (-2.0 * 1 / 8)
    e = torch.zeros(1, 1, 16, dtype=F64); e[0, 0, 2] = 1.0
    z = oracle.rope_rotate(e, torch.tensor([3]), 1e4, 8, True)[0, 0]
    assert math.isclose(float(z[2]), math.cos(ang), rel_tol=1e-14) and math.isclose(float(z[3]), math.sin(ang), rel_tol=1e-14)
    assert float(z.abs().sum()) == pytest.approx(abs(math.cos(ang)) + abs(math.sin(ang)), rel=1e-14)


# ---------------------------------------------------------------- attention with linear biases

def _with_alibi(layers, slopes):
    return [dict(w, alibi=slopes) for w in layers]


def test_linear_bias_slopes_are_the_published_sequences():
    assert synth.alibi_slopes(8).tolist() == [2.0 ** -(i + 1) for i in range(8)]
    s12 = synth.alibi_slopes(12)
    assert s12[:8].tolist() == [2.0 ** -(i + 1) for i in range(8)]
    assert torch.allclose(s12[8:].double(), torch.tensor([2.0 ** -0.5, 2.0 ** -1.5, 2.0 ** -2.5, 2.0 ** -3.5], dtype=F64), rtol=1e-7)
    assert synth.alibi_slopes(40).shape == (40,) and float(synth.alibi_slopes(40)[32]) == pytest.approx(2.0 ** -0.125, rel=1e-7)


@pytest.mark.parametrize("nq,nkv", [(4, 2), (3, 3), (4, 1)])
def test_linear_biases_match_scalar_loops(nq, nkv):
    shape = small_shape(num_q_heads=nq, num_kv_heads=nkv, hidden=12, ffn=20, head_dim=8, kv_block_size=4)
    q_lens, ctx_lens = [5, 1, 3], [0, 6, 2]
    mb = synth.make_microbatch(q_lens, ctx_lens, seed=3, block=4)
    slopes = synth.alibi_slopes(nq)
    layers = _with_alibi(draw_layers(shape, 3, "fan_in"), slopes)
    hidden = synth.draw_hidden(shape, mb.num_tokens, seed=3)
    pool = oracle_pool(shape, mb, 3)
    pool0 = pool.clone()
    out, _, _ = run_oracle(shape, mb, layers=layers, hidden=hidden, pool=pool)
    got, row0 = [], 0
    x_rows = hidden.double().tolist()
    for s, (q, c) in enumerate(zip(q_lens, ctx_lens)):
        rows = x_rows[row0:row0 + q]
        for l in range(shape.num_layers):
            w = {k: v.double().tolist() for k, v in layers[l].items()}
            ck, cv = [], []
            for j in range(c):
                blk = int(mb.block_tables[s][j // 4])
                ck.append(pool0[l, 0, blk, j % 4].tolist())
                cv.append(pool0[l, 1, blk, j % 4].tolist())
            rows = brute_force.layer_one_sequence(shape, w, rows, list(range(c, c + q)), ck, cv)
        got.extend(rows)
        row0 += q
    got = torch.tensor(got, dtype=F64)
    assert torch.allclose(out, got, rtol=1e-10, atol=1e-11), float((out - got).abs().max())
    plain, _, _ = run_oracle(shape, mb, layers=draw_layers(shape, 3, "fan_in"), hidden=hidden, pool=oracle_pool(shape, mb, 3))
    assert not torch.allclose(out, plain, rtol=1e-3)


def test_zero_slopes_are_the_rotation_at_position_zero():
    """With all slopes zero the scores carry no bias, and a rotary embedding at position 0 rotates by angle 0: the two
    stages compute the same thing, bit for bit."""
    shape = small_shape()
    mb = synth.make_microbatch([9, 1, 1, 20], [3, 33, 0, 11], seed=31)
    layers = draw_layers(shape, 31, "fan_in")
    zeros = dataclasses_replace_positions(mb, 0)
    a, _, pa = run_oracle(shape, zeros, seed=31, layers=layers)
    b, _, pb = run_oracle(shape, mb, seed=31, layers=_with_alibi(layers, torch.zeros(shape.num_q_heads)))
    assert torch.equal(a, b)
    assert torch.equal(pa.nan_to_num(nan=-7.0), pb.nan_to_num(nan=-7.0))


def dataclasses_replace_positions(mb, value):
    import dataclasses
    return dataclasses.replace(mb, positions=torch.full_like(torch.as_tensor(mb.positions), value))


def test_zero_queries_give_geometric_weights():
    """Queries of zero leave only the biases: the weight of key j for the query at index i is r^(i-j) / sum_k r^(i-k)
    with r = exp(-slope) - a closed form, evaluated here with Python floats."""
    gen = torch.Generator().manual_seed(8)
    ctx, n, nq, nkv, d = 5, 3, 4, 2, 4
    keys = torch.randn(ctx + n, nkv, d, generator=gen, dtype=F64)
    vals = torch.randn(ctx + n, nkv, d, generator=gen, dtype=F64)
    slopes = torch.tensor([0.5, 0.25, 0.0625, 1.5], dtype=F64)
    out = oracle.attention_rows(torch.zeros(n, nq, d, dtype=F64), keys, vals, ctx, slopes)
    for row in range(n):
        i = ctx + row
        for h in range(nq):
            r = math.exp(-float(slopes[h]))
            wts = [r ** (i - j) for j in range(i + 1)]
            z = sum(wts)
            for c in range(d):
                want = sum(wts[j] / z * float(vals[j, h // 2, c]) for j in range(i + 1))
                assert math.isclose(float(out[row, h, c]), want, rel_tol=1e-12, abs_tol=1e-14)
    # steeper slopes look at nearer keys: with a huge slope only the query's own key is left
    own = oracle.attention_rows(torch.zeros(n, nq, d, dtype=F64), keys, vals, ctx, torch.full((nq,), 800.0, dtype=F64))
    for row in range(n):
        assert torch.equal(own[row, 0], vals[ctx + row, 0])


def test_linear_biases_keep_the_chunking_and_decode_identities():
    """A chunk split in two, and a last prefill row against a decode row, under linear biases: distances are counted
    from the row's own logical index, whatever the chunking."""
    shape = small_shape()
    slopes = synth.alibi_slopes(shape.num_q_heads)
    layers = _with_alibi(draw_layers(shape, 12, "fan_in"), slopes)
    whole = synth.make_microbatch([11], [5], seed=12)
    hidden = synth.draw_hidden(shape, 11, seed=12)
    pool = oracle_pool(shape, whole, 12)
    want, _, pool_w = run_oracle(shape, whole, layers=layers, hidden=hidden, pool=pool.clone())
    first = synth.MicroBatch([7], [5], whole.block_tables, whole.positions[:7], whole.num_kv_blocks)
    second = synth.MicroBatch([4], [12], whole.block_tables, whole.positions[7:], whole.num_kv_blocks)
    pool2 = pool.clone()
    a, _, pool2 = run_oracle(shape, first, layers=layers, hidden=hidden[:7], pool=pool2)
    b, _, pool2 = run_oracle(shape, second, layers=layers, hidden=hidden[7:], pool=pool2)
    assert torch.allclose(torch.cat([a, b]), want, rtol=1e-11, atol=1e-12)
    # the last row alone, as a decode token over the cache the first ten rows left
    ten = synth.MicroBatch([10], [5], whole.block_tables, whole.positions[:10], whole.num_kv_blocks)
    pool3 = pool.clone()
    _, _, pool3 = run_oracle(shape, ten, layers=layers, hidden=hidden[:10], pool=pool3)
    one = synth.MicroBatch([1], [15], whole.block_tables, whole.positions[10:], whole.num_kv_blocks)
    last, _, _ = run_oracle(shape, one, layers=layers, hidden=hidden[10:], pool=pool3)
    assert torch.allclose(last[0], want[10], rtol=1e-11, atol=1e-12)


# ---------------------------------------------------------------- the cache as a store of a narrower type

# ---------------------------------------------------------------- LayerNorm, ungated GELU MLP, parallel branches

def _scalar_loops(shape, mb, layers, hidden, pool0, q_lens, ctx_lens, blk=4):
    got, row0 = [], 0
    x_rows = hidden.double().tolist()
    for s, (q, c) in enumerate(zip(q_lens, ctx_lens)):
        rows = x_rows[row0:row0 + q]
        for l in range(shape.num_layers):
            w = {k: v.double().tolist() for k, v in layers[l].items()}
            ck, cv = [], []
            for j in range(c):
                b = int(mb.block_tables[s][j // blk])
                ck.append(pool0[l, 0, b, j % blk].tolist())
                cv.append(pool0[l, 1, b, j % blk].tolist())
            rows = brute_force.layer_one_sequence(shape, w, rows, list(range(c, c + q)), ck, cv)
        got.extend(rows)
        row0 += q
    return torch.tensor(got, dtype=F64)


BLOCK_KINDS = [
    dict(norm_kind="layer"),                                                                 # LayerNorm, rest default
    dict(mlp_kind="gelu_tanh"),
    dict(mlp_kind="gelu_erf", biases=True),
    dict(parallel_block=True),
    dict(parallel_block=True, shared=True),
    dict(norm_kind="layer", mlp_kind="gelu_tanh", biases=True, alibi_zero=True),             # the GPT-2 block
    dict(norm_kind="layer", mlp_kind="gelu_erf", parallel_block=True, biases=True, alibi=True),   # Falcon, two norms
    dict(norm_kind="layer", mlp_kind="gelu_erf", parallel_block=True, shared=True),          # Falcon, one norm
    dict(norm_kind="layer", parallel_block=True, shared=True, rope_interleaved=True),        # Cohere
]


def _block_layers(shape, seed, kind):
    layers = draw_layers(shape, seed, "fan_in", block_biases=kind.get("biases", False), shared_norm=kind.get("shared", False))
    if kind.get("alibi") or kind.get("alibi_zero"):
        slopes = synth.alibi_slopes(shape.num_q_heads)
        layers = _with_alibi(layers, slopes * 0 if kind.get("alibi_zero") else slopes)
    return layers


def _block_shape(kind, **kw):
    keys = ("norm_kind", "mlp_kind", "parallel_block", "rope_interleaved")
    return small_shape(**{k: kind[k] for k in keys if k in kind}, **kw)


@pytest.mark.parametrize("kind", BLOCK_KINDS, ids=lambda k: "-".join(f"{a}={b}" for a, b in k.items()))
def test_block_kinds_match_scalar_loops(kind):
    shape = _block_shape(kind, num_q_heads=4, num_kv_heads=2, hidden=12, ffn=20, head_dim=8, kv_block_size=4)
    q_lens, ctx_lens = [5, 1, 3], [0, 6, 2]
    mb = synth.make_microbatch(q_lens, ctx_lens, seed=3, block=4)
    layers = _block_layers(shape, 3, kind)
    hidden = synth.draw_hidden(shape, mb.num_tokens, seed=3) + 0.5           # rows with a mean: LayerNorm removes it
    pool = oracle_pool(shape, mb, 3)
    pool0 = pool.clone()
    out, _, _ = run_oracle(shape, mb, layers=layers, hidden=hidden, pool=pool)
    got = _scalar_loops(shape, mb, layers, hidden, pool0, q_lens, ctx_lens)
    assert torch.allclose(out, got, rtol=1e-9, atol=1e-10), float((out - got).abs().max())
    base = small_shape(num_q_heads=4, num_kv_heads=2, hidden=12, ffn=20, head_dim=8, kv_block_size=4)
    plain, _, _ = run_oracle(base, mb, layers=draw_layers(base, 3, "fan_in"), hidden=hidden, pool=oracle_pool(base, mb, 3))
    assert not torch.allclose(out, plain, rtol=1e-3)


def test_layernorm_against_the_library_and_closed_forms():
    g = torch.Generator().manual_seed(5)
    x = torch.randn(7, 24, dtype=F64, generator=g) * 3 + 2
    gain = torch.randn(24, dtype=F64, generator=g)
    bias = torch.randn(24, dtype=F64, generator=g)
    want = torch.nn.functional.layer_norm(x, (24,), gain, bias, 1e-5)
    assert torch.allclose(oracle.layernorm(x, gain, bias, 1e-5), want, rtol=1e-12, atol=1e-13)
    want = torch.nn.functional.layer_norm(x, (24,), gain, None, 1e-5)
    assert torch.allclose(oracle.layernorm(x, gain, None, 1e-5), want, rtol=1e-12, atol=1e-13)
    y = oracle.layernorm(x, torch.ones(24, dtype=F64), None, 0.0)            # zero mean, unit variance
    assert y.mean(dim=-1).abs().max() < 1e-14
    assert ((y * y).mean(dim=-1) - 1).abs().max() < 1e-13
    shifted = oracle.layernorm(x + 10.0, gain, bias, 1e-5)                    # a shift of the row changes nothing
    assert torch.allclose(shifted, oracle.layernorm(x, gain, bias, 1e-5), rtol=1e-11, atol=1e-12)
    scaled = oracle.layernorm(x * 4.0, gain, bias, 0.0)                       # nor does its scale, without epsilon
    assert torch.allclose(scaled, oracle.layernorm(x, gain, bias, 0.0), rtol=1e-12, atol=1e-12)
    const = torch.full((2, 24), 3.25, dtype=F64)                              # no deviations: the bias alone
    assert torch.equal(oracle.layernorm(const, gain, bias, 1e-5), bias.expand(2, 24))
    # epsilon sits under the root, next to the variance: variance 1 (values +-1) divides by sqrt(1 + eps)
    pm = torch.tensor([[1.0, -1.0] * 12], dtype=F64)
    assert torch.allclose(oracle.layernorm(pm, torch.ones(24, dtype=F64), None, 3.0), pm / 2.0, rtol=1e-15)
    # and it differs from the RMSNorm exactly by the removed mean
    assert torch.allclose(oracle.layernorm(x, gain, None, 1e-5),
                          oracle.rmsnorm(x - x.mean(dim=-1, keepdim=True), gain, 1e-5), rtol=1e-12, atol=1e-13)


def test_gelu_forms_against_the_library_and_literal_values():
    z = torch.linspace(-6, 6, 241, dtype=F64)
    assert torch.allclose(oracle.gelu(z, "gelu_erf"), torch.nn.functional.gelu(z), rtol=1e-12, atol=1e-14)
    assert torch.allclose(oracle.gelu(z, "gelu_tanh"), torch.nn.functional.gelu(z, approximate="tanh"), rtol=1e-12, atol=1e-14)
    one = torch.tensor([1.0, -1.0, 0.0, 0.5], dtype=F64)
    # Phi(1) = 0.841344746068543, Phi(0.5) = 0.691462461274013 (normal distribution tables)
    assert torch.allclose(oracle.gelu(one, "gelu_erf"),
                          torch.tensor([0.841344746068543, -0.158655253931457, 0.0, 0.3457312306370065], dtype=F64), rtol=1e-13)
    # tanh form at 1: 0.5 (1 + tanh(0.7978845608 * 1.044715)) = 0.5 (1 + tanh(0.8335619..)) = 0.841191990608
    t1 = 0.5 * (1 + math.tanh(math.sqrt(2 / math.pi) * 1.044715))
    assert abs(t1 - 0.841191990608) < 1e-11
    assert torch.allclose(oracle.gelu(one[:1], "gelu_tanh"), torch.tensor([t1], dtype=F64), rtol=1e-14)
    big = torch.tensor([30.0, -30.0], dtype=F64)
    for form in ("gelu_erf", "gelu_tanh"):
        assert torch.equal(oracle.gelu(big, form), torch.tensor([30.0, -0.0], dtype=F64)) or \
            torch.equal(oracle.gelu(big, form).abs(), torch.tensor([30.0, 0.0], dtype=F64))
        assert float((oracle.gelu(z, form) - oracle.gelu(z, "gelu_erf")).abs().max()) < 5e-4   # the two forms are close
        # gelu(z) - gelu(-z) = z for both forms (Phi(z) + Phi(-z) = 1; tanh is odd)
        assert torch.allclose(oracle.gelu(z, form) - oracle.gelu(-z, form), z, rtol=1e-13, atol=1e-14)


def test_parallel_block_from_the_sequential_one():
    """With a zero output projection the attention branch adds nothing, and the MLP branch reads the same rows in either
    wiring: both blocks agree.  With a zero down projection only the attention branch remains in either.  Otherwise they
    differ.  A parallel block without a second norm equals the block given its first norm twice."""
    mb = synth.make_microbatch([6, 1, 3], [0, 9, 4], seed=8, block=16)
    seq, par = small_shape(), small_shape(parallel_block=True)
    hidden = synth.draw_hidden(seq, mb.num_tokens, seed=8)

    def both(edit):
        outs = []
        for shape in (seq, par):
            layers = draw_layers(shape, 8, "fan_in")
            for w in layers:
                edit(w)
            outs.append(run_oracle(shape, mb, layers=layers, hidden=hidden, pool=oracle_pool(shape, mb, 8))[0])
        return outs

    a, b = both(lambda w: w["wo"].zero_())
    assert torch.equal(a, b)
    a, b = both(lambda w: w["wdown"].zero_())
    assert torch.equal(a, b)
    a, b = both(lambda w: None)
    assert not torch.allclose(a, b, rtol=1e-3)
    twice = draw_layers(par, 8, "fan_in")
    for w in twice:
        w["norm2"] = w["norm1"].clone()
    shared = draw_layers(par, 8, "fan_in", shared_norm=True)
    assert all("norm2" not in w for w in shared)
    a = run_oracle(par, mb, layers=twice, hidden=hidden, pool=oracle_pool(par, mb, 8))[0]
    b = run_oracle(par, mb, layers=shared, hidden=hidden, pool=oracle_pool(par, mb, 8))[0]
    assert torch.equal(a, b)


def test_zero_block_biases_change_nothing_and_real_ones_shift_by_themselves():
    shape = small_shape(norm_kind="layer", mlp_kind="gelu_tanh", num_layers=1)
    mb = synth.make_microbatch([4, 1], [0, 5], seed=9, block=16)
    hidden = synth.draw_hidden(shape, mb.num_tokens, seed=9)
    none = draw_layers(shape, 9, "fan_in")
    zero = draw_layers(shape, 9, "fan_in", block_biases=True)
    for w in zero:
        for k in ("norm1_bias", "norm2_bias", "bo", "bup", "bdown"):
            w[k].zero_()
    a = run_oracle(shape, mb, layers=none, hidden=hidden, pool=oracle_pool(shape, mb, 9))[0]
    b = run_oracle(shape, mb, layers=zero, hidden=hidden, pool=oracle_pool(shape, mb, 9))[0]
    assert torch.equal(a, b)
    # the last bias of the block lands on the output as it is
    zero[0]["bdown"] = synth.draw_block_biases(shape, 0, seed=9)["bdown"]
    c = run_oracle(shape, mb, layers=zero, hidden=hidden, pool=oracle_pool(shape, mb, 9))[0]
    assert torch.allclose(c - a, zero[0]["bdown"].double().expand_as(a), rtol=0, atol=1e-12)


# ---------------------------------------------------------------- frequency scaling of the rotation

LLAMA31 = ("llama3", 8.0, 1.0, 4.0, 8192)          # the parameters the Llama-3.1 models are published with


def test_rope_scaling_with_factor_one_changes_nothing_and_linear_scaling_compresses_positions():
    g = torch.Generator().manual_seed(3)
    u = torch.randn(6, 3, 16, dtype=F64, generator=g)
    pos = torch.tensor([0, 4, 8, 12, 400, 8000])
    plain = oracle.rope_rotate(u, pos, 1e4)
    assert torch.equal(oracle.rope_rotate(u, pos, 1e4, scaling=("linear", 1.0)), plain)
    assert torch.equal(oracle.rope_rotate(u, pos, 1e4, scaling=("llama3", 1.0, 1.0, 4.0, 8192)), plain)
    # positions that are multiples of the factor: the scaled rotation is the plain one at position / factor
    got = oracle.rope_rotate(u, pos, 1e4, scaling=("linear", 4.0))
    want = oracle.rope_rotate(u, pos // 4, 1e4)
    assert torch.allclose(got, want, rtol=1e-12, atol=1e-12)
    assert not torch.allclose(got, plain, rtol=1e-3)


def test_wavelength_scaling_keeps_fast_pairs_and_slows_the_slow_ones():
    d, theta = 128, 5e5
    i = torch.arange(d // 2, dtype=F64)
    inv = theta ** (-2.0 * i / d)
    got = oracle.scaled_inv_freq(inv, LLAMA31)
    ratio = got / inv
    wavelength = 2 * math.pi / inv
    fast, slow = wavelength < 8192 / 4.0, wavelength > 8192 / 1.0
    assert torch.equal(ratio[fast], torch.ones(int(fast.sum()), dtype=F64))
    assert torch.allclose(ratio[slow], torch.full((int(slow.sum()),), 1 / 8.0, dtype=F64), rtol=1e-15)
    mid = ~(fast | slow)
    # theta = 500000, 64 pairs: wavelengths 2 pi theta^(i/64); 2048 and 8192 are passed after pairs 28 and 35
    assert int(fast.sum()) == 29 and int(mid.sum()) == 6 and int(slow.sum()) == 29
    assert (ratio[mid] > 1 / 8.0).all() and (ratio[mid] < 1.0).all()
    assert (ratio[1:] <= ratio[:-1] + 1e-15).all()                       # never rising with the pair index
    # continuous at the borders: a frequency exactly at a border gets the neighbouring rule's value
    for turns, want in ((4.0, 1.0), (1.0, 1 / 8.0)):
        f = torch.tensor([turns * 2 * math.pi / 8192], dtype=F64)
        for eps in (-1e-9, 1e-9):
            r = float(oracle.scaled_inv_freq(f * (1 + eps), LLAMA31) / (f * (1 + eps)))
            assert abs(r - want) < 1e-6
    # halfway between the borders in turns (2.5 of them over the trained length): the mean of both frequencies
    f = torch.tensor([2.5 * 2 * math.pi / 8192], dtype=F64)
    assert abs(float(oracle.scaled_inv_freq(f, LLAMA31) / f) - 0.5 * (1 + 1 / 8.0)) < 1e-12


@pytest.mark.parametrize("scaling", [("linear", 4.0), ("llama3", 8.0, 1.0, 4.0, 64)])
def test_rope_scaling_matches_scalar_loops(scaling):
    """Whole block with scaled rotation frequencies; the trained length of the wavelength kind is chosen so that the
    eight pairs of this small head fall into all three ranges."""
    shape = small_shape(num_q_heads=4, num_kv_heads=2, hidden=12, ffn=20, head_dim=16, kv_block_size=4, rope_theta=100.0,
                        rope_scaling=scaling)
    if scaling[0] == "llama3":
        inv = 100.0 ** (-2.0 * torch.arange(8, dtype=F64) / 16)
        r = oracle.scaled_inv_freq(inv, scaling) / inv
        assert (r == 1).any() and (r == 1 / 8.0).any() and ((r > 1 / 8.0) & (r < 1)).any()
    q_lens, ctx_lens = [5, 1, 3], [0, 6, 2]
    mb = synth.make_microbatch(q_lens, ctx_lens, seed=3, block=4, position_shift=40)
    layers = draw_layers(shape, 3, "fan_in")
    hidden = synth.draw_hidden(shape, mb.num_tokens, seed=3)
    pool = oracle_pool(shape, mb, 3)
    pool0 = pool.clone()
    out, _, _ = run_oracle(shape, mb, layers=layers, hidden=hidden, pool=pool)
    got, row0 = [], 0
    x_rows = hidden.double().tolist()
    for s, (q, c) in enumerate(zip(q_lens, ctx_lens)):
        rows = x_rows[row0:row0 + q]
        for l in range(shape.num_layers):
            w = {k: v.double().tolist() for k, v in layers[l].items()}
            ck, cv = [], []
            for j in range(c):
                b = int(mb.block_tables[s][j // 4])
                ck.append(pool0[l, 0, b, j % 4].tolist())
                cv.append(pool0[l, 1, b, j % 4].tolist())
            rows = brute_force.layer_one_sequence(shape, w, rows, list(range(c + 40, c + q + 40)), ck, cv)
        got.extend(rows)
        row0 += q
    got = torch.tensor(got, dtype=F64)
    assert torch.allclose(out, got, rtol=1e-9, atol=1e-10), float((out - got).abs().max())
    base = dataclasses.replace(shape, rope_scaling=None)
    plain, _, _ = run_oracle(base, mb, layers=layers, hidden=hidden, pool=pool0.clone())
    assert not torch.allclose(out, plain, rtol=1e-3)


def test_cache_store_type_as_wide_as_the_arithmetic_changes_nothing():
    """kv_store_dtype = the oracle's own float64: a rounding that rounds nothing; output and pool bit for bit."""
    shape = small_shape()
    mb = synth.make_microbatch([9, 1, 1, 20], [3, 33, 0, 11], seed=31)
    out0, slots0, pool0 = run_oracle(shape, mb, seed=31)
    out1, slots1, pool1 = run_oracle(shape, mb, seed=31, kv_store_dtype=F64)
    assert slots0 == slots1 and torch.equal(out0, out1)
    assert torch.equal(pool0.nan_to_num(nan=-7.0), pool1.nan_to_num(nan=-7.0))


def test_cache_store_rounds_exactly_the_appended_slots_once():
    """With a bfloat16 store, what a layer appends is what the unrounded reading appends, rounded once to
    bfloat16, at exactly the mapped slots (first layer: its input does not depend on the reading), everything
    else in the pool stays bit for bit; the new values are bfloat16 numbers."""
    shape = small_shape(num_layers=2)
    q_lens, ctx_lens = [18, 1, 1], [15, 16, 31]
    mb = synth.make_microbatch(q_lens, ctx_lens, seed=32)
    before = oracle_pool(shape, mb, 32)
    _, slots, pool_plain = run_oracle(shape, mb, seed=32, pool=before.clone())
    _, slots_r, pool_round = run_oracle(shape, mb, seed=32, pool=before.clone(), kv_store_dtype=torch.bfloat16)
    assert slots == slots_r
    flat = lambda p: p.view(shape.num_layers, 2, -1, shape.num_kv_heads, shape.head_dim)
    want = torch.zeros(mb.num_kv_blocks * 16, dtype=torch.bool)
    want[slots] = True
    b, p, r = flat(before), flat(pool_plain), flat(pool_round)
    assert torch.equal(r[:, :, ~want].nan_to_num(nan=-7.0), b[:, :, ~want].nan_to_num(nan=-7.0))
    assert torch.equal(r[0][:, want], p[0][:, want].to(torch.bfloat16).to(F64))
    assert not torch.equal(r[0][:, want], p[0][:, want])                   # the rounding did something
    new = r[:, :, want]
    assert torch.equal(new, new.to(torch.bfloat16).to(F64))                # every appended value is a bfloat16 number
    # the second layer's appends differ from the rounded plain ones only through the first layer's attention
    assert torch.allclose(r[1][:, want], p[1][:, want], rtol=0, atol=0.05)


@pytest.mark.parametrize("nq,nkv", [(4, 2), (3, 3), (4, 1)])
def test_rounded_cache_matches_scalar_loops_that_read_back_what_they_stored(nq, nkv):
    """Scalar loops in which every new key and value is rounded to bfloat16 on its way into the cache and the
    chunk that wrote them attends to the stored values."""
    shape = small_shape(num_q_heads=nq, num_kv_heads=nkv, hidden=12, ffn=20, head_dim=4, kv_block_size=4)
    q_lens, ctx_lens = [5, 1, 3], [0, 6, 2]
    mb = synth.make_microbatch(q_lens, ctx_lens, seed=3, block=4)
    layers = draw_layers(shape, 3, "fan_in")
    hidden = synth.draw_hidden(shape, mb.num_tokens, seed=3)
    pool = oracle_pool(shape, mb, 3)
    pool0 = pool.clone()
    out, _, _ = run_oracle(shape, mb, layers=layers, hidden=hidden, pool=pool, kv_store_dtype=torch.bfloat16)
    plain, _, _ = run_oracle(shape, mb, layers=layers, hidden=hidden, pool=pool0.clone())
    got, row0 = [], 0
    x_rows = hidden.double().tolist()
    for s, (q, c) in enumerate(zip(q_lens, ctx_lens)):
        rows = x_rows[row0:row0 + q]
        for l in range(shape.num_layers):
            w = {k: v.double().tolist() for k, v in layers[l].items()}
            ck, cv = [], []
            for j in range(c):
                blk = int(mb.block_tables[s][j // 4])
                ck.append(pool0[l, 0, blk, j % 4].tolist())
                cv.append(pool0[l, 1, blk, j % 4].tolist())
            rows = brute_force.layer_one_sequence_rounded_cache(shape, w, rows, list(range(c, c + q)), ck, cv)
        got.extend(rows)
        row0 += q
    got = torch.tensor(got, dtype=F64)
    assert torch.allclose(out, got, rtol=1e-10, atol=1e-11), float((out - got).abs().max())
    assert float((out - plain).abs().max()) > 1e-5           # and it is not the unrounded reading
    # the rounding helper of the scalar loops against literal bfloat16 facts: 1 + 2^-8 is a tie and goes to even
    assert brute_force.round_to_bfloat16(1.0 + 2.0 ** -8) == 1.0
    assert brute_force.round_to_bfloat16(1.0 + 3 * 2.0 ** -8) == 1.0 + 2.0 ** -6
    assert brute_force.round_to_bfloat16(-0.3) == -0.30078125


@pytest.mark.parametrize("chunks", [[5, 11, 16], [31, 1], [1] * 6 + [26]])
def test_chunked_prefill_equals_unsplit_with_a_rounded_cache(chunks):
    """Under the stored-value reading a later chunk and the writing chunk see the same keys and values, so a
    prefill cut into chunks equals the unsplit one as closely as with the unrounded pool."""
    shape = small_shape()
    n = sum(chunks)
    layers = draw_layers(shape, 7, "fan_in")
    hidden = synth.draw_hidden(shape, n, seed=7)
    mb = synth.make_microbatch([n], [0], seed=7)
    full, _, pool_full = run_oracle(shape, mb, layers=layers, hidden=hidden, kv_store_dtype=torch.bfloat16)
    pool = oracle.new_pool(oracle_shape(shape), mb.num_kv_blocks)
    outs, done = [], 0
    for c in chunks:
        pos = torch.arange(done, done + c, dtype=torch.int32)
        o, _ = oracle.stage_forward(oracle_shape(shape), layers, hidden[done:done + c], pos, [c], [done],
                                    mb.block_tables, pool, kv_store_dtype=torch.bfloat16)
        outs.append(o)
        done += c
    got = torch.cat(outs)
    assert torch.allclose(got, full, rtol=1e-11, atol=1e-12)
    used = synth.valid_slot_mask(mb, 16, include_new=True)
    assert torch.equal(pool[:, :, used], pool_full[:, :, used])
    # whereas under the unrounded reading a chunked run that stores bfloat16 between calls would differ from it
    plain, _, _ = run_oracle(shape, mb, layers=layers, hidden=hidden)
    assert float((plain - full).abs().max()) > 1e-6


# ---------------------------------------------------------------- slots and pool writes

def test_slot_mapping_closed_form_and_pool_diff():
    shape = small_shape()
    q_lens, ctx_lens = [18, 1, 1], [15, 16, 31]
    mb = synth.make_microbatch(q_lens, ctx_lens, seed=11)
    slots = oracle.slot_mapping(q_lens, ctx_lens, mb.block_tables, 16)
    # enumerate every logical position of every sequence and keep the new ones
    expect = []
    for s, (q, c) in enumerate(zip(q_lens, ctx_lens)):
        logical_to_slot = {}
        for b, blk in enumerate(mb.block_tables[s].tolist()):
            for o in range(16):
                logical_to_slot[b * 16 + o] = blk * 16 + o
        expect += [logical_to_slot[j] for j in range(c, c + q)]
    assert slots == expect and len(set(slots)) == len(slots)
    pool = oracle_pool(shape, mb, 11)
    before = pool.clone()
    _, slots2, _ = run_oracle(shape, mb, seed=11, pool=pool)
    assert slots2 == slots
    flat_b = before.view(shape.num_layers, 2, -1, shape.num_kv_heads, shape.head_dim)
    flat_a = pool.view(shape.num_layers, 2, -1, shape.num_kv_heads, shape.head_dim)
    changed = ~((flat_a == flat_b) | (torch.isnan(flat_a) & torch.isnan(flat_b))).all(dim=-1).all(dim=-1)
    want = torch.zeros(mb.num_kv_blocks * 16, dtype=torch.bool)
    want[slots] = True
    assert torch.equal(changed, want.expand(shape.num_layers, 2, -1))
    assert not torch.isnan(flat_a[:, :, slots]).any()


def test_poisoned_slots_never_reach_output():
    shape = small_shape()
    mb = synth.make_microbatch([9, 1, 1], [3, 16, 40], seed=12)
    out, _, _ = run_oracle(shape, mb, seed=12)
    assert torch.isfinite(out).all()


# ---------------------------------------------------------------- RMSNorm, RoPE, SwiGLU closed forms

def test_rmsnorm_closed_forms():
    g = torch.tensor([0.5, 2.0, -1.0, 3.0], dtype=F64)
    c, eps = 3.0, 1e-5
    a = oracle.rmsnorm(torch.full((1, 4), c, dtype=F64), g, eps)
    assert torch.allclose(a[0], g * c / math.sqrt(c * c + eps), rtol=1e-15)
    x = torch.tensor([[1.0, -2.0, 3.0, 0.5]], dtype=F64)
    ms = float((x * x).mean())
    a = oracle.rmsnorm(x, g, eps)
    assert math.isclose(float(((a / g) ** 2).mean()), 1 - eps / (ms + eps), rel_tol=1e-13)
    # scale invariance when eps is negligible
    assert torch.allclose(oracle.rmsnorm(x, g, 0.0), oracle.rmsnorm(7.0 * x, g, 0.0), rtol=1e-14)
    # eps sits inside the square root, added to the mean square
    assert math.isclose(float(oracle.rmsnorm(torch.zeros(1, 4, dtype=F64) + 1e-3, g, 1.0)[0, 1]),
                        2.0 * 1e-3 / math.sqrt(1e-6 + 1.0), rel_tol=1e-14)


def test_rope_closed_forms():
    torch.manual_seed(4)
    u = torch.randn(5, 3, 8, dtype=F64)
    pos = torch.tensor([0, 1, 7, 100, 8191])
    y = oracle.rope_rotate(u, pos, 1e4)
    assert torch.equal(y[0], u[0])                                            # position 0 is the identity
    assert torch.allclose(y.norm(dim=-1), u.norm(dim=-1), rtol=1e-13)         # rotations keep the norm
    # d = 2: a plain 2-D rotation by pos radians (theta**0 = 1)
    v = torch.tensor([[[1.0, 0.0]], [[0.0, 1.0]]], dtype=F64)
    r = oracle.rope_rotate(v, torch.tensor([2, 3]), 1e4)
    assert torch.allclose(r[0, 0], torch.tensor([math.cos(2), math.sin(2)], dtype=F64), rtol=1e-14)
    assert torch.allclose(r[1, 0], torch.tensor([-math.sin(3), math.cos(3)], dtype=F64), rtol=1e-14)
    # half-split pairing with per-pair frequency theta**(-2i/d): element i pairs with i + d/2
    d, theta, p = 8, 1e4, 5
    e = torch.zeros(1, 1, d, dtype=F64)
    e[0, 0, 1] = 1.0
    z = oracle.rope_rotate(e, torch.tensor([p]), theta)[0, 0]
    ang = p * theta ** (-2.0 * 1 / d)
    expect = torch.zeros(d, dtype=F64)
    expect[1], expect[1 + d // 2] = math.cos(ang), math.sin(ang)
    assert torch.allclose(z, expect, rtol=1e-14, atol=1e-16)
    # relative property: <R_p q, R_s k> depends on p - s only
    q, k = torch.randn(1, 1, 8, dtype=F64), torch.randn(1, 1, 8, dtype=F64)
    dot = lambda p_, s_: float((oracle.rope_rotate(q, torch.tensor([p_]), theta)
                                * oracle.rope_rotate(k, torch.tensor([s_]), theta)).sum())
    assert math.isclose(dot(9, 4), dot(105, 100), rel_tol=1e-10)
    assert not math.isclose(dot(9, 4), dot(9, 5), rel_tol=1e-3)


def test_positions_shift_leaves_fresh_prefill_unchanged_and_is_separate_from_ctx():
    shape = small_shape()
    layers = draw_layers(shape, 13, "fan_in")
    hidden = synth.draw_hidden(shape, 11, seed=13)
    mb0 = synth.make_microbatch([11], [0], seed=13)
    mb1 = synth.make_microbatch([11], [0], seed=13, position_shift=37)
    o0, s0, _ = run_oracle(shape, mb0, layers=layers, hidden=hidden)
    o1, s1, _ = run_oracle(shape, mb1, layers=layers, hidden=hidden)
    assert s0 == s1                                  # slots follow ctx + i, not positions
    assert torch.allclose(o0, o1, rtol=1e-9, atol=1e-10)   # attention sees only position differences


def test_silu_and_swiglu_limits():
    z = torch.tensor([0.0, 40.0, -40.0, 1.0], dtype=F64)
    s = oracle.silu(z)
    assert s[0] == 0.0 and math.isclose(float(s[1]), 40.0, rel_tol=1e-15) and abs(float(s[2])) < 1e-15
    assert math.isclose(float(s[3]), 1.0 / (1.0 + math.exp(-1.0)), rel_tol=1e-15)
    shape = small_shape(num_layers=1)
    mb = synth.make_microbatch([3], [0], seed=14)
    layers = draw_layers(shape, 14, "fan_in")
    layers[0]["wgate"] = torch.zeros_like(layers[0]["wgate"])
    taps = []
    out, _, _ = run_oracle(shape, mb, layers=layers, taps=taps)
    assert torch.equal(taps[0]["m"], torch.zeros_like(taps[0]["m"])) and torch.equal(out, taps[0]["h"])


def test_zero_output_projections_give_identity():
    shape = small_shape()
    mb = synth.make_microbatch([5, 1], [0, 9], seed=15)
    layers = draw_layers(shape, 15, "fan_in")
    for w in layers:
        w["wo"] = torch.zeros_like(w["wo"])
        w["wdown"] = torch.zeros_like(w["wdown"])
    hidden = synth.draw_hidden(shape, mb.num_tokens, seed=15)
    out, _, _ = run_oracle(shape, mb, seed=15, layers=layers, hidden=hidden)
    assert torch.equal(out, hidden.double())


def test_single_token_layer_reduces_to_matmul_chain():
    """One fresh token: attention returns its own value vector, so the layer is a chain of
    matrix products; cross-check against numpy float64 written with explicit transposes."""
    import numpy as np
    shape = small_shape(num_layers=1)
    mb = synth.make_microbatch([1], [0], seed=16)
    layers = draw_layers(shape, 16, "fan_in")
    hidden = synth.draw_hidden(shape, 1, seed=16)
    out, _, _ = run_oracle(shape, mb, layers=layers, hidden=hidden)
    w = {k: v.double().numpy() for k, v in layers[0].items()}
    x = hidden.double().numpy()[0]
    nq, nkv, d = shape.num_q_heads, shape.num_kv_heads, shape.head_dim
    a = x * w["norm1"] / np.sqrt(np.mean(x * x) + shape.rms_eps)
    v = (w["wqkv"][(nq + nkv) * d:] @ a).reshape(nkv, d)          # position 0: no rotation
    o = np.concatenate([v[h // (nq // nkv)] for h in range(nq)])
    h = x + w["wo"] @ o
    b = h * w["norm2"] / np.sqrt(np.mean(h * h) + shape.rms_eps)
    gate, up = w["wgate"] @ b, w["wup"] @ b
    y = h + w["wdown"] @ (gate / (1 + np.exp(-gate)) * up)
    assert np.allclose(out[0].numpy(), y, rtol=1e-12, atol=1e-13)


def test_synthetic_generator_is_deterministic_and_sliceable():
    a = synth.draw_normal_bf16(0, 5, 1000)
    b = synth.draw_normal_bf16(0, 5, 400, offset=300)
    assert torch.equal(a[300:700], b)
    idx = torch.tensor([999, 0, 512], dtype=torch.int64)
    assert torch.equal(synth.draw_normal_bf16_at(0, 5, idx), a[idx])
    assert not torch.equal(a, synth.draw_normal_bf16(1, 5, 1000))
    x = synth.draw_normal_bf16(0, 6, 200000).float()
    assert abs(float(x.mean())) < 0.01 and abs(float(x.std()) - 1.0) < 0.01
