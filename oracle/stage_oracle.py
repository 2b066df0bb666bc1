"""Plain CPU oracle of a pipeline stage's decoder-layer forward pass.

TEST INFRASTRUCTURE.  Slow, unfused, written for checking by eye.  It shares no
code with the HIP library and must not be imported by it.

What it computes.  The serving system hands each inference engine a run of
decoder layers and feeds it micro-batches that mix prefill chunks and decode
tokens; the engine's output is the activation tensor passed to the next stage
(paper section 3.2.2 "Distributed Inference Engine"; section 4.2 for the two
phases and for the payload growing with the number of processed tokens).  The
paper leaves the computation itself to its engine runtime and evaluates
Llama-family models (section 5, "Models"), so the definition used here is the
standard pre-norm Llama decoder block: RMSNorm, q/k/v projection, rotary
embedding (half-split pairing), append to a paged KV cache, causal attention
with grouped KV heads, output projection + residual, RMSNorm, SwiGLU MLP +
residual.  No biases, except an optional one on the q/k/v projection (the Qwen2
family of the paper's model table has it; it is added before the rotation),
and an optional RMSNorm over each query head and each key head (gains "qnorm",
"knorm" of head_dim elements, the stage's eps) between the bias and the
rotation, which is how the Qwen3 family of the same table (section 3.1.3)
defines its block; optionally only the first rotary_dim elements of every head
rotate, and optionally the rotation pairs neighbouring elements (2i, 2i + 1)
instead of (i, i + d/2) - the two together are the rotary embedding of the GLM /
ChatGLM families of that table; or, when a layer carries "alibi" slopes (one per
query head), no rotation at all and attention scores lowered in proportion to the
distance between query and key (attention with linear biases: the larger
Baichuan model of that table; distances are counted in logical indices of the
sequence); no final norm.  Three more switches of the shape cover the remaining dense blocks of that table
(the Falcon, GPT-2 and Cohere families): norm_kind "layer" makes both norms LayerNorms (mean removed, variance
instead of mean square, an optional bias "norm1_bias" / "norm2_bias" besides the gain); mlp_kind "gelu_tanh" or
"gelu_erf" replaces the gated MLP by down(gelu(up(b))), with optional biases "bup", "bdown" (and "bo" on the output
projection of the attention); parallel_block feeds the attention branch and the MLP branch from the same block
input x and adds both to it, y = x + attn(norm1(x)) + mlp(norm2(x)), where a layer without "norm2" feeds the
MLP from norm1(x) as well.  A block without any rotation or bias of the scores (GPT-2: positions enter outside
the layers) is the linear-bias block with zero slopes.

Numerics: every tensor is widened to `dtype` (float64 by default) on entry and
nothing is rounded afterwards.  Library primitives used as steps: matmul,
exp/softmax building blocks, cos/sin.

Loop discipline: a sequence's rows depend only on that sequence's data and on
the logical key order, never on physical block numbers.

Pins (tests/test_oracle_*.py): scalar-loop brute force of the whole block on
tiny shapes; dense masked attention; paged == contiguous (bitwise); chunked ==
unsplit; decode == last prefill row; batch-order independence; closed forms for
RMSNorm, RoPE, softmax degenerate cases; GQA == MHA with replicated heads;
zero output projections give the identity; library cross-checks (fp64 matmul
chain, torch scaled_dot_product_attention); the cache-as-a-narrower-store
switch (kv_store_dtype): a store as wide as the arithmetic changes nothing bit
for bit, a bfloat16 store rounds exactly the appended slots once, scalar loops
that read back what they stored, chunked == unsplit under it; partial rotary:
rotary_dim = head_dim is the default bit for bit, the elements past rotary_dim
are the unrotated projection, the rotated part is the rotation of a head of that
size, scalar loops with it; neighbour pairing: equal to the half-split rotation
of the head with its even elements first and its odd elements last, put back in
place (a permutation identity), a literal angle, scalar loops with it; linear
biases: zero slopes equal the rotation at position zero bit for bit, zero
queries give geometric weights (closed form), a row-constant shift of the biases
changes nothing, scalar loops with them, chunked == unsplit and decode == last
prefill row under them; LayerNorm against the library routine, zero mean and unit variance of its output, its
shift invariance, and a constant row (closed form: the bias); both GELU forms against the library routine and
literal values; the parallel block from the sequential one (zero output projection: both agree; zero down
projection: y = x + attention branch), shared norm == the same norm given twice, scalar loops with every
switch; frequency scaling of the rotation: factor 1 changes nothing bit for bit, the linear
kind equals the unscaled rotation at position / factor, the wavelength kind keeps fast pairs, divides slow pairs'
frequencies by the factor, is continuous at both borders and monotone between them, literal pair counts for the
published Llama-3.1 parameters, scalar loops with it.  The paper prints no numeric values
for this path, so parity against printed values is unpinned; parity is against
the definition.
"""
from __future__ import annotations

import dataclasses
import math
from typing import Dict, List, Optional, Sequence

import torch


@dataclasses.dataclass(frozen=True)
class OracleShape:
    num_layers: int
    hidden: int
    num_q_heads: int
    num_kv_heads: int
    head_dim: int
    ffn: int
    rms_eps: float = 1e-5
    rope_theta: float = 1e4
    kv_block_size: int = 16
    rotary_dim: int = 0          # 0: the whole head rotates; else only its first rotary_dim elements do
    rope_interleaved: bool = False   # False: pairs (i, i + d/2); True: pairs (2i, 2i + 1)
    norm_kind: str = "rms"       # "rms" | "layer": both norms of the block (rms_eps is the epsilon of either)
    mlp_kind: str = "swiglu"     # "swiglu": down(silu(gate(b)) * up(b)); "gelu_tanh" | "gelu_erf": down(gelu(up(b)))
    parallel_block: bool = False  # True: y = x + attn(norm1(x)) + mlp(norm2(x)); False: the branches in sequence
    # frequency scaling of the rotary embedding for contexts beyond the trained length: None, ("linear", factor) or
    # ("llama3", factor, low_freq_factor, high_freq_factor, original_max_position)
    rope_scaling: Optional[tuple] = None


def new_pool(shape: OracleShape, num_kv_blocks: int, dtype=torch.float64, fill=float("nan")) -> torch.Tensor:
    """The oracle's own KV pool: [layer, K|V, block, slot, kv_head, dim]."""
    return torch.full((shape.num_layers, 2, num_kv_blocks, shape.kv_block_size,
                       shape.num_kv_heads, shape.head_dim), fill, dtype=dtype)


def rmsnorm(x: torch.Tensor, gain: torch.Tensor, eps: float) -> torch.Tensor:
    """x * gain / sqrt(mean(x^2) + eps), per row."""
    ms = (x * x).mean(dim=-1, keepdim=True)
    return x * gain / torch.sqrt(ms + eps)


def layernorm(x: torch.Tensor, gain: torch.Tensor, bias: Optional[torch.Tensor], eps: float) -> torch.Tensor:
    """(x - mean) / sqrt(var + eps) * gain (+ bias), per row; var is the mean of the squared deviations."""
    mean = x.mean(dim=-1, keepdim=True)
    dev = x - mean
    var = (dev * dev).mean(dim=-1, keepdim=True)
    y = dev / torch.sqrt(var + eps) * gain
    return y if bias is None else y + bias


def block_norm(shape: "OracleShape", x: torch.Tensor, gain: torch.Tensor, bias: Optional[torch.Tensor]) -> torch.Tensor:
    """The norm in front of a branch of the block, by shape.norm_kind."""
    if shape.norm_kind == "layer":
        return layernorm(x, gain, bias, shape.rms_eps)
    assert shape.norm_kind == "rms" and bias is None
    return rmsnorm(x, gain, shape.rms_eps)


def gelu(z: torch.Tensor, form: str) -> torch.Tensor:
    """z * Phi(z) with the normal distribution function Phi ("gelu_erf"), or its tanh form
    0.5 z (1 + tanh(sqrt(2/pi) (z + 0.044715 z^3))) ("gelu_tanh")."""
    if form == "gelu_erf":
        return 0.5 * z * (1.0 + torch.erf(z / math.sqrt(2.0)))
    assert form == "gelu_tanh"
    return 0.5 * z * (1.0 + torch.tanh(math.sqrt(2.0 / math.pi) * (z + 0.044715 * z * z * z)))


def scaled_inv_freq(inv_freq: torch.Tensor, scaling: Optional[tuple]) -> torch.Tensor:
    """The rotation frequencies of a model served beyond its trained context (the Llama family the paper evaluates
    publishes its long-context members this way).

    ("linear", f): every frequency divided by f - positions are compressed by f.
    ("llama3", f, low, high, L): by wavelength w = 2 pi / frequency against the trained length L: pairs that turn
    often, w < L / high, keep their frequency; pairs that turn rarely, w > L / low, get frequency / f; between the two
    the frequency is the mix (1 - s) * frequency / f + s * frequency with s = (L / w - low) / (high - low), which is
    0 and 1 at the two borders."""
    if scaling is None:
        return inv_freq
    if scaling[0] == "linear":
        return inv_freq / float(scaling[1])
    assert scaling[0] == "llama3"
    _, f, low, high, length = scaling
    out = inv_freq.clone()
    for i in range(inv_freq.numel()):
        freq = float(inv_freq[i])
        wavelength = 2.0 * math.pi / freq
        if wavelength < length / high:
            continue
        if wavelength > length / low:
            out[i] = freq / f
        else:
            smooth = (length / wavelength - low) / (high - low)
            out[i] = (1.0 - smooth) * freq / f + smooth * freq
    return out


def rope_rotate(u: torch.Tensor, pos: torch.Tensor, theta: float, rotary_dim: int = 0,
                interleaved: bool = False, scaling: Optional[tuple] = None) -> torch.Tensor:
    """Rotary embedding.  u: [T, heads, d]; pos: [T] integers.

    Half-split pairing (the default): pair (i, i + d/2) of every head is rotated by the angle
    pos * theta**(-2i/d).  Neighbour pairing (interleaved): pair (2i, 2i + 1) is rotated by the same angle.
    Angles, cos and sin are evaluated in float64.
    scaling: see scaled_inv_freq (the frequencies theta**(-2i/d) are replaced by their scaled values).
    Partial rotary (the GLM / ChatGLM families of the paper's model table, section 3.1.3, which also pair
    neighbours): with 0 < rotary_dim < d only the first rotary_dim elements of a head rotate, as a head of that
    size would (angles pos * theta**(-2i/rotary_dim)); the rest pass through.
    """
    if rotary_dim and rotary_dim < u.shape[-1]:
        return torch.cat([rope_rotate(u[..., :rotary_dim], pos, theta, 0, interleaved, scaling), u[..., rotary_dim:]],
                         dim=-1)
    t, _, d = u.shape
    half = d // 2
    i = torch.arange(half, dtype=torch.float64)
    inv_freq = scaled_inv_freq(theta ** (-2.0 * i / d), scaling)
    ang = pos.to(torch.float64).view(t, 1) * inv_freq.view(1, half)      # [T, d/2]
    cos = torch.cos(ang).to(u.dtype).view(t, 1, half)
    sin = torch.sin(ang).to(u.dtype).view(t, 1, half)
    if interleaved:
        first, second = u[..., 0::2], u[..., 1::2]
        out = torch.empty_like(u)
        out[..., 0::2] = first * cos - second * sin
        out[..., 1::2] = second * cos + first * sin
        return out
    lo, hi = u[..., :half], u[..., half:]
    return torch.cat([lo * cos - hi * sin, hi * cos + lo * sin], dim=-1)


def silu(z: torch.Tensor) -> torch.Tensor:
    return z / (1.0 + torch.exp(-z))


def slot_mapping(q_lens: Sequence[int], ctx_lens: Sequence[int], block_tables, block: int) -> List[int]:
    """Pool slot of every new token: table[s][j // block] * block + j % block, j = ctx + i."""
    slots: List[int] = []
    for s, (q, c) in enumerate(zip(q_lens, ctx_lens)):
        for i in range(q):
            j = c + i
            slots.append(int(block_tables[s][j // block]) * block + j % block)
    return slots


def attention_rows(q: torch.Tensor, keys: torch.Tensor, values: torch.Tensor, ctx: int,
                   slopes: Optional[torch.Tensor] = None) -> torch.Tensor:
    """Causal attention of one sequence's new rows over its whole logical cache.

    q: [n, nq, d] (rotated) rows at logical indices ctx .. ctx+n-1;
    keys, values: [ctx + n, nkv, d] in logical order.  Row i sees keys 0 .. ctx+i.
    Query head h reads kv head h // (nq // nkv).  Scores are scaled by 1/sqrt(d).
    slopes [nq] (attention with linear biases): the score of the query at logical index i for the key at logical
    index j is lowered by slopes[h] * (i - j).
    """
    n, nq, d = q.shape
    nkv = keys.shape[1]
    g = nq // nkv
    total = keys.shape[0]
    out = torch.empty_like(q)
    j = torch.arange(total).view(1, total)
    limit = (ctx + torch.arange(n)).view(n, 1)
    hidden_mask = j > limit                                          # [n, total]
    for h in range(nq):
        r = h // g
        e = (q[:, h, :] @ keys[:, r, :].T) / math.sqrt(d)             # [n, total]
        if slopes is not None:
            e = e - slopes[h].to(e.dtype) * (limit - j).to(e.dtype)     # distance of key j from the row's own index
        e = e.masked_fill(hidden_mask, float("-inf"))
        e = e - e.max(dim=-1, keepdim=True).values
        w = torch.exp(e)
        w = w / w.sum(dim=-1, keepdim=True)
        out[:, h, :] = w @ values[:, r, :]
    return out


def decoder_layer(shape: OracleShape, w: Dict[str, torch.Tensor], x: torch.Tensor, pos: torch.Tensor,
                  q_lens, ctx_lens, block_tables, pool_layer: torch.Tensor, slots: List[int],
                  taps: Optional[Dict[str, torch.Tensor]] = None, kv_store_dtype=None) -> torch.Tensor:
    """One decoder layer on packed rows x [T, H]; appends to pool_layer [2, block, slot, nkv, d].

    kv_store_dtype: None keeps the appended keys/values unrounded in the oracle's pool; a torch dtype
    (the cache's storage type) rounds them once on their way into the pool, so that attention, in
    this call and in later ones, reads what a cache of that type holds."""
    dt = x.dtype
    nq, nkv, d, blk = shape.num_q_heads, shape.num_kv_heads, shape.head_dim, shape.kv_block_size
    t = x.shape[0]
    wqkv = w["wqkv"].to(dt)

    def opt(name):
        return None if w.get(name) is None else w[name].to(dt)

    a = block_norm(shape, x, w["norm1"].to(dt), opt("norm1_bias"))
    qkv = a @ wqkv.T                                                  # weights are [out, in]
    if w.get("bqkv") is not None:                                     # optional projection bias (Qwen2 family)
        qkv = qkv + w["bqkv"].to(dt)
    q = qkv[:, : nq * d].reshape(t, nq, d)
    k = qkv[:, nq * d: (nq + nkv) * d].reshape(t, nkv, d)
    v = qkv[:, (nq + nkv) * d:].reshape(t, nkv, d)
    if w.get("qnorm") is not None:                                    # optional per-head norm (Qwen3 family)
        q = rmsnorm(q, w["qnorm"].to(dt), shape.rms_eps)              # over the d elements of each head
        k = rmsnorm(k, w["knorm"].to(dt), shape.rms_eps)
    slopes = w.get("alibi")                                           # [nq]: linear biases instead of a rotation
    if slopes is None:
        q = rope_rotate(q, pos, shape.rope_theta, shape.rotary_dim, shape.rope_interleaved, shape.rope_scaling)
        k = rope_rotate(k, pos, shape.rope_theta, shape.rotary_dim, shape.rope_interleaved, shape.rope_scaling)
    # append the new tokens' keys (rotated) and values at their slots
    slot_t = torch.as_tensor(slots, dtype=torch.int64)
    k_st = k if kv_store_dtype is None else k.to(kv_store_dtype).to(dt)
    v_st = v if kv_store_dtype is None else v.to(kv_store_dtype).to(dt)
    pool_layer[0, slot_t // blk, slot_t % blk] = k_st
    pool_layer[1, slot_t // blk, slot_t % blk] = v_st
    o = torch.empty(t, nq, d, dtype=dt)
    row0 = 0
    for s, (n, c) in enumerate(zip(q_lens, ctx_lens)):
        total = c + n
        nb = (total + blk - 1) // blk
        table = torch.as_tensor(block_tables[s][:nb], dtype=torch.int64)
        keys = pool_layer[0, table].reshape(nb * blk, nkv, d)[:total]   # logical order via the table
        vals = pool_layer[1, table].reshape(nb * blk, nkv, d)[:total]
        o[row0: row0 + n] = attention_rows(q[row0: row0 + n], keys, vals, c, slopes)
        row0 += n
    branch = o.reshape(t, nq * d) @ w["wo"].to(dt).T
    if opt("bo") is not None:
        branch = branch + opt("bo")
    h = x + branch                                                    # sequential: the MLP branch starts from here
    src = x if shape.parallel_block else h
    if w.get("norm2") is None:                                        # one norm for both branches
        assert shape.parallel_block
        b = a
    else:
        b = block_norm(shape, src, w["norm2"].to(dt), opt("norm2_bias"))
    if shape.mlp_kind == "swiglu":
        m = silu(b @ w["wgate"].to(dt).T) * (b @ w["wup"].to(dt).T)
    else:
        up = b @ w["wup"].to(dt).T
        if opt("bup") is not None:
            up = up + opt("bup")
        m = gelu(up, shape.mlp_kind)
    down = m @ w["wdown"].to(dt).T
    if opt("bdown") is not None:
        down = down + opt("bdown")
    y = h + down                                                      # parallel: x + both branches
    if taps is not None:
        taps.update(a=a, q=q, k=k, v=v, attn=o.reshape(t, nq * d), h=h, b=b, m=m, x=y)
    return y


def stage_forward(shape: OracleShape, layers: Sequence[Dict[str, torch.Tensor]], hidden: torch.Tensor,
                  positions, q_lens: Sequence[int], ctx_lens: Sequence[int], block_tables,
                  pool: torch.Tensor, dtype=torch.float64,
                  taps: Optional[List[Dict[str, torch.Tensor]]] = None, kv_store_dtype=None):
    """Run the stage's layers on one micro-batch.

    hidden [T, H] (any float dtype; widened exactly), positions [T], per-sequence q_lens
    (new tokens; 1 = decode) and ctx_lens (tokens already cached), block_tables [S][...],
    pool [L, 2, blocks, slot, nkv, d] holding the cached context at the logical positions
    0 .. ctx-1 of every sequence; it is updated in place with the new tokens (unrounded, or rounded
    once to kv_store_dtype if given: see decoder_layer).
    Returns (output [T, H] in `dtype`, slot list [T]).
    """
    assert pool.dtype == dtype
    x = hidden.to(dtype)
    pos = torch.as_tensor(positions, dtype=torch.int64)
    slots = slot_mapping(q_lens, ctx_lens, block_tables, shape.kv_block_size)
    for l in range(shape.num_layers):
        tap = {} if taps is not None else None
        x = decoder_layer(shape, layers[l], x, pos, q_lens, ctx_lens, block_tables, pool[l], slots, tap, kv_store_dtype)
        if taps is not None:
            taps.append(tap)
    return x, slots
