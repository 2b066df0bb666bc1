"""Seeded synthetic inputs for one pipeline stage's forward pass.

This module only *draws inputs*: counter-based pseudo-random tensors and the
integer structure of a micro-batch (sequence lengths, block tables).  It holds
none of the stage's arithmetic, so both the HIP path and the CPU oracle used
by the tests can be fed from it without sharing any code of the method.

Every value is a pure function of (seed, stream id, linear index), computed
with integer torch ops that behave identically on CPU and on the GPU, so a
tensor can be produced directly in device memory (the large KV pools never
exist on the host) and any slice of it can be re-drawn on the host later.

The micro-batch shapes follow the workloads the serving system forms: a mix of
prefill chunks and decode tokens in one micro-batch (paper section 3.2.2,
"Distributed Inference Engine", and section 4.2 on the prefill/decode phases).
"""
from __future__ import annotations

import dataclasses
import math
from typing import Dict, List, Optional, Sequence

import torch

_M32 = 0xFFFFFFFF
# odd multipliers below 2**31 so that a 32-bit value times the multiplier
# stays inside a signed 64-bit integer before it is masked back to 32 bits
_MUL_A = 0x7FEB352D
_MUL_B = 0x6C8E9CF5
_GOLD = 0x3C6EF372  # increments between the sub-draws of one element


def _mix32(x: torch.Tensor) -> torch.Tensor:
    """32-bit avalanche hash on int64 tensors whose values lie in [0, 2**32)."""
    x = x ^ (x >> 16)
    x = (x * _MUL_A) & _M32
    x = x ^ (x >> 15)
    x = (x * _MUL_B) & _M32
    x = x ^ (x >> 16)
    return x


def _mix32_int(x: int) -> int:
    x &= _M32
    x ^= x >> 16
    x = (x * _MUL_A) & _M32
    x ^= x >> 15
    x = (x * _MUL_B) & _M32
    x ^= x >> 16
    return x


def stream_key(seed: int, stream: int) -> int:
    """One 32-bit key per (seed, stream id)."""
    return _mix32_int(_mix32_int(seed * 0x9E3779B1 + 0x7F4A7C15) ^ (stream * 0x85EBCA6B + 0xC2B2AE35))


def hash_u32(seed: int, stream: int, idx: torch.Tensor) -> torch.Tensor:
    """Uniform 32-bit integers (held in int64) for the int64 indices `idx`."""
    key = stream_key(seed, stream)
    lo = idx & _M32
    hi = (idx >> 32) & _M32
    h = _mix32(lo ^ key)
    h = _mix32((h + hi * 0x2545F491 + 0x632BE5AB) & _M32)
    return h


def normal_from_index(seed: int, stream: int, idx: torch.Tensor) -> torch.Tensor:
    """Approximately N(0,1) float32 values for the int64 indices `idx`.

    Sum of twelve 16-bit uniforms (Irwin-Hall), centred: an exact integer below
    2**24 in magnitude, scaled by one float32 constant.  Tails end at 6 sigma.
    """
    base = hash_u32(seed, stream, idx)
    total = torch.zeros_like(base)
    for k in range(6):
        h = _mix32((base + (k + 1) * _GOLD) & _M32)
        total = total + (h & 0xFFFF) + (h >> 16)
    n = 2 * total - 12 * 65535          # integer, |n| <= 786420 < 2**24
    # variance of one 16-bit uniform is (65536**2 - 1)/12, of 2*sum(12) it is 4*(65536**2-1)
    sigma = math.sqrt(4.0 * (65536.0 ** 2 - 1.0))
    return n.to(torch.float32) * torch.tensor(1.0 / sigma, dtype=torch.float32, device=idx.device)


def draw_normal_bf16(seed: int, stream: int, numel: int, *, std: float = 1.0, mean: float = 0.0,
                     device: str | torch.device = "cpu", offset: int = 0,
                     chunk: Optional[int] = None, dtype: torch.dtype = torch.bfloat16) -> torch.Tensor:
    """`numel` values mean + std*N(0,1), rounded to bf16 (or to `dtype`: the same fp32 values rounded to
    the half-precision library's float16), for indices offset..offset+numel-1."""
    device = torch.device(device)
    if chunk is None:
        chunk = (1 << 26) if device.type == "cuda" else (1 << 22)
    out = torch.empty(numel, dtype=dtype, device=device)
    std32 = torch.tensor(std, dtype=torch.float32, device=device)
    for start in range(0, numel, chunk):
        stop = min(numel, start + chunk)
        idx = torch.arange(offset + start, offset + stop, dtype=torch.int64, device=device)
        v = normal_from_index(seed, stream, idx) * std32
        if mean != 0.0:
            v = v + torch.tensor(mean, dtype=torch.float32, device=device)
        out[start:stop] = v.to(dtype)
    return out


def draw_normal_bf16_at(seed: int, stream: int, idx: torch.Tensor, *, std: float = 1.0,
                        mean: float = 0.0, dtype: torch.dtype = torch.bfloat16) -> torch.Tensor:
    """Same values as `draw_normal_bf16`, at arbitrary int64 indices."""
    v = normal_from_index(seed, stream, idx) * torch.tensor(std, dtype=torch.float32, device=idx.device)
    if mean != 0.0:
        v = v + torch.tensor(mean, dtype=torch.float32, device=idx.device)
    return v.to(dtype)


def draw_int_uniform(seed: int, stream: int, n: int, lo: int, hi: int) -> List[int]:
    """n integers uniform in [lo, hi] (inclusive), as a Python list."""
    idx = torch.arange(n, dtype=torch.int64)
    h = hash_u32(seed, stream, idx)
    return (lo + (h % (hi - lo + 1))).tolist()


# --------------------------------------------------------------------------
# stage shapes and micro-batches
# --------------------------------------------------------------------------

@dataclasses.dataclass(frozen=True)
class StageShape:
    """Dimensions of one pipeline stage (a run of identical decoder layers)."""
    name: str
    num_layers: int
    hidden: int
    num_q_heads: int
    num_kv_heads: int
    head_dim: int
    ffn: int
    rms_eps: float = 1e-5
    rope_theta: float = 1e4
    kv_block_size: int = 16
    vocab: int = 0          # vocabulary size of the model the stage is cut from (embedding / output head)
    rotary_dim: int = 0     # 0: whole heads rotate; else only the first rotary_dim elements of every head
    rope_interleaved: bool = False   # rotation pairs: (i, i + d/2), or neighbours (2i, 2i + 1)
    norm_kind: str = "rms"          # "rms" | "layer": the block's two norms
    mlp_kind: str = "swiglu"        # "swiglu" | "gelu_tanh" | "gelu_erf" (the latter two: down(gelu(up(b))), no gate)
    parallel_block: bool = False    # attention branch and MLP branch both start from the block's input
    # None, ("linear", factor) or ("llama3", factor, low_freq_factor, high_freq_factor, original_max_position)
    rope_scaling: Optional[tuple] = None

    @property
    def qkv_out(self) -> int:
        return (self.num_q_heads + 2 * self.num_kv_heads) * self.head_dim

    @property
    def params_per_layer(self) -> int:
        h, d = self.hidden, self.head_dim
        return h * self.qkv_out + self.num_q_heads * d * h + 3 * h * self.ffn


TINY = StageShape("tiny-llama-style", 2, 256, 4, 2, 64, 688, vocab=1000)
LLAMA2_7B_STAGE = StageShape("llama2-7b-8of32", 8, 4096, 32, 32, 128, 11008, vocab=32000)
QWEN2_7B_STAGE = StageShape("qwen2-7b-7of28", 7, 3584, 28, 4, 128, 18944, vocab=152064)
LLAMA3_70B_STAGE = StageShape("llama3-70b-20of80", 20, 8192, 64, 8, 128, 28672, rope_theta=5e5, vocab=128256)


@dataclasses.dataclass
class MicroBatch:
    """Integer structure of one micro-batch: sequences packed one after another."""
    q_lens: List[int]            # new tokens per sequence (1 = decode, >1 = prefill chunk)
    ctx_lens: List[int]          # tokens of the sequence already in the KV cache
    block_tables: torch.Tensor   # int32 [S, max_blocks_per_seq], -1 where unused
    positions: torch.Tensor      # int32 [T]
    num_kv_blocks: int           # blocks in (each layer's) pool

    @property
    def num_seqs(self) -> int:
        return len(self.q_lens)

    @property
    def num_tokens(self) -> int:
        return int(sum(self.q_lens))

    @property
    def max_blocks_per_seq(self) -> int:
        return int(self.block_tables.shape[1])


def blocks_needed(total_len: int, block: int) -> int:
    return (total_len + block - 1) // block


def make_microbatch(q_lens: Sequence[int], ctx_lens: Sequence[int], *, seed: int, block: int = 16,
                    spare_blocks: int = 3, paging: str = "permuted",
                    max_blocks_per_seq: Optional[int] = None,
                    position_shift: int = 0) -> MicroBatch:
    """Lay sequences out in a paged pool.

    paging="permuted": physical blocks come from a seeded permutation of the pool, so a
    sequence's blocks are scattered and interleaved with other sequences' blocks.
    paging="identity": sequence s gets consecutive blocks (a contiguous cache).
    A few spare blocks stay unallocated; table entries past a sequence's need are -1.
    """
    q_lens = [int(q) for q in q_lens]
    ctx_lens = [int(c) for c in ctx_lens]
    need = [blocks_needed(c + q, block) for q, c in zip(q_lens, ctx_lens)]
    total = sum(need) + spare_blocks
    if paging == "permuted":
        g = torch.Generator(device="cpu")
        g.manual_seed(seed * 7919 + 17)
        perm = torch.randperm(total, generator=g).tolist()
    elif paging == "identity":
        perm = list(range(total))
    else:
        raise ValueError(paging)
    width = max(need) if max_blocks_per_seq is None else max_blocks_per_seq
    width = max(width, 1)
    table = torch.full((len(q_lens), width), -1, dtype=torch.int32)
    cursor = 0
    for s, nb in enumerate(need):
        if nb:
            table[s, :nb] = torch.tensor(perm[cursor:cursor + nb], dtype=torch.int32)
        cursor += nb
    pos: List[int] = []
    for q, c in zip(q_lens, ctx_lens):
        pos.extend(range(c + position_shift, c + q + position_shift))
    return MicroBatch(q_lens, ctx_lens, table, torch.tensor(pos, dtype=torch.int32), total)


def decode_contexts(seed: int, n: int, lo: int, hi: int, stream: int = 900) -> List[int]:
    return draw_int_uniform(seed, stream, n, lo, hi)


def workload(name: str, seed: int = 0, budget: int = 256):
    """(StageShape, MicroBatch) for the named workload.

    "tiny":        2 fresh 32-token prefills + 6 decode tokens with contexts in [16,100]
    "llama2-7b":   64 decode tokens, contexts in [512,2048]
    "qwen2-7b":    one fresh 2048-token prefill chunk + 128 decode tokens, contexts in [256,4096]
    "llama3-70b":  256 decode tokens, contexts in [1024,8192]
    "sweep":       llama3-70b stage, `budget` tokens at 1 prefill : 4 decode
    """
    if name == "tiny":
        ctx = [0, 0] + decode_contexts(seed, 6, 16, 100)
        return TINY, make_microbatch([32, 32] + [1] * 6, ctx, seed=seed)
    if name == "llama2-7b":
        ctx = decode_contexts(seed, 64, 512, 2048)
        return LLAMA2_7B_STAGE, make_microbatch([1] * 64, ctx, seed=seed)
    if name == "qwen2-7b":
        ctx = [0] + decode_contexts(seed, 128, 256, 4096)
        return QWEN2_7B_STAGE, make_microbatch([2048] + [1] * 128, ctx, seed=seed)
    if name == "llama3-70b":
        ctx = decode_contexts(seed, 256, 1024, 8192)
        return LLAMA3_70B_STAGE, make_microbatch([1] * 256, ctx, seed=seed)
    if name == "sweep":
        pt = int(round(budget / 5.0))
        dt = budget - pt
        k = draw_int_uniform(seed, 901, 1, 0, 3)[0]
        ctx = [k * pt] + decode_contexts(seed, dt, 512, 8192)
        return LLAMA3_70B_STAGE, make_microbatch([pt] + [1] * dt, ctx, seed=seed)
    raise KeyError(name)


# stream ids of the tensors of a stage (one per tensor kind; the layer index is added)
STREAM_HIDDEN = 1
STREAM_KV = 2
STREAM_EMBED = 3
STREAM_FINAL_NORM = 4
STREAM_LM_HEAD = 5
STREAM_TOKEN_IDS = 6
STREAM_LAYER_BASE = 100   # + 10*layer + {0..6 weights, 7 q/k/v bias, 8 query-head norm gain, 9 key-head norm gain}
_WEIGHT_KINDS = ("norm1", "wqkv", "wo", "norm2", "wgate", "wup", "wdown")


def weight_shapes(shape: StageShape) -> Dict[str, tuple]:
    h, d, f = shape.hidden, shape.head_dim, shape.ffn
    return {
        "norm1": (h,),
        "wqkv": (shape.qkv_out, h),        # q rows, then k rows, then v rows; [out, in]
        "wo": (h, shape.num_q_heads * d),
        "norm2": (h,),
        "wgate": (f, h),
        "wup": (f, h),
        "wdown": (h, f),
    }


def draw_layer_weights(shape: StageShape, layer: int, *, seed: int, device="cpu",
                       weight_std: Optional[float] = None, dtype: torch.dtype = torch.bfloat16) -> Dict[str, torch.Tensor]:
    """bf16 (or `dtype`) weights of one layer: matrices ~ N(0, std 0.02) (or std = `weight_std`, or
    1/sqrt(fan_in) when weight_std == "fan_in"), norm gains ~ 1 + N(0, 0.02)."""
    out = {}
    for k, kind in enumerate(_WEIGHT_KINDS):
        shp = weight_shapes(shape)[kind]
        n = 1
        for s in shp:
            n *= s
        stream = STREAM_LAYER_BASE + 10 * layer + k
        if kind.startswith("norm"):
            t = draw_normal_bf16(seed, stream, n, std=0.02, mean=1.0, device=device, dtype=dtype)
        else:
            if weight_std is None:
                std = 0.02
            elif weight_std == "fan_in":
                std = 1.0 / math.sqrt(shp[1])
            else:
                std = float(weight_std)
            t = draw_normal_bf16(seed, stream, n, std=std, device=device, dtype=dtype)
        out[kind] = t.view(*shp)
    return out


STREAM_W4_BASE = 100000   # + 20*layer + {0..4 code words, 5..9 scales, 10..14 zero points} of the five matrices
_W4_MATRICES = ("wqkv", "wo", "wgate", "wup", "wdown")


def draw_w4_layer(shape: StageShape, layer: int, *, seed: int, group: int, device="cpu",
                  weight_std: float = 0.02, dtype: torch.dtype = torch.bfloat16) -> Dict[str, torch.Tensor]:
    """One layer with 4-bit group-quantised projection matrices, drawn directly in their stored form:
    code words int32 [N, K/8] of uniformly random bits (every 4-bit code is uniform in 0..15), zero points
    bf16 [N, K/group], integers uniform in 6..9, scales bf16 [N, K/group] = weight_std/4.74 * u with u uniform
    in [0.75, 1.25) (code - zero has standard deviation 4.74, so the weights they stand for have about
    `weight_std`; `dtype` replaces bf16 for scales, zero points and gains; integer arithmetic and one float32 multiplication, so CPU and GPU draws are bit-identical).
    Keys: the matrix names hold the code words, "s"/"z" + {qkv,o,gate,up,down} the scales and zero points;
    the norm gains are those of `draw_layer_weights`."""
    device = torch.device(device)
    out = {}
    for k, kind in enumerate(_WEIGHT_KINDS):
        if kind.startswith("norm"):
            out[kind] = draw_normal_bf16(seed, STREAM_LAYER_BASE + 10 * layer + k, shape.hidden, std=0.02, mean=1.0,
                                         device=device, dtype=dtype)
    shapes = weight_shapes(shape)
    for m, kind in enumerate(_W4_MATRICES):
        n, kk = shapes[kind]
        if kk % group or kk % 8:
            raise ValueError(f"{kind}: {kk} input features are not a multiple of the group size {group}")
        base = STREAM_W4_BASE + 20 * layer
        words = n * (kk // 8)
        code = torch.empty(words, dtype=torch.int32, device=device)
        chunk = 1 << 24
        for start in range(0, words, chunk):
            idx = torch.arange(start, min(words, start + chunk), dtype=torch.int64, device=device)
            h = hash_u32(seed, base + m, idx)
            code[start:start + idx.numel()] = (h - ((h >> 31) << 32)).to(torch.int32)   # the same 32 bits, signed
        groups = n * (kk // group)
        gi = torch.arange(groups, dtype=torch.int64, device=device)
        scale = (768 + hash_u32(seed, base + 5 + m, gi) % 512).to(torch.float32) * \
            torch.tensor(weight_std / 4.74 / 1024.0, dtype=torch.float32, device=device)
        zero = 6 + hash_u32(seed, base + 10 + m, gi) % 4
        suffix = kind[1:]
        out[kind] = code.view(n, kk // 8)
        out["s" + suffix] = scale.to(dtype).view(n, kk // group)
        out["z" + suffix] = zero.to(dtype).view(n, kk // group)
    return out


def alibi_slopes(num_heads: int) -> torch.Tensor:
    """The head slopes of attention with linear biases as its authors define them: for a power of two n the geometric
    sequence 2^(-8/n), 2^(-16/n), ..., 2^(-8); otherwise the slopes of the largest power of two p below n, followed by
    every second slope (the first, third, ...) of 2p until n slopes are there.  float32 [num_heads] (model constants,
    inputs of both sides)."""
    def power_of_two(n):
        start = 2.0 ** (-8.0 / n)
        return [start ** (i + 1) for i in range(n)]
    p = 1
    while p * 2 <= num_heads:
        p *= 2
    slopes = power_of_two(p)
    if p < num_heads:
        slopes += power_of_two(2 * p)[0::2][: num_heads - p]
    return torch.tensor(slopes, dtype=torch.float32)


def draw_qkv_bias(shape: StageShape, layer: int, *, seed: int, device="cpu", std: float = 0.5,
                  dtype: torch.dtype = torch.bfloat16) -> torch.Tensor:
    """bf16 bias [qkv_out] of a layer's q/k/v projection ~ N(0, std) (for the stages that have one)."""
    return draw_normal_bf16(seed, STREAM_LAYER_BASE + 10 * layer + 7, shape.qkv_out, std=std, device=device, dtype=dtype)


STREAM_BLOCK_BIAS_BASE = 200000   # + 10*layer + {0 norm1_bias, 1 norm2_bias, 2 bo, 3 bup, 4 bdown}


def draw_block_biases(shape: StageShape, layer: int, *, seed: int, device="cpu", std: float = 0.25,
                      dtype: torch.dtype = torch.bfloat16) -> Dict[str, torch.Tensor]:
    """Biases ~ N(std, std) of the blocks that have them: of the two LayerNorms [hidden], of the attention's output
    projection [hidden], and of the two matrices of an ungated MLP ([ffn] and [hidden]).  Their mean is not zero, so
    that the rows of the residual stream they are added to get a mean of their own (which a LayerNorm removes)."""
    sizes = (("norm1_bias", shape.hidden), ("norm2_bias", shape.hidden), ("bo", shape.hidden), ("bup", shape.ffn),
             ("bdown", shape.hidden))
    return {name: draw_normal_bf16(seed, STREAM_BLOCK_BIAS_BASE + 10 * layer + k, n, std=std, mean=std, device=device,
                                   dtype=dtype)
            for k, (name, n) in enumerate(sizes)}


def draw_qk_norm(shape: StageShape, layer: int, *, seed: int, device="cpu", std: float = 0.25,
                 dtype: torch.dtype = torch.bfloat16) -> Dict[str, torch.Tensor]:
    """Gains [head_dim] ~ 1 + N(0, std) of a layer's per-head query and key norms (for the stages that have them)."""
    return {name: draw_normal_bf16(seed, STREAM_LAYER_BASE + 10 * layer + k, shape.head_dim, std=std, mean=1.0,
                                   device=device, dtype=dtype)
            for name, k in (("qnorm", 8), ("knorm", 9))}


def draw_hidden(shape: StageShape, num_tokens: int, *, seed: int, device="cpu",
                dtype: torch.dtype = torch.bfloat16) -> torch.Tensor:
    return draw_normal_bf16(seed, STREAM_HIDDEN, num_tokens * shape.hidden, device=device, dtype=dtype).view(
        num_tokens, shape.hidden)


def draw_ends_weights(shape: StageShape, *, seed: int, device="cpu", head_std: float = 0.02,
                      dtype: torch.dtype = torch.bfloat16) -> Dict[str, torch.Tensor]:
    """bf16 tensors of the pipeline's two ends: embedding table [vocab, hidden] ~ N(0, 1) (so the first
    stage's input has the scale of `draw_hidden`), final norm gain ~ 1 + N(0, 0.02), output head
    [vocab, hidden] ~ N(0, head_std)."""
    v, h = shape.vocab, shape.hidden
    return {
        "embed": draw_normal_bf16(seed, STREAM_EMBED, v * h, device=device, dtype=dtype).view(v, h),
        "final_norm": draw_normal_bf16(seed, STREAM_FINAL_NORM, h, std=0.02, mean=1.0, device=device, dtype=dtype),
        "lm_head": draw_normal_bf16(seed, STREAM_LM_HEAD, v * h, std=head_std, device=device, dtype=dtype).view(v, h),
    }


def draw_token_ids(shape: StageShape, num_tokens: int, *, seed: int) -> List[int]:
    return draw_int_uniform(seed, STREAM_TOKEN_IDS, num_tokens, 0, shape.vocab - 1)


def kv_value_index(shape: StageShape, num_kv_blocks: int, layer, kv, block, slot, head, dim):
    """Linear draw index of one cached K (kv=0) or V (kv=1) element.

    The index is a function of where the element logically lives (layer, physical block, slot
    in the block, kv head, dim); it is the generator's own numbering, not a memory layout.
    All arguments broadcast; integer tensors or ints.
    """
    b, nkv, d = shape.kv_block_size, shape.num_kv_heads, shape.head_dim
    return ((((layer * 2 + kv) * num_kv_blocks + block) * b + slot) * nkv + head) * d + dim


def draw_kv_blocks(shape: StageShape, num_kv_blocks: int, layer: int, kv: int, blocks: torch.Tensor,
                   *, seed: int, dtype: torch.dtype = torch.bfloat16) -> torch.Tensor:
    """Cached values of the given physical blocks: bf16 [len(blocks), block, nkv, d] ~ N(0,1)."""
    dev = blocks.device
    b, nkv, d = shape.kv_block_size, shape.num_kv_heads, shape.head_dim
    blk = blocks.to(torch.int64).view(-1, 1, 1, 1)
    slot = torch.arange(b, dtype=torch.int64, device=dev).view(1, b, 1, 1)
    head = torch.arange(nkv, dtype=torch.int64, device=dev).view(1, 1, nkv, 1)
    dim = torch.arange(d, dtype=torch.int64, device=dev).view(1, 1, 1, d)
    idx = kv_value_index(shape, num_kv_blocks, layer, kv, blk, slot, head, dim)
    return draw_normal_bf16_at(seed, STREAM_KV, idx, dtype=dtype)


def valid_slot_mask(mb: MicroBatch, block: int = 16, *, include_new: bool = False) -> torch.Tensor:
    """bool [num_kv_blocks, block]: slots that hold cached context before the call
    (or, with include_new, context plus this call's new tokens)."""
    mask = torch.zeros(mb.num_kv_blocks, block, dtype=torch.bool)
    for s, (q, c) in enumerate(zip(mb.q_lens, mb.ctx_lens)):
        n = c + q if include_new else c
        full, rem = divmod(n, block)
        row = mb.block_tables[s].to(torch.int64)
        if full:
            mask[row[:full]] = True
        if rem:
            mask[row[full], :rem] = True
    return mask
