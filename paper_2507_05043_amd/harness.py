"""Set a stage up on the GPU from the seeded synthetic draws (device memory plumbing only)."""
from __future__ import annotations

from typing import Optional

import torch

from . import synth
from .stage import Stage, make_config


def make_stage(shape: synth.StageShape, mb: synth.MicroBatch, seed: int, weight_std=None,
               max_tokens: Optional[int] = None, alias_layers: bool = False, fill_kv: bool = True,
               device: str = "cuda:0", activation_planes: int = 0, vocab_size: int = 0,
               qkv_bias: bool = False, weight_group_size: int = 0, dtype: torch.dtype = torch.bfloat16,
               qk_norm: bool = False, weight_copies: int = 0, alibi=False, block_biases: bool = False,
               shared_norm: bool = False, pool_first: bool = False) -> Stage:
    """Draw the stage's weights on the device, size the pool and workspace for `mb`, fill the cache.
    weight_group_size > 0: 4-bit group-quantised projection weights with that group size.
    dtype: the 16-bit element type (bfloat16, or float16 for the half-precision library).
    qk_norm: per-head RMSNorm gains for queries and keys (the Qwen3 family's block).
    weight_copies: 1 = the stage keeps no second copy of its weights in operand order.
    alibi: attention with linear biases (the published head slopes; "zero": all slopes zero, a block without
    positions) instead of the rotary embedding.
    block_biases: the biases the shape's block kind can carry (of its LayerNorms, of the output and down projections,
    of an ungated MLP's first matrix).  shared_norm: a parallel block whose two branches read one norm.
    The block's kind itself (norm_kind, mlp_kind, parallel_block) comes with the shape.
    pool_first: allocate the KV pool before the weights are drawn (an engine reserves its cache when it starts)."""
    cfg = make_config(num_layers=shape.num_layers, hidden=shape.hidden, num_q_heads=shape.num_q_heads,
                      num_kv_heads=shape.num_kv_heads, head_dim=shape.head_dim, ffn=shape.ffn,
                      rms_eps=shape.rms_eps, rope_theta=shape.rope_theta, num_kv_blocks=mb.num_kv_blocks,
                      max_tokens=max_tokens or mb.num_tokens, max_seqs=mb.num_seqs,
                      max_blocks_per_seq=mb.max_blocks_per_seq,
                      kv_layer_stride_bytes=0 if alias_layers else None, activation_planes=activation_planes,
                      vocab_size=vocab_size, weight_bits=4 if weight_group_size else 0,
                      weight_group_size=weight_group_size, rotary_dim=shape.rotary_dim, weight_copies=weight_copies,
                      rope_interleaved=int(shape.rope_interleaved), norm_kind=shape.norm_kind, mlp_kind=shape.mlp_kind,
                      parallel_block=int(shape.parallel_block), rope_scaling=shape.rope_scaling)
    kv_pool = None
    if pool_first:
        from .stage import stage_kv_layer_bytes
        pool_bytes = (cfg.num_layers - 1) * cfg.kv_layer_stride_bytes + stage_kv_layer_bytes(cfg)
        kv_pool = torch.empty(pool_bytes, dtype=torch.uint8, device=device)
    if weight_group_size:
        layers = [synth.draw_w4_layer(shape, l, seed=seed, group=weight_group_size, device=device,
                                      weight_std=0.02 if weight_std is None else float(weight_std), dtype=dtype)
                  for l in range(shape.num_layers)]
    else:
        layers = [synth.draw_layer_weights(shape, l, seed=seed, device=device, weight_std=weight_std, dtype=dtype)
                  for l in range(shape.num_layers)]
    if qkv_bias:
        for l, w in enumerate(layers):
            w["bqkv"] = synth.draw_qkv_bias(shape, l, seed=seed, device=device, dtype=dtype)
    if qk_norm:
        for l, w in enumerate(layers):
            w.update(synth.draw_qk_norm(shape, l, seed=seed, device=device, dtype=dtype))
    if alibi:
        for w in layers:
            slopes = synth.alibi_slopes(shape.num_q_heads).to(device)
            w["alibi"] = slopes * 0 if alibi == "zero" else slopes
    for l, w in enumerate(layers):
        if shape.mlp_kind != "swiglu":
            del w["wgate"]
        if block_biases:
            b = synth.draw_block_biases(shape, l, seed=seed, device=device, dtype=dtype)
            if shape.norm_kind != "layer":
                del b["norm1_bias"], b["norm2_bias"]
            if shape.mlp_kind == "swiglu":
                del b["bup"]
            w.update(b)
        if shared_norm:
            del w["norm2"]
            w.pop("norm2_bias", None)
    st = Stage(cfg, layers, device=device, dtype=dtype, kv_pool=kv_pool)
    if fill_kv:
        fill_pool(st, shape, mb, seed)
    return st


def fill_pool(st: Stage, shape: synth.StageShape, mb: synth.MicroBatch, seed: int, progress: bool = False) -> None:
    """Cached context drawn into its slots; every other slot of the pool is NaN."""
    st.kv_pool.view(st.dtype).fill_(float("nan"))
    valid = synth.valid_slot_mask(mb, shape.kv_block_size)
    used = torch.nonzero(valid.any(dim=1)).flatten()
    if used.numel() == 0:
        return
    used_dev = used.to(st.device)
    m = valid[used].to(st.device).view(-1, shape.kv_block_size, 1, 1)
    nan = torch.tensor(float("nan"), dtype=st.dtype, device=st.device)
    layers = 1 if st.cfg.kv_layer_stride_bytes == 0 else shape.num_layers
    step = 4096
    for l in range(layers):
        for kv in (0, 1):
            for i in range(0, used_dev.numel(), step):
                blk = used_dev[i:i + step]
                vals = synth.draw_kv_blocks(shape, mb.num_kv_blocks, l, kv, blk, seed=seed, dtype=st.dtype)
                vals = torch.where(m[i:i + step], vals, nan)
                st.write_kv_blocks(l, kv, blk, vals)
        if progress:
            print(f"  KV pool of layer {l} filled", flush=True)
