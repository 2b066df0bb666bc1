"""Shared test plumbing: turn synthetic draws into oracle inputs (no arithmetic of the method)."""
from __future__ import annotations

from typing import Dict, List

import torch

import oracle
from paper_2507_05043_amd import synth


def oracle_shape(shape: synth.StageShape) -> oracle.OracleShape:
    return oracle.OracleShape(shape.num_layers, shape.hidden, shape.num_q_heads, shape.num_kv_heads,
                              shape.head_dim, shape.ffn, shape.rms_eps, shape.rope_theta,
                              shape.kv_block_size, shape.rotary_dim, shape.rope_interleaved,
                              shape.norm_kind, shape.mlp_kind, shape.parallel_block, shape.rope_scaling)


def draw_layers(shape: synth.StageShape, seed: int, weight_std=None, device="cpu",
                qkv_bias: bool = False, elem: torch.dtype = torch.bfloat16,
                qk_norm: bool = False, alibi=False, block_biases: bool = False,
                shared_norm: bool = False) -> List[Dict[str, torch.Tensor]]:
    """block_biases: the norms' biases (LayerNorm shapes only), bo, bdown, and for an ungated MLP bup.
    shared_norm (parallel blocks): no second norm - both branches read the first.  An ungated MLP has no wgate."""
    layers = [synth.draw_layer_weights(shape, l, seed=seed, device=device, weight_std=weight_std, dtype=elem)
              for l in range(shape.num_layers)]
    for l, w in enumerate(layers):
        if shape.mlp_kind != "swiglu":
            del w["wgate"]
        if block_biases:
            b = synth.draw_block_biases(shape, l, seed=seed, device=device, dtype=elem)
            if shape.norm_kind != "layer":
                del b["norm1_bias"], b["norm2_bias"]
            if shape.mlp_kind == "swiglu":
                del b["bup"]
            w.update(b)
        if shared_norm:
            del w["norm2"]
            w.pop("norm2_bias", None)
    if qkv_bias:
        for l, w in enumerate(layers):
            w["bqkv"] = synth.draw_qkv_bias(shape, l, seed=seed, device=device, dtype=elem)
    if qk_norm:
        for l, w in enumerate(layers):
            w.update(synth.draw_qk_norm(shape, l, seed=seed, device=device, dtype=elem))
    if alibi:
        for w in layers:
            slopes = synth.alibi_slopes(shape.num_q_heads).to(device)
            w["alibi"] = slopes * 0 if alibi == "zero" else slopes
    return layers


def oracle_pool(shape: synth.StageShape, mb: synth.MicroBatch, seed: int, dtype=torch.float64,
                elem: torch.dtype = torch.bfloat16) -> torch.Tensor:
    """Oracle-layout pool [L, 2, blocks, slot, nkv, d]: cached context drawn (as 16-bit `elem` values, widened to
    `dtype`), everything else NaN."""
    osh = oracle_shape(shape)
    pool = oracle.new_pool(osh, mb.num_kv_blocks, dtype=dtype)
    valid = synth.valid_slot_mask(mb, shape.kv_block_size)                 # [blocks, slot]
    used_blocks = torch.nonzero(valid.any(dim=1)).flatten()
    if used_blocks.numel() == 0:
        return pool
    for l in range(shape.num_layers):
        for kv in (0, 1):
            vals = synth.draw_kv_blocks(shape, mb.num_kv_blocks, l, kv, used_blocks, seed=seed, dtype=elem).to(dtype)
            m = valid[used_blocks].view(-1, shape.kv_block_size, 1, 1)
            vals = torch.where(m, vals, torch.full_like(vals, float("nan")))
            pool[l, kv, used_blocks] = vals
    return pool


def rel_l2(a: torch.Tensor, b: torch.Tensor) -> float:
    a = a.double()
    b = b.double()
    return float((a - b).norm() / b.norm().clamp_min(1e-300))
