"""Build the same seeded problem for the HIP library (on the GPU) and for the oracle (on the CPU),
and compare the two.  No arithmetic of the method lives here."""
from __future__ import annotations

import math
from typing import Dict, List, Optional, Sequence

import torch

import oracle
from paper_2507_05043_amd import Stage, synth
from paper_2507_05043_amd.harness import fill_pool, make_stage  # noqa: F401
from tests.helpers import draw_layers, oracle_pool, oracle_shape, rel_l2

REL_L2_TOL = 1e-2      # stated tolerance on bf16 output hidden states
MAX_ABS_TOL = 5e-2     # stated max-abs tolerance, scaled by max(1, rms(oracle)) beyond unit scale


def run_gpu(st: Stage, shape, mb, seed, taps_layer=None, hidden=None):
    hidden = hidden if hidden is not None else synth.draw_hidden(shape, mb.num_tokens, seed=seed, device=st.device,
                                                                 dtype=st.dtype)
    res = st.forward(hidden, mb.positions, mb.q_lens, mb.ctx_lens, mb.block_tables, want_slots=True,
                     taps_layer=taps_layer)
    torch.cuda.synchronize()
    return res


def run_oracle(shape, mb, seed, weight_std=None, dtype=torch.float64, want_taps=False, layers=None,
               elem=torch.bfloat16):
    """`elem`: the 16-bit type the inputs are drawn in (the oracle widens them exactly and computes in `dtype`)."""
    layers = layers if layers is not None else draw_layers(shape, seed, weight_std, elem=elem)
    hidden = synth.draw_hidden(shape, mb.num_tokens, seed=seed, dtype=elem)
    pool = oracle_pool(shape, mb, seed, dtype=dtype, elem=elem)
    taps = [] if want_taps else None
    out, slots = oracle.stage_forward(oracle_shape(shape), layers, hidden, mb.positions, mb.q_lens, mb.ctx_lens,
                                      mb.block_tables, pool, dtype=dtype, taps=taps)
    return out, slots, pool, taps


def check_output(gpu_out: torch.Tensor, ref: torch.Tensor, what: str = "output") -> Dict[str, float]:
    got = gpu_out.detach().cpu().double()
    ref = ref.double()
    assert torch.isfinite(got).all(), f"{what}: non-finite values"
    r = rel_l2(got, ref)
    rms = float(ref.pow(2).mean().sqrt())
    max_abs = float((got - ref).abs().max())
    bound = MAX_ABS_TOL * max(1.0, rms)
    assert r <= REL_L2_TOL, f"{what}: rel-L2 {r:.3e} > {REL_L2_TOL}"
    assert max_abs <= bound, f"{what}: max-abs {max_abs:.3e} > {bound:.3e} (rms {rms:.3f})"
    return {"rel_l2": r, "max_abs": max_abs, "rms": rms}


def check_output_stratified(gpu_out: torch.Tensor, ref: torch.Tensor, strata, what: str = "output",
                            gate_max_abs: bool = True, gate_strata: bool = False) -> Dict[str, float]:
    """The whole-output metric estimated from a stratified sample of rows.

    strata: list of (row_slice_into_the_sample, rows_in_the_population).  Every sampled row of a
    stratum stands for population/sample rows, so the sums of squared error and of squared reference
    are scaled per stratum before the ratio is taken (rows of a stratum are exact; only which
    sequences were drawn is a sample).  Also reports every stratum on its own, and with gate_strata holds
    every stratum to the tolerance by itself, so that many good rows cannot outvote a few bad ones.
    """
    got = gpu_out.detach().cpu().double()
    ref = ref.double()
    assert torch.isfinite(got).all(), f"{what}: non-finite values"
    num = den = 0.0
    per = []
    max_abs = 0.0
    for sl, population in strata:
        g, r = got[sl], ref[sl]
        w = population / g.shape[0]
        num += w * float((g - r).pow(2).sum())
        den += w * float(r.pow(2).sum())
        per.append(rel_l2(g, r))
        max_abs = max(max_abs, float((g - r).abs().max()))
    est = (num / den) ** 0.5
    rms = float(ref.pow(2).mean().sqrt())
    assert est <= REL_L2_TOL, f"{what}: estimated whole-output rel-L2 {est:.3e} > {REL_L2_TOL} (strata {per})"
    if gate_strata:
        assert max(per) <= REL_L2_TOL, f"{what}: a stratum's rel-L2 exceeds {REL_L2_TOL}: {per}"
    if gate_max_abs:
        assert max_abs <= MAX_ABS_TOL * max(1.0, rms), f"{what}: max-abs {max_abs:.3e} (rms {rms:.3f})"
    return {"rel_l2": est, "per_stratum": per, "max_abs": max_abs, "rms": rms}


def check_taps(gpu_taps: Dict[str, torch.Tensor], otap: Dict[str, torch.Tensor], x_in: torch.Tensor,
               x_in_gpu: torch.Tensor, label: str):
    """Every sub-layer output, and the two residual branches on their own, within the rel-L2 tolerance.
    A branch is what a sub-layer adds to the residual stream: each side's own output minus its own input."""
    cpu = {k: v.detach().cpu().double() for k, v in gpu_taps.items()}
    t = x_in.shape[0]
    o_qkv = torch.cat([otap["q"].reshape(t, -1), otap["k"].reshape(t, -1), otap["v"].reshape(t, -1)], dim=1)
    pairs = {
        "norm1": (cpu["a"], otap["a"]), "qkv": (cpu["qkv"], o_qkv), "attn": (cpu["attn"], otap["attn"]),
        "h": (cpu["h"], otap["h"]), "mlp": (cpu["m"], otap["m"]), "x": (cpu["x"], otap["x"]),
        "attn_branch": (cpu["h"] - x_in_gpu.detach().cpu().double(), otap["h"] - x_in.double()),
        "mlp_branch": (cpu["x"] - cpu["h"], otap["x"] - otap["h"]),
    }
    errs = {}
    for name, (g, o) in pairs.items():
        assert torch.isfinite(g).all(), f"{label} tap {name}: non-finite"
        errs[name] = rel_l2(g, o)
    bad = {k: v for k, v in errs.items() if v > REL_L2_TOL}
    assert not bad, f"{label}: taps over tolerance {bad} (all: {errs})"
    return errs


def check_pool(st: Stage, shape, mb, oracle_pool_after: torch.Tensor, before: List[List[torch.Tensor]], slots):
    """Exactly the new tokens' slots changed; their values match the oracle's; the rest is bit-identical."""
    blocks = torch.arange(mb.num_kv_blocks, device=st.device)
    nb, b = mb.num_kv_blocks, shape.kv_block_size
    want = torch.zeros(nb * b, dtype=torch.bool)
    want[slots] = True
    for l in range(shape.num_layers):
        for kv in (0, 1):
            after = st.read_kv_blocks(l, kv, blocks).cpu().reshape(nb * b, -1)
            prev = before[l][kv].reshape(nb * b, -1)
            same = (after.view(torch.int16) == prev.view(torch.int16)).all(dim=1)
            # every untouched slot is bit-identical, every mapped slot was written
            assert bool(same[~want].all()), f"layer {l} kv {kv}: a slot outside the slot mapping changed"
            assert not bool(same[want].any()), f"layer {l} kv {kv}: a mapped slot was not written"
            got = after[want].double()
            ref = oracle_pool_after[l, kv].reshape(nb * b, -1)[want].double()
            assert torch.isfinite(got).all()
            r = rel_l2(got, ref)
            assert r <= REL_L2_TOL, f"layer {l} kv {kv}: appended values rel-L2 {r:.3e}"


def snapshot_pool(st: Stage, shape, mb) -> List[List[torch.Tensor]]:
    blocks = torch.arange(mb.num_kv_blocks, device=st.device)
    return [[st.read_kv_blocks(l, kv, blocks).cpu().clone() for kv in (0, 1)] for l in range(shape.num_layers)]


def sub_problem(shape: synth.StageShape, mb: synth.MicroBatch, seqs: Sequence[int], seed: int, dtype=torch.float64,
                draw_device="cpu", elem=torch.bfloat16):
    """The oracle's view of a subset of sequences: their rows, a compact re-paged pool holding the
    same cached values (drawn by their original physical block numbers), compact block tables."""
    b = shape.kv_block_size
    cu = [0]
    for q in mb.q_lens:
        cu.append(cu[-1] + q)
    rows = torch.cat([torch.arange(cu[s], cu[s + 1]) for s in seqs])
    q_lens = [mb.q_lens[s] for s in seqs]
    ctx_lens = [mb.ctx_lens[s] for s in seqs]
    need = [synth.blocks_needed(q + c, b) for q, c in zip(q_lens, ctx_lens)]
    total = sum(need)
    width = max(need)
    table = torch.full((len(seqs), width), -1, dtype=torch.int32)
    orig = []
    cur = 0
    for i, (s, nbk) in enumerate(zip(seqs, need)):
        table[i, :nbk] = torch.arange(cur, cur + nbk, dtype=torch.int32)
        orig.append(mb.block_tables[s, :nbk].to(torch.int64))
        cur += nbk
    orig = torch.cat(orig)
    sub = synth.MicroBatch(q_lens, ctx_lens, table, mb.positions[rows], total)
    pool = oracle.new_pool(oracle_shape(shape), total, dtype=dtype)
    valid = synth.valid_slot_mask(sub, b).view(total, b, 1, 1)
    for l in range(shape.num_layers):
        for kv in (0, 1):
            # the generator gives the same bits on either device; drawing on the GPU is only faster
            vals = synth.draw_kv_blocks(shape, mb.num_kv_blocks, l, kv, orig.to(draw_device), seed=seed,
                                        dtype=elem).cpu().to(dtype)
            pool[l, kv] = torch.where(valid, vals, torch.full_like(vals, float("nan")))
    return sub, rows, pool
