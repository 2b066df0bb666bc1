"""Startup profiling of a stage: computation latency across batch sizes and sequence lengths.

The serving system's scheduler sizes its micro-batches from a table every engine measures when it
starts: how long the engine's layers take for a given number of sequences and context length (paper
section 4.1, the first of the two profiling phases).  This module produces that table for a `Stage`
by timing stage_forward on synthetic micro-batches; it holds no arithmetic of the method.

The measurement appends to the KV pool (as every forward pass does) and leaves the cached values it
finds untouched otherwise: run it before the pool holds live sequences.
"""
from __future__ import annotations

from typing import Dict, Iterable, List, Tuple

import torch

from .stage import Stage


def _decode_batch(stage: Stage, num_seqs: int, ctx_len: int):
    """A decode micro-batch of `num_seqs` sequences with `ctx_len` cached tokens each, paged one
    sequence after another from block 0 (identity paging)."""
    c = stage.cfg
    blocks_per_seq = (ctx_len + 1 + 15) // 16
    if num_seqs > c.max_seqs or num_seqs > c.max_tokens:
        raise ValueError(f"{num_seqs} sequences exceed the stage's capacity")
    if blocks_per_seq > c.max_blocks_per_seq or num_seqs * blocks_per_seq > c.num_kv_blocks:
        raise ValueError(f"{num_seqs} sequences of {ctx_len} cached tokens exceed the KV pool")
    tables = torch.full((num_seqs, c.max_blocks_per_seq), -1, dtype=torch.int32)
    for s in range(num_seqs):
        tables[s, :blocks_per_seq] = torch.arange(s * blocks_per_seq, (s + 1) * blocks_per_seq, dtype=torch.int32)
    return [ctx_len] * num_seqs, [1] * num_seqs, [ctx_len] * num_seqs, tables


def _prefill_batch(stage: Stage, chunk_len: int, ctx_len: int):
    c = stage.cfg
    blocks = (ctx_len + chunk_len + 15) // 16
    if chunk_len > c.max_tokens or blocks > c.max_blocks_per_seq or blocks > c.num_kv_blocks:
        raise ValueError(f"a chunk of {chunk_len} tokens after {ctx_len} exceeds the stage's capacity")
    tables = torch.full((1, c.max_blocks_per_seq), -1, dtype=torch.int32)
    tables[0, :blocks] = torch.arange(blocks, dtype=torch.int32)
    return list(range(ctx_len, ctx_len + chunk_len)), [chunk_len], [ctx_len], tables


def _time(stage: Stage, positions, q_lens, ctx_lens, tables, warmup: int, iters: int) -> float:
    t = sum(q_lens)
    hidden = torch.zeros(t, stage.cfg.hidden, dtype=torch.bfloat16, device=stage.device)
    out = torch.empty_like(hidden)
    for _ in range(warmup):
        stage.forward(hidden, positions, q_lens, ctx_lens, tables, out=out)
    stream = torch.cuda.current_stream(stage.device)
    begin, end = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    begin.record(stream)
    for _ in range(iters):
        stage.forward(hidden, positions, q_lens, ctx_lens, tables, out=out)
    end.record(stream)
    end.synchronize()
    return begin.elapsed_time(end) / iters


def profile_decode(stage: Stage, batch_sizes: Iterable[int], ctx_lens: Iterable[int], *, warmup: int = 2,
                   iters: int = 5) -> Dict[Tuple[int, int], float]:
    """{(num_seqs, ctx_len): milliseconds per micro-batch} for pure-decode micro-batches."""
    table = {}
    for b in batch_sizes:
        for c in ctx_lens:
            table[(b, c)] = _time(stage, *_decode_batch(stage, b, c), warmup, iters)
    return table


def profile_prefill(stage: Stage, chunk_lens: Iterable[int], ctx_lens: Iterable[int] = (0,), *, warmup: int = 2,
                    iters: int = 5) -> Dict[Tuple[int, int], float]:
    """{(chunk_len, ctx_len): milliseconds per micro-batch} for one prefill chunk after ctx_len cached tokens."""
    table = {}
    for n in chunk_lens:
        for c in ctx_lens:
            table[(n, c)] = _time(stage, *_prefill_batch(stage, n, c), warmup, iters)
    return table


def format_table(table: Dict[Tuple[int, int], float], row_name: str, col_name: str) -> List[str]:
    rows = sorted({k[0] for k in table})
    cols = sorted({k[1] for k in table})
    lines = [f"{row_name} \\ {col_name} " + " ".join(f"{c:>9d}" for c in cols)]
    for r in rows:
        lines.append(f"{r:>12d} " + " ".join(f"{table[(r, c)]:9.3f}" for c in cols))
    return lines
