"""Startup profiling of a stage: computation latency across batch sizes and sequence lengths.

The serving system's scheduler sizes its micro-batches from a table every engine measures when it
starts: how long the engine's layers take for a given number of sequences and context length (paper
section 4.1, the first of the two profiling phases).  This module produces that table for a `Stage`
from the library's stage_profile call (one point per call: synthetic micro-batch, identity paging, timed with
events on the stream); it holds no arithmetic of the method.

The measurement appends to the KV pool (as every forward pass does) and leaves the cached values it
finds untouched otherwise: run it before the pool holds live sequences.
"""
from __future__ import annotations

from typing import Dict, Iterable, List, Tuple

from .stage import Stage


def profile_decode(stage: Stage, batch_sizes: Iterable[int], ctx_lens: Iterable[int], *, warmup: int = 2,
                   iters: int = 5) -> Dict[Tuple[int, int], float]:
    """{(num_seqs, ctx_len): milliseconds per micro-batch} for pure-decode micro-batches."""
    table = {}
    for b in batch_sizes:
        for c in ctx_lens:
            table[(b, c)] = stage.profile(b, 1, c, warmup=warmup, iters=iters)
    return table


def profile_prefill(stage: Stage, chunk_lens: Iterable[int], ctx_lens: Iterable[int] = (0,), *, warmup: int = 2,
                    iters: int = 5) -> Dict[Tuple[int, int], float]:
    """{(chunk_len, ctx_len): milliseconds per micro-batch} for one prefill chunk after ctx_len cached tokens."""
    table = {}
    for n in chunk_lens:
        for c in ctx_lens:
            table[(n, c)] = stage.profile(1, n, c, warmup=warmup, iters=iters)
    return table


def format_table(table: Dict[Tuple[int, int], float], row_name: str, col_name: str) -> List[str]:
    rows = sorted({k[0] for k in table})
    cols = sorted({k[1] for k in table})
    lines = [f"{row_name} \\ {col_name} " + " ".join(f"{c:>9d}" for c in cols)]
    for r in rows:
        lines.append(f"{r:>12d} " + " ".join(f"{table[(r, c)]:9.3f}" for c in cols))
    return lines
