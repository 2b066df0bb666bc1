"""Plain CPU oracle of the two ends of the pipeline: token embedding before the
first stage, and final norm + vocabulary projection + greedy choice after the last.

TEST INFRASTRUCTURE.  Slow, unfused, written for checking by eye.  It shares no
code with the HIP library and must not be imported by it.

What it computes.  The head engine receives requests and feeds the first run
of layers; the engines after it receive intermediate activations; the system's
throughput is counted in generated tokens (paper section 3.2.2 "Distributed
Inference Engine"; section 5 "Metrics").  The paper leaves both ends to its
engine runtime and evaluates Llama-family models (section 5, "Models"), so the
definitions used here are that family's: the embedding is a row gather from a
[vocab, hidden] table; the output head is RMSNorm with its own gain, then a
bias-free projection onto the vocabulary, applied to the LAST row of every
sequence of the micro-batch (the only row whose next token is not already
known); greedy decoding takes the index of the largest logit, the smallest
index among equals.

Numerics: inputs are widened to `dtype` (float64 by default) on entry and
nothing is rounded afterwards.  Library primitive used as a step: matmul.

Pins (tests/test_oracle_ends_pins.py): scalar-loop brute force on tiny shapes;
gather against direct indexing of hand-written tables; an identity-like head
whose logits are the normalised activations themselves; invariance of the
logits under positive scaling of the hidden rows (up to eps); permutation of
vocabulary rows permutes logits; rows other than each sequence's last have no
influence; ties resolve to the smallest index; the LayerNorm head against the
library's layer_norm followed by a matmul, scalar loops, and invariance to a
shift of the hidden rows.  The paper prints no numeric
values for this path: parity against printed values is unpinned; parity is
against the definition.
"""
from __future__ import annotations

from typing import Sequence

import torch


def embed_tokens(table: torch.Tensor, token_ids: Sequence[int], dtype=torch.float64) -> torch.Tensor:
    """hidden[t] = table[token_ids[t]].  table: [vocab, hidden]; returns [T, hidden]."""
    vocab = table.shape[0]
    rows = []
    for tok in token_ids:
        tok = int(tok)
        if not 0 <= tok < vocab:
            raise ValueError(f"token id {tok} outside [0, {vocab})")
        rows.append(table[tok].to(dtype))
    if not rows:
        return torch.zeros((0, table.shape[1]), dtype=dtype)
    return torch.stack(rows)


def last_rows(q_lens: Sequence[int]) -> list:
    """Row index, in the packed [T, hidden] layout, of the last token of every sequence."""
    out, start = [], 0
    for q in q_lens:
        q = int(q)
        if q < 1:
            raise ValueError("every sequence contributes at least one row")
        out.append(start + q - 1)
        start += q
    return out


def head_logits(hidden: torch.Tensor, q_lens: Sequence[int], gain: torch.Tensor, w_vocab: torch.Tensor,
                eps: float, dtype=torch.float64, norm_kind: str = "rms", bias: torch.Tensor = None) -> torch.Tensor:
    """logits[s] = norm(hidden[last row of s]) @ w_vocab^T.  Returns [S, vocab].

    norm_kind "rms": x * gain / sqrt(mean(x^2) + eps).  "layer" (the families whose blocks use LayerNorms end with
    one too): (x - mean) / sqrt(mean((x - mean)^2) + eps) * gain (+ bias)."""
    idx = last_rows(q_lens)
    if sum(int(q) for q in q_lens) != hidden.shape[0]:
        raise ValueError("q_lens do not add up to the number of rows")
    x = hidden.to(dtype)[idx]                                        # [S, hidden]
    if norm_kind == "layer":
        dev = x - x.mean(dim=-1, keepdim=True)
        var = (dev * dev).mean(dim=-1, keepdim=True)
        xn = dev / torch.sqrt(var + eps) * gain.to(dtype)
        if bias is not None:
            xn = xn + bias.to(dtype)
    else:
        if norm_kind != "rms" or bias is not None:
            raise ValueError("an RMSNorm head has no bias")
        ms = (x * x).mean(dim=-1, keepdim=True)
        xn = x * gain.to(dtype) / torch.sqrt(ms + eps)
    return xn @ w_vocab.to(dtype).T


def greedy_tokens(logits: torch.Tensor) -> torch.Tensor:
    """Index of the largest logit of every row; among equal maxima the smallest index."""
    s, v = logits.shape
    out = torch.empty(s, dtype=torch.int64)
    for r in range(s):
        row = logits[r]
        best = row.max()
        out[r] = int(torch.nonzero(row == best).flatten()[0])
    return out
