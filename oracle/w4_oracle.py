"""Plain CPU oracle of the 4-bit group-quantised weight format.

TEST INFRASTRUCTURE.  Slow, unfused, written for checking by eye.  It shares no
code with the HIP library and must not be imported by it.

What it defines.  The paper runs its 70B model with 4-bit quantised weights
(section 5, "Models"; section 5.2, "Rent the cloud devices", names a 4-bit
AWQ checkpoint) and says nothing about the format, so the format is this repository's, of the usual
group-quantised kind: a weight matrix W [N, K] (N output features, K input
features) is stored as
    code words   32-bit [N, K/8]; element k of a row is the 4-bit field at bits
                 4*(k mod 8) .. 4*(k mod 8)+3 of word k // 8 (least significant first),
    scales       [N, K/group],
    zero points  [N, K/group]  (in code units),
and stands for
    W[n, k] = (code[n, k] - zero[n, k // group]) * scale[n, k // group].
A stage with such weights computes exactly what the stage oracle computes with
the matrices W in place of the bf16 ones: `dequantize` produces them (float64,
nothing rounded) and its result is passed to `stage_forward` unchanged.

`quantize` is the usual asymmetric min/max rule per group; it exists for the
tests (round trips), the stage never quantises.

Pins (tests/test_oracle_w4_pins.py): hand-written words against hand-written
codes; the field order against Python integer arithmetic on random words; the
formula on literal numbers; group boundaries (a change of one group's scale or
zero point moves exactly that group's columns); the round trip
quantize -> dequantize within half a scale step, exact for matrices that lie
on the grid; a stage whose bf16 weights lie on a grid gives the same output
from either representation.  The paper prints no values for this: parity
against printed values is unpinned; parity is against the definition.
"""
from __future__ import annotations

import torch


def unpack_codes(words: torch.Tensor) -> torch.Tensor:
    """words: integer tensor [N, K/8] holding 32-bit words (signed or unsigned storage; only the low 32
    bits count).  Returns the codes, int64 [N, K], each in 0..15."""
    w = words.to(torch.int64) & 0xFFFFFFFF
    n, nw = w.shape
    codes = torch.empty(n, nw * 8, dtype=torch.int64)
    for i in range(8):
        codes[:, i::8] = (w >> (4 * i)) & 15
    return codes


def dequantize(words: torch.Tensor, scales: torch.Tensor, zeros: torch.Tensor, group: int,
               dtype=torch.float64) -> torch.Tensor:
    """W[n, k] = (code[n, k] - zero[n, k // group]) * scale[n, k // group], in `dtype`, nothing rounded."""
    codes = unpack_codes(words.cpu())
    n, k = codes.shape
    assert k % group == 0 and tuple(scales.shape) == (n, k // group) == tuple(zeros.shape)
    s = scales.cpu().to(dtype).repeat_interleave(group, dim=1)
    z = zeros.cpu().to(dtype).repeat_interleave(group, dim=1)
    return (codes.to(dtype) - z) * s


def quantize(w: torch.Tensor, group: int):
    """Asymmetric min/max quantisation per group of `group` consecutive input features:
    scale = (max - min) / 15 (1 where the group is constant), zero = round(-min / scale) clamped to 0..15,
    code = round(w / scale + zero) clamped to 0..15.  Returns (words int64 [N, K/8], scales, zeros) in float64."""
    w = w.to(torch.float64)
    n, k = w.shape
    assert k % group == 0 and k % 8 == 0
    g = w.view(n, k // group, group)
    lo, hi = g.min(dim=2).values, g.max(dim=2).values
    scale = (hi - lo) / 15.0
    scale = torch.where(scale > 0, scale, torch.ones_like(scale))
    zero = torch.clamp(torch.round(-lo / scale), 0, 15)
    code = torch.clamp(torch.round(g / scale.unsqueeze(2) + zero.unsqueeze(2)), 0, 15).to(torch.int64).view(n, k)
    words = torch.zeros(n, k // 8, dtype=torch.int64)
    for i in range(8):
        words |= code[:, i::8] << (4 * i)
    return words, scale, zero


def dequantize_layer(layer: dict, group: int, dtype=torch.float64) -> dict:
    """A layer given in stored form (matrix names -> code words, 's'/'z' + name[1:] -> scales / zero points,
    everything else as it is) turned into the dict of plain matrices the stage oracle takes."""
    out = {}
    for name, t in layer.items():
        if name in ("wqkv", "wo", "wgate", "wup", "wdown"):
            out[name] = dequantize(t, layer["s" + name[1:]], layer["z" + name[1:]], group, dtype)
        elif name[0] in "sz" and ("w" + name[1:]) in layer and name[1:] in ("qkv", "o", "gate", "up", "down"):
            continue
        else:
            out[name] = t
    return out
