"""Pins of the 4-bit weight format oracle against what the definition and arithmetic fix (no GPU)."""
import random

import torch

import oracle
from oracle import w4_oracle as W
from tests.helpers import oracle_pool, oracle_shape


def test_hand_written_words():
    # 0x76543210: field i (bits 4i..4i+3) holds i, so the eight elements of the word are 0..7 in order
    words = torch.tensor([[0x76543210, 0xFEDCBA98 - (1 << 32)], [0x0000000F, 0x10000000]], dtype=torch.int64)
    codes = W.unpack_codes(words)
    assert codes[0].tolist() == list(range(16))
    assert codes[1].tolist() == [15, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 1]
    # signed 32-bit storage of the same bits gives the same codes
    assert torch.equal(W.unpack_codes(words.to(torch.int32)), codes)


def test_field_order_against_integer_arithmetic():
    rng = random.Random(3)
    vals = [[rng.getrandbits(32) for _ in range(5)] for _ in range(4)]
    codes = W.unpack_codes(torch.tensor(vals, dtype=torch.int64))
    for n in range(4):
        for k in range(40):
            assert codes[n, k].item() == (vals[n][k // 8] >> (4 * (k % 8))) % 16


def test_formula_on_literal_numbers():
    # one row, K = 16, groups of 8: codes 0..15; first group zero 3 scale 0.5, second group zero 10 scale -2
    words = torch.tensor([[0x76543210, 0xFEDCBA98]], dtype=torch.int64)
    w = W.dequantize(words, torch.tensor([[0.5, -2.0]]), torch.tensor([[3.0, 10.0]]), 8)
    want = [(c - 3) * 0.5 for c in range(8)] + [(c - 10) * -2.0 for c in range(8, 16)]
    assert w.dtype == torch.float64 and w[0].tolist() == want


def test_a_group_parameter_moves_only_its_group():
    g = torch.Generator().manual_seed(0)
    words = torch.randint(0, 1 << 32, (6, 8), generator=g, dtype=torch.int64)     # K = 64
    s = torch.rand(6, 4, generator=g, dtype=torch.float64) + 0.1
    z = torch.randint(0, 16, (6, 4), generator=g).to(torch.float64)
    base = W.dequantize(words, s, z, 16)
    s2 = s.clone(); s2[2, 1] *= 3
    z2 = z.clone(); z2[4, 3] += 1
    d1 = (W.dequantize(words, s2, z, 16) != base).nonzero().tolist()
    d2 = (W.dequantize(words, s, z2, 16) != base).nonzero().tolist()
    assert all(r == 2 and 16 <= k < 32 for r, k in d1) and d1
    assert sorted(d2) == [[4, k] for k in range(48, 64)]
    # raising a zero point by one lowers its group by exactly one scale step
    assert torch.allclose(W.dequantize(words, s, z2, 16)[4, 48:], base[4, 48:] - s[4, 3])


def test_round_trip_within_half_a_step_and_exact_on_the_grid():
    g = torch.Generator().manual_seed(1)
    w = torch.randn(8, 256, generator=g, dtype=torch.float64) * 0.02
    for group in (32, 64, 128):
        words, s, z = W.quantize(w, group)
        back = W.dequantize(words, s, z, group)
        step = s.repeat_interleave(group, dim=1)
        # the zero point is rounded too, which can push a group's end codes into the clamp: allow one step there
        assert ((back - w).abs() <= step * 1.0 + 1e-15).all()
        assert ((back - w).abs() <= step * 0.5 + 1e-15).to(torch.float64).mean() > 0.9
        # a matrix on the grid comes back exactly and re-quantises to the same codes wherever its groups span 0..15
        words2, s2, z2 = W.quantize(back, group)
        assert torch.equal(W.dequantize(words2, s2, z2, group), back) or \
            (W.dequantize(words2, s2, z2, group) - back).abs().max() <= 1e-12


def test_stage_output_is_the_same_from_either_representation():
    # weights that lie on a 4-bit grid whose values bf16 holds exactly: the stage oracle must not care
    # whether it is handed the matrices or their codes
    from paper_2507_05043_amd import synth
    shape = synth.StageShape("w4-pin", 2, 64, 2, 1, 32, 96)
    osh = oracle_shape(shape)
    group = 32
    stored = []
    for l in range(shape.num_layers):
        lw = synth.draw_w4_layer(shape, l, seed=5, group=group)
        for name in ("qkv", "o", "gate", "up", "down"):
            lw["s" + name] = torch.full_like(lw["s" + name], 2.0 ** -7)     # code - zero has at most 5 bits: exact in bf16
        stored.append(lw)
    plain = [W.dequantize_layer(lw, group) for lw in stored]
    as_bf16 = [{k: (v.to(torch.bfloat16) if v.dtype == torch.float64 else v) for k, v in lw.items()} for lw in plain]
    for a, b in zip(plain, as_bf16):
        for k in ("wqkv", "wdown"):
            assert torch.equal(a[k], b[k].to(torch.float64))
    mb = synth.make_microbatch([5, 1], [0, 20], seed=2, max_blocks_per_seq=4)
    hidden = synth.draw_hidden(shape, mb.num_tokens, seed=2)
    outs = []
    for layers in (plain, as_bf16):
        pool = oracle_pool(shape, mb, seed=2)
        out, _ = oracle.stage_forward(osh, layers, hidden, mb.positions, mb.q_lens, mb.ctx_lens, mb.block_tables, pool)
        outs.append(out)
    assert torch.isfinite(outs[0]).all() and torch.equal(outs[0], outs[1])
