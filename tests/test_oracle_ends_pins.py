"""Pins of the ends oracle (embedding gather, final norm + vocabulary projection, greedy choice)
against things other than itself: scalar loops, hand-written tables, closed forms and invariants."""
import math

import pytest
import torch

import oracle


def _rand(shape, seed, scale=1.0):
    g = torch.Generator().manual_seed(seed)
    return (torch.randn(shape, generator=g, dtype=torch.float64) * scale)


def test_embedding_is_a_row_gather_of_a_hand_written_table():
    table = torch.tensor([[0.0, 1.0, 2.0], [10.0, 11.0, 12.0], [20.0, 21.0, 22.0], [30.0, 31.0, 32.0]])
    out = oracle.embed_tokens(table, [3, 0, 0, 2])
    assert out.dtype == torch.float64
    assert out.tolist() == [[30.0, 31.0, 32.0], [0.0, 1.0, 2.0], [0.0, 1.0, 2.0], [20.0, 21.0, 22.0]]
    assert oracle.embed_tokens(table, []).shape == (0, 3)


@pytest.mark.parametrize("bad", [-1, 4, 1000])
def test_embedding_rejects_ids_outside_the_table(bad):
    with pytest.raises(ValueError):
        oracle.embed_tokens(torch.zeros(4, 3), [1, bad])


def test_last_rows_of_a_packed_batch():
    assert oracle.last_rows([3, 1, 1, 5]) == [2, 3, 4, 9]
    assert oracle.last_rows([1]) == [0]
    with pytest.raises(ValueError):
        oracle.last_rows([2, 0])


def _brute_logits(hidden, q_lens, gain, w, eps):
    """Scalar loops straight from the definition."""
    out = []
    start = 0
    for q in q_lens:
        row = hidden[start + q - 1]
        start += q
        h = len(row)
        ms = sum(float(v) * float(v) for v in row) / h
        r = 1.0 / math.sqrt(ms + eps)
        xn = [float(row[k]) * float(gain[k]) * r for k in range(h)]
        out.append([sum(xn[k] * float(w[v][k]) for k in range(h)) for v in range(len(w))])
    return torch.tensor(out, dtype=torch.float64)


@pytest.mark.parametrize("seed", [0, 1])
def test_head_logits_equal_scalar_loops(seed):
    q_lens = [3, 1, 2]
    hidden = _rand((6, 12), seed)
    gain = 1.0 + _rand((12,), seed + 10, 0.1)
    w = _rand((7, 12), seed + 20)
    got = oracle.head_logits(hidden, q_lens, gain, w, 1e-5)
    want = _brute_logits(hidden.tolist(), q_lens, gain.tolist(), w.tolist(), 1e-5)
    assert got.shape == (3, 7)
    assert torch.allclose(got, want, rtol=1e-12, atol=1e-12)


def test_identity_head_returns_the_normalised_last_rows():
    # w = I, gain = 1, eps -> 0: logits are x / rms(x); their mean square is 1
    hidden = _rand((5, 8), 3)
    logits = oracle.head_logits(hidden, [2, 3], torch.ones(8), torch.eye(8), 1e-30)
    for s, r in enumerate([1, 4]):
        x = hidden[r]
        assert torch.allclose(logits[s], x / x.pow(2).mean().sqrt(), rtol=1e-12, atol=0)
        assert abs(float(logits[s].pow(2).mean()) - 1.0) < 1e-12


def test_gain_scales_columns_before_the_projection():
    # a gain that is zero except at one coordinate leaves only that coordinate's weight column
    hidden = _rand((2, 6), 4)
    w = _rand((5, 6), 5)
    gain = torch.zeros(6, dtype=torch.float64)
    gain[2] = 3.0
    logits = oracle.head_logits(hidden, [2], gain, w, 1e-6)
    x = hidden[1]
    want = 3.0 * x[2] / torch.sqrt(x.pow(2).mean() + 1e-6) * w[:, 2]
    assert torch.allclose(logits[0], want, rtol=1e-12, atol=1e-15)


def test_logits_do_not_depend_on_the_scale_of_the_hidden_rows():
    hidden = _rand((4, 16), 6)
    gain = 1.0 + _rand((16,), 7, 0.1)
    w = _rand((9, 16), 8)
    a = oracle.head_logits(hidden, [1, 3], gain, w, 1e-12)
    b = oracle.head_logits(hidden * 37.5, [1, 3], gain, w, 1e-12)
    assert torch.allclose(a, b, rtol=1e-9, atol=1e-9)
    # with a large eps the scale does matter: eps sits inside the root
    c = oracle.head_logits(hidden, [1, 3], gain, w, 10.0)
    ms = hidden[[0, 3]].pow(2).mean(dim=-1, keepdim=True)
    assert torch.allclose(c, a * torch.sqrt((ms + 1e-12) / (ms + 10.0)), rtol=1e-9, atol=1e-12)


def test_permuting_vocabulary_rows_permutes_logits_and_only_last_rows_matter():
    hidden = _rand((7, 10), 9)
    gain = 1.0 + _rand((10,), 10, 0.1)
    w = _rand((11, 10), 11)
    q_lens = [4, 1, 2]
    base = oracle.head_logits(hidden, q_lens, gain, w, 1e-5)
    perm = torch.randperm(11, generator=torch.Generator().manual_seed(1))
    assert torch.equal(oracle.head_logits(hidden, q_lens, gain, w[perm], 1e-5), base[:, perm])
    changed = hidden.clone()
    changed[[0, 1, 2, 5]] = 123.0            # rows that are not the last of their sequence
    assert torch.equal(oracle.head_logits(changed, q_lens, gain, w, 1e-5), base)
    changed[3] += 1.0                         # a last row
    assert not torch.equal(oracle.head_logits(changed, q_lens, gain, w, 1e-5)[0], base[0])


def test_q_lens_must_cover_every_row():
    with pytest.raises(ValueError):
        oracle.head_logits(torch.zeros(5, 4), [2, 2], torch.ones(4), torch.zeros(3, 4), 1e-5)


def test_greedy_choice_takes_the_largest_logit_and_the_smallest_index_among_equals():
    logits = torch.tensor([[0.0, 2.0, 1.0, 2.0], [-1.0, -3.0, -1.0, -2.0], [5.0, 4.0, 3.0, 2.0], [1.0, 1.0, 1.0, 7.0]],
                          dtype=torch.float64)
    assert oracle.greedy_tokens(logits).tolist() == [1, 0, 0, 3]
    # against a library routine on rows without ties
    rnd = _rand((20, 50), 12)
    assert torch.equal(oracle.greedy_tokens(rnd), rnd.argmax(dim=-1))


def test_an_embedded_token_is_chosen_again_by_a_tied_head():
    # with orthogonal embedding rows, gain 1 and the output head tied to the table, the token whose
    # embedding is the hidden row gets the largest logit (cosine 1 against cosine 0)
    table = torch.eye(6, dtype=torch.float64) * 2.5
    ids = [4, 1, 5]
    hidden = oracle.embed_tokens(table, ids)
    logits = oracle.head_logits(hidden, [1, 1, 1], torch.ones(6), table, 1e-6)
    assert oracle.greedy_tokens(logits).tolist() == ids


# ---------------------------------------------------------------- the LayerNorm head

def _brute_layernorm_logits(hidden, q_lens, gain, bias, w, eps):
    """Scalar loops; the variance by the two-moment formula (the tensor code sums squared deviations)."""
    out = []
    start = 0
    for q in q_lens:
        row = [float(v) for v in hidden[start + q - 1]]
        start += q
        h = len(row)
        mean = sum(row) / h
        var = sum(v * v for v in row) / h - mean * mean
        r = 1.0 / math.sqrt(var + eps)
        xn = [(row[k] - mean) * r * float(gain[k]) + (float(bias[k]) if bias is not None else 0.0) for k in range(h)]
        out.append([sum(xn[k] * float(w[v][k]) for k in range(h)) for v in range(len(w))])
    return torch.tensor(out, dtype=torch.float64)


@pytest.mark.parametrize("with_bias", [False, True])
def test_layernorm_head_equals_scalar_loops_and_the_library(with_bias):
    q_lens = [2, 1, 4]
    hidden = _rand((7, 12), 3) + 0.75                    # rows with a mean of their own
    gain = 1.0 + _rand((12,), 13, 0.1)
    bias = _rand((12,), 23, 0.3) if with_bias else None
    w = _rand((9, 12), 33)
    got = oracle.head_logits(hidden, q_lens, gain, w, 1e-5, norm_kind="layer", bias=bias)
    want = _brute_layernorm_logits(hidden.tolist(), q_lens, gain.tolist(), None if bias is None else bias.tolist(),
                                   w.tolist(), 1e-5)
    assert torch.allclose(got, want, rtol=1e-10, atol=1e-11)
    rows = hidden.double()[oracle.last_rows(q_lens)]
    lib = torch.nn.functional.layer_norm(rows, (12,), gain.double(), None if bias is None else bias.double(), 1e-5)
    assert torch.allclose(got, lib @ w.double().T, rtol=1e-12, atol=1e-12)
    # a shift of the hidden rows changes nothing; an RMSNorm head would change
    shifted = oracle.head_logits(hidden + 3.0, q_lens, gain, w, 1e-5, norm_kind="layer", bias=bias)
    assert torch.allclose(shifted, got, rtol=1e-9, atol=1e-10)
    rms = oracle.head_logits(hidden, q_lens, gain, w, 1e-5)
    assert not torch.allclose(rms, got, rtol=1e-2)


def test_an_rmsnorm_head_takes_no_bias():
    with pytest.raises(ValueError):
        oracle.head_logits(_rand((2, 8), 1), [2], torch.ones(8), _rand((4, 8), 2), 1e-5, bias=torch.zeros(8))
