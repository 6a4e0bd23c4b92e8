"""Pins for the part of the oracle's gate that decides tokens too close to call (Sections 2.1 and 2.3:
one expert per token, picked from a frozen random projection of its hidden state).

oracle.route ranks with a library matrix product and re-evaluates, as correctly rounded exact sums,
every token whose k+1 best logits are closer than the product's rounding error.  These tests tie that
branch to exact rational arithmetic (fractions.Fraction: every float is an exact rational, so sums and
comparisons here have no rounding at all): gate bias included, gaps that are not zero but far below
the rounding error of a float64 dot product, k = 1, 2, 3, and the sign-bit gate next to zero."""
import math
from fractions import Fraction

import numpy as np
import pytest

from oracle import moe_oracle as O


def exact_rank(xt, Wg, bias=None):
    """Experts in gate order (larger exact logit first, equal logits by lower index) and the exact logits."""
    d, E = Wg.shape
    L = []
    for e in range(E):
        s = sum((Fraction(float(xt[i])) * Fraction(float(Wg[i, e])) for i in range(d)), Fraction(0))
        if bias is not None:
            s += Fraction(float(bias[e]))
        L.append(s)
    return sorted(range(E), key=lambda e: (-L[e], e)), L


def expected_weights(L, sel, renorm):
    if renorm:
        ex = [math.exp(float(L[e] - L[sel[0]])) for e in sel]
        return [v / sum(ex) for v in ex]
    m = max(L)
    ex = [math.exp(float(v - m)) for v in L]
    return [ex[e] / sum(ex) for e in sel]


def check_all_tokens(x, Wg, bias, k, renorm=1):
    r = O.route(x, Wg, k=k, bias=bias, renorm=renorm)
    for t in range(x.shape[0]):
        order, L = exact_rank(x[t], Wg, bias)
        assert r.idx[t].tolist() == order[:k], f"token {t}: {r.idx[t].tolist()} but exact arithmetic ranks {order[:k + 1]}"
        np.testing.assert_allclose(r.w[t], expected_weights(L, order[:k], renorm), rtol=0, atol=2e-7)
    return r


def near_tie_gate(rng, T, d, E, pairs, tiny):
    """Random gate in which, for every (a, b, sign) of pairs, column b is column a except for two entries
    chosen so that with x_i = x_j = 1 the exact logits differ by sign * tiny and nothing else: entry i gets
    +2^-30 and entry j gets -2^-30 + sign * tiny (both exactly representable)."""
    x = rng.standard_normal((T, d))
    Wg = rng.standard_normal((d, E)) / math.sqrt(d)
    i, j = 1, d - 2
    x[:, i] = 1.0
    x[:, j] = 1.0
    for a, b, sign in pairs:
        Wg[:, b] = Wg[:, a]
        Wg[i, a] = 0.25
        Wg[j, a] = 0.0
        Wg[i, b] = 0.25 + 2.0 ** -30
        Wg[j, b] = -(2.0 ** -30) + sign * tiny
        got = Fraction(float(Wg[i, b])) + Fraction(float(Wg[j, b])) - Fraction(float(Wg[i, a])) - Fraction(float(Wg[j, a]))
        assert got == Fraction(sign * tiny)
    return x, Wg


@pytest.mark.parametrize("k", [1, 2, 3])
def test_gaps_below_the_rounding_error_are_ranked_exactly(k):
    rng = np.random.default_rng(100 + k)
    T, d, E = 40, 64, 7
    tiny = 2.0 ** -60                     # a float64 dot product of this size is good to about 1e-15: 1e3 times coarser
    # column 5 beats column 2 by tiny although its index is higher; column 6 loses to column 0 by tiny
    x, Wg = near_tie_gate(rng, T, d, E, [(2, 5, +1), (0, 6, -1)], tiny)
    r = check_all_tokens(x, Wg, None, k)
    hit = 0
    for t in range(T):
        row = r.idx[t].tolist()
        if 2 in row:                      # 5 ranks directly above 2 wherever 2 is selected
            assert 5 in row and row.index(5) + 1 == row.index(2)
        if 6 in row:                      # and 6 directly below 0
            assert 0 in row and row.index(0) + 1 == row.index(6)
        hit += (5 in row) + (0 in row)
    assert hit > 0                        # the crafted pairs do reach the selection
    assert float(r.margin.min()) <= 2 * tiny * 1.01      # the oracle reports the exact gap, not a rounded one


@pytest.mark.parametrize("k", [1, 2, 3])
def test_gate_bias_enters_the_exact_re_evaluation(k):
    rng = np.random.default_rng(200 + k)
    T, d, E = 32, 48, 6
    x = rng.standard_normal((T, d))
    Wg = rng.standard_normal((d, E)) / math.sqrt(d)
    Wg[:, 4] = Wg[:, 1]                   # identical projections: only the bias can tell 1 and 4 apart
    Wg[:, 3] = Wg[:, 0]
    bias = rng.standard_normal(E) * 0.1
    bias[4] = bias[1] + 2.0 ** -45        # 4 wins by the bias alone, by less than the product's rounding error
    bias[3] = bias[0] - 2.0 ** -45        # 3 loses to 0 by the bias alone
    r = check_all_tokens(x, Wg, bias, k)
    for row in r.idx.tolist():
        if 1 in row:
            assert 4 in row and row.index(4) < row.index(1)
        if 3 in row:
            assert 0 in row and row.index(0) < row.index(3)
    # a bias that is dropped from the re-evaluation would rank 1 before 4 (equal projections, lower index)
    dropped = O.route(x, Wg, k=k, bias=None)
    assert any(1 in row and (4 not in row or row.index(1) < row.index(4)) for row in dropped.idx.tolist())


def test_bias_against_a_column_gap():
    rng = np.random.default_rng(7)
    T, d, E = 24, 32, 5
    tiny = 2.0 ** -58
    x, Wg = near_tie_gate(rng, T, d, E, [(1, 3, +1)], tiny)       # column 3 ahead of column 1 by tiny ...
    bias = np.zeros(E)
    bias[1] = 2.0 ** -57                                          # ... and the bias puts 1 ahead by twice that
    for k in (1, 2):
        r = check_all_tokens(x, Wg, bias, k)
        for row in r.idx.tolist():
            if 3 in row:
                assert 1 in row and row.index(1) < row.index(3)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("k,renorm", [(1, 1), (2, 1), (3, 0)])
def test_stored_precision_inputs_every_token_against_exact_rationals(dtype, k, renorm):
    rng = np.random.default_rng(300 + k)
    T, d, E = 48, 96, 9
    x = rng.standard_normal((T, d)).astype(np.float32)
    Wg = (rng.standard_normal((d, E)) / math.sqrt(d)).astype(np.float32)
    if dtype == "bf16":                  # values a bf16 tensor can hold
        x = (x.view(np.uint32) & np.uint32(0xFFFF0000)).view(np.float32)
        Wg = (Wg.view(np.uint32) & np.uint32(0xFFFF0000)).view(np.float32)
    Wg[:, 8] = Wg[:, 3]                  # an exact tie in every token
    Wg[5, 8] = Wg[5, 3] * np.float32(1.0 + 2.0 ** -7)         # except where x[:, 5] is not zero: a real, small gap
    x[::3, 5] = 0.0
    bias = (rng.standard_normal(E) * 0.05).astype(np.float32)
    bias[8] = bias[3]
    check_all_tokens(x, Wg, bias, k, renorm)
    # the oracle's own exact row agrees with the rationals to the last bit
    for t in (0, 1, 3):
        _, L = exact_rank(x[t], Wg, bias)
        got = O.exact_logits_row(x[t], Wg, bias)
        assert [float(v) for v in L] == got.tolist()


def test_sign_bits_next_to_zero():
    rng = np.random.default_rng(11)
    T, d, b = 30, 40, 3
    x = rng.standard_normal((T, d))
    Wh = rng.standard_normal((d, b)) / math.sqrt(d)
    tiny = 2.0 ** -60
    # direction 1: the projection of token t is exactly s_t * tiny with s_t in {-1, 0, +1}: all other entries
    # cancel in pairs, which a rounded sum need not notice
    Wh[:, 1] = 0.0
    x[:, 0] = 1.0
    x[:, 1] = -1.0
    x[:, 2] = 1.0
    Wh[0, 1] = 0.375
    Wh[1, 1] = 0.375
    s = np.array([(-1, 0, 1)[t % 3] for t in range(T)], dtype=np.float64)
    x[:, 2] = s                                            # x_2 * tiny is what is left
    Wh[2, 1] = tiny
    r = O.route_hash(x, Wh)
    for t in range(T):
        code = 0
        for j in range(b):
            proj = sum((Fraction(float(x[t, i])) * Fraction(float(Wh[i, j])) for i in range(d)), Fraction(0))
            code |= (1 << j) if proj > 0 else 0
        assert int(r.idx[t, 0]) == code
        assert ((int(r.idx[t, 0]) >> 1) & 1) == (1 if s[t] > 0 else 0)     # zero and negative projections give bit 0
    assert float(r.margin.min()) == 0.0 and float(np.sort(r.margin)[T // 3]) == tiny


def test_tanh_gelu_is_the_published_approximation():
    # another library's implementation of the tanh form, in float64
    import torch
    z = np.linspace(-8, 8, 641)
    want = torch.nn.functional.gelu(torch.from_numpy(z), approximate="tanh").numpy()
    np.testing.assert_allclose(O.gelu_tanh(z), want, rtol=0, atol=1e-15)
    # and its distance from the exact form: largest between |z| = 2 and 3, about 4.7e-4
    diff = np.abs(O.gelu_tanh(z) - O.gelu(z))
    assert 4.0e-4 < diff.max() < 5.5e-4 and 2.0 < abs(z[diff.argmax()]) < 3.0


def test_planted_mistakes_in_the_re_evaluation_are_caught(monkeypatch):
    """The pins above fail when the oracle's branch for close tokens is broken in the ways one would break it:
    (1) the bias left out of the exact sums, (2) floats that coincide after rounding taken for a tie,
    (3) the branch never entered."""
    rng = np.random.default_rng(201)
    x = rng.standard_normal((32, 48))
    Wg = rng.standard_normal((48, 6)) / math.sqrt(48)
    Wg[:, 4] = Wg[:, 1]
    bias = rng.standard_normal(6) * 0.1
    bias[4] = bias[1] + 2.0 ** -45
    check_all_tokens(x, Wg, bias, 2)
    xs, Ws = near_tie_gate(np.random.default_rng(101), 40, 64, 7, [(2, 5, +1), (0, 6, -1)], 2.0 ** -60)
    check_all_tokens(xs, Ws, None, 2)

    real_row, real_rank, real_dot = O.exact_logits_row, O._rank_exactly, O.exact_dot
    with monkeypatch.context() as m:
        m.setattr(O, "exact_logits_row", lambda xt, W, b=None: real_row(xt, W, None))
        m.setattr(O, "exact_dot", lambda xt, col, b=None: real_dot(xt, col, None))
        with pytest.raises(AssertionError):
            check_all_tokens(x, Wg, bias, 2)
    with monkeypatch.context() as m:
        def float_rank(Lt, xt, W64, b, k):
            order = sorted(range(Lt.shape[0]), key=lambda e: (-Lt[e], e))
            return order, 0.0
        m.setattr(O, "_rank_exactly", float_rank)
        with pytest.raises(AssertionError):
            check_all_tokens(xs, Ws, None, 2)
    with monkeypatch.context() as m:
        m.setattr(O, "exact_logits_row", lambda xt, W, b=None: O.gate_logits(xt[None, :], W, b)[0])
        m.setattr(O, "_rank_exactly", lambda Lt, xt, W64, b, k: (sorted(range(Lt.shape[0]), key=lambda e: (-Lt[e], e)), 0.0))
        with pytest.raises(AssertionError):
            check_all_tokens(xs, Ws, None, 2)
