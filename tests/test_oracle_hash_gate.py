"""Pins of the oracle's sign-bit gate (reading of CPM-2 Section 2.3: the gate is a random projection
used as a locality sensitive hashing function) by facts that do not come from it."""
from fractions import Fraction

import numpy as np

from oracle import moe_oracle as O


def _brute(x, Wh):
    """Exact rational arithmetic, plain loops."""
    out = []
    for t in range(x.shape[0]):
        code = 0
        for j in range(Wh.shape[1]):
            s = sum(Fraction(float(x[t, i])) * Fraction(float(Wh[i, j])) for i in range(x.shape[1]))
            if s > 0:
                code |= 1 << j
        out.append(code)
    return np.array(out, dtype=np.int32)


def test_hash_gate_equals_exact_rational_loops():
    rng = np.random.default_rng(3)
    for b in (1, 3, 5, 8):
        x = rng.standard_normal((40, 24)).astype(np.float32)
        Wh = rng.standard_normal((24, b)).astype(np.float32)
        r = O.route_hash(x, Wh)
        assert r.idx.shape == (40, 1) and np.array_equal(r.idx[:, 0], _brute(x, Wh))
        assert np.all(r.w == 1.0) and r.w.dtype == np.float32
        assert np.all(r.idx >= 0) and np.all(r.idx < (1 << b))


def test_axis_directions_read_coordinate_signs():
    d, b = 16, 4
    Wh = np.zeros((d, b), dtype=np.float32)
    for j in range(b):
        Wh[3 * j + 1, j] = 1.0
    rng = np.random.default_rng(5)
    x = rng.standard_normal((200, d)).astype(np.float32)
    want = sum((x[:, 3 * j + 1] > 0).astype(np.int32) << j for j in range(b))
    assert np.array_equal(O.route_hash(x, Wh).idx[:, 0], want)


def test_scaling_keeps_the_code_negation_complements_it_zero_gives_zero():
    rng = np.random.default_rng(7)
    x = rng.standard_normal((64, 32)).astype(np.float32)
    Wh = rng.standard_normal((32, 6)).astype(np.float32)
    base = O.route_hash(x, Wh).idx[:, 0]
    assert np.array_equal(O.route_hash(4.0 * x, Wh).idx[:, 0], base)
    assert np.array_equal(O.route_hash(-x, Wh).idx[:, 0], 63 - base)      # no projection is exactly zero here
    assert np.array_equal(O.route_hash(np.zeros((3, 32), dtype=np.float32), Wh).idx[:, 0], np.zeros(3, dtype=np.int32))


def test_hash_gate_is_the_top1_projection_gate_on_signed_sums():
    """argmax_e sum_j s(e, j) L_j with s = +1 where bit j of e is set, else -1, is the sign pattern of L;
    on small integers the signed sums are exact, so route() (pinned elsewhere) must agree."""
    rng = np.random.default_rng(9)
    b, d = 4, 12
    x = rng.integers(-4, 5, size=(300, d)).astype(np.float32)
    Wh = rng.integers(-3, 4, size=(d, b)).astype(np.float32)
    S = np.array([[1.0 if (e >> j) & 1 else -1.0 for e in range(1 << b)] for j in range(b)])
    top1 = O.route(x, (Wh.astype(np.float64) @ S), k=1).idx[:, 0]
    assert np.array_equal(O.route_hash(x, Wh).idx[:, 0], top1)       # includes exact zeros: lower index = bit 0


def test_sign_of_a_projection_that_plain_summation_gets_wrong():
    """2^60 + 1 - 2^60 is 1 in exact arithmetic and 0 or 2 in any fp64 summation order."""
    x = np.array([[2.0 ** 60, 1.0, -(2.0 ** 60)], [2.0 ** 60, -1.0, -(2.0 ** 60)], [2.0 ** 60, 0.0, -(2.0 ** 60)]],
                 dtype=np.float32)
    Wh = np.ones((3, 1), dtype=np.float32)
    assert O.route_hash(x, Wh).idx[:, 0].tolist() == [1, 0, 0]


def test_layer_with_hash_gate_is_the_dense_ffn_of_the_named_expert():
    rng = np.random.default_rng(11)
    T, d, f, b = 30, 8, 12, 2
    x = rng.standard_normal((T, d)).astype(np.float32)
    Wh = rng.standard_normal((d, b)).astype(np.float32)
    mats = [tuple(rng.standard_normal(s) * 0.3 for s in ((d, f), (d, f), (f, d))) for _ in range(1 << b)]
    y, r, p, _ = O.layer_forward_hash(x, Wh, lambda e: mats[e])
    code = _brute(x, Wh)
    for t in range(T):
        W_in, W_gate, W_out = mats[code[t]]
        a, g = x[t].astype(np.float64) @ W_gate, x[t].astype(np.float64) @ W_in
        want = (O.gelu(a) * g) @ W_out
        assert np.allclose(y[t], want, rtol=1e-12, atol=1e-12)
    assert int(p.counts.sum()) == T
