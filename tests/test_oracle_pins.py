"""Pins for the CPU oracle: each test ties oracle/moe_oracle.py to something that is
not the oracle itself (hand-computed values, textbook constants, a pure-Python
brute force, dense special cases computed by another library, invariants)."""
import json
import math
import os

import numpy as np
import pytest
import torch

from oracle import moe_oracle as O
from tests import brute_force as B

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def _gold(name):
    with open(os.path.join(GOLD, name)) as fh:
        return json.load(fh)


def _rand_case(seed, T, d, f, E):
    rng = np.random.default_rng(seed)
    x = rng.standard_normal((T, d))
    Wg = rng.standard_normal((d, E)) / math.sqrt(d)
    experts = [(rng.standard_normal((d, f)) * 0.3, rng.standard_normal((d, f)) * 0.3,
                rng.standard_normal((f, d)) * 0.3) for _ in range(E)]
    return x, Wg, experts


def _lists(experts):
    return [tuple(m.tolist() for m in e) for e in experts]


# ---------------------------------------------------------------- printed / textbook values

def test_gelu_matches_normal_table():
    for z, phi in _gold("normal_cdf.json")["phi"].items():
        z = float(z)
        assert abs(float(O.gelu(np.array([z]))[0]) - z * phi) < 2e-10 * max(1.0, abs(z))


def test_gelu_identities():
    z = np.linspace(-6, 6, 241)
    assert O.gelu(np.array([0.0]))[0] == 0.0
    np.testing.assert_allclose(O.gelu(z) - O.gelu(-z), z, atol=1e-15)
    np.testing.assert_allclose(O.gelu(z), [0.5 * v * (1 + math.erf(v / math.sqrt(2))) for v in z], atol=1e-15)
    # the tanh form is a different function: close, but not equal
    assert 1e-5 < np.abs(O.gelu_tanh(z) - O.gelu(z)).max() < 1e-3


def test_table1_totals_need_three_matrices_and_32_experts():
    g = _gold("table1_sizes.json")
    d, f, L, E = g["d_model"], g["d_ff"], g["layers"], g["experts"]
    dense = O.model_parameter_count(1, 3, d, f, L) / 1e9
    moe = O.model_parameter_count(E, 3, d, f, L) / 1e9
    assert round(dense) == g["dense_params_billion"]          # 10.87 B -> "11 B"
    assert round(moe) == g["moe_params_billion"]              # 198.1 B -> "198 B"
    assert round(O.model_parameter_count(1, 2, d, f, L) / 1e9) != g["dense_params_billion"]   # 8.86 B
    assert round(O.model_parameter_count(E, 2, d, f, L) / 1e9) != g["moe_params_billion"]
    assert 3 * d * f * 2 == 240 * 2 ** 20                     # one bf16 expert = 240 MiB


def test_hand_worked_example():
    g = _gold("hand_example.json")
    x, Wg = np.array(g["x"], float), np.array(g["Wg"], float)
    ex = [(np.array(e["W_in"], float), np.array(e["W_gate"], float), np.array(e["W_out"], float))
          for e in g["experts"]]
    y, r, p, _ = O.layer_forward(x, Wg, lambda e: ex[e], E=2, k=1)
    assert r.idx.tolist() == g["idx"]
    assert r.w.tolist() == g["w"]
    np.testing.assert_allclose(y, g["y"], atol=5e-10)
    # swapping the two up-projections is a different function (guards the GELU operand)
    y_sw, *_ = O.layer_forward(x, Wg, lambda e: (ex[e][1], ex[e][0], ex[e][2]), E=2, k=1)
    assert np.abs(y_sw - np.array(g["y"])).max() > 0.1


def test_hand_worked_top2_weights():
    t2 = _gold("hand_example.json")["top2"]
    x = np.array([[1.0]])
    Wg = np.array([t2["logits"]])
    r = O.route(x, Wg, k=2, renorm=1)
    assert r.idx[0].tolist() == t2["idx"]
    np.testing.assert_allclose(r.w[0], t2["w_renorm"], atol=1e-7)
    r0 = O.route(x, Wg, k=2, renorm=0)
    np.testing.assert_allclose(r0.w[0], t2["w_full"], atol=1e-7)
    np.testing.assert_allclose(r.margin[0], math.log(3.0), atol=1e-12)   # gaps: ln3, 5 -> min ln3


# ---------------------------------------------------------------- brute force on tiny inputs

@pytest.mark.parametrize("k,renorm,act", [(1, 1, 0), (2, 1, 0), (3, 1, 0), (2, 0, 0), (1, 0, 1), (3, 0, 1)])
def test_oracle_equals_brute_force(k, renorm, act):
    T, d, f, E = 9, 6, 10, 5       # d != f so a transposed operand cannot go unnoticed
    x, Wg, ex = _rand_case(10 + k, T, d, f, E)
    bias = np.linspace(-0.3, 0.3, E)
    y, r, p, _ = O.layer_forward(x, Wg, lambda e: ex[e], E=E, k=k, bias=bias, renorm=renorm, act=act)
    yb, idxb, wb = B.moe_layer(x.tolist(), Wg.tolist(), _lists(ex), k=k, bias=bias.tolist(),
                               renorm=renorm, act=act)
    assert r.idx.tolist() == idxb
    np.testing.assert_allclose(r.w, np.array(wb), rtol=0, atol=1e-7)      # w is rounded to fp32
    w_exact = np.array(wb)
    # recompute y with the brute force's own unrounded weights to compare at fp64 level
    y64 = O.combine(O.expert_ffn(p.Xp, p.offsets, lambda e: ex[e], act), p.inv, w_exact.astype(np.float64))
    np.testing.assert_allclose(y64, np.array(yb), rtol=1e-12, atol=1e-13)
    np.testing.assert_allclose(y, np.array(yb), rtol=1e-6, atol=1e-6)


def test_crafted_ties_go_to_lowest_index():
    T, d, f, E = 6, 4, 3, 6
    x, Wg, ex = _rand_case(3, T, d, f, E)
    Wg[:, 4] = Wg[:, 1]            # experts 1 and 4 always tie
    Wg[:, 5] = Wg[:, 1]
    x[2] = 0.0                     # an all-zero token: every logit is 0
    for k in (1, 2, 3):
        r = O.route(x, Wg, k=k)
        _, idxb, _ = B.moe_layer(x.tolist(), Wg.tolist(), _lists(ex), k=k)
        assert r.idx.tolist() == idxb
        assert r.idx[2].tolist() == list(range(k))
        for t in range(T):
            row = r.idx[t].tolist()
            if 4 in row:
                assert 1 in row and row.index(1) < row.index(4)
            if 5 in row:
                assert 4 in row and row.index(4) < row.index(5)
    y, *_ = O.layer_forward(x, Wg, lambda e: ex[e], E=E, k=2)
    assert np.all(y[2] == 0.0)     # FFN(0) = 0: no biases anywhere


def test_duplicate_gate_columns_tie_exactly_for_fp32_inputs():
    # a library matmul may round identical columns differently; ties are defined in exact arithmetic
    rng = np.random.default_rng(5)
    T, d, E, k = 96, 256, 12, 3
    x = rng.standard_normal((T, d)).astype(np.float32)
    Wg = (rng.standard_normal((d, E)) / 16).astype(np.float32)
    Wg[:, 7] = Wg[:, 2]
    Wg[:, 9] = Wg[:, 2]
    r = O.route(x, Wg, k=k)
    _, idxb, _ = B.moe_layer(x[:, :].astype(np.float64).tolist(), Wg.astype(np.float64).tolist(),
                             [([[0.0]] * d, [[0.0]] * d, [[0.0] * d])] * E, k=k)
    assert r.idx.tolist() == idxb                      # brute force sums with math.fsum: exact too
    for row in r.idx.tolist():
        for a, b in ((2, 7), (7, 9), (2, 9)):
            if b in row:
                assert a in row and row.index(a) < row.index(b)
    e = O.exact_logits_row(x[0], Wg)
    assert e[2] == e[7] == e[9]
    np.testing.assert_allclose(e, x[0].astype(np.float64) @ Wg.astype(np.float64), rtol=0, atol=1e-12)


# ---------------------------------------------------------------- dense special cases (another library)

def _torch_dense_ffn(x, W_in, W_gate, W_out):
    xt = torch.from_numpy(np.asarray(x, dtype=np.float64))
    a = xt @ torch.from_numpy(W_gate)
    b = xt @ torch.from_numpy(W_in)
    return ((torch.nn.functional.gelu(a) * b) @ torch.from_numpy(W_out)).numpy()


def test_single_expert_is_the_dense_ffn():
    x, Wg, ex = _rand_case(5, 17, 12, 20, 1)
    y, r, p, _ = O.layer_forward(x, Wg, lambda e: ex[0], E=1, k=1)
    np.testing.assert_allclose(y, _torch_dense_ffn(x, *ex[0]), rtol=1e-12, atol=1e-12)
    assert np.all(r.idx == 0) and np.all(r.w == 1.0)
    assert p.perm.tolist() == list(range(17))


@pytest.mark.parametrize("k", [1, 2, 4])
def test_duplicated_experts_equal_the_dense_ffn(k):
    # Section 2.3: the MoE model starts as copies of the dense model, so any routing gives the dense output
    x, Wg, ex = _rand_case(6, 23, 8, 14, 4)
    y, *_ = O.layer_forward(x, Wg, lambda e: ex[2], E=4, k=k, renorm=1)
    np.testing.assert_allclose(y, _torch_dense_ffn(x, *ex[2]), rtol=1e-6, atol=1e-6)  # w rounded to fp32


# ---------------------------------------------------------------- invariants

@pytest.mark.parametrize("k", [1, 2, 3])
def test_routing_and_permutation_invariants(k):
    T, d, E = 301, 16, 7
    rng = np.random.default_rng(8)
    x = rng.standard_normal((T, d))
    Wg = rng.standard_normal((d, E))
    r = O.route(x, Wg, k=k)
    p = O.permute(x, r.idx, E)
    A = T * k
    assert p.counts.sum() == A and p.offsets[0] == 0 and p.offsets[-1] == A
    assert np.array_equal(np.diff(p.offsets), p.counts)
    assert sorted(p.perm.tolist()) == list(range(A))
    assert np.array_equal(p.inv[p.perm], np.arange(A))
    flat = r.idx.reshape(-1)
    for e in range(E):
        seg = p.perm[p.offsets[e]:p.offsets[e + 1]]
        assert np.all(flat[seg] == e)
        assert np.all(np.diff(seg) > 0)                      # stable: ascending assignment index
    assert all(len(set(row)) == k for row in r.idx.tolist())
    np.testing.assert_allclose(r.w.sum(axis=1), 1.0, atol=2e-7)
    assert np.all(r.w >= 0)
    if k == 1:
        assert np.all(r.w == 1.0)
    # slot order: descending logit
    sel = np.take_along_axis(r.logits, r.idx.astype(np.int64), axis=1)
    assert np.all(np.diff(sel, axis=1) <= 0)
    # everything not selected is no larger than the last selected
    assert np.all(r.logits <= sel[:, :1] + 0) and np.all((r.logits >= sel[:, -1:]).sum(axis=1) >= k)
    np.testing.assert_array_equal(p.Xp, x[p.perm // k])


def test_full_softmax_weights_are_probabilities_of_selected():
    rng = np.random.default_rng(9)
    x, Wg = rng.standard_normal((40, 8)), rng.standard_normal((8, 6))
    r = O.route(x, Wg, k=2, renorm=0)
    prob = torch.softmax(torch.from_numpy(r.logits), dim=1).numpy()
    np.testing.assert_allclose(r.w, np.take_along_axis(prob, r.idx.astype(np.int64), axis=1), atol=1e-7)
    assert np.all(r.w.sum(axis=1) < 1.0)


def test_token_independence_and_expert_relabelling():
    T, d, f, E, k = 12, 8, 6, 4, 2
    x, Wg, ex = _rand_case(11, T, d, f, E)
    y, *_ = O.layer_forward(x, Wg, lambda e: ex[e], E=E, k=k)
    sh = np.random.default_rng(1).permutation(T)
    y_sh, *_ = O.layer_forward(x[sh], Wg, lambda e: ex[e], E=E, k=k)
    np.testing.assert_array_equal(y_sh, y[sh])
    for t in range(T):                                         # each token alone
        y1, *_ = O.layer_forward(x[t:t + 1], Wg, lambda e: ex[e], E=E, k=k)
        np.testing.assert_allclose(y1[0], y[t], rtol=1e-13, atol=1e-14)
    rel = np.array([2, 0, 3, 1])                               # new id -> old id
    y_rel, *_ = O.layer_forward(x, Wg[:, rel], lambda e: ex[rel[e]], E=E, k=k)
    np.testing.assert_allclose(y_rel, y, rtol=1e-13, atol=1e-14)


def test_linearity_in_down_and_in_projection():
    x, Wg, ex = _rand_case(12, 10, 8, 6, 3)
    y, *_ = O.layer_forward(x, Wg, lambda e: ex[e], E=3, k=2)
    y2, *_ = O.layer_forward(x, Wg, lambda e: (ex[e][0], ex[e][1], -2.5 * ex[e][2]), E=3, k=2)
    np.testing.assert_allclose(y2, -2.5 * y, rtol=1e-13, atol=1e-14)
    y3, *_ = O.layer_forward(x, Wg, lambda e: (3.0 * ex[e][0], ex[e][1], ex[e][2]), E=3, k=2)
    np.testing.assert_allclose(y3, 3.0 * y, rtol=1e-13, atol=1e-14)
    # ... but not in the gated projection (GELU is not linear)
    y4, *_ = O.layer_forward(x, Wg, lambda e: (ex[e][0], 3.0 * ex[e][1], ex[e][2]), E=3, k=2)
    assert np.abs(y4 - 3.0 * y).max() > 1e-3


def test_empty_inputs_and_empty_experts():
    x, Wg, ex = _rand_case(13, 5, 4, 3, 6)
    bias = np.array([0, -1e9, 0, -1e9, 0, 0.0])
    touched = []

    def src(e):
        touched.append(e)
        return ex[e]
    y, r, p, _ = O.layer_forward(x, Wg, src, E=6, k=2, bias=bias)
    assert p.counts[1] == 0 and p.counts[3] == 0
    assert 1 not in touched and 3 not in touched          # empty experts are never loaded
    x0 = np.zeros((0, 4))
    y0, r0, p0, _ = O.layer_forward(x0, Wg, src, E=6, k=2)
    assert y0.shape == (0, 4) and p0.counts.sum() == 0 and p0.offsets.tolist() == [0] * 7


def test_planted_mistakes_are_caught_by_the_pins():
    """The pins above are only worth something if plausible slips fail them: plant a few in copies
    of the oracle's steps (on the CPU) and check the brute force disagrees."""
    T, d, f, E, k = 7, 5, 4, 3, 2
    x, Wg, ex = _rand_case(14, T, d, f, E)
    yb, idxb, wb = B.moe_layer(x.tolist(), Wg.tolist(), _lists(ex), k=k)
    yb = np.array(yb)
    r = O.route(x, Wg, k=k)
    p = O.permute(x, r.idx, E)
    Yp = O.expert_ffn(p.Xp, p.offsets, lambda e: ex[e])
    good = O.combine(Yp, p.inv, r.w)
    assert np.abs(good - yb).max() < 1e-6
    wrong_inv = O.combine(Yp, p.perm, r.w)                                   # perm used for inv
    wrong_w = O.combine(Yp, p.inv, r.w[:, ::-1])                             # slots swapped
    rev = np.concatenate([[0], np.cumsum(p.counts[::-1])]).astype(np.int32)      # segments in reverse order
    wrong_seg = O.combine(O.expert_ffn(p.Xp, rev, lambda e: ex[e]), p.inv, r.w) \
        if len(set(p.counts.tolist())) > 1 else None
    for bad in (wrong_inv, wrong_w, wrong_seg):
        if bad is not None:
            assert np.abs(bad - yb).max() > 1e-3
