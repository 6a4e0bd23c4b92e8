"""Plain fp64 CPU definition of the CPM-2-MoE feed-forward layer.

TEST INFRASTRUCTURE ONLY.  Nothing on the product path may import this module;
it exists so that tests, the smoke check and the bench's CPU-baseline leg have
an independent statement of what the layer computes.  It shares no code with
the HIP kernels.

What it states (CPM-2 paper, arxiv 2106.10715):

* Section 2.1: the feed-forward layer of every Transformer block is expanded
  to several experts, and each token is sent to an expert chosen from its own
  hidden state by a gating function.
* Section 2.3 (MoE stage): the gate is a frozen random projection of the hidden
  state; all experts start as copies of the dense feed-forward layer.
* Table 1: d_model 4096, d_ff 10240.  The printed parameter totals (11 B dense,
  198 B with 32 experts) are only reproduced by a three-matrix gated expert
  (see model_parameter_count), so an expert is
      FFN_e(x) = (GELU(x W_gate[e]) * (x W_in[e])) W_out[e],   no biases.
* Section 6.2: tokens are routed and batched by expert before computation.
  Offloading and scheduling change where and when an expert runs, never the
  result, so the streamed mode has the same definition as the resident one.

Every floating-point step is evaluated in float64 from the stored-precision
inputs.  Readings of points the paper leaves open: selection is on the logits,
general top-k (k=1 is the paper's case), ties go to the lower expert index,
slots are ordered by descending logit, combine weights are the softmax over the
selected k (renorm=1; a single expert then has weight exactly 1) or the full
softmax probability (renorm=0), GELU is the exact erf form, and no token is
dropped.

Pinned by tests/test_oracle_*.py (brute-force loops, dense special cases, hand
computed values, invariants).
"""
from __future__ import annotations

import math
from fractions import Fraction
from functools import cmp_to_key
from typing import Callable, NamedTuple, Optional, Tuple

import numpy as np
from scipy.special import erf as _erf


class Routing(NamedTuple):
    idx: np.ndarray      # [T, k] int32, selected experts, slot j ordered by descending logit
    w: np.ndarray        # [T, k] float32 combine weights
    logits: np.ndarray   # [T, E] float64
    margin: np.ndarray   # [T] float64: smallest gap between consecutive ranks 0..k of the sorted logits


class Permutation(NamedTuple):
    counts: np.ndarray   # [E] int32
    offsets: np.ndarray  # [E+1] int32, exclusive prefix sum of counts
    perm: np.ndarray     # [A] int32: perm[row] = flat assignment index a = t*k + j
    inv: np.ndarray      # [A] int32: inv[a] = row
    Xp: np.ndarray       # [A, d] float64: Xp[row] = x[perm[row] // k]


def gelu(z: np.ndarray) -> np.ndarray:
    """Exact GELU: z * Phi(z), Phi the standard normal CDF."""
    z = np.asarray(z, dtype=np.float64)
    return 0.5 * z * (1.0 + _erf(z / math.sqrt(2.0)))


def gelu_tanh(z: np.ndarray) -> np.ndarray:
    """The tanh approximation of GELU (offered as act=1; never mixed with the exact form)."""
    z = np.asarray(z, dtype=np.float64)
    return 0.5 * z * (1.0 + np.tanh(math.sqrt(2.0 / math.pi) * (z + 0.044715 * z ** 3)))


def _act(act: int) -> Callable[[np.ndarray], np.ndarray]:
    if act == 0:
        return gelu
    if act == 1:
        return gelu_tanh
    raise ValueError("act must be 0 (erf GELU) or 1 (tanh GELU)")


def gate_logits(x: np.ndarray, Wg: np.ndarray, bias: Optional[np.ndarray] = None) -> np.ndarray:
    """L[t, e] = sum_i x[t, i] Wg[i, e] (+ b[e]): the random-projection gate of Section 2.3."""
    L = np.asarray(x, dtype=np.float64) @ np.asarray(Wg, dtype=np.float64)
    if bias is not None:
        L = L + np.asarray(bias, dtype=np.float64)[None, :]
    return L


def exact_logits_row(xt: np.ndarray, Wg: np.ndarray, bias: Optional[np.ndarray] = None) -> np.ndarray:
    """One token's logits as correctly rounded exact sums (math.fsum over the products, which are
    exact in fp64 for bf16/fp32 stored inputs): independent of summation order, so identical gate
    columns give identical logits and "tie" means a tie in exact arithmetic."""
    xt = np.asarray(xt, dtype=np.float64)
    Wg = np.asarray(Wg, dtype=np.float64)
    out = np.empty(Wg.shape[1], dtype=np.float64)
    for e in range(Wg.shape[1]):
        terms = (xt * Wg[:, e]).tolist()
        if bias is not None:
            terms.append(float(bias[e]))
        out[e] = math.fsum(terms)
    return out


def exact_dot(xt: np.ndarray, col: np.ndarray, bias_e: Optional[float] = None) -> Fraction:
    """sum_i xt[i] col[i] (+ bias_e) as an exact rational: every float is an integer times a power of two,
    so the products and their sum are formed in integer arithmetic with no rounding anywhere."""
    mx, ex = np.frexp(np.asarray(xt, dtype=np.float64))
    mw, ew = np.frexp(np.asarray(col, dtype=np.float64))
    ix = np.ldexp(mx, 53).astype(np.int64).tolist()          # 53-bit integer significands, exact
    iw = np.ldexp(mw, 53).astype(np.int64).tolist()
    sh = (ex.astype(np.int64) + ew.astype(np.int64)).tolist()
    low = min(sh) if sh else 0
    total = 0
    for a, b, s in zip(ix, iw, sh):
        if a and b:
            total += (a * b) << (s - low)
    out = Fraction(total) * Fraction(2) ** (low - 106)
    if bias_e is not None:
        out += Fraction(float(bias_e))
    return out


def _ranked(L: np.ndarray, k: int):
    order = np.argsort(-L, axis=1, kind="stable")   # descending logit, equal logits keep ascending expert index
    top = np.take_along_axis(L, order[:, :min(k + 1, L.shape[1])], axis=1)
    gaps = top[:, :-1] - top[:, 1:] if top.shape[1] > 1 else np.full((L.shape[0], 1), np.inf)
    return order, top, gaps.min(axis=1)


def _rank_exactly(Lt: np.ndarray, xt: np.ndarray, W64: np.ndarray, bias: Optional[np.ndarray], k: int):
    """Gate order of one token whose logits Lt are correctly rounded exact sums.  Rounding is monotone, so
    different floats are ordered like the exact values; only experts whose floats coincide are compared as
    exact rationals (they may still differ by less than the rounding), and a tie that survives goes to the
    lower expert index.  Returns (order, smallest exact gap between consecutive ranks 0..k)."""
    E = Lt.shape[0]
    exact = {}

    def value(e):
        if e not in exact:
            exact[e] = exact_dot(xt, W64[:, e], None if bias is None else bias[e])
        return exact[e]

    def before(a, b):
        if Lt[a] != Lt[b]:
            return -1 if Lt[a] > Lt[b] else 1
        va, vb = value(a), value(b)
        if va != vb:
            return -1 if va > vb else 1
        return -1 if a < b else 1

    order = sorted(range(E), key=cmp_to_key(before))
    gap = math.inf
    for r in range(min(k + 1, E) - 1):
        a, b = order[r], order[r + 1]
        gap = min(gap, float(value(a) - value(b)) if Lt[a] == Lt[b] else float(Lt[a] - Lt[b]))
    return order, gap


def route(x: np.ndarray, Wg: np.ndarray, k: int = 1, bias: Optional[np.ndarray] = None,
          renorm: int = 1) -> Routing:
    """Gate each token to its k best experts (Section 2.1: one expert per token, k = 1).

    The ranking is the one exact arithmetic gives.  The matrix product is a library matmul whose
    rounding error is at most about d * 2^-53 * |x_t| * |W_g column|; any token whose k+1 best
    logits are not separated by more than that bound gets its logits as correctly rounded exact sums
    (exact_logits_row) and is ranked by _rank_exactly.
    """
    x64 = np.asarray(x, dtype=np.float64)
    W64 = np.asarray(Wg, dtype=np.float64)
    L = gate_logits(x64, W64, bias)
    T, E = L.shape
    if not 1 <= k <= E:
        raise ValueError("need 1 <= k <= E")
    order, top, margin = _ranked(L, k)
    d = x64.shape[1]
    col = np.sqrt((W64 * W64).sum(axis=0)).max() if E else 0.0
    bound = (d + 4) * 2.0 ** -53 * (np.sqrt((x64 * x64).sum(axis=1)) * col + np.abs(top).max(axis=1))
    close = np.nonzero(margin <= 4.0 * bound)[0]
    for t in close:
        L[t] = exact_logits_row(x64[t], W64, bias)
    order, top, margin = _ranked(L, k)
    for t in close:
        order[t], margin[t] = _rank_exactly(L[t], x64[t], W64, bias, k)
    idx = order[:, :k].astype(np.int32)
    sel = np.take_along_axis(L, order[:, :k], axis=1)
    if renorm:
        ex = np.exp(sel - sel[:, :1])
        w = ex / ex.sum(axis=1, keepdims=True)
    else:
        m = L.max(axis=1, keepdims=True)
        ex = np.exp(L - m)
        w = np.take_along_axis(ex, idx.astype(np.int64), axis=1) / ex.sum(axis=1, keepdims=True)
    return Routing(idx, w.astype(np.float32), L, margin)


def route_hash(x: np.ndarray, Wh: np.ndarray) -> Routing:
    """Sign-bit reading of Section 2.3's gate (which the paper describes as a random projection that serves
    as a hashing function of the locality sensitive kind): the hidden state is projected on b random directions W_h[d, b] and the signs of the b
    projections, read as a binary number, name one of E = 2^b experts:
        idx[t] = sum_j [ x_t . W_h[:, j] > 0 ] * 2^j,        weight 1.
    A projection that is exactly zero gives bit 0.  As in route(), the decision is the one exact
    arithmetic gives: projections closer to zero than the matmul's error bound are re-evaluated with
    exact_logits_row.  margin = the smallest |projection| of the token."""
    x64 = np.asarray(x, dtype=np.float64)
    W64 = np.asarray(Wh, dtype=np.float64)
    L = gate_logits(x64, W64)
    T, b = L.shape
    if not 1 <= b <= 8:
        raise ValueError("need 1 <= bits <= 8")
    d = x64.shape[1]
    col = np.sqrt((W64 * W64).sum(axis=0)).max()
    bound = (d + 4) * 2.0 ** -53 * (np.sqrt((x64 * x64).sum(axis=1)) * col + np.abs(L).max(axis=1))
    for t in np.nonzero(np.abs(L).min(axis=1) <= 4.0 * bound)[0]:
        L[t] = exact_logits_row(x64[t], W64)
    code = ((L > 0.0).astype(np.int64) << np.arange(b, dtype=np.int64)[None, :]).sum(axis=1)
    return Routing(code.astype(np.int32)[:, None], np.ones((T, 1), dtype=np.float32), L, np.abs(L).min(axis=1))


def permute(x: np.ndarray, idx: np.ndarray, E: int) -> Permutation:
    """Batch the assignments by expert (Section 6.2), keeping flat order a = t*k + j inside an expert."""
    T, k = idx.shape
    flat = idx.reshape(-1).astype(np.int64)
    counts = np.bincount(flat, minlength=E).astype(np.int32)
    offsets = np.zeros(E + 1, dtype=np.int32)
    np.cumsum(counts, out=offsets[1:])
    perm = np.argsort(flat, kind="stable").astype(np.int32)   # rows: experts ascending, a ascending
    inv = np.empty(T * k, dtype=np.int32)
    inv[perm] = np.arange(T * k, dtype=np.int32)
    Xp = np.asarray(x, dtype=np.float64)[perm // k] if T * k else np.zeros((0, x.shape[1]))
    return Permutation(counts, offsets, perm, inv, Xp)


def expert_ffn_rows(X: np.ndarray, W_in: np.ndarray, W_gate: np.ndarray, W_out: np.ndarray,
                    act: int = 0) -> np.ndarray:
    """One expert applied to rows X[n, d]: (act(X W_gate) * (X W_in)) W_out."""
    X = np.asarray(X, dtype=np.float64)
    a = X @ np.asarray(W_gate, dtype=np.float64)
    b = X @ np.asarray(W_in, dtype=np.float64)
    h = _act(act)(a) * b
    return h @ np.asarray(W_out, dtype=np.float64)


ExpertSource = Callable[[int], Tuple[np.ndarray, np.ndarray, np.ndarray]]  # e -> (W_in, W_gate, W_out)


def expert_ffn(Xp: np.ndarray, offsets: np.ndarray, experts: ExpertSource, act: int = 0) -> np.ndarray:
    """Yp[r] = FFN_e(Xp[r]) for every row r of expert e's segment; empty experts are never touched."""
    A, d = Xp.shape
    Yp = np.zeros((A, d), dtype=np.float64)
    for e in range(len(offsets) - 1):
        lo, hi = int(offsets[e]), int(offsets[e + 1])
        if hi > lo:
            W_in, W_gate, W_out = experts(e)
            Yp[lo:hi] = expert_ffn_rows(Xp[lo:hi], W_in, W_gate, W_out, act)
    return Yp


def combine(Yp: np.ndarray, inv: np.ndarray, w: np.ndarray) -> np.ndarray:
    """y[t] = sum_j w[t, j] Yp[inv[t*k + j]]: the selected experts' outputs replace the FFN output."""
    T, k = w.shape
    y = np.zeros((T, Yp.shape[1]), dtype=np.float64)
    w64 = np.asarray(w, dtype=np.float64)
    inv2 = np.asarray(inv).reshape(T, k)
    for j in range(k):
        y += w64[:, j:j + 1] * Yp[inv2[:, j]]
    return y


def layer_forward_hash(x: np.ndarray, Wh: np.ndarray, experts: ExpertSource, act: int = 0):
    """The layer with the sign-bit gate: route_hash -> permute -> expert FFNs -> combine (weights are 1)."""
    r = route_hash(x, Wh)
    p = permute(x, r.idx, 1 << np.asarray(Wh).shape[1])
    Yp = expert_ffn(p.Xp, p.offsets, experts, act)
    return combine(Yp, p.inv, r.w), r, p, Yp


def layer_forward(x: np.ndarray, Wg: np.ndarray, experts: ExpertSource, E: int, k: int = 1,
                  bias: Optional[np.ndarray] = None, renorm: int = 1, act: int = 0):
    """The whole layer: route -> batch by expert -> expert FFNs -> weighted un-permute."""
    r = route(x, Wg, k, bias, renorm)
    p = permute(x, r.idx, E)
    Yp = expert_ffn(p.Xp, p.offsets, experts, act)
    y = combine(Yp, p.inv, r.w)
    return y, r, p, Yp


def model_parameter_count(n_experts: int = 1, ffn_matrices: int = 3, d: int = 4096, f: int = 10240,
                          layers: int = 24) -> int:
    """Weights in the encoder-decoder stack of Table 1 (embeddings and norms left out).

    Encoder block: self-attention (4 d^2) + FFN; decoder block: self- and cross-attention
    (8 d^2) + FFN; every FFN holds n_experts experts of ffn_matrices d-by-f matrices.
    """
    ffn = n_experts * ffn_matrices * d * f
    return layers * (4 * d * d + ffn) + layers * (8 * d * d + ffn)
