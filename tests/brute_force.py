"""Second, independent statement of the MoE layer, used only to pin the oracle.

Pure-Python loops over scalars (math.erf, math.exp; no numpy arithmetic, no
permutation, no offsets): every token is pushed through EVERY expert densely,
then the k-sparse gate weights pick what is kept.  Follows the same passages of
the CPM-2 paper as the oracle (Section 2.1 for "one expert per token chosen by a
gate", Section 2.3 for the projection gate, Table 1 for the expert shape).
"""
import math


def _gelu(z):
    return 0.5 * z * (1.0 + math.erf(z / math.sqrt(2.0)))


def _gelu_tanh(z):
    return 0.5 * z * (1.0 + math.tanh(math.sqrt(2.0 / math.pi) * (z + 0.044715 * z * z * z)))


def dense_ffn_token(xt, W_in, W_gate, W_out, act=0):
    d, f = len(W_in), len(W_in[0])
    g = _gelu if act == 0 else _gelu_tanh
    h = []
    for c in range(f):
        a = math.fsum(xt[i] * W_gate[i][c] for i in range(d))
        b = math.fsum(xt[i] * W_in[i][c] for i in range(d))
        h.append(g(a) * b)
    dout = len(W_out[0])
    return [math.fsum(h[c] * W_out[c][o] for c in range(f)) for o in range(dout)]


def moe_layer(x, Wg, experts, k=1, bias=None, renorm=1, act=0):
    """x: T lists of d floats; Wg: d lists of E; experts: list of (W_in, W_gate, W_out) nested lists.
    Returns (y, idx, w) as nested lists."""
    T, d, E = len(x), len(Wg), len(Wg[0])
    ys, idxs, ws = [], [], []
    for t in range(T):
        logit = [math.fsum(x[t][i] * Wg[i][e] for i in range(d)) + (bias[e] if bias is not None else 0.0)
                 for e in range(E)]
        # k picks: repeatedly take the largest remaining logit, first index wins a tie
        left = list(range(E))
        pick = []
        for _ in range(k):
            best = left[0]
            for e in left[1:]:
                if logit[e] > logit[best]:
                    best = e
            pick.append(best)
            left.remove(best)
        if renorm:
            z = [math.exp(logit[e] - logit[pick[0]]) for e in pick]
            s = math.fsum(z)
            wt = [v / s for v in z]
        else:
            m = max(logit)
            s = math.fsum(math.exp(v - m) for v in logit)
            wt = [math.exp(logit[e] - m) / s for e in pick]
        mask = [0.0] * E
        for e, v in zip(pick, wt):
            mask[e] = v
        outs = [dense_ffn_token(x[t], *experts[e], act=act) for e in range(E)]   # all experts, densely
        dout = len(outs[0])
        ys.append([math.fsum(mask[e] * outs[e][o] for e in range(E)) for o in range(dout)])
        idxs.append(pick)
        ws.append(wt)
    return ys, idxs, ws
