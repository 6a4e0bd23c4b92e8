"""GPU parity of every stage of the layer against the CPU oracle, called through the C ABI.

Bars: routing indices, counts, offsets and permutation bit-exact; fp32 outputs within 1e-5 and
bf16 outputs within 1e-2 normalised L2 of the fp64 oracle evaluated on the same stored inputs."""
import numpy as np
import pytest
import torch

import moe_workloads as W
import paper_2106_10715_amd as M
from oracle import moe_oracle as O
from paper_2106_10715_amd import harness as H

pytestmark = pytest.mark.gpu

TOL = {"f32": 1e-5, "bf16": 1e-2}


def rel_l2(got, ref):
    ref = np.asarray(ref, dtype=np.float64)
    den = np.linalg.norm(ref)
    return float(np.linalg.norm(np.asarray(got, dtype=np.float64) - ref) / (den if den > 0 else 1.0))


def rounded(a, dtype):
    a = np.ascontiguousarray(a, dtype=np.float32).copy()
    return W.round_to_bf16(a) if dtype == "bf16" else a


def make_inputs(seed, T, d, E, dtype, bias=False):
    rng = np.random.default_rng(seed)
    x = rounded(rng.standard_normal((T, d)), dtype)
    Wg = rounded(rng.standard_normal((d, E)) / np.sqrt(d), dtype)
    b = rng.standard_normal(E).astype(np.float32) * 0.5 if bias else None
    return x, Wg, b


def gpu_route(cfg, x, Wg, b, dtype):
    T, k = cfg.T, cfg.k
    dx, dW = H.to_device(x, dtype), H.to_device(Wg, dtype)
    db = torch.from_numpy(b).cuda() if b is not None else None
    idx = torch.full((T, k), -7, dtype=torch.int32, device="cuda")
    w = torch.full((T, k), -7.0, dtype=torch.float32, device="cuda")
    ws = torch.empty(M.moe_workspace_bytes(cfg), dtype=torch.uint8, device="cuda")
    M.moe_route(cfg, dx, dW, db, idx, w, ws)
    torch.cuda.synchronize()
    return idx.cpu().numpy(), w.cpu().numpy()


# ------------------------------------------------------------------------------------------- route

ROUTE_CASES = [
    # T, d, E, k, dtype, renorm, bias
    (64, 256, 4, 1, "f32", 1, False),          # the tiny fp32 configuration's gate
    (1, 64, 1, 1, "bf16", 1, False),
    (63, 128, 8, 2, "bf16", 1, True),
    (257, 512, 32, 1, "bf16", 1, False),
    (130, 192, 33, 3, "bf16", 0, True),
    (100, 256, 64, 2, "bf16", 1, True),
    (77, 128, 100, 8, "f32", 0, False),
    (50, 64, 256, 4, "bf16", 1, True),
    (33, 4096, 32, 1, "bf16", 1, False),       # the paper's width
    (19, 320, 8, 8, "f32", 1, True),           # k = E
    (90, 256, 100, 2, "bf16", 0, True),        # four expert blocks: the largest per-wave partial tiles (dynamic LDS)
    (40, 128, 160, 3, "bf16", 1, False),       # five expert blocks: one shared tile, waves add in turn
    (4100, 128, 32, 1, "bf16", 1, False),      # enough tokens for 16-token gate blocks (shorter batches use 8)
    (8200, 64, 64, 2, "bf16", 0, True),        # and for full 32-token blocks, ragged last block
    (8200, 128, 32, 1, "bf16", 1, False),      # 32-token blocks of up to 32 experts: two blocks per compute unit
]


@pytest.mark.parametrize("T,d,E,k,dtype,renorm,bias", ROUTE_CASES)
def test_route_matches_oracle(T, d, E, k, dtype, renorm, bias):
    x, Wg, b = make_inputs(100 + T + E, T, d, E, dtype, bias)
    cfg = M.MoeCfg.make(T, d, 64, E, k, dtype, renorm)
    idx, w = gpu_route(cfg, x, Wg, b, dtype)
    ref = O.route(x, Wg, k, b, renorm)
    assert np.array_equal(idx, ref.idx), f"min oracle margin {ref.margin.min():.3e}"
    assert rel_l2(w, ref.w) <= 1e-5
    assert np.abs(w - ref.w).max() <= 2e-5
    if renorm and k == 1:
        assert np.all(w == 1.0)


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_route_ties_and_near_ties(dtype):
    T, d, E, k = 96, 256, 12, 3
    x, Wg, _ = make_inputs(5, T, d, E, dtype)
    Wg[:, 7] = Wg[:, 2]                      # exact ties between experts 2, 7, 9
    Wg[:, 9] = Wg[:, 2]
    x[10] = 0.0                              # all logits exactly 0
    x[11] = 0.0
    # near ties that fp32 accumulation cannot resolve: expert 5 = expert 4 except one tiny coordinate
    Wg[:, 5] = Wg[:, 4]
    Wg[3, 5] = rounded(np.array([Wg[3, 4] * (1 + 2.0 ** -7)]), dtype)[0]
    cfg = M.MoeCfg.make(T, d, 64, E, k, dtype)
    idx, w = gpu_route(cfg, x, Wg, None, dtype)
    ref = O.route(x, Wg, k)
    assert np.array_equal(idx, ref.idx)
    assert idx[10].tolist() == [0, 1, 2] and idx[11].tolist() == [0, 1, 2]
    assert rel_l2(w, ref.w) <= 1e-5
    # the case is only meaningful if some decisions really were inside fp32 noise
    assert (ref.margin < 1e-6).sum() >= 2


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
@pytest.mark.parametrize("E,k,twins", [(12, 3, 2), (40, 2, 20)])
def test_route_ties_between_different_columns(dtype, E, k, twins):
    """Columns that are not the same and still give exactly the same projection for every token (entries i and j
    swapped, and the tokens have x_i = x_j): a tie in exact arithmetic, which sums rounded in different orders
    need not notice.  The gate must take it for a tie (lower expert first), few twins (one by one) and many (the
    block-wide pass) alike, and with a bias that breaks the tie by one unit in the last place of an fp32 it must
    follow the bias."""
    T, d = 90, 256
    x, Wg, _ = make_inputs(17, T, d, E, dtype)
    i, j = 5, 201
    first = 3
    pairs = [((i + 7 * n) % d, (j + 11 * n) % d) for n in range(1, twins)]
    for a, b in pairs:                            # every token has the same value in all coordinates that get swapped
        x[:, a] = x[:, i]
        x[:, b] = x[:, i]
    for n, (a, b) in enumerate(pairs, 1):         # twins of column `first`: the same entries, two of them swapped
        Wg[:, first + n] = Wg[:, first]
        Wg[a, first + n], Wg[b, first + n] = Wg[b, first], Wg[a, first]
    cfg = M.MoeCfg.make(T, d, 64, E, k, dtype)
    idx, w = gpu_route(cfg, x, Wg, None, dtype)
    ref = O.route(x, Wg, k)
    assert np.array_equal(idx, ref.idx)
    assert (idx == first).any()
    for slot in range(k - 1):                     # wherever a twin is selected, the next slot holds the next twin
        sel = (idx[:, slot] >= first) & (idx[:, slot] < first + twins - 1)
        assert np.all(idx[sel, slot + 1] == idx[sel, slot] + 1)
    bias = np.zeros(E, dtype=np.float32)
    bias[first + 1] = np.float32(2.0 ** -20)      # now the second twin is ahead of the first, by far less than the fp32 noise
    idx2, _ = gpu_route(cfg, x, Wg, bias, dtype)
    ref2 = O.route(x, Wg, k, bias)
    assert np.array_equal(idx2, ref2.idx)
    sel = idx2[:, 0] == first + 1
    assert sel.any() and np.all(idx2[sel, 1] == first)


def test_route_gap_far_below_the_last_place_of_an_fp64_logit():
    """fp32 inputs: two columns whose exact projections differ by 2^-83 of their size: an fp64 sum cannot tell them
    apart; the pair arithmetic of the re-evaluation can, and the higher-numbered expert, which is ahead, comes first."""
    T, d, E, k = 40, 128, 6, 2
    x, Wg, _ = make_inputs(23, T, d, E, "f32")
    x[:, 9] = np.float32(2.0 ** -60)
    Wg[:, 4] = Wg[:, 1]
    Wg[9, 1] = np.float32(1.0)
    Wg[9, 4] = np.float32(1.0 + 2.0 ** -23)
    cfg = M.MoeCfg.make(T, d, 64, E, k, "f32")
    idx, w = gpu_route(cfg, x, Wg, None, "f32")
    ref = O.route(x, Wg, k)
    assert np.array_equal(idx, ref.idx)
    sel = idx[:, 0] == 4
    assert sel.any() and np.all(idx[sel, 1] == 1) and not (idx[:, 0] == 1).any()
    assert 0.0 < ref.margin.min() < 1e-24


@pytest.mark.parametrize("E,k", [(40, 2), (200, 8)])
def test_route_many_columns_too_close_to_call(E, k):
    """More tied columns than the gate re-evaluates one by one (twenty identical experts, and tokens that are
    all zero): the block-wide fp64 pass decides, ties still go to the lower expert index."""
    T, d = 70, 256
    x, Wg, _ = make_inputs(11, T, d, E, "bf16")
    for e in range(3, 23):
        Wg[:, e] = Wg[:, 3]
    x[5] = 0.0
    x[69] = 0.0
    cfg = M.MoeCfg.make(T, d, 64, E, k, "bf16")
    idx, w = gpu_route(cfg, x, Wg, None, "bf16")
    ref = O.route(x, Wg, k)
    assert np.array_equal(idx, ref.idx)
    assert idx[5].tolist() == list(range(k)) and idx[69].tolist() == list(range(k))
    assert rel_l2(w, ref.w) <= 1e-5
    # some tokens select the twenty twins: they must come out as expert 3, then 4, ...
    assert (idx == 3).any()
    for j in range(k - 1):
        sel = (idx[:, j] >= 3) & (idx[:, j] < 22)
        assert np.all(idx[sel, j + 1] == idx[sel, j] + 1)


@pytest.mark.parametrize("T,d,bits,dtype", [(64, 256, 2, "f32"), (257, 512, 5, "bf16"), (130, 192, 8, "bf16"),
                                           (50, 64, 1, "bf16"), (33, 4096, 5, "bf16"), (77, 128, 6, "f32")])
def test_hash_gate_matches_oracle(T, d, bits, dtype):
    """Sign-bit gate: expert id = sign pattern of log2(E) projections, weight exactly 1 (integer result)."""
    x, Wh, _ = make_inputs(300 + T + bits, T, d, bits, dtype)
    cfg = M.MoeCfg.make(T, d, 64, 1 << bits, 1, dtype, gate=M.GATE_HASH)
    idx, w = gpu_route(cfg, x, Wh, None, dtype)
    ref = O.route_hash(x, Wh)
    assert np.array_equal(idx, ref.idx), f"min oracle margin {ref.margin.min():.3e}"
    assert np.all(w == 1.0)


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_hash_gate_on_and_near_the_boundaries(dtype):
    """Tokens exactly on a hyperplane (projection 0 -> bit 0), and tokens whose projection is far below what
    fp32 accumulation resolves: both sides must take the exact sign."""
    T, d, bits = 64, 256, 4
    x, Wh, _ = make_inputs(9, T, d, bits, dtype)
    x[5] = 0.0                                             # every projection exactly zero
    Wh[:, 2] = 0.0
    Wh[7, 2] = 1.0                                         # direction 2 reads coordinate 7
    x[6, 7] = 0.0                                          # exactly on hyperplane 2
    x[8, 7] = rounded(np.array([2.0 ** -100]), dtype)[0]   # barely on the positive side
    x[9, 7] = -x[8, 7]
    # a projection that cancels to a tiny value: direction 3 = (1, -1, 0, ...) on nearly equal coordinates
    Wh[:, 3] = 0.0
    Wh[0, 3], Wh[1, 3] = 1.0, -1.0
    x[10, 0] = rounded(np.array([1.0 + 2.0 ** -7]), dtype)[0]
    x[10, 1] = 1.0
    x[11, 0], x[11, 1] = 1.0, x[10, 0]
    x[12, 0] = x[12, 1] = 3.0                              # exact cancellation
    cfg = M.MoeCfg.make(T, d, 64, 1 << bits, 1, dtype, gate=M.GATE_HASH)
    idx, w = gpu_route(cfg, x, Wh, None, dtype)
    ref = O.route_hash(x, Wh)
    assert np.array_equal(idx, ref.idx)
    assert idx[5, 0] == 0
    assert (idx[6, 0] >> 2) & 1 == 0 and (idx[8, 0] >> 2) & 1 == 1 and (idx[9, 0] >> 2) & 1 == 0
    assert (idx[10, 0] >> 3) & 1 == 1 and (idx[11, 0] >> 3) & 1 == 0 and (idx[12, 0] >> 3) & 1 == 0
    assert np.all(w == 1.0)


def test_hash_gate_rejects_what_it_cannot_take():
    ws = torch.empty(1 << 20, dtype=torch.uint8, device="cuda")
    z = torch.zeros((8, 64), dtype=torch.bfloat16, device="cuda")
    i = torch.zeros((8, 1), dtype=torch.int32, device="cuda")
    wv = torch.zeros((8, 1), dtype=torch.float32, device="cuda")
    b = torch.zeros(8, dtype=torch.float32, device="cuda")
    for E, k in ((6, 1), (1, 1), (8, 2)):
        with pytest.raises(M.MoeError):
            M.moe_route(M.MoeCfg.make(8, 64, 64, E, k, "bf16", gate=M.GATE_HASH), z, z, None, i, wv, ws)
    with pytest.raises(M.MoeError):
        M.moe_route(M.MoeCfg.make(8, 64, 64, 8, 1, "bf16", gate=M.GATE_HASH), z, z, b, i, wv, ws)


def test_route_dead_experts_get_nothing():
    T, d, E, k = 200, 128, 16, 2
    x, Wg, _ = make_inputs(6, T, d, E, "bf16")
    b = np.zeros(E, dtype=np.float32)
    b[[3, 8, 15]] = W.DEAD_BIAS
    cfg = M.MoeCfg.make(T, d, 64, E, k, "bf16")
    idx, w = gpu_route(cfg, x, Wg, b, "bf16")
    ref = O.route(x, Wg, k, b)
    assert np.array_equal(idx, ref.idx)
    assert not np.isin(idx, [3, 8, 15]).any()
    np.testing.assert_allclose(w.sum(axis=1), 1.0, atol=3e-7)


# ------------------------------------------------------------------------------------------- permute

def gpu_permute(cfg, x, idx_np, dtype, with_rows=True):
    A = cfg.T * cfg.k
    dx = H.to_device(x, dtype)
    didx = torch.from_numpy(np.ascontiguousarray(idx_np, dtype=np.int32)).cuda()
    counts = torch.full((cfg.E,), -1, dtype=torch.int32, device="cuda")
    offsets = torch.full((cfg.E + 1,), -1, dtype=torch.int32, device="cuda")
    perm = torch.full((A,), -1, dtype=torch.int32, device="cuda")
    inv = torch.full((A,), -1, dtype=torch.int32, device="cuda")
    Xp = torch.zeros((A, cfg.d), dtype=cfg.torch_dtype, device="cuda") if with_rows else None
    ws = torch.empty(M.moe_workspace_bytes(cfg), dtype=torch.uint8, device="cuda")
    M.moe_permute(cfg, dx, didx, counts, offsets, perm, inv, Xp, ws)
    torch.cuda.synchronize()
    return counts.cpu().numpy(), offsets.cpu().numpy(), perm.cpu().numpy(), inv.cpu().numpy(), Xp


@pytest.mark.parametrize("T,d,E,k,dtype,skew", [
    (64, 256, 4, 1, "f32", 0.0),
    (1, 64, 1, 1, "bf16", 0.0),
    (1025, 64, 7, 1, "bf16", 0.0),           # crosses a chunk boundary by one
    (3000, 128, 32, 2, "bf16", 1.2),         # several chunks, ragged tail, skewed
    (2048, 64, 256, 4, "bf16", 0.0),
    (5000, 64, 64, 2, "f32", 2.0),           # heavy skew, some experts empty
    (999, 192, 3, 3, "bf16", 0.0),           # k = E
    (16384, 64, 32, 1, "bf16", 0.0),         # the largest batch one block still sorts alone
    (16385, 64, 32, 1, "bf16", 0.0),         # one more: per-chunk histograms, scan and scatter kernels
    (9000, 64, 64, 2, "bf16", 1.5),          # those kernels with several chunks, skew and empty experts
])
def test_permute_matches_oracle(T, d, E, k, dtype, skew):
    rng = np.random.default_rng(T + E)
    x = rounded(rng.standard_normal((T, d)), dtype)
    p = (np.arange(1, E + 1) ** -skew) if skew else np.ones(E)
    p = p / p.sum()
    idx = np.stack([rng.choice(E, size=k, replace=False, p=p) for _ in range(T)]).astype(np.int32)
    cfg = M.MoeCfg.make(T, d, 64, E, k, dtype)
    counts, offsets, perm, inv, Xp = gpu_permute(cfg, x, idx, dtype)
    ref = O.permute(x, idx, E)
    assert np.array_equal(counts, ref.counts)
    assert np.array_equal(offsets, ref.offsets)
    assert np.array_equal(perm, ref.perm)
    assert np.array_equal(inv, ref.inv)
    assert np.array_equal(H.to_f64(Xp), ref.Xp)       # pure data movement: exact


def test_permute_is_deterministic_and_index_only_mode():
    T, d, E, k = 4100, 64, 16, 2
    rng = np.random.default_rng(1)
    x = rounded(rng.standard_normal((T, d)), "bf16")
    idx = np.stack([rng.choice(E, size=k, replace=False) for _ in range(T)]).astype(np.int32)
    cfg = M.MoeCfg.make(T, d, 64, E, k, "bf16")
    a = gpu_permute(cfg, x, idx, "bf16")
    b = gpu_permute(cfg, x, idx, "bf16", with_rows=False)
    for u, v in zip(a[:4], b[:4]):
        assert np.array_equal(u, v)


def test_permute_all_tokens_to_one_expert():
    T, d, E = 2500, 64, 9
    x = rounded(np.random.default_rng(2).standard_normal((T, d)), "bf16")
    idx = np.full((T, 1), 4, dtype=np.int32)
    cfg = M.MoeCfg.make(T, d, 64, E, 1, "bf16")
    counts, offsets, perm, inv, Xp = gpu_permute(cfg, x, idx, "bf16")
    assert counts.tolist() == [0, 0, 0, 0, T, 0, 0, 0, 0]
    assert np.array_equal(perm, np.arange(T)) and np.array_equal(inv, np.arange(T))
    assert offsets.tolist() == [0] * 5 + [T] * 5


# ------------------------------------------------------------------------------------------- pack

def packed_reference(W_in, W_gate, W_out):
    """The packed bf16 layout as the header defines it, written out with plain loops over fragments."""
    d, f = W_in.shape
    out = []

    def frag(Wm, s, col0):
        fr = np.empty(512, dtype=np.uint16)
        for l in range(64):
            for j in range(8):
                fr[8 * l + j] = Wm[16 * s + 8 * (l // 32) + j, col0 + l % 32]
        return fr
    gate, win, wout = W.bf16_bits(W_gate), W.bf16_bits(W_in), W.bf16_bits(W_out)
    for n in range(f // 32):
        for s in range(d // 16):
            out.append(frag(gate, s, 32 * n))
            out.append(frag(win, s, 32 * n))
    for p in range(d // 64):
        for s in range(f // 16):
            out.append(frag(wout, s, 64 * p))
            out.append(frag(wout, s, 64 * p + 32))
    return np.concatenate(out)


def test_pack_layout_bf16_and_f32():
    d, f = 128, 192
    rng = np.random.default_rng(3)
    mats = [rounded(rng.standard_normal(s), "bf16") for s in ((d, f), (d, f), (f, d))]
    cfg = M.MoeCfg.make(1, d, f, 1, 1, "bf16")
    dev = [H.to_device(m, "bf16") for m in mats]
    out = torch.zeros(M.moe_expert_bytes(cfg), dtype=torch.uint8, device="cuda")
    M.moe_pack_weights(cfg, dev[0], dev[1], dev[2], out)
    torch.cuda.synchronize()
    got = out.cpu().numpy().view(np.uint16)
    assert np.array_equal(got, packed_reference(*mats))
    cfg32 = M.MoeCfg.make(1, d, f, 1, 1, "f32")
    dev32 = [H.to_device(m, "f32") for m in mats]
    out32 = torch.zeros(M.moe_expert_bytes(cfg32), dtype=torch.uint8, device="cuda")
    M.moe_pack_weights(cfg32, dev32[0], dev32[1], dev32[2], out32)
    torch.cuda.synchronize()
    got32 = out32.cpu().numpy().view(np.float32)
    assert np.array_equal(got32, np.concatenate([mats[1].ravel(), mats[0].ravel(), mats[2].ravel()]))


# ------------------------------------------------------------------------------------------- expert FFN

def run_ffn(T, d, f, E, k, dtype, counts, act=0, seed=0):
    """Rows already batched by expert with the given counts; returns (gpu Yp, oracle Yp)."""
    A = int(np.sum(counts))
    assert A == T * k
    rng = np.random.default_rng(seed)
    Xp = rounded(rng.standard_normal((A, d)), dtype)
    ex = [(rounded(rng.standard_normal((d, f)) * 0.05, dtype), rounded(rng.standard_normal((d, f)) * 0.05, dtype),
           rounded(rng.standard_normal((f, d)) * 0.05, dtype)) for _ in range(E)]
    offsets = np.concatenate([[0], np.cumsum(counts)]).astype(np.int32)
    cfg = M.MoeCfg.make(T, d, f, E, k, dtype, 1, act)
    wl = W.Workload("t", T, d, f, E, k, dtype, 0)
    packed, _ = H.pack_experts(wl, cfg, experts=lambda e: ex[e])
    dXp = H.to_device(Xp, dtype)
    doff = torch.from_numpy(offsets).cuda()
    Yp = torch.full((A, d), float("nan"), dtype=cfg.torch_dtype, device="cuda")
    ws = torch.empty(M.moe_workspace_bytes(cfg), dtype=torch.uint8, device="cuda")
    M.moe_expert_ffn(cfg, dXp, doff, packed, Yp, ws)
    torch.cuda.synchronize()
    ref = O.expert_ffn(Xp.astype(np.float64), offsets, lambda e: ex[e], act)
    return H.to_f64(Yp), ref, offsets


@pytest.mark.parametrize("d,f,E,counts,dtype,act", [
    (256, 512, 4, [20, 0, 37, 7], "f32", 0),                 # fp32 path, an empty expert
    (128, 192, 5, [130, 0, 1, 300, 69], "bf16", 0),          # several row tiles, ragged tails, empty expert
    (64, 64, 3, [1, 1, 1], "bf16", 0),                       # smallest legal shape: idle waves in the block
    (192, 320, 2, [129, 127], "bf16", 1),                    # tanh GELU
    (320, 128, 6, [0, 0, 64, 0, 0, 200], "f32", 1),
    (512, 1024, 3, [257, 128, 31], "bf16", 0),
    (256, 384, 3, [700, 0, 310], "bf16", 0),                 # few experts of many rows: the down-projection's tiles are cut lower than the up-projection's
    (1024, 256, 8, [250, 260, 241, 283, 256, 255, 257, 246], "bf16", 0),   # 8 experts of about a tile each: two down tiles per expert
])
def test_expert_ffn_matches_oracle(d, f, E, counts, dtype, act):
    A = sum(counts)
    got, ref, offsets = run_ffn(A, d, f, E, 1, dtype, counts, act, seed=d + f)
    assert np.isfinite(got).all()
    assert rel_l2(got, ref) <= TOL[dtype]
    for e in range(E):                                        # per segment, so a bad small expert cannot hide
        lo, hi = offsets[e], offsets[e + 1]
        if hi > lo:
            assert rel_l2(got[lo:hi], ref[lo:hi]) <= TOL[dtype], f"expert {e}"


# ------------------------------------------------------------------------------------------- combine

@pytest.mark.parametrize("T,d,k,dtype", [(64, 256, 1, "f32"), (301, 128, 2, "bf16"), (77, 192, 8, "bf16"),
                                         (50, 64, 3, "f32")])
def test_combine_matches_oracle(T, d, k, dtype):
    rng = np.random.default_rng(T)
    A = T * k
    Yp = rounded(rng.standard_normal((A, d)), dtype)
    inv = rng.permutation(A).astype(np.int32)
    w = rng.random((T, k)).astype(np.float32)
    w /= w.sum(axis=1, keepdims=True)
    cfg = M.MoeCfg.make(T, d, 64, 8, k, dtype)
    y = torch.empty((T, d), dtype=cfg.torch_dtype, device="cuda")
    M.moe_combine(cfg, H.to_device(Yp, dtype), torch.from_numpy(inv).cuda(), torch.from_numpy(w).cuda(), y)
    torch.cuda.synchronize()
    ref = O.combine(Yp.astype(np.float64), inv, w)
    got = H.to_f64(y)
    assert rel_l2(got, ref) <= (1e-6 if dtype == "f32" else 4e-3)     # one rounding to storage


def _random_ffn_case(seed):
    rng = np.random.default_rng(seed)
    d = int(rng.choice([64, 128, 192, 256, 448, 1024]))
    f = int(rng.choice([64, 128, 320, 576, 1024]))
    E = int(rng.integers(1, 9))
    kind = seed % 3
    if kind == 0:
        counts = [int(c) for c in rng.integers(0, 70, size=E)]
    elif kind == 1:
        counts = [int(c) for c in rng.choice([0, 1, 31, 32, 33, 255, 256, 257, 300, 513], size=E)]
    else:
        counts = [int(800 / (i + 1) ** 1.3) for i in range(E)]
    if sum(counts) == 0:
        counts[0] = 5
    return d, f, E, counts


@pytest.mark.parametrize("seed", range(56))
def test_expert_ffn_random_shapes(seed):
    """Seeded sweep over widths, depths and segment lengths (empty, one row, around the 32-row block and the
    256-row tile, several tiles, skewed): every segment on its own against the oracle."""
    d, f, E, counts = _random_ffn_case(1000 + seed)
    got, ref, offsets = run_ffn(sum(counts), d, f, E, 1, "bf16", counts, seed % 2, seed=seed)
    assert np.isfinite(got).all()
    for e in range(E):
        lo, hi = offsets[e], offsets[e + 1]
        if hi > lo:
            assert rel_l2(got[lo:hi], ref[lo:hi]) <= TOL["bf16"], f"expert {e}: d={d} f={f} counts={counts}"
