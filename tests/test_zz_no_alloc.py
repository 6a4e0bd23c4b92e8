"""moe_permute_static, the batching entry point for callers that cannot allocate (its scratch is a fixed
array inside the library), against moe_permute with a caller workspace: bit for bit, on two calls in a row,
the second with a smaller input, on both sides of the size at which the kernels start to use the scratch."""
import numpy as np
import pytest
import torch

import paper_2106_10715_amd as M

pytestmark = pytest.mark.gpu


def _run(which, cfg, x, idx, ws):
    T, k, E, d = cfg.T, cfg.k, cfg.E, cfg.d
    A = T * k
    t = lambda shape, dt: torch.full(shape, -7, dtype=dt, device="cuda")
    out = dict(counts=t((E,), torch.int32), offsets=t((E + 1,), torch.int32), perm=t((A,), torch.int32),
               inv=t((A,), torch.int32), Xp=torch.zeros((A, d), dtype=torch.bfloat16, device="cuda"))
    if which == "static":
        M.moe_permute_static(cfg, x, idx, out["counts"], out["offsets"], out["perm"], out["inv"], out["Xp"])
    else:
        M.moe_permute(cfg, x, idx, out["counts"], out["offsets"], out["perm"], out["inv"], out["Xp"], ws)
    torch.cuda.synchronize()
    return out


def _case(seed, T, k, E, d=128):
    g = torch.Generator(device="cpu").manual_seed(seed)
    x = torch.randn((T, d), generator=g).to(torch.bfloat16).cuda()
    # skewed expert ids, distinct within a token, a few experts without any token
    scores = torch.randn((T, E), generator=g) + torch.linspace(2.0, -2.0, E)[None, :]
    scores[:, E // 2] = -1e9
    idx = scores.topk(k, dim=1).indices.to(torch.int32).cuda()
    cfg = M.MoeCfg.make(T, d, 64, E, k)
    ws = torch.empty(M.moe_workspace_bytes(cfg), dtype=torch.uint8, device="cuda")
    return cfg, x, idx, ws


def test_static_scratch_permute_equals_workspace_permute_on_consecutive_calls():
    # chunked kernels (scratch in use): 45 chunks x 37 experts, then a smaller call that leaves most of the
    # previous call's scratch contents in place, then a short batch (one-block kernel, no scratch), then large again
    for seed, (T, k, E) in enumerate([(23001, 2, 37), (17011, 1, 9), (3000, 2, 64), (40000, 1, 256)]):
        cfg, x, idx, ws = _case(seed, T, k, E)
        got = _run("static", cfg, x, idx, None)
        want = _run("ws", cfg, x, idx, ws)
        for name in want:
            assert torch.equal(got[name], want[name]), f"case {seed} (T {T}, k {k}, E {E}): {name} differs"
        assert int(got["offsets"][-1]) == T * k and int(got["counts"][E // 2]) == 0
        assert np.array_equal(np.sort(got["perm"].cpu().numpy()), np.arange(T * k))


def test_static_scratch_permute_rejects_what_its_array_cannot_hold():
    cfg, x, idx, ws = _case(5, 1000, 1, 8)
    big = M.MoeCfg.make(262144 + 1, 128, 64, 8, 1)
    with pytest.raises(M.MoeError, match="at most 262144"):
        M.moe_permute_static(big, x, idx, ws, ws, ws, ws, None)       # rejected before anything is read
    empty = M.MoeCfg.make(0, 128, 64, 8, 1)
    counts = torch.full((8,), -1, dtype=torch.int32, device="cuda")
    offsets = torch.full((9,), -1, dtype=torch.int32, device="cuda")
    M.moe_permute_static(empty, None, None, counts, offsets, None, None, None)
    torch.cuda.synchronize()
    assert counts.tolist() == [0] * 8 and offsets.tolist() == [0] * 9
