"""Seeded synthetic inputs for the CPM-2-MoE feed-forward layer.

This module only *draws* numbers: it holds no step of the layer itself (no
logits, no routing, no FFN arithmetic).  Both the CPU oracle's tests and the
HIP path's tests/bench take their inputs from here, so the two sides consume
bit-identical stored-precision values.

Shapes follow Table 1 of the CPM-2 paper (d_model 4096, d_ff 10240) and the
32-expert setting of Section 6; the trained weights and the 40 real instances
of Section 6.2 are not available, so seeded Gaussian tensors stand in for
them:

    x        ~ N(0, 1)              hidden states            [T, d]
    W_g      ~ N(0, std 1/sqrt(d))  frozen random-projection gate (Section 2.3) [d, E]
    W_in, W_gate ~ N(0, std 0.02)   expert up-projections    [d, f] each
    W_out    ~ N(0, std 0.02)       expert down-projection   [f, d]

Every tensor is produced by a Philox counter-based stream keyed by
(seed, tensor id, expert id, chunk), so one expert can be regenerated alone
without holding the other experts in memory.  Values are returned as float32
arrays that are already rounded (round-to-nearest-even) to the storage
precision of the workload (bf16 or fp32), so "x" means exactly the same real
numbers on both sides.
"""
from __future__ import annotations

import os
from concurrent.futures import ThreadPoolExecutor
from dataclasses import dataclass, replace
from typing import Optional, Tuple

import numpy as np

# tensor ids for the Philox key
_TID_X, _TID_WG, _TID_WIN, _TID_WGATE, _TID_WOUT, _TID_PERM = 1, 2, 3, 4, 5, 6
_CHUNKS = 8  # row chunks per tensor, one Philox stream each (parallel fill)


@dataclass(frozen=True)
class Workload:
    name: str
    T: int            # tokens
    d: int            # d_model
    f: int            # d_ff
    E: int            # experts
    k: int            # experts per token (the paper uses 1)
    dtype: str        # "bf16" | "f32": storage precision of x, W_g and expert weights
    seed: int
    renorm: int = 1   # 1: softmax over the selected k; 0: full-softmax probability
    zipf_s: Optional[float] = None   # skewed loads: per-expert gate bias
    n_dead: int = 0                  # experts whose bias guarantees zero tokens
    streamed: bool = False           # experts live in pinned host memory
    gate: str = "topk"               # "topk": projection on E directions; "hash": sign bits of log2(E) projections

    @property
    def A(self) -> int:
        return self.T * self.k

    def with_tokens(self, T: int) -> "Workload":
        return replace(self, T=T, name=f"{self.name}-T{T}")


# The configurations the layer is measured on.  c1 is the small fp32 case a
# CPU finishes instantly; c3 is the CPM-2-MoE layer of Table 1 with the 32 experts
# of Section 6.2; c4a/c4b are the same layer with host-streamed experts; c5 is the
# load-imbalance stress (the imbalance problem of Section 6.2).
CONFIGS = {
    "c1": Workload("c1-tiny-f32", T=64, d=256, f=512, E=4, k=1, dtype="f32", seed=1001),
    "c2": Workload("c2-resident-E8", T=2048, d=4096, f=10240, E=8, k=1, dtype="bf16", seed=1002),
    "c3": Workload("c3-cpm2moe-E32", T=4096, d=4096, f=10240, E=32, k=1, dtype="bf16", seed=1003),
    "c4a": Workload("c4a-streamed-T512", T=512, d=4096, f=10240, E=32, k=1, dtype="bf16",
                    seed=1003, streamed=True),
    "c4b": Workload("c4b-streamed-T8192", T=8192, d=4096, f=10240, E=32, k=1, dtype="bf16",
                    seed=1003, streamed=True),
    "c5": Workload("c5-zipf-E64-top2", T=16384, d=4096, f=10240, E=64, k=2, dtype="bf16",
                   seed=1005, zipf_s=1.2, n_dead=4),
    # token-throughput regime: a fine-tuning batch of about 2^16 tokens (Section 4.1), 2048 tokens per
    # expert, every expert bound by the matrix cores instead of by streaming its weights
    "c6": Workload("c6-T65536-E32", T=65536, d=4096, f=10240, E=32, k=1, dtype="bf16", seed=1006),
}

# Bias of an expert that must receive no token at all.
DEAD_BIAS = -1.0e9


def round_to_bf16(a: np.ndarray) -> np.ndarray:
    """Round float32 values to the nearest bf16 (ties to even), in place; returns a."""
    u = a.view(np.uint32)
    u += np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))
    u &= np.uint32(0xFFFF0000)
    return a


def bf16_bits(a: np.ndarray) -> np.ndarray:
    """uint16 bit patterns of a float32 array that already holds bf16 values."""
    return (np.ascontiguousarray(a).view(np.uint32) >> np.uint32(16)).astype(np.uint16)


def _n_threads() -> int:
    return max(1, min(16, os.cpu_count() or 1))


def _fill_chunk(out: np.ndarray, seed: int, tid: int, expert: int, chunk: int,
                std: float, dtype: str) -> None:
    key = np.array([np.uint64(seed), np.uint64((tid << 40) | (expert << 8) | chunk)],
                   dtype=np.uint64)
    g = np.random.Generator(np.random.Philox(key=key))
    g.standard_normal(out=out, dtype=np.float32)
    if std != 1.0:
        out *= np.float32(std)
    if dtype == "bf16":
        round_to_bf16(out)


def _gaussian(shape: Tuple[int, int], seed: int, tid: int, expert: int, std: float,
              dtype: str, pool: Optional[ThreadPoolExecutor] = None,
              out: Optional[np.ndarray] = None) -> np.ndarray:
    rows, cols = shape
    if out is None:
        out = np.empty(shape, dtype=np.float32)
    flat = out.reshape(-1)
    n = flat.size
    bounds = [(n * c) // _CHUNKS for c in range(_CHUNKS + 1)]
    jobs = [(flat[bounds[c]:bounds[c + 1]], seed, tid, expert, c, std, dtype)
            for c in range(_CHUNKS) if bounds[c + 1] > bounds[c]]
    if pool is None or n < (1 << 20):
        for j in jobs:
            _fill_chunk(*j)
    else:
        list(pool.map(lambda j: _fill_chunk(*j), jobs))
    return out


def _fit_load_bias(p: np.ndarray, k: int, seed: int, n: int = 120000,
                   iters: int = 25) -> np.ndarray:
    """Biases b_r such that i.i.d. N(0,1) scores plus b put a share p_r of the
    top-k picks on rank r.  Gaussian scores are probit- not Gumbel-distributed, so
    b = ln p does not do it; this fixed-point iteration on a private sample of
    standard normals (not on the workload's tensors) does.  Deterministic in seed."""
    live = p.size
    key = np.array([np.uint64(seed), np.uint64(7 << 40)], dtype=np.uint64)
    z = np.random.Generator(np.random.Philox(key=key)).standard_normal((n, live), dtype=np.float32)
    b = 0.8 * np.log(p)
    for _ in range(iters):
        s = z + b.astype(np.float32)
        top = np.argpartition(-s, k, axis=1)[:, :k] if k < live else np.tile(np.arange(live), (n, 1))
        share = np.bincount(top.ravel(), minlength=live) / top.size
        share = np.maximum(share, 0.1 / top.size)
        b += 0.5 * (np.log(p) - np.log(share))
        b -= b.max()
    return b


def make_pool() -> ThreadPoolExecutor:
    return ThreadPoolExecutor(max_workers=_n_threads())


def gen_x(wl: Workload, pool: Optional[ThreadPoolExecutor] = None) -> np.ndarray:
    """Hidden states x[T, d], float32 holding storage-precision values."""
    if wl.T == 0:
        return np.empty((0, wl.d), dtype=np.float32)
    return _gaussian((wl.T, wl.d), wl.seed, _TID_X, 0, 1.0, wl.dtype, pool)


def gen_gate(wl: Workload) -> Tuple[np.ndarray, Optional[np.ndarray]]:
    """Gate projection W_g[d, E] and, for skewed workloads, the bias b[E] (fp32); for the hashing gate
    W_g[d, log2 E] and no bias."""
    if wl.gate == "hash":
        bits = wl.E.bit_length() - 1
        assert 1 << bits == wl.E and wl.k == 1 and wl.zipf_s is None
        return _gaussian((wl.d, bits), wl.seed, _TID_WG, 0, 1.0 / np.sqrt(wl.d), wl.dtype), None
    Wg = _gaussian((wl.d, wl.E), wl.seed, _TID_WG, 0, 1.0 / np.sqrt(wl.d), wl.dtype)
    bias = None
    if wl.zipf_s is not None:
        live = wl.E - wl.n_dead
        p = np.arange(1, live + 1, dtype=np.float64) ** (-wl.zipf_s)
        p /= p.sum()
        by_rank = np.full(wl.E, DEAD_BIAS, dtype=np.float64)
        by_rank[:live] = _fit_load_bias(p, wl.k, wl.seed)
        key = np.array([np.uint64(wl.seed), np.uint64(_TID_PERM << 40)], dtype=np.uint64)
        order = np.random.Generator(np.random.Philox(key=key)).permutation(wl.E)
        bias = np.empty(wl.E, dtype=np.float32)
        bias[order] = by_rank.astype(np.float32)   # rank r lives at expert id order[r]
    return Wg, bias


def gen_expert(wl: Workload, e: int, pool: Optional[ThreadPoolExecutor] = None,
               out: Optional[Tuple[np.ndarray, np.ndarray, np.ndarray]] = None
               ) -> Tuple[np.ndarray, np.ndarray, np.ndarray]:
    """(W_in[d,f], W_gate[d,f], W_out[f,d]) of expert e, float32 holding storage values."""
    o = out if out is not None else (None, None, None)
    W_in = _gaussian((wl.d, wl.f), wl.seed, _TID_WIN, e, 0.02, wl.dtype, pool, o[0])
    W_gate = _gaussian((wl.d, wl.f), wl.seed, _TID_WGATE, e, 0.02, wl.dtype, pool, o[1])
    W_out = _gaussian((wl.f, wl.d), wl.seed, _TID_WOUT, e, 0.02, wl.dtype, pool, o[2])
    return W_in, W_gate, W_out


def expert_bytes(wl: Workload) -> int:
    """Bytes of one expert's three matrices in storage precision."""
    es = 2 if wl.dtype == "bf16" else 4
    return 3 * wl.d * wl.f * es
