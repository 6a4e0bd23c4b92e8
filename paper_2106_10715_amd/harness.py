"""Plumbing shared by the tests, the smoke check and the bench: moves a seeded workload
(moe_workloads) into device memory and packs its experts with the library's own pack kernel.
No step of the layer is computed here."""
from __future__ import annotations

from dataclasses import dataclass
from typing import Optional

import numpy as np
import torch

import moe_workloads as W

from . import binding as B


def to_device(a: np.ndarray, dtype: str, device="cuda") -> torch.Tensor:
    """float32 array holding storage-precision values -> device tensor of the storage type."""
    if dtype == "bf16":
        bits = torch.from_numpy(W.bf16_bits(a).view(np.int16))
        return bits.to(device).view(torch.bfloat16).reshape(a.shape)
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).to(device)


def to_f64(t: torch.Tensor) -> np.ndarray:
    return t.detach().to(torch.float32).cpu().numpy().astype(np.float64)


def cfg_of(wl: W.Workload, act: int = 0) -> B.MoeCfg:
    return B.MoeCfg.make(wl.T, wl.d, wl.f, wl.E, wl.k, wl.dtype, wl.renorm, act, B.GATE_HASH if wl.gate == "hash" else B.GATE_TOPK)


@dataclass
class DeviceLayer:
    wl: W.Workload
    cfg: B.MoeCfg
    x: torch.Tensor                 # [T, d]
    Wg: torch.Tensor                # [d, E]
    bias: Optional[torch.Tensor]    # [E] fp32 or None
    packed: Optional[torch.Tensor]  # [E, expert_bytes] uint8 on the device (resident mode)
    host_packed: Optional[torch.Tensor]   # same, pinned host memory (streamed mode)
    ws: torch.Tensor                # workspace, uint8
    y: torch.Tensor                 # [T, d]


def pack_experts(wl: W.Workload, cfg: B.MoeCfg, experts=None, device="cuda", to_host: bool = False,
                 pool=None, keep_device: bool = True):
    """Generates (or takes from `experts(e)`) every expert, uploads it row-major, packs it on the GPU.
    Returns (device tensor or None, pinned host tensor or None), each [E, expert_bytes] uint8."""
    eb = B.moe_expert_bytes(cfg)
    dev = torch.empty((wl.E, eb), dtype=torch.uint8, device=device) if keep_device else None
    host = torch.empty((wl.E, eb), dtype=torch.uint8, pin_memory=True) if to_host else None
    scratch = torch.empty(eb, dtype=torch.uint8, device=device) if not keep_device else None
    bufs = None
    own_pool = pool is None and experts is None
    if own_pool:
        pool = W.make_pool()
    try:
        for e in range(wl.E):
            if experts is not None:
                W_in, W_gate, W_out = experts(e)
            else:
                if bufs is None:
                    bufs = (np.empty((wl.d, wl.f), np.float32), np.empty((wl.d, wl.f), np.float32),
                            np.empty((wl.f, wl.d), np.float32))
                W_in, W_gate, W_out = W.gen_expert(wl, e, pool, bufs)
            d_in, d_gate, d_out = (to_device(m, wl.dtype, device) for m in (W_in, W_gate, W_out))
            dst = dev[e] if keep_device else scratch
            B.moe_pack_weights(cfg, d_in, d_gate, d_out, dst)
            if host is not None:
                host[e].copy_(dst)
            torch.cuda.synchronize()
    finally:
        if own_pool:
            pool.shutdown()
    return dev, host


def build_layer(wl: W.Workload, act: int = 0, resident: bool = True, host_copy: bool = False,
                experts=None, device="cuda") -> DeviceLayer:
    cfg = cfg_of(wl, act)
    pool = W.make_pool()
    try:
        x = to_device(W.gen_x(wl, pool), wl.dtype, device)
        Wg_np, bias_np = W.gen_gate(wl)
        Wg = to_device(Wg_np, wl.dtype, device)
        bias = torch.from_numpy(bias_np).to(device) if bias_np is not None else None
        packed, host = pack_experts(wl, cfg, experts, device, to_host=host_copy, pool=pool, keep_device=resident)
    finally:
        pool.shutdown()
    ws = torch.empty(B.moe_workspace_bytes(cfg), dtype=torch.uint8, device=device)
    y = torch.empty((wl.T, wl.d), dtype=cfg.torch_dtype, device=device)
    return DeviceLayer(wl, cfg, x, Wg, bias, packed, host, ws, y)
