"""ctypes binding of include/moe355.h -- argument marshalling only."""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional

import torch

MOE_F32, MOE_BF16 = 0, 1
_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB: Optional[C.CDLL] = None


class MoeError(RuntimeError):
    pass


class MoeCfg(C.Structure):
    _fields_ = [("T", C.c_int32), ("d", C.c_int32), ("f", C.c_int32), ("E", C.c_int32), ("k", C.c_int32),
                ("dtype", C.c_int32), ("renorm", C.c_int32), ("act", C.c_int32), ("gate", C.c_int32),
                ("gate_packed", C.c_int32)]

    @classmethod
    def make(cls, T, d, f, E, k=1, dtype="bf16", renorm=1, act=0, gate=0, gate_packed=0) -> "MoeCfg":
        code = {"bf16": MOE_BF16, "f32": MOE_F32}[dtype] if isinstance(dtype, str) else int(dtype)
        return cls(T, d, f, E, k, code, renorm, act, gate, gate_packed)

    def with_packed_gate(self, on: bool = True) -> "MoeCfg":
        """A copy of this cfg whose W_g arguments are (or are not) the block written by moe_pack_gate."""
        return MoeCfg(self.T, self.d, self.f, self.E, self.k, self.dtype, self.renorm, self.act, self.gate, 1 if on else 0)

    @property
    def torch_dtype(self):
        return torch.bfloat16 if self.dtype == MOE_BF16 else torch.float32


def lib_path() -> str:
    """The library next to this file, or the build named by the environment variable MOE355_LIB."""
    return os.environ.get("MOE355_LIB") or os.path.join(_HERE, "libmoe355.so")


def lib() -> C.CDLL:
    """The loaded library; raises if it was never built (python -m paper_2106_10715_amd.build)."""
    global _LIB
    if _LIB is None:
        path = lib_path()
        if not os.path.exists(path):
            raise MoeError(f"{path} is missing: build it with `python paper_2106_10715_amd/build.py`; "
                           "there is no non-HIP fallback")
        L = C.CDLL(path)
        p, i32p, f32p, cfgp = C.c_void_p, C.c_void_p, C.c_void_p, C.POINTER(MoeCfg)
        L.moe_last_error.restype = C.c_char_p
        L.moe_last_error.argtypes = []
        sigs = {
            "moe_workspace_bytes": [cfgp, C.POINTER(C.c_size_t)],
            "moe_expert_bytes": [cfgp, C.POINTER(C.c_size_t)],
            "moe_pack_weights": [cfgp, p, p, p, p, p],
            "moe_gate_bytes": [cfgp, C.POINTER(C.c_size_t)],
            "moe_pack_gate": [cfgp, p, p, p],
            "moe_route": [cfgp, p, p, f32p, i32p, f32p, p, p],
            "moe_permute": [cfgp, p, i32p, i32p, i32p, i32p, i32p, p, p, p],
            "moe_permute_static": [cfgp, p, i32p, i32p, i32p, i32p, i32p, p, p],
            "moe_expert_ffn": [cfgp, p, i32p, p, p, p, p],
            "moe_combine": [cfgp, p, i32p, f32p, p, p],
            "moe_layer_forward": [cfgp, p, p, f32p, p, p, p, p, p],
            "moe_stream_ctx_create": [cfgp, p, C.c_size_t, p, C.c_int32, C.POINTER(C.c_void_p)],
            "moe_stream_ctx_destroy": [p],
            "moe_stream_ctx_stats": [p, C.POINTER(C.c_int32), C.POINTER(C.c_size_t), C.POINTER(C.c_float)],
            "moe_schedule_order": [C.POINTER(C.c_int32), C.c_int32, C.c_double, C.c_int32, C.POINTER(C.c_int32),
                                   C.POINTER(C.c_int32), C.POINTER(C.c_int32)],
            "moe_stream_ctx_set_order": [p, C.c_int32, C.c_double, C.c_int32],
            "moe_stream_ctx_last_order": [p, C.POINTER(C.c_int32), C.POINTER(C.c_int32), C.POINTER(C.c_int32)],
            "moe_stream_slots_that_fit": [C.POINTER(MoeCfg), C.c_size_t, C.POINTER(C.c_int32)],
            "moe_stream_ctx_keep_experts": [p, C.c_int32],
            "moe_stream_ctx_prefetch": [p, C.c_int32],
            "moe_stream_ctx_share_loader": [p, p],
            "moe_plan_slots": [C.POINTER(C.c_int32), C.c_int32, C.c_int32, C.POINTER(C.c_int32), C.POINTER(C.c_int64),
                               C.POINTER(C.c_int64), C.POINTER(C.c_int32), C.POINTER(C.c_int32)],
            "moe_timer_create": [C.c_int32, C.c_int32, C.POINTER(C.c_void_p)],
            "moe_timer_destroy": [p],
            "moe_timer_reset": [p],
            "moe_timer_read": [p, C.POINTER(C.c_float), C.c_int32, C.POINTER(C.c_int32)],
            "moe_layer_forward_timed": [cfgp, p, p, f32p, p, p, p, p, p],
        }
        for name, args in sigs.items():
            fn = getattr(L, name)
            fn.restype = C.c_int
            fn.argtypes = args
        _LIB = L
    return _LIB


def _check(rc: int) -> None:
    if rc != 0:
        raise MoeError(f"moe355 error {rc}: {lib().moe_last_error().decode()}")


def _ptr(t: Optional[torch.Tensor]):
    if t is None:
        return None
    if not t.is_contiguous():
        raise MoeError("tensors passed to moe355 must be contiguous")
    return C.c_void_p(t.data_ptr())


def _stream(stream: Optional[torch.cuda.Stream]):
    s = stream if stream is not None else torch.cuda.current_stream()
    return C.c_void_p(s.cuda_stream)


def moe_workspace_bytes(cfg: MoeCfg) -> int:
    n = C.c_size_t(0)
    _check(lib().moe_workspace_bytes(C.byref(cfg), C.byref(n)))
    return n.value


def moe_expert_bytes(cfg: MoeCfg) -> int:
    n = C.c_size_t(0)
    _check(lib().moe_expert_bytes(C.byref(cfg), C.byref(n)))
    return n.value


def moe_pack_weights(cfg, W_in_e, W_gate_e, W_out_e, packed_e, stream=None) -> None:
    _check(lib().moe_pack_weights(C.byref(cfg), _ptr(W_in_e), _ptr(W_gate_e), _ptr(W_out_e), _ptr(packed_e),
                                  _stream(stream)))


def moe_gate_bytes(cfg: MoeCfg) -> int:
    n = C.c_size_t(0)
    _check(lib().moe_gate_bytes(C.byref(cfg), C.byref(n)))
    return n.value


def moe_pack_gate(cfg, W_g, gate_packed, stream=None) -> None:
    _check(lib().moe_pack_gate(C.byref(cfg), _ptr(W_g), _ptr(gate_packed), _stream(stream)))


def moe_route(cfg, x, W_g, gate_bias, idx, w, ws, stream=None) -> None:
    _check(lib().moe_route(C.byref(cfg), _ptr(x), _ptr(W_g), _ptr(gate_bias), _ptr(idx), _ptr(w), _ptr(ws),
                           _stream(stream)))


def moe_permute(cfg, x, idx, counts, offsets, perm, inv, Xp, ws, stream=None) -> None:
    _check(lib().moe_permute(C.byref(cfg), _ptr(x), _ptr(idx), _ptr(counts), _ptr(offsets), _ptr(perm), _ptr(inv),
                             _ptr(Xp), _ptr(ws), _stream(stream)))


def moe_permute_static(cfg, x, idx, counts, offsets, perm, inv, Xp, stream=None) -> None:
    _check(lib().moe_permute_static(C.byref(cfg), _ptr(x), _ptr(idx), _ptr(counts), _ptr(offsets), _ptr(perm), _ptr(inv),
                                    _ptr(Xp), _stream(stream)))


def moe_expert_ffn(cfg, Xp, offsets, W_packed, Yp, ws, stream=None) -> None:
    _check(lib().moe_expert_ffn(C.byref(cfg), _ptr(Xp), _ptr(offsets), _ptr(W_packed), _ptr(Yp), _ptr(ws),
                                _stream(stream)))


def moe_combine(cfg, Yp, inv, w, y, stream=None) -> None:
    _check(lib().moe_combine(C.byref(cfg), _ptr(Yp), _ptr(inv), _ptr(w), _ptr(y), _stream(stream)))


class StreamCtx:
    """Host-streamed expert mode: experts in pinned host memory, K device slots, a copy stream."""

    def __init__(self, cfg: MoeCfg, host_experts: torch.Tensor, dev_slots: torch.Tensor, K: int = 2):
        if not host_experts.is_pinned():
            raise MoeError("host_experts must be pinned host memory")
        self._keep = (host_experts, dev_slots)
        self._h = C.c_void_p(None)
        _check(lib().moe_stream_ctx_create(C.byref(cfg), _ptr(host_experts), moe_expert_bytes(cfg), _ptr(dev_slots),
                                           K, C.byref(self._h)))

    @property
    def handle(self):
        return self._h

    def stats(self):
        n, b, ms = C.c_int32(0), C.c_size_t(0), C.c_float(0)
        _check(lib().moe_stream_ctx_stats(self._h, C.byref(n), C.byref(b), C.byref(ms)))
        return {"n_loaded": n.value, "bytes": b.value, "copy_ms": ms.value}

    def set_order(self, policy: int, tokens_per_load: float = 1.0, K: int = 0) -> None:
        _check(lib().moe_stream_ctx_set_order(self._h, policy, tokens_per_load, K))

    def keep_experts(self, on: bool = True) -> None:
        _check(lib().moe_stream_ctx_keep_experts(self._h, 1 if on else 0))

    def share_loader(self, owner: "StreamCtx") -> None:
        _check(lib().moe_stream_ctx_share_loader(self._h, owner.handle))
        self._owner = owner                      # the owner's stream must outlive this context

    def prefetch(self, expert: int) -> None:
        _check(lib().moe_stream_ctx_prefetch(self._h, int(expert)))

    def last_order(self):
        order = (C.c_int32 * 256)()
        n, ok = C.c_int32(0), C.c_int32(0)
        _check(lib().moe_stream_ctx_last_order(self._h, order, C.byref(n), C.byref(ok)))
        return list(order[:n.value]), bool(ok.value)

    def close(self):
        if self._h:
            lib().moe_stream_ctx_destroy(self._h)
            self._h = C.c_void_p(None)

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


def moe_layer_forward(cfg, x, W_g, gate_bias, W_packed, sctx: Optional[StreamCtx], y, ws, stream=None) -> None:
    _check(lib().moe_layer_forward(C.byref(cfg), _ptr(x), _ptr(W_g), _ptr(gate_bias), _ptr(W_packed),
                                   sctx.handle if sctx is not None else None, _ptr(y), _ptr(ws), _stream(stream)))


ORDER_ASCENDING, ORDER_GREEDY = 0, 1
GATE_TOPK, GATE_HASH = 0, 1


def moe_schedule_order(counts, tokens_per_load: float, K: int):
    """(order of the non-empty experts, satisfiable) for host token counts; argument marshalling only."""
    E = len(counts)
    c = (C.c_int32 * E)(*[int(v) for v in counts])
    order = (C.c_int32 * E)()
    n, ok = C.c_int32(0), C.c_int32(0)
    _check(lib().moe_schedule_order(c, E, float(tokens_per_load), int(K), order, C.byref(n), C.byref(ok)))
    return list(order[:n.value]), bool(ok.value)


def moe_plan_slots(order, slot_expert, slot_tick, tick: int):
    """(slot_of, load, slot_expert_after, slot_tick_after, tick_after); argument marshalling only."""
    n, K = len(order), len(slot_expert)
    o = (C.c_int32 * max(n, 1))(*[int(v) for v in order])
    se = (C.c_int32 * K)(*[int(v) for v in slot_expert])
    st = (C.c_int64 * K)(*[int(v) for v in slot_tick])
    tk = C.c_int64(int(tick))
    so, ld = (C.c_int32 * max(n, 1))(), (C.c_int32 * max(n, 1))()
    _check(lib().moe_plan_slots(o, n, K, se, st, C.byref(tk), so, ld))
    return list(so[:n]), [bool(v) for v in ld[:n]], list(se), list(st), tk.value


def moe_stream_slots_that_fit(cfg: MoeCfg, reserve_bytes: int = 0) -> int:
    K = C.c_int32(0)
    _check(lib().moe_stream_slots_that_fit(C.byref(cfg), int(reserve_bytes), C.byref(K)))
    return K.value


STAGES = ("route", "permute", "ffn_up", "ffn_down", "combine")
TIME_STAGES, TIME_UP_KERNEL = 0, 1


class Timer:
    """Event timing of resident layer calls (moe_timer_* of the library): all five stages, or the expert
    up-projection kernel alone."""

    def __init__(self, max_calls: int, mode: int = TIME_STAGES):
        self._h = C.c_void_p(None)
        self.mode = mode
        self.max_calls = max_calls
        _check(lib().moe_timer_create(max_calls, mode, C.byref(self._h)))

    @property
    def handle(self):
        return self._h

    def reset(self) -> None:
        _check(lib().moe_timer_reset(self._h))

    def read(self):
        """Per recorded call: {stage: ms} (all stages) or the kernel's ms (up-projection kernel alone)."""
        width = len(STAGES) if self.mode == TIME_STAGES else 1
        buf = (C.c_float * (self.max_calls * width))()
        n = C.c_int32(0)
        _check(lib().moe_timer_read(self._h, buf, self.max_calls, C.byref(n)))
        got = min(n.value, self.max_calls)
        if self.mode == TIME_STAGES:
            return [{s: buf[c * width + i] for i, s in enumerate(STAGES)} for c in range(got)]
        return [buf[c] for c in range(got)]

    def close(self) -> None:
        if self._h:
            lib().moe_timer_destroy(self._h)
            self._h = C.c_void_p(None)

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


def moe_layer_forward_timed(cfg, x, W_g, gate_bias, W_packed, y, ws, timer: Timer, stream=None) -> None:
    _check(lib().moe_layer_forward_timed(C.byref(cfg), _ptr(x), _ptr(W_g), _ptr(gate_bias), _ptr(W_packed), _ptr(y),
                                         _ptr(ws), _stream(stream), timer.handle))
