#!/usr/bin/env python3
"""Throughput of the CPM-2-MoE feed-forward layer on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload c3|c2|c5|c6|c4a|c4b] [--tokens T]

A step is one moe_layer_forward (route -> permute -> expert FFNs -> combine) over one batch of
seeded synthetic tokens that is already resident in HBM.  Prints ONE JSON line: whole-layer
tokens/s, the roofline figure of the dominant kernel (the fused gate/in up-projection of the expert
FFNs; duration measured with HIP events on the launch stream inside every tenth timed step), per-stage
times, the same step replayed from a captured HIP graph, a short host-streamed leg on the same weights
(host-to-device rate and load/compute overlap: the other half of the metric), and the CPU oracle timed on
the host cores on a bounded sample of the same workload.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E, published
MFMA_BF16_PEAK_TFLOPS = 2500.0  # MI355X dense bf16 matrix peak, published


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=None,
                    help="timed steps (default 200 with resident experts, 30 with host-streamed ones)")
    ap.add_argument("--warmup", type=int, default=None,
                    help="untimed steps before them (default 30 resident: the first twenty or so steps after an idle "
                         "GPU run 2-3 %% slower than the steady state; 5 streamed)")
    ap.add_argument("--workload", default="c3", choices=["c2", "c3", "c4a", "c4b", "c5", "c6"])
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-streaming-leg", action="store_true",
                    help="resident c3 run: leave out the short host-streamed leg (T 512, the same weights) that fills the "
                         "'streaming' record")
    ap.add_argument("--no-graph", action="store_true", help="resident run: leave out the captured-graph replay")
    ap.add_argument("--no-mfma-leg", action="store_true",
                    help="resident c3 run: leave out the short leg at T 65536 on the same experts (2048 tokens per expert: the "
                         "regime bound by the matrix cores), which fills the 'mfma_leg' record")
    ap.add_argument("--tokens", type=int, default=None,
                    help="run the workload's layer on this many tokens instead of its own count (a sweep over batch sizes; "
                         "the figure the workload is quoted on is the one without this option)")
    ap.add_argument("--streamed", action="store_true", help="run the workload with host-streamed experts even if it is defined resident")
    ap.add_argument("--slots", type=int, default=4,
                    help="device slots of the streamed mode (with 4 or more, the copy stream waits for freed slots once "
                         "per K/2 copies instead of before every copy)")
    ap.add_argument("--layers", type=int, default=1,
                    help="streamed workloads: run a stack of this many layers (own context and slots each, the same host "
                         "weights, layer l+1 fed with layer l's output) and report what is exposed per layer when the layers "
                         "run one by one against per model when the next layer's first expert is prefetched under the "
                         "current layer (Section 6.2: only the first expert waits for its parameters)")
    ap.add_argument("--order", default="ascending", choices=["ascending", "greedy"],
                    help="streamed mode: expert execution order (greedy = the paper's Section 6.2 schedule)")
    ap.add_argument("--keep-experts", action="store_true",
                    help="streamed mode: slots keep their experts between steps (with --slots >= experts only the "
                         "warm-up loads anything); not the measured streamed configuration, which reloads every step")
    ap.add_argument("--tokens-per-load", type=float, default=None,
                    help="greedy order: tokens whose computation lasts as long as one expert load "
                         "(default: from the published peaks, beta = expert bytes / 64 GB/s, alpha = 6 d f / 2.5 PFLOP/s)")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run one plain 1 GiB device-to-device copy (a kernel of known traffic, for scaling "
                         "FETCH_SIZE / WRITE_SIZE counters of a rocprofv3 --pmc run)")
    return ap.parse_args()


def measured_traffic(workload: str, which: str):
    """HBM bytes per launch of an expert FFN kernel as the FETCH_SIZE / WRITE_SIZE counters of rocprofv3
    gave them (table written next to the library from the counter runs summarised under profiles/), or
    None when there is no figure for this workload or the kernel source has changed since."""
    import hashlib
    pkg = os.path.join(ROOT, "paper_2106_10715_amd")
    try:
        tab = json.load(open(os.path.join(pkg, "ffn_traffic.json")))
        sha = hashlib.sha256(open(os.path.join(pkg, "csrc", "ffn.hip"), "rb").read()).hexdigest()
    except OSError:
        return None
    if tab.get("source_sha256") != sha or workload not in tab:
        return None
    t = tab[workload][which]
    return {"read_bytes": t["read_bytes"], "write_bytes": t["write_bytes"], "bytes": t["read_bytes"] + t["write_bytes"],
            "source": "replayed, not measured by this run: rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE of an earlier run "
                      f"(summary under profiles/, {tab.get('profile', 'ffn_hbm_traffic')}); valid for ffn.hip sha256 {sha[:12]}"}


def cpu_baseline(wl, counts):
    """The oracle as it stands, timed on the host cores on a bounded sample: routing and batching of
    the whole batch, then the expert FFN of the first experts' complete segments until about
    15 s of CPU work is spent (the combine, a scaled row copy, is left out of the sample).  tokens/s = sampled assignments / (their FFN time + the
    proportional share of routing time)."""
    import numpy as np

    import moe_workloads as W
    from oracle import moe_oracle as O

    x = W.gen_x(wl)
    Wg, bias = W.gen_gate(wl)
    t0 = time.perf_counter()
    r = O.route(x, Wg, wl.k, bias, wl.renorm)
    p = O.permute(x, r.idx, wl.E)
    t_route = time.perf_counter() - t0
    assert np.array_equal(p.counts, counts), "oracle and GPU disagree on expert counts"
    pool = W.make_pool()
    done, t_ffn, experts = 0, 0.0, 0
    budget = 15.0
    try:
        for e in range(wl.E):
            n = int(p.counts[e])
            if n == 0:
                continue
            mats = W.gen_expert(wl, int(e), pool)                 # input generation is not timed
            lo = int(p.offsets[e])
            t1 = time.perf_counter()
            O.expert_ffn_rows(p.Xp[lo:lo + n], *mats)
            t_ffn += time.perf_counter() - t1
            done += n
            experts += 1
            if t_ffn > budget:
                break
    finally:
        pool.shutdown()
    A = wl.T * wl.k
    total = t_ffn + t_route * done / A
    try:
        import threadpoolctl
        threads = max((i.get("num_threads", 1) for i in threadpoolctl.threadpool_info()), default=1)
    except Exception:
        threads = os.cpu_count() or 1
    return {"value": (done / wl.k) / total, "unit": "tokens/s", "cores": int(threads), "kind": "oracle",
            "sample": f"route+permute of all {wl.T} tokens ({t_route:.2f} s, charged pro rata) and fp64 expert FFN of "
                      f"{experts} complete expert segments = {done} assignments ({t_ffn:.2f} s)"}


def streamed_leg(M, torch, np, cfg, x, gate, bias, host_packed, y, ws, wl, steps, warmup, n_slots, order="ascending",
                 keep=False, tokens_per_load=None):
    """Host-streamed steps of the layer (Section 6.2: experts in pinned host memory, loaded on a copy stream
    while earlier experts compute): per-step time, host-to-device rate over the copy window, and how much of
    the shorter of (the same copies alone, the same layer with resident experts) the streamed step hides."""
    eb = M.moe_expert_bytes(cfg)
    slots = torch.empty((n_slots, eb), dtype=torch.uint8, device="cuda")
    ctx = M.StreamCtx(cfg, host_packed, slots, n_slots)
    if keep:
        ctx.keep_experts(True)
    if order == "greedy":
        # Section 6.2 takes alpha and beta from the peak rates of the machine
        tpl = tokens_per_load or (eb / 64e9) / (6.0 * wl.d * wl.f / (MFMA_BF16_PEAK_TFLOPS * 1e12))
        ctx.set_order(M.ORDER_GREEDY, tpl, n_slots)

    def step():
        M.moe_layer_forward(cfg, x, gate, bias, None, ctx, y, ws)

    for _ in range(warmup):
        step()
    torch.cuda.synchronize()
    copy_ms, copy_bytes, loaded = [], 0, []
    t0 = time.perf_counter()
    for _ in range(steps):
        step()
        st = ctx.stats()                         # per-call copy figures; the wait is part of the streamed step anyway
        copy_ms.append(st["copy_ms"])
        copy_bytes = st["bytes"]
        loaded.append(st["n_loaded"])
    torch.cuda.synchronize()
    ms_per_step = (time.perf_counter() - t0) * 1e3 / steps
    cm = float(np.mean(copy_ms))
    h2d = copy_bytes / (cm * 1e-3) / 1e9 if cm > 0 else 0.0
    roof = {"bound": "h2d", "achieved": h2d, "peak": 64.0, "unit": "GB/s", "frac": h2d / 64.0, "traffic": None,
            "kernel": "hipMemcpyAsync pinned host -> HBM slot (copy stream)", "avg_copy_window_ms": cm,
            "bytes_per_step": copy_bytes, "note": "peak = PCIe Gen5 x16 raw, one direction"}
    rec = {"workload": wl.name, "T": wl.T, "slots": n_slots, "order": order, "steps": steps, "warmup": warmup,
           "tokens_per_s": wl.T / (ms_per_step * 1e-3), "h2d_gbs": h2d, "h2d_frac_of_64_gbs": h2d / 64.0,
           "copy_window_ms": cm, "step_ms": ms_per_step, "copy_share_of_step": cm / ms_per_step if ms_per_step > 0 else 0.0,
           "experts_loaded_per_step": float(np.mean(loaded))}
    counts = torch.empty(cfg.E, dtype=torch.int32, device="cuda")
    idx = torch.empty((wl.T, wl.k), dtype=torch.int32, device="cuda")
    w = torch.empty((wl.T, wl.k), dtype=torch.float32, device="cuda")
    offsets = torch.empty(cfg.E + 1, dtype=torch.int32, device="cuda")
    perm = torch.empty(wl.A, dtype=torch.int32, device="cuda")
    inv = torch.empty(wl.A, dtype=torch.int32, device="cuda")
    M.moe_route(cfg, x, gate, bias, idx, w, ws)
    M.moe_permute(cfg, x, idx, counts, offsets, perm, inv, None, ws)
    torch.cuda.synchronize()
    live_experts = [int(e) for e in np.nonzero(counts.cpu().numpy())[0]]
    if not keep:
        # Overlap of loading and computing (Section 6.2: separate streams so that the two run side by side):
        # the same copies alone (back to back on a side stream, nothing else running), the same layer alone
        # (experts resident), and how much of the shorter of the two the streamed step hides.
        side = torch.cuda.Stream()
        ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        alone_ms = []
        for _ in range(3):
            torch.cuda.synchronize()
            with torch.cuda.stream(side):
                ev0.record(side)
                for i, e in enumerate(live_experts):
                    slots[i % n_slots].copy_(host_packed[e], non_blocking=True)
                ev1.record(side)
            ev1.synchronize()
            alone_ms.append(ev0.elapsed_time(ev1))
        copy_alone_ms = float(np.mean(alone_ms[1:]))
        resident = torch.empty((cfg.E, eb), dtype=torch.uint8, device="cuda")
        resident.copy_(host_packed)
        torch.cuda.synchronize()
        for _ in range(3):
            M.moe_layer_forward(cfg, x, gate, bias, resident, None, y, ws)
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        for _ in range(10):
            M.moe_layer_forward(cfg, x, gate, bias, resident, None, y, ws)
        torch.cuda.synchronize()
        compute_alone_ms = (time.perf_counter() - t1) * 1e3 / 10
        del resident
        shorter = min(copy_alone_ms, compute_alone_ms)
        copy_alone_gbs = len(live_experts) * eb / (copy_alone_ms * 1e-3) / 1e9
        rec.update({
            "copy_alone_ms": copy_alone_ms, "copy_alone_gbs": copy_alone_gbs, "compute_alone_ms": compute_alone_ms,
            "exposed_ms": ms_per_step - max(copy_alone_ms, compute_alone_ms),
            "overlap": (copy_alone_ms + compute_alone_ms - ms_per_step) / shorter,
            "overlap_note": "(copies alone + layer alone - streamed step) / the shorter of the two; 1 = the shorter one is "
                            "hidden completely; exposed_ms = streamed step - the longer of the two",
            "h2d_frac_of_copies_alone": h2d / copy_alone_gbs})
    if order == "greedy":
        o, ok = ctx.last_order()
        rec.update({"order_first": o[:8], "order_last": o[-4:], "constraints_satisfiable": ok})
    ctx.close()
    del slots
    return ms_per_step, roof, rec, counts.cpu().numpy()


def stack_leg(M, torch, np, cfg, x, gate, bias, host_packed, wl, n_layers, n_slots, steps, warmup):
    """A stack of streamed layers (each with its own context and slots; layer l+1 reads layer l's output; all layers load
    through the copy streams of the first, moe_stream_ctx_share_loader).  Slots keep their experts, so that an expert
    requested ahead of its layer's call is found resident by it:
      one by one   every layer's call is waited for before the next is issued, nothing is requested ahead
      pipelined    as soon as the call of layer l has returned (its loads are queued), the first expert of layer l+1 is
                   requested (moe_stream_ctx_prefetch), so that it is loaded while layer l finishes and layer l+1
                   routes; the calls follow each other without a wait in between
    Both load every non-empty expert of every layer in every pass (what the slots hold is forgotten between passes)."""
    eb = M.moe_expert_bytes(cfg)
    ctxs, keep = [], []
    for _ in range(n_layers):
        slots = torch.empty((n_slots, eb), dtype=torch.uint8, device="cuda")
        ctx = M.StreamCtx(cfg, host_packed, slots, n_slots)
        if ctxs:
            ctx.share_loader(ctxs[0])            # one loader (two copy streams) for the whole stack
        ctxs.append(ctx)
        keep.append(slots)
    ws = torch.empty(M.moe_workspace_bytes(cfg), dtype=torch.uint8, device="cuda")
    acts = [x] + [torch.empty_like(x) for _ in range(n_layers)]
    counts = torch.empty(cfg.E, dtype=torch.int32, device="cuda")

    def first_expert(l):
        """The expert layer l will run first (ascending order: its lowest non-empty expert), by the staged calls."""
        idx = torch.empty((wl.T, wl.k), dtype=torch.int32, device="cuda")
        w = torch.empty((wl.T, wl.k), dtype=torch.float32, device="cuda")
        offsets = torch.empty(cfg.E + 1, dtype=torch.int32, device="cuda")
        perm = torch.empty(wl.A, dtype=torch.int32, device="cuda")
        inv = torch.empty(wl.A, dtype=torch.int32, device="cuda")
        M.moe_route(cfg, acts[l], gate, bias, idx, w, ws)
        M.moe_permute(cfg, acts[l], idx, counts, offsets, perm, inv, None, ws)
        torch.cuda.synchronize()
        return int(np.nonzero(counts.cpu().numpy())[0][0])

    def one_pass(pipelined, firsts):
        for ctx in ctxs:                         # every pass loads everything: forget what the slots hold
            ctx.keep_experts(False)
            ctx.keep_experts(True)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        ends = []
        for l in range(n_layers):
            M.moe_layer_forward(cfg, acts[l], gate, bias, None, ctxs[l], acts[l + 1], ws)
            if pipelined and l + 1 < n_layers:
                ctxs[l + 1].prefetch(firsts[l + 1])
            if not pipelined:
                torch.cuda.synchronize()
                ends.append((time.perf_counter() - t0) * 1e3)
        torch.cuda.synchronize()
        per_layer.append([round(b - a, 3) for a, b in zip([0.0] + ends, ends)])
        return (time.perf_counter() - t0) * 1e3, sum(c.stats()["n_loaded"] for c in ctxs)

    per_layer = []
    # a first pass fixes the activations of every layer (and with them which expert each layer runs first)
    one_pass(False, None)
    firsts = [first_expert(l) for l in range(n_layers)]
    res = {}
    for name, pipelined in (("one_by_one", False), ("pipelined", True)):
        for _ in range(warmup):
            one_pass(pipelined, firsts)
        ms, loads = zip(*[one_pass(pipelined, firsts) for _ in range(steps)])
        res[name] = {"ms_per_pass": float(np.mean(ms)), "ms_passes": [round(float(v), 3) for v in ms],
                     "loads_in_calls_per_pass": float(np.mean(loads))}
        if not pipelined:
            res[name]["ms_per_layer_last_pass"] = per_layer[-1]
    for c in reversed(ctxs):                     # the owner of the shared copy stream last
        c.close()
    return res


def main():
    args = parse()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py measures one GPU: the layer is built and measured on a single MI355X (--gpus 1); "
              "sharding over several GPUs is described in the design notes, not built", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch

    import moe_workloads as W
    import paper_2106_10715_amd as M
    from paper_2106_10715_amd import harness as H

    if not torch.cuda.is_available():
        print("bench.py needs a GPU", file=sys.stderr)
        sys.exit(2)
    torch.cuda.set_device(0)
    M.lib()                                     # fails loudly if the HIP library is not built
    wl = W.CONFIGS[args.workload]
    if args.tokens is not None:
        if args.tokens < 1:
            sys.exit("bench.py: --tokens must be positive")
        wl = wl.with_tokens(args.tokens)
    if args.streamed and not wl.streamed:
        import dataclasses
        wl = dataclasses.replace(wl, streamed=True, name=wl.name + "-streamed")
    if args.steps is None:
        args.steps = 30 if wl.streamed else 200
    if args.warmup is None:
        args.warmup = 5 if wl.streamed else 30
    if args.steps < 1 or args.warmup < 0:
        sys.exit("bench.py: --steps must be positive and --warmup not negative")
    # the default run (the layer the metric is quoted on, experts resident) also runs a short streamed leg on the
    # same weights, which needs them in pinned host memory as well
    streaming_leg = (not wl.streamed and args.workload == "c3" and args.tokens is None and not args.no_streaming_leg)
    t_setup = time.perf_counter()
    L = H.build_layer(wl, resident=not wl.streamed, host_copy=wl.streamed or streaming_leg)
    # the gate is frozen (Section 2.3): packed once, like the experts
    gate = torch.empty(M.moe_gate_bytes(L.cfg), dtype=torch.uint8, device="cuda")
    M.moe_pack_gate(L.cfg, L.Wg, gate)
    cfg = L.cfg.with_packed_gate()
    torch.cuda.synchronize()
    print(f"[bench] {wl.name}: inputs resident after {time.perf_counter() - t_setup:.1f} s", file=sys.stderr, flush=True)
    A, d, f, es = wl.A, wl.d, wl.f, 2 if wl.dtype == "bf16" else 4

    out = {
        "metric": "MoE-FFN tokens/s (d4096,ff10240,E32,bf16)" if args.workload in ("c3", "c4a", "c4b")
                  else f"MoE-FFN tokens/s (d{d},ff{f},E{wl.E},{wl.dtype})",
        "value": None, "unit": "tokens/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": None, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": wl.dtype, "data": "synthetic",
    }

    if wl.streamed:
        ms_per_step, roof, rec, counts = streamed_leg(M, torch, np, cfg, L.x, gate, L.bias, L.host_packed, L.y, L.ws, wl,
                                                      args.steps, args.warmup, args.slots, args.order, args.keep_experts,
                                                      args.tokens_per_load)
        out["roofline"] = roof
        out["streaming"] = rec
        if args.layers > 1:
            st = stack_leg(M, torch, np, cfg, L.x, gate, L.bias, L.host_packed, wl, args.layers, args.slots,
                           max(3, args.steps // 4), 2)
            if "copy_alone_ms" in rec:
                for v in st.values():
                    if not isinstance(v, dict):
                        continue
                    v["exposed_ms_per_pass"] = v["ms_per_pass"] - args.layers * rec["copy_alone_ms"]
                    v["exposed_ms_per_layer"] = v["exposed_ms_per_pass"] / args.layers
            out["stack"] = {"layers": args.layers, **st,
                            "note": "exposed = pass time - layers x (the same copies alone); one_by_one pays the first load's "
                                    "lead-in and the last expert's tail once per layer, pipelined once per model"}
    else:
        def step():
            M.moe_layer_forward(cfg, L.x, gate, L.bias, L.packed, None, L.y, L.ws)

        if args.calibrate_copy:
            src = torch.zeros(1 << 30, dtype=torch.uint8, device="cuda")
            dst = torch.empty_like(src)
            torch.cuda.synchronize()
            dst.copy_(src)
            torch.cuda.synchronize()
            del src, dst
        # The two short legs that fill the other halves of the metric run first, the host-streamed one (mostly copies)
        # before the one at T 65536 (heavy matrix load), and the resident measurement follows at once: after an idle
        # spell (the set-up generates weights on the host for seconds) the first ten to twenty layer steps run 5-30 %
        # slow while the GPU's power management settles, which a run of 5 warm-up and 20 timed steps would mostly
        # measure; straight after the T 65536 leg the first steps already run at the steady rate.
        if streaming_leg:
            # the other half of the metric: the same layer and weights with host-streamed experts, on the short batch
            # of the streamed configuration (T 512); a few steps are enough, every step moves all 32 experts
            wls = W.CONFIGS["c4a"]
            cfgs = H.cfg_of(wls).with_packed_gate()
            xs = H.to_device(W.gen_x(wls), wls.dtype)
            wss = torch.empty(M.moe_workspace_bytes(cfgs), dtype=torch.uint8, device="cuda")
            ys = torch.empty((wls.T, wls.d), dtype=cfgs.torch_dtype, device="cuda")
            _, sroof, srec, _ = streamed_leg(M, torch, np, cfgs, xs, gate, None, L.host_packed, ys, wss, wls, 5, 2,
                                             args.slots)
            srec["roofline"] = sroof
            out["streaming"] = srec
        if args.workload == "c3" and args.tokens is None and not args.no_mfma_leg:
            # "% of the MFMA peak" is only meaningful where the matrix cores bind: the same layer and experts on a batch of
            # 2^16 tokens (a fine-tuning batch of Section 4.1), every expert with about 2048 rows
            wlm = wl.with_tokens(65536)
            cfgm = H.cfg_of(wlm).with_packed_gate()
            xm = H.to_device(W.gen_x(wlm), wlm.dtype)
            wsm = torch.empty(M.moe_workspace_bytes(cfgm), dtype=torch.uint8, device="cuda")
            ym = torch.empty((wlm.T, wlm.d), dtype=cfgm.torch_dtype, device="cuda")
            for _ in range(3):
                M.moe_layer_forward(cfgm, xm, gate, L.bias, L.packed, None, ym, wsm)
            torch.cuda.synchronize()
            n_m = 10
            t1 = time.perf_counter()
            for _ in range(n_m):
                M.moe_layer_forward(cfgm, xm, gate, L.bias, L.packed, None, ym, wsm)
            torch.cuda.synchronize()
            m_ms = (time.perf_counter() - t1) * 1e3 / n_m
            tm = M.Timer(4, M.TIME_STAGES)
            for _ in range(4):
                M.moe_layer_forward_timed(cfgm, xm, gate, L.bias, L.packed, ym, wsm, tm)
            torch.cuda.synchronize()
            st = tm.read()
            tm.close()
            upm = float(np.mean([c["ffn_up"] for c in st]))
            dnm = float(np.mean([c["ffn_down"] for c in st]))
            fl = 6.0 * d * f * wlm.A
            out["mfma_leg"] = {"workload": wlm.name, "T": wlm.T, "steps": n_m, "ms_per_step": m_ms, "tokens_per_s": wlm.T / (m_ms * 1e-3),
                               "ffn_up_ms": upm, "ffn_down_ms": dnm, "ffn_tflops": fl / ((upm + dnm) * 1e-3) / 1e12,
                               "mfma_frac": fl / ((upm + dnm) * 1e-3) / 1e12 / MFMA_BF16_PEAK_TFLOPS,
                               "up_kernel_tflops": 4.0 * d * f * wlm.A / (upm * 1e-3) / 1e12, "peak_tflops": MFMA_BF16_PEAK_TFLOPS,
                               "note": "the layer and experts of the run above on 65536 tokens; kernel times from 4 extra steps with "
                                       "events between the stages (ffn_up includes the work-list kernel)"}
            del xm, wsm, ym
        if "mfma_leg" in out:
            out["order_note"] = ("the streaming and mfma legs ran before the warm-up and timed steps of the resident measurement "
                                 "(GPU under load when the warm-up starts); with them after it, the first steps after the idle "
                                 "set-up run slow and 20 timed steps after 5 warm-up steps measure about 3 % more per step")
        for _ in range(args.warmup):
            step()
        torch.cuda.synchronize()
        # two events around the dominant kernel in every tenth step, every third in short runs (each event costs
        # the step some 7 us of idle time between two kernels): those steps go through the timed entry point
        every = 10 if args.steps >= 100 else 3
        up_timer = M.Timer((args.steps + every - 1) // every, M.TIME_UP_KERNEL)
        t0 = time.perf_counter()
        for i in range(args.steps):
            if i % every == 0:
                M.moe_layer_forward_timed(cfg, L.x, gate, L.bias, L.packed, L.y, L.ws, up_timer)
            else:
                step()
        torch.cuda.synchronize()
        ms_per_step = (time.perf_counter() - t0) * 1e3 / args.steps
        up_samples = up_timer.read()
        up_timer.close()
        up_ms = float(np.mean(up_samples))
        # per-stage breakdown from extra steps outside the timed region (events between all stages cost
        # a few microseconds of idle time each, which the timed steps do not pay)
        n_extra = min(args.steps, 10)
        stage_timer = M.Timer(n_extra, M.TIME_STAGES)
        for _ in range(n_extra):
            M.moe_layer_forward_timed(cfg, L.x, gate, L.bias, L.packed, L.y, L.ws, stage_timer)
        torch.cuda.synchronize()
        per_call = stage_timer.read()
        stage_timer.close()
        # what the run did, read back through the staged calls
        lay_counts = torch.empty(wl.E, dtype=torch.int32, device="cuda")
        idx = torch.empty((wl.T, wl.k), dtype=torch.int32, device="cuda")
        w = torch.empty((wl.T, wl.k), dtype=torch.float32, device="cuda")
        offsets = torch.empty(wl.E + 1, dtype=torch.int32, device="cuda")
        perm = torch.empty(wl.A, dtype=torch.int32, device="cuda")
        inv = torch.empty(wl.A, dtype=torch.int32, device="cuda")
        M.moe_route(cfg, L.x, gate, L.bias, idx, w, L.ws)
        M.moe_permute(cfg, L.x, idx, lay_counts, offsets, perm, inv, None, L.ws)
        torch.cuda.synchronize()
        counts = lay_counts.cpu().numpy()
    live = int((counts > 0).sum())
    out["value"] = wl.T / (ms_per_step * 1e-3)
    out["ms_per_step"] = ms_per_step
    out["config"] = {"workload": wl.name, "T": wl.T, "d_model": d, "d_ff": f, "experts": wl.E, "top_k": wl.k,
                     "mode": f"host-streamed experts (K={args.slots} slots, {args.order} order"
                             f"{', experts kept between steps' if args.keep_experts else ''})" if wl.streamed
                             else "experts resident in HBM",
                     "gate": "packed once (moe_pack_gate)",
                     "non_empty_experts": live, "max_tokens_per_expert": int(counts.max()),
                     "min_tokens_per_expert": int(counts.min())}
    ffn_flops = 6.0 * d * f * A
    if not wl.streamed:
        stage_ms = {s: float(np.mean([c[s] for c in per_call])) for s in M.STAGES}
        # Algorithmic bytes: W_gate+W_in of every non-empty expert once and Xp once for the up kernel, W_out once
        # and Yp once for the down kernel.  H[A,f] goes through HBM between the two (written by up, read by
        # down): traffic of this implementation, reported separately and not counted as algorithmic.
        up_bytes = live * 2 * d * f * es + A * d * es
        down_bytes = live * d * f * es + A * d * es
        up_gbs = up_bytes / (up_ms * 1e-3) / 1e9
        up_tflops = 4.0 * d * f * A / (up_ms * 1e-3) / 1e12
        # the up kernel is bound by whichever roofline gives the longer time for this workload
        t_hbm = up_bytes / (HBM_PEAK_GBS * 1e9)
        t_mfma = 4.0 * d * f * A / (MFMA_BF16_PEAK_TFLOPS * 1e12)
        traffic = measured_traffic(args.workload, "up") if args.tokens is None else None
        if t_hbm >= t_mfma:
            roof = {"bound": "hbm", "achieved": up_gbs, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                    "frac": up_gbs / HBM_PEAK_GBS, "traffic": traffic}
        else:
            roof = {"bound": "mfma", "achieved": up_tflops, "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s",
                    "frac": up_tflops / MFMA_BF16_PEAK_TFLOPS, "traffic": traffic}
        roof.update({"kernel": "ffn_mfma_kernel<true> (expert up-projection, gate/in fused)",
                     "avg_launch_ms": up_ms, "timed_launches": f"{len(up_samples)} of the {args.steps} timed steps (every {every}th)",
                     "algorithmic_bytes_per_launch": up_bytes,
                     "algorithmic_flops_per_launch": 4.0 * d * f * A, "h_staging_bytes_per_launch": A * f * es})
        out["roofline"] = roof
        ffn_ms = stage_ms["ffn_up"] + stage_ms["ffn_down"]
        out["stages_ms"] = stage_ms          # ffn_up here includes the work-list kernel that precedes the up kernel
        out["stages_note"] = f"stage times from {n_extra} extra steps after the timed region"
        out["ffn"] = {"tflops": ffn_flops / (ffn_ms * 1e-3) / 1e12,
                      "mfma_frac": ffn_flops / (ffn_ms * 1e-3) / 1e12 / MFMA_BF16_PEAK_TFLOPS,
                      "weight_gbs": live * 3 * d * f * es / (ffn_ms * 1e-3) / 1e9,
                      "down_gbs": down_bytes / (stage_ms["ffn_down"] * 1e-3) / 1e9}
        if not args.no_graph:
            # the same step recorded once into a HIP graph (kernel launches only) and replayed
            g = torch.cuda.CUDAGraph()
            with torch.cuda.graph(g):
                step()
            torch.cuda.synchronize()
            for _ in range(min(args.warmup, 10)):
                g.replay()
            torch.cuda.synchronize()
            t1 = time.perf_counter()
            for _ in range(args.steps):
                g.replay()
            torch.cuda.synchronize()
            g_ms = (time.perf_counter() - t1) * 1e3 / args.steps
            out["graph"] = {"ms_per_step": g_ms, "tokens_per_s": wl.T / (g_ms * 1e-3), "steps": args.steps,
                            "note": "the same layer call captured once in a HIP graph and replayed; value/ms_per_step above "
                                    "are the eager launches"}
            del g
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(wl, counts)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
