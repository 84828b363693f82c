"""Benchmark of the MoHGE layer on one MI355X.

A step is one pass of the whole hot path (route -> permute -> expert FFN up/down -> combine;
with --backward also the auxiliary losses and the backward pass) over one batch of seeded
synthetic input already resident in HBM.  Prints ONE JSON line: whole-layer tokens/s of the
headline workload (the largest single-GPU configuration, `large_prefill_skewed`), the roofline
of its dominant kernel (live HIP-event timing), the CPU oracle timed on this machine's host cores on
a bounded sample, and `all_configs`: the same measurements for the other named configurations.
"""
from __future__ import annotations

import argparse
import hashlib
import json
import os
import re
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_MFMA_BF16 = 2.5e15     # FLOP/s, dense bf16, MI355X
PEAK_VALU_F32 = 157.3e12    # FLOP/s, fp32 vector ALU (256 CUs x 4 SIMDs x 64 lanes x 2 FLOP at 2.4 GHz)
PEAK_HBM = 8.0e12           # B/s
HEADLINE = "large_prefill_skewed"
# (workload, backward) pairs reported under all_configs next to the headline
OTHERS = (("tiny_f32", False), ("mid_prefill", False), ("decode", False), ("training", False),
          ("training", True), ("paper_14b", False))

KERNEL_SOURCES = ("ffn_tiled.hip", "tiled.h", "ffn_skinny.hip", "skinny.h", "ffn.hip", "common.h")


def kernel_source_hash() -> str:
    """Hash of the sources of the expert-network kernels: a traffic figure measured with
    rocprofv3 counters is only quoted while the kernels it was measured on are unchanged."""
    h = hashlib.sha256()
    for name in KERNEL_SOURCES:
        with open(os.path.join(ROOT, "paper_2604_23108_amd", "csrc", name), "rb") as f:
            h.update(f.read())
    return h.hexdigest()[:16]


def measured_traffic(tag: str):
    """HBM bytes per launch of the dominant kernel of workload `tag`, from the rocprofv3 counter
    summary under profiles/ (FETCH_SIZE and WRITE_SIZE, each scaled by what the same counter reads
    for a plain device copy of known size): (bytes, file) if that summary was made with the
    present kernel sources, else (None, reason)."""
    path = os.path.join(ROOT, "profiles", f"{tag.replace('/', '_')}_rocprofv3.md")
    if not os.path.exists(path):
        return None, "no counter summary under profiles/ for this workload"
    text = open(path).read()
    m_hash = re.search(r"^kernel_source_hash: (\w+)", text, re.M)
    m_traffic = re.search(r"^traffic_bytes_per_launch: ([0-9.e+]+)", text, re.M)
    if not m_hash or not m_traffic:
        return None, f"{os.path.relpath(path, ROOT)} carries no traffic line"
    if m_hash.group(1) != kernel_source_hash():
        return None, f"{os.path.relpath(path, ROOT)} was measured on other kernel sources"
    return float(m_traffic.group(1)), os.path.relpath(path, ROOT)


def event_time(fn, iters, torch):
    """Average milliseconds per call of fn(), HIP events on the stream the kernels use."""
    start, stop = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    for _ in range(3):          # untimed: the first launches of a call in a process run slower
        fn()
    start.record()
    for _ in range(iters):
        fn()
    stop.record()
    stop.synchronize()
    return start.elapsed_time(stop) / iters


def event_time_inner(before, fn, iters, torch):
    """Average milliseconds of fn() alone when every fn() needs a before() first: one pair of
    HIP events around each fn(), on the stream the kernels use."""
    for _ in range(3):
        before()
        fn()
    pairs = []
    for _ in range(iters):
        before()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        fn()
        e1.record()
        pairs.append((e0, e1))
    torch.cuda.synchronize()
    return sum(a.elapsed_time(b) for a, b in pairs) / iters


def probe_timed(fn, torch):
    for _ in range(3):
        work = fn()
    a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    a.record()
    for _ in range(10):
        fn()
    b.record()
    b.synchronize()
    return work / (a.elapsed_time(b) / 10 * 1e-3)


def box_probe(torch, BB):
    """Ceilings of this box: TB/s of kernels that only read (1.25 GiB, every byte once), TFLOP/s of a
    kernel that only issues bf16 MFMAs; HIP events around 10 launches each."""
    buf = torch.ones(1280 << 20, dtype=torch.uint8, device="cuda")
    out = torch.zeros(1 << 20, dtype=torch.uint8, device="cuda")
    res = {}
    timed = lambda fn: probe_timed(fn, torch) / 1e12
    res["read_contiguous_TBs"] = round(timed(lambda: BB.mohge_probe_read(buf, 0, False, out)), 3)
    for row in (2048, 4096, 8192):
        for stag in (False, True):
            key = "read_rows_%d%s_TBs" % (row, "_staggered" if stag else "")
            res[key] = round(timed(lambda: BB.mohge_probe_read(buf, row, stag, out)), 3)
    # one round of workgroups of the decode up projection's size (about 940 active workgroups)
    small = buf[: 940 * 128 * 8192]
    res["read_rows_8192_940_workgroups_TBs"] = round(timed(lambda: BB.mohge_probe_read(small, 8192, False, out)), 3)
    tf = timed(lambda: BB.mohge_probe_mfma(out, 20000))
    res["mfma_bf16_only_TFLOPs"] = round(tf, 1)
    res["mfma_clock_implied_GHz"] = round(tf * 1e12 / (256 * 4 * 1024.0) / 1e9, 3)   # 1024 FLOP per clock and SIMD
    return res


def cpu_baseline(w, inp, budget_s=12.0):
    """The oracle as it stands on a bounded sample: the first n tokens of the workload
    through route -> permute -> experts -> combine, n sized to about `budget_s` seconds."""
    import oracle
    from synth import LayerInputs, Tensor

    def run(n):
        sw = w.replace(T=n)
        sub = LayerInputs(sw, Tensor(inp.x.f32[:n]), inp.w_group, inp.w_expert, inp.w_gate, inp.w_up,
                          inp.w_down, inp.expert_logit_bias)
        t0 = time.perf_counter()
        oracle.layer(sw, sub)
        return time.perf_counter() - t0

    n = min(w.T, 16)
    t = run(n)              # (also widens the bf16 weights to the float32 the oracle reads, once)
    t = run(n)
    per_tok = t / n
    n2 = int(max(n, min(w.T, budget_s / max(per_tok, 1e-9))))
    if n2 > n:
        t = run(n2)
        n = n2
    return {"value": n / t, "unit": "tokens/s", "cores": oracle.num_threads(), "kind": "oracle",
            "sample": f"first {n} of {w.T} tokens of {w.name} through the whole layer (fp64 C oracle, OpenMP), {t:.1f} s"}


def tile_phases(torch, BB, cfg, L, x):
    """Where the clocks of the fused expert launch go (counters of the benchmark library)."""
    import numpy as np
    cyc = BB.cycles_buffer()
    opts = BB.FfnOptions(cycles=cyc)
    BB.mohge_bench_expert_ffn(cfg, x, L.perm, L.offsets, L.w13, L.w2, L.y_perm, L.ws_ffn, opts)
    torch.cuda.synchronize()
    c = cyc.cpu().numpy().astype(np.float64)
    d, q = c[0], c[1]
    busy = d[:, :4].sum(1)
    ticks = q[:, 1] + q[:, 3]
    clk = (q[:, 0] + q[:, 2]).sum() / max(ticks.sum(), 1) / 10.0
    return {
        "core_clock_GHz": round(float(clk), 3),
        "share_setup_wait_mainloop_epilogue": [round(float(v), 4) for v in d[:, :4].sum(0) / busy.sum()],
        "clocks_per_stage": round(float(d[:, 2].sum() / max(d[:, 5].sum(), 1)), 1),
        "busy_clocks_per_workgroup_min_mean_max": [int(busy.min()), int(busy.mean()), int(busy.max())],
        "alive_us_min_mean_max": [round(float(v), 1) for v in ((q[:, 5] - q[:, 4]).min() / 100, (q[:, 5] - q[:, 4]).mean() / 100, (q[:, 5] - q[:, 4]).max() / 100)],
        "clocks_waiting_for_row_blocks_mean_max": [int(d[:, 6].mean()), int(d[:, 6].max())],
        "tiles_that_waited": int(d[:, 7].sum()), "tiles": int(d[:, 4].sum()),
    }


def decode_timeline(torch, BB, M, L, x):
    """When the pieces of the single-launch decode layer ran (time stamps of the benchmark library)."""
    import numpy as np
    cfg = L.cfg
    tr = BB.decode_trace_buffer(cfg)
    for _ in range(3):
        tr.zero_()
        BB.mohge_bench_decode_layer(cfg, x, L.w_group, L.w_expert, L.bias, L.w13, L.w2, L.group_idx, L.expert_idx,
                                    L.gates, L.y, L.ws_decode, 0, tr)
        torch.cuda.synchronize()
    t = tr.cpu().numpy().astype(np.float64) / 100.0                      # microseconds
    counts = np.bincount(L.expert_idx.cpu().numpy().reshape(-1), minlength=cfg.n_experts)
    F_e = np.repeat(np.asarray(cfg.d_ff), cfg.experts_per_group)
    n_route = ((cfg.T + 15) // 16) * ((cfg.n_groups + cfg.n_experts + 15) // 16) * ((cfg.d + 255) // 256)
    nA = n_route + (cfg.T + 3) // 4
    U = int(((counts > 0) * (F_e // 64)).sum())
    D = int((counts > 0).sum()) * ((cfg.d + 127) // 128)
    t0 = t[:nA + U + D, 0].min()
    s, a, e = t[:, 0] - t0, t[:, 1] - t0, t[:, 3] - t0
    up, dn = slice(nA, nA + U), slice(nA + U, nA + U + D)
    r = lambda v: round(float(v), 1)
    return {"unit": "us after the first piece started", "route_tasks": n_route, "up_units": U, "down_units": D,
            "route_done": r(e[:n_route].max()), "routing_published": r(e[n_route:nA].max()),
            "first_up_unit_streams": r(s[up].min()), "up_unit_us_median_max": [r(np.median((e - s)[up])), r((e - s)[up].max())],
            "last_up_unit_done": r(e[up].max()), "first_expert_complete": r(a[dn].min()),
            "down_units_waited_us_median_max": [r(np.median((a - s)[dn])), r((a - s)[dn].max())],
            "last_down_unit_done": r(e[dn].max())}


def measure(args, name, backward, torch, M, BB, steps, warmup, full):
    """One workload: K steps between events, per-call times, roofline of the dominant kernel."""
    import numpy as np
    from paper_2604_23108_amd.device_layer import DeviceLayer, to_dev
    from synth import WORKLOADS, generate

    w = WORKLOADS[name]
    inp = generate(w)
    dl = DeviceLayer(w, inp, training=backward, backward=backward)
    L, cfg, x = dl.layer, dl.cfg, dl.x
    dy = None
    if backward:
        if inp.dy is None:
            sys.exit("bench.py: --backward needs a workload that draws dy (e.g. --workload training)")
        dy = to_dev(inp.dy, True)
    quant = full and (args.fp8_weights or args.mxfp4_weights)
    if quant:
        if w.T > 32 or backward or (args.fp8_weights and args.mxfp4_weights):
            sys.exit("bench.py: --fp8-weights / --mxfp4-weights (one of them) are for decode workloads (T <= 32), forward only")
        L.use_fp8_weights() if args.fp8_weights else L.use_mxfp4_weights()

    weight_sets = None
    flip = [0]
    if full and args.alternate_weights:
        if w.T > 32:
            sys.exit("bench.py: --alternate-weights is for decode workloads (T <= 32)")
        clone = lambda ts: None if ts is None else tuple([t.clone() for t in part] for part in ts)
        weight_sets = [(L.w13, L.w2, L.w8, L.w4),
                       ([t.clone() for t in L.w13], [t.clone() for t in L.w2], clone(L.w8), clone(L.w4))]

    def flipw():
        if weight_sets:
            flip[0] ^= 1
            L.w13, L.w2, L.w8, L.w4 = weight_sets[flip[0]]
        return True

    single = full and args.single_launch
    if single and (w.T > 32 or backward or quant or w.dtype != "bf16"):
        sys.exit("bench.py: --single-launch is the bf16 decode layer as one launch (T <= 32, forward only)")

    def step():
        flipw()
        if single:
            L.forward_decode(x)
        else:
            L.forward(x)
        if backward:
            L.backward(x, dy)

    if full and args.graph:
        # the timed step is one replay of a HIP graph that holds exactly the launches of step()
        L.capture(x, dy)
        step = L.replay
    for _ in range(warmup):
        step()
    torch.cuda.synchronize()
    # exactly K steps between a synchronisation on either side: the wall clock, and a pair of
    # HIP events around the same K steps on the launch stream
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    e0.record()
    for _ in range(steps):
        step()
    e1.record()
    torch.cuda.synchronize()
    ms_wall = (time.perf_counter() - t0) * 1e3 / steps
    ms_events = e0.elapsed_time(e1) / steps
    # a fused launch whose tiles gave up waiting would have written NaN: say so rather than time it
    for call, ws in ((M.CALL_FFN_SAVED, getattr(L, "saved", None)) if backward else (M.CALL_EXPERT_FFN, L.ws_ffn),
                     (M.CALL_EXPERT_FFN_BWD, getattr(L, "ws_ffn_bwd", None)) if backward else (None, None)):
        if call is not None and M.mohge_fused_status(cfg, call, ws) != 0:
            sys.exit(f"bench.py: {name}: {M.mohge_last_error()}")
    # the same steps once more, each between its own pair of HIP events: median and minimum
    pairs = []
    for _ in range(steps):
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        step()
        b.record()
        pairs.append((a, b))
    torch.cuda.synchronize()
    step_ms = sorted(a.elapsed_time(b) for a, b in pairs)

    # per-call timing with HIP events (state from the last step is valid input for each call)
    it = max(10, steps)
    calls = {
        "route": lambda: M.mohge_route(cfg, x, L.w_group, L.w_expert, L.bias, L.group_idx, L.expert_idx, L.gates, L.gs, L.es1, L.ws_route),
        "permute": lambda: M.mohge_permute(cfg, L.expert_idx, L.counts, L.offsets, L.perm, L.inv_perm, None, None, L.ws_permute),
        "ffn": (lambda: flipw() and M.mohge_expert_ffn_w8(cfg, x, L.perm, L.offsets, *L.w8, L.y_perm, L.ws_ffn)) if quant and args.fp8_weights
               else (lambda: flipw() and M.mohge_expert_ffn_w4(cfg, x, L.perm, L.offsets, *L.w4, L.y_perm, L.ws_ffn)) if quant
               else (lambda: flipw() and M.mohge_expert_ffn(cfg, x, L.perm, L.offsets, L.w13, L.w2, L.y_perm, L.ws_ffn)),
        "ffn_up": lambda: flipw() and M.mohge_expert_ffn_up(cfg, x, L.perm, L.offsets, L.w13, L.ws_ffn),
        "ffn_down": lambda: flipw() and M.mohge_expert_ffn_down(cfg, L.ws_ffn, L.offsets, L.w2, L.y_perm),
        "combine": lambda: M.mohge_combine(cfg, L.y_perm, L.inv_perm, L.gates, L.y),
    }
    if backward:
        calls.update({
            "ffn_train_fwd": lambda: M.mohge_expert_ffn_train(cfg, x, L.perm, L.offsets, L.w13, L.w2, L.y_perm, L.saved),
            "aux_loss": lambda: M.mohge_aux_loss(cfg, L.gs, L.es1, L.group_idx, L.expert_idx, L.losses, L.stats, L.ws_aux),
            "combine_bwd": lambda: M.mohge_combine_bwd(cfg, dy, L.y_perm, L.inv_perm, L.gates, L.dgates, L.dy_perm),
            "ffn_bwd": lambda: M.mohge_expert_ffn_bwd(cfg, x, L.perm, L.offsets, L.w13, L.w2, L.saved, L.dy_perm,
                                                      L.dx_perm, L.dw13, L.dw2, L.ws_ffn_bwd),
            "route_bwd": lambda: M.mohge_route_bwd(cfg, x, L.w_group, L.w_expert, L.gs, L.es1, L.group_idx,
                                                   L.expert_idx, L.gates, L.dgates, L.stats, L.dx_perm, L.inv_perm,
                                                   L.dx, L.dw_group, L.dw_expert, L.dz, L.ws_route_bwd),
        })
    if w.T <= 32 and w.dtype == "bf16" and not quant and not backward:
        # the same layer as one launch (mohge_decode_layer)
        calls["decode_layer"] = lambda: flipw() and L.forward_decode(x) is not None
    if not full:
        keep = ("ffn", "route", "combine", "permute", "decode_layer") + (("ffn_up",) if w.T <= 32 else ()) + (("ffn_train_fwd", "ffn_bwd") if backward else ())
        calls = {k: v for k, v in calls.items() if k in keep}
    call_ms = {k: event_time(f, it, torch) for k, f in calls.items()}
    fused_alone = w.T > 32 and w.dtype == "bf16" and not backward
    if fused_alone:
        # the product launch of mohge_expert_ffn by itself; its tile schedule (a separate small
        # launch) is rebuilt before every timed launch, outside the event pair
        ffn_part = lambda p: BB.mohge_bench_expert_ffn(cfg, x, L.perm, L.offsets, L.w13, L.w2, L.y_perm, L.ws_ffn, None, p)
        call_ms["ffn_tiles"] = event_time_inner(lambda: ffn_part(1), lambda: ffn_part(2), it, torch)

    if "decode_layer" in call_ms:
        if M.mohge_fused_status(cfg, M.CALL_DECODE_LAYER, L.ws_decode) != 0:
            sys.exit(f"bench.py: {name}: {M.mohge_last_error()}")
        L.forward(x)                       # (the per-call state below is that of the separate calls)
    if full and args.copy_calibration:
        src = torch.empty(256 << 20, dtype=torch.uint8, device="cuda")
        for _ in range(3):
            dst = src.clone()
        torch.cuda.synchronize()
        del src, dst

    counts = L.counts.cpu().numpy().astype(np.int64)
    F_e = np.repeat(np.asarray(w.d_ff, np.int64), w.experts_per_group)
    elt = 2 if w.dtype == "bf16" else 4
    flops_up = float((counts * 4 * w.d * F_e).sum())
    flops_down = float((counts * 2 * w.d * F_e).sum())
    touched = counts > 0
    bytes_up = float((touched * 2 * w.d * F_e * elt).sum() + w.T * w.d * elt + (counts * F_e * elt).sum())
    bytes_down = float((touched * w.d * F_e * elt).sum() + (counts * F_e * elt).sum() + w.n_pairs * w.d * elt)
    P = w.n_pairs
    bytes_route = float(w.T * w.d * elt + (w.n_experts + w.n_groups) * w.d * 4 + w.T * (w.k_groups * 4 + w.k_experts * 8))
    bytes_combine = float((P + w.T) * w.d * elt + P * 8)

    decode = w.T <= 32
    tag = name
    if decode and quant:
        # fp8: one byte per weight plus an fp32 scale per row; mxfp4: half a byte per weight plus
        # a scale byte per 32 weights; activations stay bf16
        if args.fp8_weights:
            wb_up, wb_down = 2 * w.d * F_e + 2 * F_e * 4, w.d * F_e + w.d * 4
        else:
            wb_up, wb_down = 2 * w.d * F_e * (0.5 + 1 / 32), w.d * F_e * (0.5 + 1 / 32)
        b8_up = float((touched * wb_up).sum() + w.T * w.d * elt + (counts * F_e * elt).sum())
        b8_down = float((touched * wb_down).sum() + (counts * F_e * elt).sum() + w.n_pairs * w.d * elt)
        ach = (b8_up + b8_down) / (call_ms["ffn"] * 1e-3)
        kname = "ffn_skinny_q_kernel<up, %d> + <down, %d>" % ((8, 8) if args.fp8_weights else (4, 4))
        tag = name + ("/fp8" if args.fp8_weights else "/mxfp4")
        roof = {"kernel": kname + " (one call of the quantised-weight entry point)", "bound": "hbm",
                "achieved": ach / 1e9, "peak": PEAK_HBM / 1e9, "unit": "GB/s", "frac": ach / PEAK_HBM}
    elif w.dtype != "bf16":
        # the fp32 path (correctness configuration): plain fused multiply-adds on the vector ALUs
        ach = (flops_up + flops_down) / (call_ms["ffn"] * 1e-3)
        roof = {"kernel": "ffn_f32_kernel<up> + <down> (one mohge_expert_ffn call)", "bound": "alu",
                "achieved": ach / 1e12, "peak": PEAK_VALU_F32 / 1e12, "unit": "TFLOP/s", "frac": ach / PEAK_VALU_F32}
    elif decode:
        ach = bytes_up / (call_ms["ffn_up"] * 1e-3)
        roof = {"kernel": "ffn_skinny_kernel<up> (one mohge_expert_ffn_up call)", "bound": "hbm",
                "achieved": ach / 1e9, "peak": PEAK_HBM / 1e9, "unit": "GB/s", "frac": ach / PEAK_HBM}
    else:
        # the step's expert networks are one launch (up and down tiles together) plus its schedule
        key = "ffn_train_fwd" if backward else "ffn_tiles" if fused_alone else "ffn"
        ach = (flops_up + flops_down) / (call_ms[key] * 1e-3)
        roof = {"kernel": "ffn_fused_kernel<up, down> (the product launch of mohge_expert_ffn, timed alone)" if fused_alone
                          else "ffn_fused_kernel + its schedule kernel (one %s call)" %
                          ("mohge_expert_ffn_train" if backward else "mohge_expert_ffn"),
                "bound": "mfma", "achieved": ach / 1e12, "peak": PEAK_MFMA_BF16 / 1e12, "unit": "TFLOP/s",
                "frac": ach / PEAK_MFMA_BF16}
        # The bound of a launch is the resource whose peak allows it the least: with few rows per expert
        # (the paper's layer shapes: every weight byte is used by one row block) moving the algorithmic
        # bytes at the HBM peak takes longer than the multiply-adds at the matrix-core peak.
        t_mfma, t_hbm = (flops_up + flops_down) / PEAK_MFMA_BF16, (bytes_up + bytes_down) / PEAK_HBM
        if t_hbm > t_mfma and not backward:
            ach_b = (bytes_up + bytes_down) / (call_ms[key] * 1e-3)
            roof.update({"bound": "hbm", "achieved": ach_b / 1e9, "peak": PEAK_HBM / 1e9, "unit": "GB/s",
                         "frac": ach_b / PEAK_HBM, "frac_of_mfma_peak": ach / PEAK_MFMA_BF16})
        roof["least_time_ms"] = {"mfma": round(t_mfma * 1e3, 5), "hbm": round(t_hbm * 1e3, 5)}
    roof["traffic"], roof["traffic_source"] = measured_traffic(tag + ("_backward" if backward else ""))
    parts = {
        "step_ms_median": round(step_ms[len(step_ms) // 2], 5), "step_ms_min": round(step_ms[0], 5),
        "call_ms": {k: round(v, 5) for k, v in call_ms.items()},
        "route_gbs": bytes_route / (call_ms["route"] * 1e-3) / 1e9,
        "route_tflops_f32": 2.0 * w.T * w.d * (w.n_experts + w.n_groups) / (call_ms["route"] * 1e-3) / 1e12,
        "combine_gbs": bytes_combine / (call_ms["combine"] * 1e-3) / 1e9,
        "count_min": int(counts.min()), "count_max": int(counts.max()),
    }
    if "ffn_up" in call_ms and "ffn_down" in call_ms:
        t_ffn = (call_ms["ffn_up"] + call_ms["ffn_down"]) * 1e-3
        parts.update({"ffn_up_down_tflops": (flops_up + flops_down) / t_ffn / 1e12,
                      "ffn_up_down_frac_mfma": (flops_up + flops_down) / t_ffn / PEAK_MFMA_BF16,
                      "ffn_up_down_gbs": (bytes_up + bytes_down) / t_ffn / 1e9,
                      "ffn_up_down_frac_hbm": (bytes_up + bytes_down) / t_ffn / PEAK_HBM})
    if backward:
        # the five backward products: dH and dW_down cost what the down projection costs,
        # dX and dW13 what the up projection costs
        flops_bwd = 2.0 * (flops_up + flops_down)
        parts["ffn_bwd_tflops"] = flops_bwd / (call_ms["ffn_bwd"] * 1e-3) / 1e12
        parts["ffn_bwd_frac_mfma"] = flops_bwd / (call_ms["ffn_bwd"] * 1e-3) / PEAK_MFMA_BF16
        parts["step"] = "forward (activations kept) + aux losses + backward"
    if full and args.tile_phases and fused_alone:
        parts["tile_phases"] = tile_phases(torch, BB, cfg, L, x)
    if full and args.decode_timeline and "decode_layer" in call_ms:
        parts["decode_layer_timeline"] = decode_timeline(torch, BB, M, L, x)
    res = dict(w=w, inp=inp, ms_events=ms_events, ms_wall=ms_wall, roof=roof, parts=parts, quant=quant)
    del dl, L
    return res


def placement_report(args, torch, M):
    """The paper's per-GPU load table (section 3.4.1, load-balance experiment) for R virtual GPUs:
    the GPU router's expert choices for a workload replayed through the allocation rule."""
    import numpy as np
    from paper_2604_23108_amd import placement
    from paper_2604_23108_amd.device_layer import DeviceLayer
    from synth import WORKLOADS, generate
    R = args.placement_report
    w = WORKLOADS[args.workload or "paper_14b"]
    dl = DeviceLayer(w, generate(w), training=False)
    dl.layer.forward(dl.x)
    torch.cuda.synchronize()
    eidx = dl.layer.expert_idx.cpu().numpy()
    out = {"placement_report": {"workload": w.name, "virtual_gpus": R, "ideal_share": 1.0 / R}}
    for mode in ("contiguous", "strided"):
        rep = placement.load_report(eidx, w.n_groups, w.experts_per_group, R, w.d_ff, mode)
        print(placement.format_report(rep, f"{w.name}: share of every group's routed pairs per virtual GPU "
                                           f"({mode} all-size sets, {R} GPUs, ideal {100.0 / R:.2f} %)"), file=sys.stderr)
        out["placement_report"][mode] = {
            "share_by_group_percent": np.round(100 * rep["share_by_group"], 2).tolist(),
            "flop_share_percent": np.round(100 * rep["flop_share"], 2).tolist(),
            "max_abs_deviation_percent": round(float(100 * np.abs(rep["share_by_group"] - 1.0 / R).max()), 3)}
    print(json.dumps(out))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--workload", default=None, help=f"default: {HEADLINE}, with the other named configurations "
                    "under all_configs; naming a workload measures that one alone")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-all-configs", action="store_true", help="the headline workload only")
    ap.add_argument("--backward", action="store_true",
                    help="training step: forward (keeping activations, with the auxiliary losses) + backward")
    ap.add_argument("--graph", action="store_true",
                    help="replay the step as one HIP graph instead of plain launches (measured: no faster, "
                         "the step is not bound by host launch overhead)")
    ap.add_argument("--fp8-weights", action="store_true",
                    help="decode workloads: stream per-row quantised FP8 E4M3 expert weights (mohge_expert_ffn_w8)")
    ap.add_argument("--mxfp4-weights", action="store_true",
                    help="decode workloads: stream MXFP4 expert weights (mohge_expert_ffn_w4)")
    ap.add_argument("--alternate-weights", action="store_true",
                    help="decode workloads: keep two copies of the expert weights and alternate between them "
                         "step by step, so that nothing of a step's weights can be left in the last-level cache")
    ap.add_argument("--box-probe", action="store_true",
                    help="instead of the layer: measure what the box delivers (pure reads in several access "
                         "patterns, back-to-back bf16 MFMAs) and print one JSON line")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run a plain 256 MiB device copy (for scaling rocprofv3 FETCH_SIZE / WRITE_SIZE)")
    ap.add_argument("--single-launch", action="store_true",
                    help="decode workloads: the step is ONE launch (mohge_decode_layer) instead of the four calls")
    ap.add_argument("--decode-timeline", action="store_true",
                    help="decode workloads: add when the pieces of the single-launch layer ran (benchmark library's time stamps)")
    ap.add_argument("--tile-phases", action="store_true",
                    help="prefill workloads: add the clock breakdown of the fused expert launch (setup, wait, main "
                         "loop, epilogue, core clock, idle tail) from the benchmark library's counters")
    ap.add_argument("--placement-report", type=int, default=0, metavar="R",
                    help="instead of timing: route the workload (default paper_14b) on the GPU and print the share "
                         "of every group's routed pairs that each of R virtual GPUs would receive under the "
                         "All-size Group-decoupling Allocation")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on one GPU only (no collectives, no sharding); use --gpus 1")

    import torch
    import paper_2604_23108_amd as M
    from paper_2604_23108_amd import bench_binding as BB

    if args.box_probe:
        print(json.dumps({"box_probe": box_probe(torch, BB)}))
        return
    if args.placement_report:
        placement_report(args, torch, M)
        return
    name = args.workload or HEADLINE
    r = measure(args, name, args.backward, torch, M, BB, args.steps, args.warmup, True)
    w, roof, parts = r["w"], r["roof"], r["parts"]
    # the same kind of work with nothing else going on, measured now on this machine (see box_probe)
    if w.dtype == "bf16":
        out = torch.zeros(1 << 20, dtype=torch.uint8, device="cuda")
        if roof["bound"] == "mfma":
            ceil = probe_timed(lambda: BB.mohge_probe_mfma(out, 20000), torch) / 1e12
            what = "a kernel of nothing but bf16 MFMAs on operands with full mantissas (clock under that load)"
        else:
            buf = torch.ones(1 << 30, dtype=torch.uint8, device="cuda")
            ceil = probe_timed(lambda: BB.mohge_probe_read(buf, 0, False, out), torch) / 1e9
            what = "a kernel that only reads 1 GiB in contiguous streams"
            del buf
        roof["measured_ceiling"] = {"value": ceil, "unit": roof["unit"], "what": what}
        roof["frac_of_measured_ceiling"] = roof["achieved"] / ceil
    res = {
        "metric": "MoHGE layer tokens/sec + expert-FFN % bf16 MFMA peak (decode: % HBM BW)",
        "value": w.T / (r["ms_events"] * 1e-3), "unit": "tokens/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": r["ms_events"], "ms_per_step_wall": r["ms_wall"],
        "timing": "ms_per_step: HIP events around the K steps on the launch stream; ms_per_step_wall: host clock "
                  "around the same K steps between two synchronisations",
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": ("bf16 (expert weights fp8 e4m3)" if args.fp8_weights else "bf16 (expert weights mxfp4)" if args.mxfp4_weights else "bf16") if w.dtype == "bf16" else "f32",
        "data": "synthetic", "launch": "hip graph replay of the step" if args.graph else
                                       "eager, the layer as one launch (mohge_decode_layer)" if args.single_launch else "eager",
        "config": {"workload": w.name, "T": w.T, "d": w.d, "groups_x_experts": f"{w.n_groups}x{w.experts_per_group}",
                   "d_ff": list(w.d_ff), "k_groups": w.k_groups, "k_experts": w.k_experts,
                   "select_mode": "per_group" if w.select_mode == 1 else "global", "seed": w.seed,
                   **({"backward": True} if args.backward else {}),
                   **({"alternate_weights": True} if args.alternate_weights else {})},
        "roofline": roof,
        "parts": parts,
    }
    if not args.no_cpu_baseline:
        res["cpu_baseline"] = cpu_baseline(w, r["inp"])
    del r
    if args.workload is None and not args.no_all_configs:
        allc = {}
        for oname, bwd in OTHERS:
            torch.cuda.empty_cache()
            o = measure(args, oname, bwd, torch, M, BB, max(10, args.steps // 2), max(3, args.warmup // 2), False)
            ow = o["w"]
            allc[oname + ("_backward" if bwd else "")] = {
                "T": ow.T, "dtype": "bf16" if ow.dtype == "bf16" else "f32",
                "ms_per_step": round(o["ms_events"], 5), "tokens_per_s": ow.T / (o["ms_events"] * 1e-3),
                "roofline": {k: o["roof"][k] for k in ("kernel", "bound", "achieved", "peak", "unit", "frac", "traffic", "traffic_source")},
                "call_ms": o["parts"]["call_ms"],
                **({"ffn_bwd_frac_mfma": o["parts"]["ffn_bwd_frac_mfma"]} if bwd else {})}
            del o
        res["all_configs"] = allc
    print(json.dumps(res))


if __name__ == "__main__":
    main()
