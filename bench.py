#!/usr/bin/env python3
"""Benchmark of the sliced causal attention hot path on one MI355X.

One "step" = one pass of the whole hot path over one synthetic microbatch: forward of every slice
in order against its cached K/V prefix, then backward of every slice in reverse order with dK/dV
accumulated in fp32 (the call order of the slice-wise schedule, paper Sec. 4.1.2).  Inputs are
resident in HBM before the timed region.  Prints ONE JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload llama70b_tp8_share] [--slices n] [--no-cpu-baseline]

The headline (`value`, `ms_per_step`) is timed with nothing but the library's kernels on the stream.  The per-kernel
breakdown behind `roofline` comes from a SECOND pass of the same steps in which every kernel is bracketed by HIP
events on the stream it runs on.  `cpu_baseline` times the fp64 oracle on a sample of the same seeded tensors, and
`parity` compares the library's result on that same sample with what the oracle returned there (outside any timing).
"""
import argparse
import json
import math
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0      # MI355X dense bf16 MFMA peak


def visible_pairs(s, q_offset, kv_begin, kv_end):
    """Visible (query row, key) pairs of one causal call, per query head."""
    total = 0
    full_rows_from = max(0, kv_end - 1 - q_offset)          # rows r >= this see the whole range
    full_rows_from = min(full_rows_from, s)
    # rows r < full_rows_from see keys kv_begin .. q_offset + r
    lo_r = max(0, kv_begin - q_offset)                      # first row that sees anything
    if lo_r < full_rows_from:
        n = full_rows_from - lo_r
        first = q_offset + lo_r + 1 - kv_begin
        total += n * first + n * (n - 1) // 2
    total += (s - full_rows_from) * max(0, kv_end - kv_begin)
    return total


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=3)
    ap.add_argument("--warmup", type=int, default=1)
    ap.add_argument("--workload", default="llama70b_tp8_share")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--slices", type=int, default=None,
                    help="cut the workload's sequence into this many slices instead of its own count (slice-length sweep)")
    ap.add_argument("--chunked", action="store_true",
                    help="K/V and the dK/dV accumulators as one allocation per slice (the paper's chunked cache) instead of one buffer")
    ap.add_argument("--no-fwd-ranges", action="store_true",
                    help="never cut a forward call into key ranges (for comparison on workloads with short slices)")
    ap.add_argument("--schedule-sim", default=None, metavar="P,M[,V]",
                    help="also time every slice's forward and backward call and feed the times to the slice-wise 1F1B "
                         "schedule simulator with P pipeline devices, M microbatches and V stages per device (default 1; "
                         "adds a 'schedule_sim' object)")
    ap.add_argument("--probe-dq-atomics", action="store_true",
                    help="instead of the benchmark: time the float32 atomic adds a fused (scores-once) backward would need "
                         "for dq, in that kernel's access pattern, alone and under a stream of matrix instructions")
    args = ap.parse_args()
    if args.probe_dq_atomics:
        return probe_dq_atomics()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (no collectives, no sharding); --gpus %d is not supported" % args.gpus,
              file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    import paper_2504_14519_amd as sp
    from synth_inputs import CONFIGS, normal_bf16

    cfg_id = [i for i, c in CONFIGS.items() if c["name"] == args.workload]
    if not cfg_id:
        sys.exit("unknown workload %s" % args.workload)
    cfg_id = cfg_id[0]
    c = CONFIGS[cfg_id]
    N, n, Hq, Hkv, D = c["N"], c["n"], c["Hq"], c["Hkv"], c["D"]
    if args.slices:
        if N % args.slices or (N // args.slices) % 256:
            sys.exit("--slices must cut the sequence into equal slices of a multiple of 256 rows")
        n = args.slices
    s = N // n
    first_slice = n - n // 8 if c["name"] == "longest" else 0     # the longest config runs its final eighth only
    scale = 1.0 / math.sqrt(D)
    dev = "cuda:0"

    def to_dev(bits):
        return torch.from_numpy(bits.view(np.int16)).view(torch.bfloat16).to(dev)

    q = to_dev(normal_bf16((1, N, Hq, D), cfg_id, "q")) if first_slice == 0 else None
    if q is None:   # only the slices that run need queries
        qn = normal_bf16((1, (n - first_slice) * s, Hq, D), cfg_id, "q")
        don = normal_bf16((1, (n - first_slice) * s, Hq, D), cfg_id, "do")
        q, do = to_dev(qn), to_dev(don)
    else:
        do = to_dev(normal_bf16((1, N, Hq, D), cfg_id, "do"))
    k = to_dev(normal_bf16((1, N, Hkv, D), cfg_id, "k"))
    v = to_dev(normal_bf16((1, N, Hkv, D), cfg_id, "v"))
    slices = list(range(first_slice, n))
    nrun = len(slices)
    outs = [torch.empty((1, s, Hq, D), device=dev, dtype=torch.bfloat16) for _ in slices]
    lses = [torch.empty((1, Hq, s), device=dev, dtype=torch.float32) for _ in slices]
    dq = torch.empty((1, nrun * s, Hq, D), device=dev, dtype=torch.bfloat16)
    dk_acc = torch.zeros((1, N, Hkv, D), device=dev, dtype=torch.float32)
    dv_acc = torch.zeros((1, N, Hkv, D), device=dev, dtype=torch.float32)
    dk_out = torch.empty((1, N, Hkv, D), device=dev, dtype=torch.bfloat16)
    dv_out = torch.empty((1, N, Hkv, D), device=dev, dtype=torch.bfloat16)
    # one workspace for every backward call of the step: the largest any slice asks for
    ws_bytes = max(sp.slimpipe_attn_workspace_bytes(sp.make_params(q[:, :s], k, outs[0], i * s, 0, (i + 1) * s, True, scale), True)
                   for i in slices)
    ws = torch.empty(ws_bytes, device=dev, dtype=torch.uint8)
    # forward: room for partial results when a slice's query blocks would not fill the GPU (0 for the 256K workload)
    fws_bytes = 0 if args.no_fwd_ranges else max(
        sp.slimpipe_attn_workspace_bytes(sp.make_params(q[:, :s], k, outs[0], i * s, 0, (i + 1) * s, True, scale), False) for i in slices)
    fws = torch.empty(fws_bytes, device=dev, dtype=torch.uint8) if fws_bytes else None

    def qs(j):
        return slice(j * s, (j + 1) * s)

    if args.chunked:
        # one allocation per slice, as the paper keeps its cache; the contiguous buffers are dropped
        kc = [k[:, i * s:(i + 1) * s].clone() for i in range(n)]
        vc = [v[:, i * s:(i + 1) * s].clone() for i in range(n)]
        dkc = [torch.zeros((1, s, Hkv, D), device=dev, dtype=torch.float32) for _ in range(n)]
        dvc = [torch.zeros((1, s, Hkv, D), device=dev, dtype=torch.float32) for _ in range(n)]
        dkoc = [dk_out[:, i * s:(i + 1) * s] for i in range(n)]
        dvoc = [dv_out[:, i * s:(i + 1) * s] for i in range(n)]
        del k, v, dk_acc, dv_acc

        def fwd_call(j):
            i = slices[j]
            sp.slimpipe_attn_fwd_chunked(q[:, qs(j)], kc, vc, i * s, 0, (i + 1) * s, True, scale, out=outs[j], lse=lses[j], workspace=fws)

        def bwd_call(j):
            i = slices[j]
            sp.slimpipe_attn_bwd_chunked(q[:, qs(j)], kc, vc, outs[j], do[:, qs(j)], lses[j], i * s, 0, (i + 1) * s, dkc, dvc,
                                         True, scale, dq=dq[:, qs(j)], dq_dtype=sp.BF16, dkv_accumulate=(j != nrun - 1),
                                         workspace=ws)

        def finalize():
            for i in range(n):
                sp.slimpipe_attn_finalize_bf16(dkc[i], dkoc[i])
                sp.slimpipe_attn_finalize_bf16(dvc[i], dvoc[i])
    else:
        def fwd_call(j):
            i = slices[j]
            sp.slimpipe_attn_fwd(q[:, qs(j)], k, v, i * s, 0, (i + 1) * s, True, scale, out=outs[j], lse=lses[j], workspace=fws)

        def bwd_call(j):
            i = slices[j]
            # the last slice to run backward first overwrites its dK/dV rows; earlier slices add to them
            sp.slimpipe_attn_bwd(q[:, qs(j)], k, v, outs[j], do[:, qs(j)], lses[j], i * s, 0, (i + 1) * s, dk_acc, dv_acc,
                                 True, scale, dq=dq[:, qs(j)], dq_dtype=sp.BF16, dkv_accumulate=(j != nrun - 1), workspace=ws)

        def finalize():
            sp.slimpipe_attn_finalize_bf16(dk_acc, dk_out)
            sp.slimpipe_attn_finalize_bf16(dv_acc, dv_out)

    def step(mark=None):
        """Forward of every slice in sequence order, backward in reverse order, dK/dV to bf16."""
        for j in range(nrun):
            fwd_call(j)
            if mark:
                mark("F", j)
        for j in reversed(range(nrun)):
            bwd_call(j)
            if mark:
                mark("B", j)
        finalize()

    pairs = [visible_pairs(s, i * s, 0, (i + 1) * s) for i in slices]
    pairs_total = sum(pairs)
    flops_step = 14.0 * D * Hq * pairs_total            # fwd 4D + bwd 10D per visible pair per q head
    flops_step_model = 12.0 * D * Hq * pairs_total

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    # pass 1, the headline: nothing on the stream but the library's kernels
    sp.slimpipe_attn_profile_enable(False)
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_per_step = (t1 - t0) * 1e3 / args.steps
    value = flops_step / (ms_per_step * 1e-3) / 1e12
    # pass 2, the breakdown: the same steps with every kernel bracketed by HIP events on its stream
    sp.slimpipe_attn_profile_enable(True)
    sp.slimpipe_attn_profile_read()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    ms_per_step_pass2 = (time.perf_counter() - t0) * 1e3 / args.steps
    prof = sp.slimpipe_attn_profile_read()
    sp.slimpipe_attn_profile_enable(False)

    # Flop per visible pair and q head, in units of D.  "issued": what each kernel computes (S = QK^T and dP = dO V^T are
    # computed by BOTH backward kernels).  "credited": the 10*D of the backward counted once, the duplicated 4*D split
    # evenly between dq and dk/dv, so that the credited figures add up to the 14*D of `value`.
    issued = {"fwd": 4.0, "dq": 6.0, "dkdv": 8.0}
    credited = {"fwd": 4.0, "dq": 4.0, "dkdv": 6.0}
    kshare = {kk: prof[kk][0] for kk in issued}
    dom = max(kshare, key=kshare.get)
    dom_ms, dom_n = prof[dom]
    per_d = D * Hq * pairs_total * args.steps

    def rate(flop_units, ms):
        return flop_units * per_d / (ms * 1e-3) / 1e12 if ms > 0 else 0.0

    achieved = rate(credited[dom], dom_ms)
    bwd_ms = sum(prof[kk][0] for kk in ("delta", "dq", "dq_reduce", "dkdv", "dkdv_reduce"))
    roofline = {
        "bound": "mfma", "kernel": dom, "achieved": round(achieved, 1), "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s",
        "frac": round(achieved / PEAK_BF16_TFLOPS, 4), "traffic": stored_traffic(c["name"], dom),
        "flop_accounting": "credited: %g*D per visible pair and q head for %s (S and dP, which both backward kernels "
                           "compute, counted once and split between them); the kernel issues %g*D" % (credited[dom], dom, issued[dom]),
        "achieved_issued": round(rate(issued[dom], dom_ms), 1), "frac_issued": round(rate(issued[dom], dom_ms) / PEAK_BF16_TFLOPS, 4),
        "launches": int(dom_n), "avg_launch_ms": round(dom_ms / max(1, dom_n), 4),
        "flops_per_launch_avg_credited": credited[dom] * per_d / max(1, dom_n),
        "kernel_ms_per_step": {kk: round(prof[kk][0] / args.steps, 3) for kk in prof},
        "kernel_tflops_issued": {kk: round(rate(issued[kk], prof[kk][0]), 1) for kk in issued if prof[kk][0] > 0},
        "kernel_tflops_credited": {kk: round(rate(credited[kk], prof[kk][0]), 1) for kk in issued if prof[kk][0] > 0},
        "backward_tflops_10D": round(rate(10.0, bwd_ms), 1),
        "ms_per_step_with_event_bracketing": round(ms_per_step_pass2, 3),
    }

    # the HBM-bound companions, against the 8 TB/s roof: algorithmic bytes over HIP-event time.  delta reads dO and out
    # (bf16) and writes one float per row and head; finalize reads the fp32 dK/dV accumulators and writes bf16
    aux_bytes = {"delta": nrun * s * Hq * (2 * D * 2 + 4.0), "finalize": 2 * N * Hkv * D * 6.0}
    roofline["hbm_bound_kernels_GBps"] = {kk: round(b * args.steps / (prof[kk][0] * 1e-3) / 1e9, 1)
                                          for kk, b in aux_bytes.items() if prof[kk][0] > 0}

    # what a pure stream of the same MFMA instruction sustains on this GPU (after the timed region): with
    # random operands the chip is power limited, which is the regime the attention kernels run in
    roofline["mfma_stream_tflops"] = {"constant_operands": round(sp.slimpipe_attn_mfma_rate(False), 1),
                                      "random_operands": round(sp.slimpipe_attn_mfma_rate(True), 1)}
    # the same matrix work on every compute unit, timed per XCD: workgroups are handed to the XCDs round-robin, so the
    # slowest XCD sets the time of a launch of equal workgroups (what the other XCDs idle at its end is lost)
    xr = sp.slimpipe_attn_xcd_rate()
    ends = [e for _, _, e in xr.values()]
    roofline["xcd_spread"] = {"mean_workgroup_ms_by_xcd": {str(x): round(m_, 3) for x, (_, m_, _) in xr.items()},
                              "last_end_ms_by_xcd": {str(x): round(e, 3) for x, (_, _, e) in xr.items()},
                              "slowest_over_mean": round(max(ends) / (sum(ends) / len(ends)), 4)}
    roofline["issued_frac_of_mfma_stream_random"] = round(roofline["achieved_issued"] / max(roofline["mfma_stream_tflops"]["random_operands"], 1e-9), 4)

    out = {
        "metric": "sliced causal attn fwd+bwd TFLOP/s and % of MI355X bf16 MFMA peak",
        "value": round(value, 2), "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 3), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": c["name"], "seq": N, "slices": n, "slice_len": s, "slices_run": [slices[0], slices[-1]],
                   "q_heads": Hq, "kv_heads": Hkv, "head_dim": D, "flop_convention": "14*D per visible pair per q head",
                   "kv_layout": "one chunk per slice" if args.chunked else "contiguous",
                   "fwd_key_ranges_workspace_bytes": fws_bytes},
        "pct_of_bf16_peak": round(100.0 * value / PEAK_BF16_TFLOPS, 2),
        "value_model_flops_12D": round(flops_step_model / (ms_per_step * 1e-3) / 1e12, 2),
        "roofline": roofline,
    }

    if args.schedule_sim:
        out["schedule_sim"] = schedule_sim(args.schedule_sim, n, nrun, slices, step, torch)
    if not args.no_cpu_baseline:
        out["cpu_baseline"], out["parity"] = cpu_baseline_and_parity(sp, torch, q, k if not args.chunked else torch.cat(kc, dim=1),
                                                                     v if not args.chunked else torch.cat(vc, dim=1), do, c, n, s,
                                                                     first_slice, scale)
    print(json.dumps(out), flush=True)


def probe_dq_atomics():
    """One JSON line per variant.  Shape: one backward call of the 256K workload's slice 15 (16384 rows, 8 q heads) over
    256 key tiles (one round of workgroups per head on a 256-CU chip would be 32; 256 x 8 = 2048 workgroups = 8 rounds).
    Needed rate: a fused backward at R TFLOP/s (10*D = 1280 flop per pair and head) makes R/1280 T pairs/s; with
    rows_per_step = 32 it adds 4 bytes of dq per pair, with 64 it adds 2."""
    import paper_2504_14519_amd as sp
    s_q, heads, key_tiles = 16384, 8, 256
    for rows in (32, 64):
        pairs = float(s_q) * 256 * key_tiles * heads
        bytes_total = pairs * (4.0 if rows == 32 else 2.0)
        for placement in (0, 1):
            for rotate in (0, 1):
                for filler, atomics in ((0, True), (40 * rows // 32, False), (40 * rows // 32, True)):
                    ms, ok, mism = sp.slimpipe_attn_dq_atomic_probe(s_q, heads, key_tiles, rows, placement, rotate, filler, atomics)
                    ms, ok, mism = sp.slimpipe_attn_dq_atomic_probe(s_q, heads, key_tiles, rows, placement, rotate, filler, atomics)
                    print(json.dumps({"probe": "dq_atomics", "rows_per_step": rows, "placement": placement, "rotate": rotate,
                                      "filler_mfma_per_step": filler, "atomics": atomics, "ms": round(ms, 3),
                                      "atomic_TBps": round(bytes_total / (ms * 1e-3) / 1e12, 3) if atomics else None,
                                      "equiv_fused_bwd_TFLOPs": round(pairs * 1280.0 / (ms * 1e-3) / 1e12, 1),
                                      "sum_ok": ok, "wg_not_on_xcd_w_mod_8": mism}), flush=True)


def schedule_sim(spec, n, nrun, slices, step, torch):
    """Per-slice attention times of this GPU (events on the stream the calls go to, after each slice's forward
    call and each slice's backward call, inside one more pass of the step) -> what the paper's schedule makes of
    them: bubble fraction without the context exchange and with it, accumulated activation (Sec. 4.1.3, 4.2)."""
    from paper_2504_14519_amd.schedule_sim import simulate_interleaved, simulate_lockstep, accumulated_fraction_interleaved
    parts = [int(x) for x in spec.split(",")]
    p_dev, m_mb, v_st = parts[0], parts[1], (parts[2] if len(parts) > 2 else 1)
    if nrun != n or slices[0] != 0:
        return {"error": "needs a workload that runs every slice"}
    marks = []

    def mark(kind, j):
        e = torch.cuda.Event(enable_timing=True)
        e.record()
        marks.append((kind, j, e))

    mark("start", -1)
    step(mark)
    torch.cuda.synchronize()
    t = {"F": [0.0] * n, "B": [0.0] * n}
    for (_, _, e0), (kind, j, e1) in zip(marks[:-1], marks[1:]):
        t[kind][j] = e0.elapsed_time(e1)
    res = {"p": p_dev, "m": m_mb, "n": n, "v": v_st, "fwd_ms_by_slice": [round(x, 3) for x in t["F"]],
           "bwd_ms_by_slice": [round(x, 3) for x in t["B"]],
           "accumulated_activation_fraction_of_Ma": round(accumulated_fraction_interleaved(p_dev, n, v_st, max(m_mb, 2 * p_dev)), 4),
           "warmup_cooldown_bound_(p-1)/(nvm)": round((p_dev - 1.0) / (n * v_st * m_mb), 5), "bubble_fraction": {}}
    for mode in (None, "pairwise", "balanced", "ideal"):
        r = simulate_interleaved(p_dev, n, m_mb, v_st, t["F"], t["B"], exchange=mode)
        res["bubble_fraction"][mode or "no_exchange"] = round(r["bubble_fraction"], 5)
    # the same with aligned columns of passes (each as long as its slowest pass): bubble of the last device, and the
    # part of it that the paper's closed forms count (the columns the device has no pass in)
    lock = {mode: simulate_lockstep(p_dev, n, m_mb, t["F"], t["B"], exchange=mode, v=v_st) for mode in (None, "pairwise", "balanced", "ideal")}
    res["lockstep_last_device_bubble_fraction"] = {(mode or "no_exchange"): round(r["bubble_fraction"][-1], 5) for mode, r in lock.items()}
    res["lockstep_last_device_absent_columns_fraction"] = round(lock["ideal"]["absent_fraction"][-1], 5)
    res["long_context_figure_(p-1)p/((n+1)nvm)"] = round((p_dev - 1.0) * p_dev / ((n + 1.0) * n * v_st * m_mb), 5)
    return res


def stored_traffic(workload, kernel):
    """HBM-side bytes per launch of `kernel` from the committed rocprofv3 counter summary (FETCH_SIZE and
    WRITE_SIZE runs scaled by a plain streaming kernel), or None if there is none for this workload."""
    path = os.path.join(ROOT, "profiles", "bench_%s_counters.txt" % workload)
    try:
        for line in open(path):
            f = line.split()
            if len(f) == 3 and f[0] == "traffic_bytes_per_launch" and f[1] == kernel:
                return float(f[2])
    except OSError:
        pass
    return None


def cpu_baseline_and_parity(sp, torch, q, k, v, do, c, n, s, first_slice, scale):
    """The fp64 oracle, as it stands, timed on the host cores on a bounded sample of the workload's own tensors: the
    first `rows` rows of one slice (all heads) as a call of their own against their whole prefix.  The same call then
    runs through the library (outside any timing) and the two results are compared: `parity`."""
    import numpy as np
    from oracle import attn_fwd, attn_bwd
    Hq, Hkv, D = c["Hq"], c["Hkv"], c["D"]
    i = min(first_slice + 2, n - 1)               # third slice that runs: cached slices + the diagonal block
    j = i - first_slice                            # its index among the query slices held on the device
    budget = 1.4e8 * 8 / Hq                        # (row, key) pairs per head: 10-20 s of host work on 16 cores
    rows = int(min(s, 4096, max(256, budget // (i * s + 2048) // 256 * 256)))
    kv_end = i * s + rows
    rs = slice(j * s, j * s + rows)

    def f64(t):
        return t.to(torch.float32).cpu().numpy().astype(np.float64)

    q64, do64, k64, v64 = f64(q[:, rs]), f64(do[:, rs]), f64(k[:, :kv_end]), f64(v[:, :kv_end])
    t0 = time.perf_counter()
    o_ref, l_ref = attn_fwd(q64, k64, v64, i * s, 0, kv_end, True, scale)
    dq_ref, dk_ref, dv_ref = attn_bwd(q64, k64, v64, o_ref, do64, l_ref, i * s, 0, kv_end, True, scale)
    dt = time.perf_counter() - t0
    pairs = visible_pairs(rows, i * s, 0, kv_end)
    tf = 14.0 * D * Hq * pairs / dt / 1e12
    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        cores = os.cpu_count()
    sample = ("fwd+bwd of the first %d rows of slice %d (all %d q heads, the workload's own tensors) against keys [0,%d), "
              "fp64 numpy; %.1f s" % (rows, i, Hq, kv_end, dt))
    base = {"value": round(tf, 5), "unit": "TFLOP/s", "cores": int(cores), "kind": "oracle", "sample": sample}

    # the library on the same call: forward, then backward from ITS OWN out / lse (the whole chain against the oracle's)
    kk, vv = k[:, :kv_end], v[:, :kv_end]
    out, lse = sp.slimpipe_attn_fwd(q[:, rs], kk, vv, i * s, 0, kv_end, True, scale)
    dk = torch.zeros((1, kv_end, Hkv, D), device=q.device, dtype=torch.float32)
    dv = torch.zeros_like(dk)
    dq = sp.slimpipe_attn_bwd(q[:, rs], kk, vv, out, do[:, rs], lse, i * s, 0, kv_end, dk, dv, True, scale, dq_dtype=sp.F32,
                              dkv_accumulate=False)
    torch.cuda.synchronize()

    def rel(x, ref):
        x = x.cpu().numpy().astype(np.float64)
        return float(np.linalg.norm(x - ref) / np.linalg.norm(ref))

    og, lg = f64(out), lse.cpu().numpy().astype(np.float64)
    finite = bool(np.isfinite(og).all() and np.isfinite(lg).all() and torch.isfinite(dq).all() and torch.isfinite(dk).all()
                  and torch.isfinite(dv).all())
    parity = {"sample": "the cpu_baseline sample: GPU forward -> GPU backward against oracle forward -> oracle backward",
              "out_max_abs": float(np.abs(og - o_ref).max()), "lse_max_abs": float(np.abs(lg - l_ref).max()),
              "dq_rel_l2": rel(dq, dq_ref), "dk_rel_l2": rel(dk, dk_ref), "dv_rel_l2": rel(dv, dv_ref), "all_finite": finite,
              "tolerances": {"out_max_abs": 1e-2, "lse_max_abs": 1e-3, "grad_rel_l2": 2e-2}}
    parity["within_tolerance"] = bool(finite and parity["out_max_abs"] <= 1e-2 and parity["lse_max_abs"] <= 1e-3 and
                                      max(parity["dq_rel_l2"], parity["dk_rel_l2"], parity["dv_rel_l2"]) <= 2e-2)
    return base, parity


if __name__ == "__main__":
    main()
