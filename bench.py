#!/usr/bin/env python3
"""Benchmark of the MoE-layer forward (Algorithm 1 without the all-reduce) on one MI355X.

A "step" is one moe_layer_forward call: gate, permutation, slice, both grouped expert GEMMs and the
combine (slice and combine done by the GEMMs' own loads and stores on the top-1 path), over one
batch of synthetic tokens already resident in HBM.  The default workload is the
headline configuration (T=8192, d=2048, F=8192, E=8, top-1, bf16).

Prints ONE JSON line: layer tokens/s as `value`, a `roofline` object for the dominant kernel (the
GeLU grouped GEMM) timed with HIP events recorded inside the timed region, per-stage timings, and a
`cpu_baseline` object: the fp64 oracle timed on the host cores on a bounded token sample.
"""

from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0   # MI355X dense bf16 MFMA
PEAK_HBM_GBS = 8000.0       # MI355X HBM3E
TRAFFIC_FILE = os.path.join(ROOT, "profiles", "grouped_gemm_{workload}_hbm_traffic.txt")


def measured_traffic(workload, stage):
    """HBM bytes per launch of one of the grouped GEMMs ("ffn_up" / "ffn_down"), from the committed
    rocprofv3 --pmc summary (the counters cannot be read from inside this process).  None when
    there is no summary for this workload."""
    try:
        text = open(TRAFFIC_FILE.format(workload=workload)).read()
    except OSError:
        return None
    if f"workload: {workload}" not in text:
        return None
    for line in text.splitlines():
        if line.startswith(f"traffic_bytes_per_launch[{stage}]:"):
            return float(line.split(":")[1])
    return None


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def cpu_baseline(lc, inp, sample_tokens):
    """The oracle as it stands, on the first `sample_tokens` tokens of the same workload."""
    from oracle import ppmoe_oracle as O
    from paper_2304_11414_amd import synth
    try:
        from threadpoolctl import threadpool_info
        threads = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        threads = os.cpu_count() or 1
    mv = synth.math_views(inp)
    xs = inp["x"][:sample_tokens]
    t0 = time.perf_counter()
    O.layer_forward(xs, mv["Wg"], inp["bias"], mv["W1"], mv["W2"], E=lc.E, k=lc.top_k,
                    local_begin=lc.local_begin, local_count=lc.n_local,
                    capacity_factor=lc.capacity_factor, renorm=lc.renorm_topk)
    dt = time.perf_counter() - t0
    return {"value": xs.shape[0] / dt, "unit": "tokens/s", "cores": int(threads), "kind": "oracle",
            "sample": f"whole layer (numpy fp64, its matmuls on the BLAS numpy links, {threads} threads) on "
                      f"the first {xs.shape[0]} of {lc.T} tokens, all {lc.n_local} local experts' "
                      f"weights, {dt:.2f} s"}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=30)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--settle", type=int, default=80,
                    help="layer calls made before the warm-up steps so that the device's power management has "
                         "settled (from idle it boosts, over-corrects for about 10 ms and takes about 25 ms "
                         "of load to reach the clock it then keeps): the timed steps measure steady state")
    ap.add_argument("--config", type=int, default=1, help="index into synth.CONFIGS (1 = headline)")
    ap.add_argument("--cpu-sample", type=int, default=8192, help="tokens the CPU oracle is timed on")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--dtype", choices=("bf16", "f16"), default=None,
                    help="run the (bf16) workload in this 16-bit type instead (f16: the paper's own precision)")
    ap.add_argument("--no-backward", action="store_true",
                    help="skip the (untimed-region) measurement of moe_layer_backward")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run the library's plain copy kernel on 1 GiB (reference of known "
                         "traffic for rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs)")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on ONE GPU only (no collectives, no sharding); "
                 "--gpus must be 1")

    import torch
    from paper_2304_11414_amd import binding as B
    from paper_2304_11414_amd import synth

    if not torch.cuda.is_available():
        sys.exit("bench.py: no GPU visible")
    B.load_library()
    B.moe_init()          # one-time set-up of the device (the only call here that synchronises by itself)
    lc = synth.CONFIGS[args.config]
    if args.dtype is not None and lc.in_dtype != "f32" and args.dtype != lc.in_dtype:
        lc = lc.scaled(name=f"{lc.name}_{args.dtype}", in_dtype=args.dtype,
                       out_dtype=args.dtype if lc.out_dtype != "f32" else "f32")
    log(f"[bench] workload {lc.name}: T={lc.T} d={lc.d} F={lc.F} E={lc.E} local={lc.n_local} "
        f"top_k={lc.top_k} cf={lc.capacity_factor} {lc.in_dtype}->{lc.out_dtype}")
    inp = synth.make_inputs(lc)
    cfg = B.config_from(lc)
    tmap = {"bf16": torch.bfloat16, "f16": torch.float16, "f32": torch.float32}
    tdt, odt = tmap[lc.in_dtype], tmap[lc.out_dtype]
    dev = {k: (torch.from_numpy(v).cuda().to(tdt) if k != "bias" else torch.from_numpy(v).cuda())
           for k, v in inp.items() if v is not None}
    bias = dev.get("bias")
    ws = torch.empty(B.moe_workspace_bytes(cfg), dtype=torch.uint8, device="cuda")
    out = torch.empty((lc.T, lc.d), dtype=odt, device="cuda")

    def step(events=None):
        B.moe_layer_forward(cfg, dev["x"], dev["Wg_t"], bias, dev["W1_t"], dev["W2_t"], out, ws,
                            stage_events=events)

    for _ in range(max(0, args.settle)):
        step()
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    if args.calibrate_copy:
        src = torch.empty(1 << 30, dtype=torch.uint8, device="cuda")
        dst = torch.empty_like(src)
        src.fill_(1)
        for _ in range(3):
            B.moe_copy_bytes(src, dst)
        torch.cuda.synchronize()
        del src, dst

    # Timed region 1: K steps, nothing but the layer calls -> tokens/s.
    K = args.steps
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(K):
        step()
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    ms_per_step = wall * 1e3 / K
    assert B.moe_ffn_check(cfg, ws, True) == 0, "a hand-over of partial sums did not arrive (timed region)"

    # The same K steps replayed from a HIP graph holding one layer call (second reported number:
    # what a caller that captures the layer pays per step, without the host's launch work).
    graph_ms_per_step = None
    try:
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.stream(side):
            step()
            torch.cuda.synchronize()
            with torch.cuda.graph(graph, stream=side):
                step()
        torch.cuda.current_stream().wait_stream(side)
        for _ in range(max(0, args.settle) + args.warmup):   # (the capture left the device idle: settle again)
            graph.replay()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(K):
            graph.replay()
        torch.cuda.synchronize()
        graph_ms_per_step = (time.perf_counter() - t0) * 1e3 / K
        assert B.moe_ffn_check(cfg, ws, True) == 0, "a hand-over of partial sums did not arrive (graph replays)"
        del graph
    except Exception as exc:   # (a failed capture must not cost the run its headline number)
        log(f"[bench] graph replay not measured: {exc!r}")

    # Timed region 2: the same K steps with HIP events recorded on the stream around every stage
    # (each record costs a few microseconds, which is why region 1 carries the headline number).
    events = [[B.moe_event_create() for _ in range(B.MOE_NUM_STAGES + 1)] for _ in range(K)]
    for _ in range(max(0, args.settle)):
        step()
    torch.cuda.synchronize()
    for i in range(K):
        step(events[i])
    torch.cuda.synchronize()
    assert B.moe_ffn_check(cfg, ws, True) == 0, "a hand-over of partial sums did not arrive (event region)"

    stage_ms = np.zeros(B.MOE_NUM_STAGES)
    for i in range(K):
        for s in range(B.MOE_NUM_STAGES):
            stage_ms[s] += B.moe_event_elapsed_ms(events[i][s], events[i][s + 1])
    stage_ms /= K
    ev_total = float(np.mean([B.moe_event_elapsed_ms(e[0], e[-1]) for e in events]))
    for e in events:
        for h in e:
            B.moe_event_destroy(h)

    # Empirical ceilings of this device, measured here with the library's own helpers: a plain
    # copy kernel (HBM) and a register-resident MFMA loop with the GEMM's launch shape (matrix
    # cores; random operands draw more power and settle at a lower clock than constant ones).
    def timed(fn, reps):
        fn()
        e0, e1 = B.moe_event_create(), B.moe_event_create()
        torch.cuda.synchronize()
        B.moe_event_record(e0)
        for _ in range(reps):
            fn()
        B.moe_event_record(e1)
        torch.cuda.synchronize()
        ms = B.moe_event_elapsed_ms(e0, e1) / reps
        B.moe_event_destroy(e0)
        B.moe_event_destroy(e1)
        return ms
    ceilings = {}
    src = torch.empty(1 << 30, dtype=torch.uint8, device="cuda")
    dst = torch.empty_like(src)
    src.fill_(1)
    ceilings["copy_gbs"] = round(2 * src.numel() / (timed(lambda: B.moe_copy_bytes(src, dst), 10) * 1e-3) / 1e9, 1)
    del src, dst
    sink = torch.empty(65536, dtype=torch.float32, device="cuda")
    for name, rnd in (("mfma_random_tflops", 1), ("mfma_constant_tflops", 0)):
        fl = []
        ms = timed(lambda: fl.append(B.moe_mfma_probe(100000, rnd, sink)), 3)
        ceilings[name] = round(fl[-1] / (ms * 1e-3) / 1e12, 1)

    # The row-movement kernels on their own (K3 slice, K6 combine): on the fused top-1 path the layer
    # does not run them, so their bandwidth is measured through the stage entry points, on the
    # layer's own routing, back to back (launch gaps included).
    views = B.workspace_views(cfg, ws)
    step()
    torch.cuda.synchronize()
    rows_max = max(B.moe_max_rows(cfg), 1)
    xs = torch.empty((rows_max, lc.d), dtype=tdt, device="cuda")
    ys = torch.empty((rows_max, lc.d), dtype=tdt, device="cuda").normal_()
    out2 = torch.empty_like(out)
    def timed_graph(fn, reps=20):
        """Mean time of one call, `reps` calls replayed from a HIP graph (kernel time without the
        host's launch gaps, which are a sixth of a 12 us kernel)."""
        fn(None)
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        g = torch.cuda.CUDAGraph()
        with torch.cuda.stream(side):
            with torch.cuda.graph(g, stream=side):
                for _ in range(reps):
                    fn(side)
        torch.cuda.current_stream().wait_stream(side)
        torch.cuda.synchronize()
        return timed(g.replay, 3) / reps
    standalone_ms = {
        "slice": timed_graph(lambda st: B.moe_slice_rows(cfg, dev["x"], views["perm"], views["offsets"], xs, stream=st)),
        "combine": timed_graph(lambda st: B.moe_combine(cfg, ys, views["inv_perm"], views["gate_w"], out2, stream=st))}
    # What clock the two GEMMs run at (the library's in-kernel read-out), each launched alone a few
    # times on the layer's routing; and, for context, the vendor library's dense GEMM (torch.matmul)
    # on the same two shapes with all rows in one group -- no ragged groups, no activation.
    gemm_clock, dense = {}, {}
    if lc.in_dtype != "f32" and int(views["offsets"][-1].item()) > 0:
        rows_now = int(views["offsets"][-1].item())
        Hs = torch.empty((rows_max, lc.F), dtype=tdt, device="cuda")
        fws = torch.empty(B.moe_ffn_workspace_bytes(cfg), dtype=torch.uint8, device="cuda")
        for name, call in (("ffn_up", lambda: B.moe_expert_ffn_up(cfg, xs, views["offsets"], dev["W1_t"], Hs, fws)),
                           ("ffn_down", lambda: B.moe_expert_ffn_down(cfg, Hs, views["offsets"], dev["W2_t"], ys, fws))):
            ms = timed(call, 5)
            ghz, us = B.moe_ffn_clock(cfg, fws, False)
            gemm_clock[name] = {"shader_ghz": round(ghz, 3), "first_block_us": round(us, 1), "alone_ms": round(ms, 5)}
        assert B.moe_ffn_check(cfg, fws, False) == 0
        del Hs, fws
        a_up = torch.randn((rows_now, lc.d), device="cuda").to(tdt)
        w_up = (torch.randn((lc.F, lc.d), device="cuda") * 0.02).to(tdt)
        ms_up = timed(lambda: torch.matmul(a_up, w_up.t()), 10)
        del a_up
        a_dn = torch.randn((rows_now, lc.F), device="cuda").to(tdt)
        w_dn = w_up.view(lc.d, lc.F)                            # (same layout as W2[i]: [d, F], F contiguous)
        ms_dn = timed(lambda: torch.matmul(a_dn, w_dn.t()), 10)
        del a_dn, w_up, w_dn
        fl = 2.0 * rows_now * lc.d * lc.F
        dense = {"what": "torch.matmul (vendor BLAS), one dense group of all kept rows, no activation",
                 "up_ms": round(ms_up, 5), "down_ms": round(ms_dn, 5),
                 "up_frac_of_mfma_peak": round(fl / (ms_up * 1e-3) / 1e12 / PEAK_BF16_TFLOPS, 4),
                 "down_frac_of_mfma_peak": round(fl / (ms_dn * 1e-3) / 1e12 / PEAK_BF16_TFLOPS, 4)}
    del xs, ys, out2

    counts = views["counts"].cpu().numpy()
    A = int(views["offsets"][-1].item())
    eb = 4 if lc.in_dtype == "f32" else 2
    ob = 4 if lc.out_dtype == "f32" else 2
    k = lc.top_k
    flops_up = 2.0 * A * lc.d * lc.F
    flops_dn = 2.0 * A * lc.F * lc.d
    flops_router = 2.0 * lc.T * lc.d * lc.E
    bytes_gate = lc.T * lc.d * eb + lc.E * lc.d * eb + 8 * k * lc.T
    bytes_slice = A * (2 * lc.d * eb + 4)
    bytes_combine = A * lc.d * eb + lc.T * (lc.d * ob + 8 * k)
    names = B.STAGE_NAMES
    st = dict(zip(names, stage_ms.tolist()))
    tflops_up = flops_up / (st["ffn_up"] * 1e-3) / 1e12
    tflops_dn = flops_dn / (st["ffn_down"] * 1e-3) / 1e12
    detail = {
        "stage_ms": {n: round(v, 5) for n, v in st.items()},
        "event_ms_per_step": round(ev_total, 5),
        "kept_rows": A, "expert_rows": counts.tolist(),
        "drop_rate": round(1.0 - A / max(1, k * lc.T), 5) if lc.n_local == lc.E else None,
        "layer_tflops": round((flops_router + flops_up + flops_dn) / (ms_per_step * 1e-3) / 1e12, 2),
        "ffn_up_tflops": round(tflops_up, 2), "ffn_down_tflops": round(tflops_dn, 2),
        "ffn_frac_of_mfma_peak": round((flops_up + flops_dn) / ((st["ffn_up"] + st["ffn_down"]) * 1e-3)
                                       / 1e12 / PEAK_BF16_TFLOPS, 4),
        "empirical_ceilings": ceilings,
        "gemm_clock": gemm_clock,
        "dense_gemm_library": dense,
        "ffn_frac_of_mfma_random_ceiling": round((flops_up + flops_dn) / ((st["ffn_up"] + st["ffn_down"]) * 1e-3)
                                                 / 1e12 / ceilings["mfma_random_tflops"], 4),
        "gate_gbs": round(bytes_gate / (st["gate"] * 1e-3) / 1e9, 1),
        "layer_fuses": {"slice": bool(B.moe_layer_fuses(cfg) & B.MOE_FUSE_SLICE),
                        "combine": bool(B.moe_layer_fuses(cfg) & B.MOE_FUSE_COMBINE)},
        "standalone_ms": {n: round(v, 5) for n, v in standalone_ms.items()},
        "slice_gbs": round(bytes_slice / (standalone_ms["slice"] * 1e-3) / 1e9, 1),
        "combine_gbs": round(bytes_combine / (standalone_ms["combine"] * 1e-3) / 1e9, 1),
        "slice_frac_of_hbm_peak": round(bytes_slice / (standalone_ms["slice"] * 1e-3) / 1e9 / PEAK_HBM_GBS, 4),
        "combine_frac_of_hbm_peak": round(bytes_combine / (standalone_ms["combine"] * 1e-3) / 1e9 / PEAK_HBM_GBS, 4),
    }
    # The dominant kernel is whichever of the two grouped GEMMs (same kernel template, equal FLOPs)
    # takes longer.  Which roof bounds it: the matrix cores, unless streaming the local experts' weights
    # once from HBM already takes longer than the FLOPs at peak (few rows per expert: workload 4).
    dom = "ffn_up" if st["ffn_up"] >= st["ffn_down"] else "ffn_down"
    dom_tflops = tflops_up if dom == "ffn_up" else tflops_dn
    gemm_bytes = lc.n_local * lc.d * lc.F * eb + A * (lc.d + lc.F) * eb      # weights once + both activations
    t_mfma = flops_up / (PEAK_BF16_TFLOPS * 1e12)
    t_hbm = gemm_bytes / (PEAK_HBM_GBS * 1e9)
    detail["gemm_roof"] = {"flops_per_gemm": flops_up, "bytes_per_gemm": gemm_bytes,
                           "time_at_mfma_peak_us": round(t_mfma * 1e6, 2), "time_at_hbm_peak_us": round(t_hbm * 1e6, 2),
                           "ffn_up_frac_of_roof": round(max(t_mfma, t_hbm) / (st["ffn_up"] * 1e-3), 4),
                           "ffn_down_frac_of_roof": round(max(t_mfma, t_hbm) / (st["ffn_down"] * 1e-3), 4)}
    if t_hbm > t_mfma:
        dom_gbs = gemm_bytes / (st[dom] * 1e-3) / 1e9
        roofline = {"bound": "hbm", "kernel": f"grouped_gemm_bf16_fast_kernel ({dom})", "achieved": dom_gbs,
                    "peak": PEAK_HBM_GBS, "unit": "GB/s", "frac": dom_gbs / PEAK_HBM_GBS,
                    "traffic": measured_traffic(lc.name, dom)}
    else:
        roofline = {"bound": "mfma", "kernel": f"grouped_gemm_bf16_fast_kernel ({dom})", "achieved": dom_tflops,
                    "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s", "frac": dom_tflops / PEAK_BF16_TFLOPS,
                    "traffic": measured_traffic(lc.name, dom)}

    # The layer's backward (a NEXT row of the scope, outside the timed forward regions): a few calls,
    # timed with events; its five grouped GEMMs are 2.5 x the forward's FLOPs.
    if lc.in_dtype != "f32" and not args.no_backward:
        try:
            d_out = torch.randn((lc.T, lc.d), device="cuda").to(odt)
            dx = torch.empty((lc.T, lc.d), dtype=tdt, device="cuda")
            dWg = torch.empty((lc.E, lc.d), dtype=torch.float32, device="cuda")
            dW1 = torch.empty((lc.n_local, lc.F, lc.d), dtype=torch.float32, device="cuda")
            dW2 = torch.empty((lc.n_local, lc.d, lc.F), dtype=torch.float32, device="cuda")
            bws = torch.empty(B.moe_layer_backward_workspace_bytes(cfg), dtype=torch.uint8, device="cuda")
            bw_ms = timed(lambda: B.moe_layer_backward(cfg, dev["x"], dev["Wg_t"], bias, dev["W1_t"], dev["W2_t"],
                                                       d_out, dx, dWg, None, dW1, dW2, bws), 5)
            detail["backward"] = {"ms_per_call": round(bw_ms, 4),
                                  "gemm_tflops": round(5 * flops_up / (bw_ms * 1e-3) / 1e12, 1),
                                  "ratio_to_forward": round(bw_ms / ms_per_step, 2)}
            # The training pair that keeps the forward's intermediates instead of recomputing them.
            saved = torch.empty(B.moe_layer_saved_bytes(cfg), dtype=torch.uint8, device="cuda")
            ft_ms = timed(lambda: B.moe_layer_forward_train(cfg, dev["x"], dev["Wg_t"], bias, dev["W1_t"], dev["W2_t"],
                                                            out, None, None, None, saved, ws), 5)
            bs_ms = timed(lambda: B.moe_layer_backward_saved(cfg, dev["x"], dev["Wg_t"], dev["W1_t"], dev["W2_t"],
                                                             d_out, saved, dx, dWg, None, dW1, dW2, bws), 5)
            detail["backward"].update({"forward_train_ms": round(ft_ms, 4), "backward_saved_ms": round(bs_ms, 4),
                                       "saved_gemm_tflops": round(4 * flops_up / (bs_ms * 1e-3) / 1e12, 1),
                                       "train_step_ratio_to_forward": round((ft_ms + bs_ms) / ms_per_step, 2)})
            del d_out, dx, dWg, dW1, dW2, bws, saved
        except Exception as exc:   # (the backward is not part of the headline number)
            log(f"[bench] backward not measured: {exc!r}")
    log("[bench] " + json.dumps(detail))

    result = {
        "metric": "MoE-layer fwd tokens/s at d=2048,E=8,top-1 bf16; % MFMA peak (GEMM), % HBM (slice)",
        "value": lc.T / (ms_per_step * 1e-3),
        "unit": "tokens/s",
        "n_gpus": 1, "steps": K, "warmup": args.warmup,
        "ms_per_step": ms_per_step,
        "graph_ms_per_step": graph_ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": lc.in_dtype, "data": "synthetic",
        "config": {"workload": f"{lc.name}: T={lc.T} d={lc.d} F={lc.F} E={lc.E} local={lc.n_local} "
                               f"top_k={lc.top_k} capacity_factor={lc.capacity_factor} "
                               f"{lc.in_dtype} in / {lc.out_dtype} out, seed {lc.seed}"},
        "roofline": roofline,
        "detail": detail,
    }
    if not args.no_cpu_baseline:
        log("[bench] timing the CPU oracle on a token sample")
        result["cpu_baseline"] = cpu_baseline(lc, inp, min(args.cpu_sample, lc.T))
    print(json.dumps(result), flush=True)


if __name__ == "__main__":
    main()
