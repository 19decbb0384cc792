#!/usr/bin/env python3
"""Benchmark of the AES-SpMM hot path on one MI355X.

One step = one pass of the whole hot path over one synthetic graph already
resident in HBM:
    aes_sample_build -> aes_spmm_f32 -> aes_quantize_features -> aes_spmm_q8
The default workload is the largest graph ("products_like": 2.45 M nodes,
~120 M edges, F = 128, W = 64, int8 features with per-row scales).

Prints ONE JSON line.  `value` is the step's algorithmic bytes (no-reuse model:
8 B per sampled slot + one feature row per slot + the output, see
`algorithmic_bytes`) divided by the step time.

`roofline` describes the dominant kernel (the fp32 SpMM), timed with HIP events
inside the timed region:
  achieved   algorithmic bytes / time: an EFFECTIVE rate.  A feature row that
             many slots reference is fetched once and then served by L2 or the
             Infinity Cache, so this rate may exceed what HBM delivers and is not
             a fraction of any roof.
  traffic    bytes that crossed the L2 <-> fabric boundary in one launch
             (rocprofv3 FETCH_SIZE + WRITE_SIZE of a recorded profile under
             profiles/; reads served by the Infinity Cache are included - no
             counter on this chip separates them from HBM reads)
  frac       traffic / time / 8 TB/s: an upper bound on the HBM fraction of the
             timed launch, never above 1
  hbm_anchor the same kernels on the same plan with every column index replaced
             by a uniformly random row of a 2 GiB / 8 GiB feature table, measured
             in this run: no reuse is possible, the gathers come from HBM, so
             algorithmic bytes = HBM bytes and the rate is the kernel's fraction
             of the HBM roof proper
`cpu_baseline` is the CPU oracle timed on the same workload on this machine's host
cores; `max_rel_err` compares the outputs of the TIMED kernels with it.
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

HBM_PEAK_GBPS = 8000.0          # MI355X published HBM3E peak
TRAFFIC_FILE = os.path.join(ROOT, "profiles", "hbm_traffic.json")


def algorithmic_bytes(n_rows, S, F, elem_bytes, per_row_scale):
    """Bytes one multiply over a plan must move if nothing is reused:
    (col, val) per slot, one feature row per slot, Y once, s_rowptr (no row_perm: natural row order)."""
    b = 8 * S + S * F * elem_bytes + 4 * n_rows * F + 8 * n_rows
    if per_row_scale:
        b += 4 * S
    return b


def build_bytes(n_rows, S):
    """rowptr in, sampled (col, val) in and out, s_rowptr out (no row_perm requested)."""
    return 8 * (n_rows + 1) + 8 * S + 8 * S + 8 * (n_rows + 1)


def quantize_bytes(n, F, groups):
    return 4 * n * F + n * F + 8 * groups


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="products_like")
    ap.add_argument("--width", type=int, default=0, help="sampling width W (default: the workload's first)")
    ap.add_argument("--cpu-rows", type=int, default=-1,
                    help="rows in the CPU oracle's sample (-1: all rows, 0: skip the CPU baseline)")
    ap.add_argument("--no-hbm-anchor", action="store_true",
                    help="skip the cache-defeating runs of the multiply kernels (random columns over 2 GiB / 8 GiB tables)")
    ap.add_argument("--copy-probe", action="store_true",
                    help="mark the run as a counter-calibration run (kept for the rocprofv3 command lines; the "
                         "plain 1 GiB read + 1 GiB write elementwise kernel they scale against always runs)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (no collectives, no sharding); use --gpus 1", file=sys.stderr)
        return 2

    import numpy as np
    import torch

    import paper_2503_18427_amd as aes
    from workloads import configs

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    aes.library()
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)

    t_gen = time.time()
    d = configs.make(args.workload, dev)
    w = d["workload"]
    W = args.width or w.widths[0]
    n, F, nnz = d["n"], d["F"], d["nnz"]
    rowptr, colidx, val, X = d["rowptr"], d["colidx"], d["val"], d["X"]
    torch.cuda.synchronize()
    t_gen = time.time() - t_gen

    scheme, gran = w.q_scheme, w.q_granularity
    groups = {0: 1, 1: F, 2: n}[gran]
    plan = aes.aes_sample_build(rowptr, colidx, val, n, W, 0)
    ws_build = torch.empty(max(aes.aes_sample_workspace_bytes(n), 8), dtype=torch.uint8, device=dev)
    ws_q = torch.empty(max(aes.aes_quantize_workspace_bytes(n, F, gran), 8), dtype=torch.uint8, device=dev)
    Y = torch.empty((n, F), dtype=torch.float32, device=dev)
    Yq = torch.empty((n, F), dtype=torch.float32, device=dev)
    qbuf = (torch.empty((n, F), dtype=torch.int8 if scheme == 1 else torch.uint8, device=dev),
            torch.empty(groups, dtype=torch.float32, device=dev), torch.empty(groups, dtype=torch.float32, device=dev))
    torch.cuda.synchronize()
    S = int(plan.s_rowptr[-1].item())

    legs = ["sample_build", "spmm_f32", "quantize", "spmm_q8"]
    leg_bytes = {
        "sample_build": build_bytes(n, S),
        "spmm_f32": algorithmic_bytes(n, S, F, 4, False),
        "quantize": quantize_bytes(n, F, groups),
        "spmm_q8": algorithmic_bytes(n, S, F, 1, gran == 2),
    }

    def step(events=None):
        marks = []

        def mark():
            if events is not None:
                e = torch.cuda.Event(enable_timing=True)
                e.record()
                marks.append(e)

        mark()
        aes.aes_sample_build(rowptr, colidx, val, n, W, 0, out=plan, workspace=ws_build)
        mark()
        aes.aes_spmm_f32(plan, X, Y)
        mark()
        aes.aes_quantize_features(X, scheme, gran, out=qbuf, workspace=ws_q)
        mark()
        aes.aes_spmm_q8(plan, qbuf[0], scheme, gran, qbuf[1], qbuf[2], Yq)
        mark()
        if events is not None:
            events.append(marks)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    events = []
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step(events)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_per_step = (t1 - t0) * 1e3 / args.steps

    leg_ms = {k: 0.0 for k in legs}
    for marks in events:
        for i, k in enumerate(legs):
            leg_ms[k] += marks[i].elapsed_time(marks[i + 1])
    leg_ms = {k: v / args.steps for k, v in leg_ms.items()}
    total_bytes = sum(leg_bytes.values())
    value = total_bytes / (ms_per_step * 1e-3) / 1e9
    leg_gbps = {k: leg_bytes[k] / (leg_ms[k] * 1e-3) / 1e9 for k in legs}

    def recorded(leg):
        """Per-launch L2 <-> fabric bytes of a leg's kernel from the recorded rocprofv3 profile, or None."""
        try:
            with open(TRAFFIC_FILE) as f:
                return json.load(f).get(f"{args.workload}:W{W}:{leg}")
        except (OSError, ValueError):
            return None

    rec = recorded("spmm_f32")
    traffic = rec["hbm_bytes"] if rec else None
    t_f32 = leg_ms["spmm_f32"] * 1e-3
    traffic_gbps = traffic / t_f32 / 1e9 if traffic else None
    # Compulsory traffic with a perfect cache: every distinct feature row once.
    distinct_cols = int(torch.unique(plan.s_col[:S]).numel()) if S > 0 else 0
    compulsory = 8 * S + distinct_cols * F * 4 + 4 * n * F + 8 * n
    t_min_ms = compulsory / (HBM_PEAK_GBPS * 1e9) * 1e3
    if traffic_gbps is not None:
        frac, frac_basis = min(1.0, traffic_gbps / HBM_PEAK_GBPS), (
            "recorded L2<->fabric traffic of this kernel on this workload / this run's kernel time / peak; Infinity "
            "Cache hits are inside the traffic, so this bounds the HBM fraction from above")
    else:
        frac, frac_basis = min(1.0, leg_gbps["spmm_f32"] / HBM_PEAK_GBPS), (
            "no recorded traffic for this workload and width: algorithmic rate / peak, capped at 1 (cache reuse "
            "can lift the algorithmic rate above the HBM roof)")
    roofline = {
        "kernel": "spmm_rows_kernel (aes_spmm_f32)",
        "bound": "hbm",
        "achieved": leg_gbps["spmm_f32"],
        "achieved_is": "algorithmic bytes (8S + 4SF + 4nF + 8n, no reuse) / average kernel time: an effective rate, "
                       "not a fraction of the HBM roof when feature rows are re-served by L2 / Infinity Cache",
        "peak": HBM_PEAK_GBPS,
        "unit": "GB/s",
        "frac": frac,
        "frac_is": frac_basis,
        "traffic": traffic,
        "traffic_GBps": traffic_gbps,
        "traffic_source": (rec.get("source") if rec else None),
        "traffic_is": "FETCH_SIZE + WRITE_SIZE per launch from two rocprofv3 --pmc runs, each scaled by a known-size "
                      "copy; a recorded profile, not measured in this run",
        "traffic_over_algorithmic": (traffic / leg_bytes["spmm_f32"]) if traffic else None,
        "algorithmic_bytes": leg_bytes["spmm_f32"],
        "avg_ms": leg_ms["spmm_f32"],
        "perfect_cache_model": {"distinct_feature_rows": distinct_cols, "compulsory_bytes": compulsory,
                                "t_min_ms": t_min_ms, "t_min_over_t": t_min_ms / leg_ms["spmm_f32"]},
    }

    def leg_record(k):
        r = {"ms": leg_ms[k], "GBps": leg_gbps[k], "bytes": leg_bytes[k]}
        rk = recorded(k)
        if rk:
            r["traffic_bytes"] = rk["hbm_bytes"]
            r["traffic_GBps"] = rk["hbm_bytes"] / (leg_ms[k] * 1e-3) / 1e9
            r["traffic_frac_of_peak"] = min(1.0, r["traffic_GBps"] / HBM_PEAK_GBPS)
        return r

    out = {
        "metric": "effective SpMM GB/s over the hot path (sample build + fp32 SpMM + int8 quantise + int8 SpMM; "
                  "algorithmic bytes / time)",
        "value": value,
        "unit": "GB/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": ms_per_step,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f32",
        "data": "synthetic",
        "config": {"workload": args.workload, "n_nodes": n, "nnz": nnz, "F": F, "W": W, "slots": S,
                   "int8": {"scheme": "symmetric_rne_i8" if scheme == 1 else "affine_floor_u8",
                            "granularity": ["tensor", "column", "row"][gran]},
                   "generate_s": round(t_gen, 2)},
        "legs": {k: leg_record(k) for k in legs},
        "gflops": {"spmm_f32": 2.0 * S * F / (leg_ms["spmm_f32"] * 1e-3) / 1e9,
                   "spmm_q8": 2.0 * S * F / (leg_ms["spmm_q8"] * 1e-3) / 1e9},
        "roofline": roofline,
    }

    # Outside the timed step: the single-kernel (sample on the fly) forms of both multiplies, and a
    # plain elementwise kernel that reads 1 GiB and writes 1 GiB (the stream ceiling of this machine, and
    # the known-size reference the rocprofv3 HBM counters are scaled with).
    def timed(fn, iters=5):
        fn()
        ev = [torch.cuda.Event(enable_timing=True) for _ in range(iters + 1)]
        ev[0].record()
        for i in range(iters):
            fn()
            ev[i + 1].record()
        torch.cuda.synchronize()
        return sorted(ev[i].elapsed_time(ev[i + 1]) for i in range(iters))[iters // 2]

    # Error figures first: Y and Yq still hold what the TIMED kernels (aes_spmm_f32 / aes_spmm_q8 on the
    # plan) wrote; the untimed single-kernel forms below overwrite them afterwards.
    if args.cpu_rows != 0:
        n_cpu = n if args.cpu_rows < 0 else min(args.cpu_rows, n)
        out["cpu_baseline"], out["max_rel_err"] = cpu_baseline(
            d, plan, Y, Yq, qbuf, W, scheme, gran, n_cpu, leg_bytes, total_bytes, S)
        out["max_rel_err"]["outputs_of"] = "the timed aes_spmm_f32 / aes_spmm_q8 launches of the last step"

    t_ff = timed(lambda: aes.aes_spmm_fused_f32(rowptr, colidx, val, n, W, X, Y=Y))
    t_fq = timed(lambda: aes.aes_spmm_fused_q8(rowptr, colidx, val, n, W, qbuf[0], scheme, gran, qbuf[1], qbuf[2],
                                               Y=Yq))
    out["fused_single_kernel"] = {"spmm_fused_f32_ms": t_ff, "spmm_fused_q8_ms": t_fq,
                                  "vs_build_plus_spmm_f32": (leg_ms["sample_build"] + leg_ms["spmm_f32"]) / t_ff}
    src = torch.ones(1 << 28, dtype=torch.float32, device=dev)
    dst = torch.empty_like(src)
    t_cp = timed(lambda: torch.mul(src, 1.0, out=dst), iters=3)
    out["stream_copy_GBps"] = 2.0 * (1 << 30) / (t_cp * 1e-3) / 1e9
    del src, dst
    if roofline["traffic_GBps"] is not None:
        roofline["traffic_over_stream_copy"] = roofline["traffic_GBps"] / out["stream_copy_GBps"]

    # The HBM roof proper: the timed kernels on the same plan (same rows, same slot counts, same launch) with
    # the column indices replaced by uniformly random rows of a feature table far larger than the caches
    # (L2 32 MiB, Infinity Cache 256 MiB), so nothing is reused and algorithmic bytes are HBM bytes.
    # Two table sizes: 2 GiB (at most 1/8 of the gathers can be served by the Infinity Cache; address
    # translation is still comfortable) and 8 GiB (no cache can matter, but random 512-byte gathers over so
    # many pages saturate the address-translation path: rocprofv3 shows the L2 TLB busy 98 % of the time).
    # Skipped when the workload's own feature matrix is already that large (then the timed legs are the
    # anchor) or when memory is short.
    def anchor(table_bytes):
        gen = torch.Generator(device=dev)
        gen.manual_seed(7)
        res = {}
        rows_f32 = table_bytes // (4 * F)
        Xa = torch.empty((rows_f32, F), dtype=torch.float32, device=dev).normal_(generator=gen)
        ca = torch.randint(0, rows_f32, (S,), dtype=torch.int32, device=dev, generator=gen)
        pa = aes.Plan(n, rows_f32, W, plan.s_rowptr, ca, plan.s_val, None, None)
        t_a = timed(lambda: aes.aes_spmm_f32(pa, Xa, Y))
        g_a = leg_bytes["spmm_f32"] / (t_a * 1e-3) / 1e9
        res["spmm_f32"] = {"ms": t_a, "GBps": g_a, "frac": g_a / HBM_PEAK_GBPS,
                           "over_stream_copy": g_a / out["stream_copy_GBps"], "table_rows": rows_f32}
        del Xa, ca, pa
        rows_q8 = table_bytes // F
        Xqa = torch.randint(-127, 128, (rows_q8, F), dtype=torch.int8, device=dev, generator=gen)
        ca = torch.randint(0, rows_q8, (S,), dtype=torch.int32, device=dev, generator=gen)
        groups_a = {0: 1, 1: F, 2: rows_q8}[gran]
        sa = torch.rand(groups_a, device=dev, generator=gen) + 0.5
        za = torch.zeros(groups_a, device=dev)
        pa = aes.Plan(n, rows_q8, W, plan.s_rowptr, ca, plan.s_val, None, None)
        t_q = timed(lambda: aes.aes_spmm_q8(pa, Xqa, scheme, gran, sa, za, Yq))
        g_q = leg_bytes["spmm_q8"] / (t_q * 1e-3) / 1e9
        res["spmm_q8"] = {"ms": t_q, "GBps": g_q, "frac": g_q / HBM_PEAK_GBPS, "table_rows": rows_q8}
        return res

    if not args.no_hbm_anchor and S > 0 and X.numel() * 4 < (2 << 30):
        roofline["hbm_anchor"] = {
            "what": "the timed kernels (aes_spmm_f32, aes_spmm_q8) on the same plan rows and launch, columns uniformly "
                    "random over a feature table of the given size (no reuse: algorithmic bytes = HBM bytes), measured "
                    "in this run; per-node int8 scales, where used, are gathered over the same random nodes"}
        for label, table_bytes in (("table_2GiB", 2 << 30), ("table_8GiB", 8 << 30)):
            try:
                torch.cuda.empty_cache()
                free, _ = torch.cuda.mem_get_info()
                if free < table_bytes + 4 * S + (4 << 30):
                    raise RuntimeError(f"only {free >> 30} GiB free")
                roofline["hbm_anchor"][label] = anchor(table_bytes)
            except (RuntimeError, torch.OutOfMemoryError) as exc:   # never let the anchor cost the bench line
                roofline["hbm_anchor"][label] = {"skipped": str(exc)[:200]}
    print(json.dumps(out))
    return 0


def cpu_baseline(d, plan, Y, Yq, qbuf, W, scheme, gran, n_rows_sample, leg_bytes, total_bytes, S):
    """The CPU oracle on a bounded sample of the same workload, on this machine's host
    cores; also the GPU-vs-oracle error on the sampled rows."""
    import numpy as np
    import torch

    import oracle as orc

    n, F = d["n"], d["F"]
    rowptr, colidx, val = (d[k].cpu().numpy() for k in ("rowptr", "colidx", "val"))
    X = d["X"].cpu().numpy()
    rng = np.random.default_rng(0)
    if n_rows_sample >= n:
        rows = np.arange(n, dtype=np.int64)
    else:
        rows = np.sort(rng.choice(n, size=n_rows_sample, replace=False)).astype(np.int64)

    t = time.perf_counter()
    ref = orc.sample_build(rowptr, colidx, val, W, 0, want_eid=False)
    t_build = time.perf_counter() - t
    slots_rows = int((ref[0][rows + 1] - ref[0][rows]).sum())

    t = time.perf_counter()
    Yref, Yabs = orc.spmm_plan(ref[0], ref[1], ref[2], X, rows=rows, want_abs=True)
    t_f32 = time.perf_counter() - t

    # The oracle quantises X itself; nothing it consumes comes from the GPU path.
    nq = n
    t = time.perf_counter()
    oq, osc, ozr = orc.quantize(X, scheme, gran)
    t_quant = time.perf_counter() - t
    codes_ok = bool(np.array_equal(qbuf[0].cpu().numpy(), oq)
                    and np.array_equal(qbuf[1].cpu().numpy().view(np.uint32), osc.view(np.uint32)))

    t = time.perf_counter()
    Yqref, Yqabs = orc.spmm_q8(ref[0], ref[1], ref[2], oq, scheme, gran, osc, ozr, rows=rows, want_abs=True)
    t_q8 = time.perf_counter() - t

    # one host core, on a bounded row sample (the full workload would take ~16 x longer)
    n_st = min(100_000, rows.size)
    rows_st = rows[:: max(1, rows.size // n_st)][:n_st]
    slots_st = int((ref[0][rows_st + 1] - ref[0][rows_st]).sum())
    threads = orc.num_threads()
    orc.set_num_threads(1)
    t = time.perf_counter()
    orc.spmm_plan(ref[0], ref[1], ref[2], X, rows=rows_st)
    t_st = time.perf_counter() - t
    orc.set_num_threads(threads)
    # the exact (unsampled) product on the same bounded row sample, all cores: the CSR is its own W = 0 plan
    nnz_st = int((rowptr[rows_st + 1] - rowptr[rows_st]).sum())
    t = time.perf_counter()
    orc.spmm_plan(rowptr, colidx, val, X, rows=rows_st)
    t_exact = time.perf_counter() - t

    groups_q = {0: 1, 1: F, 2: nq}[gran]
    rate = {
        "sample_build": leg_bytes["sample_build"] / t_build,
        "spmm_f32": algorithmic_bytes(n_rows_sample, slots_rows, F, 4, False) / t_f32,
        "quantize": quantize_bytes(nq, F, groups_q) / t_quant,
        "spmm_q8": algorithmic_bytes(n_rows_sample, slots_rows, F, 1, gran == 2) / t_q8,
    }
    est_step_s = sum(leg_bytes[k] / rate[k] for k in rate)

    rows_t = torch.from_numpy(rows).to(Y.device)
    Yg = Y[rows_t].cpu().numpy().astype(np.float64)
    Yqg = Yq[rows_t].cpu().numpy().astype(np.float64)
    e32 = float(np.max(np.abs(Yg - Yref) / np.where(Yabs > 0, Yabs, 1.0)))
    e8 = float(np.max(np.abs(Yqg - Yqref) / np.where(Yqabs > 0, Yqabs, 1.0)))
    plan_ok = bool(np.array_equal(plan.s_rowptr.cpu().numpy(), ref[0])
                   and np.array_equal(plan.s_col[:S].cpu().numpy(), ref[1]))

    base = {
        "value": total_bytes / est_step_s / 1e9,
        "unit": "GB/s",
        "cores": orc.num_threads(),
        "kind": "oracle",
        "sample": f"sample build on all rows; fp32 and int8 SpMM on {n_rows_sample} of {n} rows "
                  f"({slots_rows} slots; the int8 leg dequantises all of X first, as the oracle defines it); "
                  f"quantise on all {nq} feature rows; each leg's rate scaled to the full step's bytes",
        "seconds": {"sample_build": t_build, "spmm_f32": t_f32, "quantize": t_quant, "spmm_q8": t_q8},
        "leg_GBps": {k: v / 1e9 for k, v in rate.items()},
        "single_thread": {"spmm_f32_GBps": algorithmic_bytes(rows_st.size, slots_st, F, 4, False) / t_st / 1e9,
                          "rows": int(rows_st.size), "seconds": t_st},
        "exact_spmm": {"GBps": algorithmic_bytes(rows_st.size, nnz_st, F, 4, False) / t_exact / 1e9,
                       "rows": int(rows_st.size), "entries": nnz_st, "seconds": t_exact},
    }
    errs = {"fp32_vs_oracle": e32, "int8_vs_oracle_dequantised": e8, "plan_bit_exact": plan_ok,
            "int8_codes_and_scales_bit_exact": codes_ok,
            "rows_checked": n_rows_sample}
    return base, errs


if __name__ == "__main__":
    sys.exit(main())
