"""Measurement studies around the hot path, on one MI355X.

    python studies.py width-sweep [workload]
    python studies.py strategies  [workload]
    python studies.py loading     [workload]
    python studies.py layer       [workload]
    python studies.py graph       [workload]
    python studies.py sampling-rate [workload]
    python studies.py folded      [workload]
    python studies.py inline      [workload]
    python studies.py table-size

They reproduce the *shape* of the paper's evaluation on the synthetic workloads
(the paper's datasets are not available): kernel time and error against the
exact product per width W (Sec. 4.2), the per-row sampling-rate distribution
(Fig. 5), the adaptive strategy against the fixed AFS / SFS granularities
(Sec. 3.3), and what 8-bit features save when they are loaded from the host
(Sec. 3.1, Table 3).  Every product of the method is computed by the library's
kernels; torch is only used for norms, quantiles and host-to-device copies.
Output: markdown tables on stdout.
"""
from __future__ import annotations

import os
import sys

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

import torch  # noqa: E402

import paper_2503_18427_amd as aes  # noqa: E402
from workloads import configs  # noqa: E402


def _time_ms(fn, iters: int = 10, warmup: int = 2) -> float:
    """Median HIP-event time of fn() on the current stream."""
    for _ in range(warmup):
        fn()
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(iters + 1)]
    ev[0].record()
    for i in range(iters):
        fn()
        ev[i + 1].record()
    torch.cuda.synchronize()
    ts = sorted(ev[i].elapsed_time(ev[i + 1]) for i in range(iters))
    return ts[len(ts) // 2]


_evict = None


def _time_ms_cold(fn, iters: int = 5) -> float:
    """Median time of fn() when a 1 GiB buffer is overwritten before every call, so
    that neither L2 nor the 256 MB Infinity Cache holds the operands."""
    global _evict
    if _evict is None:
        _evict = torch.empty(1 << 28, dtype=torch.float32, device="cuda")
    ts = []
    for i in range(iters + 1):
        _evict.fill_(float(i))
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        fn()
        b.record()
        torch.cuda.synchronize()
        if i > 0:
            ts.append(a.elapsed_time(b))
    return sorted(ts)[len(ts) // 2]


def _rel_fro(Y: torch.Tensor, Yex: torch.Tensor) -> float:
    return float(torch.linalg.vector_norm((Y - Yex).double()) / torch.linalg.vector_norm(Yex.double()))


def _bytes(n, S, F, e, per_row_scale=False):
    return 8 * S + S * F * e + 4 * n * F + 8 * n + (4 * S if per_row_scale else 0)


def width_sweep(name: str) -> None:
    d = configs.make(name, "cuda")
    w = d["workload"]
    n, F, X = d["n"], d["F"], d["X"]
    scheme, gran = w.q_scheme, w.q_granularity
    q = aes.aes_quantize_features(X, scheme, gran)
    csr = (d["rowptr"], d["colidx"], d["val"])
    exact = aes.aes_sample_build(*csr, n, 0)
    Yex = aes.aes_spmm_f32(exact, X)
    t_ex = _time_ms(lambda: aes.aes_spmm_f32(exact, X, Yex))
    deg = (d["rowptr"][1:] - d["rowptr"][:-1]).double()
    print(f"### width sweep, `{name}`: n = {n}, nnz = {d['nnz']}, F = {F}, exact SpMM {t_ex:.3f} ms "
          f"({_bytes(n, d['nnz'], F, 4) / t_ex / 1e6:.0f} GB/s effective)\n")
    print("| W | slots S | sampled rows | median / mean row sampling rate | build ms | fp32 ms (cold) | fp32 GB/s | "
          "fused fp32 ms | int8 ms (cold) | int8 GB/s | speedup vs exact | rel. Frobenius error fp32 | int8 |")
    print("|---|---|---|---|---|---|---|---|---|---|---|---|---|")
    Y = torch.empty_like(Yex)
    for W in w.widths:
        plan = aes.aes_sample_build(*csr, n, W)
        S = int(plan.s_rowptr[-1])
        slots = (plan.s_rowptr[1:] - plan.s_rowptr[:-1]).double()
        rate = torch.where(deg > 0, slots / deg.clamp(min=1), torch.ones_like(deg))
        t_b = _time_ms(lambda: aes.aes_sample_build(*csr, n, W, out=plan))
        t32 = _time_ms(lambda: aes.aes_spmm_f32(plan, X, Y))
        t32c = _time_ms_cold(lambda: aes.aes_spmm_f32(plan, X, Y))
        e32 = _rel_fro(Y, Yex)
        t_f = _time_ms(lambda: aes.aes_spmm_fused_f32(*csr, n, W, X, Y=Y))
        t8 = _time_ms(lambda: aes.aes_spmm_q8(plan, q[0], scheme, gran, q[1], q[2], Y))
        t8c = _time_ms_cold(lambda: aes.aes_spmm_q8(plan, q[0], scheme, gran, q[1], q[2], Y))
        e8 = _rel_fro(Y, Yex)
        print(f"| {W} | {S} | {float((deg > W).double().mean()) * 100:.1f} % | "
              f"{float(rate.median()):.3f} / {float(rate.mean()):.3f} | {t_b:.3f} | {t32:.3f} ({t32c:.3f}) | "
              f"{_bytes(n, S, F, 4) / t32 / 1e6:.0f} | {t_f:.3f} | {t8:.3f} ({t8c:.3f}) | "
              f"{_bytes(n, S, F, 1, gran == 2) / t8 / 1e6:.0f} | {t_ex / t32:.2f}x | {e32:.4f} | {e8:.4f} |")
    print()


def strategies(name: str) -> None:
    d = configs.make(name, "cuda")
    w = d["workload"]
    n, F, X = d["n"], d["F"], d["X"]
    csr = (d["rowptr"], d["colidx"], d["val"])
    exact = aes.aes_sample_build(*csr, n, 0)
    Yex = aes.aes_spmm_f32(exact, X)
    Y = torch.empty_like(Yex)
    print(f"### adaptive vs fixed granularity, `{name}` (error = relative Frobenius distance to the exact product; "
          f"times: plan build / fused single kernel, ms)\n")
    print("| W | adaptive err | AFS err | SFS err | adaptive build / fused | AFS build / fused | SFS build / fused |")
    print("|---|---|---|---|---|---|---|")
    for W in w.widths:
        row = [f"| {W} "]
        errs, times = [], []
        for strat in (aes.AES_STRATEGY_ADAPTIVE, aes.AES_STRATEGY_AFS, aes.AES_STRATEGY_SFS):
            plan = aes.aes_sample_build(*csr, n, W, strategy=strat)
            aes.aes_spmm_f32(plan, X, Y)
            errs.append(_rel_fro(Y, Yex))
            tb = _time_ms(lambda: aes.aes_sample_build(*csr, n, W, strategy=strat, out=plan))
            tf = _time_ms(lambda: aes.aes_spmm_fused_f32(*csr, n, W, X, strategy=strat, Y=Y))
            times.append(f"{tb:.3f} / {tf:.3f}")
        print(f"| {W} | " + " | ".join(f"{e:.4f}" for e in errs) + " | " + " | ".join(times) + " |")
    print()


def loading(name: str) -> None:
    """Host-to-device feature loading: float32 vs 8-bit (+ stand-alone Eq. 2 pass) vs 8-bit fused."""
    d = configs.make(name, "cuda")
    w = d["workload"]
    n, F, X = d["n"], d["F"], d["X"]
    scheme, gran = w.q_scheme, w.q_granularity
    W = w.widths[0]
    plan = aes.aes_sample_build(d["rowptr"], d["colidx"], d["val"], n, W)
    q = aes.aes_quantize_features(X, scheme, gran)
    X_host = X.cpu().pin_memory()
    Xq_host = q[0].cpu().pin_memory()
    sc_host, zr_host = q[1].cpu().pin_memory(), q[2].cpu().pin_memory()
    X_dev = torch.empty_like(X)
    Xq_dev = torch.empty_like(q[0])
    sc_dev, zr_dev = torch.empty_like(q[1]), torch.empty_like(q[2])
    Y = torch.empty((n, F), device="cuda")

    def load_f32():
        X_dev.copy_(X_host, non_blocking=True)

    def load_q8():
        Xq_dev.copy_(Xq_host, non_blocking=True)
        sc_dev.copy_(sc_host, non_blocking=True)
        zr_dev.copy_(zr_host, non_blocking=True)

    t_l32 = _time_ms(load_f32, iters=5)
    t_l8 = _time_ms(load_q8, iters=5)
    t_dq = _time_ms(lambda: aes.aes_dequantize_features(Xq_dev, scheme, gran, sc_dev, zr_dev, X_dev))
    t_s32 = _time_ms(lambda: aes.aes_spmm_f32(plan, X_dev, Y))
    t_s8 = _time_ms(lambda: aes.aes_spmm_q8(plan, Xq_dev, scheme, gran, sc_dev, zr_dev, Y))
    print(f"### feature loading, `{name}` (n = {n}, F = {F}, W = {W}; pinned host memory, one stream; ms)\n")
    print("| pipeline | load | dequantise | SpMM | total | loading share | load time saved vs fp32 |")
    print("|---|---|---|---|---|---|---|")
    rows = [("fp32 features", t_l32, 0.0, t_s32),
            ("8-bit load + stand-alone Eq. 2 pass + fp32 SpMM (the paper's pipeline)", t_l8, t_dq, t_s32),
            ("8-bit load + fused dequantising SpMM", t_l8, 0.0, t_s8)]
    for label, tl, td, ts in rows:
        tot = tl + td + ts
        print(f"| {label} | {tl:.3f} | {td:.3f} | {ts:.3f} | {tot:.3f} | {tl / tot * 100:.1f} % | "
              f"{(1 - tl / t_l32) * 100:.1f} % |")
    print(f"\nhost-to-device rates: fp32 {X.numel() * 4 / t_l32 / 1e6:.1f} GB/s, "
          f"8-bit {(q[0].numel() + 8 * q[1].numel()) / t_l8 / 1e6:.1f} GB/s\n")
    # The loading share against the sampling width (the layout of the paper's Table 3): loading and the
    # Eq. 2 pass do not depend on W, the multiply does.
    widths = (16, 32, 64, 128, 256, 512, 1024)
    print(f"loading share of (load + dequantise + SpMM) against W, `{name}`:\n")
    print("| pipeline | " + " | ".join(f"W = {x}" for x in widths) + " |")
    print("|---|" + "---|" * len(widths))
    shares = {label: [] for label, *_ in rows}
    for Wx in widths:
        px = aes.aes_sample_build(d["rowptr"], d["colidx"], d["val"], n, Wx)
        tx32 = _time_ms(lambda: aes.aes_spmm_f32(px, X_dev, Y), iters=5)
        tx8 = _time_ms(lambda: aes.aes_spmm_q8(px, Xq_dev, scheme, gran, sc_dev, zr_dev, Y), iters=5)
        for (label, tl, td, _), ts in zip(rows, (tx32, tx32, tx8)):
            shares[label].append(tl / (tl + td + ts) * 100)
        del px
    for label, vals in shares.items():
        print(f"| {label} | " + " | ".join(f"{v:.1f} %" for v in vals) + " |")
    print()


def layer(name: str) -> None:
    """One GNN layer H = (A_s X) Theta: fused kernel vs SpMM followed by a library GEMM."""
    d = configs.make(name, "cuda")
    w = d["workload"]
    n, F, X = d["n"], d["F"], d["X"]
    g = torch.Generator(device="cuda")
    g.manual_seed(7)
    print(f"### fused layer, `{name}` (n = {n}, F = {F}; ms)\n")
    scheme, gran = w.q_scheme, w.q_granularity
    q = aes.aes_quantize_features(X, scheme, gran)
    print("| W | Fo | aes_spmm_f32 | library GEMM (torch.matmul, fp32) | sum | aes_gcn_layer_f32 | saved | "
          "max abs difference | aes_spmm_q8 | + GEMM | aes_gcn_layer_q8 | saved |")
    print("|---|---|---|---|---|---|---|---|---|---|---|---|")
    for W in w.widths:
        plan = aes.aes_sample_build(d["rowptr"], d["colidx"], d["val"], n, W)
        for Fo in (64, F):
            Theta = torch.randn((F, Fo), device="cuda", generator=g) / F ** 0.5
            Y = torch.empty((n, F), device="cuda")
            H0 = torch.empty((n, Fo), device="cuda")
            H1 = torch.empty((n, Fo), device="cuda")
            t_s = _time_ms(lambda: aes.aes_spmm_f32(plan, X, Y))
            t_g = _time_ms(lambda: torch.matmul(Y, Theta, out=H0))
            t_f = _time_ms(lambda: aes.aes_gcn_layer_f32(plan, X, Theta, H1))
            diff = float((H0 - H1).abs().max())
            t_s8 = _time_ms(lambda: aes.aes_spmm_q8(plan, q[0], scheme, gran, q[1], q[2], Y))
            t_f8 = _time_ms(lambda: aes.aes_gcn_layer_q8(plan, q[0], scheme, gran, q[1], q[2], Theta, H1))
            print(f"| {W} | {Fo} | {t_s:.3f} | {t_g:.3f} | {t_s + t_g:.3f} | {t_f:.3f} | "
                  f"{(1 - t_f / (t_s + t_g)) * 100:.1f} % | {diff:.2e} | {t_s8:.3f} | {t_s8 + t_g:.3f} | {t_f8:.3f} | "
                  f"{(1 - t_f8 / (t_s8 + t_g)) * 100:.1f} % |")
    print()


def folded(name: str) -> None:
    """8-bit SpMM with per-node scales: gathered per slot vs folded into the plan once."""
    d = configs.make(name, "cuda")
    w = d["workload"]
    n, F, X = d["n"], d["F"], d["X"]
    W = w.widths[0]
    plan = aes.aes_sample_build(d["rowptr"], d["colidx"], d["val"], n, W)
    S = int(plan.s_rowptr[-1])
    Y = torch.empty((n, F), device="cuda")
    t32 = _time_ms(lambda: aes.aes_spmm_f32(plan, X, Y), iters=5)
    print(f"### per-node scales gathered vs folded, `{name}` (n = {n}, S = {S}, F = {F}, W = {W}; ms; fp32 SpMM {t32:.3f})\n")
    print("| scheme | aes_spmm_q8 per row | fold pass | aes_spmm_q8 folded | speedup of the multiply | vs fp32 SpMM | "
          "max abs difference |")
    print("|---|---|---|---|---|---|---|")
    for scheme, label in ((aes.AES_Q_SYMMETRIC_RNE_I8, "symmetric int8"), (aes.AES_Q_AFFINE_FLOOR_U8, "affine uint8")):
        q = aes.aes_quantize_features(X, scheme, aes.AES_Q_PER_ROW)
        t_row = _time_ms(lambda: aes.aes_spmm_q8(plan, q[0], scheme, aes.AES_Q_PER_ROW, q[1], q[2], Y), iters=5)
        big = n * F > 2 ** 31                      # no second copy of Y for the very large workloads
        Y0 = None if big else Y.clone()
        fplan, bias = aes.aes_plan_fold_row_constants(plan, scheme, q[1], q[2])
        t_fold = _time_ms(lambda: aes.aes_plan_fold_row_constants(plan, scheme, q[1], q[2], s_val_folded=fplan.s_val,
                                                                  row_bias=bias), iters=5)
        t_f = _time_ms(lambda: aes.aes_spmm_q8(fplan, q[0], scheme, aes.AES_Q_PER_ROW_FOLDED, None, bias, Y), iters=5)
        diff = "-" if big else f"{float((Y - Y0).abs().max()):.1e}"
        print(f"| {label} | {t_row:.3f} | {t_fold:.3f} | {t_f:.3f} | {t_row / t_f:.2f}x | {t32 / t_f:.2f}x | {diff} |")
        del q, fplan, Y0
    print()


def inline(name: str) -> None:
    """8-bit SpMM with per-node constants: gathered from arrays of their own, read from the node's own
    row of codes (AES_Q_PER_ROW_INLINE), or folded into the plan, on the workload's graph at several
    feature widths (the paper's own widths, 100 / 500 / 602, leave room in a row's last 128-byte line;
    128 and 256 do not)."""
    from workloads import graphs
    w = configs.WORKLOADS[name]
    rowptr, colidx, val = configs.make_graph(w, "cuda")
    n, W = w.n, w.widths[0]
    plan = aes.aes_sample_build(rowptr, colidx, val, n, W)
    S = int(plan.s_rowptr[-1])
    print(f"### per-node constants: own arrays vs inside the rows vs folded, `{name}` graph (n = {n}, S = {S}, W = {W}; ms)\n")
    print("| F | scheme | bytes per row of codes (own arrays / inside) | aes_quantize_features (own / inside) | "
          "aes_spmm_q8 own arrays | inside the rows | folded plan | inside vs own | bit-identical |")
    print("|---|---|---|---|---|---|---|---|---|")
    for F in (100, 128, 500, 602):
        if n * F * 4 > 8 * 2 ** 30:
            continue
        X = graphs.features(n, F, w.x_dist, w.seed + 1000, torch.device("cuda"))
        Y = torch.empty((n, F), device="cuda")
        for scheme, label in ((aes.AES_Q_SYMMETRIC_RNE_I8, "symmetric int8"), (aes.AES_Q_AFFINE_FLOOR_U8, "affine uint8")):
            ld_own = (F + 127) // 128 * 128                  # rows on whole 128-byte lines in both layouts
            qdtype = torch.uint8 if scheme == aes.AES_Q_AFFINE_FLOOR_U8 else torch.int8
            own_buf = torch.empty((n, ld_own), dtype=qdtype, device="cuda")
            own = (own_buf[:, :F], torch.empty(n, device="cuda"), torch.empty(n, device="cuda"))
            t_qo = _time_ms(lambda: aes.aes_quantize_features(X, scheme, aes.AES_Q_PER_ROW, out=own), iters=5)
            ld_in = aes.aes_quantize_inline_ld(F, scheme)
            in_buf = torch.empty((n, ld_in), dtype=qdtype, device="cuda")
            t_qi = _time_ms(lambda: aes.aes_quantize_features(X, scheme, aes.AES_Q_PER_ROW_INLINE, out=in_buf), iters=5)
            q_in = aes.aes_quantize_features(X, scheme, aes.AES_Q_PER_ROW_INLINE, out=in_buf)
            t_own = _time_ms(lambda: aes.aes_spmm_q8(plan, own[0], scheme, aes.AES_Q_PER_ROW, own[1], own[2], Y), iters=5)
            Y0 = Y.clone()
            t_in = _time_ms(lambda: aes.aes_spmm_q8(plan, q_in[0], scheme, aes.AES_Q_PER_ROW_INLINE, None, None, Y), iters=5)
            same = bool(torch.equal(Y, Y0))
            fplan, bias = aes.aes_plan_fold_row_constants(plan, scheme, own[1], own[2])
            t_f = _time_ms(lambda: aes.aes_spmm_q8(fplan, own[0], scheme, aes.AES_Q_PER_ROW_FOLDED, None, bias, Y), iters=5)
            print(f"| {F} | {label} | {ld_own} / {ld_in} | {t_qo:.3f} / {t_qi:.3f} | {t_own:.3f} | {t_in:.3f} | {t_f:.3f} | "
                  f"{t_own / t_in:.2f}x | {same} |")
            del own_buf, own, in_buf, q_in, fplan, Y0
        del X, Y
    print()


def sampling_rate(name: str) -> None:
    """Distribution of the per-row sampling rate slots / row_nnz (the quantity of the paper's Fig. 5)."""
    d = configs.make(name, "cuda")
    n = d["n"]
    deg = (d["rowptr"][1:] - d["rowptr"][:-1]).double()
    print(f"### per-row sampling rate, `{name}` (n = {n}, nnz = {d['nnz']}): share of rows whose rate is at most x\n")
    xs = (0.05, 0.1, 0.2, 0.4, 0.6, 0.8, 0.99)
    print("| W | " + " | ".join(f"x = {x}" for x in xs) + " | mean rate | edges kept |")
    print("|---|" + "---|" * (len(xs) + 2))
    for W in (16, 32, 64, 128, 256, 512, 1024):
        plan = aes.aes_sample_build(d["rowptr"], d["colidx"], d["val"], n, W)
        slots = (plan.s_rowptr[1:] - plan.s_rowptr[:-1]).double()
        rate = torch.where(deg > 0, slots / deg.clamp(min=1), torch.ones_like(deg))
        cdf = " | ".join(f"{float((rate <= x).double().mean()) * 100:.1f} %" for x in xs)
        print(f"| {W} | {cdf} | {float(rate.mean()):.3f} | {float(slots.sum() / deg.sum()) * 100:.1f} % |")
    print()


def graph(name: str) -> None:
    """One whole step launched eagerly vs replayed from a captured HIP graph (small, launch-bound workloads)."""
    d = configs.make(name, "cuda")
    w = d["workload"]
    n, F, X = d["n"], d["F"], d["X"]
    scheme, gran = w.q_scheme, w.q_granularity
    W = w.widths[0]
    csr = (d["rowptr"], d["colidx"], d["val"])
    plan = aes.aes_sample_build(*csr, n, W)
    ws_b = torch.empty(max(aes.aes_sample_workspace_bytes(n), 8), dtype=torch.uint8, device="cuda")
    ws_q = torch.empty(max(aes.aes_quantize_workspace_bytes(n, F, gran), 8), dtype=torch.uint8, device="cuda")
    q = aes.aes_quantize_features(X, scheme, gran)
    Y = torch.empty((n, F), device="cuda")
    Yq = torch.empty((n, F), device="cuda")

    def step():
        aes.aes_sample_build(*csr, n, W, out=plan, workspace=ws_b)
        aes.aes_spmm_f32(plan, X, Y)
        aes.aes_quantize_features(X, scheme, gran, out=q, workspace=ws_q)
        aes.aes_spmm_q8(plan, q[0], scheme, gran, q[1], q[2], Yq)

    t_eager = _time_ms(step, iters=50, warmup=5)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        step()
    torch.cuda.current_stream().wait_stream(side)
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        step()
    t_graph = _time_ms(g.replay, iters=50, warmup=5)
    print(f"### whole step, eager launches vs HIP-graph replay, `{name}` (W = {W}): "
          f"{t_eager:.3f} ms vs {t_graph:.3f} ms\n")


def table_size(_name=None):
    """Where the multiply saturates: a synthetic plan (2^20 rows x 32 slots, uniformly random columns, no
    reuse beyond what the table size forces) over feature tables that fit L2, the Infinity Cache, or
    neither.  Separates what the kernel can issue from what each level of the memory system delivers."""
    from paper_2503_18427_amd import Plan
    n_rows, W = 1 << 20, 32
    S = n_rows * W
    gen = torch.Generator(device="cuda")
    gen.manual_seed(1)
    s_rowptr = torch.arange(n_rows + 1, device="cuda", dtype=torch.int64) * W
    s_val = torch.rand(S, device="cuda", generator=gen)
    print("### synthetic plan, uniformly random columns: algorithmic GB/s against the size of the feature table "
          f"({n_rows} rows x {W} slots)\n")
    print("| F | table rows | fp32 table MiB | aes_spmm_f32 ms | GB/s | int8 table MiB | aes_spmm_q8 ms (per column) | GB/s |")
    print("|---|---|---|---|---|---|---|---|")
    for F in (128, 256):
        Y = torch.empty(n_rows, F, device="cuda")
        for log_cols in (11, 13, 15, 17, 19, 21):
            n_cols = 1 << log_cols
            s_col = torch.randint(0, n_cols, (S,), device="cuda", dtype=torch.int32, generator=gen)
            X = torch.randn(n_cols, F, device="cuda", generator=gen)
            plan = Plan(n_rows, n_cols, W, s_rowptr, s_col, s_val, None, None)
            t32 = _time_ms(lambda: aes.aes_spmm_f32(plan, X, Y))
            q = aes.aes_quantize_features(X, aes.AES_Q_SYMMETRIC_RNE_I8, aes.AES_Q_PER_COLUMN)
            t8 = _time_ms(lambda: aes.aes_spmm_q8(plan, q[0], aes.AES_Q_SYMMETRIC_RNE_I8, aes.AES_Q_PER_COLUMN,
                                                  q[1], q[2], Y))
            b32, b8 = _bytes(n_rows, S, F, 4), _bytes(n_rows, S, F, 1)
            print(f"| {F} | 2^{log_cols} | {n_cols * F * 4 / 2**20:.0f} | {t32:.3f} | {b32 / t32 / 1e6:.0f} | "
                  f"{n_cols * F / 2**20:.1f} | {t8:.3f} | {b8 / t8 / 1e6:.0f} |")
    print()


def main(argv) -> int:
    if len(argv) < 2 or argv[1] not in ("width-sweep", "strategies", "loading", "layer", "graph", "sampling-rate", "folded", "inline", "table-size"):
        print(__doc__)
        return 2
    assert torch.cuda.is_available(), "the studies need a GPU"
    name = argv[2] if len(argv) > 2 else {"width-sweep": "rmat20", "strategies": "reddit_like",
                                          "loading": "products_like", "layer": "products_like", "graph": "arxiv_like", "sampling-rate": "reddit_like", "folded": "products_like", "inline": "products_like", "table-size": None}[argv[1]]
    {"width-sweep": width_sweep, "strategies": strategies, "loading": loading, "layer": layer,
     "graph": graph, "sampling-rate": sampling_rate, "folded": folded, "inline": inline, "table-size": table_size}[argv[1]](name)
    return 0


if __name__ == "__main__":
    sys.exit(main(sys.argv))
