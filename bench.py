#!/usr/bin/env python3
"""Benchmark of the contraction hot path on one MI355X.

A "step" is one pass of the whole path for one contraction: sb_contract() parses the mode strings,
plans the evaluation, selects a kernel and launches it on tensors that are already resident in
HBM.  The headline workload is the large cube C_mnp = sum_k A_km B_knp at 512^4 in fp32 evaluated
as one StridedBatchedGemm over p; the other benchmark contractions are timed too.

Prints ONE JSON line: metric / value (GFLOP/s) / ms_per_step ..., plus
  "roofline":     achieved vs peak for the headline kernel (HIP events on the launch stream; median, min
                  and max over at least 30 timed iterations), the HBM traffic measured with rocprofv3
                  counters (read from profiles/bench_default_hbm_traffic.txt), and under "configs" one
                  compact row per benchmark configuration (kernel time, achieved rate, fraction of the
                  roofline, the same over rotating buffers for working sets the last-level cache holds);
  "cpu_baseline": the CPU oracle timed on the host cores on a bounded sample of the same workload, with
                  all cores and with one thread (the paper's CPU figures are serial);
  "baselines":    the conventional evaluation on the same GPU, twice: explicit mode permutation with this
                  library's own permute kernel followed by this library's own GEMM (same GEMM code, so the
                  difference is the copy), and torch's permute/copy + vendor GEMM;
  "workloads":    the details behind "configs".
Every timed output buffer is checked afterwards: a few thousand of its elements against the oracle.
"""
import argparse
import json
import os
import re
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

# MI355X published peaks used for the roofline fractions
PEAK = {"hbm": 8000.0,                                   # GB/s
        "mfma": {"f64": 78.6, "f32": 157.3, "bf16": 2500.0}}   # TFLOP/s, dense
ESIZE = {"f64": 8, "f32": 4, "bf16": 2}
UNIT_ROUNDOFF = {"f64": 2.0 ** -53, "f32": 2.0 ** -24, "bf16": 2.0 ** -24}      # of the accumulation
OUT_ROUNDOFF = {"f64": 0.0, "f32": 0.0, "bf16": 2.0 ** -8}                        # of the stored result
TOL = {"f64": 1e-12, "f32": 1e-5, "bf16": 2e-2}
# which roofline binds each workload: dense high-intensity contractions are priced against the
# matrix cores, the batch-dominated / output-dominated ones against HBM
BOUND = {1: "hbm", 3: "hbm", 40: "mfma", 41: "mfma", 5: "hbm"}
SHORT = {1: "cfg1", 3: "cfg3", 40: "cfg4a", 41: "cfg4b", 5: "cfg5"}
MIB = 1 << 20
TRAFFIC_FILE = os.path.join(ROOT, "profiles", "bench_default_hbm_traffic.txt")
LLC_BYTES = 256 << 20      # Infinity Cache: working sets below this can be served without touching HBM


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=30)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--workload", type=int, default=41, help="headline workload id (inputs.WORKLOADS)")
    ap.add_argument("--only-headline", action="store_true", help="skip the other workloads")
    ap.add_argument("--prewarm-ms", type=float, default=100.0,
                    help="keep the device busy with another kernel for this long before the headline's warm-up steps (0: off)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-torch-baseline", action="store_true")
    ap.add_argument("--sweeps", action="store_true",
                    help="instead of the other workloads, add the size sweeps (cubic tensors, n = 8 .. 512) to the line")
    ap.add_argument("--sweeps-summary", default=None, help="with --sweeps: also write the sweeps as a text table to this file")
    ap.add_argument("--no-bf16-family", action="store_true", help="skip the dense bf16 products (the profiler commands under profiles/ do)")
    ap.add_argument("--no-tucker", action="store_true", help="skip the Tucker/HOOI timings (tens of thousands of small launches)")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run one device copy of known size (to scale rocprofv3 byte counters)")
    return ap.parse_args()


def dev(x, dtype):
    import torch
    from paper_1606_05696_amd import inputs
    flat = np.ascontiguousarray(x.ravel(order="F"))
    if dtype == "bf16":
        return torch.from_numpy(inputs.bf16_bits(flat).view(np.int16)).cuda().view(torch.bfloat16)
    return torch.from_numpy(flat).cuda()


def strip(s):
    return "".join(c for c in s if c.isalpha())


def workload_numbers(w):
    ext = w["ext"]
    nel = lambda s: int(np.prod([ext[c] for c in strip(s)], dtype=np.int64))
    labels = set(strip(w["A"])) | set(strip(w["B"]))
    flops = 2 * int(np.prod([ext[c] for c in labels], dtype=np.int64))
    nbytes = (nel(w["A"]) + nel(w["B"]) + nel(w["C"])) * ESIZE[w["dtype"]]    # each tensor touched once (beta = 0)
    return flops, nbytes


def time_steps(fn, steps, warmup):
    """Wall time per step (host clock around a synchronised region) and device time per launch
    (HIP events recorded on the launch stream around the same region)."""
    import torch
    for _ in range(warmup):
        fn()
    torch.cuda.synchronize()
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    ev0.record()
    for _ in range(steps):
        fn()
    ev1.record()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    return (t1 - t0) * 1e3 / steps, ev0.elapsed_time(ev1) / steps


def time_stats(fn, iters=30, warmup=10, target_us=200.0, max_inner=256):
    """Device time per launch as median / min / max over `iters` timed iterations (HIP events on the
    launch stream).  An iteration is `inner` back-to-back launches, enough of them to last about
    target_us, so that event resolution and launch gaps do not dominate the small workloads."""
    import torch
    for _ in range(warmup):
        fn()
    torch.cuda.synchronize()
    _, probe_ms = time_steps(fn, 5, 0)
    inner = int(min(max_inner, max(1, round(target_us / max(probe_ms * 1e3, 1e-3)))))
    evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(iters)]
    for e0, e1 in evs:
        e0.record()
        for _ in range(inner):
            fn()
        e1.record()
    torch.cuda.synchronize()
    us = np.array([e0.elapsed_time(e1) for e0, e1 in evs]) * 1e3 / inner
    return dict(median_us=float(np.median(us)), min_us=float(us.min()), max_us=float(us.max()), iters=iters,
                launches_per_iter=inner)


def measured_peaks(dtypes):
    """What this device sustains, for pricing next to the published peaks: the matrix-core rate of a
    pure-MFMA kernel per element type (sb_probe_mfma) and the rate of a 1 GiB device copy."""
    import torch
    import paper_1606_05696_amd as sb
    out = {}
    scratch = torch.empty(1 << 19, dtype=torch.float32, device="cuda")          # 2 MiB
    for dt in dtypes:
        flops = [0.0]

        def probe():
            flops[0] = sb.sb_probe_mfma(dt, 2048, scratch)[1]

        _, ms = time_steps(probe, 5, 2)
        out["mfma_%s_tflops" % dt] = flops[0] / ms / 1e9
    src = torch.empty(1 << 28, dtype=torch.float32, device="cuda")              # 1 GiB
    dst = torch.empty_like(src)
    _, ms = time_steps(lambda: dst.copy_(src), 5, 2)
    out["hbm_copy_gbps"] = 2.0 * src.numel() * 4 / ms / 1e6                      # read + write
    del src, dst
    torch.cuda.empty_cache()
    return out


def measured_traffic():
    """HBM-side bytes per launch of each workload's kernel, from the rocprofv3 counter summary kept
    under profiles/ (lines `workload <name> fetch_MiB write_MiB total_MiB`), with the commit it was
    taken at.  Measured offline with the profiler, not in this run."""
    out = {"source": os.path.relpath(TRAFFIC_FILE, ROOT), "commit": None, "bytes": {}}
    try:
        for ln in open(TRAFFIC_FILE):
            f = ln.split()
            if len(f) >= 5 and f[0] == "workload":
                out["bytes"][f[1]] = int(float(f[4]) * MIB)
            elif len(f) >= 2 and f[0] == "commit":
                out["commit"] = f[1]
    except OSError:
        out["source"] = None
    return out


def check_output(tC, dimsC, modesA, A, modesB, B, modesC, dtype, nsamples=3000, seed=99):
    """A few thousand elements of a timed output buffer against the oracle (eq. (1) at those positions):
    relative Frobenius error of the sample and the worst element relative to the running-error bound
    (K + 4) u K amax bmax (+ the output rounding for bf16)."""
    import torch
    from oracle import oracle
    rng = np.random.default_rng(seed)
    idx = np.stack([rng.integers(0, d, nsamples) for d in dimsC], axis=1).astype(np.int64)
    corners = np.array([[0] * len(dimsC), [d - 1 for d in dimsC]], dtype=np.int64)
    idx = np.concatenate([idx, corners])
    ld = np.cumprod([1] + list(dimsC[:-1])).astype(np.int64)
    off = torch.from_numpy(idx @ ld).cuda()
    got = tC[off].to(torch.float64).cpu().numpy()
    ref = oracle.contract_at(strip(modesA), A, strip(modesB), B, strip(modesC), idx, wide=(dtype == "f64"))
    K = int(np.prod([A.shape[strip(modesA).index(c)] for c in set(strip(modesA)) & set(strip(modesB))]))
    acc = (K + 4) * UNIT_ROUNDOFF[dtype] * K * float(np.abs(A).max()) * float(np.abs(B).max())
    bound = OUT_ROUNDOFF[dtype] * (np.abs(ref) + acc) + acc
    den = np.linalg.norm(ref)
    rel = float(np.linalg.norm(got - ref) / den) if den > 0 else float(np.linalg.norm(got))
    worst = float(np.max(np.abs(got - ref) / bound))
    ok = bool(np.isfinite(got).all() and rel <= TOL[dtype] and worst <= 1.0)
    return dict(samples=int(idx.shape[0]), rel_fro=rel, worst_error_over_bound=worst, ok=ok)


def roofline_of(bound, dtype, flops, nbytes, us):
    if bound == "mfma":
        ach, peak, unit = flops / us / 1e6, PEAK["mfma"][dtype], "TFLOP/s"
    else:
        ach, peak, unit = nbytes / us / 1e3, PEAK["hbm"], "GB/s"
    return dict(bound=bound, achieved=ach, peak=peak, unit=unit, frac=ach / peak)


def run_workload(cfg, steps, warmup, traffic, torch_baseline=True, evaluations=None, prewarm_ms=0.0):
    """One benchmark configuration: wall time over `steps` steps (the headline figure), kernel time as
    median / min / max, the cold-cache variant, the output check, the conventional baselines."""
    import torch
    import paper_1606_05696_amd as sb
    from paper_1606_05696_amd import inputs
    w = inputs.WORKLOADS[cfg]
    dtype = w["dtype"]
    A, B = inputs.workload_tensors(cfg)
    ext = w["ext"]
    dA, dB, dC = ([ext[c] for c in w[t]] for t in "ABC")
    tA, tB = dev(A, dtype), dev(B, dtype)
    tC = torch.empty(int(np.prod(dC)), dtype=tA.dtype, device="cuda")
    ma, mb, mc = w["eval"]
    flops, nbytes = workload_numbers(w)
    rc, plan = sb.sb_contract_plan(ma, mb, mc, dA, dB)

    def step():
        sb.sb_contract(ma, mb, mc, 1.0, tA, dA, tB, dB, 0.0, tC, dC)

    if prewarm_ms > 0:
        # Generating and uploading the inputs took seconds of host time with the GPU idle, and the chip
        # needs tens of milliseconds of work to come back to its sustained clocks: a few warm-up steps of a
        # 1 ms kernel do not get there.  Another kernel (the pure-MFMA probe, not the measured one) keeps the
        # device busy for prewarm_ms first; the W warm-up steps and the K timed steps follow directly.
        scratch = torch.empty(1 << 19, dtype=torch.float32, device="cuda")
        src = torch.empty(1 << 27, dtype=torch.float32, device="cuda")
        dst = torch.empty_like(src)
        _, pair_ms = time_steps(lambda: (dst.copy_(src), sb.sb_probe_mfma(dtype, 2048, scratch)), 4, 1)
        for _ in range(int(prewarm_ms / max(pair_ms, 1e-3)) + 1):      # queued without gaps; the warm-up steps follow on the same stream
            dst.copy_(src)
            sb.sb_probe_mfma(dtype, 2048, scratch)
    ms, kernel_ms = time_steps(step, steps, warmup)
    kernel = sb.sb_last_kernel()
    stats = time_stats(step, iters=max(30, steps), warmup=2)
    tC.fill_(float("nan"))
    step()
    check = check_output(tC, dC, ma, A, mb, B, mc, dtype)
    out = dict(workload=w["name"], short=SHORT[cfg], dtype=dtype, evaluation=plan.text(), kernel_family=kernel,
               ms_per_step=ms, kernel_ms=kernel_ms, kernel_us=stats, gflops=flops / ms / 1e6, flops=flops, bytes=nbytes,
               check=check)
    bound = BOUND[cfg]
    out["roofline"] = roofline_of(bound, dtype, flops, nbytes, kernel_ms * 1e3)
    out["roofline"]["traffic"] = traffic["bytes"].get(SHORT[cfg])
    if bound == "hbm" and nbytes > (8 << 20) and nbytes < 2 * LLC_BYTES:
        # same launch over rotating copies of B and C whose total size is twice the last-level
        # cache, so that no launch finds its operands cached from the previous one
        nsets = int(2 * LLC_BYTES // nbytes) + 1
        sets = [(tB.clone(), torch.empty_like(tC)) for _ in range(nsets)]
        state = {"i": 0}

        def cold_step():
            b, c = sets[state["i"] % nsets]
            state["i"] += 1
            sb.sb_contract(ma, mb, mc, 1.0, tA, dA, b, dB, 0.0, c, dC)

        _, cold_ms = time_steps(cold_step, max(steps, 2 * nsets), nsets)
        out["cold_cache"] = dict(kernel_ms=cold_ms, buffer_sets=nsets, achieved=nbytes / cold_ms / 1e6,
                                 frac=nbytes / cold_ms / 1e6 / PEAK["hbm"], unit="GB/s")
        del sets
    if evaluations:
        # the other evaluations of the same contraction (flattened / partly flattened / batched elsewhere):
        # the flat-versus-batched comparison of section IV-B on this machine
        rows = []
        for name, (ea, eb, ec) in evaluations:
            rc2, plan2 = sb.sb_contract_plan(ea, eb, ec, dA, dB)

            def other():
                sb.sb_contract(ea, eb, ec, 1.0, tA, dA, tB, dB, 0.0, tC, dC)

            st = time_stats(other, iters=30, warmup=5)
            fam = sb.sb_last_kernel()
            tC.fill_(float("nan"))
            other()
            chk = check_output(tC, dC, ea, A, eb, B, ec, dtype, nsamples=1000)
            r = roofline_of(bound, dtype, flops, nbytes, st["median_us"])
            rows.append(dict(name=name, evaluation=plan2.text(), kernel_family=fam, kernel_us=st, achieved=r["achieved"],
                             unit=r["unit"], frac=r["frac"], check_ok=chk["ok"]))
        out["evaluations"] = rows
    out["conventional_own"] = conventional_own(ma, mb, mc, ext, dtype, tA, tB, tC, flops)
    if torch_baseline:
        out["torch_matmul"] = conventional_baseline(cfg, tA, tB, dA, dB, dC, steps, warmup, flops)
    del tA, tB, tC
    torch.cuda.empty_cache()
    return out, (A, B)


def conventional_baseline(cfg, tA, tB, dA, dB, dC, steps, warmup, flops):
    """The conventional evaluation on the same GPU with the vendor's code: bring the operands into
    matricised form (explicit permute + copy where the layout needs one) and call the vendor GEMM through
    torch.  A column-major tensor with extents (d0, d1, ..) is a row-major torch tensor of shape (.., d1, d0)."""
    import torch
    from paper_1606_05696_amd import inputs
    w = inputs.WORKLOADS[cfg]
    a = tA.view(*reversed(dA))
    b = tB.view(*reversed(dB))
    la, lb, lc = w["A"][::-1], w["B"][::-1], w["C"][::-1]     # torch (row-major) index order
    expr = "%s,%s->%s" % (la, lb, lc)

    def step():
        return torch.einsum(expr, a, b).contiguous()

    ms, _ = time_steps(step, steps, warmup)
    return dict(ms_per_step=ms, gflops=flops / ms / 1e6, how="torch.einsum('%s') + contiguous()" % expr)


def matricise(ma, mb, mc):
    """The conventional algorithm of section II-D for C_mc = A_ma B_mb with one contracted index: the tensor
    that holds C's first mode becomes the left matrix (free modes, k), the other the right matrix
    (k, free modes), free modes in C's order; C is permuted back if it is not (left modes, right modes).
    Returns (left is A?, perm of the left tensor, perm of the right tensor, perm of the product back to C,
    rows, cols); a perm is None where the tensor already has the wanted mode order."""
    ma, mb, mc = strip(ma), strip(mb), strip(mc)
    k = (set(ma) & set(mb)).pop()
    left_is_a = mc[0] in ma
    L, R = (ma, mb) if left_is_a else (mb, ma)
    rows = [c for c in mc if c in L]
    cols = [c for c in mc if c in R]
    want_l, want_r, have_c = rows + [k], [k] + cols, rows + cols
    perm = lambda have, want: None if list(have) == list(want) else [list(have).index(c) for c in want]
    return left_is_a, perm(L, want_l), perm(R, want_r), perm(have_c, mc), rows, cols


def conventional_own(ma, mb, mc, ext, dtype, tA, tB, tC, flops, iters=30):
    """The conventional evaluation with THIS library's kernels: explicit mode permutations (sb_permute)
    into matricised form, one plain GEMM (sb_gemm with batch 1: the same GEMM code the copy-free path
    runs), a permutation of the result where needed.  kappa = number of permutation kernels."""
    import torch
    import paper_1606_05696_amd as sb
    left_is_a, pl, pr, pc, rows, cols = matricise(ma, mb, mc)
    sa, sb_, sc = strip(ma), strip(mb), strip(mc)
    tL, tR = (tA, tB) if left_is_a else (tB, tA)
    mL, mR = (sa, sb_) if left_is_a else (sb_, sa)
    k = (set(sa) & set(sb_)).pop()
    M = int(np.prod([ext[c] for c in rows], dtype=np.int64)) if rows else 1
    N = int(np.prod([ext[c] for c in cols], dtype=np.int64)) if cols else 1
    K = ext[k]
    bufL = torch.empty_like(tL) if pl else tL
    bufR = torch.empty_like(tR) if pr else tR
    bufC = torch.empty_like(tC) if pc else tC
    dL, dR = [ext[c] for c in mL], [ext[c] for c in mR]
    dP = [ext[c] for c in rows + cols]

    def run():
        if pl:
            sb.sb_permute(dL, pl, tL, bufL, dt=dtype)
        if pr:
            sb.sb_permute(dR, pr, tR, bufR, dt=dtype)
        sb.sb_gemm("N", "N", M, N, K, 1.0, bufL, M, 0, bufR, K, 0, 0.0, bufC, M, 0, 1, dt=dtype)
        if pc:
            sb.sb_permute(dP, pc, bufC, tC, dt=dtype)

    st = time_stats(run, iters=iters, warmup=3)
    kappa = sum(1 for p in (pl, pr, pc) if p)
    return dict(kappa=kappa, us=st["median_us"], min_us=st["min_us"], max_us=st["max_us"], gflops=flops / st["median_us"] / 1e3,
                how="%d x sb_permute + sb_gemm(N, N, %d, %d, %d, batch 1)" % (kappa, M, N, K))


def run_table2_cases(steps, warmup, torch_baseline=True):
    """cfg2: every order-2 x order-3 single-mode contraction (Table II) at extent 64, fp32, in the
    evaluation SB_AUTO picks, against the conventional route (explicit permutation + GEMM) in this
    library's own kernels and in torch's.  These calls are launch-bound: the figure of merit is time per
    call, back to back.  Also 1008 enqueues in a row twice: cycling through the 36 cases (no case finds its
    plan in the eight-entry cache, so parsing and planning are inside every call) and case by case (28
    calls of each in a row: every call but the first finds its plan)."""
    import itertools
    import torch
    import paper_1606_05696_amd as sb
    from paper_1606_05696_amd import inputs
    n = 64
    rows = []
    ext = dict(m=n, n=n, p=n, k=n)
    tC = torch.empty(n ** 3, dtype=torch.float32, device="cuda")
    A = inputs.uniform_tensor(21, [n, n], np.float32)
    B = inputs.uniform_tensor(22, [n, n, n], np.float32)
    tA, tB = dev(A, "f32"), dev(B, "f32")
    cases = []
    for free_a in "mnp":
        rest = [c for c in "mnp" if c != free_a]
        for ma in (free_a + "k", "k" + free_a):
            for perm in itertools.permutations(["k"] + rest):
                cases.append((ma, "".join(perm)))
    flops = 2 * n ** 4
    all_ok = True
    for ma, mb in cases:
        rc, plan = sb.sb_contract_plan(ma, mb, "mnp", [n, n], [n, n, n])

        def ours():
            sb.sb_contract(ma, mb, "mnp", 1.0, tA, [n, n], tB, [n, n, n], 0.0, tC, [n, n, n])

        st = time_stats(ours, iters=30, warmup=warmup)
        tC.fill_(float("nan"))
        ours()
        chk = check_output(tC, [n, n, n], ma, A, mb, B, "mnp", "f32", nsamples=300)
        all_ok = all_ok and chk["ok"]
        own = conventional_own(ma, mb, "mnp", ext, "f32", tA, tB, tC, flops, iters=10)
        row = dict(A=ma, B=mb, evaluation=plan.text(), exceptional=int(plan.exceptional), us_per_call=st["median_us"],
                   min_us=st["min_us"], max_us=st["max_us"], kappa=own["kappa"], conventional_own_us=own["us"])
        if torch_baseline:
            a, b = tA.view(n, n), tB.view(n, n, n)
            expr = "%s,%s->pnm" % (ma[::-1], mb[::-1])
            row["conventional_torch_us"] = time_stats(lambda: torch.einsum(expr, a, b).contiguous(), iters=10, warmup=3)["median_us"]
        rows.append(row)

    def enqueue(order, cache):
        sb.sb_plan_cache_enable(cache)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for ma, mb in order:
            sb.sb_contract(ma, mb, "mnp", 1.0, tA, [n, n], tB, [n, n, n], 0.0, tC, [n, n, n])
        t1 = time.perf_counter()              # host time to enqueue
        torch.cuda.synchronize()
        t2 = time.perf_counter()
        sb.sb_plan_cache_enable(True)
        return dict(calls=len(order), host_us_per_call=(t1 - t0) * 1e6 / len(order), total_us_per_call=(t2 - t0) * 1e6 / len(order))

    cycling = cases * 28                                    # 1008 calls, consecutive calls always differ
    grouped = [c for c in cases for _ in range(28)]         # the same 1008 calls, case by case
    enqueue(cycling[:72], True)                             # warm-up
    back_to_back = dict(cycling_cases_plan_cache_defeated=enqueue(cycling, True), case_by_case_plan_cache_hits=enqueue(grouped, True),
                        cycling_cases_plan_cache_off=enqueue(cycling, False))
    ours = np.array([r["us_per_call"] for r in rows])
    own = np.array([r["conventional_own_us"] for r in rows])
    kap = np.array([r["kappa"] for r in rows])
    out = dict(workload="cfg2: all 36 order-2 x order-3 contractions at 64^4, f32, SB_AUTO evaluation", short="cfg2",
               median_us_per_call=float(np.median(ours)), max_us_per_call=float(ours.max()),
               mean_gflops=float(flops / ours.mean() / 1e3), all_outputs_ok=bool(all_ok),
               conventional_own_mean_us={int(kv): float(own[kap == kv].mean()) for kv in sorted(set(kap))},
               speedup_over_conventional_own_by_kappa={int(kv): float((own[kap == kv] / ours[kap == kv]).mean()) for kv in sorted(set(kap))},
               case_1_3=next(r for r in rows if (r["A"], r["B"]) == ("mk", "nkp")),
               case_2_4=next(r for r in rows if (r["A"], r["B"]) == ("km", "pkn")),
               back_to_back_1008_enqueues=back_to_back, cases=rows)
    if torch_baseline:
        conv = np.array([r["conventional_torch_us"] for r in rows])
        out["conventional_torch_mean_us"] = float(conv.mean())
        out["speedup_over_conventional_torch_mean"] = float((conv / ours).mean())
    return out


def run_exceptional_cases(steps, warmup, n=512, torch_baseline=True, dtypes=("f32", "f64")):
    """Two exceptional cases of Table II (3.6 and 6.4, the ones section III-E writes out) at n^4 in
    fp32 and fp64: the extended-operation kernel against the two-step route the paper benchmarks it
    against (explicit mode transposition + GEMM), in this library's own kernels and in torch's."""
    import torch
    import paper_1606_05696_amd as sb
    from paper_1606_05696_amd import inputs
    rows = []
    flops = 2 * n ** 4
    ext = dict(m=n, n=n, p=n, k=n)
    for dtype in dtypes:
        npdt, tdt = (np.float32, torch.float32) if dtype == "f32" else (np.float64, torch.float64)
        A = inputs.uniform_tensor(31, [n, n], npdt)
        B = inputs.uniform_tensor(32, [n, n, n], npdt)
        tA, tB = dev(A, dtype), dev(B, dtype)
        tC = torch.empty(n ** 3, dtype=tdt, device="cuda")
        for case, ma, mb in (("3.6", "nk", "pmk"), ("6.4", "kp", "nkm")):
            rc, plan = sb.sb_contract_plan(ma, mb, "mnp", [n, n], [n, n, n])

            def ours():
                sb.sb_contract(ma, mb, "mnp", 1.0, tA, [n, n], tB, [n, n, n], 0.0, tC, [n, n, n], dt=dtype)

            st = time_stats(ours, iters=max(30, steps), warmup=warmup)
            family = sb.sb_last_kernel()
            tC.fill_(float("nan"))
            ours()
            chk = check_output(tC, [n, n, n], ma, A, mb, B, "mnp", dtype, nsamples=1000)
            own = conventional_own(ma, mb, "mnp", ext, dtype, tA, tB, tC, flops, iters=10)
            t_ours = st["median_us"] / 1e3
            row = dict(case=case, dtype=dtype, evaluation=plan.text(), kernel_family=family, kernel_ms=t_ours, kernel_us=st,
                       gflops=flops / t_ours / 1e6, frac_of_mfma_peak=flops / t_ours / 1e9 / PEAK["mfma"][dtype],
                       check_ok=chk["ok"], conventional_own=own, speedup_over_conventional_own=own["us"] / st["median_us"])
            if dtype == "f32":
                row["frac_of_fp32_mfma_peak"] = row["frac_of_mfma_peak"]
            if torch_baseline:
                a, b = tA.view(n, n), tB.view(n, n, n)
                expr = "%s,%s->pnm" % (ma[::-1], mb[::-1])
                _, t_conv = time_steps(lambda: torch.einsum(expr, a, b).contiguous(), steps, warmup)
                row["conventional_torch_ms"] = t_conv
                row["speedup_over_conventional_torch"] = t_conv / t_ours
            rows.append(row)
        del tA, tB, tC
    return dict(workload="exceptional cases 3.6 and 6.4 at %d^4, %s: extended-operation kernel" % (n, " and ".join(dtypes)), short="ext-op", cases=rows)


def run_bf16_family(torch_baseline=True, settle_ms=150.0):
    """Large dense bf16 products (section IV-B: a batched evaluation must not trail the flat GEMM) through
    sb_gemm in the three operand layouts: 4096^3 flat, eight batches of 2048^3 and 512 batches of 512^3.
    A dense bf16 product runs this chip against its power limit, so the device is kept busy (the same call,
    queued without gaps) for settle_ms before each timing, and the operands are normal random numbers: the
    4096^3 T,N product is timed on all-zero operands too, which shows how much of the rate the data decide.
    The vendor's batched GEMM (torch.bmm on the same buffers) is timed the same way."""
    import torch
    import paper_1606_05696_amd as sb
    from paper_1606_05696_amd import inputs

    def settled(fn):
        # batches of 20 calls, each batch waited for: the queue never holds more than that, however slow a
        # call is (under a profiler that serialises dispatches a loop bounded by host time alone would
        # queue tens of thousands)
        t0 = time.perf_counter()
        while (time.perf_counter() - t0) * 1e3 < settle_ms:
            for _ in range(20):
                fn()
            torch.cuda.synchronize()
        for _ in range(20):
            fn()
        return time_stats(fn, iters=30, warmup=5, target_us=400.0)

    layouts = {"T,N": ("km", "kn"), "N,N": ("mk", "kn"), "N,T": ("mk", "nk")}        # stored modes, first one contiguous
    rows = []
    for (n, batch) in ((4096, 1), (2048, 8), (512, 512)):
        ext = dict(m=n, n=n, k=n, p=batch)
        flops = 2 * n ** 3 * batch
        for name, (ma, mb) in layouts.items():
            mc = "mn"
            dA, dB, dC = ([ext[c] for c in m + "p"] for m in (ma, mb, mc))       # the batch is the last, slowest mode of all three
            A = inputs.make_tensor(7 * n + batch, dA, "bf16")
            B = inputs.make_tensor(7 * n + batch + 1, dB, "bf16")
            tA, tB = dev(A, "bf16"), dev(B, "bf16")
            tC = torch.empty(int(np.prod(dC)), dtype=torch.bfloat16, device="cuda")

            opA, opB = name.split(",")

            def ours():
                sb.sb_gemm(opA, opB, n, n, n, 1.0, tA, n, n * n, tB, n, n * n, 0.0, tC, n, n * n, batch, dt="bf16")

            st = settled(ours)
            family = sb.sb_last_kernel()
            tC.fill_(float("nan"))
            ours()
            # eq. (1) has no index common to all three tensors: the first and the last batch are checked as matrices
            ok = True
            for q in sorted({0, batch - 1}):
                chk = check_output(tC[q * n * n:(q + 1) * n * n], [n, n], ma, np.asfortranarray(A[:, :, q]), mb, np.asfortranarray(B[:, :, q]),
                                   mc, "bf16", nsamples=1000)
                ok = ok and chk["ok"]
            tf = flops / st["median_us"] / 1e6
            row = dict(layout=name, n=n, batch=batch, kernel_family=family, kernel_us=st, tflops=tf, frac_of_bf16_mfma_peak=tf / PEAK["mfma"]["bf16"],
                       check_ok=ok)
            if torch_baseline:
                # the same buffers as (batch, rows, cols) views: the stored matrices are column-major
                va = tA.view(batch, n, n).transpose(1, 2) if ma.startswith("m") else tA.view(batch, n, n)        # (m, k)
                vb = tB.view(batch, n, n) if mb.startswith("k") else tB.view(batch, n, n).transpose(1, 2)        # (n, k)
                sv = settled(lambda: torch.bmm(va, vb.transpose(1, 2)))
                row["vendor_us"] = sv["median_us"]
                row["vendor_tflops"] = flops / sv["median_us"] / 1e6
            if n == 4096 and name == "T,N":
                tA.zero_(); tB.zero_()
                row["tflops_on_zero_operands"] = flops / settled(ours)["median_us"] / 1e6
                if torch_baseline:
                    row["vendor_tflops_on_zero_operands"] = flops / settled(lambda: torch.bmm(va, vb.transpose(1, 2)))["median_us"] / 1e6
            rows.append(row)
            del tA, tB, tC
    return dict(workload="dense bf16 products 4096^3, 2048^3 x 8, 512^3 x 512 in three layouts", short="bf16-gemm", cases=rows)


def run_sweeps(steps, warmup):
    """Size sweeps over cubic tensors in fp32, the shapes of the paper's GPU plots (section IV):
    batches of n small GEMMs (n x n x n) against the vendor's strided-batched GEMM; case 1.1 in its
    three evaluations (flattened, batched in p, batched in n); the exceptional case 6.4 with the
    extended operation, as batched matrix-vector products and by transposition + GEMM; n matrix-vector products of n x n matrices (the BatchedGemv end).
    """
    import torch
    import paper_1606_05696_amd as sb
    from paper_1606_05696_amd import inputs
    sizes = [8, 16, 32, 64, 128, 256, 512]
    out = {}
    reps = lambda n: max(steps, 200) if n <= 128 else steps

    rows = []
    for n in sizes:      # n independent GEMMs of n x n x n, every operand batched (stride n^2)
        tA = dev(inputs.uniform_tensor(51, [n, n, n], np.float32), "f32")
        tB = dev(inputs.uniform_tensor(52, [n, n, n], np.float32), "f32")
        tC = torch.empty(n ** 3, dtype=torch.float32, device="cuda")

        def ours():
            sb.sb_gemm("N", "N", n, n, n, 1.0, tA, n, n * n, tB, n, n * n, 0.0, tC, n, n * n, n, dt="f32")

        a3, b3, c3 = tA.view(n, n, n), tB.view(n, n, n), tC.view(n, n, n)

        def vendor():      # row-major views: C_p^T = B_p^T A_p^T
            torch.bmm(b3, a3, out=c3)

        _, t_ours = time_steps(ours, reps(n), warmup)
        _, t_vend = time_steps(vendor, reps(n), warmup)
        flops, nbytes = 2 * n ** 4, 3 * 4 * n ** 3
        rows.append(dict(n=n, us=t_ours * 1e3, gflops=flops / t_ours / 1e6, gbps=nbytes / t_ours / 1e6,
                         vendor_bmm_us=t_vend * 1e3, kernel_family=sb.sb_last_kernel()))
    out["batched_gemm_n_of_nxnxn"] = rows

    rows = []
    for n in sizes:      # case 1.1, C_mnp = A_mk B_knp: flattened, batched in p, batched in n
        tA = dev(inputs.uniform_tensor(53, [n, n], np.float32), "f32")
        tB = dev(inputs.uniform_tensor(54, [n, n, n], np.float32), "f32")
        tC = torch.empty(n ** 3, dtype=torch.float32, device="cuda")
        row = dict(n=n)
        for name, (ma, mb, mc) in (("flat", ("mk", "k(np)", "m(np)")), ("batch_p", ("mk", "kn[p]", "mn[p]")),
                                   ("batch_n", ("mk", "k[n]p", "m[n]p"))):
            def ours():
                sb.sb_contract(ma, mb, mc, 1.0, tA, [n, n], tB, [n, n, n], 0.0, tC, [n, n, n])
            _, t = time_steps(ours, reps(n), warmup)
            row[name + "_us"] = t * 1e3
            row[name + "_gflops"] = 2 * n ** 4 / t / 1e6
        rows.append(row)
    out["case_1_1_flat_vs_batched"] = rows

    rows = []
    for n in sizes[2:]:  # exceptional case 6.4, C_mnp = B_nkm A_kp
        tA = dev(inputs.uniform_tensor(55, [n, n], np.float32), "f32")
        tB = dev(inputs.uniform_tensor(56, [n, n, n], np.float32), "f32")
        tC = torch.empty(n ** 3, dtype=torch.float32, device="cuda")
        row = dict(n=n)
        for name, strat in (("extended_op", "auto"), ("batched_gemv", "level2")):
            def ours():
                sb.sb_contract("kp", "nkm", "mnp", 1.0, tA, [n, n], tB, [n, n, n], 0.0, tC, [n, n, n], strat=strat)
            _, t = time_steps(ours, reps(n) if name == "extended_op" else max(3, steps // 4), min(warmup, 3))
            row[name + "_us"] = t * 1e3
        a, b = tA.view(n, n), tB.view(n, n, n)

        def conventional():
            return torch.einsum("pk,mkn->pnm", a, b).contiguous()

        _, t = time_steps(conventional, reps(n), warmup)
        row["transpose_gemm_us"] = t * 1e3
        row["extended_op_gflops"] = 2 * n ** 4 / row["extended_op_us"] / 1e3
        rows.append(row)
    out["case_6_4_exceptional"] = rows

    rows = []
    for n in sizes[2:] + [1024]:      # n matrix-vector products y_p = op(A_p) x_p with n x n matrices: level 2, HBM-bound
        tA = dev(inputs.uniform_tensor(57, [n, n, n], np.float32), "f32")
        tx = dev(inputs.uniform_tensor(58, [n, n], np.float32), "f32")
        ty = torch.empty(n * n, dtype=torch.float32, device="cuda")
        row = dict(n=n)
        nbytes = 4 * (n ** 3 + 2 * n * n)
        for name, op in (("gemv_n", "N"), ("gemv_t", "T")):
            def ours():
                sb.sb_gemm(op, "N", n, 1, n, 1.0, tA, n, n * n, tx, n, n, 0.0, ty, n, n, n, dt="f32")
            _, t = time_steps(ours, reps(n), warmup)
            row[name + "_us"] = t * 1e3
            row[name + "_gbps"] = nbytes / t / 1e6
            row[name + "_frac_of_hbm_peak"] = nbytes / t / 1e6 / PEAK["hbm"]
            row[name + "_kernel_family"] = sb.sb_last_kernel()
        a3, x3, y3 = tA.view(n, n, n), tx.view(n, 1, n), ty.view(n, 1, n)

        def vendor():      # row-major views: y_p^T = x_p^T A_p^T
            torch.bmm(x3, a3, out=y3)

        _, t = time_steps(vendor, reps(n), warmup)
        row["vendor_bmm_us"] = t * 1e3
        rows.append(row)
    out["batched_gemv_n_of_nxn"] = rows
    return out



def run_batched_gemv(steps, warmup, n=512):
    """n matrix-vector products y_p = op(A_p) x_p with n x n fp32 matrices, both layouts: the level-2 end
    of the primitive (thin kernels), bound by reading the matrices once."""
    import torch
    import paper_1606_05696_amd as sb
    from paper_1606_05696_amd import inputs
    tA = dev(inputs.uniform_tensor(57, [n, n, n], np.float32), "f32")
    tx = dev(inputs.uniform_tensor(58, [n, n], np.float32), "f32")
    ty = torch.empty(n * n, dtype=torch.float32, device="cuda")
    nbytes = 4 * (n ** 3 + 2 * n * n)
    out = dict(workload="%d matrix-vector products of %d x %d, f32: y_[p] = op(A_[p]) x_[p]" % (n, n, n), short="gemv",
               algorithmic_bytes=nbytes, cases=[])
    for op in ("N", "T"):
        def ours():
            sb.sb_gemm(op, "N", n, 1, n, 1.0, tA, n, n * n, tx, n, n, 0.0, ty, n, n, n, dt="f32")
        st = time_stats(ours, iters=max(30, steps), warmup=warmup)
        t = st["median_us"] / 1e3
        out["cases"].append(dict(op=op, kernel_family=sb.sb_last_kernel(), us=st["median_us"], kernel_us=st, gbps=nbytes / t / 1e6,
                                 frac_of_hbm_peak=nbytes / t / 1e6 / PEAK["hbm"]))
    return out


def run_tucker(sizes=(128, 512), core=10, iterations=20, oracle_n=128, with_oracle=True):
    """The application study of section IV-C: HOOI (Algorithm 1) on cubic n^3 tensors with a 10^3 core,
    fp32, every contraction through sb_contract.  Reports time per iteration (steps 4-9: five
    contractions and three Gram / eigensolver / back-multiplication rounds), the one-off
    initialisation (step 2) and, at one size, the numpy oracle's time per iteration on the host."""
    import torch
    import paper_1606_05696_amd as sb
    from paper_1606_05696_amd import inputs
    rows = []
    for n in sizes:
        T = inputs.lowrank_noise_tensor(61, [n, n, n], (core,) * 3, noise=0.05, dtype=np.float32)
        tT = dev(T, "f32")
        fac = [torch.zeros(n * core, dtype=torch.float32, device="cuda") for _ in range(3)]
        tG = torch.zeros(core ** 3, dtype=torch.float32, device="cuda")
        ws = torch.empty(sb.sb_tucker_workspace("f32", n, n, n, core, core, core)[1], dtype=torch.uint8, device="cuda")

        def run(its, init):
            sb.sb_tucker_hooi(tT, (n, n, n), (core,) * 3, its, fac[0], fac[1], fac[2], tG, ws, init=init, dt="f32")

        run(2, True)                                   # warm-up (first-use set-up of every kernel)
        _, t_init = time_steps(lambda: run(0, True), 3, 1)
        _, t_loop = time_steps(lambda: run(iterations, False), 3, 1)
        _, t_tail = time_steps(lambda: run(0, False), 3, 1)      # step 11 alone
        row = dict(n=n, core=core, iterations_timed=iterations, ms_per_iteration=(t_loop - t_tail) / iterations,
                   init_ms=t_init - t_tail, core_ms=t_tail,
                   fit=float(torch.linalg.vector_norm(tG) / torch.linalg.vector_norm(tT)))
        if with_oracle and n == oracle_n:
            from oracle import tucker_oracle
            T64 = T.astype(np.float64)
            start = tucker_oracle.hosvd_init(T64, (core,) * 3)
            t0 = time.perf_counter()
            tucker_oracle.hooi(T64, (core,) * 3, 1, init=start)
            row["cpu_oracle_ms_per_iteration"] = (time.perf_counter() - t0) * 1e3
        rows.append(row)
        del tT, ws
    return dict(workload="Tucker/HOOI (Algorithm 1): cubic tensors, core %d^3, f32" % core, cases=rows)



def cpu_baseline(cfg, tensors, budget_s=12.0):
    """Time the CPU oracle, as it stands, on a bounded sample of the workload: the leading part of the
    last mode of C (a whole number of slices), sized from a two-slice probe to take about budget_s with
    every core; then once more with ONE thread on a sample a tenth of that time long (the paper's CPU
    figures are serial)."""
    import ctypes
    from oracle import oracle
    from paper_1606_05696_amd import inputs
    w = inputs.WORKLOADS[cfg]
    A, B = tensors
    wide = w["dtype"] == "f64"
    last = w["C"][-1]
    ext = w["ext"]
    in_a = last in w["A"]

    def run(nslices):
        sl = lambda X, modes: X[tuple(slice(0, nslices) if c == last else slice(None) for c in modes)]
        As = np.asfortranarray(sl(A, w["A"])) if in_a else A
        Bs = B if in_a else np.asfortranarray(sl(B, w["B"]))
        t0 = time.perf_counter()
        oracle.contract(w["A"], As, w["B"], Bs, w["C"], wide=wide)
        return time.perf_counter() - t0

    flops_per_slice = workload_numbers(w)[0] / ext[last]
    probe = min(2, ext[last])
    t_probe = run(probe)
    n = int(max(probe, min(ext[last], budget_s / max(t_probe / probe, 1e-9))))
    t = run(n) if n > probe else t_probe
    threads = int(os.environ.get("OMP_NUM_THREADS", os.cpu_count() or 1))
    acc = "long double" if wide else "double"
    out = dict(value=flops_per_slice * n / t / 1e9, unit="GFLOP/s", cores=threads, kind="oracle",
               sample="%d of %d slices of mode %s of C (%.3g GFLOP in %.2f s, %s accumulation)"
                      % (n, ext[last], last, flops_per_slice * n / 1e9, t, acc))
    try:        # the oracle's loops are OpenMP-parallel: one thread through the OpenMP runtime it is linked to
        omp = ctypes.CDLL("libgomp.so.1")
        omp.omp_set_num_threads(1)
        n1 = int(max(1, min(ext[last], round(4.0 * n / max(t * threads, 1e-9)))))      # about four seconds of one core
        t1 = run(n1)
        omp.omp_set_num_threads(threads)
        out["one_thread"] = dict(value=flops_per_slice * n1 / t1 / 1e9, unit="GFLOP/s", cores=1,
                                 sample="%d slices (%.3g GFLOP in %.2f s)" % (n1, flops_per_slice * n1 / 1e9, t1))
    except OSError:
        out["one_thread"] = None
    return out


def config_rows(head, others):
    """The compact per-configuration table under "roofline": one row per benchmark configuration (and per
    evaluation of cfg5), kernel time as the median of the timed iterations."""
    rows = []
    for r in [head] + [o for o in others if "roofline" in o]:
        rf = roofline_of(r["roofline"]["bound"], r["dtype"], r["flops"], r["bytes"], r["kernel_us"]["median_us"])
        row = dict(config=r["short"], kernel_family=r["kernel_family"], kernel_us=r["kernel_us"]["median_us"], min_us=r["kernel_us"]["min_us"],
                   max_us=r["kernel_us"]["max_us"], bound=rf["bound"], achieved=rf["achieved"], unit=rf["unit"], frac=rf["frac"],
                   cold_frac=r.get("cold_cache", {}).get("frac"), traffic=r["roofline"].get("traffic"),
                   algorithmic_bytes=r["bytes"], check_ok=r["check"]["ok"])
        rows.append(row)
        for e in r.get("evaluations", []):
            rows.append(dict(config="%s %s" % (r["short"], e["name"]), kernel_family=e["kernel_family"], kernel_us=e["kernel_us"]["median_us"],
                             min_us=e["kernel_us"]["min_us"], max_us=e["kernel_us"]["max_us"], bound=rf["bound"], achieved=e["achieved"],
                             unit=e["unit"], frac=e["frac"], cold_frac=None, traffic=None, algorithmic_bytes=r["bytes"], check_ok=e["check_ok"]))
    for o in others:
        if o.get("short") == "cfg2":
            rows.append(dict(config="cfg2 (36 cases, per call)", kernel_family=None, kernel_us=o["median_us_per_call"], min_us=None,
                             max_us=o["max_us_per_call"], bound="launch", achieved=None, unit=None, frac=None, cold_frac=None,
                             traffic=None, algorithmic_bytes=2113536, check_ok=o["all_outputs_ok"]))
        elif o.get("short") == "ext-op":
            for c in o["cases"]:
                rows.append(dict(config="ext-op case %s 512^4%s" % (c["case"], "" if c["dtype"] == "f32" else " " + c["dtype"]),
                                 kernel_family=c["kernel_family"], kernel_us=c["kernel_us"]["median_us"],
                                 min_us=c["kernel_us"]["min_us"], max_us=c["kernel_us"]["max_us"], bound="mfma", achieved=c["gflops"] / 1e3,
                                 unit="TFLOP/s", frac=c["frac_of_mfma_peak"], cold_frac=None, traffic=None,
                                 algorithmic_bytes=ESIZE[c["dtype"]] * (512 ** 2 + 2 * 512 ** 3), check_ok=c["check_ok"]))
        elif o.get("short") == "bf16-gemm":
            for c in o["cases"]:
                rows.append(dict(config="bf16 %s %d^3 x %d" % (c["layout"], c["n"], c["batch"]), kernel_family=c["kernel_family"],
                                 kernel_us=c["kernel_us"]["median_us"], min_us=c["kernel_us"]["min_us"], max_us=c["kernel_us"]["max_us"], bound="mfma",
                                 achieved=c["tflops"], unit="TFLOP/s", frac=c["frac_of_bf16_mfma_peak"], cold_frac=None, traffic=None,
                                 algorithmic_bytes=2 * 3 * c["n"] ** 2 * c["batch"], check_ok=c["check_ok"]))
        elif o.get("short") == "gemv":
            for c in o["cases"]:
                rows.append(dict(config="gemv %s 512 x 512^2" % c["op"], kernel_family=c["kernel_family"], kernel_us=c["kernel_us"]["median_us"],
                                 min_us=c["kernel_us"]["min_us"], max_us=c["kernel_us"]["max_us"], bound="hbm", achieved=c["gbps"], unit="GB/s",
                                 frac=c["frac_of_hbm_peak"], cold_frac=None, traffic=None, algorithmic_bytes=o["algorithmic_bytes"], check_ok=None))
    return rows


def sweeps_text(sw):
    """The size sweeps as a plain text table (kept under profiles/ as sweeps_summary.txt)."""
    out = ["Size sweeps over cubic fp32 tensors (the shapes of the paper's GPU plots, section IV), one MI355X.",
           "command: python3 bench.py --sweeps --no-cpu-baseline --no-tucker --sweeps-summary <this file>",
           "times are microseconds per call (HIP events around back-to-back calls); kf = kernel family", ""]
    for name, rows in sw.items():
        keys = list(rows[0].keys())
        out.append(name)
        out.append("  " + " ".join("%22s" % k for k in keys))
        for r in rows:
            out.append("  " + " ".join("%22s" % (("%.2f" % r[k]) if isinstance(r[k], float) else r[k]) for k in keys))
        out.append("")
    return "\n".join(out)


def main():
    args = parse_args()
    if args.gpus != 1:
        print("bench.py measures one GPU: the contraction path has no multi-GPU part (every box here has "
              "one GPU); run with --gpus 1", file=sys.stderr)
        sys.exit(2)
    import torch
    import paper_1606_05696_amd as sb
    from paper_1606_05696_amd import inputs
    sb.binding.load()
    torch.cuda.set_device(0)

    if args.calibrate_copy:
        src = torch.empty(1 << 28, dtype=torch.float32, device="cuda").fill_(1.0)     # 1 GiB
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    traffic = measured_traffic()
    tb = not args.no_torch_baseline
    cfg5_forms = [("flat (mp)(nq)", ("(mp)k", "k(nq)", "(mp)(nq)")), ("(mp)n[q]", ("(mp)k", "kn[q]", "(mp)n[q]")),
                  ("m[p](nq)", ("m[p]k", "k(nq)", "m[p](nq)"))]
    cfg4_forms = [("batched in n", ("km", "k[n]p", "m[n]p")), ("flat m(np)", ("km", "k(np)", "m(np)"))]
    forms = {5: cfg5_forms, 41: cfg4_forms}
    # what the box itself sustains (pure-MFMA kernels, a 1 GiB copy) is measured first: these run the chip for
    # some tens of milliseconds, so the headline's few warm-up steps do not start from idle clocks
    peaks = measured_peaks(sorted({v["dtype"] for v in inputs.WORKLOADS.values()}))
    head, tensors = run_workload(args.workload, args.steps, args.warmup, traffic, tb, forms.get(args.workload), prewarm_ms=args.prewarm_ms)
    w = inputs.WORKLOADS[args.workload]
    roof = head["roofline"]
    measured = peaks["mfma_%s_tflops" % w["dtype"]] if roof["bound"] == "mfma" else peaks["hbm_copy_gbps"]
    roof["measured_peak"] = measured
    roof["frac_of_measured"] = roof["achieved"] / measured
    roof["traffic_source"] = "%s (rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE, offline, commit %s)" % (traffic["source"], traffic["commit"])
    roof["kernel_us"] = head["kernel_us"]
    result = {
        "metric": "GFLOP/s per contraction (StridedBatchedGemm path), 1 GPU",
        "value": head["gflops"], "unit": "GFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": head["ms_per_step"], "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": w["dtype"], "data": "synthetic",
        "config": {"workload": w["name"], "evaluation": head["evaluation"], "kernel_family": head["kernel_family"],
                   "flops_per_step": head["flops"], "algorithmic_bytes_per_step": head["bytes"], "output_check": head["check"],
                   "device_prewarm_ms": args.prewarm_ms},
        "roofline": roof,
    }
    result["measured_peaks"] = peaks
    result["baselines"] = {"conventional_same_gpu_own_kernels": head["conventional_own"]}
    if tb:
        result["baselines"]["conventional_same_gpu"] = head["torch_matmul"]
    if not args.no_cpu_baseline:
        result["cpu_baseline"] = cpu_baseline(args.workload, tensors)
    del tensors
    others = []
    if args.sweeps:
        result["sweeps"] = run_sweeps(args.steps, args.warmup)
        if args.sweeps_summary:
            with open(args.sweeps_summary, "w") as f:
                f.write(sweeps_text(result["sweeps"]))
    elif not args.only_headline:
        for cfg in inputs.WORKLOADS:
            if cfg == args.workload:
                continue
            steps = args.steps if cfg in (40, 41) else max(args.steps, 200)
            r, _ = run_workload(cfg, steps, args.warmup, traffic, tb, forms.get(cfg))
            others.append(r)
        others.append(run_table2_cases(max(args.steps, 200), args.warmup, tb))
        others.append(run_exceptional_cases(args.steps, args.warmup, torch_baseline=tb))
        others.append(run_batched_gemv(args.steps, args.warmup))
        if not args.no_bf16_family:
            others.append(run_bf16_family(tb))
        if not args.no_tucker:
            others.append(run_tucker(with_oracle=not args.no_cpu_baseline))
        result["workloads"] = others
    roof["configs"] = config_rows(head, others)
    print(json.dumps(result))


if __name__ == "__main__":
    main()
