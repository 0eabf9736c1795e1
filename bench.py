#!/usr/bin/env python3
"""Benchmark of the contraction hot path on one MI355X.

A "step" is one pass of the whole path for one contraction: sb_contract() parses the mode strings,
plans the evaluation, selects a kernel and launches it on tensors that are already resident in
HBM.  The headline workload is the large cube C_mnp = sum_k A_km B_knp at 512^4 in fp32 evaluated
as one StridedBatchedGemm over p; the other benchmark contractions are timed too and reported in
the same JSON line under "workloads".

Prints ONE JSON line: metric / value (GFLOP/s) / ms_per_step ..., plus
  "roofline":     achieved vs peak for the dominant kernel (HIP events on the launch stream),
  "cpu_baseline": the CPU oracle timed on the host cores on a bounded sample of the same workload,
  "baselines":    the conventional evaluation on the same GPU (torch permute/copy + vendor GEMM).
"""
import argparse
import json
import os
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
# which roofline binds each workload: dense high-intensity contractions are priced against the
# matrix cores, the batch-dominated / output-dominated ones against HBM
BOUND = {1: "hbm", 3: "hbm", 40: "mfma", 41: "mfma", 5: "hbm"}
# HBM-side bytes per launch from rocprofv3 --pmc FETCH_SIZE + WRITE_SIZE, scaled by the same counters'
# readings for a 1 GiB copy (profiles/bench_default_hbm_traffic.txt); measured offline, not in this run
MIB = 1 << 20
MEASURED_TRAFFIC = {41: int(1127.02 * MIB), 40: int(2564.64 * MIB), 3: int(128.14 * MIB), 5: int(41.29 * MIB),
                    1: int(0.65 * MIB)}


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=30)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--workload", type=int, default=41, help="headline workload id (inputs.WORKLOADS)")
    ap.add_argument("--only-headline", action="store_true", help="skip the other workloads")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-torch-baseline", action="store_true")
    ap.add_argument("--sweeps", action="store_true",
                    help="instead of the other workloads, add the size sweeps (cubic tensors, n = 8 .. 512) to the line")
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


def workload_numbers(w):
    ext = w["ext"]
    strip = lambda s: "".join(c for c in s if c.isalpha())
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


LLC_BYTES = 256 << 20      # Infinity Cache: working sets below this can be served without touching HBM


def run_workload(cfg, steps, warmup, torch_baseline=True):
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

    ms, kernel_ms = time_steps(step, steps, warmup)
    kernel = sb.sb_last_kernel()
    out = dict(workload=w["name"], dtype=dtype, evaluation=plan.text(), kernel_family=kernel,
               ms_per_step=ms, kernel_ms=kernel_ms, gflops=flops / ms / 1e6, flops=flops, bytes=nbytes)
    bound = BOUND[cfg]
    if bound == "mfma":
        ach, peak, unit = flops / kernel_ms / 1e9, PEAK["mfma"][dtype], "TFLOP/s"
    else:
        ach, peak, unit = nbytes / kernel_ms / 1e6, PEAK["hbm"], "GB/s"
    out["roofline"] = dict(bound=bound, achieved=ach, peak=peak, unit=unit, frac=ach / peak,
                           traffic=MEASURED_TRAFFIC.get(cfg))
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
    if torch_baseline:
        out["torch_matmul"] = conventional_baseline(cfg, tA, tB, dA, dB, dC, steps, warmup, flops)
    del tA, tB, tC
    torch.cuda.empty_cache()
    return out, (A, B)


def conventional_baseline(cfg, tA, tB, dA, dB, dC, steps, warmup, flops):
    """The conventional evaluation on the same GPU: bring the operands into matricised form
    (explicit permute + copy where the layout needs one) and call the vendor GEMM through torch.
    A column-major tensor with extents (d0, d1, ..) is a row-major torch tensor of shape (.., d1, d0)."""
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


def run_table2_cases(steps, warmup):
    """cfg2: every order-2 x order-3 single-mode contraction (Table II) at extent 64, fp32, in the
    evaluation SB_AUTO picks, against the conventional route (explicit permute/copy + vendor GEMM).
    These calls are launch-bound: the figure of merit is time per call, back to back."""
    import itertools
    import torch
    import paper_1606_05696_amd as sb
    from paper_1606_05696_amd import inputs
    n = 64
    rows = []
    tC = torch.empty(n ** 3, dtype=torch.float32, device="cuda")
    for free_a in "mnp":
        rest = [c for c in "mnp" if c != free_a]
        for ma in (free_a + "k", "k" + free_a):
            for perm in itertools.permutations(["k"] + rest):
                mb = "".join(perm)
                tA = dev(inputs.uniform_tensor(21, [n, n], np.float32), "f32")
                tB = dev(inputs.uniform_tensor(22, [n, n, n], np.float32), "f32")
                rc, plan = sb.sb_contract_plan(ma, mb, "mnp", [n, n], [n, n, n])

                def ours():
                    sb.sb_contract(ma, mb, "mnp", 1.0, tA, [n, n], tB, [n, n, n], 0.0, tC, [n, n, n])

                a, b = tA.view(n, n), tB.view(n, n, n)
                expr = "%s,%s->pnm" % (ma[::-1], mb[::-1])

                def conventional():
                    return torch.einsum(expr, a, b).contiguous()

                _, t_ours = time_steps(ours, steps, warmup)
                _, t_conv = time_steps(conventional, steps, warmup)
                rows.append(dict(A=ma, B=mb, evaluation=plan.text(), exceptional=int(plan.exceptional),
                                 us_per_call=t_ours * 1e3, conventional_us_per_call=t_conv * 1e3))
    flops = 2 * n ** 4
    ours = np.array([r["us_per_call"] for r in rows])
    conv = np.array([r["conventional_us_per_call"] for r in rows])
    return dict(workload="cfg2: all 36 order-2 x order-3 contractions at 64^4, f32, SB_AUTO evaluation",
                calls_timed_per_case=steps, mean_us_per_call=float(ours.mean()), max_us_per_call=float(ours.max()),
                mean_gflops=float(flops / ours.mean() / 1e3),
                conventional_mean_us_per_call=float(conv.mean()),
                speedup_over_conventional_mean=float((conv / ours).mean()),
                speedup_over_conventional_min=float((conv / ours).min()),
                speedup_over_conventional_max=float((conv / ours).max()),
                cases=rows)


def run_exceptional_cases(steps, warmup, n=512):
    """Two exceptional cases of Table II (3.6 and 6.4, the ones section III-E writes out) at n^4 in
    fp32: the extended-operation kernel against the two-step route the paper benchmarks it against
    (explicit mode transposition + GEMM, here torch permute/copy + vendor GEMM)."""
    import torch
    import paper_1606_05696_amd as sb
    from paper_1606_05696_amd import inputs
    rows = []
    tA = dev(inputs.uniform_tensor(31, [n, n], np.float32), "f32")
    tB = dev(inputs.uniform_tensor(32, [n, n, n], np.float32), "f32")
    tC = torch.empty(n ** 3, dtype=torch.float32, device="cuda")
    flops = 2 * n ** 4
    for case, ma, mb in (("3.6", "nk", "pmk"), ("6.4", "kp", "nkm")):
        rc, plan = sb.sb_contract_plan(ma, mb, "mnp", [n, n], [n, n, n])

        def ours():
            sb.sb_contract(ma, mb, "mnp", 1.0, tA, [n, n], tB, [n, n, n], 0.0, tC, [n, n, n])

        a, b = tA.view(n, n), tB.view(n, n, n)
        expr = "%s,%s->pnm" % (ma[::-1], mb[::-1])

        def conventional():
            return torch.einsum(expr, a, b).contiguous()

        _, t_ours = time_steps(ours, steps, warmup)
        family = sb.sb_last_kernel()
        _, t_conv = time_steps(conventional, steps, warmup)
        rows.append(dict(case=case, evaluation=plan.text(), kernel_family=family, kernel_ms=t_ours,
                         gflops=flops / t_ours / 1e6, frac_of_fp32_mfma_peak=flops / t_ours / 1e9 / PEAK["mfma"]["f32"],
                         conventional_ms=t_conv, speedup_over_conventional=t_conv / t_ours))
    return dict(workload="exceptional cases 3.6 and 6.4 at %d^4, f32: extended-operation kernel" % n, cases=rows)


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
    out = dict(workload="%d matrix-vector products of %d x %d, f32: y_[p] = op(A_[p]) x_[p]" % (n, n, n),
               algorithmic_bytes=nbytes, cases=[])
    for op in ("N", "T"):
        def ours():
            sb.sb_gemm(op, "N", n, 1, n, 1.0, tA, n, n * n, tx, n, n, 0.0, ty, n, n, n, dt="f32")
        _, t = time_steps(ours, max(steps, 100), warmup)
        out["cases"].append(dict(op=op, kernel_family=sb.sb_last_kernel(), us=t * 1e3, gbps=nbytes / t / 1e6,
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
    last mode of C (a whole number of slices), sized from a two-slice probe to take about budget_s."""
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
    return dict(value=flops_per_slice * n / t / 1e9, unit="GFLOP/s", cores=threads, kind="oracle",
                sample="%d of %d slices of mode %s of C (%.3g GFLOP in %.2f s, %s accumulation)"
                       % (n, ext[last], last, flops_per_slice * n / 1e9, t, "long double" if wide else "double"))


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

    head, tensors = run_workload(args.workload, args.steps, args.warmup, not args.no_torch_baseline)
    w = inputs.WORKLOADS[args.workload]
    peaks = measured_peaks(sorted({v["dtype"] for v in inputs.WORKLOADS.values()}))
    measured = peaks["mfma_%s_tflops" % w["dtype"]] if head["roofline"]["bound"] == "mfma" else peaks["hbm_copy_gbps"]
    head["roofline"]["measured_peak"] = measured
    head["roofline"]["frac_of_measured"] = head["roofline"]["achieved"] / measured
    result = {
        "metric": "GFLOP/s per contraction (StridedBatchedGemm path), 1 GPU",
        "value": head["gflops"], "unit": "GFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": head["ms_per_step"], "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": w["dtype"], "data": "synthetic",
        "config": {"workload": w["name"], "evaluation": head["evaluation"], "kernel_family": head["kernel_family"],
                   "flops_per_step": head["flops"], "algorithmic_bytes_per_step": head["bytes"]},
        "roofline": head["roofline"],
    }
    result["measured_peaks"] = peaks
    if not args.no_torch_baseline:
        result["baselines"] = {"conventional_same_gpu": head["torch_matmul"]}
    if not args.no_cpu_baseline:
        result["cpu_baseline"] = cpu_baseline(args.workload, tensors)
    del tensors
    if args.sweeps:
        result["sweeps"] = run_sweeps(args.steps, args.warmup)
    elif not args.only_headline:
        others = []
        for cfg in inputs.WORKLOADS:
            if cfg == args.workload:
                continue
            steps = args.steps if cfg in (40, 41) else max(args.steps, 200)
            r, _ = run_workload(cfg, steps, args.warmup, not args.no_torch_baseline)
            others.append(r)
        others.append(run_table2_cases(max(args.steps, 200), args.warmup))
        others.append(run_exceptional_cases(args.steps, args.warmup))
        others.append(run_batched_gemv(args.steps, args.warmup))
        if not args.no_tucker:
            others.append(run_tucker(with_oracle=not args.no_cpu_baseline))
        result["workloads"] = others
    print(json.dumps(result))


if __name__ == "__main__":
    main()
