#!/usr/bin/env python3
"""Benchmark of the compression hot path (all three mode contractions for all replicas) on one MI355X.

One "step" = one full pass Y_p = X x1 U_p x2 V_p x3 W_p, p = 0..P-1, over one synthetic tensor of the
chosen configuration, inputs resident in HBM (or generated on chip) when the timed region starts.
Prints ONE JSON line: whole-job throughput in input elements/s, the roofline of the dominant kernel
(fused mode-1/2, MFMA-bound) measured live with HIP events, and the CPU oracle timed on a bounded sample.
"""
import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_TFLOPS = {"f32": 157.3, "bf16": 2500.0}   # MI355X dense MFMA peaks


def recorded_traffic(tag):
    """HBM-side bytes of one launch of the dominant kernel of workload `tag`, from the rocprofv3 --pmc FETCH_SIZE /
    WRITE_SIZE passes summarised in profiles/*_<tag>_hbm_counters.txt (their line "traffic_bytes_per_launch = N":
    both counters scaled by what they read on a plain device copy of known size).  Counter passes are separate runs,
    so this is the recorded figure of the same command, not one measured by this script; None when no summary exists."""
    import glob
    import re
    for path in sorted(glob.glob(os.path.join(ROOT, "profiles", "*_%s_hbm_counters.txt" % tag))):
        m = re.search(r"^traffic_bytes_per_launch\s*=\s*([0-9.eE+]+)", open(path).read(), re.M)
        if m:
            return float(m.group(1))
    return None


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=None)
    ap.add_argument("--warmup", type=int, default=None)
    ap.add_argument("--config", default=os.environ.get("EXAT_BENCH_CONFIG", "cfg5"),
                    help="cfg1..cfg5 (default cfg5: the 1e12-element bf16 configuration generated on chip, the one the "
                         "target of the task is stated on; one step = one pass over the whole tensor)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--calib-copy", action="store_true",
                    help="after the timed region, run one plain 256 MiB device copy (a kernel of known traffic "
                         "that calibrates the FETCH_SIZE / WRITE_SIZE counters in a rocprofv3 --pmc run)")
    ap.add_argument("--kslices", type=int, default=0,
                    help="development aid: compress only the first N frontal slices (generated configs); "
                         "the reported numbers then refer to that sub-box, not to the configuration")
    ap.add_argument("--blocks", action="store_true",
                    help="materialised configurations only: the block-streamed form of Sec. 4.3 (every dI x dJ x dK block, "
                         "resident in HBM as its own array, through exat_compress_block, then exat_finalize) instead of the "
                         "one-shot call on the whole tensor; the algorithmic flops stay those of the three modes once each, "
                         "so the per-block repetition of modes 2 and 3 shows up as a lower fraction")
    ap.add_argument("--slab", type=int, default=0,
                    help="with --blocks: compress the blocks in slabs of this many block layers along k per call "
                         "(exat_compress_blocks; all blocks of a slab resident at once) instead of one call per block")
    ap.add_argument("--mfma-ceiling", action="store_true",
                    help="measure what the matrix cores of this GPU sustain when a kernel issues nothing but MFMAs "
                         "(exat_probe_mfma: bf16 32x32x16 and fp32 32x32x2, constant and random operands) and print it")
    ap.add_argument("--split", action="store_true",
                    help="fp32 materialised configurations only: run the contractions on the fp16 matrix cores with "
                         "two-piece operands (EXAT_F32_SPLIT) instead of fp32 MFMA; reported against the fp16 MFMA peak")
    ap.add_argument("--two-stage", action="store_true",
                    help="fp32 materialised configurations only: the two-stage compression of Sec. 4.4 (sparse first "
                         "stage to 2L x 2M x 2N with 4 entries per column, then the dense replicas on its output); the "
                         "roofline object then describes the HBM-bound first-stage kernel")
    ap.add_argument("--cpals", action="store_true",
                    help="the decomposition stage on the configuration's proxy tensors: 10 sweeps of batched CP-ALS (Alg. 1) "
                         "over the P tensors of L x M x N that the compression of the same synthetic tensor produced (fp32 "
                         "materialised configurations); value then counts proxy-tensor elements swept per second")
    ap.add_argument("--ls", action="store_true",
                    help="the join of the replicas: the stacked least-squares solves of Eq. 4 for the three modes, on the "
                         "configuration's own stacked compression matrices (needs P*L >= 1.5 I: cfg3); value then counts "
                         "matrix elements streamed per second (two passes over the stacked matrix per iteration)")
    return ap.parse_args()


def mfma_ceiling(args):
    """The MFMA-only rate of this machine: the ceiling of any kernel here, next to the published peak."""
    import torch
    from paper_2311_13693_amd import exat
    torch.cuda.set_device(0)
    torch.zeros(1, device="cuda")            # the device is initialised through torch, as everywhere in this file
    out = {"metric": "MFMA-only rate of this GPU (measurement aid: no compression work)", "unit": "TFLOP/s", "n_gpus": 1,
           "workgroups": 256, "waves_per_workgroup": 8, "rates": {}}
    # about 100 ms per launch: 64 MFMAs per iteration and wave, two waves per SIMD
    for name, kind, iters, peak in (("bf16_32x32x16", 0, 40000, PEAK_TFLOPS["bf16"]), ("f32_32x32x2", 1, 20000, PEAK_TFLOPS["f32"])):
        for operands in ("constant", "random"):
            tf, ghz = exat.probe_mfma(kind, operands == "random", iters, 256)
            out["rates"]["%s, %s operands" % (name, operands)] = {"tflops": tf, "core_ghz": ghz, "published_peak": peak, "frac": tf / peak}
    print(json.dumps(out))


def cpals(args):
    """One step = `SWEEPS` sweeps of Alg. 1 over all P proxy tensors (the output of one compression pass)."""
    import torch
    from paper_2311_13693_amd import exat
    import workloads as wl
    SWEEPS = 10
    cfg = wl.CONFIGS[args.config]
    assert cfg.materialised and cfg.dtype == "f32", "--cpals needs a materialised fp32 configuration"
    steps = args.steps if args.steps is not None else 50
    warmup = args.warmup if args.warmup is not None else 50      # warm up for ~50 ms of load: the chip's clock settles under load
    torch.cuda.set_device(0)
    A, B, C = wl.cp_factors(cfg)
    U, V, W = wl.compression_matrices(cfg)
    dev = lambda a: torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).cuda()
    gen = exat.make_gen(dev(A.T), dev(B.T), dev(C.T), cfg.seed, cfg.sigma)
    plan = exat.Plan(exat.make_desc(cfg.I, cfg.J, cfg.K, cfg.L, cfg.M, cfg.N, cfg.P, cfg.dI, cfg.dJ, cfg.dK, exat.EXAT_F32))
    plan.set_factors(dev(U), dev(V), dev(W))
    whole = exat.make_desc(cfg.I, cfg.J, cfg.K, cfg.L, cfg.M, cfg.N, cfg.P, cfg.I, cfg.J, cfg.K, exat.EXAT_F32)
    X = torch.empty(cfg.elements, dtype=torch.float32, device="cuda")
    exat.gen_block(whole, gen, 0, 0, 0, X)
    Y = plan.compress(X)                      # the proxy tensors: input of the timed region, resident in HBM
    torch.cuda.synchronize()
    del X
    L, M, N, P, R = cfg.L, cfg.M, cfg.N, cfg.P, cfg.R
    rng = np.random.default_rng(cfg.seed & 0xFFFFFFFF)
    start = [rng.standard_normal((P, R, d)).astype(np.float32) for d in (L, M, N)]   # [p][r][d] = column-major d x R
    S = [torch.from_numpy(s).cuda() for s in start]
    F = [s.clone() for s in S]
    work = torch.empty(exat.lib().exat_cpals_workspace_floats(L, M, N, P), dtype=torch.float32, device="cuda")

    def step():
        for f, s in zip(F, S):
            f.copy_(s)
        exat.cpals(Y, L, M, N, P, R, SWEEPS, F[0], F[1], F[2], work)
    for _ in range(warmup):
        step()
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    ks, ke = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    kms = []
    e0.record()
    for _ in range(steps):
        for f, s in zip(F, S):
            f.copy_(s)
        ks.record()                           # the library's kernels run on torch's current stream
        exat.cpals(Y, L, M, N, P, R, SWEEPS, F[0], F[1], F[2], work)
        ke.record()
        ke.synchronize()
        kms.append(ks.elapsed_time(ke))
    e1.record()
    torch.cuda.synchronize()
    ms_step, ms_k = e0.elapsed_time(e1) / steps, float(np.mean(kms))
    flops = 3 * 2.0 * L * M * N * R * P * SWEEPS          # the three MTTKRPs of a sweep, factored form
    achieved = flops / (ms_k * 1e-3) / 1e12
    out = {
        "metric": "input tensor elements compressed/sec + TTM TFLOP/s (% MFMA peak), 1 MI355X",
        "value": P * L * M * N * SWEEPS / (ms_step * 1e-3), "unit": "elements/s",
        "n_gpus": 1, "steps": steps, "warmup": warmup, "ms_per_step": ms_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": "%s decomposition stage: %d sweeps of CP-ALS (rank %d) over the %d proxy tensors of %dx%dx%d; "
                               "elements = proxy-tensor elements x sweeps" % (cfg.name, SWEEPS, R, P, L, M, N)},
        "kernel_ms": {"all_launches": ms_k, "per_sweep": ms_k / SWEEPS},
        "roofline": {"bound": "alu", "kernel": "k_cpals_mttkrp + k_cpals_solve", "achieved": achieved, "peak": 157.3, "unit": "TFLOP/s",
                     "frac": achieved / 157.3, "traffic": None},
    }
    Yh = Y.cpu().numpy().reshape((L, M, N, P), order="F")
    if not args.no_cpu_baseline:
        import oracle
        from threadpoolctl import threadpool_info
        nrep = min(P, 4)
        t0 = time.perf_counter()
        for p in range(nrep):
            oracle.cp_als(Yh[..., p], start[0][p].T, start[1][p].T, start[2][p].T, SWEEPS)
        t = (time.perf_counter() - t0) * P / nrep
        cores = max([int(lib.get("num_threads", 1)) for lib in threadpool_info()] + [1])
        out["cpu_baseline"] = {"value": P * L * M * N * SWEEPS / t, "unit": "elements/s", "cores": cores, "kind": "oracle",
                               "sample": "replicas 0..%d of %d, %d sweeps each (numpy fp64), scaled to all replicas" % (nrep - 1, P, SWEEPS),
                               "seconds_full": t, "extrapolated": nrep < P}
    plan.close()
    print(json.dumps(out))


def ls(args):
    """One step = the three stacked least-squares solves (Eq. 4) that join the replicas' factors, one per mode."""
    import torch
    from paper_2311_13693_amd import exat
    import workloads as wl
    ITERS, TOL = 40, 1e-6
    cfg = wl.CONFIGS[args.config]
    if 2 * cfg.P * cfg.L < 3 * cfg.I:
        print("bench.py --ls: %s stacks %d rows for %d unknowns; the fp32 iteration needs P*L >= 1.5 I (use cfg3)"
              % (cfg.name, cfg.P * cfg.L, cfg.I), file=sys.stderr)
        sys.exit(2)
    steps = args.steps if args.steps is not None else 30
    warmup = args.warmup if args.warmup is not None else 30
    torch.cuda.set_device(0)
    P, R = cfg.P, cfg.R
    dims = ((cfg.L, cfg.I), (cfg.M, cfg.J), (cfg.N, cfg.K))
    rng = np.random.default_rng(cfg.seed & 0xFFFFFFFF)
    mats, stacks, hosts = [], [], []
    for Uh, Fh, (Ld, Id) in zip(wl.compression_matrices(cfg), wl.cp_factors(cfg), dims):
        # replica factors U_p A (the Kronecker property) plus estimation noise, in the layout the CP-ALS writes
        Ah = Uh.astype(np.float64) @ Fh.astype(np.float64)
        Ah = (Ah + 0.05 * np.abs(Ah).mean() * rng.standard_normal(Ah.shape)).astype(np.float32)
        flat = np.concatenate([Ah[p * Ld:(p + 1) * Ld].reshape(-1, order="F") for p in range(P)])
        mats.append(torch.from_numpy(np.ascontiguousarray(Uh, dtype=np.float32)).cuda())
        stacks.append(torch.from_numpy(flat).cuda())
        hosts.append((Uh, Ah))
    Xs = [torch.empty(Id * R, dtype=torch.float32, device="cuda") for _, Id in dims]
    rel = [torch.empty(R, dtype=torch.float32, device="cuda") for _ in dims]
    works = [torch.empty(exat.lib().exat_ls_workspace_floats(P, Ld, Id, R), dtype=torch.float32, device="cuda") for Ld, Id in dims]

    def step():
        for (Ld, Id), Ud, Ad, Xd, rd, wk in zip(dims, mats, stacks, Xs, rel, works):
            exat.ls(Ud, P, Ld, Id, Ad, R, ITERS, TOL, Xd, rd, wk)
    for _ in range(warmup):
        step()
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()                                   # the library's kernels run on torch's current stream
    for _ in range(steps):
        step()
    e1.record()
    torch.cuda.synchronize()
    ms_step = e0.elapsed_time(e1) / steps
    passes = 2 * ITERS + 1
    elements = sum(P * Ld * Id for Ld, Id in dims) * passes
    achieved = 4.0 * elements / (ms_step * 1e-3) / 1e9
    out = {
        "metric": "input tensor elements compressed/sec + TTM TFLOP/s (% MFMA peak), 1 MI355X",
        "value": elements / (ms_step * 1e-3), "unit": "elements/s",
        "n_gpus": 1, "steps": steps, "warmup": warmup, "ms_per_step": ms_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": "%s join of the replicas: stacked least squares (Eq. 4) for the three modes, %d x %d matrices, "
                               "%d right-hand sides, %d CGLS iterations each; elements = matrix elements x passes over the matrix"
                               % (cfg.name, P * cfg.L, cfg.I, R, ITERS)},
        "kernel_ms": {"all_launches": ms_step, "per_iteration": ms_step / (3 * ITERS)},
        "relres_max": max(float(r.max()) for r in rel),
        "roofline": {"bound": "hbm", "kernel": "k_ls_up + k_ls_down", "achieved": achieved, "peak": 8000.0, "unit": "GB/s",
                     "frac": achieved / 8000.0, "traffic": None},
    }
    if not args.no_cpu_baseline:
        import oracle
        from threadpoolctl import threadpool_info
        t = 0.0
        for (Uh, Ah), (Ld, Id) in zip(hosts, dims):
            t0 = time.perf_counter()
            oracle.stacked_ls(Uh.reshape(P, Ld, Id), Ah)
            t += time.perf_counter() - t0
        cores = max([int(lib.get("num_threads", 1)) for lib in threadpool_info()] + [1])
        out["cpu_baseline"] = {"value": elements / t, "unit": "elements/s", "cores": cores, "kind": "oracle",
                               "sample": "the same three solves (numpy lstsq, fp64), counted with the GPU's element figure",
                               "seconds_full": t, "extrapolated": False}
    print(json.dumps(out))


def two_stage(args):
    """One step = sparse first stage over X (resident in HBM) + dense multi-replica second stage on its output."""
    import torch
    from paper_2311_13693_amd import exat
    import workloads as wl
    cfg = wl.CONFIGS[args.config]
    assert cfg.materialised and cfg.dtype == "f32", "--two-stage needs a materialised fp32 configuration"
    ts = wl.TwoStage(cfg)
    steps = args.steps if args.steps is not None else (20 if cfg.elements > 5e8 else 200)
    warmup = args.warmup if args.warmup is not None else (20 if cfg.elements > 5e8 else 200)
    torch.cuda.set_device(0)
    A, B, C = wl.cp_factors(cfg)
    dev = lambda a: torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).cuda()
    gen = exat.make_gen(dev(A.T), dev(B.T), dev(C.T), cfg.seed, cfg.sigma)
    whole = exat.make_desc(cfg.I, cfg.J, cfg.K, cfg.L, cfg.M, cfg.N, cfg.P, cfg.I, cfg.J, cfg.K, exat.EXAT_F32)
    X = torch.empty(cfg.elements, dtype=torch.float32, device="cuda")
    exat.gen_block(whole, gen, 0, 0, 0, X)
    mats = wl.first_stage_matrices(ts)
    U2, V2, W2 = wl.second_stage_matrices(ts)
    st = exat.Stage1(cfg.I, cfg.J, cfg.K, *mats)
    c2 = ts.second
    plan = exat.Plan(exat.make_desc(c2.I, c2.J, c2.K, c2.L, c2.M, c2.N, c2.P, c2.dI, c2.dJ, c2.dK, exat.EXAT_F32))
    plan.set_factors(dev(U2), dev(V2), dev(W2))
    X1 = torch.empty(ts.A1 * ts.B1 * ts.C1, dtype=torch.float32, device="cuda")
    Y = plan.new_y()

    def step():
        st.apply(X, X1)
        plan.compress(X1, Y)
    st.set_timing(True)
    for _ in range(warmup):
        step()
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    k12, k3 = [], []
    e0.record()
    for _ in range(steps):
        step()
        a, b = st.last_timing()
        k12.append(a); k3.append(b)
    e1.record()
    torch.cuda.synchronize()
    if args.calib_copy:
        src = torch.ones(64 << 20, dtype=torch.float32, device="cuda")
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
    ms_step = e0.elapsed_time(e1) / steps
    ms12, ms3 = float(np.mean(k12)), float(np.mean(k3))
    # context for the roofline fraction: what a plain read-only pass over the same tensor (a library reduction)
    # reaches on this machine; not part of the timed region
    for _ in range(3):
        X.sum()
    r0, r1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    r0.record()
    for _ in range(10):
        X.sum()
    r1.record()
    torch.cuda.synchronize()
    ms_read = r0.elapsed_time(r1) / 10
    achieved = 4.0 * cfg.elements / (ms12 * 1e-3) / 1e9    # algorithmic bytes: every fp32 element of X once
    out = {
        "metric": "input tensor elements compressed/sec + TTM TFLOP/s (% MFMA peak), 1 MI355X",
        "value": cfg.elements / (ms_step * 1e-3), "unit": "elements/s",
        "n_gpus": 1, "steps": steps, "warmup": warmup, "ms_per_step": ms_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": "%s two-stage: %dx%dx%d f32 -> %dx%dx%d (sparse sign matrices, %d entries per column) -> "
                               "P=%d replicas of %dx%dx%d" % (cfg.name, cfg.I, cfg.J, cfg.K, ts.A1, ts.B1, ts.C1,
                                                              ts.nnz_per_col, cfg.P, cfg.L, cfg.M, cfg.N),
                   "sigma": cfg.sigma},
        "kernel_ms": {"stage1_mode12": ms12, "stage1_mode3": ms3},
        "read_only_pass_over_X": {"what": "torch.sum over the same tensor", "ms": ms_read,
                                  "GB/s": 4.0 * cfg.elements / (ms_read * 1e-3) / 1e9},
        "roofline": {"bound": "hbm", "kernel": "k_stage1_mfma (k_stage1_mode12 when U or V is no bf16 matrix)", "achieved": achieved, "peak": 8000.0, "unit": "GB/s",
                     "frac": achieved / 8000.0, "traffic": recorded_traffic(cfg.name + "_two_stage")},
    }
    if not args.no_cpu_baseline:
        import oracle
        Xh = X.cpu().numpy().reshape((cfg.I, cfg.J, cfg.K), order="F")
        nrep = 1 if cfg.elements > 5e8 else 2
        t0 = time.perf_counter()
        oracle.two_stage(Xh, *mats, U2, V2, W2, cfg.P, replicas=list(range(nrep)))
        t = (time.perf_counter() - t0) * cfg.P / nrep
        from threadpoolctl import threadpool_info
        cores = max([int(lib.get("num_threads", 1)) for lib in threadpool_info()] + [1])   # numpy's BLAS pool
        out["cpu_baseline"] = {"value": cfg.elements / t, "unit": "elements/s", "cores": cores, "kind": "oracle",
                               "sample": "replicas 0..%d of %d over the whole tensor (numpy fp64), scaled to all replicas"
                                         % (nrep - 1, cfg.P), "seconds_full": t, "extrapolated": nrep < cfg.P}
    plan.close(); st.close()
    print(json.dumps(out))


def cpu_baseline(cfg, A, B, C, U, V, W, budget_s=15.0):
    """Times the oracle as it stands on a bounded sample of the workload: (block, replica) units of the
    configuration's own block decomposition (Sec. 4.3), taken in order until the time budget is spent
    (or everything is done), then scaled by units_total / units_done."""
    import oracle
    nb = (cfg.I // cfg.dI, cfg.J // cfg.dJ, cfg.K // cfg.dK)
    units_total = nb[0] * nb[1] * nb[2] * cfg.P
    done, t_gen, t_comp = 0, 0.0, 0.0
    for bk in range(nb[2]):
        for bj in range(nb[1]):
            for bi in range(nb[0]):
                box = (bi * cfg.dI, (bi + 1) * cfg.dI, bj * cfg.dJ, (bj + 1) * cfg.dJ, bk * cfg.dK, (bk + 1) * cfg.dK)
                t0 = time.perf_counter()
                Xb = oracle.gen_box(A, B, C, cfg.seed, cfg.sigma, box)     # input preparation, not counted
                t_gen += time.perf_counter() - t0
                for p in range(cfg.P):
                    t0 = time.perf_counter()
                    oracle.comp_box(Xb, U, V, W, cfg.P, box, replicas=[p])
                    t_comp += time.perf_counter() - t0
                    done += 1
                    if t_comp >= budget_s:
                        break
                if t_comp >= budget_s or t_gen >= 2 * budget_s:
                    break
            if t_comp >= budget_s or t_gen >= 2 * budget_s:
                break
        if t_comp >= budget_s or t_gen >= 2 * budget_s:
            break
    t_full = t_comp * units_total / done
    return {"value": cfg.elements / t_full, "unit": "elements/s", "cores": oracle.num_threads(), "kind": "oracle",
            "sample": "%d of %d (block %dx%dx%d, replica) units of the same workload, %.1f s measured, scaled to all units"
                      % (done, units_total, cfg.dI, cfg.dJ, cfg.dK, t_comp),
            "seconds_full": t_full, "extrapolated": done < units_total}


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (no collectives are part of it); "
              "run with --gpus 1. Throughput at N GPUs is not measured.", file=sys.stderr)
        sys.exit(2)
    if args.mfma_ceiling:
        return mfma_ceiling(args)
    if args.two_stage:
        return two_stage(args)
    if args.cpals:
        return cpals(args)
    if args.ls:
        return ls(args)
    import torch
    from paper_2311_13693_amd import exat
    import workloads as wl
    cfg = wl.CONFIGS[args.config]
    big = cfg.elements > 5e10
    # A pass over the small configurations takes about a millisecond, and the chip needs some 50 ms of load before
    # its clock has settled (cfg2: 1.18 ms per pass after 3 warm-up passes, 1.105 ms after 50 or more), so their
    # defaults warm up for ~100 ms and time as long again.
    steps = args.steps if args.steps is not None else (2 if big else (5 if cfg.elements > 5e8 else 100))
    warmup = args.warmup if args.warmup is not None else (1 if big else (3 if cfg.elements > 5e8 else 100))

    torch.cuda.set_device(0)
    A, B, C = wl.cp_factors(cfg)
    U, V, W = wl.compression_matrices(cfg)
    dev = lambda a: torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).cuda()
    gen = exat.make_gen(dev(A.T), dev(B.T), dev(C.T), cfg.seed, cfg.sigma)
    split = args.split and cfg.dtype == "f32" and cfg.materialised
    dt = exat.EXAT_BF16 if cfg.dtype == "bf16" else (exat.EXAT_F32_SPLIT if split else exat.EXAT_F32)
    plan = exat.Plan(exat.make_desc(cfg.I, cfg.J, cfg.K, cfg.L, cfg.M, cfg.N, cfg.P, cfg.dI, cfg.dJ, cfg.dK, dt))
    t0 = time.perf_counter()
    plan.set_factors(dev(U), dev(V), dev(W))
    torch.cuda.synchronize()
    t_prep = time.perf_counter() - t0
    X = None
    if cfg.materialised:
        # X resident in HBM before the timed region, produced by the library's own block generator
        whole = exat.make_desc(cfg.I, cfg.J, cfg.K, cfg.L, cfg.M, cfg.N, cfg.P, cfg.I, cfg.J, cfg.K, dt)
        X = torch.empty(cfg.elements, dtype=torch.bfloat16 if cfg.dtype == "bf16" else torch.float32, device="cuda")
        exat.gen_block(whole, gen, 0, 0, 0, X)
    Y = plan.new_y()
    box, frac = None, 1.0
    if args.kslices and not cfg.materialised:
        box, frac = (0, cfg.I, 0, cfg.J, 0, args.kslices), args.kslices / cfg.K
    step = (lambda: plan.compress(X, Y)) if cfg.materialised else (lambda: plan.compress_gen(gen, box, Y))
    blocks = None
    if args.blocks and cfg.materialised:
        bdesc = exat.make_desc(cfg.I, cfg.J, cfg.K, cfg.L, cfg.M, cfg.N, cfg.P, cfg.dI, cfg.dJ, cfg.dK, dt)
        blocks = []
        for bk in range(cfg.K // cfg.dK):
            for bj in range(cfg.J // cfg.dJ):
                for bi in range(cfg.I // cfg.dI):
                    t = torch.empty(cfg.dI * cfg.dJ * cfg.dK, dtype=X.dtype, device="cuda")
                    exat.gen_block(bdesc, gen, bi, bj, bk, t)
                    blocks.append((bi, bj, bk, t))
        del X
        X = None

        nbi, nbj, nbk = cfg.I // cfg.dI, cfg.J // cfg.dJ, cfg.K // cfg.dK
        slabs = []
        if args.slab > 0:
            per_layer = nbi * nbj
            for bk0 in range(0, nbk, args.slab):
                bk1 = min(nbk, bk0 + args.slab)
                slabs.append(([t for _, _, _, t in blocks[bk0 * per_layer:bk1 * per_layer]], bk0, bk1))

        def step():
            if slabs:
                for ts, bk0, bk1 in slabs:
                    plan.compress_blocks(ts, 0, nbj, bk0, bk1)
            else:
                for bi, bj, bk, t in blocks:
                    plan.compress_block(t, bi, bj, bk)
            plan.finalize(Y)

    plan.set_timing(True)
    # whatever --warmup says, a configuration with passes of about a millisecond gets at least 100 untimed passes
    # before the timed ones (the clock has to settle, see above); reported as untimed_passes_before_warmup
    settle = max(0, 100 - warmup) if cfg.elements <= 5e8 else 0
    for _ in range(settle + warmup):
        step()
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    k12, k3 = [], []
    e0.record()
    for _ in range(steps):
        step()                         # back to back: nothing waits inside the timed region
    e1.record()
    torch.cuda.synchronize()
    calls_per_step = (len(slabs) if slabs else len(blocks)) if blocks else 1
    covered = max(1, min(steps, 128 // calls_per_step))   # whole passes inside the library's ring of 128 timed calls
    for age in range(min(covered * calls_per_step, 128)):
        a, b = plan.timing_of(age)
        k12.append(a); k3.append(b)
    if args.calib_copy:
        src = torch.ones(64 << 20, dtype=torch.float32, device="cuda")
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
    ms_step = e0.elapsed_time(e1) / steps
    ms12, ms3 = float(np.sum(k12)) / covered, float(np.sum(k3)) / covered   # per pass (a pass is one call, or one call per block)

    PL = cfg.P * cfg.L
    f12 = 2.0 * PL * (cfg.elements + cfg.M * cfg.J * cfg.K) * frac   # algorithmic flops of the fused mode-1/2 launch
    achieved = f12 / (ms12 * 1e-3) / 1e12
    peak = PEAK_TFLOPS["bf16" if split else cfg.dtype]   # fp16 and bf16 MFMA peaks are equal
    out = {
        "metric": "input tensor elements compressed/sec + TTM TFLOP/s (% MFMA peak), 1 MI355X",
        "value": cfg.elements * frac / (ms_step * 1e-3), "unit": "elements/s",
        "n_gpus": 1, "steps": steps, "warmup": warmup, "untimed_passes_before_warmup": settle, "ms_per_step": ms_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": ("f32 as two fp16 pieces (fp32 accumulate)" if split else "f32") if cfg.dtype == "f32" else "bf16 (fp32 accumulate)",
        "data": "synthetic",
        "config": {"workload": "%s: %dx%dx%d %s, R=%d, P=%d, L=M=N=%d, %s" % (
            cfg.name, cfg.I, cfg.J, cfg.K, cfg.dtype, cfg.R, cfg.P, cfg.L,
            (("block-streamed from HBM in %dx%dx%d blocks, " % (cfg.dI, cfg.dJ, cfg.dK)) +
             (("slabs of %d block layers per call (exat_compress_blocks + exat_finalize)" % args.slab) if slabs
              else "one call per block (exat_compress_block + exat_finalize)")) if blocks
            else ("materialised in HBM" if cfg.materialised else "generated on chip")),
            "sigma": cfg.sigma},
        "ttm_tflops": cfg.flops * frac / (ms_step * 1e-3) / 1e12,
        "ttm_frac_of_mfma_peak": cfg.flops * frac / (ms_step * 1e-3) / 1e12 / peak,
        "kernel_ms": {"mode12": ms12, "mode3": ms3},
        "operand_prep_ms": t_prep * 1e3,
        "roofline": {"bound": "mfma", "kernel": "k_mode12_split" if split else ("k_mode12_v4" if (cfg.dtype == "bf16" and not cfg.materialised) else "k_mode12_v3"), "achieved": achieved, "peak": peak, "unit": "TFLOP/s",
                     "frac": achieved / peak,
                     "traffic": recorded_traffic(cfg.name) if (frac == 1.0 and not split and not blocks) else None},
    }
    # what this machine sustains when a kernel issues nothing but MFMAs of the same kind on changing operands (after the
    # timed region; context for `frac`, which stays against the published peak)
    tf_only, ghz_only = exat.probe_mfma(0 if (cfg.dtype == "bf16" or split) else 1, True, 40000 if (cfg.dtype == "bf16" or split) else 20000, 256)
    out["mfma_only_on_this_box"] = {"tflops": tf_only, "core_ghz": ghz_only, "operands": "random",
                                    "instruction": "32x32x16 bf16" if (cfg.dtype == "bf16" or split) else "32x32x2 f32"}
    if cfg.materialised:
        out["hbm_algorithmic_gbps"] = cfg.elements * (2 if cfg.dtype == "bf16" else 4) / (ms12 * 1e-3) / 1e9
    if frac != 1.0:
        out["config"]["sub_box_k_slices"] = args.kslices
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(cfg, A, B, C, U, V, W)
    plan.close()
    print(json.dumps(out))


if __name__ == "__main__":
    main()
