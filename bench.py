#!/usr/bin/env python3
"""Benchmark of the SAP-scheduled Lasso round on one MI355X.

A "step" is one scheduling round (Algorithm 1's loop body: draw candidates, candidate Gram, greedy rho
filter, x_j^T r, soft-threshold update, residual update).  The default workload is the largest
configuration that fits one GPU: the fifth of the workload list, dense Lasso with N = 50000 rows,
J = 1000000 fp32 columns (200 GB resident in HBM), 30 % near-duplicate columns, L' = 8000 candidates
per round (Section 5, "Datasets": it stands in for the paper's 450 x 1,000,000 synthetic design).
Inputs are synthetic, generated on the GPU and resident in HBM before the timed region.

Prints ONE JSON line: whole-job coordinate updates per second, plus
  roofline     -- the candidate-Gram MFMA tile kernel against the fp32 matrix peak, its duration
                  measured with HIP events on the solver's stream inside the timed region
  hbm_streams  -- the two HBM streams of a round (x_j^T r for the kept set; the residual update)
  hbm_pass     -- the pass over all J columns (the stopping test)
  cpu_baseline -- the CPU oracle timed on this machine's host cores, at one thread and at all of them, on a
                  bounded sample of the same workload (a reported baseline, not a target)
  secondary    -- (default workload only) the second configuration (N = 10000, J = 100000, L' = 1000)
                  inside its initial sweep and after it (rounds >= J / L')

Other modes: --sweep (size sweep of the Gram, the kept-set dot products and the residual update) and
--compare-schedulers (objective against rounds and time for the schedulers Section 5.1 compares).
"""
from __future__ import annotations

import argparse
import ctypes
import glob
import json
import os
import re
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

MFMA_FP32_PEAK_TFLOPS = 157.3
VALU_FP32_PEAK_TFLOPS = 157.3         # 256 compute units x 128 lanes x 2 flop x 2.4 GHz
HBM_PEAK_GBPS = 8000.0
DEFAULT_WORKLOAD = "c5_dense_duplicates"

WORKLOADS = {
    # name -> (config key of synth.lasso_inputs, overrides)
    "c2_dense_block_corr": ("c2_dense_block_corr", {}),
    "c1_dense_iid": ("c1_dense_iid", {}),
    "c3_genotype": ("c3_genotype", {}),
    # the third configuration stored as 2-bit genotype counts (16 rows per 32-bit word)
    "c3_genotype_packed": ("c3_genotype_packed", {}),
    "c4_sparse_csc": ("c4_sparse_csc", {}),
    # the fifth configuration's rows, duplicate structure and L'=8000 with J cut to fit quick runs
    "c5_dense_duplicates_j60k": ("c5_dense_duplicates", dict(j=60000, nnz=200, rounds=20)),
    # the fifth configuration at full size: 50000 x 1000000 fp32 = 200 GB of X resident in HBM
    "c5_dense_duplicates": ("c5_dense_duplicates", {}),
    "c2_small": ("c2_dense_block_corr", dict(n=2000, j=8000, nnz=40, l_prime=500, rounds=16)),
}


def measured_traffic(kernel: str, workload: str, route: str):
    """HBM bytes per launch (read + written) of a kernel, from the rocprofv3 --pmc summaries under
    profiles/ (FETCH_SIZE and WRITE_SIZE, already scaled by the copy-kernel calibration stated there).
    A summary carries one line per measured launch shape:
        #@ traffic kernel=<k> workload=<w> route=<r> fetch_bytes=<n> write_bytes=<n>
    Returns None when no summary covers this kernel, workload and route."""
    pat = re.compile(r"^#@ traffic kernel=(\S+) workload=(\S+) route=(\S+) fetch_bytes=(\d+) write_bytes=(\d+)")
    for path in sorted(glob.glob(os.path.join(ROOT, "profiles", "*.txt"))):
        try:
            with open(path) as f:
                for line in f:
                    m = pat.match(line)
                    if m and (m.group(1), m.group(2), m.group(3)) == (kernel, workload, route):
                        return {"bytes": int(m.group(4)) + int(m.group(5)), "fetch_bytes": int(m.group(4)),
                                "write_bytes": int(m.group(5)), "source": os.path.relpath(path, ROOT)}
        except OSError:
            continue
    return None


def design_args(p, host=False):
    """The design matrix of a synthetic problem as constructor arguments: of the library (device
    tensors, packed codes where the workload has them) or, with host, of the oracle (numpy; a packed
    design as the fp32 matrix its codes stand for)."""
    if host:
        if p.layout in ("dense", "geno2"):
            return dict(x=p.x.cpu().numpy())
        return dict(values=p.values.cpu().numpy(), row_idx=p.row_idx.cpu().numpy(), col_ptr=p.col_ptr.cpu().numpy(),
                    n=p.n)
    if p.layout == "dense":
        return dict(x=p.x)
    if p.layout == "geno2":
        return dict(codes=p.codes, col_mean=p.col_mean, col_scale=p.col_scale, n=p.n)
    return dict(values=p.values, row_idx=p.row_idx, col_ptr=p.col_ptr, n=p.n)


# ---------------------------------------------------------------------------------------------------
# host cores: what they are, and how many of them the oracle's OpenMP loops use
# ---------------------------------------------------------------------------------------------------
def cpu_model() -> str:
    try:
        with open("/proc/cpuinfo") as f:
            for line in f:
                if line.lower().startswith("model name"):
                    return line.split(":", 1)[1].strip()
    except OSError:
        pass
    return "unknown"


class OmpThreads:
    """Number of threads of the OpenMP runtime the oracle library is linked with (the oracle itself is
    not touched: this is the runtime's own omp_set_num_threads)."""

    def __init__(self):
        self.lib = None
        for name in ("libgomp.so.1", "libgomp.so"):
            try:
                self.lib = ctypes.CDLL(name)
                break
            except OSError:
                continue
        self.all = int(self.lib.omp_get_max_threads()) if self.lib else 1

    def set(self, n: int) -> int:
        if self.lib:
            self.lib.omp_set_num_threads(int(n))
            return int(n)
        return 1


def _timed(f):
    t0 = time.perf_counter()
    out = f()
    return time.perf_counter() - t0, out


def cpu_baseline_rounds(p, args, rounds_done, wall, budget_s):
    """Whole oracle rounds from round 0 on the workload's own arrays (configurations the host can hold):
    at all cores, then at one thread, each inside its share of the budget."""
    from oracle.oracle import OracleLasso
    omp = OmpThreads()
    okw = dict(y=p.y.cpu().numpy(), lam=p.lam, rho=p.rho, eta=p.eta, l_prime=p.l_prime, seed=p.seed,
               p_max=args.p_max, dynamic=args.deps == "dynamic", no_deps=args.deps == "none",
               priority=args.priority, n_shards=args.shards, loss=args.loss)
    host = design_args(p, host=True)
    legs = {}
    for name, threads, share in (("all_cores", omp.all, 0.6), ("one_thread", 1, 0.4)):
        omp.set(threads)
        o = OracleLasso(**host, **okw)
        n_upd = n_rounds = 0
        tc = time.perf_counter()
        while True:
            n_upd += len(o.round()["kept"])
            n_rounds += 1
            el = time.perf_counter() - tc
            if n_rounds >= args.steps or el + el / n_rounds > budget_s * share:
                break
        el = time.perf_counter() - tc
        legs[name] = {"threads": threads, "rounds": n_rounds, "seconds": round(el, 3), "updates": n_upd,
                      "updates_per_s": round(n_upd / el, 2), "rounds_per_s": round(n_rounds / el, 4),
                      "objective_after_sample": float(o.objective())}
    omp.set(omp.all)
    a = legs["all_cores"]
    return {"value": a["updates_per_s"], "unit": "updates/s", "cores": a["threads"], "kind": "oracle",
            "sample": f"first {a['rounds']} rounds of the same workload from round 0, whole oracle rounds "
                      f"({a['seconds']} s at {a['threads']} threads; {legs['one_thread']['rounds']} rounds, "
                      f"{legs['one_thread']['seconds']} s at 1 thread)",
            "value_one_thread": legs["one_thread"]["updates_per_s"], "rounds_per_s": a["rounds_per_s"],
            "cpu_model": cpu_model(), "nproc": os.cpu_count(), "legs": legs,
            "objective_after_sample": a["objective_after_sample"], "seconds_to_that_objective": a["seconds"]}


def cpu_baseline_large(p, args, make_solver, ms_per_round, budget_s):
    """Configurations the host cannot hold (200 GB of X; 3.2 TFLOP of Gram per round): round 0 of the
    same workload, with the oracle's own stage functions applied to what the round touches.
      * Step 1 whole: keys for all J coordinates and the draw of L' candidates.
      * Step 2: the candidate columns are gathered from the GPU's copy of X; R complete rows of the
        L' x L' candidate Gram are computed (each row = L' dot products of N terms, the unit the whole
        Gram is made of) and the time is scaled to the (L'+1)/2 row-equivalents of the upper triangle
        that oracle_gram_dense computes; the greedy walk is timed on an L' x L' identity matrix.
      * eq. (2), Step 4 and the residual update whole, on the kept set of the GPU's round 0 (the kept set
        needs the whole Gram, which the CPU does not compute here; the GPU's is the oracle's by the
        parity tests).
    Each piece at one thread and at all cores.  updates/s = |B_1| of that round / the summed time."""
    import numpy as np
    import torch
    from oracle import oracle as orc
    omp = OmpThreads()
    g = make_solver()
    beta0, dbeta0, r0, _ = g.get_state()
    f_start = g.objective()
    g.round()
    lr = g.last_round()
    cand, kept_pos = lr["cand"].cpu().numpy(), lr["kept_pos"].cpu().numpy()
    f_gpu = g.objective()
    g.close()
    L, k = len(cand), len(kept_pos)
    xs = p.x[lr["cand"].long()].cpu().numpy()                      # (L, N) gathered candidate columns
    beta0, dbeta0, r0 = beta0.cpu().numpy(), dbeta0.cpu().numpy(), r0.cpu().numpy()
    local = np.arange(L, dtype=np.int32)
    eye = np.eye(L, dtype=np.float32)
    # rows per leg: the Gram rows take most of the budget; a row costs about N * L' / 1.8e9 s on one core
    row_s = p.n * L / 1.8e9
    legs = {}
    f_ref = None
    for name, threads, share in (("all_cores", omp.all, 0.5), ("one_thread", 1, 0.5)):
        omp.set(threads)
        n_rows = int(max(4, min(L, budget_s * share * 0.6 / (row_s / threads))))
        t_keys, keys = _timed(lambda: orc.priority_keys(dbeta0, p.eta, p.seed, 0))
        t_draw, ref_cand = _timed(lambda: orc.draw(keys, p.l_prime))
        same_draw = bool(np.array_equal(ref_cand, cand))
        rows = np.linspace(0, L - 1, n_rows).astype(np.int32)
        t_rows, _ = _timed(lambda: orc.gram_rows_dense(xs, local, rows))
        t_gram = t_rows / n_rows * (L + 1) / 2.0
        t_filter, _ = _timed(lambda: orc.greedy_filter(eye, p.rho, 0))
        b, d, r = beta0.copy(), dbeta0.copy(), r0.copy()

        def upd():
            z = orc.dots_dense(xs, kept_pos, r)
            delta = orc.update(cand[kept_pos], z, p.lam, b, d)
            orc.residual_dense(xs, kept_pos, delta, r)
        t_upd, _ = _timed(upd)
        f_ref = orc.objective(r, b, p.lam)
        total = t_keys + t_draw + t_gram + t_filter + t_upd
        legs[name] = {"threads": threads, "gram_rows_timed": n_rows, "gram_rows_s": round(t_rows, 3),
                      "keys_and_draw_s": round(t_keys + t_draw, 3), "gram_s_extrapolated": round(t_gram, 2),
                      "filter_s": round(t_filter, 3), "dots_update_residual_s": round(t_upd, 3),
                      "round_s_extrapolated": round(total, 2), "updates_per_s": round(k / total, 3),
                      "cpu_seconds_spent": round(t_keys + t_draw + t_rows + t_filter + t_upd, 2),
                      "candidate_list_equals_gpu": same_draw}
    omp.set(omp.all)
    a, o1 = legs["all_cores"], legs["one_thread"]
    return {"value": a["updates_per_s"], "unit": "updates/s", "cores": a["threads"], "kind": "oracle",
            "sample": (f"round 0 of the same workload on its gathered candidate columns: keys and draw over all "
                       f"J = {p.j}, {a['gram_rows_timed']} complete rows of the {L} x {L} candidate Gram at {a['threads']} "
                       f"threads ({o1['gram_rows_timed']} at 1 thread), the greedy walk on an identity matrix, "
                       f"x_j^T r / update / residual for the {k} kept columns"),
            "extrapolation": (f"Gram time = time per row x (L'+1)/2 = {(L + 1) / 2:.0f} row-equivalents (the upper triangle "
                              f"oracle_gram_dense computes); round time = keys + draw + that + walk + update; "
                              f"updates/s = {k} kept coordinates / round time"),
            "value_one_thread": o1["updates_per_s"], "rounds_per_s": round(1.0 / a["round_s_extrapolated"], 6),
            "cpu_model": cpu_model(), "nproc": os.cpu_count(), "legs": legs,
            "objective_start": f_start, "objective_after_sample": float(f_ref), "gpu_objective_at_that_round": f_gpu,
            "seconds_to_that_objective": a["round_s_extrapolated"],
            "seconds_to_that_objective_one_thread": o1["round_s_extrapolated"],
            "gpu_seconds_to_that_objective": round(ms_per_round * 1e-3, 6)}


# ---------------------------------------------------------------------------------------------------
# other modes
# ---------------------------------------------------------------------------------------------------
def run_sweep(args) -> int:
    """Size sweep of the three per-round kernels that have a roofline: the candidate Gram (fp32 MFMA),
    the dot products of the kept set and the residual update (HBM streams).  Each point is a synthetic
    i.i.d. design with exactly L' columns (every column is a candidate in every round), a threshold no
    pair reaches (every candidate is kept) and lambda = 0 (every kept coordinate moves): k = k1 = L'.
    Kernel times are the library's per-stage HIP events averaged over the timed rounds.  The dot products
    are taken by their own kernel for every list length (a short list would otherwise fold them into the
    Gram launch); the residual update takes the route the library picks for the shape."""
    import torch
    import paper_1312_5766_amd as pk
    pk.load()
    dev = torch.device("cuda:0")
    print(f"{'N':>6} {'L=k':>5} | {'gram us':>9} {'TFLOP/s':>8} {'frac':>5} {'tile':>4} {'mask us':>7} | {'dots MB':>8} {'us':>7} {'GB/s':>6} "
          f"{'frac':>5} | {'resid us':>8} {'GB/s':>6} {'frac':>5}", flush=True)
    for n in args.sweep_rows:
        for l in args.sweep_l_prime:
            if 4.0 * n * l > 8e9:
                continue
            gen = torch.Generator(device=dev)
            gen.manual_seed(1000003 * n + l)
            x = torch.randn((l, n), generator=gen, device=dev, dtype=torch.float32)
            x /= x.norm(dim=1, keepdim=True)
            y = torch.randn(n, generator=gen, device=dev, dtype=torch.float32)
            s = pk.StradsLasso(x=x, y=y, lam=0.0, rho=2.0, eta=1e-6, l_prime=l, seed=0)
            s.set_tuning("dots_with_gram", 0)      # the kept-set dot products as a kernel of their own, so that they can be timed
            for t in args.tune:
                name, value = t.split("=")
                try:
                    s.set_tuning(name, int(value))
                except pk.StradsError as e:            # a route the shape has no room for: the point keeps the default
                    print(f"# N={n} L'={l}: {name}={value} refused ({e})", flush=True)
            edge = s.gram_tile_edge()
            for _ in range(2):
                s.round()
            # every round starts from the same state, so the values stay finite whatever Jacobi does with L' columns
            beta, dbeta, r, _t = [a.clone() if isinstance(a, torch.Tensor) else a for a in s.get_state()]
            rounds = args.sweep_rounds
            s.set_tuning("profile_rounds", rounds)
            s.set_tuning("profile_level", 2)
            kept = moved = 0
            for t in range(rounds):
                s.set_state(beta, dbeta, r, 2 + t)
                info = s.round(want_info=True)
                kept += info.n_kept
                moved += info.n_moved
            st = s.stage_times()
            s.close()
            k, k1 = kept / rounds, moved / rounds
            gram_tf = n * l * (l - 1) / (st["gram_tiles"] * 1e-3) / 1e12 if st["gram_tiles"] > 0 else 0.0
            dots_gb = 4.0 * n * (k + 1) / (st["update"] * 1e-3) / 1e9 if st["update"] > 0 else 0.0
            res_gb = (4.0 * n * k1 + 8.0 * n) / (st["residual"] * 1e-3) / 1e9
            print(f"{n:>6} {l:>5} | {st['gram_tiles'] * 1e3:>9.1f} {gram_tf:>8.1f} {gram_tf / MFMA_FP32_PEAK_TFLOPS:>5.3f} "
                  f"{edge:>4} {st['gram_mask'] * 1e3:>7.1f} | "
                  f"{4e-6 * n * (k + 1):>8.1f} {st['update'] * 1e3:>7.1f} {dots_gb:>6.0f} {dots_gb / HBM_PEAK_GBPS:>5.3f} | "
                  f"{st['residual'] * 1e3:>8.1f} {res_gb:>6.0f} {res_gb / HBM_PEAK_GBPS:>5.3f}", flush=True)
            del x, y, s
    return 0


def run_compare_schedulers(args) -> int:
    """Objective against rounds and time for the schedulers Section 5.1 compares, on one workload:
    strads (priority (delta beta)^2 + eta, dependency check among all candidates: Algorithm 1),
    strads-dynamic (dependencies only between candidates that move), static-corr (uniform draw, same
    check), shotgun (uniform draw, no check; --p-max coordinates per round).  Every scheduler starts
    from beta = 0 on the same inputs; one JSON line per scheduler."""
    import torch
    import paper_1312_5766_amd as pk
    from synth import lasso_inputs as si
    pk.load()
    dev = torch.device("cuda:0")
    key, over = WORKLOADS[args.workload]
    p = si.make(key, device=dev, **over)
    base = dict(y=p.y, lam=p.lam, rho=p.rho, eta=p.eta, l_prime=p.l_prime, seed=p.seed, **design_args(p))
    modes = {"strads": dict(), "strads-dynamic": dict(dynamic=True), "static-corr": dict(priority="uniform"),
             "shotgun": dict(priority="uniform", no_deps=True, p_max=args.p_max)}
    every = max(1, args.check_every)
    for name, kw in modes.items():
        g = pk.StradsLasso(**base, **kw)
        g.round()                               # first-launch costs stay out of the clock
        torch.cuda.synchronize()
        g.close()
        g = pk.StradsLasso(**base, **kw)
        traj = [(0, 0.0, g.objective())]
        done, t_run = 0, 0.0
        while done < args.steps:
            n = min(every, args.steps - done)
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            try:
                info = g.run(n)
            except pk.StradsError as e:         # unchecked updates of correlated columns can diverge (Section 2)
                traj.append((done + n, None, str(e)))
                break
            torch.cuda.synchronize()
            t_run += time.perf_counter() - t0
            done += n
            traj.append((done, round(t_run * 1e3, 3), float(info.objective)))
        print(json.dumps({"scheduler": name, "workload": args.workload, "rounds": done,
                          "ms_total": round(t_run * 1e3, 2), "trajectory_round_ms_objective": traj}), flush=True)
        g.close()
    return 0


# ---------------------------------------------------------------------------------------------------
# the benchmark
# ---------------------------------------------------------------------------------------------------
def kkt_pass(g, p, shards, torch):
    """The HBM-bound pass: x_j^T r for all J columns (the stopping test streams X once), timed by the
    library's events around its kernels (the read-back of the result is not part of the pass)."""
    torch.cuda.synchronize()
    kkt_times = []
    if shards == 1:
        g.set_tuning("profile_level", 1)
        g.kkt()
        for _ in range(3):
            viol = g.kkt()
            kkt_times.append(g.last_kkt_ms())
        g.set_tuning("profile_level", 0)
    else:
        # stage profiling is not available with scheduler shards: events around the whole call instead
        # (they include the read-back of the result, a few microseconds)
        g.kkt()
        for _ in range(3):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            viol = g.kkt()
            e1.record()
            torch.cuda.synchronize()
            kkt_times.append(e0.elapsed_time(e1))
    kkt_ms = sum(kkt_times) / len(kkt_times)
    if p.layout == "dense":
        kkt_bytes = 4.0 * p.n * p.j
    elif p.layout == "geno2":
        kkt_bytes = 4.0 * float(p.codes.numel())
    else:
        kkt_bytes = 8.0 * float(p.values.numel())
    kkt_gbps = kkt_bytes / (kkt_ms * 1e-3) / 1e9
    out = {"kernel": "k_kkt", "bound": "hbm", "bytes": kkt_bytes, "ms": round(kkt_ms, 4),
           "achieved": round(kkt_gbps, 1), "peak": HBM_PEAK_GBPS, "unit": "GB/s",
           "frac": round(kkt_gbps / HBM_PEAK_GBPS, 4)}
    if p.layout == "geno2":
        # on packed codes the pass moves 16 times fewer bytes and is bound by the vector ALU instead:
        # one multiply-add (2 flop) per entry of X on the fp32 vector pipes (157.3 TFLOP/s)
        tf = 2.0 * p.n * p.j / (kkt_ms * 1e-3) / 1e12
        out = {"kernel": "k_geno_dots", "bound": "alu", "flops": 2.0 * p.n * p.j, "bytes": kkt_bytes,
               "ms": round(kkt_ms, 4), "achieved": round(tf, 2), "peak": VALU_FP32_PEAK_TFLOPS,
               "unit": "TFLOP/s", "frac": round(tf / VALU_FP32_PEAK_TFLOPS, 4), "codes_gbps": round(kkt_gbps, 1)}
    return out, viol


def gram_roofline(p, L, stage, workload, rides, tile_edge=128):
    gram_flops = float(p.n) * L * (L - 1)          # algorithmic: every unordered pair once, 2 flops per row
    ach = gram_flops / (stage["gram_tiles"] * 1e-3) / 1e12
    kernel = {256: "k_gram_tiles256", 64: "k_gram_direct"}.get(tile_edge, "k_gram_tiles")
    tr = measured_traffic(kernel, workload, "with_dots" if rides else "tiles_only")
    return {"bound": "mfma", "kernel": kernel, "achieved": round(ach, 3),
            "peak": MFMA_FP32_PEAK_TFLOPS, "unit": "TFLOP/s", "frac": round(ach / MFMA_FP32_PEAK_TFLOPS, 4),
            "traffic": tr["bytes"] if tr else None, "traffic_source": tr["source"] if tr else None,
            "avg_ms": round(stage["gram_tiles"], 5), "launches": stage["rounds"], "flops_per_launch": gram_flops,
            "launch_also_carries": "x_j^T r of every candidate (4*N*L' bytes)" if rides else None}


def stream_leg(make_solver, p, steps, workload, skip_rounds=0):
    """The two HBM streams of a round (x_j^T r for the kept set; the residual update), timed per stage on
    a second pass over the same trajectory with every stage bracketed by events (not the headline run:
    the extra events and the per-round readback of |B| and the mover count cost a few microseconds).
    For a short candidate list the timed run folds both into other launches; this leg then switches
    the folding off, so that the two kernels can be timed on their own."""
    v = make_solver()
    short = p.l_prime <= 4096
    if short:
        v.set_tuning("dots_with_gram", 0)
        v.set_tuning("residual_fused", 0)
    if skip_rounds:
        v.run(skip_rounds)
    v.set_tuning("profile_rounds", max(steps, 1))
    v.set_tuning("profile_level", 2)
    kept = moved = 0
    for _ in range(steps):
        ri = v.round(want_info=True)
        kept += ri.n_kept
        moved += ri.n_moved
    st2 = v.stage_times()
    v.set_tuning("profile_level", 0)
    v.close()
    if not (st2["rounds"] > 0 and st2["update"] > 0 and st2["residual"] > 0):
        return None
    k, k1 = kept / st2["rounds"], moved / st2["rounds"]
    dots_b, res_b = 4.0 * p.n * (k + 1), 4.0 * p.n * k1 + 8.0 * p.n
    dots_g, res_g = dots_b / (st2["update"] * 1e-3) / 1e9, res_b / (st2["residual"] * 1e-3) / 1e9
    td = measured_traffic("k_dots_update", workload, "general")
    tr = measured_traffic("k_residual", workload, "general")
    return {
        "dots": {"kernel": "k_dots_update", "bytes": round(dots_b), "ms": round(st2["update"], 5),
                 "achieved": round(dots_g, 1), "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                 "frac": round(dots_g / HBM_PEAK_GBPS, 4), "avg_kept": round(k, 1),
                 "traffic": td["bytes"] if td else None},
        "residual": {"kernel": "k_residual", "bytes": round(res_b),
                     "ms": round(st2["residual"], 5), "achieved": round(res_g, 1), "peak": HBM_PEAK_GBPS,
                     "unit": "GB/s", "frac": round(res_g / HBM_PEAK_GBPS, 4), "avg_moved": round(k1, 1),
                     "traffic": tr["bytes"] if tr else None},
        "stage_ms": {kk: round(vv, 5) for kk, vv in st2.items() if kk != "rounds"},
        "route": ("general route forced for this leg (dots_with_gram=0, residual_fused=0); the timed "
                  "run folds both kernels into other launches") if short else "as in the timed run",
    }


def timed_window(g, steps, torch):
    """`steps` rounds enqueued back to back on an existing solver, the Gram kernel bracketed by events."""
    g.set_tuning("profile_rounds", max(steps, 1))
    g.set_tuning("profile_level", 1)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    info = g.run(steps)
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    stage = g.stage_times()
    g.set_tuning("profile_level", 0)
    return info, wall, stage


def secondary_c2(args, pk, si, torch, dev):
    """The second configuration (N = 10000, J = 100000, block-correlated columns, L' = 1000): a window
    inside the initial sweep over all coordinates (rounds 0 .. K) and one after it (from round J / L',
    where the priorities have taken over and far fewer of the 1000 candidates move)."""
    p = si.make("c2_dense_block_corr", device=dev)
    torch.cuda.synchronize()
    kw = dict(x=p.x, y=p.y, lam=p.lam, rho=p.rho, eta=p.eta, l_prime=p.l_prime, seed=p.seed)
    K = max(1, min(args.steps, 100))
    g = pk.StradsLasso(**kw)
    g.run(min(args.warmup, 10))
    g.close()
    g = pk.StradsLasso(**kw)
    out = {"config": {"workload": "c2_dense_block_corr", "n": p.n, "j": p.j, "l_prime": p.l_prime, "lambda": p.lam}}
    sweep_rounds = (p.j + p.l_prime - 1) // p.l_prime
    for name, start in (("sweep_window", 0), ("post_sweep_window", sweep_rounds)):
        if start > 0:
            already = int(g.get_state()[3])
            if start > already:
                g.run(start - already)
        first = int(g.get_state()[3])
        info, wall, stage = timed_window(g, K, torch)
        blk = {"first_round": first, "rounds": K, "ms_per_step": round(wall / K * 1e3, 4),
               "value": round(int(info.updates_done) / wall, 1), "unit": "updates/s",
               "avg_kept": round(int(info.updates_done) / K, 1), "objective_end": float(info.objective)}
        if stage["rounds"] > 0 and stage["gram_tiles"] > 0:
            blk["roofline"] = gram_roofline(p, g.L, stage, "c2_dense_block_corr", rides=True)
        out[name] = blk
    pass_, viol = kkt_pass(g, p, 1, torch)
    out["hbm_pass"] = pass_
    g.close()
    out["hbm_streams_sweep"] = stream_leg(lambda: pk.StradsLasso(**kw), p, K, "c2_dense_block_corr")
    out["hbm_streams_post_sweep"] = stream_leg(lambda: pk.StradsLasso(**kw), p, K, "c2_dense_block_corr",
                                               skip_rounds=sweep_rounds)
    if args.cpu_seconds > 0:
        class A:                                  # the oracle's options for this block: Algorithm 1 as printed
            pass
        a = A()
        a.p_max, a.deps, a.priority, a.shards, a.loss, a.steps = 0, "static", "squared", 1, "squared", K
        out["cpu_baseline"] = cpu_baseline_rounds(p, a, K, 0.0, min(args.cpu_seconds, 12.0))
        ms = out["sweep_window"]["ms_per_step"]
        out["cpu_baseline"]["gpu_seconds_for_the_same_rounds"] = round(
            out["cpu_baseline"]["legs"]["all_cores"]["rounds"] * ms * 1e-3, 6)
    del p
    torch.cuda.empty_cache()
    return out


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=100)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--workload", default=DEFAULT_WORKLOAD, choices=sorted(WORKLOADS))
    ap.add_argument("--cpu-seconds", type=float, default=24.0, help="budget of the oracle timing (0 = skip)")
    ap.add_argument("--profile-level", type=int, default=1, choices=(0, 1, 2),
                    help="HIP-event timing inside the timed region: 1 = Gram kernel only, 2 = every stage")
    ap.add_argument("--split-k", type=int, default=0)
    ap.add_argument("--tune", action="append", default=[], metavar="NAME=VALUE",
                    help="strads_lasso_set_tuning knob applied to every solver of the run (repeatable)")
    ap.add_argument("--deps", default="static", choices=("static", "dynamic", "none"),
                    help="dependency rule of Step 2: static = Algorithm 1 as printed (the headline workload); "
                         "dynamic = only pairs of candidates that both move are checked; "
                         "none = no check (Shotgun when combined with --priority uniform)")
    ap.add_argument("--priority", default="squared", choices=("squared", "linear", "uniform"),
                    help="weight of Step 1's draw: (delta beta)^2+eta (headline), |delta beta|+eta, or 1")
    ap.add_argument("--loss", default="squared", choices=("squared", "logistic"),
                    help="loss of eq. (1); logistic: the workload's design with labels drawn from its planted "
                         "coefficients (dense workloads; not the headline)")
    ap.add_argument("--p-max", type=int, default=0, help="cap on the kept set (Algorithm 1's P); 0 = none")
    ap.add_argument("--shards", type=int, default=1,
                    help="scheduler shards taking turns (Section 3); > 1 overlaps the shards' scheduling work on "
                         "separate streams (the headline workload uses 1: Algorithm 1 with one scheduler)")
    ap.add_argument("--kkt-tol", type=float, default=0.0,
                    help="> 0: --steps is an upper bound and the run stops once the optimality violation is "
                         "<= kkt_tol * lambda, tested every --check-every rounds (each test streams X once)")
    ap.add_argument("--check-every", type=int, default=25)
    ap.add_argument("--graph-rounds", type=int, default=0,
                    help="> 0: strads_lasso_run records this many rounds once as a HIP graph and replays it "
                         "(default 0: every round is enqueued; on this runtime a replay does not run the "
                         "shards' branches concurrently)")
    ap.add_argument("--no-variants", action="store_true",
                    help="skip the extra legs that time the same workload with 4 scheduler shards and with "
                         "dynamic dependencies (reported under 'variants'; the headline value is unaffected)")
    ap.add_argument("--no-secondary", action="store_true",
                    help="skip the block on the second configuration that the default workload's line carries")
    ap.add_argument("--library-route", action="store_true",
                    help="also time, for scale, the library route for Step 2 (torch gather of the candidate "
                         "columns + the vendor GEMM of the panel with its transpose, fp32)")
    ap.add_argument("--pmc-calibration", action="store_true",
                    help="after the timed region run one elementwise kernel of known traffic (reads 1 GiB, "
                         "writes 1 GiB) so that a rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE run of this command "
                         "carries its own scale factor")
    ap.add_argument("--sweep", action="store_true", help="size sweep of Gram / dots / residual kernels, then exit")
    ap.add_argument("--sweep-rows", type=int, nargs="+", default=[10000, 50000])
    ap.add_argument("--sweep-l-prime", type=int, nargs="+", default=[32, 128, 256, 512, 1024, 2048, 4096, 8192])
    ap.add_argument("--sweep-rounds", type=int, default=6)
    ap.add_argument("--compare-schedulers", action="store_true",
                    help="objective against rounds and time for the four schedulers on --workload (--steps rounds, "
                         "objective read every --check-every rounds), then exit")
    args = ap.parse_args()

    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs the whole scheduling round on ONE GPU (scheduler and workers "
              "collapse onto it); there is no multi-GPU path to time. Run with --gpus 1.", file=sys.stderr)
        return 2

    import torch
    import paper_1312_5766_amd as pk
    from synth import lasso_inputs as si

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 2
    pk.load()                                   # fails loudly if the HIP library is not built
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    if args.sweep:
        return run_sweep(args)
    if args.compare_schedulers:
        return run_compare_schedulers(args)
    if args.graph_rounds > 0:
        # HIP-graph replay of groups of rounds needs a stream that can be captured (the legacy default
        # stream cannot); otherwise the default stream is used: a stream of our own would take one of
        # the four hardware queues away from the scheduler shards
        torch.cuda.set_stream(torch.cuda.Stream(dev))

    key, over = WORKLOADS[args.workload]
    over = dict(over)
    workload_name, fit_note = args.workload, None
    if args.workload == "c5_dense_duplicates":
        # 200 GB of X plus about 3 GB of workspaces and gathered panels: if this GPU exposes less, the
        # largest J that fits is used and the line says so
        free, _total = torch.cuda.mem_get_info()
        need = 4.0 * 50000 * 1000000 + 6e9
        if free < need:
            j_fit = int((free - 6e9) / (4.0 * 50000)) // 1000 * 1000
            over.update(j=j_fit, nnz=max(10, j_fit // 500))
            workload_name = f"c5_dense_duplicates_j{j_fit}"
            fit_note = f"only {free / 1e9:.0f} GB of HBM free: J cut from 1000000 to {j_fit}"
            print(f"bench.py: {fit_note}", file=sys.stderr, flush=True)
    t0 = time.time()
    p = si.make(key, device=dev, **over)
    if args.loss == "logistic":
        p = si.with_labels(p)
    torch.cuda.synchronize()
    t_gen = time.time() - t0
    print(f"bench.py: inputs for {workload_name} generated in {t_gen:.1f} s", file=sys.stderr, flush=True)

    def fresh():
        kw = dict(y=p.y, lam=p.lam, rho=p.rho, eta=p.eta, l_prime=p.l_prime, seed=p.seed, p_max=args.p_max,
                  dynamic=args.deps == "dynamic", no_deps=args.deps == "none", priority=args.priority,
                  n_shards=args.shards, loss=args.loss)
        h = pk.StradsLasso(**design_args(p), **kw)
        for t in args.tune:
            name, value = t.split("=")
            h.set_tuning(name, int(value))
        if args.split_k:
            h.set_tuning("gram_split_k", args.split_k)
        return h

    # warm-up on a throw-away handle, so that the timed region is the configuration's own
    # trajectory from round 0
    g = fresh()
    for _ in range(args.warmup):
        g.round()
    torch.cuda.synchronize()
    g.close()
    print("bench.py: warm-up done", file=sys.stderr, flush=True)

    g = fresh()
    tile_edge = g.gram_tile_edge()
    if args.graph_rounds > 0:
        g.set_tuning("graph_rounds", args.graph_rounds)
    f0 = g.objective()
    if args.shards > 1:
        args.profile_level = 0                  # stages of different shards overlap: no per-stage timing
    g.set_tuning("profile_rounds", max(args.steps, 1))
    g.set_tuning("profile_level", args.profile_level)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    rounds_done = updates = 0
    if args.kkt_tol > 0:
        # a run to tolerance can take minutes: it is made in segments of whole check intervals, with a
        # progress line after each (the only cost is one extra synchronisation per segment)
        seg = max(args.check_every, 1) * max(1, 20000 // max(args.check_every, 1))
        while True:
            info = g.run(min(seg, args.steps - rounds_done), args.kkt_tol, args.check_every)
            rounds_done += int(info.rounds_done)
            updates += int(info.updates_done)
            print(f"bench.py: {rounds_done} rounds, {time.perf_counter() - t0:.1f} s, objective {info.objective:.6f}, "
                  f"violation {info.kkt_violation:.3e}", file=sys.stderr, flush=True)
            if info.converged or rounds_done >= args.steps or info.rounds_done == 0:
                break
    else:
        info = g.run(args.steps)                # enqueues K rounds, waits once at the end
        rounds_done, updates = int(info.rounds_done), int(info.updates_done)
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    stage = g.stage_times() if args.profile_level else {"rounds": 0}
    g.set_tuning("profile_level", 0)
    f1 = float(info.objective)
    ms_per_step = wall / max(rounds_done, 1) * 1e3
    print(f"bench.py: timed region done ({rounds_done} rounds, {ms_per_step:.3f} ms each)", file=sys.stderr, flush=True)

    all_columns, viol = kkt_pass(g, p, args.shards, torch)
    g.close()

    streams = None
    if args.profile_level and args.shards == 1 and args.deps == "static" and p.layout == "dense":
        streams = stream_leg(fresh, p, args.steps, workload_name)

    # the same workload and round count under the two widenings of the schedule (not the headline)
    variants = None
    headline = (args.deps == "static" and args.shards == 1 and args.priority == "squared" and args.kkt_tol == 0
                and args.p_max == 0 and args.loss == "squared")
    if headline and not args.no_variants:
        variants = {}
        legs = {"shards4": dict(n_shards=4), "dynamic": dict(dynamic=True)}
        for name, extra in legs.items():
            kw = dict(y=p.y, lam=p.lam, rho=p.rho, eta=p.eta, l_prime=p.l_prime, seed=p.seed, **extra)
            v = pk.StradsLasso(**design_args(p), **kw)
            v.run(min(args.warmup, 10))
            v.close()
            v = pk.StradsLasso(**design_args(p), **kw)
            torch.cuda.synchronize()
            tv = time.perf_counter()
            iv = v.run(args.steps)
            torch.cuda.synchronize()
            wv = time.perf_counter() - tv
            variants[name] = {"value": round(int(iv.updates_done) / wv, 1), "unit": "updates/s",
                              "ms_per_step": round(wv / max(args.steps, 1) * 1e3, 4), "updates": int(iv.updates_done),
                              "objective_end": float(iv.objective)}
            v.close()
        print("bench.py: variants done", file=sys.stderr, flush=True)

    if args.pmc_calibration:
        a = torch.ones(1 << 28, dtype=torch.float32, device=dev)
        b = torch.empty_like(a)
        torch.cuda.synchronize()
        torch.add(a, 1.0, out=b)                 # 2^28 floats in, 2^28 floats out
        torch.cuda.synchronize()
        del a, b

    L, N = min(p.l_prime, p.j // max(1, args.shards)), p.n
    roofline = None
    if (args.profile_level and stage["rounds"] > 0 and stage["gram_tiles"] > 0 and p.layout in ("dense", "geno2")
            and args.deps == "static"):
        # does the launch carry the candidates' dot products?  (the library's rule, see "dots_with_gram")
        rides = (p.layout == "dense" and args.shards <= 1 and p.l_prime <= 4096
                 and "dots_with_gram=0" not in [t.replace(" ", "") for t in args.tune])
        rides = rides and tile_edge != 256
        roofline = gram_roofline(p, L, stage, workload_name, rides, tile_edge)

    # for scale: the library route for the same Step 2 (gather the candidate columns, then the vendor
    # GEMM on the panel and its transpose, fp32), timed live on this machine
    if roofline is not None and p.layout == "dense" and args.library_route:
        torch.backends.cuda.matmul.allow_tf32 = False
        idx = torch.randperm(p.j, device=dev)[:L]
        reps = 10 if float(N) * L * L < 1e12 else 2

        def _time(f):
            f()
            torch.cuda.synchronize()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for _ in range(reps):
                f()
            e1.record()
            torch.cuda.synchronize()
            return e0.elapsed_time(e1) / reps

        t_gather = _time(lambda: p.x[idx])
        panel = p.x[idx]
        t_mm = _time(lambda: panel @ panel.T)
        del panel
        roofline["library_route"] = {"what": "torch gather of the candidate columns + torch.mm(panel, panel.T), fp32",
                                     "gather_ms": round(t_gather, 5), "gemm_ms": round(t_mm, 5),
                                     "gemm_tflops_executed": round(2.0 * N * L * L / (t_mm * 1e-3) / 1e12, 2)}

    cpu = None
    if args.cpu_seconds > 0:
        host_bytes = 4.0 * p.n * p.j if p.layout == "dense" else 0.0
        gram_macs = 0.5 * p.n * float(L) * L if p.layout != "csc" else 0.0
        if p.layout == "dense" and headline and (host_bytes > 16e9 or gram_macs > 3e10):
            cpu = cpu_baseline_large(p, args, fresh, ms_per_step, args.cpu_seconds)
        else:
            cpu = cpu_baseline_rounds(p, args, rounds_done, wall, args.cpu_seconds)
            cpu["gpu_seconds_for_the_same_rounds"] = round(cpu["legs"]["all_cores"]["rounds"] * ms_per_step * 1e-3, 6)
        print("bench.py: oracle timing done", file=sys.stderr, flush=True)

    secondary = None
    if args.workload == DEFAULT_WORKLOAD and headline and not args.no_secondary:
        secondary = {"c2_dense_block_corr": secondary_c2(args, pk, si, torch, dev)}

    out = {
        "metric": "coordinate_updates_per_sec", "value": round(updates / wall, 1), "unit": "updates/s",
        "n_gpus": 1, "steps": rounds_done, "warmup": args.warmup, "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": workload_name, "n": p.n, "j": p.j, "l_prime": p.l_prime, "rho": p.rho,
                   "eta": p.eta, "lambda": p.lam, "rounds": rounds_done, "deps": args.deps, "priority": args.priority,
                   "p_max": args.p_max, "shards": args.shards, "loss": args.loss, "parallelism": "1 GPU",
                   "x_bytes": 4.0 * p.n * p.j if p.layout == "dense" else None, "note": fit_note},
        "rounds_per_s": round(rounds_done / wall, 2), "updates": updates, "seconds": round(wall, 4),
        "kkt_tol": args.kkt_tol, "converged": int(info.converged), "graph_replays": int(info.graph_replays),
        "objective_start": f0, "objective_end": f1, "kkt_violation_end": viol,
        "roofline": roofline,
        "hbm_pass": all_columns,
        "stage_ms": {k: round(v, 5) for k, v in stage.items() if k != "rounds"},
        "hbm_streams": streams,
        "cpu_baseline": cpu,
        "variants": variants,
        "secondary": secondary,
        "input_generation_s": round(t_gen, 2),
    }
    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
