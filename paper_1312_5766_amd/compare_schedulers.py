#!/usr/bin/env python3
"""Objective against rounds and time for the schedulers Section 5.1 compares, on one workload.

  strads          priority (delta beta)^2 + eta, dependency check among all candidates (Algorithm 1)
  strads-dynamic  the same priority, dependencies only between candidates that move (Section 1,
                  "Dynamic Block Structures"; Step 4)
  static-corr     uniform draw, same dependency check ("static correlation scheduler")
  shotgun         uniform draw, no check; --shotgun-p coordinates per round

Every scheduler starts from beta = 0 on the same synthetic inputs and runs --rounds rounds; the
objective of eq. (1) is read every --every rounds (one stream synchronisation each).  Prints one
JSON line per scheduler.  Needs a GPU: all rounds run in the library's HIP kernels.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--workload", default="c2_dense_block_corr")
    ap.add_argument("--rounds", type=int, default=2000)
    ap.add_argument("--every", type=int, default=100)
    ap.add_argument("--shotgun-p", type=int, default=0, help="coordinates per Shotgun round (0 = all L' drawn)")
    args = ap.parse_args()

    import torch
    import paper_1312_5766_amd as pk
    from synth import lasso_inputs as si

    pk.load()
    dev = torch.device("cuda:0")
    p = si.make(args.workload, device=dev)
    base = dict(y=p.y, lam=p.lam, rho=p.rho, eta=p.eta, l_prime=p.l_prime, seed=p.seed)
    if p.layout == "dense":
        base["x"] = p.x
    else:
        base.update(values=p.values, row_idx=p.row_idx, col_ptr=p.col_ptr, n=p.n)
    modes = {
        "strads": dict(),
        "strads-dynamic": dict(dynamic=True),
        "static-corr": dict(priority="uniform"),
        "shotgun": dict(priority="uniform", no_deps=True, p_max=args.shotgun_p),
    }
    for name, kw in modes.items():
        g = pk.StradsLasso(**base, **kw)
        g.round()                               # first-launch costs stay out of the clock
        torch.cuda.synchronize()
        g.close()
        g = pk.StradsLasso(**base, **kw)
        traj = [(0, 0.0, g.objective())]
        done, t_run = 0, 0.0
        while done < args.rounds:
            n = min(args.every, args.rounds - done)
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            info = g.run(n)
            torch.cuda.synchronize()
            t_run += time.perf_counter() - t0
            done += n
            traj.append((done, round(t_run * 1e3, 3), float(info.objective)))
            if not (info.objective == info.objective) or info.objective > 1e30:
                break
        print(json.dumps({"scheduler": name, "workload": args.workload, "rounds": done,
                          "ms_total": round(t_run * 1e3, 2), "kkt_violation": g.kkt(),
                          "trajectory_round_ms_objective": traj}))
        g.close()
    return 0


if __name__ == "__main__":
    sys.exit(main())
