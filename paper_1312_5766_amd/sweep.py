"""Size sweep of the three per-round kernels that have a roofline: the candidate Gram (fp32 MFMA), the
dot products of the kept set and the residual update (HBM streams).

    python -m paper_1312_5766_amd.sweep [--rows 50000] [--rounds 6]

Each point is a synthetic i.i.d. design with exactly L' columns (so every column is a candidate in
every round), a threshold no pair reaches (every candidate is kept) and lambda = 0 (every kept
coordinate moves): k = k1 = L'.  Kernel times are the library's own per-stage HIP events
(strads_lasso_stage_times), averaged over the timed rounds.  Algorithmic work: Gram N L'(L'-1) flop;
dots 4 N (k+1) bytes; residual 4 N k1 + 8 N bytes.
"""
import argparse
import json
import sys

import torch

import paper_1312_5766_amd as pk

MFMA_FP32_PEAK_TFLOPS = 157.3
HBM_PEAK_GBPS = 8000.0


def point(n: int, l: int, rounds: int, dev) -> dict:
    g = torch.Generator(device=dev)
    g.manual_seed(1000003 * n + l)
    x = torch.randn((l, n), generator=g, device=dev, dtype=torch.float32)
    x /= x.norm(dim=1, keepdim=True)
    y = torch.randn(n, generator=g, device=dev, dtype=torch.float32)
    s = pk.StradsLasso(x=x, y=y, lam=0.0, rho=2.0, eta=1e-6, l_prime=l, seed=0)
    for _ in range(2):
        s.round()
    # every round starts from the same state, so the values stay finite whatever Jacobi does with L' columns
    beta, dbeta, r, _t = [a.clone() if isinstance(a, torch.Tensor) else a for a in s.get_state()]
    s.set_tuning("profile_rounds", rounds)
    s.set_tuning("profile_level", 2)       # every stage bracketed by events
    kept = moved = 0
    for t in range(rounds):
        s.set_state(beta, dbeta, r, 2 + t)
        info = s.round(want_info=True)
        kept += info.n_kept
        moved += info.n_moved
    st = s.stage_times()
    s.set_tuning("profile_level", 0)
    s.close()
    k, k1 = kept / rounds, moved / rounds
    gram_tf = n * l * (l - 1) / (st["gram_tiles"] * 1e-3) / 1e12 if st["gram_tiles"] > 0 else 0.0
    dots_gb = 4.0 * n * (k + 1) / (st["update"] * 1e-3) / 1e9
    res_gb = (4.0 * n * k1 + 8.0 * n) / (st["residual"] * 1e-3) / 1e9
    return {"n": n, "l_prime": l, "k": k, "k1": k1,
            "gram_us": round(st["gram_tiles"] * 1e3, 1), "gram_tflops": round(gram_tf, 1),
            "gram_frac": round(gram_tf / MFMA_FP32_PEAK_TFLOPS, 3),
            "dots_mb": round(4e-6 * n * (k + 1), 1), "dots_us": round(st["update"] * 1e3, 1),
            "dots_gbps": round(dots_gb), "dots_frac": round(dots_gb / HBM_PEAK_GBPS, 3),
            "residual_us": round(st["residual"] * 1e3, 1), "residual_gbps": round(res_gb),
            "residual_frac": round(res_gb / HBM_PEAK_GBPS, 3)}


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--rows", type=int, nargs="+", default=[10000, 50000])
    ap.add_argument("--l-prime", type=int, nargs="+", default=[32, 128, 256, 512, 1024, 2048, 4096, 8192])
    ap.add_argument("--rounds", type=int, default=6)
    ap.add_argument("--json", action="store_true")
    args = ap.parse_args()
    pk.load()
    dev = torch.device("cuda:0")
    rows = []
    hdr = (f"{'N':>6} {'L=k':>5} | {'gram us':>9} {'TFLOP/s':>8} {'frac':>5} | {'dots MB':>8} {'us':>7} {'GB/s':>6} {'frac':>5} | "
           f"{'resid us':>8} {'GB/s':>6} {'frac':>5}")
    if not args.json:
        print(hdr, flush=True)
    for n in args.rows:
        for l in args.l_prime:
            if 4.0 * n * l > 8e9:
                continue
            p = point(n, l, args.rounds, dev)
            rows.append(p)
            if not args.json:
                print(f"{p['n']:>6} {p['l_prime']:>5} | {p['gram_us']:>9} {p['gram_tflops']:>8} {p['gram_frac']:>5} | "
                      f"{p['dots_mb']:>8} {p['dots_us']:>7} {p['dots_gbps']:>6} {p['dots_frac']:>5} | "
                      f"{p['residual_us']:>8} {p['residual_gbps']:>6} {p['residual_frac']:>5}", flush=True)
    if args.json:
        print(json.dumps(rows))
    return 0


if __name__ == "__main__":
    sys.exit(main())
