"""Perturbation size under the checkpoint strategies of Section 5.4, on a synthetic
drifting store, using only the library's entry points.

A store drifts for `iters` iterations (every block moves by its own heavy-tailed scale per
iteration).  Five set-ups keep their own running checkpoint c:

  traditional   full checkpoint every `period` iterations, FULL recovery  (||c - x||)
  partial       full checkpoint every `period` iterations, partial recovery of the lost set
  priority      fraction 1/period of the blocks every iteration, chosen by scar_select_topk
  round         same fraction, chosen round-robin (scar_select_round)
  random        same fraction, chosen uniformly at random (scar_select_random)

so that all of them write the same number of blocks per `period` iterations (Section 4.2).
After every iteration a failure that loses a fresh random `lost_fraction` of the blocks is
imagined and the perturbation it would cause, ||c_S - x_S|| (Appendix A.3), is measured with
scar_perturbation_norm (nothing is recovered, so the run continues undisturbed).  The
iteration-cost bound of Theorem 3.1 grows with this norm; the paper's datasets and trainers
are not here, so the norm is what this study can report.

    python -m paper_1810_07354_amd.strategy_study [--blocks N] [--block-len L] [--iters T]
"""
import argparse
import json

import numpy as np
import torch

from . import scar
from . import workloads as wl


def run(n_blocks=16384, block_len=1024, iters=48, period=8, lost_fraction=0.5, seed=0, device="cuda:0"):
    g = torch.Generator(device=device)
    g.manual_seed(seed)
    n = n_blocks * block_len
    x = torch.empty(n, dtype=torch.float32, device=device).normal_(0.0, 0.02, generator=g)
    # per-block drift scale: log-normal, so a few blocks move much more than the rest
    scale = torch.empty(n_blocks, device=device).log_normal_(-7.0, 1.0, generator=g)
    ws = scar.new_workspace(n_blocks, device)
    k = wl.k_of_fraction(1.0 / period, n_blocks)
    n_lost = int(n_blocks * lost_fraction)
    names = ["traditional", "partial", "priority", "round", "random"]
    ckpt = {name: x.clone() for name in names}            # running checkpoint = x(0) (Section 4.2)
    everything = torch.arange(n_blocks, dtype=torch.int32, device=device)
    norms = {name: [] for name in names}
    for t in range(1, iters + 1):
        x.view(n_blocks, block_len).add_(
            torch.empty(n_blocks, block_len, device=device).normal_(generator=g) * scale[:, None])
        for name in names:
            c = ckpt[name]
            if name in ("traditional", "partial"):
                if t % period == 0:
                    scar.checkpoint_commit(x, c, block_len, everything)
            else:
                if name == "priority":
                    idx = scar.select_topk(scar.block_scores(x, c, block_len), k, ws)
                elif name == "round":
                    idx = scar.select_round(n_blocks, k, (t - 1) * k, device)
                else:
                    idx = scar.select_random(n_blocks, k, seed, t, ws)
                scar.checkpoint_commit(x, c, block_len, idx)
        lost = torch.from_numpy(
            wl.random_lost_blocks(n_blocks, n_lost, seed + 1000 + t).view(np.int32).copy()).to(device)
        for name in names:
            which = None if name == "traditional" else lost
            out = scar.perturbation_norm(x, ckpt[name], block_len, which, ws)
            norms[name].append(scar.read_norm(out)[1])
    mean = {name: float(np.mean(v)) for name, v in norms.items()}
    return {"n_blocks": n_blocks, "block_len": block_len, "iters": iters, "period": period,
            "fraction_per_checkpoint": 1.0 / period, "lost_fraction": lost_fraction,
            "mean_perturbation_norm": mean,
            "relative_to_traditional": {n_: mean[n_] / mean["traditional"] for n_ in names}}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--blocks", type=int, default=16384)
    ap.add_argument("--block-len", type=int, default=1024)
    ap.add_argument("--iters", type=int, default=48)
    ap.add_argument("--period", type=int, default=8)
    ap.add_argument("--lost-fraction", type=float, default=0.5)
    ap.add_argument("--contraction", type=float, default=None,
                    help="contraction factor c of the training update: also print Theorem 3.1's bound")
    ap.add_argument("--dist0", type=float, default=100.0, help="||x(0) - x*|| for the bound")
    ap.add_argument("--fail-at", type=int, default=50, help="iteration of the failure for the bound")
    args = ap.parse_args()
    res = run(args.blocks, args.block_len, args.iters, args.period, args.lost_fraction)
    if args.contraction is not None:
        from . import bound
        res["iteration_cost_bound"] = {
            name: bound.iteration_cost_bound([norm], args.contraction, args.dist0, args.fail_at)
            for name, norm in res["mean_perturbation_norm"].items()}
    print(json.dumps(res))


if __name__ == "__main__":
    main()
