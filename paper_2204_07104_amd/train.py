"""Training driver: the loop the paper's experiments run (Section 5.1), on a seeded synthetic tensor.

    python -m paper_2204_07104_amd.train [--dims 3000 2000 1000] [--nnz 3300000] [--J 8] [--R 8] ...

Every step draws a fresh sample set Psi and takes one SGD step with the step sizes
gamma_t = alpha / (1 + beta t^1.5) (Section 5.1, `ftk_step_size`); every `--report-every` steps RMSE and
MAE are taken on a held-out set Gamma that training never sees (`ftk_evaluate`).  The real datasets of the
paper are not available here, so the tensor is planted: a rank-`--planted-rank` CP model with factors
U(0.3, 1) plus Gaussian noise, observed at uniformly random coordinates, split at random into Omega and
Gamma.  Argument marshalling and the loop only: every step of the method runs in the library.
"""
from __future__ import annotations

import argparse
import sys
import time
from typing import List, Optional, Sequence, Tuple

import numpy as np

from . import binding


def planted_tensor(dims: Sequence[int], nnz: int, rank: int, noise: float,
                   seed: int) -> Tuple[List[np.ndarray], np.ndarray]:
    """Coordinates (uniform, with repetition) and values sum_r prod_n U^(n)[i_n, r] + noise * N(0, 1)."""
    rng = np.random.default_rng(seed)
    factors = [rng.uniform(0.3, 1.0, (int(d), rank)) for d in dims]
    idx = [rng.integers(0, int(d), nnz).astype(np.int32) for d in dims]
    terms = np.ones((nnz, rank))
    for n in range(len(dims)):
        terms *= factors[n][idx[n]]
    vals = (terms.sum(axis=1) + noise * rng.standard_normal(nnz)).astype(np.float32)
    return idx, vals


def train(dims: Sequence[int], nnz: int, J: Sequence[int], R: int, n_samples: int, steps: int,
          alpha_A: float, beta_A: float, alpha_B: float, beta_B: float, lambda_A: float, lambda_B: float,
          holdout: float = 0.1, planted_rank: int = 4, noise: float = 0.05, seed: int = 1,
          mode: str = "sync", sampling: str = "entries", report_every: int = 50,
          out=sys.stdout) -> List[Tuple[int, float, float]]:
    """Runs the loop; returns [(step, RMSE on Gamma, MAE on Gamma)] at step 0 and at every report."""
    idx, vals = planted_tensor(dims, nnz, planted_rank, noise, seed)
    n_test = max(1, int(round(nnz * holdout)))
    n_train = nnz - n_test
    if n_train < 1:
        raise ValueError("nothing left to train on")
    tr_idx, tr_vals = [np.ascontiguousarray(i[:n_train]) for i in idx], np.ascontiguousarray(vals[:n_train])
    te_idx, te_vals = [np.ascontiguousarray(i[n_train:]) for i in idx], np.ascontiguousarray(vals[n_train:])
    history: List[Tuple[int, float, float]] = []
    with binding.FastTucker(dims, tr_idx, tr_vals, J, R, seed + 1) as ft:
        ft.ftk_set_mode({"sync": binding.FTK_SYNC, "hogwild": binding.FTK_HOGWILD,
                         "modewise": binding.FTK_HOGWILD_MODEWISE}[mode])
        if sampling == "tiles":
            ft.ftk_set_sampling(binding.FTK_SAMPLE_TILES)
        print("# %d-order tensor %s, |Omega| = %d, |Gamma| = %d, J = %s, R = %d, |Psi| = %d, kernel %s, %s step"
              % (len(dims), "x".join(str(d) for d in dims), n_train, n_test, list(J), R, n_samples,
                 ft.ftk_kernel_name(), mode), file=out)
        print("# %6s %11s %11s %10s %10s %9s" % ("step", "lr_A", "lr_B", "RMSE(G)", "MAE(G)", "seconds"), file=out)
        t0 = time.perf_counter()

        def report(t: int, lr_A: float, lr_B: float) -> None:
            rmse, mae = ft.ftk_evaluate(te_idx, te_vals)
            history.append((t, rmse, mae))
            print("  %6d %11.4e %11.4e %10.6f %10.6f %9.3f" % (t, lr_A, lr_B, rmse, mae, time.perf_counter() - t0),
                  file=out, flush=True)

        report(0, alpha_A, alpha_B)
        for t in range(steps):
            lr_A = binding.ftk_step_size(alpha_A, beta_A, t)
            lr_B = binding.ftk_step_size(alpha_B, beta_B, t)
            ft.ftk_sample(seed * 1_000_003 + t, n_samples)
            ft.ftk_sgd_step(lr_A, lr_B, lambda_A, lambda_B)
            if (t + 1) % report_every == 0 or t + 1 == steps:
                report(t + 1, lr_A, lr_B)
    return history


def main(argv: Optional[Sequence[str]] = None) -> int:
    ap = argparse.ArgumentParser(description=__doc__.split("\n")[0])
    ap.add_argument("--dims", type=int, nargs="+", default=[3000, 2000, 1000])
    ap.add_argument("--nnz", type=int, default=3_300_000, help="stored entries before the split into Omega and Gamma")
    ap.add_argument("--holdout", type=float, default=0.1, help="fraction of the entries held out as Gamma")
    ap.add_argument("--J", type=int, nargs="+", default=[8], help="one rank for all modes, or one per mode")
    ap.add_argument("--R", type=int, default=8)
    ap.add_argument("--psi", type=int, default=300_000, help="|Psi| per step")
    ap.add_argument("--steps", type=int, default=300)
    ap.add_argument("--alpha-A", type=float, default=1e-3)
    ap.add_argument("--beta-A", type=float, default=0.005)
    ap.add_argument("--alpha-B", type=float, default=1.0)
    ap.add_argument("--beta-B", type=float, default=0.005)
    ap.add_argument("--lambda-A", type=float, default=1e-3)
    ap.add_argument("--lambda-B", type=float, default=1e-3)
    ap.add_argument("--planted-rank", type=int, default=4)
    ap.add_argument("--noise", type=float, default=0.05)
    ap.add_argument("--seed", type=int, default=1)
    ap.add_argument("--mode", default="sync", choices=["sync", "hogwild", "modewise"])
    ap.add_argument("--sampling", default="entries", choices=["entries", "tiles"])
    ap.add_argument("--report-every", type=int, default=50)
    a = ap.parse_args(argv)
    J = a.J * len(a.dims) if len(a.J) == 1 else a.J
    if len(J) != len(a.dims):
        ap.error("--J takes one value or one per mode")
    train(a.dims, a.nnz, J, a.R, a.psi, a.steps, a.alpha_A, a.beta_A, a.alpha_B, a.beta_B, a.lambda_A, a.lambda_B,
          a.holdout, a.planted_rank, a.noise, a.seed, a.mode, a.sampling, a.report_every)
    return 0


if __name__ == "__main__":
    sys.exit(main())
