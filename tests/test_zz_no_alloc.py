"""ftk_sgd_step_noalloc, the entry point for callers that cannot allocate: its partial tables live in the
library's static device array.  Held to ftk_sgd_step (and to the oracle) at the parity bar, on two calls in
a row of which the second has the smaller sample set, so the second call finds the array full of the first
call's tables."""
import numpy as np
import pytest

import oracle
from paper_2204_07104_amd import binding, synth

pytestmark = pytest.mark.gpu

RTOL, ATOL = 1e-4, 1e-6


def close(got, want, what):
    for n, (g, w) in enumerate(zip(got, want)):
        err = np.abs(g.astype(np.float64) - w.astype(np.float64))
        excess = float((err - (ATOL + RTOL * np.abs(w.astype(np.float64)))).max())
        assert excess <= 0.0, "%s[%d]: %.3e over tolerance" % (what, n, excess)


@pytest.mark.parametrize("kernel,dims,zipf,J,R", [
    ("mfma16", (9_000, 2_500, 300), (1.1, 1.1, None), (16, 16, 16), 16),
    ("tiled", (5_000, 1_200, 90), (1.1, None, None), (20, 32, 12), 24),
    # 64-wide blocks: the factor-row tables are part of the context's parameter allocation, the core-gradient tables use the static array
    ("tiled", (5_000, 1_200, 90), (1.1, None, None), (64, 40, 52), 48),
])
def test_step_without_allocation_matches_the_allocating_step(kernel, dims, zipf, J, R):
    print("[case] no-alloc step, kernel=%s" % kernel, flush=True)
    w = synth.tiny_workload(3, dims, 150_000, J, R, 1, seed=83, values="int1to5", zipf=zipf)
    scale = max(1.0, float(R) * float(np.prod([j / 16.0 for j in J])))
    lr_A, lr_B = 2e-4 / scale ** 2, 1e-3 / scale ** 2
    idx, vals = synth.make_tensor(w)
    A, B = oracle.init_factors(w.init_seed, w.dims, w.J, w.R)
    flags = binding.FTK_LAYOUT_EXACT
    with binding.FastTucker(w.dims, idx, vals, w.J, w.R, w.init_seed, flags=flags) as ref, \
            binding.FastTucker(w.dims, idx, vals, w.J, w.R, w.init_seed, flags=flags) as ft:
        for f in (ref, ft):
            f.ftk_set_kernel(kernel)
            assert f.ftk_kernel_name() == kernel
        ft.ftk_set_timing(True)      # must not make the call create events
        for t, M in enumerate([40_013, 3_001]):     # the second call is the smaller one
            pos = oracle.sample_positions(700 + t, M, w.nnz)
            ref.ftk_sample(700 + t, M)
            ref.ftk_sgd_step(lr_A, lr_B, w.lambda_A, w.lambda_B)
            ft.ftk_sample(700 + t, M)
            ft.ftk_sgd_step_noalloc(lr_A, lr_B, w.lambda_A, w.lambda_B)
            oracle.sgd_step_sync(w.dims, idx, vals, A, B, pos, lr_A, lr_B, w.lambda_A, w.lambda_B)
            rA, rB = ref.ftk_get_factors()
            gA, gB = ft.ftk_get_factors()
            close(gA, rA, "A vs ftk_sgd_step, call %d" % t)
            close(gB, rB, "B vs ftk_sgd_step, call %d" % t)
            for g, o in zip(gA + gB, A + B):
                err = np.abs(g.astype(np.float64) - o)
                assert float((err - (t + 1) * (ATOL + RTOL * np.abs(o))).max()) <= 0.0, "vs oracle, call %d" % t
        assert ft.ftk_get_timing(binding.FTK_K_GRAD)[1] == 0      # nothing was recorded: no events were made
        # the two entry points mix freely on one context
        ft.ftk_sample(900, 5_000)
        ft.ftk_sgd_step(lr_A, lr_B, w.lambda_A, w.lambda_B)
        ft.ftk_sgd_step_noalloc(lr_A, lr_B, w.lambda_A, w.lambda_B)
        ref.ftk_sample(900, 5_000)
        ref.ftk_sgd_step(lr_A, lr_B, w.lambda_A, w.lambda_B)
        ref.ftk_sgd_step(lr_A, lr_B, w.lambda_A, w.lambda_B)
        close(ft.ftk_get_factors()[0], ref.ftk_get_factors()[0], "A after mixing the entry points")
        assert max(float(np.abs(a - a0).max()) for a, a0 in zip(A, oracle.init_factors(w.init_seed, w.dims, w.J, w.R)[0])) > 1e-3


def test_refusals_of_the_step_without_allocation():
    print("[case] no-alloc step, refusals", flush=True)
    w = synth.tiny_workload(3, (50, 40, 30), 2_000, (8, 8, 8), 8, 500)
    idx, vals = synth.make_tensor(w)
    with binding.FastTucker(w.dims, idx, vals, w.J, w.R) as ft:
        with pytest.raises(binding.FtkError) as e:
            ft.ftk_sgd_step_noalloc(1e-3, 1e-3, 0.0, 0.0)      # no Psi yet
        assert e.value.code == binding.FTK_ESTATE
        ft.ftk_sample(1, 500)
        ft.ftk_set_kernel("generic")
        with pytest.raises(binding.FtkError) as e:
            ft.ftk_sgd_step_noalloc(1e-3, 1e-3, 0.0, 0.0)
        assert e.value.code == binding.FTK_EUNSUPPORTED
        ft.ftk_set_kernel("auto")
        ft.ftk_sgd_step_noalloc(1e-3, 1e-3, 0.0, 0.0)
    # a shape whose partial tables exceed the static array: one mode, so that nearly all of a CU's LDS is table
    # (about 2 100 rows of 64 bytes per workgroup, 34 MB over 256 workgroups), and every row hit often enough to be in it
    w = synth.tiny_workload(1, (6_000,), 100_000, (16,), 16, 600_000)
    idx, vals = synth.make_tensor(w)
    with binding.FastTucker(w.dims, idx, vals, w.J, w.R) as ft:
        ft.ftk_sample(1, w.n_samples)
        with pytest.raises(binding.FtkError) as e:
            ft.ftk_sgd_step_noalloc(1e-12, 1e-12, 0.0, 0.0)
        assert e.value.code == binding.FTK_EUNSUPPORTED and "bytes" in str(e.value)
        ft.ftk_sgd_step(1e-12, 1e-12, 0.0, 0.0)               # the allocating call still serves it
