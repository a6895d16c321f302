"""Parity of the HIP path against the CPU oracle (needs an MI355X: run with -m gpu).

Bars (from the benchmark spec): sampled index sets bit-exact; after one synchronous step every
parameter within 1e-4 relative / 1e-6 absolute of the oracle; RMSE over 10 steps within 1e-3
relative.  Everything goes through the C ABI (binding.FastTucker); every input is seeded.
"""
import numpy as np
import pytest

import oracle
from paper_2204_07104_amd import binding, synth

pytestmark = pytest.mark.gpu

RTOL, ATOL = 1e-4, 1e-6


def announce(msg):
    print("[case] " + msg, flush=True)


def assert_params_close(got, want, what):
    for n, (g, w) in enumerate(zip(got, want)):
        err = np.abs(g.astype(np.float64) - w.astype(np.float64))
        bound = ATOL + RTOL * np.abs(w.astype(np.float64))
        worst = float((err - bound).max())
        assert worst <= 0.0, "%s[%d]: max excess over tolerance %.3e (max abs err %.3e)" % (what, n, worst, float(err.max()))


# step sizes for one-step comparisons: large enough that the most frequently hit rows and the core
# factors move by percents (the benchmark's own step sizes are chosen for many stable steps)
TEST_STEP_SIZES = {
    "C1": dict(lr_A=1e-3, lr_B=1e-3),
    "C2": dict(lr_A=1e-8, lr_B=1e-2),
    "C3": dict(lr_A=1e-11, lr_B=1e-4),
    "C4": dict(lr_A=4e-3, lr_B=1.0),
    "C5": dict(lr_A=5e-13, lr_B=1e-6),
}


def oracle_state(w):
    return oracle.init_factors(w.init_seed, w.dims, w.J, w.R)


def one_step_case(w, idx, vals, A0=None, B0=None, seed=None, kernel=None, tiles=False, flags=0):
    seed = w.sample_seed0 if seed is None else seed
    draw = oracle.sample_positions_tiles if tiles else oracle.sample_positions
    with binding.FastTucker(w.dims, idx, vals, w.J, w.R, w.init_seed, flags=flags) as ft:
        if tiles:
            ft.ftk_set_sampling(binding.FTK_SAMPLE_TILES)
        if kernel:
            ft.ftk_set_kernel(kernel)
            if kernel != "auto":
                assert ft.ftk_kernel_name() == kernel.split(":")[0]
        if A0 is not None:
            ft.ftk_set_factors(A0, B0)
            A, B = [a.copy() for a in A0], [b.copy() for b in B0]
        else:
            A, B = oracle_state(w)
            gA, gB = ft.ftk_get_factors()
            for x, y in zip(gA + gB, A + B):
                assert np.array_equal(x, y), "initial parameters differ from the oracle's"
        ft.ftk_sample(seed, w.n_samples)
        pos = ft.ftk_get_samples()
        want = draw(seed, w.n_samples, w.nnz)
        assert np.array_equal(pos, want), "sample set differs from the oracle's"
        ft.ftk_sgd_step(w.lr_A, w.lr_B, w.lambda_A, w.lambda_B)
        gA, gB = ft.ftk_get_factors()
    oracle.sgd_step_sync(w.dims, idx, vals, A, B, want, w.lr_A, w.lr_B, w.lambda_A, w.lambda_B)
    assert_params_close(gA, A, "A")
    assert_params_close(gB, B, "B")
    return gA, gB, A, B


# ------------------------------------------------------------------------------------------------
# sampling and initialisation: bit-exact
# ------------------------------------------------------------------------------------------------
@pytest.mark.parametrize("nnz,M,seed", [(1, 5, 0), (3, 64, 7), (100_000, 1, 1000), (100_000, 63, 1001),
                                        (100_000, 65, 1002), (100_000, 10_000, 1003),
                                        (999_983, 262_145, 0xFEDCBA9876543210), (50_000_000, 100_003, 42)])
def test_sample_set_bit_exact(nnz, M, seed):
    announce("sample nnz=%d M=%d seed=%d" % (nnz, M, seed))
    idx = [np.zeros(nnz, dtype=np.int32)]
    vals = np.zeros(nnz, dtype=np.float32)
    with binding.FastTucker((1,), idx, vals, (1,), 1) as ft:
        ft.ftk_sample(seed, M)
        got = ft.ftk_get_samples()
        # a second draw with another seed replaces Psi; drawing fewer keeps the buffers
        ft.ftk_sample(seed + 1, max(1, M // 2))
        got2 = ft.ftk_get_samples()
    assert np.array_equal(got, oracle.sample_positions(seed, M, nnz))
    assert np.array_equal(got2, oracle.sample_positions(seed + 1, max(1, M // 2), nnz))


@pytest.mark.parametrize("nnz,M,seed", [(1, 70, 3), (50, 130, 4), (64, 64, 5), (65, 200, 6), (1000, 1000, 7),
                                        (100_000, 10_001, 8), (999_983, 262_145, 2**63 + 11)])
def test_tile_sampling_sample_set_bit_exact(nnz, M, seed):
    """The tile-sampling variant: positions (in the caller's numbering) bit-exact against the oracle,
    and switching back restores the default rule."""
    announce("tile sampling nnz=%d M=%d seed=%d" % (nnz, M, seed))
    idx = [np.zeros(nnz, dtype=np.int32)]
    vals = np.zeros(nnz, dtype=np.float32)
    with binding.FastTucker((1,), idx, vals, (1,), 1) as ft:
        ft.ftk_set_sampling(binding.FTK_SAMPLE_TILES)
        ft.ftk_sample(seed, M)
        got = ft.ftk_get_samples()
        ft.ftk_set_sampling(binding.FTK_SAMPLE_ENTRIES)
        back = ft.ftk_get_samples()
        with pytest.raises(binding.FtkError):
            ft.ftk_set_sampling(2)
    assert np.array_equal(got, oracle.sample_positions_tiles(seed, M, nnz))
    assert np.array_equal(back, oracle.sample_positions(seed, M, nnz))


@pytest.mark.parametrize("kernel", ["auto", "generic", "tiled"])
@pytest.mark.parametrize("order,dims,nnz,J,R,M", [
    (3, (700, 500, 90), 30_011, (16, 16, 16), 16, 7_013),
    (3, (300, 200, 50), 20_000, (24, 40, 9), 20, 5_000),
    (4, (60, 50, 40, 30), 9_999, (8, 8, 8, 8), 8, 3_001),
])
def test_one_step_with_tile_sampling(order, dims, nnz, J, R, M, kernel):
    """One synchronous step on a tile-sampled Psi, every kernel variant: the entries are read from the
    reordered copy of the tensor, the gradients must be those of the oracle's positions."""
    announce("tile-sampled step order=%d J=%r kernel=%s" % (order, J, kernel))
    w = synth.tiny_workload(order, dims, nnz, J, R, M, seed=21 + order, values="normal")
    w = synth.replace(w, lr_A=1e-4, lr_B=1e-4)
    idx, vals = synth.make_tensor(w)
    one_step_case(w, idx, vals, kernel=kernel, tiles=True)


def test_initial_parameters_bit_exact():
    announce("init")
    w = synth.tiny_workload(3, (1000, 37, 5), 50, (8, 5, 3), 6, 10)
    idx, vals = synth.make_tensor(w)
    for seed in (0, 1, 0xABCDEF0123456789):
        with binding.FastTucker(w.dims, idx, vals, w.J, w.R, seed) as ft:
            gA, gB = ft.ftk_get_factors()
        A, B = oracle.init_factors(seed, w.dims, w.J, w.R)
        for x, y in zip(gA + gB, A + B):
            assert np.array_equal(x, y)


# ------------------------------------------------------------------------------------------------
# one synchronous step
# ------------------------------------------------------------------------------------------------
def test_c1_one_step_and_ten_step_rmse():
    w = synth.WORKLOADS["C1"]
    announce("C1 full size")
    idx, vals = synth.make_tensor(w)
    one_step_case(w, idx, vals)
    A, B = oracle_state(w)
    with binding.FastTucker(w.dims, idx, vals, w.J, w.R, w.init_seed) as ft:
        r0 = ft.ftk_rmse()
        assert r0 == pytest.approx(oracle.rmse(w.dims, idx, vals, A, B), rel=1e-5)
        prev = r0
        for t in range(10):
            ft.ftk_sample(w.sample_seed0 + t, w.n_samples)
            ft.ftk_sgd_step(w.lr_A, w.lr_B, w.lambda_A, w.lambda_B)
            pos = oracle.sample_positions(w.sample_seed0 + t, w.n_samples, w.nnz)
            oracle.sgd_step_sync(w.dims, idx, vals, A, B, pos, w.lr_A, w.lr_B, w.lambda_A, w.lambda_B)
            got, want = ft.ftk_rmse(), oracle.rmse(w.dims, idx, vals, A, B)
            assert got == pytest.approx(want, rel=1e-3), "step %d" % t
            assert got < prev
            prev = got
        assert ft.ftk_mae() == pytest.approx(oracle.errors(w.dims, idx, vals, A, B)[1], rel=1e-3)


def test_ten_steps_rmse_scaled_c2_both_kernels():
    """10 synchronous steps on the C2 recipe at reduced size (J = R = 16: the matrix-core kernels),
    RMSE after every step within 1e-3 relative of the oracle's, for the specialised and the generic
    gradient kernel, and for the specialised kernel under the tile-sampling rule."""
    w = synth.WORKLOADS["C2"].scaled(nnz=300_000, n_samples=30_000, dims=(4_800, 1_777, 220))
    w = synth.replace(w, lr_A=2e-7, lr_B=1e-4)
    idx, vals = synth.make_tensor(w)
    for kernel, tiles in (("auto", False), ("generic", False), ("auto", True)):
        announce("10 steps scaled C2, kernel=%s%s" % (kernel, ", tile sampling" if tiles else ""))
        draw = oracle.sample_positions_tiles if tiles else oracle.sample_positions
        A, B = oracle_state(w)
        with binding.FastTucker(w.dims, idx, vals, w.J, w.R, w.init_seed) as ft:
            ft.ftk_set_kernel(kernel)
            if tiles:
                ft.ftk_set_sampling(binding.FTK_SAMPLE_TILES)
            assert ft.ftk_kernel_name() == ("mfma16" if kernel == "auto" else "generic")
            first = None
            for t in range(10):
                ft.ftk_sample(w.sample_seed0 + t, w.n_samples)
                ft.ftk_sgd_step(w.lr_A, w.lr_B, w.lambda_A, w.lambda_B)
                pos = draw(w.sample_seed0 + t, w.n_samples, w.nnz)
                oracle.sgd_step_sync(w.dims, idx, vals, A, B, pos, w.lr_A, w.lr_B, w.lambda_A, w.lambda_B)
                got, want = ft.ftk_rmse(), oracle.rmse(w.dims, idx, vals, A, B)
                assert got == pytest.approx(want, rel=1e-3), "step %d" % t
                first = got if first is None else first
            assert got < first          # it learns
            gA, gB = ft.ftk_get_factors()
        # after 10 steps the parameters themselves are still close (errors do not blow up)
        for g, o in zip(gA + gB, A + B):
            assert float(np.abs(g.astype(np.float64) - o).max()) <= 1e-3 * (1.0 + float(np.abs(o).max()))


TINY = [
    # order, dims, nnz, J, R, M
    (10, (12, 9, 15, 7, 20, 6, 11, 8, 5, 13), 9000, (4,) * 10, 4, 2100),   # the highest order the paper scales to
    (9, (30, 8, 8, 8, 8, 8, 8, 8, 25), 5000, (3, 2, 4, 2, 3, 2, 4, 2, 3), 5, 1300),
    (9, (30, 8, 8, 8, 8, 8, 8, 8, 25), 3000, (3, 2, 20, 2, 3, 2, 4, 2, 3), 5, 700),   # order 9 with a rank above 16: no matrix-core instance
    (7, (40, 30, 20, 10, 10, 10, 10), 8000, (8,) * 7, 8, 3000),             # tiled kernel at order 7
    (3, (40, 30, 20), 4000, (64, 64, 64), 64, 700),
    (3, (200, 300, 20), 20000, (24, 40, 9), 20, 5000),      # ranks that are no multiple of 16, padded tiles
    (2, (5000, 3), 30000, (32, 32), 48, 20001),             # a 3-row mode: everything collides
    (1, (50,), 200, (4,), 3, 100),
    (2, (40, 30), 500, (3, 5), 4, 333),
    (3, (20, 30, 10), 2000, (2, 3, 4), 2, 1000),
    (3, (64, 64, 64), 5000, (16, 16, 16), 16, 4097),
    (3, (30, 30, 30), 3000, (8, 8, 8), 16, 64),
    (4, (9, 8, 7, 6), 1500, (2, 2, 2, 2), 3, 777),
    (5, (6, 5, 4, 3, 7), 800, (2, 1, 3, 2, 2), 5, 129),
    (6, (50,) * 6, 4000, (8,) * 6, 16, 2049),
    (6, (40, 30, 20, 10, 12, 9), 4000, (16,) * 6, 16, 1500),  # J = R = 16 at order 6: "auto" is the tiled kernel there
    (8, (5,) * 8, 600, (2,) * 8, 2, 65),
    (3, (10, 10, 10), 100, (5, 7, 3), 11, 1),
    (3, (300, 200, 100), 3000, (32, 32, 32), 32, 513),
    (3, (3, 2, 2), 1, (4, 4, 4), 4, 200),          # one stored entry, every sample a duplicate
]


@pytest.mark.parametrize("layout", ["padded", "exact"])
@pytest.mark.parametrize("kernel", ["auto", "generic", "tiled", "mfma16", "rows"])
@pytest.mark.parametrize("order,dims,nnz,J,R,M", TINY)
def test_one_step_small_shapes(order, dims, nnz, J, R, M, kernel, layout):
    """Every gradient-kernel variant on every small shape: "auto" is the specialised J = R = 16 kernel
    where it applies (ranks up to 16 are held padded to 16 for it unless the exact layout is asked for)
    and the tiled matrix-core kernel elsewhere."""
    flags = binding.FTK_LAYOUT_EXACT if layout == "exact" else 0
    announce("tiny order=%d dims=%r J=%r R=%d M=%d kernel=%s layout=%s" % (order, dims, J, R, M, kernel, layout))
    w = synth.tiny_workload(order, dims, nnz, J, R, M, seed=11 + order, values="normal")
    w = synth.replace(w, lr_A=1e-2, lr_B=1e-2)
    idx, vals = synth.make_tensor(w)
    if kernel == "tiled" and order > 8 and (max(J) > 16 or R > 16):   # orders 9, 10 are built for ranks up to 16: must say so
        with pytest.raises(binding.FtkError) as e:
            one_step_case(w, idx, vals, kernel=kernel, flags=flags)
        assert e.value.code == binding.FTK_EUNSUPPORTED
        return
    if kernel == "rows":
        # the tiled kernel's shapes with every (possibly padded) J_n a multiple of four; refused elsewhere
        padded = layout == "padded" and 2 <= order <= 5 and max(J) <= 16 and R <= 16
        fits = padded or (all(j % 4 == 0 for j in J) and max(J) <= 64 and R <= 64 and (order <= 8 or (max(J) <= 16 and R <= 16)))
        if not fits:
            with pytest.raises(binding.FtkError) as e:
                one_step_case(w, idx, vals, kernel=kernel, flags=flags)
            assert e.value.code == binding.FTK_EUNSUPPORTED
            return
    if kernel == "mfma16":
        # by name: where the (possibly padded) ranks are all 16 and the order is at most 6, also at order 6,
        # which "auto" gives to the tiled kernel; refused elsewhere
        fits = 2 <= order <= 6 and ((set(J) == {16} and R == 16) or (layout == "padded" and order <= 5 and max(J) <= 16 and R <= 16))
        fits = fits or (order == 1 and J == (16,) and R == 16)
        if not fits:
            with pytest.raises(binding.FtkError) as e:
                one_step_case(w, idx, vals, kernel=kernel, flags=flags)
            assert e.value.code == binding.FTK_EUNSUPPORTED
            return
    one_step_case(w, idx, vals, kernel=kernel, flags=flags)


def _random_case(case_seed):
    """A shape nobody picked by hand: order 1..6, ragged ranks (now and then 16 everywhere, now and then
    past the matrix-core kernels' limit), a skewed mode, sample counts off every tile boundary."""
    rng = np.random.default_rng(1000 + case_seed)
    order = int(rng.integers(1, 7))
    dims = tuple(int(x) for x in rng.integers(2, 400, size=order))
    flavour = case_seed % 4
    if flavour == 0:
        J, R = (16,) * order, 16
    elif flavour == 1:
        J, R = tuple(int(x) for x in rng.integers(1, 17, size=order)), int(rng.integers(1, 17))
    elif flavour == 2:
        J, R = tuple(int(x) for x in rng.integers(1, 65, size=order)), int(rng.integers(1, 65))
    else:
        J, R = tuple(int(x) for x in rng.integers(1, 90, size=order)), int(rng.integers(1, 90))
    nnz = int(rng.integers(50, 20_000))
    M = int(rng.integers(1, 6_000))
    zipf = tuple(1.1 if (n == 0 and dims[0] > 50) else None for n in range(order))
    return order, dims, nnz, J, R, M, zipf


@pytest.mark.parametrize("case_seed", range(24))
def test_one_step_random_shapes(case_seed):
    order, dims, nnz, J, R, M, zipf = _random_case(case_seed)
    announce("random case %d: order=%d dims=%r J=%r R=%d nnz=%d M=%d" % (case_seed, order, dims, J, R, nnz, M))
    w = synth.tiny_workload(order, dims, nnz, J, R, M, seed=300 + case_seed, values="normal", zipf=zipf)
    # a step small enough for any of these shapes (predictions of order R (J/16)^N at the start)
    scale = max(1.0, float(R) * float(np.prod([max(j, 1) / 16.0 for j in J])))
    w = synth.replace(w, lr_A=1e-4 / scale ** 2, lr_B=1e-4 / scale ** 2)
    idx, vals = synth.make_tensor(w)
    # every variant that is built for the shape: the tiled kernel keeps B and its transpose, padded, in LDS
    # (high orders with ranks above 32 do not fit), the one-lane-per-sample kernel keeps N R columns per lane
    # there; a shape none of them takes is refused by ftk_create with FTK_EUNSUPPORTED
    ran = []
    # the default layout (ranks up to 16 padded to 16) with the kernel the library picks, the exact layout
    # with every variant
    exact = binding.FTK_LAYOUT_EXACT
    for kernel, tiles, flags in ((None, False, 0), (None, case_seed % 2 == 0, exact), ("generic", False, exact),
                                 ("tiled", case_seed % 2 == 1, exact)):
        try:
            gA, gB, A, B = one_step_case(w, idx, vals, kernel=kernel, tiles=tiles, flags=flags)
            assert all(np.isfinite(x).all() for x in A + B)
            ran.append(kernel or "auto")
        except binding.FtkError as e:
            assert e.code == binding.FTK_EUNSUPPORTED, e
    announce("random case %d ran on: %s" % (case_seed, ", ".join(ran) or "no variant (shape refused)"))
    assert ran or order * R > 256


@pytest.mark.parametrize("order,dims,J,R,kernel", [
    (3, (900, 300, 40), (16, 16, 16), 16, None),
    (3, (500, 200, 30), (20, 7, 33), 12, None),
    (3, (9_000, 3_000, 40), (20, 8, 32), 12, "rows"),     # the lists are re-planned (and grow) with |Psi|
])
def test_sample_count_changing_from_step_to_step(order, dims, J, R, kernel):
    """|Psi| changes every step (1 sample, one group, many groups, back): the number of workgroups, the rows
    kept in the workgroup tables and the partial tables the update pass reads all follow it.  Parameters
    against the oracle after every step, both sampling rules."""
    w = synth.tiny_workload(order, dims, 40_000, J, R, 1, seed=77, values="normal", zipf=(1.1, None, None))
    scale = max(1.0, float(R) * float(np.prod([j / 16.0 for j in J])))
    lr = 3e-5 / scale ** 2
    idx, vals = synth.make_tensor(w)
    for tiles in (False, True):
        draw = oracle.sample_positions_tiles if tiles else oracle.sample_positions
        A, B = oracle_state(w)
        with binding.FastTucker(w.dims, idx, vals, w.J, w.R, w.init_seed) as ft:
            if kernel:
                ft.ftk_set_kernel(kernel)
                assert ft.ftk_kernel_name() == kernel
            if tiles:
                ft.ftk_set_sampling(binding.FTK_SAMPLE_TILES)
            for t, M in enumerate([700, 64, 9_000, 1, 3_329, 130, 20_000, 65]):
                announce("changing |Psi|: step %d with %d samples%s" % (t, M, ", tiles" if tiles else ""))
                ft.ftk_sample(500 + t, M)
                ft.ftk_sgd_step(lr, lr, w.lambda_A, w.lambda_B)
                oracle.sgd_step_sync(w.dims, idx, vals, A, B, draw(500 + t, M, w.nnz), lr, lr, w.lambda_A, w.lambda_B)
                gA, gB = ft.ftk_get_factors()
                for g, o in zip(gA + gB, A + B):
                    err = np.abs(g.astype(np.float64) - o)
                    assert float((err - (t + 1) * (ATOL + RTOL * np.abs(o))).max()) <= 0.0, "step %d" % t


def test_rows_whose_length_is_no_multiple_of_four_next_to_table_rows():
    """The update pass scans the accumulator four floats at a time while other blocks of the same launch
    update the rows kept in the workgroups' tables: with J_n = 50 a group of four floats can hold the end of
    one row and the start of the next, and an element must never be written by both (a lost update once
    showed up as one wrong element now and then).  Same small shape, several fresh contexts."""
    w = synth.tiny_workload(4, (153, 311, 144, 358), 1227, (48, 40, 25, 50), 22, 3329, seed=302, values="normal")
    w = synth.replace(w, lr_A=1.5e-10, lr_B=1.5e-10)
    idx, vals = synth.make_tensor(w)
    for rep in range(12):
        announce("straddling rows, repetition %d" % rep)
        one_step_case(w, idx, vals)


@pytest.mark.parametrize("order,dims,J,R,zipf", [
    (3, (2_000, 700, 90), (20, 28, 12), 20, (1.2, 1.1, None)),          # 32-wide blocks, ranks off the block size
    (3, (2_000, 700, 90), (20, 36, 52), 24, (1.2, 1.1, None)),          # 64-wide blocks
    (4, (900, 500, 300, 60), (4, 8, 12, 16), 8, (1.1, None, 1.3, None)),   # 16-wide, order 4
    (3, (2_000, 700, 90), (18, 36, 50), 24, (1.2, 1.1, None)),          # the same with rows that are no multiple of 16 bytes
])
def test_matrix_core_kernel_with_ranks_off_the_block_size(order, dims, J, R, zipf):
    """The general matrix-core kernel on ranks that are multiples of four but not of 16 (rows fetched 16
    bytes per lane, blocks partly padding) and on ranks that are not (rows fetched float by float), with
    skewed modes so that all three routes of the factor-row gradients carry rows, over several groups and a
    ragged last one; both sampling rules."""
    w = synth.tiny_workload(order, dims, 60_000, J, R, 5_003, seed=411, values="normal", zipf=zipf)
    scale = max(1.0, float(R) * float(np.prod([j / 16.0 for j in J])))
    w = synth.replace(w, lr_A=1e-4 / scale ** 2, lr_B=1e-4 / scale ** 2)
    idx, vals = synth.make_tensor(w)
    for tiles in (False, True):
        announce("ranks off the block size: J=%r R=%d%s" % (J, R, ", tiles" if tiles else ""))
        one_step_case(w, idx, vals, kernel="tiled", tiles=tiles, flags=binding.FTK_LAYOUT_EXACT)


@pytest.mark.parametrize("kernel", [None, "rows"])
@pytest.mark.parametrize("name,nnz,M,dims", [
    ("C2", 200_000, 20_000, (4_800, 1_777, 220)),
    ("C3", 100_000, 5_000, (10_000, 6_250, 300)),
    ("C4", 200_000, 20_000, (1_000,) * 6),
    ("C5", 50_000, 2_000, (4_800, 1_777, 220)),
])
def test_one_step_scaled_workloads(name, nnz, M, dims, kernel):
    announce("scaled %s%s" % (name, ", kernel rows" if kernel else ""))
    w = synth.replace(synth.WORKLOADS[name].scaled(nnz=nnz, n_samples=M, dims=dims), **TEST_STEP_SIZES[name])
    idx, vals = synth.make_tensor(w)
    one_step_case(w, idx, vals, kernel=kernel)


def test_signed_parameters_and_hot_rows():
    """Parameters of both signs (cancellation in the sums) and a mode with 2 rows (every sample
    collides on it)."""
    announce("signed parameters, 2-row mode")
    w = synth.tiny_workload(3, (500, 2, 40), 20_000, (8, 8, 8), 8, 30_000, seed=5, values="normal")
    w = synth.replace(w, lr_A=1e-4, lr_B=1e-3)
    idx, vals = synth.make_tensor(w)
    rng = np.random.default_rng(3)
    A0 = [rng.uniform(-0.6, 0.6, size=(w.dims[n], w.J[n])).astype(np.float32) for n in range(3)]
    B0 = [rng.uniform(-0.6, 0.6, size=(w.J[n], w.R)).astype(np.float32) for n in range(3)]
    one_step_case(w, idx, vals, A0, B0)


# ------------------------------------------------------------------------------------------------
# rows that leave the chip one sample at a time: every single update has to be visible
# ------------------------------------------------------------------------------------------------
def frequency_rank(col, rows):
    """Rank of every row of a mode by how often it occurs in Omega: most frequent first, ties by ascending
    row number (the ranking ftk_get_table_rows refers to)."""
    counts = np.bincount(col, minlength=rows)
    by_rank = np.argsort(-counts, kind="stable")
    rank = np.empty(rows, dtype=np.int64)
    rank[by_rank] = np.arange(rows)
    return rank


COLD_ROW_CASES = [
    # kernel, dims, power-law exponent per mode, J, R, stored entries, |Psi| (ragged last group), lr_A
    ("mfma16", (40_000, 60_000, 1_500), (1.1, None, None), (16, 16, 16), 16, 400_000, 60_013, 1e-2),
    ("mfma16", (60_000, 30_000), (None, 1.1), (16, 16), 16, 300_000, 50_001, 1e-2),
    # |Psi| large enough for the turns that share their Philox blocks: shares of 11 and 7 tiles for the two waves of a SIMD
    # (one pair of turns and a turn of three tiles; two plain turns), and the ragged end of Psi inside the last share
    ("mfma16", (400_000, 600_000, 1_500), (1.1, None, None), (16, 16, 16), 16, 1_200_000, 300_007, 1e-2),
    ("mfma16", (20_000, 50_000, 300, 40, 1_200), (1.1, None, None, None, None), (16,) * 5, 16, 300_000, 40_007, 0.3),
    ("tiled", (30_000, 50_000, 900), (1.1, None, None), (32, 32, 32), 32, 300_000, 40_011, 1e-2),   # 32-wide blocks
    ("tiled", (40_000, 60_000, 1_500), (1.1, None, None), (16, 16, 16), 16, 400_000, 60_013, 1e-2),
    # 64-wide blocks: the table rows (here the 100 evenly hit rows of the last mode beyond its first 16) are summed in
    # per-workgroup tables in global memory by the same atomics as the rows outside the tables
    ("tiled", (30_000, 50_000, 100), (1.1, None, None), (64, 64, 64), 64, 300_000, 40_011, 3e-3),
    ("rows", (30_000, 50_000, 100), (1.1, None, None), (64, 64, 64), 64, 300_000, 40_011, 3e-3),
    # the same rows through the lists of the row-owning workgroups instead of atomics: row number in a spare lane
    # (J_n = 8, 20), in a store of its own (J_n = 16, 32), and with lists so short that many rows fall back to atomics
    ("rows", (30_000, 50_000, 900), (1.1, None, None), (32, 32, 32), 32, 300_000, 40_011, 1e-2),
    ("rows", (40_000, 60_000, 1_500), (1.1, None, None), (16, 16, 16), 16, 400_000, 60_013, 1e-2),
    ("rows", (40_000, 60_000, 1_500), (1.1, None, None), (8, 20, 8), 16, 400_000, 60_013, 1e-2),
    ("rows:tight", (40_000, 60_000, 1_500), (1.1, None, None), (8, 20, 8), 16, 400_000, 60_013, 1e-2),
    ("rows:tight", (30_000, 50_000, 900), (1.1, None, None), (32, 32, 32), 32, 300_000, 40_011, 1e-2),
    ("rows", (20_000, 50_000, 300, 40, 1_200, 700), (1.1, None, None, None, None, None), (8,) * 6, 16, 300_000, 40_007, 1.0),
]


def cold_row_inputs(dims, zipf, J, R, nnz, M, lr_A):
    """Many more rows than any on-chip table holds, most of them hit 0 to 3 times by Psi, and parameters of
    both signs sized so that ONE hit moves a row's elements by about a hundred tolerances."""
    w = synth.tiny_workload(len(dims), dims, nnz, J, R, M, seed=613, values="int1to5", zipf=zipf)
    w = synth.replace(w, lr_A=lr_A, lr_B=1e-2)
    idx, vals = synth.make_tensor(w)
    rng = np.random.default_rng(97)
    A0 = [rng.uniform(-0.5, 0.5, size=(w.dims[n], w.J[n])).astype(np.float32) for n in range(w.order)]
    B0 = [rng.uniform(-0.5, 0.5, size=(w.J[n], w.R)).astype(np.float32) for n in range(w.order)]
    return w, idx, vals, A0, B0


def single_hit_rows_that_moved(w, idx, pos, K, A0, A1, least=1e-3):
    """Rows outside the on-chip tables (rank >= K[n]) that exactly one sample of Psi hits and whose largest
    element change under the oracle's step exceeds `least`; returns their number over all modes."""
    total = 0
    for n in range(w.order):
        hits = np.bincount(idx[n][pos], minlength=w.dims[n])
        cold = frequency_rank(idx[n], w.dims[n]) >= int(K[n])
        moved = np.abs(A1[n].astype(np.float64) - A0[n].astype(np.float64)).max(axis=1)
        total += int(np.count_nonzero((hits == 1) & cold & (moved > least)))
    return total


@pytest.mark.parametrize("tiles", [False, True])
@pytest.mark.parametrize("kernel,dims,zipf,J,R,nnz,M,lr_A", COLD_ROW_CASES)
def test_rows_outside_the_tables_hit_once_or_twice(kernel, dims, zipf, J, R, nnz, M, lr_A, tiles):
    """The route that carries the rows no table holds (compacted lists of float atomics): tens of thousands
    of rows per mode, far more than fit on chip, most of them hit by a single sample.  The step is sized so
    that one hit moves an element by ~1e-3 to 1e-2 against a tolerance of ~1e-5: a dropped, doubled or
    misdirected update of a single row fails the comparison.  The test itself checks that power: at least
    10 000 rows outside the tables with exactly one hit each move by more than 1e-3 under the oracle's step."""
    announce("rows outside the tables: kernel=%s dims=%r J=%r%s" % (kernel, dims, J, ", tile sampling" if tiles else ""))
    w, idx, vals, A0, B0 = cold_row_inputs(dims, zipf, J, R, nnz, M, lr_A)
    draw = oracle.sample_positions_tiles if tiles else oracle.sample_positions
    with binding.FastTucker(w.dims, idx, vals, w.J, w.R, w.init_seed, flags=binding.FTK_LAYOUT_EXACT) as ft:
        ft.ftk_set_kernel(kernel)
        assert ft.ftk_kernel_name() == kernel.split(":")[0]
        if tiles:
            ft.ftk_set_sampling(binding.FTK_SAMPLE_TILES)
        ft.ftk_set_factors(A0, B0)
        ft.ftk_sample(w.sample_seed0, w.n_samples)
        K, top = ft.ftk_get_table_rows()
        pos = ft.ftk_get_samples()
        want = draw(w.sample_seed0, w.n_samples, w.nnz)
        assert np.array_equal(pos, want), "sample set differs from the oracle's"
        ft.ftk_sgd_step(w.lr_A, w.lr_B, w.lambda_A, w.lambda_B)
        gA, gB = ft.ftk_get_factors()
    A, B = [a.copy() for a in A0], [b.copy() for b in B0]
    oracle.sgd_step_sync(w.dims, idx, vals, A, B, want, w.lr_A, w.lr_B, w.lambda_A, w.lambda_B)
    # all three routes carry rows: a one-hot mode, table rows, and far more rows than the tables hold
    assert int(top.max()) == 16 and int(K.sum()) > int(top.sum()), (K, top)
    assert sum(w.dims) > 20 * int(K.sum()), (K, w.dims)
    n_single = single_hit_rows_that_moved(w, idx, want, K, A0, A)
    announce("  tables hold %r rows, %d single-hit rows outside them move by more than 1e-3" % (K.tolist(), n_single))
    assert n_single >= 10_000, n_single
    assert_params_close(gA, A, "A")
    assert_params_close(gB, B, "B")


@pytest.mark.parametrize("kernel", ["mfma16", "tiled"])
def test_every_sample_is_taken_exactly_once_whatever_the_size_of_psi(kernel):
    """The waves' shares of Psi (whole tiles, dealt to workgroups, SIMDs and the two waves of a SIMD; turns in pairs
    where |Psi| allows) at sample counts around every edge of that deal: fewer samples than a tile, than waves, one
    tile per wave and one sample more, the first count that takes the paired turns and its neighbours, a count
    that leaves every wave whole tiles.  Inputs as in the test above: one hit moves a row by about a hundred
    tolerances, so a sample left out or taken twice fails the comparison."""
    announce("shares of Psi at edge sizes, kernel=%s" % kernel)
    dims, zipf, J, R = (400_000, 600_000, 1_500), (1.1, None, None), (16, 16, 16), 16
    w, idx, vals, A0, B0 = cold_row_inputs(dims, zipf, J, R, 1_200_000, 1, 1e-2)
    with binding.FastTucker(w.dims, idx, vals, w.J, w.R, w.init_seed, flags=binding.FTK_LAYOUT_EXACT) as ft:
        ft.ftk_set_kernel(kernel)
        for M in (1, 15, 17, 2_047, 2_048 * 16, 2_048 * 16 + 1, 262_079, 262_081, 262_145, 2_048 * 16 * 9):
            ft.ftk_set_factors(A0, B0)
            ft.ftk_sample(w.sample_seed0 + M, M)
            ft.ftk_sgd_step(w.lr_A, w.lr_B, w.lambda_A, w.lambda_B)
            gA, gB = ft.ftk_get_factors()
            pos = oracle.sample_positions(w.sample_seed0 + M, M, w.nnz)
            A, B = [a.copy() for a in A0], [b.copy() for b in B0]
            oracle.sgd_step_sync(w.dims, idx, vals, A, B, pos, w.lr_A, w.lr_B, w.lambda_A, w.lambda_B)
            assert_params_close(gA, A, "A, |Psi| = %d" % M)
            assert_params_close(gB, B, "B, |Psi| = %d" % M)
            if M >= 2_047:
                moved = max(float(np.abs(a.astype(np.float64) - a0).max()) for a, a0 in zip(A, A0))
                assert moved > 1e-3, (M, moved)


# ------------------------------------------------------------------------------------------------
# invariants and error paths through the ABI
# ------------------------------------------------------------------------------------------------
def test_zero_learning_rate_leaves_parameters_bit_identical():
    announce("lr = 0")
    w = synth.tiny_workload(3, (50, 40, 30), 2000, (8, 8, 8), 8, 1500)
    idx, vals = synth.make_tensor(w)
    with binding.FastTucker(w.dims, idx, vals, w.J, w.R, 3) as ft:
        A0, B0 = ft.ftk_get_factors()
        ft.ftk_sample(1, w.n_samples)
        ft.ftk_sgd_step(0.0, 0.0, 0.5, 0.5)
        A1, B1 = ft.ftk_get_factors()
    for x, y in zip(A0 + B0, A1 + B1):
        assert np.array_equal(x, y)


@pytest.mark.parametrize("kernel,J,R", [("auto", (16, 16, 16), 16), ("tiled", (16, 16, 16), 16), ("tiled", (32, 32, 32), 32),
                                        ("tiled", (64, 64, 64), 64), ("rows", (8, 8, 8), 8), ("generic", (5, 6, 7), 3)])
def test_a_diverged_run_still_returns(kernel, J, R):
    """A step size far too large turns the parameters into inf and NaN.  The header promises only that every
    call still returns: the compare-and-swap loops compare bit patterns, so NaN does not keep them turning."""
    announce("diverged run, kernel=%s J=%r" % (kernel, J))
    w = synth.tiny_workload(3, (300, 200, 100), 20_000, J, R, 9_001)
    idx, vals = synth.make_tensor(w)
    with binding.FastTucker(w.dims, idx, vals, w.J, w.R, 3, flags=binding.FTK_LAYOUT_EXACT) as ft:
        ft.ftk_set_kernel(kernel)
        for t in range(4):
            ft.ftk_sample(t, w.n_samples)
            ft.ftk_sgd_step(1e30, 1e30, 0.1, 0.1)
        A, B = ft.ftk_get_factors()
        assert not np.isfinite(ft.ftk_rmse())
    assert not all(np.isfinite(a).all() for a in A)


def test_repeating_a_step_reuses_psi_and_accumulators_are_clean():
    """Two steps on the same Psi equal two oracle steps on it: nothing is left over in the
    gradient accumulators between steps."""
    announce("two steps on one Psi")
    w = synth.tiny_workload(3, (60, 50, 40), 3000, (4, 4, 4), 4, 2500)
    idx, vals = synth.make_tensor(w)
    A, B = oracle.init_factors(9, w.dims, w.J, w.R)
    pos = oracle.sample_positions(77, w.n_samples, w.nnz)
    with binding.FastTucker(w.dims, idx, vals, w.J, w.R, 9) as ft:
        ft.ftk_sample(77, w.n_samples)
        for _ in range(2):
            ft.ftk_sgd_step(1e-2, 1e-2, 1e-2, 1e-2)
            oracle.sgd_step_sync(w.dims, idx, vals, A, B, pos, 1e-2, 1e-2, 1e-2, 1e-2)
        gA, gB = ft.ftk_get_factors()
    assert_params_close(gA, A, "A")
    assert_params_close(gB, B, "B")


def test_rmse_and_mae_match_oracle():
    announce("rmse / mae")
    for order, dims, J, R in [(3, (100, 90, 80), (8, 8, 8), 8), (2, (50, 60), (3, 7), 5), (6, (20,) * 6, (8,) * 6, 16),
                              (3, (300, 200, 100), (16, 16, 16), 16), (1, (500,), (16,), 16), (4, (30, 20, 10, 40), (16,) * 4, 16)]:
        w = synth.tiny_workload(order, dims, 20_011, J, R, 10, seed=21)
        idx, vals = synth.make_tensor(w)
        A, B = oracle.init_factors(4, w.dims, w.J, w.R)
        with binding.FastTucker(w.dims, idx, vals, w.J, w.R, 4) as ft:
            rm, ma = ft.ftk_rmse(), ft.ftk_mae()
        want_rm, want_ma = oracle.errors(w.dims, idx, vals, A, B)
        assert rm == pytest.approx(want_rm, rel=1e-5)
        assert ma == pytest.approx(want_ma, rel=1e-5)


@pytest.mark.parametrize("order,dims,J,R", [
    (3, (700, 500, 90), (16, 16, 16), 16),      # matrix-core kernel for J = R = 16
    (3, (300, 200, 50), (24, 40, 9), 20),       # tiled kernel, padded ranks
    (4, (60, 50, 40, 30), (8, 8, 8, 8), 8),
    (2, (900, 800), (80, 3), 70),               # generic kernel
])
def test_held_out_set_evaluation_matches_oracle(order, dims, J, R):
    """ftk_evaluate on entries that are NOT the stored ones (other seed, other length, ragged tail)
    after two steps of training, against the oracle's error sums over the same entries."""
    announce("held-out evaluation order=%d J=%r R=%d" % (order, J, R))
    w = synth.tiny_workload(order, dims, 30_000, J, R, 4_000, seed=5, values="normal")
    w = synth.replace(w, lr_A=1e-5, lr_B=1e-5)    # two steps that lower the error on every one of the shapes
    idx, vals = synth.make_tensor(w)
    held = synth.replace(w, nnz=12_345, data_seed=w.data_seed + 77)
    hidx, hvals = synth.make_tensor(held)
    A, B = oracle_state(w)
    with binding.FastTucker(w.dims, idx, vals, w.J, w.R, w.init_seed) as ft:
        for t in range(2):
            ft.ftk_sample(w.sample_seed0 + t, w.n_samples)
            ft.ftk_sgd_step(w.lr_A, w.lr_B, w.lambda_A, w.lambda_B)
            pos = oracle.sample_positions(w.sample_seed0 + t, w.n_samples, w.nnz)
            oracle.sgd_step_sync(w.dims, idx, vals, A, B, pos, w.lr_A, w.lr_B, w.lambda_A, w.lambda_B)
        got_rmse, got_mae = ft.ftk_evaluate(hidx, hvals)
        # a row number outside the mode is refused, and the context stays usable
        bad = [a.copy() for a in hidx]
        bad[order - 1][17] = dims[order - 1]
        with pytest.raises(binding.FtkError) as e:
            ft.ftk_evaluate(bad, hvals)
        assert e.value.code == binding.FTK_EINVAL
        again = ft.ftk_evaluate(hidx, hvals)
    want_rmse, want_mae = oracle.errors(w.dims, hidx, hvals, A, B)
    assert abs(got_rmse - want_rmse) <= 1e-4 * want_rmse, (got_rmse, want_rmse)
    assert abs(got_mae - want_mae) <= 1e-4 * want_mae, (got_mae, want_mae)
    assert again == pytest.approx((got_rmse, got_mae), rel=1e-12)    # block sums are added in any order


def test_call_order_and_bad_input_errors():
    announce("error paths")
    w = synth.tiny_workload(3, (10, 10, 10), 100, (2, 2, 2), 2, 10)
    idx, vals = synth.make_tensor(w)
    with binding.FastTucker(w.dims, idx, vals, w.J, w.R) as ft:
        with pytest.raises(binding.FtkError) as ei:
            ft.ftk_sgd_step(0.1, 0.1, 0.0, 0.0)
        assert ei.value.code == binding.FTK_ESTATE
        with pytest.raises(binding.FtkError) as ei:
            ft.ftk_get_samples()
        assert ei.value.code == binding.FTK_ESTATE
        with pytest.raises(binding.FtkError) as ei:
            ft.ftk_sample(1, 0)
        assert ei.value.code == binding.FTK_EINVAL
        with pytest.raises(binding.FtkError) as ei:
            ft.ftk_set_kernel("no-such-kernel")
        assert ei.value.code == binding.FTK_EUNSUPPORTED
        ft.ftk_sample(1, 10)
        ft.ftk_sgd_step(0.1, 0.1, 0.0, 0.0)      # and now it works
    bad = [a.copy() for a in idx]
    bad[1][17] = 10                               # == dims[1]: out of range
    with pytest.raises(binding.FtkError) as ei:
        binding.FastTucker(w.dims, bad, vals, w.J, w.R)
    assert ei.value.code == binding.FTK_EINVAL
    bad[1][17] = -1
    with pytest.raises(binding.FtkError) as ei:
        binding.FastTucker(w.dims, bad, vals, w.J, w.R)
    assert ei.value.code == binding.FTK_EINVAL


def test_device_pointers_and_caller_stream():
    """COO handed over as torch device tensors, work enqueued on torch's current stream."""
    import torch
    announce("device pointers + stream")
    w = synth.tiny_workload(3, (80, 70, 60), 5000, (8, 8, 8), 8, 3000)
    idx, vals = synth.make_tensor(w)
    d_idx = [torch.from_numpy(a).cuda() for a in idx]
    d_vals = torch.from_numpy(vals).cuda()
    A, B = oracle.init_factors(2, w.dims, w.J, w.R)
    stream = torch.cuda.Stream()
    with torch.cuda.stream(stream):
        with binding.FastTucker(w.dims, d_idx, d_vals, w.J, w.R, 2) as ft:
            del d_idx, d_vals                      # the library keeps its own copy
            ft.ftk_set_stream(torch.cuda.current_stream().cuda_stream)
            ft.ftk_sample(5, w.n_samples)
            ft.ftk_sgd_step(1e-2, 1e-2, 1e-2, 1e-2)
            gA, gB = ft.ftk_get_factors()
    pos = oracle.sample_positions(5, w.n_samples, w.nnz)
    oracle.sgd_step_sync(w.dims, idx, vals, A, B, pos, 1e-2, 1e-2, 1e-2, 1e-2)
    assert_params_close(gA, A, "A")
    assert_params_close(gB, B, "B")


def test_timing_slots_count_launches():
    announce("timing")
    w = synth.tiny_workload(3, (80, 70, 60), 5000, (8, 8, 8), 8, 3000)
    idx, vals = synth.make_tensor(w)
    with binding.FastTucker(w.dims, idx, vals, w.J, w.R) as ft:
        ft.ftk_set_timing(True)
        for t in range(3):
            ft.ftk_sample(t, w.n_samples)
            ft.ftk_sgd_step(1e-3, 1e-3, 1e-2, 1e-2)
        for slot in (binding.FTK_K_GRAD, binding.FTK_K_APPLY):
            ms, cnt = ft.ftk_get_timing(slot)
            assert cnt == 3 and ms > 0.0
        # Psi is only materialised as arrays when something needs them
        ms, cnt = ft.ftk_get_timing(binding.FTK_K_SAMPLE)
        assert cnt == (3 if ft.ftk_kernel_name() == "generic" else 0)
        ft.ftk_get_samples()
        assert ft.ftk_get_timing(binding.FTK_K_SAMPLE)[1] == cnt + (0 if ft.ftk_kernel_name() == "generic" else 1)
        ft.ftk_set_timing(False)


# ------------------------------------------------------------------------------------------------
# the benchmark workload at full size, in the configuration bench.py times
# ------------------------------------------------------------------------------------------------
def test_c2_full_size_one_step():
    """C2 (order-3, 1e8 stored entries, J = R = 16, |Psi| = 1e6): the sample set bit-exact and every
    parameter after one step against the oracle (which needs a few seconds for 1e6 samples)."""
    # step sizes large enough that the most-hit rows and the core factors move by a few percent:
    # the comparison has to see the gradients, not just the unchanged parameters
    w = synth.replace(synth.WORKLOADS["C2"], lr_A=1e-8, lr_B=1e-2)
    announce("C2 full size: generating")
    idx, vals = synth.make_tensor(w)
    announce("C2 full size: step")
    gA, gB, A, B = one_step_case(w, idx, vals)
    A0, B0 = oracle_state(w)
    moved_A = max(float(np.abs(a.astype(np.float64) - a0).max()) for a, a0 in zip(A, A0))
    moved_B = max(float(np.abs(b.astype(np.float64) - b0).max()) for b, b0 in zip(B, B0))
    assert moved_A > 1e-2, moved_A
    assert moved_B > 1e-2, moved_B


@pytest.mark.parametrize("name", ["C3", "C4", "C5", "C2 at J = R = 8", "C4 with row owners"])
def test_other_workloads_full_size_one_step(name):
    """The other named workloads at full size, on the kernel the library picks for them: the sample
    set bit-exact and every parameter after one synchronous step against the oracle (up to half a
    minute of one host core for the 4e6 samples of C3 and the 64 x 64 contractions of C5).  The C2
    tensor at J = R = 8, the paper's most used ranks, runs on the J = R = 16 kernel through the padded
    layout: the same comparison at full size for that route."""
    kernel = None
    if name == "C2 at J = R = 8":
        w = synth.replace(synth.WORKLOADS["C2"], J=(8, 8, 8), R=8, lr_A=1e-7, lr_B=1e-2)
    elif name == "C4 with row owners":     # the "rows" kernel at full size: 12e6 list entries per step
        w = synth.replace(synth.WORKLOADS["C4"], **TEST_STEP_SIZES["C4"])
        kernel = "rows"
    else:
        w = synth.replace(synth.WORKLOADS[name], **TEST_STEP_SIZES[name])
    announce("%s full size: generating" % name)
    idx, vals = synth.make_tensor(w)
    announce("%s full size: step" % name)
    gA, gB, A, B = one_step_case(w, idx, vals, kernel=kernel)
    A0, B0 = oracle_state(w)
    assert all(np.isfinite(a).all() for a in A + B)
    moved_A = max(float(np.abs(a.astype(np.float64) - a0).max()) for a, a0 in zip(A, A0))
    moved_B = max(float(np.abs(b.astype(np.float64) - b0).max()) for b, b0 in zip(B, B0))
    announce("%s full size: largest change of A %.3e, of B %.3e" % (name, moved_A, moved_B))
    assert moved_A > 1e-4, moved_A
    assert moved_B > 1e-4, moved_B


# ------------------------------------------------------------------------------------------------
# in-place (Hogwild) mode: judged on its RMSE curve
# ------------------------------------------------------------------------------------------------
@pytest.mark.parametrize("name,nnz,M,dims,lr_A,lr_B,kernel,mode", [
    ("C1", 100_000, 10_000, (1000, 800, 600), 1e-3, 1e-3, "auto", binding.FTK_HOGWILD),
    ("C2", 300_000, 30_000, (4_800, 1_777, 220), 2e-7, 1e-4, "auto", binding.FTK_HOGWILD),
    ("C2", 300_000, 30_000, (4_800, 1_777, 220), 2e-7, 1e-4, "generic", binding.FTK_HOGWILD),
    # the general matrix-core kernel at all three block widths (its row gradients' factor -lr_A rides in an operand table)
    ("C1", 100_000, 10_000, (1000, 800, 600), 1e-3, 1e-3, "tiled", binding.FTK_HOGWILD),
    ("C3", 100_000, 10_000, (10_000, 6_250, 300), 3e-9, 3e-7, "auto", binding.FTK_HOGWILD),
    # 64-wide ranks: the in-place pass adds to A and to the workgroups' tables behind it through one buffer
    ("C5", 100_000, 10_000, (4_800, 1_777, 220), 3e-11, 1e-8, "auto", binding.FTK_HOGWILD),
    ("C1", 100_000, 10_000, (1000, 800, 600), 1e-3, 1e-3, "auto", binding.FTK_HOGWILD_MODEWISE),
    ("C2", 300_000, 30_000, (4_800, 1_777, 220), 2e-7, 1e-4, "auto", binding.FTK_HOGWILD_MODEWISE),
    ("C1", 100_000, 10_000, (1000, 800, 600), 1e-3, 1e-3, "generic", binding.FTK_HOGWILD_MODEWISE),
    ("C2", 300_000, 30_000, (4_800, 1_777, 220), 2e-7, 1e-4, "generic", binding.FTK_HOGWILD_MODEWISE),
    # the mode-by-mode order on the general matrix-core kernel, at its three block widths
    ("C1", 100_000, 10_000, (1000, 800, 600), 1e-3, 1e-3, "tiled", binding.FTK_HOGWILD_MODEWISE),
    ("C3", 100_000, 10_000, (10_000, 6_250, 300), 3e-9, 3e-7, "auto", binding.FTK_HOGWILD_MODEWISE),
    ("C5", 100_000, 10_000, (4_800, 1_777, 220), 3e-11, 1e-8, "auto", binding.FTK_HOGWILD_MODEWISE),
])
def test_hogwild_mode_rmse_curve(name, nnz, M, dims, lr_A, lr_B, kernel, mode):
    """10 steps with factor rows updated in place.  The result depends on scheduling, so it is held
    to the sequential in-place oracle (Algorithm 1's printed order) only through the RMSE after every
    step (3 % relative: concurrent samples see rows a little staler than the sequential order does,
    most visibly on the rows a tenth of all samples hit), and it has to learn."""
    announce("hogwild %s kernel=%s mode=%d" % (name, kernel, mode))
    w = synth.replace(synth.WORKLOADS[name].scaled(nnz=nnz, n_samples=M, dims=dims), lr_A=lr_A, lr_B=lr_B)
    idx, vals = synth.make_tensor(w)
    A, B = oracle_state(w)
    with binding.FastTucker(w.dims, idx, vals, w.J, w.R, w.init_seed) as ft:
        ft.ftk_set_kernel(kernel)
        ft.ftk_set_mode(mode)
        start = ft.ftk_rmse()
        prev = start
        for t in range(10):
            ft.ftk_sample(w.sample_seed0 + t, w.n_samples)
            ft.ftk_sgd_step(w.lr_A, w.lr_B, w.lambda_A, w.lambda_B)
            pos = oracle.sample_positions(w.sample_seed0 + t, w.n_samples, w.nnz)
            oracle.sgd_step_hogwild(w.dims, idx, vals, A, B, pos, w.lr_A, w.lr_B, w.lambda_A, w.lambda_B)
            got, want = ft.ftk_rmse(), oracle.rmse(w.dims, idx, vals, A, B)
            assert got == pytest.approx(want, rel=3e-2), "step %d" % t
            assert got < prev
            prev = got
        # switching back gives the synchronous step again (nothing left over in the accumulators)
        ft.ftk_set_mode(binding.FTK_SYNC)
        A0, B0 = ft.ftk_get_factors()
        ft.ftk_sample(5, w.n_samples)
        ft.ftk_sgd_step(w.lr_A, w.lr_B, w.lambda_A, w.lambda_B)
        gA, gB = ft.ftk_get_factors()
    pos = oracle.sample_positions(5, w.n_samples, w.nnz)
    oracle.sgd_step_sync(w.dims, idx, vals, A0, B0, pos, w.lr_A, w.lr_B, w.lambda_A, w.lambda_B)
    assert_params_close(gA, A0, "A")
    assert_params_close(gB, B0, "B")


@pytest.mark.parametrize("kernel,N,J,R,lr_A,lr_B", [
    ("mfma16", 3, (16, 8, 12), 8, 5e-2, 1e-2), ("generic", 3, (16, 8, 12), 8, 5e-2, 1e-2),
    ("mfma16", 5, (16, 16, 16, 16, 16), 16, 1e-3, 1e-2), ("mfma16", 2, (4, 16), 11, 5e-2, 1e-2),
    # the general matrix-core kernel: one, two and four blocks of 16 ranks, and orders the J_n = R = 16 kernel is not built for
    ("tiled", 3, (16, 8, 12), 8, 5e-2, 1e-2), ("tiled", 3, (32, 24, 20), 24, 3e-5, 1e-3), ("tiled", 3, (64, 48, 40), 48, 3e-7, 1e-5),
    ("tiled", 4, (32, 32, 16, 20), 32, 3e-6, 1e-3), ("tiled", 6, (32, 16, 32, 16, 32, 16), 32, 3e-7, 1e-4),
    ("tiled", 7, (16,) * 7, 16, 1e-4, 1e-3),
    # ranks that are no multiples of four: rows fetched float by float
    ("tiled", 3, (6, 10, 7), 5, 5e-2, 1e-2), ("tiled", 3, (18, 30, 9), 20, 3e-4, 1e-3), ("tiled", 2, (50, 33), 40, 1e-5, 1e-5)])
def test_modewise_in_place_step_equals_the_printed_order_when_no_row_is_shared(kernel, N, J, R, lr_A, lr_B):
    """Every stored entry has rows of its own in every mode, and Psi holds no position twice: then
    no two samples touch the same row, running them at once changes nothing, and one step in
    FTK_HOGWILD_MODEWISE has to give what Algorithm 1 gives when its lines are followed one sample
    after the other -- parameter by parameter.  The step is large enough that following the modes in
    turn matters: the same step with all gradients taken at the starting rows lands elsewhere.
    On the matrix cores (both kernels, ranks padded to blocks of 16) and on the one-lane-per-sample kernels."""
    announce("modewise in-place, conflict-free, kernel=%s order=%d" % (kernel, N))
    nnz = 6000
    rng = np.random.default_rng(11)
    dims = (nnz,) * N
    idx = [rng.permutation(nnz).astype(np.int32) for _ in range(N)]
    vals = rng.uniform(1.0, 5.0, nnz).astype(np.float32)
    M, seed = 60, 0
    while True:   # a sample set without repeated positions (about three in four seeds at this size)
        pos = oracle.sample_positions(seed, M, nnz)
        if len(set(pos.tolist())) == M:
            break
        seed += 1
    lam_A, lam_B = 1e-2, 1e-2
    A, B = oracle.init_factors(3, dims, J, R)
    A_sync, B_sync = [a.copy() for a in A], [b.copy() for b in B]
    with binding.FastTucker(dims, idx, vals, J, R, 3) as ft:
        ft.ftk_set_kernel(kernel)
        assert ft.ftk_kernel_name() == kernel
        ft.ftk_set_mode(binding.FTK_HOGWILD_MODEWISE)
        ft.ftk_sample(seed, M)
        assert np.array_equal(ft.ftk_get_samples(), pos)
        ft.ftk_sgd_step(lr_A, lr_B, lam_A, lam_B)
        gA, gB = ft.ftk_get_factors()
    oracle.sgd_step_hogwild(dims, idx, vals, A, B, pos, lr_A, lr_B, lam_A, lam_B)
    oracle.sgd_step_sync(dims, idx, vals, A_sync, B_sync, pos, lr_A, lr_B, lam_A, lam_B)
    assert_params_close(gA, A, "A")
    assert_params_close(gB, B, "B")
    # teeth: the order is visible at this step size
    far = max(float(np.max(np.abs(A[n] - A_sync[n]) / (np.abs(A[n]) + 1e-6))) for n in range(1, N))
    assert far > 1e-3, far
    assert max(float(np.max(np.abs(B[n] - B_sync[n]))) for n in range(N)) > 1e-5


# ------------------------------------------------------------------------------------------------
# the training loop of the paper's experiments, end to end: decaying step sizes, held-out Gamma
# ------------------------------------------------------------------------------------------------
@pytest.mark.parametrize("mode,sampling", [("sync", "entries"), ("sync", "tiles"), ("hogwild", "entries"),
                                           ("modewise", "entries")])
def test_training_driver_learns_a_planted_tensor(mode, sampling):
    """paper_2204_07104_amd.train on a small planted tensor: RMSE and MAE on the held-out entries (never
    sampled) fall to a fifth of where they start, in every mode and under both sampling rules."""
    import io
    from paper_2204_07104_amd import train
    announce("training driver, %s step, %s sampling" % (mode, sampling))
    out = io.StringIO()
    hist = train.train((300, 200, 100), 66_000, (8, 8, 8), 8, n_samples=6_000, steps=200,
                       alpha_A=5e-3, beta_A=0.05, alpha_B=1.0, beta_B=0.05, lambda_A=1e-3, lambda_B=1e-3,
                       holdout=0.1, planted_rank=4, noise=0.05, seed=1, mode=mode, sampling=sampling,
                       report_every=50, out=out)
    assert [h[0] for h in hist] == [0, 50, 100, 150, 200]
    (_, rmse0, mae0), (_, rmse1, mae1) = hist[0], hist[-1]
    assert np.isfinite([rmse1, mae1]).all()
    assert rmse1 < 0.2 * rmse0, out.getvalue()
    assert mae1 < 0.2 * mae0, out.getvalue()
    assert mae1 <= rmse1


def test_three_contexts_interleaved():
    """Three contexts of different shapes alive at once, stepping in turn (the same kernel instantiations with
    different LDS sizes, tables and grids): each follows its own oracle as if it were alone."""
    announce("three contexts interleaved")
    w1 = synth.replace(synth.WORKLOADS["C2"].scaled(nnz=200_000, n_samples=20_000, dims=(4_800, 1_777, 220)), lr_A=2e-7, lr_B=1e-4)
    w2 = synth.replace(synth.tiny_workload(3, (60, 50, 40), 3_000, (16, 16, 16), 16, 700, seed=5, values="normal"),
                       lr_A=1e-6, lr_B=1e-6)
    w3 = synth.replace(synth.tiny_workload(3, (300, 200, 100), 9_000, (32, 20, 32), 24, 2_500, seed=6, values="normal"),
                       lr_A=1e-8, lr_B=1e-8)
    cases = []
    for w in (w1, w2, w3):
        idx, vals = synth.make_tensor(w)
        A, B = oracle_state(w)
        cases.append((w, idx, vals, A, B, binding.FastTucker(w.dims, idx, vals, w.J, w.R, w.init_seed)))
    try:
        for t in range(3):
            for w, idx, vals, A, B, ft in cases:
                ft.ftk_sample(900 + t, w.n_samples)
            for w, idx, vals, A, B, ft in reversed(cases):
                ft.ftk_sgd_step(w.lr_A, w.lr_B, w.lambda_A, w.lambda_B)
            for w, idx, vals, A, B, ft in cases:
                pos = oracle.sample_positions(900 + t, w.n_samples, w.nnz)
                oracle.sgd_step_sync(w.dims, idx, vals, A, B, pos, w.lr_A, w.lr_B, w.lambda_A, w.lambda_B)
        for w, idx, vals, A, B, ft in cases:
            gA, gB = ft.ftk_get_factors()
            A0, B0 = oracle_state(w)
            assert all(np.isfinite(o).all() for o in A + B)
            assert max(float(np.abs(a - a0).max()) for a, a0 in zip(A, A0)) > 1e-5   # the steps moved something
            for g, o in zip(gA + gB, A + B):
                err = np.abs(g.astype(np.float64) - o)
                assert float((err - 3 * (ATOL + RTOL * np.abs(o))).max()) <= 0.0, w.name
            assert ft.ftk_rmse() == pytest.approx(oracle.rmse(w.dims, idx, vals, A, B), rel=1e-5)
    finally:
        for case in cases:
            case[-1].close()
