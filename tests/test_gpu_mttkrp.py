"""GPU parity of the fused MTTKRP (cals_mttkrp through the C-ABI) against the CPU oracle.

Bar (floating point, fp64): per-element |gpu - oracle| <= 1e-12 * sum|terms| of that element
(for non-negative data that is the element itself, i.e. the relative error)."""
import numpy as np
import pytest

import oracle as O
from workloads import get_config, make_tensor, random_tensor, uniform_factors

pytestmark = pytest.mark.gpu
TOL = 1e-12


def _torch():
    import torch
    return torch


def _fused(dims, ranks, seed, signed=False):
    facs = [uniform_factors(dims, r, seed + k) for k, r in enumerate(ranks)]
    U = [np.hstack([f[n] for f in facs]) for n in range(len(dims))]
    if signed:
        U = [2.0 * u - 1.0 for u in U]
    return U


def _abs_scale(T, U, mode):
    """sum of |terms| per output element = MTTKRP of |T| with |U| (oracle definition, non-negative data)."""
    return O.mttkrp(np.abs(T), [np.abs(u) for u in U], mode)


def _gpu_mttkrp(T, U, pad_to=None, poison=True, rows_after=0, stats_out=None):
    """rows_after: the multi-matrices are views of larger device buffers with that many NaN rows after the last
    factor row (every read of the kernel stays in mapped memory, and a read past the last row poisons the result)."""
    import paper_2010_04678_amd as P
    torch = _torch()
    dims = tuple(T.shape[::-1])
    R = U[0].shape[1]
    ld = pad_to if pad_to is not None else R
    ctx = P.Context(max_total_rank=max(ld, 1) if T.ndim > 3 else max(R, 1))
    Td = torch.from_numpy(T).cuda()
    ctx.submit_tensor(Td)
    Ud = []
    for n in range(T.ndim):
        big = torch.full((dims[n] + rows_after, ld), float("nan") if poison else 0.0, dtype=torch.float64, device="cuda")
        buf = big[:dims[n]]
        buf[:, :R] = torch.from_numpy(np.ascontiguousarray(U[n])).cuda()
        Ud.append(buf)
    out = []
    for mode in range(1, T.ndim + 1):
        M = torch.full((dims[mode - 1], ld), 777.0, dtype=torch.float64, device="cuda")
        ctx.mttkrp(mode, Ud, M, total_rank=R)
        torch.cuda.synchronize()
        Mh = M.cpu().numpy()
        assert np.all(Mh[:, R:] == 777.0), "columns beyond total_rank must not be touched"
        out.append(Mh[:, :R])
    if stats_out is not None:
        stats_out.append(ctx.stats())
    ctx.close()
    return out


CASES = [
    # dims, ranks, signed
    ((17, 13, 11), [3, 1, 5], True),            # odd sizes, ragged everywhere, one 16-column tile
    ((32, 32, 32), [1, 2, 3, 4, 5] * 2, False), # config 1 shape
    ((70, 9, 150), [7] * 5, True),              # two 16-row tiles + tail, contraction much longer than a stage
    ((5, 3, 2), [1], True),                     # smaller than any tile; contracted index shorter than a stage
    ((3, 130, 2), [20, 20, 20, 3], False),      # tiny fast index for modes 2,3 (general wrap path), 4 column tiles
    ((129, 65, 33), list(range(1, 21)) + [11] * 20, True),   # 430 columns = 27 tiles: several column blocks, two launches
    ((40, 24, 20), [20] * 30, False),           # 600 columns = 38 tiles
    ((24, 20, 18), [20] * 21, True),            # 420 columns = 27 tiles (cfg 4's width)
    ((300, 7, 5), [5] * 3, False),              # odd leading dimension (one column per lane), four row tiles per wavefront
]


@pytest.mark.parametrize("dims,ranks,signed", CASES)
def test_mttkrp_matches_oracle_elementwise(dims, ranks, signed):
    T = random_tensor(dims, 7 + dims[0], signed=signed)
    U = _fused(dims, ranks, 100 + dims[1], signed=signed)
    got = _gpu_mttkrp(T, U, pad_to=sum(ranks) + 5)
    for mode in (1, 2, 3):
        want = O.mttkrp(T, U, mode)
        scale = _abs_scale(T, U, mode)
        err = np.abs(got[mode - 1] - want)
        assert np.all(np.isfinite(got[mode - 1]))
        assert np.all(err <= TOL * scale + 1e-300), (mode, float((err / (scale + 1e-300)).max()))


@pytest.mark.parametrize("wn_max", [14, 8, 5])
@pytest.mark.parametrize("dims,ranks,signed", [c for c in CASES if sum(c[1]) >= 192])
def test_mttkrp_every_column_block_width(dims, ranks, signed, wn_max):
    # the library chooses between wide column blocks (up to 14 tiles of 16 columns, fewest passes over the tensor) and
    # narrow ones (up to 8) by a cost model; here each is forced (development knob of the launch planner), so that the
    # kernels of every block width are compared with the oracle whatever the model prefers for these small tensors
    import os
    T = random_tensor(dims, 7 + dims[0], signed=signed)
    U = _fused(dims, ranks, 100 + dims[1], signed=signed)
    os.environ["CALS_MTTKRP_WNMAX"] = str(wn_max)
    try:
        got = _gpu_mttkrp(T, U, pad_to=sum(ranks) + 5)
    finally:
        del os.environ["CALS_MTTKRP_WNMAX"]
    for mode in (1, 2, 3):
        want = O.mttkrp(T, U, mode)
        scale = _abs_scale(T, U, mode)
        err = np.abs(got[mode - 1] - want)
        assert np.all(np.isfinite(got[mode - 1]))
        assert np.all(err <= TOL * scale + 1e-300), (mode, wn_max, float((err / (scale + 1e-300)).max()))


WM_CASES = [((180, 20, 16), [20] * 5, True),          # 180 rows = one 192-row workgroup of three row tiles per wavefront
            ((16, 180, 20), [20] * 7, False),         # the same for an inner mode, 9 column tiles
            ((20, 16, 200), [11] * 4, True),          # two such workgroups in the last mode
            ((129, 65, 33), list(range(1, 21)) + [11] * 20, True),
            ((70, 9, 150), [7] * 5, True)]


@pytest.mark.parametrize("wm", [1, 2, 3, 4])
@pytest.mark.parametrize("dims,ranks,signed", WM_CASES)
def test_mttkrp_every_row_tile_count(dims, ranks, signed, wm):
    # the planner picks 1, 2, 3 or 4 row tiles per wavefront from the row count, the width and the mode's layout; here
    # each is forced on the tile kernel (development knobs, column blocks of up to 9 tiles so that three row tiles
    # stay within the accumulator budget), so that every count meets every read mode whatever the planner prefers
    import os
    T = random_tensor(dims, 11 + dims[0], signed=signed)
    U = _fused(dims, ranks, 200 + dims[1], signed=signed)
    env = {"CALS_MTTKRP_WM": str(wm), "CALS_MTTKRP_KERNEL": "1", "CALS_MTTKRP_WNMAX": "7" if wm == 4 else "9"}
    os.environ.update(env)
    try:
        got = _gpu_mttkrp(T, U, pad_to=sum(ranks) + 2)
    finally:
        for k in env:
            del os.environ[k]
    for mode in (1, 2, 3):
        want = O.mttkrp(T, U, mode)
        scale = _abs_scale(T, U, mode)
        err = np.abs(got[mode - 1] - want)
        assert np.all(np.isfinite(got[mode - 1]))
        assert np.all(err <= TOL * scale + 1e-300), (mode, wm, float((err / (scale + 1e-300)).max()))


@pytest.mark.parametrize("force", ["1", "0"])
@pytest.mark.parametrize("dims,ranks,signed", [c for c in CASES if c[0][0] >= 16 and c[0][0] % 4 != 0] +
                         [((19, 6, 5), [2, 3], True), ((33, 4, 3), [16] * 3, False), ((255, 7, 3), [5, 9, 20], True)])
def test_mttkrp_first_mode_not_a_multiple_of_four(dims, ranks, signed, force):
    # tensors whose first mode is not a multiple of 4 (the paper's datasets: 405, 255, 299): modes 2 and up read runs of
    # I1 contiguous elements that are not 16-byte aligned.  Narrow launches read them with padded runs and shifted
    # 16-byte loads, wide ones element by element; here each way is forced at every width (development knob)
    import os
    T = random_tensor(dims, 11 + dims[0], signed=signed)
    U = _fused(dims, ranks, 300 + dims[1], signed=signed)
    os.environ["CALS_MTTKRP_CONTIGU"] = force
    try:
        got = _gpu_mttkrp(T, U, pad_to=sum(ranks) + 3)
    finally:
        del os.environ["CALS_MTTKRP_CONTIGU"]
    for mode in (1, 2, 3):
        want = O.mttkrp(T, U, mode)
        scale = _abs_scale(T, U, mode)
        err = np.abs(got[mode - 1] - want)
        assert np.all(np.isfinite(got[mode - 1]))
        assert np.all(err <= TOL * scale + 1e-300), (mode, force, float((err / (scale + 1e-300)).max()))


@pytest.mark.parametrize("dims,ranks,pad", [((37, 5, 4), [20] * 4, 3), ((37, 5, 4), [20] * 4, 4), ((255, 7, 3), [5, 9, 20], 3),
                                            ((255, 7, 3), [5, 9, 20], 2), ((33, 4, 3), [16] * 3, 0), ((19, 6, 5), [2, 3], 1)])
def test_padded_run_reads_never_touch_rows_after_the_factor(dims, ranks, pad):
    # padded-run reads count the first mode rounded up to 4; the up to three padding positions have no factor row.
    # The multi-matrices here are followed in memory by NaN rows: a kernel that fetched a row past the end would turn
    # every output of that column into NaN (0 * NaN).  Odd and even leading dimensions (one / two columns per lane),
    # widths below and above 64 columns (packed and per-row production of the Khatri-Rao tile)
    import os
    T = random_tensor(dims, 13 + dims[0], signed=True)
    U = _fused(dims, ranks, 400 + dims[1], signed=True)
    os.environ["CALS_MTTKRP_CONTIGU"] = "1"
    try:
        got = _gpu_mttkrp(T, U, pad_to=sum(ranks) + pad, rows_after=8)
    finally:
        del os.environ["CALS_MTTKRP_CONTIGU"]
    for mode in (1, 2, 3):
        want = O.mttkrp(T, U, mode)
        scale = _abs_scale(T, U, mode)
        assert np.all(np.isfinite(got[mode - 1])), mode
        assert np.all(np.abs(got[mode - 1] - want) <= TOL * scale + 1e-300), (mode, pad)


ROWS_CASES = [
    # dims, ranks, signed: fast contracted index a multiple of 4 and at least 16 in every mode
    ((200, 24, 20), list(range(1, 11)) * 2, False),      # configuration 2's row count and width (110): 13 row tiles
    ((48, 40, 36), [2, 7, 1, 12, 9], True),              # 3 row tiles, 2 column tiles
    ((52, 200, 16), [20] * 6 + [8], True),               # 52 rows (mode 1), 200 (mode 2), 16 (mode 3); 128 columns
    ((180, 20, 16), [16, 20, 20, 8], False),             # 12 of 13 row tiles live
    ((100, 36, 20), [13, 20, 7], True),                  # 7 row tiles
    ((300, 20, 16), [20] * 5 + [3], False),              # several row blocks when a small variant is forced
    ((64, 32, 28), [1], True),                           # a single column
]


@pytest.mark.parametrize("variant", [(4, 2), (4, 4), (7, 2), (13, 2)])
@pytest.mark.parametrize("dims,ranks,signed", ROWS_CASES)
def test_mttkrp_rows_kernel_every_variant(dims, ranks, signed, variant):
    # the second kernel of the fused MTTKRP (a wavefront holds all row tiles of its row block, lanes form their own
    # Khatri-Rao values, four wavefronts share the contraction range): every variant forced in turn (development
    # knobs of the launch planner, read when the context is created), both tensor read modes (mode 1: row pairs; modes
    # 2 and 3: contiguous contraction), full and ragged tiles, one and several row blocks and column groups
    import os
    T = random_tensor(dims, 17 + dims[0], signed=signed)
    U = _fused(dims, ranks, 500 + dims[1], signed=signed)
    R = sum(ranks)
    env = {"CALS_MTTKRP_KERNEL": "2", "CALS_MTTKRP_ROWS_WMB": str(variant[0]), "CALS_MTTKRP_ROWS_WNB": str(variant[1])}
    for pad in (R + (R % 2), (R + 15) // 16 * 16 + 16):
        st = []
        os.environ.update(env)
        try:
            got = _gpu_mttkrp(T, U, pad_to=pad, stats_out=st)
        finally:
            for k in env:
                del os.environ[k]
        # a variant takes a width when its column tiles split into groups of wnb and wnb - 1 tiles
        nt, wnb = (R + 15) // 16, variant[1]
        groups = (nt + wnb - 1) // wnb
        takes = groups * wnb - nt <= groups
        assert st[0].mttkrp_rows_launches == (3 if takes else 0), "every mode of these shapes suits the rows kernel"
        for mode in (1, 2, 3):
            want = O.mttkrp(T, U, mode)
            scale = _abs_scale(T, U, mode)
            assert np.all(np.isfinite(got[mode - 1]))
            assert np.all(np.abs(got[mode - 1] - want) <= TOL * scale + 1e-300), (mode, variant, pad)


def test_mttkrp_rows_kernel_is_chosen_for_short_modes_and_is_bit_reproducible():
    # left to itself the planner gives the 200-row modes of a configuration-2-shaped problem to the rows kernel
    # (one row block, four column groups); its four-wavefront exchange and the split-K reduction add in a fixed order
    cfg = get_config(2)
    dims = (200, 200, 40)
    T = make_tensor(cfg, dims)
    U = _fused(dims, cfg.ranks, 300)
    st = []
    a = _gpu_mttkrp(T, U, pad_to=112, stats_out=st)
    b = _gpu_mttkrp(T, U, pad_to=112)
    assert st[0].mttkrp_rows_launches >= 2
    for mode in range(3):
        assert np.array_equal(a[mode], b[mode])
        want = O.mttkrp(T, U, mode + 1)
        assert np.all(np.abs(a[mode] - want) <= TOL * np.abs(want))


def test_mttkrp_config2_shape_reduced_depth():
    # configuration 2's fused width (110) on a tensor with its row count but fewer slabs (oracle stays fast)
    cfg = get_config(2)
    dims = (200, 200, 24)
    T = make_tensor(cfg, dims)
    U = _fused(dims, cfg.ranks, 300)
    got = _gpu_mttkrp(T, U)
    for mode in (1, 2, 3):
        want = O.mttkrp(T, U, mode)
        rel = np.abs(got[mode - 1] - want) / np.abs(want)
        assert rel.max() <= TOL, (mode, rel.max())


def test_mttkrp_is_bit_reproducible_and_fusion_is_exact():
    # Eq. (2): a model's block of the fused result equals its solo MTTKRP.  With a fixed split of the
    # contraction range the GPU result is also run-to-run identical.
    dims, ranks = (48, 40, 36), [2, 7, 1, 12, 9]
    T = random_tensor(dims, 55, signed=True)
    U = _fused(dims, ranks, 500, signed=True)
    a = _gpu_mttkrp(T, U)
    b = _gpu_mttkrp(T, U)
    for mode in range(3):
        assert np.array_equal(a[mode], b[mode])
    c0 = 0
    for r in ranks:
        solo = _gpu_mttkrp(T, [u[:, c0:c0 + r] for u in U])
        for mode in range(3):
            scale = _abs_scale(T, [u[:, c0:c0 + r] for u in U], mode + 1)
            assert np.all(np.abs(solo[mode] - a[mode][:, c0:c0 + r]) <= 1e-13 * scale)
        c0 += r


def _gpu_mttkrp_reuse(T, U, pad_to=None):
    """Mode-2 and mode-3 MTTKRPs through the two-step path (contraction with U1 first)."""
    import paper_2010_04678_amd as P
    torch = _torch()
    dims = (T.shape[2], T.shape[1], T.shape[0])
    R = U[0].shape[1]
    ld = pad_to if pad_to is not None else R
    ctx = P.Context(max_total_rank=max(ld, 1), flags=P.CTX_REUSE)
    ctx.submit_tensor(torch.from_numpy(T).cuda())
    Ud = []
    for n in range(3):
        buf = torch.full((dims[n], ld), float("nan"), dtype=torch.float64, device="cuda")
        buf[:, :R] = torch.from_numpy(np.ascontiguousarray(U[n])).cuda()
        Ud.append(buf)
    M2 = torch.full((dims[1], ld), 777.0, dtype=torch.float64, device="cuda")
    M3 = torch.full((dims[2], ld), 777.0, dtype=torch.float64, device="cuda")
    ctx.mttkrp_reuse(Ud, M2, M3, total_rank=R)
    torch.cuda.synchronize()
    out = []
    for M in (M2, M3):
        Mh = M.cpu().numpy()
        assert np.all(Mh[:, R:] == 777.0), "columns beyond total_rank must not be touched"
        out.append(Mh[:, :R])
    ctx.close()
    return out


@pytest.mark.parametrize("dims,ranks,signed", CASES)
def test_two_step_mttkrp_matches_oracle_elementwise(dims, ranks, signed):
    # the mode-2 and mode-3 results of the two-step path (tensor contracted with the mode-1 factors first) are the
    # plain MTTKRPs: same bar, against the same definition
    T = random_tensor(dims, 7 + dims[0], signed=signed)
    U = _fused(dims, ranks, 100 + dims[1], signed=signed)
    R = sum(ranks)
    for pad in (R + 5, (R + 15) // 16 * 16):       # odd and 16-aligned leading dimension (one / two columns per lane)
        got = _gpu_mttkrp_reuse(T, U, pad_to=pad)
        for k, mode in enumerate((2, 3)):
            want = O.mttkrp(T, U, mode)
            scale = _abs_scale(T, U, mode)
            err = np.abs(got[k] - want)
            assert np.all(np.isfinite(got[k]))
            assert np.all(err <= TOL * scale + 1e-300), (mode, pad, float((err / (scale + 1e-300)).max()))


def _random_cases(n, seed):
    rng = np.random.default_rng(seed)
    out = []
    for _ in range(n):
        dims = tuple(int(rng.choice([1, 2, 3, 5, 8, 15, 16, 17, 31, 32, 33, 48, 64, 65, 96, 100, 127, 128, 130])) for _ in range(3))
        if dims[0] * dims[1] * dims[2] > 600000:
            dims = (dims[0], min(dims[1], 33), dims[2])
        total = int(rng.choice([1, 2, 7, 15, 16, 17, 31, 32, 33, 47, 48, 49, 63, 64, 65, 100, 112, 113, 130, 224, 225]))
        ranks, left = [], total
        while left > 0:
            r = int(min(left, rng.integers(1, 33)))
            ranks.append(r)
            left -= r
        out.append((dims, ranks, bool(rng.integers(0, 2)), int(rng.integers(0, 3))))
    return out


@pytest.mark.parametrize("dims,ranks,signed,padkind", _random_cases(36, 2024))
def test_mttkrp_seeded_random_shapes(dims, ranks, signed, padkind):
    # shapes and widths around every tile, stage, pairing and packing boundary of the kernel (16-row and 16-column
    # tiles, 4-/16-index stages, two-rows-per-load in mode 1, packed production up to 64 columns), plain and two-step
    T = random_tensor(dims, 11 + sum(dims), signed=signed)
    U = _fused(dims, ranks, 200 + dims[2], signed=signed)
    R = sum(ranks)
    pad = [R, R + 1, (R + 15) // 16 * 16][padkind]
    got = _gpu_mttkrp(T, U, pad_to=pad)
    got2 = _gpu_mttkrp_reuse(T, U, pad_to=pad)
    for mode in (1, 2, 3):
        want = O.mttkrp(T, U, mode)
        scale = _abs_scale(T, U, mode)
        assert np.all(np.abs(got[mode - 1] - want) <= TOL * scale + 1e-300), (mode, "plain")
        if mode > 1:
            assert np.all(np.abs(got2[mode - 2] - want) <= TOL * scale + 1e-300), (mode, "two-step")
