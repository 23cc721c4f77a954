"""The entry point that allocates nothing (cals_mttkrp_noalloc: split-K partials in a fixed device array) against
cals_mttkrp, through the C-ABI: same launch plan and kernels, so the results must be bit-identical, and both must
meet the parity bar against the oracle.  Two calls in a row share the array; the second is smaller, so it runs on
the first one's leftovers."""
import numpy as np
import pytest

import oracle as O
from workloads import random_tensor, uniform_factors

pytestmark = pytest.mark.gpu
TOL = 1e-12


def _setup(dims, ranks, seed):
    import torch
    import paper_2010_04678_amd as P
    T = random_tensor(dims, seed, signed=True)
    facs = [uniform_factors(dims, r, seed + 10 + k) for k, r in enumerate(ranks)]
    U = [2.0 * np.hstack([f[n] for f in facs]) - 1.0 for n in range(len(dims))]
    R = U[0].shape[1]
    ld = (R + 15) // 16 * 16
    ctx = P.Context(max_total_rank=ld)
    Td = torch.from_numpy(T).cuda()
    ctx.submit_tensor(Td)
    Ud = []
    for n in range(len(dims)):
        buf = torch.zeros((dims[n], ld), dtype=torch.float64, device="cuda")
        buf[:, :R] = torch.from_numpy(np.ascontiguousarray(U[n])).cuda()
        Ud.append(buf)
    return ctx, T, U, Ud, R, ld


def _compare(ctx, T, U, Ud, R, ld, dims):
    import torch
    for mode in range(1, len(dims) + 1):
        a = torch.full((dims[mode - 1], ld), 777.0, dtype=torch.float64, device="cuda")
        b = torch.full((dims[mode - 1], ld), 777.0, dtype=torch.float64, device="cuda")
        ctx.mttkrp(mode, Ud, a, total_rank=R)
        ctx.mttkrp(mode, Ud, b, total_rank=R, no_alloc=True)
        torch.cuda.synchronize()
        ah, bh = a.cpu().numpy(), b.cpu().numpy()
        assert np.array_equal(ah, bh), (mode, float(np.abs(ah - bh).max()))
        assert np.all(bh[:, R:] == 777.0)
        want = O.mttkrp(T, U, mode)
        scale = O.mttkrp(np.abs(T), [np.abs(u) for u in U], mode)
        assert np.all(np.abs(bh[:, :R] - want) <= TOL * scale + 1e-300), mode


def test_no_alloc_mttkrp_two_calls_in_a_row_the_second_smaller():
    import torch
    # first call: several column blocks, many splits (about 4 MB of partials); second: one tile, a few splits
    big_dims, big_ranks = (129, 65, 33), list(range(1, 21)) + [11] * 20
    small_dims, small_ranks = (17, 13, 11), [3, 1, 5]
    ctx1, T1, U1, Ud1, R1, ld1 = _setup(big_dims, big_ranks, 901)
    ctx2, T2, U2, Ud2, R2, ld2 = _setup(small_dims, small_ranks, 902)
    _compare(ctx1, T1, U1, Ud1, R1, ld1, big_dims)
    _compare(ctx2, T2, U2, Ud2, R2, ld2, small_dims)
    # and once more the large one, now on the small one's leftovers
    _compare(ctx1, T1, U1, Ud1, R1, ld1, big_dims)
    ctx1.close()
    ctx2.close()
    torch.cuda.empty_cache()


def test_no_alloc_mttkrp_order_4_and_refusal_beyond_the_fixed_array():
    import torch
    import paper_2010_04678_amd as P
    dims, ranks = (12, 10, 9, 7), [4, 9, 20]
    ctx, T, U, Ud, R, ld = _setup(dims, ranks, 903)
    _compare(ctx, T, U, Ud, R, ld, dims)
    ctx.close()
    # a launch whose partials cannot fit 256 MiB: mode 1 of a 40000 x 16 x 16 tensor at 512 columns with the split
    # count forced to 2 (planner knob, read when the context is created): 2 x 40000 x 512 doubles = 328 MB.
    # Nothing is enqueued and the error names the reason
    import os
    I1, w = 40000, 512
    os.environ["CALS_MTTKRP_SPLITS"] = "2"
    try:
        ctx = P.Context(max_total_rank=w)
    finally:
        del os.environ["CALS_MTTKRP_SPLITS"]
    Td = torch.ones((16, 16, I1), dtype=torch.float64, device="cuda")
    ctx.submit_tensor(Td)
    Ud = [None] + [torch.ones((16, w), dtype=torch.float64, device="cuda") for _ in range(2)]
    M = torch.zeros((I1, w), dtype=torch.float64, device="cuda")
    ctx.mttkrp(1, Ud, M)                      # the allocating entry point takes it
    torch.cuda.synchronize()
    assert float(M.min()) == 256.0 and float(M.max()) == 256.0
    M.zero_()
    with pytest.raises(P.CalsError) as info:
        ctx.mttkrp(1, Ud, M, no_alloc=True)
    assert info.value.code == P.binding.E_TOOLARGE and "scratch" in str(info.value)
    torch.cuda.synchronize()
    assert float(M.abs().max()) == 0.0        # nothing ran
    ctx.close()
    del Td, M
    torch.cuda.empty_cache()
