"""GPU parity for tensors of order above 3 (cals_submit_tensor_nd and everything behind it) against the CPU oracle.

Same bars as for order 3: MTTKRP per element within 1e-12 of the sum of the absolute values of its terms; fits
within 1e-8, factors within 1e-6 relative, identical iteration counts, statuses and retirement order."""
import numpy as np
import pytest

import oracle as O
from workloads import low_rank_tensor, random_tensor, uniform_factors

from test_gpu_cals import compare, run_gpu
from test_gpu_mttkrp import TOL, _abs_scale, _fused, _gpu_mttkrp

pytestmark = pytest.mark.gpu

ND_CASES = [
    # dims, ranks, signed
    ((7, 5, 6, 4), [3, 1, 5], True),               # odd sizes, every run shorter than a stage somewhere
    ((20, 18, 17, 16), [5] * 4, False),            # fast run of 16+ rows in every mode (wrap and affine paths)
    ((33, 4, 3, 35), [20, 20, 3], True),           # long first and last modes, tiny inner modes
    ((3, 40, 2, 3), [7, 9], False),                # tiny fast index (general path), long inner mode
    ((6, 5, 4, 3, 5), [2, 7, 1, 12], True),        # order 5: runs of two modes on both sides
    ((9, 1, 8, 1, 7), [4, 4], False),              # singleton modes inside
    ((4, 3, 2, 3, 2, 4), list(range(1, 9)), True),  # order 6
    ((16, 16, 16, 16), [20] * 13, False),          # 260 columns: several column tiles, split contraction
    ((5, 7, 23, 19), [6, 11], True),               # two-step: the second step's range cut into ragged slices
]


@pytest.mark.parametrize("dims,ranks,signed", ND_CASES)
def test_mttkrp_order_n_matches_oracle_elementwise(dims, ranks, signed):
    T = random_tensor(dims, 17 + dims[0], signed=signed)
    U = _fused(dims, ranks, 400 + dims[1], signed=signed)
    got = _gpu_mttkrp(T, U, pad_to=sum(ranks) + 5)
    for mode in range(1, len(dims) + 1):
        want = O.mttkrp(T, U, mode)
        scale = _abs_scale(T, U, mode)
        err = np.abs(got[mode - 1] - want)
        assert np.all(np.isfinite(got[mode - 1]))
        assert np.all(err <= TOL * scale + 1e-300), (mode, float((err / (scale + 1e-300)).max()))


def test_mttkrp_order_n_seeded_random_shapes():
    rng = np.random.default_rng(20260)
    for case in range(16):
        N = int(rng.integers(4, 7))
        dims = tuple(int(d) for d in rng.integers(1, [0, 0, 0, 0, 24, 12, 7][N], size=N))
        ranks = [int(r) for r in rng.integers(1, 21, size=int(rng.integers(1, 6)))]
        T = random_tensor(dims, 3000 + case, signed=True)
        U = _fused(dims, ranks, 3100 + case, signed=True)
        got = _gpu_mttkrp(T, U, pad_to=sum(ranks) + int(rng.integers(0, 3)))
        for mode in range(1, N + 1):
            want = O.mttkrp(T, U, mode)
            scale = _abs_scale(T, U, mode)
            err = np.abs(got[mode - 1] - want)
            assert np.all(err <= TOL * scale + 1e-300), (case, dims, ranks, mode)


def _models(dims, ranks, seed, flags=0, tol=1e-5, max_iters=30, alpha=1.2):
    out = []
    for k, r in enumerate(ranks):
        f = flags[k % len(flags)] if isinstance(flags, (list, tuple)) else flags
        out.append(dict(rank=r, init=uniform_factors(dims, r, seed + k), tol=[tol, -1.0][k % 2],
                        max_iters=[max_iters, 9][k % 2], flags=f, ls_alpha=alpha))
    return out


@pytest.mark.parametrize("dims", [(12, 10, 9, 8), (7, 6, 5, 4, 6), (40, 3, 4, 300)])
def test_order_n_queue_matches_oracle(dims):
    T = low_rank_tensor(dims, 4, 500 + dims[0], noise=0.05)
    ranks = [3, 1, 4, 2, 5, 3, 2, 6]
    models = _models(dims, ranks, 600)
    for rstar, slots in [(sum(ranks), 0), (9, 3)]:
        ref = O.cals(T, models, rstar, slots)
        results, facs, st = run_gpu(T, models, rstar, slots, rounds_per_call=3)
        compare(results, facs, ref, models)
        assert st.rounds == ref["rounds"]
        assert abs(st.tensor_norm_sq - O.norm_sq(T)) <= 1e-12 * st.tensor_norm_sq


def test_order_4_nonneg_linesearch_and_plain_models_together():
    dims = (11, 9, 8, 7)
    T = np.maximum(low_rank_tensor(dims, 3, 700, noise=0.05), 0.0)
    ranks = [2, 3, 4, 1, 5, 2, 3]
    models = _models(dims, ranks, 710, flags=[O.FLAG_NONNEG, O.FLAG_LINESEARCH, 0], max_iters=40, alpha=1.2)
    ref = O.cals(T, models, 12, 4)
    assert max(ref["iters"]) > 9
    results, facs, st = run_gpu(T, models, 12, 4, rounds_per_call=5)
    compare(results, facs, ref, models)
    ls = [r for r in results if models[r.model_id]["flags"] == O.FLAG_LINESEARCH]
    assert sum(r.ls_accepted for r in ls) > 0
    for r in results:
        if models[r.model_id]["flags"] == O.FLAG_NONNEG:
            assert min(u.min() for u in facs[r.model_id][0]) >= 0.0


def test_order_4_with_a_trailing_singleton_equals_the_order_3_run_on_the_gpu():
    dims3 = (14, 12, 10)
    T3 = low_rank_tensor(dims3, 3, 720, noise=0.1)
    T4 = np.ascontiguousarray(T3.reshape((1,) + T3.shape))
    ranks = [2, 4, 3]
    m3 = [dict(rank=r, init=uniform_factors(dims3, r, 730 + k), tol=-1.0, max_iters=12, flags=0, ls_alpha=1.0)
          for k, r in enumerate(ranks)]
    m4 = [dict(m, init=list(m["init"]) + [np.ones((1, m["rank"]))]) for m in m3]
    r3, f3, _ = run_gpu(T3, m3, 9)
    r4, f4, _ = run_gpu(T4, m4, 9)
    for a, b in zip(r3, r4):
        assert a.model_id == b.model_id and a.iters == b.iters
        assert abs(a.fit - b.fit) <= 1e-9
        Ua, la = f3[a.model_id]
        Ub, lb = f4[b.model_id]
        for n in range(2):
            assert np.allclose(Ua[n], Ub[n], rtol=1e-7, atol=1e-9)
        assert np.allclose(Ua[2] * la, Ub[2] * (lb * Ub[3][0]), rtol=1e-7, atol=1e-9)


def test_order_n_argument_errors_and_reuse_flag():
    import paper_2010_04678_amd as P
    ctx = P.Context(max_total_rank=8)
    with pytest.raises(P.CalsError) as e:
        ctx.submit_tensor(np.zeros((2,) * 7))
    assert e.value.code == -1                                   # order above CALS_MAX_MODES
    ctx.close()
    dims = (6, 5, 4, 3)
    T = random_tensor(dims, 5)
    ctx = P.Context(max_total_rank=8, flags=P.CTX_REUSE)        # two-step sweeps: same results up to rounding order
    ctx.submit_tensor(T)
    with pytest.raises(ValueError):
        ctx.enqueue_model(uniform_factors(dims[:3], 2, 1))      # three matrices for a four-mode tensor
    init = uniform_factors(dims, 2, 1)
    ctx.enqueue_model(init, tol=-1.0, max_iters=5)
    ctx.run()
    (r,) = ctx.poll_retired()
    ref = O.cp_als(T, init, tol=-1.0, max_iters=5)
    assert r.iters == 5 and abs(r.fit - ref["fit"]) <= 1e-8
    ctx.close()


@pytest.mark.parametrize("seed", list(range(8)))
def test_seeded_random_order_n_queues_match_oracle(seed):
    # random small jobs on tensors of order 3 to 5: dims, ranks, tolerances, caps, R*, slot limits and all four
    # combinations of the two extensions (plain, NONNEG, LINESEARCH, both); some with a tall mode
    rng = np.random.default_rng(8000 + seed)
    N = int(rng.choice([3, 4, 4, 5]))
    dims = [int(rng.choice([2, 3, 5, 8, 11, 17])) for _ in range(N)]
    if seed % 4 == 3:
        dims[int(rng.integers(0, N))] = int(rng.choice([270, 300]))           # row-blocked update kernels
    dims = tuple(dims)
    T = low_rank_tensor(dims, int(rng.integers(2, 5)), 8100 + seed, noise=0.05)
    models = []
    for k in range(int(rng.integers(3, 10))):
        r = int(rng.choice([1, 2, 3, 4, 5, 7, 8, 9, 12, 16, 17, 20, 21, 32]))
        models.append(dict(rank=r, init=uniform_factors(dims, r, 8200 + 100 * seed + k),
                           tol=float(rng.choice([-1.0, 1e-3, 1e-5])), max_iters=int(rng.integers(2, 22)),
                           flags=int(rng.choice([0, 1, 2, 3])), ls_alpha=float(rng.choice([1.1, 1.3, 2.0, 3.0]))))
    rmax = max(m["rank"] for m in models)
    rstar = int(rng.integers(rmax, rmax + 40))
    slots = int(rng.choice([0, 2, 3, 5]))
    ref = O.cals(T, models, rstar, slots)
    results, facs, st = run_gpu(T, models, rstar, slots, rounds_per_call=int(rng.integers(1, 9)))
    compare(results, facs, ref, models)
    assert st.rounds == ref["rounds"]


def _gpu_mttkrp_reuse_nd(T, U, pad_to):
    import torch
    import paper_2010_04678_amd as P
    dims = tuple(T.shape[::-1])
    R = U[0].shape[1]
    ld = pad_to
    ctx = P.Context(max_total_rank=ld, flags=P.CTX_REUSE)
    ctx.submit_tensor(torch.from_numpy(T).cuda())
    Ud, Md = [], []
    for n in range(T.ndim):
        buf = torch.full((dims[n], ld), float("nan"), dtype=torch.float64, device="cuda")
        buf[:, :R] = torch.from_numpy(np.ascontiguousarray(U[n])).cuda()
        Ud.append(buf)
        Md.append(torch.full((dims[n], ld), 777.0, dtype=torch.float64, device="cuda"))
    ctx.mttkrp_reuse_nd(Ud, Md, total_rank=R)
    torch.cuda.synchronize()
    out = [m.cpu().numpy() for m in Md]
    ctx.close()
    for n in range(1, T.ndim):
        assert np.all(out[n][:, R:] == 777.0)
    return [m[:, :R] for m in out]


@pytest.mark.parametrize("dims,ranks,signed", ND_CASES)
def test_two_step_mttkrp_order_n_matches_oracle_elementwise(dims, ranks, signed):
    T = random_tensor(dims, 17 + dims[0], signed=signed)
    U = _fused(dims, ranks, 400 + dims[1], signed=signed)
    pad = (sum(ranks) + 5 + 1) // 2 * 2 if dims[0] % 2 else sum(ranks) + 5       # even and odd leading dimensions
    got = _gpu_mttkrp_reuse_nd(T, U, pad_to=pad)
    for mode in range(2, len(dims) + 1):
        want = O.mttkrp(T, U, mode)
        scale = _abs_scale(T, U, mode)
        err = np.abs(got[mode - 1] - want)
        assert np.all(np.isfinite(got[mode - 1]))
        assert np.all(err <= TOL * scale + 1e-300), (mode, float((err / (scale + 1e-300)).max()))


def test_two_step_line_search_order_4_with_a_long_first_mode():
    # line search only (no clipping), first mode far longer than the buffer is wide: the extrapolated point's
    # contraction is the combination of the stored ones, and the chain of contractions is rebuilt from it
    import paper_2010_04678_amd as P
    dims = (350, 5, 4, 6)
    T = low_rank_tensor(dims, 3, 850, noise=0.02)
    models = _models(dims, [3, 1, 4, 2, 5, 3, 2], 860, flags=[O.FLAG_LINESEARCH, O.FLAG_LINESEARCH, 0], alpha=1.5)
    ref = O.cals(T, models, 10, 3)
    results, facs, st = run_gpu(T, models, 10, 3, rounds_per_call=4, ctx_flags=P.CTX_REUSE)
    compare(results, facs, ref, models)
    assert st.rounds == ref["rounds"]
    assert sum(r.ls_accepted for r in results) > 0


@pytest.mark.parametrize("dims", [(12, 10, 9, 8), (7, 6, 5, 4, 6), (300, 3, 4, 40)])
def test_two_step_sweeps_order_n_match_oracle(dims):
    import paper_2010_04678_amd as P
    T = np.abs(low_rank_tensor(dims, 4, 500 + dims[0], noise=0.05))
    ranks = [3, 1, 4, 2, 5, 3, 2, 6]
    models = _models(dims, ranks, 600, flags=[0, O.FLAG_LINESEARCH, O.FLAG_NONNEG, O.FLAG_NONNEG | O.FLAG_LINESEARCH])
    ref = O.cals(T, models, 12, 4)
    results, facs, st = run_gpu(T, models, 12, 4, rounds_per_call=3, ctx_flags=P.CTX_REUSE)
    compare(results, facs, ref, models)
    assert st.rounds == ref["rounds"]
