"""Edge and degenerate cases of the CALS path on the GPU, each against the CPU oracle: empty queue, extreme ranks,
a singleton dimension, total rank that fills R* exactly, a tall mode with the widest model (row-blocked update),
and an all-zero tensor (every model fails numerically at once)."""
import numpy as np
import pytest

import oracle as O
from workloads import random_tensor, uniform_factors

from test_gpu_cals import compare, run_gpu

pytestmark = pytest.mark.gpu


def _model(dims, rank, seed, **kw):
    m = dict(rank=rank, init=uniform_factors(dims, rank, seed), tol=-1.0, max_iters=5, flags=0, ls_alpha=1.0)
    m.update(kw)
    return m


def _lowrank_tensor(dims, R, seed, noise=0.01):
    A = uniform_factors(dims, R, seed)
    T = np.einsum("ir,jr,kr->kji", *A)
    return np.ascontiguousarray(T + noise * random_tensor(dims, seed + 1, signed=True) * np.sqrt((T ** 2).mean()))


def test_empty_queue_is_a_no_op():
    import paper_2010_04678_amd as P
    ctx = P.Context(max_total_rank=16)
    ctx.submit_tensor(random_tensor((4, 3, 2), 1))
    assert ctx.iterate(3) == 0
    ctx.run()
    assert ctx.poll_retired() == []
    st = ctx.stats()
    assert st.rounds == 0 and st.n_active == 0 and st.models_queued == 0 and st.models_retired == 0
    ctx.close()


def test_rank_1_and_rank_32_side_by_side_fill_rstar_exactly():
    # total rank 32 + 1 + 4 = 37 = R*: not a multiple of the 16-column tile; the widest model the library takes
    dims = (40, 33, 21)
    T = _lowrank_tensor(dims, 6, 11)
    models = [_model(dims, 32, 1, max_iters=4), _model(dims, 1, 2), _model(dims, 4, 3, tol=1e-4, max_iters=40)]
    ref = O.cals(T, models, 37, 0)
    results, facs, st = run_gpu(T, models, 37)
    compare(results, facs, ref, models)
    assert max(ref["total_rank_log"]) == 37


def test_head_of_line_blocking_when_next_model_does_not_fit():
    # R* = 10: the rank-8 model blocks the queue although the rank-2 model behind it would fit (Alg. 3 fill rule)
    dims = (12, 10, 8)
    T = _lowrank_tensor(dims, 3, 21)
    models = [_model(dims, 6, 1, max_iters=3), _model(dims, 8, 2, max_iters=2), _model(dims, 2, 3, max_iters=2)]
    ref = O.cals(T, models, 10, 0)
    results, facs, st = run_gpu(T, models, 10, rounds_per_call=1)
    compare(results, facs, ref, models)
    assert [r.model_id for r in results] == [0, 1, 2]
    assert st.rounds == 3 + 2


def test_one_slot_runs_the_models_one_after_the_other_with_the_same_results():
    # one slot = plain CP-ALS, model after model (what bench.py --one-at-a-time times); the models of a concurrent run
    # do not influence each other, so both runs agree with the oracle and with each other
    from workloads import get_config, make_models, make_tensor
    cfg = get_config(1)
    T = make_tensor(cfg)
    models = make_models(cfg)
    for k, m in enumerate(models):
        m["tol"] = [-1.0, 1e-5][k % 2]
    ref = O.cals(T, models, max(m["rank"] for m in models), 1)
    assert list(ref["retire_order"]) == list(range(len(models)))        # a queue of one slot keeps the input order
    one, facs1, st1 = run_gpu(T, models, max(m["rank"] for m in models), 1, rounds_per_call=5)
    compare(one, facs1, ref, models)
    assert st1.rounds == sum(r.iters for r in one)
    many, facsm, stm = run_gpu(T, models, cfg.max_total_rank, cfg.max_slots)
    assert stm.rounds == max(r.iters for r in many)
    by_id = {r.model_id: r for r in many}
    for r in one:
        q = by_id[r.model_id]
        assert (r.iters, r.status) == (q.iters, q.status) and abs(r.fit - q.fit) <= 1e-8
        for a, b in zip(facs1[r.model_id][0], facsm[r.model_id][0]):
            assert np.abs(a - b).max() <= 1e-6 * max(1.0, np.abs(b).max())


def test_round_log_follows_the_queue():
    # one record per round: fused width and number of active models as Alg. 3's fill and removal loops leave them
    import torch
    import paper_2010_04678_amd as P
    dims = (20, 16, 12)
    T = _lowrank_tensor(dims, 3, 4100)
    ranks, iters = [4, 3, 5, 2, 6], [3, 5, 2, 4, 3]
    for flags in (0, P.CTX_TIMING):
        ctx = P.Context(max_total_rank=10, max_slots=2, flags=flags)
        ctx.submit_tensor(torch.from_numpy(T).cuda())
        for k, (r, it) in enumerate(zip(ranks, iters)):
            ctx.enqueue_model(uniform_factors(dims, r, 4200 + k), tol=-1.0, max_iters=it)
        ctx.iterate(4)
        part = ctx.round_log()
        ctx.run()
        log = ctx.round_log()
        st = ctx.stats()
        assert log[:len(part)] == part or flags               # timings of earlier rounds do not change afterwards
        assert [r[0] for r in log] == list(range(st.rounds))
        # replay: two slots, R* = 10: (4,3) -> 3 rounds, model 0 leaves; (3,5): 5+3 > 10 blocks ... computed by hand below
        active, nxt, left, want = [], 0, list(iters), []
        while nxt < len(ranks) or active:
            while nxt < len(ranks) and len(active) < 2 and sum(ranks[k] for k in active) + ranks[nxt] <= 10:
                active.append(nxt); nxt += 1
            want.append((len(active), sum(ranks[k] for k in active)))
            for k in active:
                left[k] -= 1
            active = [k for k in active if left[k] > 0]
        assert [(r[1], r[2]) for r in log] == want
        assert abs(sum(r[4] for r in log) - st.mttkrp_flops) <= 1e-9 * st.mttkrp_flops
        assert all(r[4] == 2.0 * 3 * r[2] * 20 * 16 * 12 for r in log)
        assert all((r[3] > 0.0) == bool(flags) for r in log)
        assert ctx.round_log(first_round=2, cap=3) == log[2:5]
        ctx.close()


def test_singleton_dimension():
    dims = (1, 9, 7)                                      # a matrix in disguise: mode-1 factors are 1 x R
    T = random_tensor(dims, 3)
    models = [_model(dims, 1, 1, max_iters=6), _model(dims, 1, 2, max_iters=6), _model(dims, 2, 5, max_iters=6)]
    ref = O.cals(T, models, 8, 0)
    results, facs, st = run_gpu(T, models, 8)
    compare(results, facs, ref, models)


def test_tall_mode_row_blocked_update_with_widest_model():
    # 700 rows: the update of mode 1 runs as row blocks (two launches); 300 rows: two blocks with a ragged tail
    dims = (700, 300, 3)
    T = _lowrank_tensor(dims, 5, 31)
    models = [_model(dims, 32, 1, max_iters=3), _model(dims, 3, 2, tol=1e-5, max_iters=30), _model(dims, 17, 4, max_iters=4)]
    ref = O.cals(T, models, 64, 0)
    results, facs, st = run_gpu(T, models, 64)
    compare(results, facs, ref, models)


def test_all_zero_tensor_fails_every_model_numerically():
    import paper_2010_04678_amd as P
    dims = (6, 5, 4)
    T = np.zeros((4, 5, 6))
    models = [_model(dims, 2, 1), _model(dims, 3, 2)]
    ref = O.cals(T, models, 8, 0)
    results, facs, st = run_gpu(T, models, 8)
    assert [r.model_id for r in results] == list(ref["retire_order"]) == [0, 1]
    for r in results:
        assert r.status == P.NUMERICAL == ref["status"][r.model_id]
        assert r.iters == ref["iters"][r.model_id] == 0


def test_nonneg_ranks_at_the_kernel_width_boundaries():
    # the non-negative update is compiled for widths 4, 8, ..., 32: ranks on both sides of each boundary, and 1 and 32
    dims = (37, 29, 23)
    T = np.ascontiguousarray(random_tensor(dims, 900, signed=True) * 0.25 +
                             np.einsum("ir,jr,kr->kji", *uniform_factors(dims, 5, 901)))
    models = [_model(dims, r, 910 + r, flags=O.FLAG_NONNEG, max_iters=6) for r in (1, 4, 5, 8, 9, 12, 13, 16, 17, 20, 21, 24, 25, 28, 29, 32)]
    R = sum(m["rank"] for m in models)
    ref = O.cals(T, models, R, 0)
    results, facs, st = run_gpu(T, models, R, 0, rounds_per_call=2)
    compare(results, facs, ref, models)
    for r in results:
        assert min(u.min() for u in facs[r.model_id][0]) >= 0.0


def test_yardsticks_return_plausible_rates():
    import torch
    import paper_2010_04678_amd as P
    ctx = P.Context(max_total_rank=16)
    assert ctx.yardstick(3) >= 1 and ctx.yardstick(2) > 100.0          # compute units, MHz
    buf = torch.ones(1 << 24, dtype=torch.float64, device="cuda")      # 128 MiB
    assert ctx.yardstick(1, buf, reps=2) > 100.0                       # GB/s
    assert ctx.yardstick(0, reps=1) > 1.0                              # TFLOP/s
    for bad in (dict(kind=7), dict(kind=1, buf=None), dict(kind=0, reps=0)):
        with pytest.raises(P.CalsError) as e:
            ctx.yardstick(bad.get("kind", 0), bad.get("buf"), bad.get("reps", 1))
        assert e.value.code == -1
    ctx.close()


def test_cp_cals_driver_matches_per_model_oracle_runs():
    # the convenience driver: every model equals its own plain CP-ALS (Alg. 1), whatever R* it picks
    import paper_2010_04678_amd as P
    dims = (30, 26, 22)
    T = _lowrank_tensor(dims, 4, 77, noise=0.05)
    inits = [uniform_factors(dims, r, 700 + k) for k, r in enumerate([2, 5, 3, 7, 4, 1, 6])]
    for two_step in (False, True, None):      # None: the driver decides (suggest_two_step)
        out = P.cp_cals(T, inits, tol=1e-5, max_iters=60, max_total_rank=12, two_step=two_step)
        assert len(out) == len(inits)
        for k, (res, U, lam) in enumerate(out):
            ref = O.cp_als(T, inits[k], tol=1e-5, max_iters=60)
            assert res.model_id == k and res.iters == ref["iters"] and res.status == ref["status"]
            assert abs(res.fit - ref["fit"]) <= 1e-8
            for n in range(3):
                a = U[n] * (lam[None, :] if n == 2 else 1.0)
                b = ref["U"][n] * (ref["lam"][None, :] if n == 2 else 1.0)
                assert (np.linalg.norm(a - b, axis=0) / np.linalg.norm(b, axis=0)).max() <= 1e-6


def test_cp_cals_with_modes_reordered_by_length():
    # reorder_modes: the library gets the tensor with its modes sorted by decreasing length and sweeps them in that
    # order; the result is the oracle's CP-ALS on that transposed tensor, handed back in the caller's mode order
    import torch
    import paper_2010_04678_amd as P
    dims = (12, 40, 25)                                   # I1, I2, I3 -> order of decreasing length: modes 2, 3, 1
    T = _lowrank_tensor(dims, 3, 91, noise=0.05)          # numpy shape (I3, I2, I1)
    inits = [uniform_factors(dims, r, 900 + k) for k, r in enumerate([2, 4, 3, 5])]
    order = [1, 2, 0]
    Tp = np.ascontiguousarray(np.transpose(T, [2 - order[j] for j in (2, 1, 0)]))
    assert Tp.shape == (12, 25, 40)
    assert Tp[3, 7, 11] == T[7, 11, 3]                    # element (i2, i3, i1) of the new tensor = (i1, i2, i3) of the old
    for Tin in (T, torch.from_numpy(T).cuda()):
        out = P.cp_cals(Tin, inits, tol=1e-6, max_iters=40, reorder_modes=True)
        for k, (res, U, lam) in enumerate(out):
            ref = O.cp_als(Tp, [inits[k][order[j]] for j in range(3)], tol=1e-6, max_iters=40)
            assert res.iters == ref["iters"] and res.status == ref["status"] and abs(res.fit - ref["fit"]) <= 1e-8
            assert [u.shape[0] for u in U] == list(dims)
            assert np.abs(lam - ref["lam"]).max() <= 1e-6 * np.abs(ref["lam"]).max()
            for j in range(3):
                a, b = U[order[j]], ref["U"][j]
                assert (np.linalg.norm(a - b, axis=0) / np.linalg.norm(b, axis=0)).max() <= 1e-6
    # already sorted: nothing is copied, same result as without the option
    T2 = _lowrank_tensor((40, 25, 12), 3, 92, noise=0.05)
    in2 = [uniform_factors((40, 25, 12), 3, 950)]
    a = P.cp_cals(T2, in2, tol=-1.0, max_iters=5, reorder_modes=True)[0]
    b = P.cp_cals(T2, in2, tol=-1.0, max_iters=5)[0]
    assert a[0].fit == b[0].fit and all(np.array_equal(x, y) for x, y in zip(a[1], b[1]))


@pytest.mark.parametrize("seed", list(range(10)))
def test_seeded_random_queues_match_oracle(seed):
    # random small jobs: dims, ranks, tolerances, iteration caps, R*, slot limits and a mix of plain, non-negative and
    # line-search models; with and without two-step sweeps.  Same bars as everywhere (compare()).
    import paper_2010_04678_amd as P
    rng = np.random.default_rng(5000 + seed)
    dims = tuple(int(rng.choice([3, 8, 17, 24, 33, 40])) for _ in range(3))
    if seed % 5 == 4:
        dims = (int(rng.choice([260, 300, 513])), dims[1], min(dims[2], 8))      # a tall mode: row-blocked update
    T = _lowrank_tensor(dims, int(rng.integers(2, 6)), 6000 + seed, noise=0.05)
    if seed % 3 == 1:
        T = np.ascontiguousarray(np.abs(T))
    models = []
    for k in range(int(rng.integers(3, 12))):
        r = int(rng.choice([1, 2, 3, 4, 5, 7, 8, 9, 12, 16, 17, 20, 32], p=[.1, .1, .1, .1, .1, .1, .08, .08, .08, .06, .04, .04, .02]))
        kind = int(rng.choice([0, 1, 2], p=[.5, .25, .25]))
        models.append(dict(rank=r, init=uniform_factors(dims, r, 7000 + 100 * seed + k),
                           tol=float(rng.choice([-1.0, 1e-3, 1e-5])), max_iters=int(rng.integers(2, 26)),
                           flags=[0, O.FLAG_NONNEG, O.FLAG_LINESEARCH][kind], ls_alpha=float(rng.choice([1.1, 1.3, 2.0]))))
    rmax = max(m["rank"] for m in models)
    rstar = int(rng.integers(rmax, rmax + 40))
    slots = int(rng.choice([0, 2, 3, 5]))
    ref = O.cals(T, models, rstar, slots)
    for flags in (0, P.CTX_REUSE):
        results, facs, st = run_gpu(T, models, rstar, slots, rounds_per_call=int(rng.integers(1, 9)), ctx_flags=flags)
        compare(results, facs, ref, models)


@pytest.mark.parametrize("dims", [(100003, 30, 20), (20, 30, 100003), (7, 200001, 5)])
def test_very_long_modes(dims):
    # one mode of 1e5 rows and more: many row blocks in the contraction, the row-blocked update at its block cap,
    # long contraction ranges for the two short modes; MTTKRP element-wise and three iterations of a small queue
    from test_gpu_mttkrp import TOL, _abs_scale, _fused, _gpu_mttkrp
    T = _lowrank_tensor(dims, 3, 4100, noise=0.1)
    U = _fused(dims, [3, 8, 20, 1], 4200)
    got = _gpu_mttkrp(T, U, pad_to=37)
    for mode in (1, 2, 3):
        want = O.mttkrp(T, U, mode)
        err = np.abs(got[mode - 1] - want)
        assert np.all(err <= TOL * _abs_scale(T, U, mode) + 1e-300), mode
    models = [_model(dims, r, 4300 + r, max_iters=3, flags=f) for r, f in [(2, 0), (5, O.FLAG_LINESEARCH), (3, O.FLAG_NONNEG), (17, 0)]]
    ref = O.cals(T, models, 27, 0)
    results, facs, st = run_gpu(T, models, 27, 0, rounds_per_call=2)
    compare(results, facs, ref, models)
