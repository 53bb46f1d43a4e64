"""Host-side planner (C ABI, include/bapipe_plan.h) against the CPU oracle and against what the paper fixes:
the printed table formulas on worked numbers, Eq. (1) in closed form, brute force over every contiguous
partition of short layer lists.  No GPU is touched."""
import math
import random

import pytest

from oracle import plan as O
from paper_2012_12544_amd import binding as B


# ------------------------------------------------------------------ oracle pins (paper / mathematics)
def test_oracle_tables_on_worked_numbers():
    # Table I with M = 8, N = 3 (the figure's case), F = 1, B = 2: 10 slots of 3, bubble 2/10
    c = O.schedule_cost(O.S_1F1B_AS, 8, 3, 1, 1.0, 2.0, 0.5, 10.0, 7.0)
    assert c["minibatch_time"] == 30.0 and c["bubble_fraction"] == 0.2
    assert c["features_memory"] == 30.0 and c["weights_memory"] == 14.0 and c["bandwidth_demand"] == 10.0
    f = O.schedule_cost(O.S_FBP_AS, 8, 3, 1, 1.0, 2.0, 0.5, 10.0, 7.0)
    assert f["features_memory"] == 60.0 and f["bandwidth_demand"] == 20.0 / 3.0 and f["minibatch_time"] == 30.0
    # Table II, same case, SR = 0.5: SNO exposes N + M - 2 - ceil(7/3) = 6 round trips, SO only N - 1 = 2
    sno = O.schedule_cost(O.S_1F1B_SNO, 8, 3, 2, 1.0, 2.0, 0.5, 10.0, 7.0)
    so = O.schedule_cost(O.S_1F1B_SO, 8, 3, 2, 1.0, 2.0, 0.5, 10.0, 7.0)
    assert sno["minibatch_time"] == 36.0 and so["minibatch_time"] == 32.0
    assert sno["bubble_fraction"] == (2 * 4.0 + 4 * 1.0) / 36.0 and so["bubble_fraction"] == 8.0 / 32.0
    assert sno["features_memory"] == 20.0 and so["features_memory"] == 40.0
    assert sno["in_flight"] == 2 and so["in_flight"] == 4


def test_oracle_table_invariants():
    rng = random.Random(5)
    for _ in range(200):
        M, N = rng.randint(1, 40), rng.randint(1, 9)
        F, Bt, SR = rng.uniform(0.1, 5), rng.uniform(0.1, 9), rng.uniform(0, 3)
        i = rng.randint(1, N)
        sno = O.schedule_cost(O.S_1F1B_SNO, M, N, i, F, Bt, SR, 3.0, 2.0)
        so = O.schedule_cost(O.S_1F1B_SO, M, N, i, F, Bt, SR, 3.0, 2.0)
        asy = O.schedule_cost(O.S_1F1B_AS, M, N, i, F, Bt, SR, 3.0, 2.0)
        # useful work is M (F + B): time = work / (1 - bubble) for every schedule
        for c in (sno, so, asy):
            assert math.isclose(c["minibatch_time"] * (1 - c["bubble_fraction"]), M * (F + Bt), rel_tol=1e-12)
        # overlap never loses, and without transfers the synchronous schedules are the asynchronous one
        assert so["minibatch_time"] <= sno["minibatch_time"] + 1e-12
        z = O.schedule_cost(O.S_1F1B_SNO, M, N, i, F, Bt, 0.0, 3.0, 2.0)
        assert z["minibatch_time"] == asy["minibatch_time"] and math.isclose(z["bubble_fraction"], asy["bubble_fraction"])
        assert so["features_memory"] == 2 * sno["features_memory"]
    # one accelerator: no bubble, no exposed transfer
    one = O.schedule_cost(O.S_1F1B_SO, 5, 1, 1, 1.0, 1.0, 9.0, 1.0, 1.0)
    assert one["bubble_fraction"] == 0.0 and one["minibatch_time"] == 10.0


def test_oracle_ideal_time_closed_forms():
    # identical accelerators: T = T_1 / N; one twice as fast as the other: harmonic combination
    f = [[1.0, 2.0, 3.0]] * 4
    assert math.isclose(O.ideal_stage_ms(f, f), 12.0 / 4)
    assert math.isclose(O.ideal_stage_ms([[3.0], [6.0]], [[0.0], [0.0]]), 2.0)


def test_oracle_brute_force_on_a_hand_case():
    p = dict(fwd_ms=[[1, 1, 1, 5, 1, 1]] * 3, bwd_ms=[[0] * 6] * 3, out_bytes=[1] * 6, weight_bytes=[0] * 6,
             stash_bytes=[0] * 6, n_micro=4, schedule=O.S_1F1B_SO)
    assert O.best_bottleneck(p) == 5           # [1 1 1 | 5 | 1 1]
    assert len(list(O.all_partitions(6, 3))) == math.comb(5, 2)
    # the cut after layer 3 forbidden (large output): the 5 must share a stage
    p["out_bytes"] = [1, 1, 1, 9, 1, 1]
    assert O.best_bottleneck(p, a_th=2) == 6   # [1 1 | 1 5 | 1 1] or [1 1 1 | 5 1 | 1]


# ------------------------------------------------------------------ C ABI against the oracle
SCHEDULES = [B.PLAN_1F1B_AS, B.PLAN_FBP_AS, B.PLAN_1F1B_SNO, B.PLAN_1F1B_SO]


def test_schedule_cost_matches_the_tables():
    rng = random.Random(11)
    for _ in range(300):
        s = rng.choice(SCHEDULES)
        M, N = rng.randint(1, 64), rng.randint(1, 8)
        i = rng.randint(1, N)
        F, Bt, SR, a, w = rng.uniform(0.01, 5), rng.uniform(0.01, 9), rng.uniform(0, 3), rng.uniform(0, 1e9), rng.uniform(0, 1e9)
        got, ref = B.bapipe_schedule_cost(s, M, N, i, F, Bt, SR, a, w), O.schedule_cost(s, M, N, i, F, Bt, SR, a, w)
        for k, v in ref.items():
            assert got[k] == v if isinstance(v, int) else math.isclose(got[k], v, rel_tol=1e-14, abs_tol=0.0), (k, got, ref)


def test_schedule_cost_rejects_bad_arguments():
    for args in [(9, 1, 1, 1, 1, 1, 0, 0, 0), (0, 0, 1, 1, 1, 1, 0, 0, 0), (0, 1, 2, 3, 1, 1, 0, 0, 0),
                 (0, 1, 1, 1, 0.0, 1, 0, 0, 0), (0, 1, 1, 1, 1, 1, -1.0, 0, 0)]:
        with pytest.raises(B.BapipeError) as e:
            B.bapipe_schedule_cost(*args)
        assert e.value.status == B.E_INVALID


def test_schedule_choice():
    # the paper's trade-off: overlap (SO) wins when its doubled features fit, otherwise it needs half-size
    # micro-batches (twice as many, each a bit less efficient) and may lose to the naive schedule
    w, a_full, a_half = [1e9, 1e9], [4e9, 4e9], [2e9, 2e9]
    cands = [dict(schedule=B.PLAN_1F1B_SNO, n_micro=8, F=1.0, B=2.0, SR=0.5, a=a_full),
             dict(schedule=B.PLAN_1F1B_SO, n_micro=8, F=1.0, B=2.0, SR=0.5, a=a_full),
             dict(schedule=B.PLAN_1F1B_SO, n_micro=16, F=0.6, B=1.2, SR=0.25, a=a_half)]
    assert B.bapipe_schedule_choose(cands, w)[0] == 1                                  # unlimited memory
    assert B.bapipe_schedule_choose(cands, w, [2e9 + 2 * 4e9] * 2)[0] == 0              # SO at full size needs 4 x 4e9 on stage 1
    slow_half = [cands[0], cands[1], dict(cands[2], F=0.9, B=1.8)]
    assert B.bapipe_schedule_choose(slow_half, w, [2e9 + 2 * 4e9] * 2)[0] == 0
    fast_half = [cands[0], cands[1], dict(cands[2], F=0.5, B=1.0)]
    assert B.bapipe_schedule_choose(fast_half, w, [2e9 + 2 * 4e9] * 2)[0] == 2
    with pytest.raises(B.BapipeError) as e:
        B.bapipe_schedule_choose(cands, w, [1e9] * 2)
    assert e.value.status == B.E_UNSUPPORTED
    rng = random.Random(23)
    for _ in range(200):
        N = rng.randint(1, 5)
        ww = [rng.uniform(0, 2e9) for _ in range(N)]
        cs = [dict(schedule=rng.choice(SCHEDULES), n_micro=rng.randint(1, 32), F=rng.uniform(0.1, 3), B=rng.uniform(0.1, 6),
                   SR=rng.uniform(0, 1), a=[rng.uniform(0, 4e9) for _ in range(N)]) for _ in range(rng.randint(1, 5))]
        cap = [rng.choice([0.0, 4e9, 1.6e10, 6e10]) for _ in range(N)]
        ref = O.choose_schedule(cs, ww, cap)
        if ref is None:
            with pytest.raises(B.BapipeError):
                B.bapipe_schedule_choose(cs, ww, cap)
        else:
            assert B.bapipe_schedule_choose(cs, ww, cap)[0] == ref


def random_profile(rng, L, N, hetero):
    speed = [rng.uniform(0.5, 2.0) if hetero else 1.0 for _ in range(N)]
    base_f = [rng.choice([0.05, 0.2, 1.0, 3.0]) * rng.uniform(0.5, 1.5) for _ in range(L)]
    base_b = [2 * f * rng.uniform(0.8, 1.2) for f in base_f]
    return dict(fwd_ms=[[f * s for f in base_f] for s in speed], bwd_ms=[[b * s for b in base_b] for s in speed],
                out_bytes=[rng.choice([1e5, 1e6, 8e6]) for _ in range(L)],
                weight_bytes=[rng.choice([0.0, 1e5, 4e6]) for _ in range(L)],
                stash_bytes=[rng.choice([0.0, 1e6, 6e6]) for _ in range(L)])


def valid_partition(sb, L, N):
    return len(sb) == N + 1 and sb[0] == 0 and sb[-1] == L and all(sb[n] < sb[n + 1] for n in range(N))


@pytest.mark.parametrize("hetero", [False, True])
def test_unconstrained_partition_is_the_brute_force_optimum(hetero):
    rng = random.Random(3 + hetero)
    for _ in range(120):
        L = rng.randint(1, 12)
        N = rng.randint(1, min(L, 5))
        p = random_profile(rng, L, N, hetero)
        sb, rep = B.bapipe_partition(p["fwd_ms"], p["bwd_ms"], p["out_bytes"], p["weight_bytes"], p["stash_bytes"],
                                     n_micro=8, schedule=B.PLAN_1F1B_SO)
        assert valid_partition(sb, L, N)
        ref = O.best_bottleneck(dict(p, n_micro=8, schedule=O.S_1F1B_SO))
        mine = max(O.stage_ms(p["fwd_ms"], p["bwd_ms"], n, sb[n], sb[n + 1]) for n in range(N))
        assert mine == ref == rep["bottleneck_ms"]                 # same sums in the same order: exact
        assert rep["seed_bottleneck_ms"] >= ref
        assert math.isclose(rep["ideal_stage_ms"], O.ideal_stage_ms(p["fwd_ms"], p["bwd_ms"]), rel_tol=1e-14)
        assert ref >= rep["ideal_stage_ms"] * (1 - 1e-12) or hetero   # identical accelerators: T is a lower bound
        assert rep["comm_bottleneck"] == 0 and rep["memory_tuned"] == 0 and rep["a_th_bytes"] == 0.0


def test_identical_layers_split_evenly():
    sb, rep = B.bapipe_partition([[1.0] * 12] * 4, [[2.0] * 12] * 4, [1.0] * 12, [0.0] * 12, [0.0] * 12)
    assert sb == [0, 3, 6, 9, 12] and rep["bottleneck_ms"] == 9.0 == rep["ideal_stage_ms"] == rep["seed_bottleneck_ms"]
    # a twice faster second accelerator takes twice the layers (Eq. (1): T = 1/(1/36 + 1/18) = 12)
    sb, rep = B.bapipe_partition([[1.0] * 12, [0.5] * 12], [[2.0] * 12, [1.0] * 12], [1.0] * 12, [0.0] * 12, [0.0] * 12)
    assert sb == [0, 4, 12] and rep["bottleneck_ms"] == 12.0 == rep["ideal_stage_ms"]


@pytest.mark.parametrize("schedule", SCHEDULES)
def test_constrained_partition_flow(schedule):
    """Flags reported by the library decide which constraint set the result is optimal for; the result
    itself must satisfy what the flow promises."""
    rng = random.Random(17 + schedule)
    seen = {"comm": 0, "mem": 0, "both": 0, "none": 0, "infeasible": 0}
    for _ in range(300):
        L = rng.randint(2, 11)
        N = rng.randint(2, min(L, 4))
        p = random_profile(rng, L, N, hetero=rng.random() < 0.5)
        p.update(n_micro=rng.randint(1, 8), schedule=schedule, link_bytes_per_ms=rng.choice([0.0, 2e5, 2e6, 2e7]),
                 mem_capacity=[rng.choice([0.0, 2e7, 6e7, 2e8]) for _ in range(N)])
        try:
            sb, rep = B.bapipe_partition(p["fwd_ms"], p["bwd_ms"], p["out_bytes"], p["weight_bytes"], p["stash_bytes"],
                                         p["mem_capacity"], p["link_bytes_per_ms"], p["n_micro"], schedule)
        except B.BapipeError as e:
            assert e.status == B.E_UNSUPPORTED
            rep = e.report
            a_th = rep["a_th_bytes"] if rep["comm_bottleneck"] else None
            assert O.best_bottleneck(p, a_th=a_th, use_memory=bool(rep["memory_tuned"])) is None
            seen["infeasible"] += 1
            continue
        assert valid_partition(sb, L, N)
        T = O.ideal_stage_ms(p["fwd_ms"], p["bwd_ms"])
        if rep["comm_bottleneck"]:
            assert math.isclose(rep["a_th_bytes"], T * p["link_bytes_per_ms"], rel_tol=1e-14)
            assert all(p["out_bytes"][sb[n + 1] - 1] <= rep["a_th_bytes"] for n in range(N - 1))
        else:
            assert rep["a_th_bytes"] == 0.0 and not O.needs_more_bandwidth(p, sb)
        assert all(O.stage_fits(p, n, sb[n], sb[n + 1]) for n in range(N))
        ref = O.best_bottleneck(p, a_th=rep["a_th_bytes"] if rep["comm_bottleneck"] else None,
                                use_memory=bool(rep["memory_tuned"]))
        mine = max(O.stage_ms(p["fwd_ms"], p["bwd_ms"], n, sb[n], sb[n + 1]) for n in range(N))
        assert mine == ref == rep["bottleneck_ms"]
        assert ref >= O.best_bottleneck(p)                         # constraints never help
        seen[("both" if rep["memory_tuned"] else "comm") if rep["comm_bottleneck"] else ("mem" if rep["memory_tuned"] else "none")] += 1
    assert seen["none"] and seen["comm"] and seen["mem"], seen     # the sweep exercises every branch


def test_partition_rejects_bad_arguments():
    ok = dict(fwd_ms=[[1.0, 1.0]], bwd_ms=[[1.0, 1.0]], out_bytes=[1.0, 1.0], weight_bytes=[0.0, 0.0], stash_bytes=[0.0, 0.0])
    with pytest.raises(B.BapipeError) as e:                          # more accelerators than layers
        B.bapipe_partition([[1.0]] * 2, [[1.0]] * 2, [1.0], [0.0], [0.0])
    assert e.value.status == B.E_INVALID
    with pytest.raises(B.BapipeError) as e:
        B.bapipe_partition([[-1.0, 1.0]], ok["bwd_ms"], ok["out_bytes"], ok["weight_bytes"], ok["stash_bytes"])
    assert e.value.status == B.E_INVALID
    with pytest.raises(B.BapipeError) as e:
        B.bapipe_partition(ok["fwd_ms"], ok["bwd_ms"], ok["out_bytes"], ok["weight_bytes"], ok["stash_bytes"], n_micro=0)
    assert e.value.status == B.E_INVALID
    assert B.load().bapipe_partition(None, None, None) == B.E_INVALID
