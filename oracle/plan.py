"""CPU oracle of the host-side planner (test infrastructure only: nothing in the product imports it).

Schedule cost model: the four columns of Tables I and II written out as printed.
Balanced partition (Sec. III-C): the definition - among all ways of cutting L layers into N contiguous
non-empty stages (brute force over every combination of N-1 cut points), the smallest possible time of
the slowest stage, optionally restricted to cuts after layers whose output is at most a_th
(coarse-grained network) and to stages that fit their accelerator's memory."""
import itertools
import math

S_1F1B_AS, S_FBP_AS, S_1F1B_SNO, S_1F1B_SO = range(4)


def schedule_cost(schedule, M, N, i, F, B, SR, a, w):
    """Tables I / II; stage index i is 1-based."""
    steady = (M + N - 1) * (F + B)
    if schedule in (S_1F1B_AS, S_FBP_AS):
        time = steady
        bubble = (N - 1) / (M + N - 1)
    elif schedule == S_1F1B_SNO:
        c = math.ceil((M - 1) / N)
        time = steady + (N + M - 2 - c) * 2 * SR
        bubble = ((N - 1) * (F + B + 2 * SR) + (M - 1 - c) * 2 * SR) / time
    else:
        time = steady + (N - 1) * 2 * SR
        bubble = (N - 1) * (F + B + 2 * SR) / time
    doubled = schedule in (S_FBP_AS, S_1F1B_SO)
    features = (2 if doubled else 1) * (N - i + 1) * a
    bandwidth = 2 * a / (F + B) if schedule == S_FBP_AS else a / F
    return dict(minibatch_time=time, bubble_fraction=bubble, features_memory=features, weights_memory=2 * w,
                bandwidth_demand=bandwidth, in_flight=min(M, (2 if doubled else 1) * (N - i + 1)))


def ideal_stage_ms(fwd, bwd):
    """Eq. (1): T = 1 / sum_n 1/T_n with T_n the whole network's F+B time on accelerator n."""
    return 1.0 / sum(1.0 / sum(f + b for f, b in zip(fr, br)) for fr, br in zip(fwd, bwd))


def stage_ms(fwd, bwd, n, lo, hi):
    return sum(fwd[n][l] + bwd[n][l] for l in range(lo, hi))


def stage_fits(p, n, lo, hi):
    cap = p["mem_capacity"][n] if p.get("mem_capacity") else 0.0
    if not cap > 0.0:
        return True
    N = len(p["fwd_ms"])
    depth = schedule_cost(p["schedule"], p["n_micro"], N, n + 1, 1.0, 1.0, 0.0, 1.0, 0.0)["in_flight"]
    return 2.0 * sum(p["weight_bytes"][lo:hi]) + depth * sum(p["stash_bytes"][lo:hi]) <= cap


def needs_more_bandwidth(p, sb):
    """Some boundary's transfer cannot hide behind the compute of the stage sending or receiving it."""
    bw = p.get("link_bytes_per_ms", 0.0)
    if not bw > 0.0:
        return False
    N = len(p["fwd_ms"])
    for n in range(N - 1):
        a = p["out_bytes"][sb[n + 1] - 1]
        for m in (n, n + 1):
            F = sum(p["fwd_ms"][m][sb[m]:sb[m + 1]])
            B = sum(p["bwd_ms"][m][sb[m]:sb[m + 1]])
            if schedule_cost(p["schedule"], 1, 1, 1, F, B, 0.0, a, 0.0)["bandwidth_demand"] > bw:
                return True
    return False


def all_partitions(L, N):
    for cuts in itertools.combinations(range(1, L), N - 1):
        yield (0,) + cuts + (L,)


def best_bottleneck(p, a_th=None, use_memory=False):
    """Smallest slowest-stage time over every admissible partition (None if there is none)."""
    fwd, bwd = p["fwd_ms"], p["bwd_ms"]
    N, L = len(fwd), len(fwd[0])
    best = None
    for sb in all_partitions(L, N):
        if a_th is not None and any(p["out_bytes"][sb[n + 1] - 1] > a_th for n in range(N - 1)):
            continue
        if use_memory and not all(stage_fits(p, n, sb[n], sb[n + 1]) for n in range(N)):
            continue
        t = max(stage_ms(fwd, bwd, n, sb[n], sb[n + 1]) for n in range(N))
        if best is None or t < best:
            best = t
    return best


def choose_schedule(candidates, w, capacity=None):
    """Index of the memory-feasible candidate with the smallest mini-batch time (first wins ties), or None."""
    N = len(w)
    best = None
    for c, k in enumerate(candidates):
        costs = [schedule_cost(k["schedule"], k["n_micro"], N, i, k["F"], k["B"], k["SR"], k["a"][i - 1], w[i - 1])
                 for i in range(1, N + 1)]
        fits = all(not (capacity and capacity[i] > 0) or costs[i]["in_flight"] * k["a"][i] + 2 * w[i] <= capacity[i]
                   for i in range(N))
        if fits and (best is None or costs[0]["minibatch_time"] < best[1]):
            best = (c, costs[0]["minibatch_time"])
    return None if best is None else best[0]
