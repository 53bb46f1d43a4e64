// Host-side planner: pipeline-schedule cost model (Tables I and II) and balanced partition
// explorer (Sec. III-C).  No device code, no global state.
#include <cmath>
#include <limits>
#include <vector>

#include "../../include/bapipe_plan.h"

namespace {

bool known_schedule(int s) { return s >= BAPIPE_PLAN_1F1B_AS && s <= BAPIPE_PLAN_1F1B_SO; }

// micro-batches whose features stage i (1-based) of N holds at once: "Features memory" row / a,
// never more than the M micro-batches that exist
int in_flight(int schedule, int M, int N, int i)
{
    int d = N - i + 1;
    if (schedule == BAPIPE_PLAN_FBP_AS || schedule == BAPIPE_PLAN_1F1B_SO) d *= 2;
    return d < M ? d : M;
}

// "Bandwidth" row: bytes per time unit that hide a transfer of `a` bytes behind the stage's compute
double bandwidth_row(int schedule, double a, double F, double B)
{
    return schedule == BAPIPE_PLAN_FBP_AS ? 2.0 * a / (F + B) : a / F;
}

int ceil_div(int a, int b) { return (a + b - 1) / b; }

struct Net {
    const bapipe_plan_input_t *in;
    int L, N;
    double f(int n, int l) const { return in->fwd_ms[(size_t)n * L + l]; }
    double b(int n, int l) const { return in->bwd_ms[(size_t)n * L + l]; }
    // F + B of layers [lo, hi) on accelerator n, summed in layer order
    double span_ms(int n, int lo, int hi) const
    {
        double t = 0.0;
        for (int l = lo; l < hi; ++l) t += f(n, l) + b(n, l);
        return t;
    }
    double span_fwd(int n, int lo, int hi) const
    {
        double t = 0.0;
        for (int l = lo; l < hi; ++l) t += f(n, l);
        return t;
    }
    double span_bwd(int n, int lo, int hi) const
    {
        double t = 0.0;
        for (int l = lo; l < hi; ++l) t += b(n, l);
        return t;
    }
    bool fits(int n, int lo, int hi) const
    {
        const double cap = in->mem_capacity ? in->mem_capacity[n] : 0.0;
        if (!(cap > 0.0)) return true;
        double w = 0.0, s = 0.0;
        for (int l = lo; l < hi; ++l) {
            w += in->weight_bytes[l];
            s += in->stash_bytes[l];
        }
        return 2.0 * w + in_flight(in->schedule, in->n_micro, N, n + 1) * s <= cap;
    }
    double bottleneck(const std::vector<int> &sb) const
    {
        double m = 0.0;
        for (int n = 0; n < N; ++n) m = std::fmax(m, span_ms(n, sb[n], sb[n + 1]));
        return m;
    }
};

// Eq. (1): with T_n the time of the whole network on accelerator n, equal stage times are
// T = 1 / sum_n (1 / T_n)
double ideal_stage_ms(const Net &net)
{
    double inv = 0.0;
    for (int n = 0; n < net.N; ++n) inv += 1.0 / net.span_ms(n, 0, net.L);
    return 1.0 / inv;
}

// Seed: each stage takes layers until its running time is as close to T as it gets (leaving one
// layer for every later stage); then single boundaries move by one layer while that makes the
// slowest stage strictly faster.
std::vector<int> seeded_partition(const Net &net, double T)
{
    const int L = net.L, N = net.N;
    std::vector<int> sb(N + 1, 0);
    sb[N] = L;
    for (int n = 0; n + 1 < N; ++n) {
        const int lo = sb[n], max_hi = L - (N - 1 - n);
        int best_hi = lo + 1;
        double best_gap = std::numeric_limits<double>::infinity(), t = 0.0;
        for (int hi = lo + 1; hi <= max_hi; ++hi) {
            t += net.f(n, hi - 1) + net.b(n, hi - 1);
            const double gap = std::fabs(t - T);
            if (gap < best_gap) {
                best_gap = gap;
                best_hi = hi;
            }
        }
        sb[n + 1] = best_hi;
    }
    bool moved = true;
    while (moved) {
        moved = false;
        double cur = net.bottleneck(sb);
        for (int k = 1; k < N; ++k) {
            for (int d = -1; d <= 1; d += 2) {
                const int nb = sb[k] + d;
                if (nb <= sb[k - 1] || nb >= sb[k + 1]) continue;
                const int old = sb[k];
                sb[k] = nb;
                const double t = net.bottleneck(sb);
                if (t < cur) {
                    cur = t;
                    moved = true;
                } else {
                    sb[k] = old;
                }
            }
        }
    }
    return sb;
}

// Contiguous partition with the smallest slowest stage among those whose boundaries are allowed
// (boundary_ok[l]: a stage may end after layer l) and, if use_memory, whose stages fit their
// accelerator.  best[n][e] = min over b of max(best[n-1][b], time of stage n on [b, e)); the first
// b that reaches the minimum is kept.  Returns false if no such partition exists.
bool exact_partition(const Net &net, const std::vector<char> &boundary_ok, bool use_memory, std::vector<int> &sb)
{
    const int L = net.L, N = net.N;
    const double INF = std::numeric_limits<double>::infinity();
    std::vector<std::vector<double>> best(N, std::vector<double>(L + 1, INF));
    std::vector<std::vector<int>> from(N, std::vector<int>(L + 1, -1));
    for (int n = 0; n < N; ++n) {
        const int b_lo = n == 0 ? 0 : n, b_hi = n == 0 ? 0 : L - (N - n);       // first layer of stage n
        for (int b = b_lo; b <= b_hi; ++b) {
            if (n > 0 && (!boundary_ok[b - 1] || best[n - 1][b] == INF)) continue;
            const double before = n == 0 ? 0.0 : best[n - 1][b];
            double t = 0.0;
            const int e_hi = L - (N - 1 - n);
            for (int e = b + 1; e <= e_hi; ++e) {
                t += net.f(n, e - 1) + net.b(n, e - 1);
                if (n == N - 1 && e != L) continue;
                if (use_memory && !net.fits(n, b, e)) continue;
                const double v = std::fmax(before, t);
                if (v < best[n][e]) {
                    best[n][e] = v;
                    from[n][e] = b;
                }
            }
        }
    }
    if (best[N - 1][L] == INF) return false;
    sb.assign(N + 1, 0);
    sb[N] = L;
    for (int n = N - 1; n > 0; --n) sb[n] = from[n][sb[n + 1]];
    return true;
}

bool needs_more_bandwidth(const Net &net, const std::vector<int> &sb)
{
    const double bw = net.in->link_bytes_per_ms;
    if (!(bw > 0.0)) return false;
    for (int n = 0; n + 1 < net.N; ++n) {
        const double a = net.in->out_bytes[sb[n + 1] - 1];
        // the sender overlaps the transfer with its own compute, the receiver with its own
        for (int side = 0; side < 2; ++side) {
            const int m = n + side;
            const double F = net.span_fwd(m, sb[m], sb[m + 1]), B = net.span_bwd(m, sb[m], sb[m + 1]);
            if (bandwidth_row(net.in->schedule, a, F, B) > bw) return true;
        }
    }
    return false;
}

bool all_fit(const Net &net, const std::vector<int> &sb)
{
    for (int n = 0; n < net.N; ++n)
        if (!net.fits(n, sb[n], sb[n + 1])) return false;
    return true;
}

}  // namespace

extern "C" int bapipe_schedule_cost(int schedule, int M, int N, int i, double F, double B, double SR, double a,
                                    double w, bapipe_schedule_cost_t *out)
{
    if (!out || !known_schedule(schedule) || M < 1 || N < 1 || i < 1 || i > N || !(F > 0.0) || !(B > 0.0) ||
        !(SR >= 0.0) || !(a >= 0.0) || !(w >= 0.0))
        return BAPIPE_E_INVALID;
    bapipe_schedule_cost_t c;
    const double steady = (double)(M + N - 1) * (F + B);
    switch (schedule) {
    case BAPIPE_PLAN_1F1B_AS:
    case BAPIPE_PLAN_FBP_AS:
        // Table I: transfers are hidden completely
        c.minibatch_time = steady;
        c.bubble_fraction = (double)(N - 1) / (double)(M + N - 1);
        break;
    case BAPIPE_PLAN_1F1B_SNO: {
        // Table II: N + M - 2 - ceil((M-1)/N) round trips of 2 SR stay exposed
        const int exposed = N + M - 2 - ceil_div(M - 1, N);
        c.minibatch_time = steady + (double)exposed * 2.0 * SR;
        c.bubble_fraction = ((double)(N - 1) * (F + B + 2.0 * SR) + (double)(M - 1 - ceil_div(M - 1, N)) * 2.0 * SR) /
                            c.minibatch_time;
        break;
    }
    default:
        // 1F1B-SO: only the N-1 fill / drain round trips stay exposed
        c.minibatch_time = steady + (double)(N - 1) * 2.0 * SR;
        c.bubble_fraction = (double)(N - 1) * (F + B + 2.0 * SR) / c.minibatch_time;
        break;
    }
    const bool doubled = schedule == BAPIPE_PLAN_FBP_AS || schedule == BAPIPE_PLAN_1F1B_SO;
    c.features_memory = (doubled ? 2.0 : 1.0) * (double)(N - i + 1) * a;
    c.weights_memory = 2.0 * w;
    c.bandwidth_demand = bandwidth_row(schedule, a, F, B);
    c.in_flight = in_flight(schedule, M, N, i);
    *out = c;
    return BAPIPE_OK;
}

extern "C" int bapipe_schedule_choose(const bapipe_schedule_candidate_t *cand, int n_cand, int N, const double *w,
                                      const double *capacity, int *best, bapipe_schedule_cost_t *cost)
{
    if (!cand || n_cand < 1 || N < 1 || !w || !best) return BAPIPE_E_INVALID;
    int pick = -1;
    bapipe_schedule_cost_t pick_cost{};
    for (int c = 0; c < n_cand; ++c) {
        const bapipe_schedule_candidate_t &k = cand[c];
        if (!k.a) return BAPIPE_E_INVALID;
        bool fits = true;
        bapipe_schedule_cost_t first{};
        for (int i = 1; i <= N; ++i) {
            bapipe_schedule_cost_t sc;
            const int st = bapipe_schedule_cost(k.schedule, k.n_micro, N, i, k.F, k.B, k.SR, k.a[i - 1], w[i - 1], &sc);
            if (st != BAPIPE_OK) return st;
            if (i == 1) first = sc;
            const double cap = capacity ? capacity[i - 1] : 0.0;
            // memory actually held: the in-flight count never exceeds the M micro-batches that exist
            if (cap > 0.0 && (double)sc.in_flight * k.a[i - 1] + sc.weights_memory > cap) fits = false;
        }
        if (fits && (pick < 0 || first.minibatch_time < pick_cost.minibatch_time)) {
            pick = c;
            pick_cost = first;
        }
    }
    if (pick < 0) return BAPIPE_E_UNSUPPORTED;
    *best = pick;
    if (cost) *cost = pick_cost;
    return BAPIPE_OK;
}

extern "C" int bapipe_partition(const bapipe_plan_input_t *in, int *stage_begin, bapipe_plan_report_t *report)
{
    if (!in || !stage_begin || !report || in->n_layers < 1 || in->n_acc < 1 || in->n_acc > in->n_layers ||
        !in->fwd_ms || !in->bwd_ms || !in->out_bytes || !in->weight_bytes || !in->stash_bytes || in->n_micro < 1 ||
        !known_schedule(in->schedule))
        return BAPIPE_E_INVALID;
    Net net{in, in->n_layers, in->n_acc};
    for (int n = 0; n < net.N; ++n) {
        double whole = 0.0;
        for (int l = 0; l < net.L; ++l) {
            if (!(net.f(n, l) >= 0.0) || !(net.b(n, l) >= 0.0)) return BAPIPE_E_INVALID;
            whole += net.f(n, l) + net.b(n, l);
        }
        if (!(whole > 0.0)) return BAPIPE_E_INVALID;
    }
    for (int l = 0; l < net.L; ++l)
        if (!(in->out_bytes[l] >= 0.0) || !(in->weight_bytes[l] >= 0.0) || !(in->stash_bytes[l] >= 0.0)) return BAPIPE_E_INVALID;

    bapipe_plan_report_t rep{};
    rep.ideal_stage_ms = ideal_stage_ms(net);

    // 1. inter-layer partition, communication and memory ignored
    std::vector<int> sb = seeded_partition(net, rep.ideal_stage_ms);
    rep.seed_bottleneck_ms = net.bottleneck(sb);
    std::vector<char> boundary_ok(net.L, 1);
    std::vector<int> ex;
    if (exact_partition(net, boundary_ok, false, ex) && net.bottleneck(ex) < rep.seed_bottleneck_ms) sb = ex;

    // 2. / 3. communication test and memory fine-tune; tuning for memory may create a communication
    // bottleneck, so the test is repeated once the partition has moved
    bool restricted = false, use_memory = false;
    for (int round = 0; round < 3; ++round) {
        bool changed = false;
        if (!restricted && needs_more_bandwidth(net, sb)) {
            rep.comm_bottleneck = 1;
            rep.a_th_bytes = rep.ideal_stage_ms * in->link_bytes_per_ms;
            for (int l = 0; l < net.L; ++l) boundary_ok[l] = in->out_bytes[l] <= rep.a_th_bytes;
            restricted = changed = true;
        }
        if (!use_memory && !all_fit(net, sb)) {
            rep.memory_tuned = 1;
            use_memory = changed = true;
        }
        if (!changed) break;
        if (!exact_partition(net, boundary_ok, use_memory, sb)) {
            *report = rep;
            return BAPIPE_E_UNSUPPORTED;
        }
    }
    rep.bottleneck_ms = net.bottleneck(sb);
    for (int n = 0; n <= net.N; ++n) stage_begin[n] = sb[n];
    *report = rep;
    return BAPIPE_OK;
}
