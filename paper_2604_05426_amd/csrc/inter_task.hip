// Dynamic inter-task scheduling (paper Sec. 6.2): n tasks with profiled durations d_i and GPU requirements g_i on G GPUs,
// every task holds its GPUs for its whole duration, minimise the makespan (P | size_j | C_max), re-plan on every task
// arrival and completion.  Host code only.
//
// The paper hands its constraint program (start times, GPU assignment x_ig, pair orders y_ij, big-M disjunctions per
// shared GPU) to a general solver.  Here the structure is used directly:
//   * GPUs are interchangeable, so all that matters of a partial schedule is when each GPU falls idle; concrete GPUs
//     are handed out afterwards in order of start time;
//   * a schedule in which no task can start earlier with the others left alone is reproduced by starting its tasks in
//     the order of their start times, each as early as possible but not before the one before it, and some such schedule
//     is optimal.  The solver walks these lists depth first; a node is the set of started tasks plus the sorted idle
//     times of the GPUs, clipped to the last start (the front no later task goes behind).  A branch is cut when a lower
//     bound (ends so far, earliest possible end of a waiting task, work left against the capacity between the idle times
//     and the incumbent's makespan) shows that nothing below it can be strictly better than the incumbent, or when the
//     same node has been expanded before (different lists lead to the same idle times).
// Cutting only on "cannot be strictly better" leaves the answer what full enumeration of the lists would give: the first
// one, in the candidate order (g descending, d descending, index ascending; tasks with equal d and g in index order,
// tasks that come out with equal starts in candidate order), that reaches the optimum.
#include <algorithm>
#include <cmath>
#include <cstring>
#include <string>
#include <unordered_set>
#include <vector>

#include "common.h"

using mlora::set_error;

namespace {

constexpr double kEps = 1e-9;            // two times closer than this are the same time
constexpr size_t kMaxSeenBytes = (size_t)128 << 20;   // memory bound of the table of expanded nodes (the search stays exact without it)
constexpr int64_t kMaxNodes = 4000000;      // search budget (about a second); beyond it the best schedule found so far is returned

struct Solver {
    int n = 0, G = 0;
    double now = 0.0;
    std::vector<double> d;            // by candidate position
    std::vector<int> g, idx;          // GPUs needed, caller's index
    std::vector<char> used;
    std::vector<double> cur, best;    // starts by candidate position
    double best_mk = INFINITY;
    double root_lb = 0.0;
    bool done = false;
    bool out_of_budget = false;
    int64_t nodes = 0;
    std::unordered_set<std::string> seen;

    // idle: sorted idle times of the G GPUs, all >= front
    void dfs(int depth, double mk, double front, int last, const double* idle, uint32_t mask) {
        if (done) return;
        if (++nodes > kMaxNodes && best_mk < INFINITY) { done = out_of_budget = true; return; }
        if (depth == n) {
            if (mk < best_mk - kEps) {
                best_mk = mk;
                best = cur;
                if (best_mk <= root_lb + kEps) done = true;   // nothing can be strictly better than the root bound
            }
            return;
        }
        if (mk >= best_mk - kEps) return;
        if (best_mk < INFINITY) {
            double work = 0.0;
            for (int p = 0; p < n; ++p) {
                if (used[p]) continue;
                if (idle[g[p] - 1] + d[p] >= best_mk - kEps) return;
                work += d[p] * g[p];
            }
            double room = 0.0;
            for (int q = 0; q < G; ++q) room += std::max(0.0, best_mk - kEps - idle[q]);
            if (work > room + kEps) return;
        }
        // the same started set with the same idle times, ends so far and last position has been expanded before: every
        // list below it has been seen with the same makespan (what was cut then was cut against a makespan no smaller
        // than today's incumbent)
        if (depth > 0 && depth < n - 1) {
            std::string key(sizeof(uint32_t) + sizeof(int) + sizeof(double) * (size_t)(G + 1), '\0');
            char* w = &key[0];
            std::memcpy(w, &mask, sizeof mask); w += sizeof mask;
            // the last position matters only while a waiting task could still start at the front itself
            int tie = -1;
            for (int p = 0; p < last; ++p)
                if (!used[p] && idle[g[p] - 1] <= front + kEps) { tie = last; break; }
            std::memcpy(w, &tie, sizeof tie); w += sizeof tie;
            std::memcpy(w, &mk, sizeof mk); w += sizeof mk;
            std::memcpy(w, idle, sizeof(double) * (size_t)G);
            if (seen.count(key)) return;
            if (seen.size() * (key.size() + 64) < kMaxSeenBytes) seen.insert(std::move(key));   // 64: node and bucket overhead
        }
        double next[MLORA_MAX_CLUSTER_GPUS];
        for (int p = 0; p < n; ++p) {
            if (used[p]) continue;
            bool twin_waiting = false;     // equal tasks only in index order
            for (int q = 0; q < p; ++q)
                if (!used[q] && d[q] == d[p] && g[q] == g[p]) { twin_waiting = true; break; }
            if (twin_waiting) continue;
            const double s = idle[g[p] - 1];                // >= front: the idle times are clipped to it
            if (p < last && s <= front + kEps) continue;    // equal starts only in candidate order
            // the g[p] GPUs that have been idle longest take the task; the others idle before s count as idle from s
            const double e = s + d[p];
            int m = 0;
            for (int q = g[p]; q < G; ++q) next[m++] = std::max(idle[q], s);
            // merge g[p] copies of e into the (sorted) rest
            int pos = m;
            while (pos > 0 && next[pos - 1] > e) --pos;
            for (int q = m - 1; q >= pos; --q) next[q + g[p]] = next[q];
            for (int q = 0; q < g[p]; ++q) next[pos + q] = e;
            used[p] = 1;
            cur[p] = s;
            double child[MLORA_MAX_CLUSTER_GPUS];
            std::memcpy(child, next, sizeof(double) * (size_t)G);
            dfs(depth + 1, std::max(mk, e), s, p, child, mask | (1u << p));
            used[p] = 0;
            if (done) return;
        }
    }
    // starts[i] by caller index; returns the makespan
    double solve(int n_, const double* dur, const int32_t* need, int G_, const double* release, double now_,
                 double* starts) {
        n = n_; G = G_; now = now_;
        std::vector<double> rel(G, now);
        if (release)
            for (int q = 0; q < G; ++q) rel[q] = std::max(release[q], now);
        std::sort(rel.begin(), rel.end());
        idx.resize(n);
        for (int i = 0; i < n; ++i) idx[i] = i;
        std::stable_sort(idx.begin(), idx.end(), [&](int a, int b) {
            if (need[a] != need[b]) return need[a] > need[b];
            return dur[a] > dur[b];
        });
        d.resize(n); g.resize(n);
        for (int p = 0; p < n; ++p) { d[p] = dur[idx[p]]; g[p] = need[idx[p]]; }
        used.assign(n, 0);
        cur.assign(n, 0.0);
        best.assign(n, 0.0);
        best_mk = INFINITY;
        done = out_of_budget = false;
        nodes = 0;
        seen.clear();
        // root bound: longest single task from its earliest possible start, and total work against capacity
        root_lb = now;
        double work = 0.0;
        for (int p = 0; p < n; ++p) {
            root_lb = std::max(root_lb, rel[g[p] - 1] + d[p]);
            work += d[p] * g[p];
        }
        {   // smallest C with sum_q max(0, C - rel_q) >= work
            double acc = 0.0;     // capacity before rel[q] from GPUs 0..q-1
            for (int q = 0; q < G; ++q) {
                const double nxt = q + 1 < G ? rel[q + 1] : INFINITY;
                const double cap_at_next = nxt == INFINITY ? INFINITY : acc + (q + 1) * (nxt - rel[q]);
                if (work <= cap_at_next) {
                    root_lb = std::max(root_lb, rel[q] + (work - acc) / (q + 1));
                    break;
                }
                acc = cap_at_next;
            }
        }
        if (n == 0) return now;
        dfs(0, now, now, -1, rel.data(), 0u);
        for (int p = 0; p < n; ++p) starts[idx[p]] = best[p];
        return best_mk;
    }
};

// GPUs in order of start time (ties: candidate order), lowest idle index first
void hand_out_gpus(int n, const double* dur, const int32_t* need, int G, const double* release, double now,
                   const double* starts, uint64_t* masks) {
    std::vector<double> free_at(G, now);
    if (release)
        for (int q = 0; q < G; ++q) free_at[q] = std::max(release[q], now);
    std::vector<int> cand(n), order(n);
    for (int i = 0; i < n; ++i) cand[i] = i;
    std::stable_sort(cand.begin(), cand.end(), [&](int a, int b) {
        if (need[a] != need[b]) return need[a] > need[b];
        return dur[a] > dur[b];
    });
    std::vector<int> pos(n);
    for (int p = 0; p < n; ++p) pos[cand[p]] = p;
    for (int i = 0; i < n; ++i) order[i] = i;
    std::sort(order.begin(), order.end(), [&](int a, int b) {
        if (starts[a] != starts[b]) return starts[a] < starts[b];
        return pos[a] < pos[b];
    });
    for (int i : order) {
        uint64_t m = 0;
        int got = 0;
        for (int q = 0; q < G && got < need[i]; ++q)
            if (free_at[q] <= starts[i] + kEps) {
                m |= (uint64_t)1 << q;
                free_at[q] = starts[i] + dur[i];
                ++got;
            }
        masks[i] = m;
    }
}

bool bad_task(double duration, int32_t gpus, int32_t G) {
    return !(duration > 0.0) || !std::isfinite(duration) || gpus < 1 || gpus > G;
}

}  // namespace

extern "C" int multi_lora_schedule_tasks(int32_t n, const double* durations, const int32_t* gpus_needed, int32_t G,
                                         const double* release, double now, double* starts, uint64_t* gpu_masks,
                                         double* makespan, int32_t* proved_optimal) {
    if (n < 0 || n > MLORA_MAX_TASKS || G < 1 || G > MLORA_MAX_CLUSTER_GPUS || !std::isfinite(now)) {
        set_error("schedule: n in [0, MLORA_MAX_TASKS], G in [1, MLORA_MAX_CLUSTER_GPUS], finite now");
        return MLORA_ERR_SHAPE;
    }
    if (!makespan || (n > 0 && (!durations || !gpus_needed || !starts || !gpu_masks))) {
        set_error("schedule: NULL argument");
        return MLORA_ERR_NULL;
    }
    for (int32_t i = 0; i < n; ++i)
        if (bad_task(durations[i], gpus_needed[i], G)) {
            set_error("schedule: a task needs a positive finite duration and 1..G GPUs");
            return MLORA_ERR_SHAPE;
        }
    if (release)
        for (int32_t q = 0; q < G; ++q)
            if (!std::isfinite(release[q])) {
                set_error("schedule: release times must be finite");
                return MLORA_ERR_SHAPE;
            }
    Solver s;
    *makespan = s.solve(n, durations, gpus_needed, G, release, now, starts);
    if (proved_optimal) *proved_optimal = s.out_of_budget ? 0 : 1;
    if (n > 0) hand_out_gpus(n, durations, gpus_needed, G, release, now, starts, gpu_masks);
    return MLORA_OK;
}

// ---- event-driven re-planning -------------------------------------------------------------------

struct mlora_cluster {
    int32_t G = 0;
    struct Pending { int32_t id; double d; int32_t g; double planned; };
    struct Running { int32_t id; double start, est_end; uint64_t mask; };
    std::vector<Pending> pending;     // submission order
    std::vector<Running> running;
    double planned_makespan = 0.0;
    int32_t next_id = 0;

    void release_times(double now, std::vector<double>& rel) const {
        rel.assign(G, now);
        for (const Running& r : running)
            for (int q = 0; q < G; ++q)
                if (r.mask >> q & 1) rel[q] = std::max(r.est_end, now);    // an overrun estimate counts as "now"
    }
    void replan(double now) {
        std::vector<double> rel;
        release_times(now, rel);
        const int n = (int)pending.size();
        std::vector<double> d(n), starts(n);
        std::vector<int32_t> g(n);
        for (int i = 0; i < n; ++i) { d[i] = pending[i].d; g[i] = pending[i].g; }
        Solver s;
        double mk = s.solve(n, d.data(), g.data(), G, rel.data(), now, starts.data());
        for (int i = 0; i < n; ++i) pending[i].planned = starts[i];
        for (double r : rel) mk = std::max(mk, r);
        planned_makespan = mk;
    }
};

extern "C" int multi_lora_cluster_create(mlora_cluster** out, int32_t G) {
    if (!out) { set_error("cluster create: NULL argument"); return MLORA_ERR_NULL; }
    *out = nullptr;
    if (G < 1 || G > MLORA_MAX_CLUSTER_GPUS) {
        set_error("cluster create: G in [1, MLORA_MAX_CLUSTER_GPUS]");
        return MLORA_ERR_SHAPE;
    }
    mlora_cluster* c = new mlora_cluster();
    c->G = G;
    *out = c;
    return MLORA_OK;
}

extern "C" int multi_lora_cluster_destroy(mlora_cluster* cluster) {
    delete cluster;
    return MLORA_OK;
}

extern "C" int multi_lora_cluster_submit(mlora_cluster* cluster, double now, double duration, int32_t gpus,
                                         int32_t* task_id) {
    if (!cluster || !task_id) { set_error("cluster submit: NULL argument"); return MLORA_ERR_NULL; }
    if (bad_task(duration, gpus, cluster->G) || !std::isfinite(now)) {
        set_error("cluster submit: a task needs a positive finite duration and 1..G GPUs");
        return MLORA_ERR_SHAPE;
    }
    if ((int)cluster->pending.size() >= MLORA_MAX_TASKS) {
        set_error("cluster submit: MLORA_MAX_TASKS tasks are already waiting");
        return MLORA_ERR_SHAPE;
    }
    *task_id = cluster->next_id++;
    cluster->pending.push_back({*task_id, duration, gpus, 0.0});
    cluster->replan(now);
    return MLORA_OK;
}

extern "C" int multi_lora_cluster_complete(mlora_cluster* cluster, double now, int32_t task_id) {
    if (!cluster) { set_error("cluster complete: NULL argument"); return MLORA_ERR_NULL; }
    for (size_t i = 0; i < cluster->running.size(); ++i)
        if (cluster->running[i].id == task_id) {
            cluster->running.erase(cluster->running.begin() + (std::ptrdiff_t)i);
            cluster->replan(now);
            return MLORA_OK;
        }
    set_error("cluster complete: task is not running");
    return MLORA_ERR_SHAPE;
}

extern "C" int multi_lora_cluster_poll(mlora_cluster* cluster, double now, int32_t* task_ids, uint64_t* gpu_masks,
                                       int32_t cap, int32_t* count) {
    if (!cluster || !count || (cap > 0 && (!task_ids || !gpu_masks))) {
        set_error("cluster poll: NULL argument");
        return MLORA_ERR_NULL;
    }
    mlora_cluster& c = *cluster;
    // tasks that are due, by planned start, ties in candidate order (g descending, d descending, submission order)
    std::vector<int> due;
    for (int i = 0; i < (int)c.pending.size(); ++i)
        if (c.pending[i].planned <= now + kEps) due.push_back(i);
    std::stable_sort(due.begin(), due.end(), [&](int a, int b) {
        const auto &x = c.pending[a], &y = c.pending[b];
        if (x.planned != y.planned) return x.planned < y.planned;
        if (x.g != y.g) return x.g > y.g;
        return x.d > y.d;
    });
    uint64_t busy = 0;
    for (const auto& r : c.running) busy |= r.mask;
    bool stale = false;
    std::vector<int> started;      // indices into pending
    std::vector<uint64_t> masks;
    for (int i : due) {
        const auto& t = c.pending[i];
        uint64_t m = 0;
        int got = 0;
        for (int q = 0; q < c.G && got < t.g; ++q)
            if (!(busy >> q & 1)) { m |= (uint64_t)1 << q; ++got; }
        if (got < t.g) { stale = true; continue; }        // a running task has overrun its estimate
        if (t.planned < now - kEps) stale = true;          // started late: what is planned behind it moves
        busy |= m;
        started.push_back(i);
        masks.push_back(m);
    }
    *count = (int32_t)started.size();
    for (size_t j = 0; j < started.size() && (int32_t)j < cap; ++j) {
        task_ids[j] = c.pending[started[j]].id;
        gpu_masks[j] = masks[j];
    }
    for (size_t j = 0; j < started.size(); ++j) {
        const auto& t = c.pending[started[j]];
        c.running.push_back({t.id, now, now + t.d, masks[j]});
    }
    std::vector<int> gone = started;
    std::sort(gone.begin(), gone.end());
    for (size_t j = gone.size(); j-- > 0;) c.pending.erase(c.pending.begin() + gone[j]);
    if (stale) c.replan(now);
    if (*count > cap) {
        set_error("cluster poll: output arrays too small (the tasks have been started)");
        return MLORA_ERR_SHAPE;
    }
    return MLORA_OK;
}

extern "C" int multi_lora_cluster_plan(const mlora_cluster* cluster, int32_t* task_ids, double* planned_starts,
                                       int32_t cap, int32_t* count, double* planned_makespan) {
    if (!cluster || !count || (cap > 0 && (!task_ids || !planned_starts))) {
        set_error("cluster plan: NULL argument");
        return MLORA_ERR_NULL;
    }
    *count = (int32_t)cluster->pending.size();
    if (planned_makespan) *planned_makespan = cluster->planned_makespan;
    for (int32_t i = 0; i < *count && i < cap; ++i) {
        task_ids[i] = cluster->pending[i].id;
        planned_starts[i] = cluster->pending[i].planned;
    }
    if (*count > cap) {
        set_error("cluster plan: output arrays too small");
        return MLORA_ERR_SHAPE;
    }
    return MLORA_OK;
}
