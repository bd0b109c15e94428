// The scheduler's outer loop (paper Section 4.3) and the score it maximises (Section 5.1, SLO attainment).
// Host code, no device work.
//
// A deployment is a partition of the GPU pool into independent pipeline groups (model replicas), each described by
// its count vector tau over the GPU types.  The paper names the search's ingredients -- K-means over the
// communication matrices for the start, the number of groups from the elbow of the inertia curve, the merge / split /
// swap mutations, an early memory check, a layer partition that starts even and is then made proportional to the
// stages' memory, a task simulator that turns the replicas' latencies into an expected SLO attainment -- and leaves
// the driver around them open.  What this file fixes on top of the paper:
//   request queue   requests in arrival order, never dropped; a replica serves one request at a time; a request goes
//                   to the replica where it would finish earliest (lowest index on ties); it is on time when
//                   finish <= arrival + deadline.
//   random draws    draw(seed, c) = output c + 1 of the SplitMix64 sequence started at seed; an index below n is
//                   draw mod n; iteration `it` uses counters 5 it .. 5 it + 4 (member, operator, two groups, type).
//   K-means         a point per GPU type present, weighted by its GPU count; features: the type's row of hop latencies
//                   over the largest latency, then its row of per-byte times over the largest per-byte time; seeds:
//                   the heaviest point, then the point farthest from its nearest seed; Lloyd rounds to a fixed point.
//   elbow           on the curve ((M-1)/(n-1), W_M / W_1) the point farthest below the chord between its ends.
//   group plan      per stage count S: even partition -> layout DP -> memory-proportional partition -> layout DP,
//                   the cheaper of the two; the cheapest S (fewest stages on ties).
//   population      an offspring that applies, passes the early checks and has a plan joins the population while
//                   there is room, else replaces the member of lowest attainment (oldest first) unless it scores lower.
#include <algorithm>
#include <cmath>
#include <cstdint>
#include <limits>
#include <map>
#include <vector>

#include "../../include/hexgen.h"

namespace {
const double kInf = std::numeric_limits<double>::infinity();
const double kNaN = std::numeric_limits<double>::quiet_NaN();
typedef std::vector<int> Tau;

bool pool_ok(const hexgen_pool_t *p) {
    if (!p || p->n_types <= 0 || p->n_types > 8 || !p->count || !p->m_d || !p->c_d || !p->mem_bytes || !p->tp_alpha ||
        !p->tp_beta || !p->pp_alpha || !p->pp_beta)
        return false;
    for (int k = 0; k < p->n_types; ++k)
        if (p->count[k] < 0 || p->count[k] > 64) return false;
    return true;
}

// the hop links between the GPU types that are present must be usable numbers: latency >= 0, bandwidth > 0
bool links_ok(const hexgen_pool_t *p) {
    for (int a = 0; a < p->n_types; ++a)
        for (int b = 0; b < p->n_types; ++b) {
            if (p->count[a] == 0 || p->count[b] == 0) continue;
            const double al = p->pp_alpha[a * p->n_types + b], be = p->pp_beta[a * p->n_types + b];
            if (!(al >= 0.0) || !(be > 0.0) || std::isinf(al) || std::isinf(be)) return false;
        }
    return true;
}

int total(const Tau &t) {
    int s = 0;
    for (int v : t) s += v;
    return s;
}

// ---- request queue -------------------------------------------------------------------------------------------------
double attainment(int n_req, const double *arrival, const int *cls, int n_rep, int n_cls, const double *latency,
                  const double *deadline, double *finish_out) {
    std::vector<double> free_at(n_rep, 0.0);
    long on_time = 0;
    for (int q = 0; q < n_req; ++q) {
        const int c = cls ? cls[q] : 0;
        int pick = 0;
        double pick_f = 0.0;
        for (int r = 0; r < n_rep; ++r) {
            const double f = std::max(arrival[q], free_at[r]) + latency[(size_t)r * n_cls + c];
            if (r == 0 || f < pick_f) { pick = r; pick_f = f; }
        }
        free_at[pick] = pick_f;
        if (finish_out) finish_out[q] = pick_f;
        if (pick_f <= arrival[q] + deadline[c]) ++on_time;
    }
    return (double)on_time / (double)n_req;
}

// ---- K-means start ---------------------------------------------------------------------------------------------------
struct Clustering {
    std::vector<int> label;
    double inertia;
};

double dist2(const std::vector<double> &a, const std::vector<double> &b) {
    double s = 0.0;
    for (size_t d = 0; d < a.size(); ++d) s += (a[d] - b[d]) * (a[d] - b[d]);
    return s;
}

Clustering lloyd(const std::vector<std::vector<double>> &pt, const std::vector<double> &w, int m) {
    const int n = (int)pt.size();
    std::vector<std::vector<double>> centre;
    int heavy = 0;
    for (int i = 1; i < n; ++i)
        if (w[i] > w[heavy]) heavy = i;
    centre.push_back(pt[heavy]);
    while ((int)centre.size() < m) {
        int far = 0;
        double far_d = -1.0;
        for (int i = 0; i < n; ++i) {
            double d = kInf;
            for (const auto &c : centre) d = std::min(d, dist2(pt[i], c));
            if (d > far_d) { far = i; far_d = d; }
        }
        centre.push_back(pt[far]);
    }
    Clustering out;
    out.label.assign(n, -1);
    for (int round = 0; round < 100; ++round) {
        std::vector<int> now(n);
        for (int i = 0; i < n; ++i) {
            int best = 0;
            double best_d = dist2(pt[i], centre[0]);
            for (int c = 1; c < m; ++c) {
                const double d = dist2(pt[i], centre[c]);
                if (d < best_d) { best = c; best_d = d; }
            }
            now[i] = best;
        }
        if (now == out.label) break;
        out.label = now;
        for (int c = 0; c < m; ++c) {
            double wsum = 0.0;
            std::vector<double> acc(pt[0].size(), 0.0);
            for (int i = 0; i < n; ++i) {
                if (out.label[i] != c) continue;
                wsum += w[i];
                for (size_t d = 0; d < acc.size(); ++d) acc[d] += w[i] * pt[i][d];
            }
            if (wsum == 0.0) continue;           // an empty cluster keeps its centre
            for (size_t d = 0; d < acc.size(); ++d) centre[c][d] = acc[d] / wsum;
        }
    }
    out.inertia = 0.0;
    for (int i = 0; i < n; ++i) out.inertia += w[i] * dist2(pt[i], centre[out.label[i]]);
    return out;
}

int elbow(const std::vector<double> &inertia) {
    const int n = (int)inertia.size();
    if (n == 1 || !(inertia[0] > 0.0)) return 1;
    const double y_last = inertia[n - 1] / inertia[0];
    int best = 1;
    double best_d = 0.0;
    for (int m = 1; m <= n; ++m) {
        const double x = (double)(m - 1) / (double)(n - 1);
        const double d = (1.0 - (1.0 - y_last) * x) - inertia[m - 1] / inertia[0];
        if (d > best_d) { best = m; best_d = d; }
    }
    return best;
}

std::vector<Tau> initial_groups(const hexgen_pool_t *p) {
    const int NT = p->n_types;
    std::vector<int> present;
    for (int k = 0; k < NT; ++k)
        if (p->count[k] > 0) present.push_back(k);
    std::vector<Tau> groups;
    if (present.empty()) return groups;
    double a_max = 0.0, t_max = 0.0;
    for (int a : present)
        for (int b : present) {
            a_max = std::max(a_max, p->pp_alpha[a * NT + b]);
            t_max = std::max(t_max, 1.0 / p->pp_beta[a * NT + b]);
        }
    std::vector<std::vector<double>> pt;
    std::vector<double> w;
    for (int a : present) {
        std::vector<double> f;
        for (int b : present) f.push_back(a_max > 0.0 ? p->pp_alpha[a * NT + b] / a_max : 0.0);
        for (int b : present) f.push_back((1.0 / p->pp_beta[a * NT + b]) / t_max);
        pt.push_back(f);
        w.push_back((double)p->count[a]);
    }
    std::vector<Clustering> runs;
    std::vector<double> inertia;
    for (int m = 1; m <= (int)present.size(); ++m) {
        runs.push_back(lloyd(pt, w, m));
        inertia.push_back(runs.back().inertia);
    }
    const int m = elbow(inertia);
    for (int c = 0; c < m; ++c) {
        Tau tau(NT, 0);
        for (size_t i = 0; i < present.size(); ++i)
            if (runs[m - 1].label[i] == c) tau[present[i]] = p->count[present[i]];
        if (total(tau) > 0) groups.push_back(tau);
    }
    return groups;
}

// ---- one group's pipeline --------------------------------------------------------------------------------------------
struct Plan {
    double latency = kInf;
    std::vector<int> layers, type, count;
};

Plan plan_group(const hexgen_pool_t *pool, const hexgen_task_t *task, const Tau &tau, int total_layers, int max_stages,
                int pow2) {
    hexgen_pool_t sub = *pool;
    sub.count = tau.data();
    Plan best;
    const int s_max = std::min(std::min(max_stages, total(tau)), total_layers);
    for (int S = 1; S <= s_max; ++S) {
        std::vector<int> even(S), type(S), count(S);
        for (int j = 0; j < S; ++j) even[j] = total_layers / S + (j < total_layers % S ? 1 : 0);
        const double c1 = hexgen_sched_pipeline_layout(&sub, task, S, even.data(), pow2, type.data(), count.data());
        if (!(c1 < kInf)) continue;
        Plan cand;
        cand.latency = c1;
        cand.layers = even;
        cand.type = type;
        cand.count = count;
        std::vector<double> mem(S);
        for (int j = 0; j < S; ++j) mem[j] = pool->mem_bytes[type[j]] * count[j];
        std::vector<int> prop(S), type2(S), count2(S);
        if (hexgen_sched_repartition_layers(total_layers, S, mem.data(), prop.data()) && prop != even) {
            const double c2 = hexgen_sched_pipeline_layout(&sub, task, S, prop.data(), pow2, type2.data(), count2.data());
            if (c2 < c1) {
                cand.latency = c2;
                cand.layers = prop;
                cand.type = type2;
                cand.count = count2;
            }
        }
        if (cand.latency < best.latency) best = cand;
    }
    return best;
}

uint64_t draw(uint64_t seed, uint64_t counter) {
    uint64_t z = seed + (counter + 1) * 0x9E3779B97F4A7C15ull;
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    return z ^ (z >> 31);
}
}  // namespace

extern "C" {

double hexgen_slo_attainment(int n_req, const double *arrival, const int *cls, int n_replicas, int n_classes,
                             const double *latency, const double *deadline, double *finish_out) try {
    if (n_req <= 0 || !arrival || n_replicas <= 0 || n_classes <= 0 || !latency || !deadline) return kNaN;
    for (int q = 0; q < n_req; ++q) {
        if (!(arrival[q] >= (q ? arrival[q - 1] : 0.0))) return kNaN;          // sorted, non-negative, no NaN
        if (cls && (cls[q] < 0 || cls[q] >= n_classes)) return kNaN;
    }
    for (int i = 0; i < n_replicas * n_classes; ++i)
        if (!(latency[i] > 0.0)) return kNaN;
    return attainment(n_req, arrival, cls, n_replicas, n_classes, latency, deadline, finish_out);
} catch (...) {      // no exception (an allocation failure) may cross the C boundary
    return kNaN;
}

unsigned long long hexgen_sched_draw(unsigned long long seed, unsigned long long counter) { return draw(seed, counter); }

int hexgen_sched_initial_groups(const hexgen_pool_t *pool, int *groups) try {
    if (!pool_ok(pool) || !links_ok(pool) || !groups) return 0;
    const std::vector<Tau> g = initial_groups(pool);
    for (size_t i = 0; i < g.size(); ++i)
        for (int k = 0; k < pool->n_types; ++k) groups[i * pool->n_types + k] = g[i][k];
    return (int)g.size();
} catch (...) {      // no exception (an allocation failure) may cross the C boundary
    return 0;
}

double hexgen_sched_plan_group(const hexgen_pool_t *pool, const hexgen_task_t *task, const int *tau, int total_layers,
                               int max_stages, int pow2_degrees_only, int *n_stages, int *layers, int *stage_type,
                               int *stage_count) try {
    if (!pool_ok(pool) || !task || !tau || total_layers <= 0 || max_stages <= 0 || max_stages > 64) return kNaN;
    Tau t(tau, tau + pool->n_types);
    for (int k = 0; k < pool->n_types; ++k)
        if (t[k] < 0 || t[k] > pool->count[k]) return kNaN;
    const Plan p = plan_group(pool, task, t, total_layers, max_stages, pow2_degrees_only);
    if (std::isnan(p.latency)) return kNaN;
    if (n_stages) *n_stages = (int)p.layers.size();
    for (size_t j = 0; j < p.layers.size(); ++j) {
        if (layers) layers[j] = p.layers[j];
        if (stage_type) stage_type[j] = p.type[j];
        if (stage_count) stage_count[j] = p.count[j];
    }
    return p.latency;
} catch (...) {      // no exception (an allocation failure) may cross the C boundary
    return kNaN;
}

double hexgen_sched_search(const hexgen_pool_t *pool, const hexgen_task_t *task, const hexgen_search_t *cfg, int n_req,
                           const double *arrival, double deadline, int max_groups, int *n_groups, int *group_tau,
                           double *group_latency, int *group_n_stages, int *stage_layers, int *stage_type,
                           int *stage_count, double *history) try {
    if (!pool_ok(pool) || !links_ok(pool) || !task || !cfg || n_req <= 0 || !arrival || !(deadline > 0.0) || max_groups <= 0 || !n_groups ||
        !group_tau || cfg->total_layers <= 0 || cfg->max_stages <= 0 || cfg->max_stages > 64 || cfg->n_iter < 0 ||
        cfg->pop_size <= 0 || cfg->max_group_states <= 0)
        return kNaN;
    for (int q = 0; q < n_req; ++q)
        if (!(arrival[q] >= (q ? arrival[q - 1] : 0.0))) return kNaN;
    const int NT = pool->n_types;

    std::map<Tau, Plan> plans;
    auto plan = [&](const Tau &tau) -> const Plan & {
        auto it = plans.find(tau);
        if (it == plans.end())
            it = plans.emplace(tau, plan_group(pool, task, tau, cfg->total_layers, cfg->max_stages, cfg->pow2_degrees_only)).first;
        return it->second;
    };
    auto admissible = [&](const Tau &tau) {
        if (total(tau) <= 0 || !hexgen_sched_group_can_hold(NT, tau.data(), pool->mem_bytes, cfg->model_bytes)) return false;
        long states = 1;
        for (int v : tau) {
            states *= v + 1;
            if (states > cfg->max_group_states) return false;
        }
        return plan(tau).latency < kInf;
    };
    typedef std::vector<Tau> Groups;
    auto fitness = [&](const Groups &g) {
        std::vector<double> lat;
        for (const Tau &t : g) lat.push_back(plan(t).latency);
        return attainment(n_req, arrival, nullptr, (int)lat.size(), 1, lat.data(), &deadline, nullptr);
    };
    auto all_admissible = [&](const Groups &g) {
        for (const Tau &t : g)
            if (!admissible(t)) return false;
        return true;
    };

    Groups start = initial_groups(pool);
    if (start.empty() || !all_admissible(start)) {
        // a start with a cluster that cannot serve the model falls back to the whole pool as one group
        start.assign(1, Tau(pool->count, pool->count + NT));
        if (!admissible(start[0])) return kNaN;
    }
    struct Member { Groups groups; double score; };
    std::vector<Member> population;
    population.push_back(Member{start, fitness(start)});
    Member best = population[0];
    for (int it = 0; it < cfg->n_iter; ++it) {
        uint64_t u[5];
        for (int j = 0; j < 5; ++j) u[j] = draw(cfg->seed, 5ull * (uint64_t)it + j);
        const Groups &parent = population[u[0] % population.size()].groups;
        const int op = (int)(u[1] % 3), n_g = (int)parent.size();
        Groups child, fresh;
        bool applies = false;
        if (op == 0 && n_g >= 2) {                    // merge groups i and j
            const int i = (int)(u[2] % n_g);
            int j = (int)(u[3] % (n_g - 1));
            if (j >= i) ++j;
            Tau merged(NT);
            hexgen_sched_merge(NT, parent[i].data(), parent[j].data(), merged.data());
            for (int x = 0; x < n_g; ++x)
                if (x != i && x != j) child.push_back(parent[x]);
            child.push_back(merged);
            fresh.push_back(merged);
            applies = true;
        } else if (op == 1) {                         // split group i
            const int i = (int)(u[2] % n_g);
            Tau lo(NT), hi(NT);
            hexgen_sched_split(NT, parent[i].data(), lo.data(), hi.data());
            if (total(lo) > 0 && total(hi) > 0) {
                child = parent;
                child[i] = lo;
                child.push_back(hi);
                fresh = {lo, hi};
                applies = true;
            }
        } else if (op == 2 && n_g >= 2) {             // one GPU from group j to group i
            const int i = (int)(u[2] % n_g);
            int j = (int)(u[3] % (n_g - 1));
            if (j >= i) ++j;
            std::vector<int> held;
            for (int k = 0; k < NT; ++k)
                if (parent[j][k] > 0) held.push_back(k);
            const int k = held[u[4] % held.size()];
            child = parent;
            hexgen_sched_swap(NT, child[i].data(), child[j].data(), k);
            fresh.push_back(child[i]);
            if (total(child[j]) == 0) child.erase(child.begin() + j);
            else fresh.push_back(child[j]);
            applies = true;
        }
        if (applies && all_admissible(fresh)) {
            const double f = fitness(child);
            if ((int)population.size() < cfg->pop_size) {
                population.push_back(Member{child, f});
            } else {
                size_t worst = 0;
                for (size_t x = 1; x < population.size(); ++x)
                    if (population[x].score < population[worst].score) worst = x;
                if (f >= population[worst].score) {
                    population.erase(population.begin() + worst);
                    population.push_back(Member{child, f});
                }
            }
            if (f > best.score) best = Member{child, f};
        }
        if (history) history[it] = best.score;
    }

    if ((int)best.groups.size() > max_groups) return kNaN;
    *n_groups = (int)best.groups.size();
    for (size_t g = 0; g < best.groups.size(); ++g) {
        const Plan &p = plan(best.groups[g]);
        for (int k = 0; k < NT; ++k) group_tau[g * NT + k] = best.groups[g][k];
        if (group_latency) group_latency[g] = p.latency;
        if (group_n_stages) group_n_stages[g] = (int)p.layers.size();
        for (size_t j = 0; j < p.layers.size(); ++j) {
            const size_t o = g * cfg->max_stages + j;
            if (stage_layers) stage_layers[o] = p.layers[j];
            if (stage_type) stage_type[o] = p.type[j];
            if (stage_count) stage_count[o] = p.count[j];
        }
    }
    return best.score;
} catch (...) {      // no exception (an allocation failure) may cross the C boundary
    return kNaN;
}

}  // extern "C"
