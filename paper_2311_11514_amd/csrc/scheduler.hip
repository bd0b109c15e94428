// Pipeline layout by dynamic programming (paper Section 4.2, Algorithm 1) and the mutation operators and layer
// re-partition rule of the search (Section 4.3).  Host code, no device work.
//
// A pipeline group holds count[k] GPUs of each of n_types types; a layer partition l_1 .. l_S is given; every stage
// runs on tau_k GPUs of ONE type (the paper's heuristic).  DP[j; tau] of the paper is the cheapest way to serve the
// first j stages with the GPU multiset tau.  The pipeline-hop term of the end-to-end cost couples consecutive
// stages through their types, so the state here also records the type of stage j: DP[j; tau; k].  Stage costs come
// from the cost-model functions of this library (Eqs. 3, 4, 6), hops from Eq. 5 with one link per type pair.
#include <cmath>
#include <limits>
#include <vector>

#include "../../include/hexgen.h"

namespace {
const double kInf = std::numeric_limits<double>::infinity();
const double kNaN = std::numeric_limits<double>::quiet_NaN();

bool bad_pool(const hexgen_pool_t *p) {
    if (!p || p->n_types <= 0 || p->n_types > 8 || !p->count || !p->m_d || !p->c_d || !p->mem_bytes || !p->tp_alpha ||
        !p->tp_beta || !p->pp_alpha || !p->pp_beta)
        return true;
    for (int k = 0; k < p->n_types; ++k)
        if (p->count[k] < 0 || p->count[k] > 64) return true;
    return false;
}

double stage_cost(const hexgen_pool_t *p, const hexgen_task_t *t, int layers, int k, int n) {
    if (hexgen_cost_mem(t->hidden, t->params_factor, t->bytes_per_elem, t->batch, t->s_in, t->s_out, layers, n) >
        p->mem_bytes[k])
        return kInf;
    std::vector<double> m(n, p->m_d[k]), c(n, p->c_d[k]), al((size_t)n * n, p->tp_alpha[k]), be((size_t)n * n, p->tp_beta[k]);
    return hexgen_cost_comp(t->hidden, t->params_factor, t->bytes_per_elem, t->batch, t->s_in, t->s_out, layers, n, m.data(),
                            c.data()) +
           hexgen_cost_comm_tp(t->hidden, t->bytes_per_elem, t->batch, t->s_in, t->s_out, layers, n, al.data(), be.data());
}
}  // namespace

extern "C" {

double hexgen_sched_pipeline_layout(const hexgen_pool_t *pool, const hexgen_task_t *task, int n_stages, const int *layers,
                                    int pow2_degrees_only, int *stage_type, int *stage_count) try {
    if (bad_pool(pool) || !task || n_stages <= 0 || n_stages > 64 || !layers) return kNaN;
    for (int j = 0; j < n_stages; ++j)
        if (layers[j] <= 0) return kNaN;
    const int NT = pool->n_types;
    // mixed-radix index of a count vector tau, 0 <= tau_k <= count[k]
    std::vector<long> radix(NT, 1);
    long n_tau = 1;
    for (int k = 0; k < NT; ++k) { radix[k] = n_tau; n_tau *= pool->count[k] + 1; }
    if (n_tau > (1L << 22)) return kNaN;
    auto digit = [&](long idx, int k) { return (int)((idx / radix[k]) % (pool->count[k] + 1)); };
    const size_t states = (size_t)n_tau * NT;
    std::vector<double> prev(states, kInf), cur(states, kInf);
    // parent[j][state] = (type, count) chosen for stage j and the predecessor's type, for the back-track
    struct Step { short k_prev, n; };
    std::vector<std::vector<Step>> parent(n_stages, std::vector<Step>(states, Step{-1, 0}));
    std::vector<double> hop((size_t)NT * NT, 0.0);
    for (int a = 0; a < NT; ++a)
        for (int b = 0; b < NT; ++b)
            hop[(size_t)a * NT + b] = hexgen_cost_comm_pp(task->hidden, task->bytes_per_elem, task->batch, task->s_in, task->s_out,
                                                          1, 1, pool->pp_alpha + a * NT + b, pool->pp_beta + a * NT + b);
    for (int j = 0; j < n_stages; ++j) {
        std::fill(cur.begin(), cur.end(), kInf);
        for (int k = 0; k < NT; ++k) {
            for (int n = 1; n <= pool->count[k]; ++n) {
                if (pow2_degrees_only && (n & (n - 1))) continue;
                const double sc = stage_cost(pool, task, layers[j], k, n);
                if (!(sc < kInf)) continue;
                if (std::isnan(sc)) return kNaN;
                if (j == 0) {
                    const size_t s = (size_t)(n * radix[k]) * NT + k;
                    if (sc < cur[s]) { cur[s] = sc; parent[0][s] = Step{-1, (short)n}; }
                    continue;
                }
                for (long tau = 0; tau < n_tau; ++tau) {
                    if (digit(tau, k) + n > pool->count[k]) continue;
                    for (int kp = 0; kp < NT; ++kp) {
                        const double base = prev[(size_t)tau * NT + kp];
                        if (!(base < kInf)) continue;
                        const double c = base + hop[(size_t)kp * NT + k] + sc;
                        const size_t s = (size_t)(tau + n * radix[k]) * NT + k;
                        if (c < cur[s]) { cur[s] = c; parent[j][s] = Step{(short)kp, (short)n}; }
                    }
                }
            }
        }
        prev.swap(cur);
    }
    // best entry of the last row; GPUs may stay unused
    double best = kInf;
    size_t best_s = 0;
    for (size_t s = 0; s < states; ++s)
        if (prev[s] < best) { best = prev[s]; best_s = s; }
    if (!(best < kInf)) return kInf;
    if (stage_type && stage_count) {
        size_t s = best_s;
        for (int j = n_stages - 1; j >= 0; --j) {
            const int k = (int)(s % NT);
            const Step st = parent[j][s];
            stage_type[j] = k;
            stage_count[j] = st.n;
            if (j > 0) s = (size_t)((long)(s / NT) - st.n * radix[k]) * NT + st.k_prev;
        }
    }
    return best;
} catch (...) {      // no exception (an allocation failure) may cross the C boundary
    return kNaN;
}

int hexgen_sched_merge(int n_types, const int *tau1, const int *tau2, int *out) {
    if (n_types <= 0 || !tau1 || !tau2 || !out) return 0;
    for (int k = 0; k < n_types; ++k) out[k] = tau1[k] + tau2[k];
    return 1;
}

int hexgen_sched_split(int n_types, const int *tau, int *out1, int *out2) {
    if (n_types <= 0 || !tau || !out1 || !out2) return 0;
    for (int k = 0; k < n_types; ++k) { out1[k] = tau[k] / 2; out2[k] = tau[k] - tau[k] / 2; }
    return 1;
}

int hexgen_sched_swap(int n_types, int *tau1, int *tau2, int type) {
    if (n_types <= 0 || !tau1 || !tau2 || type < 0 || type >= n_types || tau2[type] < 1) return 0;
    tau1[type] += 1;
    tau2[type] -= 1;
    return 1;
}

int hexgen_sched_group_can_hold(int n_types, const int *tau, const double *mem_bytes, double model_bytes) {
    if (n_types <= 0 || !tau || !mem_bytes) return 0;
    double total = 0.0;
    for (int k = 0; k < n_types; ++k) total += tau[k] * mem_bytes[k];
    return total >= model_bytes ? 1 : 0;
}

int hexgen_sched_repartition_layers(int total_layers, int n_stages, const double *stage_mem, int *layers_out) try {
    if (n_stages <= 0 || total_layers < n_stages || !stage_mem || !layers_out) return 0;
    double tot = 0.0;
    for (int j = 0; j < n_stages; ++j) {
        if (!(stage_mem[j] > 0.0)) return 0;
        tot += stage_mem[j];
    }
    const int extra = total_layers - n_stages;
    std::vector<double> frac(n_stages);
    int given = 0;
    for (int j = 0; j < n_stages; ++j) {
        const double ideal = extra * stage_mem[j] / tot;
        const double fl = std::floor(ideal);
        layers_out[j] = 1 + (int)fl;
        frac[j] = ideal - fl;
        given += layers_out[j];
    }
    for (int rest = total_layers - given; rest > 0; --rest) {      // largest fractional part first, first stage on ties
        int pick = 0;
        for (int j = 1; j < n_stages; ++j)
            if (frac[j] > frac[pick]) pick = j;
        layers_out[pick] += 1;
        frac[pick] = -1.0;
    }
    return 1;
} catch (...) {      // no exception (an allocation failure) may cross the C boundary
    return 0;
}

}  // extern "C"
