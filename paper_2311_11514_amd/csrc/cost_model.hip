// The paper's inference cost model (Table 1; Appendix "Modeling the Generative Inference Cost", Eqs. 3-6) as host
// functions of the library: plain arithmetic, no device work.  A scheduler evaluates these for every candidate
// stage; the measured rates of this machine (bench.py) are what goes in for m_d and c_d.
#include <cmath>
#include <limits>

#include "../../include/hexgen.h"

namespace {
const double kNaN = std::numeric_limits<double>::quiet_NaN();
bool bad_task(int hidden, int bytes, int batch, int s_in, int s_out) {
    return hidden <= 0 || bytes <= 0 || batch <= 0 || s_in < 0 || s_out < 0;
}
double vmax_inv(const double *v, int n) {        // max_d (1 / v_d) = 1 / min_d v_d, NaN for a non-positive rate
    double lo = v[0];
    for (int i = 0; i < n; ++i) {
        if (!(v[i] > 0.0)) return kNaN;
        if (v[i] < lo) lo = v[i];
    }
    return 1.0 / lo;
}
}  // namespace

extern "C" {

double hexgen_cost_comp_prefill(int hidden, double params_factor, int bytes_per_elem, int batch, int s_in, int s_out,
                                int layers, int n_dev, const double *m_d, const double *c_d) {
    (void)m_d;
    if (bad_task(hidden, bytes_per_elem, batch, s_in, s_out) || layers < 0 || n_dev <= 0 || !c_d || !(params_factor > 0.0))
        return kNaN;
    const double H2 = (double)hidden * hidden;
    return 2.0 * params_factor * H2 * batch * s_in / n_dev * vmax_inv(c_d, n_dev) * layers;
}

double hexgen_cost_comp_decode(int hidden, double params_factor, int bytes_per_elem, int batch, int s_in, int s_out,
                               int layers, int n_dev, const double *m_d, const double *c_d) {
    if (bad_task(hidden, bytes_per_elem, batch, s_in, s_out) || layers < 0 || n_dev <= 0 || !m_d || !c_d ||
        !(params_factor > 0.0))
        return kNaN;
    const double H2 = (double)hidden * hidden;
    const double scan = params_factor * H2 * bytes_per_elem / n_dev * vmax_inv(m_d, n_dev);
    const double flops = 2.0 * params_factor * H2 * batch / n_dev * vmax_inv(c_d, n_dev);
    return (scan + flops) * layers * s_out;
}

double hexgen_cost_comp(int hidden, double params_factor, int bytes_per_elem, int batch, int s_in, int s_out, int layers,
                        int n_dev, const double *m_d, const double *c_d) {
    return hexgen_cost_comp_prefill(hidden, params_factor, bytes_per_elem, batch, s_in, s_out, layers, n_dev, m_d, c_d) +
           hexgen_cost_comp_decode(hidden, params_factor, bytes_per_elem, batch, s_in, s_out, layers, n_dev, m_d, c_d);
}

double hexgen_cost_comm_tp(int hidden, int bytes_per_elem, int batch, int s_in, int s_out, int layers, int n_dev,
                           const double *alpha, const double *beta) {
    if (bad_task(hidden, bytes_per_elem, batch, s_in, s_out) || layers < 0 || n_dev <= 0) return kNaN;
    if (n_dev == 1) return 0.0;
    if (!alpha || !beta) return kNaN;
    const double row = (double)batch * hidden * bytes_per_elem;
    double worst_prefill = 0.0, worst_step = 0.0;
    for (int d = 0; d < n_dev; ++d) {
        double sp = 0.0, ss = 0.0;
        for (int e = 0; e < n_dev; ++e) {
            if (e == d) continue;
            const double a = alpha[d * n_dev + e], bw = beta[d * n_dev + e];
            if (!(bw > 0.0) || !(a >= 0.0)) return kNaN;
            sp += a + row * s_in / (n_dev * bw);
            ss += a + row / (n_dev * bw);
        }
        worst_prefill = std::fmax(worst_prefill, sp);
        worst_step = std::fmax(worst_step, ss);
    }
    return worst_prefill * 4.0 * layers + worst_step * 4.0 * s_out * layers;
}

double hexgen_cost_comm_pp(int hidden, int bytes_per_elem, int batch, int s_in, int s_out, int n_from, int n_to,
                           const double *alpha, const double *beta) {
    if (bad_task(hidden, bytes_per_elem, batch, s_in, s_out) || n_from <= 0 || n_to <= 0 || !alpha || !beta) return kNaN;
    const double row = (double)batch * hidden * bytes_per_elem;
    double best_prefill = INFINITY, best_step = INFINITY;
    for (int i = 0; i < n_from * n_to; ++i) {
        if (!(beta[i] > 0.0) || !(alpha[i] >= 0.0)) return kNaN;
        best_prefill = std::fmin(best_prefill, alpha[i] + row * s_in / beta[i]);
        best_step = std::fmin(best_step, alpha[i] + row / beta[i]);
    }
    return best_prefill + best_step * s_out;
}

double hexgen_cost_mem(int hidden, double params_factor, int bytes_per_elem, int batch, int s_in, int s_out, int layers,
                       int n_dev) {
    if (bad_task(hidden, bytes_per_elem, batch, s_in, s_out) || layers < 0 || n_dev <= 0 || !(params_factor > 0.0)) return kNaN;
    const double H = hidden, s = (double)s_in + s_out;
    return (params_factor * H * H * bytes_per_elem / n_dev + 2.0 * batch * s * H * bytes_per_elem / n_dev) * layers +
           4.0 * batch * s * H * bytes_per_elem;
}

}  // extern "C"
