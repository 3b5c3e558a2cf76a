// Host-side scalar pieces of DeCo-SGD: the DeCo rule (Algorithm 3), its objective phi, the
// iteration-time model of Section 4 (Theorem 3 and the recurrence it is proved from) and the
// look-up-table implementation of Section 4.5.  No device code.
#include <cmath>
#include <cstdint>
#include <new>
#include <vector>

#include "ddef.h"

namespace {

bool positive_finite(double v) { return std::isfinite(v) && v > 0.0; }

// Largest ratio that keeps the transfer of one message hidden: behind tau compute slots
// minus the latency, and within one compute slot; never more than the whole gradient.
double hidden_ratio(double tau, double sent_per_second, double b_s, double t_comp_s) {
    double r = (tau * t_comp_s - b_s) * sent_per_second;
    const double one_slot = t_comp_s * sent_per_second;
    if (one_slot < r) r = one_slot;
    return r > 1.0 ? 1.0 : r;
}

}  // namespace

struct ddef_lut {
    double a_min = 0, a_max = 0, step = 0;
    double v_g = 0, b = 0, t_comp = 0;
    std::vector<uint32_t> tau;
    std::vector<double> delta;
    std::vector<char> valid;
};

extern "C" {

double ddef_phi(double delta, double tau) {
    if (!(delta > 0.0) || !(delta <= 1.0) || !(tau >= 0.0)) return NAN;
    return (1.0 - delta) / (delta * std::pow(1.0 - delta / 2.0, tau));
}

double ddef_phi_prime(double delta, double tau) {
    const double phi = ddef_phi(delta, tau);
    return phi / delta;                                   // NaN stays NaN outside the domain
}

static int deco_scan(bool non_iid, double v_g_bits, double a_bps, double b_s, double t_comp_s, uint32_t* tau,
                     double* delta) {
    if (!tau || !delta) return DDEF_EINVAL;
    if (!positive_finite(v_g_bits) || !positive_finite(a_bps) || !positive_finite(t_comp_s)) return DDEF_EINVAL;
    if (!std::isfinite(b_s) || b_s < 0.0) return DDEF_EINVAL;
    const double sent_per_second = a_bps / v_g_bits;      // fraction of the gradient per second
    const double first = std::ceil((b_s + 1.0 / sent_per_second) / t_comp_s);
    const double last = std::ceil(b_s / t_comp_s);
    if (first > 4.0e9) return DDEF_EINVAL;
    bool have = false;
    double phi_min = INFINITY;
    for (double cand = first; cand >= last; cand -= 1.0) {
        const double ratio = hidden_ratio(cand, sent_per_second, b_s, t_comp_s);
        if (!(ratio > 0.0)) continue;                     // nothing can be sent in time: no phi
        const double phi = non_iid ? ddef_phi_prime(ratio, cand) : ddef_phi(ratio, cand);
        if (phi <= phi_min) { phi_min = phi; *tau = (uint32_t)cand; *delta = ratio; have = true; }
    }
    return have ? DDEF_OK : DDEF_EINVAL;
}

int ddef_deco(double v_g_bits, double a_bps, double b_s, double t_comp_s, uint32_t* tau, double* delta) {
    return deco_scan(false, v_g_bits, a_bps, b_s, t_comp_s, tau, delta);
}

int ddef_deco_noniid(double v_g_bits, double a_bps, double b_s, double t_comp_s, uint32_t* tau, double* delta) {
    return deco_scan(true, v_g_bits, a_bps, b_s, t_comp_s, tau, delta);
}

int ddef_corner_compression_only(double v_g_bits, double a_bps, double t_comp_s, double* delta) {
    if (!delta) return DDEF_EINVAL;
    if (!positive_finite(v_g_bits) || !positive_finite(a_bps) || !positive_finite(t_comp_s)) return DDEF_EINVAL;
    const double one_slot = t_comp_s * a_bps / v_g_bits;     // share of the gradient one T_comp carries
    *delta = one_slot > 1.0 ? 1.0 : one_slot;
    return DDEF_OK;
}

int ddef_corner_delay_only(double v_g_bits, double a_bps, double b_s, double t_comp_s, uint32_t tau_max,
                           uint32_t* tau) {
    if (!tau) return DDEF_EINVAL;
    if (!positive_finite(v_g_bits) || !positive_finite(a_bps) || !positive_finite(t_comp_s)) return DDEF_EINVAL;
    if (!std::isfinite(b_s) || b_s < 0.0) return DDEF_EINVAL;
    const double slots = std::ceil((b_s + v_g_bits / a_bps) / t_comp_s);     // where Algorithm 3's scan starts
    *tau = slots > (double)tau_max ? tau_max : (uint32_t)slots;
    return DDEF_OK;
}

double ddef_t_avg_model(uint32_t tau, double delta, double v_g_bits, double a_bps, double b_s, double t_comp_s) {
    const double transfer = delta * v_g_bits / a_bps;
    double t = (t_comp_s + b_s + transfer) / ((double)tau + 1.0);
    if (transfer > t) t = transfer;
    if (t_comp_s > t) t = t_comp_s;
    return t;
}

double ddef_t_avg_simulate(uint32_t tau, double delta, double v_g_bits, double a_bps, double b_s,
                           double t_comp_s, uint64_t iterations) {
    if (iterations == 0) return NAN;
    // done_compute[k], done_send[k]: end of the k-th computation / of putting message k on the
    // wire; message k arrives b later.  Computation k+1 needs computation k and the arrival of
    // message k - tau (messages with index <= 0 count as arrived at time 0).
    const double transfer = delta * v_g_bits / a_bps;
    std::vector<double> done_compute(iterations + 1, 0.0), done_send(iterations + 1, 0.0);
    for (uint64_t k = 0; k < iterations; ++k) {
        double wait_for = done_compute[k];
        if (k > tau) {
            const double arrived = done_send[k - tau] + b_s;
            if (arrived > wait_for) wait_for = arrived;
        }
        done_compute[k + 1] = wait_for + t_comp_s;
        const double wire_free = done_send[k] > done_compute[k + 1] ? done_send[k] : done_compute[k + 1];
        done_send[k + 1] = wire_free + transfer;
    }
    return (done_send[iterations] + b_s) / (double)iterations;
}

int ddef_lut_build(double v_g_bits, double a_min_bps, double a_max_bps, uint32_t points, double b_s,
                   double t_comp_s, ddef_lut** out) {
    if (!out) return DDEF_EINVAL;
    *out = nullptr;
    if (!positive_finite(v_g_bits) || !positive_finite(a_min_bps) || !positive_finite(a_max_bps) ||
        !positive_finite(t_comp_s) || !std::isfinite(b_s) || b_s < 0.0)
        return DDEF_EINVAL;
    if (points < 2 || points > (1u << 20) || !(a_max_bps > a_min_bps)) return DDEF_EINVAL;
    ddef_lut* lut = new (std::nothrow) ddef_lut;
    if (!lut) return DDEF_ENOMEM;
    lut->a_min = a_min_bps; lut->a_max = a_max_bps;
    lut->step = (a_max_bps - a_min_bps) / (double)(points - 1);
    lut->v_g = v_g_bits; lut->b = b_s; lut->t_comp = t_comp_s;
    lut->tau.assign(points, 0u); lut->delta.assign(points, 0.0); lut->valid.assign(points, 0);
    for (uint32_t i = 0; i < points; ++i) {
        const double a = i + 1 == points ? a_max_bps : a_min_bps + lut->step * (double)i;
        uint32_t tau = 0;
        double delta = 0.0;
        if (ddef_deco(v_g_bits, a, b_s, t_comp_s, &tau, &delta) == DDEF_OK) {
            lut->tau[i] = tau; lut->delta[i] = delta; lut->valid[i] = 1;
        }
    }
    *out = lut;
    return DDEF_OK;
}

int ddef_lut_query(const ddef_lut* lut, double a_bps, uint32_t* tau, double* delta, int* from_table) {
    if (!lut || !tau || !delta || !positive_finite(a_bps)) return DDEF_EINVAL;
    if (a_bps >= lut->a_min && a_bps <= lut->a_max) {
        size_t i = (size_t)std::floor((a_bps - lut->a_min) / lut->step + 0.5);     // nearest sample point
        if (i >= lut->tau.size()) i = lut->tau.size() - 1;
        if (lut->valid[i]) {
            *tau = lut->tau[i]; *delta = lut->delta[i];
            if (from_table) *from_table = 1;
            return DDEF_OK;
        }
    }
    if (from_table) *from_table = 0;
    return ddef_deco(lut->v_g, a_bps, lut->b, lut->t_comp, tau, delta);   // outside the table: decide online
}

int ddef_lut_destroy(ddef_lut* lut) {
    if (!lut) return DDEF_EINVAL;
    delete lut;
    return DDEF_OK;
}

}  // extern "C"
