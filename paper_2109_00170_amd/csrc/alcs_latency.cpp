// Host side of the latency model of arXiv 2109.00170, Section 3.3: a layer's run time as the
// piecewise-linear interpolant of a few (non-zero weights, measured time) pairs, Eqs. (4)-(6),
// and the network's run time as a constant plus the sum over its layers, Eq. (2).  The pairs are
// measured with alcs_sparse_conv_timed; nothing here touches the GPU.
#include <cmath>

#include "alcs.h"

namespace {

bool table_ok(const double *k, const double *t, int n) {
    if (!k || !t || n < 2) return false;
    for (int i = 0; i < n; ++i)
        if (!std::isfinite(k[i]) || !std::isfinite(t[i])) return false;
    for (int i = 0; i + 1 < n; ++i)
        if (!(k[i] < k[i + 1])) return false;
    return true;
}

// The sum of Eq. (4) telescopes: every interval that lies wholly below s adds t[i+1] - t[i], the
// interval that holds s adds its slope times the part below s, so only that interval is looked at.
double interpolate(const double *k, const double *t, int n, double s) {
    if (!(s > k[0])) return t[0];
    if (s >= k[n - 1]) return t[n - 1];
    int lo = 0, hi = n - 1;  // k[lo] <= s < k[hi]
    while (hi - lo > 1) {
        const int mid = (lo + hi) / 2;
        if (s >= k[mid]) lo = mid;
        else hi = mid;
    }
    const double w = (s - k[lo]) / (k[hi] - k[lo]);
    return t[lo] + w * (t[hi] - t[lo]);
}

}  // namespace

extern "C" int alcs_latency_estimate(const double *k_host, const double *t_host, int n, double s,
                                      double *estimate_out) {
    if (!estimate_out || !table_ok(k_host, t_host, n) || std::isnan(s)) return ALCS_E_INVALID_ARG;
    *estimate_out = interpolate(k_host, t_host, n, s);
    return ALCS_OK;
}

extern "C" int alcs_network_latency(double tau, const double *k_host, const double *t_host,
                                     const int *n_host, int L, const double *s_host, double *latency_out) {
    if (!latency_out || L < 0 || !std::isfinite(tau)) return ALCS_E_INVALID_ARG;
    if (L > 0 && (!n_host || !s_host)) return ALCS_E_INVALID_ARG;
    long long first = 0;
    for (int l = 0; l < L; ++l) {
        if (n_host[l] < 2 || !table_ok(k_host + first, t_host + first, n_host[l]) || std::isnan(s_host[l]))
            return ALCS_E_INVALID_ARG;
        first += n_host[l];
    }
    double total = tau;
    first = 0;
    for (int l = 0; l < L; ++l) {
        total += interpolate(k_host + first, t_host + first, n_host[l], s_host[l]);
        first += n_host[l];
    }
    *latency_out = total;
    return ALCS_OK;
}
