// Host-side planning helpers of the prefill path (no device code): the batching dynamic program of Sec. 5.3
// (requests sorted by length, elastic instances sorted; f[i][k] = cheapest input latency of the first i requests
// on the first k instances; interval sums from prefix arrays; last split points recorded for the backtrack) and the
// least-squares fit of the iteration-time model of Sec. 5.5 (alpha + beta * sum(len) + gamma * sum(len^2)).
#include <math.h>

#include <vector>

#include "esp_common.h"

namespace esp {

// Solves min || A x - y || for A = [1, s1, s2] (n x 3) by Householder QR on column-scaled A.  A column whose
// remaining part is negligible (e.g. an all-zero or duplicate column) gets coefficient 0.
static bool lstsq3(const double* s1, const double* s2, const double* y, const double* w, int n, double x[3]) {
    std::vector<long double> a((size_t)n * 3), b(n);
    long double scale[3] = {1.0L, 0.0L, 0.0L};
    for (int i = 0; i < n; ++i) {
        scale[1] = fmaxl(scale[1], fabsl((long double)s1[i]));
        scale[2] = fmaxl(scale[2], fabsl((long double)s2[i]));
    }
    for (int c = 1; c < 3; ++c) if (scale[c] == 0.0L) scale[c] = 1.0L;
    for (int i = 0; i < n; ++i) {
        const long double wi = w ? (long double)w[i] : 1.0L;    // the sample's equation times its weight
        a[(size_t)i * 3 + 0] = wi;
        a[(size_t)i * 3 + 1] = wi * (long double)s1[i] / scale[1];
        a[(size_t)i * 3 + 2] = wi * (long double)s2[i] / scale[2];
        b[i] = wi * (long double)y[i];
    }
    bool live[3] = {true, true, true};
    long double rdiag[3] = {0, 0, 0};
    for (int c = 0; c < 3; ++c) {
        long double norm = 0;
        for (int i = c; i < n; ++i) norm += a[(size_t)i * 3 + c] * a[(size_t)i * 3 + c];
        norm = sqrtl(norm);
        long double full = 0;
        for (int i = 0; i < n; ++i) full += a[(size_t)i * 3 + c] * a[(size_t)i * 3 + c];
        if (c >= n || norm <= 1e-13L * sqrtl(full) || norm == 0.0L) { live[c] = false; continue; }
        const long double alpha = a[(size_t)c * 3 + c] > 0 ? -norm : norm;
        std::vector<long double> v(n, 0.0L);
        for (int i = c; i < n; ++i) v[i] = a[(size_t)i * 3 + c];
        v[c] -= alpha;
        long double vv = 0;
        for (int i = c; i < n; ++i) vv += v[i] * v[i];
        if (vv == 0.0L) { live[c] = false; continue; }
        for (int cc = c; cc < 3; ++cc) {
            long double dot = 0;
            for (int i = c; i < n; ++i) dot += v[i] * a[(size_t)i * 3 + cc];
            const long double f = 2.0L * dot / vv;
            for (int i = c; i < n; ++i) a[(size_t)i * 3 + cc] -= f * v[i];
        }
        long double dot = 0;
        for (int i = c; i < n; ++i) dot += v[i] * b[i];
        const long double f = 2.0L * dot / vv;
        for (int i = c; i < n; ++i) b[i] -= f * v[i];
        rdiag[c] = a[(size_t)c * 3 + c];
    }
    long double sol[3] = {0, 0, 0};
    for (int c = 2; c >= 0; --c) {
        if (!live[c]) continue;
        long double r = b[c];
        for (int cc = c + 1; cc < 3; ++cc) if (live[cc]) r -= a[(size_t)c * 3 + cc] * sol[cc];
        sol[c] = r / rdiag[c];
    }
    for (int c = 0; c < 3; ++c) x[c] = (double)(sol[c] / scale[c]);
    return true;
}

}  // namespace esp

using namespace esp;

extern "C" {

esp_status esp_fit_prefill_model(const double* sum_len, const double* sum_len_sq, const double* seconds,
                                 const double* weights, int32_t n, double* coef) {
    if (!sum_len || !sum_len_sq || !seconds || !coef) return fail(ESP_ERR_INVALID_ARG, "fit: null argument");
    if (n < 3) return fail(ESP_ERR_INVALID_ARG, "fit: needs at least 3 samples, got %d", n);
    for (int i = 0; i < n; ++i)
        if (!isfinite(sum_len[i]) || !isfinite(sum_len_sq[i]) || !isfinite(seconds[i]))
            return fail(ESP_ERR_INVALID_ARG, "fit: sample %d is not finite", i);
    if (weights)
        for (int i = 0; i < n; ++i)
            if (!isfinite(weights[i]) || weights[i] < 0.0) return fail(ESP_ERR_INVALID_ARG, "fit: weight %d is negative or not finite", i);
    lstsq3(sum_len, sum_len_sq, seconds, weights, n, coef);
    return ESP_OK;
}

}  // extern "C"

// The dynamic program.  `monotone`: the search for the last batch of (first i requests, first k instances) starts at
// the split points of its neighbours, split_req[i][k-1] and split_ins[i-1][k] (the lower halves of the two
// inequalities of Eq. 6, the halves that are known when the table is filled row by row).
static esp_status plan_batches(const int64_t* req_len, int32_t n_req, const int64_t* free_slots, int32_t n_inst,
                               const double* coefs, int32_t* req_cuts, int32_t* inst_cuts, int32_t* n_batches,
                               double* cost, int32_t* split_req, int32_t* split_ins, bool monotone) {
    if (!req_len || !free_slots || !coefs || !req_cuts || !inst_cuts || !n_batches || !cost)
        return fail(ESP_ERR_INVALID_ARG, "plan: null argument");
    if (n_req < 1 || n_inst < 1) return fail(ESP_ERR_INVALID_ARG, "plan: needs at least one request and one instance");
    for (int i = 0; i < n_req; ++i) {
        if (req_len[i] < 1) return fail(ESP_ERR_INVALID_ARG, "plan: request %d has length %lld", i, (long long)req_len[i]);
        if (i > 0 && req_len[i] > req_len[i - 1]) return fail(ESP_ERR_INVALID_ARG, "plan: requests must be sorted by length, longest first");
    }
    for (int k = 0; k < n_inst; ++k)
        if (free_slots[k] < 0) return fail(ESP_ERR_INVALID_ARG, "plan: instance %d has negative free slots", k);
    const int n = n_req, m = n_inst;
    // prefix sums: tokens, squared tokens, reciprocal lengths of requests; free slots of instances
    std::vector<double> s1(n + 1, 0.0), s2(n + 1, 0.0), sinv(n + 1, 0.0);
    std::vector<long double> d(n + 1, 0.0L), v(m + 1, 0.0L);
    for (int i = 0; i < n; ++i) {
        const double x = (double)req_len[i];
        s1[i + 1] = s1[i] + x; s2[i + 1] = s2[i] + x * x; sinv[i + 1] = sinv[i] + 1.0 / x;
        d[i + 1] = d[i] + (long double)req_len[i];
    }
    for (int k = 0; k < m; ++k) v[k + 1] = v[k] + (long double)free_slots[k];
    const double inf = INFINITY;
    const size_t W = (size_t)m + 1;
    std::vector<double> f((size_t)(n + 1) * W, inf);
    std::vector<int32_t> sr((size_t)(n + 1) * W, -1), si((size_t)(n + 1) * W, -1);
    f[0] = 0.0;
    for (int i = 1; i <= n; ++i)
        for (int k = 1; k <= m; ++k) {
            double best = inf; int bj = -1, bl = -1;
            int j0 = 0, l0 = 0;
            if (monotone) {
                if (k > 1 && sr[(size_t)i * W + k - 1] >= 0) j0 = sr[(size_t)i * W + k - 1];
                if (i > 1 && si[(size_t)(i - 1) * W + k] >= 0) l0 = si[(size_t)(i - 1) * W + k];
            }
            for (int pass = 0; pass < 2 && best == inf; ++pass) {
                if (pass == 1) {                        // nothing fits inside the bounds: search the whole range
                    if (j0 == 0 && l0 == 0) break;
                    j0 = 0; l0 = 0;
                }
                for (int j = j0; j < i; ++j)            // the last batch holds requests j .. i-1
                    for (int l = l0; l < k; ++l) {      // on instances l .. k-1
                        const double prev = f[(size_t)j * W + l];
                        if (prev == inf) continue;
                        if (d[i] - d[j] > v[k] - v[l]) continue;
                        const double* c = coefs + 3 * (size_t)(k - l - 1);
                        const double t = c[0] + c[1] * (s1[i] - s1[j]) + c[2] * (s2[i] - s2[j]);
                        const double total = prev + t * (sinv[i] - sinv[j]);
                        if (total < best) { best = total; bj = j; bl = l; }
                    }
            }
            f[(size_t)i * W + k] = best; sr[(size_t)i * W + k] = bj; si[(size_t)i * W + k] = bl;
        }
    if (split_req) for (size_t t = 0; t < sr.size(); ++t) split_req[t] = sr[t];
    if (split_ins) for (size_t t = 0; t < si.size(); ++t) split_ins[t] = si[t];
    int bk = -1; double best = inf;
    for (int k = 1; k <= m; ++k)
        if (f[(size_t)n * W + k] < best) { best = f[(size_t)n * W + k]; bk = k; }
    *cost = best;
    *n_batches = 0;
    if (bk < 0) return ESP_OK;                          // nothing fits: no plan, cost = +inf
    int nb = 0;
    for (int i = n, k = bk; i > 0;) {                   // backtrack, last batch first
        req_cuts[nb] = i; inst_cuts[nb] = k; ++nb;
        const int j = sr[(size_t)i * W + k], l = si[(size_t)i * W + k];
        i = j; k = l;
    }
    for (int a = 0, b = nb - 1; a < b; ++a, --b) {
        int t = req_cuts[a]; req_cuts[a] = req_cuts[b]; req_cuts[b] = t;
        t = inst_cuts[a]; inst_cuts[a] = inst_cuts[b]; inst_cuts[b] = t;
    }
    *n_batches = nb;
    return ESP_OK;
}

extern "C" {

esp_status esp_plan_prefill_batches(const int64_t* req_len, int32_t n_req, const int64_t* free_slots, int32_t n_inst,
                                    const double* coefs, int32_t* req_cuts, int32_t* inst_cuts, int32_t* n_batches,
                                    double* cost, int32_t* split_req, int32_t* split_ins) {
    return plan_batches(req_len, n_req, free_slots, n_inst, coefs, req_cuts, inst_cuts, n_batches, cost, split_req, split_ins, false);
}

esp_status esp_plan_prefill_batches_monotone(const int64_t* req_len, int32_t n_req, const int64_t* free_slots, int32_t n_inst,
                                             const double* coefs, int32_t* req_cuts, int32_t* inst_cuts, int32_t* n_batches,
                                             double* cost, int32_t* split_req, int32_t* split_ins) {
    return plan_batches(req_len, n_req, free_slots, n_inst, coefs, req_cuts, inst_cuts, n_batches, cost, split_req, split_ins, true);
}

}  // extern "C"
