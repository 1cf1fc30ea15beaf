/*
 * esp_oracle.c -- TEST INFRASTRUCTURE, NOT PRODUCT CODE.
 *
 * A plain, slow, fp64 CPU statement of what one GPU's share of elastic
 * sequence-parallel (ESP) attention computes.  Only tests, the smoke check and
 * the benchmark's cpu_baseline leg may call it.  It shares no code, header or
 * table with the HIP path and must never be reachable from the product path.
 *
 * What the method computes (LoongServe, arXiv 2404.09526):
 *   - Sec. 2.3 / Fig. 1: in sequence-parallel prefill every instance attends
 *     its local queries q_i to each key-value segment kv_j that passes by and,
 *     after all rounds, forms the final output.  One (q_i, kv_j) meeting is a
 *     "partial attention": softmax attention restricted to the keys of that one
 *     segment, causal by the tokens' global positions (striped permutation).
 *   - Sec. 4.2 / Fig. 8: in (multi-master) distributed decoding each instance
 *     computes attention of a request's single query token against the
 *     key-value rows that this instance holds, and the results are sent back
 *     and combined at the master.
 *   - Sec. 6: the KV cache pool is paged at the granularity of one token, so a
 *     request's rows sit at arbitrary slots; the ESP kernels keep the accuracy
 *     of the original attention.  Hence the result of partial attention
 *     followed by the combination is exactly softmax attention, and this file
 *     writes out that definition: two passes, no blocking, no online rescaling.
 *   - Sec. 4.1 / Fig. 7: during prefill, instances of the shrunken group save
 *     selected key-value rows into pool slots named by the scaling plan
 *     (oracle_kv_append: a pure copy of 16-bit patterns).
 *
 * Readings where the paper is silent (softmax scale is an argument; LSE is the
 * natural log of the sum of exponentials of the scaled scores; a key is
 * visible iff kv_pos <= q_pos; an empty visible set gives O = 0, LSE = -inf;
 * query head h reads KV head h / (Hq/Hkv); the combination is the
 * log-sum-exp weighted average) are listed in the design document.
 *
 * All inputs are bf16 bit patterns (uint16) unless stated; all arithmetic is
 * double precision on the exact values of those inputs; outputs are double.
 */
#include <math.h>
#ifdef _OPENMP
#include <omp.h>
#endif
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

static double bf16_bits_to_double(uint16_t bits)
{
    uint32_t u = ((uint32_t)bits) << 16; /* bf16 is the top half of an IEEE float */
    float f;
    memcpy(&f, &u, sizeof f);
    return (double)f;
}

/*
 * Softmax attention of ONE query vector (one row, one head) over a set of
 * n key/value rows.  Row j of the set is row rows[j] of k/v when rows != NULL,
 * else row lo + j.  k and v are [*, Hkv, D]; kvh selects the KV head.
 * pos (nullable) gives the global position of each k/v row (indexed like k);
 * with causal != 0 only rows with pos <= qpos are visible.
 * Writes O[D] and *lse.  s is scratch for n doubles.
 */
static void attend_one(const uint16_t *qvec, const uint16_t *k, const uint16_t *v,
                       int64_t Hkv, int64_t D, int64_t kvh,
                       const int32_t *rows, int64_t lo, int64_t n,
                       const int32_t *pos, int32_t qpos, int causal, double scale,
                       double *O, double *lse, double *s)
{
    double qd[1024];
    for (int64_t d = 0; d < D; ++d) qd[d] = bf16_bits_to_double(qvec[d]);

    /* pass 1: scaled scores of the visible keys, and their maximum */
    double m = -INFINITY;
    int64_t nvis = 0;
    for (int64_t j = 0; j < n; ++j) {
        int64_t r = rows ? (int64_t)rows[j] : lo + j;
        if (causal && pos[r] > qpos) { s[j] = -INFINITY; continue; }
        const uint16_t *kr = k + (r * Hkv + kvh) * D;
        double dot = 0.0;
        for (int64_t d = 0; d < D; ++d) dot += qd[d] * bf16_bits_to_double(kr[d]);
        s[j] = scale * dot;
        if (s[j] > m) m = s[j];
        ++nvis;
    }
    for (int64_t d = 0; d < D; ++d) O[d] = 0.0;
    if (nvis == 0) { *lse = -INFINITY; return; }

    /* pass 2: the normaliser */
    double l = 0.0;
    for (int64_t j = 0; j < n; ++j)
        if (s[j] != -INFINITY) l += exp(s[j] - m);
    double L = m + log(l);
    *lse = L;

    /* pass 3: probability-weighted sum of the value rows */
    for (int64_t j = 0; j < n; ++j) {
        if (s[j] == -INFINITY) continue;
        int64_t r = rows ? (int64_t)rows[j] : lo + j;
        const uint16_t *vr = v + (r * Hkv + kvh) * D;
        double p = exp(s[j] - L);
        for (int64_t d = 0; d < D; ++d) O[d] += p * bf16_bits_to_double(vr[d]);
    }
}

/*
 * Partial attention (Sec. 2.3, Fig. 1; kernel remarks in Sec. 6) for a list of
 * sampled (query row, query head) pairs.  Sample i uses query row s_row[i],
 * head s_head[i] and the key rows [s_kv_lo[i], s_kv_hi[i]) of the shard (the
 * rows of the request that the query belongs to).
 *   q [Tq,Hq,D], k/v [Tkv,Hkv,D] bf16 bits; q_pos [Tq], kv_pos [Tkv] int32.
 *   O_out [n,D], LSE_out [n] double.
 * Returns 0, or -1 on bad arguments / allocation failure.
 */
int oracle_partial_attn(const uint16_t *q, const uint16_t *k, const uint16_t *v,
                        const int32_t *q_pos, const int32_t *kv_pos,
                        int64_t Hq, int64_t Hkv, int64_t D, double scale, int causal,
                        int64_t n, const int64_t *s_row, const int64_t *s_head,
                        const int64_t *s_kv_lo, const int64_t *s_kv_hi,
                        double *O_out, double *LSE_out)
{
    if (D > 1024 || Hkv <= 0 || Hq % Hkv != 0) return -1;
    int64_t G = Hq / Hkv;
    int64_t max_n = 1;
    for (int64_t i = 0; i < n; ++i)
        if (s_kv_hi[i] - s_kv_lo[i] > max_n) max_n = s_kv_hi[i] - s_kv_lo[i];
    int fail = 0;
#pragma omp parallel
    {
        double *s = (double *)malloc(sizeof(double) * (size_t)max_n);
        if (!s) {
#pragma omp atomic write
            fail = 1;
        }
#pragma omp for schedule(dynamic, 1)
        for (int64_t i = 0; i < n; ++i) {
            if (!s) continue;
            int64_t r = s_row[i], h = s_head[i];
            attend_one(q + (r * Hq + h) * D, k, v, Hkv, D, h / G,
                       NULL, s_kv_lo[i], s_kv_hi[i] - s_kv_lo[i],
                       kv_pos, causal ? q_pos[r] : 0, causal, scale,
                       O_out + i * D, LSE_out + i, s);
        }
        free(s);
    }
    return fail ? -1 : 0;
}

/*
 * Decode partial attention (Sec. 4.2, Fig. 8; token-granular pool of Sec. 6)
 * for sampled (request, head) pairs: one query token per request against the
 * pool rows slot_idx[seq_offsets[b] .. seq_offsets[b+1]) that this instance
 * holds for request b.  No mask: every resident token precedes the query.
 *   q [B,Hq,D]; k_pool/v_pool [S,Hkv,D] bf16 bits.
 *   O_out [n,D], LSE_out [n] double.
 */
int oracle_partial_attn_decode(const uint16_t *q, const uint16_t *k_pool, const uint16_t *v_pool,
                               const int32_t *slot_idx, const int32_t *seq_offsets,
                               int64_t Hq, int64_t Hkv, int64_t D, double scale,
                               int64_t n, const int64_t *s_req, const int64_t *s_head,
                               double *O_out, double *LSE_out)
{
    if (D > 1024 || Hkv <= 0 || Hq % Hkv != 0) return -1;
    int64_t G = Hq / Hkv;
    int64_t max_n = 1;
    for (int64_t i = 0; i < n; ++i) {
        int64_t len = seq_offsets[s_req[i] + 1] - seq_offsets[s_req[i]];
        if (len > max_n) max_n = len;
    }
    int fail = 0;
#pragma omp parallel
    {
        double *s = (double *)malloc(sizeof(double) * (size_t)max_n);
        if (!s) {
#pragma omp atomic write
            fail = 1;
        }
#pragma omp for schedule(dynamic, 1)
        for (int64_t i = 0; i < n; ++i) {
            if (!s) continue;
            int64_t b = s_req[i], h = s_head[i];
            int64_t lo = seq_offsets[b], len = seq_offsets[b + 1] - lo;
            attend_one(q + (b * Hq + h) * D, k_pool, v_pool, Hkv, D, h / G,
                       slot_idx + lo, 0, len, NULL, 0, 0, scale,
                       O_out + i * D, LSE_out + i, s);
        }
        free(s);
    }
    return fail ? -1 : 0;
}

/*
 * Combination of P partial results of the same n (row, head) pairs into the
 * result over the union of their key sets ("generate the final output",
 * Sec. 2.3; "send results back to the master", Sec. 4.2).  With
 * m = max_p LSE_p and w_p = exp(LSE_p - m):
 *   O = sum_p w_p O_p / sum_p w_p,   LSE = m + ln sum_p w_p.
 * A partial with LSE = -inf (empty key set) has weight 0; if all are -inf the
 * result is O = 0, LSE = -inf.
 *   O_parts [P,n,D], LSE_parts [P,n], O_out [n,D], LSE_out [n]; all double.
 */
int oracle_merge_partials(const double *O_parts, const double *LSE_parts,
                          int64_t P, int64_t n, int64_t D,
                          double *O_out, double *LSE_out)
{
    for (int64_t i = 0; i < n; ++i) {
        double m = -INFINITY;
        for (int64_t p = 0; p < P; ++p)
            if (LSE_parts[p * n + i] > m) m = LSE_parts[p * n + i];
        for (int64_t d = 0; d < D; ++d) O_out[i * D + d] = 0.0;
        if (m == -INFINITY) { LSE_out[i] = -INFINITY; continue; }
        double wsum = 0.0;
        for (int64_t p = 0; p < P; ++p) {
            double L = LSE_parts[p * n + i];
            if (L == -INFINITY) continue;
            double w = exp(L - m);
            wsum += w;
            for (int64_t d = 0; d < D; ++d) O_out[i * D + d] += w * O_parts[(p * n + i) * D + d];
        }
        for (int64_t d = 0; d < D; ++d) O_out[i * D + d] /= wsum;
        LSE_out[i] = m + log(wsum);
    }
    return 0;
}

/*
 * KV append / selective retention (Sec. 4.1, Fig. 7; Sec. 4.2 "saves
 * key-value tensors into its local pool"): row t of k and v is copied, bit for
 * bit, to slot slot_idx[t] of the pools; a negative slot means "do not keep".
 *   k, v [T,row_elems]; pools [S,row_elems]; 16-bit patterns.
 * Returns 0, or -1 if a slot is >= S.
 */
int oracle_kv_append(const uint16_t *k, const uint16_t *v, const int32_t *slot_idx,
                     int64_t T, int64_t row_elems, int64_t S,
                     uint16_t *k_pool, uint16_t *v_pool)
{
    for (int64_t t = 0; t < T; ++t) {
        int64_t s = slot_idx[t];
        if (s < 0) continue;
        if (s >= S) return -1;
        memcpy(k_pool + s * row_elems, k + t * row_elems, sizeof(uint16_t) * (size_t)row_elems);
        memcpy(v_pool + s * row_elems, v + t * row_elems, sizeof(uint16_t) * (size_t)row_elems);
    }
    return 0;
}

/* Number of OpenMP threads a parallel region of this library gets. */
int oracle_num_threads(void)
{
    int n = 1;
#pragma omp parallel
    {
#pragma omp single
        n =
#ifdef _OPENMP
            omp_get_num_threads();
#else
            1;
#endif
    }
    return n;
}
