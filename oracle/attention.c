/*
 * CPU oracle for causal grouped-query scaled-dot-product attention.
 *
 * TEST INFRASTRUCTURE ONLY.  Nothing on the product path may call, link or import this file; it
 * exists so that the HIP kernels can be checked element by element against the plain definition.
 * It shares no code with the HIP path.
 *
 * What it computes is the attention equation of the paper's background section (Eq. 2):
 *     Attention(q_i, K, V) = softmax(q_i K^T * scale) V
 * evaluated separately for every request, with K, V in R^{L' x (H x D)} (L' = context length so
 * far, H = KV heads, D = head dimension), written out directly:
 *   - two passes over the keys (scores and their maximum first, then the weighted sum),
 *   - no tiling, no running ("online") softmax, no reordering,
 *   - every product and sum in double precision; bf16 inputs are widened exactly.
 *
 * Readings the paper leaves open (each is a parameter or documented here):
 *   - "scale": the equation divides by an unnamed scale; the caller passes the multiplier
 *     (1/sqrt(D) in all workloads).
 *   - causality: query row i of a request whose context holds kv_len tokens, the last q_len of
 *     which are the queries themselves, sees keys 0 .. kv_len - q_len + i (inclusive).
 *   - grouped-query attention: query head h reads KV head h / (Hq / H).
 *   - layouts: Q and O are [rows, Hq, D]; K and V are [kv_len, H, D] (token-major, as a
 *     [B, L, H, D] cache stores one request).
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

static inline double bf16_to_double(uint16_t b) {
    uint32_t u = ((uint32_t)b) << 16;
    float f;
    memcpy(&f, &u, sizeof f);
    return (double)f;
}

int oracle_num_threads(void) {
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/*
 * Softmax probabilities of one query vector against n keys of one KV head.
 *   q      : D bf16 values
 *   k      : keys, [n, H, D] bf16, this function reads head kvh
 *   p_out  : n doubles, p_j = exp(s_j - max_j s_j) / sum_j exp(s_j - max_j s_j),
 *            s_j = scale * sum_d q[d] * k[j, kvh, d]
 * Returned value: the maximum score (useful for tests).
 */
double oracle_softmax_row(const uint16_t* q, const uint16_t* k, int64_t n, int H, int D, int kvh,
                          double scale, double* p_out) {
    double m = -INFINITY;
    for (int64_t j = 0; j < n; ++j) {
        const uint16_t* kj = k + ((size_t)j * H + kvh) * D;
        double s = 0.0;
        for (int d = 0; d < D; ++d) s += bf16_to_double(q[d]) * bf16_to_double(kj[d]);
        s *= scale;
        p_out[j] = s;
        if (s > m) m = s;
    }
    double denom = 0.0;
    for (int64_t j = 0; j < n; ++j) {
        p_out[j] = exp(p_out[j] - m);
        denom += p_out[j];
    }
    for (int64_t j = 0; j < n; ++j) p_out[j] /= denom;
    return m;
}

/*
 * Attention output for a set of query rows of ONE request.
 *   q       : [q_len, Hq, D] bf16, the request's query rows
 *   k, v    : [kv_len, H, D] bf16, the request's whole context (already including the q_len
 *             newest tokens)
 *   rows    : indices in [0, q_len) of the rows to evaluate, or NULL for all rows 0..q_len-1
 *   n_rows  : number of entries of rows (or q_len when rows == NULL)
 *   out     : [n_rows, Hq, D] doubles
 * Returns 0, or -1 on an invalid argument (kv_len < q_len, Hq % H != 0, row out of range).
 */
int oracle_attention_request(const uint16_t* q, const uint16_t* k, const uint16_t* v, int64_t q_len,
                             int64_t kv_len, int Hq, int H, int D, double scale, const int32_t* rows,
                             int64_t n_rows, double* out) {
    if (kv_len < q_len || H <= 0 || Hq % H != 0 || D <= 0) return -1;
    if (rows) {
        for (int64_t r = 0; r < n_rows; ++r)
            if (rows[r] < 0 || rows[r] >= q_len) return -1;
    } else if (n_rows != q_len) {
        return -1;
    }
    const int group = Hq / H;
    int failed = 0;
#pragma omp parallel
    {
        double* p = (double*)malloc(sizeof(double) * (size_t)(kv_len > 0 ? kv_len : 1));
        if (!p) {
#pragma omp atomic write
            failed = 1;
        }
#pragma omp for collapse(2) schedule(dynamic, 1)
        for (int64_t r = 0; r < n_rows; ++r) {
            for (int h = 0; h < Hq; ++h) {
                if (!p) continue;
                const int64_t i = rows ? rows[r] : r;
                const int64_t n = kv_len - q_len + i + 1; /* visible keys */
                const int kvh = h / group;
                const uint16_t* qi = q + ((size_t)i * Hq + h) * D;
                oracle_softmax_row(qi, k, n, H, D, kvh, scale, p);
                double* o = out + ((size_t)r * Hq + h) * D;
                for (int d = 0; d < D; ++d) o[d] = 0.0;
                for (int64_t j = 0; j < n; ++j) {
                    const uint16_t* vj = v + ((size_t)j * H + kvh) * D;
                    const double pj = p[j];
                    for (int d = 0; d < D; ++d) o[d] += pj * bf16_to_double(vj[d]);
                }
            }
        }
        free(p);
    }
    return failed ? -1 : 0;
}
