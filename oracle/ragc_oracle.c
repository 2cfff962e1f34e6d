/*
 * CPU oracle for prefix-cached prefill attention.  TEST INFRASTRUCTURE ONLY:
 * nothing on the product path may call this; it exists so that tests, the smoke
 * check and the benchmark's cpu_baseline leg have an independent, slow and
 * obviously correct answer to compare the HIP kernels with.  It shares no code,
 * header or table with them.
 *
 * What it computes.  The paper reuses the cached key/value tensors of the
 * retrieved documents and computes only the request tokens (Sec. 3.2 "Full
 * prefill computation"); the result must be the one full recomputation would
 * give (Sec. 9: the exact KV cache is preserved, generation is unchanged).  The
 * attention itself is the standard scaled dot-product attention the paper cites
 * (Sec. 1, Sec. 5.1: a token's state depends on the tokens before it), for
 * multi-head and grouped-query layouts (Sec. 6).  So for one request with P
 * cached tokens and N new tokens, query head h reading kv head g = h / (Hq/Hkv),
 * and new token i (absolute position P+i):
 *
 *     s_j = scale * sum_d q[i,h,d] * k[j,g,d]          j = 0 .. P+i  (inclusive)
 *     w_j = exp(s_j - max_j s_j) / sum_j' exp(s_j' - max s)
 *     o[i,h,:] = sum_j w_j * v[j,g,:]
 *
 * written out below exactly like that, in fp64, one row at a time, with no
 * blocking, no online rescaling and no reordering.  k and v are the LOGICAL
 * sequence (cached prefix rows then new rows); the oracle never sees block
 * tables, so the paged gather of the HIP path is verified independently.
 *
 * Pins (tests marked "not gpu"): hand-worked D=1 case, single-key case returns
 * V, q=0 gives running means, a dominant key returns its V row, P=0 equals a
 * library causal attention, an independent numpy full-sequence recomputation,
 * causality and GQA invariances.
 */
#include <math.h>
#include <stdlib.h>
#include <string.h>

/* Returns 0 on success, -1 on bad arguments, -2 on allocation failure.
 *   q      [N][Hq][D]      new-token queries
 *   k, v   [P+N][Hkv][D]   logical key/value sequence
 *   rows   n_rows pairs (i, h), or NULL for all N*Hq rows in (i, h) order
 *   out    [n_rows][D]  (or [N][Hq][D] when rows == NULL)
 *   wsum   optional [n_rows]: sum of the softmax weights of each row
 *   threads  OpenMP threads over rows (<= 0: runtime default)
 */
int ragc_oracle_prefill_attn(const double* q, const double* k, const double* v,
                             int P, int N, int Hq, int Hkv, int D, double scale,
                             const int* rows, long n_rows, double* out, double* wsum,
                             int threads)
{
    if (!q || !k || !v || !out || P < 0 || N < 0 || Hq <= 0 || Hkv <= 0 || D <= 0) return -1;
    if (Hq % Hkv != 0) return -1;
    const int G = Hq / Hkv;
    const long total = rows ? n_rows : (long)N * Hq;
    int failed = 0;
#ifdef _OPENMP
#pragma omp parallel num_threads(threads > 0 ? threads : 1) if (threads != 1)
#endif
    {
        double* w = (double*)malloc(sizeof(double) * (size_t)(P + N > 0 ? P + N : 1));
        if (!w) {
#ifdef _OPENMP
#pragma omp atomic write
#endif
            failed = 1;
        }
#ifdef _OPENMP
#pragma omp for schedule(dynamic, 8)
#endif
        for (long r = 0; r < total; ++r) {
            if (!w) continue;
            const int i = rows ? rows[2 * r] : (int)(r / Hq);
            const int h = rows ? rows[2 * r + 1] : (int)(r % Hq);
            if (i < 0 || i >= N || h < 0 || h >= Hq) {
#ifdef _OPENMP
#pragma omp atomic write
#endif
                failed = 2;
                continue;
            }
            const int g = h / G;
            const int visible = P + i + 1; /* a token sees the prefix, earlier new tokens and itself */
            const double* qi = q + ((size_t)i * Hq + h) * D;
            double smax = -INFINITY;
            for (int j = 0; j < visible; ++j) {
                const double* kj = k + ((size_t)j * Hkv + g) * D;
                double dot = 0.0;
                for (int d = 0; d < D; ++d) dot += qi[d] * kj[d];
                w[j] = scale * dot;
                if (w[j] > smax) smax = w[j];
            }
            double denom = 0.0;
            for (int j = 0; j < visible; ++j) {
                w[j] = exp(w[j] - smax);
                denom += w[j];
            }
            double* o = out + (size_t)r * D;
            for (int d = 0; d < D; ++d) o[d] = 0.0;
            double ws = 0.0;
            for (int j = 0; j < visible; ++j) {
                const double wj = w[j] / denom;
                const double* vj = v + ((size_t)j * Hkv + g) * D;
                ws += wj;
                for (int d = 0; d < D; ++d) o[d] += wj * vj[d];
            }
            if (wsum) wsum[r] = ws;
        }
        free(w);
    }
    if (failed == 1) return -2;
    if (failed == 2) return -1;
    return 0;
}

int ragc_oracle_max_threads(void)
{
#ifdef _OPENMP
    extern int omp_get_max_threads(void);
    return omp_get_max_threads();
#else
    return 1;
#endif
}
