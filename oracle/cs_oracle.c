/*
 * CPU oracle for the co-serving attention hot path -- TEST INFRASTRUCTURE ONLY.
 *
 * Plain fp64 softmax attention over the LOGICAL (unpaged) key/value sequence of one
 * request, exactly as the definition reads: a new token at absolute position p attends
 * keys 0..p of its own request (prior context plus the causal part of its own chunk;
 * paper Sec. 4.2, the P(P+C) attention term and the chunked-prefill paragraph), with
 * grouped-query heads (kv head = query head / group size) and a caller-given scale.
 *
 * No blocking, no online softmax, no paging: scores for one (query, head) are written to
 * a buffer, the maximum is subtracted, the exponentials are normalised and the values are
 * averaged.  Inputs are float32 arrays holding bf16-representable numbers; they are
 * widened to double exactly.  Nothing here is shared with the HIP library.
 *
 * Build: gcc -O2 -fopenmp -shared -fPIC cs_oracle.c -o libcs_oracle.so -lm
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#ifdef _OPENMP
#include <omp.h>
#endif

/*
 * q        [nq][Hq][D]   float   query rows of ONE request
 * pos      [nq]          int32   absolute position of each query row (chunk row i of a
 *                                request with prior context C has pos = C + i; a decode
 *                                token has pos = C)
 * k, v     [n][Hkv][D]   float   logical keys / values of that request, n > max(pos)
 * out      [nq][Hq][D]   double  attention output
 * wsum     [nq][Hq]      double  (nullable) sum of the normalised weights of each row,
 *                                returned so a test can check it equals 1
 * returns 0, or -1 on bad arguments, -2 if a position is outside [0, n)
 */
int cs_ref_attention_seq(const float* q, const int32_t* pos, int32_t nq,
                         const float* k, const float* v, int32_t n,
                         int32_t Hq, int32_t Hkv, int32_t D, double scale,
                         double* out, double* wsum)
{
    if (!q || !pos || !k || !v || !out) return -1;
    if (nq < 0 || n <= 0 || Hq <= 0 || Hkv <= 0 || D <= 0 || Hq % Hkv != 0) return -1;
    const int32_t G = Hq / Hkv;
    int32_t maxpos = -1;
    for (int32_t i = 0; i < nq; ++i) {
        if (pos[i] < 0 || pos[i] >= n) return -2;
        if (pos[i] > maxpos) maxpos = pos[i];
    }
    int failed = 0;
#pragma omp parallel
    {
        double* s = (double*)malloc(sizeof(double) * (size_t)(maxpos + 2));
        if (!s) {
#pragma omp atomic write
            failed = 1;
        }
#pragma omp for collapse(2) schedule(dynamic, 1)
        for (int32_t i = 0; i < nq; ++i) {
            for (int32_t h = 0; h < Hq; ++h) {
                if (!s) continue;
                const int32_t g = h / G;          /* kv head shared by this query head */
                const int32_t p = pos[i];         /* last visible key                 */
                const float* qv = q + ((size_t)i * Hq + h) * D;
                double m = -INFINITY;
                for (int32_t j = 0; j <= p; ++j) {
                    const float* kv = k + ((size_t)j * Hkv + g) * D;
                    double acc = 0.0;
                    for (int32_t d = 0; d < D; ++d) acc += (double)qv[d] * (double)kv[d];
                    s[j] = scale * acc;
                    if (s[j] > m) m = s[j];
                }
                double denom = 0.0;
                for (int32_t j = 0; j <= p; ++j) { s[j] = exp(s[j] - m); denom += s[j]; }
                double* o = out + ((size_t)i * Hq + h) * D;
                for (int32_t d = 0; d < D; ++d) o[d] = 0.0;
                double wtot = 0.0;
                for (int32_t j = 0; j <= p; ++j) {
                    const double w = s[j] / denom;
                    wtot += w;
                    const float* vv = v + ((size_t)j * Hkv + g) * D;
                    for (int32_t d = 0; d < D; ++d) o[d] += w * (double)vv[d];
                }
                if (wsum) wsum[(size_t)i * Hq + h] = wtot;
            }
        }
        free(s);
    }
    return failed ? -1 : 0;
}

/* Number of threads the parallel region above will use (reported by the benchmark). */
int cs_ref_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}
