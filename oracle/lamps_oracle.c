/*
 * CPU oracle for the decode hot path under LAMPS (arXiv 2410.18248).
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain, fp64 statement of
 * what the GPU library must compute.  Only the test-suite, the smoke check and
 * the benchmark's cpu_baseline leg may build, link or call it; the product
 * path never does, and nothing here shares code with the HIP sources.
 *
 * What is stated here:
 *   - single-query attention of one decode iteration, Section 2.2 of the
 *     paper (the unnumbered equation h_out = softmax(q K^T / sqrt(d_h)) V),
 *     evaluated over the LOGICAL (un-paged) key/value sequence of each
 *     running request.  Requests that sit in an API call (Preserve / Discard /
 *     Swap, Section 1 and Section 4.2) are not in the running batch
 *     (Algorithm 1) and their output rows are left untouched.
 *   - grouped-query head mapping: query head h reads key/value head
 *     h / (H / H_kv).  The paper shows one head; heads are independent.
 *
 * Arithmetic: every stored element (fp32 or bf16 bit pattern) is widened
 * exactly to double; all sums are plain left-to-right double sums; no
 * blocking, no online rescaling, no reordering.
 *
 * Pins (tests/test_oracle_*.py): brute-force dense evaluation without max
 * subtraction, torch's float64 softmax/matmul, closed forms (one token, equal
 * keys, constant values, zero query, dominant key), invariants (row
 * permutation, key shift, value scaling, convex hull), GQA == MHA on repeated
 * heads, exactness of the bf16 widening.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#ifdef _OPENMP
#include <omp.h>
#endif

enum { ORACLE_F32 = 0, ORACLE_BF16 = 1 };

/* bf16 is the upper half of an IEEE binary32: widening is exact. */
static double widen(const void *base, size_t i, int dtype)
{
    if (dtype == ORACLE_F32) {
        return (double)((const float *)base)[i];
    } else {
        uint32_t bits = (uint32_t)((const uint16_t *)base)[i] << 16;
        float f;
        memcpy(&f, &bits, sizeof f);
        return (double)f;
    }
}

/* Exposed so a test can pin the widening against a library conversion. */
double lamps_oracle_widen(const void *base, int64_t i, int dtype)
{
    return widen(base, (size_t)i, dtype);
}

/*
 * One (request, query head): Section 2.2 equation, literally.
 *   q      : D elements
 *   K, V   : logical sequences, element (t, g, d) at ((t*Hkv)+g)*D + d
 *   C      : number of cached positions attended to
 *   o      : D doubles out
 *   p      : scratch, C doubles
 */
static void attend_one(int dtype, int Hkv, int D, double scale, const void *q,
                       size_t q_off, const void *K, const void *V, int g,
                       int C, double *o, double *p)
{
    int t, d;
    double m = -INFINITY, Z = 0.0;

    for (d = 0; d < D; ++d)
        o[d] = 0.0;
    if (C <= 0)
        return; /* empty context: empty weighted sum */

    for (t = 0; t < C; ++t) {
        size_t row = ((size_t)t * Hkv + g) * D;
        double s = 0.0;
        for (d = 0; d < D; ++d)
            s += widen(q, q_off + d, dtype) * widen(K, row + d, dtype);
        s *= scale;
        p[t] = s;
        if (s > m)
            m = s;
    }
    for (t = 0; t < C; ++t) {
        p[t] = exp(p[t] - m);
        Z += p[t];
    }
    for (t = 0; t < C; ++t) {
        size_t row = ((size_t)t * Hkv + g) * D;
        for (d = 0; d < D; ++d)
            o[d] += p[t] * widen(V, row + d, dtype);
    }
    for (d = 0; d < D; ++d)
        o[d] /= Z;
}

/*
 * One layer of one decode iteration for a batch.
 *   q        : [B][H][D] elements of `dtype`
 *   K[r],V[r]: logical sequences of request r, [C_r][Hkv][D]; may be NULL when
 *              the request is not running or C_r == 0
 *   ctx_lens : [B]
 *   running  : [B], 0 = paused (row of `out` is not written)
 *   scale    : softmax scale; pass 1/sqrt(D) for the paper's equation
 *   out      : [B][H][D] doubles
 * Returns 0, or -1 on bad arguments / allocation failure.
 */
int lamps_oracle_decode_attn(int dtype, int B, int H, int Hkv, int D,
                             double scale, const void *q,
                             const void *const *K, const void *const *V,
                             const int32_t *ctx_lens, const uint8_t *running,
                             double *out, int nthreads)
{
    int G, fail = 0;
    long pair, npairs;

    if (B < 0 || H <= 0 || Hkv <= 0 || D <= 0 || H % Hkv != 0)
        return -1;
    if (dtype != ORACLE_F32 && dtype != ORACLE_BF16)
        return -1;
    G = H / Hkv;
    npairs = (long)B * H;
#ifdef _OPENMP
    if (nthreads > 0)
        omp_set_num_threads(nthreads);
#else
    (void)nthreads;
#endif

#pragma omp parallel for schedule(dynamic, 1)
    for (pair = 0; pair < npairs; ++pair) {
        int r = (int)(pair / H), h = (int)(pair % H);
        int C = ctx_lens[r];
        double *p;
        if (!running[r])
            continue;
        p = (double *)malloc(sizeof(double) * (size_t)(C > 0 ? C : 1));
        if (!p) {
            fail = 1;
            continue;
        }
        attend_one(dtype, Hkv, D, scale, q, ((size_t)r * H + h) * D, K[r], V[r],
                   h / G, C, out + ((size_t)r * H + h) * D, p);
        free(p);
    }
    return fail ? -1 : 0;
}

/* Processors OpenMP may use here; the caller picks `nthreads` from it. */
int lamps_oracle_max_threads(void)
{
#ifdef _OPENMP
    return omp_get_num_procs();
#else
    return 1;
#endif
}
