/*
 * ef_oracle.c -- CPU oracle for dist-EF-blockSGDM (arxiv 1905.10936).
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, single-threaded, plain-C
 * statement of what the hot path computes.  It shares no code with the HIP
 * library and must never be called from the product path; only the tests, the
 * smoke check and the benchmark's cpu_baseline leg load it.
 *
 * What it follows:
 *   - blockwise scaled-sign compressor C_B            : Section 3.2
 *   - worker / server / parameter update of one step  : Algorithm 4
 *     (Algorithm 3 is the mu = 0 case, Eq. (1) is the B = 1 case)
 *   - parameter update with weight decay outside compression : Appendix A
 *   - phi(v) of Proposition 1 and delta of the non-block compressor : Section 3.2
 *   - one bit per coordinate for the sign in {-1, +1},
 *     one fp32 scale per block                        : Appendix A, Section 3.2
 *
 * Readings where the paper is silent (kept identical on the GPU side by
 * construction of the tests, not by shared code):
 *   - sign(0): bit = (p >= 0), so +0 and -0 both encode +1.
 *   - arithmetic: fp32, round-to-nearest-even, one rounding per written
 *     operation, evaluated left to right, never fused (build with
 *     -ffp-contract=off).
 *   - ||.||_1 of a block: accumulated in double, ascending index, divided by
 *     d_b in double, rounded once to float.
 *   - (1/M) sum_i: fp32 running sum in worker order starting from +0, then one
 *     fp32 division by (float)M.
 *   - eta_{t-1}/eta_t: one fp32 division; eta_{-1} = 0 gives ratio 0.
 *   - Appendix A update, per coordinate, one rounding per operation:
 *     lx = lambda*x ; mt = mu*mt + lx ; x = x - eta*((Delta + mu*mt) + lx).
 *   - packing: flat index j -> bit (j mod 64) of 64-bit word floor(j/64),
 *     least significant bit first; bits past d are 0.
 *
 * Pins (tests/test_oracle_pins.py): every function here is pinned by closed
 * forms, the paper's constant-magnitude example, the Proposition 1 energy
 * identity, the Lemma 3 recurrence, brute force on tiny inputs, the exactly
 * rounded L1 norm of blocks of up to 10^6 elements, and special cases
 * (identity compressor, M = 1, majority vote).  The Algorithm 3 worker
 * is pinned to the Algorithm 4 worker at mu = 0 (the reduction Section 4.1
 * states) and to the brute force; the Appendix A update to efo_apply at
 * lambda = 0, to a float64 run of the decay-momentum recursion on dyadic values
 * (zero payload) and to the brute force.  efo_quality is pinned by the closed
 * form the paper prints for the constant-magnitude example, by one-hot blocks
 * (ratio 1/d_b exactly), by B = 1 (phi = delta) and by the approximation
 * inequality of Definition 1 measured on the oracle's own compressor output.
 * Nothing is unpinned.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#define EFO_OK 0
#define EFO_BAD_ARG -1
#define EFO_BAD_OFFSETS -2
#define EFO_NO_MEM -3

/* Partition check: offs[0] = 0 < offs[1] < ... < offs[B] = d (Section 3.2:
 * every block has d_b >= 1 elements, d_b is a denominator). */
int efo_check_offsets(const int64_t *offs, int64_t B, int64_t d)
{
    int64_t b;
    if (!offs || B < 1 || d < 1)
        return EFO_BAD_OFFSETS;
    if (offs[0] != 0 || offs[B] != d)
        return EFO_BAD_OFFSETS;
    for (b = 0; b < B; ++b)
        if (offs[b + 1] <= offs[b])
            return EFO_BAD_OFFSETS;
    return EFO_OK;
}

int64_t efo_sign_words(int64_t d)
{
    return (d + 63) / 64;
}

/* C_B(v), Section 3.2: block b -> (||v_Gb||_1 / d_b, sign(v_Gb)).
 * signs: uint64[ceil(d/64)], scales: float[B]. */
int efo_compress(const float *v, int64_t d, const int64_t *offs, int64_t B,
                 uint64_t *signs, float *scales)
{
    int64_t b, j;
    int rc = efo_check_offsets(offs, B, d);
    if (rc)
        return rc;
    if (!v || !signs || !scales)
        return EFO_BAD_ARG;
    memset(signs, 0, (size_t)efo_sign_words(d) * sizeof(uint64_t));
    for (b = 0; b < B; ++b) {
        double l1 = 0.0;
        int64_t db = offs[b + 1] - offs[b];
        for (j = offs[b]; j < offs[b + 1]; ++j) {
            l1 += (double)fabsf(v[j]);
            if (v[j] >= 0.0f)
                signs[j / 64] |= (uint64_t)1 << (j % 64);
        }
        scales[b] = (float)(l1 / (double)db);
    }
    return EFO_OK;
}

/* Inverse view of the payload: out_j = +scale_b(j) if bit j is set, else
 * -scale_b(j).  This is the vector Delta of Algorithm 4. */
int efo_decode(const uint64_t *signs, const float *scales, int64_t d,
               const int64_t *offs, int64_t B, float *out)
{
    int64_t b, j;
    int rc = efo_check_offsets(offs, B, d);
    if (rc)
        return rc;
    if (!signs || !scales || !out)
        return EFO_BAD_ARG;
    for (b = 0; b < B; ++b)
        for (j = offs[b]; j < offs[b + 1]; ++j) {
            int bit = (int)((signs[j / 64] >> (j % 64)) & 1u);
            out[j] = bit ? scales[b] : -scales[b];
        }
    return EFO_OK;
}

/* One worker's part of iteration t of Algorithm 4:
 *   m <- mu*m + g
 *   p  = mu*m + g + (eta_prev/eta)*e        (uses the updated m)
 *   Delta = C_B(p)  -> (signs, scales)
 *   e <- p - Delta
 */
int efo_worker_step(const float *g, float *m, float *e, int64_t d,
                    const int64_t *offs, int64_t B, float mu, float eta_prev,
                    float eta, uint64_t *signs, float *scales)
{
    int64_t j;
    float r, *p, *delta;
    int rc = efo_check_offsets(offs, B, d);
    if (rc)
        return rc;
    if (!g || !m || !e || !signs || !scales)
        return EFO_BAD_ARG;
    if (!(mu >= 0.0f && mu < 1.0f) || !(eta > 0.0f) || !(eta_prev >= 0.0f))
        return EFO_BAD_ARG;
    p = (float *)malloc((size_t)d * sizeof(float));
    delta = (float *)malloc((size_t)d * sizeof(float));
    if (!p || !delta) {
        free(p);
        free(delta);
        return EFO_NO_MEM;
    }
    r = eta_prev / eta;
    for (j = 0; j < d; ++j) {
        float mm = mu * m[j];
        float mnew = mm + g[j];
        float t1, t2, t3;
        m[j] = mnew;
        t1 = mu * mnew;
        t2 = t1 + g[j];
        t3 = r * e[j];
        p[j] = t2 + t3;
    }
    rc = efo_compress(p, d, offs, B, signs, scales);
    if (!rc)
        rc = efo_decode(signs, scales, d, offs, B, delta);
    if (!rc)
        for (j = 0; j < d; ++j)
            e[j] = p[j] - delta[j];
    free(p);
    free(delta);
    return rc;
}

/* One worker's part of iteration t of Algorithm 3 (no momentum):
 *   p  = g + (eta_prev/eta)*e
 *   Delta = C_B(p)  -> (signs, scales)
 *   e <- p - Delta
 */
int efo_worker_step_sgd(const float *g, float *e, int64_t d, const int64_t *offs,
                        int64_t B, float eta_prev, float eta, uint64_t *signs,
                        float *scales)
{
    int64_t j;
    float r, *p, *delta;
    int rc = efo_check_offsets(offs, B, d);
    if (rc)
        return rc;
    if (!g || !e || !signs || !scales)
        return EFO_BAD_ARG;
    if (!(eta > 0.0f) || !(eta_prev >= 0.0f))
        return EFO_BAD_ARG;
    p = (float *)malloc((size_t)d * sizeof(float));
    delta = (float *)malloc((size_t)d * sizeof(float));
    if (!p || !delta) {
        free(p);
        free(delta);
        return EFO_NO_MEM;
    }
    r = eta_prev / eta;
    for (j = 0; j < d; ++j) {
        float t = r * e[j];
        p[j] = g[j] + t;
    }
    rc = efo_compress(p, d, offs, B, signs, scales);
    if (!rc)
        rc = efo_decode(signs, scales, d, offs, B, delta);
    if (!rc)
        for (j = 0; j < d; ++j)
            e[j] = p[j] - delta[j];
    free(p);
    free(delta);
    return rc;
}

/* Server part of iteration t of Algorithm 4:
 *   ptilde = (1/M) sum_i Delta_i + (eta_prev/eta)*etilde
 *   Deltatilde = C_B(ptilde) -> (out_signs, out_scales)
 *   etilde <- ptilde - Deltatilde
 * signs: uint64[M][W], scales: float[M][B], worker-major.
 */
int efo_server_step(int M, const uint64_t *signs, const float *scales,
                    float *te, int64_t d, const int64_t *offs, int64_t B,
                    float eta_prev, float eta, uint64_t *out_signs,
                    float *out_scales)
{
    int64_t j, W = efo_sign_words(d);
    int i;
    float r, *tp, *delta, *acc;
    int rc = efo_check_offsets(offs, B, d);
    if (rc)
        return rc;
    if (M < 1 || !signs || !scales || !te || !out_signs || !out_scales)
        return EFO_BAD_ARG;
    if (!(eta > 0.0f) || !(eta_prev >= 0.0f))
        return EFO_BAD_ARG;
    tp = (float *)malloc((size_t)d * sizeof(float));
    delta = (float *)malloc((size_t)d * sizeof(float));
    acc = (float *)malloc((size_t)d * sizeof(float));
    if (!tp || !delta || !acc) {
        free(tp);
        free(delta);
        free(acc);
        return EFO_NO_MEM;
    }
    r = eta_prev / eta;
    for (j = 0; j < d; ++j)
        acc[j] = 0.0f;
    for (i = 0; i < M && !rc; ++i) {
        rc = efo_decode(signs + (int64_t)i * W, scales + (int64_t)i * B, d,
                        offs, B, delta);
        if (!rc)
            for (j = 0; j < d; ++j)
                acc[j] = acc[j] + delta[j];
    }
    if (!rc) {
        for (j = 0; j < d; ++j) {
            float avg = acc[j] / (float)M;
            float t = r * te[j];
            tp[j] = avg + t;
        }
        rc = efo_compress(tp, d, offs, B, out_signs, out_scales);
    }
    if (!rc)
        rc = efo_decode(out_signs, out_scales, d, offs, B, delta);
    if (!rc)
        for (j = 0; j < d; ++j)
            te[j] = tp[j] - delta[j];
    free(tp);
    free(delta);
    free(acc);
    return rc;
}

/* Parameter update of Algorithm 4: x <- x - eta * Deltatilde. */
int efo_apply(float *x, const uint64_t *signs, const float *scales, int64_t d,
              const int64_t *offs, int64_t B, float eta)
{
    int64_t j;
    float *delta;
    int rc = efo_check_offsets(offs, B, d);
    if (rc)
        return rc;
    if (!x || !signs || !scales || !(eta > 0.0f))
        return EFO_BAD_ARG;
    delta = (float *)malloc((size_t)d * sizeof(float));
    if (!delta)
        return EFO_NO_MEM;
    rc = efo_decode(signs, scales, d, offs, B, delta);
    if (!rc)
        for (j = 0; j < d; ++j) {
            float u = eta * delta[j];
            x[j] = x[j] - u;
        }
    free(delta);
    return rc;
}

/* Parameter update with the weight decay kept outside the compressed signal
 * (Appendix A): an extra momentum mt for the decay term on every machine,
 *   mt <- mu*mt + lambda*x
 *   x  <- x - eta * (Deltatilde + mu*mt + lambda*x)     (updated mt, old x)
 * evaluated in fp32, one rounding per operation, left to right. */
int efo_apply_wd(float *x, float *mt, const uint64_t *signs, const float *scales,
                 int64_t d, const int64_t *offs, int64_t B, float eta, float mu,
                 float lambda)
{
    int64_t j;
    float *delta;
    int rc = efo_check_offsets(offs, B, d);
    if (rc)
        return rc;
    if (!x || !mt || !signs || !scales || !(eta > 0.0f))
        return EFO_BAD_ARG;
    if (!(mu >= 0.0f && mu < 1.0f) || !(lambda >= 0.0f))
        return EFO_BAD_ARG;
    delta = (float *)malloc((size_t)d * sizeof(float));
    if (!delta)
        return EFO_NO_MEM;
    rc = efo_decode(signs, scales, d, offs, B, delta);
    if (!rc)
        for (j = 0; j < d; ++j) {
            float lx = lambda * x[j];
            float a = mu * mt[j];
            float mnew = a + lx;
            float b = mu * mnew;
            float u1 = delta[j] + b;
            float u = u1 + lx;
            float step = eta * u;
            mt[j] = mnew;
            x[j] = x[j] - step;
        }
    free(delta);
    return rc;
}

/* How well the compressors approximate v (Definition 1):
 *   phi(v)   = min_b ||v_Gb||_1^2 / (d_b ||v_Gb||_2^2)   for C_B   (Proposition 1)
 *   delta(v) = ||v||_1^2 / (d ||v||_2^2)                 for the non-block compressor, Eq. (1)
 * in double, sums in ascending index order.  A block (or vector) of zeros is
 * reproduced exactly by the compressor and counts as ratio 1.
 */
int efo_quality(const float *v, int64_t d, const int64_t *offs, int64_t B,
                double *phi, double *delta)
{
    int64_t b, j;
    double l1 = 0.0, l2 = 0.0, best = 1.0;
    int rc = efo_check_offsets(offs, B, d);
    if (rc)
        return rc;
    if (!v || !phi || !delta)
        return EFO_BAD_ARG;
    for (b = 0; b < B; ++b) {
        double a1 = 0.0, a2 = 0.0;
        for (j = offs[b]; j < offs[b + 1]; ++j) {
            double a = fabs((double)v[j]);
            a1 += a;
            a2 += a * a;
        }
        if (a2 > 0.0) {
            double ratio = a1 * a1 / ((double)(offs[b + 1] - offs[b]) * a2);
            if (ratio < best)
                best = ratio;
        }
    }
    for (j = 0; j < d; ++j) {
        double a = fabs((double)v[j]);
        l1 += a;
        l2 += a * a;
    }
    *phi = best;
    *delta = l2 > 0.0 ? l1 * l1 / ((double)d * l2) : 1.0;
    return EFO_OK;
}

/* One whole iteration for M workers that share x (they all pull the same
 * Deltatilde, so one copy of x stands for all of them).
 * g, m, e: float[M][d]; wsigns: uint64[M][W]; wscales: float[M][B]. */
int efo_step(int M, const float *g, float *m, float *e, float *te, float *x,
             int64_t d, const int64_t *offs, int64_t B, float mu,
             float eta_prev, float eta, uint64_t *wsigns, float *wscales,
             uint64_t *ssigns, float *sscales)
{
    int i, rc = EFO_OK;
    int64_t W = efo_sign_words(d);
    if (M < 1)
        return EFO_BAD_ARG;
    for (i = 0; i < M && !rc; ++i)
        rc = efo_worker_step(g + (int64_t)i * d, m + (int64_t)i * d,
                             e + (int64_t)i * d, d, offs, B, mu, eta_prev,
                             eta, wsigns + (int64_t)i * W,
                             wscales + (int64_t)i * B);
    if (!rc)
        rc = efo_server_step(M, wsigns, wscales, te, d, offs, B, eta_prev,
                             eta, ssigns, sscales);
    if (!rc)
        rc = efo_apply(x, ssigns, sscales, d, offs, B, eta);
    return rc;
}
