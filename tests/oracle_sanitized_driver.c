/* Runs every entry point of the CPU oracle on small ragged layouts with buffers
 * of exactly the documented sizes; built by tests/test_oracle_sanitized.py with
 * AddressSanitizer and UndefinedBehaviorSanitizer, so that an access outside a
 * buffer, a shift out of range or a signed overflow inside the oracle ends the
 * program with an error.  It also checks the closed form of C_B on the
 * hand-built example v = [3, -1, 0, -4 | 0.5] (Section 3.2; sign(0) read as +1).
 * Test infrastructure only. */
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

int efo_check_offsets(const int64_t *offs, int64_t B, int64_t d);
int64_t efo_sign_words(int64_t d);
int efo_compress(const float *v, int64_t d, const int64_t *offs, int64_t B, uint64_t *signs, float *scales);
int efo_decode(const uint64_t *signs, const float *scales, int64_t d, const int64_t *offs, int64_t B, float *out);
int efo_worker_step(const float *g, float *m, float *e, int64_t d, const int64_t *offs, int64_t B, float mu,
                    float eta_prev, float eta, uint64_t *signs, float *scales);
int efo_worker_step_sgd(const float *g, float *e, int64_t d, const int64_t *offs, int64_t B, float eta_prev, float eta,
                        uint64_t *signs, float *scales);
int efo_server_step(int M, const uint64_t *signs, const float *scales, float *te, int64_t d, const int64_t *offs,
                    int64_t B, float eta_prev, float eta, uint64_t *out_signs, float *out_scales);
int efo_apply(float *x, const uint64_t *signs, const float *scales, int64_t d, const int64_t *offs, int64_t B,
              float eta);
int efo_apply_wd(float *x, float *mt, const uint64_t *signs, const float *scales, int64_t d, const int64_t *offs,
                 int64_t B, float eta, float mu, float lambda);
int efo_quality(const float *v, int64_t d, const int64_t *offs, int64_t B, double *phi, double *delta);
int efo_step(int M, const float *g, float *m, float *e, float *te, float *x, int64_t d, const int64_t *offs,
             int64_t B, float mu, float eta_prev, float eta, uint64_t *wsigns, float *wscales, uint64_t *ssigns,
             float *sscales);

static uint32_t rng_state = 12345u;
static float next_value(void)
{
    rng_state = rng_state * 1664525u + 1013904223u;
    if ((rng_state >> 28) == 0u)
        return 0.0f; /* some exact zeros */
    return ((float)(rng_state >> 8) / 8388608.0f - 1.0f) * 3.0f;
}

#define REQUIRE(cond)                                                        \
    do {                                                                     \
        if (!(cond)) {                                                       \
            fprintf(stderr, "line %d: %s failed\n", __LINE__, #cond);        \
            return 1;                                                        \
        }                                                                    \
    } while (0)

static int run_layout(const int64_t *offs, int64_t B, int M)
{
    const int64_t d = offs[B], W = efo_sign_words(d);
    float *g = malloc(sizeof(float) * (size_t)(M * d)), *m = calloc((size_t)(M * d), sizeof(float));
    float *e = calloc((size_t)(M * d), sizeof(float)), *te = calloc((size_t)d, sizeof(float));
    float *x = calloc((size_t)d, sizeof(float)), *mt = calloc((size_t)d, sizeof(float));
    float *dec = malloc(sizeof(float) * (size_t)d);
    uint64_t *ws = malloc(sizeof(uint64_t) * (size_t)(M * W)), *ss = malloc(sizeof(uint64_t) * (size_t)W);
    float *wc = malloc(sizeof(float) * (size_t)(M * B)), *sc = malloc(sizeof(float) * (size_t)B);
    double phi, delta;
    int i, t;
    int64_t j;
    REQUIRE(g && m && e && te && x && mt && dec && ws && ss && wc && sc);
    REQUIRE(efo_check_offsets(offs, B, d) == 0);
    for (t = 0; t < 3; ++t) {
        const float eta_prev = t ? 0.1f : 0.0f, eta = t == 2 ? 0.05f : 0.1f;
        for (j = 0; j < M * d; ++j)
            g[j] = next_value();
        REQUIRE(efo_step(M, g, m, e, te, x, d, offs, B, 0.9f, eta_prev, eta, ws, wc, ss, sc) == 0);
        for (i = 0; i < M; ++i) {
            REQUIRE(efo_worker_step(g + i * d, m + i * d, e + i * d, d, offs, B, 0.9f, eta_prev, eta, ws + i * W,
                                    wc + i * B) == 0);
            REQUIRE(efo_worker_step_sgd(g + i * d, e + i * d, d, offs, B, eta_prev, eta, ws + i * W, wc + i * B) == 0);
        }
        REQUIRE(efo_server_step(M, ws, wc, te, d, offs, B, eta_prev, eta, ss, sc) == 0);
        REQUIRE(efo_apply(x, ss, sc, d, offs, B, eta) == 0);
        REQUIRE(efo_apply_wd(x, mt, ss, sc, d, offs, B, eta, 0.9f, 5e-4f) == 0);
        REQUIRE(efo_compress(g, d, offs, B, ss, sc) == 0);
        REQUIRE(efo_decode(ss, sc, d, offs, B, dec) == 0);
        REQUIRE(efo_quality(g, d, offs, B, &phi, &delta) == 0);
        REQUIRE(phi > 0.0 && phi <= 1.0 && delta > 0.0 && delta <= 1.0);
        if (d % 64)
            REQUIRE((ss[W - 1] >> (d % 64)) == 0u); /* padding bits stay 0 */
    }
    free(g); free(m); free(e); free(te); free(x); free(mt); free(dec); free(ws); free(ss); free(wc); free(sc);
    return 0;
}

int main(void)
{
    /* closed form of C_B */
    {
        const float v[5] = {3.0f, -1.0f, 0.0f, -4.0f, 0.5f};
        const int64_t offs[3] = {0, 4, 5};
        uint64_t signs[1];
        float scales[2], dec[5];
        const float want[5] = {2.0f, -2.0f, 2.0f, -2.0f, 0.5f};
        REQUIRE(efo_compress(v, 5, offs, 2, signs, scales) == 0);
        REQUIRE(signs[0] == 0x15u && scales[0] == 2.0f && scales[1] == 0.5f);
        REQUIRE(efo_decode(signs, scales, 5, offs, 2, dec) == 0);
        REQUIRE(memcmp(dec, want, sizeof want) == 0);
    }
    {
        const int64_t a[2] = {0, 1};                                   /* d = 1 */
        const int64_t b[6] = {0, 1, 64, 65, 127, 200};                 /* word boundaries inside and between blocks */
        const int64_t c[4] = {0, 63, 128, 129};
        const int64_t e[3] = {0, 4097, 8192};
        int64_t many[302];
        int k;
        for (k = 0; k <= 301; ++k)
            many[k] = k;                                               /* 301 blocks of one element */
        REQUIRE(run_layout(a, 1, 1) == 0);
        REQUIRE(run_layout(b, 5, 3) == 0);
        REQUIRE(run_layout(c, 3, 2) == 0);
        REQUIRE(run_layout(e, 2, 4) == 0);
        REQUIRE(run_layout(many, 301, 2) == 0);
    }
    /* rejected partitions must not be touched */
    {
        const int64_t bad1[3] = {0, 2, 2}, bad2[3] = {1, 2, 3}, bad3[3] = {0, 3, 2};
        REQUIRE(efo_check_offsets(bad1, 2, 2) != 0);
        REQUIRE(efo_check_offsets(bad2, 2, 3) != 0);
        REQUIRE(efo_check_offsets(bad3, 2, 2) != 0);
    }
    puts("oracle sanitized run ok");
    return 0;
}
