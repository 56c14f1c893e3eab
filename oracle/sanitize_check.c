/* Runs every entry point of the oracle once on small, exactly sized heap buffers, for a build with
 * -fsanitize=address,undefined (tests/test_oracle_sanitize.py compiles and runs it): an access outside
 * a buffer, a signed overflow, a bad shift or a misaligned access ends the program with a report.
 * TEST INFRASTRUCTURE ONLY, like the oracle itself; sizes include ragged ones (n < ld, n not a
 * multiple of anything, k = n, one candidate). */
#include <stdio.h>

#include "eck_oracle.c"

#define CHECK(cond)                                                         \
    do {                                                                    \
        if (!(cond)) {                                                      \
            fprintf(stderr, "sanitize_check: %s failed (line %d)\n", #cond, __LINE__); \
            return 1;                                                       \
        }                                                                   \
    } while (0)

static float unit(uint64_t *s)
{
    *s = *s * 6364136223846793005ull + 1442695040888963407ull;
    return (float)((*s >> 40) & 0xFFFF) / 65536.0f;
}

static int one_space(const int32_t *pb, int32_t kind, int n_feat)
{
    void *sp = orc_space_create(pb, kind);
    CHECK(sp != NULL);
    int32_t G = 0;
    uint32_t radix[16];
    uint64_t size = 0;
    CHECK(orc_space_info(sp, &G, radix, &size) == ORC_OK && G >= 1 && G <= 16);
    const uint64_t n = 37, ld = 41, P = 5;
    uint16_t *genes = (uint16_t *)malloc((size_t)G * ld * 2), *par = (uint16_t *)malloc((size_t)G * P * 2);
    uint16_t *child = (uint16_t *)malloc((size_t)G * ld * 2);
    memset(genes, 0, (size_t)G * ld * 2);
    CHECK(orc_enumerate(sp, ORC_MODE_SAMPLE, 7, 0, 1000, n, NULL, 0, 0, genes, ld) == ORC_OK);
    if (size && size >= n) CHECK(orc_enumerate(sp, ORC_MODE_EXHAUSTIVE, 0, 0, size - n, n, NULL, 0, 0, child, ld) == ORC_OK);
    CHECK(orc_enumerate(sp, ORC_MODE_SAMPLE, 9, 0, 0, P, NULL, 0, 0, par, P) == ORC_OK);
    memset(child, 0, (size_t)G * ld * 2);
    CHECK(orc_enumerate(sp, ORC_MODE_MUTATE, 9, 1, 0, n, par, (uint32_t)P, 429496729u, child, ld) == ORC_OK);
    CHECK(orc_enumerate(sp, ORC_MODE_CROSSOVER, 9, 2, 0, n, par, (uint32_t)P, 0xFFFFFFFFu, child, ld) == ORC_OK);
    uint8_t *keep = (uint8_t *)malloc(n);
    CHECK(orc_dedup(child, ld, n, G, keep) == ORC_OK && keep[0] == 1);
    uint64_t *raw = (uint64_t *)malloc((size_t)n_feat * ld * 8);
    float *f32 = (float *)malloc((size_t)n_feat * ld * 4);
    uint16_t *b16 = (uint16_t *)malloc((size_t)n_feat * ld * 2);
    uint8_t *legal = (uint8_t *)malloc(n);
    memset(raw, 0, (size_t)n_feat * ld * 8);
    memset(f32, 0, (size_t)n_feat * ld * 4);
    memset(b16, 0, (size_t)n_feat * ld * 2);
    CHECK(orc_features(sp, genes, ld, n, n_feat, raw, f32, b16, legal) == ORC_OK);
    CHECK(orc_features(sp, child, ld, 1, n_feat, raw, f32, b16, legal) == ORC_OK);
    free(genes); free(par); free(child); free(keep); free(raw); free(f32); free(b16); free(legal);
    orc_space_destroy(sp);
    return 0;
}

int main(void)
{
    uint64_t s = 1;
    /* problems: op, dim[8], elem_bytes, 5 hardware parameters */
    const int32_t gemm[15] = {ORC_OP_GEMM, 1, 96, 80, 48, 0, 0, 0, 0, 2, 8, 64, 16384, 1024, 8};
    const int32_t bgemm[15] = {ORC_OP_BGEMM, 3, 40, 100, 20, 0, 0, 0, 0, 4, 6, 64, 16384, 512, 4};
    const int32_t conv[15] = {ORC_OP_CONV2D, 2, 6, 8, 9, 7, 3, 3, 2 | (1 << 16), 2, 8, 64, 65536, 2048, 16};
    const int32_t mv[15] = {ORC_OP_GEMM, 1, 64, 1, 4096, 0, 0, 0, 0, 2, 8, 64, 65536, 2048, 16};
    if (one_space(gemm, ORC_SPACE_KNOB, 32) || one_space(bgemm, ORC_SPACE_KNOB, 64) ||
        one_space(gemm, ORC_SPACE_SPLIT, 64) || one_space(bgemm, ORC_SPACE_SPLIT, 32) ||
        one_space(conv, ORC_SPACE_SPLIT, 64) || one_space(conv, ORC_SPACE_SPLIT_XRED, 64) ||
        one_space(mv, ORC_SPACE_SPLIT_XRED, 64))
        return 1;
    {
        uint32_t cnt = orc_split_table(360, NULL, 0);
        uint32_t *tab = (uint32_t *)malloc((size_t)cnt * 16);
        CHECK(orc_split_table(360, tab, cnt) == cnt && tab[0] == 1 && tab[3] == 360);
        free(tab);
        CHECK(orc_transform(0) == 0.0f && orc_transform(UINT64_MAX) > 63.9f && orc_transform(1023) == 10.0f);
        CHECK(orc_bf16_rne(1.0f) == 0x3F80 && orc_bf16_to_f32(0x3F80) == 1.0f);
        (void)orc_hash(~0ull, ~0u, ~0ull, 15);
    }
    /* model: forward, magnitude, gradient, update */
    {
        const int32_t w[4] = {6, 5, 3, 1};
        const uint64_t P = orc_param_count(3, w), n = 19, ld = 24;
        CHECK(P == 6 * 5 + 5 + 5 * 3 + 3 + 3 + 1);
        float *theta = (float *)malloc(P * 4), *feat = (float *)malloc(6 * ld * 4), *e = (float *)malloc(16 * 4);
        double *out = (double *)malloc(n * 8), *state = (double *)malloc((3 * P + 1) * 8), *grad = (double *)malloc(P * 8);
        double *y = (double *)malloc(16 * 8);
        for (uint64_t i = 0; i < P; ++i) theta[i] = unit(&s) - 0.5f;
        for (uint64_t i = 0; i < 6 * ld; ++i) feat[i] = 8.0f * unit(&s);
        CHECK(orc_score(3, w, theta, feat, ld, n, 0, out) == ORC_OK);
        CHECK(orc_score(3, w, theta, feat, ld, n, 1, out) == ORC_OK);
        CHECK(orc_score_magnitude(3, w, theta, feat, ld, n, out) == ORC_OK);
        for (uint64_t i = 0; i < 3 * P + 1; ++i) state[i] = i < P ? (double)theta[i] : 0.0;
        for (int i = 0; i < 16; ++i) { e[i] = 1.0f + unit(&s); y[i] = (double)e[i]; }
        (void)orc_batch_gradient(3, w, state, feat, ld, y, 4, 8, grad);
        double snr, loss;
        CHECK(orc_update(3, w, 0, state, feat, ld, e, 16, 5, 8, 1e-3, 0.9, 0.999, 1e-8, &snr, &loss) == ORC_OK);
        CHECK(orc_update(3, w, 1, state, feat, ld, e, 16, 3, 4, 1e-3, 0.9, 0.999, 1e-8, &snr, &loss) == ORC_OK);
        CHECK(snr == snr && loss == loss);
        e[3] = 0.0f;
        CHECK(orc_update(3, w, 0, state, feat, ld, e, 16, 1, 8, 1e-3, 0.9, 0.999, 1e-8, &snr, &loss) == ORC_OK && snr != snr);
        free(theta); free(feat); free(e); free(out); free(state); free(grad); free(y);
        (void)orc_loss(0.5, 0.25);
        (void)orc_loss_grad(0.5, 0.25);
        CHECK(orc_k_step(1.0, 5.0, 1.0, 64) < 1.0 && orc_k_step(0.0, 5.0, 1.0, 64) == 0.0);
    }
    /* selection */
    {
        const uint64_t n = 90;
        float *en = (float *)malloc(n * 4), *lat = (float *)malloc(n * 4);
        uint8_t *legal = (uint8_t *)malloc(n);
        for (uint64_t i = 0; i < n; ++i) { en[i] = unit(&s) - 0.5f; lat[i] = unit(&s) - 0.3f; legal[i] = (i % 7) != 0; }
        en[5] = NAN; lat[11] = NAN; en[17] = -0.0f; en[18] = 0.0f; lat[20] = INFINITY;
        uint32_t *idx = (uint32_t *)malloc(90 * 4), *cnt = (uint32_t *)malloc(90 * 4);
        float *eo = (float *)malloc(90 * 4);
        CHECK(orc_topk(en, lat, legal, n, 3, 30, ORC_SEL_THRESHOLD, 1.1f, 0, idx, eo, cnt) == ORC_OK);
        CHECK(orc_topk(en, lat, legal, n, 3, 7, ORC_SEL_THRESHOLD, INFINITY, 0, idx, eo, cnt) == ORC_OK);
        CHECK(orc_topk(en, lat, legal, n, 1, 30, ORC_SEL_RANK, 0.0f, 40, idx, eo, cnt) == ORC_OK);
        CHECK(orc_topk(en, NULL, NULL, n, 90, 1, ORC_SEL_THRESHOLD, 1.1f, 0, idx, eo, cnt) == ORC_OK);
        CHECK(orc_topk(en, lat, NULL, n, 1, 90, ORC_SEL_RANK, 0.0f, 90, idx, eo, cnt) != 12345);
        free(en); free(lat); free(legal); free(idx); free(cnt); free(eo);
    }
    /* tree ensemble */
    {
        const int32_t F = 5, depth = 3, T = 4;
        const uint64_t n = 50, ld = 53;
        const uint32_t nodes = 7, leaves = 8;
        float *feat = (float *)malloc(F * ld * 4), *e = (float *)malloc(n * 4);
        for (uint64_t i = 0; i < F * ld; ++i) feat[i] = 40.0f * unit(&s);
        for (uint64_t i = 0; i < n; ++i) e[i] = 0.5f + feat[i] / 40.0f + 0.5f * feat[ld + i] / 40.0f;
        uint8_t *nf = (uint8_t *)malloc(T * nodes);
        float *nt = (float *)malloc(T * nodes * 4), *lf = (float *)malloc(T * leaves * 4);
        double snr, loss, *out = (double *)malloc(n * 8);
        CHECK(orc_trees_boost(F, depth, 0, 3, nf, nt, lf, 0.5, feat, ld, e, n, 0.3, 1.0, &snr, &loss) == ORC_OK);
        CHECK(snr == snr && loss == loss);
        e[7] = -1.0f;
        CHECK(orc_trees_boost(F, depth, 3, 1, nf, nt, lf, 0.5, feat, ld, e, n, 0.3, 1.0, &snr, &loss) == ORC_OK && snr != snr);
        CHECK(orc_trees_predict(F, depth, T, nf, nt, lf, 0.5, feat, ld, n, 0, out) == ORC_OK);
        CHECK(orc_trees_predict(F, depth, T, nf, nt, lf, 0.5, feat, ld, n, 1, out) == ORC_OK);
        free(feat); free(e); free(nf); free(nt); free(lf); free(out);
    }
    printf("sanitize_check ok\n");
    return 0;
}
