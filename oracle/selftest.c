/* Memory-safety self-test of the CPU oracle (test infrastructure only).
 *
 * Built with -fsanitize=address,undefined by tests/test_oracle_sanitize.py and run as a
 * separate process: every entry point is called once on small inputs whose buffers are sized
 * exactly, so an out-of-bounds access, a misaligned or overflowing operation aborts the run.
 * It checks no values (the pins do that); it returns 0 when every call returned normally. */
#include "dqn_oracle.c"

#include <stdio.h>

static uint64_t rs = 88172645463325252ull;
static uint32_t rnd(void) { rs ^= rs << 13; rs ^= rs >> 7; rs ^= rs << 17; return (uint32_t)(rs >> 11); }

int main(void)
{
    const int K = 5, dueling = 1, B = 3;
    const int64_t n = orc_param_count(K, dueling);
    float *theta = malloc(n * sizeof(float)), *target = malloc(n * sizeof(float));
    float *v = calloc(n, sizeof(float)), *m = calloc(n, sizeof(float));
    double *grads = malloc(n * sizeof(double));
    for (int64_t i = 0; i < n; ++i) {
        theta[i] = ((float)(rnd() % 2001) - 1000.f) * 2e-5f;
        target[i] = ((float)(rnd() % 2001) - 1000.f) * 2e-5f;
    }
    const size_t SB = (size_t)B * IN_C * IN_H * IN_W;
    uint8_t *s = malloc(SB), *sn = malloc(SB);
    for (size_t i = 0; i < SB; ++i) { s[i] = (uint8_t)rnd(); sn[i] = (uint8_t)rnd(); }
    int32_t a[3] = {0, 4, 2}, a_star[3];
    float r[3] = {-1.f, 0.f, 1.f}, w[3] = {1.f, 0.5f, 0.25f};
    uint8_t done[3] = {0, 1, 0};
    double q[3 * 5], qn[3 * 5], qt[3 * 5], y[3], td[3], loss, hid[3 * 512];
    int rc = 0;

    rc |= orc_forward_q(theta, K, dueling, 0, s, B, q, hid);
    rc |= orc_forward_q(theta, K, dueling, 1, s, B, q, NULL);
    for (int quant = 0; quant < 2; ++quant)
        for (int centered = 0; centered < 2; ++centered) {
            orc_config cfg = {K, dueling, 1, 1, 1.0, 0.99, 2.5e-4, 0.95, 0.01, centered, quant};
            rc |= orc_train_step(&cfg, B, theta, target, v, centered ? m : NULL, s, sn, a, r, done, w, q, qn, qt,
                                 a_star, y, td, &loss, grads);
        }
    {
        orc_config cfg = {4, 0, 0, 0, 1.0, 0.99, 2.5e-4, 0.95, 0.01, 0, 0};  /* plain head, Eq.8, squared loss */
        const int64_t n4 = orc_param_count(4, 0);
        int32_t a4[3] = {0, 3, 1};
        rc |= n4 > n;
        rc |= orc_train_step(&cfg, B, theta, target, v, NULL, s, sn, a4, r, done, NULL, q, qn, qt, a_star, y, td,
                             &loss, grads);
    }
    {
        int32_t acts[3];
        double qa[3 * 5];
        rc |= orc_act(theta, K, dueling, 0, s, B, 0.3, 77, acts, qa);
    }
    {   /* sum-tree: a capacity that is not a power of two */
        const int64_t cap = 37, L = 64;
        float raw[37], *tree = malloc(2 * L * sizeof(float)), is_w[16], z[16], maxp = 1.f;
        int32_t idx[16];
        double dist[16];
        for (int i = 0; i < cap; ++i) raw[i] = 0.01f + (float)(rnd() % 1000) * 1e-3f;
        orc_tree_build(raw, cap, L, 0.6, tree);
        rc |= orc_per_sample(tree, L, cap, 16, 0.4, 5, 0, idx, is_w, z);
        rc |= orc_per_sample(tree, L, cap, 16, 0.4, 5, 1, idx, is_w, z);
        orc_tree_descend(tree, L, z, 16, idx);
        orc_per_sample_cumsum(tree, L, cap, z, 16, idx, dist);
        float tdv[16];
        for (int i = 0; i < 16; ++i) tdv[i] = (float)(rnd() % 100) * 0.03f;
        tdv[3] = NAN;
        rc |= orc_per_update(tree, L, cap, idx, tdv, 16, 0.6, 1e-6, &maxp);
        /* store path across a wrap, with episode ends */
        int64_t cursor = 0, seq = 0;
        uint8_t ring_done[37] = {0}, dn[100];
        for (int i = 0; i < 100; ++i) dn[i] = rnd() % 11 == 0;
        orc_tree_build(raw, 0, L, 0.6, tree);
        orc_replay_store(tree, L, cap, &cursor, &seq, ring_done, dn, 100, 0.6, maxp);
        rc |= !(tree[1] >= 0.f) || cursor != 100 % cap || seq != 100;
        free(tree);
    }
    {   /* gather across the ring ends */
        const int64_t cap = 6, F = IN_H * IN_W;
        uint8_t *ring = malloc(cap * F), *gs = malloc(2 * 4 * F), *gn = malloc(2 * 4 * F);
        for (int64_t i = 0; i < cap * F; ++i) ring[i] = (uint8_t)rnd();
        int32_t gi[2] = {0, 5};
        orc_gather(ring, cap, gi, 2, gs, gn);
        free(ring); free(gs); free(gn);
    }
    {   /* preprocessing: odd sizes, with and without a grey table */
        const int H = 53, W = 211;
        uint8_t *raw = malloc(2 * H * W), *out = malloc(2 * IN_H * IN_W);
        double *val = malloc(2 * IN_H * IN_W * sizeof(double));
        float lut[256];
        for (int i = 0; i < 2 * H * W; ++i) raw[i] = (uint8_t)rnd();
        for (int i = 0; i < 256; ++i) lut[i] = (float)(255 - i);
        orc_preprocess(raw, 2, H, W, lut, out, val);
        orc_preprocess(raw, 2, H, W, NULL, out, NULL);
        free(raw); free(out); free(val);
    }
    {
        orc_schedule sc = {50000, 4, 30000, 5000000, 100000000, 1.0, 0.1, 0.4, 1.0};
        double e, b;
        int32_t tr, sy;
        orc_schedule_at(&sc, 1, &e, &b, &tr, &sy);
        orc_schedule_at(&sc, 123456789, &e, &b, &tr, &sy);
        double rw[4] = {1.0, 0.0, -1.0, 1.0};
        rc |= !(orc_discounted_return(rw, 4, 0.99) == orc_discounted_return(rw, 4, 0.99));
    }
    free(theta); free(target); free(v); free(m); free(grads); free(s); free(sn);
    printf(rc ? "selftest: a call failed (rc %d)\n" : "selftest: ok\n", rc);
    return rc ? 1 : 0;
}
