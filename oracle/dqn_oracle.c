/*
 * CPU oracle for the deep Q-learning minibatch training step (arxiv 1804.05834).
 *
 * THIS IS TEST INFRASTRUCTURE.  It is a plain, slow, obviously-correct
 * implementation that the GPU library is checked against.  It shares no code
 * with the GPU path and nothing in the product may call it.
 *
 * Arithmetic: parameters and inputs are fp32 (or uint8) values; every sum and
 * product is taken in double.  A value is rounded to fp32 only where the method
 * stores it as state: the parameters, the RMSProp accumulators and the
 * sum-tree nodes.
 *
 * Layouts (canonical, row-major):
 *   states      uint8 [n][4][84][84]
 *   activations double [n][C][H][W]
 *   conv weight float  [O][C][kh][kw]          (cross-correlation, no padding)
 *   fc weight   float  [out][in], fc1 input index = c*49 + h*7 + w
 *   parameter blob: conv1.W conv1.b conv2.W conv2.b conv3.W conv3.b fc1.W fc1.b
 *                   then  plain head : out.W[K][512] out.b[K]
 *                   or    dueling    : V.W[1][512] V.b[1] A.W[K][512] A.b[K]
 *
 * Reduced-precision mode (quant = 1): the throughput configuration computes with
 * "bf16 weights/activations, fp32 accumulation and fp32 master weights".  A ReLU
 * mask is a yes/no decision taken on a rounded number, so to compare gradients the
 * checker has to take those decisions on the same numbers: in this mode the conv
 * and fc1 weight matrices, the outputs of conv1-3 and the activation gradients
 * that flow back through fc1 and the convolutions are rounded to bf16
 * (round-to-nearest-even from the fp32 value); biases, the 512-unit hidden layer,
 * the head, all sums and the master parameters keep full precision.  Gradients
 * are taken at the rounded weights and applied to the master weights.
 *
 * Pins (tests/test_oracle_*.py): Eq.1 closed form, a brute-forced tabular MDP
 * for the targets, the Eq.13 identities, finite differences and an independent
 * autograd for the gradients, closed forms for RMSProp, exact integer
 * sum-trees and a brute-force cumulative-sum sampler.  The composed whole step
 * has no worked numeric example in the paper: "parity unpinned" beyond the
 * composition of those pins.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

#define IN_C 4
#define IN_H 84
#define IN_W 84
#define C1_O 32
#define C1_K 8
#define C1_S 4
#define C1_H 20
#define C2_O 64
#define C2_K 4
#define C2_S 2
#define C2_H 9
#define C3_O 64
#define C3_K 3
#define C3_S 1
#define C3_H 7
#define FC_IN (C3_O * C3_H * C3_H) /* 3136 */
#define FC_OUT 512

/* ------------------------------------------------------------------ */
/* bf16 rounding: the value is first an fp32 number (what an fp32 accumulator
 * holds), then rounded to the nearest bf16 (8 significant bits), ties to even. */
/* ------------------------------------------------------------------ */
double orc_round_bf16(double x)
{
    float f = (float)x;
    uint32_t u;
    memcpy(&u, &f, 4);
    if ((u & 0x7F800000u) == 0x7F800000u) return (double)f; /* inf / nan unchanged */
    u += 0x7FFFu + ((u >> 16) & 1u);
    u &= 0xFFFF0000u;
    memcpy(&f, &u, 4);
    return (double)f;
}

static void round_array_bf16(double *x, int64_t n)
{
    for (int64_t i = 0; i < n; ++i) x[i] = orc_round_bf16(x[i]);
}

/* ------------------------------------------------------------------ */
/* Counter-based draws.  A 64-bit mixer (the SplitMix64 output function
 * applied to seed + (ctr+1)*golden-gamma); the top 24 bits scaled by 2^-24
 * give a uniform in [0,1) that is exact in fp32.                       */
/* ------------------------------------------------------------------ */
uint64_t orc_mix64(uint64_t seed, uint64_t ctr)
{
    uint64_t z = seed + (ctr + 1u) * 0x9E3779B97F4A7C15ull;
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    return z ^ (z >> 31);
}

float orc_draw_u24(uint64_t seed, uint64_t ctr)
{
    return (float)(orc_mix64(seed, ctr) >> 40) * (1.0f / 16777216.0f);
}

/* ------------------------------------------------------------------ */
/* Eq.1: discounted return R_t = sum_{t'=t}^{T} gamma^(t'-t) r_t'.     */
/* ------------------------------------------------------------------ */
double orc_discounted_return(const double *r, int64_t n, double gamma)
{
    double ret = 0.0, g = 1.0;
    for (int64_t k = 0; k < n; ++k) {
        ret += g * r[k];
        g *= gamma;
    }
    return ret;
}

/* ------------------------------------------------------------------ */
/* Parameter blob bookkeeping (Section 3, the five layers).            */
/* ------------------------------------------------------------------ */
typedef struct {
    int64_t c1w, c1b, c2w, c2b, c3w, c3b, f1w, f1b;
    int64_t vw, vb; /* dueling only (else -1) */
    int64_t aw, ab; /* advantage stream, or the plain output layer */
    int64_t total;
} orc_layout;

static orc_layout make_layout(int K, int dueling)
{
    orc_layout L;
    int64_t o = 0;
    L.c1w = o; o += (int64_t)C1_O * IN_C * C1_K * C1_K;
    L.c1b = o; o += C1_O;
    L.c2w = o; o += (int64_t)C2_O * C1_O * C2_K * C2_K;
    L.c2b = o; o += C2_O;
    L.c3w = o; o += (int64_t)C3_O * C2_O * C3_K * C3_K;
    L.c3b = o; o += C3_O;
    L.f1w = o; o += (int64_t)FC_OUT * FC_IN;
    L.f1b = o; o += FC_OUT;
    if (dueling) {
        L.vw = o; o += FC_OUT;
        L.vb = o; o += 1;
    } else {
        L.vw = L.vb = -1;
    }
    L.aw = o; o += (int64_t)K * FC_OUT;
    L.ab = o; o += K;
    L.total = o;
    return L;
}

int64_t orc_param_count(int32_t K, int32_t dueling)
{
    return make_layout(K, dueling).total;
}

/* offsets of the 8 (plain) or 10 (dueling) tensors + total, for tests */
void orc_param_offsets(int32_t K, int32_t dueling, int64_t *out12)
{
    orc_layout L = make_layout(K, dueling);
    out12[0] = L.c1w; out12[1] = L.c1b; out12[2] = L.c2w; out12[3] = L.c2b;
    out12[4] = L.c3w; out12[5] = L.c3b; out12[6] = L.f1w; out12[7] = L.f1b;
    out12[8] = L.vw;  out12[9] = L.vb;  out12[10] = L.aw; out12[11] = L.ab;
}

/* ------------------------------------------------------------------ */
/* Layers.  Convolution = cross-correlation, stride s, no padding:
 *   y[o,i,j] = b[o] + sum_{c,p,q} W[o,c,p,q] * x[c, i*s+p, j*s+q]     */
/* ------------------------------------------------------------------ */
static void conv_fwd(const double *x, int C, int H, int W, const float *w, const float *b,
                     int O, int k, int s, int relu, double *y)
{
    int OH = (H - k) / s + 1, OW = (W - k) / s + 1;
    for (int o = 0; o < O; ++o)
        for (int i = 0; i < OH; ++i)
            for (int j = 0; j < OW; ++j) {
                double acc = (double)b[o];
                for (int c = 0; c < C; ++c)
                    for (int p = 0; p < k; ++p)
                        for (int q = 0; q < k; ++q)
                            acc += (double)w[((o * C + c) * k + p) * k + q] *
                                   x[(c * H + i * s + p) * W + j * s + q];
                if (relu && acc < 0.0) acc = 0.0;
                y[(o * OH + i) * OW + j] = acc;
            }
}

/* dy is the gradient w.r.t. the conv output BEFORE any activation.
 * dx (may be NULL) is overwritten; dw, db are accumulated into.       */
static void conv_bwd(const double *x, int C, int H, int W, const float *w, int O, int k, int s,
                     const double *dy, double *dx, double *dw, double *db)
{
    int OH = (H - k) / s + 1, OW = (W - k) / s + 1;
    if (dx) memset(dx, 0, sizeof(double) * C * H * W);
    for (int o = 0; o < O; ++o)
        for (int i = 0; i < OH; ++i)
            for (int j = 0; j < OW; ++j) {
                double g = dy[(o * OH + i) * OW + j];
                if (g == 0.0) continue;
                db[o] += g;
                for (int c = 0; c < C; ++c)
                    for (int p = 0; p < k; ++p)
                        for (int q = 0; q < k; ++q) {
                            int wi = ((o * C + c) * k + p) * k + q;
                            int xi = (c * H + i * s + p) * W + j * s + q;
                            dw[wi] += g * x[xi];
                            if (dx) dx[xi] += g * (double)w[wi];
                        }
            }
}

static void fc_fwd(const double *x, int nin, const float *w, const float *b, int nout, int relu,
                   double *y)
{
    for (int o = 0; o < nout; ++o) {
        double acc = (double)b[o];
        for (int i = 0; i < nin; ++i) acc += (double)w[(int64_t)o * nin + i] * x[i];
        if (relu && acc < 0.0) acc = 0.0;
        y[o] = acc;
    }
}

static void fc_bwd(const double *x, int nin, const float *w, int nout, const double *dy,
                   double *dx, double *dw, double *db)
{
    if (dx) memset(dx, 0, sizeof(double) * nin);
    for (int o = 0; o < nout; ++o) {
        double g = dy[o];
        if (g == 0.0) continue;
        db[o] += g;
        for (int i = 0; i < nin; ++i) {
            dw[(int64_t)o * nin + i] += g * x[i];
            if (dx) dx[i] += g * (double)w[(int64_t)o * nin + i];
        }
    }
}

/* per-sample activation record */
typedef struct {
    double x0[IN_C * IN_H * IN_W];
    double a1[C1_O * C1_H * C1_H];
    double a2[C2_O * C2_H * C2_H];
    double a3[FC_IN];
    double h[FC_OUT];
    double adv[64]; /* A stream (or plain Q) */
    double v;
} orc_acts;

/* Forward of one sample (Section 3 layer list; ReLU after conv1-3 and fc1,
 * linear output; Eq.13 for the dueling head with both streams reading the
 * same 512-unit hidden layer).                                         */
static void net_forward_one(const float *P, const orc_layout *L, int K, int dueling, int quant,
                            const uint8_t *s, orc_acts *A, double *q)
{
    for (int i = 0; i < IN_C * IN_H * IN_W; ++i) A->x0[i] = (double)s[i] / 255.0;
    conv_fwd(A->x0, IN_C, IN_H, IN_W, P + L->c1w, P + L->c1b, C1_O, C1_K, C1_S, 1, A->a1);
    if (quant) round_array_bf16(A->a1, C1_O * C1_H * C1_H);
    conv_fwd(A->a1, C1_O, C1_H, C1_H, P + L->c2w, P + L->c2b, C2_O, C2_K, C2_S, 1, A->a2);
    if (quant) round_array_bf16(A->a2, C2_O * C2_H * C2_H);
    conv_fwd(A->a2, C2_O, C2_H, C2_H, P + L->c3w, P + L->c3b, C3_O, C3_K, C3_S, 1, A->a3);
    if (quant) round_array_bf16(A->a3, FC_IN);
    fc_fwd(A->a3, FC_IN, P + L->f1w, P + L->f1b, FC_OUT, 1, A->h);
    fc_fwd(A->h, FC_OUT, P + L->aw, P + L->ab, K, 0, A->adv);
    if (dueling) {
        fc_fwd(A->h, FC_OUT, P + L->vw, P + L->vb, 1, 0, &A->v);
        double mean = 0.0;
        for (int a = 0; a < K; ++a) mean += A->adv[a];
        mean /= (double)K;
        for (int a = 0; a < K; ++a) q[a] = A->v + (A->adv[a] - mean);
    } else {
        A->v = 0.0;
        for (int a = 0; a < K; ++a) q[a] = A->adv[a];
    }
}

/* Copy of a parameter blob with the conv1-3 and fc1 weight matrices rounded to
 * bf16 (reduced-precision mode); biases and the head are copied unchanged.   */
static float *quantized_copy(const float *P, const orc_layout *L)
{
    float *Q = (float *)malloc(sizeof(float) * (size_t)L->total);
    if (!Q) return NULL;
    memcpy(Q, P, sizeof(float) * (size_t)L->total);
    const int64_t beg[4] = {L->c1w, L->c2w, L->c3w, L->f1w};
    const int64_t end[4] = {L->c1b, L->c2b, L->c3b, L->f1b};
    for (int t = 0; t < 4; ++t)
        for (int64_t i = beg[t]; i < end[t]; ++i) Q[i] = (float)orc_round_bf16((double)P[i]);
    return Q;
}

/* Q-values of n states.  q: double [n][K].  hidden (may be NULL): [n][512].
 * quant: 0 full precision / 1 reduced-precision mode (see the file header).  */
int32_t orc_forward_q(const float *params, int32_t K, int32_t dueling, int32_t quant,
                      const uint8_t *states, int64_t n, double *q, double *hidden)
{
    if (K < 1 || K > 64) return -1;
    orc_layout L = make_layout(K, dueling);
    float *Pq = quant ? quantized_copy(params, &L) : NULL;
    if (quant && !Pq) return -2;
    if (quant) params = Pq;
    int fail = 0;
#pragma omp parallel for schedule(dynamic, 1)
    for (int64_t j = 0; j < n; ++j) {
        orc_acts *A = (orc_acts *)malloc(sizeof(orc_acts));
        if (!A) { fail = 1; continue; }
        net_forward_one(params, &L, K, dueling, quant, states + j * (IN_C * IN_H * IN_W), A, q + j * K);
        if (hidden) memcpy(hidden + j * FC_OUT, A->h, sizeof(double) * FC_OUT);
        free(A);
    }
    free(Pq);
    return fail ? -2 : 0;
}

/* The layer outputs of n states (after ReLU; conv outputs [C][H][W] per state):
 * a1 [n][32][20][20], a2 [n][64][9][9], a3 [n][64][7][7], h [n][512]; any may be
 * NULL.  Same arithmetic as orc_forward_q (it calls the same per-sample forward). */
int32_t orc_forward_acts(const float *params, int32_t K, int32_t dueling, int32_t quant,
                         const uint8_t *states, int64_t n, double *a1, double *a2, double *a3,
                         double *h)
{
    if (K < 1 || K > 64) return -1;
    orc_layout L = make_layout(K, dueling);
    float *Pq = quant ? quantized_copy(params, &L) : NULL;
    if (quant && !Pq) return -2;
    if (quant) params = Pq;
    int fail = 0;
#pragma omp parallel for schedule(dynamic, 1)
    for (int64_t j = 0; j < n; ++j) {
        orc_acts *A = (orc_acts *)malloc(sizeof(orc_acts));
        double q[64];
        if (!A) { fail = 1; continue; }
        net_forward_one(params, &L, K, dueling, quant, states + j * (IN_C * IN_H * IN_W), A, q);
        if (a1) memcpy(a1 + j * (C1_O * C1_H * C1_H), A->a1, sizeof(A->a1));
        if (a2) memcpy(a2 + j * (C2_O * C2_H * C2_H), A->a2, sizeof(A->a2));
        if (a3) memcpy(a3 + j * FC_IN, A->a3, sizeof(A->a3));
        if (h) memcpy(h + j * FC_OUT, A->h, sizeof(A->h));
        free(A);
    }
    free(Pq);
    return fail ? -2 : 0;
}

int32_t orc_forward(const float *params, int32_t K, int32_t dueling, const uint8_t *states,
                    int64_t n, double *q, double *hidden)
{
    return orc_forward_q(params, K, dueling, 0, states, n, q, hidden);
}

/* argmax with the lowest index winning ties */
static int argmax_low(const double *q, int K)
{
    int best = 0;
    for (int a = 1; a < K; ++a)
        if (q[a] > q[best]) best = a;
    return best;
}

/* ------------------------------------------------------------------ */
/* Targets and loss (Eq.7-9, Alg.1 target lines).
 *   a*  = argmax_a Q_online(s',a)   (double_q, Eq.9)
 *         argmax_a Q_target(s',a)   (Eq.8)
 *   y   = r + gamma (1-done) Q_target(s',a*)
 *   td  = y - Q_online(s,a)
 *   l   = 0.5 td^2                         (loss_kind 0, matches Eq.7)
 *         0.5 td^2 if |td|<=kappa else kappa(|td|-0.5 kappa)   (loss_kind 1)
 *   L   = (1/B) sum_j w_j l_j
 *   dL/dQ(s_j,a) = -(1/B) w_j clip(td_j,-kappa,kappa) [a==a_j]   (no clip for kind 0)
 * w may be NULL (all ones).  dq (may be NULL): double [B][K].          */
/* ------------------------------------------------------------------ */
int32_t orc_target_loss(int32_t B, int32_t K, int32_t double_q, int32_t loss_kind, double kappa,
                        double gamma, const double *q_s, const double *q_next_online,
                        const double *q_next_target, const int32_t *a, const float *r,
                        const uint8_t *done, const float *w, int32_t *a_star, double *y,
                        double *td, double *loss, double *dq)
{
    double total = 0.0;
    for (int j = 0; j < B; ++j) {
        if (a[j] < 0 || a[j] >= K) return -1;
        const double *sel = double_q ? q_next_online + (int64_t)j * K : q_next_target + (int64_t)j * K;
        int as = argmax_low(sel, K);
        double boot = done[j] ? 0.0 : gamma * q_next_target[(int64_t)j * K + as];
        double yj = (double)r[j] + boot;
        double d = yj - q_s[(int64_t)j * K + a[j]];
        double wj = w ? (double)w[j] : 1.0;
        double l, dl; /* dl = d l / d td */
        if (loss_kind == 1 && fabs(d) > kappa) {
            l = kappa * (fabs(d) - 0.5 * kappa);
            dl = d > 0 ? kappa : -kappa;
        } else {
            l = 0.5 * d * d;
            dl = d;
        }
        total += wj * l;
        if (a_star) a_star[j] = as;
        if (y) y[j] = yj;
        if (td) td[j] = d;
        if (dq) {
            for (int k = 0; k < K; ++k) dq[(int64_t)j * K + k] = 0.0;
            dq[(int64_t)j * K + a[j]] = -wj * dl / (double)B;
        }
    }
    if (loss) *loss = total / (double)B;
    return 0;
}

/* ------------------------------------------------------------------ */
/* RMSProp (named in Table 1; form: v <- rho v + (1-rho) g^2,
 * theta <- theta - lr g / sqrt(v + eps); centered variant keeps
 * m <- rho m + (1-rho) g and uses sqrt(v - m^2 + eps)).
 * theta, v, m are fp32 state; the arithmetic is double.               */
/* ------------------------------------------------------------------ */
void orc_rmsprop(int64_t n, float *theta, float *v, float *m, const double *g, double lr,
                 double rho, double eps, int32_t centered)
{
    for (int64_t i = 0; i < n; ++i) {
        double vi = rho * (double)v[i] + (1.0 - rho) * g[i] * g[i];
        float vf = (float)vi;
        double denom;
        if (centered) {
            double mi = rho * (double)m[i] + (1.0 - rho) * g[i];
            float mf = (float)mi;
            m[i] = mf;
            denom = sqrt((double)vf - (double)mf * (double)mf + eps);
        } else {
            denom = sqrt((double)vf + eps);
        }
        v[i] = vf;
        theta[i] = (float)((double)theta[i] - lr * g[i] / denom);
    }
}

/* ------------------------------------------------------------------ */
/* Whole training step on an explicit minibatch.                       */
/* ------------------------------------------------------------------ */
typedef struct {
    int32_t num_actions, dueling, double_q, loss_kind;
    double huber_delta, gamma, lr, rms_decay, rms_eps;
    int32_t rms_centered;
    int32_t quant; /* 0 full precision / 1 reduced-precision mode (see the file header) */
} orc_config;

/* Gradient of L w.r.t. all online parameters: forward on s (online),
 * forward on s' (online and target), targets+loss, exact reverse mode.
 * grads: double [param_count], overwritten.  All q_* / y / td / a_star /
 * loss outputs may be NULL.                                            */
int32_t orc_loss_grad(const orc_config *cfg, int32_t B, const float *theta,
                      const float *theta_target, const uint8_t *s, const uint8_t *s_next,
                      const int32_t *a, const float *r, const uint8_t *done, const float *w,
                      double *q_s, double *q_next_online, double *q_next_target,
                      int32_t *a_star, double *y, double *td, double *loss, double *grads)
{
    int K = cfg->num_actions, due = cfg->dueling;
    if (K < 1 || K > 64 || B < 1) return -1;
    orc_layout L = make_layout(K, due);
    const int64_t SS = IN_C * IN_H * IN_W;

    double *qs = (double *)malloc(sizeof(double) * (size_t)B * K * 4);
    orc_acts *acts = (orc_acts *)malloc(sizeof(orc_acts) * (size_t)B);
    if (!qs || !acts) { free(qs); free(acts); return -2; }
    double *qno = qs + (size_t)B * K, *qnt = qno + (size_t)B * K, *dq = qnt + (size_t)B * K;
    /* the weights the network computes with: the parameters themselves, or
     * their bf16-rounded copies in reduced-precision mode */
    const int quant = cfg->quant;
    float *Wq = quant ? quantized_copy(theta, &L) : NULL;
    float *Wtq = quant ? quantized_copy(theta_target, &L) : NULL;
    if (quant && (!Wq || !Wtq)) { free(qs); free(acts); free(Wq); free(Wtq); return -2; }
    const float *W = quant ? Wq : theta, *Wt = quant ? Wtq : theta_target;

#pragma omp parallel for schedule(dynamic, 1)
    for (int j = 0; j < B; ++j) {
        orc_acts *tmp = (orc_acts *)malloc(sizeof(orc_acts));
        net_forward_one(W, &L, K, due, quant, s + j * SS, &acts[j], qs + (int64_t)j * K);
        net_forward_one(W, &L, K, due, quant, s_next + j * SS, tmp, qno + (int64_t)j * K);
        net_forward_one(Wt, &L, K, due, quant, s_next + j * SS, tmp, qnt + (int64_t)j * K);
        free(tmp);
    }
    int32_t rc = orc_target_loss(B, K, cfg->double_q, cfg->loss_kind, cfg->huber_delta, cfg->gamma,
                                 qs, qno, qnt, a, r, done, w, a_star, y, td, loss, dq);
    if (rc) { free(qs); free(acts); free(Wq); free(Wtq); return rc; }
    if (q_s) memcpy(q_s, qs, sizeof(double) * (size_t)B * K);
    if (q_next_online) memcpy(q_next_online, qno, sizeof(double) * (size_t)B * K);
    if (q_next_target) memcpy(q_next_target, qnt, sizeof(double) * (size_t)B * K);

    if (grads) {
        memset(grads, 0, sizeof(double) * (size_t)L.total);
        /* Threads own contiguous runs of samples and accumulate into private
         * buffers, which are then added up in thread order. */
        int nthreads = 1;
#ifdef _OPENMP
        nthreads = omp_get_max_threads();
        if (nthreads > B) nthreads = B;
#endif
        double *priv = (double *)calloc((size_t)nthreads * (size_t)L.total, sizeof(double));
        if (!priv) { free(qs); free(acts); free(Wq); free(Wtq); return -2; }
#pragma omp parallel num_threads(nthreads)
        {
            int tid = 0;
#ifdef _OPENMP
            tid = omp_get_thread_num();
#endif
            double *G = priv + (size_t)tid * (size_t)L.total;
            double *dh = (double *)malloc(sizeof(double) * FC_OUT);
            double *dh2 = (double *)malloc(sizeof(double) * FC_OUT);
            double *d3 = (double *)malloc(sizeof(double) * FC_IN);
            double *d2 = (double *)malloc(sizeof(double) * C2_O * C2_H * C2_H);
            double *d1 = (double *)malloc(sizeof(double) * C1_O * C1_H * C1_H);
            /* static contiguous chunks: thread t owns samples [t*B/T, (t+1)*B/T) */
            int j0 = (int)((int64_t)tid * B / nthreads), j1 = (int)((int64_t)(tid + 1) * B / nthreads);
            for (int j = j0; j < j1; ++j) {
                const orc_acts *A = &acts[j];
                const double *dqj = dq + (int64_t)j * K;
                double dadv[64], dv = 0.0;
                if (due) {
                    /* Q_a = V + A_a - mean A  =>  dV = sum dQ, dA_a = dQ_a - mean dQ */
                    double sum = 0.0;
                    for (int k = 0; k < K; ++k) sum += dqj[k];
                    dv = sum;
                    for (int k = 0; k < K; ++k) dadv[k] = dqj[k] - sum / (double)K;
                } else {
                    for (int k = 0; k < K; ++k) dadv[k] = dqj[k];
                }
                fc_bwd(A->h, FC_OUT, W + L.aw, K, dadv, dh, G + L.aw, G + L.ab);
                if (due) {
                    fc_bwd(A->h, FC_OUT, W + L.vw, 1, &dv, dh2, G + L.vw, G + L.vb);
                    for (int i = 0; i < FC_OUT; ++i) dh[i] += dh2[i];
                }
                for (int i = 0; i < FC_OUT; ++i)
                    if (A->h[i] <= 0.0) dh[i] = 0.0;
                if (quant) round_array_bf16(dh, FC_OUT);
                fc_bwd(A->a3, FC_IN, W + L.f1w, FC_OUT, dh, d3, G + L.f1w, G + L.f1b);
                for (int i = 0; i < FC_IN; ++i)
                    if (A->a3[i] <= 0.0) d3[i] = 0.0;
                if (quant) round_array_bf16(d3, FC_IN);
                conv_bwd(A->a2, C2_O, C2_H, C2_H, W + L.c3w, C3_O, C3_K, C3_S, d3, d2,
                         G + L.c3w, G + L.c3b);
                for (int i = 0; i < C2_O * C2_H * C2_H; ++i)
                    if (A->a2[i] <= 0.0) d2[i] = 0.0;
                if (quant) round_array_bf16(d2, C2_O * C2_H * C2_H);
                conv_bwd(A->a1, C1_O, C1_H, C1_H, W + L.c2w, C2_O, C2_K, C2_S, d2, d1,
                         G + L.c2w, G + L.c2b);
                for (int i = 0; i < C1_O * C1_H * C1_H; ++i)
                    if (A->a1[i] <= 0.0) d1[i] = 0.0;
                if (quant) round_array_bf16(d1, C1_O * C1_H * C1_H);
                conv_bwd(A->x0, IN_C, IN_H, IN_W, W + L.c1w, C1_O, C1_K, C1_S, d1, NULL,
                         G + L.c1w, G + L.c1b);
            }
            free(dh); free(dh2); free(d3); free(d2); free(d1);
        }
        for (int t = 0; t < nthreads; ++t) {
            const double *G = priv + (size_t)t * (size_t)L.total;
            for (int64_t i = 0; i < L.total; ++i) grads[i] += G[i];
        }
        free(priv);
    }
    free(qs);
    free(acts);
    free(Wq);
    free(Wtq);
    return 0;
}

/* One full step: gradient, then RMSProp on theta / rms_v (/ rms_m).   */
int32_t orc_train_step(const orc_config *cfg, int32_t B, float *theta, const float *theta_target,
                       float *rms_v, float *rms_m, const uint8_t *s, const uint8_t *s_next,
                       const int32_t *a, const float *r, const uint8_t *done, const float *w,
                       double *q_s, double *q_next_online, double *q_next_target,
                       int32_t *a_star, double *y, double *td, double *loss, double *grads)
{
    int64_t n = orc_param_count(cfg->num_actions, cfg->dueling);
    double *g = grads ? grads : (double *)malloc(sizeof(double) * (size_t)n);
    if (!g) return -2;
    int32_t rc = orc_loss_grad(cfg, B, theta, theta_target, s, s_next, a, r, done, w, q_s,
                               q_next_online, q_next_target, a_star, y, td, loss, g);
    if (rc == 0)
        orc_rmsprop(n, theta, rms_v, rms_m, g, cfg->lr, cfg->rms_decay, cfg->rms_eps,
                    cfg->rms_centered);
    if (!grads) free(g);
    return rc;
}

/* ------------------------------------------------------------------ */
/* Acting (Alg.1, action-selection lines): per environment e,
 *   u = draw(seed, 2e); if u < epsilon: a = floor(draw(seed, 2e+1) * K)
 *   else a = argmax_a Q(obs_e, a), lowest index on ties.               */
/* ------------------------------------------------------------------ */
int32_t orc_act(const float *params, int32_t K, int32_t dueling, int32_t quant, const uint8_t *obs,
                int64_t E, double epsilon, uint64_t draw_seed, int32_t *actions, double *q)
{
    double *qq = q ? q : (double *)malloc(sizeof(double) * (size_t)E * K);
    if (!qq) return -2;
    int32_t rc = orc_forward_q(params, K, dueling, quant, obs, E, qq, NULL);
    if (rc == 0) {
        for (int64_t e = 0; e < E; ++e) {
            float u = orc_draw_u24(draw_seed, 2u * (uint64_t)e);
            if ((double)u < epsilon) {
                float u2 = orc_draw_u24(draw_seed, 2u * (uint64_t)e + 1u);
                int act = (int)floor((double)u2 * (double)K);
                actions[e] = act < K ? act : K - 1;
            } else {
                actions[e] = argmax_low(qq + e * K, K);
            }
        }
    }
    if (!q) free(qq);
    return rc;
}

/* ------------------------------------------------------------------ */
/* Prioritized replay (Eq.10-12, Alg.2 sampling / weighting / priority
 * lines) on a binary sum-tree stored as a heap: tree[1] is the root,
 * tree[2i], tree[2i+1] the children of i, leaves at tree[L .. 2L-1]
 * (L a power of two >= capacity), tree[0] unused (kept 0).
 * Leaves hold fp32(p^alpha); each internal node is fp32(left + right). */
/* ------------------------------------------------------------------ */
static float leaf_value(double p, double alpha) { return (float)pow(p, alpha); }

void orc_tree_build(const float *raw_p, int64_t n, int64_t L, double alpha, float *tree)
{
    tree[0] = 0.0f;
    for (int64_t i = 0; i < L; ++i) tree[L + i] = i < n ? leaf_value((double)raw_p[i], alpha) : 0.0f;
    for (int64_t i = L - 1; i >= 1; --i) tree[i] = tree[2 * i] + tree[2 * i + 1];
}

/* Prefix descent for one mass z; returns the leaf slot (not clamped).
 * Eq.10 gives a transition of priority zero the probability zero, and Eq.11's
 * small constant exists so that no stored transition has it; a leaf of value 0
 * is a slot that holds no drawable transition.  In exact arithmetic the
 * descent never enters a subtree whose sum is 0.  In fp32 it can: a parent is
 * the ROUNDED sum of its children, so z < parent does not imply
 * z - left < right, and fp32(u * total) can equal the total.  The rule
 * therefore turns left whenever nothing lies to the right (right == 0): with
 * a positive total every visited node then has a positive sum, and the leaf
 * reached is a stored transition with P(j) > 0 -- the rightmost one of the
 * subtree when z overshoots it.                                            */
static int64_t tree_descend(const float *tree, int64_t L, float z)
{
    int64_t node = 1;
    while (node < L) {
        float left = tree[2 * node], right = tree[2 * node + 1];
        if (z < left || right == 0.0f) {
            node = 2 * node;
        } else {
            z = z - left;
            node = 2 * node + 1;
        }
    }
    return node - L;
}

/* The descent alone, for given masses z (not clamped to the stored size). */
void orc_tree_descend(const float *tree, int64_t L, const float *z, int32_t n, int32_t *idx)
{
    for (int j = 0; j < n; ++j) idx[j] = (int32_t)tree_descend(tree, L, z[j]);
}

/* B draws.  n_stored = number of stored transitions (the N of Eq.12); the slots that may hold a
 * transition are [0, limit) (limit = n_stored for one stream written from slot 0; with many
 * environment streams, each in a sub-ring of its own, the stored transitions are not the first
 * n_stored slots).
 * independent: z = fp32(u_j * total); stratified: z = fp32((j+u_j)*fp32(total/B)).
 * w_j = (n_stored * P(j))^-beta, then divided by the maximum over the minibatch.
 * Returns -4 if the tree is empty (total <= 0).                        */
int32_t orc_per_sample_n(const float *tree, int64_t L, int64_t limit, int64_t n_stored, int32_t B,
                         double beta, uint64_t draw_seed, int32_t stratified, int32_t *idx, float *is_w,
                         float *z_out)
{
    float total = tree[1];
    if (!(total > 0.0f) || n_stored < 1 || limit < 1) return -4;
    float seg = total / (float)B;
    double wmax = 0.0;
    double *wr = (double *)malloc(sizeof(double) * (size_t)B);
    if (!wr) return -2;
    for (int j = 0; j < B; ++j) {
        float u = orc_draw_u24(draw_seed, (uint64_t)j);
        float z = stratified ? ((float)j + u) * seg : u * total;
        int64_t slot = tree_descend(tree, L, z);
        if (slot > limit - 1) slot = limit - 1;
        idx[j] = (int32_t)slot;
        if (z_out) z_out[j] = z;
        double P = (double)tree[L + slot] / (double)total;
        wr[j] = pow((double)n_stored * P, -beta);
        if (wr[j] > wmax) wmax = wr[j];
    }
    for (int j = 0; j < B; ++j) is_w[j] = (float)(wr[j] / wmax);
    free(wr);
    return 0;
}

int32_t orc_per_sample(const float *tree, int64_t L, int64_t size, int32_t B, double beta,
                       uint64_t draw_seed, int32_t stratified, int32_t *idx, float *is_w,
                       float *z_out)
{
    return orc_per_sample_n(tree, L, size, size, B, beta, draw_seed, stratified, idx, is_w, z_out);
}

/* Definitional sampler: smallest slot whose inclusive cumulative sum of the
 * leaves (in double) exceeds z (a slot with a zero leaf never is that slot).  Also returns the distance from z to the
 * nearest bucket boundary, so a caller can accept an off-by-a-bucket index
 * when z sits within rounding of that boundary.                         */
void orc_per_sample_cumsum(const float *tree, int64_t L, int64_t size, const float *z, int32_t B,
                           int32_t *idx, double *boundary_dist)
{
    for (int j = 0; j < B; ++j) {
        double c = 0.0, zz = (double)z[j], lo = 0.0;
        int64_t slot = -1, last = size - 1; /* last: the last slot with a non-zero leaf */
        for (int64_t i = 0; i < size; ++i) {
            if (tree[L + i] > 0.0f) last = i;
            lo = c;
            c += (double)tree[L + i];
            if (c > zz) { slot = i; break; }
        }
        if (slot < 0) { slot = last; } /* z at or beyond the exact total: the last drawable slot */
        idx[j] = (int32_t)slot;
        if (boundary_dist) {
            double d1 = fabs(zz - lo), d2 = fabs(c - zz);
            boundary_dist[j] = d1 < d2 ? d1 : d2;
        }
    }
}

/* Priority update: for j = 0..n-1 in order, leaf[idx_j] <- fp32((|td_j|+eps)^alpha)
 * and every ancestor is recomputed as left+right (so the last occurrence of a
 * repeated index wins).  max_p <- max(max_p, |td_j| + eps).  An entry whose
 * error is not finite is skipped (the paper does not consider it; a NaN
 * priority would poison every sum above it).                           */
int32_t orc_per_update(float *tree, int64_t L, int64_t size, const int32_t *idx, const float *td_abs,
                       int32_t n, double alpha, double eps, float *max_p)
{
    for (int j = 0; j < n; ++j) {
        if (idx[j] < 0 || idx[j] >= size) return -1;
        float p = (float)((double)fabsf(td_abs[j]) + eps);
        if (!isfinite(p)) continue;
        int64_t node = L + idx[j];
        tree[node] = leaf_value((double)p, alpha);
        for (node >>= 1; node >= 1; node >>= 1) tree[node] = tree[2 * node] + tree[2 * node + 1];
        if (max_p && p > *max_p) *max_p = p;
    }
    return 0;
}

/* ------------------------------------------------------------------ */
/* Frame-stack gather from a ring of single frames: transition i has
 * s = frames[(i-3..i) mod N], s' = frames[(i-2..i+1) mod N].           */
/* ------------------------------------------------------------------ */
void orc_gather(const uint8_t *frames, int64_t capacity, const int32_t *idx, int32_t B, uint8_t *s,
                uint8_t *s_next)
{
    const int64_t F = IN_H * IN_W;
    for (int j = 0; j < B; ++j)
        for (int k = 0; k < 5; ++k) {
            int64_t slot = (((int64_t)idx[j] - 3 + k) % capacity + capacity) % capacity;
            const uint8_t *src = frames + slot * F;
            if (k < 4) memcpy(s + ((int64_t)j * 4 + k) * F, src, (size_t)F);
            if (k > 0) memcpy(s_next + ((int64_t)j * 4 + k - 1) * F, src, (size_t)F);
        }
}

/* ------------------------------------------------------------------ */
/* Store path (Alg.1 "store transition"; Alg.2 "store transition ... with
 * maximal priority").  One environment stream; time step t goes to ring slot
 * t mod N and carries (x_t, a_t, r_t, done_t); transition i is
 * (s = frames i-3..i, a_i, r_i, s' = frames i-2..i+1).  Only the part that
 * decides what can be sampled is modelled here (frames themselves are a plain
 * copy): the done flags and the sum-tree.
 *
 * Written out one time step at a time.  When time step q lands in slot h:
 *   - transition h-1 becomes complete (its s' now ends in x_q).  It enters
 *     the tree with the maximal priority seen so far, leaf = fp32(max_p^alpha),
 *     unless its state stack would reach back before the stream's start
 *     (q-1 < 3) or across an episode end (done at i-3, i-2 or i-1): such a
 *     stack mixes two episodes, the paper does not say what the preprocessing
 *     does there, and the reading taken is that it is never sampled (leaf 0).
 *   - slot h itself (its transition waits for the next frame) and slots
 *     h+1 .. h+3, whose five-frame windows now mix the newest frames with the
 *     oldest: leaf 0.
 * Every ancestor is recomputed as left + right.                            */
/* ------------------------------------------------------------------ */
static void set_leaf(float *tree, int64_t L, int64_t slot, float v)
{
    int64_t node = L + slot;
    tree[node] = v;
    for (node >>= 1; node >= 1; node >>= 1) tree[node] = tree[2 * node] + tree[2 * node + 1];
}

void orc_replay_store(float *tree, int64_t L, int64_t capacity, int64_t *cursor, int64_t *seq,
                      uint8_t *done_ring, const uint8_t *done_new, int64_t n, double alpha, float max_p)
{
    for (int64_t t = 0; t < n; ++t) {
        const int64_t h = *cursor, q = *seq;
        done_ring[h] = done_new ? done_new[t] : 0;
        if (q >= 1) {
            const int64_t i = (h - 1 + capacity) % capacity;
            int valid = q - 1 >= 3;
            for (int k = 1; k <= 3 && valid; ++k)
                if (done_ring[((i - k) % capacity + capacity) % capacity]) valid = 0;
            set_leaf(tree, L, i, valid ? leaf_value((double)max_p, alpha) : 0.0f);
        }
        for (int k = 0; k < 4; ++k) set_leaf(tree, L, (h + k) % capacity, 0.0f);
        *cursor = (h + 1) % capacity;
        *seq = q + 1;
    }
}

/* ------------------------------------------------------------------ */
/* Schedules of Table 1, as functions of the environment step t = 1, 2, ...:
 * a value that goes "a -> b (1 -> T steps)" is a at t = 1, b at t >= T and
 * linear in between; an update happens when t is past the learning start and
 * t = 0 mod the update period (Alg.2 "if t = 0 mod K"); the target network is
 * copied when t = 0 mod the target period.                                */
/* ------------------------------------------------------------------ */
typedef struct {
    int64_t learning_start, update_period, target_period, eps_steps, beta_steps;
    double eps_start, eps_end, beta_start, beta_end;
} orc_schedule;

static double ramp(double a, double b, int64_t t, int64_t T)
{
    if (T <= 1 || t >= T) return b;
    if (t <= 1) return a;
    return a + (b - a) * (double)(t - 1) / (double)(T - 1);
}

void orc_schedule_at(const orc_schedule *s, int64_t t, double *epsilon, double *beta, int32_t *train,
                     int32_t *sync_target)
{
    *epsilon = ramp(s->eps_start, s->eps_end, t, s->eps_steps);
    *beta = ramp(s->beta_start, s->beta_end, t, s->beta_steps);
    *train = t > s->learning_start && t % s->update_period == 0;
    *sync_target = t % s->target_period == 0;
}

/* ------------------------------------------------------------------ */
/* Frame preprocessing (Sec.3: palette frame -> grey-scale -> linear
 * interpolation to 84 x 84).  raw: [n][H][W] bytes; grey(y,x) = lut[raw] if a
 * 256-entry table is given (the emulator's palette -> luminance map, which the
 * paper does not print), else the byte itself.  Output pixel (i,j) samples
 * the source at the centre-aligned coordinate
 *     sy = (i + 1/2) H/84 - 1/2,   sx = (j + 1/2) W/84 - 1/2
 * (the convention of library "linear" resizing), clamped to the image, and
 * blends the four neighbours bilinearly; the result is rounded to the
 * nearest integer (ties to even) and clipped to 0..255.  val (optional)
 * receives the unrounded value.  Pinned against a library bilinear resize
 * and closed forms; parity with OpenCV's own fixed-point rounding (the
 * library the paper names) is unpinned: it is not available here.       */
/* ------------------------------------------------------------------ */
void orc_preprocess(const uint8_t *raw, int64_t n, int32_t H, int32_t W, const float *lut, uint8_t *out,
                    double *val)
{
    for (int64_t f = 0; f < n; ++f)
        for (int i = 0; i < IN_H; ++i)
            for (int j = 0; j < IN_W; ++j) {
                double sy = (i + 0.5) * (double)H / IN_H - 0.5, sx = (j + 0.5) * (double)W / IN_W - 0.5;
                if (sy < 0) sy = 0;
                if (sx < 0) sx = 0;
                if (sy > H - 1) sy = H - 1;
                if (sx > W - 1) sx = W - 1;
                int y0 = (int)floor(sy), x0 = (int)floor(sx);
                int y1 = y0 + 1 < H ? y0 + 1 : H - 1, x1 = x0 + 1 < W ? x0 + 1 : W - 1;
                double fy = sy - y0, fx = sx - x0;
                const uint8_t *im = raw + f * (int64_t)H * W;
#define GREY(y, x) (lut ? (double)lut[im[(int64_t)(y) * W + (x)]] : (double)im[(int64_t)(y) * W + (x)])
                double top = GREY(y0, x0) * (1 - fx) + GREY(y0, x1) * fx;
                double bot = GREY(y1, x0) * (1 - fx) + GREY(y1, x1) * fx;
#undef GREY
                double v = top * (1 - fy) + bot * fy;
                double r = rint(v);
                if (r < 0) r = 0;
                if (r > 255) r = 255;
                int64_t o = (f * IN_H + i) * IN_W + j;
                out[o] = (uint8_t)r;
                if (val) val[o] = v;
            }
}
