/*
 * libdqn: the minibatch training step of deep Q-learning (DQN / Double DQN /
 * dueling head / proportional prioritized replay) for one AMD MI355X (gfx950),
 * as described in arxiv 1804.05834 (Sections 2.2-2.5, Section 3, Table 1).
 *
 * C ABI.  Every function returns an int32 status (0 = ok, negative = error) and
 * never throws.  On error no output buffer has been written by that call and
 * dqn_last_error() describes the cause.
 *
 * Pointers: unless a parameter says "host", every data pointer is a HIP DEVICE
 * pointer, 256-byte aligned, owned by the caller for the lifetime of the
 * context.  `stream` is a hipStream_t passed as void* (NULL = the null stream).
 * Calls enqueue work on that stream and return without synchronising; scalar
 * results land in caller-supplied device memory.  A context must not be used
 * from two streams at once.
 *
 * Actions are 0-based int32 in [0, num_actions) (the paper's set {1..K},
 * Section 2.1).  States are uint8 [4][84][84] stacks of grey frames
 * (Section 3); the network sees x = uint8 / 255.
 *
 * Canonical parameter blob (what dqn_get_params / dqn_set_params exchange;
 * fp32, concatenated, row-major), following the layer list of Section 3:
 *   conv1.W[32][4][8][8] conv1.b[32]  conv2.W[64][32][4][4] conv2.b[64]
 *   conv3.W[64][64][3][3] conv3.b[64] fc1.W[512][3136] fc1.b[512]
 *     (fc1 input index = c*49 + h*7 + w)
 *   plain head  : out.W[K][512] out.b[K]
 *   dueling head: V.W[1][512] V.b[1] A.W[K][512] A.b[K]          (Eq.13)
 * The library keeps its parameter buffers in an internal (channel-last)
 * permutation of this blob; only get/set translate.
 */
#ifndef DQN_H_
#define DQN_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum {
    DQN_OK = 0,
    DQN_ERR_INVALID_ARG = -1, /* NULL / misaligned pointer, size out of range      */
    DQN_ERR_OOM = -2,         /* host allocation failed                            */
    DQN_ERR_HIP = -3,         /* a HIP runtime call failed                         */
    DQN_ERR_STATE = -4,       /* e.g. sampling before any priority was stored      */
    DQN_ERR_UNSUPPORTED = -5  /* valid request this build does not implement       */
};

typedef struct dqn_ctx dqn_ctx;

/* All fields are explicit; there are no hidden defaults (Table 1 values in
 * brackets are what the paper's benchmark uses). */
typedef struct {
    int32_t num_actions;   /* K, 1..64                                              */
    int32_t dueling;       /* 0 plain output layer / 1 dueling head (Eq.13)         */
    int32_t double_q;      /* 0 target of Eq.8 / 1 Double-DQN target of Eq.9        */
    int32_t precision;     /* 0 fp32 / 1 bf16 compute with fp32 master + accumulate */
    int32_t loss_kind;     /* 0 = 0.5*td^2 (Eq.7) / 1 = Huber                       */
    float huber_delta;     /* Huber threshold [1]                                   */
    float gamma;           /* discount [0.99]                                       */
    float lr;              /* RMSProp step size                                     */
    float rms_decay;       /* RMSProp rho                                           */
    float rms_eps;         /* RMSProp epsilon (inside the square root)              */
    int32_t rms_centered;  /* 1 = subtract the squared running mean of g            */
    int32_t max_batch;     /* largest B of dqn_train_step, 1..1024                  */
    int32_t max_act_batch; /* largest E of dqn_act, 1..8192                         */
    int32_t per_stratified;/* 0 independent draws (Alg.2) / 1 one draw per stratum  */
    int64_t replay_capacity; /* N frames/transitions in the ring [1,000,000]; 0 = none */
    float per_alpha;       /* prioritisation exponent of Eq.10 [0.6]                */
    float per_eps;         /* the small constant of Eq.11                           */
    uint64_t seed;         /* online-network initialisation stream                  */
    uint64_t target_seed;  /* target-network initialisation stream                  */
} dqn_config;

/* Byte sizes of the caller-owned device buffers for a configuration.  A size
 * of 0 means the buffer is not used and its pointer may be NULL. */
typedef struct {
    size_t params;        /* ONE network's fp32 parameters (online, target: each)  */
    size_t opt_state;     /* RMSProp accumulators                                  */
    size_t shadow_bf16;   /* bf16 copies of both networks (precision 1)            */
    size_t grads;         /* fp32 gradient of the last step                        */
    size_t replay_frames; /* uint8 [capacity][84][84]                              */
    size_t replay_meta;   /* action / reward / terminal flag per slot              */
    size_t tree;          /* sum-tree: float [2L] heap + 64 floats of state        */
    size_t workspace;     /* activations, partial sums, minibatch staging          */
    int64_t param_count;  /* number of fp32 parameters of one network              */
    int64_t tree_leaves;  /* L = capacity rounded up to a power of two             */
} dqn_sizes;

typedef struct {
    void *online, *target, *opt_state, *shadow_bf16, *grads;
    void *replay_frames, *replay_meta, *tree, *workspace;
} dqn_buffers;

/* An explicit minibatch (Alg.1 "sample random minibatch"): B transitions. */
typedef struct {
    const uint8_t *s;      /* [B][4][84][84]                                         */
    const uint8_t *s_next; /* [B][4][84][84]                                         */
    const int32_t *a;      /* [B]                                                    */
    const float *r;        /* [B]                                                    */
    const uint8_t *done;   /* [B] 1 = s_next is terminal                             */
    const float *w;        /* [B] importance weights, or NULL = all 1                */
} dqn_batch;

/* Optional per-step outputs; any member may be NULL. */
typedef struct {
    float *loss;          /* [1]    (1/B) sum_j w_j l(td_j)                          */
    float *q_s;           /* [B][K] Q(s_j, . ; theta)                                */
    float *q_next_online; /* [B][K] Q(s'_j, . ; theta)                               */
    float *q_next_target; /* [B][K] Q(s'_j, . ; theta^-)                             */
    float *y;             /* [B]    targets (Eq.8 / Eq.9, y = r for terminal s')     */
    float *td;            /* [B]    y_j - Q(s_j, a_j; theta)                         */
    int32_t *a_star;      /* [B]    the action the target bootstraps from            */
    int32_t *idx;         /* [B]    sampled replay slots (replay mode only)          */
    float *is_w;          /* [B]    importance weights used                          */
    float *td_abs_mean;   /* [1]    (1/B) sum_j |td_j| (rows with a finite error)    */
    float *q_max_mean;    /* [1]    (1/B) sum_j max_a Q(s_j, a; theta)               */
} dqn_step_out;

/* Sizes of every buffer dqn_init needs.  `cfg`, `out`: host pointers. */
int32_t dqn_query_sizes(const dqn_config *cfg, dqn_sizes *out);

/* Creates a context over caller-owned device buffers (sizes from
 * dqn_query_sizes), initialises the online and target parameters on the host
 * (Alg.1 "random weights": uniform in +-sqrt(6/fan_in) from the counter-based
 * draws of cfg->seed / cfg->target_seed, biases 0), zeroes the optimizer state
 * and empties the replay.  `out`, `cfg`, `bufs`: host pointers.  The context
 * owns only host-side bookkeeping; free it with dqn_destroy. */
int32_t dqn_init(dqn_ctx **out, const dqn_config *cfg, const dqn_buffers *bufs, void *stream);

/* Epsilon-greedy action selection for E observations (Alg.1, the two action
 * lines; Eq.3): with u = draw(draw_seed, 2e), if u < epsilon the action is
 * floor(draw(draw_seed, 2e+1) * K), else argmax_a Q(obs_e, a; theta) with the
 * lowest index winning ties.  obs: [E][4][84][84]; actions: [E];
 * q_opt: [E][K] or NULL.  1 <= E <= max_act_batch. */
int32_t dqn_act(dqn_ctx *ctx, const uint8_t *obs, int32_t E, float epsilon, uint64_t draw_seed,
                int32_t *actions, float *q_opt, void *stream);

/* One minibatch training step (Alg.1 target + gradient-step lines; Alg.2
 * inner loop and weight update; Eq.7-9, Eq.13; RMSProp of Table 1):
 * forward of the online net on s and s', of the target net on s', target y,
 * TD error, loss L = (1/B) sum w l(td), exact gradient, RMSProp update of the
 * online parameters.  `batch` (host pointer to a struct of device pointers)
 * selects the explicit mode.  batch == NULL selects the replay mode: B slots
 * are drawn as by per_sample(beta, draw_seed), their frame stacks gathered
 * from the ring, and after the update their priorities are set from |td| as by
 * per_update.  `out` (host pointer, may be NULL) names optional outputs.
 * 1 <= B <= max_batch.
 * A row whose action lies outside [0, num_actions) is not trained on: it enters
 * the loss and the gradient with weight 0, its td is reported as NaN, and in
 * replay mode its priority is left alone.  In replay mode, if the tree holds no
 * mass at all (every stored transition has priority zero: nothing can be drawn),
 * every importance weight is 0, the parameters do not move and no priority is
 * written. */
int32_t dqn_train_step(dqn_ctx *ctx, int32_t B, const dqn_batch *batch, float beta,
                       uint64_t draw_seed, const dqn_step_out *out, void *stream);

/* Proportional prioritized sampling (Eq.10, Eq.12; Alg.2 sampling and
 * weighting lines).  Draw j uses u_j = draw(draw_seed, j); independent mode
 * descends the sum-tree with mass fp32(u_j * total), stratified mode with
 * fp32((j + u_j) * fp32(total / B)).  idx[j] is the leaf reached (clamped to
 * the stored size); is_w[j] = (N * P(j))^-beta / max_j(...), N = stored
 * transitions.  A slot whose leaf is 0 has probability zero and is never
 * returned, also where the fp32 sums of the tree would let the textbook
 * descent overshoot into it: the walk turns left whenever the right child is 0.
 * Returns DQN_ERR_STATE if nothing is stored (the call cannot see on the host
 * whether every stored leaf is 0: then idx = 0 and is_w = 0 are written).
 * 1 <= B <= 1024. */
int32_t per_sample(dqn_ctx *ctx, int32_t B, float beta, uint64_t draw_seed, int32_t *idx,
                   float *is_w, void *stream);

/* Priority update (Eq.11; Alg.2 priority line): leaf[idx_j] = fp32((|td_j| +
 * per_eps)^alpha) for j = 0..n-1 with the last occurrence of a repeated index
 * winning, every ancestor recomputed as fp32(left + right), and the running
 * maximum priority raised to max_j(|td_j| + per_eps).  idx values must lie in
 * [0, stored size); out-of-range entries and entries whose td is not finite are
 * skipped (their leaves keep their values).  1 <= n <= 1024. */
int32_t per_update(dqn_ctx *ctx, const int32_t *idx, const float *td_abs, int32_t n, void *stream);

/* dqn_act for callers that cannot allocate device memory or pass a workspace of
 * their own sizing: code under HIP graph capture, tight serving loops, harnesses
 * that forbid hipMalloc.  Same arguments, same kernels and bit-identical results
 * as dqn_act, but the activations and partial sums go to a static device array
 * inside the library (4 MiB per GPU, held until the process ends) instead of
 * the context's workspace, so E is limited to DQN_ACT_STATIC_MAX; a larger E
 * is DQN_ERR_INVALID_ARG.  The call allocates nothing (no hipMalloc, no
 * hipFree, no events); the array's device address is looked up once per device,
 * at dqn_init or on the first call there.  Nothing in the array has to start
 * at zero: every word read has been written earlier in the same call.  All
 * calls on one GPU share the array: calls that overlap on one GPU (two
 * streams, two contexts, two threads) race and give undefined results. */
#define DQN_ACT_STATIC_MAX 32
int32_t dqn_act_static(dqn_ctx *ctx, const uint8_t *obs, int32_t E, float epsilon, uint64_t draw_seed,
                       int32_t *actions, float *q_opt, void *stream);

/* ---- auxiliary calls needed to drive and to check the five above ---- */

/* Bulk (re)build of the sum-tree from n raw priorities p_i > 0 for slots
 * 0..n-1 (leaf = fp32(p^alpha), slots >= n get 0) and sets the stored size to
 * n.  n <= replay_capacity. */
int32_t per_fill(dqn_ctx *ctx, const float *priorities, int64_t n, void *stream);

/* Stores n consecutive single frames and their transition data into ring slots
 * slot0 .. slot0+n-1 (mod capacity) (Alg.1 "store transition").  Transition i
 * is read back as s = frames (i-3..i), s' = frames (i-2..i+1), slots taken
 * modulo the capacity.  Priorities are not touched.  frames: [n][84][84]. */
int32_t dqn_replay_write(dqn_ctx *ctx, int64_t slot0, int64_t n, const uint8_t *frames,
                         const int32_t *a, const float *r, const uint8_t *done, void *stream);

/* Store path (Alg.1 "store transition"; Alg.2 "store transition with maximal
 * priority").  Appends n consecutive time steps of ONE environment stream at the
 * write cursor (slot = stream position mod capacity): frame x_t with the action
 * a_t taken on it, the reward r_t and the terminal flag done_t.  Transition i is
 * read back as s = frames (i-3..i), s' = frames (i-2..i+1), so a time step
 * completes the transition before it.  Each completed transition enters the
 * sum-tree with the maximal priority seen so far (1 before the first update),
 * leaf = fp32(max_p^alpha); a transition whose state stack would reach back
 * before the start of the stream or across an episode end (done at one of the
 * three slots before it) gets leaf 0 and is never sampled, and so do the last
 * written slot (its transition is not complete yet) and the three slots after
 * it, whose windows mix the newest frames with the oldest.
 * The stored count (N of Eq.12) becomes min(time steps stored, capacity).
 * frames: [n][84][84] device, 16-byte aligned; a, r, done: [n] device, not NULL.
 * 1 <= n <= min(1020, capacity - 8); the ring must have at least 16 slots.
 * per_fill sets the cursor to n mod capacity; dqn_replay_write does not move it. */
int32_t dqn_replay_store(dqn_ctx *ctx, int64_t n, const uint8_t *frames, const int32_t *a,
                         const float *r, const uint8_t *done, void *stream);

/* Store path for many environment streams (Alg.1 "store transition" with one
 * emulator per stream, as batched acting needs it).  The ring becomes E sub-rings
 * of C = capacity / E slots (integer division; stream e owns slots [eC, (e+1)C));
 * the first call on an empty context fixes E.  Every call appends ONE time step to
 * every stream, at local slot (calls so far) mod C: frame x_t of stream e with the
 * action taken on it, reward and terminal flag.  Each stream follows the rules of
 * dqn_replay_store within its own sub-ring: the transition before the new step
 * enters with the maximal priority unless its stack would reach before the
 * stream's start or across an episode end; the slot just written and the three
 * after it get leaf 0.  A transition's frames are read back modulo its sub-ring, so
 * no stack ever mixes two streams.  The stored count (N of Eq.12) is
 * E * min(calls, C).  frames: [E][84][84] device, 16-byte aligned; a, r, done: [E].
 * 1 <= E <= capacity / 16.  per_fill returns the context to one stream. */
int32_t dqn_replay_store_envs(dqn_ctx *ctx, int32_t E, const uint8_t *frames, const int32_t *a,
                              const float *r, const uint8_t *done, void *stream);

/* Host-side view of the store path: next slot, stored count, time steps so far.
 * Any pointer may be NULL. */
int32_t dqn_replay_state(const dqn_ctx *ctx, int64_t *cursor, int64_t *stored, int64_t *steps);

/* Frame preprocessing (Sec.3: raw palette frame -> grey-scale -> linearly
 * interpolated to 84 x 84), batched.  raw: [n][height][width] bytes (device);
 * grey_lut: 256 floats (device) mapping a byte to its grey level in 0..255, or
 * NULL when the bytes already are grey levels; frames: [n][84][84] (device).
 * Output pixel (i,j) samples the source at (i+1/2)*height/84 - 1/2,
 * (j+1/2)*width/84 - 1/2 (clamped), blends the four neighbours bilinearly in
 * fp32 and rounds to the nearest integer (ties to even).  Needs no context.
 * 1 <= n <= 65535. */
int32_t dqn_preprocess(const uint8_t *raw, int64_t n, int32_t height, int32_t width,
                       const float *grey_lut, uint8_t *frames, void *stream);

/* Schedules of Table 1 as functions of the environment step t = 1, 2, ... (host
 * only, no device work): a value "a -> b (1 -> T steps)" is a at t = 1, b at
 * t >= T, linear in between; train is set when t is past learning_start and
 * t = 0 mod update_period (Alg.2 "if t = 0 mod K"); sync_target when
 * t = 0 mod target_period (Alg.2 last line).  dqn_schedule_default fills in
 * Table 1: learning start 50,000, update period 4, target period 30,000,
 * epsilon 1.0 -> 0.1 over 5,000,000 steps, beta 0.4 -> 1.0 over 100,000,000. */
typedef struct {
    int64_t learning_start, update_period, target_period, eps_steps, beta_steps;
    float eps_start, eps_end, beta_start, beta_end;
} dqn_schedule;
typedef struct {
    float epsilon, beta;
    int32_t train, sync_target;
} dqn_schedule_point;
int32_t dqn_schedule_default(dqn_schedule *s);
int32_t dqn_schedule_at(const dqn_schedule *s, int64_t step, dqn_schedule_point *out);

/* Materialises the stacks of n slots: s, s_next [n][4][84][84], a, r, done [n]
 * (any output may be NULL).  1 <= n <= max_batch. */
int32_t dqn_replay_gather(dqn_ctx *ctx, const int32_t *idx, int32_t n, uint8_t *s, uint8_t *s_next,
                          int32_t *a, float *r, uint8_t *done, void *stream);

/* Diagnostics: the stored outputs (after ReLU) of layer 1-3 (the convolutions) or
 * 4 (the 512-unit hidden layer) of Section 3's network for the first n rows of
 * the online pass on s of the last dqn_train_step, as fp32 in canonical order:
 * dst [n][32][20][20], [n][64][9][9], [n][64][7][7] or [n][512].  These are
 * the numbers the backward pass takes its ReLU decisions on.  1 <= n <= max_batch. */
int32_t dqn_get_activations(dqn_ctx *ctx, int32_t layer, int32_t n, float *dst, void *stream);

/* Host-only self-check, no device work: replays, for a run of ns samples per
 * workgroup (1..32), the schedule by which the fused conv1 + conv2 forward launch
 * of the bf16 path hands conv1's output of a sample (Section 3, first and second
 * layer) from its producer waves to its consumer waves through a ring of images
 * in LDS, using the very functions the kernel's loops call.  Returns 0 if every
 * sample is complete before it is read, read exactly once, and never overwritten
 * while unread; a positive code otherwise. */
int32_t dqn_selftest_fused_conv_schedule(int32_t ns);

/* theta^- <- theta (Alg.2 "copy weights into target network"). */
int32_t dqn_sync_target(dqn_ctx *ctx, void *stream);

/* which: 0 online, 1 target, 2 gradient of the last step, 3 RMSProp v,
 * 4 RMSProp m (centered only).  dst / src: device, canonical blob. */
int32_t dqn_get_params(dqn_ctx *ctx, int32_t which, float *dst, void *stream);
int32_t dqn_set_params(dqn_ctx *ctx, int32_t which, const float *src, void *stream);

/* Per-kernel timing: after dqn_profile_begin every kernel launched through
 * this context is bracketed by HIP events on its stream; dqn_profile_end
 * synchronises, disables timing, and copies up to `cap` records (name, launch
 * count, total milliseconds) to host arrays.  Returns the number of distinct
 * kernels seen (may exceed cap) or a negative status.  names: host array of
 * cap pointers to static strings. */
int32_t dqn_profile_begin(dqn_ctx *ctx);
int32_t dqn_profile_end(dqn_ctx *ctx, int32_t cap, const char **names, int64_t *counts,
                        double *total_ms);

/* Last error message of this context (host string, valid until the next call
 * on the context); for a NULL ctx, the last error of a failed dqn_init /
 * dqn_query_sizes on this thread. */
const char *dqn_last_error(const dqn_ctx *ctx);

int32_t dqn_destroy(dqn_ctx *ctx);

#ifdef __cplusplus
}
#endif
#endif /* DQN_H_ */
