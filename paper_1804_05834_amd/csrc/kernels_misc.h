// Everything around the GEMMs: the head (dueling combine, argmax, Bellman
// target, Huber loss and their gradients), RMSProp, the sum-tree, the
// frame-stack gather, epsilon-greedy selection and layout permutations.
#pragma once
#include <hip/hip_runtime.h>
#include <hip/hip_bf16.h>
#include <stdint.h>

#include "net.h"
#include "sumtree.h"

namespace misc {

// Barrier that orders LDS traffic only: global loads and stores issued earlier stay in flight
// across it (__syncthreads() would first wait for every one of them to complete).
__device__ __forceinline__ void sync_lds()
{
    asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
}

__device__ __forceinline__ float wave_sum(float v)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
    return v;
}

__device__ __forceinline__ float block_max_1024(float v, float *sh /*16*/)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
    __syncthreads();
    if (lane == 0) sh[wave] = v;
    __syncthreads();
    float r = sh[0];
    for (int w = 1; w < (int)(blockDim.x >> 6); ++w) r = fmaxf(r, sh[w]);
    return r;
}

// ------------------------------------------------------------------ head
// Rows of the head: dueling -> row 0 is the state value V, rows 1..K the
// advantages (Eq.13); plain -> rows 0..K-1 are the Q outputs.  Offsets are
// relative to the head section of the parameter blob.
__device__ __forceinline__ int head_w_off(int r, int K, int dueling)
{
    if (!dueling) return r * net::HID;
    return r == 0 ? 0 : net::HID + 1 + (r - 1) * net::HID;
}
__device__ __forceinline__ int head_b_off(int r, int K, int dueling)
{
    if (!dueling) return K * net::HID + r;
    return r == 0 ? net::HID : net::HID + 1 + K * net::HID + (r - 1);
}

constexpr int MAXR = 65;  // up to 64 actions + V

// The dot products of the head for the three passes of a training row at once: 3R of length 512 spread
// over groups of 16 lanes, so the whole head takes two rounds of a 512-thread workgroup instead
// of one wave per row in turn.  The weights of a round do not depend on the hidden layer, so
// head_rows3_load requests them while the fc1 partial sums are still being added up, and
// head_rows3_dot only reads LDS.
struct HeadRound {
    float w[net::HID / 16];
    float b;
    int d;  // dot product number: pass = d / R, row = d % R; -1: none
};
__device__ __forceinline__ void head_rows3_load(HeadRound &H, int round, const float *head_on, const float *head_tg,
                                                int K, int dueling, int tid)
{
    const int R = K + (dueling ? 1 : 0);
    const int grp = tid >> 4, l = tid & 15;
    const int d = grp + 32 * round;
    H.d = d < 3 * R ? d : -1;
    if (H.d < 0) return;
    const int p = d / R, r = d - p * R;
    const float *head = p == 2 ? head_tg : head_on;
    const float *w = head + head_w_off(r, K, dueling);
#pragma unroll
    for (int k = 0; k < net::HID / 16; ++k) H.w[k] = w[l + 16 * k];
    H.b = head[head_b_off(r, K, dueling)];
}
__device__ __forceinline__ void head_rows3_dot(const HeadRound &H, const float (*hid)[net::HID] /*LDS [3][512]*/,
                                               int K, int dueling, float (*raw)[65] /*LDS [3][65]*/, int tid)
{
    if (H.d < 0) return;  // uniform within the 16-lane group
    const int R = K + (dueling ? 1 : 0);
    const int l = tid & 15;
    const int p = H.d / R, r = H.d - p * R;
    const float *x = hid[p];
    float acc = 0.f;
#pragma unroll
    for (int k = 0; k < net::HID / 16; ++k) acc += H.w[k] * x[l + 16 * k];
#pragma unroll
    for (int o = 8; o > 0; o >>= 1) acc += __shfl_xor(acc, o, 64);
    if (l == 0) raw[p][r] = acc + H.b;
}

struct HeadArgs {
    const float *part;  // fc1 partial sums [nsplit][3B][512]: rows s | s' online | s' target
    int nsplit;
    long split_stride;
    int B, K, dueling, double_q, loss_kind;
    float kappa, gamma;
    const float *f1b_on, *f1b_tg;    // fc1 biases
    const float *head_on, *head_tg;  // head sections of the two parameter blobs
    const int32_t *a;
    const float *r;
    const uint8_t *done;
    const float *w;  // may be nullptr
    int w_raw;       // 1: w holds unnormalised importance weights; divide by their maximum here
    float *h_s;      // [B][512] hidden layer of the online net on s
    void *dh;        // [B][512] gradient w.r.t. the fc1 pre-activation (fp32, or bf16 if dh_bf16)
    int dh_bf16;
    float *dA;       // [B][R]   gradient w.r.t. the head rows
    float *td_abs;   // [B] |td_j|; NaN for a row the priority update must skip
    float *loss_j;   // [B] w_j * l(td_j)
    float *qmax_j;   // [B] max_a Q(s_j, a; theta)
    float *q_s, *q_no, *q_nt, *y, *td;  // optional outputs
    int32_t *a_star;
    float *is_w;
};

// One workgroup per minibatch row: finishes fc1 (split reduction, bias, ReLU)
// for the three passes, evaluates the head three times, forms the target
// (Eq.8 / Eq.9), the TD error, the loss term and the gradient w.r.t. the
// head rows, and back-propagates through the head into the hidden layer.
//
// The kernel is a chain of latencies, so it is written to have ONE round trip to memory: every
// global operand (partial sums and biases first, then the head weights of the dot products, the
// thread's column of the online head for the back-propagation, the raw importance weights, the
// row's transition) is requested before anything is waited for, in the order of first use.  The
// dueling combine (Eq.13) and the argmax run on one wave per pass with lane a holding action a.
// NS: the number of reduction splits of fc1 (A.nsplit), a template argument so that the loads of the
// partial sums are unconditional: behind a run-time test the compiler adds a split to its sum right where
// it is loaded, and the kernel then waits for its first load before it has requested the second.
constexpr int HEAD_MAX_SPLITS = 7;   // most reduction splits of fc1
template <int NS>
__global__ __launch_bounds__(512) void k_head_train(HeadArgs A)
{
    __shared__ float hid[3][net::HID];
    __shared__ float raw[3][MAXR];
    __shared__ float q[3][64];
    __shared__ float shm[16];
    __shared__ float res_q[3];     // Q(s, a_j; theta), max_a Q(s, a; theta), -
    __shared__ int res_as[3];      // argmax_a of pass p
    const int j = blockIdx.x, tid = threadIdx.x;
    const int K = A.K, R = K + (A.dueling ? 1 : 0);
    const bool norm = A.w && A.w_raw;

    // ---- every global load, in the order of first use
    float ps[3][NS];
    const long row[3] = {(long)j, (long)A.B + j, 2L * A.B + j};
#pragma unroll
    for (int p = 0; p < 3; ++p)
#pragma unroll
        for (int sp = 0; sp < NS; ++sp) ps[p][sp] = A.part[sp * A.split_stride + row[p] * net::HID + tid];
    const float b_on = A.f1b_on[tid], b_tg = A.f1b_tg[tid];
    HeadRound H0, H1;
    head_rows3_load(H0, 0, A.head_on, A.head_tg, K, A.dueling, tid);
    head_rows3_load(H1, 1, A.head_on, A.head_tg, K, A.dueling, tid);
    const int aj_raw = A.a[j];
    const bool dn = A.done[j] != 0;
    const float rj = A.r[j];
    const float wj = A.w ? A.w[j] : 1.f;
    float w0 = 0.f, w1 = 0.f;   // raw importance weights tid and tid + 512 (B <= 1024), for their maximum
    if (norm) {
        w0 = tid < A.B ? A.w[tid] : 0.f;
        w1 = tid + 512 < A.B ? A.w[tid + 512] : 0.f;
    }
    __builtin_amdgcn_sched_barrier(0);

    // ---- hidden layer: split sums in split order, bias, ReLU
    {
        float acc[3] = {0.f, 0.f, 0.f};
#pragma unroll
        for (int p = 0; p < 3; ++p) {
#pragma unroll
            for (int sp = 0; sp < NS; ++sp) acc[p] += ps[p][sp];
        }
        const float hs = fmaxf(acc[0] + b_on, 0.f);
        hid[0][tid] = hs;
        hid[1][tid] = fmaxf(acc[1] + b_on, 0.f);
        hid[2][tid] = fmaxf(acc[2] + b_tg, 0.f);
        A.h_s[(long)j * net::HID + tid] = hs;
    }
    __syncthreads();
    // column tid of the online head, for the back-propagation into the hidden layer at the end: requested
    // here, behind the operands the dot products wait for, and in flight until the last phase
    constexpr int HW_PRE = 24;
    float hw[HW_PRE];
#pragma unroll
    // (unconditional, row index clamped: a value chosen between a loaded one and a constant would be waited
    // for right here, in front of the dot products)
    for (int r = 0; r < HW_PRE; ++r) hw[r] = A.head_on[head_w_off(r < R ? r : R - 1, K, A.dueling) + tid];
    __builtin_amdgcn_sched_barrier(0);
    head_rows3_dot(H0, hid, K, A.dueling, raw, tid);
    head_rows3_dot(H1, hid, K, A.dueling, raw, tid);
    for (int round = 2; 32 * round < 3 * R; ++round) {  // more than 64 dot products: K > 20
        head_rows3_load(H0, round, A.head_on, A.head_tg, K, A.dueling, tid);
        head_rows3_dot(H0, hid, K, A.dueling, raw, tid);
    }
    if (norm) {  // per-wave maxima of the raw weights; thread 0 combines them below
        float wmax = fmaxf(w0, w1);
#pragma unroll
        for (int o = 32; o > 0; o >>= 1) wmax = fmaxf(wmax, __shfl_xor(wmax, o, 64));
        if ((tid & 63) == 0) shm[tid >> 6] = wmax;
    }
    __syncthreads();
    const bool a_ok = aj_raw >= 0 && aj_raw < K;
    const int aj = a_ok ? aj_raw : 0;
    if (tid < 192) {
        // wave p: lane a holds Q_a of pass p (Eq.13: V + A_a - mean A, or the plain outputs)
        const int p = tid >> 6, a = tid & 63;
        const float v = a < K ? raw[p][A.dueling ? 1 + a : a] : 0.f;
        float qa = v;
        if (A.dueling) qa = raw[p][0] + (v - wave_sum(v) / (float)K);
        if (a < K) q[p][a] = qa;
        // argmax with the lowest index winning ties; lanes past K never win
        float bv = a < K ? qa : -3.4028234663852886e38f;
        int bi = a < K ? a : 64;
#pragma unroll
        for (int o = 32; o > 0; o >>= 1) {
            const float ov = __shfl_xor(bv, o, 64);
            const int oi = __shfl_xor(bi, o, 64);
            if (ov > bv || (ov == bv && oi < bi)) { bv = ov; bi = oi; }
        }
        const float q_aj = __shfl(qa, aj, 64);
        if (a == 0) {
            res_as[p] = bi;
            if (p == 0) { res_q[0] = q_aj; res_q[1] = bv; }
        }
    }
    __syncthreads();
    if (tid == 0) {
        float wnorm = 1.f;
        if (norm) {
            float m = shm[0];
            for (int v = 1; v < 8; ++v) m = fmaxf(m, shm[v]);
            wnorm = m > 0.f ? 1.f / m : 0.f;   // no mass in the tree: every weight is 0
        }
        const int as = res_as[A.double_q ? 1 : 2];
        const float boot = dn ? 0.f : A.gamma * q[2][as];
        const float y = rj + boot;
        const float d = y - res_q[0];
        // an action outside [0, K) cannot be trained on: the row contributes nothing (weight 0), its TD
        // error is reported as NaN and the priority update skips it
        const float w = !a_ok ? 0.f : A.w ? wj * wnorm : 1.f;
        float l, dl;
        if (A.loss_kind == 1 && fabsf(d) > A.kappa) {
            l = A.kappa * (fabsf(d) - 0.5f * A.kappa);
            dl = d > 0.f ? A.kappa : -A.kappa;
        } else {
            l = 0.5f * d * d;
            dl = d;
        }
        shm[8] = -w * dl / (float)A.B;  // dL/dQ(s_j, a_j)
        // a drawn row whose raw weight is 0 came from a tree without mass: its slot holds nothing to update
        const bool skip = !a_ok || (norm && !(wj > 0.f));
        A.td_abs[j] = skip ? __int_as_float(0x7fc00000) : fabsf(d);
        A.loss_j[j] = w * l;
        A.qmax_j[j] = res_q[1];
        if (A.y) A.y[j] = y;
        if (A.td) A.td[j] = a_ok ? d : __int_as_float(0x7fc00000);
        if (A.a_star) A.a_star[j] = as;
        if (A.is_w) A.is_w[j] = w;
    }
    if (A.q_s && tid >= 64 && tid < 64 + K) A.q_s[(long)j * K + tid - 64] = q[0][tid - 64];
    if (A.q_no && tid >= 128 && tid < 128 + K) A.q_no[(long)j * K + tid - 128] = q[1][tid - 128];
    if (A.q_nt && tid >= 192 && tid < 192 + K) A.q_nt[(long)j * K + tid - 192] = q[2][tid - 192];
    __syncthreads();
    {
        // gradient w.r.t. the head rows (dueling: dV = g, dA_a = [a = a_j] g - g / K), every thread for itself
        const float g = shm[8];
        const float gk = A.dueling ? g / (float)K : 0.f;
        const int hit = A.dueling ? 1 + aj : aj;
        if (tid < R) A.dA[(long)j * R + tid] = (A.dueling && tid == 0) ? g : (tid == hit ? g : 0.f) - gk;
        float acc = 0.f;
#pragma unroll
        for (int r = 0; r < HW_PRE; ++r)
            if (r < R) acc += ((A.dueling && r == 0) ? g : (r == hit ? g : 0.f) - gk) * hw[r];
        for (int r = HW_PRE; r < R; ++r)
            acc += ((A.dueling && r == 0) ? g : (r == hit ? g : 0.f) - gk) * A.head_on[head_w_off(r, K, A.dueling) + tid];
        const float gmask = hid[0][tid] > 0.f ? acc : 0.f;
        if (A.dh_bf16) static_cast<__hip_bfloat16 *>(A.dh)[(long)j * net::HID + tid] = __float2bfloat16(gmask);
        else static_cast<float *>(A.dh)[(long)j * net::HID + tid] = gmask;
    }
}

struct HeadWgradArgs {
    const float *dA;      // [B][R]
    const float *h_s;     // [B][512]
    const float *loss_j;  // [B]
    float *ghead;         // head section of the gradient partial buffer
    float *loss_out;      // optional
    float *loss_slot;     // always written
    int B, K, dueling;
    const float *td_abs;  // [B]
    const float *qmax_j;  // [B]
    float *td_abs_mean;   // optional [1]: (1/B) sum_j |td_j| over the rows with a finite error
    float *q_max_mean;    // optional [1]: (1/B) sum_j max_a Q(s_j, a; theta)
};

// Head weight gradient: dW[r][i] = sum_j dA[j][r] h[j][i], db[r] = sum_j dA[j][r].
// grid (R, 16): block (r, c) owns hidden units [32c, 32c+32); its 512 threads split the
// minibatch sixteen ways and combine through LDS in a fixed order.  Block (0,0) also folds the
// per-row loss terms into L = (1/B) sum_j w_j l_j.
// NG = threads / 32 groups over the minibatch; lds: NG * 34 floats.  Row r, hidden units [32c, 32c+32).
template <int NG>
__device__ __forceinline__ void head_wgrad_body(const HeadWgradArgs &A, int r, int c, float *lds)
{
    float(*red)[33] = reinterpret_cast<float(*)[33]>(lds);
    float *redb = lds + NG * 33;
    const int il = threadIdx.x & 31, jg = threadIdx.x >> 5;
    const int i = c * 32 + il;
    const int R = A.K + (A.dueling ? 1 : 0);
    float acc = 0.f, accb = 0.f;
#pragma unroll 8
    for (int j = jg; j < A.B; j += NG) {
        float d = A.dA[(long)j * R + r];
        acc += d * A.h_s[(long)j * net::HID + i];
        accb += d;
    }
    red[jg][il] = acc;
    if (il == 0) redb[jg] = accb;
    __syncthreads();
    if (jg == 0) {
        float s = red[0][il];
#pragma unroll
        for (int g = 1; g < NG; ++g) s += red[g][il];
        A.ghead[head_w_off(r, A.K, A.dueling) + i] = s;
        if (il == 0 && c == 0) {
            float sb = redb[0];
#pragma unroll
            for (int g = 1; g < NG; ++g) sb += redb[g];
            A.ghead[head_b_off(r, A.K, A.dueling)] = sb;
        }
    }
    if (r == 0 && c == 0 && (int)threadIdx.x >= NG * 32 - 64) {  // the last wave sums the loss terms
        const int lane = threadIdx.x & 63;
        float s = 0.f, sd = 0.f, sq = 0.f;
        for (int j = lane; j < A.B; j += 64) {
            s += A.loss_j[j];
            const float d = A.td_abs[j];
            if (d <= 3.4028234e38f) sd += d;   // false for NaN
            sq += A.qmax_j[j];
        }
        s = wave_sum(s) / (float)A.B;
        sd = wave_sum(sd) / (float)A.B;
        sq = wave_sum(sq) / (float)A.B;
        if (lane == 0) {
            *A.loss_slot = s;
            if (A.loss_out) *A.loss_out = s;
            if (A.td_abs_mean) *A.td_abs_mean = sd;
            if (A.q_max_mean) *A.q_max_mean = sq;
        }
    }
}

__global__ __launch_bounds__(512) void k_head_wgrad(HeadWgradArgs A)
{
    __shared__ float lds[16 * 34];
    head_wgrad_body<16>(A, blockIdx.x, blockIdx.y, lds);
}

struct HeadActArgs {
    const float *part;
    int nsplit;
    long split_stride;
    int E, K, dueling;
    const float *f1b, *head;
    float epsilon;
    uint64_t seed;
    int32_t *actions;
    float *q_out;  // optional [E][K]
};

// Acting (Alg.1 action lines): finish fc1, evaluate the head, pick the action.  One workgroup per
// observation, built like the training head: every global operand (the partial sums of the thread's two
// hidden units, the biases, the head weights of the first 32 dot products, spread over groups of 16 lanes)
// is requested before anything is waited for, the dueling combine (Eq.13) and the argmax run on one wave
// with lane a holding action a, and the arithmetic is that of k_head_train, so Q(s, .) has the same bits
// here and there.  NS: reduction splits of fc1 (A.nsplit), a template argument so that the loads are
// unconditional.
__device__ __forceinline__ void head_rows1_load(HeadRound &H, int round, const float *head, int K, int dueling, int tid)
{
    const int R = K + (dueling ? 1 : 0);
    const int grp = tid >> 4, l = tid & 15;
    const int d = grp + 16 * round;
    H.d = d < R ? d : -1;
    const int r = d < R ? d : R - 1;   // clamped: the loads are unconditional
    const float *w = head + head_w_off(r, K, dueling);
#pragma unroll
    for (int k = 0; k < net::HID / 16; ++k) H.w[k] = w[l + 16 * k];
    H.b = head[head_b_off(r, K, dueling)];
}
__device__ __forceinline__ void head_rows1_dot(const HeadRound &H, const float *hid /*LDS [512]*/, float *raw /*LDS*/, int tid)
{
    const int l = tid & 15;
    float acc = 0.f;
#pragma unroll
    for (int k = 0; k < net::HID / 16; ++k) acc += H.w[k] * hid[l + 16 * k];
#pragma unroll
    for (int o = 8; o > 0; o >>= 1) acc += __shfl_xor(acc, o, 64);
    if (l == 0 && H.d >= 0) raw[H.d] = acc + H.b;
}
template <int NS>
__global__ __launch_bounds__(256) void k_head_act(HeadActArgs A)
{
    __shared__ float hid[net::HID];
    __shared__ float raw[MAXR];
    const int e = blockIdx.x, tid = threadIdx.x;
    const int K = A.K, R = K + (A.dueling ? 1 : 0);
    float ps[2][NS];
#pragma unroll
    for (int u = 0; u < 2; ++u)
#pragma unroll
        for (int sp = 0; sp < NS; ++sp) ps[u][sp] = A.part[sp * A.split_stride + (long)e * net::HID + tid + 256 * u];
    const float b0 = A.f1b[tid], b1 = A.f1b[tid + 256];
    HeadRound H0, H1;
    head_rows1_load(H0, 0, A.head, K, A.dueling, tid);
    head_rows1_load(H1, 1, A.head, K, A.dueling, tid);
    __builtin_amdgcn_sched_barrier(0);
    {
        float acc[2] = {0.f, 0.f};
#pragma unroll
        for (int u = 0; u < 2; ++u)
#pragma unroll
            for (int sp = 0; sp < NS; ++sp) acc[u] += ps[u][sp];
        hid[tid] = fmaxf(acc[0] + b0, 0.f);
        hid[tid + 256] = fmaxf(acc[1] + b1, 0.f);
    }
    __syncthreads();
    head_rows1_dot(H0, hid, raw, tid);
    head_rows1_dot(H1, hid, raw, tid);
    for (int round = 2; 16 * round < R; ++round) {   // more than 32 dot products: K > 31
        head_rows1_load(H0, round, A.head, K, A.dueling, tid);
        head_rows1_dot(H0, hid, raw, tid);
    }
    __syncthreads();
    if (tid < 64) {
        const int a = tid;
        const float v = a < K ? raw[A.dueling ? 1 + a : a] : 0.f;
        float qa = v;
        if (A.dueling) qa = raw[0] + (v - wave_sum(v) / (float)K);
        // argmax with the lowest index winning ties; lanes past K never win
        float bv = a < K ? qa : -3.4028234663852886e38f;
        int bi = a < K ? a : 64;
#pragma unroll
        for (int o = 32; o > 0; o >>= 1) {
            const float ov = __shfl_xor(bv, o, 64);
            const int oi = __shfl_xor(bi, o, 64);
            if (ov > bv || (ov == bv && oi < bi)) { bv = ov; bi = oi; }
        }
        if (a == 0) {
            int act = bi;
            const float u = draw_u24(A.seed, 2ull * (uint64_t)e);
            if (u < A.epsilon) {
                const float u2 = draw_u24(A.seed, 2ull * (uint64_t)e + 1ull);
                act = min((int)floorf(u2 * (float)K), K - 1);
            }
            A.actions[e] = act;
        }
        if (A.q_out && a < K) A.q_out[(long)e * K + a] = qa;
    }
}
// the launch for a run-time number of splits
inline void launch_head_act(const HeadActArgs &H, hipStream_t st)
{
    switch (H.nsplit) {
    case 1: k_head_act<1><<<H.E, 256, 0, st>>>(H); break;
    case 2: k_head_act<2><<<H.E, 256, 0, st>>>(H); break;
    case 3: k_head_act<3><<<H.E, 256, 0, st>>>(H); break;
    case 4: k_head_act<4><<<H.E, 256, 0, st>>>(H); break;
    case 5: k_head_act<5><<<H.E, 256, 0, st>>>(H); break;
    case 6: k_head_act<6><<<H.E, 256, 0, st>>>(H); break;
    default: k_head_act<7><<<H.E, 256, 0, st>>>(H); break;
    }
}

// --------------------------------------------------------------- RMSProp
// g = sum of the reduction splits (fixed order); v <- rho v + (1-rho) g^2;
// theta <- theta - lr g / sqrt(v + eps)   [centered: sqrt(v - m^2 + eps)].
// Each layer is a segment with its own block range.  A segment whose gradient
// arrives in several splits uses 64 parameters x 4 split-groups per block, so
// the split sum is spread over four times the threads and combined in LDS;
// a single-split segment (fc1, head) is a plain 256-parameters-per-block sweep.
struct RmsSeg {
    long begin, count;  // range of the blob
    const float *part;  // [nsplit][count]
    int nsplit;
    long stride;
    int block_begin;    // first blockIdx.x of this segment
};
struct RmsArgs {
    RmsSeg seg[5];
    float *theta, *v, *m, *g;
    __hip_bfloat16 *shadow;  // bf16 copy of theta (same order) or nullptr
    __hip_bfloat16 *w2t;     // with it: conv2's weights once more, as [tap][channel in][channel out] (or nullptr)
    float lr, rho, eps;
};

// What the update reads of parameter i
struct RmsOld { float v, th, m; };
__device__ __forceinline__ RmsOld rms_load(const RmsArgs &A, long i) { return RmsOld{A.v[i], A.theta[i], A.m ? A.m[i] : 0.f}; }
// store_g: false where the gradient already stands in A.g (a single partial written there by its kernel)
__device__ __forceinline__ void rms_apply(const RmsArgs &A, long i, float g, const RmsOld &old, bool store_g = true)
{
    float v = A.rho * old.v + (1.f - A.rho) * g * g;
    float denom;
    if (A.m) {
        float m = A.rho * old.m + (1.f - A.rho) * g;
        A.m[i] = m;
        denom = sqrtf(v - m * m + A.eps);
    } else {
        denom = sqrtf(v + A.eps);
    }
    float th = old.th - A.lr * g / denom;
    A.v[i] = v;
    A.theta[i] = th;
    if (store_g) A.g[i] = g;
    if (A.shadow) A.shadow[i] = __float2bfloat16(th);
    if (A.w2t && i >= net::C2W && i < net::C2W + 64 * 512) {
        const int t = (int)(i - net::C2W);   // [channel out][tap][channel in]
        A.w2t[(t & 511) * 64 + (t >> 9)] = __float2bfloat16(th);
    }
}
// every operand is requested before the first store: the buffers may overlap as far as the compiler
// knows, so a load behind a store would wait for the arithmetic in front of that store
__device__ __forceinline__ void rms_update(const RmsArgs &A, long i, float g, bool store_g = true)
{
    const RmsOld old = rms_load(A, i);
    rms_apply(A, i, g, old, store_g);
}

// The segment that workgroup bx belongs to.  A macro, to be used on the KERNEL PARAMETER itself: picked
// through a reference or a copy of the argument structure, the segment array ends up in scratch memory.
#define RMS_SELECT_SEGMENT(A, bx, S)                                  \
    misc::RmsSeg S = (A).seg[0];                                     \
    {                                                                \
        int s_ = 0;                                                  \
        _Pragma("unroll") for (int t_ = 1; t_ < 5; ++t_)             \
            if ((bx) >= (A).seg[t_].block_begin) s_ = t_;            \
        if (s_ == 1) S = (A).seg[1];                                 \
        if (s_ == 2) S = (A).seg[2];                                 \
        if (s_ == 3) S = (A).seg[3];                                 \
        if (s_ == 4) S = (A).seg[4];                                 \
    }

// workgroup bx (256 threads) of the update, in segment S; red: 256 floats of LDS
__device__ __forceinline__ void rmsprop_block(const RmsArgs &A, const RmsSeg &S, int bx, float (*red)[64])
{
    const int tid = threadIdx.x;
    if (S.nsplit > 1) {
        const int pl = tid & 63, sg = tid >> 6;
        const long o = (long)(bx - S.block_begin) * 64 + pl;
        // what the update reads is requested along with the partial sums (by every thread, from a clamped
        // index: no branch, no wait), not in a round trip of its own behind their sum
        const RmsOld old = rms_load(A, S.begin + (o < S.count ? o : 0));
        float g = 0.f;
        if (o < S.count) {
#pragma unroll 8
            for (int t = sg; t < S.nsplit; t += 4) g += S.part[t * S.stride + o];
        }
        red[sg][pl] = g;
        __syncthreads();
        if (sg == 0 && o < S.count)
            rms_apply(A, S.begin + o, (red[0][pl] + red[1][pl]) + (red[2][pl] + red[3][pl]), old);
    } else {
        const long o = (long)(bx - S.block_begin) * 256 + tid;
        if (o < S.count) rms_update(A, S.begin + o, S.part[o], S.part != A.g + S.begin);
    }
}
__global__ __launch_bounds__(256) void k_rmsprop(RmsArgs A)
{
    __shared__ float red[4][64];
    RMS_SELECT_SEGMENT(A, (int)blockIdx.x, S)
    rmsprop_block(A, S, blockIdx.x, red);
}

// conv2's weights [channel out][tap][channel in] (fp32, internal order) as bf16 [tap][channel in][channel out]:
// the layout in which the input gradient of conv2 finds the eight output channels of a matrix-instruction
// operand next to each other (its reduction runs over the output channels)
__global__ void k_w2_transposed(const float *w2, __hip_bfloat16 *w2t)
{
    const int t = blockIdx.x * blockDim.x + threadIdx.x;
    if (t < 64 * 512) w2t[(t & 511) * 64 + (t >> 9)] = __float2bfloat16(w2[t]);
}

// fp32 -> bf16 copy (round to nearest even)
__global__ void k_to_bf16(const float *src, __hip_bfloat16 *dst, long n)
{
    long i = (long)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) dst[i] = __float2bfloat16(src[i]);
}

// ------------------------------------------------- layout permutations
// canonical blob <-> internal blob (see net.h).  dir 0: dst(internal) from
// src(canonical); dir 1: dst(canonical) from src(internal).
__global__ void k_permute(const float *src, float *dst, long n, int dir)
{
    long e = (long)blockIdx.x * blockDim.x + threadIdx.x;  // canonical index
    if (e >= n) return;
    long in = e;
    if (e >= net::C2W && e < net::C2B) {  // [o][c][p][q] -> [o][p][q][c]
        long t = e - net::C2W;
        int q = t % 4, p = (t / 4) % 4, c = (t / 16) % 32, o = t / 512;
        in = net::C2W + ((o * 4 + p) * 4 + q) * 32 + c;
    } else if (e >= net::C3W && e < net::C3B) {
        long t = e - net::C3W;
        int q = t % 3, p = (t / 3) % 3, c = (t / 9) % 64, o = t / 576;
        in = net::C3W + ((o * 3 + p) * 3 + q) * 64 + c;
    } else if (e >= net::F1W && e < net::F1B) {  // [o][c*49 + hw] -> [o][hw*64 + c]
        long t = e - net::F1W;
        int k = t % 3136, o = t / 3136;
        int c = k / 49, hw = k % 49;
        in = net::F1W + (long)o * 3136 + hw * 64 + c;
    }
    if (dir == 0) dst[in] = src[e];
    else dst[e] = src[in];
}

__global__ void k_fill(float *p, float v, long n)
{
    long i = (long)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i] = v;
}

// ------------------------------------------------------------- sum-tree
// Heap layout: tree[1] root, children of i at 2i and 2i+1, leaves at
// tree[L..2L); tree[2L] holds the running maximum priority.
__global__ void k_tree_leaves(float *tree, long L, const float *p, long n, float alpha)
{
    long i = (long)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= L) return;
    tree[L + i] = i < n ? (float)pow((double)p[i], (double)alpha) : 0.f;
    if (i == 0) tree[0] = 0.f;
}
__global__ void k_tree_level(float *tree, long first, long count)
{
    long i = (long)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= count) return;
    long node = first + i;
    tree[node] = tree[2 * node] + tree[2 * node + 1];
}

// Rebuild of the internal nodes from the leaves, 12 levels per launch: the tree over Lcur leaves
// (leaves at tree[Lcur, 2 Lcur)) is cut into blocks of BL = min(Lcur, 4096) leaves; a workgroup loads
// its block's leaves, forms the block's sub-tree in LDS level by level (node = left + right in fp32,
// so every node has the bits any other order of repair gives) and writes its BL - 1 internal
// nodes.  The block roots are the leaves of the tree one launch up: Lcur >> 12 of them.
// The block of BL leaves number b of the tree over Lcur leaves; t: 2 * 4096 floats of LDS
__device__ __forceinline__ void tree_block(float *tree, long Lcur, int BL, long b, float *t)
{
    const long root = Lcur / BL + b;          // heap index of the block root
    for (int i = threadIdx.x; i < BL; i += 256) t[BL + i] = tree[Lcur + b * BL + i];
    for (int first = BL >> 1; first >= 1; first >>= 1) {
        __syncthreads();
        for (int i = threadIdx.x; i < first; i += 256) t[first + i] = t[2 * (first + i)] + t[2 * (first + i) + 1];
    }
    __syncthreads();
    // local node p at depth d (p in [2^d, 2^(d+1))) is heap node (root << d) + (p - 2^d)
    for (int p = 1 + threadIdx.x; p < BL; p += 256) {
        const int d = 31 - __clz(p);
        tree[(root << d) + (p - (1 << d))] = t[p];
    }
}
__global__ __launch_bounds__(256) void k_tree_rebuild(float *tree, long Lcur, int BL)
{
    __shared__ float t[2 * 4096];             // local heap: t[1] block root, leaves at t[BL, 2 BL)
    tree_block(tree, Lcur, BL, blockIdx.x, t);
}
// One thread per stream: the leaves the new time step settles, by the rules of the one-stream store
// path applied to the stream's own sub-ring (see k_store_priorities): the transition at local slot
// l - 1 has just become complete and enters with leaf = fp32(max_p^alpha) unless its state stack
// would reach back before the stream's start (t - 1 < 3) or across an episode end; the slot just
// written and the three after it get leaf 0.  Reads only transition data of earlier time steps.
// The internal nodes are rebuilt afterwards.
__device__ __forceinline__ void store_leaves_env(float *tree, long L, long C, long l, long t, long e,
                                                 const uint8_t *done, float alpha)
{
    const long base = e * C;
    auto at = [&](long k) { long q = (l + k) % C; if (q < 0) q += C; return base + q; };
    if (t >= 1) {
        bool valid = t - 1 >= 3;
        for (int k = 2; k <= 4; ++k)
            if (done[at(-k)]) valid = false;
        tree[L + at(-1)] = valid ? (float)pow((double)tree[2 * L], (double)alpha) : 0.f;
    }
    for (int k = 0; k < 4; ++k) tree[L + at(k)] = 0.f;
}
// grid (E): frame and transition data of stream e (waves 0..3), and its leaves (one thread of the last wave)
__global__ __launch_bounds__(256) void k_replay_write_envs(uint8_t *frames, int32_t *meta_a, float *meta_r,
                                                           uint8_t *meta_done, long C, long l,
                                                           const uint8_t *src, const int32_t *a,
                                                           const float *r, const uint8_t *done,
                                                           float *tree, long L, long t, float alpha)
{
    const long e = blockIdx.x, slot = e * C + l;
    if (threadIdx.x == 192) store_leaves_env(tree, L, C, l, t, e, meta_done, alpha);
    const uint4 *s = reinterpret_cast<const uint4 *>(src + e * net::FRAME);
    uint4 *d = reinterpret_cast<uint4 *>(frames + slot * net::FRAME);
    for (int t4 = threadIdx.x; t4 < net::FRAME / 16; t4 += 256) d[t4] = s[t4];
    if (threadIdx.x == 0) {
        meta_a[slot] = a[e];
        meta_r[slot] = r[e];
        meta_done[slot] = done[e];
    }
}

__global__ __launch_bounds__(256) void k_per_sample(SampleArgs A)
{
    const int lane = threadIdx.x & 63;
    const int j = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (j >= A.B) return;
    const int jj[1] = {j};
    long slot[1];
    float leaf[1];
    const float total = per_sample_walk<1>(A, jj, lane, slot, leaf);
    if (lane == 0) per_sample_emit(A, j, slot[0], total, leaf[0]);
}

// w_j <- w_j / max_j w_j over the minibatch (single workgroup)
__global__ __launch_bounds__(1024) void k_per_normalise(float *is_w, int B)
{
    __shared__ float sh[16];
    const int j = threadIdx.x;
    const float w = j < B ? is_w[j] : 0.f;
    const float wmax = block_max_1024(w, sh);
    if (j < B) is_w[j] = wmax > 0.f ? w / wmax : 0.f;
}

// Leaf-to-root repair by the threads of ONE workgroup, each starting from its own distinct leaf
// with the leaf's new value v: a level is one exchange through memory: every walker publishes
// its node, the workgroup meets, every walker reads its sibling as it now stands and forms
// parent = left + right (fp32; the sum is commutative, so walkers whose paths have merged hold
// identical values and store them to the same word; the result is bit-identical to repairing
// the paths one after another).  All walkers sit on one compute unit, so workgroup scope is
// enough: a store is complete before the barrier and the load after it sees it.  Every thread
// of the workgroup must call this (it contains barriers).
// W walkers per thread (a thread's walkers take the levels together).
template <int W>
__device__ __forceinline__ void tree_walk(float *tree, int (&node)[W], float (&v)[W], const bool (&walk)[W], int levels)
{
#pragma unroll
    for (int w = 0; w < W; ++w)
        if (walk[w]) __hip_atomic_store(&tree[node[w]], v[w], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
    for (int l = 0; l < levels; ++l) {
        __syncthreads();
        float vs[W];
#pragma unroll
        for (int w = 0; w < W; ++w)
            vs[w] = walk[w] ? __hip_atomic_load(&tree[node[w] ^ 1], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP) : 0.f;
#pragma unroll
        for (int w = 0; w < W; ++w)
            if (walk[w]) {
                v[w] = v[w] + vs[w];
                node[w] >>= 1;
                __hip_atomic_store(&tree[node[w]], v[w], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
            }
    }
}
__device__ __forceinline__ void tree_walk(float *tree, int node, float v, bool walk, int levels)
{
    int n1[1] = {node};
    float v1[1] = {v};
    const bool w1[1] = {walk};
    tree_walk<1>(tree, n1, v1, w1, levels);
}

// Priority update (Eq.11): a single workgroup, one thread per entry.  Repeated
// slots are settled first ("last occurrence wins" is an integer maximum over
// entry numbers in an LDS hash table keyed by leaf).  The surviving entries
// then repair the tree level by level, parent = left + right in fp32; the sum
// is commutative, so the result is bit-identical to a sequential repair.
constexpr int PU_SLOTS = 2048;  // hash slots (at most 1024 live keys)
__device__ __forceinline__ int pu_hash(int key) { return (int)(((unsigned)key * 2654435761u) >> 21); }
// returns the slot of `key`; *first is set when this call created it
__device__ __forceinline__ int pu_insert(int *keys, int key, bool *first)
{
    int h = pu_hash(key);
    for (;;) {
        const int old = atomicCAS(&keys[h], -1, key);
        if (old == -1 || old == key) {
            *first = old == -1;
            return h;
        }
        h = (h + 1) & (PU_SLOTS - 1);
    }
}
__device__ __forceinline__ int pu_find(const int *keys, int key)
{
    int h = pu_hash(key);
    for (;;) {
        const int k = keys[h];
        if (k == key) return h;
        if (k == -1) return -1;
        h = (h + 1) & (PU_SLOTS - 1);
    }
}

struct PerUpdateArgs {
    float *tree;
    long L;
    int levels;
    long size;
    const int32_t *idx;
    const float *td_abs;
    int n;
    float alpha, eps;
    int leaves_fixed;   // 1: priority exponent 0 over a tree of ones: a leaf's new value is its old one, so
                        // only the running maximum priority is updated and no node is read or written
};
constexpr int PU_LDS_WORDS = 2 * PU_SLOTS + 16;  // LDS of per_update_body, in 4-byte words

// The whole workgroup must call this; it handles W entries per thread (W * blockDim.x >= n).
// lds: PU_LDS_WORDS words.  With `state` the walk stops after `first_levels` levels and leaves
// every walker (node, value, active) there, for per_update_resume to take to the root later:
// entry j at state[j], state[STATE_STRIDE + j], state[2 * STATE_STRIDE + j].
constexpr int STATE_STRIDE = 1024;
template <int W = 1>
__device__ __forceinline__ void per_update_body(const PerUpdateArgs &A, int *lds, int first_levels = -1,
                                                int *state = nullptr)
{
    int *keys = lds, *ivals = lds + PU_SLOTS;  // ivals: largest entry number naming the slot's leaf
    float *sh = reinterpret_cast<float *>(lds + 2 * PU_SLOTS);
    float *tree = A.tree;
    const long L = A.L, size = A.size;
    const int levels = A.levels, n = A.n;
    const int32_t *idx = A.idx;
    const float *td_abs = A.td_abs;
    const float alpha = A.alpha, eps = A.eps;
    const int tid = threadIdx.x, nt = blockDim.x;
    int my[W];
    float p[W];
#pragma unroll
    for (int w = 0; w < W; ++w) {
        const int j = tid + w * nt;
        my[w] = -1;
        p[w] = 0.f;
        if (j < n) {
            const int v = idx[j];
            p[w] = (float)((double)fabsf(td_abs[j]) + (double)eps);
            // an entry with a slot outside the ring or a non-finite error is skipped: its leaf keeps
            // its value, and the tree stays a tree of finite sums
            if (v >= 0 && v < size && p[w] <= 3.4028234663852886e38f) my[w] = v;   // finite: false for NaN and infinity
        }
    }
    for (int t = tid; t < PU_SLOTS; t += nt) { keys[t] = -1; ivals[t] = -1; }
    __syncthreads();
    int node[W], slot[W];
    float pm = 0.f;
#pragma unroll
    for (int w = 0; w < W; ++w) {
        const bool valid = my[w] >= 0;
        node[w] = (int)L + (valid ? my[w] : 0);
        slot[w] = 0;
        if (valid) {
            bool first;
            slot[w] = pu_insert(keys, node[w], &first);
            atomicMax(&ivals[slot[w]], tid + w * nt);
            pm = fmaxf(pm, p[w]);
        }
    }
    const float pmax = block_max_1024(pm, sh);  // contains barriers
    if (tid == 0) tree[2 * L] = fmaxf(tree[2 * L], pmax);
    if (A.leaves_fixed) return;   // uniform for the workgroup
    // One walker per distinct leaf (the last entry naming it) walks to the root.  A level is one
    // exchange through memory: every walker publishes its node, the workgroup meets, every
    // walker reads its sibling as it now stands.  Walkers whose paths have merged hold the same
    // value and store it to the same word.
    bool walk[W];
    float v[W];
#pragma unroll
    for (int w = 0; w < W; ++w) {
        walk[w] = my[w] >= 0 && ivals[slot[w]] == tid + w * nt;
        v[w] = (float)pow((double)p[w], (double)alpha);
    }
    tree_walk<W>(tree, node, v, walk, state ? first_levels : levels);
    if (state) {
#pragma unroll
        for (int w = 0; w < W; ++w) {
            const int j = tid + w * nt;
            if (j < STATE_STRIDE) {
                state[j] = node[w];
                state[STATE_STRIDE + j] = __float_as_int(v[w]);
                state[2 * STATE_STRIDE + j] = walk[w] ? 1 : 0;
            }
        }
    }
}

// A later part of a split priority update: the walkers that the part before left `done_levels`
// levels above their leaves climb `walk_levels` more (to the root if that is all that is left;
// otherwise they are left in `state` again).  Same workgroup shape as the first part.
template <int W>
__device__ __forceinline__ void per_update_resume(const PerUpdateArgs &A, int done_levels, int walk_levels, int *state)
{
    const int tid = threadIdx.x, nt = blockDim.x;
    if (A.leaves_fixed) return;
    int node[W];
    float v[W];
    bool walk[W];
#pragma unroll
    for (int w = 0; w < W; ++w) {
        const int j = tid + w * nt;
        const bool in = j < A.n && j < STATE_STRIDE;
        node[w] = in ? state[j] : 1;
        v[w] = in ? __int_as_float(state[STATE_STRIDE + j]) : 0.f;
        walk[w] = in && state[2 * STATE_STRIDE + j] != 0;
    }
    const bool last = done_levels + walk_levels >= A.levels;
    tree_walk<W>(A.tree, node, v, walk, last ? A.levels - done_levels : walk_levels);
    if (!last) {
#pragma unroll
        for (int w = 0; w < W; ++w) {
            const int j = tid + w * nt;
            if (j < A.n && j < STATE_STRIDE) {
                state[j] = node[w];
                state[STATE_STRIDE + j] = __float_as_int(v[w]);
            }
        }
    }
}

__global__ __launch_bounds__(1024) void k_per_update(PerUpdateArgs A)
{
    __shared__ int lds[PU_LDS_WORDS];
    per_update_body<1>(A, lds);
}

// Store path (Alg.2 "store transition with maximal priority"): n time steps have just been
// written to ring slots h0 .. h0+n-1 (stream positions seq0 .. seq0+n-1).  Thread j settles
// the leaf of slot h0-1+j: for j < n that transition has just become complete (its s' ends in a
// new frame) and enters with leaf = fp32(max_p^alpha), unless its state stack would reach back
// before the start of the stream or across an episode end (done at one of the three slots
// before it), in which case it is never sampled (leaf 0); the last written slot (not complete
// yet) and the three after it, whose windows mix the newest frames with the oldest (j = n ..
// n+3), get leaf 0.
// One workgroup, n + 4 <= 1024 distinct slots, then the same level-by-level walk as above.
__global__ __launch_bounds__(1024) void k_store_priorities(float *tree, long L, int levels, long cap,
                                                           long h0, long seq0, int n,
                                                           const uint8_t *done, float alpha)
{
    const int j = threadIdx.x;
    const bool walk = j < n + 4;
    long slot = (h0 - 1 + j) % cap;
    if (slot < 0) slot += cap;
    float v = 0.f;
    if (j < n) {
        const long q = seq0 - 1 + j;  // stream position of the transition's own frame
        bool valid = q >= 3;
#pragma unroll
        for (int k = 1; k <= 3; ++k) {
            long sk = slot - k;
            if (sk < 0) sk += cap;
            if (done[sk]) valid = false;
        }
        if (valid) v = (float)pow((double)tree[2 * L], (double)alpha);
    }
    tree_walk(tree, (int)(L + slot), v, walk, levels);
}

// Frame preprocessing (Sec.3: palette frame -> grey-scale -> linear interpolation to 84 x 84).
// One thread per output pixel, grid (ceil(7056/256), n).  grey = lut[byte] or the byte itself;
// centre-aligned source coordinate, clamped; bilinear blend; round to nearest even.
__global__ __launch_bounds__(256) void k_preprocess(const uint8_t *raw, int H, int W, const float *lut, uint8_t *out)
{
    const int o = blockIdx.x * 256 + threadIdx.x;
    if (o >= net::FRAME) return;
    const int i = o / 84, j = o % 84;
    const uint8_t *im = raw + (long)blockIdx.y * H * W;
    // the source coordinate (i + 1/2) H/84 - 1/2 = ((2i+1) H - 84) / 168 is kept as an exact
    // fraction, so only the blend itself is rounded
    const int ny = min(max((2 * i + 1) * H - 84, 0), 168 * (H - 1));
    const int nx = min(max((2 * j + 1) * W - 84, 0), 168 * (W - 1));
    const int y0 = ny / 168, x0 = nx / 168;
    const int y1 = min(y0 + 1, H - 1), x1 = min(x0 + 1, W - 1);
    const float fy = (float)(ny % 168) / 168.f, fx = (float)(nx % 168) / 168.f;
    auto grey = [&](int y, int x) {
        const uint8_t b = im[(long)y * W + x];
        return lut ? lut[b] : (float)b;
    };
    const float top = grey(y0, x0) * (1.f - fx) + grey(y0, x1) * fx;
    const float bot = grey(y1, x0) * (1.f - fx) + grey(y1, x1) * fx;
    const float v = top * (1.f - fy) + bot * fy;
    out[(long)blockIdx.y * net::FRAME + o] = (uint8_t)fminf(fmaxf(rintf(v), 0.f), 255.f);
}

// Stored layer outputs back in the canonical order: src [n][P][C] (channel-last, fp32 or bf16) ->
// dst fp32 [n][C][P].  One thread per element.
__global__ __launch_bounds__(256) void k_read_act(const void *src, int is_bf16, long n, int P, int Cn, float *dst)
{
    const long e = (long)blockIdx.x * 256 + threadIdx.x;   // canonical index
    if (e >= n * P * Cn) return;
    const long row = e / ((long)P * Cn);
    const int c = (int)((e / P) % Cn), pos = (int)(e % P);
    const long in = (row * P + pos) * Cn + c;
    dst[e] = is_bf16 ? __uint_as_float((uint32_t) static_cast<const uint16_t *>(src)[in] << 16)
                     : static_cast<const float *>(src)[in];
}

// Copies up to eleven short arrays of 4-byte words; grid (blocks, items).
struct CopyOutArgs {
    struct Item {
        uint32_t *dst;
        const uint32_t *src;
        int words;
    } item[11];
};
__global__ __launch_bounds__(256) void k_copy_out(CopyOutArgs A)
{
    const CopyOutArgs::Item it = A.item[blockIdx.y];
    const int t = blockIdx.x * 256 + threadIdx.x;
    if (t < it.words) it.dst[t] = it.src[t];
}

// --------------------------------------------------------------- replay
// Slot `off` frames away from slot i (off in [-3, 1]), wrapping inside the sub-ring that i lies in:
// the whole ring (sub == cap: one stream), or one environment stream's share of it.
__device__ __forceinline__ long ring_slot(long i, long off, long cap, long sub)
{
    const long base = sub == cap ? 0 : (i / sub) * sub;
    long l = (i - base + off) % sub;
    if (l < 0) l += sub;
    return base + l;
}

struct GatherArgs {
    const uint8_t *frames;  // ring [cap][7056]
    const int32_t *meta_a;
    const float *meta_r;
    const uint8_t *meta_done;
    long cap;
    const int32_t *idx;  // [n]
    uint8_t *stack5;     // [n][5][7056] or nullptr
    uint8_t *s, *s_next; // [n][4][7056] or nullptr
    int32_t *a;
    float *r;
    uint8_t *done;
    long sub;            // length of the sub-ring a window wraps in (the capacity for one stream)
};

// Frame-stack gather: transition i reads ring slots i-3 .. i+1 (mod cap);
// grid (n, 5), 16 bytes per thread per trip.
__global__ __launch_bounds__(256) void k_gather(GatherArgs A)
{
    const int j = blockIdx.x, k = blockIdx.y;
    long i = A.idx[j];
    i = i < 0 ? 0 : (i >= A.cap ? A.cap - 1 : i);  // keeps every access inside the ring
    const long slot = ring_slot(i, k - 3, A.cap, A.sub);
    const uint4 *src = reinterpret_cast<const uint4 *>(A.frames + slot * net::FRAME);
    uint4 *d0 = A.stack5 ? reinterpret_cast<uint4 *>(A.stack5 + ((long)j * 5 + k) * net::FRAME) : nullptr;
    uint4 *d1 = (A.s && k < 4) ? reinterpret_cast<uint4 *>(A.s + ((long)j * 4 + k) * net::FRAME) : nullptr;
    uint4 *d2 = (A.s_next && k > 0) ? reinterpret_cast<uint4 *>(A.s_next + ((long)j * 4 + k - 1) * net::FRAME) : nullptr;
    for (int t = threadIdx.x; t < net::FRAME / 16; t += 256) {
        uint4 v = src[t];
        if (d0) d0[t] = v;
        if (d1) d1[t] = v;
        if (d2) d2[t] = v;
    }
    if (k == 0 && threadIdx.x == 0) {
        if (A.a) A.a[j] = A.meta_a[i];
        if (A.r) A.r[j] = A.meta_r[i];
        if (A.done) A.done[j] = A.meta_done[i];
    }
}

// Sampling and the frame-stack gather in one launch (grid (B, 5), 256 threads): the first wave of
// every workgroup repeats the draw of its transition (five workgroups per transition do the same
// descent; it costs less than a launch), workgroup (j, 0) also emits the draw's outputs, then all
// threads copy frame k of the stack.
__global__ __launch_bounds__(256) void k_sample_gather(SampleArgs S, GatherArgs A)
{
    __shared__ long slot_sh;
    const int j = blockIdx.x, k = blockIdx.y;
    if (threadIdx.x < 64) {
        const int jj[1] = {j};
        long slot[1];
        float leaf[1];
        const float total = per_sample_walk<1>(S, jj, threadIdx.x, slot, leaf);
        if (threadIdx.x == 0) {
            slot_sh = slot[0];
            if (k == 0) per_sample_emit(S, j, slot[0], total, leaf[0]);
        }
    }
    __syncthreads();
    const long i = slot_sh;
    const long slot = ring_slot(i, k - 3, A.cap, A.sub);
    const uint4 *src = reinterpret_cast<const uint4 *>(A.frames + slot * net::FRAME);
    uint4 *d0 = reinterpret_cast<uint4 *>(A.stack5 + ((long)j * 5 + k) * net::FRAME);
    for (int t = threadIdx.x; t < net::FRAME / 16; t += 256) d0[t] = src[t];
}

// Ring store: n frames into slots slot0.. (mod cap); grid (n).
__global__ __launch_bounds__(256) void k_replay_write(uint8_t *frames, int32_t *meta_a, float *meta_r,
                                                      uint8_t *meta_done, long cap, long slot0,
                                                      const uint8_t *src, const int32_t *a,
                                                      const float *r, const uint8_t *done)
{
    const long j = blockIdx.x;
    const long slot = (slot0 + j) % cap;
    const uint4 *s = reinterpret_cast<const uint4 *>(src + j * net::FRAME);
    uint4 *d = reinterpret_cast<uint4 *>(frames + slot * net::FRAME);
    for (int t = threadIdx.x; t < net::FRAME / 16; t += 256) d[t] = s[t];
    if (threadIdx.x == 0) {
        if (a) meta_a[slot] = a[j];
        if (r) meta_r[slot] = r[j];
        if (done) meta_done[slot] = done[j];
    }
}

}  // namespace misc
