// fp32 implicit-GEMM kernels on the CDNA4 matrix cores (v_mfma_f32_32x32x2_f32).
//
// Three kernel shapes cover the whole network (Section 3; the forward /
// backward / calculateGradient split of the paper's Layer class is kept as
// three kernel families):
//   k_fwd   : Y[m][n]  = sum_k  A(m,k) * W[n][k]            (conv1-3, fc1 forward)
//   k_dgrad : dX[m][c] = sum_(tap,o) dY(m,tap,o) * W[o][tap][c]   (input gradients)
//   k_wgrad : dW[o][k] = sum_m  dY[m][o] * A(m,k)           (weight gradients)
// A(m,k) is the im2col view of a channel-last activation tensor, formed on the
// fly while staging tiles in LDS; it never exists in memory.
//
// MFMA 32x32x2 operand layout (64-lane wave, lane = 32*h + i):
//   a-operand: A[i][k=h]     b-operand: B[k=h][j=i]
//   result   : acc[r] = D[8*(r/4) + 4*h + r%4][i]
// The reduction order inside a tile is free as long as both operands agree, so
// a lane that reads LDS along k takes 4 consecutive k (one 128-bit read) and
// feeds them to 4 MFMAs: MFMA t pairs k = 4*h + t of both operands.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "net.h"

typedef float v16f __attribute__((ext_vector_type(16)));
typedef float v4f __attribute__((ext_vector_type(4)));

namespace g32 {

constexpr int BK = 32;      // reduction elements staged per iteration
constexpr int LDK = BK + 4; // LDS row stride of a k-contiguous tile (floats)

__device__ __forceinline__ v16f mfma(float a, float b, v16f c)
{
    return __builtin_amdgcn_mfma_f32_32x32x2f32(a, b, c, 0, 0, 0);
}

__device__ __forceinline__ v4f ld4(const float *p) { return *reinterpret_cast<const v4f *>(p); }
// Four input elements as they lie in memory, and their conversion: a staging register holds the raw form,
// so that nothing waits for a load before the tile of the stage before has been multiplied
__device__ __forceinline__ v4f ld4raw(const float *p) { return *reinterpret_cast<const v4f *>(p); }
__device__ __forceinline__ uint32_t ld4raw(const uint8_t *p) { return *reinterpret_cast<const uint32_t *>(p); }
__device__ __forceinline__ v4f cvt4(v4f v) { return v; }
__device__ __forceinline__ v4f cvt4(uint32_t u)
{
    v4f r;
    r.x = (float)(u & 0xFFu);
    r.y = (float)((u >> 8) & 0xFFu);
    r.z = (float)((u >> 16) & 0xFFu);
    r.w = (float)(u >> 24);
    return r;
}
__device__ __forceinline__ v4f ld4(const uint8_t *p)
{
    uint32_t u = *reinterpret_cast<const uint32_t *>(p);
    v4f r;
    r.x = (float)(u & 0xFFu);
    r.y = (float)((u >> 8) & 0xFFu);
    r.z = (float)((u >> 16) & 0xFFu);
    r.w = (float)(u >> 24);
    return r;
}

// ---------------------------------------------------------------------------
// Forward geometries: row m = (sample, out_y, out_x); k = position inside the
// receptive field in the order the weights are stored.
// ---------------------------------------------------------------------------
struct GConv1 {  // 8x8 stride 4, uint8 CHW input, k = (c, p, q)
    using in_t = uint8_t;
    static constexpr int K = 256, N = 32, P = 400;
    static __device__ __forceinline__ long row_off(int m, long xs)
    {
        int n = m / 400, r = m % 400, i = r / 20, j = r % 20;
        return (long)n * xs + (i * 4) * 84 + j * 4;
    }
    static __device__ __forceinline__ int k_off(int k) { return (k >> 6) * 7056 + ((k >> 3) & 7) * 84 + (k & 7); }
};
struct GConv2 {  // 4x4 stride 2 over 20x20x32, k = (p, q, c)
    using in_t = float;
    static constexpr int K = 512, N = 64, P = 81;
    static __device__ __forceinline__ long row_off(int m, long xs)
    {
        int n = m / 81, r = m % 81, i = r / 9, j = r % 9;
        return (long)n * xs + ((i * 2) * 20 + j * 2) * 32;
    }
    static __device__ __forceinline__ int k_off(int k) { return (k >> 7) * 640 + (k & 127); }
};
struct GConv3 {  // 3x3 stride 1 over 9x9x64, k = (p, q, c)
    using in_t = float;
    static constexpr int K = 576, N = 64, P = 49;
    static __device__ __forceinline__ long row_off(int m, long xs)
    {
        int n = m / 49, r = m % 49, i = r / 7, j = r % 7;
        return (long)n * xs + (i * 9 + j) * 64;
    }
    static __device__ __forceinline__ int k_off(int k) { return (k / 192) * 576 + (k % 192); }
};
struct GFc1 {  // dense 3136 -> 512 on the flattened conv3 output
    using in_t = float;
    static constexpr int K = 3136, N = 512, P = 1;
    static __device__ __forceinline__ long row_off(int m, long xs) { return (long)m * xs; }
    static __device__ __forceinline__ int k_off(int k) { return k; }
};

// One launch serves up to three independent (input, weights, output) row
// ranges: the online net on s, the online net on s' and the target net on s'.
struct FwdSeg {
    const void *x;      // input activations (uint8 for conv1, float otherwise)
    const float *w;     // [N][K]
    const float *bias;  // [N] or nullptr (raw partial sums, no activation)
    float *y;           // [M][N] (+ z*split_stride per reduction split)
    int M;              // rows
    int tile_begin;     // first blockIdx.x of this segment
    long xs;            // elements between consecutive samples of x
};
struct FwdArgs {
    FwdSeg seg[3];
    int nseg;
    int klen;           // reduction elements per blockIdx.z
    long split_stride;  // elements between the outputs of consecutive splits
    float scale;        // multiplies the accumulated sum (1/255 for conv1)
};

// KS > 1 cuts every staged reduction slab into KS slices of 32, one per group of waves: the
// workgroup then has KS times the threads, the same loads per thread and KS times the bytes in
// flight, and the reduction loop is KS times shorter.  The KS partial tiles are added through
// LDS at the end.  This is what the small-batch launches use: with few rows there are few
// tiles, and a long dependent chain of short stages per tile is pure latency.
template <int NWT, int KS>
__device__ __forceinline__ void reduce_slices(v16f &acc, float *red /*LDS, (KS-1)*NWT*1024 floats*/, int ks,
                                              int w2, int lane)
{
    if constexpr (KS > 1) {
        __syncthreads();  // every wave is done reading the staged tiles
        if (ks > 0) {
            float *dst = red + ((ks - 1) * NWT + w2) * 1024;
#pragma unroll
            for (int r = 0; r < 16; ++r) dst[r * 64 + lane] = acc[r];
        }
        __syncthreads();
        if (ks == 0) {
#pragma unroll
            for (int s = 0; s < KS - 1; ++s) {
                const float *src = red + (s * NWT + w2) * 1024;
#pragma unroll
                for (int r = 0; r < 16; ++r) acc[r] += src[r * 64 + lane];
            }
        }
    }
}

template <class G, int BM, int BN, int KS = 1>
__global__ __launch_bounds__((BM / 32) * (BN / 32) * KS * 64) void k_fwd(FwdArgs A)
{
    constexpr int NWT = (BM / 32) * (BN / 32), T = NWT * KS * 64;
    constexpr int BKS = BK * KS, LD = BKS + 4, CPR = BKS / 4, RPP = T / CPR;
    constexpr int NA = BM * CPR / T, NB = BN * CPR / T;
    static_assert(NA * T == BM * CPR && NB * T == BN * CPR && G::K % BKS == 0, "tile/threads mismatch");
    static_assert((BM + BN) * LD >= (KS - 1) * NWT * 1024, "reduction scratch does not fit the tiles");
    using in_t = typename G::in_t;
    __shared__ __attribute__((aligned(16))) float smem[(BM + BN) * LD];
    float *As = smem, *Bs = smem + BM * LD;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    // tile order: column tiles of one row tile together, reduction splits apart
    const int t = net::tile_of_workgroup();
    const int by = t % (int)gridDim.y, bx = (t / (int)gridDim.y) % (int)gridDim.x, bz = t / (int)(gridDim.y * gridDim.x);
    FwdSeg S = A.seg[0];
    if (A.nseg > 1 && bx >= A.seg[1].tile_begin) S = A.seg[1];
    if (A.nseg > 2 && bx >= A.seg[2].tile_begin) S = A.seg[2];
    const int m0 = (bx - S.tile_begin) * BM, n0 = by * BN;
    const int kbeg = bz * A.klen, kend = kbeg + A.klen;
    const in_t *x = static_cast<const in_t *>(S.x);

    const int lr = tid / CPR, kq = (tid % CPR) * 4;
    long aoff[NA];
#pragma unroll
    for (int i = 0; i < NA; ++i) {
        int m = m0 + lr + i * RPP;
        aoff[i] = m < S.M ? G::row_off(m, S.xs) : -1;
    }
    v4f ra[NA], rb[NB];
    auto gload = [&](int k0) {
        const int ko = G::k_off(k0 + kq);
#pragma unroll
        for (int i = 0; i < NA; ++i) ra[i] = aoff[i] >= 0 ? ld4(x + aoff[i] + ko) : v4f{0, 0, 0, 0};
#pragma unroll
        for (int i = 0; i < NB; ++i)
            rb[i] = ld4(S.w + (long)(n0 + lr + i * RPP) * G::K + k0 + kq);
    };
    auto sstore = [&]() {
#pragma unroll
        for (int i = 0; i < NA; ++i) *reinterpret_cast<v4f *>(&As[(lr + i * RPP) * LD + kq]) = ra[i];
#pragma unroll
        for (int i = 0; i < NB; ++i) *reinterpret_cast<v4f *>(&Bs[(lr + i * RPP) * LD + kq]) = rb[i];
    };

    const int ks = wave / NWT, w2 = wave % NWT;
    const int wm = w2 % (BM / 32), wn = w2 / (BM / 32);
    const int li = lane & 31, h = lane >> 5;
    const float *ap = &As[(wm * 32 + li) * LD + ks * BK + 4 * h];
    const float *bp = &Bs[(wn * 32 + li) * LD + ks * BK + 4 * h];
    v16f acc = {0};
    const int col = n0 + wn * 32 + li;
    const float bias = S.bias ? S.bias[col] : 0.f;   // requested here, used in the epilogue

    gload(kbeg);
    sstore();
    __syncthreads();
    for (int k0 = kbeg; k0 < kend; k0 += BKS) {
        const bool more = k0 + BKS < kend;
        if (more) gload(k0 + BKS);
#pragma unroll
        for (int kk = 0; kk < BK; kk += 8) {
            v4f a = ld4(ap + kk), b = ld4(bp + kk);
            acc = mfma(a.x, b.x, acc);
            acc = mfma(a.y, b.y, acc);
            acc = mfma(a.z, b.z, acc);
            acc = mfma(a.w, b.w, acc);
        }
        __syncthreads();
        if (more) {
            sstore();
            __syncthreads();
        }
    }
    reduce_slices<NWT, KS>(acc, smem, ks, w2, lane);
    if (ks != 0) return;

    // all values first, then the stores: a wait for the bias inside the bounds-checked branches would be
    // repeated in every branch, and since stores count as outstanding memory operations too, each store
    // would then wait for the one before it to be acknowledged
    float *y = S.y + (long)bz * A.split_stride;
    float v[16];
#pragma unroll
    for (int r = 0; r < 16; ++r) {
        v[r] = acc[r] * A.scale;
        if (S.bias) v[r] = fmaxf(v[r] + bias, 0.f);
    }
#pragma unroll
    for (int r = 0; r < 16; ++r) {
        int m = m0 + wm * 32 + 8 * (r / 4) + 4 * h + (r % 4);
        if (m < S.M) y[(long)m * G::N + col] = v[r];
    }
}

// ---------------------------------------------------------------------------
// Input gradient.  For a stride-S convolution the input pixels fall into S*S
// parity classes (h mod S, w mod S); a pixel of class (a,b) only meets the
// kernel taps p = a + S*u, q = b + S*v, so each class is its own dense GEMM
// over (KH/S)*(KW/S) taps with no multiplications by structural zeros:
//   dX[n][S*h'+a][S*w'+b][c] = sum_{u,v,o} dY[n][h'-u][w'-v][o] * W[o][a+S*u][b+S*v][c]
// (out-of-range dY positions contribute 0).  The result is multiplied by the
// ReLU mask of the layer below (its stored output > 0).
// ---------------------------------------------------------------------------
template <int S_, int TH_, int TW_, int OH_, int OW_, int HP_, int WP_, int CO_, int CI_, int KH_,
          int KW_, int H_, int W_>
struct DGeom {
    static constexpr int S = S_, TH = TH_, TW = TW_, OH = OH_, OW = OW_, HP = HP_, WP = WP_,
                         CO = CO_, CI = CI_, KH = KH_, KW = KW_, H = H_, W = W_;
    static constexpr int K = TH * TW * CO;  // reduction length per class
    static constexpr int PP = HP * WP;      // rows per sample per class
};
using DConv2 = DGeom<2, 2, 2, 9, 9, 10, 10, 64, 32, 4, 4, 20, 20>;
using DConv3 = DGeom<1, 3, 3, 7, 7, 9, 9, 64, 64, 3, 3, 9, 9>;
using DFc1 = DGeom<1, 1, 1, 1, 1, 1, 1, 512, 3136, 1, 1, 1, 1>;

struct DgradArgs {
    const float *dy;    // [B][OH][OW][CO] gradient w.r.t. this layer's pre-activation
    const float *w;     // [CO][KH][KW][CI]
    const float *xact;  // [B][H][W][CI] this layer's input (ReLU output of the layer below)
    float *dx;          // [B][H][W][CI] gradient w.r.t. the pre-activation of the layer below
    int B;
};

// LDS floats of an input-gradient tile
template <int BM, int BN, int KS> constexpr int dgrad_lds() { return BM * (BK * KS + 4) + BK * KS * (BN + 4); }

// Tile number t of a grid of (gx, gy, gz) tiles, computed by the first (BM/32)(BN/32) KS waves of
// the workgroup (a launch may hold wider workgroups: the waves beyond leave at once; a barrier
// counts only the waves that are still there).  Tile order: the parity classes of one row tile
// together, then the row tiles of one column tile.
// The whole reduction is requested before the first stage is staged where it is at most four stages long
// (every layer at the tile shapes of the small-batch step): the tile is then one round trip to memory, not
// one per stage; so are the stored activations the epilogue masks with (the ReLU of the layer below).
template <class D, int BM, int BN, int KS>
__device__ __forceinline__ void dgrad_tile(const DgradArgs &A, int t, int gx, int gz, float *smem)
{
    constexpr int NWT = (BM / 32) * (BN / 32), T = NWT * KS * 64;
    constexpr int BKS = BK * KS, LD = BKS + 4, CPR = BKS / 4, RPP = T / CPR;
    constexpr int NA = BM * CPR / T;
    constexpr int LDB = BN + 4;            // LDS row stride of the [k][c] weight tile
    constexpr int BROWS = T / (BN / 4);    // weight-tile rows filled per pass
    constexpr int NBL = BKS / BROWS;
    static_assert(NA * T == BM * CPR && NBL * BROWS == BKS && D::K % BKS == 0 && D::CO % 4 == 0, "tile/threads mismatch");
    static_assert(BM * LD + BKS * LDB >= (KS - 1) * NWT * 1024, "reduction scratch does not fit the tiles");
    if ((int)threadIdx.x >= T) return;
    float *As = smem, *Bs = smem + BM * LD;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int bz = t % gz, bx = (t / gz) % gx, by = t / (gz * gx);
    const int m0 = bx * BM, n0 = by * BN;
    const int ca = bz / D::S, cb = bz % D::S;
    const int Mc = A.B * D::PP;

    const int lr = tid / CPR, kq = (tid % CPR) * 4;
    int rn[NA], rh[NA], rw[NA];
#pragma unroll
    for (int i = 0; i < NA; ++i) {
        int m = m0 + lr + i * RPP;
        if (m < Mc) {
            rn[i] = m / D::PP;
            int r = m % D::PP;
            rh[i] = r / D::WP;
            rw[i] = r % D::WP;
        } else {
            rn[i] = -1; rh[i] = 0; rw[i] = 0;
        }
    }
    const int br = tid / (BN / 4), bc = (tid % (BN / 4)) * 4;
    constexpr int NST = D::K / BKS;             // reduction stages
    constexpr bool ALLPRE = NST <= 4;           // all of them in flight at once
    constexpr int NREG = ALLPRE ? NST : 1;
    v4f ra[NREG][NA], rb[NREG][NBL];
    auto gload = [&](int k0, v4f (&qa)[NA], v4f (&qb)[NBL]) {
        {   // a staged slab may span several kernel taps: each thread derives the tap of its chunk
            const int k = k0 + kq, tap = k / D::CO, o = k % D::CO;
            const int u = tap / D::TW, v = tap % D::TW;
#pragma unroll
            for (int i = 0; i < NA; ++i) {
                int ii = rh[i] - u, jj = rw[i] - v;
                bool ok = rn[i] >= 0 && ii >= 0 && ii < D::OH && jj >= 0 && jj < D::OW;
                qa[i] = ok ? ld4(A.dy + ((long)(rn[i] * D::OH + ii) * D::OW + jj) * D::CO + o)
                           : v4f{0, 0, 0, 0};
            }
        }
#pragma unroll
        for (int i = 0; i < NBL; ++i) {
            const int k = k0 + br + i * BROWS, tap = k / D::CO, o = k % D::CO;
            const int p = ca + D::S * (tap / D::TW), q = cb + D::S * (tap % D::TW);
            qb[i] = ld4(A.w + ((long)(o * D::KH + p) * D::KW + q) * D::CI + n0 + bc);
        }
    };
    auto sstore = [&](const v4f (&qa)[NA], const v4f (&qb)[NBL]) {
#pragma unroll
        for (int i = 0; i < NA; ++i) *reinterpret_cast<v4f *>(&As[(lr + i * RPP) * LD + kq]) = qa[i];
#pragma unroll
        for (int i = 0; i < NBL; ++i) *reinterpret_cast<v4f *>(&Bs[(br + i * BROWS) * LDB + bc]) = qb[i];
    };

    const int ks = wave / NWT, w2 = wave % NWT;
    const int wm = w2 % (BM / 32), wn = w2 / (BM / 32);
    const int li = lane & 31, h = lane >> 5;
    const float *ap = &As[(wm * 32 + li) * LD + ks * BK + 4 * h];
    const float *bp = &Bs[(ks * BK + 4 * h) * LDB + wn * 32 + li];
    v16f acc = {0};
    auto compute = [&]() {
#pragma unroll
        for (int kk = 0; kk < BK; kk += 8) {
            v4f a = ld4(ap + kk);
            acc = mfma(a.x, bp[(kk + 0) * LDB], acc);
            acc = mfma(a.y, bp[(kk + 1) * LDB], acc);
            acc = mfma(a.z, bp[(kk + 2) * LDB], acc);
            acc = mfma(a.w, bp[(kk + 3) * LDB], acc);
        }
    };
    // where this lane's results go (-1: no such row), and the stored activations there
    const int col = n0 + wn * 32 + li;
    int off[16];
    float xm[16];
    // (the loads are unconditional, from a clamped address: a value chosen between a loaded one and a
    // constant would make the compiler wait for the load right here)
    auto epilogue_loads = [&]() {
        if (__builtin_amdgcn_readfirstlane(ks) != 0) return;   // only the waves of slice 0 write the tile
#pragma unroll
        for (int g = 0; g < 4; ++g) {
            const int mg = m0 + wm * 32 + 8 * g + 4 * h;
            int n = mg / D::PP, rr = mg % D::PP;
            int ph = rr / D::WP, pw = rr % D::WP;
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const int r = 4 * g + j;
                const int o = ((n * D::H + D::S * ph + ca) * D::W + D::S * pw + cb) * D::CI + col;
                const bool valid = mg + j < Mc;
                off[r] = valid ? o : -1;
                xm[r] = A.xact[valid ? o : 0];
                if (++pw == D::WP) {
                    pw = 0;
                    if (++ph == D::HP) { ph = 0; ++n; }
                }
            }
        }
    };

    if constexpr (ALLPRE) {
#pragma unroll
        for (int st = 0; st < NST; ++st) gload(st * BKS, ra[st], rb[st]);
        epilogue_loads();
#pragma unroll
        for (int st = 0; st < NST; ++st) {
            if (st) __syncthreads();   // every wave has read the stage before
            sstore(ra[st], rb[st]);
            __syncthreads();
            compute();
        }
    } else {
        gload(0, ra[0], rb[0]);
        epilogue_loads();
        sstore(ra[0], rb[0]);
        __syncthreads();
        for (int k0 = 0; k0 < D::K; k0 += BKS) {
            const bool more = k0 + BKS < D::K;
            if (more) gload(k0 + BKS, ra[0], rb[0]);
            compute();
            __syncthreads();
            if (more) {
                sstore(ra[0], rb[0]);
                __syncthreads();
            }
        }
    }
    reduce_slices<NWT, KS>(acc, smem, ks, w2, lane);
    if (ks != 0) return;

#pragma unroll
    for (int r = 0; r < 16; ++r)
        if (off[r] >= 0) A.dx[off[r]] = xm[r] > 0.f ? acc[r] : 0.f;
}
template <class D, int BM, int BN, int KS = 1>
__global__ __launch_bounds__((BM / 32) * (BN / 32) * KS * 64) void k_dgrad(DgradArgs A)
{
    __shared__ __attribute__((aligned(16))) float smem[dgrad_lds<BM, BN, KS>()];
    dgrad_tile<D, BM, BN, KS>(A, net::tile_of_workgroup(), gridDim.x, gridDim.z, smem);
}

// ---------------------------------------------------------------------------
// Weight gradient: dW[o][k] = sum_m dY[m][o] * A(m,k), db[o] = sum_m dY[m][o].
// The reduction runs over all output positions of all samples; it is cut into
// blockIdx.z splits of consecutive rows, each writing its own partial result
// ([W..., b...] per split), which the optimizer kernel adds up in a fixed order
// (no floating-point atomics, so results are reproducible).
// ---------------------------------------------------------------------------
struct WgradArgs {
    const float *dy;   // [B*P][N]
    const void *x;     // layer input (uint8 for conv1)
    float *part;       // [splits][N*K + N]
    int B;
    int rps;           // reduction rows (output positions) per split, a multiple of 32
    long xs;           // elements between consecutive samples of x
    long part_stride;  // elements between consecutive splits
    float scale;       // multiplies dW (1/255 for conv1)
};

// LDS of one weight-gradient tile pair, in floats
template <int BMO, int BNK> constexpr int wgrad_lds() { return BK * (BMO + 4) + BK * (BNK + 4); }

// One weight-gradient tile: output channels [by*BMO, +BMO) x im2col columns [bx*BNK, +BNK) over the
// rows of split bz, computed by the first T threads of the workgroup; Ys/Xs are the workgroup's LDS.
template <class G, int BMO, int BNK>
__device__ __forceinline__ void wgrad_tile(const WgradArgs &A, int bx, int by, int bz, float *lds)
{
    constexpr int T = (BMO / 32) * (BNK / 32) * 64;
    constexpr int LDY = BMO + 4, LDX = BNK + 4;
    constexpr int YR = T / (BMO / 4), XR = T / (BNK / 4);  // tile rows filled per pass
    constexpr int NY = (BK + YR - 1) / YR, NX = (BK + XR - 1) / XR;
    using in_t = typename G::in_t;
    if ((int)threadIdx.x >= T) return;   // a wider workgroup: the waves beyond the tile's leave at once
    float *Ys = lds, *Xs = lds + BK * LDY;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int kc0 = bx * BNK, o0 = by * BMO;
    const int mbeg = bz * A.rps;
    const int mend = min(mbeg + A.rps, A.B * G::P);
    const in_t *x = static_cast<const in_t *>(A.x);

    const int yr = tid / (BMO / 4), yc = (tid % (BMO / 4)) * 4;
    const int xr = tid / (BNK / 4), xc = (tid % (BNK / 4)) * 4;
    const int xko = G::k_off(kc0 + xc);
    using raw_t = decltype(ld4raw(x));
    v4f ry[NY];
    raw_t rx[NX];
    auto gload = [&](int mb) {
#pragma unroll
        for (int i = 0; i < NY; ++i) {
            int r = yr + i * YR, m = mb + r;
            ry[i] = (r < BK && m < mend) ? ld4(A.dy + (long)m * G::N + o0 + yc) : v4f{0, 0, 0, 0};
        }
#pragma unroll
        for (int i = 0; i < NX; ++i) {
            int r = xr + i * XR, m = mb + r;
            rx[i] = (r < BK && m < mend) ? ld4raw(x + G::row_off(m, A.xs) + xko) : raw_t{};
        }
    };
    auto sstore = [&]() {
#pragma unroll
        for (int i = 0; i < NY; ++i) {
            int r = yr + i * YR;
            if (r < BK) *reinterpret_cast<v4f *>(&Ys[r * LDY + yc]) = ry[i];
        }
#pragma unroll
        for (int i = 0; i < NX; ++i) {
            int r = xr + i * XR;
            if (r < BK) *reinterpret_cast<v4f *>(&Xs[r * LDX + xc]) = cvt4(rx[i]);
        }
    };

    const int wo = wave % (BMO / 32), wk = wave / (BMO / 32);
    const int li = lane & 31, h = lane >> 5;
    const float *yp = &Ys[(4 * h) * LDY + wo * 32 + li];
    const float *xp = &Xs[(4 * h) * LDX + wk * 32 + li];
    const bool do_bias = bx == 0 && wk == 0;
    v16f acc = {0}, accb = {0};

    if (mbeg < mend) {
        gload(mbeg);
        sstore();
    }
    __syncthreads();
    for (int mb = mbeg; mb < mend; mb += BK) {
        const bool more = mb + BK < mend;
        if (more) gload(mb + BK);
#pragma unroll
        for (int kk = 0; kk < BK; kk += 8) {
#pragma unroll
            for (int t = 0; t < 4; ++t) {
                float a = yp[(kk + t) * LDY], b = xp[(kk + t) * LDX];
                acc = mfma(a, b, acc);
                if (do_bias) accb = mfma(a, 1.0f, accb);
            }
        }
        __syncthreads();
        if (more) {
            sstore();
            __syncthreads();
        }
    }

    float *part = A.part + (long)bz * A.part_stride;
    const int col = kc0 + wk * 32 + li;
#pragma unroll
    for (int r = 0; r < 16; ++r) {
        int o = o0 + wo * 32 + 8 * (r / 4) + 4 * h + (r % 4);
        part[(long)o * G::K + col] = acc[r] * A.scale;
        if (do_bias && li == 0) part[(long)G::N * G::K + o] = accb[r];
    }
}

// tile number -> (bx, by, bz) of a grid (gx, gy, gz): with row splits (conv layers) all tiles of one
// split together; without (fc1) all output tiles of one input-column tile together
__device__ __forceinline__ void wgrad_tile_of(int t, int gx, int gy, int gz, int &bx, int &by, int &bz)
{
    if (gz > 1) {
        bx = t % gx; by = (t / gx) % gy; bz = t / (gx * gy);
    } else {
        by = t % gy; bx = t / gy; bz = 0;
    }
}

template <class G, int BMO, int BNK>
__global__ __launch_bounds__((BMO / 32) * (BNK / 32) * 64) void k_wgrad(WgradArgs A)
{
    __shared__ __attribute__((aligned(16))) float lds[wgrad_lds<BMO, BNK>()];
    int bx, by, bz;
    wgrad_tile_of(net::tile_of_workgroup(), gridDim.x, gridDim.y, gridDim.z, bx, by, bz);
    wgrad_tile<G, BMO, BNK>(A, bx, by, bz, lds);
}

}  // namespace g32
