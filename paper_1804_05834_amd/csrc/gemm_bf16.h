// bf16 implicit-GEMM kernels on the CDNA4 matrix cores
// (v_mfma_f32_32x32x16_bf16: bf16 operands, fp32 accumulation).
//
// Same three kernel families and the same geometries as gemm_fp32.h; what
// differs is the staging:
//   * a reduction stage is 64 elements (128 bytes per row), moved as 16-byte
//     chunks; conv1 converts its uint8 pixels to bf16 while staging (integers
//     up to 255 are exact in bf16);
//   * an operand whose reduction index is the SLOW index in memory (weights in
//     the input-gradient kernel, both operands of the weight-gradient kernel)
//     is staged as it lies in memory, [reduction][column], and read with the
//     LDS transpose load (ds_read_b64_tr_b16), which hands each lane four
//     consecutive reduction elements of its column: within a group of 16 lanes,
//     lane s addresses row s/4, columns 4*(s%4)..+3 of a 4x16 block and lane d
//     receives column d of that block.
//
// MFMA 32x32x16 operand layout (lane = 32*h + i): a-operand A[i][8h..8h+7],
// b-operand B[8h..8h+7][i], result acc[r] = D[8*(r/4) + 4*h + r%4][i].
//
// Kernels whose output is channel-last ([position][channel]) feed the WEIGHT
// fragment as the a-operand and the activation fragment as the b-operand, i.e.
// they compute the transposed tile: a lane then owns one output position and 4
// groups of 4 consecutive channels, which it stores as 8-byte pieces (instead of
// sixteen 2-byte stores at a 64-byte row stride).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "gemm_fp32.h"

namespace gbf {

typedef __bf16 v8bf __attribute__((ext_vector_type(8)));
typedef short v4s __attribute__((ext_vector_type(4)));
typedef uint16_t bf16_t;  // storage type

constexpr int BK = 64;       // reduction elements per stage
constexpr int LDK = BK + 8;  // LDS row stride (elements) of a k-contiguous tile: 144 bytes

__device__ __forceinline__ v16f mfma(v8bf a, v8bf b, v16f c)
{
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
}

__device__ __forceinline__ bf16_t f2bf(float f)  // round to nearest even
{
    return __builtin_bit_cast(bf16_t, (__bf16)f);
}
// four floats -> four bf16 in 8 bytes
__device__ __forceinline__ uint2 pack4(float a, float b, float c, float d)
{
    typedef __bf16 v2bf __attribute__((ext_vector_type(2)));
    v2bf lo = {(__bf16)a, (__bf16)b}, hi = {(__bf16)c, (__bf16)d};
    return uint2{__builtin_bit_cast(uint32_t, lo), __builtin_bit_cast(uint32_t, hi)};
}
__device__ __forceinline__ float bf2f(bf16_t b) { return __uint_as_float((uint32_t)b << 16); }

// 8 consecutive reduction elements as one 16-byte value
__device__ __forceinline__ uint4 ld8(const bf16_t *p) { return *reinterpret_cast<const uint4 *>(p); }
__device__ __forceinline__ uint32_t pack2_u8(uint32_t lo, uint32_t hi)
{
    return (__float_as_uint((float)lo) >> 16) | (__float_as_uint((float)hi) & 0xFFFF0000u);
}
__device__ __forceinline__ uint4 ld8(const uint8_t *p)  // 8 pixels -> 8 bf16 (exact)
{
    uint32_t a = *reinterpret_cast<const uint32_t *>(p), b = *reinterpret_cast<const uint32_t *>(p + 4);
    uint4 r;
    r.x = pack2_u8(a & 0xFFu, (a >> 8) & 0xFFu);
    r.y = pack2_u8((a >> 16) & 0xFFu, a >> 24);
    r.z = pack2_u8(b & 0xFFu, (b >> 8) & 0xFFu);
    r.w = pack2_u8((b >> 16) & 0xFFu, b >> 24);
    return r;
}

// Barrier that orders LDS traffic only: global loads and stores issued earlier stay in flight
// across it (__syncthreads() would wait for all of them first).
__device__ __forceinline__ void sync_lds()
{
    asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
}

__device__ __forceinline__ v8bf frag_k(const bf16_t *p)  // 8 consecutive k of one row
{
    return *reinterpret_cast<const v8bf *>(p);
}
// 8 consecutive reduction rows of one column out of a [reduction][column] tile.
// p points at (row0 + s/4, col_block + 4*(s%4)) for this lane; ld = row stride.
__device__ __forceinline__ v8bf frag_tr(const bf16_t *p, int ld)
{
    typedef __attribute__((address_space(3))) v4s *lds_v4s;
    v4s lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_v4s)(p));
    v4s hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_v4s)(p + 4 * ld));
    typedef short v8s __attribute__((ext_vector_type(8)));
    v8s r = {lo.x, lo.y, lo.z, lo.w, hi.x, hi.y, hi.z, hi.w};
    return __builtin_bit_cast(v8bf, r);
}

using g32::GConv1;
using g32::GConv2;
using g32::GConv3;
using g32::GFc1;

template <class G> struct in_type { using t = bf16_t; };
template <> struct in_type<GConv1> { using t = uint8_t; };

// ---------------------------------------------------------------------------
struct FwdSeg {
    const void *x;      // uint8 (conv1) or bf16 activations
    const bf16_t *w;    // [N][K] bf16 copy of the weights
    const float *bias;  // [N] fp32 (master copy) or nullptr
    void *y;            // bf16 [M][N], or fp32 raw partial sums when RAW
    int M;
    int tile_begin;
    long xs;
};
struct FwdArgs {
    FwdSeg seg[3];
    int nseg;
    int klen;
    long split_stride;
    float scale;
};

// Workgroup tile BM x BN; each wave owns WM x WN MFMA blocks of 32x32.
template <class G, int BM, int BN, int WM, int WN, bool RAW>
__global__ __launch_bounds__((BM / (32 * WM)) * (BN / (32 * WN)) * 64) void k_fwd(FwdArgs A)
{
    constexpr int WAVES_M = BM / (32 * WM), WAVES_N = BN / (32 * WN), T = WAVES_M * WAVES_N * 64;
    constexpr int NA = BM * 8 / T, NB = (BN * 8 + T - 1) / T;
    static_assert(NA * T == BM * 8, "tile/threads mismatch");
    using in_t = typename in_type<G>::t;
    __shared__ __attribute__((aligned(16))) bf16_t As[BM * LDK];
    __shared__ __attribute__((aligned(16))) bf16_t Bs[BN * LDK];

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

    const int lr = tid >> 3, kq = (tid & 7) * 8;
    long aoff[NA];
#pragma unroll
    for (int i = 0; i < NA; ++i) {
        int m = m0 + lr + i * (T / 8);
        aoff[i] = m < S.M ? G::row_off(m, S.xs) : -1;
    }
    uint4 ra[NA], rb[NB];
    auto gload = [&](int k0) {
        const int ko = G::k_off(k0 + kq);
#pragma unroll
        for (int i = 0; i < NA; ++i) ra[i] = aoff[i] >= 0 ? ld8(x + aoff[i] + ko) : uint4{0, 0, 0, 0};
#pragma unroll
        for (int i = 0; i < NB; ++i) {
            int r = lr + i * (T / 8);
            if (r < BN) rb[i] = ld8(S.w + (long)(n0 + r) * G::K + k0 + kq);
        }
    };
    auto sstore = [&]() {
#pragma unroll
        for (int i = 0; i < NA; ++i) *reinterpret_cast<uint4 *>(&As[(lr + i * (T / 8)) * LDK + kq]) = ra[i];
#pragma unroll
        for (int i = 0; i < NB; ++i) {
            int r = lr + i * (T / 8);
            if (r < BN) *reinterpret_cast<uint4 *>(&Bs[r * LDK + kq]) = rb[i];
        }
    };

    const int wm = wave % WAVES_M, wn = wave / WAVES_M;
    const int li = lane & 31, h = lane >> 5;
    const bf16_t *ap = &As[(wm * 32 * WM + li) * LDK + 8 * h];
    const bf16_t *bp = &Bs[(wn * 32 * WN + li) * LDK + 8 * h];
    v16f acc[WM][WN];
#pragma unroll
    for (int a = 0; a < WM; ++a)
#pragma unroll
        for (int b = 0; b < WN; ++b) acc[a][b] = v16f{0};

    // bias of this lane's channels, requested before the loop so the epilogue does not wait for it
    v4f bias_r[WN][4];
    if (!RAW) {
#pragma unroll
        for (int b = 0; b < WN; ++b)
#pragma unroll
            for (int g = 0; g < 4; ++g)
                bias_r[b][g] = *reinterpret_cast<const v4f *>(S.bias + n0 + (wn * WN + b) * 32 + 8 * g + 4 * h);
    }

    gload(kbeg);
    sstore();
    __syncthreads();
    for (int k0 = kbeg; k0 < kend; k0 += BK) {
        const bool more = k0 + BK < kend;
        if (more) gload(k0 + BK);
#pragma unroll
        for (int kk = 0; kk < BK; kk += 16) {
            v8bf fa[WM], fb[WN];
#pragma unroll
            for (int a = 0; a < WM; ++a) fa[a] = frag_k(ap + a * 32 * LDK + kk);
#pragma unroll
            for (int b = 0; b < WN; ++b) fb[b] = frag_k(bp + b * 32 * LDK + kk);
#pragma unroll
            for (int a = 0; a < WM; ++a)
#pragma unroll
                for (int b = 0; b < WN; ++b) acc[a][b] = mfma(fb[b], fa[a], acc[a][b]);  // transposed tile
        }
        __syncthreads();
        if (more) {
            sstore();
            __syncthreads();
        }
    }

    // acc[a][b][4g + j] = Y[row m = block a, lane li][channel = block b, 8g + 4h + j]
    if constexpr (RAW) {
#pragma unroll
        for (int a = 0; a < WM; ++a) {
            const int m = m0 + (wm * WM + a) * 32 + li;
            if (m >= S.M) continue;
            float *y = static_cast<float *>(S.y) + (long)bz * A.split_stride;
#pragma unroll
            for (int b = 0; b < WN; ++b)
#pragma unroll
                for (int g = 0; g < 4; ++g) {
                    const int col = n0 + (wn * WN + b) * 32 + 8 * g + 4 * h;
                    *reinterpret_cast<v4f *>(y + (long)m * G::N + col) =
                        v4f{acc[a][b][4 * g] * A.scale, acc[a][b][4 * g + 1] * A.scale,
                            acc[a][b][4 * g + 2] * A.scale, acc[a][b][4 * g + 3] * A.scale};
                }
        }
    } else {
        // bias + ReLU, the bf16 tile goes through LDS (the operand tiles are no longer read: the
        // loop ends on a barrier) and leaves as whole rows, 16 bytes per lane
        static_assert(RAW || BN <= BK, "the output tile is staged in the A tile's LDS");
#pragma unroll
        for (int a = 0; a < WM; ++a)
#pragma unroll
            for (int b = 0; b < WN; ++b)
#pragma unroll
                for (int g = 0; g < 4; ++g) {
                    const int col = (wn * WN + b) * 32 + 8 * g + 4 * h;
                    const v4f bv = bias_r[b][g];
                    *reinterpret_cast<uint2 *>(&As[((wm * WM + a) * 32 + li) * LDK + col]) =
                        pack4(fmaxf(acc[a][b][4 * g] * A.scale + bv.x, 0.f), fmaxf(acc[a][b][4 * g + 1] * A.scale + bv.y, 0.f),
                              fmaxf(acc[a][b][4 * g + 2] * A.scale + bv.z, 0.f), fmaxf(acc[a][b][4 * g + 3] * A.scale + bv.w, 0.f));
                }
        __syncthreads();
        constexpr int CH = BN / 8;
        static_assert((BM * CH) % T == 0, "tile/threads mismatch");
#pragma unroll
        for (int i = 0; i < BM * CH / T; ++i) {
            const int c = tid + i * T, row = c / CH, ch = c % CH;
            if (m0 + row < S.M)
                *reinterpret_cast<uint4 *>(static_cast<bf16_t *>(S.y) + (long)(m0 + row) * G::N + n0 + ch * 8) =
                    *reinterpret_cast<const uint4 *>(&As[row * LDK + ch * 8]);
        }
    }
}

// ---------------------------------------------------------------------------
using g32::DConv2;
using g32::DConv3;
using g32::DFc1;

struct DgradArgs {
    const bf16_t *dy;    // [B][OH][OW][CO]
    const bf16_t *w;     // [CO][KH][KW][CI] bf16 copy of the weights
    const bf16_t *xact;  // [B][H][W][CI] layer input (ReLU output of the layer below)
    bf16_t *dx;          // [B][H][W][CI]
    int B;
};

template <class D, int BM, int BN, int WM, int WN>
__global__ __launch_bounds__((BM / (32 * WM)) * (BN / (32 * WN)) * 64) void k_dgrad(DgradArgs A)
{
    constexpr int WAVES_M = BM / (32 * WM), WAVES_N = BN / (32 * WN), T = WAVES_M * WAVES_N * 64;
    constexpr int NA = BM * 8 / T;
    constexpr int LDB = BN + 8;          // row stride of the [k][c] weight tile
    constexpr int BCH = BN / 8;          // 16-byte chunks per weight-tile row
    constexpr int BROWS = T / BCH;       // rows filled per pass
    constexpr int NBL = (BK + BROWS - 1) / BROWS;
    static_assert(NA * T == BM * 8 && D::CO % BK == 0, "tile/threads mismatch");
    __shared__ __attribute__((aligned(16))) bf16_t As[BM * LDK];
    __shared__ __attribute__((aligned(16))) bf16_t Bs[BK * LDB];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    // tile order: the parity classes of one row tile together, then the row tiles of one column tile
    const int t = net::tile_of_workgroup();
    const int bz = t % (int)gridDim.z, bx = (t / (int)gridDim.z) % (int)gridDim.x, by = t / (int)(gridDim.z * gridDim.x);
    const int m0 = bx * BM, n0 = by * BN;
    const int ca = bz / D::S, cb = bz % D::S;
    const int Mc = A.B * D::PP;

    const int lr = tid >> 3, kq = (tid & 7) * 8;
    int rn[NA], rh[NA], rw[NA];
#pragma unroll
    for (int i = 0; i < NA; ++i) {
        int m = m0 + lr + i * (T / 8);
        if (m < Mc) {
            rn[i] = m / D::PP;
            int r = m % D::PP;
            rh[i] = r / D::WP;
            rw[i] = r % D::WP;
        } else {
            rn[i] = -1; rh[i] = 0; rw[i] = 0;
        }
    }
    const int br = tid / BCH, bc = (tid % BCH) * 8;
    uint4 ra[NA], rb[NBL];
    auto gload = [&](int k0) {
        const int tap = k0 / D::CO, o0 = k0 % D::CO;
        const int u = tap / D::TW, v = tap % D::TW;
#pragma unroll
        for (int i = 0; i < NA; ++i) {
            int ii = rh[i] - u, jj = rw[i] - v;
            bool ok = rn[i] >= 0 && ii >= 0 && ii < D::OH && jj >= 0 && jj < D::OW;
            ra[i] = ok ? ld8(A.dy + ((long)(rn[i] * D::OH + ii) * D::OW + jj) * D::CO + o0 + kq)
                       : uint4{0, 0, 0, 0};
        }
        const int p = ca + D::S * u, q = cb + D::S * v;
#pragma unroll
        for (int i = 0; i < NBL; ++i) {
            int r = br + i * BROWS;
            if (r < BK) rb[i] = ld8(A.w + ((long)((o0 + r) * D::KH + p) * D::KW + q) * D::CI + n0 + bc);
        }
    };
    auto sstore = [&]() {
#pragma unroll
        for (int i = 0; i < NA; ++i) *reinterpret_cast<uint4 *>(&As[(lr + i * (T / 8)) * LDK + kq]) = ra[i];
#pragma unroll
        for (int i = 0; i < NBL; ++i) {
            int r = br + i * BROWS;
            if (r < BK) *reinterpret_cast<uint4 *>(&Bs[r * LDB + bc]) = rb[i];
        }
    };

    const int wm = wave % WAVES_M, wn = wave / WAVES_M;
    const int li = lane & 31, h = lane >> 5, s16 = lane & 15, half = (lane >> 4) & 1;
    const bf16_t *ap = &As[(wm * 32 * WM + li) * LDK + 8 * h];
    // transpose-read base: row 8h + s/4, column (wave block) + 16*half + 4*(s%4)
    const bf16_t *bp = &Bs[(8 * h + (s16 >> 2)) * LDB + wn * 32 * WN + 16 * half + 4 * (s16 & 3)];
    v16f acc[WM][WN];
#pragma unroll
    for (int a = 0; a < WM; ++a)
#pragma unroll
        for (int b = 0; b < WN; ++b) acc[a][b] = v16f{0};

    // where this lane's results go, and the stored activations there (the ReLU mask), requested
    // before the loop so the epilogue does not wait for them
    long obase[WM];
    uint2 xa[WM][WN][4];
#pragma unroll
    for (int a = 0; a < WM; ++a) {
        const int m = m0 + (wm * WM + a) * 32 + li;
        obase[a] = -1;
        if (m < Mc) {
            const int n = m / D::PP, rr = m % D::PP;
            const int hh = D::S * (rr / D::WP) + ca, ww = D::S * (rr % D::WP) + cb;
            obase[a] = ((long)(n * D::H + hh) * D::W + ww) * D::CI + n0 + wn * WN * 32 + 4 * h;
        }
#pragma unroll
        for (int b = 0; b < WN; ++b)
#pragma unroll
            for (int g = 0; g < 4; ++g)
                xa[a][b][g] = obase[a] >= 0 ? *reinterpret_cast<const uint2 *>(A.xact + obase[a] + b * 32 + 8 * g)
                                            : uint2{0, 0};
    }

    gload(0);
    sstore();
    __syncthreads();
    for (int k0 = 0; k0 < D::K; k0 += BK) {
        const bool more = k0 + BK < D::K;
        if (more) gload(k0 + BK);
#pragma unroll
        for (int kk = 0; kk < BK; kk += 16) {
            v8bf fa[WM], fb[WN];
#pragma unroll
            for (int a = 0; a < WM; ++a) fa[a] = frag_k(ap + a * 32 * LDK + kk);
#pragma unroll
            for (int b = 0; b < WN; ++b) fb[b] = frag_tr(bp + kk * LDB + b * 32, LDB);
#pragma unroll
            for (int a = 0; a < WM; ++a)
#pragma unroll
                for (int b = 0; b < WN; ++b) acc[a][b] = mfma(fb[b], fa[a], acc[a][b]);  // transposed tile
        }
        __syncthreads();
        if (more) {
            sstore();
            __syncthreads();
        }
    }

    // acc[a][b][4g + j] = dX[position m = block a, lane li][channel = block b, 8g + 4h + j]
#pragma unroll
    for (int a = 0; a < WM; ++a) {
        if (obase[a] < 0) continue;
#pragma unroll
        for (int b = 0; b < WN; ++b) {
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                const uint2 x = xa[a][b][g];
                // ReLU mask of the layer below: its stored output is > 0
                const float v0 = (int16_t)(x.x & 0xFFFFu) > 0 ? acc[a][b][4 * g] : 0.f;
                const float v1 = (int16_t)(x.x >> 16) > 0 ? acc[a][b][4 * g + 1] : 0.f;
                const float v2 = (int16_t)(x.y & 0xFFFFu) > 0 ? acc[a][b][4 * g + 2] : 0.f;
                const float v3 = (int16_t)(x.y >> 16) > 0 ? acc[a][b][4 * g + 3] : 0.f;
                *reinterpret_cast<uint2 *>(A.dx + obase[a] + b * 32 + 8 * g) = pack4(v0, v1, v2, v3);
            }
        }
    }
}

// ---------------------------------------------------------------------------
struct WgradArgs {
    const bf16_t *dy;  // [B*P][N]
    const void *x;     // layer input: uint8 (conv1) or bf16
    float *part;       // [splits][N*K + N] fp32
    int B;
    int rps;           // reduction rows per split, a multiple of 64
    long xs;
    long part_stride;
    float scale;
};

template <class G, int BMO, int BNK, int WM, int WN>
__global__ __launch_bounds__((BMO / (32 * WM)) * (BNK / (32 * WN)) * 64) void k_wgrad(WgradArgs A)
{
    constexpr int WAVES_M = BMO / (32 * WM), WAVES_N = BNK / (32 * WN), T = WAVES_M * WAVES_N * 64;
    constexpr int LDY = BMO + 8, LDX = BNK + 8;
    constexpr int YCH = BMO / 8, XCH = BNK / 8;          // 16-byte chunks per tile row
    constexpr int YR = T / YCH, XR = T / XCH;            // rows filled per pass
    constexpr int NY = (BK + YR - 1) / YR, NX = (BK + XR - 1) / XR;
    using in_t = typename in_type<G>::t;
    __shared__ __attribute__((aligned(16))) bf16_t Ys[BK * LDY];
    __shared__ __attribute__((aligned(16))) bf16_t Xs[BK * LDX];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    // tile order: with row splits (conv layers) all tiles of one split together; without
    // (fc1) all output tiles of one input-column tile together
    const int t = net::tile_of_workgroup();
    int bx, by, bz;
    if (gridDim.z > 1) {
        bx = t % (int)gridDim.x; by = (t / (int)gridDim.x) % (int)gridDim.y; bz = t / (int)(gridDim.x * gridDim.y);
    } else {
        by = t % (int)gridDim.y; bx = t / (int)gridDim.y; bz = 0;
    }
    const int kc0 = bx * BNK, o0 = by * BMO;
    const int mbeg = bz * A.rps;
    const int mend = min(mbeg + A.rps, A.B * G::P);
    const in_t *x = static_cast<const in_t *>(A.x);

    const int yr = tid / YCH, yc = (tid % YCH) * 8;
    const int xr = tid / XCH, xc = (tid % XCH) * 8;
    const int xko = G::k_off(kc0 + xc);
    uint4 ry[NY], rx[NX];
    auto gload = [&](int mb) {
#pragma unroll
        for (int i = 0; i < NY; ++i) {
            int r = yr + i * YR, m = mb + r;
            ry[i] = (r < BK && m < mend) ? ld8(A.dy + (long)m * G::N + o0 + yc) : uint4{0, 0, 0, 0};
        }
#pragma unroll
        for (int i = 0; i < NX; ++i) {
            int r = xr + i * XR, m = mb + r;
            rx[i] = (r < BK && m < mend) ? ld8(x + G::row_off(m, A.xs) + xko) : uint4{0, 0, 0, 0};
        }
    };
    auto sstore = [&]() {
#pragma unroll
        for (int i = 0; i < NY; ++i) {
            int r = yr + i * YR;
            if (r < BK) *reinterpret_cast<uint4 *>(&Ys[r * LDY + yc]) = ry[i];
        }
#pragma unroll
        for (int i = 0; i < NX; ++i) {
            int r = xr + i * XR;
            if (r < BK) *reinterpret_cast<uint4 *>(&Xs[r * LDX + xc]) = rx[i];
        }
    };

    const int wo = wave % WAVES_M, wk = wave / WAVES_M;
    const int li = lane & 31, h = lane >> 5, s16 = lane & 15, half = (lane >> 4) & 1;
    const int trow = 8 * h + (s16 >> 2), tcol = 16 * half + 4 * (s16 & 3);
    const bf16_t *yp = &Ys[trow * LDY + wo * 32 * WM + tcol];
    const bf16_t *xp = &Xs[trow * LDX + wk * 32 * WN + tcol];
    const bool do_bias = bx == 0 && wk == 0;
    v16f acc[WM][WN], accb[WM];
#pragma unroll
    for (int a = 0; a < WM; ++a) {
        accb[a] = v16f{0};
#pragma unroll
        for (int b = 0; b < WN; ++b) acc[a][b] = v16f{0};
    }
    v8bf ones;
#pragma unroll
    for (int e = 0; e < 8; ++e) ones[e] = (__bf16)1.0f;

    if (mbeg < mend) {
        gload(mbeg);
        sstore();
    }
    __syncthreads();
    for (int mb = mbeg; mb < mend; mb += BK) {
        const bool more = mb + BK < mend;
        if (more) gload(mb + BK);
#pragma unroll
        for (int kk = 0; kk < BK; kk += 16) {
            v8bf fa[WM], fb[WN];
#pragma unroll
            for (int a = 0; a < WM; ++a) fa[a] = frag_tr(yp + kk * LDY + a * 32, LDY);
#pragma unroll
            for (int b = 0; b < WN; ++b) fb[b] = frag_tr(xp + kk * LDX + b * 32, LDX);
#pragma unroll
            for (int a = 0; a < WM; ++a) {
#pragma unroll
                for (int b = 0; b < WN; ++b) acc[a][b] = mfma(fa[a], fb[b], acc[a][b]);
                if (do_bias) accb[a] = mfma(fa[a], ones, accb[a]);
            }
        }
        __syncthreads();
        if (more) {
            sstore();
            __syncthreads();
        }
    }

    float *part = A.part + (long)bz * A.part_stride;
#pragma unroll
    for (int a = 0; a < WM; ++a) {
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            int o = o0 + (wo * WM + a) * 32 + 8 * (r / 4) + 4 * h + (r % 4);
#pragma unroll
            for (int b = 0; b < WN; ++b) {
                int col = kc0 + (wk * WN + b) * 32 + li;
                part[(long)o * G::K + col] = acc[a][b][r] * A.scale;
            }
            if (do_bias && li == 0) part[(long)G::N * G::K + o] = accb[a][r];
        }
    }
}



// ===========================================================================
// conv1 (8x8 stride 4 over the uint8 frame stack), specialised.
//
// The generic kernels gather conv1's im2col rows from global memory in 4/8-byte
// pieces at 84-byte strides, which is address-bound.  Here one workgroup owns
// one sample: its four 84x84 frames are read once with 16-byte loads -- from a
// materialised state, or straight from the replay ring through the sampled
// slot (the frame-stack gather fused into the loader) -- converted to bf16 and
// kept in LDS as [4][84][84].  Every operand of the 8x8/4 convolution is then
// an LDS read at a computed address:
//   forward : pixel row of A = 8 consecutive q for one (c,p): 16 bytes;
//             all of W (32x256 bf16) sits in registers as 16 b-operands;
//   wgrad   : 8 consecutive pixels of one im2col column, fetched with the LDS
//             transpose load, whose lanes each supply their own address.
// ===========================================================================
namespace c1 {
constexpr int FR = 84 * 84;       // elements per frame
constexpr int XIN = 4 * FR;       // staged state, elements

struct Src {                      // where the four frames of sample n come from
    const uint8_t *x;             // explicit states [n][4][84][84] (idx == nullptr) or the ring
    long xs;                      // bytes between samples (explicit)
    const int32_t *idx;           // sampled slots (ring mode)
    long cap;                     // ring capacity
    int shift;                    // 0: frames i-3..i (s), 1: frames i-2..i+1 (s')
};

// The sampled slot of sample n (ring mode; 0 otherwise).  Fetched one sample ahead of the frame
// loads that depend on it, so that the two memory latencies do not add up.
// The value stays in a vector register until it is used (frame_ptr makes it scalar): were it
// made scalar where it is loaded, the wave would wait for every outstanding load right there.
__device__ __forceinline__ int sample_slot(const Src &S, int n)
{
    int zero;
    asm volatile("v_mov_b32 %0, 0" : "=v"(zero));  // opaque, so the load below is a vector load
    return S.idx ? S.idx[n + zero] : 0;
}

__device__ __forceinline__ const uint8_t *frame_ptr(const Src &S, int n, int slot_n, int k)
{
    if (!S.idx) return S.x + (long)n * S.xs + (long)k * FR;
    long i = __builtin_amdgcn_readfirstlane(slot_n);
    i = i < 0 ? 0 : (i >= S.cap ? S.cap - 1 : i);
    long slot = i - 3 + k + S.shift;  // within [-3, cap+1]: one wrap at most (cap >= 5)
    if (slot < 0) slot += S.cap;
    if (slot >= S.cap) slot -= S.cap;
    return S.x + slot * FR;
}

// Staging of frames k0 .. k0+NF-1 of sample n as bf16 into xin[(k-k0)*FR ...], in two halves so
// that the global loads of the next sample can be in flight while the current one is computed:
// stage_load issues every 16-byte load of a thread, stage_store converts (16 pixels -> 16 bf16)
// and writes two 16-byte LDS stores per load.
template <int T, int NF> struct Staged {
    static constexpr int CH = FR / 8, TOT = NF * CH, NL = (TOT + T - 1) / T;
    uint2 raw[NL];
};
template <int T, int NF>
__device__ __forceinline__ void stage_load(Staged<T, NF> &R, const Src &S, int n, int slot_n, int k0, int tid)
{
    using ST = Staged<T, NF>;
    // the (workgroup-uniform) frame addresses first, so that the slot lookup does not sit
    // between the frame loads and serialise them
    const uint8_t *f[4];
#pragma unroll
    for (int k = 0; k < 4; ++k) f[k] = frame_ptr(S, n, slot_n, k0 + (k < NF ? k : 0));
#pragma unroll
    for (int i = 0; i < ST::NL; ++i) {
        const int t = tid + i * T;
        if (t < ST::TOT) {
            const int k = t / ST::CH;
            const uint8_t *fp = k == 0 ? f[0] : k == 1 ? f[1] : k == 2 ? f[2] : f[3];
            R.raw[i] = *reinterpret_cast<const uint2 *>(fp + (t % ST::CH) * 8);
        }
    }
}
// 8 pixels -> 8 bf16 -> one 16-byte LDS store; consecutive lanes write consecutive 16 bytes
template <int T, int NF>
__device__ __forceinline__ void stage_store(bf16_t *xin, const Staged<T, NF> &R, int tid)
{
    using ST = Staged<T, NF>;
#pragma unroll
    for (int i = 0; i < ST::NL; ++i) {
        const int t = tid + i * T;
        if (t < ST::TOT) {
            const uint2 r = R.raw[i];
            uint4 o;
            o.x = pack2_u8(r.x & 0xFFu, (r.x >> 8) & 0xFFu);
            o.y = pack2_u8((r.x >> 16) & 0xFFu, r.x >> 24);
            o.z = pack2_u8(r.y & 0xFFu, (r.y >> 8) & 0xFFu);
            o.w = pack2_u8((r.y >> 16) & 0xFFu, r.y >> 24);
            *reinterpret_cast<uint4 *>(xin + t * 8) = o;  // frames are contiguous in xin: (t/CH)*FR + (t%CH)*8 == t*8
        }
    }
}

struct FwdSeg {
    Src src;
    const bf16_t *w;    // [32][256] bf16
    const float *bias;  // [32]
    bf16_t *y;          // [n][400][32]
    int n;              // samples
    int first;          // index of the segment's first sample in the launch-wide sample list
};
struct FwdArgs {
    FwdSeg seg[3];
    int nseg;
    int total;          // samples of all segments
};

// One output block of 32 pixels x 32 channels: bias, 1/255, ReLU, bf16, 32 contiguous bytes per lane.
// acc[4g + j] = Y[pixel li of the block][channel 16h + 4g + j]
__device__ __forceinline__ void conv1_store(const v16f &acc, const v4f (&bias)[4], bf16_t *y, int m, int h)
{
    constexpr float sc = 1.0f / 255.0f;
    uint2 o[4];
#pragma unroll
    for (int g4 = 0; g4 < 4; ++g4) {
        const v4f bv = bias[g4];
        o[g4] = pack4(fmaxf(acc[4 * g4] * sc + bv.x, 0.f), fmaxf(acc[4 * g4 + 1] * sc + bv.y, 0.f),
                      fmaxf(acc[4 * g4 + 2] * sc + bv.z, 0.f), fmaxf(acc[4 * g4 + 3] * sc + bv.w, 0.f));
    }
    uint4 *d = reinterpret_cast<uint4 *>(y + m * 32 + 16 * h);
    d[0] = uint4{o[0].x, o[0].y, o[1].x, o[1].y};
    d[1] = uint4{o[2].x, o[2].y, o[3].x, o[3].y};
}

// Weight fragments for the 16 reduction steps.  MFMA row i carries output channel
// ch(i) = 16*((i>>2)&1) + 4*(i>>3) + (i&3), so that the 16 results of a lane (rows 8g + 4h + j)
// are the 16 consecutive channels 16h + 4g + j of its pixel.
__device__ __forceinline__ void conv1_weights(v8bf (&wb)[16], const bf16_t *w, int li, int h)
{
    const int ch = 16 * ((li >> 2) & 1) + 4 * (li >> 3) + (li & 3);
#pragma unroll
    for (int t = 0; t < 16; ++t) wb[t] = __builtin_bit_cast(v8bf, ld8(w + ch * 256 + 16 * t + 8 * h));
}

// The MFMA loop of one sample for one wave: row blocks `wave` and (TWO) `wave + 8` of the 13
// blocks of 32 output pixels, 16 reduction steps each.  Straight-line code, no lane-dependent
// control flow, and the im2col fragments are fetched from LDS one group of four steps ahead
// of the MFMAs that consume them, so the LDS latency is hidden behind the matrix unit.
template <bool TWO>
__device__ __forceinline__ void conv1_blocks(const bf16_t *xin, const v8bf (&wa)[16], const v4f (&bias)[4],
                                             bf16_t *y, int wave, int li, int h)
{
    const int m0 = wave * 32 + li;
    int m1 = (wave + 8) * 32 + li;
    if (m1 > 399) m1 = 399;  // rows past the end read a valid pixel and are not stored
    const bf16_t *px0 = xin + (4 * (m0 / 20)) * 84 + 4 * (m0 % 20) + h * 84;
    const bf16_t *px1 = xin + (4 * (m1 / 20)) * 84 + 4 * (m1 % 20) + h * 84;
    auto frag = [&](const bf16_t *px, int t) {
        // k = 16t + 8h: channel t/4, kernel row (2t + h) % 8; 16 bytes at an 8-byte-aligned address
        const uint2 *q = reinterpret_cast<const uint2 *>(px + (t >> 2) * FR + ((2 * t) & 7) * 84);
        return __builtin_bit_cast(v8bf, uint4{q[0].x, q[0].y, q[1].x, q[1].y});
    };
    v16f acc0 = {0}, acc1 = {0};
    v8bf f0[2][4], f1[2][4];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        f0[0][j] = frag(px0, j);
        if constexpr (TWO) f1[0][j] = frag(px1, j);
    }
#pragma unroll
    for (int grp = 0; grp < 4; ++grp) {
        const int cur = grp & 1, nxt = cur ^ 1;
        if (grp < 3) {
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                f0[nxt][j] = frag(px0, 4 * (grp + 1) + j);
                if constexpr (TWO) f1[nxt][j] = frag(px1, 4 * (grp + 1) + j);
            }
        }
        // the scheduler would otherwise sink every read to just above its MFMA, which leaves
        // one LDS access in flight per wave and the matrix unit waiting on LDS latency
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            acc0 = mfma(wa[4 * grp + j], f0[cur][j], acc0);  // transposed tile
            if constexpr (TWO) acc1 = mfma(wa[4 * grp + j], f1[cur][j], acc1);
        }
        __builtin_amdgcn_sched_barrier(0);
    }
    const int mm = (wave + 8) * 32 + li;
    conv1_store(acc0, bias, y, m0, h);
    if (TWO && mm < 400) conv1_store(acc1, bias, y, mm, h);
}

// The samples [g0, g1) of one segment.  Weights and bias stay in registers; the frames of the
// next sample are loaded while the current one is computed, and the ring slot of the sample
// after that is already on its way.
__device__ __forceinline__ void conv1_fwd_range(const FwdSeg &S, int g0, int g1, bf16_t *xin, int tid)
{
    const int lane = tid & 63, li = lane & 31, h = lane >> 5;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);  // scalar: the block choice below is a uniform branch
    Staged<512, 4> R;
    stage_load<512, 4>(R, S.src, g0, sample_slot(S.src, g0), 0, tid);
    int slot_next = g0 + 1 < g1 ? sample_slot(S.src, g0 + 1) : 0;
    v8bf wa[16];
    conv1_weights(wa, S.w, li, h);
    v4f bias[4];  // this lane's 16 channels: 16h + 4g + j
#pragma unroll
    for (int g4 = 0; g4 < 4; ++g4) bias[g4] = *reinterpret_cast<const v4f *>(S.bias + 16 * h + 4 * g4);
    // Everything requested so far has arrived before the loop starts.  Without this the first
    // MFMA of every sample waits for "all outstanding vector loads" on account of the weight
    // registers, and that includes the next sample's frames requested a moment earlier.
    __builtin_amdgcn_s_waitcnt(0x0F70);  // vmcnt(0)
    for (int g = g0; g < g1; ++g) {
        sync_lds();  // the previous sample is no longer read
        stage_store<512, 4>(xin, R, tid);
        sync_lds();
        if (g + 1 < g1) {
            stage_load<512, 4>(R, S.src, g + 1, slot_next, 0, tid);
            if (g + 2 < g1) slot_next = sample_slot(S.src, g + 2);
        }
        // 13 blocks of 32 output pixels (the last one half empty): waves 0-4 take two, 5-7 one
        bf16_t *y = S.y + (long)g * (400 * 32);
        if (wave + 8 < 13) conv1_blocks<true>(xin, wa, bias, y, wave, li, h);
        else conv1_blocks<false>(xin, wa, bias, y, wave, li, h);
    }
}

// Persistent workgroups: workgroup b owns samples [b*total/G, (b+1)*total/G) of the launch-wide
// list (segment after segment).
__global__ __launch_bounds__(512) void k_conv1_fwd(FwdArgs A)
{
    __shared__ __attribute__((aligned(16))) bf16_t xin[XIN];
    const int g0 = (int)((long)blockIdx.x * A.total / gridDim.x);
    const int g1 = (int)((long)(blockIdx.x + 1) * A.total / gridDim.x);
    for (int s = 0; s < A.nseg; ++s) {
        FwdSeg S = A.seg[0];
        if (s == 1) S = A.seg[1];
        if (s == 2) S = A.seg[2];
        const int lo = max(g0, S.first) - S.first, hi = min(g1, S.first + S.n) - S.first;
        if (lo < hi) conv1_fwd_range(S, lo, hi, xin, threadIdx.x);
    }
}

struct WgradArgs {
    Src src;
    const bf16_t *dy;  // [B][400][32]
    float *part;       // [nsplit][32*256 + 32]
    int B;
    int nsplit;        // = gridDim.x; workgroup z sums samples z, z+nsplit, ...
};

constexpr int LDY1 = 40;  // row stride (elements) of the staged dY tile

// grid (nsplit, 2): a workgroup takes one channel pair y (frames 2y, 2y+1 = im2col columns
// 128y .. 128y+127), so a workgroup stages half a state and two workgroups fit one CU.
__global__ __launch_bounds__(256) void k_conv1_wgrad(WgradArgs A)
{
    __shared__ __attribute__((aligned(16))) bf16_t xin[2 * FR];
    __shared__ __attribute__((aligned(16))) bf16_t dys[400 * LDY1];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;  // wave = block of 32 im2col columns
    const int li = lane & 31, h = lane >> 5, s16 = lane & 15, half = (lane >> 4) & 1;
    // the two channel pairs of one sample split run next to each other: same dY, same ring slots
    const int tile = net::tile_of_workgroup();
    const int cp = tile & 1, split = tile >> 1;
    typedef __attribute__((address_space(3))) v4s *lds_v4s;

    // this lane's share of the transpose loads: reduction row offset s/4 (+4 for the second
    // load), columns 16*half + 4*(s%4) .. +3 of the wave's 32-column block
    const int rsub = 8 * h + (s16 >> 2);
    const int kc = 32 * wave + 16 * half + 4 * (s16 & 3);       // column within the pair: (c, p, q0)
    const int xoff = (kc >> 6) * FR + ((kc >> 3) & 7) * 84 + (kc & 7);
    const bf16_t *yp = dys + rsub * LDY1 + 16 * half + 4 * (s16 & 3);

    v16f acc = {0}, accb = {0};
    v8bf ones;
#pragma unroll
    for (int e = 0; e < 8; ++e) ones[e] = (__bf16)1.0f;
    const bool do_bias = cp == 0 && wave == 0;

    Staged<256, 2> R;
    uint4 ry[7];
    auto load_sample = [&](int n, int slot_n) {
        stage_load<256, 2>(R, A.src, n, slot_n, 2 * cp, tid);
        const bf16_t *dyn = A.dy + (long)n * (400 * 32);
#pragma unroll
        for (int i = 0; i < 7; ++i) {
            const int t = tid + i * 256;
            if (t < 1600) ry[i] = ld8(dyn + (t >> 2) * 32 + (t & 3) * 8);
        }
    };
    // the ring slot of a sample is fetched one sample ahead of the frame loads that need it
    if (split < A.B) load_sample(split, sample_slot(A.src, split));
    int slot_next = split + A.nsplit < A.B ? sample_slot(A.src, split + A.nsplit) : 0;
    for (int n = split; n < A.B; n += A.nsplit) {
        __syncthreads();  // the previous sample's tiles are no longer read
        stage_store<256, 2>(xin, R, tid);
#pragma unroll
        for (int i = 0; i < 7; ++i) {
            const int t = tid + i * 256;
            if (t < 1600) *reinterpret_cast<uint4 *>(dys + (t >> 2) * LDY1 + (t & 3) * 8) = ry[i];
        }
        __syncthreads();
        if (n + A.nsplit < A.B) {
            load_sample(n + A.nsplit, slot_next);  // in flight during the MFMA loop
            if (n + 2 * A.nsplit < A.B) slot_next = sample_slot(A.src, n + 2 * A.nsplit);
        }
#pragma unroll 5
        for (int t = 0; t < 25; ++t) {  // 16 output pixels per step
            v8bf fa = frag_tr(yp + 16 * t * LDY1, LDY1);
            const int m0 = 16 * t + rsub, m1 = m0 + 4;
            const bf16_t *x0 = xin + xoff + (4 * (m0 / 20)) * 84 + 4 * (m0 % 20);
            const bf16_t *x1 = xin + xoff + (4 * (m1 / 20)) * 84 + 4 * (m1 % 20);
            v4s lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_v4s)x0);
            v4s hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_v4s)x1);
            typedef short v8s __attribute__((ext_vector_type(8)));
            v8s xb = {lo.x, lo.y, lo.z, lo.w, hi.x, hi.y, hi.z, hi.w};
            acc = mfma(fa, __builtin_bit_cast(v8bf, xb), acc);
            if (do_bias) accb = mfma(fa, ones, accb);
        }
    }

    float *part = A.part + (long)split * (32 * 256 + 32);
#pragma unroll
    for (int r = 0; r < 16; ++r) {
        const int o = 8 * (r / 4) + 4 * h + (r % 4);
        part[o * 256 + 128 * cp + 32 * wave + li] = acc[r] * (1.0f / 255.0f);
        if (do_bias && li == 0) part[32 * 256 + o] = accb[r];
    }
}
}  // namespace c1
}  // namespace gbf
