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
    uint32_t u = __float_as_uint(f);
    u += 0x7FFFu + ((u >> 16) & 1u);
    return (bf16_t)(u >> 16);
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
    const int bx = blockIdx.x;
    FwdSeg S = A.seg[0];
    if (A.nseg > 1 && bx >= A.seg[1].tile_begin) S = A.seg[1];
    if (A.nseg > 2 && bx >= A.seg[2].tile_begin) S = A.seg[2];
    const int m0 = (bx - S.tile_begin) * BM, n0 = blockIdx.y * BN;
    const int kbeg = blockIdx.z * A.klen, kend = kbeg + A.klen;
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
                for (int b = 0; b < WN; ++b) acc[a][b] = mfma(fa[a], fb[b], acc[a][b]);
        }
        __syncthreads();
        if (more) {
            sstore();
            __syncthreads();
        }
    }

#pragma unroll
    for (int b = 0; b < WN; ++b) {
        const int col = n0 + (wn * WN + b) * 32 + li;
        const float bias = (!RAW && S.bias) ? S.bias[col] : 0.f;
#pragma unroll
        for (int a = 0; a < WM; ++a) {
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                int m = m0 + (wm * WM + a) * 32 + 8 * (r / 4) + 4 * h + (r % 4);
                if (m < S.M) {
                    float v = acc[a][b][r] * A.scale;
                    if (RAW) {
                        (static_cast<float *>(S.y) + (long)blockIdx.z * A.split_stride)[(long)m * G::N + col] = v;
                    } else {
                        v = fmaxf(v + bias, 0.f);
                        static_cast<bf16_t *>(S.y)[(long)m * G::N + col] = f2bf(v);
                    }
                }
            }
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
    const int m0 = blockIdx.x * BM, n0 = blockIdx.y * BN;
    const int ca = blockIdx.z / D::S, cb = blockIdx.z % D::S;
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
                for (int b = 0; b < WN; ++b) acc[a][b] = mfma(fa[a], fb[b], acc[a][b]);
        }
        __syncthreads();
        if (more) {
            sstore();
            __syncthreads();
        }
    }

#pragma unroll
    for (int b = 0; b < WN; ++b) {
        const int col = n0 + (wn * WN + b) * 32 + li;
#pragma unroll
        for (int a = 0; a < WM; ++a) {
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                int m = m0 + (wm * WM + a) * 32 + 8 * (r / 4) + 4 * h + (r % 4);
                if (m < Mc) {
                    int n = m / D::PP, rr = m % D::PP;
                    int hh = D::S * (rr / D::WP) + ca, ww = D::S * (rr % D::WP) + cb;
                    long off = ((long)(n * D::H + hh) * D::W + ww) * D::CI + col;
                    A.dx[off] = (int16_t)A.xact[off] > 0 ? f2bf(acc[a][b][r]) : (bf16_t)0;
                }
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
    const int kc0 = blockIdx.x * BNK, o0 = blockIdx.y * BMO;
    const int mbeg = blockIdx.z * A.rps;
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
    const bool do_bias = blockIdx.x == 0 && wk == 0;
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

    float *part = A.part + (long)blockIdx.z * A.part_stride;
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

}  // namespace gbf
