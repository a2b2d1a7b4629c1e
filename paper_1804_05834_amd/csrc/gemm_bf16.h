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
#include "sumtree.h"

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

// v_mfma_f32_16x16x32_bf16 (lane = 16*g + i): a-operand A[i][8g..8g+7], b-operand B[8g..8g+7][i],
// result acc[j] = D[4g + j][i]
__device__ __forceinline__ v4f mfma16(v8bf a, v8bf b, v4f c)
{
    return __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b, c, 0, 0, 0);
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
// 8 pixels in two words -> 8 bf16 (exact): the upper halves of the floats, merged pairwise by a byte permute
__device__ __forceinline__ uint4 cvt8_u8(uint32_t a, uint32_t b)
{
    auto pk = [](float lo, float hi) { return __builtin_amdgcn_perm(__float_as_uint(hi), __float_as_uint(lo), 0x07060302u); };
    uint4 o;
    o.x = pk((float)(a & 0xFFu), (float)((a >> 8) & 0xFFu));
    o.y = pk((float)((a >> 16) & 0xFFu), (float)(a >> 24));
    o.z = pk((float)(b & 0xFFu), (float)((b >> 8) & 0xFFu));
    o.w = pk((float)((b >> 16) & 0xFFu), (float)(b >> 24));
    return o;
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
    // written with the builtins so that the compiler's own wait counting knows that every LDS operation
    // of the wave has completed here (behind an inline-asm barrier it waits for all of them again)
    __builtin_amdgcn_s_waitcnt(0xC07F);   // lgkmcnt(0)
    __builtin_amdgcn_s_barrier();
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

// Dispatch-order number u of `total` workgroups -> tile number, die-aware as net::tile_of_workgroup
// (a launch that holds two problems numbers each of them by itself).
__device__ __forceinline__ int tile_of(int u, int total)
{
    const int die = u & 7, slot = u >> 3, q = total >> 3, r = total & 7;
    return die * q + (die < r ? die : r) + slot;
}

// ---------------------------------------------------------------------------
// fc1 forward for many rows (Section 3 fourth layer: 3136 -> 512): raw fp32 partial sums of a few
// reduction splits, which the head kernel adds up.
//
// 128 x 128 output tile per workgroup of four waves, 64 x 64 per wave (2 x 2 MFMA blocks, so every
// LDS fragment feeds two matrix instructions), reduction stages of 64 elements in LDS tiles that are
// double-buffered: ONE barrier per stage and sixteen 32x32x16 MFMAs per wave between two barriers.
// While stage s is multiplied, stage s+1 goes from registers to the other LDS buffer and stage s+3
// is requested from memory.  The 49 stages of the reduction are dealt out evenly to the splits.
// Measured per stage and workgroup in the steady state: 16 MFMAs per wave take 250 ns, with the LDS
// reads beside them 285 ns, with the 32 KB of LDS writes as well 430 ns: the loop is bound by LDS
// bandwidth (96 KB per stage and compute unit), not by the matrix pipe.
// Tile order: the four column tiles of one row tile and split next to each other (they share the
// activations), row tiles of one split after each other (they share the weights).
// ---------------------------------------------------------------------------
namespace f1 {
constexpr int BM = 128, BN = 128;
constexpr int TILE = BM * LDK;                   // elements of one operand tile in LDS
constexpr int LDS_BYTES = 2 * 2 * TILE * 2;      // two operands, two buffers: 73,728 bytes
constexpr int STAGES = GFc1::K / BK;             // 49

struct Args {
    FwdSeg seg[3];      // tile_begin counts row tiles of BM rows; y = fp32 [M][512] of split 0
    int nseg;
    int nsplit;
    int tiles_m;        // row tiles of all segments
    long split_stride;  // elements between the partial sums of consecutive splits
};

// Barrier that orders LDS traffic only, written with the builtins so that the compiler's own wait
// counting knows that every LDS operation of the wave has completed at this point.
__device__ __forceinline__ void lds_barrier()
{
    __builtin_amdgcn_s_waitcnt(0xC07F);   // lgkmcnt(0)
    __builtin_amdgcn_s_barrier();
}

__global__ __launch_bounds__(256, 2) void k_fc1_fwd(Args A)
{
    extern __shared__ __attribute__((aligned(16))) bf16_t lds[];
    bf16_t *As = lds, *Bs = lds + 2 * TILE;      // [buffer][row][LDK]
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int t = tile_of(blockIdx.x, gridDim.x);
    const int by = t & 3, bx = (t >> 2) % A.tiles_m, bz = (t >> 2) / A.tiles_m;
    FwdSeg S = A.seg[0];
    if (A.nseg > 1 && bx >= A.seg[1].tile_begin) S = A.seg[1];
    if (A.nseg > 2 && bx >= A.seg[2].tile_begin) S = A.seg[2];
    const int m0 = (bx - S.tile_begin) * BM, n0 = by * BN;
    const int s0 = STAGES * bz / A.nsplit, n = STAGES * (bz + 1) / A.nsplit - s0;
    const bf16_t *x = static_cast<const bf16_t *>(S.x);

    // staging: 16-byte piece c = tid + 256 i of a 128 x 64 tile is row c / 8, elements 8 (c % 8) .. +7
    const int lr = tid >> 3, kq = (tid & 7) * 8;
    const bf16_t *pa[4], *pb[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        int m = m0 + lr + 32 * i;
        if (m > S.M - 1) m = S.M - 1;             // rows past the end repeat the last row; they are never stored
        pa[i] = x + (long)m * S.xs + kq;
        pb[i] = S.w + (long)(n0 + lr + 32 * i) * GFc1::K + kq;
    }
    typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));   // a native vector: stays in registers
    struct Regs { u32x4 a[4], b[4]; };
    Regs R0, R1;                                  // two stages on their way from memory
    auto gload = [&](Regs &R, int st) {
        const int k0 = (s0 + st) * BK;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            R.a[i] = *reinterpret_cast<const u32x4 *>(pa[i] + k0);
            R.b[i] = *reinterpret_cast<const u32x4 *>(pb[i] + k0);
        }
    };
    auto sstore = [&](const Regs &R, int buf) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            *reinterpret_cast<u32x4 *>(&As[buf * TILE + (lr + 32 * i) * LDK + kq]) = R.a[i];
            *reinterpret_cast<u32x4 *>(&Bs[buf * TILE + (lr + 32 * i) * LDK + kq]) = R.b[i];
        }
    };
    const int wm = wave & 1, wn = wave >> 1;
    const int li = lane & 31, h = lane >> 5;
    const int apo = (wm * 64 + li) * LDK + 8 * h, bpo = (wn * 64 + li) * LDK + 8 * h;
    v16f acc[2][2];
#pragma unroll
    for (int a = 0; a < 2; ++a)
#pragma unroll
        for (int b = 0; b < 2; ++b) acc[a][b] = v16f{0};
    struct Frag { v8bf a[2], b[2]; };             // the operands of one 16-deep step of the wave's 64 x 64
    auto rd = [&](int buf, int kk) {
        Frag F;
        const bf16_t *ap = As + buf * TILE + apo + kk, *bp = Bs + buf * TILE + bpo + kk;
        F.a[0] = frag_k(ap); F.a[1] = frag_k(ap + 32 * LDK);
        F.b[0] = frag_k(bp); F.b[1] = frag_k(bp + 32 * LDK);
        return F;
    };
    auto mm = [&](const Frag &F) {
#pragma unroll
        for (int a = 0; a < 2; ++a)
#pragma unroll
            for (int b = 0; b < 2; ++b) acc[a][b] = mfma(F.b[b], F.a[a], acc[a][b]);  // transposed tile
    };

    gload(R0, 0);
    if (n > 1) gload(R1, 1);
    sstore(R0, 0);
    if (n > 2) gload(R0, 2);
    lds_barrier();
    Frag cur = rd(0, 0);
    // Stage i out of buffer buf.  NX holds stage i + 1 (requested two stages ago) and is refilled with
    // stage i + 3.  The operands of a step are requested before the matrix instructions of the step
    // before it; the barrier sits in front of the stage's last step, whose matrix instructions then
    // cover the barrier and the first LDS reads of the next stage.  The other buffer was last read
    // before the previous barrier, so it may be written at any point of this stage.
    auto stage = [&](int i, int buf, Regs &NX) {
        Frag f1 = rd(buf, 16);
        __builtin_amdgcn_sched_barrier(0);
        mm(cur);
        __builtin_amdgcn_sched_barrier(0);
        Frag f2 = rd(buf, 32);
        if (i + 1 < n) sstore(NX, buf ^ 1);
        __builtin_amdgcn_sched_barrier(0);
        mm(f1);
        __builtin_amdgcn_sched_barrier(0);
        Frag f3 = rd(buf, 48);
        if (i + 3 < n) gload(NX, i + 3);
        __builtin_amdgcn_sched_barrier(0);
        mm(f2);
        __builtin_amdgcn_sched_barrier(0);
        lds_barrier();
        if (i + 1 < n) cur = rd(buf ^ 1, 0);
        __builtin_amdgcn_sched_barrier(0);
        mm(f3);
        __builtin_amdgcn_sched_barrier(0);
    };
    for (int i = 0; i < n; i += 2) {              // unrolled by two: the register sets alternate statically
        stage(i, 0, R1);
        if (i + 1 < n) stage(i + 1, 1, R0);
    }

    // acc[a][b][4g + j] = Y[row block a, lane li][column block b, 8g + 4h + j].  The tile leaves through LDS
    // (the operand buffers are no longer read: the loop ends on a barrier), so that it is written as whole
    // 512-byte rows, two per wave and instruction, instead of 32-byte pieces of 32 different rows.
    constexpr int LDO = BN + 4;                   // fp32 row stride of the staged output tile
    static_assert(BM * LDO * 4 <= LDS_BYTES, "the output tile is staged in the operand buffers");
    float *ot = reinterpret_cast<float *>(lds);
#pragma unroll
    for (int a = 0; a < 2; ++a)
#pragma unroll
        for (int b = 0; b < 2; ++b)
#pragma unroll
            for (int g = 0; g < 4; ++g)
                *reinterpret_cast<v4f *>(&ot[((wm * 2 + a) * 32 + li) * LDO + (wn * 2 + b) * 32 + 8 * g + 4 * h]) =
                    v4f{acc[a][b][4 * g], acc[a][b][4 * g + 1], acc[a][b][4 * g + 2], acc[a][b][4 * g + 3]};
    lds_barrier();
    float *y = static_cast<float *>(S.y) + (long)bz * A.split_stride;
#pragma unroll
    for (int i = 0; i < 16; ++i) {
        const int r = (tid >> 5) + 8 * i, cq = (tid & 31) * 4, m = m0 + r;
        if (m < S.M) *reinterpret_cast<v4f *>(y + (long)m * GFc1::N + n0 + cq) = *reinterpret_cast<const v4f *>(&ot[r * LDO + cq]);
    }
}
}  // namespace f1

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

// DB: the LDS tiles are double-buffered, which leaves one barrier per reduction stage instead of two
// (for the layers whose stages are so short that the barriers dominate them), and a wave with a
// single output block alternates between two accumulators so that consecutive MFMAs do not wait
// for each other's result.
// LDS elements of an input-gradient tile
template <int BM, int BN, bool DB> constexpr int dgrad_lds() { return (DB ? 2 : 1) * (BM * LDK + BK * (BN + 8)); }

// Tile number t of a (gx, gy, gz) grid of tiles; tile order: the parity classes of one row tile
// together, then the row tiles of one column tile.
template <class D, int BM, int BN, int WM, int WN, bool DB>
__device__ __forceinline__ void dgrad_tile(const DgradArgs &A, int t, int gx, int gz, bf16_t *lds)
{
    constexpr int WAVES_M = BM / (32 * WM), WAVES_N = BN / (32 * WN), T = WAVES_M * WAVES_N * 64;
    constexpr int NA = BM * 8 / T;
    constexpr int LDB = BN + 8;          // row stride of the [k][c] weight tile
    constexpr int BCH = BN / 8;          // 16-byte chunks per weight-tile row
    constexpr int BROWS = T / BCH;       // rows filled per pass
    constexpr int NBL = (BK + BROWS - 1) / BROWS;
    static_assert(NA * T == BM * 8 && D::CO % BK == 0, "tile/threads mismatch");
    constexpr int NBUF = DB ? 2 : 1;
    constexpr bool ACC2 = DB && WM * WN == 1;
    bf16_t(*As2)[BM * LDK] = reinterpret_cast<bf16_t(*)[BM * LDK]>(lds);
    bf16_t(*Bs2)[BK * LDB] = reinterpret_cast<bf16_t(*)[BK * LDB]>(lds + NBUF * BM * LDK);

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int bz = t % gz, bx = (t / gz) % gx, by = t / (gz * gx);
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
    auto sstore = [&](int buf) {
        bf16_t *As = As2[buf], *Bs = Bs2[buf];
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
    const int apo = (wm * 32 * WM + li) * LDK + 8 * h;
    // transpose-read base: row 8h + s/4, column (wave block) + 16*half + 4*(s%4)
    const int bpo = (8 * h + (s16 >> 2)) * LDB + wn * 32 * WN + 16 * half + 4 * (s16 & 3);
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
        // (unconditional, from a clamped address: a value chosen between a loaded one and a constant would
        // be waited for right here, in front of the first stage's loads)
        const long ob = obase[a] >= 0 ? obase[a] : 0;
#pragma unroll
        for (int b = 0; b < WN; ++b)
#pragma unroll
            for (int g = 0; g < 4; ++g) xa[a][b][g] = *reinterpret_cast<const uint2 *>(A.xact + ob + b * 32 + 8 * g);
    }

    v16f acc2 = {0};   // second accumulator (ACC2 only)
    auto compute = [&](int buf) {
        const bf16_t *ap = As2[buf] + apo, *bp = Bs2[buf] + bpo;
        // the fragments of a 16-deep step are requested before the matrix instructions of the step before it
        auto frags = [&](int kk, v8bf (&fa)[WM], v8bf (&fb)[WN]) {
#pragma unroll
            for (int a = 0; a < WM; ++a) fa[a] = frag_k(ap + a * 32 * LDK + kk);
#pragma unroll
            for (int b = 0; b < WN; ++b) fb[b] = frag_tr(bp + kk * LDB + b * 32, LDB);
        };
        v8bf fa[WM], fb[WN], fan[WM], fbn[WN];
        frags(0, fa, fb);
#pragma unroll
        for (int kk = 0; kk < BK; kk += 16) {
            if (kk + 16 < BK) frags(kk + 16, fan, fbn);
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int a = 0; a < WM; ++a)
#pragma unroll
                for (int b = 0; b < WN; ++b) {  // transposed tile
                    if (ACC2 && (kk & 16)) acc2 = mfma(fb[b], fa[a], acc2);
                    else acc[a][b] = mfma(fb[b], fa[a], acc[a][b]);
                }
            __builtin_amdgcn_sched_barrier(0);
            if (kk + 16 < BK) {
#pragma unroll
                for (int a = 0; a < WM; ++a) fa[a] = fan[a];
#pragma unroll
                for (int b = 0; b < WN; ++b) fb[b] = fbn[b];
            }
        }
    };
    gload(0);
    if constexpr (DB) {
        int s = 0;
        for (int k0 = 0; k0 < D::K; k0 += BK, s ^= 1) {
            sstore(s);
            if (k0 + BK < D::K) gload(k0 + BK);
            sync_lds();   // buffer s is complete; every wave is past the previous stage, which read buffer s^1
            compute(s);
        }
        if (ACC2) acc[0][0] += acc2;
    } else {
        sstore(0);
        __syncthreads();
        for (int k0 = 0; k0 < D::K; k0 += BK) {
            const bool more = k0 + BK < D::K;
            if (more) gload(k0 + BK);
            compute(0);
            __syncthreads();
            if (more) {
                sstore(0);
                __syncthreads();
            }
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

// LDS elements of a weight-gradient tile
template <int BMO, int BNK, bool DB> constexpr int wgrad_lds() { return (DB ? 2 : 1) * BK * (BMO + 8 + BNK + 8); }

// Tile number t of a (gx, gy, gz) grid of tiles; tile order: with row splits (conv layers) all
// tiles of one split together; without (fc1) all output tiles of one input-column tile together.
// DB: double-buffered LDS tiles (one barrier per reduction stage) and, for a wave with a single
// output block, two alternating accumulators, as in the input gradient.
template <class G, int BMO, int BNK, int WM, int WN, bool DB>
__device__ __forceinline__ void wgrad_tile(const WgradArgs &A, int t, int gx, int gy, int gz, bf16_t *lds)
{
    constexpr int WAVES_M = BMO / (32 * WM), WAVES_N = BNK / (32 * WN), T = WAVES_M * WAVES_N * 64;
    constexpr int LDY = BMO + 8, LDX = BNK + 8;
    constexpr int YCH = BMO / 8, XCH = BNK / 8;          // 16-byte chunks per tile row
    constexpr int YR = T / YCH, XR = T / XCH;            // rows filled per pass
    constexpr int NY = (BK + YR - 1) / YR, NX = (BK + XR - 1) / XR;
    using in_t = typename in_type<G>::t;
    constexpr int NBUF = DB ? 2 : 1;
    constexpr bool ACC2 = DB && WM * WN <= 2;   // two alternating accumulators per output block
    bf16_t(*Ys2)[BK * LDY] = reinterpret_cast<bf16_t(*)[BK * LDY]>(lds);
    bf16_t(*Xs2)[BK * LDX] = reinterpret_cast<bf16_t(*)[BK * LDX]>(lds + NBUF * BK * LDY);

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    int bx, by, bz;
    if (gz > 1) {
        bx = t % gx; by = (t / gx) % gy; bz = t / (gx * gy);
    } else {
        by = t % gy; bx = t / gy; bz = 0;
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
    auto sstore = [&](int buf) {
        bf16_t *Ys = Ys2[buf], *Xs = Xs2[buf];
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
    const int ypo = trow * LDY + wo * 32 * WM + tcol, xpo = trow * LDX + wk * 32 * WN + tcol;
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

    v16f acc2[WM][WN];   // second accumulators (ACC2 only)
#pragma unroll
    for (int a = 0; a < WM; ++a)
#pragma unroll
        for (int b = 0; b < WN; ++b) acc2[a][b] = v16f{0};
    auto compute = [&](int buf) {
        const bf16_t *yp = Ys2[buf] + ypo, *xp = Xs2[buf] + xpo;
        // the fragments of a 16-deep step are requested before the matrix instructions of the step before it
        auto frags = [&](int kk, v8bf (&fa)[WM], v8bf (&fb)[WN]) {
#pragma unroll
            for (int a = 0; a < WM; ++a) fa[a] = frag_tr(yp + kk * LDY + a * 32, LDY);
#pragma unroll
            for (int b = 0; b < WN; ++b) fb[b] = frag_tr(xp + kk * LDX + b * 32, LDX);
        };
        v8bf fa[WM], fb[WN], fan[WM], fbn[WN];
        frags(0, fa, fb);
#pragma unroll
        for (int kk = 0; kk < BK; kk += 16) {
            if (kk + 16 < BK) frags(kk + 16, fan, fbn);
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int a = 0; a < WM; ++a) {
#pragma unroll
                for (int b = 0; b < WN; ++b) {
                    if (ACC2 && (kk & 16)) acc2[a][b] = mfma(fa[a], fb[b], acc2[a][b]);
                    else acc[a][b] = mfma(fa[a], fb[b], acc[a][b]);
                }
                if (do_bias) accb[a] = mfma(fa[a], ones, accb[a]);
            }
            __builtin_amdgcn_sched_barrier(0);
            if (kk + 16 < BK) {
#pragma unroll
                for (int a = 0; a < WM; ++a) fa[a] = fan[a];
#pragma unroll
                for (int b = 0; b < WN; ++b) fb[b] = fbn[b];
            }
        }
    };
    if constexpr (DB) {
        if (mbeg < mend) gload(mbeg);
        int sb = 0;
        for (int mb = mbeg; mb < mend; mb += BK, sb ^= 1) {
            sstore(sb);
            if (mb + BK < mend) gload(mb + BK);
            sync_lds();   // buffer sb is complete; every wave is past the previous stage, which read buffer sb^1
            compute(sb);
        }
        if (ACC2) {
#pragma unroll
            for (int a = 0; a < WM; ++a)
#pragma unroll
                for (int b = 0; b < WN; ++b) acc[a][b] += acc2[a][b];
        }
    } else {
        if (mbeg < mend) {
            gload(mbeg);
            sstore(0);
        }
        __syncthreads();
        for (int mb = mbeg; mb < mend; mb += BK) {
            const bool more = mb + BK < mend;
            if (more) gload(mb + BK);
            compute(0);
            __syncthreads();
            if (more) {
                sstore(0);
                __syncthreads();
            }
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

// The input gradient and the weight gradient of one layer go into ONE launch of 64x64 tiles (both
// read the layer's dY and depend on nothing else that is computed in the backward pass): nd
// input-gradient tiles, then nw weight-gradient tiles.
struct PairGrid {
    int nd, dgx, dgz;        // input gradient: tiles, grid x and z
    int nw, wgx, wgy, wgz;   // weight gradient: tiles, grid
};

// ===========================================================================
// conv1 (8x8 stride 4 over the uint8 frame stack), specialised.
//
// The generic kernels gather conv1's im2col rows from global memory in 4/8-byte
// pieces at 84-byte strides, which is address-bound.  Here the 84x84 frames are
// read with 16-byte loads -- from a materialised state, or straight from the
// replay ring through the sampled slot (the frame-stack gather fused into the
// loader) -- converted to bf16 and kept in LDS, and every operand of the 8x8/4
// convolution is an LDS read at a computed address:
//   forward : one WAVE stages the 20 input rows under 4 output rows of the four
//             frames in LDS of its own and reads them as two-row "quads";
//             all of W (32x256 bf16) sits in registers (see k_conv1_fwd);
//   wgrad   : one WORKGROUP stages two whole frames of a sample; 8 consecutive
//             pixels of one im2col column are fetched with the LDS transpose
//             load, whose lanes each supply their own address.
// ===========================================================================
namespace c1 {
constexpr int FR = 84 * 84;       // elements per frame

struct Src {                      // where the four frames of sample n come from
    const uint8_t *x;             // explicit states [n][4][84][84] (idx == nullptr) or the ring
    long xs;                      // bytes between samples (explicit)
    const int32_t *idx;           // sampled slots (ring mode)
    long cap;                     // ring capacity
    int shift;                    // 0: frames i-3..i (s), 1: frames i-2..i+1 (s')
    int sub;                      // length of the sub-ring a window wraps in: the capacity (one stream),
                                  // or the share of one environment stream when the ring holds many
};

// First slot of the sub-ring that slot i lies in.
__device__ __forceinline__ long sub_ring_base(const Src &S, long i)
{
    return (long)S.sub == S.cap ? 0 : (long)((uint32_t)i / (uint32_t)S.sub) * S.sub;
}

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
    const long base = sub_ring_base(S, i);
    long slot = i - base - 3 + k + S.shift;  // within [-3, sub+1]: one wrap at most (sub >= 5)
    if (slot < 0) slot += S.sub;
    if (slot >= S.sub) slot -= S.sub;
    return S.x + (base + slot) * FR;
}

// Staging of frames k0 .. k0+NF-1 of sample n as bf16 into xin[(k-k0)*FR ...], in two halves so
// that the global loads of the next sample can be in flight while the current one is computed:
// stage_load issues every 16-byte load of a thread, stage_store converts (16 pixels -> 16 bf16)
// and writes two 16-byte LDS stores per load.
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));   // a native vector: stays in registers
template <int T, int NF> struct Staged {
    static constexpr int CH = FR / 16, TOT = NF * CH, NL = (TOT + T - 1) / T;
    u32x4 raw[NL];
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
        int t = tid + i * T;
        if (t > ST::TOT - 1) t = ST::TOT - 1;   // the last pass repeats a piece rather than branching
        const int k = t / ST::CH;
        const uint8_t *fp = k == 0 ? f[0] : k == 1 ? f[1] : k == 2 ? f[2] : f[3];
        R.raw[i] = *reinterpret_cast<const u32x4 *>(fp + (t % ST::CH) * 16);
    }
}
// 16 pixels -> 16 bf16 -> two 16-byte LDS stores; consecutive lanes write consecutive 32 bytes
template <int T, int NF>
__device__ __forceinline__ void stage_store(bf16_t *xin, const Staged<T, NF> &R, int tid)
{
    using ST = Staged<T, NF>;
#pragma unroll
    for (int i = 0; i < ST::NL; ++i) {
        const int t = tid + i * T;
        if (t < ST::TOT) {
            const u32x4 r = R.raw[i];
            uint4 *d = reinterpret_cast<uint4 *>(xin + t * 16);  // frames are contiguous in xin: (t/CH)*FR + (t%CH)*16 == t*16
            d[0] = cvt8_u8(r.x, r.y);
            d[1] = cvt8_u8(r.z, r.w);
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
    int draw;           // replay mode: the kernel draws sample g of every segment itself (draw g of `samp`);
                        // segment 0 publishes the draws
    misc::SampleArgs samp;
};

// Forward pass, one WAVE per unit of work and no workgroup barrier anywhere.
//
// A unit is a strip of 4 output rows of one sample: 80 output pixels = 16 lanes x 5 consecutive
// pixels of one output row.  Its receptive field, input rows 16s .. 16s+19 of the four frames
// (13,440 bytes as bf16), sits in a part of LDS that belongs to this wave alone, so staging,
// matrix instructions and stores of different waves never wait for each other.
//
// v_mfma_f32_16x16x32_bf16, weights as the a-operand (row r = channel 8*(r/4) + 4*hh + r%4 for
// channel half hh), pixels as the b-operand (column n = lane % 16: output row n/4 of the strip,
// pixels 5*(n%4) .. +4 of that row).  Reduction step (c, xh) covers frame c, all 8 kernel rows,
// kernel columns 4xh .. 4xh+3: lane group kg = lane/16 holds kernel rows 2kg and 2kg+1, four
// columns each.  With that split the operand of pixel j at step (c, xh) is the "quad"
//   q[c][j + xh] = { input row 2kg, columns 4(j+xh)..+3 ; input row 2kg+1, same columns },
// i.e. six quads per frame serve all five pixels and both column halves, each fetched by ONE
// two-address LDS read, and every input element is read from LDS 2.4 times instead of 4.
// The result of lane (n, g = lane/16) is channels 8g .. 8g+7 of its pixels: 16 bytes per store.
constexpr int SROWS = 20;               // input rows per strip
constexpr int STRIP = 4 * SROWS * 84;   // elements per strip (four frames)
constexpr int UNITS = 5;                // strips per sample
constexpr int CHUNKS = STRIP / 16;      // 16-byte pieces of a strip's pixels: 420
constexpr int MAX_DRAWS = 8;            // samples one wave may draw for itself

struct StripRaw { u32x4 raw[7]; };      // this lane's pieces lane, lane + 64, ... of a strip
struct StripOff { uint32_t off[7]; };   // their byte offsets within four frames that are contiguous in memory

// The pixels of strip `strip` of sample g.  Four frames of a ring sample are contiguous unless
// they straddle the end of the ring (or its start, for the first slots); explicit states always are.
__device__ __forceinline__ void strip_load(StripRaw &R, const Src &S, int g, int slot_g, int strip, int lane,
                                           const StripOff &O)
{
    const uint8_t *base;
    bool contig = true;
    long b = 0, rb = 0;                           // first frame's slot within its sub-ring; the sub-ring's first slot
    if (!S.idx) {
        base = S.x + (long)g * S.xs;
    } else {
        long i = __builtin_amdgcn_readfirstlane(slot_g);
        i = i < 0 ? 0 : (i >= S.cap ? S.cap - 1 : i);
        rb = sub_ring_base(S, i);
        b = i - rb - 3 + S.shift;                 // within [-3, sub - 2]
        contig = b >= 0 && b + 3 < S.sub;
        base = S.x + (rb + b) * FR;
    }
    if (contig) {   // one scalar base, per-lane offsets that never change
        base += strip * (16 * 84);
#pragma unroll
        for (int i = 0; i < 7; ++i)
            if (i < 6 || lane < CHUNKS - 384) R.raw[i] = *reinterpret_cast<const u32x4 *>(base + O.off[i]);
    } else {
#pragma unroll
        for (int i = 0; i < 7; ++i) {
            const int t = lane + 64 * i;
            if (t < CHUNKS) {
                long slot = b + t / (CHUNKS / 4);
                if (slot < 0) slot += S.sub;
                if (slot >= S.sub) slot -= S.sub;
                R.raw[i] = *reinterpret_cast<const u32x4 *>(S.x + (rb + slot) * FR + strip * (16 * 84) + (t % (CHUNKS / 4)) * 16);
            }
        }
    }
}
// 16 pixels -> 16 bf16 -> two 16-byte LDS stores; consecutive lanes write consecutive 32 bytes
__device__ __forceinline__ void strip_store(bf16_t *xs, const StripRaw &R, int lane)
{
#pragma unroll
    for (int i = 0; i < 7; ++i) {
        const int t = lane + 64 * i;
        if (t < CHUNKS) {
            const u32x4 r = R.raw[i];
            uint4 *d = reinterpret_cast<uint4 *>(xs + t * 16);
            d[0] = cvt8_u8(r.x, r.y);
            d[1] = cvt8_u8(r.z, r.w);
        }
    }
}

// Units [u0, u1) of one segment (unit = UNITS * sample + strip), processed by one wave.  Weights and
// bias stay in registers; the pixels of the next unit are loaded while the current one is computed,
// and the ring slot of the unit after that is already on its way.
//
// In draw mode the kernel has drawn the samples itself (see k_conv1_fwd) and `slots` holds them;
// otherwise the slots are read from S.src.idx, where a sampling kernel left them.
__device__ __forceinline__ void conv1_fwd_units(const FwdSeg &S, int u0, int u1, bf16_t *xs, const int *slots, int lane)
{
    const int n = lane & 15, kg = lane >> 4, oyl = n >> 2, q = n & 3;
    StripOff O;
#pragma unroll
    for (int i = 0; i < 7; ++i) {
        const int t = lane + 64 * i;
        O.off[i] = t < CHUNKS ? (t / (CHUNKS / 4)) * FR + (t % (CHUNKS / 4)) * 16 : 0;
    }
    StripRaw R;
    int g = u0 / UNITS, strip = u0 % UNITS;   // current unit
    int gn = g, sn = strip + 1;               // next unit
    if (sn == UNITS) { sn = 0; ++gn; }
    // draw mode: slots[] holds the slots of this wave's samples of this segment, first one at index 0
    const int gfirst = g;
    auto slot_of = [&](int gq) { return slots ? slots[gq - gfirst] : sample_slot(S.src, gq); };
    strip_load(R, S.src, g, slot_of(g), strip, lane, O);
    int slot_next = u0 + 1 < u1 ? slot_of(gn) : 0;
    v8bf wa[8][2];   // [2c + xh][channel half]
#pragma unroll
    for (int st = 0; st < 8; ++st)
#pragma unroll
        for (int hh = 0; hh < 2; ++hh) {
            const int ch = 8 * (n >> 2) + 4 * hh + (n & 3);
            const bf16_t *p = S.w + ch * 256 + (st >> 1) * 64 + (2 * kg) * 8 + 4 * (st & 1);
            const uint2 lo = *reinterpret_cast<const uint2 *>(p), hi = *reinterpret_cast<const uint2 *>(p + 8);
            wa[st][hh] = __builtin_bit_cast(v8bf, uint4{lo.x, lo.y, hi.x, hi.y});
        }
    const v4f b0 = *reinterpret_cast<const v4f *>(S.bias + 8 * kg), b1 = *reinterpret_cast<const v4f *>(S.bias + 8 * kg + 4);
    // LDS byte address of this lane's first quad of frame 0; a frame is SROWS * 84 elements further
    const uint32_t px = (uint32_t)(uintptr_t)(xs + (4 * oyl + 2 * kg) * 84 + 20 * q);
    const uint32_t yoff = ((20 * oyl + 5 * q) * 32 + 8 * kg) * 2;   // bytes, within the unit's 80 output pixels
    for (int u = u0; u < u1; ++u) {
        strip_store(xs, R, lane);   // LDS operations of one wave complete in order: no wait needed around this
        if (u + 1 < u1) {
            strip_load(R, S.src, gn, slot_next, sn, lane, O);
            int g2 = gn;
            if (sn + 1 == UNITS) ++g2;
            if (u + 2 < u1) slot_next = slot_of(g2);
        }
        struct Quads { uint4 q[6]; };
        // The compiler would pair neighbouring columns of ONE row into a two-address read and then
        // shuffle registers; the pairing wanted here is the same columns of TWO rows (21 eight-byte
        // steps apart), which lands each quad in the four consecutive registers the MFMA reads.
        // These reads are invisible to the compiler's wait counting: the waits are written out.
        auto quads = [&](int c) {
            typedef uint32_t v4u __attribute__((ext_vector_type(4)));
            const uint32_t addr = px + c * (SROWS * 84 * 2);
            Quads Q;
#define C1_RD2(JJ) { v4u t; asm volatile("ds_read2_b64 %0, %1 offset0:%2 offset1:%3" : "=v"(t) : "v"(addr), "n"(JJ), "n"(JJ + 21)); Q.q[JJ] = uint4{t.x, t.y, t.z, t.w}; }
            C1_RD2(0) C1_RD2(1) C1_RD2(2) C1_RD2(3) C1_RD2(4) C1_RD2(5)
#undef C1_RD2
            return Q;
        };
        v4f acc[5][2];
#pragma unroll
        for (int j = 0; j < 5; ++j) acc[j][0] = acc[j][1] = v4f{0, 0, 0, 0};
        Quads cur = quads(0);
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            Quads nxt = cur;
            asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");   // `cur` has arrived
            if (c < 3) nxt = quads(c + 1);                        // in flight during the 20 MFMAs below
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int xh = 0; xh < 2; ++xh)
#pragma unroll
                for (int j = 0; j < 5; ++j) {
                    const v8bf b = __builtin_bit_cast(v8bf, cur.q[j + xh]);
                    acc[j][0] = mfma16(wa[2 * c + xh][0], b, acc[j][0]);
                    acc[j][1] = mfma16(wa[2 * c + xh][1], b, acc[j][1]);
                }
            __builtin_amdgcn_sched_barrier(0);
            cur = nxt;
        }
        // bias, 1/255, ReLU, bf16; the 80 pixels of a unit are contiguous in y
        uint8_t *yb = reinterpret_cast<uint8_t *>(S.y) + ((long)g * 400 + 80 * strip) * 64;
        constexpr float sc = 1.0f / 255.0f;
#pragma unroll
        for (int j = 0; j < 5; ++j) {
            const v4f a0 = acc[j][0], a1 = acc[j][1];
            const uint2 lo = pack4(fmaxf(a0.x * sc + b0.x, 0.f), fmaxf(a0.y * sc + b0.y, 0.f),
                                   fmaxf(a0.z * sc + b0.z, 0.f), fmaxf(a0.w * sc + b0.w, 0.f));
            const uint2 hi = pack4(fmaxf(a1.x * sc + b1.x, 0.f), fmaxf(a1.y * sc + b1.y, 0.f),
                                   fmaxf(a1.z * sc + b1.z, 0.f), fmaxf(a1.w * sc + b1.w, 0.f));
            *reinterpret_cast<uint4 *>(yb + yoff + j * 64) = uint4{lo.x, lo.y, hi.x, hi.y};
        }
        g = gn; strip = sn;
        if (++sn == UNITS) { sn = 0; ++gn; }
    }
}

// Draw mode (replay: every segment has the same n samples, sample g of a segment is draw g).
// The wave walks the sum-tree (Eq.10) for the samples of its unit range [u0, u1) before it requests
// a pixel: two draws per walk, its range touches two samples as a rule and never more than
// MAX_DRAWS (the host sizes the grid accordingly).  slots[k] = slot of the k-th sample of the
// range; with `publish`, the wave that owns strip 0 of a sample of segment 0 writes the index, the
// raw importance weight and the transition data for the kernels that follow.
__device__ __forceinline__ void draw_slots(const misc::SampleArgs &P, int n, int u0, int u1, int *slots, int lane,
                                           bool publish)
{
    const int gs0 = u0 / UNITS, gs1 = (u1 - 1) / UNITS;   // launch-wide sample numbers
#pragma unroll 1
    for (int ga = gs0; ga <= gs1; ga += 2) {
        const int gb = ga + 1 <= gs1 ? ga + 1 : ga;
        const int jj[2] = {ga % n, gb % n};
        long sl[2];
        float leaf[2];
        const float total = misc::per_sample_walk<2>(P, jj, lane, sl, leaf);
        if (lane == 0) {
            slots[ga - gs0] = (int)sl[0];
            slots[gb - gs0] = (int)sl[1];
        }
        // lanes 0 and 1 publish one draw each
        if (lane == 0 && publish && ga < n && UNITS * ga >= u0) misc::per_sample_emit(P, ga, sl[0], total, leaf[0]);
        if (lane == 1 && publish && gb < n && gb != ga) misc::per_sample_emit(P, gb, sl[1], total, leaf[1]);
    }
}

// Wave w of the launch owns units [w*U/W, (w+1)*U/W) of the launch-wide list (segment after segment,
// U = UNITS * samples, W = 4 * gridDim.x).  Two workgroups of four waves fit one CU.
__global__ __launch_bounds__(256, 2) void k_conv1_fwd(FwdArgs A)
{
    __shared__ __attribute__((aligned(16))) bf16_t lds[4 * STRIP];
    __shared__ int slot_tab[4][MAX_DRAWS];
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    bf16_t *xs = lds + wave * STRIP;
    const long nw = (long)gridDim.x * 4, wid = (long)blockIdx.x * 4 + wave, units = (long)A.total * UNITS;
    const int u0 = (int)(wid * units / nw), u1 = (int)((wid + 1) * units / nw);
    if (A.draw && u0 < u1) draw_slots(A.samp, A.seg[0].n, u0, u1, slot_tab[wave], lane, true);
    for (int s = 0; s < A.nseg; ++s) {
        FwdSeg S = A.seg[0];
        if (s == 1) S = A.seg[1];
        if (s == 2) S = A.seg[2];
        const int lo = max(u0, UNITS * S.first) - UNITS * S.first;
        const int hi = min(u1, UNITS * (S.first + S.n)) - UNITS * S.first;
        // the first sample of [lo, hi) is launch-wide sample S.first + lo / UNITS
        if (lo < hi) conv1_fwd_units(S, lo, hi, xs, A.draw ? slot_tab[wave] + (S.first + lo / UNITS - u0 / UNITS) : nullptr, lane);
    }
}


// ---------------------------------------------------------------------------
// The same forward pass in fp32 (v_mfma_f32_16x16x4_f32), for the full-precision path.
//
// Units and lanes as above (strip of 4 output rows, 16 lanes x 5 pixels), but the strip stays in
// LDS as the uint8 it is (6,720 bytes per wave, no conversion while staging): the MFMA takes one
// reduction element per lane and instruction, lane group kg supplies kernel row 4yq + kg, and a
// lane's six 4-byte words of that row (pixels 4jj .. 4jj+3 of its run) serve, byte by byte, the
// kernel columns of all five pixels: word jj is columns 0-3 of pixel jj and columns 4-7 of pixel
// jj-1.  One v_cvt_f32_ubyte per byte, 24 per 40 MFMAs.
// A wave holds the weights of 16 output channels (64 registers): waves work in pairs, one channel
// half each.  KS = 2 (small batches: fewer units than SIMDs) also cuts the reduction in two, frames
// 0-1 and 2-3, over two such pairs, which then add their sums through LDS in a fixed order.
// The first wave of a group can copy its strip to a gathered stack (the weight-gradient kernel of
// this path reads a materialised state): segment 0 supplies frames 0-3, segment 1 its last frame.
// ---------------------------------------------------------------------------
constexpr int RAWSTRIP = 4 * SROWS * 84;   // bytes of one strip as uint8
struct FwdSegF {
    Src src;
    const float *w;     // [32][256] fp32, k = (c, ky, kx)
    const float *bias;  // [32]
    float *y;           // [n][400][32]
    int n;
    int first;
    uint8_t *stack;     // [n][5][84][84] or nullptr
    int stack_mode;     // 1: frames 0-3 of the sample to stack frames 0-3; 2: frame 3 to stack frame 4
};
struct FwdArgsF {
    FwdSegF seg[3];
    int nseg;
    int total;
    int draw;
    misc::SampleArgs samp;
};

__device__ __forceinline__ v4f mfma4(float a, float b, v4f c)
{
    return __builtin_amdgcn_mfma_f32_16x16x4f32(a, b, c, 0, 0, 0);
}

template <int KS>
__device__ __forceinline__ void conv1_fwd_units_f32(const FwdSegF &S, int u0, int u1, int hh, int ks, uint8_t *xs,
                                                    v4f *red, const int *slots, int lane)
{
    constexpr int NCY = 8 / KS;   // (frame, kernel-row half) pairs of this wave
    const int n = lane & 15, kg = lane >> 4, oyl = n >> 2, q = n & 3;
    const bool first_wave = hh == 0 && ks == 0;
    StripOff O;
#pragma unroll
    for (int i = 0; i < 7; ++i) {
        const int t = lane + 64 * i;
        O.off[i] = t < CHUNKS ? (t / (CHUNKS / 4)) * FR + (t % (CHUNKS / 4)) * 16 : 0;
    }
    const int gfirst = u0 / UNITS;
    auto slot_of = [&](int gq) { return slots ? slots[gq - gfirst] : sample_slot(S.src, gq); };
    StripRaw R;
    strip_load(R, S.src, gfirst, slot_of(gfirst), u0 % UNITS, lane, O);
    int slot_next = u0 + 1 < u1 ? slot_of((u0 + 1) / UNITS) : 0;
    // weights: wa[8 cyl + 4 xh + b] = W[16hh + n][frame, kernel row 4yq + kg of pair NCY ks + cyl][4 xh + b]
    float wa[8 * NCY];
#pragma unroll
    for (int cyl = 0; cyl < NCY; ++cyl) {
        const int cy = NCY * ks + cyl;
        const float *p = S.w + (16 * hh + n) * 256 + (cy >> 1) * 64 + (4 * (cy & 1) + kg) * 8;
        const v4f lo = *reinterpret_cast<const v4f *>(p), hi = *reinterpret_cast<const v4f *>(p + 4);
        wa[8 * cyl + 0] = lo.x; wa[8 * cyl + 1] = lo.y; wa[8 * cyl + 2] = lo.z; wa[8 * cyl + 3] = lo.w;
        wa[8 * cyl + 4] = hi.x; wa[8 * cyl + 5] = hi.y; wa[8 * cyl + 6] = hi.z; wa[8 * cyl + 7] = hi.w;
    }
    const v4f bias = *reinterpret_cast<const v4f *>(S.bias + 16 * hh + 4 * kg);
    const uint8_t *px = xs + (4 * oyl + kg) * 84 + 20 * q;
    for (int u = u0; u < u1; ++u) {
        const int g = u / UNITS, strip = u % UNITS;
#pragma unroll
        for (int i = 0; i < 7; ++i) {
            const int t = lane + 64 * i;
            if (t < CHUNKS) {
                *reinterpret_cast<u32x4 *>(xs + t * 16) = R.raw[i];
                // rows 16s .. 16s+15 of the frames are this strip's own (the last strip owns all 20)
                const int fr = t / (CHUNKS / 4), off = (t % (CHUNKS / 4)) * 16;
                if (first_wave && S.stack && (off < 16 * 84 || strip == UNITS - 1) && (S.stack_mode == 1 || fr == 3))
                    *reinterpret_cast<u32x4 *>(S.stack + ((long)g * 5 + (S.stack_mode == 1 ? fr : 4)) * FR + strip * (16 * 84) + off) = R.raw[i];
            }
        }
        if (u + 1 < u1) {
            strip_load(R, S.src, (u + 1) / UNITS, slot_next, (u + 1) % UNITS, lane, O);
            if (u + 2 < u1) slot_next = slot_of((u + 2) / UNITS);
        }
        v4f acc[5];
#pragma unroll
        for (int j = 0; j < 5; ++j) acc[j] = v4f{0, 0, 0, 0};
#pragma unroll
        for (int cyl = 0; cyl < NCY; ++cyl) {
            const int cy = NCY * ks + cyl;   // frame cy / 2, kernel rows 4 (cy % 2) + kg
            const uint8_t *p = px + (cy >> 1) * (SROWS * 84) + (cy & 1) * (4 * 84);
            uint32_t d[6];
#pragma unroll
            for (int jj = 0; jj < 6; ++jj) d[jj] = *reinterpret_cast<const uint32_t *>(p + 4 * jj);
            float f[6][4];
#pragma unroll
            for (int jj = 0; jj < 6; ++jj) {
                f[jj][0] = (float)(d[jj] & 0xFFu);
                f[jj][1] = (float)((d[jj] >> 8) & 0xFFu);
                f[jj][2] = (float)((d[jj] >> 16) & 0xFFu);
                f[jj][3] = (float)(d[jj] >> 24);
            }
#pragma unroll
            for (int xh = 0; xh < 2; ++xh)
#pragma unroll
                for (int b = 0; b < 4; ++b)
#pragma unroll
                    for (int j = 0; j < 5; ++j) acc[j] = mfma4(wa[8 * cyl + 4 * xh + b], f[j + xh][b], acc[j]);
        }
        if constexpr (KS == 2) {   // frames 2-3 join frames 0-1; the buffer alternates, so one barrier per unit
            v4f *r = red + (((u - u0) & 1) * 2 + hh) * (5 * 64);
            if (ks == 1) {
#pragma unroll
                for (int j = 0; j < 5; ++j) r[j * 64 + lane] = acc[j];
            }
            sync_lds();
            if (ks == 0) {
#pragma unroll
                for (int j = 0; j < 5; ++j) acc[j] += r[j * 64 + lane];
            }
        }
        if (ks == 0) {
            float *y = S.y + ((long)g * 400 + 20 * (4 * strip + oyl) + 5 * q) * 32 + 16 * hh + 4 * kg;
            constexpr float sc = 1.0f / 255.0f;
#pragma unroll
            for (int j = 0; j < 5; ++j) {
                v4f o;
                o.x = fmaxf(acc[j].x * sc + bias.x, 0.f);
                o.y = fmaxf(acc[j].y * sc + bias.y, 0.f);
                o.z = fmaxf(acc[j].z * sc + bias.z, 0.f);
                o.w = fmaxf(acc[j].w * sc + bias.w, 0.f);
                *reinterpret_cast<v4f *>(y + j * 32) = o;
            }
        }
    }
}

// KS = 1: the four waves of a workgroup are two pairs, each with a unit range of its own.
// KS = 2: they are one group of four on one unit range.
template <int KS>
__global__ __launch_bounds__(256, 2) void k_conv1_fwd_f32(FwdArgsF A)
{
    __shared__ __attribute__((aligned(16))) uint8_t lds[4 * RAWSTRIP];
    __shared__ __attribute__((aligned(16))) v4f red[KS == 2 ? 2 * 2 * 5 * 64 : 1];
    __shared__ int slot_tab[4][MAX_DRAWS];
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int hh = wave & 1, ks = KS == 2 ? wave >> 1 : 0;
    const long ng = (long)gridDim.x * (KS == 2 ? 1 : 2), gid = KS == 2 ? (long)blockIdx.x : (long)blockIdx.x * 2 + (wave >> 1);
    const long units = (long)A.total * UNITS;
    const int u0 = (int)(gid * units / ng), u1 = (int)((gid + 1) * units / ng);
    if (A.draw && u0 < u1) draw_slots(A.samp, A.seg[0].n, u0, u1, slot_tab[wave], lane, hh == 0 && ks == 0);
    for (int s = 0; s < A.nseg; ++s) {
        FwdSegF S = A.seg[0];
        if (s == 1) S = A.seg[1];
        if (s == 2) S = A.seg[2];
        const int lo = max(u0, UNITS * S.first) - UNITS * S.first;
        const int hi = min(u1, UNITS * (S.first + S.n)) - UNITS * S.first;
        if (lo < hi)
            conv1_fwd_units_f32<KS>(S, lo, hi, hh, ks, lds + wave * RAWSTRIP, red,
                                    A.draw ? slot_tab[wave] + (S.first + lo / UNITS - u0 / UNITS) : nullptr, lane);
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
constexpr int WG1_LDS = 2 * FR + 400 * LDY1;   // LDS elements of a workgroup
// tile = 2 * split + channel pair
__device__ __forceinline__ void conv1_wgrad_block(const WgradArgs &A, int tile, bf16_t *lds)
{
    bf16_t *xin = lds, *dys = lds + 2 * FR;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;  // wave = block of 32 im2col columns
    const int li = lane & 31, h = lane >> 5, s16 = lane & 15, half = (lane >> 4) & 1;
    // the two channel pairs of one sample split run next to each other: same dY, same ring slots
    const int cp = tile & 1, split = tile >> 1;
    typedef __attribute__((address_space(3))) v4s *lds_v4s;

    // this lane's share of the transpose loads: reduction row offset s/4 (+4 for the second
    // load), columns 16*half + 4*(s%4) .. +3 of the wave's 32-column block
    const int rsub = 8 * h + (s16 >> 2);
    const int kc = 32 * wave + 16 * half + 4 * (s16 & 3);       // column within the pair: (c, p, q0)
    const int xoff = (kc >> 6) * FR + ((kc >> 3) & 7) * 84 + (kc & 7);
    const bf16_t *yp = dys + rsub * LDY1 + 16 * half + 4 * (s16 & 3);
    const bf16_t *xw = xin + xoff + 4 * rsub;   // the window of output pixel rsub

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
        // the operands of step t + 1 are requested before the matrix instruction of step t
        auto operands = [&](int t, v8bf &fa, v8bf &fb) {   // 16 output pixels per step
            fa = frag_tr(yp + 16 * t * LDY1, LDY1);
            // pixel m = 16t + rsub (and m + 4) of the 20-wide output: its window starts at input row 4(m/20),
            // column 4(m%20).  16t = 20q + r with q, r known at compile time, so the lane only has to see
            // whether r + rsub runs over into the next row: no division
            const int q = (16 * t) / 20, r = (16 * t) % 20;
            const bf16_t *x0 = xw + (336 * q + 4 * r) + (rsub >= 20 - r ? 256 : 0);
            const bf16_t *x1 = xw + (336 * q + 4 * r + 16) + (rsub + 4 >= 20 - r ? 256 : 0);
            v4s lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_v4s)x0);
            v4s hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_v4s)x1);
            typedef short v8s __attribute__((ext_vector_type(8)));
            v8s xb = {lo.x, lo.y, lo.z, lo.w, hi.x, hi.y, hi.z, hi.w};
            fb = __builtin_bit_cast(v8bf, xb);
        };
        v8bf fa, fb, fan, fbn;
        operands(0, fa, fb);
#pragma unroll
        for (int t = 0; t < 25; ++t) {
            fan = fa; fbn = fb;
            if (t + 1 < 25) operands(t + 1, fan, fbn);
            __builtin_amdgcn_sched_barrier(0);
            acc = mfma(fa, fb, acc);
            if (do_bias) accb = mfma(fa, ones, accb);
            __builtin_amdgcn_sched_barrier(0);
            fa = fan; fb = fbn;
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
__global__ __launch_bounds__(256) void k_conv1_wgrad(WgradArgs A)
{
    __shared__ __attribute__((aligned(16))) bf16_t lds[WG1_LDS];
    conv1_wgrad_block(A, net::tile_of_workgroup(), lds);
}
}  // namespace c1

// ===========================================================================
// conv2 and conv3 forward, one sample per workgroup at a time ("ps" = per sample).
//
// The generic kernels above cut the batch into row tiles and walk the reduction in stages with
// two barriers each; for these two layers a stage holds a handful of MFMAs, so the walk is a
// chain of latencies.  Here a persistent workgroup of four waves keeps its share of the WEIGHTS in
// registers (32 output channels x the whole reduction per wave), copies one sample's input
// (25.6 KB / 10.4 KB) into LDS with one barrier per sample, double-buffered, and every b-operand
// is a single 16-byte LDS read at base + immediate offset: no index arithmetic in the loop.
//
// v_mfma_f32_16x16x32_bf16, weights as the a-operand (row r = channel 32hh + 8(r/4) + 4cb + r%4 for
// the wave's channel half hh and channel block cb), output positions as the b-operand columns; one
// reduction step is one kernel tap x 32 input channels, lane group kg = lane/16 takes 8 of them.
// Wave (ph, hh) owns half of the position blocks and half of the channels; the result of lane
// (n, g = lane/16) is channels 32hh + 8g .. +7 of its positions: 16 bytes per store.
//
// LDS layout of a sample: pixels in raster order, padded so that the pixels which the 16 lanes of
// one lane group read (two apart for the stride-2 layer, neighbours for the stride-1 layer) start
// 144 bytes apart, i.e. one 16-byte bank group further each: conflict-free.
// ===========================================================================
namespace ps {
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));   // a native vector: stays in registers across barriers

struct Seg {
    const bf16_t *x;    // [n][positions in][channels in]
    const bf16_t *w;    // [64][K] bf16, K = (tap, channel)
    const float *bias;  // [64]
    bf16_t *y;          // [n][positions out][64]
    int n;              // samples
    int first;          // index of the segment's first sample in the launch-wide sample list
};
struct Args {
    Seg seg[3];
    int nseg;
    int total;
};

// G: layer geometry.  IN_PIX pixels of IN_CH channels in, OUT x OUT positions out, TAPS x TAPS
// kernel with stride STRIDE, IN_W pixels per input row.
struct G2 { static constexpr int IN_PIX = 400, IN_CH = 32, IN_W = 20, OUT = 9, TAPS = 4, STRIDE = 2; };
struct G3 { static constexpr int IN_PIX = 81, IN_CH = 64, IN_W = 9, OUT = 7, TAPS = 3, STRIDE = 1; };

template <class G> struct Shape {
    static constexpr int PB = G::IN_CH * 2;                        // bytes per pixel
    static constexpr int GROUP = 128 / PB;                         // pixels per 128-byte group: 2 / 1
    static constexpr int GB = 144;                                 // LDS bytes per group (128 + 16)
    static constexpr int SAMPLE = (G::IN_PIX / GROUP + (G::IN_PIX % GROUP ? 1 : 0)) * GB;
    static constexpr int K = G::TAPS * G::TAPS * G::IN_CH;
    static constexpr int STEPS = K / 32;                           // reduction steps: 16 / 18
    static constexpr int SPT = G::IN_CH / 32;                      // steps per tap: 1 / 2
    static constexpr int WROW = K * 2 + 16;                        // LDS bytes per weight row in transit
    static constexpr int NPOS = G::OUT * G::OUT;                   // 81 / 49
    static constexpr int NBLK = (NPOS + 31) / 32;                  // position blocks per wave: 3 / 2
    static constexpr int CHUNKS = G::IN_PIX * PB / 16;             // 16-byte pieces of a sample: 1600 / 648
    static constexpr int NLD = (CHUNKS + 255) / 256;               // pieces per thread: 7 / 3
    static constexpr int WCH = 32 * K * 2 / 16 / 256;              // weight pieces per thread and half: 8 / 9
    static constexpr int LDS = 32 * WROW > 2 * SAMPLE ? 32 * WROW : 2 * SAMPLE;
    // LDS byte offset of 16-byte piece c of pixel q
    static __device__ __forceinline__ uint32_t at(int q, int c) { return (q / GROUP) * GB + (q % GROUP) * PB + c * 16; }
};

template <class G> struct Raw { u32x4 r[Shape<G>::NLD]; };
template <class G>
__device__ __forceinline__ void load_sample(Raw<G> &R, const bf16_t *x, int tid)
{
    using S = Shape<G>;
    const u32x4 *p = reinterpret_cast<const u32x4 *>(x);
#pragma unroll
    for (int i = 0; i < S::NLD; ++i) { const int t = tid + 256 * i; R.r[i] = p[t < S::CHUNKS ? t : S::CHUNKS - 1]; }
}
template <class G>
__device__ __forceinline__ void store_sample(uint8_t *buf, const Raw<G> &R, int tid)
{
    using S = Shape<G>;
    constexpr int CPP = S::PB / 16;   // pieces per pixel
#pragma unroll
    for (int i = 0; i < S::NLD; ++i) {
        const int t = tid + 256 * i;
        if (t < S::CHUNKS) *reinterpret_cast<u32x4 *>(buf + S::at(t / CPP, t % CPP)) = R.r[i];
    }
}

// Samples [g0, g1) of one segment.
template <class G>
__device__ __forceinline__ void run(const Seg &S, int g0, int g1, uint8_t *lds, int tid)
{
    using H = Shape<G>;
    const int lane = tid & 63, n = lane & 15, kg = lane >> 4;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6), ph = wave & 1, hh = wave >> 1;
    Raw<G> R;
    load_sample<G>(R, S.x + (long)g0 * (G::IN_PIX * G::IN_CH), tid);   // on its way while the weights are fetched
    // The workgroup fetches each half of the weight matrix once, coalesced, into LDS; the two waves
    // that own the half pick their fragments from there.
    v8bf wa[H::STEPS][2];
    for (int half = 0; half < 2; ++half) {
        const u32x4 *src = reinterpret_cast<const u32x4 *>(S.w + half * 32 * H::K);
        sync_lds();   // LDS is free (the previous segment's last sample has been read)
#pragma unroll
        for (int i = 0; i < H::WCH; ++i) {
            const int c = tid + 256 * i;   // row c / (K/8), piece c % (K/8)
            *reinterpret_cast<u32x4 *>(lds + (c / (H::K / 8)) * H::WROW + (c % (H::K / 8)) * 16) = src[c];
        }
        sync_lds();
        if (hh == half) {
#pragma unroll
            for (int st = 0; st < H::STEPS; ++st)
#pragma unroll
                for (int cb = 0; cb < 2; ++cb) {
                    const int chl = 8 * (n >> 2) + 4 * cb + (n & 3);
                    wa[st][cb] = __builtin_bit_cast(v8bf, *reinterpret_cast<const uint4 *>(lds + chl * H::WROW + st * 64 + kg * 16));
                }
        }
    }
    const v4f b0 = *reinterpret_cast<const v4f *>(S.bias + 32 * hh + 8 * kg);
    const v4f b1 = *reinterpret_cast<const v4f *>(S.bias + 32 * hh + 8 * kg + 4);
    // this lane's positions and the LDS offset of their first tap; positions past the end read a
    // valid pixel and are not stored
    uint32_t base[H::NBLK];
    int pos[H::NBLK];
#pragma unroll
    for (int b = 0; b < H::NBLK; ++b) {
        int p = 16 * (H::NBLK * ph + b) + n;
        pos[b] = p;
        if (p > H::NPOS - 1) p = H::NPOS - 1;
        base[b] = H::at(G::STRIDE * (G::IN_W * (p / G::OUT) + (p % G::OUT)), kg);
    }
    sync_lds();   // the weight rows have been read
    store_sample<G>(lds + (g0 & 1) * H::SAMPLE, R, tid);
    load_sample<G>(R, S.x + (long)min(g0 + 1, g1 - 1) * (G::IN_PIX * G::IN_CH), tid);
    for (int g = g0; g < g1; ++g) {
        sync_lds();   // buffer g&1 is complete; buffer (g+1)&1 is no longer read
        if (g + 1 < g1) store_sample<G>(lds + ((g + 1) & 1) * H::SAMPLE, R, tid);
        // the last loads repeat the last sample: redundant, never out of range
        load_sample<G>(R, S.x + (long)min(g + 2, g1 - 1) * (G::IN_PIX * G::IN_CH), tid);
        const uint8_t *buf = lds + (g & 1) * H::SAMPLE;
        v4f acc[H::NBLK][2];
#pragma unroll
        for (int b = 0; b < H::NBLK; ++b) acc[b][0] = acc[b][1] = v4f{0, 0, 0, 0};
        // byte offset of reduction step st: pixel (ky, kx) further, second half of its channels for odd
        // steps of the 64-channel layer
        auto step_off = [](int st) {
            const int tap = st / H::SPT, ky = tap / G::TAPS, kx = tap % G::TAPS;
            return (int)H::at(G::IN_W * ky + kx, 0) + (st % H::SPT) * 64;
        };
        // the operands of step st+1 are requested before the matrix instructions of step st
        uint4 cur[H::NBLK], nxt[H::NBLK];
#pragma unroll
        for (int b = 0; b < H::NBLK; ++b) cur[b] = *reinterpret_cast<const uint4 *>(buf + base[b] + step_off(0));
#pragma unroll
        for (int st = 0; st < H::STEPS; ++st) {
            if (st + 1 < H::STEPS) {
#pragma unroll
                for (int b = 0; b < H::NBLK; ++b) nxt[b] = *reinterpret_cast<const uint4 *>(buf + base[b] + step_off(st + 1));
            }
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int b = 0; b < H::NBLK; ++b) {
                const v8bf bb = __builtin_bit_cast(v8bf, cur[b]);
                acc[b][0] = mfma16(wa[st][0], bb, acc[b][0]);
                acc[b][1] = mfma16(wa[st][1], bb, acc[b][1]);
            }
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int b = 0; b < H::NBLK; ++b) cur[b] = nxt[b];
        }
        bf16_t *y = S.y + (long)g * (H::NPOS * 64) + 32 * hh + 8 * kg;
#pragma unroll
        for (int b = 0; b < H::NBLK; ++b) {
            // unconditional: a lane past the last position has computed the last position once more (its
            // operand address was clamped to that pixel) and stores the same bits there.  Without a branch
            // the compiler can count these stores, and the wait for the next sample's pixels, requested
            // before them, does not wait for their acknowledgement as well.
            const v4f a0 = acc[b][0], a1 = acc[b][1];
            const uint2 lo = pack4(fmaxf(a0.x + b0.x, 0.f), fmaxf(a0.y + b0.y, 0.f), fmaxf(a0.z + b0.z, 0.f), fmaxf(a0.w + b0.w, 0.f));
            const uint2 hi = pack4(fmaxf(a1.x + b1.x, 0.f), fmaxf(a1.y + b1.y, 0.f), fmaxf(a1.z + b1.z, 0.f), fmaxf(a1.w + b1.w, 0.f));
            *reinterpret_cast<uint4 *>(y + (pos[b] < H::NPOS ? pos[b] : H::NPOS - 1) * 64) = uint4{lo.x, lo.y, hi.x, hi.y};
        }
    }
}

// Workgroup b owns samples [b*total/G, (b+1)*total/G) of the launch-wide list; two workgroups fit one CU.
template <class G>
__global__ __launch_bounds__(256, 2) void k_conv_fwd_ps(Args A)
{
    __shared__ __attribute__((aligned(16))) uint8_t lds[Shape<G>::LDS];
    const int g0 = (int)((long)blockIdx.x * A.total / gridDim.x);
    const int g1 = (int)((long)(blockIdx.x + 1) * A.total / gridDim.x);
    for (int s = 0; s < A.nseg; ++s) {
        Seg S = A.seg[0];
        if (s == 1) S = A.seg[1];
        if (s == 2) S = A.seg[2];
        const int lo = max(g0, S.first) - S.first, hi = min(g1, S.first + S.n) - S.first;
        if (lo < hi) run<G>(S, lo, hi, lds, threadIdx.x);
    }
}
}  // namespace ps

// ===========================================================================
// conv1 + conv2 forward in ONE launch (Section 2.1 network): conv1's output of a sample never leaves
// the CU unless a later kernel reads it (the backward pass reads it for the training rows only).
//
// A workgroup of eight waves owns a run of samples of one segment.  Waves 0-3 are PRODUCERS: each
// computes one conv1 strip per interval exactly as c1::k_conv1_fwd does (strip staged in LDS of its
// own, weights in registers, next strip's pixels in flight) and writes the 80 x 32 result into the
// sample's place in a ring of three LDS images, in the layout ps::run reads.  Waves 4-7 are
// CONSUMERS: they hold conv2's weights in registers as ps::k_conv_fwd_ps does and, in every interval
// in which a sample has become complete, compute its conv2 output out of the ring.  One barrier per
// interval.  Strips are dealt out in order, four per interval, five per sample: sample k is complete
// after interval floor((5k+4)/4) and is consumed in the first interval i with 4i >= 5k+5, which is a
// different interval for every k; the producers are then at most two samples ahead of the sample
// being read, so three images suffice.
//
// Replay mode: the workgroup draws its samples first (Eq.10 walk, two draws per wave and walk, all
// eight waves), while the consumers' weight loads are in flight; the workgroups of segment 0 publish
// the draws.  Otherwise the slots (ring mode) are copied into LDS from where a sampling kernel left them.
// Workgroups are dealt out per segment, so none pays the start-up twice.
// ===========================================================================
namespace c12 {
using c1::Src;
using c1::StripOff;
using c1::StripRaw;
using c1::STRIP;
using c1::UNITS;
using S2 = ps::Shape<ps::G2>;
using ps::u32x4;

struct Seg {
    Src src;
    const bf16_t *w1;   // [32][256]
    const float *b1;    // [32]
    bf16_t *y1;         // [n][400][32], or nullptr: conv1's output is not kept
    const bf16_t *w2;   // [64][512]
    const float *b2;    // [64]
    bf16_t *y2;         // [n][81][64]
    int n;              // samples
};
struct Args {
    Seg seg[3];
    int nseg;
    int draw;           // replay mode: sample g of every segment is draw g of `samp`; segment 0 publishes
    misc::SampleArgs samp;
};

constexpr int NRING = 3;                                    // conv1 images in LDS
constexpr int MAX_PER_WG = 32;                              // samples one workgroup may own (slot table)
constexpr int STRIPS_B = 4 * STRIP * 2;                     // 53,760 bytes: one strip per producer wave
constexpr int RING_B = NRING * S2::SAMPLE;                  // 86,400 bytes
constexpr int LDS_BYTES = STRIPS_B + RING_B + MAX_PER_WG * 8 + 16;   // + slot table, leaf values, total
// The hand-over schedule, as functions the kernel's loops and the host-side check
// (schedule_is_safe, behind dqn_selftest_fused_conv_schedule) both call.
constexpr int PRODUCERS = 4;                                // producer waves: strips per interval
__host__ __device__ constexpr int intervals(int ns) { return (UNITS * ns + PRODUCERS - 1) / PRODUCERS + 1; }
// sample that strip u of a run belongs to, and the image of the ring that holds a sample
__host__ __device__ constexpr int sample_of_strip(int u) { return u / UNITS; }
__host__ __device__ constexpr int image_of_sample(int k) { return k % NRING; }
// is sample kc consumed in interval i?  (its last strip was produced in an earlier interval)
__host__ __device__ constexpr bool consumed_in(int kc, int i) { return UNITS * kc + UNITS <= PRODUCERS * i; }

// Replays the schedule on the host for a run of ns samples: a sample is complete before it is read, it
// is read exactly once, and no strip is written into an image that still holds a sample which has
// not been read or is being read in the same interval.  Returns 0 if safe, else a code naming the failure.
inline int schedule_is_safe(int ns)
{
    if (ns < 1 || ns > MAX_PER_WG) return 1;
    int holds[NRING], written[MAX_PER_WG], consumed[MAX_PER_WG];
    for (int r = 0; r < NRING; ++r) holds[r] = -1;
    for (int k = 0; k < ns; ++k) written[k] = consumed[k] = 0;
    int kc = 0;
    for (int i = 0; i < intervals(ns); ++i) {
        int reading = -1;
        if (kc < ns && consumed_in(kc, i)) {
            if (written[kc] != UNITS || holds[image_of_sample(kc)] != kc) return 2;   // read before complete
            reading = kc;
        }
        for (int u = PRODUCERS * i; u < PRODUCERS * i + PRODUCERS && u < UNITS * ns; ++u) {
            const int k = sample_of_strip(u), img = image_of_sample(k);
            if (holds[img] != k) {
                if (holds[img] >= 0 && !consumed[holds[img]]) return 3;               // overwrites an unread sample
                if (reading >= 0 && image_of_sample(reading) == img) return 4;        // overwrites the sample being read
                holds[img] = k;
            }
            ++written[k];
        }
        if (reading >= 0) { consumed[reading] = 1; ++kc; }
    }
    for (int k = 0; k < ns; ++k)
        if (!consumed[k] || written[k] != UNITS) return 5;                             // something left over
    return 0;
}

// samples [lo, hi) of segment S, consumer wave (ph, hh) = (position half, channel half)
__device__ __forceinline__ void run_consumer(const Seg &S, int lo, int hi, const uint8_t *ring, const v8bf (&wa)[16][2],
                                             int lane, int ph, int hh)
{
    const int n = lane & 15, kg = lane >> 4;
    const int ns = hi - lo, nint = intervals(ns);
    const v4f b0 = *reinterpret_cast<const v4f *>(S.b2 + 32 * hh + 8 * kg);
    const v4f b1 = *reinterpret_cast<const v4f *>(S.b2 + 32 * hh + 8 * kg + 4);
    uint32_t base[3];
    int pos[3];
#pragma unroll
    for (int b = 0; b < 3; ++b) {
        int p = 16 * (3 * ph + b) + n;
        pos[b] = p;
        if (p > 80) p = 80;   // positions past the end read a valid pixel and are not stored
        base[b] = S2::at(2 * (20 * (p / 9) + (p % 9)), kg);
    }
    int kc = 0;   // next sample to consume
    for (int i = 0; i < nint; ++i) {
        if (kc < ns && consumed_in(kc, i)) {
            const uint8_t *buf = ring + image_of_sample(kc) * S2::SAMPLE;
            v4f acc[3][2];
#pragma unroll
            for (int b = 0; b < 3; ++b) acc[b][0] = acc[b][1] = v4f{0, 0, 0, 0};
            // the operands of step st+1 are requested before the matrix instructions of step st
            uint4 cur[3], nxt[3];
#pragma unroll
            for (int b = 0; b < 3; ++b) cur[b] = *reinterpret_cast<const uint4 *>(buf + base[b]);
#pragma unroll
            for (int st = 0; st < 16; ++st) {
                if (st < 15) {
                    const int off = (int)S2::at(20 * ((st + 1) >> 2) + ((st + 1) & 3), 0);
#pragma unroll
                    for (int b = 0; b < 3; ++b) nxt[b] = *reinterpret_cast<const uint4 *>(buf + base[b] + off);
                }
                __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                for (int b = 0; b < 3; ++b) {
                    const v8bf bb = __builtin_bit_cast(v8bf, cur[b]);
                    acc[b][0] = mfma16(wa[st][0], bb, acc[b][0]);
                    acc[b][1] = mfma16(wa[st][1], bb, acc[b][1]);
                }
                __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                for (int b = 0; b < 3; ++b) cur[b] = nxt[b];
            }
            bf16_t *y = S.y2 + (long)(lo + kc) * (81 * 64) + 32 * hh + 8 * kg;
#pragma unroll
            for (int b = 0; b < 3; ++b) {
                if (pos[b] < 81) {
                    const v4f a0 = acc[b][0], a1 = acc[b][1];
                    const uint2 l2 = pack4(fmaxf(a0.x + b0.x, 0.f), fmaxf(a0.y + b0.y, 0.f), fmaxf(a0.z + b0.z, 0.f), fmaxf(a0.w + b0.w, 0.f));
                    const uint2 h2 = pack4(fmaxf(a1.x + b1.x, 0.f), fmaxf(a1.y + b1.y, 0.f), fmaxf(a1.z + b1.z, 0.f), fmaxf(a1.w + b1.w, 0.f));
                    *reinterpret_cast<uint4 *>(y + pos[b] * 64) = uint4{l2.x, l2.y, h2.x, h2.y};
                }
            }
            ++kc;
        }
        sync_lds();
    }
}

// samples [lo, hi) of segment S, producer wave w: strips w, w + 4, ... of the run's strip list.
// R holds the pixels of strip w (requested by the caller); slots: the run's ring slots (ring mode).
__device__ __forceinline__ void run_producer(const Seg &S, int lo, int hi, bf16_t *xs, uint8_t *ring, const int *slots,
                                             StripRaw &R, const StripOff &O, int lane, int w)
{
    const int n = lane & 15, kg = lane >> 4, oyl = n >> 2, q = n & 3;
    const int ns = hi - lo, nstrips = UNITS * ns, nint = intervals(ns);
    v8bf wa[8][2];   // [2c + xh][channel half], as in c1::conv1_fwd_units
#pragma unroll
    for (int st = 0; st < 8; ++st)
#pragma unroll
        for (int h2 = 0; h2 < 2; ++h2) {
            const int ch = 8 * (n >> 2) + 4 * h2 + (n & 3);
            const bf16_t *p = S.w1 + ch * 256 + (st >> 1) * 64 + (2 * kg) * 8 + 4 * (st & 1);
            const uint2 l2 = *reinterpret_cast<const uint2 *>(p), hi2 = *reinterpret_cast<const uint2 *>(p + 8);
            wa[st][h2] = __builtin_bit_cast(v8bf, uint4{l2.x, l2.y, hi2.x, hi2.y});
        }
    const v4f b0 = *reinterpret_cast<const v4f *>(S.b1 + 8 * kg), b1 = *reinterpret_cast<const v4f *>(S.b1 + 8 * kg + 4);
    const uint32_t px = (uint32_t)(uintptr_t)(xs + (4 * oyl + 2 * kg) * 84 + 20 * q);
    int u = w;
    for (int i = 0; i < nint; ++i) {
        if (u < nstrips) {
            const int k = sample_of_strip(u), strip = u % UNITS;
            c1::strip_store(xs, R, lane);   // LDS operations of one wave complete in order
            const int un = u + PRODUCERS;
            if (un < nstrips) c1::strip_load(R, S.src, lo + un / UNITS, S.src.idx ? slots[un / UNITS] : 0, un % UNITS, lane, O);
            struct Quads { uint4 q[6]; };
            auto quads = [&](int c) {   // see c1::conv1_fwd_units
                typedef uint32_t v4u __attribute__((ext_vector_type(4)));
                const uint32_t addr = px + c * (c1::SROWS * 84 * 2);
                Quads Q;
#define C12_RD2(JJ) { v4u t; asm volatile("ds_read2_b64 %0, %1 offset0:%2 offset1:%3" : "=v"(t) : "v"(addr), "n"(JJ), "n"(JJ + 21)); Q.q[JJ] = uint4{t.x, t.y, t.z, t.w}; }
                C12_RD2(0) C12_RD2(1) C12_RD2(2) C12_RD2(3) C12_RD2(4) C12_RD2(5)
#undef C12_RD2
                return Q;
            };
            v4f acc[5][2];
#pragma unroll
            for (int j = 0; j < 5; ++j) acc[j][0] = acc[j][1] = v4f{0, 0, 0, 0};
            Quads cur = quads(0);
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                Quads nxt = cur;
                asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");   // `cur` has arrived
                if (c < 3) nxt = quads(c + 1);
                __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                for (int xh = 0; xh < 2; ++xh)
#pragma unroll
                    for (int j = 0; j < 5; ++j) {
                        const v8bf b = __builtin_bit_cast(v8bf, cur.q[j + xh]);
                        acc[j][0] = mfma16(wa[2 * c + xh][0], b, acc[j][0]);
                        acc[j][1] = mfma16(wa[2 * c + xh][1], b, acc[j][1]);
                    }
                __builtin_amdgcn_sched_barrier(0);
                cur = nxt;
            }
            // bias, 1/255, ReLU, bf16: into the sample's image in the ring and, where kept, to memory
            uint8_t *img = ring + image_of_sample(k) * S2::SAMPLE;
            uint8_t *yb = S.y1 ? reinterpret_cast<uint8_t *>(S.y1) + ((long)(lo + k) * 400 + 80 * strip) * 64 +
                                     ((20 * oyl + 5 * q) * 32 + 8 * kg) * 2
                               : nullptr;
            constexpr float sc = 1.0f / 255.0f;
#pragma unroll
            for (int j = 0; j < 5; ++j) {
                const v4f a0 = acc[j][0], a1 = acc[j][1];
                const uint2 l2 = pack4(fmaxf(a0.x * sc + b0.x, 0.f), fmaxf(a0.y * sc + b0.y, 0.f),
                                       fmaxf(a0.z * sc + b0.z, 0.f), fmaxf(a0.w * sc + b0.w, 0.f));
                const uint2 h2 = pack4(fmaxf(a1.x * sc + b1.x, 0.f), fmaxf(a1.y * sc + b1.y, 0.f),
                                       fmaxf(a1.z * sc + b1.z, 0.f), fmaxf(a1.w * sc + b1.w, 0.f));
                const uint4 v = uint4{l2.x, l2.y, h2.x, h2.y};
                *reinterpret_cast<uint4 *>(img + S2::at(80 * strip + 20 * oyl + 5 * q + j, kg)) = v;
                if (yb) *reinterpret_cast<uint4 *>(yb + j * 64) = v;
            }
            u = un;
        }
        sync_lds();
    }
}

// Segment t owns workgroups [G t / nseg, G (t+1) / nseg); each of them an even share of its samples.
// The host sizes the grid so that no share exceeds MAX_PER_WG.  Dynamic LDS: LDS_BYTES.
__global__ __launch_bounds__(512) void k_conv12_fwd(Args A)
{
    extern __shared__ __attribute__((aligned(16))) uint8_t lds[];
    int s = 0, w0 = 0, w1 = 1;
    for (int t = 0; t < A.nseg; ++t) {
        const int a = (int)((long)gridDim.x * t / A.nseg), b = (int)((long)gridDim.x * (t + 1) / A.nseg);
        if ((int)blockIdx.x >= a && (int)blockIdx.x < b) { s = t; w0 = a; w1 = b; }
    }
    Seg S = A.seg[0];
    if (s == 1) S = A.seg[1];
    if (s == 2) S = A.seg[2];
    const int lo = (int)((long)((int)blockIdx.x - w0) * S.n / (w1 - w0));
    const int hi = (int)((long)((int)blockIdx.x - w0 + 1) * S.n / (w1 - w0));
    if (lo >= hi) return;   // the whole workgroup
    const int ns = hi - lo;
    uint8_t *ring = lds + STRIPS_B;
    int *slots = reinterpret_cast<int *>(lds + STRIPS_B + RING_B);
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);

    float *leafv = reinterpret_cast<float *>(slots + MAX_PER_WG);   // [MAX_PER_WG] leaf values, then the total

    // The slots of the run: drawn here, two per wave and walk, or copied from the index list.  Nothing but
    // the slot stands between a draw and the first pixel request, so the walk leaves the leaf's value and
    // the total in LDS, and what is published per draw (publish_draws) is written after the barrier by a
    // wave that has nothing else to do yet.
    auto fill_slots = [&]() {
        if (!S.src.idx) return;
        if (A.draw) {
#pragma unroll 1
            for (int k = 2 * wave; k < ns; k += 16) {
                const int kb = k + 1 < ns ? k + 1 : k;
                const int jj[2] = {lo + k, lo + kb};
                long sl[2];
                float leaf[2];
                const float total = misc::per_sample_walk<2>(A.samp, jj, lane, sl, leaf);
                if (lane == 0) {
                    slots[k] = (int)sl[0];
                    slots[kb] = (int)sl[1];
                    leafv[k] = leaf[0];
                    leafv[kb] = leaf[1];
                    if (k == 0) leafv[MAX_PER_WG] = total;
                }
            }
        } else {
            for (int k = tid; k < ns; k += 512) slots[k] = S.src.idx[lo + k];
        }
    };
    // index, raw importance weight and transition data of the segment-0 draws, one draw per lane
    auto publish_draws = [&]() {
        if (S.src.idx && A.draw && s == 0 && lane < ns)
            misc::per_sample_emit(A.samp, lo + lane, slots[lane], leafv[MAX_PER_WG], leafv[lane]);
    };

    if (wave >= 4) {
        const int n = lane & 15, kg = lane >> 4, ph = wave & 1, hh = (wave >> 1) & 1;
        // this wave's share of conv2's weights, straight into a-operand registers (row 8(n/4) + 4cb + n%4 of
        // channel half hh, reduction elements 32st + 8kg .. +7); on its way while the slots are found
        v8bf wa[16][2];
#pragma unroll
        for (int st = 0; st < 16; ++st)
#pragma unroll
            for (int cb = 0; cb < 2; ++cb) {
                const int chl = 8 * (n >> 2) + 4 * cb + (n & 3);
                wa[st][cb] = __builtin_bit_cast(v8bf, *reinterpret_cast<const uint4 *>(S.w2 + (32 * hh + chl) * 512 + st * 32 + kg * 8));
            }
        fill_slots();
        sync_lds();   // the slot table is complete
        if (wave == 4) publish_draws();   // the consumers wait for the first image anyway
        run_consumer(S, lo, hi, ring, wa, lane, ph, hh);
    } else {
        StripOff O;
#pragma unroll
        for (int i = 0; i < 7; ++i) {
            const int t = lane + 64 * i;
            O.off[i] = t < c1::CHUNKS ? (t / (c1::CHUNKS / 4)) * c1::FR + (t % (c1::CHUNKS / 4)) * 16 : 0;
        }
        fill_slots();
        sync_lds();   // the slot table is complete
        StripRaw R;
        if (wave < UNITS * ns) c1::strip_load(R, S.src, lo + wave / UNITS, S.src.idx ? slots[wave / UNITS] : 0, wave % UNITS, lane, O);
        run_producer(S, lo, hi, reinterpret_cast<bf16_t *>(lds) + wave * STRIP, ring, slots, R, O, lane, wave);
    }
}
}  // namespace c12

// ===========================================================================
// Input gradient of conv2, one sample per workgroup (Section 2.1 network, backward pass of the
// Section 2.2 loss).  dX[pixel][ci] = sum over taps and co of dY[position][co] W[co][tap][ci]:
// the reduction runs over (tap, co), so the weights are needed with co as the reduction index and
// ci as the block row.  They are fetched once per workgroup in their natural [co][tap][ci] layout,
// passed through LDS in two halves of 32 output channels, and read back with the transposing LDS
// load (ds_read_tr16_b64) straight into a-operand registers, where they stay for all samples.
//
// A sample's dY image sits in LDS at a 144-byte pixel pitch inside a border of zeros (written
// once), so taps that fall outside the image read zeros: no bounds test, and every b-operand is a
// single 16-byte read at a per-lane base + immediate offset.  The next sample's dY is in flight
// while the current one is multiplied.  The ReLU mask is the stored activation at the result's
// own place (16 bytes per lane per block, prefetched); the lane's 8 results are 8 consecutive
// channels, stored as 16 bytes.
//
// The kernel is 4x4 with stride 2, so the 20x20 input pixels fall into four stride-parity classes
// (y%2, x%2); a pixel of class (py, px) is reached by the four taps (py + 2ty, px + 2tx) only.
// Wave = class: 100 pixels = 7 position blocks, 4 taps x 64 co = 8 reduction steps, 64 weight
// registers.  (The same scheme for the 3x3 stride-1 layer needs 144 weight registers per wave; it
// is faster alone but leaves no room for the kernels that run beside it, and is not used.)
// ===========================================================================
namespace dps {
using ps::u32x4;
constexpr int PIX = 144;             // LDS bytes per dY pixel (128 + 16)
constexpr int IMG = 11 * 11 * PIX;   // the 9x9 image inside a border of one zero pixel

struct Args {
    const bf16_t *dy;    // [B][positions out][64]
    const bf16_t *w;     // [64][taps][channels in]
    const bf16_t *xact;  // [B][pixels in][channels in], the layer input after ReLU
    bf16_t *dx;          // [B][pixels in][channels in]
    int B;
};

// a-operand of v_mfma_f32_16x16x32_bf16 out of a [reduction][column] tile in LDS: lane 16kg + s gets
// reduction rows 8kg .. 8kg+7 of block row s.  The 16 block rows are four runs of four consecutive
// tile columns; colbyte is the byte offset of the run that block row s belongs to.
__device__ __forceinline__ v8bf frag_tr16(const uint8_t *tile, int pitch, int lane, int colbyte)
{
    typedef __attribute__((address_space(3))) v4s *lds_v4s;
    typedef short v8s __attribute__((ext_vector_type(8)));
    const int s = lane & 15, kg = lane >> 4;
    const uint8_t *p = tile + (8 * kg + (s >> 2)) * pitch + colbyte;
    const v4s lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_v4s)(p));
    const v4s hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_v4s)(p + 4 * pitch));
    const v8s r = {lo.x, lo.y, lo.z, lo.w, hi.x, hi.y, hi.z, hi.w};
    return __builtin_bit_cast(v8bf, r);
}

// 8 results of a lane through the ReLU mask (activation bits > 0 as a signed 16-bit test) to 16 bytes
__device__ __forceinline__ uint4 masked8(const uint4 m, const v4f a0, const v4f a1)
{
    auto keep = [](uint32_t w2, int hi, float v) { return (int16_t)(hi ? (w2 >> 16) : (w2 & 0xFFFFu)) > 0 ? v : 0.f; };
    const uint2 lo = pack4(keep(m.x, 0, a0.x), keep(m.x, 1, a0.y), keep(m.y, 0, a0.z), keep(m.y, 1, a0.w));
    const uint2 hi = pack4(keep(m.z, 0, a1.x), keep(m.z, 1, a1.y), keep(m.w, 0, a1.z), keep(m.w, 1, a1.w));
    return uint4{lo.x, lo.y, hi.x, hi.y};
}

constexpr int W2PITCH = 512 * 2 + 16;   // LDS bytes per conv2 weight row in transit (one co: 16 taps x 32 ci)

// dy [B][81][64], w [64][4][4][32], xact and dx [B][400][32]; workgroup `bid` of `nblocks`
__device__ __forceinline__ void conv2_dgrad_ps_body(const Args &A, int bid, int nblocks, uint8_t *lds)
{
    uint8_t *img = lds, *wt = lds + IMG;
    const int tid = threadIdx.x, lane = tid & 63, n = lane & 15, kg = lane >> 4;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6), py = wave >> 1, px = wave & 1;
    const int g0 = (int)((long)bid * A.B / nblocks), g1 = (int)((long)(bid + 1) * A.B / nblocks);
    if (g0 >= g1) return;
    // a sample's dY is 648 pieces of 16 bytes; the first sample's is on its way while the weights pass through
    u32x4 r0, r1, r2;
    auto load_dy = [&](int g) {
        const u32x4 *p = reinterpret_cast<const u32x4 *>(A.dy + (long)g * (81 * 64));
        r0 = p[tid]; r1 = p[tid + 256]; r2 = p[tid < 136 ? tid + 512 : 647];
    };
    load_dy(g0);
    for (int i = tid; i < IMG / 16; i += 256) *reinterpret_cast<u32x4 *>(img + i * 16) = u32x4{0, 0, 0, 0};
    // wa[2 tap + co half][ci block], tap = 2ty + tx = kernel element (py + 2ty, px + 2tx); block row s of ci
    // block cb is input channel 8(s/4) + 4cb + s%4, so a lane's 8 results are 8 consecutive channels
    v8bf wa[8][2];
    for (int half = 0; half < 2; ++half) {
        const u32x4 *src = reinterpret_cast<const u32x4 *>(A.w + half * 32 * 512);
        sync_lds();
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const int c = tid + 256 * i;   // row (co) c / 64, 16-byte piece c % 64
            *reinterpret_cast<u32x4 *>(wt + (c >> 6) * W2PITCH + (c & 63) * 16) = src[c];
        }
        sync_lds();
#pragma unroll
        for (int tap = 0; tap < 4; ++tap)
#pragma unroll
            for (int cb = 0; cb < 2; ++cb) {
                const int ky = py + 2 * (tap >> 1), kx = px + 2 * (tap & 1);
                const int col = (ky * 4 + kx) * 32 + 8 * (n & 3) + 4 * cb;
                wa[2 * tap + half][cb] = frag_tr16(wt, W2PITCH, lane, col * 2);
            }
    }
    // pixel (2a + py, 2b + px) takes dY positions (a - ty, b - tx); image pixel (a - ty + 1, b - tx + 1) holds them.
    // base = the (ty, tx) = (1, 1) corner, i.e. image pixel (a, b)
    uint32_t base[7];
    int pos[7];
#pragma unroll
    for (int b = 0; b < 7; ++b) {
        int p = 16 * b + n;
        pos[b] = p;
        if (p > 99) p = 99;
        base[b] = ((p / 10) * 11 + (p % 10)) * PIX + kg * 16;
    }
    for (int g = g0; g < g1; ++g) {
        sync_lds();   // the previous sample's image (and, the first time, the weights in transit) has been read
#define DPS_ST(I, V) { const int t = tid + 256 * I; const int q = t >> 3; *reinterpret_cast<u32x4 *>(img + ((q / 9 + 1) * 11 + q % 9 + 1) * PIX + (t & 7) * 16) = V; }
        DPS_ST(0, r0) DPS_ST(1, r1)
        if (tid < 136) DPS_ST(2, r2)
#undef DPS_ST
        if (g + 1 < g1) load_dy(g + 1);
        const long obase = (long)g * (400 * 32) + 8 * kg;
        uint4 mk[7];
#pragma unroll
        for (int b = 0; b < 7; ++b) {
            const int p = pos[b] > 99 ? 99 : pos[b];
            const int y = 2 * (p / 10) + py, x = 2 * (p % 10) + px;
            mk[b] = *reinterpret_cast<const uint4 *>(A.xact + obase + (y * 20 + x) * 32);
        }
        sync_lds();
#pragma unroll
        for (int b = 0; b < 7; ++b) {
            v4f acc0 = {0, 0, 0, 0}, acc1 = {0, 0, 0, 0};
#pragma unroll
            for (int st = 0; st < 8; ++st) {
                const int tap = st >> 1, ty = tap >> 1, tx = tap & 1;
                const int off = ((1 - ty) * 11 + (1 - tx)) * PIX + (st & 1) * 64;
                const v8bf bb = __builtin_bit_cast(v8bf, *reinterpret_cast<const uint4 *>(img + base[b] + off));
                acc0 = mfma16(wa[st][0], bb, acc0);
                acc1 = mfma16(wa[st][1], bb, acc1);
            }
            if (pos[b] < 100) {
                const int p = pos[b];
                const int y = 2 * (p / 10) + py, x = 2 * (p % 10) + px;
                *reinterpret_cast<uint4 *>(A.dx + obase + (y * 20 + x) * 32) = masked8(mk[b], acc0, acc1);
            }
        }
    }
}
constexpr int PS_LDS = IMG + 32 * W2PITCH;   // bytes

// conv2's input gradient AND conv1's weight gradient of a sample in one workgroup (Section 2.1 network,
// backward pass of the Section 2.2 loss): conv1's dY is needed by nothing but conv1's weight gradient,
// sample by sample, so the workgroup that forms it keeps it in LDS, in the layout the weight gradient
// stages it in, and goes on to the weight gradient of the same sample (c1::conv1_wgrad_block's loop,
// both channel pairs one after the other, the frames read from the ring or the explicit states while
// the input gradient is computed).  conv1's dY is never written to memory, and the launch of conv1's
// weight gradient, with its hand-over, is gone.  Workgroup b takes samples b, b + nblocks, ... and
// writes ONE partial of conv1's weight gradient: the same samples in the same order as split b of
// c1::k_conv1_wgrad with nblocks splits, so the partials have the same bits.
struct FusedArgs {
    Args d;           // dx is not used
    c1::Src src;      // where the frames of sample n come from
    float *part1;     // [nblocks][32*256 + 32]
    const bf16_t *w2t;  // conv2's weights as [tap][channel in][channel out]
};
constexpr int FUSED_DYS = 400 * c1::LDY1 * 2;             // 32,000 bytes: conv1's dY as the weight gradient reads it
constexpr int FUSED_XIN = 2 * c1::FR * 2;                 // 28,224 bytes: two frames as bf16
constexpr int FUSED_LDS = FUSED_DYS + FUSED_XIN + IMG;    // 77,648 bytes

__device__ __forceinline__ void conv2_dgrad_conv1_wgrad_body(const FusedArgs &F, int bid, int nblocks, uint8_t *lds)
{
    using c1::FR;
    using c1::LDY1;
    const Args &A = F.d;
    bf16_t *dys = reinterpret_cast<bf16_t *>(lds), *xin = reinterpret_cast<bf16_t *>(lds + FUSED_DYS);
    uint8_t *img = lds + FUSED_DYS + FUSED_XIN;
    const int tid = threadIdx.x, lane = tid & 63, n = lane & 15, kg = lane >> 4;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6), py = wave >> 1, px = wave & 1;
    if (bid >= A.B) return;
    u32x4 r0, r1, r2;
    auto load_dy = [&](int g) {
        const u32x4 *p = reinterpret_cast<const u32x4 *>(A.dy + (long)g * (81 * 64));
        r0 = p[tid]; r1 = p[tid + 256]; r2 = p[tid < 136 ? tid + 512 : 647];
    };
    load_dy(bid);
    int slot_g = c1::sample_slot(F.src, bid);
    for (int i = tid; i < IMG / 16; i += 256) *reinterpret_cast<u32x4 *>(img + i * 16) = u32x4{0, 0, 0, 0};
    // conv2's weights, wa[2 tap + co half][ci block] as in conv2_dgrad_ps_body, straight from the copy that
    // keeps the output channels next to each other: the eight reduction elements of a lane are 16 bytes
    v8bf wa[8][2];
#pragma unroll
    for (int tap = 0; tap < 4; ++tap)
#pragma unroll
        for (int half = 0; half < 2; ++half)
#pragma unroll
            for (int cb = 0; cb < 2; ++cb) {
                const int ky = py + 2 * (tap >> 1), kx = px + 2 * (tap & 1);
                const int ci = 8 * (n >> 2) + 4 * cb + (n & 3);
                wa[2 * tap + half][cb] = __builtin_bit_cast(
                    v8bf, *reinterpret_cast<const uint4 *>(F.w2t + (((ky * 4 + kx) * 32 + ci) * 64 + 32 * half + 8 * kg)));
            }
    // position 16b + n of the wave's parity class (block b), clamped; its dY corner in the image; its pixel
    auto pos_of = [&](int b) { const int p = 16 * b + n; return p > 99 ? 99 : p; };
    auto base_of = [&](int p) { return (uint32_t)(((p / 10) * 11 + (p % 10)) * PIX + kg * 16); };
    auto pixel_of = [&](int p) { return (2 * (p / 10) + py) * 20 + 2 * (p % 10) + px; };
    // conv1's weight gradient: this lane's share as in c1::conv1_wgrad_block (wave = block of 32 im2col columns)
    typedef __attribute__((address_space(3))) v4s *lds_v4s;
    const int li = lane & 31, h = lane >> 5, s16 = lane & 15, half = (lane >> 4) & 1;
    const int rsub = 8 * h + (s16 >> 2);
    const int kc = 32 * wave + 16 * half + 4 * (s16 & 3);
    const int xoff = (kc >> 6) * FR + ((kc >> 3) & 7) * 84 + (kc & 7);
    const bf16_t *yp = dys + rsub * LDY1 + 16 * half + 4 * (s16 & 3);
    const bf16_t *xw = xin + xoff + 4 * rsub;   // the window of output pixel rsub
    v16f acc[2] = {v16f{0}, v16f{0}}, accb = {0};
    v8bf ones;
#pragma unroll
    for (int e = 0; e < 8; ++e) ones[e] = (__bf16)1.0f;
    c1::Staged<256, 2> R, R2;   // the frames of the two channel pairs

    for (int g = bid; g < A.B; g += nblocks) {
        sync_lds();   // the previous sample's image, dY tile and frames have been read (the first time: the image is cleared)
#define DPS_ST(I, V) { const int t = tid + 256 * I; const int q = t >> 3; *reinterpret_cast<u32x4 *>(img + ((q / 9 + 1) * 11 + q % 9 + 1) * PIX + (t & 7) * 16) = V; }
        DPS_ST(0, r0) DPS_ST(1, r1)
        if (tid < 136) DPS_ST(2, r2)
#undef DPS_ST
        const int gn = g + nblocks;
        if (gn < A.B) load_dy(gn);
        const bf16_t *xg = A.xact + (long)g * (400 * 32) + 8 * kg;
        // ReLU masks two blocks ahead of their use (all seven at once would cost 28 registers)
        uint4 mk0 = *reinterpret_cast<const uint4 *>(xg + pixel_of(pos_of(0)) * 32);
        uint4 mk1 = *reinterpret_cast<const uint4 *>(xg + pixel_of(pos_of(1)) * 32);
        // the sample's four frames are on their way while the input gradient is computed
        c1::stage_load<256, 2>(R, F.src, g, slot_g, 0, tid);
        c1::stage_load<256, 2>(R2, F.src, g, slot_g, 2, tid);
        const int slot_n = gn < A.B ? c1::sample_slot(F.src, gn) : 0;
        sync_lds();
        // the operand of reduction step st + 1 (of the next block after a block's last step) is requested before
        // the matrix instructions of step st
        auto operand = [&](int b, int st) {
            const int tap = st >> 1, ty = tap >> 1, tx = tap & 1;
            const int off = ((1 - ty) * 11 + (1 - tx)) * PIX + (st & 1) * 64;
            return *reinterpret_cast<const uint4 *>(img + base_of(pos_of(b)) + off);
        };
        uint4 cur = operand(0, 0);
#pragma unroll
        for (int b = 0; b < 7; ++b) {
            const int p = pos_of(b);
            const uint4 mk = mk0;
            mk0 = mk1;
            if (b + 2 < 7) mk1 = *reinterpret_cast<const uint4 *>(xg + pixel_of(pos_of(b + 2)) * 32);
            v4f acc0 = {0, 0, 0, 0}, acc1 = {0, 0, 0, 0};
#pragma unroll
            for (int st = 0; st < 8; ++st) {
                uint4 nxt = cur;
                if (st < 7) nxt = operand(b, st + 1);
                else if (b < 6) nxt = operand(b + 1, 0);
                __builtin_amdgcn_sched_barrier(0);
                const v8bf bb = __builtin_bit_cast(v8bf, cur);
                acc0 = mfma16(wa[st][0], bb, acc0);
                acc1 = mfma16(wa[st][1], bb, acc1);
                __builtin_amdgcn_sched_barrier(0);
                cur = nxt;
            }
            if (16 * b + n < 100) *reinterpret_cast<uint4 *>(dys + pixel_of(p) * LDY1 + 8 * kg) = masked8(mk, acc0, acc1);
        }
#pragma unroll
        for (int cp = 0; cp < 2; ++cp) {
            if (cp == 1) sync_lds();   // the first pair's frames have been read
            c1::stage_store<256, 2>(xin, cp == 0 ? R : R2, tid);
            sync_lds();   // the dY tile and the pair's frames are complete
            const bool do_bias = cp == 0 && wave == 0;
            // the operands of step t + 1 are requested before the matrix instruction of step t
            auto operands = [&](int t, v8bf &fa, v8bf &fb) {   // 16 output pixels per step
                fa = frag_tr(yp + 16 * t * LDY1, LDY1);
                // see c1::conv1_wgrad_block: no division
                const int q = (16 * t) / 20, r = (16 * t) % 20;
                const bf16_t *x0 = xw + (336 * q + 4 * r) + (rsub >= 20 - r ? 256 : 0);
                const bf16_t *x1 = xw + (336 * q + 4 * r + 16) + (rsub + 4 >= 20 - r ? 256 : 0);
                v4s lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_v4s)x0);
                v4s hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_v4s)x1);
                typedef short v8s __attribute__((ext_vector_type(8)));
                v8s xb = {lo.x, lo.y, lo.z, lo.w, hi.x, hi.y, hi.z, hi.w};
                fb = __builtin_bit_cast(v8bf, xb);
            };
            v8bf fa, fb, fan, fbn;
            operands(0, fa, fb);
#pragma unroll
            for (int t = 0; t < 25; ++t) {
                fan = fa; fbn = fb;
                if (t + 1 < 25) operands(t + 1, fan, fbn);
                __builtin_amdgcn_sched_barrier(0);
                acc[cp] = mfma(fa, fb, acc[cp]);
                if (do_bias) accb = mfma(fa, ones, accb);
                __builtin_amdgcn_sched_barrier(0);
                fa = fan; fb = fbn;
            }
        }
        slot_g = slot_n;
    }

    float *part = F.part1 + (long)bid * (32 * 256 + 32);
#pragma unroll
    for (int cp = 0; cp < 2; ++cp)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const int o = 8 * (r / 4) + 4 * h + (r % 4);
            part[o * 256 + 128 * cp + 32 * wave + li] = acc[cp][r] * (1.0f / 255.0f);
            if (cp == 0 && wave == 0 && li == 0) part[32 * 256 + o] = accb[r];
        }
}
}  // namespace dps
}  // namespace gbf
