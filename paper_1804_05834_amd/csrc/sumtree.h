// Counter-based draws and proportional sampling from the sum-tree (Eq.10, Eq.12): the device
// functions shared by the sampling kernel, the fused sample-and-gather kernel and the conv1
// kernel that draws its own transitions.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace misc {

// ----------------------------------------------------------------- draws
// 64-bit counter mixer (SplitMix64 output function on seed + (ctr+1)*gamma);
// a uniform in [0,1) is its top 24 bits times 2^-24.
__host__ __device__ __forceinline__ uint64_t mix64(uint64_t seed, uint64_t ctr)
{
    uint64_t z = seed + (ctr + 1ull) * 0x9E3779B97F4A7C15ull;
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    return z ^ (z >> 31);
}
__host__ __device__ __forceinline__ float draw_u24(uint64_t seed, uint64_t ctr)
{
    return (float)(mix64(seed, ctr) >> 40) * (1.0f / 16777216.0f);
}

// Optional per-slot transition data to carry along with the draw.
struct MetaGather {
    const int32_t *meta_a;
    const float *meta_r;
    const uint8_t *meta_done;
    int32_t *a;
    float *r;
    uint8_t *done;
};

// Proportional sampling (Eq.10, Eq.12), one WAVE per draw.  The descent is the
// sequential rule "z < left ? go left : (z -= left, go right)" in fp32, except that it also
// turns left when the right child is 0: a parent is the ROUNDED sum of its children, so a mass
// below the parent can still overshoot the right child, and the walk would end on a leaf of
// value 0, a slot that holds no drawable transition (Eq.10 gives it probability zero; its
// importance weight would be infinite).  With a positive total every node visited is positive.
// The memory side is batched: at a node x the wave fetches the whole 6-level subtree
// below x in one round trip (lane l reads local heap node l of levels 1..5 and
// node l of level 6), then walks those 6 levels out of registers with lane
// shuffles.  20 levels cost 4 dependent round trips instead of 20, and every
// fetch is a contiguous run of the heap array.
// is_w receives the RAW weight (N P(j))^-beta; k_per_normalise (or the consumer)
// divides by the minibatch maximum.
struct SampleArgs {
    const float *tree;
    long L;
    int levels;
    long size;
    int B;
    float beta;
    uint64_t seed;
    int stratified;
    int32_t *idx;
    float *is_w;
    MetaGather G;
    int uniform;   // 1: every stored slot has leaf 1 (priority exponent 0, tree built by a bulk fill): no tree reads
    long limit;    // slots that may hold a transition are [0, limit): `size` for one stream; with many
                   // environment streams the stored transitions are not the first `size` slots
};

// The mass the draws are scaled by: the root of the tree; in uniform mode the number of stored slots
// (the root of a tree of ones), without a memory access.
__device__ __forceinline__ float sample_total(const SampleArgs &A) { return A.uniform ? (float)A.size : A.tree[1]; }

// Draw j by one wave; every lane returns the slot.
__device__ __forceinline__ long per_sample_descend(const SampleArgs &A, int j, int lane, float total)
{
    const float *tree = A.tree;
    const float u = draw_u24(A.seed, (uint64_t)j);
    float z = A.stratified ? __fmul_rn((float)j + u, total / (float)A.B) : __fmul_rn(u, total);
    if (A.uniform) {
        // a tree whose stored leaves are all 1 holds exact integers, and its descent returns floor(z)
        long slot = (long)z;
        return slot > A.limit - 1 ? A.limit - 1 : slot;
    }
    long node = 1;
    const int lj = lane >= 2 ? 31 - __clz(lane) : 0;  // level of local heap node `lane`
    for (int done = 0; done < A.levels;) {
        const int r = min(6, A.levels - done);  // levels walked in this round
        float va = 0.f, vb = 0.f;
        if (lane >= 2 && lane < (2 << min(r, 5))) va = tree[(node << lj) + (lane - (1 << lj))];
        if (r == 6) vb = tree[(node << 6) + lane];
        int cur = 1;  // local heap index
        for (int t = 0; t < r; ++t) {
            const int c = 2 * cur;  // left child
            const float left = c < 64 ? __shfl(va, c, 64) : __shfl(vb, c - 64, 64);
            const float right = c < 64 ? __shfl(va, c + 1, 64) : __shfl(vb, c - 63, 64);
            if (z < left || right == 0.f) {   // nothing on the right: a zero leaf is never drawn
                cur = c;
            } else {
                z = z - left;
                cur = c + 1;
            }
        }
        node = (node << r) + (cur - (1 << r));
        done += r;
    }
    long slot = node - A.L;
    if (slot > A.limit - 1) slot = A.limit - 1;
    return slot;
}

// Draws j0 and j1 by one wave at once: the same walk as above for each, with the two fetches of a
// round issued together, so the pair costs the four round trips of one.
__device__ __forceinline__ void per_sample_descend2(const SampleArgs &A, int j0, int j1, int lane, float total,
                                                    long &slot0, long &slot1)
{
    const float *tree = A.tree;
    const int jj[2] = {j0, j1};
    float z[2];
    long node[2] = {1, 1};
#pragma unroll
    for (int d = 0; d < 2; ++d) {
        const float u = draw_u24(A.seed, (uint64_t)jj[d]);
        z[d] = A.stratified ? __fmul_rn((float)jj[d] + u, total / (float)A.B) : __fmul_rn(u, total);
    }
    if (A.uniform) {
        slot0 = (long)z[0];
        slot1 = (long)z[1];
        if (slot0 > A.limit - 1) slot0 = A.limit - 1;
        if (slot1 > A.limit - 1) slot1 = A.limit - 1;
        return;
    }
    const int lj = lane >= 2 ? 31 - __clz(lane) : 0;
    for (int done = 0; done < A.levels;) {
        const int r = min(6, A.levels - done);
        float va[2] = {0.f, 0.f}, vb[2] = {0.f, 0.f};
#pragma unroll
        for (int d = 0; d < 2; ++d) {
            if (lane >= 2 && lane < (2 << min(r, 5))) va[d] = tree[(node[d] << lj) + (lane - (1 << lj))];
            if (r == 6) vb[d] = tree[(node[d] << 6) + lane];
        }
#pragma unroll
        for (int d = 0; d < 2; ++d) {
            int cur = 1;
            for (int t = 0; t < r; ++t) {
                const int c = 2 * cur;
                const float left = c < 64 ? __shfl(va[d], c, 64) : __shfl(vb[d], c - 64, 64);
                const float right = c < 64 ? __shfl(va[d], c + 1, 64) : __shfl(vb[d], c - 63, 64);
                if (z[d] < left || right == 0.f) {
                    cur = c;
                } else {
                    z[d] = z[d] - left;
                    cur = c + 1;
                }
            }
            node[d] = (node[d] << r) + (cur - (1 << r));
        }
        done += r;
    }
    slot0 = node[0] - A.L;
    slot1 = node[1] - A.L;
    if (slot0 > A.limit - 1) slot0 = A.limit - 1;
    if (slot1 > A.limit - 1) slot1 = A.limit - 1;
}

// What one lane writes for draw j once the slot is known: index, raw weight, transition data.
__device__ __forceinline__ void per_sample_emit(const SampleArgs &A, int j, long slot, float total)
{
    A.idx[j] = (int32_t)slot;
    if (A.uniform) {
        A.is_w[j] = 1.f;   // (N * 1/N)^-beta
    } else {
        const double P = (double)A.tree[A.L + slot] / (double)total;
        // a tree without mass (every stored transition has priority zero) has nothing to draw: weight 0
        A.is_w[j] = total > 0.f ? (float)pow((double)A.size * P, -(double)A.beta) : 0.f;
    }
    if (A.G.a) {
        A.G.a[j] = A.G.meta_a[slot];
        A.G.r[j] = A.G.meta_r[slot];
        A.G.done[j] = A.G.meta_done[slot];
    }
}

}  // namespace misc
