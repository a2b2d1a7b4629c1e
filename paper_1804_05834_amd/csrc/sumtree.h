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
// shuffles.  20 levels cost 3 dependent round trips instead of 20 (the round at the
// root is wider where that saves one, see first_round_levels), and every fetch is a
// contiguous run of the heap array.
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

// Draws jj[0 .. ND) by one wave at once: the fetches of a round are issued together, so ND draws cost the
// round trips of one.  Every lane returns the slots, the values of the leaves reached and (the function's
// value) the mass the draws were scaled by.  Lane 1 of the first round reads the root along with the
// subtree below it, and the leaf's value is the child chosen in the last step: neither the total nor the
// leaf costs a memory round trip of its own.
// Levels of the walk's first round.  The top of the tree is ONE contiguous run of the heap array, so a round
// that starts at the root can take 7 or 8 levels (255 / 511 nodes: four / eight loads per lane, issued
// together) where that saves the walk a dependent round trip: 19 or 20 levels in three rounds, not four.
__device__ __forceinline__ int first_round_levels(int levels)
{
    const int m = levels % 6;
    return levels > 6 && (m == 1 || m == 2) ? 6 + m : min(6, levels);
}

template <int ND>
__device__ __forceinline__ float per_sample_walk(const SampleArgs &A, const int (&jj)[ND], int lane, long (&slot)[ND],
                                                 float (&leaf)[ND])
{
    auto mass = [&](int j, float total) {
        const float u = draw_u24(A.seed, (uint64_t)j);
        return A.stratified ? __fmul_rn((float)j + u, total / (float)A.B) : __fmul_rn(u, total);
    };
    if (A.uniform) {
        // a tree whose stored leaves are all 1 holds exact integers, and its descent returns floor(z)
        const float total = sample_total(A);
#pragma unroll
        for (int d = 0; d < ND; ++d) {
            const long sl = (long)mass(jj[d], total);
            slot[d] = sl > A.limit - 1 ? A.limit - 1 : sl;
            leaf[d] = 1.f;
        }
        return total;
    }
    const float *tree = A.tree;
    float total = 0.f, z[ND];
    long node[ND];
#pragma unroll
    for (int d = 0; d < ND; ++d) { node[d] = 1; z[d] = 0.f; leaf[d] = 0.f; }
    if (A.levels == 0) {   // a tree of one leaf
        total = tree[1];
#pragma unroll
        for (int d = 0; d < ND; ++d) leaf[d] = total;
    }
    const int lj = lane >= 1 ? 31 - __clz(lane) : 0;  // level of local heap node `lane`
    int done = 0;
    const int r0 = first_round_levels(A.levels);
    if (r0 > 6) {
        // the wide first round: lane l holds nodes l, 64 + l, ... of the top 2^(r0+1) nodes; the walk is the
        // same in every lane, so each lane picks the register its own node of the wanted run sits in and
        // the exchange takes the wanted lane's
        float v[8];
#pragma unroll
        for (int q = 0; q < 8; ++q) {
            const int n = 64 * q + lane;
            v[q] = n >= 1 && n < (2 << r0) ? tree[n] : 0.f;
        }
        total = __shfl(v[0], 1, 64);
#pragma unroll
        for (int d = 0; d < ND; ++d) {
            z[d] = mass(jj[d], total);
            int cur = 1;
#pragma unroll
            for (int t = 0; t < 8; ++t) {
                if (t >= r0) continue;
                const int c = 2 * cur;  // left child, below 2^(t+1)... its run of 64 nodes: c >> 6
                float m;
                if (t < 5) m = v[0];
                else if (t == 5) m = v[1];
                else if (t == 6) m = (c & 64) ? v[3] : v[2];
                else m = (c & 128) ? ((c & 64) ? v[7] : v[6]) : ((c & 64) ? v[5] : v[4]);
                const float left = __shfl(m, c & 63, 64), right = __shfl(m, (c & 63) + 1, 64);
                if (z[d] < left || right == 0.f) {
                    cur = c;
                    leaf[d] = left;
                } else {
                    z[d] = z[d] - left;
                    cur = c + 1;
                    leaf[d] = right;
                }
            }
            node[d] = cur;
        }
        done = r0;
    }
    while (done < A.levels) {
        const int r = min(6, A.levels - done);  // levels walked in this round
        float va[ND], vb[ND];
#pragma unroll
        for (int d = 0; d < ND; ++d) {
            va[d] = vb[d] = 0.f;
            if (lane >= (done ? 2 : 1) && lane < (2 << min(r, 5))) va[d] = tree[(node[d] << lj) + (lane - (1 << lj))];
            if (r == 6) vb[d] = tree[(node[d] << 6) + lane];
        }
        if (done == 0) {
            total = __shfl(va[0], 1, 64);
#pragma unroll
            for (int d = 0; d < ND; ++d) z[d] = mass(jj[d], total);
        }
#pragma unroll
        for (int d = 0; d < ND; ++d) {
            int cur = 1;  // local heap index
            for (int t = 0; t < r; ++t) {
                const int c = 2 * cur;  // left child
                const float left = c < 64 ? __shfl(va[d], c, 64) : __shfl(vb[d], c - 64, 64);
                const float right = c < 64 ? __shfl(va[d], c + 1, 64) : __shfl(vb[d], c - 63, 64);
                if (z[d] < left || right == 0.f) {   // nothing on the right: a zero leaf is never drawn
                    cur = c;
                    leaf[d] = left;
                } else {
                    z[d] = z[d] - left;
                    cur = c + 1;
                    leaf[d] = right;
                }
            }
            node[d] = (node[d] << r) + (cur - (1 << r));
        }
        done += r;
    }
#pragma unroll
    for (int d = 0; d < ND; ++d) {
        slot[d] = node[d] - A.L;
        if (slot[d] > A.limit - 1) {   // not reached while the tree has mass: slots past the limit hold zero leaves
            slot[d] = A.limit - 1;
            leaf[d] = tree[A.L + slot[d]];
        }
    }
    return total;
}

// What one lane writes for draw j once the walk has ended: index, raw weight (from the leaf's value and
// the total the walk returned), transition data.
__device__ __forceinline__ void per_sample_emit(const SampleArgs &A, int j, long slot, float total, float leaf)
{
    A.idx[j] = (int32_t)slot;
    if (A.uniform) {
        A.is_w[j] = 1.f;   // (N * 1/N)^-beta
    } else {
        const double P = (double)leaf / (double)total;
        // a tree without mass (every stored transition has priority zero) has nothing to draw: weight 0
        A.is_w[j] = total > 0.f ? (float)pow((double)A.size * P, -(double)A.beta) : 0.f;
    }
    if (A.G.a) {   // the three loads first: behind a store the compiler would hold a load back
        const int32_t a = A.G.meta_a[slot];
        const float r = A.G.meta_r[slot];
        const uint8_t d = A.G.meta_done[slot];
        A.G.a[j] = a;
        A.G.r[j] = r;
        A.G.done[j] = d;
    }
}

}  // namespace misc
