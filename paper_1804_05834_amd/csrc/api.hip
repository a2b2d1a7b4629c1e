// C ABI of libdqn (see include/dqn.h): host-side bookkeeping, workspace layout
// and the launch schedule of the training step.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cmath>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <new>
#include <string>
#include <vector>

#include "../../include/dqn.h"
#include "gemm_bf16.h"
#include "gemm_fp32.h"
#include "kernels_misc.h"
#include "net.h"

// Scratch memory of dqn_act_static, the entry point for callers that cannot allocate: activations and
// fc1 partial sums of up to DQN_ACT_STATIC_MAX observations.  Each GPU the library runs on holds its own
// copy of this array, at its own address, until the process ends.  In host code the array's name is
// only a stand-in for the symbol; the device address is looked up once per device (below).
constexpr size_t SCRATCH_BYTES = 4u << 20;
static __device__ __align__(256) uint8_t scratch[SCRATCH_BYTES];

namespace {

thread_local std::string g_err;  // errors without a context

constexpr int MAX_DEVICES = 64;
uint8_t *g_scratch_ptr[MAX_DEVICES];   // device address of `scratch` on each device, once looked up

// The address of `scratch` on the current device (looked up on first use on that device, with that
// device current; no allocation), or nullptr.
uint8_t *scratch_of_current_device()
{
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= MAX_DEVICES) return nullptr;
    if (!g_scratch_ptr[dev]) {
        void *p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess) {
            (void)hipGetLastError();
            return nullptr;
        }
        g_scratch_ptr[dev] = static_cast<uint8_t *>(p);
    }
    return g_scratch_ptr[dev];
}

constexpr int MAX_WSPLIT = 64;   // most reduction splits of a conv2/conv3 weight gradient
constexpr int MAX_WSPLIT1 = 256; // ... of the conv1 weight gradient (one output tile only)

struct Workspace {
    // minibatch staging (replay mode)
    uint8_t *stack5;
    int32_t *b_idx, *b_a;
    float *b_w, *b_r, *td_abs, *loss_j, *qmax_j, *loss_slot;
    int *pu_state;   // walkers of a priority update that is split over two launches
    gbf::bf16_t *w2t;  // bf16 only: the online conv2 weights as [tap][channel in][channel out] (see misc::k_w2_transposed)
    uint8_t *b_done;
    // activations, channel-last, rows = samples of all passes (fp32 or bf16 by precision)
    void *act1, *act2, *act3;
    float *f1part, *h_s;
    size_t f1rows;   // rows of 512 partial sums that f1part holds (rows of a launch x reduction splits)
    // backward (dh, d3, d2, d1: fp32 or bf16 by precision)
    float *dA;
    void *dh, *d3, *d2, *d1;
    // gradient partial sums per layer, [split][W..., b...]
    float *gp1, *gp2, *gp3;
    // step outputs staged here when the step is replayed from a recording
    float *o_loss, *o_q, *o_y, *o_td, *o_isw;  // o_q: [3][max_batch][K]
    int32_t *o_astar;
    size_t total;
};

size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

constexpr size_t MAX_STEP_GRAPHS = 16;  // recorded steps kept per context (one per batch size)

// reduction splits of the fc1 forward GEMM (3136 = 98*32 = 49*64 reduction elements)
int fc1_splits(long M, int precision)
{
    if (precision == 1) return M <= 2048 ? 7 : 1;
    return M <= 512 ? 7 : M <= 1536 ? 2 : 1;
}

Workspace carve(const dqn_config &c, uint8_t *base)
{
    Workspace w{};
    size_t off = 0;
    auto take = [&](size_t bytes) {
        uint8_t *p = base ? base + off : nullptr;
        off += align_up(bytes, 256);
        return p;
    };
    const size_t MB = (size_t)c.max_batch;
    const size_t rows = std::max<size_t>(3 * MB, (size_t)c.max_act_batch);
    const size_t R = (size_t)c.num_actions + (c.dueling ? 1 : 0);
    w.stack5 = take(MB * 5 * net::FRAME);
    w.b_idx = (int32_t *)take(MB * 4);
    w.b_a = (int32_t *)take(MB * 4);
    w.b_w = (float *)take(MB * 4);
    w.b_r = (float *)take(MB * 4);
    w.td_abs = (float *)take(MB * 4);
    w.loss_j = (float *)take(MB * 4);
    w.qmax_j = (float *)take(MB * 4);
    w.loss_slot = (float *)take(256);
    w.pu_state = (int *)take(3 * misc::STATE_STRIDE * 4);
    w.w2t = (gbf::bf16_t *)take(c.precision == 1 ? net::L2N * 2 : 0);
    w.b_done = take(MB);
    const size_t es = c.precision == 1 ? 2 : 4;  // bytes per activation element
    w.act1 = take(rows * net::A1 * es);
    w.act2 = take(rows * net::A2 * es);
    w.act3 = take(rows * net::A3 * es);
    size_t f1rows = std::max({std::min<size_t>(rows, 192) * 14, std::min<size_t>(rows, 512) * 7,
                              std::min<size_t>(rows, 1536) * 2, rows});
    if (c.precision == 1) f1rows = std::max(f1rows, std::min<size_t>(rows, 2048) * 7);
    w.f1part = (float *)take(f1rows * net::HID * 4);
    w.f1rows = f1rows;
    w.h_s = (float *)take(MB * net::HID * 4);
    w.dA = (float *)take(MB * R * 4);
    w.dh = take(MB * net::HID * es);
    w.d3 = take(MB * net::A3 * es);
    w.d2 = take(MB * net::A2 * es);
    w.d1 = take(MB * net::A1 * es);
    w.gp1 = (float *)take((size_t)MAX_WSPLIT1 * net::L1N * 4);
    w.gp2 = (float *)take((size_t)MAX_WSPLIT * net::L2N * 4);
    w.gp3 = (float *)take((size_t)MAX_WSPLIT * net::L3N * 4);
    w.o_loss = (float *)take(256);
    w.o_q = (float *)take(3 * MB * (size_t)c.num_actions * 4);
    w.o_y = (float *)take(MB * 4);
    w.o_td = (float *)take(MB * 4);
    w.o_isw = (float *)take(MB * 4);
    w.o_astar = (int32_t *)take(MB * 4);
    w.total = off;
    return w;
}

struct ProfRec {
    const char *name;
    hipEvent_t e0, e1;
};

}  // namespace

struct dqn_ctx {
    dqn_config cfg;
    dqn_buffers buf;
    dqn_sizes sz;
    Workspace ws;
    int64_t n;       // parameters per network
    int R;           // head rows
    long L;          // tree leaves (power of two)
    int levels;      // log2(L)
    long stored;     // transitions with a priority
    float *theta, *theta_t, *rms_v, *rms_m, *grads;
    int32_t *meta_a;
    float *meta_r;
    uint8_t *meta_done;
    float *tree;
    // side stream: kernels off the critical chain (weight gradients, priority update) overlap
    // the input-gradient chain of the backward pass
    int num_cu = 256;  // compute units of the device
    // bf16: conv1 + conv2 forward run as one launch (gbf::c12) from this many samples per launch on;
    // INT_MAX: never (the launch needs 140 KB of LDS per workgroup, granted at initialisation)
    int conv12_min = INT32_MAX;
    // bf16: fc1 forward as 128 x 128 tiles (gbf::f1) from this many rows per launch on; needs 72 KB of LDS
    float *gp4 = nullptr, *gp5 = nullptr;   // where fc1's and the head's weight gradients are written: inside `grads`
    bool fused_bwd = false;   // conv2's input gradient and conv1's weight gradient in one workgroup per sample
    bool fc1_big = false;
    int fc1_big_rows = 512, fc1_big_splits = 0;
    hipStream_t side = nullptr;
    hipStream_t side2 = nullptr;  // the single-workgroup priority update gets a lane of its own
    hipEvent_t ev_fork = nullptr, ev_a = nullptr, ev_b = nullptr, ev_c = nullptr, ev_join = nullptr, ev_join2 = nullptr;
    // Uniform replay (priority exponent 0, the "without prioritized replay" settings of Sec.4) over a tree
    // that a bulk fill built: every stored leaf is 1 and stays 1, the descent returns floor(z) and every
    // importance weight is 1, so sampling reads no tree node and the priority update writes none.  The store
    // path gives leaf 0 to slots that hold no whole transition: after it the tree is walked again.
    bool leaves_all_one = false;
    // The ring as sub-rings: one environment stream (sub = capacity) or, after dqn_replay_store_envs, `envs`
    // streams of `sub` slots each.  slot_limit: slots that may hold a transition are [0, slot_limit).
    int envs = 0;
    long sub = 0, slot_limit = 0;
    int64_t cursor = 0;  // next ring slot of the store path
    int64_t seq = 0;     // time steps stored so far (stream position of the next one)
    bool prof = false;
    std::vector<ProfRec> recs;
    std::string err;
    // Optional: the replay-mode training step (everything after the sampling kernel, whose
    // arguments change every step) is recorded once per batch size into a HIP graph and replayed.
    // Recording happens on `cap`, so the caller may pass the legacy default stream, which
    // cannot be captured.  Recordings live until dqn_destroy.
    hipStream_t cap = nullptr;
    bool graph_off = true;   // cleared by DQN_GRAPH=1; set again after a failed recording
    struct StepGraph {
        int32_t B;
        hipGraph_t graph;
        hipGraphExec_t exec;
    };
    std::vector<StepGraph> graphs;
};

namespace {

int32_t fail(dqn_ctx *c, int32_t code, const std::string &msg)
{
    if (c) c->err = msg;
    else g_err = msg;
    return code;
}

bool aligned(const void *p, size_t a) { return ((uintptr_t)p % a) == 0; }

void drop_graphs(dqn_ctx *c)
{
    for (dqn_ctx::StepGraph &g : c->graphs) {
        if (g.exec) (void)hipGraphExecDestroy(g.exec);
        if (g.graph) (void)hipGraphDestroy(g.graph);
    }
    c->graphs.clear();
}

const char *check_config(const dqn_config &c)
{
    if (c.num_actions < 1 || c.num_actions > 64) return "num_actions must be in 1..64";
    if (c.dueling < 0 || c.dueling > 1 || c.double_q < 0 || c.double_q > 1) return "dueling/double_q must be 0 or 1";
    if (c.precision < 0 || c.precision > 1) return "precision must be 0 (fp32) or 1 (bf16)";
    if (c.loss_kind < 0 || c.loss_kind > 1) return "loss_kind must be 0 or 1";
    if (!(c.huber_delta > 0.f)) return "huber_delta must be > 0";
    if (!(c.gamma >= 0.f && c.gamma <= 1.f)) return "gamma must be in [0,1]";
    if (!(c.lr >= 0.f) || !(c.rms_decay >= 0.f && c.rms_decay < 1.f) || !(c.rms_eps > 0.f))
        return "lr >= 0, 0 <= rms_decay < 1, rms_eps > 0 required";
    if (c.rms_centered < 0 || c.rms_centered > 1) return "rms_centered must be 0 or 1";
    if (c.max_batch < 1 || c.max_batch > 1024) return "max_batch must be in 1..1024";
    if (c.max_act_batch < 1 || c.max_act_batch > 8192) return "max_act_batch must be in 1..8192";
    if (c.per_stratified < 0 || c.per_stratified > 1) return "per_stratified must be 0 or 1";
    if (c.replay_capacity < 0 || c.replay_capacity > (1ll << 30)) return "replay_capacity out of range";
    if (c.replay_capacity > 0 && c.replay_capacity < 5) return "replay_capacity must be 0 or >= 5";
    if (c.replay_capacity > 0 && (!(c.per_alpha >= 0.f) || !(c.per_eps > 0.f))) return "per_alpha >= 0 and per_eps > 0 required";
    return nullptr;
}

long tree_leaves(int64_t cap)
{
    long L = 1;
    while (L < cap) L <<= 1;
    return L;
}

template <class F>
void launch(dqn_ctx *c, const char *name, hipStream_t st, F &&f)
{
    if (c->prof) {
        ProfRec r{name, nullptr, nullptr};
        if (hipEventCreate(&r.e0) == hipSuccess && hipEventCreate(&r.e1) == hipSuccess) {
            (void)hipEventRecord(r.e0, st);
            f();
            (void)hipEventRecord(r.e1, st);
            c->recs.push_back(r);
            return;
        }
    }
    f();
}

// Every internal node of the sum-tree from its leaves, twelve levels per launch.
void rebuild_tree(dqn_ctx *c, hipStream_t st)
{
    for (long Lcur = c->L; Lcur >= 2; Lcur >>= 12) {
        const int BL = (int)std::min<long>(Lcur, 4096);
        launch(c, "tree_rebuild", st, [&] { misc::k_tree_rebuild<<<dim3((unsigned)(Lcur / BL)), 256, 0, st>>>(c->tree, Lcur, BL); });
        if (Lcur <= 4096) break;
    }
}

int uniform_replay(const dqn_ctx *c)
{
    const char *off = std::getenv("DQN_NO_UNIFORM_FAST_PATH");   // for A/B measurements
    return c->leaves_all_one && !(off && off[0] == '1') ? 1 : 0;
}

int32_t hip_status(dqn_ctx *c, const char *where)
{
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return fail(c, DQN_ERR_HIP, std::string(where) + ": " + hipGetErrorString(e));
    return DQN_OK;
}

dim3 grid1(long n, int block) { return dim3((unsigned)((n + block - 1) / block)); }

// ----- host-side initial weights: uniform in +-sqrt(6/fan_in), biases 0 -----
void he_uniform_host(std::vector<float> &blob, int K, int dueling, uint64_t seed)
{
    struct T { int64_t count; int fan_in; };
    std::vector<T> spec = {{8192, 256}, {32, 0}, {32768, 512}, {64, 0}, {36864, 576}, {64, 0},
                           {1605632, 3136}, {512, 0}};
    if (dueling) { spec.push_back({512, 512}); spec.push_back({1, 0}); }
    spec.push_back({(int64_t)K * 512, 512});
    spec.push_back({K, 0});
    int64_t e = 0;
    for (const T &t : spec) {
        float bound = t.fan_in ? (float)std::sqrt(6.0 / (double)t.fan_in) : 0.f;
        for (int64_t i = 0; i < t.count; ++i, ++e) {
            float centred = 2.0f * misc::draw_u24(seed, (uint64_t)e) - 1.0f;
            blob[(size_t)e] = t.fan_in ? centred * bound : 0.f;
        }
    }
}

void permute(dqn_ctx *c, const float *src, float *dst, int dir, hipStream_t st)
{
    launch(c, "permute", st, [&] { misc::k_permute<<<grid1(c->n, 256), 256, 0, st>>>(src, dst, c->n, dir); });
}

float *which_buffer(dqn_ctx *c, int which)
{
    switch (which) {
    case 0: return c->theta;
    case 1: return c->theta_t;
    case 2: return c->grads;
    case 3: return c->rms_v;
    case 4: return c->rms_m;
    default: return nullptr;
    }
}

// ----- forward of up to three passes through conv1..fc1 -----
struct Pass {
    const uint8_t *x;    // uint8 states, or the replay ring when idx is set
    long xs;             // bytes between samples (states)
    int net;             // 0 online / 1 target parameters
    int n;               // samples
    const int32_t *idx;  // ring mode: sampled slots (or where the forward kernel leaves them); frames are read from the ring
    int shift;           // ring mode: 0 = s (frames i-3..i), 1 = s' (frames i-2..i+1)
    uint8_t *stack;      // fp32 ring mode: where conv1 leaves a gathered copy of the frames for the weight gradient
    int stack_mode;      // 1: frames 0-3 of the sample to stack frames 0-3; 2: frame 3 to stack frame 4
};

const float *theta_of(dqn_ctx *c, int net) { return net ? c->theta_t : c->theta; }
const gbf::bf16_t *shadow_of(dqn_ctx *c, int net)
{
    const gbf::bf16_t *sh = (const gbf::bf16_t *)c->buf.shadow_bf16;
    return sh + (net ? align_up((size_t)c->n * 2, 256) / 2 : 0);
}

// Launch shapes of the conv1 forward kernels for `samples` samples (all passes), and whether a wave's
// (wave group's) share of strips spans few enough samples for it to draw them itself.
struct Conv1Plan {
    bool ks2;        // fp32: four waves per strip (fewer wave pairs than SIMDs)
    int grid;
    bool draw_fits;
};
Conv1Plan conv1_plan_f32(int samples, int num_cu)
{
    const int units = samples * gbf::c1::UNITS;
    Conv1Plan P;
    P.ks2 = 2 * units <= 4 * num_cu;
    P.grid = P.ks2 ? std::min(units, 2 * num_cu) : std::min((units + 1) / 2, 2 * num_cu);
    const int groups = P.ks2 ? P.grid : 2 * P.grid;
    const int upg = (units + groups - 1) / groups + 1;   // strips per group of waves, at most
    P.draw_fits = (upg + gbf::c1::UNITS - 1) / gbf::c1::UNITS + 1 <= gbf::c1::MAX_DRAWS;
    return P;
}
Conv1Plan conv1_plan_bf16(int samples, int num_cu)
{
    const int units = samples * gbf::c1::UNITS;
    Conv1Plan P;
    P.ks2 = false;
    // one wave per strip of a sample, four waves per workgroup, two workgroups resident per CU
    P.grid = std::min((units + 3) / 4, 2 * num_cu);
    const int upw = (units + 4 * P.grid - 1) / (4 * P.grid) + 1;
    P.draw_fits = (upw + gbf::c1::UNITS - 1) / gbf::c1::UNITS + 1 <= gbf::c1::MAX_DRAWS;
    return P;
}
// bf16: conv1 + conv2 as one launch, one workgroup per CU, for passes of n[0..npass) samples?
bool fused12_fits(const dqn_ctx *c, const int *n, int npass, bool draw)
{
    long rows = 0;
    for (int i = 0; i < npass; ++i) rows += n[i];
    if (rows < c->conv12_min || npass > c->num_cu) return false;
    const int grid12 = (int)std::min<long>(rows, c->num_cu);
    for (int i = 0; i < npass; ++i) {
        const int wgs = (int)((long)grid12 * (i + 1) / npass - (long)grid12 * i / npass);
        if (wgs < 1 || (n[i] + wgs - 1) / wgs > gbf::c12::MAX_PER_WG) return false;
        if (draw && n[i] != n[0]) return false;
    }
    return true;
}
// Can the first forward kernel of a replay-mode step of batch B draw the transitions itself?  If not
// (few compute units and a large batch), a sampling launch runs in front of the step.
bool in_kernel_draw_fits(const dqn_ctx *c, int B)
{
    if (c->cfg.precision == 0) return conv1_plan_f32(3 * B, c->num_cu).draw_fits;
    const int n[3] = {B, B, B};
    return fused12_fits(c, n, 3, true) || conv1_plan_bf16(3 * B, c->num_cu).draw_fits;
}

int32_t forward_trunk_f32(dqn_ctx *c, const Workspace &w, const Pass *pass, int npass, int *nsplit_out,
                          long *split_stride_out, hipStream_t st, const misc::SampleArgs *draw)
{
    using namespace g32;
    float *act1 = (float *)w.act1, *act2 = (float *)w.act2, *act3 = (float *)w.act3;
    long row0[3];
    long rows = 0;
    for (int i = 0; i < npass; ++i) { row0[i] = rows; rows += pass[i].n; }

    auto build = [&](FwdArgs &A, int BM, int P, auto xptr, auto xstride, int64_t woff, int64_t boff,
                     float *ybase, long ystride, bool with_bias) {
        int tile = 0;
        A.nseg = npass;
        for (int i = 0; i < npass; ++i) {
            FwdSeg &S = A.seg[i];
            const float *theta = theta_of(c, pass[i].net);
            S.x = xptr(i);
            S.xs = xstride(i);
            S.w = theta + woff;
            S.bias = with_bias ? theta + boff : nullptr;
            S.y = ybase + row0[i] * ystride;
            S.M = pass[i].n * P;
            S.tile_begin = tile;
            tile += (S.M + BM - 1) / BM;
        }
        for (int i = npass; i < 3; ++i) A.seg[i] = A.seg[0];
        return tile;
    };

    // Few rows (small batches): the reduction slab of every stage is sliced over extra waves
    // (KS > 1), which shortens the dependent chain of stages per tile.
    const bool small = rows * 81 < 64 * 512;
    {  // conv1: one wave per strip of a sample and channel half; a small batch also halves the reduction
        using namespace gbf;
        c1::FwdArgsF A{};
        A.nseg = npass;
        int first = 0;
        for (int i = 0; i < npass; ++i) {
            const float *theta = theta_of(c, pass[i].net);
            A.seg[i] = c1::FwdSegF{c1::Src{pass[i].x, pass[i].xs, pass[i].idx, (long)c->cfg.replay_capacity, pass[i].shift, (int)c->sub},
                                   theta + net::C1W, theta + net::C1B, act1 + row0[i] * net::A1, pass[i].n, first,
                                   pass[i].stack, pass[i].stack_mode};
            first += pass[i].n;
        }
        for (int i = npass; i < 3; ++i) A.seg[i] = A.seg[0];
        A.total = first;
        A.draw = draw != nullptr;
        if (draw) A.samp = *draw;
        const Conv1Plan plan = conv1_plan_f32(first, c->num_cu);
        const bool ks2 = plan.ks2;
        const int grid = plan.grid;
        if (draw && !plan.draw_fits)   // the caller asks in_kernel_draw_fits first
            return fail(c, DQN_ERR_INVALID_ARG, "forward: batch too large for in-kernel sampling");
        if (ks2) launch(c, "conv1_fwd", st, [&] { c1::k_conv1_fwd_f32<2><<<dim3(grid), 256, 0, st>>>(A); });
        else launch(c, "conv1_fwd", st, [&] { c1::k_conv1_fwd_f32<1><<<dim3(grid), 256, 0, st>>>(A); });
    }
    {  // conv2
        FwdArgs A{};
        int BM = small ? 32 : 64;
        int tiles = build(A, BM, 81, [&](int i) { return (const void *)(act1 + row0[i] * net::A1); },
                          [&](int) { return (long)net::A1; }, net::C2W, net::C2B, act2, net::A2, true);
        A.klen = GConv2::K; A.split_stride = 0; A.scale = 1.0f;
        if (small) launch(c, "conv2_fwd", st, [&] { k_fwd<GConv2, 32, 32, 4><<<dim3(tiles, 2, 1), 256, 0, st>>>(A); });
        else launch(c, "conv2_fwd", st, [&] { k_fwd<GConv2, 64, 64><<<dim3(tiles, 1, 1), 256, 0, st>>>(A); });
    }
    {  // conv3
        FwdArgs A{};
        int BM = small ? 32 : 64;
        int tiles = build(A, BM, 49, [&](int i) { return (const void *)(act2 + row0[i] * net::A2); },
                          [&](int) { return (long)net::A2; }, net::C3W, net::C3B, act3, net::A3, true);
        A.klen = GConv3::K; A.split_stride = 0; A.scale = 1.0f;
        if (small) launch(c, "conv3_fwd", st, [&] { k_fwd<GConv3, 32, 32, 3><<<dim3(tiles, 2, 1), 192, 0, st>>>(A); });
        else launch(c, "conv3_fwd", st, [&] { k_fwd<GConv3, 64, 64><<<dim3(tiles, 1, 1), 256, 0, st>>>(A); });
    }
    {  // fc1: raw partial sums per reduction split; the head kernels finish it
        FwdArgs A{};
        const int ns = fc1_splits(rows, 0);
        int tiles = build(A, 32, 1, [&](int i) { return (const void *)(act3 + row0[i] * net::A3); },
                          [&](int) { return (long)net::A3; }, net::F1W, net::F1B, w.f1part, net::HID, false);
        A.klen = GFc1::K / ns; A.split_stride = rows * net::HID; A.scale = 1.0f;
        // few rows: the reduction of a split is sliced over seven wave groups of the workgroup as well
        if (rows <= 192) launch(c, "fc1_fwd", st, [&] { k_fwd<GFc1, 32, 32, 7><<<dim3(tiles, 16, ns), 448, 0, st>>>(A); });
        else launch(c, "fc1_fwd", st, [&] { k_fwd<GFc1, 32, 64><<<dim3(tiles, 8, ns), 128, 0, st>>>(A); });
        *nsplit_out = ns;
        *split_stride_out = rows * net::HID;
    }
    return hip_status(c, "forward");
}

// draw != nullptr: the conv1 kernel draws the transitions itself (replay mode; no sampling kernel ran)
int32_t forward_trunk_bf16(dqn_ctx *c, const Workspace &w, const Pass *pass, int npass, int *nsplit_out,
                           long *split_stride_out, hipStream_t st, const misc::SampleArgs *draw)
{
    using namespace gbf;
    bf16_t *act1 = (bf16_t *)w.act1, *act2 = (bf16_t *)w.act2, *act3 = (bf16_t *)w.act3;
    long row0[3];
    long rows = 0;
    for (int i = 0; i < npass; ++i) { row0[i] = rows; rows += pass[i].n; }

    auto build = [&](FwdArgs &A, int BM, int P, auto xptr, auto xstride, int64_t woff, int64_t boff,
                     auto yptr, bool with_bias) {
        int tile = 0;
        A.nseg = npass;
        for (int i = 0; i < npass; ++i) {
            FwdSeg &S = A.seg[i];
            S.x = xptr(i);
            S.xs = xstride(i);
            S.w = shadow_of(c, pass[i].net) + woff;
            S.bias = with_bias ? theta_of(c, pass[i].net) + boff : nullptr;
            S.y = yptr(i);
            S.M = pass[i].n * P;
            S.tile_begin = tile;
            tile += (S.M + BM - 1) / BM;
        }
        for (int i = npass; i < 3; ++i) A.seg[i] = A.seg[0];
        return tile;
    };

    // conv1 + conv2 as one launch, one workgroup per CU (faster from a handful of samples on)
    const int pass_n[3] = {pass[0].n, npass > 1 ? pass[1].n : 0, npass > 2 ? pass[2].n : 0};
    const bool fused12 = fused12_fits(c, pass_n, npass, draw != nullptr);
    const int grid12 = (int)std::min<long>(rows, c->num_cu);
    if (fused12) {
        c12::Args A{};
        A.nseg = npass;
        for (int i = 0; i < npass; ++i) {
            c12::Seg &S = A.seg[i];
            S.src = c1::Src{pass[i].x, pass[i].xs, pass[i].idx, (long)c->cfg.replay_capacity, pass[i].shift, (int)c->sub};
            S.w1 = shadow_of(c, pass[i].net) + net::C1W;
            S.b1 = theta_of(c, pass[i].net) + net::C1B;
            // only the backward pass reads conv1's output, and only the rows of the first pass of a training step
            S.y1 = npass == 3 && i == 0 ? act1 + row0[i] * net::A1 : nullptr;
            S.w2 = shadow_of(c, pass[i].net) + net::C2W;
            S.b2 = theta_of(c, pass[i].net) + net::C2B;
            S.y2 = act2 + row0[i] * net::A2;
            S.n = pass[i].n;
        }
        for (int i = npass; i < 3; ++i) A.seg[i] = A.seg[0];
        A.draw = draw != nullptr;
        if (draw) A.samp = *draw;
        launch(c, "conv12_fwd", st, [&] { c12::k_conv12_fwd<<<dim3(grid12), 512, c12::LDS_BYTES, st>>>(A); });
    } else
    {  // conv1: persistent waves, strips of the frames staged in LDS (read from the ring in ring mode)
        c1::FwdArgs A{};
        A.nseg = npass;
        int first = 0;
        for (int i = 0; i < npass; ++i) {
            c1::FwdSeg &S = A.seg[i];
            S.src = c1::Src{pass[i].x, pass[i].xs, pass[i].idx, (long)c->cfg.replay_capacity, pass[i].shift, (int)c->sub};
            S.w = shadow_of(c, pass[i].net) + net::C1W;
            S.bias = theta_of(c, pass[i].net) + net::C1B;
            S.y = act1 + row0[i] * net::A1;
            S.n = pass[i].n;
            S.first = first;
            first += pass[i].n;
        }
        for (int i = npass; i < 3; ++i) A.seg[i] = A.seg[0];
        A.total = first;
        A.draw = draw != nullptr;
        if (draw) A.samp = *draw;
        // a wave that draws for itself holds at most MAX_DRAWS slots: its units span that many samples at most
        const Conv1Plan plan = conv1_plan_bf16(first, c->num_cu);
        const int grid = plan.grid;
        if (draw && !plan.draw_fits)   // the caller asks in_kernel_draw_fits first
            return fail(c, DQN_ERR_INVALID_ARG, "forward: batch too large for in-kernel sampling");
        launch(c, "conv1_fwd", st, [&] { c1::k_conv1_fwd<<<dim3(grid), 256, 0, st>>>(A); });
    }
    // conv2, conv3: persistent workgroups that keep the weights in registers and take one sample at a time
    auto per_sample = [&](ps::Args &A, const bf16_t *x, long xs, int64_t woff, int64_t boff, bf16_t *y, long ys) {
        A.nseg = npass;
        int first = 0;
        for (int i = 0; i < npass; ++i) {
            A.seg[i] = ps::Seg{x + row0[i] * xs, shadow_of(c, pass[i].net) + woff, theta_of(c, pass[i].net) + boff,
                               y + row0[i] * ys, pass[i].n, first};
            first += pass[i].n;
        }
        for (int i = npass; i < 3; ++i) A.seg[i] = A.seg[0];
        A.total = first;
        return std::min(first, 2 * c->num_cu);
    };
    if (!fused12) {
        ps::Args A{};
        const int grid = per_sample(A, act1, net::A1, net::C2W, net::C2B, act2, net::A2);
        launch(c, "conv2_fwd", st, [&] { ps::k_conv_fwd_ps<ps::G2><<<dim3(grid), 256, 0, st>>>(A); });
    }
    {
        ps::Args A{};
        const int grid = per_sample(A, act2, net::A2, net::C3W, net::C3B, act3, net::A3);
        launch(c, "conv3_fwd", st, [&] { ps::k_conv_fwd_ps<ps::G3><<<dim3(grid), 256, 0, st>>>(A); });
    }
    if (c->fc1_big && rows >= c->fc1_big_rows) {
        // many rows: 128 x 128 tiles, double-buffered stages, few reduction splits
        f1::Args A{};
        A.nseg = npass;
        int tile = 0;
        for (int i = 0; i < npass; ++i) {
            A.seg[i] = FwdSeg{act3 + row0[i] * net::A3, shadow_of(c, pass[i].net) + net::F1W, nullptr,
                              w.f1part + row0[i] * net::HID, pass[i].n, tile, (long)net::A3};
            tile += (pass[i].n + f1::BM - 1) / f1::BM;
        }
        for (int i = npass; i < 3; ++i) A.seg[i] = A.seg[0];
        A.tiles_m = tile;
        // as many splits as it takes to give about three quarters of the compute units a workgroup, seven at
        // most: every further split is another 3 MB of partial sums per 1536 rows to write and to read back
        // (measured at 1536 rows: 3 / 4 / 5 / 6 / 7 splits give 151.3 / 149.8 / 152 / 153.5 / 152.6 us per step)
        int ns = c->fc1_big_splits > 0 ? c->fc1_big_splits : (3 * c->num_cu / 4 + 2 * tile) / (4 * tile);
        ns = std::max<long>(1, std::min<long>({(long)ns, 7L, (long)(w.f1rows / (size_t)rows)}));
        A.nsplit = ns;
        A.split_stride = rows * net::HID;
        launch(c, "fc1_fwd", st, [&] { f1::k_fc1_fwd<<<dim3(4 * tile * ns), 256, f1::LDS_BYTES, st>>>(A); });
        *nsplit_out = ns;
        *split_stride_out = rows * net::HID;
    } else {
        FwdArgs A{};
        const int ns = fc1_splits(rows, 1);
        int tiles = build(A, 64, 1, [&](int i) { return (const void *)(act3 + row0[i] * net::A3); },
                          [&](int) { return (long)net::A3; }, net::F1W, net::F1B,
                          [&](int i) { return (void *)(w.f1part + row0[i] * net::HID); }, false);
        A.klen = GFc1::K / ns; A.split_stride = rows * net::HID; A.scale = 1.0f;
        launch(c, "fc1_fwd", st, [&] { k_fwd<GFc1, 64, 128, 1, 2, true><<<dim3(tiles, 4, ns), 256, 0, st>>>(A); });
        *nsplit_out = ns;
        *split_stride_out = rows * net::HID;
    }
    return hip_status(c, "forward");
}

// w: where the activations and the fc1 partial sums go (the context's workspace, or a view of the
// library's static scratch array)
int32_t forward_trunk(dqn_ctx *c, const Workspace &w, const Pass *pass, int npass, int *ns, long *ss, hipStream_t st,
                      const misc::SampleArgs *draw = nullptr)
{
    return c->cfg.precision == 1 ? forward_trunk_bf16(c, w, pass, npass, ns, ss, st, draw)
                                 : forward_trunk_f32(c, w, pass, npass, ns, ss, st, draw);
}

// reduction rows per split (a multiple of `unit`) and the resulting number of splits
void split_rows(long M, int tiles, int cap, int unit, int *rps, int *ns)
{
    long want = std::max<long>(1, 512 / tiles);
    long by_rows = std::max<long>(1, M / 64);
    long n = std::min<long>({want, by_rows, (long)cap});
    long r = ((M + n - 1) / n + unit - 1) / unit * unit;
    *rps = (int)r;
    *ns = (int)((M + r - 1) / r);
}

// fork/join between the caller's stream and the side stream (no-ops when they are the same)
void ev_record(hipEvent_t e, hipStream_t on, hipStream_t other)
{
    if (on != other) (void)hipEventRecord(e, on);
}
void ev_wait(hipStream_t waiter, hipEvent_t e, hipStream_t other)
{
    if (waiter != other) (void)hipStreamWaitEvent(waiter, e, 0);
}

// The priority update (one workgroup, twenty tree levels one after the other, needs only the TD
// errors) rides in other launches as their workgroup 0 (bf16: the backward launches of fc1, conv3 and conv2 and the RMSProp launch; fp32: those three backward launches), four entries per
// thread and a share of the levels per launch (the first part, which also settles the duplicates and
// raises the new priorities to the power alpha, takes the fewest): each part is shorter than the
// launch it sits in, so the update costs no launch, no stream and no event.
struct SplitUpdate {
    misc::PerUpdateArgs update;
    int *state;
    int upto[3];        // tree levels walked when part 0, 1, 2 ends (part 3 goes to the root)
    int on;             // 0: no update in this step
};
// part k of the update (k = 0: settle duplicates, write the leaves, first levels)
__device__ __forceinline__ void update_part(const SplitUpdate &U, int k, int *lds)
{
    if (k == 0) misc::per_update_body<4>(U.update, lds, U.upto[0], U.state);
    else misc::per_update_resume<4>(U.update, U.upto[k - 1], k < 3 ? U.upto[k] - U.upto[k - 1] : U.update.levels, U.state);
}

// RMSProp after workgroup 0, which finishes the priority update (conv1's weight-gradient launch
// fills every workgroup slot of the chip with its own 512 workgroups; RMSProp's are many and short)
__global__ __launch_bounds__(256) void k_rmsprop_pu(misc::RmsArgs A, SplitUpdate U)
{
    __shared__ float red[4][64];
    if (blockIdx.x == 0) return update_part(U, 3, nullptr);
    const int bx = (int)blockIdx.x - 1;
    RMS_SELECT_SEGMENT(A, bx, S)
    misc::rmsprop_block(A, S, bx, red);
}

// ----- RMSProp over a subset of the layers (bit i of `layers`: conv1, conv2, conv3, fc1, head) -----
enum : unsigned { RMS_CONV1 = 1, RMS_CONV2 = 2, RMS_CONV3 = 4, RMS_FC1 = 8, RMS_HEAD = 16, RMS_ALL = 31 };
void launch_rmsprop(dqn_ctx *c, unsigned layers, int ns1, int ns2, int ns3, hipStream_t st,
                    const SplitUpdate *last_part = nullptr)
{
    const dqn_config &cfg = c->cfg;
    const Workspace &w = c->ws;
    const long cnt[5] = {net::L1N, net::L2N, net::L3N, net::L4N, net::head_count(cfg.num_actions, cfg.dueling)};
    const long beg[5] = {net::C1W, net::C2W, net::C3W, net::F1W, net::HEAD};
    // fc1's and the head's weight gradients have a single partial: they are written straight into the
    // gradient buffer (c->gp4, c->gp5), and RMSProp does not store them there once more
    const float *part[5] = {w.gp1, w.gp2, w.gp3, c->gp4, c->gp5};
    const int nsp[5] = {ns1, ns2, ns3, 1, 1};
    misc::RmsArgs RA{};
    int blk = 0, k = 0;
    for (int i = 0; i < 5; ++i) {
        if (!(layers >> i & 1)) continue;
        RA.seg[k++] = {beg[i], cnt[i], part[i], nsp[i], nsp[i] > 1 ? cnt[i] : 0, blk};
        const long per = nsp[i] > 1 ? 64 : 256;
        blk += (int)((cnt[i] + per - 1) / per);
    }
    for (; k < 5; ++k) RA.seg[k].block_begin = 0x7fffffff;  // never selected
    RA.theta = c->theta; RA.v = c->rms_v; RA.m = c->rms_m; RA.g = c->grads;
    RA.shadow = cfg.precision == 1 ? (__hip_bfloat16 *)c->buf.shadow_bf16 : nullptr;
    RA.w2t = cfg.precision == 1 ? (__hip_bfloat16 *)w.w2t : nullptr;
    RA.lr = cfg.lr; RA.rho = cfg.rms_decay; RA.eps = cfg.rms_eps;
    if (last_part && last_part->on) launch(c, "rmsprop", st, [&] { k_rmsprop_pu<<<blk + 1, 256, 0, st>>>(RA, *last_part); });
    else launch(c, "rmsprop", st, [&] { misc::k_rmsprop<<<blk, 256, 0, st>>>(RA); });
}

// What rides in the launches of the backward pass beside the trunk's gradients: the head's weight
// gradient and the priority update (Eq.11) of the transitions just trained on.
struct SmallTail {
    misc::HeadWgradArgs head;
    misc::PerUpdateArgs update;
    bool with_update;
};

// ----- fp32 on one stream: one backward launch per layer, as in the bf16 step -----
// The layer's input-gradient tiles and its weight-gradient tiles share a launch (both read the
// layer's dY); the input gradients of a small batch are 100-200 workgroups, so the weight
// gradient rides in what the launch leaves free.  fc1's launch also takes the head's weight
// gradient; workgroup 0 of each launch is part PART of the priority update.  A launch has the width of its widest tile
// (256 / 384 / 512 threads); in a narrower tile the waves beyond leave at once.
struct PairF32 {
    int nd, dgx, dgz;        // input gradient: tiles, grid x and z
    int nw, wgx, wgy, wgz;   // weight gradient: tiles, grid
};
template <class D, int BM, int BN, int KS, class G, int TH, bool HEAD, int PART>
__global__ __launch_bounds__(TH) void k_layer_bwd_f32(g32::DgradArgs DA, g32::WgradArgs WA, PairF32 P,
                                                      misc::HeadWgradArgs H, SplitUpdate U)
{
    using namespace g32;
    constexpr int LD = dgrad_lds<BM, BN, KS>(), LW = wgrad_lds<64, 64>();
    constexpr int L0 = LD > LW ? LD : LW;
    constexpr int L = PART == 0 && misc::PU_LDS_WORDS > L0 ? misc::PU_LDS_WORDS : L0;
    __shared__ __attribute__((aligned(16))) float lds[L];
    if (U.on && blockIdx.x == 0) return update_part(U, PART, reinterpret_cast<int *>(lds));
    const int id = (int)blockIdx.x - U.on;
    if (id < P.nd) {
        // dispatch order -> tile number, die-aware within the group
        const int die = id & 7, slot = id >> 3, q = P.nd >> 3, r = P.nd & 7;
        dgrad_tile<D, BM, BN, KS>(DA, die * q + (die < r ? die : r) + slot, P.dgx, P.dgz, lds);
    } else if (id < P.nd + P.nw) {
        int bx, by, bz;
        wgrad_tile_of(id - P.nd, P.wgx, P.wgy, P.wgz, bx, by, bz);
        wgrad_tile<G, 64, 64>(WA, bx, by, bz, lds);
    } else if (HEAD) {
        if ((int)threadIdx.x >= 256) return;
        const int u = id - P.nd - P.nw;
        misc::head_wgrad_body<8>(H, u / 16, u % 16, lds);
    }
}

// ----- backward through fc1, conv3, conv2, conv1 (no input gradient for conv1) -----
// The input-gradient chain and conv1's weight gradient run on st; the weight gradients of fc1,
// conv3 and conv2 run on sd behind the events the chain records.  All of st's kernels are
// enqueued before any of sd's: handing the host from one stream to another costs more than a
// launch, and the device does not care in which order the host filled the two queues.
void backward_f32(dqn_ctx *c, int B, const uint8_t *s, long xs, int *ns1, int *ns2, int *ns3, hipStream_t st,
                  hipStream_t sd, const SmallTail *tail)
{
    using namespace g32;
    const Workspace &w = c->ws;
    float *act1 = (float *)w.act1, *act2 = (float *)w.act2, *act3 = (float *)w.act3;
    float *dh = (float *)w.dh, *d3 = (float *)w.d3, *d2 = (float *)w.d2, *d1 = (float *)w.d1;
    const bool small = B <= 128;
    int rps1, rps2, rps3;
    split_rows((long)B * 400, 1, MAX_WSPLIT1, 32, &rps1, ns1);
    split_rows((long)B * 81, 8, MAX_WSPLIT, 32, &rps2, ns2);
    split_rows((long)B * 49, 9, MAX_WSPLIT, 32, &rps3, ns3);
    const WgradArgs G1{d1, s, w.gp1, B, rps1, xs, net::L1N, 1.0f / 255.0f};
    const WgradArgs G2{d2, act1, w.gp2, B, rps2, net::A1, net::L2N, 1.0f};
    const WgradArgs G3{d3, act2, w.gp3, B, rps3, net::A2, net::L3N, 1.0f};
    const WgradArgs G4{dh, act3, c->gp4, B, (B + 31) / 32 * 32, net::A3, 0, 1.0f};
    if (sd == st) {
        // the priority update in three parts: few levels beside fc1's short launch, the rest in halves
        const int lv = c->levels;
        const SplitUpdate U{tail->update, w.pu_state, {lv / 10, 11 * lv / 20, 11 * lv / 20}, tail->with_update ? 1 : 0};
        const misc::HeadWgradArgs &HW = tail->head;
        {
            DgradArgs D{dh, c->theta + net::F1W, act3, d3, B};
            const int gx = (B + 31) / 32;
            const int nh = c->R * 16 + U.on;
            if (small) {
                PairF32 P{gx * 98, gx, 1, 49 * 8, 49, 8, 1};
                launch(c, "fc1_bwd", st, [&] {
                    k_layer_bwd_f32<DFc1, 32, 32, 4, GFc1, 256, true, 0><<<P.nd + P.nw + nh, 256, 0, st>>>(D, G4, P, HW, U);
                });
            } else {
                PairF32 P{gx * 49, gx, 1, 49 * 8, 49, 8, 1};
                launch(c, "fc1_bwd", st, [&] {
                    k_layer_bwd_f32<DFc1, 32, 64, 1, GFc1, 256, true, 0><<<P.nd + P.nw + nh, 256, 0, st>>>(D, G4, P, HW, U);
                });
            }
        }
        {
            DgradArgs D{d3, c->theta + net::C3W, act2, d2, B};
            if (small) {
                const int gx = (int)(((long)B * 81 + 31) / 32);
                PairF32 P{gx * 2, gx, 1, 9 * *ns3, 9, 1, *ns3};
                launch(c, "conv3_bwd", st, [&] {
                    k_layer_bwd_f32<DConv3, 32, 32, 6, GConv3, 384, false, 1><<<P.nd + P.nw + U.on, 384, 0, st>>>(D, G3, P, HW, U);
                });
            } else {
                const int gx = (int)(((long)B * 81 + 63) / 64);
                PairF32 P{gx, gx, 1, 9 * *ns3, 9, 1, *ns3};
                launch(c, "conv3_bwd", st, [&] {
                    k_layer_bwd_f32<DConv3, 64, 64, 1, GConv3, 256, false, 1><<<P.nd + P.nw + U.on, 256, 0, st>>>(D, G3, P, HW, U);
                });
            }
        }
        {
            DgradArgs D{d2, c->theta + net::C2W, act1, d1, B};
            const int gx = (int)(((long)B * 100 + 63) / 64);
            PairF32 P{gx * 4, gx, 4, 8 * *ns2, 8, 1, *ns2};
            launch(c, "conv2_bwd", st, [&] {
                k_layer_bwd_f32<DConv2, 64, 32, 4, GConv2, 512, false, 3><<<P.nd + P.nw + U.on, 512, 0, st>>>(D, G2, P, HW, U);
            });
        }
        if (B <= 64) launch(c, "conv1_wgrad", st, [&] { k_wgrad<GConv1, 32, 128><<<dim3(2, 1, *ns1), 256, 0, st>>>(G1); });
        else launch(c, "conv1_wgrad", st, [&] { k_wgrad<GConv1, 32, 256><<<dim3(1, 1, *ns1), 512, 0, st>>>(G1); });
        return;
    }
    {
        DgradArgs D{dh, c->theta + net::F1W, act3, d3, B};
        launch(c, "fc1_dgrad", st, [&] { k_dgrad<DFc1, 32, 64><<<dim3((B + 31) / 32, 49, 1), 128, 0, st>>>(D); });
        ev_record(c->ev_a, st, sd);
    }
    {
        DgradArgs D{d3, c->theta + net::C3W, act2, d2, B};
        long M = (long)B * 81;
        launch(c, "conv3_dgrad", st, [&] { k_dgrad<DConv3, 64, 64><<<dim3((M + 63) / 64, 1, 1), 256, 0, st>>>(D); });
        ev_record(c->ev_b, st, sd);
    }
    {
        DgradArgs D{d2, c->theta + net::C2W, act1, d1, B};
        long M = (long)B * 100;
        launch(c, "conv2_dgrad", st, [&] { k_dgrad<DConv2, 64, 32, 4><<<dim3((M + 63) / 64, 1, 4), 512, 0, st>>>(D); });
    }
    // large batch on three streams: the input-gradient chain and conv1's weight gradient on st, the other
    // weight gradients on sd behind the events of their input gradients
    launch(c, "conv1_wgrad", st, [&] { k_wgrad<GConv1, 32, 256><<<dim3(1, 1, *ns1), 512, 0, st>>>(G1); });
    launch(c, "fc1_wgrad", sd, [&] { k_wgrad<GFc1, 64, 64><<<dim3(49, 8, 1), 256, 0, sd>>>(G4); });
    ev_wait(sd, c->ev_a, st);
    launch(c, "conv3_wgrad", sd, [&] { k_wgrad<GConv3, 64, 64><<<dim3(9, 1, *ns3), 256, 0, sd>>>(G3); });
    ev_wait(sd, c->ev_b, st);
    launch(c, "conv2_wgrad", sd, [&] { k_wgrad<GConv2, 64, 64><<<dim3(8, 1, *ns2), 256, 0, sd>>>(G2); });
}

// fc1's backward pair (see gbf::k_bwd_pair) with the head's weight gradient as a third group of
// workgroups (row r, 32 hidden units each): all three need only what the head kernel left.
__global__ __launch_bounds__(256) void k_fc1_head_bwd(gbf::DgradArgs DA, gbf::WgradArgs WA, gbf::PairGrid P,
                                                      misc::HeadWgradArgs H, SplitUpdate U)
{
    using namespace gbf;
    constexpr int LD = dgrad_lds<64, 64, true>(), LW = wgrad_lds<64, 64, true>();
    static_assert((LD > LW ? LD : LW) * 2 >= 8 * 34 * 4 && (LD > LW ? LD : LW) * 2 >= misc::PU_LDS_WORDS * 4, "LDS");
    __shared__ __attribute__((aligned(16))) bf16_t lds[LD > LW ? LD : LW];
    if (U.on && blockIdx.x == 0) return update_part(U, 0, reinterpret_cast<int *>(lds));
    const int id = (int)blockIdx.x - U.on;
    if (id < P.nd) {
        dgrad_tile<DFc1, 64, 64, 1, 1, true>(DA, tile_of(id, P.nd), P.dgx, P.dgz, lds);
    } else if (id < P.nd + P.nw) {
        wgrad_tile<GFc1, 64, 64, 1, 1, true>(WA, tile_of(id - P.nd, P.nw), P.wgx, P.wgy, P.wgz, lds);
    } else {
        const int u = id - P.nd - P.nw;
        misc::head_wgrad_body<8>(H, u / 16, u % 16, reinterpret_cast<float *>(lds));
    }
}

// conv3's backward pair after workgroup 0
__global__ __launch_bounds__(256) void k_conv3_bwd_pu(gbf::DgradArgs DA, gbf::WgradArgs WA, gbf::PairGrid P, SplitUpdate U)
{
    using namespace gbf;
    constexpr int LD = dgrad_lds<64, 64, true>(), LW = wgrad_lds<64, 64, true>();
    __shared__ __attribute__((aligned(16))) bf16_t lds[LD > LW ? LD : LW];
    if (U.on && blockIdx.x == 0) return update_part(U, 1, reinterpret_cast<int *>(lds));
    const int id = (int)blockIdx.x - U.on;
    if (id < P.nd) dgrad_tile<DConv3, 64, 64, 1, 1, true>(DA, tile_of(id, P.nd), P.dgx, P.dgz, lds);
    else wgrad_tile<GConv3, 64, 64, 1, 1, true>(WA, tile_of(id - P.nd, P.nw), P.wgx, P.wgy, P.wgz, lds);
}

// conv2's backward pair after workgroup 0: the per-sample input gradient (nps workgroups) and the
// tiled weight gradient (nw workgroups); both read conv2's dY
__global__ __launch_bounds__(256, 2) void k_conv2_bwd_pu(gbf::dps::Args PA, gbf::WgradArgs WA, int nps, int nw, int wgx,
                                                         int wgy, int wgz, SplitUpdate U)
{
    using namespace gbf;
    constexpr int LW = wgrad_lds<64, 64, true>() * 2;   // bytes
    constexpr int LB = dps::PS_LDS > LW ? dps::PS_LDS : LW;
    __shared__ __attribute__((aligned(16))) uint8_t lds[LB];
    if (U.on && blockIdx.x == 0) return update_part(U, 2, reinterpret_cast<int *>(lds));
    const int id = (int)blockIdx.x - U.on;
    if (id < nps) dps::conv2_dgrad_ps_body(PA, id, nps, lds);
    else wgrad_tile<GConv2, 64, 64, 1, 1, true>(WA, tile_of(id - nps, nw), wgx, wgy, wgz, reinterpret_cast<bf16_t *>(lds));
}

// conv2's launch with conv1's weight gradient inside the per-sample workgroups (dps::conv2_dgrad_conv1_wgrad_body):
// workgroup 0 as above, nps workgroups of samples, nw weight-gradient tiles.  Dynamic LDS: dps::FUSED_LDS.
__global__ __launch_bounds__(256, 2) void k_conv21_bwd_pu(gbf::dps::FusedArgs FA, gbf::WgradArgs WA, int nps, int nw, int wgx,
                                                          int wgy, int wgz, SplitUpdate U)
{
    using namespace gbf;
    static_assert(dps::FUSED_LDS >= wgrad_lds<64, 128, true>() * 2 && dps::FUSED_LDS >= misc::PU_LDS_WORDS * 4, "LDS");
    extern __shared__ __attribute__((aligned(16))) uint8_t lds_dyn[];
    if (U.on && blockIdx.x == 0) return update_part(U, 2, reinterpret_cast<int *>(lds_dyn));
    const int id = (int)blockIdx.x - U.on;
    if (id < nps) dps::conv2_dgrad_conv1_wgrad_body(FA, id, nps, lds_dyn);
    else wgrad_tile<GConv2, 64, 128, 1, 2, true>(WA, tile_of(id - nps, nw), wgx, wgy, wgz, reinterpret_cast<bf16_t *>(lds_dyn));
}

// bf16: one stream and one launch per layer, the layer's input gradient and weight gradient side by
// side in it (both read the layer's dY and nothing else that the backward pass computes).  Events
// between streams cost more than they gain here: a record or a wait on the critical stream adds
// about 4 us to the gap between two kernels, and a kernel on another stream starts 11-14 us after
// the kernel it waits for has ended.
void backward_bf16(dqn_ctx *c, int B, const Pass &ps, int *ns1, int *ns2, int *ns3, hipStream_t st,
                   const misc::HeadWgradArgs &head, const SplitUpdate &U)
{
    using namespace gbf;
    const Workspace &w = c->ws;
    bf16_t *act1 = (bf16_t *)w.act1, *act2 = (bf16_t *)w.act2, *act3 = (bf16_t *)w.act3;
    bf16_t *dh = (bf16_t *)w.dh, *d3 = (bf16_t *)w.d3, *d2 = (bf16_t *)w.d2, *d1 = (bf16_t *)w.d1;
    const bf16_t *sh = shadow_of(c, 0);
    int rps;
    {
        DgradArgs D{dh, sh + net::F1W, act3, d3, B};
        WgradArgs G{dh, act3, c->gp4, B, (B + 63) / 64 * 64, net::A3, 0, 1.0f};
        const int gx = (B + 63) / 64;
        PairGrid P{gx * 49, gx, 1, 49 * 8, 49, 8, 1};
        const int nh = c->R * 16;
        launch(c, "fc1_bwd", st, [&] { k_fc1_head_bwd<<<P.nd + P.nw + nh + U.on, 256, 0, st>>>(D, G, P, head, U); });
    }
    {
        DgradArgs D{d3, sh + net::C3W, act2, d2, B};
        const int nd = (int)(((long)B * 81 + 63) / 64);
        // four workgroups of this launch fit one CU: where fewer splits let the whole launch run in one
        // round of workgroups, take fewer (B = 512: 41 instead of 56; 153.2 against 154.6 us/step)
        int cap3 = (4 * c->num_cu - 1 - nd) / 9;
        if (cap3 < 32 || cap3 > MAX_WSPLIT) cap3 = MAX_WSPLIT;
        split_rows((long)B * 49, 9, cap3, 64, &rps, ns3);
        WgradArgs G{d3, act2, w.gp3, B, rps, net::A2, net::L3N, 1.0f};
        PairGrid P{nd, nd, 1, 9 * *ns3, 9, 1, *ns3};
        launch(c, "conv3_bwd", st, [&] { k_conv3_bwd_pu<<<P.nd + P.nw + U.on, 256, 0, st>>>(D, G, P, U); });
    }
    {   // conv2: the per-sample input gradient, at most one workgroup per CU, beside the tiled weight gradient
        dps::Args P{d2, sh + net::C2W, act1, d1, B};
        split_rows((long)B * 81, 8, MAX_WSPLIT, 64, &rps, ns2);
        WgradArgs G{d2, act1, w.gp2, B, rps, net::A1, net::L2N, 1.0f};
        const int nw = 8 * *ns2, gz = *ns2;
        if (c->fused_bwd) {
            // conv1's weight gradient inside the per-sample workgroups: one partial per workgroup.  Two workgroups
            // of this launch fit one CU, so the weight-gradient tiles are 64 x 128: a quarter of the row splits'
            // tiles fewer, and the launch runs in one round of workgroups at B = 512
            const int nps = std::min({B, c->num_cu, MAX_WSPLIT1});
            const int nw2 = 4 * gz;
            dps::FusedArgs F{P, c1::Src{ps.x, ps.xs, ps.idx, (long)c->cfg.replay_capacity, ps.shift, (int)c->sub}, w.gp1, w.w2t};
            launch(c, "conv21_bwd", st, [&] {
                k_conv21_bwd_pu<<<nps + nw2 + U.on, 256, dps::FUSED_LDS, st>>>(F, G, nps, nw2, 4, 1, gz, U);
            });
            *ns1 = nps;
            return;
        }
        const int nps = std::min(B, c->num_cu);
        launch(c, "conv2_bwd", st, [&] { k_conv2_bwd_pu<<<nps + nw + U.on, 256, 0, st>>>(P, G, nps, nw, 8, 1, gz, U); });
    }
    {   // conv1: one workgroup per split of samples, frames staged in LDS
        *ns1 = std::min(B, MAX_WSPLIT1);
        c1::WgradArgs G{c1::Src{ps.x, ps.xs, ps.idx, (long)c->cfg.replay_capacity, ps.shift, (int)c->sub}, d1, w.gp1, B, *ns1};
        launch(c, "conv1_wgrad", st, [&] { c1::k_conv1_wgrad<<<dim3(*ns1, 2), 256, 0, st>>>(G); });
    }
}

}  // namespace

// ============================================================================
extern "C" {

const char *dqn_last_error(const dqn_ctx *ctx) { return ctx ? ctx->err.c_str() : g_err.c_str(); }

int32_t dqn_query_sizes(const dqn_config *cfg, dqn_sizes *out)
{
    if (!cfg || !out) return fail(nullptr, DQN_ERR_INVALID_ARG, "dqn_query_sizes: NULL argument");
    if (const char *m = check_config(*cfg)) return fail(nullptr, DQN_ERR_INVALID_ARG, m);
    dqn_sizes s{};
    const int64_t n = net::param_count(cfg->num_actions, cfg->dueling);
    s.param_count = n;
    s.params = align_up((size_t)n * 4, 256);
    s.opt_state = s.params * (cfg->rms_centered ? 2 : 1);
    s.shadow_bf16 = cfg->precision == 1 ? 2 * align_up((size_t)n * 2, 256) : 0;
    s.grads = s.params;
    const int64_t cap = cfg->replay_capacity;
    s.replay_frames = (size_t)cap * net::FRAME;
    s.replay_meta = cap ? align_up((size_t)cap * 4, 256) * 2 + align_up((size_t)cap, 256) : 0;
    s.tree_leaves = cap ? tree_leaves(cap) : 0;
    s.tree = cap ? ((size_t)2 * s.tree_leaves + 64) * 4 : 0;
    s.workspace = carve(*cfg, nullptr).total;
    *out = s;
    return DQN_OK;
}

int32_t dqn_init(dqn_ctx **out, const dqn_config *cfg, const dqn_buffers *b, void *stream)
{
    if (!out || !cfg || !b) return fail(nullptr, DQN_ERR_INVALID_ARG, "dqn_init: NULL argument");
    *out = nullptr;
    dqn_sizes sz;
    int32_t rc = dqn_query_sizes(cfg, &sz);
    if (rc) return rc;
    const void *req[] = {b->online, b->target, b->opt_state, b->grads, b->workspace};
    for (const void *p : req)
        if (!p || !aligned(p, 256)) return fail(nullptr, DQN_ERR_INVALID_ARG, "dqn_init: a required buffer is NULL or not 256-byte aligned");
    if (cfg->precision == 1 && (!b->shadow_bf16 || !aligned(b->shadow_bf16, 256)))
        return fail(nullptr, DQN_ERR_INVALID_ARG, "dqn_init: shadow_bf16 buffer required for precision 1");
    if (cfg->replay_capacity > 0) {
        const void *rp[] = {b->replay_frames, b->replay_meta, b->tree};
        for (const void *p : rp)
            if (!p || !aligned(p, 256)) return fail(nullptr, DQN_ERR_INVALID_ARG, "dqn_init: replay buffers are NULL or not 256-byte aligned");
    }
    dqn_ctx *c = new (std::nothrow) dqn_ctx();
    if (!c) return fail(nullptr, DQN_ERR_OOM, "dqn_init: out of host memory");
    c->cfg = *cfg;
    c->buf = *b;
    c->sz = sz;
    c->n = sz.param_count;
    c->R = cfg->num_actions + (cfg->dueling ? 1 : 0);
    c->ws = carve(*cfg, (uint8_t *)b->workspace);
    c->theta = (float *)b->online;
    c->theta_t = (float *)b->target;
    c->rms_v = (float *)b->opt_state;
    c->rms_m = cfg->rms_centered ? (float *)((uint8_t *)b->opt_state + sz.params) : nullptr;
    c->grads = (float *)b->grads;
    c->gp4 = c->grads + net::F1W;
    c->gp5 = c->grads + net::HEAD;
    c->L = sz.tree_leaves;
    c->levels = 0;
    while ((1l << c->levels) < c->L) ++c->levels;
    c->stored = 0;
    c->sub = (long)cfg->replay_capacity;
    if (cfg->replay_capacity > 0) {
        size_t stride = align_up((size_t)cfg->replay_capacity * 4, 256);
        c->meta_a = (int32_t *)b->replay_meta;
        c->meta_r = (float *)((uint8_t *)b->replay_meta + stride);
        c->meta_done = (uint8_t *)b->replay_meta + 2 * stride;
        c->tree = (float *)b->tree;
    }
    hipStream_t st = (hipStream_t)stream;

    std::vector<float> blob;
    try {
        blob.resize((size_t)c->n);
    } catch (...) {
        delete c;
        return fail(nullptr, DQN_ERR_OOM, "dqn_init: out of host memory");
    }
    for (int net_i = 0; net_i < 2; ++net_i) {
        he_uniform_host(blob, cfg->num_actions, cfg->dueling, net_i ? cfg->target_seed : cfg->seed);
        // the gradient buffer doubles as the staging area for the canonical blob
        if (hipMemcpyAsync(c->grads, blob.data(), (size_t)c->n * 4, hipMemcpyHostToDevice, st) != hipSuccess ||
            hipStreamSynchronize(st) != hipSuccess) {
            std::string m = std::string("dqn_init: upload failed: ") + hipGetErrorString(hipGetLastError());
            delete c;
            return fail(nullptr, DQN_ERR_HIP, m);
        }
        permute(c, c->grads, net_i ? c->theta_t : c->theta, 0, st);
    }
    long nopt = (long)(sz.opt_state / 4);
    misc::k_fill<<<grid1(nopt, 256), 256, 0, st>>>(c->rms_v, 0.f, nopt);
    misc::k_fill<<<grid1(c->n, 256), 256, 0, st>>>(c->grads, 0.f, c->n);
    if (cfg->replay_capacity > 0) {
        long nt = 2 * c->L + 64;
        misc::k_fill<<<grid1(nt, 256), 256, 0, st>>>(c->tree, 0.f, nt);
        misc::k_fill<<<1, 64, 0, st>>>(c->tree + 2 * c->L, 1.0f, 1);  // maximal priority starts at 1
    }
    if (cfg->precision == 1) {
        __hip_bfloat16 *sh = (__hip_bfloat16 *)b->shadow_bf16;
        size_t half = align_up((size_t)c->n * 2, 256) / 2;
        misc::k_to_bf16<<<grid1(c->n, 256), 256, 0, st>>>(c->theta, sh, c->n);
        misc::k_to_bf16<<<grid1(c->n, 256), 256, 0, st>>>(c->theta_t, sh + half, c->n);
        misc::k_w2_transposed<<<grid1(64 * 512, 256), 256, 0, st>>>(c->theta + net::C2W, (__hip_bfloat16 *)c->ws.w2t);
    }
    if (hipStreamSynchronize(st) != hipSuccess || hipGetLastError() != hipSuccess) {
        delete c;
        return fail(nullptr, DQN_ERR_HIP, "dqn_init: device initialisation failed");
    }
    (void)scratch_of_current_device();   // set-up: the address of the static scratch array on this device
    {
        int dev = 0, cus = 0;
        if (hipGetDevice(&dev) == hipSuccess &&
            hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess && cus > 0)
            c->num_cu = cus;
    }
    // DQN_CONV12_MIN_SAMPLES in the environment moves the batch size from which the fused conv1 + conv2
    // forward launch is used (samples of all passes of a launch; a huge value switches it off)
    if (cfg->precision == 1 &&
        hipFuncSetAttribute((const void *)gbf::c12::k_conv12_fwd, hipFuncAttributeMaxDynamicSharedMemorySize,
                            gbf::c12::LDS_BYTES) == hipSuccess) {
        const char *m = std::getenv("DQN_CONV12_MIN_SAMPLES");
        c->conv12_min = m && m[0] ? std::atoi(m) : 8;
    } else {
        (void)hipGetLastError();
    }
    // DQN_FUSED_BWD=0 in the environment keeps conv1's weight gradient a launch of its own
    if (cfg->precision == 1 &&
        hipFuncSetAttribute((const void *)k_conv21_bwd_pu, hipFuncAttributeMaxDynamicSharedMemorySize,
                            gbf::dps::FUSED_LDS) == hipSuccess) {
        const char *m = std::getenv("DQN_FUSED_BWD");
        c->fused_bwd = !(m && m[0] == '0');
    } else {
        (void)hipGetLastError();
    }
    if (cfg->precision == 1 &&
        hipFuncSetAttribute((const void *)gbf::f1::k_fc1_fwd, hipFuncAttributeMaxDynamicSharedMemorySize,
                            gbf::f1::LDS_BYTES) == hipSuccess) {
        c->fc1_big = true;
        if (const char *m = std::getenv("DQN_FC1_BIG_ROWS")) if (m[0]) c->fc1_big_rows = std::atoi(m);
        if (const char *m = std::getenv("DQN_FC1_SPLITS")) if (m[0]) c->fc1_big_splits = std::atoi(m);
    } else {
        (void)hipGetLastError();
    }
    // side stream at the default priority; if anything fails the step simply runs on one stream
    // (DQN_SINGLE_STREAM=1 in the environment keeps everything on the caller's stream)
    const char *single = std::getenv("DQN_SINGLE_STREAM");
    if ((single && single[0] == '1') || hipStreamCreateWithFlags(&c->side, hipStreamNonBlocking) != hipSuccess)
        c->side = nullptr;
    if (c->side && hipStreamCreateWithFlags(&c->side2, hipStreamNonBlocking) != hipSuccess) c->side2 = nullptr;
    // DQN_GRAPH=1 replays the step from a recorded HIP graph.  Off by default: on this runtime a
    // graph launch costs the host about as much as the plain launches it replaces and the
    // step is bound by the device either way.
    const char *graph = std::getenv("DQN_GRAPH");
    c->graph_off = !(graph && graph[0] == '1');
    if (!c->graph_off && hipStreamCreateWithFlags(&c->cap, hipStreamNonBlocking) != hipSuccess) c->cap = nullptr;
    hipEvent_t *evs[6] = {&c->ev_fork, &c->ev_a, &c->ev_b, &c->ev_c, &c->ev_join, &c->ev_join2};
    for (hipEvent_t *e : evs)
        if (c->side && hipEventCreateWithFlags(e, hipEventDisableTiming) != hipSuccess) {
            (void)hipStreamDestroy(c->side);
            if (c->side2) (void)hipStreamDestroy(c->side2);
            c->side = c->side2 = nullptr;
        }
    (void)hipGetLastError();
    *out = c;
    return DQN_OK;
}

int32_t dqn_destroy(dqn_ctx *ctx)
{
    if (!ctx) return DQN_OK;
    for (ProfRec &r : ctx->recs) {
        (void)hipEventDestroy(r.e0);
        (void)hipEventDestroy(r.e1);
    }
    if (!ctx->graphs.empty()) (void)hipDeviceSynchronize();  // no recording is destroyed while it may still run
    drop_graphs(ctx);
    for (hipStream_t sx : {ctx->side, ctx->side2, ctx->cap})
        if (sx) {
            (void)hipStreamSynchronize(sx);
            (void)hipStreamDestroy(sx);
        }
    for (hipEvent_t e : {ctx->ev_fork, ctx->ev_a, ctx->ev_b, ctx->ev_c, ctx->ev_join, ctx->ev_join2})
        if (e) (void)hipEventDestroy(e);
    delete ctx;
    return DQN_OK;
}

int32_t dqn_profile_begin(dqn_ctx *c)
{
    if (!c) return DQN_ERR_INVALID_ARG;
    c->prof = true;
    return DQN_OK;
}

int32_t dqn_profile_end(dqn_ctx *c, int32_t cap, const char **names, int64_t *counts, double *total_ms)
{
    if (!c || cap < 0 || (cap > 0 && (!names || !counts || !total_ms))) return DQN_ERR_INVALID_ARG;
    c->prof = false;
    if (hipDeviceSynchronize() != hipSuccess) return fail(c, DQN_ERR_HIP, "dqn_profile_end: synchronise failed");
    int32_t distinct = 0;
    for (ProfRec &r : c->recs) {
        float ms = 0.f;
        (void)hipEventElapsedTime(&ms, r.e0, r.e1);
        int32_t k = 0;
        for (; k < distinct && k < cap; ++k)
            if (names[k] == r.name || std::strcmp(names[k], r.name) == 0) break;
        if (k == distinct) {
            if (k < cap) { names[k] = r.name; counts[k] = 0; total_ms[k] = 0.0; }
            ++distinct;
        }
        if (k < cap) { counts[k] += 1; total_ms[k] += ms; }
        (void)hipEventDestroy(r.e0);
        (void)hipEventDestroy(r.e1);
    }
    c->recs.clear();
    return distinct;
}

int32_t dqn_get_params(dqn_ctx *c, int32_t which, float *dst, void *stream)
{
    if (!c) return DQN_ERR_INVALID_ARG;
    float *src = which_buffer(c, which);
    if (!src) return fail(c, which == 4 ? DQN_ERR_STATE : DQN_ERR_INVALID_ARG, "dqn_get_params: no such buffer");
    if (!dst || !aligned(dst, 16)) return fail(c, DQN_ERR_INVALID_ARG, "dqn_get_params: dst is NULL or misaligned");
    permute(c, src, dst, 1, (hipStream_t)stream);
    return hip_status(c, "dqn_get_params");
}

int32_t dqn_set_params(dqn_ctx *c, int32_t which, const float *src, void *stream)
{
    if (!c) return DQN_ERR_INVALID_ARG;
    float *dst = which_buffer(c, which);
    if (!dst) return fail(c, which == 4 ? DQN_ERR_STATE : DQN_ERR_INVALID_ARG, "dqn_set_params: no such buffer");
    if (!src || !aligned(src, 16)) return fail(c, DQN_ERR_INVALID_ARG, "dqn_set_params: src is NULL or misaligned");
    hipStream_t st = (hipStream_t)stream;
    permute(c, src, dst, 0, st);
    if (c->cfg.precision == 1 && which <= 1) {
        __hip_bfloat16 *sh = (__hip_bfloat16 *)c->buf.shadow_bf16;
        size_t half = align_up((size_t)c->n * 2, 256) / 2;
        misc::k_to_bf16<<<grid1(c->n, 256), 256, 0, st>>>(dst, sh + (which ? half : 0), c->n);
        if (which == 0) misc::k_w2_transposed<<<grid1(64 * 512, 256), 256, 0, st>>>(c->theta + net::C2W, (__hip_bfloat16 *)c->ws.w2t);
    }
    return hip_status(c, "dqn_set_params");
}

int32_t dqn_get_activations(dqn_ctx *c, int32_t layer, int32_t n, float *dst, void *stream)
{
    if (!c) return DQN_ERR_INVALID_ARG;
    if (layer < 1 || layer > 4) return fail(c, DQN_ERR_INVALID_ARG, "dqn_get_activations: layer must be 1..4");
    if (n < 1 || n > c->cfg.max_batch || !dst) return fail(c, DQN_ERR_INVALID_ARG, "dqn_get_activations: n out of range or dst NULL");
    const Workspace &w = c->ws;
    const void *src[4] = {w.act1, w.act2, w.act3, w.h_s};
    const int P[4] = {400, 81, 49, 1}, Cn[4] = {32, 64, 64, net::HID};
    const int k = layer - 1;
    const long total = (long)n * P[k] * Cn[k];
    hipStream_t st = (hipStream_t)stream;
    misc::k_read_act<<<grid1(total, 256), 256, 0, st>>>(src[k], k < 3 && c->cfg.precision == 1, n, P[k], Cn[k], dst);
    return hip_status(c, "dqn_get_activations");
}

int32_t dqn_selftest_fused_conv_schedule(int32_t ns)
{
    return gbf::c12::schedule_is_safe(ns);
}

int32_t dqn_sync_target(dqn_ctx *c, void *stream)
{
    if (!c) return DQN_ERR_INVALID_ARG;
    hipStream_t st = (hipStream_t)stream;
    if (hipMemcpyAsync(c->theta_t, c->theta, (size_t)c->n * 4, hipMemcpyDeviceToDevice, st) != hipSuccess)
        return fail(c, DQN_ERR_HIP, "dqn_sync_target: copy failed");
    if (c->cfg.precision == 1) {
        __hip_bfloat16 *sh = (__hip_bfloat16 *)c->buf.shadow_bf16;
        size_t half = align_up((size_t)c->n * 2, 256) / 2;
        if (hipMemcpyAsync(sh + half, sh, (size_t)c->n * 2, hipMemcpyDeviceToDevice, st) != hipSuccess)
            return fail(c, DQN_ERR_HIP, "dqn_sync_target: copy failed");
    }
    return DQN_OK;
}

// ------------------------------------------------------------ replay
int32_t per_fill(dqn_ctx *c, const float *priorities, int64_t n, void *stream)
{
    if (!c) return DQN_ERR_INVALID_ARG;
    if (c->cfg.replay_capacity <= 0) return fail(c, DQN_ERR_STATE, "per_fill: context has no replay");
    if (n < 0 || n > c->cfg.replay_capacity) return fail(c, DQN_ERR_INVALID_ARG, "per_fill: n out of range");
    if (n > 0 && (!priorities || !aligned(priorities, 16))) return fail(c, DQN_ERR_INVALID_ARG, "per_fill: priorities NULL or misaligned");
    hipStream_t st = (hipStream_t)stream;
    const long L = c->L;
    launch(c, "tree_leaves", st, [&] {
        misc::k_tree_leaves<<<grid1(L, 256), 256, 0, st>>>(c->tree, L, priorities, n, c->cfg.per_alpha);
    });
    rebuild_tree(c, st);
    c->envs = 0;
    c->sub = (long)c->cfg.replay_capacity;
    c->slot_limit = n;
    c->stored = n;
    c->seq = n;
    c->cursor = n % c->cfg.replay_capacity;
    c->leaves_all_one = c->cfg.per_alpha == 0.f && n <= (1 << 24);   // sums of ones are exact up to 2^24
    return hip_status(c, "per_fill");
}

int32_t per_sample(dqn_ctx *c, int32_t B, float beta, uint64_t draw_seed, int32_t *idx, float *is_w, void *stream)
{
    if (!c) return DQN_ERR_INVALID_ARG;
    if (c->cfg.replay_capacity <= 0 || c->stored <= 0) return fail(c, DQN_ERR_STATE, "per_sample: nothing stored");
    if (B < 1 || B > 1024) return fail(c, DQN_ERR_INVALID_ARG, "per_sample: B must be in 1..1024");
    if (!idx || !is_w || !aligned(idx, 4) || !aligned(is_w, 4)) return fail(c, DQN_ERR_INVALID_ARG, "per_sample: NULL or misaligned output");
    if (!(beta >= 0.f)) return fail(c, DQN_ERR_INVALID_ARG, "per_sample: beta must be >= 0");
    hipStream_t st = (hipStream_t)stream;
    launch(c, "per_sample", st, [&] {
        misc::k_per_sample<<<(B + 3) / 4, 256, 0, st>>>(misc::SampleArgs{
            c->tree, c->L, c->levels, c->stored, B, beta, draw_seed, c->cfg.per_stratified, idx, is_w, misc::MetaGather{},
            uniform_replay(c), c->slot_limit});
    });
    launch(c, "per_normalise", st, [&] { misc::k_per_normalise<<<1, 1024, 0, st>>>(is_w, B); });
    return hip_status(c, "per_sample");
}

int32_t per_update(dqn_ctx *c, const int32_t *idx, const float *td_abs, int32_t n, void *stream)
{
    if (!c) return DQN_ERR_INVALID_ARG;
    if (c->cfg.replay_capacity <= 0 || c->stored <= 0) return fail(c, DQN_ERR_STATE, "per_update: nothing stored");
    if (n < 1 || n > 1024) return fail(c, DQN_ERR_INVALID_ARG, "per_update: n must be in 1..1024");
    if (!idx || !td_abs) return fail(c, DQN_ERR_INVALID_ARG, "per_update: NULL argument");
    hipStream_t st = (hipStream_t)stream;
    launch(c, "per_update", st, [&] {
        misc::k_per_update<<<1, (n + 63) / 64 * 64, 0, st>>>(
            misc::PerUpdateArgs{c->tree, c->L, c->levels, c->slot_limit, idx, td_abs, n, c->cfg.per_alpha, c->cfg.per_eps, 0});
    });
    return hip_status(c, "per_update");
}

int32_t dqn_replay_write(dqn_ctx *c, int64_t slot0, int64_t n, const uint8_t *frames, const int32_t *a,
                         const float *r, const uint8_t *done, void *stream)
{
    if (!c) return DQN_ERR_INVALID_ARG;
    const int64_t cap = c->cfg.replay_capacity;
    if (cap <= 0) return fail(c, DQN_ERR_STATE, "dqn_replay_write: context has no replay");
    if (slot0 < 0 || slot0 >= cap || n < 1 || n > cap) return fail(c, DQN_ERR_INVALID_ARG, "dqn_replay_write: slot range out of bounds");
    if (!frames || !aligned(frames, 16)) return fail(c, DQN_ERR_INVALID_ARG, "dqn_replay_write: frames NULL or not 16-byte aligned");
    hipStream_t st = (hipStream_t)stream;
    launch(c, "replay_write", st, [&] {
        misc::k_replay_write<<<dim3((unsigned)n), 256, 0, st>>>((uint8_t *)c->buf.replay_frames, c->meta_a, c->meta_r,
                                                                c->meta_done, cap, slot0, frames, a, r, done);
    });
    return hip_status(c, "dqn_replay_write");
}

int32_t dqn_replay_store(dqn_ctx *c, int64_t n, const uint8_t *frames, const int32_t *a, const float *r,
                         const uint8_t *done, void *stream)
{
    if (!c) return DQN_ERR_INVALID_ARG;
    const int64_t cap = c->cfg.replay_capacity;
    if (cap <= 0) return fail(c, DQN_ERR_STATE, "dqn_replay_store: context has no replay");
    if (cap < 16) return fail(c, DQN_ERR_STATE, "dqn_replay_store: needs a ring of at least 16 slots");
    if (c->envs > 0) return fail(c, DQN_ERR_STATE, "dqn_replay_store: the ring holds many environment streams (dqn_replay_store_envs); per_fill resets it");
    if (n < 1 || n > 1020 || n > cap - 8) return fail(c, DQN_ERR_INVALID_ARG, "dqn_replay_store: n must be in 1..min(1020, capacity-8)");
    if (!frames || !aligned(frames, 16) || !a || !r || !done)
        return fail(c, DQN_ERR_INVALID_ARG, "dqn_replay_store: NULL argument or frames not 16-byte aligned");
    hipStream_t st = (hipStream_t)stream;
    const int64_t h0 = c->cursor;
    launch(c, "replay_write", st, [&] {
        misc::k_replay_write<<<dim3((unsigned)n), 256, 0, st>>>((uint8_t *)c->buf.replay_frames, c->meta_a, c->meta_r,
                                                                c->meta_done, cap, h0, frames, a, r, done);
    });
    launch(c, "store_priorities", st, [&] {
        misc::k_store_priorities<<<1, (int)((n + 4 + 63) / 64 * 64), 0, st>>>(c->tree, c->L, c->levels, cap, h0, c->seq,
                                                                             (int)n, c->meta_done, c->cfg.per_alpha);
    });
    c->leaves_all_one = false;
    c->cursor = (h0 + n) % cap;
    c->seq += n;
    c->stored = std::min<int64_t>(c->seq, cap);
    c->slot_limit = c->stored;
    return hip_status(c, "dqn_replay_store");
}

int32_t dqn_replay_store_envs(dqn_ctx *c, int32_t E, const uint8_t *frames, const int32_t *a, const float *r,
                              const uint8_t *done, void *stream)
{
    if (!c) return DQN_ERR_INVALID_ARG;
    const int64_t cap = c->cfg.replay_capacity;
    if (cap <= 0) return fail(c, DQN_ERR_STATE, "dqn_replay_store_envs: context has no replay");
    if (E < 1 || cap / E < 16) return fail(c, DQN_ERR_INVALID_ARG, "dqn_replay_store_envs: E must be in 1..capacity/16");
    if (!frames || !aligned(frames, 16) || !a || !r || !done)
        return fail(c, DQN_ERR_INVALID_ARG, "dqn_replay_store_envs: NULL argument or frames not 16-byte aligned");
    if (c->envs == 0 && c->seq != 0)
        return fail(c, DQN_ERR_STATE, "dqn_replay_store_envs: the ring already holds one stream; start from an empty context");
    if (c->envs != 0 && c->envs != E) return fail(c, DQN_ERR_INVALID_ARG, "dqn_replay_store_envs: the number of streams is fixed by the first call");
    hipStream_t st = (hipStream_t)stream;
    const long C = (long)(cap / E);
    const long t = (long)c->seq, l = t % C;
    // two launches: the time steps with the leaves they settle, then the tree above the leaves
    launch(c, "replay_write", st, [&] {
        misc::k_replay_write_envs<<<dim3((unsigned)E), 256, 0, st>>>((uint8_t *)c->buf.replay_frames, c->meta_a, c->meta_r,
                                                                     c->meta_done, C, l, frames, a, r, done, c->tree, c->L,
                                                                     t, c->cfg.per_alpha);
    });
    rebuild_tree(c, st);
    c->envs = E;
    c->sub = C;
    c->slot_limit = (long)E * C;
    c->leaves_all_one = false;
    c->seq += 1;
    c->cursor = c->seq % C;
    c->stored = (long)E * std::min<int64_t>(c->seq, C);
    return hip_status(c, "dqn_replay_store_envs");
}

int32_t dqn_replay_state(const dqn_ctx *c, int64_t *cursor, int64_t *stored, int64_t *steps)
{
    if (!c) return DQN_ERR_INVALID_ARG;
    if (cursor) *cursor = c->cursor;
    if (stored) *stored = c->stored;
    if (steps) *steps = c->seq;
    return DQN_OK;
}

int32_t dqn_preprocess(const uint8_t *raw, int64_t n, int32_t height, int32_t width, const float *grey_lut,
                       uint8_t *frames, void *stream)
{
    if (!raw || !frames) return fail(nullptr, DQN_ERR_INVALID_ARG, "dqn_preprocess: NULL argument");
    if (n < 1 || n > 65535 || height < 1 || width < 1 || height > 4096 || width > 4096)
        return fail(nullptr, DQN_ERR_INVALID_ARG, "dqn_preprocess: n must be in 1..65535, height and width in 1..4096");
    hipStream_t st = (hipStream_t)stream;
    misc::k_preprocess<<<dim3((net::FRAME + 255) / 256, (unsigned)n), 256, 0, st>>>(raw, height, width, grey_lut, frames);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return fail(nullptr, DQN_ERR_HIP, std::string("dqn_preprocess: ") + hipGetErrorString(e));
    return DQN_OK;
}

int32_t dqn_schedule_default(dqn_schedule *s)
{
    if (!s) return DQN_ERR_INVALID_ARG;
    s->learning_start = 50000; s->update_period = 4; s->target_period = 30000;
    s->eps_steps = 5000000; s->beta_steps = 100000000;
    s->eps_start = 1.0f; s->eps_end = 0.1f; s->beta_start = 0.4f; s->beta_end = 1.0f;
    return DQN_OK;
}

int32_t dqn_schedule_at(const dqn_schedule *s, int64_t step, dqn_schedule_point *out)
{
    if (!s || !out || step < 1 || s->update_period < 1 || s->target_period < 1) return DQN_ERR_INVALID_ARG;
    auto ramp = [](double a, double b, int64_t t, int64_t T) {
        if (T <= 1 || t >= T) return b;
        return a + (b - a) * (double)(t - 1) / (double)(T - 1);
    };
    out->epsilon = (float)ramp(s->eps_start, s->eps_end, step, s->eps_steps);
    out->beta = (float)ramp(s->beta_start, s->beta_end, step, s->beta_steps);
    out->train = step > s->learning_start && step % s->update_period == 0;
    out->sync_target = step % s->target_period == 0;
    return DQN_OK;
}

int32_t dqn_replay_gather(dqn_ctx *c, const int32_t *idx, int32_t n, uint8_t *s, uint8_t *s_next, int32_t *a,
                          float *r, uint8_t *done, void *stream)
{
    if (!c) return DQN_ERR_INVALID_ARG;
    if (c->cfg.replay_capacity <= 0) return fail(c, DQN_ERR_STATE, "dqn_replay_gather: context has no replay");
    if (n < 1 || n > c->cfg.max_batch || !idx) return fail(c, DQN_ERR_INVALID_ARG, "dqn_replay_gather: n out of range or idx NULL");
    if ((s && !aligned(s, 16)) || (s_next && !aligned(s_next, 16))) return fail(c, DQN_ERR_INVALID_ARG, "dqn_replay_gather: outputs must be 16-byte aligned");
    hipStream_t st = (hipStream_t)stream;
    misc::GatherArgs G{(const uint8_t *)c->buf.replay_frames, c->meta_a, c->meta_r, c->meta_done,
                       (long)c->cfg.replay_capacity, idx, nullptr, s, s_next, a, r, done, c->sub};
    launch(c, "gather", st, [&] { misc::k_gather<<<dim3(n, 5), 256, 0, st>>>(G); });
    return hip_status(c, "dqn_replay_gather");
}

// ------------------------------------------------------------ acting
int32_t dqn_act(dqn_ctx *c, const uint8_t *obs, int32_t E, float epsilon, uint64_t draw_seed, int32_t *actions,
                float *q_opt, void *stream)
{
    if (!c) return DQN_ERR_INVALID_ARG;
    if (E < 1 || E > c->cfg.max_act_batch) return fail(c, DQN_ERR_INVALID_ARG, "dqn_act: E out of range");
    if (!obs || !actions || !aligned(obs, 16)) return fail(c, DQN_ERR_INVALID_ARG, "dqn_act: NULL or misaligned argument");
    if (!(epsilon >= 0.f && epsilon <= 1.f)) return fail(c, DQN_ERR_INVALID_ARG, "dqn_act: epsilon must be in [0,1]");
    hipStream_t st = (hipStream_t)stream;
    Pass p{obs, net::STATE, 0, E, nullptr, 0};
    int ns;
    long ss;
    int32_t rc = forward_trunk(c, c->ws, &p, 1, &ns, &ss, st);
    if (rc) return rc;
    misc::HeadActArgs H{c->ws.f1part, ns, ss, E, c->cfg.num_actions, c->cfg.dueling, c->theta + net::F1B,
                        c->theta + net::HEAD, epsilon, draw_seed, actions, q_opt};
    if (ns < 1 || ns > misc::HEAD_MAX_SPLITS) return fail(c, DQN_ERR_STATE, "dqn_act: unexpected number of fc1 reduction splits");
    launch(c, "head_act", st, [&] { misc::launch_head_act(H, st); });
    return hip_status(c, "dqn_act");
}

int32_t dqn_act_static(dqn_ctx *c, const uint8_t *obs, int32_t E, float epsilon, uint64_t draw_seed,
                       int32_t *actions, float *q_opt, void *stream)
{
    if (!c) return DQN_ERR_INVALID_ARG;
    if (E < 1 || E > DQN_ACT_STATIC_MAX)
        return fail(c, DQN_ERR_INVALID_ARG, "dqn_act_static: E must be in 1..DQN_ACT_STATIC_MAX (32): the static scratch array holds no more");
    if (!obs || !actions || !aligned(obs, 16)) return fail(c, DQN_ERR_INVALID_ARG, "dqn_act_static: NULL or misaligned argument");
    if (!(epsilon >= 0.f && epsilon <= 1.f)) return fail(c, DQN_ERR_INVALID_ARG, "dqn_act_static: epsilon must be in [0,1]");
    uint8_t *base = scratch_of_current_device();
    if (!base) return fail(c, DQN_ERR_HIP, "dqn_act_static: the address of the static scratch array is not available on this device");
    // a view of the scratch array laid out like the part of the workspace that acting uses; every word a
    // kernel reads from it has been written by an earlier kernel of this call, so nothing is cleared
    Workspace w{};
    const size_t es = c->cfg.precision == 1 ? 2 : 4, n = DQN_ACT_STATIC_MAX;
    size_t off = 0;
    auto take = [&](size_t bytes) { uint8_t *q = base + off; off += align_up(bytes, 256); return q; };
    w.act1 = take(n * net::A1 * es);
    w.act2 = take(n * net::A2 * es);
    w.act3 = take(n * net::A3 * es);
    w.f1part = (float *)take(n * 14 * net::HID * 4);
    w.f1rows = n * 14;
    static_assert(DQN_ACT_STATIC_MAX * (size_t)(net::A1 + net::A2 + net::A3) * 4 + DQN_ACT_STATIC_MAX * 14 * (size_t)net::HID * 4 + 4 * 256
                      <= SCRATCH_BYTES, "scratch array too small");
    hipStream_t st = (hipStream_t)stream;
    Pass p{obs, net::STATE, 0, E, nullptr, 0};
    int ns;
    long ss;
    const bool prof = c->prof;   // per-kernel timing creates events: not on this path
    c->prof = false;
    int32_t rc = forward_trunk(c, w, &p, 1, &ns, &ss, st);
    if (rc == DQN_OK) {
        misc::HeadActArgs H{w.f1part, ns, ss, E, c->cfg.num_actions, c->cfg.dueling, c->theta + net::F1B,
                            c->theta + net::HEAD, epsilon, draw_seed, actions, q_opt};
        if (ns < 1 || ns > misc::HEAD_MAX_SPLITS) {
            c->prof = prof;
            return fail(c, DQN_ERR_STATE, "dqn_act_static: unexpected number of fc1 reduction splits");
        }
        misc::launch_head_act(H, st);
        rc = hip_status(c, "dqn_act_static");
    }
    c->prof = prof;
    return rc;
}

// ------------------------------------------------------------ training
static misc::SampleArgs sample_args(dqn_ctx *c, int32_t B, float beta, uint64_t draw_seed)
{
    const Workspace &w = c->ws;
    // raw importance weights; the head kernel divides by their maximum
    return misc::SampleArgs{c->tree, c->L, c->levels, c->stored, B, beta, draw_seed, c->cfg.per_stratified,
                            w.b_idx, w.b_w,
                            misc::MetaGather{c->meta_a, c->meta_r, c->meta_done, w.b_a, w.b_r, w.b_done}, uniform_replay(c),
                            c->slot_limit};
}

// The sampling kernel of a replay-mode step.  The fp32 path copies the drawn frame stacks next
// (its conv1 reads a materialised stack): there the two are one launch.
static void enqueue_sample(dqn_ctx *c, int32_t B, float beta, uint64_t draw_seed, hipStream_t st)
{
    const misc::SampleArgs S = sample_args(c, B, beta, draw_seed);
    if (c->cfg.precision == 0) {
        misc::GatherArgs G{(const uint8_t *)c->buf.replay_frames, c->meta_a, c->meta_r, c->meta_done,
                           (long)c->cfg.replay_capacity, c->ws.b_idx, c->ws.stack5, nullptr, nullptr, nullptr, nullptr, nullptr,
                           c->sub};
        launch(c, "sample_gather", st, [&] { misc::k_sample_gather<<<dim3(B, 5), 256, 0, st>>>(S, G); });
        return;
    }
    launch(c, "per_sample", st, [&] { misc::k_per_sample<<<(B + 3) / 4, 256, 0, st>>>(S); });
}

// Enqueues every kernel of one training step on st (and on the side streams, which fork from
// st and join it again before the function returns).  In replay mode the sampling kernel has
// been enqueued by the caller.
// draw != nullptr (bf16 replay mode): no sampling kernel has run, the first forward kernel draws.
static int32_t enqueue_step(dqn_ctx *c, int32_t B, const dqn_batch *batch, const dqn_step_out *out, hipStream_t st,
                            const misc::SampleArgs *draw = nullptr)
{
    const dqn_config &cfg = c->cfg;
    const Workspace &w = c->ws;
    dqn_step_out O{};
    if (out) O = *out;

    const uint8_t *s, *sn;
    const int32_t *ring_idx = nullptr;
    long xs;
    const int32_t *a;
    const float *r, *isw;
    const uint8_t *done;
    if (batch) {
        if (!batch->s || !batch->s_next || !batch->a || !batch->r || !batch->done)
            return fail(c, DQN_ERR_INVALID_ARG, "dqn_train_step: batch has a NULL member");
        if (!aligned(batch->s, 16) || !aligned(batch->s_next, 16))
            return fail(c, DQN_ERR_INVALID_ARG, "dqn_train_step: states must be 16-byte aligned");
        s = batch->s; sn = batch->s_next; xs = net::STATE;
        a = batch->a; r = batch->r; done = batch->done; isw = batch->w;
    } else {
        a = w.b_a; r = w.b_r; done = w.b_done; isw = w.b_w;
        if (cfg.precision == 1 || draw) {
            // the conv1 forward kernel reads the five frames of a transition straight from the ring (bf16: so
            // does the conv1 weight gradient; fp32: the forward kernel leaves it a gathered copy)
            ring_idx = w.b_idx;
            s = sn = (const uint8_t *)c->buf.replay_frames; xs = 0;
        } else {
            // the frame stacks were copied by the sampling launch
            s = w.stack5; sn = w.stack5 + net::FRAME; xs = 5 * net::FRAME;
        }
    }
    const bool stacking = !batch && cfg.precision == 0 && draw;

    // forward: online(s), online(s'), target(s') in one launch per layer
    Pass passes[3] = {{s, xs, 0, B, ring_idx, 0, stacking ? w.stack5 : nullptr, 1},
                      {sn, xs, 0, B, ring_idx, 1, stacking ? w.stack5 : nullptr, 2},
                      {sn, xs, 1, B, ring_idx, 1, nullptr, 0}};
    int ns;
    long ss;
    int32_t rc = forward_trunk(c, w, passes, 3, &ns, &ss, st, draw);
    if (rc) return rc;
    // the drawn indices exist once the sampling kernel, or the first forward kernel, has run
    if (!batch && O.idx && hipMemcpyAsync(O.idx, w.b_idx, (size_t)B * 4, hipMemcpyDeviceToDevice, st) != hipSuccess)
        return fail(c, DQN_ERR_HIP, "dqn_train_step: copy failed");

    misc::HeadArgs H{};
    H.part = w.f1part; H.nsplit = ns; H.split_stride = ss;
    H.B = B; H.K = cfg.num_actions; H.dueling = cfg.dueling; H.double_q = cfg.double_q; H.loss_kind = cfg.loss_kind;
    H.kappa = cfg.huber_delta; H.gamma = cfg.gamma;
    H.f1b_on = c->theta + net::F1B; H.f1b_tg = c->theta_t + net::F1B;
    H.head_on = c->theta + net::HEAD; H.head_tg = c->theta_t + net::HEAD;
    H.a = a; H.r = r; H.done = done; H.w = isw; H.w_raw = batch ? 0 : 1;
    H.h_s = w.h_s; H.dh = w.dh; H.dh_bf16 = cfg.precision == 1; H.dA = w.dA; H.td_abs = w.td_abs; H.loss_j = w.loss_j;
    H.qmax_j = w.qmax_j;
    H.q_s = O.q_s; H.q_no = O.q_next_online; H.q_nt = O.q_next_target; H.y = O.y; H.td = O.td;
    H.a_star = O.a_star; H.is_w = O.is_w;
    if (ns < 1 || ns > misc::HEAD_MAX_SPLITS) return fail(c, DQN_ERR_STATE, "dqn_train_step: unexpected number of fc1 reduction splits");
    launch(c, "head_train", st, [&] {
        switch (ns) {
        case 1: misc::k_head_train<1><<<B, 512, 0, st>>>(H); break;
        case 2: misc::k_head_train<2><<<B, 512, 0, st>>>(H); break;
        case 3: misc::k_head_train<3><<<B, 512, 0, st>>>(H); break;
        case 4: misc::k_head_train<4><<<B, 512, 0, st>>>(H); break;
        case 5: misc::k_head_train<5><<<B, 512, 0, st>>>(H); break;
        case 6: misc::k_head_train<6><<<B, 512, 0, st>>>(H); break;
        default: misc::k_head_train<7><<<B, 512, 0, st>>>(H); break;
        }
    });

    // large fp32 batches fork: the weight gradients of the trunk go to one side stream, the head
    // weight gradient and the priority update to another; they join again before the optimizer.
    // Their kernels are long enough (50-120 us) to repay the events; everything else stays on st
    // with one backward launch per layer.
    // measured: 645 against 665 us/step at B = 512 with the streams, 547 against 536 at 384, 277 against 245 at 128
    const bool multi = c->side && cfg.precision == 0 && B > 448;
    hipStream_t sd = multi ? c->side : st;
    hipStream_t sp = multi ? (c->side2 ? c->side2 : c->side) : st;
    if (sd != st || sp != st) (void)hipEventRecord(c->ev_fork, st);
    ev_wait(sd, c->ev_fork, st);
    if (sp != sd) ev_wait(sp, c->ev_fork, st);
    misc::HeadWgradArgs HW{w.dA, w.h_s, w.loss_j, c->gp5, O.loss, w.loss_slot, B, cfg.num_actions, cfg.dueling,
                           w.td_abs, w.qmax_j, O.td_abs_mean, O.q_max_mean};
    // the indices come from the sampling kernel, so the ring capacity bounds them
    misc::PerUpdateArgs PU{c->tree, c->L, c->levels, (long)cfg.replay_capacity, w.b_idx, w.td_abs, B,
                           cfg.per_alpha, cfg.per_eps, uniform_replay(c)};
    // one stream: they ride in the launches of the backward pass (see backward_bf16, backward_f32)
    SmallTail tail{HW, PU, !batch};
    const bool fuse_tail = sd == st;
    if (!fuse_tail) {
        launch(c, "head_wgrad", sp, [&] { misc::k_head_wgrad<<<dim3(c->R, 16), 512, 0, sp>>>(HW); });
        if (!batch) launch(c, "per_update", sp, [&] { misc::k_per_update<<<1, (B + 63) / 64 * 64, 0, sp>>>(PU); });
    }
    if (sp != sd) (void)hipEventRecord(c->ev_join2, sp);

    int ns1, ns2, ns3;
    // bf16: the update in four parts: beside fc1's, conv3's and conv2's gradients and inside the RMSProp launch
    const int lv = c->levels;
    // (of 20 levels: 2, 5, 7 and 6; the RMSProp launch is the one its part can outlast, fc1's the shortest)
    const SplitUpdate U{PU, w.pu_state, {lv / 10, 7 * lv / 20, 7 * lv / 10}, batch ? 0 : 1};
    if (cfg.precision == 1) backward_bf16(c, B, passes[0], &ns1, &ns2, &ns3, st, HW, U);
    else backward_f32(c, B, stacking ? w.stack5 : s, stacking ? 5L * net::FRAME : xs, &ns1, &ns2, &ns3, st, sd,
                      fuse_tail ? &tail : nullptr);
    ev_record(c->ev_join, sd, st);
    ev_wait(st, c->ev_join, sd);
    if (sp != sd) (void)hipStreamWaitEvent(st, c->ev_join2, 0);

    launch_rmsprop(c, RMS_ALL, ns1, ns2, ns3, st, cfg.precision == 1 ? &U : nullptr);
    return hip_status(c, "dqn_train_step");
}

// Records the replay-mode step for batch size B (everything after the sampling kernel, with the
// outputs staged in the workspace); returns nullptr if this runtime cannot do it.
static dqn_ctx::StepGraph *record_step_graph(dqn_ctx *c, int32_t B)
{
    const Workspace &w = c->ws;
    const size_t BK = (size_t)c->cfg.max_batch * c->cfg.num_actions;
    dqn_step_out O{};
    O.loss = w.o_loss; O.q_s = w.o_q; O.q_next_online = w.o_q + BK; O.q_next_target = w.o_q + 2 * BK;
    O.y = w.o_y; O.td = w.o_td; O.a_star = w.o_astar; O.is_w = w.o_isw;  // idx: already in b_idx
    O.td_abs_mean = w.o_loss + 1; O.q_max_mean = w.o_loss + 2;
    if (hipStreamBeginCapture(c->cap, hipStreamCaptureModeRelaxed) != hipSuccess) {
        (void)hipGetLastError();
        return nullptr;
    }
    const int32_t rc = enqueue_step(c, B, nullptr, &O, c->cap);
    hipGraph_t g = nullptr;
    const hipError_t e = hipStreamEndCapture(c->cap, &g);
    hipGraphExec_t x = nullptr;
    if (rc != DQN_OK || e != hipSuccess || !g || hipGraphInstantiate(&x, g, nullptr, nullptr, 0) != hipSuccess) {
        if (g) (void)hipGraphDestroy(g);
        (void)hipGetLastError();
        return nullptr;
    }
    c->graphs.push_back({B, g, x});
    return &c->graphs.back();
}

int32_t dqn_train_step(dqn_ctx *c, int32_t B, const dqn_batch *batch, float beta, uint64_t draw_seed,
                       const dqn_step_out *out, void *stream)
{
    if (!c) return DQN_ERR_INVALID_ARG;
    if (B < 1 || B > c->cfg.max_batch) return fail(c, DQN_ERR_INVALID_ARG, "dqn_train_step: B out of range");
    hipStream_t st = (hipStream_t)stream;
    if (batch) return enqueue_step(c, B, batch, out, st);
    if (c->cfg.replay_capacity <= 0 || c->stored <= 0) return fail(c, DQN_ERR_STATE, "dqn_train_step: replay is empty");
    if (!(beta >= 0.f)) return fail(c, DQN_ERR_INVALID_ARG, "dqn_train_step: beta must be >= 0");
    const bool graphs = !c->prof && !c->graph_off && c->cap && c->side;
    if (!graphs && !in_kernel_draw_fits(c, B)) {
        enqueue_sample(c, B, beta, draw_seed, st);
        return enqueue_step(c, B, nullptr, out, st);
    }
    if (!graphs) {
        // the first forward kernel draws the transitions (and, in fp32, gathers their frames for the
        // weight gradient): one launch less on the critical path
        const misc::SampleArgs S = sample_args(c, B, beta, draw_seed);
        return enqueue_step(c, B, nullptr, out, st, &S);
    }
    enqueue_sample(c, B, beta, draw_seed, st);

    dqn_ctx::StepGraph *g = nullptr;
    if (graphs) {
        for (dqn_ctx::StepGraph &x : c->graphs)
            if (x.B == B) g = &x;
        if (!g && c->graphs.size() < MAX_STEP_GRAPHS) {
            g = record_step_graph(c, B);
            if (!g) c->graph_off = true;  // this runtime cannot record the step: plain launches from now on
        }
    }
    if (!g) return enqueue_step(c, B, nullptr, out, st);

    if (hipGraphLaunch(g->exec, st) != hipSuccess) {
        c->graph_off = true;
        return fail(c, DQN_ERR_HIP, std::string("dqn_train_step: graph launch: ") + hipGetErrorString(hipGetLastError()));
    }
    if (out) {  // hand the staged outputs to the caller
        const Workspace &w = c->ws;
        const size_t BK = (size_t)c->cfg.max_batch * c->cfg.num_actions;
        const int nq = B * c->cfg.num_actions;
        misc::CopyOutArgs A{};
        int n = 0;
        auto add = [&](void *dst, const void *src, int words) {
            if (dst) A.item[n++] = {(uint32_t *)dst, (const uint32_t *)src, words};
        };
        add(out->loss, w.o_loss, 1);
        add(out->q_s, w.o_q, nq);
        add(out->q_next_online, w.o_q + BK, nq);
        add(out->q_next_target, w.o_q + 2 * BK, nq);
        add(out->y, w.o_y, B);
        add(out->td, w.o_td, B);
        add(out->a_star, w.o_astar, B);
        add(out->idx, w.b_idx, B);
        add(out->is_w, w.o_isw, B);
        add(out->td_abs_mean, w.o_loss + 1, 1);
        add(out->q_max_mean, w.o_loss + 2, 1);
        if (n) misc::k_copy_out<<<dim3((nq + 255) / 256, n), 256, 0, st>>>(A);
    }
    return hip_status(c, "dqn_train_step");
}

}  // extern "C"
