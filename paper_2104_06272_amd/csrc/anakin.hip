// Host side of libanakin: the C ABI, configuration checks, workspace layout,
// one-time initialisation (parameters, env states, mazes) and the step
// scheduler.  The host only enqueues a fixed kernel sequence on one stream
// (paper section 3.1: the host "is exclusively used to schedule"); all state
// stays in the caller's device workspace between calls (section 2.3).
#include <math.h>
#include <stdlib.h>
#include <string.h>
#include <mutex>
#include <new>
#include <vector>
#include <utility>
#include "internal.h"

using namespace ank;

static thread_local std::string g_create_error;

// ---- the library's own update scratch, for callers that cannot allocate (anakin_learn_static) --------------
// One array per GPU (every device that loads the library holds its own copy until the process ends).  In host
// code the array's name is only a stand-in: its device address is asked for once per device, with that device
// current, and kept here; kernels receive that address like any other scratch pointer.
static __device__ __align__(256) unsigned char scratch[ANAKIN_STATIC_SCRATCH_BYTES];
constexpr int MAX_DEVICES = 64;
static std::mutex g_scratch_mutex;
static void* g_scratch_ptr[MAX_DEVICES];

static hipError_t resolve_static_scratch(int device)
{
    if (device < 0 || device >= MAX_DEVICES) return hipErrorInvalidDevice;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (g_scratch_ptr[device]) return hipSuccess;
    int current = -1;
    hipError_t e = hipGetDevice(&current);
    if (e != hipSuccess) return e;
    if (current != device && (e = hipSetDevice(device)) != hipSuccess) return e;
    void* p = nullptr;
    e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (current != device) (void)hipSetDevice(current);
    if (e != hipSuccess) return e;
    g_scratch_ptr[device] = p;
    return hipSuccess;
}

namespace ank { void fill_rollout_args(anakin* h, RolloutArgs& a); }

static size_t align256(size_t x) { return (x + 255) & ~(size_t)255; }

static bool is_pow2_in(int v, int lo, int hi) { return v >= lo && v <= hi && (v & (v - 1)) == 0; }

// ---- configuration -------------------------------------------------------
static int build_shapes(const anakin_env_cfg* env, const anakin_net_cfg* net, int B, int T,
                        EnvDims& ed, NetShape& ns, std::string& err)
{
    if (!env || !net) { err = "null configuration"; return ANAKIN_E_INVALID_ARG; }
    if (B <= 0 || T <= 0 || B % 16 != 0) { err = "B must be a positive multiple of 16 and T positive"; return ANAKIN_E_BAD_CONFIG; }
    if ((long long)B * (T + 1) >= (1ll << 30)) { err = "B*(T+1) too large"; return ANAKIN_E_BAD_CONFIG; }
    ed.kind = env->kind; ed.rows = env->rows; ed.cols = env->cols; ed.max_steps = env->max_steps;
    memset(&ns, 0, sizeof ns);
    if (env->kind == ANAKIN_ENV_CATCH) {
        if (env->rows < 2 || env->cols < 1 || env->rows > 255 || env->cols > 255) { err = "catch: rows in 2..255, cols in 1..255"; return ANAKIN_E_BAD_CONFIG; }
        ns.D = env->rows * env->cols; ns.A = 3;
    } else if (env->kind == ANAKIN_ENV_PENDULUM) {
        if (env->max_steps < 1) { err = "pendulum: max_steps >= 1"; return ANAKIN_E_BAD_CONFIG; }
        ns.D = 3; ns.A = 1;
    } else if (env->kind == ANAKIN_ENV_MAZE) {
        if (env->rows < 2 || env->cols < 2 || env->rows * env->cols > 256 || env->max_steps < 1 || env->max_steps > 65535 ||
            !(env->p_wall >= 0.0f && env->p_wall < 1.0f)) { err = "maze: 4..256 cells, max_steps in 1..65535, p_wall in [0,1)"; return ANAKIN_E_BAD_CONFIG; }
        ns.D = 3 * env->rows * env->cols; ns.A = 4;
    } else { err = "unknown env kind"; return ANAKIN_E_BAD_CONFIG; }
    if (net->policy != ANAKIN_POLICY_CATEGORICAL && net->policy != ANAKIN_POLICY_TANH_GAUSSIAN) { err = "unknown policy"; return ANAKIN_E_BAD_CONFIG; }
    if ((net->policy == ANAKIN_POLICY_TANH_GAUSSIAN) != (env->kind == ANAKIN_ENV_PENDULUM)) { err = "tanh-gaussian policy goes with the pendulum, categorical with catch and maze"; return ANAKIN_E_BAD_CONFIG; }
    if (net->dtype != ANAKIN_DTYPE_FP32 && net->dtype != ANAKIN_DTYPE_BF16) { err = "unknown dtype"; return ANAKIN_E_BAD_CONFIG; }
    if (net->n_hidden < 1 || net->n_hidden > MAX_LAYERS) { err = "n_hidden in 1..4"; return ANAKIN_E_BAD_CONFIG; }
    ns.L = net->n_hidden; ns.policy = net->policy; ns.bf16 = net->dtype == ANAKIN_DTYPE_BF16;
    ns.NH = net->policy == ANAKIN_POLICY_CATEGORICAL ? ns.A + 1 : 3;
    ns.NHP = ns.NH <= 4 ? 4 : 8;
    ns.dims[0] = ns.D;
    for (int l = 0; l < ns.L; ++l) {
        if (!is_pow2_in(net->hidden[l], 32, 1024)) { err = "hidden widths must be powers of two in 32..1024"; return ANAKIN_E_BAD_CONFIG; }
        ns.dims[l + 1] = net->hidden[l];
    }
    long long off = 0;
    for (int l = 0; l < ns.L; ++l) {
        ns.w_off[l] = (int)off; off += (long long)ns.dims[l] * ns.dims[l + 1];
        ns.b_off[l] = (int)off; off += ns.dims[l + 1];
    }
    ns.wh_off = (int)off; off += (long long)ns.dims[ns.L] * ns.NH;
    ns.bh_off = (int)off; off += ns.NH;
    ns.P = (int)off;
    if (!(net->gamma >= 0.0f && net->gamma <= 1.0f) || !(net->lambda_ >= 0.0f && net->lambda_ <= 1.0f) ||
        !(net->lr > 0.0f) || !(net->beta1 >= 0.0f && net->beta1 < 1.0f) || !(net->beta2 >= 0.0f && net->beta2 < 1.0f) ||
        !(net->eps > 0.0f)) { err = "hyper-parameters out of range"; return ANAKIN_E_BAD_CONFIG; }
    if (rollout_pick_tile(ns, B) == 0) { err = "no rollout tile fits B and the hidden widths"; return ANAKIN_E_BAD_CONFIG; }
    return ANAKIN_OK;
}

// split-K factor for a reduction over M samples feeding `tiles` output tiles:
// chunks are multiples of 16 rows; aim for about 1024 workgroups, at most max_splits splits
static int pick_splits(int M, int tiles, int max_splits, int quantum = 16)
{
    int cap = 1024 / (tiles > 0 ? tiles : 1);
    if (cap > max_splits) cap = max_splits;
    if (cap < 1) cap = 1;
    int s = M / quantum;
    while (s > cap && s % 2 == 0) s /= 2;
    return s > 0 ? s : 1;
}

// largest split count <= cap whose chunks are whole multiples of `quantum` rows (1 if none)
static int pick_divisor_splits(int M, int quantum, int cap)
{
    for (int s = cap; s > 1; --s) if (M % (s * quantum) == 0) return s;
    return M % quantum == 0 ? 1 : 0;
}

// The scratch of the backward pass: per-sample head gradients, dZ_l, split-K partial sums, first-stage partials
// of the head gradient.  Nothing here outlives one update and every byte is written before it is read.  Offsets
// are placed from `base` (a workspace offset, or SCRATCH_TAG for the static array); returns the bytes taken.
static size_t carve_update_scratch(const EnvDims& ed, const NetShape& ns, int B, int T, const int* splits, int splits_w, int head_fan,
                                   Layout& L, size_t base)
{
    size_t off = 0;
    auto take = [&](size_t bytes) { size_t o = off; off = align256(off + bytes); return base + o; };
    const size_t tn = (size_t)T * B;
    L.dhead = take(tn * ns.NHP * 4);
    for (int l = 0; l < MAX_LAYERS; ++l) {
        const size_t w = l < ns.L ? (size_t)ns.dims[l + 1] : 0;
        L.dz[l] = take(tn * w * 4);
    }
    for (int l = 0; l < MAX_REGIONS; ++l) {
        size_t cnt = 0;
        if (l < ns.L) cnt = (size_t)ns.dims[l] * ns.dims[l + 1] + ns.dims[l + 1];
        else if (l == ns.L) cnt = (size_t)ns.dims[ns.L] * ns.NH + ns.NH;
        size_t floats = cnt * (size_t)(l <= ns.L ? splits[l] : 0);
        if (l == 0 && splits_w > 0) {
            // wall-plane partials, agent-plane partials, column sums (see launch_backward_bf16)
            const size_t plane = (size_t)ed.rows * ed.cols * ns.dims[1];
            const size_t pieces = plane * ((size_t)splits_w + splits[0]) + (size_t)ns.dims[1] * splits_w;
            if (pieces > floats) floats = pieces;
        }
        L.part[l] = take(floats * 4);
    }
    L.head_stage = take(head_fan > 1 ? (size_t)splits[ns.L] * head_fan * ((size_t)ns.dims[ns.L] * ns.NH + ns.NH) * 4 : 0);
    return off;
}

static void carve(const EnvDims& ed, const NetShape& ns, int B, int T, const int* splits, int splits_w, int head_fan, int loss_blocks, Layout& L)
{
    size_t off = 0;
    auto take = [&](size_t bytes) { size_t o = off; off = align256(off + bytes); return o; };
    const size_t P = (size_t)ns.P, n = (size_t)B, tn = (size_t)T * B, t1n = (size_t)(T + 1) * B;
    L.theta = take(P * 4); L.grad = take(P * 4); L.m = take(P * 4); L.v = take(P * 4);
    L.w_bf16 = take(ns.bf16 ? P * 2 : 0); L.wt_bf16 = take(ns.bf16 ? P * 2 : 0);
    L.theta0 = take(P * 4); L.w0_bf16 = take(ns.bf16 ? P * 2 : 0);
    L.w_src = L.theta; L.w16_src = L.w_bf16;
    L.s0 = take(n * 4); L.f0 = take(n * 4); L.f1 = take(n * 4); L.walls = take(n * 8 * 4);
    L.tr_s0 = take(t1n * 4); L.tr_f0 = take(t1n * 4); L.tr_f1 = take(t1n * 4);
    L.tr_act = take(tn); L.tr_eps = take(tn * 4); L.tr_actf = take(tn * 4);
    L.tr_rew = take(tn * 4); L.tr_done = take(tn);
    L.tr_val = take(t1n * 4); L.tr_head = take(t1n * ns.NHP * 4);
    L.adv = take(tn * 4); L.ret = take(tn * 4);
    for (int l = 0; l < MAX_LAYERS; ++l) {
        const size_t w = l < ns.L ? (size_t)ns.dims[l + 1] : 0;
        L.act[l] = take(tn * w * 4);
        L.mask[l] = L.act[l] + tn * w * 2;                       // packed bf16 activations use the lower half only
    }
    off += carve_update_scratch(ed, ns, B, T, splits, splits_w, head_fan, L, off);
    L.prefix = take(ns.bf16 ? (size_t)B * ns.dims[1] * 4 : 0);
    L.loss_part = take((size_t)(loss_blocks + T) * 8 * 4);     // + T: with N updates per unroll every chunk rounds its block count up
    // decoupled steps: behaviour parameters, second record set, the learner's forward results
    const bool dec = true;
    L.theta_b = take(dec ? P * 4 : 0);
    L.w_bf16_b = take(ns.bf16 ? P * 2 : 0); L.wt_bf16_b = take(ns.bf16 ? P * 2 : 0);
    L.prefix_b = take(ns.bf16 ? (size_t)B * ns.dims[1] * 4 : 0);
    L.alt_tr_s0 = take(dec ? t1n * 4 : 0); L.alt_tr_f0 = take(dec ? t1n * 4 : 0); L.alt_tr_f1 = take(dec ? t1n * 4 : 0);
    L.alt_tr_act = take(dec ? tn : 0); L.alt_tr_eps = take(dec ? tn * 4 : 0); L.alt_tr_actf = take(dec ? tn * 4 : 0);
    L.alt_tr_rew = take(dec ? tn * 4 : 0); L.alt_tr_done = take(dec ? tn : 0);
    L.alt_tr_val = take(dec ? t1n * 4 : 0); L.alt_tr_head = take(dec ? t1n * ns.NHP * 4 : 0);
    L.head_new = take(dec ? t1n * ns.NHP * 4 : 0); L.val_new = take(dec ? t1n * 4 : 0); L.eps_new = take(dec ? tn * 4 : 0);
    L.path = take(ed.kind == ENV_PENDULUM && !ns.bf16 ? tn * 2 * 4 : 0);
    L.small_part = take(small_fused_part_bytes(ed, ns, B, T));
    L.counters = take(256);
    L.total = off;
}

static void plan(const EnvDims& ed, const NetShape& ns, int B, int T, int* splits, int* splits_w, int* head_fan, int* loss_blocks)
{
    const int M = B * T;
    for (int l = 0; l < MAX_REGIONS; ++l) splits[l] = 0;
    for (int l = 0; l < ns.L; ++l) {
        const int tiles = ((ns.dims[l] + 127) / 128) * ((ns.dims[l + 1] + 127) / 128);
        splits[l] = pick_splits(M, tiles, 256);
    }
    splits[ns.L] = pick_splits(M, (ns.dims[ns.L] + 127) / 128, 256);
    if (!ns.bf16)
        for (int l = 1; l < ns.L; ++l)
            if (ns.dims[l] == 256 && ns.dims[l + 1] == 256) {
                // persistent 256 x 256 dW kernel, 32-sample steps.  It shares its launch with the dX kernel of the
                // layer and the two kinds of workgroup run side by side, one per compute unit: half the units take
                // a dW chunk each, the other half a dX row range each (their costs per sample are within 10 %).
                // Compared with one chunk per unit followed by one row range per unit this halves the partial sums
                // (256 KB per chunk, written here, read by Adam) and every unit pays one prologue instead of two.
                const int s = pick_divisor_splits(M, 32, 128);
                // a sample count without a usable divisor (few, long chunks) stays with the tiled kernels
                const int tiles32 = M / 32;
                if (s > 0 && s >= (tiles32 < 64 ? tiles32 : 64)) splits[l] = s;
            }
    if (ed.kind != ENV_MAZE) splits[0] = pick_splits(M, 2 * ((ns.dims[1] + WG - 1) / WG), 512);   // scatter kernel: more, smaller chunks
    if (ed.kind == ENV_CATCH && ns.dims[0] < 64 && !ns.bf16) {
        // matrix-core scatter: 64-sample steps, about two workgroups (of 128 columns) per CU
        const int s = pick_divisor_splits(M, 64, 256);
        if (s > 0) splits[0] = s;
    }
    if (const int s = first_fused_splits(ns, ed.kind, M, splits[1])) splits[0] = s;                           // first layer folded into the dX product of the second
    if (ns.L == 1 && ed.kind != ENV_MAZE) { splits[0] = pick_splits(M, 1, 1024); splits[1] = splits[0]; }                                     // fused one-layer update: one chunking for both regions
    if (ns.L == 1 && ed.kind == ENV_CATCH && !ns.bf16 && ns.dims[1] == 32 && B % 256 == 0) {
        // the single-launch update (scan, loss and backward pass): a workgroup owns whole blocks of 256 envs; at most
        // 512 workgroups -- two per compute unit, which is what fits one at a time -- so that a large batch pays the
        // workgroup's prologue (W1 into LDS, 51 KB of sums cleared) and its tail once per two blocks or more, and the
        // optimiser kernel adds half as many partial gradients (measured on B = 262144: 1024 -> 512 workgroups
        // 151.5 -> 146 us and 10.5 -> 7.9 us in the optimiser kernel; 256 workgroups 220 us)
        int s = B / 256;
        while (s > 512 && s % 2 == 0) s /= 2;
        if (s <= 1024) { splits[0] = s; splits[1] = s; }
    }
    // the head-gradient pass streams the last hidden layer: many small workgroups, summed in two levels
    const bool bfp = rollout_bf16_ok(ns, ed, B);
    const int hq = bfp ? 64 : (M % 32 == 0 ? 32 : 16);  // row quantum of the head pass
    if (bfp) splits[ns.L] = pick_splits(M, (ns.dims[ns.L] + 127) / 128, 256, 64);
    *splits_w = 0;
    if (bfp) {
        // 256 x 256 tiles where both sides of a layer are multiples of 256: about one workgroup per CU
        for (int l = 1; l < ns.L; ++l)
            if (ns.dims[l] % 256 == 0 && ns.dims[l + 1] % 256 == 0)
                splits[l] = pick_splits(M, (ns.dims[l] / 256) * (ns.dims[l + 1] / 256), 64, 128);   // chunks: pairs of 64-sample stages
        const int cells = ed.rows * ed.cols;
        if (ed.kind == ENV_MAZE && cells % 256 == 0 && ns.dims[1] % 256 == 0 && M % 128 == 0) {
            const int tiles = (cells / 256) * (ns.dims[1] / 256);
            splits[0] = pick_splits(M, tiles, 128, 128);           // agent plane: all B*T samples
            *splits_w = pick_splits(2 * B, tiles, 64, 128);        // wall plane: time-summed, two bf16 terms per env
        }
    }
    int fan = 1;
    bool one_stage = false;
    if (!ns.bf16 && ns.dims[ns.L] % 64 == 0 && M % 32 == 0) {
        // matrix-core head pass: two workgroups per CU stream enough on their own, and their partials go straight to Adam
        const int s = pick_divisor_splits(M, 32, 512);
        if (s >= 64) { splits[ns.L] = s; one_stage = true; }
    }
    if (heads_fused_shape(ns, M)) {
        // the head gradients come out of the top layer's dW product: same chunks, one partial per chunk
        const int st = splits[ns.L - 1];
        if (st > 0 && M % st == 0 && (M / st) % 32 == 0) { splits[ns.L] = st; one_stage = true; }
    }
    if (bfp && bf16_top_fused(ns, M, splits[ns.L - 1])) {
        // the head gradients come out of the top layer's dW product here too
        splits[ns.L] = splits[ns.L - 1]; one_stage = true;
    }
    while (!one_stage && fan < 16 && (M / hq) % (splits[ns.L] * fan * 2) == 0 && M / (splits[ns.L] * fan * 2) >= 2 * hq) fan *= 2;
    *head_fan = fan;
    *loss_blocks = (M + WG - 1) / WG;
}

extern "C" size_t anakin_workspace_bytes(const anakin_env_cfg* env, const anakin_net_cfg* net, int32_t B, int32_t T)
{
    EnvDims ed; NetShape ns; std::string err;
    if (build_shapes(env, net, B, T, ed, ns, err) != ANAKIN_OK) return 0;
    int splits[MAX_REGIONS], sw, lb, fan;
    plan(ed, ns, B, T, splits, &sw, &fan, &lb);
    if (lb < B / 8) lb = B / 8;                                  // as in anakin_create
    Layout L;
    carve(ed, ns, B, T, splits, sw, fan, lb, L);
    return L.total;
}

// ---- one-time initialisation on the host ----------------------------------
// Glorot-uniform weights: W = a (2u - 1), a = sqrt(6 / (fan_in + fan_out)); each head
// group (logits / value / mu / log_sigma) has its own fan_out and its own group id;
// element e of a group takes word e % 4 of the draw with index e / 4.
static void init_group(uint64_t seed, uint32_t gid, float* W, int ld, int col0, int fan_in, int fan_out)
{
    const float a = (float)sqrt(6.0 / (double)(fan_in + fan_out));
    for (int i = 0; i < fan_in; ++i)
        for (int j = 0; j < fan_out; ++j) {
            const uint32_t e = (uint32_t)(i * fan_out + j);
            const u32x4 w = philox(seed, e >> 2, gid, DOM_PARAM);
            const uint32_t word = (e & 3) == 0 ? w.x : (e & 3) == 1 ? w.y : (e & 3) == 2 ? w.z : w.w;
            W[(size_t)i * ld + col0 + j] = a * fmaf(2.0f, u01(word), -1.0f);
        }
}

static void init_params_host(const NetShape& ns, uint64_t seed, std::vector<float>& th)
{
    th.assign((size_t)ns.P, 0.0f);
    uint32_t gid = 0;
    for (int l = 0; l < ns.L; ++l) init_group(seed, gid++, th.data() + ns.w_off[l], ns.dims[l + 1], 0, ns.dims[l], ns.dims[l + 1]);
    float* Wh = th.data() + ns.wh_off;
    const int HL = ns.dims[ns.L];
    if (ns.policy == POLICY_CATEGORICAL) {
        init_group(seed, gid++, Wh, ns.NH, 0, HL, ns.A);
        init_group(seed, gid++, Wh, ns.NH, ns.A, HL, 1);
    } else {
        for (int c = 0; c < 3; ++c) init_group(seed, gid++, Wh, ns.NH, c, HL, 1);
    }
}

// maze walls for one env: redraw until the goal is reachable from the start
static void make_maze(const EnvDims& ed, float p_wall, uint64_t seed, int env, uint32_t w[8])
{
    const int R = ed.rows, C = ed.cols, n = R * C;
    const uint32_t thr = (uint32_t)floor((double)p_wall * 4294967296.0);
    std::vector<int> frontier;
    std::vector<char> seen((size_t)n);
    for (uint32_t attempt = 0;; ++attempt) {
        for (int i = 0; i < 8; ++i) w[i] = 0;
        for (int blk = 0; blk * 4 < n; ++blk) {
            const u32x4 d = philox(seed, (uint32_t)env, (uint64_t)attempt | ((uint64_t)blk << 32), DOM_MAZE);
            const uint32_t ws[4] = {d.x, d.y, d.z, d.w};
            for (int i = 0; i < 4 && blk * 4 + i < n; ++i)
                if (ws[i] < thr) w[(blk * 4 + i) >> 5] |= 1u << ((blk * 4 + i) & 31);
        }
        w[0] &= ~1u;
        w[(n - 1) >> 5] &= ~(1u << ((n - 1) & 31));
        // depth-first reachability from the start cell
        std::fill(seen.begin(), seen.end(), 0);
        frontier.clear();
        frontier.push_back(0); seen[0] = 1;
        bool ok = false;
        while (!frontier.empty()) {
            const int c = frontier.back(); frontier.pop_back();
            if (c == n - 1) { ok = true; break; }
            const int r = c / C, col = c % C;
            const int cand[4] = {r > 0 ? c - C : -1, col + 1 < C ? c + 1 : -1, r + 1 < R ? c + C : -1, col > 0 ? c - 1 : -1};
            for (int d : cand)
                if (d >= 0 && !seen[d] && !((w[d >> 5] >> (d & 31)) & 1u)) { seen[d] = 1; frontier.push_back(d); }
        }
        if (ok) return;
    }
}

#define HIPCHK(h, call)                                                                   \
    do {                                                                                  \
        hipError_t e_ = (call);                                                           \
        if (e_ != hipSuccess) {                                                           \
            (h)->err = std::string(#call) + ": " + hipGetErrorString(e_);                 \
            return ANAKIN_E_HIP;                                                          \
        }                                                                                 \
    } while (0)

static int upload(anakin* h, size_t off, const void* src, size_t bytes)
{
    if (bytes == 0) return ANAKIN_OK;
    HIPCHK(h, hipMemcpyAsync(h->ws + off, src, bytes, hipMemcpyHostToDevice, h->stream));
    HIPCHK(h, hipStreamSynchronize(h->stream));
    return ANAKIN_OK;
}
static int download(anakin* h, void* dst, size_t off, size_t bytes)
{
    if (bytes == 0) return ANAKIN_OK;
    HIPCHK(h, hipMemcpyAsync(dst, h->ws + off, bytes, hipMemcpyDeviceToHost, h->stream));
    HIPCHK(h, hipStreamSynchronize(h->stream));
    return ANAKIN_OK;
}

// packed <-> row form of the env state
static void pack_state(const EnvDims& ed, const int32_t* si, const float* sf, uint32_t& s0, float& f0, float& f1)
{
    f0 = 0.0f; f1 = 0.0f;
    if (ed.kind == ENV_CATCH) s0 = catch_pack(si[0], si[1], si[2]);
    else if (ed.kind == ENV_PENDULUM) { s0 = (uint32_t)si[0]; f0 = sf[0]; f1 = sf[1]; }
    else s0 = (uint32_t)si[0] | ((uint32_t)si[1] << 16);
}
static void unpack_state(const EnvDims& ed, uint32_t s0, float f0, float f1, int32_t* si, float* sf)
{
    si[0] = si[1] = si[2] = si[3] = 0; sf[0] = sf[1] = 0.0f;
    if (ed.kind == ENV_CATCH) { si[0] = (int32_t)(s0 & 0xff); si[1] = (int32_t)((s0 >> 8) & 0xff); si[2] = (int32_t)((s0 >> 16) & 0xff); }
    else if (ed.kind == ENV_PENDULUM) { si[0] = (int32_t)s0; sf[0] = f0; sf[1] = f1; }
    else { si[0] = (int32_t)(s0 & 0xffff); si[1] = (int32_t)(s0 >> 16); }
}

extern "C" int32_t anakin_create(anakin_t** out, const anakin_env_cfg* env, const anakin_net_cfg* net,
                                 int32_t B, int32_t T, uint64_t seed, void* d_workspace, size_t workspace_bytes,
                                 void* hip_stream)
{
    if (!out) { g_create_error = "null output pointer"; return ANAKIN_E_INVALID_ARG; }
    *out = nullptr;
    EnvDims ed; NetShape ns;
    int rc = build_shapes(env, net, B, T, ed, ns, g_create_error);
    if (rc != ANAKIN_OK) return rc;
    if (!d_workspace) { g_create_error = "null workspace"; return ANAKIN_E_INVALID_ARG; }
    if (((uintptr_t)d_workspace & 255u) != 0) { g_create_error = "workspace must be 256-byte aligned"; return ANAKIN_E_MISALIGNED; }
    anakin* h = new (std::nothrow) anakin();
    if (!h) { g_create_error = "out of host memory"; return ANAKIN_E_INVALID_ARG; }
    h->env_cfg = *env; h->net_cfg = *net; h->env = ed; h->net = ns; h->B = B; h->T = T;
    h->seed = seed; h->gstep = 0; h->adam_t = 0; h->have_traj = 0; h->mode = 0; h->prof_on = 0; h->traj_packed = 0; h->traj_no_acts = 0;
    h->pathwise = 0; h->metric_blocks = 0;
    h->traj_decoupled = 0; h->actor_stream = nullptr; h->actor_stream_owned = 0; h->ev_fork = nullptr; h->ev_join = nullptr;
    h->ws = static_cast<char*>(d_workspace); h->ws_bytes = workspace_bytes;
    h->scratch = nullptr;
    h->stream = static_cast<hipStream_t>(hip_stream);
    plan(ed, ns, B, T, h->splits, &h->splits_w, &h->head_fan, &h->loss_blocks);
    // returns and loss in one launch write one block of sums per eight envs where the unroll is short
    if (h->loss_blocks < B / 8) h->loss_blocks = B / 8;
    carve(ed, ns, B, T, h->splits, h->splits_w, h->head_fan, h->loss_blocks, h->lay);
    if (h->lay.total > workspace_bytes) {
        g_create_error = "workspace too small: need " + std::to_string(h->lay.total) + " bytes";
        delete h; return ANAKIN_E_WORKSPACE_TOO_SMALL;
    }
    {
        // the device the workspace lives on (the current one if the runtime cannot tell), and this device's copy
        // of the static scratch array: resolved here, at set-up, so that anakin_learn_static has nothing left to do
        int dev = 0;
        hipPointerAttribute_t attr;
        if (hipPointerGetAttributes(&attr, d_workspace) == hipSuccess) dev = attr.device;
        else { (void)hipGetLastError(); if (hipGetDevice(&dev) != hipSuccess) dev = 0; }
        h->device = dev;
        const hipError_t es = resolve_static_scratch(dev);
        if (es != hipSuccess) { g_create_error = std::string("hipGetSymbolAddress(static scratch): ") + hipGetErrorString(es); delete h; return ANAKIN_E_HIP; }
    }
    h->n_updates = 1; h->chunks_sequential = 0;
    h->TM = rollout_pick_tile(ns, B);
    h->TM_mfma = rollout_pick_tile_mfma(ns, B);
    h->TM_res = rollout_resident_tile(ns, ed.kind, B);
    h->bf16_path = rollout_bf16_ok(ns, ed, B) ? 1 : 0;

    auto fail = [&](int code) { g_create_error = h->err; delete h; return code; };
    // parameters and optimiser state
    std::vector<float> th;
    init_params_host(ns, seed, th);
    if ((rc = upload(h, h->lay.theta, th.data(), th.size() * 4)) != ANAKIN_OK) return fail(rc);
    hipError_t e = hipMemsetAsync(h->ws + h->lay.grad, 0, (size_t)ns.P * 4, h->stream);
    if (e == hipSuccess) e = hipMemsetAsync(h->ws + h->lay.m, 0, (size_t)ns.P * 4, h->stream);
    if (e == hipSuccess) e = hipMemsetAsync(h->ws + h->lay.v, 0, (size_t)ns.P * 4, h->stream);
    // the metrics are sums over these blocks: zero until the first update has written them
    if (e == hipSuccess) e = hipMemsetAsync(h->ws + h->lay.loss_part, 0, (size_t)(h->loss_blocks + T) * 8 * 4, h->stream);
    if (e == hipSuccess) e = hipMemsetAsync(h->ws + h->lay.counters, 0, 256, h->stream);
    if (e != hipSuccess) { h->err = std::string("hipMemsetAsync: ") + hipGetErrorString(e); return fail(ANAKIN_E_HIP); }
    if (ns.bf16) {
        e = launch_refresh_bf16(h);
        if (e != hipSuccess) { h->err = std::string("refresh_bf16: ") + hipGetErrorString(e); return fail(ANAKIN_E_HIP); }
    }
    // initial env states
    std::vector<uint32_t> s0((size_t)B), walls(ed.kind == ENV_MAZE ? (size_t)B * 8 : 0);
    std::vector<float> f0((size_t)B, 0.0f), f1((size_t)B, 0.0f);
    for (int b = 0; b < B; ++b) {
        const u32x4 w = philox(seed, (uint32_t)b, 0, DOM_INIT);
        if (ed.kind == ENV_CATCH) s0[b] = catch_reset(ed, w.x);
        else if (ed.kind == ENV_PENDULUM) { EnvState st; pendulum_reset(st, w.x, w.y); s0[b] = st.s0; f0[b] = st.f0; f1[b] = st.f1; }
        else {
            uint32_t wl[8];
            make_maze(ed, env->p_wall, seed, b, wl);
            for (int k = 0; k < 8; ++k) walls[(size_t)k * B + b] = wl[k];      // word-major [8][B]
            s0[b] = 0;
        }
    }
    if ((rc = upload(h, h->lay.s0, s0.data(), (size_t)B * 4)) != ANAKIN_OK) return fail(rc);
    if ((rc = upload(h, h->lay.f0, f0.data(), (size_t)B * 4)) != ANAKIN_OK) return fail(rc);
    if ((rc = upload(h, h->lay.f1, f1.data(), (size_t)B * 4)) != ANAKIN_OK) return fail(rc);
    if ((rc = upload(h, h->lay.walls, walls.data(), walls.size() * 4)) != ANAKIN_OK) return fail(rc);
    e = hipStreamSynchronize(h->stream);
    if (e != hipSuccess) { h->err = std::string("hipStreamSynchronize: ") + hipGetErrorString(e); return fail(ANAKIN_E_HIP); }
    *out = h;
    return ANAKIN_OK;
}

extern "C" int32_t anakin_destroy(anakin_t* h)
{
    if (!h) return ANAKIN_E_INVALID_ARG;
    (void)prof_resolve(h);
    for (hipEvent_t e : h->prof_pool) (void)hipEventDestroy(e);
    if (h->actor_stream) { (void)hipStreamSynchronize(h->actor_stream); if (h->actor_stream_owned) (void)hipStreamDestroy(h->actor_stream); }
    if (h->ev_fork) (void)hipEventDestroy(h->ev_fork);
    if (h->ev_join) (void)hipEventDestroy(h->ev_join);
    delete h;
    return ANAKIN_OK;
}

namespace ank {
void fill_rollout_args(anakin* h, RolloutArgs& a)
{
    const Layout& L = h->lay;
    a.env = h->env; a.net = h->net; a.theta = at<const float>(h, L.theta);
    a.B = h->B; a.T = h->T; a.seed = h->seed; a.gstep = h->gstep;
    a.keep_acts = one_layer_fused(h) ? 0 : 1;
    rollout_lds_bytes(h->net, h->env, h->TM, &a.ldx);
    TrajPtrs& t = a.tp;
    t.s0 = at<uint32_t>(h, L.s0); t.f0 = at<float>(h, L.f0); t.f1 = at<float>(h, L.f1); t.walls = at<const uint32_t>(h, L.walls);
    t.tr_s0 = at<uint32_t>(h, L.tr_s0); t.tr_f0 = at<float>(h, L.tr_f0); t.tr_f1 = at<float>(h, L.tr_f1);
    t.tr_act = at<uint8_t>(h, L.tr_act); t.tr_eps = at<float>(h, L.tr_eps); t.tr_actf = at<float>(h, L.tr_actf);
    t.tr_rew = at<float>(h, L.tr_rew); t.tr_done = at<uint8_t>(h, L.tr_done);
    t.tr_val = at<float>(h, L.tr_val); t.tr_head = at<float>(h, L.tr_head);
    for (int l = 0; l < MAX_LAYERS; ++l) { t.act[l] = at<float>(h, L.act[l]); t.mask[l] = at<uint32_t>(h, L.mask[l]); }
}
}  // namespace ank

#define NEED(h) do { if (!(h)) return ANAKIN_E_INVALID_ARG; } while (0)

// ---- per-kernel timing ----------------------------------------------------------
namespace ank {
static hipEvent_t prof_event(anakin* h)
{
    if (!h->prof_pool.empty()) { hipEvent_t e = h->prof_pool.back(); h->prof_pool.pop_back(); return e; }
    hipEvent_t e = nullptr;
    if (hipEventCreate(&e) != hipSuccess) return nullptr;
    return e;
}
ProfScope::ProfScope(anakin* h_, const char* name) : h(h_), idx(-1)
{
    if (!h->prof_on) return;
    int id = -1;
    for (size_t i = 0; i < h->prof_totals.size(); ++i) if (h->prof_totals[i].name == name) { id = (int)i; break; }
    if (id < 0) { h->prof_totals.push_back({name, 0, 0.0}); id = (int)h->prof_totals.size() - 1; }
    anakin::ProfPending p{id, prof_event(h), prof_event(h)};
    if (!p.start || !p.stop) return;
    (void)hipEventRecord(p.start, h->stream);
    h->prof_pending.push_back(p);
    idx = (int)h->prof_pending.size() - 1;
}
ProfScope::~ProfScope()
{
    if (idx >= 0) (void)hipEventRecord(h->prof_pending[(size_t)idx].stop, h->stream);
}
hipError_t prof_resolve(anakin* h)
{
    hipError_t e = hipStreamSynchronize(h->stream);
    if (e != hipSuccess) return e;
    for (const auto& p : h->prof_pending) {
        float ms = 0.0f;
        if (hipEventElapsedTime(&ms, p.start, p.stop) == hipSuccess) {
            h->prof_totals[(size_t)p.name].calls += 1;
            h->prof_totals[(size_t)p.name].ms += (double)ms;
        }
        h->prof_pool.push_back(p.start); h->prof_pool.push_back(p.stop);
    }
    h->prof_pending.clear();
    return hipSuccess;
}
}  // namespace ank

extern "C" int32_t anakin_profile(anakin_t* h, int32_t enable)
{
    NEED(h);
    HIPCHK(h, prof_resolve(h));
    if (enable) h->prof_totals.clear();
    h->prof_on = enable ? 1 : 0;
    return ANAKIN_OK;
}

extern "C" int32_t anakin_kernel_times(anakin_t* h, anakin_kernel_time* out, int32_t cap, int32_t* n)
{
    NEED(h);
    if (!n || (cap > 0 && !out)) return ANAKIN_E_INVALID_ARG;
    HIPCHK(h, prof_resolve(h));
    *n = (int32_t)h->prof_totals.size();
    for (int32_t i = 0; i < *n && i < cap; ++i) {
        memset(&out[i], 0, sizeof out[i]);
        strncpy(out[i].name, h->prof_totals[(size_t)i].name.c_str(), sizeof(out[i].name) - 1);
        out[i].calls = h->prof_totals[(size_t)i].calls;
        out[i].total_ms = h->prof_totals[(size_t)i].ms;
    }
    return ANAKIN_OK;
}

extern "C" int32_t anakin_rollout(anakin_t* h)
{
    NEED(h);
    if (bf16_mfma(h)) HIPCHK(h, launch_rollout_bf16(h));
    else HIPCHK(h, launch_rollout(h));
    h->traj_packed = bf16_mfma(h) ? 1 : 0;
    h->traj_no_acts = one_layer_fused(h) ? 1 : 0;
    h->traj_decoupled = 0;
    h->gstep += (uint64_t)h->T;
    h->have_traj = 1;
    return ANAKIN_OK;
}

// loss, backward pass and Adam on the samples the handle's layout and T currently describe
static int32_t run_update(anakin* h, bool loss_done = false)
{
    if (!loss_done) HIPCHK(h, launch_head_grad(h));
    if (h->traj_packed) HIPCHK(h, launch_backward_bf16(h));
    else if (h->traj_no_acts) HIPCHK(h, launch_learn_one_layer(h));
    else HIPCHK(h, launch_backward(h));
    HIPCHK(h, launch_adam(h));
    return ANAKIN_OK;
}

extern "C" int32_t anakin_learn(anakin_t* h)
{
    NEED(h);
    if (!h->have_traj) { h->err = "learn needs a stored trajectory: call anakin_rollout first"; return ANAKIN_E_STATE; }
    if (h->traj_decoupled) { h->err = "the stored unroll was collected by a decoupled step (older parameters, no activations): continue with anakin_step_decoupled"; return ANAKIN_E_STATE; }
    if (h->traj_packed != (bf16_mfma(h) ? 1 : 0)) { h->err = "the mode changed between rollout and learn"; return ANAKIN_E_STATE; }
    if (h->traj_no_acts != (one_layer_fused(h) ? 1 : 0)) { h->err = "the mode changed between rollout and learn"; return ANAKIN_E_STATE; }
    if (catch_fused_ok(h)) {
        // scan, loss, backward pass in one launch; then Adam
        HIPCHK(h, launch_learn_catch_fused(h));
        HIPCHK(h, launch_adam(h));
        h->have_traj = 0;
        return ANAKIN_OK;
    }
    if (small_fused_ok(h)) {
        // scan, loss, backward pass and Adam in one launch
        HIPCHK(h, launch_learn_small_fused(h));
        h->have_traj = 0;
        return ANAKIN_OK;
    }
    const bool fused_loss = scan_loss_ok(h);
    if (fused_loss) HIPCHK(h, launch_scan_loss(h));
    else HIPCHK(h, launch_returns(h));
    if (h->pathwise) {
        if (h->n_updates != 1) { h->err = "the pathwise policy gradient takes one update per unroll (chunks would cut the adjoint)"; return ANAKIN_E_BAD_CONFIG; }
        HIPCHK(h, launch_pathwise(h));
    }
    if (h->n_updates == 1) {
        int32_t rc = run_update(h, fused_loss);
        if (rc != ANAKIN_OK) return rc;
        h->have_traj = 0;
        return ANAKIN_OK;
    }
    // Several updates on one unroll: chunk k is the time steps [k T/n, (k+1) T/n).  Default: every chunk's gradient is
    // taken at the parameters the unroll was acted with (the stored forward pass), so the backward kernels read a copy
    // of the weights made now while Adam moves the live ones.  Sequential mode: chunk k's gradient at the parameters
    // after k updates (the forward pass is repeated before each further chunk).  The kernels see a chunk as a shorter
    // unroll: T and the offsets of the per-sample arrays are switched for the duration of one update.
    const Layout full = h->lay;
    const NetShape& n = h->net;
    const int T = h->T, B = h->B, Ts = T / h->n_updates;
    const bool seq = h->chunks_sequential != 0;
    if (!seq) {
        HIPCHK(h, hipMemcpyAsync(h->ws + full.theta0, h->ws + full.theta, (size_t)n.P * 4, hipMemcpyDeviceToDevice, h->stream));
        if (n.bf16) HIPCHK(h, hipMemcpyAsync(h->ws + full.w0_bf16, h->ws + full.w_bf16, (size_t)n.P * 2, hipMemcpyDeviceToDevice, h->stream));
    }
    int full_splits[MAX_REGIONS];
    for (int l = 0; l < MAX_REGIONS; ++l) full_splits[l] = h->splits[l];
    const int full_sw = h->splits_w, full_fan = h->head_fan, full_lb = h->loss_blocks;
    int32_t rc = ANAKIN_OK;
    for (int k = 0; k < h->n_updates && rc == ANAKIN_OK; ++k) {
        if (seq && k > 0) {
            // sequential reading: the chunk's gradient is taken at the parameters as they are now, so the forward
            // pass over the stored states is repeated with them (activations, head outputs, values; for the Gaussian
            // policy also the noise that reproduces the stored sample), on the whole unroll's layout
            h->lay = full; h->T = T;
            hipError_t e = bf16_mfma(h) ? launch_replay_bf16(h) : launch_replay_forward(h);
            if (e == hipSuccess) e = launch_eps_now(h);
            if (e != hipSuccess) { h->err = std::string("replay of the forward pass: ") + hipGetErrorString(e); rc = ANAKIN_E_HIP; break; }
        }
        for (int l = 0; l < MAX_REGIONS; ++l) h->splits[l] = h->sub_splits[l];
        h->splits_w = h->sub_splits_w; h->head_fan = h->sub_head_fan; h->loss_blocks = h->sub_loss_blocks;
        h->T = Ts;
        const size_t r0 = (size_t)k * Ts * B;                         // first sample of the chunk
        Layout& L = h->lay;
        L = full;
        if (seq) {
            L.w_src = full.theta; L.w16_src = full.w_bf16;
            if (k > 0) { L.tr_head = full.head_new; L.tr_eps = full.eps_new; }
        } else {
            L.w_src = full.theta0; L.w16_src = n.bf16 ? full.w0_bf16 : full.w_bf16;
        }
        L.tr_s0 += r0 * 4; L.tr_f0 += r0 * 4; L.tr_f1 += r0 * 4;
        L.tr_act += r0; L.tr_eps += r0 * 4; L.tr_actf += r0 * 4; L.tr_rew += r0 * 4; L.tr_done += r0;
        L.tr_val += r0 * 4; L.tr_head += r0 * n.NHP * 4;
        L.adv += r0 * 4; L.ret += r0 * 4;
        for (int l = 0; l < n.L; ++l) { L.act[l] += r0 * n.dims[l + 1] * (h->traj_packed ? 2 : 4); L.mask[l] += r0 * n.dims[l + 1] / 4; }
        L.loss_part += (size_t)k * h->sub_loss_blocks * 8 * 4;
        rc = run_update(h);
        for (int l = 0; l < MAX_REGIONS; ++l) h->splits[l] = full_splits[l];
        h->splits_w = full_sw; h->head_fan = full_fan; h->loss_blocks = full_lb;
    }
    h->lay = full; h->T = T;
    for (int l = 0; l < MAX_REGIONS; ++l) h->splits[l] = full_splits[l];
    h->splits_w = full_sw; h->head_fan = full_fan; h->loss_blocks = full_lb;
    if (rc != ANAKIN_OK) return rc;
    h->have_traj = 0;
    return ANAKIN_OK;
}

extern "C" int32_t anakin_learn_static(anakin_t* h)
{
    NEED(h);
    if (h->prof_on) { h->err = "anakin_learn_static: switch per-kernel timing off first (it creates events)"; return ANAKIN_E_STATE; }
    Layout probe = h->lay;
    const size_t need = carve_update_scratch(h->env, h->net, h->B, h->T, h->splits, h->splits_w, h->head_fan, probe, SCRATCH_TAG);
    if (need > (size_t)ANAKIN_STATIC_SCRATCH_BYTES) {
        h->err = "anakin_learn_static: the update of this configuration needs " + std::to_string(need) + " bytes of scratch, the static array holds " +
                 std::to_string((size_t)ANAKIN_STATIC_SCRATCH_BYTES) + ": use anakin_learn, or fewer envs / a shorter unroll / a narrower net";
        return ANAKIN_E_WORKSPACE_TOO_SMALL;
    }
    void* base = nullptr;
    {
        std::lock_guard<std::mutex> lock(g_scratch_mutex);
        base = (h->device >= 0 && h->device < MAX_DEVICES) ? g_scratch_ptr[h->device] : nullptr;
    }
    if (!base) { h->err = "anakin_learn_static: no static scratch on this handle's device"; return ANAKIN_E_STATE; }
    const Layout keep = h->lay;
    h->lay = probe;                                   // the same layout with the update's scratch inside the static array
    h->scratch = static_cast<char*>(base);
    const int32_t rc = anakin_learn(h);
    h->lay = keep;
    h->scratch = nullptr;
    return rc;
}

extern "C" int32_t anakin_set_policy_gradient(anakin_t* h, int32_t kind)
{
    NEED(h);
    if (kind != ANAKIN_PG_SCORE_FUNCTION && kind != ANAKIN_PG_PATHWISE) { h->err = "unknown policy-gradient kind"; return ANAKIN_E_INVALID_ARG; }
    if (kind == ANAKIN_PG_PATHWISE && !pathwise_ok(h)) {
        h->err = "the pathwise policy gradient needs the pendulum with the tanh-Gaussian policy, an fp32 net of two equal hidden layers of 64, 128 or 256 units, and B a multiple of 16";
        return ANAKIN_E_BAD_CONFIG;
    }
    h->pathwise = kind == ANAKIN_PG_PATHWISE ? 1 : 0;
    return ANAKIN_OK;
}

extern "C" int32_t anakin_set_updates_per_unroll(anakin_t* h, int32_t n_updates)
{
    NEED(h);
    if (n_updates < 1 || h->T % n_updates != 0) { h->err = "updates per unroll: T must be a positive multiple of it"; return ANAKIN_E_BAD_CONFIG; }
    if (n_updates == 1) { h->n_updates = 1; return ANAKIN_OK; }
    int sw = 0, fan = 1, lb = 0;
    int sp[MAX_REGIONS];
    plan(h->env, h->net, h->B, h->T / n_updates, sp, &sw, &fan, &lb);
    // the scratch buffers were sized for the full unroll: a chunk's plan has to fit them
    bool ok = (sw > 0) == (h->splits_w > 0) && lb * n_updates <= h->loss_blocks + h->T && sp[h->net.L] * fan <= h->splits[h->net.L] * h->head_fan;
    for (int l = 0; l <= h->net.L && ok; ++l) ok = sp[l] > 0 && sp[l] <= h->splits[l];
    if (ok && sw > 0) ok = sw <= h->splits_w;
    if (!ok) { h->err = "updates per unroll: the chunk size does not fit the kernels' row granularity for this B and T"; return ANAKIN_E_BAD_CONFIG; }
    for (int l = 0; l < MAX_REGIONS; ++l) h->sub_splits[l] = sp[l];
    h->sub_splits_w = sw; h->sub_head_fan = fan; h->sub_loss_blocks = lb;
    h->n_updates = n_updates;
    return ANAKIN_OK;
}

extern "C" int32_t anakin_set_update_chunk_mode(anakin_t* h, int32_t mode)
{
    NEED(h);
    if (mode != ANAKIN_CHUNKS_AT_ACTING_PARAMETERS && mode != ANAKIN_CHUNKS_SEQUENTIAL) { h->err = "unknown chunk mode"; return ANAKIN_E_INVALID_ARG; }
    h->chunks_sequential = mode == ANAKIN_CHUNKS_SEQUENTIAL ? 1 : 0;
    return ANAKIN_OK;
}

extern "C" int32_t anakin_step(anakin_t* h)
{
    if (h && h->prof_pending.size() > 8192) HIPCHK(h, prof_resolve(h));
    int32_t rc = anakin_rollout(h);
    if (rc != ANAKIN_OK) return rc;
    return anakin_learn(h);
}

// ---- decoupled acting and learning on one device -------------------------------------
// The two record sets change roles by exchanging their offsets in the layout.
static void swap_record_sets(Layout& L)
{
    std::swap(L.tr_s0, L.alt_tr_s0); std::swap(L.tr_f0, L.alt_tr_f0); std::swap(L.tr_f1, L.alt_tr_f1);
    std::swap(L.tr_act, L.alt_tr_act); std::swap(L.tr_eps, L.alt_tr_eps); std::swap(L.tr_actf, L.alt_tr_actf);
    std::swap(L.tr_rew, L.alt_tr_rew); std::swap(L.tr_done, L.alt_tr_done);
    std::swap(L.tr_val, L.alt_tr_val); std::swap(L.tr_head, L.alt_tr_head);
}

extern "C" int32_t anakin_step_decoupled(anakin_t* h)
{
    NEED(h);
    if (h->n_updates != 1) { h->err = "decoupled steps apply one update per unroll"; return ANAKIN_E_BAD_CONFIG; }
    if (h->pathwise) { h->err = "decoupled steps use the score-function gradient"; return ANAKIN_E_BAD_CONFIG; }
    if (h->prof_pending.size() > 8192) HIPCHK(h, prof_resolve(h));
    if (!h->actor_stream) {
        // no stream given by the caller (anakin_set_actor_stream): one of the library's own, default priority
        HIPCHK(h, hipStreamCreateWithFlags(&h->actor_stream, hipStreamNonBlocking));
        h->actor_stream_owned = 1;
    }
    if (!h->ev_fork) HIPCHK(h, hipEventCreateWithFlags(&h->ev_fork, hipEventDisableTiming));
    if (!h->ev_join) HIPCHK(h, hipEventCreateWithFlags(&h->ev_join, hipEventDisableTiming));
    const NetShape& n = h->net;
    hipStream_t learner = h->stream;
    // the actor's parameters: the learner's as they are now, before this step's update touches them
    HIPCHK(h, hipMemcpyAsync(h->ws + h->lay.theta_b, h->ws + h->lay.theta, (size_t)n.P * 4, hipMemcpyDeviceToDevice, learner));
    const bool mc = bf16_mfma(h);                                 // bf16 net on the matrix-core path: packed activations
    if (mc) {
        HIPCHK(h, hipMemcpyAsync(h->ws + h->lay.w_bf16_b, h->ws + h->lay.w_bf16, (size_t)n.P * 2, hipMemcpyDeviceToDevice, learner));
        HIPCHK(h, hipMemcpyAsync(h->ws + h->lay.wt_bf16_b, h->ws + h->lay.wt_bf16, (size_t)n.P * 2, hipMemcpyDeviceToDevice, learner));
    }
    HIPCHK(h, hipEventRecord(h->ev_fork, learner));
    HIPCHK(h, hipStreamWaitEvent(h->actor_stream, h->ev_fork, 0));
    // actor: T steps into the free record set, on its own stream
    swap_record_sets(h->lay);
    h->stream = h->actor_stream;
    hipError_t e = mc ? launch_rollout_bf16_behaviour(h) : launch_rollout_behaviour(h);
    h->stream = learner;
    swap_record_sets(h->lay);
    HIPCHK(h, e);
    const bool join_recorded = hipEventRecord(h->ev_join, h->actor_stream) == hipSuccess;
    // learner: one off-policy update on the unroll of the previous step.  Whatever happens in it, the layout is
    // put back, the record set the actor is filling becomes the stored unroll and the handle's stream is ordered
    // behind the actor, so an error leaves the handle consistent and the fresh unroll usable.
    auto learner_update = [&]() -> int32_t {
        if (!h->have_traj) return ANAKIN_OK;
        HIPCHK(h, mc ? launch_replay_bf16(h) : launch_replay_forward(h));
        HIPCHK(h, launch_vtrace(h));
        const int no_acts = h->traj_no_acts;
        h->traj_packed = mc ? 1 : 0; h->traj_no_acts = one_layer_fused(h) ? 1 : 0;
        const Layout keep = h->lay;
        h->lay.tr_head = keep.head_new; h->lay.tr_eps = keep.eps_new;   // the loss kernel reads the learner's heads
        const int32_t r = run_update(h);
        h->lay = keep;
        h->traj_no_acts = no_acts;
        return r;
    };
    const int32_t rc = learner_update();
    swap_record_sets(h->lay);
    hipError_t ej = join_recorded ? hipStreamWaitEvent(learner, h->ev_join, 0) : hipErrorUnknown;
    if (ej != hipSuccess) ej = hipStreamSynchronize(h->actor_stream);     // order by waiting on the host instead
    h->traj_packed = mc ? 1 : 0; h->traj_no_acts = one_layer_fused(h) ? 1 : 0; h->traj_decoupled = 1;
    h->gstep += (uint64_t)h->T;
    h->have_traj = 1;
    if (rc != ANAKIN_OK) return rc;
    HIPCHK(h, ej);
    return ANAKIN_OK;
}

extern "C" int32_t anakin_set_actor_stream(anakin_t* h, void* hip_stream)
{
    NEED(h);
    if (!hip_stream) { h->err = "the actor stream must be a stream of its own (not the null stream)"; return ANAKIN_E_INVALID_ARG; }
    if (static_cast<hipStream_t>(hip_stream) == h->stream) { h->err = "the actor stream must differ from the handle's stream"; return ANAKIN_E_INVALID_ARG; }
    if (h->actor_stream) {
        HIPCHK(h, hipStreamSynchronize(h->actor_stream));
        if (h->actor_stream_owned) HIPCHK(h, hipStreamDestroy(h->actor_stream));
    }
    h->actor_stream = static_cast<hipStream_t>(hip_stream);
    h->actor_stream_owned = 0;
    return ANAKIN_OK;
}

// ---- introspection ----------------------------------------------------------
extern "C" int32_t anakin_param_count(const anakin_t* h, int64_t* out)
{
    if (!h || !out) return ANAKIN_E_INVALID_ARG;
    *out = h->net.P;
    return ANAKIN_OK;
}

static int check_n(anakin* h, const void* p, size_t n)
{
    if (!p) { h->err = "null pointer"; return ANAKIN_E_INVALID_ARG; }
    if (n != (size_t)h->net.P) { h->err = "length must equal the parameter count"; return ANAKIN_E_INVALID_ARG; }
    return ANAKIN_OK;
}

extern "C" int32_t anakin_get_params(anakin_t* h, float* dst, size_t n)
{
    NEED(h); int rc = check_n(h, dst, n); if (rc) return rc;
    return download(h, dst, h->lay.theta, n * 4);
}
extern "C" int32_t anakin_set_params(anakin_t* h, const float* src, size_t n)
{
    NEED(h); int rc = check_n(h, src, n); if (rc) return rc;
    if ((rc = upload(h, h->lay.theta, src, n * 4)) != ANAKIN_OK) return rc;
    if (h->net.bf16) {
        HIPCHK(h, launch_refresh_bf16(h));
        HIPCHK(h, hipStreamSynchronize(h->stream));
    }
    return ANAKIN_OK;
}
extern "C" int32_t anakin_get_grads(anakin_t* h, float* dst, size_t n)
{
    NEED(h); int rc = check_n(h, dst, n); if (rc) return rc;
    return download(h, dst, h->lay.grad, n * 4);
}
extern "C" int32_t anakin_get_opt_state(anakin_t* h, float* m, float* v, int32_t* step, size_t n)
{
    NEED(h); int rc = check_n(h, m, n); if (rc) return rc;
    rc = check_n(h, v, n); if (rc) return rc;
    if (!step) return ANAKIN_E_INVALID_ARG;
    if ((rc = download(h, m, h->lay.m, n * 4)) != ANAKIN_OK) return rc;
    if ((rc = download(h, v, h->lay.v, n * 4)) != ANAKIN_OK) return rc;
    *step = h->adam_t;
    return ANAKIN_OK;
}
extern "C" int32_t anakin_set_opt_state(anakin_t* h, const float* m, const float* v, int32_t step, size_t n)
{
    NEED(h); int rc = check_n(h, m, n); if (rc) return rc;
    rc = check_n(h, v, n); if (rc) return rc;
    if (step < 0) { h->err = "negative step"; return ANAKIN_E_INVALID_ARG; }
    if ((rc = upload(h, h->lay.m, m, n * 4)) != ANAKIN_OK) return rc;
    if ((rc = upload(h, h->lay.v, v, n * 4)) != ANAKIN_OK) return rc;
    h->adam_t = step;
    return ANAKIN_OK;
}

extern "C" int32_t anakin_get_env_state(anakin_t* h, int32_t* si, float* sf)
{
    NEED(h);
    if (!si || !sf) return ANAKIN_E_INVALID_ARG;
    const size_t B = (size_t)h->B;
    std::vector<uint32_t> s0(B); std::vector<float> f0(B), f1(B);
    int rc;
    if ((rc = download(h, s0.data(), h->lay.s0, B * 4)) != ANAKIN_OK) return rc;
    if ((rc = download(h, f0.data(), h->lay.f0, B * 4)) != ANAKIN_OK) return rc;
    if ((rc = download(h, f1.data(), h->lay.f1, B * 4)) != ANAKIN_OK) return rc;
    for (size_t b = 0; b < B; ++b) unpack_state(h->env, s0[b], f0[b], f1[b], si + b * 4, sf + b * 2);
    return ANAKIN_OK;
}
extern "C" int32_t anakin_set_env_state(anakin_t* h, const int32_t* si, const float* sf)
{
    NEED(h);
    if (!si || !sf) return ANAKIN_E_INVALID_ARG;
    const size_t B = (size_t)h->B;
    std::vector<uint32_t> s0(B); std::vector<float> f0(B), f1(B);
    for (size_t b = 0; b < B; ++b) {
        const int32_t* s = si + b * 4;
        bool ok = true;
        if (h->env.kind == ENV_CATCH) ok = s[0] >= 0 && s[0] < h->env.cols && s[1] >= 0 && s[1] < h->env.rows - 1 && s[2] >= 0 && s[2] < h->env.cols;
        else if (h->env.kind == ENV_PENDULUM) ok = s[0] >= 0 && s[0] < h->env.max_steps;
        else ok = s[0] >= 0 && s[0] < h->env.rows * h->env.cols && s[1] >= 0 && s[1] < h->env.max_steps;
        if (!ok) { h->err = "env state out of range"; return ANAKIN_E_INVALID_ARG; }
        pack_state(h->env, s, sf + b * 2, s0[b], f0[b], f1[b]);
    }
    int rc;
    if ((rc = upload(h, h->lay.s0, s0.data(), B * 4)) != ANAKIN_OK) return rc;
    if ((rc = upload(h, h->lay.f0, f0.data(), B * 4)) != ANAKIN_OK) return rc;
    return upload(h, h->lay.f1, f1.data(), B * 4);
}
extern "C" int32_t anakin_get_walls(anakin_t* h, uint32_t* out)
{
    NEED(h);
    if (!out) return ANAKIN_E_INVALID_ARG;
    if (h->env.kind != ENV_MAZE) { h->err = "walls exist for the maze only"; return ANAKIN_E_STATE; }
    const size_t B = (size_t)h->B;
    std::vector<uint32_t> w(B * 8);
    int rc = download(h, w.data(), h->lay.walls, B * 8 * 4);
    if (rc) return rc;
    for (size_t b = 0; b < B; ++b) for (int k = 0; k < 8; ++k) out[b * 8 + k] = w[(size_t)k * B + b];
    return ANAKIN_OK;
}
extern "C" int32_t anakin_get_global_step(const anakin_t* h, uint64_t* out)
{
    if (!h || !out) return ANAKIN_E_INVALID_ARG;
    *out = h->gstep;
    return ANAKIN_OK;
}
extern "C" int32_t anakin_set_global_step(anakin_t* h, uint64_t g) { NEED(h); h->gstep = g; return ANAKIN_OK; }

extern "C" int32_t anakin_get_trajectory(anakin_t* h, anakin_traj_view* v)
{
    NEED(h);
    if (!v) return ANAKIN_E_INVALID_ARG;
    HIPCHK(h, hipStreamSynchronize(h->stream));
    const Layout& L = h->lay;
    memset(v, 0, sizeof *v);
    v->B = h->B; v->T = h->T; v->num_heads = h->net.NH; v->head_stride = h->net.NHP; v->n_hidden = h->net.L;
    for (int l = 0; l < h->net.L; ++l) v->hidden[l] = h->net.dims[l + 1];
    v->act_is_bf16 = h->traj_packed ? 2 : (h->traj_no_acts ? -1 : 0);
#define SETP(field, off) v->field = h->ws + (off); v->off_##field = (off)
    SETP(state_s0, L.tr_s0); SETP(state_f0, L.tr_f0); SETP(state_f1, L.tr_f1);
    SETP(action, L.tr_act); SETP(eps, L.tr_eps); SETP(action_f, L.tr_actf);
    SETP(reward, L.tr_rew); SETP(done, L.tr_done); SETP(value, L.tr_val); SETP(head, L.tr_head);
    SETP(adv, L.adv); SETP(ret, L.ret);
#undef SETP
    for (int l = 0; l < h->net.L; ++l) { v->act[l] = h->ws + L.act[l]; v->off_act[l] = L.act[l]; }
    return ANAKIN_OK;
}

extern "C" int32_t anakin_get_metrics(anakin_t* h, anakin_metrics* out)
{
    NEED(h);
    if (!out) return ANAKIN_E_INVALID_ARG;
    // with several updates per unroll every chunk wrote its own run of blocks
    const int blocks = h->n_updates > 1 ? (h->metric_blocks > 0 ? h->n_updates * h->sub_loss_blocks : 0) : h->metric_blocks;
    std::vector<float> part((size_t)blocks * 8);
    int rc = download(h, part.data(), h->lay.loss_part, part.size() * 4);
    if (rc) return rc;
    double s[5] = {0, 0, 0, 0, 0};
    for (int b = 0; b < blocks; ++b) for (int k = 0; k < 5; ++k) s[k] += (double)part[(size_t)b * 8 + k];
    const double M = (double)h->B * h->T;
    out->policy_loss = s[0] / M; out->value_loss = s[1] / M; out->entropy_loss = s[2] / M;
    out->loss = out->policy_loss + out->value_loss + out->entropy_loss;
    out->reward_sum = s[3];
    out->episodes = (int64_t)llround(s[4]);
    out->nonfinite = !(isfinite(out->loss) && isfinite(out->reward_sum));
    return out->nonfinite ? ANAKIN_E_NONFINITE : ANAKIN_OK;
}

extern "C" int32_t anakin_get_plan(const anakin_t* h, anakin_plan* out)
{
    if (!h || !out) return ANAKIN_E_INVALID_ARG;
    memset(out, 0, sizeof *out);
    const NetShape& n = h->net;
    out->n_hidden = n.L;
    for (int l = 0; l <= n.L; ++l) out->splits[l] = h->splits[l];
    out->splits_walls = h->splits_w;
    out->head_fan = h->head_fan;
    out->bf16_matrix_path = bf16_mfma(h) ? 1 : 0;
    if (out->bf16_matrix_path)
        for (int l = 1; l < n.L; ++l)
            out->dx_rows[l] = bf16_dx_resident(n, h->B * h->T, l) ? bf16_dx_rows_per_workgroup(h->B * h->T, n.dims[l], n.dims[l + 1]) : 0;
    out->updates_per_unroll = h->n_updates;
    return ANAKIN_OK;
}

extern "C" int32_t anakin_set_mode(anakin_t* h, int32_t flags)
{
    NEED(h);
    if (flags & ~(ANAKIN_MODE_VALU_GEMM | ANAKIN_MODE_CANONICAL_ACTING | ANAKIN_MODE_STREAM_WEIGHTS)) { h->err = "unknown mode flag"; return ANAKIN_E_INVALID_ARG; }
    const int ref = ANAKIN_MODE_CANONICAL_ACTING | ANAKIN_MODE_VALU_GEMM;
    if (h->net.bf16 && h->bf16_path && (flags & ref) != 0 && (flags & ref) != ref) {
        h->err = "bf16 networks: the two reference-path flags go together (activation storage differs between the paths)";
        return ANAKIN_E_INVALID_ARG;
    }
    h->mode = flags;
    return ANAKIN_OK;
}

extern "C" const char* anakin_last_error(const anakin_t* h)
{
    return h ? h->err.c_str() : g_create_error.c_str();
}
