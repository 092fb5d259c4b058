// Acting: one persistent launch runs the whole T-step unroll (paper figure 2
// top; section 2.1 loop).  A workgroup owns a tile of TM environments for all T
// steps -- environments never interact, so no grid-wide synchronisation is
// needed -- and per step does: observe, policy/value forward, sample, env step,
// trajectory write.  Env state lives in registers, activations in LDS, the
// trajectory and the hidden activations (reused by the update, paper section
// 3.1) go to HBM time-major.
//
// The forward pass follows the canonical order: every output starts from its
// bias and accumulates x_k * W[k][j] by fused multiply-add for k ascending.
// Each thread owns an RM x 4 register tile of a layer's outputs and walks k
// from 0 upwards, which is exactly that order, so logits are reproducible bit
// for bit and independent of the tiling.  One-hot observations (Catch, Maze)
// turn the first layer into a gather-sum of weight rows in ascending row
// order: fma(0,w,acc) = acc and fma(1,w,acc) = acc + w, the same bits.
#include "internal.h"

namespace ank {

__device__ __forceinline__ float4 ld4(const float* p) { return *reinterpret_cast<const float4*>(p); }
__device__ __forceinline__ float bfr(float x) { return bf16_to_f(bf16_bits(x)); }

template <bool BF>
__device__ __forceinline__ float4 ldw4(const float* p)
{
    float4 w = ld4(p);
    if (BF) { w.x = bfr(w.x); w.y = bfr(w.y); w.z = bfr(w.z); w.w = bfr(w.w); }
    return w;
}

template <int RM, bool BF>
__device__ __forceinline__ void finish_rows(float (&acc)[RM][4], float* __restrict__ Y, int ldx, int m0, int c0,
                                            float* __restrict__ gout, int N)
{
#pragma unroll
    for (int r = 0; r < RM; ++r) {
        float4 o;
        o.x = acc[r][0] > 0.0f ? acc[r][0] : 0.0f;
        o.y = acc[r][1] > 0.0f ? acc[r][1] : 0.0f;
        o.z = acc[r][2] > 0.0f ? acc[r][2] : 0.0f;
        o.w = acc[r][3] > 0.0f ? acc[r][3] : 0.0f;
        if (BF) { o.x = bfr(o.x); o.y = bfr(o.y); o.z = bfr(o.z); o.w = bfr(o.w); }
        *reinterpret_cast<float4*>(Y + (m0 + r) * ldx + c0) = o;
        if (gout) *reinterpret_cast<float4*>(gout + (size_t)(m0 + r) * N + c0) = o;
    }
}

// Y[TM][N] = relu(X[TM][K] W[K][N] + b), X and Y in LDS (row stride ldx), W in global memory
template <int RM, bool BF>
__device__ __forceinline__ void dense_layer(const float* __restrict__ X, float* __restrict__ Y, int ldx,
                                            const float* __restrict__ W, const float* __restrict__ bias,
                                            int K, int N, int tid, float* __restrict__ gout)
{
    const int CG = N >> 2, tn = tid % CG, m0 = (tid / CG) * RM, c0 = tn << 2;
    float acc[RM][4];
    const float4 b = ld4(bias + c0);
#pragma unroll
    for (int r = 0; r < RM; ++r) { acc[r][0] = b.x; acc[r][1] = b.y; acc[r][2] = b.z; acc[r][3] = b.w; }
    const float* wp = W + c0;
    for (int k0 = 0; k0 < K; k0 += 4) {
        const float4 w0 = ldw4<BF>(wp + (size_t)(k0 + 0) * N);
        const float4 w1 = ldw4<BF>(wp + (size_t)(k0 + 1) * N);
        const float4 w2 = ldw4<BF>(wp + (size_t)(k0 + 2) * N);
        const float4 w3 = ldw4<BF>(wp + (size_t)(k0 + 3) * N);
#pragma unroll
        for (int r = 0; r < RM; ++r) {
            const float4 x = ld4(X + (m0 + r) * ldx + k0);
            acc[r][0] = fmaf(x.x, w0.x, acc[r][0]); acc[r][1] = fmaf(x.x, w0.y, acc[r][1]);
            acc[r][2] = fmaf(x.x, w0.z, acc[r][2]); acc[r][3] = fmaf(x.x, w0.w, acc[r][3]);
            acc[r][0] = fmaf(x.y, w1.x, acc[r][0]); acc[r][1] = fmaf(x.y, w1.y, acc[r][1]);
            acc[r][2] = fmaf(x.y, w1.z, acc[r][2]); acc[r][3] = fmaf(x.y, w1.w, acc[r][3]);
            acc[r][0] = fmaf(x.z, w2.x, acc[r][0]); acc[r][1] = fmaf(x.z, w2.y, acc[r][1]);
            acc[r][2] = fmaf(x.z, w2.z, acc[r][2]); acc[r][3] = fmaf(x.z, w2.w, acc[r][3]);
            acc[r][0] = fmaf(x.w, w3.x, acc[r][0]); acc[r][1] = fmaf(x.w, w3.y, acc[r][1]);
            acc[r][2] = fmaf(x.w, w3.z, acc[r][2]); acc[r][3] = fmaf(x.w, w3.w, acc[r][3]);
        }
    }
    finish_rows<RM, BF>(acc, Y, ldx, m0, c0, gout, N);
}

// per-env observation descriptor in LDS: 12 words per env
//   Catch: [0] ball cell, [1] paddle cell;  Pendulum: [0..2] = (cos, sin, theta_dot) as floats;
//   Maze: [0..7] wall words, [8] agent cell
constexpr int OBS_WORDS = 12;

// first layer: gather-sum for the one-hot boards, three fmas for the pendulum
template <int ENV, int RM, bool BF>
__device__ __forceinline__ void first_layer(const RolloutArgs& a, const uint32_t* __restrict__ obs,
                                            float* __restrict__ Y, int ldx, int tid, float* __restrict__ gout)
{
    const int N = a.net.dims[1];
    const int CG = N >> 2, tn = tid % CG, m0 = (tid / CG) * RM, c0 = tn << 2;
    const float* wp = a.theta + a.net.w_off[0] + c0;
    float acc[RM][4];
    const float4 b = ld4(a.theta + a.net.b_off[0] + c0);
#pragma unroll
    for (int r = 0; r < RM; ++r) { acc[r][0] = b.x; acc[r][1] = b.y; acc[r][2] = b.z; acc[r][3] = b.w; }
    if (ENV == ENV_CATCH) {
#pragma unroll
        for (int r = 0; r < RM; ++r) {
#pragma unroll
            for (int which = 0; which < 2; ++which) {
                const int cell = (int)obs[(m0 + r) * OBS_WORDS + which];
                const float4 w = ldw4<BF>(wp + (size_t)cell * N);
                acc[r][0] += w.x; acc[r][1] += w.y; acc[r][2] += w.z; acc[r][3] += w.w;
            }
        }
    } else if (ENV == ENV_PENDULUM) {
#pragma unroll
        for (int k = 0; k < 3; ++k) {
            const float4 w = ldw4<BF>(wp + (size_t)k * N);
#pragma unroll
            for (int r = 0; r < RM; ++r) {
                float x = f_from_bits(obs[(m0 + r) * OBS_WORDS + k]);
                if (BF) x = bfr(x);
                acc[r][0] = fmaf(x, w.x, acc[r][0]); acc[r][1] = fmaf(x, w.y, acc[r][1]);
                acc[r][2] = fmaf(x, w.z, acc[r][2]); acc[r][3] = fmaf(x, w.w, acc[r][3]);
            }
        }
    } else {
        const int n = a.env.rows * a.env.cols;
        for (int c = 0; c < n; ++c) {                       // wall plane, ascending cell index
            const float4 w = ldw4<BF>(wp + (size_t)c * N);
#pragma unroll
            for (int r = 0; r < RM; ++r) {
                if ((obs[(m0 + r) * OBS_WORDS + (c >> 5)] >> (c & 31)) & 1u) {
                    acc[r][0] += w.x; acc[r][1] += w.y; acc[r][2] += w.z; acc[r][3] += w.w;
                }
            }
        }
#pragma unroll
        for (int r = 0; r < RM; ++r) {                      // agent plane
            const int cell = (int)obs[(m0 + r) * OBS_WORDS + 8];
            const float4 w = ldw4<BF>(wp + (size_t)(n + cell) * N);
            acc[r][0] += w.x; acc[r][1] += w.y; acc[r][2] += w.z; acc[r][3] += w.w;
        }
        {                                                   // goal plane: always the last cell
            const float4 w = ldw4<BF>(wp + (size_t)(3 * n - 1) * N);
#pragma unroll
            for (int r = 0; r < RM; ++r) { acc[r][0] += w.x; acc[r][1] += w.y; acc[r][2] += w.z; acc[r][3] += w.w; }
        }
    }
    finish_rows<RM, BF>(acc, Y, ldx, m0, c0, gout, N);
}

template <int ENV, bool BF>
__device__ __forceinline__ void run_first_layer(const RolloutArgs& a, int TM, const uint32_t* obs, float* Y, int tid, float* gout)
{
    const int RM = TM * a.net.dims[1] / 1024;
    switch (RM) {
        case 1: first_layer<ENV, 1, BF>(a, obs, Y, a.ldx, tid, gout); break;
        case 2: first_layer<ENV, 2, BF>(a, obs, Y, a.ldx, tid, gout); break;
        case 4: first_layer<ENV, 4, BF>(a, obs, Y, a.ldx, tid, gout); break;
        case 8: first_layer<ENV, 8, BF>(a, obs, Y, a.ldx, tid, gout); break;
        default: first_layer<ENV, 16, BF>(a, obs, Y, a.ldx, tid, gout); break;
    }
}

template <bool BF>
__device__ __forceinline__ void run_dense_layer(const RolloutArgs& a, int TM, int l, const float* X, float* Y, int tid, float* gout)
{
    const int K = a.net.dims[l], N = a.net.dims[l + 1];
    const float* W = a.theta + a.net.w_off[l];
    const float* bias = a.theta + a.net.b_off[l];
    const int RM = TM * N / 1024;
    switch (RM) {
        case 1: dense_layer<1, BF>(X, Y, a.ldx, W, bias, K, N, tid, gout); break;
        case 2: dense_layer<2, BF>(X, Y, a.ldx, W, bias, K, N, tid, gout); break;
        case 4: dense_layer<4, BF>(X, Y, a.ldx, W, bias, K, N, tid, gout); break;
        case 8: dense_layer<8, BF>(X, Y, a.ldx, W, bias, K, N, tid, gout); break;
        default: dense_layer<16, BF>(X, Y, a.ldx, W, bias, K, N, tid, gout); break;
    }
}

template <int ENV, bool BF>
__global__ __launch_bounds__(WG) void rollout_kernel(const RolloutArgs a, const int TM)
{
    extern __shared__ float4 smem4[];
    float* smem = reinterpret_cast<float*>(smem4);
    const int ldx = a.ldx, NH = a.net.NH, NHP = a.net.NHP, L = a.net.L, HL = a.net.dims[a.net.L];
    float* bufA = smem;
    float* bufB = bufA + TM * ldx;
    float* whs = bufB + TM * ldx;                 // [HL][NHP] head weights
    float* bhs = whs + HL * NHP;                  // [8] head biases
    float* heads = bhs + 8;                       // [TM][NHP]
    uint32_t* obs = reinterpret_cast<uint32_t*>(heads + TM * NHP);   // [TM][OBS_WORDS]

    const int tid = threadIdx.x;
    const int b0 = blockIdx.x * TM;
    const int B = a.B, T = a.T;
    const TrajPtrs& tp = a.tp;

    // head weights into LDS once
    for (int i = tid; i < HL * NHP; i += WG) {
        const int k = i / NHP, j = i - k * NHP;
        float w = 0.0f;
        if (j < NH) { w = a.theta[a.net.wh_off + k * NH + j]; if (BF) w = bfr(w); }
        whs[i] = w;
    }
    if (tid < 8) bhs[tid] = tid < NH ? a.theta[a.net.bh_off + tid] : 0.0f;

    // env state of this thread's environment (threads 0..TM-1)
    EnvState st{0u, 0.0f, 0.0f};
    const bool owner = tid < TM;
    const int b = b0 + tid;
    if (owner) {
        st.s0 = tp.s0[b];
        if (ENV == ENV_PENDULUM) { st.f0 = tp.f0[b]; st.f1 = tp.f1[b]; }
        if (ENV == ENV_MAZE) {
            for (int w = 0; w < 8; ++w) obs[tid * OBS_WORDS + w] = tp.walls[(size_t)w * B + b];
        }
    }

    for (int t = 0; t <= T; ++t) {
        const size_t tb = (size_t)t * B + b;
        // ---- observe -------------------------------------------------------
        if (owner) {
            tp.tr_s0[tb] = st.s0;
            if (ENV == ENV_CATCH) {
                int bc, pc;
                catch_obs_cells(a.env, st.s0, bc, pc);
                obs[tid * OBS_WORDS + 0] = (uint32_t)bc;
                obs[tid * OBS_WORDS + 1] = (uint32_t)pc;
            } else if (ENV == ENV_PENDULUM) {
                tp.tr_f0[tb] = st.f0;
                tp.tr_f1[tb] = st.f1;
                float sn, cs;
                det_sincos(st.f0, sn, cs);
                obs[tid * OBS_WORDS + 0] = bits_from_f(cs);
                obs[tid * OBS_WORDS + 1] = bits_from_f(sn);
                obs[tid * OBS_WORDS + 2] = bits_from_f(st.f1);
            } else {
                obs[tid * OBS_WORDS + 8] = st.s0 & 0xffffu;
            }
        }
        __syncthreads();
        // ---- forward -------------------------------------------------------
        const bool keep = t < T;                 // the bootstrap evaluation keeps no activations
        float* g0 = keep ? tp.act[0] + ((size_t)t * B + b0) * a.net.dims[1] : nullptr;
        run_first_layer<ENV, BF>(a, TM, obs, bufA, tid, g0);
        __syncthreads();
        float* cur = bufA;
        float* nxt = bufB;
        for (int l = 1; l < L; ++l) {
            float* gl = keep ? tp.act[l] + ((size_t)t * B + b0) * a.net.dims[l + 1] : nullptr;
            run_dense_layer<BF>(a, TM, l, cur, nxt, tid, gl);
            __syncthreads();
            float* tmp = cur; cur = nxt; nxt = tmp;
        }
        for (int idx = tid; idx < TM * NH; idx += WG) {
            const int m = idx % TM, j = idx / TM;
            float acc = bhs[j];
            const float* x = cur + m * ldx;
            for (int k0 = 0; k0 < HL; k0 += 4) {
                const float4 xv = ld4(x + k0);
                acc = fmaf(xv.x, whs[(k0 + 0) * NHP + j], acc);
                acc = fmaf(xv.y, whs[(k0 + 1) * NHP + j], acc);
                acc = fmaf(xv.z, whs[(k0 + 2) * NHP + j], acc);
                acc = fmaf(xv.w, whs[(k0 + 3) * NHP + j], acc);
            }
            heads[m * NHP + j] = acc;
        }
        __syncthreads();
        // ---- sample, step, record -------------------------------------------
        if (owner) {
            const float4 h0 = ld4(heads + tid * NHP);
            const float4 h1 = NHP == 8 ? ld4(heads + tid * NHP + 4) : make_float4(0.0f, 0.0f, 0.0f, 0.0f);
            const float hv[8] = {h0.x, h0.y, h0.z, h0.w, h1.x, h1.y, h1.z, h1.w};
            float* hd = tp.tr_head + tb * NHP;
            *reinterpret_cast<float4*>(hd) = h0;
            if (NHP == 8) *reinterpret_cast<float4*>(hd + 4) = h1;
            float val = hv[0];
#pragma unroll
            for (int j = 1; j < 8; ++j) if (j == NH - 1) val = hv[j];
            tp.tr_val[tb] = val;
            if (t < T) {
                const uint64_t gt = a.gstep + (uint64_t)t;
                const u32x4 wa = philox(a.seed, (uint32_t)b, gt, DOM_ACTION);
                float r; int done;
                if (ENV == ENV_PENDULUM) {
                    float eps, act;
                    sample_gaussian(hv[0], hv[1], wa.x, wa.y, eps, act);
                    tp.tr_eps[tb] = eps;
                    tp.tr_actf[tb] = act;
                    const u32x4 wr = philox(a.seed, (uint32_t)b, gt, DOM_RESET);
                    pendulum_step(a.env, st, act, wr.x, wr.y, r, done);
                } else {
                    const int act = sample_categorical<8>(hv, a.net.A, u01(wa.x));
                    tp.tr_act[tb] = (uint8_t)act;
                    if (ENV == ENV_CATCH) {
                        const u32x4 wr = philox(a.seed, (uint32_t)b, gt, DOM_RESET);
                        catch_step(a.env, st, act, wr.x, r, done);
                    } else {
                        const uint32_t* wl = obs + tid * OBS_WORDS;
                        maze_step(a.env, st, act, [wl](int c) { return ((wl[c >> 5] >> (c & 31)) & 1u) != 0u; }, r, done);
                    }
                }
                tp.tr_rew[tb] = r;
                tp.tr_done[tb] = (uint8_t)done;
            }
        }
        // the next observe phase writes obs words that only the first layer reads, and
        // two barriers separate that read from this point
    }
    if (owner) {
        tp.s0[b] = st.s0;
        if (ENV == ENV_PENDULUM) { tp.f0[b] = st.f0; tp.f1[b] = st.f1; }
    }
}

int rollout_pick_tile(const NetShape& net, int B)
{
    int lo = 16, hi = 256;
    for (int l = 1; l <= net.L; ++l) {
        const int N = net.dims[l];
        const int mn = 1024 / N > 1 ? 1024 / N : 1;      // RM >= 1
        const int mx = 16 * 1024 / N;                    // RM <= 16
        if (mn > lo) lo = mn;
        if (mx < hi) hi = mx;
    }
    int best = 0;
    for (int tm = 16; tm <= 256; tm *= 2) {
        if (tm < lo || tm > hi || B % tm) continue;
        if (!best) best = tm;                            // smallest valid tile
        if (B / tm >= 256) best = tm;                    // largest tile that still fills the chip
    }
    return best;
}

size_t rollout_lds_bytes(const NetShape& net, const EnvDims&, int TM, int* ldx_out)
{
    int hmax = 0;
    for (int l = 1; l <= net.L; ++l) hmax = net.dims[l] > hmax ? net.dims[l] : hmax;
    const int ldx = hmax + 4;
    if (ldx_out) *ldx_out = ldx;
    size_t words = (size_t)2 * TM * ldx + (size_t)net.dims[net.L] * net.NHP + 8 + (size_t)TM * net.NHP + (size_t)TM * OBS_WORDS;
    return words * 4;
}

template <int ENV, bool BF>
static hipError_t launch_one(anakin* h, const RolloutArgs& a, size_t lds)
{
    auto kern = rollout_kernel<ENV, BF>;
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return e;
    ProfScope prof(h, "rollout");
    hipLaunchKernelGGL(kern, dim3(h->B / h->TM), dim3(WG), lds, h->stream, a, h->TM);
    return hipGetLastError();
}

void fill_rollout_args(anakin* h, RolloutArgs& a);

hipError_t launch_rollout(anakin* h)
{
    RolloutArgs a;
    fill_rollout_args(h, a);
    const size_t lds = rollout_lds_bytes(h->net, h->env, h->TM, nullptr);
    const bool bf = h->net.bf16 != 0;
    switch (h->env.kind) {
        case ENV_CATCH:    return bf ? launch_one<ENV_CATCH, true>(h, a, lds) : launch_one<ENV_CATCH, false>(h, a, lds);
        case ENV_PENDULUM: return bf ? launch_one<ENV_PENDULUM, true>(h, a, lds) : launch_one<ENV_PENDULUM, false>(h, a, lds);
        default:           return bf ? launch_one<ENV_MAZE, true>(h, a, lds) : launch_one<ENV_MAZE, false>(h, a, lds);
    }
}

}  // namespace ank
