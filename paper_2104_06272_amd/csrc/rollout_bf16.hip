// Acting for bf16 networks on the matrix cores (paper figure 2 top; section 2.1
// loop).  Same persistent structure as the fp32 kernels: a workgroup owns 64
// environments for the whole unroll, env state in registers, activations in
// LDS (bf16), trajectory and hidden activations to HBM.
//
// Numerics (bf16 workload): weights and layer inputs are bfloat16, products are
// exact in fp32, accumulation is fp32 inside v_mfma_f32_32x32x16_bf16, bias and
// ReLU are applied in fp32 and the result is rounded to bfloat16 for the next
// layer; head outputs stay fp32.  The accumulation order inside the bf16 MFMA
// is the hardware's, so head outputs agree with a sequential fp32 chain only
// to rounding; sampling and env stepping downstream are exact functions of the
// head outputs the kernel stores.
//
// The first layer is a gather-sum over the 0/1 observation in fp32.  For the
// maze the wall plane never changes, so its contribution (bias + wall rows) is
// computed once per launch, on the matrix cores, into a per-env prefix; each
// step adds the agent row and the goal row.  Hidden activations are written
// to HBM sample-packed (see learn_bf16.hip).
//
// Operand layout of v_mfma_f32_32x32x16_bf16 (verified on gfx950): lane l feeds
// A[row l%32][k 8*(l/32) .. +7] and B[k 8*(l/32) .. +7][col l%32]; accumulator
// register r of lane l is D[row 8*(r/4) + 4*(l/32) + r%4][col l%32].
#include "internal.h"

namespace ank {

typedef __bf16 bf8 __attribute__((ext_vector_type(8)));
typedef float f16v __attribute__((ext_vector_type(16)));

constexpr int BTM = 64;                 // envs per workgroup
constexpr int BOBS = 12;                // observation words per env (as in the fp32 kernels)

__device__ __forceinline__ float bf2f(uint16_t h) { return bf16_to_f(h); }

struct RolloutBf16Args {
    EnvDims env;
    NetShape net;
    TrajPtrs tp;                         // tp.act[] point to bf16 buffers here
    const float* theta;                  // fp32 master (biases are read from here)
    const uint16_t* w;                   // bf16 copy of theta, same indexing
    const uint16_t* wt;                  // bf16 copy with every weight matrix transposed ([N][K])
    float* prefix;                       // [B][H1] first-layer prefix (bias + wall rows)
    int B, T, ldx;                       // ldx: LDS row stride in bf16 elements
    uint64_t seed, gstep;
};

// hidden layer on the matrix cores: Y[64][N] = relu(X[64][K] W + b), X and Y bf16 in LDS
template <int NT>
__device__ __forceinline__ void bf16_layer(const uint16_t* __restrict__ X, uint16_t* __restrict__ Y, int ldx,
                                           const uint16_t* __restrict__ Wt, const float* __restrict__ bias,
                                           int K, int N, int tid)
{
    const int lane = tid & 63, wave = tid >> 6, l32 = lane & 31, kg = lane >> 5;
    const int n0 = wave * (N >> 2);
    f16v acc[2][NT];
#pragma unroll
    for (int t = 0; t < NT; ++t) {
        const float b = bias[n0 + 32 * t + l32];
#pragma unroll
        for (int r = 0; r < 16; ++r) { acc[0][t][r] = b; acc[1][t][r] = b; }
    }
    const uint16_t* xa = X + l32 * ldx + 8 * kg;
    const uint16_t* wb = Wt + (size_t)(n0 + l32) * K + 8 * kg;
    constexpr int U = 2;                                        // k-steps per prefetch block
    bf8 bc[U][NT], bn[U][NT];
#pragma unroll
    for (int u = 0; u < U; ++u)
#pragma unroll
        for (int t = 0; t < NT; ++t) bc[u][t] = *reinterpret_cast<const bf8*>(wb + (size_t)(32 * t) * K + 16 * u);
    for (int k0 = 0; k0 < K; k0 += 16 * U) {
        if (k0 + 16 * U < K) {
#pragma unroll
            for (int u = 0; u < U; ++u)
#pragma unroll
                for (int t = 0; t < NT; ++t)
                    bn[u][t] = *reinterpret_cast<const bf8*>(wb + (size_t)(32 * t) * K + k0 + 16 * U + 16 * u);
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const bf8 a0 = *reinterpret_cast<const bf8*>(xa + k0 + 16 * u);
            const bf8 a1 = *reinterpret_cast<const bf8*>(xa + 32 * ldx + k0 + 16 * u);
#pragma unroll
            for (int t = 0; t < NT; ++t) {
                acc[0][t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a0, bc[u][t], acc[0][t], 0, 0, 0);
                acc[1][t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a1, bc[u][t], acc[1][t], 0, 0, 0);
            }
        }
#pragma unroll
        for (int u = 0; u < U; ++u)
#pragma unroll
            for (int t = 0; t < NT; ++t) bc[u][t] = bn[u][t];
    }
#pragma unroll
    for (int mt = 0; mt < 2; ++mt)
#pragma unroll
        for (int t = 0; t < NT; ++t)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int row = mt * 32 + 8 * (r >> 2) + 4 * kg + (r & 3);
                const float v = acc[mt][t][r] > 0.0f ? acc[mt][t][r] : 0.0f;
                Y[row * ldx + n0 + 32 * t + l32] = bf16_bits(v);
            }
}

__device__ __forceinline__ void run_bf16_layer(const uint16_t* X, uint16_t* Y, int ldx, const uint16_t* Wt, const float* bias,
                                               int K, int N, int tid)
{
    switch (N >> 7) {                                           // tiles per wavefront: N / 4 / 32
        case 1: bf16_layer<1>(X, Y, ldx, Wt, bias, K, N, tid); break;
        case 2: bf16_layer<2>(X, Y, ldx, Wt, bias, K, N, tid); break;
        default: bf16_layer<4>(X, Y, ldx, Wt, bias, K, N, tid); break;
    }
}

// copy of a [64][N] bf16 tile from LDS to the sample-packed activation buffer P8[M/8][N][8]
// (eight consecutive samples of one feature adjacent): piece (group g, column c) gathers a
// column of eight rows from LDS and is stored with one 16-byte write, coalesced across c.
// g: first group of this tile in the buffer.
__device__ __forceinline__ void store_tile_packed(const uint16_t* __restrict__ Y, int ldx, uint16_t* __restrict__ gP,
                                                  size_t g, int N, int tid)
{
    for (int p = tid; p < 8 * N; p += WG) {
        const int gi = p / N, c = p - gi * N;
        const uint16_t* y = Y + (gi * 8) * ldx + c;
        uint32_t w[4];
#pragma unroll
        for (int q = 0; q < 4; ++q) w[q] = (uint32_t)y[(2 * q) * ldx] | ((uint32_t)y[(2 * q + 1) * ldx] << 16);
        *reinterpret_cast<uint4*>(gP + ((g + gi) * N + c) * 8) = make_uint4(w[0], w[1], w[2], w[3]);
    }
}

template <int ENV>
__global__ __launch_bounds__(WG) void rollout_bf16_kernel(const RolloutBf16Args a)
{
    extern __shared__ uint4 smem4[];
    uint16_t* bufA = reinterpret_cast<uint16_t*>(smem4);
    const int ldx = a.ldx, NH = a.net.NH, NHP = a.net.NHP, L = a.net.L, HL = a.net.dims[a.net.L];
    const int H1 = a.net.dims[1], D = a.net.dims[0];
    uint16_t* bufB = bufA + BTM * ldx;
    float* heads = reinterpret_cast<float*>(bufB + BTM * ldx);   // [64][NHP]
    uint32_t* obs = reinterpret_cast<uint32_t*>(heads + BTM * NHP);
    uint32_t* rng = obs + BTM * BOBS;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int b0 = blockIdx.x * BTM;
    const int B = a.B, T = a.T;
    const TrajPtrs& tp = a.tp;
    const uint16_t* w1 = a.w + a.net.w_off[0];

    EnvState st{0u, 0.0f, 0.0f};
    const bool owner = tid < BTM;
    const int b = b0 + tid;
    if (owner) {
        st.s0 = tp.s0[b];
        if (ENV == ENV_PENDULUM) { st.f0 = tp.f0[b]; st.f1 = tp.f1[b]; }
        if (ENV == ENV_MAZE) for (int w = 0; w < 8; ++w) obs[tid * BOBS + w] = tp.walls[(size_t)w * B + b];
    }
    __syncthreads();
    // first-layer prefix per env: the bias, plus -- for the maze -- the contribution of the wall
    // plane, which never changes: prefix[64][H1] = b1 + Walls[64][cells] W1[cells][H1] on the matrix cores
    if (ENV == ENV_MAZE) {
        const int n = a.env.rows * a.env.cols;
        const int l32 = lane & 31, kg = lane >> 5;
        const int n0 = wave * (H1 >> 2);
        const int NT1 = H1 >> 7;                                 // 32-column tiles per wavefront (1, 2 or 4)
        f16v acc[2][4];
#pragma unroll
        for (int t4 = 0; t4 < 4; ++t4) {
            const float bb = t4 < NT1 ? a.theta[a.net.b_off[0] + n0 + 32 * t4 + l32] : 0.0f;
#pragma unroll
            for (int r = 0; r < 16; ++r) { acc[0][t4][r] = bb; acc[1][t4][r] = bb; }
        }
        const uint16_t* wb = a.wt + a.net.w_off[0] + (size_t)(n0 + l32) * D + 8 * kg;     // W1^T: [H1][D]
        for (int k0 = 0; k0 < n; k0 += 16) {
            bf8 av[2];
#pragma unroll
            for (int mt = 0; mt < 2; ++mt) {
                const int cell = k0 + 8 * kg;
                const uint32_t bits = (obs[(mt * 32 + l32) * BOBS + (cell >> 5)] >> (cell & 31)) & 0xffu;
#pragma unroll
                for (int q = 0; q < 8; ++q) av[mt][q] = ((bits >> q) & 1u) ? (__bf16)1.0f : (__bf16)0.0f;
            }
#pragma unroll
            for (int t4 = 0; t4 < 4; ++t4) {
                if (t4 < NT1) {
                    const bf8 bv = *reinterpret_cast<const bf8*>(wb + (size_t)(32 * t4) * D + k0);
                    acc[0][t4] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(av[0], bv, acc[0][t4], 0, 0, 0);
                    acc[1][t4] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(av[1], bv, acc[1][t4], 0, 0, 0);
                }
            }
        }
#pragma unroll
        for (int mt = 0; mt < 2; ++mt)
#pragma unroll
            for (int t4 = 0; t4 < 4; ++t4)
                if (t4 < NT1) {
#pragma unroll
                    for (int r = 0; r < 16; ++r) {
                        const int row = mt * 32 + 8 * (r >> 2) + 4 * kg + (r & 3);
                        a.prefix[(size_t)(b0 + row) * H1 + n0 + 32 * t4 + l32] = acc[mt][t4][r];
                    }
                }
    } else {
        for (int c = tid; c < H1; c += WG) {
            const float bb = a.theta[a.net.b_off[0] + c];
            for (int m = 0; m < BTM; ++m) a.prefix[(size_t)(b0 + m) * H1 + c] = bb;
        }
    }
    __syncthreads();

    for (int t = 0; t <= T; ++t) {
        const size_t tb = (size_t)t * B + b;
        if (owner) {
            tp.tr_s0[tb] = st.s0;
            if (ENV == ENV_CATCH) {
                int bc, pc;
                catch_obs_cells(a.env, st.s0, bc, pc);
                obs[tid * BOBS + 0] = (uint32_t)bc; obs[tid * BOBS + 1] = (uint32_t)pc;
            } else if (ENV == ENV_PENDULUM) {
                tp.tr_f0[tb] = st.f0; tp.tr_f1[tb] = st.f1;
                float sn, cs;
                det_sincos(st.f0, sn, cs);
                obs[tid * BOBS + 0] = bits_from_f(bf16_to_f(bf16_bits(cs)));
                obs[tid * BOBS + 1] = bits_from_f(bf16_to_f(bf16_bits(sn)));
                obs[tid * BOBS + 2] = bits_from_f(bf16_to_f(bf16_bits(st.f1)));
            } else {
                obs[tid * BOBS + 8] = st.s0 & 0xffffu;
            }
        }
        __syncthreads();
        const bool keep = t < T;
        // ---- first layer: fp32 gather-sum / three fmas, rounded to bf16 ----------
        for (int c = 2 * tid; c < H1; c += 2 * WG) {
#pragma unroll 8
            for (int m = 0; m < BTM; ++m) {
                const float2 p = *reinterpret_cast<const float2*>(a.prefix + (size_t)(b0 + m) * H1 + c);
                float vx = p.x, vy = p.y;
                if (ENV == ENV_PENDULUM) {
#pragma unroll
                    for (int k = 0; k < 3; ++k) {
                        const float x = f_from_bits(obs[m * BOBS + k]);
                        const uint32_t ww = *reinterpret_cast<const uint32_t*>(w1 + (size_t)k * H1 + c);
                        vx = fmaf(x, bf2f((uint16_t)(ww & 0xffffu)), vx); vy = fmaf(x, bf2f((uint16_t)(ww >> 16)), vy);
                    }
                } else {
                    const int n = a.env.rows * a.env.cols;
                    const int r0 = ENV == ENV_CATCH ? (int)obs[m * BOBS + 0] : n + (int)obs[m * BOBS + 8];
                    const int r1 = ENV == ENV_CATCH ? (int)obs[m * BOBS + 1] : 3 * n - 1;
                    const uint32_t w0 = *reinterpret_cast<const uint32_t*>(w1 + (size_t)r0 * H1 + c);
                    const uint32_t w1v = *reinterpret_cast<const uint32_t*>(w1 + (size_t)r1 * H1 + c);
                    vx += bf2f((uint16_t)(w0 & 0xffffu)); vy += bf2f((uint16_t)(w0 >> 16));
                    vx += bf2f((uint16_t)(w1v & 0xffffu)); vy += bf2f((uint16_t)(w1v >> 16));
                }
                vx = vx > 0.0f ? vx : 0.0f; vy = vy > 0.0f ? vy : 0.0f;
                *reinterpret_cast<uint32_t*>(bufA + m * ldx + c) = (uint32_t)bf16_bits(vx) | ((uint32_t)bf16_bits(vy) << 16);
            }
        }
        __syncthreads();
        const size_t g8 = ((size_t)t * B + b0) >> 3;             // first sample group of this tile
        if (keep) store_tile_packed(bufA, ldx, reinterpret_cast<uint16_t*>(tp.act[0]), g8, H1, tid);
        uint16_t* cur = bufA;
        uint16_t* nxt = bufB;
        for (int l = 1; l < L; ++l) {
            const int K = a.net.dims[l], N = a.net.dims[l + 1];
            run_bf16_layer(cur, nxt, ldx, a.wt + a.net.w_off[l], a.theta + a.net.b_off[l], K, N, tid);
            __syncthreads();
            if (keep) store_tile_packed(nxt, ldx, reinterpret_cast<uint16_t*>(tp.act[l]), g8, N, tid);
            uint16_t* tmp = cur; cur = nxt; nxt = tmp;
        }
        // ---- heads: two wavefronts, one 32-env tile each, columns >= NH are zero ----
        if (wave < 2) {
            const int l32 = lane & 31, kg = lane >> 5;
            const bool real = l32 < NH;
            const float bv = real ? a.theta[a.net.bh_off + l32] : 0.0f;
            f16v acc;
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[r] = bv;
            const uint16_t* xa = cur + (wave * 32 + l32) * ldx + 8 * kg;
            const uint16_t* wb = a.wt + a.net.wh_off + (size_t)(real ? l32 : 0) * HL + 8 * kg;   // heads stored [NH][HL]
            for (int k0 = 0; k0 < HL; k0 += 16) {
                const bf8 av = *reinterpret_cast<const bf8*>(xa + k0);
                bf8 bvv = *reinterpret_cast<const bf8*>(wb + k0);
                if (!real) {
#pragma unroll
                    for (int q = 0; q < 8; ++q) bvv[q] = (__bf16)0.0f;
                }
                acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(av, bvv, acc, 0, 0, 0);
            }
            if (real) {
#pragma unroll
                for (int r = 0; r < 16; ++r) heads[(wave * 32 + 8 * (r >> 2) + 4 * kg + (r & 3)) * NHP + l32] = acc[r];
            }
        } else if (t < T) {
            // the other two wavefronts produce this step's random draws meanwhile
            for (int e = tid - 2 * 64; e < BTM; e += 2 * 64) {
                const u32x4 w = philox(a.seed, (uint32_t)(b0 + e), a.gstep + (uint64_t)t, DOM_ACTION);
                rng[e * 4] = w.x;
                rng[e * 4 + 1] = w.y;
            }
        }
        __syncthreads();
        if (owner) {
            float hv[8] = {0, 0, 0, 0, 0, 0, 0, 0};
#pragma unroll
            for (int j = 0; j < 8; ++j) if (j < NH) hv[j] = heads[tid * NHP + j];
            float* hd = tp.tr_head + tb * NHP;
            *reinterpret_cast<float4*>(hd) = make_float4(hv[0], hv[1], hv[2], hv[3]);
            if (NHP == 8) *reinterpret_cast<float4*>(hd + 4) = make_float4(hv[4], hv[5], hv[6], hv[7]);
            float val = hv[0];
#pragma unroll
            for (int j = 1; j < 8; ++j) if (j == NH - 1) val = hv[j];
            tp.tr_val[tb] = val;
            if (t < T) {
                const uint2 dr = *reinterpret_cast<const uint2*>(rng + tid * 4);
                float r; int done;
                if (ENV == ENV_PENDULUM) {
                    float eps, act;
                    sample_gaussian(hv[0], hv[1], dr.x, dr.y, eps, act);
                    tp.tr_eps[tb] = eps; tp.tr_actf[tb] = act;
                    pendulum_step(a.env, st, act, 0u, 0u, r, done);
                    if (done) {
                        const u32x4 wr = philox(a.seed, (uint32_t)b, a.gstep + (uint64_t)t, DOM_RESET);
                        pendulum_reset(st, wr.x, wr.y);
                    }
                } else {
                    const int act = sample_categorical<8>(hv, a.net.A, u01(dr.x));
                    tp.tr_act[tb] = (uint8_t)act;
                    if (ENV == ENV_CATCH) {
                        catch_step(a.env, st, act, 0u, r, done);
                        if (done) {
                            const u32x4 wr = philox(a.seed, (uint32_t)b, a.gstep + (uint64_t)t, DOM_RESET);
                            st.s0 = catch_reset(a.env, wr.x);
                        }
                    } else {
                        const uint32_t* wl = obs + tid * BOBS;
                        maze_step(a.env, st, act, [wl](int c) { return ((wl[c >> 5] >> (c & 31)) & 1u) != 0u; }, r, done);
                    }
                }
                tp.tr_rew[tb] = r;
                tp.tr_done[tb] = (uint8_t)done;
            }
        }
    }
    if (owner) {
        tp.s0[b] = st.s0;
        if (ENV == ENV_PENDULUM) { tp.f0[b] = st.f0; tp.f1[b] = st.f1; }
    }
}

// can this net act on the bf16 matrix-core path?
bool rollout_bf16_ok(const NetShape& net, int B)
{
    if (!net.bf16 || B % BTM) return false;
    for (int l = 1; l <= net.L; ++l) if (net.dims[l] > 512 || net.dims[l] < 128) return false;   // 1..4 tiles of 32 columns per wavefront
    if (net.dims[net.L] % 16) return false;
    return true;
}

void fill_rollout_args(anakin* h, RolloutArgs& a);

hipError_t launch_rollout_bf16(anakin* h)
{
    RolloutArgs base;
    fill_rollout_args(h, base);
    RolloutBf16Args a;
    a.env = base.env; a.net = base.net; a.tp = base.tp; a.theta = base.theta;
    a.w = at<const uint16_t>(h, h->lay.w_bf16); a.wt = at<const uint16_t>(h, h->lay.wt_bf16);
    a.prefix = at<float>(h, h->lay.prefix);
    a.B = h->B; a.T = h->T; a.seed = h->seed; a.gstep = h->gstep;
    int hmax = 0;
    for (int l = 1; l <= h->net.L; ++l) hmax = h->net.dims[l] > hmax ? h->net.dims[l] : hmax;
    a.ldx = hmax + 8;
    const size_t lds = (size_t)2 * BTM * a.ldx * 2 + (size_t)BTM * h->net.NHP * 4 + (size_t)BTM * (BOBS + 4) * 4;
    auto launch = [&](auto kern) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) return e;
        ProfScope prof(h, "rollout");
        hipLaunchKernelGGL(kern, dim3(h->B / BTM), dim3(WG), lds, h->stream, a);
        return hipGetLastError();
    };
    switch (h->env.kind) {
        case ENV_CATCH:    return launch(rollout_bf16_kernel<ENV_CATCH>);
        case ENV_PENDULUM: return launch(rollout_bf16_kernel<ENV_PENDULUM>);
        default:           return launch(rollout_bf16_kernel<ENV_MAZE>);
    }
}

}  // namespace ank
