// Acting for bf16 networks on the matrix cores (paper figure 2 top; section 2.1
// loop).  Same persistent structure as the fp32 kernels: a workgroup of eight
// wavefronts owns 64 environments for the whole unroll, env state in registers,
// activations in LDS (bf16), trajectory and hidden activations to HBM.
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
// maze the wall plane and the goal never change, so their contribution (bias +
// wall rows + goal row) is computed once per launch, on the matrix cores, and
// then lives in registers for the whole unroll; each step adds the agent row.
// Hidden activations go to HBM sample-packed (see learn_bf16.hip) straight
// from registers: the accumulator layout of the MFMA holds four consecutive
// samples of one column, half of a packed group.
//
// Weights of the hidden layers are read from L2 in operand tiles (one KiB per
// wavefront load, see internal.h), prefetched four 16-input steps ahead into a
// double register buffer; two wavefronts per SIMD cover the rest of the latency.
//
// Operand layout of v_mfma_f32_32x32x16_bf16 (verified on gfx950): lane l feeds
// A[row l%32][k 8*(l/32) .. +7] and B[k 8*(l/32) .. +7][col l%32]; accumulator
// register r of lane l is D[row 8*(r/4) + 4*(l/32) + r%4][col l%32].
#include "internal.h"

namespace ank {

typedef __bf16 bf8 __attribute__((ext_vector_type(8)));
typedef float f16v __attribute__((ext_vector_type(16)));

constexpr int BTM = 64;                 // envs per workgroup
constexpr int BWG = 512;                // threads per workgroup: two wavefronts per SIMD
constexpr int BOBS = 12;                // observation words per env (as in the fp32 kernels)

typedef __bf16 bf2 __attribute__((ext_vector_type(2)));
typedef uint32_t u32v2 __attribute__((ext_vector_type(2)));
typedef uint32_t u32v4 __attribute__((ext_vector_type(4)));

__device__ __forceinline__ float bf2f(uint16_t h) { return bf16_to_f(h); }
// two floats rounded to bfloat16 (round to nearest even), low half first
__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi)
{
    bf2 v;
    v[0] = (__bf16)lo; v[1] = (__bf16)hi;
    return __builtin_bit_cast(uint32_t, v);
}
__device__ __forceinline__ float relu(float x) { return x > 0.0f ? x : 0.0f; }
// two packed ReLU outputs (never negative, never -0) -> 1 in bit 0 resp. bit 16 where the half is not zero
__device__ __forceinline__ uint32_t nonzero_flags_pk(uint32_t w)
{
    uint32_t r;
    const uint32_t one = 0x00010001u;
    asm("v_pk_min_u16 %0, %1, %2" : "=v"(r) : "v"(w), "v"(one));
    return r;
}

struct RolloutBf16Args {
    EnvDims env;
    NetShape net;
    TrajPtrs tp;                         // tp.act[] point to bf16 buffers here
    const float* theta;                  // fp32 master (biases are read from here)
    const uint16_t* w;                   // bf16 copy of theta, same indexing
    const uint16_t* wt;                  // bf16 copy in matrix-core operand tiles (heads: [NH][HL])
    float* prefix;                       // [B][H1] first-layer prefix (bias + wall rows + goal row), maze only
    int B, T, ldx;                       // ldx: LDS row stride in bf16 elements
    int keep_acts;                       // store the packed hidden activations for the update
    uint64_t seed, gstep;
};

// Hidden layer on the matrix cores: Y[64][N] = relu(X[64][K] W + b), X and Y bf16 in LDS.
// Wavefront w computes columns [32*NT*w, 32*NT*(w+1)); wavefronts past N stay idle.
// gP: sample-packed copy of Y in HBM (null: not kept), g8: first sample group of this tile.
template <int NT>
__device__ __forceinline__ void bf16_layer(const uint16_t* __restrict__ X, uint16_t* __restrict__ Y, int ldx,
                                           const uint16_t* __restrict__ Wt, const float* __restrict__ bias,
                                           int K, int N, int wave, int lane, uint16_t* __restrict__ gP, size_t g8,
                                           uint32_t* __restrict__ gM)
{
    const int l32 = lane & 31, kg = lane >> 5;
    const int n0 = wave * 32 * NT;
    if (n0 >= N) return;
    f16v acc[2][NT];
#pragma unroll
    for (int t = 0; t < NT; ++t) {
        const float b = bias[n0 + 32 * t + l32];
#pragma unroll
        for (int r = 0; r < 16; ++r) { acc[0][t][r] = b; acc[1][t][r] = b; }
    }
    const uint16_t* xa = X + l32 * ldx + 8 * kg;
    const int KS = K >> 4;                                       // 16-input steps: 8, 16 or 32
    const uint16_t* wb = Wt + ((size_t)(n0 >> 5) * KS << 9) + lane * 8;
    constexpr int U = 4;                                         // steps per prefetch block
    bf8 w0[U][NT], w1[U][NT];
    auto load = [&](bf8 (&d)[U][NT], int s) {
#pragma unroll
        for (int u = 0; u < U; ++u)
#pragma unroll
            for (int t = 0; t < NT; ++t) d[u][t] = *reinterpret_cast<const bf8*>(wb + ((size_t)(t * KS + s + u) << 9));
    };
    auto compute = [&](const bf8 (&d)[U][NT], int s) {
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const bf8 a0 = *reinterpret_cast<const bf8*>(xa + 16 * (s + u));
            const bf8 a1 = *reinterpret_cast<const bf8*>(xa + 32 * ldx + 16 * (s + u));
#pragma unroll
            for (int t = 0; t < NT; ++t) {
                acc[0][t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a0, d[u][t], acc[0][t], 0, 0, 0);
                acc[1][t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a1, d[u][t], acc[1][t], 0, 0, 0);
            }
        }
    };
    // the scheduling barriers keep every block of loads ahead of the MFMAs of the block before it
    load(w0, 0);
    for (int s = 0; s < KS; s += 2 * U) {
        load(w1, s + U);
        __builtin_amdgcn_sched_barrier(0);
        compute(w0, s);
        if (s + 2 * U < KS) load(w0, s + 2 * U);
        __builtin_amdgcn_sched_barrier(0);
        compute(w1, s + U);
    }
    // register group r/4 of lane (l32, kg) holds rows 8*(r/4) + 4*kg + 0..3 of column l32
#pragma unroll
    for (int mt = 0; mt < 2; ++mt)
#pragma unroll
        for (int t = 0; t < NT; ++t) {
            const int col = n0 + 32 * t + l32;
            uint32_t mk = 0u;
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                const int row = mt * 32 + 8 * g + 4 * kg;
                const uint32_t p01 = pack_bf16x2(relu(acc[mt][t][4 * g]), relu(acc[mt][t][4 * g + 1]));
                const uint32_t p23 = pack_bf16x2(relu(acc[mt][t][4 * g + 2]), relu(acc[mt][t][4 * g + 3]));
                Y[(row + 0) * ldx + col] = (uint16_t)p01; Y[(row + 1) * ldx + col] = (uint16_t)(p01 >> 16);
                Y[(row + 2) * ldx + col] = (uint16_t)p23; Y[(row + 3) * ldx + col] = (uint16_t)(p23 >> 16);
                if (gP) {
                    // written once, read by the update: streaming stores leave the weights in L2
                    u32v2 pv; pv[0] = p01; pv[1] = p23;
                    __builtin_nontemporal_store(pv, reinterpret_cast<u32v2*>(gP + ((g8 + mt * 4 + g) * N + col) * 8 + 4 * kg));
                    mk |= (nonzero_flags_pk(p01) << (2 * g)) | (nonzero_flags_pk(p23) << (2 * g + 1));
                }
            }
            if (gP) __builtin_nontemporal_store(mk, gM + relu_mask_index((g8 >> 2) + mt, kg, N, col));
        }
}

// The same layer for nets whose hidden layers all have this width, with the weight stream running
// across layer boundaries: the first two blocks of the next layer's weights are requested before this
// layer's activations are stored.  Loads and stores of a wavefront complete in issue order, so a load
// issued behind the activation stores is not seen as complete until the stores are acknowledged;
// issued ahead of them it costs nothing, and the next layer starts without waiting.
// w0/w1: on entry steps 0..2U-1 of this layer (bf16_layer_first loads them for the first one); on exit,
// with Wt_next, steps 0..2U-1 of the next.
template <int NT>
__device__ __forceinline__ void bf16_layer_stream(const uint16_t* __restrict__ X, uint16_t* __restrict__ Y, int ldx,
                                                  const uint16_t* __restrict__ Wt, const uint16_t* __restrict__ Wt_next,
                                                  const float* __restrict__ bias, int K, int N, int wave, int lane,
                                                  uint16_t* __restrict__ gP, size_t g8, uint32_t* __restrict__ gM,
                                                  bf8 (&w0)[4][NT], bf8 (&w1)[4][NT])
{
    constexpr int U = 4;
    const int l32 = lane & 31, kg = lane >> 5;
    const int n0 = wave * 32 * NT;
    if (n0 >= N) return;
    f16v acc[2][NT];
#pragma unroll
    for (int t = 0; t < NT; ++t) {
        const float b = bias[n0 + 32 * t + l32];
#pragma unroll
        for (int r = 0; r < 16; ++r) { acc[0][t][r] = b; acc[1][t][r] = b; }
    }
    const uint16_t* xa = X + l32 * ldx + 8 * kg;
    const int KS = K >> 4;                                       // the next layer has the same K and N
    const size_t wave_off = ((size_t)(n0 >> 5) * KS << 9) + lane * 8;
    const uint16_t* wb = Wt + wave_off;
    const uint16_t* wn = Wt_next ? Wt_next + wave_off : wb;
    auto load = [&](bf8 (&d)[U][NT], const uint16_t* base, int s) {
#pragma unroll
        for (int u = 0; u < U; ++u)
#pragma unroll
            for (int t = 0; t < NT; ++t) d[u][t] = *reinterpret_cast<const bf8*>(base + ((size_t)(t * KS + s + u) << 9));
    };
    auto compute = [&](const bf8 (&d)[U][NT], int s) {
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const bf8 a0 = *reinterpret_cast<const bf8*>(xa + 16 * (s + u));
            const bf8 a1 = *reinterpret_cast<const bf8*>(xa + 32 * ldx + 16 * (s + u));
#pragma unroll
            for (int t = 0; t < NT; ++t) {
                acc[0][t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a0, d[u][t], acc[0][t], 0, 0, 0);
                acc[1][t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a1, d[u][t], acc[1][t], 0, 0, 0);
            }
        }
    };
    for (int s = 0; s < KS; s += 2 * U) {
        const bool last = s + 2 * U >= KS;
        __builtin_amdgcn_sched_barrier(0);
        compute(w0, s);
        if (!last) load(w0, wb, s + 2 * U);
        else if (Wt_next) load(w0, wn, 0);
        __builtin_amdgcn_sched_barrier(0);
        compute(w1, s + U);
        if (!last) load(w1, wb, s + 3 * U);
        else if (Wt_next) load(w1, wn, U);
    }
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int mt = 0; mt < 2; ++mt)
#pragma unroll
        for (int t = 0; t < NT; ++t) {
            const int col = n0 + 32 * t + l32;
            uint32_t mk = 0u;
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                const int row = mt * 32 + 8 * g + 4 * kg;
                const uint32_t p01 = pack_bf16x2(relu(acc[mt][t][4 * g]), relu(acc[mt][t][4 * g + 1]));
                const uint32_t p23 = pack_bf16x2(relu(acc[mt][t][4 * g + 2]), relu(acc[mt][t][4 * g + 3]));
                Y[(row + 0) * ldx + col] = (uint16_t)p01; Y[(row + 1) * ldx + col] = (uint16_t)(p01 >> 16);
                Y[(row + 2) * ldx + col] = (uint16_t)p23; Y[(row + 3) * ldx + col] = (uint16_t)(p23 >> 16);
                if (gP) {
                    u32v2 pv; pv[0] = p01; pv[1] = p23;
                    __builtin_nontemporal_store(pv, reinterpret_cast<u32v2*>(gP + ((g8 + mt * 4 + g) * N + col) * 8 + 4 * kg));
                    mk |= (nonzero_flags_pk(p01) << (2 * g)) | (nonzero_flags_pk(p23) << (2 * g + 1));
                }
            }
            if (gP) __builtin_nontemporal_store(mk, gM + relu_mask_index((g8 >> 2) + mt, kg, N, col));
        }
}

template <int NT>
__device__ __forceinline__ void bf16_layer_first(const uint16_t* __restrict__ Wt, int K, int N, int wave, int lane,
                                                 bf8 (&w0)[4][NT], bf8 (&w1)[4][NT])
{
    const int n0 = wave * 32 * NT;
    if (n0 >= N) return;
    const int KS = K >> 4;
    const uint16_t* wb = Wt + ((size_t)(n0 >> 5) * KS << 9) + lane * 8;
#pragma unroll
    for (int u = 0; u < 4; ++u)
#pragma unroll
        for (int t = 0; t < NT; ++t) {
            w0[u][t] = *reinterpret_cast<const bf8*>(wb + ((size_t)(t * KS + u) << 9));
            w1[u][t] = *reinterpret_cast<const bf8*>(wb + ((size_t)(t * KS + 4 + u) << 9));
        }
}

__device__ __forceinline__ void run_bf16_layer(const uint16_t* X, uint16_t* Y, int ldx, const uint16_t* Wt, const float* bias,
                                               int K, int N, int wave, int lane, uint16_t* gP, size_t g8, uint32_t* gM)
{
    if (N >= 512) bf16_layer<2>(X, Y, ldx, Wt, bias, K, N, wave, lane, gP, g8, gM);
    else bf16_layer<1>(X, Y, ldx, Wt, bias, K, N, wave, lane, gP, g8, gM);
}

// H1: width of the first hidden layer (128, 256 or 512).  Thread (pair of columns cp, env slice eq)
// owns columns 2*cp, 2*cp+1 of the first layer for EPT = H1/16 consecutive environments.
// REPLAY: the learner's pass over a stored unroll (decoupled acting and learning): states from the stored
// snapshots, head outputs and values to tp.tr_head / tp.tr_val (pointed at the learner's buffers), nothing
// sampled or stepped.
template <int ENV, int H1, bool UNI, bool REPLAY>
__global__ __launch_bounds__(BWG) void rollout_bf16_kernel(const RolloutBf16Args a)
{
    extern __shared__ uint4 smem4[];
    uint16_t* bufA = reinterpret_cast<uint16_t*>(smem4);
    const int ldx = a.ldx, NH = a.net.NH, NHP = a.net.NHP, L = a.net.L, HL = a.net.dims[a.net.L];
    const int D = a.net.dims[0];
    const int ldh = HL + 8;
    uint16_t* bufB = bufA + BTM * ldx;
    uint16_t* whs = bufB + BTM * ldx;                            // [8][HL + 8] head weights, rows >= NH zero
    float* hp = reinterpret_cast<float*>(whs + 8 * ldh);         // [4][64][8] partial head sums per quarter of HL
    uint32_t* obs = reinterpret_cast<uint32_t*>(hp + 4 * BTM * 8);
    uint32_t* rng = obs + BTM * BOBS;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int b0 = blockIdx.x * BTM;
    const int B = a.B, T = a.T;
    const TrajPtrs& tp = a.tp;
    const uint16_t* w1 = a.w + a.net.w_off[0];
    constexpr int EPT = H1 / 16;
    const int cp = tid % (H1 / 2), eq = tid / (H1 / 2);
    const int c = 2 * cp, e0 = eq * EPT;

    EnvState st{0u, 0.0f, 0.0f};
    const bool owner = tid < BTM;
    const int b = b0 + tid;
    float hb[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) hb[j] = j < NH ? a.theta[a.net.bh_off + j] : 0.0f;
    if (owner) {
        if (!REPLAY) {
            st.s0 = tp.s0[b];
            if (ENV == ENV_PENDULUM) { st.f0 = tp.f0[b]; st.f1 = tp.f1[b]; }
        }
        if (ENV == ENV_MAZE) for (int w = 0; w < 8; ++w) obs[tid * BOBS + w] = tp.walls[(size_t)w * B + b];
    }
    for (int i = tid; i < 8 * ldh; i += BWG) {
        const int k = i / ldh, j = i - k * ldh;
        whs[i] = (k < NH && j < HL) ? a.wt[a.net.wh_off + (size_t)k * HL + j] : (uint16_t)0;
    }
    __syncthreads();
    // first-layer constants of this thread: the bias, plus -- for the maze -- the contribution of the wall
    // plane and of the goal cell, which never change: prefix[64][H1] = b1 + Walls[64][cells] W1[cells][H1]
    // on the matrix cores, handed over through HBM once per launch
    float pre[ENV == ENV_MAZE ? EPT : 1][2];
    const float bias0 = a.theta[a.net.b_off[0] + c], bias1 = a.theta[a.net.b_off[0] + c + 1];
    if (ENV == ENV_MAZE) {
        const int n = a.env.rows * a.env.cols;
        const int l32 = lane & 31, kg = lane >> 5;
        constexpr int NT1 = H1 >= 512 ? 2 : 1;
        const int n0 = wave * 32 * NT1;
        if (n0 < H1) {
            f16v acc[2][NT1];
#pragma unroll
            for (int t4 = 0; t4 < NT1; ++t4) {
                const float bb = a.theta[a.net.b_off[0] + n0 + 32 * t4 + l32];
#pragma unroll
                for (int r = 0; r < 16; ++r) { acc[0][t4][r] = bb; acc[1][t4][r] = bb; }
            }
            const int KS = D >> 4;
            const uint16_t* wb = a.wt + a.net.w_off[0] + ((size_t)(n0 >> 5) * KS << 9) + lane * 8;   // operand tiles of W1
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
                for (int t4 = 0; t4 < NT1; ++t4) {
                    const bf8 bv = *reinterpret_cast<const bf8*>(wb + ((size_t)(t4 * KS + (k0 >> 4)) << 9));
                    acc[0][t4] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(av[0], bv, acc[0][t4], 0, 0, 0);
                    acc[1][t4] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(av[1], bv, acc[1][t4], 0, 0, 0);
                }
            }
#pragma unroll
            for (int mt = 0; mt < 2; ++mt)
#pragma unroll
                for (int t4 = 0; t4 < NT1; ++t4)
#pragma unroll
                    for (int r = 0; r < 16; ++r) {
                        const int row = mt * 32 + 8 * (r >> 2) + 4 * kg + (r & 3);
                        a.prefix[(size_t)(b0 + row) * H1 + n0 + 32 * t4 + l32] = acc[mt][t4][r];
                    }
        }
        __syncthreads();
        const uint32_t goal = *reinterpret_cast<const uint32_t*>(w1 + (size_t)(3 * n - 1) * H1 + c);
        const float g0 = bf2f((uint16_t)(goal & 0xffffu)), g1 = bf2f((uint16_t)(goal >> 16));
#pragma unroll
        for (int m = 0; m < EPT; ++m) {
            const float2 p = *reinterpret_cast<const float2*>(a.prefix + (size_t)(b0 + e0 + m) * H1 + c);
            pre[ENV == ENV_MAZE ? m : 0][0] = p.x + g0;
            pre[ENV == ENV_MAZE ? m : 0][1] = p.y + g1;
        }
    }
    float wp[3][2] = {{0, 0}, {0, 0}, {0, 0}};                   // pendulum: the three rows of W1
    if (ENV == ENV_PENDULUM) {
#pragma unroll
        for (int k = 0; k < 3; ++k) {
            const uint32_t ww = *reinterpret_cast<const uint32_t*>(w1 + (size_t)k * H1 + c);
            wp[k][0] = bf2f((uint16_t)(ww & 0xffffu)); wp[k][1] = bf2f((uint16_t)(ww >> 16));
        }
    }

    const int tid_outer = tid;
    for (int t = 0; t <= T; ++t) {
        // everything derived from the thread index is recomputed every step from a value the compiler
        // cannot see through: dozens of loop-invariant addresses would otherwise be kept in registers
        // across the whole time loop, on top of the 2 * EPT prefix values, and spilled
        int tid_step = tid_outer;
        asm volatile("" : "+v"(tid_step));
        const int tid = tid_step, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
        const int cp = tid % (H1 / 2), eq = tid / (H1 / 2);
        const int c = 2 * cp, e0 = eq * EPT;
        const bool owner = tid < BTM;
        const int b = b0 + tid;
        const size_t tb = (size_t)t * B + b;
        if (owner) {
            if (REPLAY) {
                st.s0 = tp.tr_s0[tb];
                if (ENV == ENV_PENDULUM) { st.f0 = tp.tr_f0[tb]; st.f1 = tp.tr_f1[tb]; }
            } else {
                tp.tr_s0[tb] = st.s0;
                if (ENV == ENV_PENDULUM) { tp.tr_f0[tb] = st.f0; tp.tr_f1[tb] = st.f1; }
            }
            if (ENV == ENV_CATCH) {
                int bc, pc;
                catch_obs_cells(a.env, st.s0, bc, pc);
                obs[tid * BOBS + 0] = (uint32_t)bc; obs[tid * BOBS + 1] = (uint32_t)pc;
            } else if (ENV == ENV_PENDULUM) {
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
        const bool keep = t < T && a.keep_acts;
        const size_t g8 = ((size_t)t * B + b0) >> 3;             // first sample group of this tile
        // the last wavefront draws this step's random numbers while it waits for its weight rows
        if (!REPLAY && wave == 7 && t < T) {
            const u32x4 w = philox(a.seed, (uint32_t)(b0 + lane), a.gstep + (uint64_t)t, DOM_ACTION);
            rng[lane * 2] = ENV == ENV_PENDULUM ? bits_from_f(gaussian_noise(w.x, w.y)) : w.x;   // the noise is ready when the heads are
            rng[lane * 2 + 1] = w.y;
        }
        // ---- first layer: fp32 gather-sum / three fmas, rounded to bf16 ----------
        {
            const int n = a.env.rows * a.env.cols;
            uint32_t r0[ENV == ENV_PENDULUM ? 1 : EPT], r1[ENV == ENV_CATCH ? EPT : 1];
            if (ENV != ENV_PENDULUM) {
                // all weight-row loads of this thread in flight before the first is used
#pragma unroll
                for (int m = 0; m < EPT; ++m) {
                    const int row0 = ENV == ENV_CATCH ? (int)obs[(e0 + m) * BOBS + 0] : n + (int)obs[(e0 + m) * BOBS + 8];
                    r0[ENV == ENV_PENDULUM ? 0 : m] = *reinterpret_cast<const uint32_t*>(w1 + (size_t)row0 * H1 + c);
                    if (ENV == ENV_CATCH)
                        r1[ENV == ENV_CATCH ? m : 0] = *reinterpret_cast<const uint32_t*>(w1 + (size_t)obs[(e0 + m) * BOBS + 1] * H1 + c);
                }
            }
            uint16_t* actP = keep ? reinterpret_cast<uint16_t*>(tp.act[0]) : nullptr;
            // with 32 environments per thread (H1 = 512) a thread holds whole 32-sample stages of its two columns
            // and writes their ReLU masks (both row halves); narrower first layers leave the mask to the activations
            uint32_t mkx[2] = {0u, 0u}, mky[2] = {0u, 0u};
#pragma unroll
            for (int m0 = 0; m0 < EPT; m0 += 8) {
                float v[8][2];
#pragma unroll
                for (int q = 0; q < 8; ++q) {
                    const int m = m0 + q;
                    float vx = ENV == ENV_MAZE ? pre[ENV == ENV_MAZE ? m : 0][0] : bias0;
                    float vy = ENV == ENV_MAZE ? pre[ENV == ENV_MAZE ? m : 0][1] : bias1;
                    if (ENV == ENV_PENDULUM) {
#pragma unroll
                        for (int k = 0; k < 3; ++k) {
                            const float x = f_from_bits(obs[(e0 + m) * BOBS + k]);
                            vx = fmaf(x, wp[k][0], vx); vy = fmaf(x, wp[k][1], vy);
                        }
                    } else {
                        const uint32_t g = r0[ENV == ENV_PENDULUM ? 0 : m];
                        vx += bf2f((uint16_t)(g & 0xffffu)); vy += bf2f((uint16_t)(g >> 16));
                        if (ENV == ENV_CATCH) {
                            const uint32_t g1 = r1[ENV == ENV_CATCH ? m : 0];
                            vx += bf2f((uint16_t)(g1 & 0xffffu)); vy += bf2f((uint16_t)(g1 >> 16));
                        }
                    }
                    v[q][0] = relu(vx); v[q][1] = relu(vy);
                }
                uint32_t px[4], py[4];
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    px[q] = pack_bf16x2(v[2 * q][0], v[2 * q + 1][0]);
                    py[q] = pack_bf16x2(v[2 * q][1], v[2 * q + 1][1]);
                    // rows m0+2q and m0+2q+1 of the LDS tile, both columns as one 4-byte store
                    *reinterpret_cast<uint32_t*>(bufA + (e0 + m0 + 2 * q) * ldx + c) = (px[q] & 0xffffu) | (py[q] << 16);
                    *reinterpret_cast<uint32_t*>(bufA + (e0 + m0 + 2 * q + 1) * ldx + c) = (px[q] >> 16) | (py[q] & 0xffff0000u);
                }
                if (actP) {
                    u32v4* dst = reinterpret_cast<u32v4*>(actP + ((g8 + (e0 >> 3)) * H1 + c) * 8) + (size_t)(m0 >> 3) * H1;   // 16-byte units: one group of eight samples is H1 of them
                    u32v4 vx4, vy4;
#pragma unroll
                    for (int q = 0; q < 4; ++q) { vx4[q] = px[q]; vy4[q] = py[q]; }
                    __builtin_nontemporal_store(vx4, dst);
                    __builtin_nontemporal_store(vy4, dst + 1);
                    if (EPT == 32) {
#pragma unroll
                        for (int k2 = 0; k2 < 2; ++k2) {
                            mkx[k2] |= (nonzero_flags_pk(px[2 * k2]) << (m0 >> 2)) | (nonzero_flags_pk(px[2 * k2 + 1]) << ((m0 >> 2) + 1));
                            mky[k2] |= (nonzero_flags_pk(py[2 * k2]) << (m0 >> 2)) | (nonzero_flags_pk(py[2 * k2 + 1]) << ((m0 >> 2) + 1));
                        }
                    }
                }
            }
            if (actP && EPT == 32) {
#pragma unroll
                for (int k2 = 0; k2 < 2; ++k2) {
                    u32v2 mv; mv[0] = mkx[k2]; mv[1] = mky[k2];
                    __builtin_nontemporal_store(mv, reinterpret_cast<u32v2*>(tp.mask[0] + relu_mask_index((g8 >> 2) + (e0 >> 5), k2, H1, c)));
                }
            }
        }
        __syncthreads();
        uint16_t* cur = bufA;
        uint16_t* nxt = bufB;
        if (UNI) {
            constexpr int NTU = H1 >= 512 ? 2 : 1;
            bf8 w0[4][NTU], w1[4][NTU];
            bf16_layer_first<NTU>(a.wt + a.net.w_off[1], H1, H1, wave, lane, w0, w1);
            for (int l = 1; l < L; ++l) {
                bf16_layer_stream<NTU>(cur, nxt, ldx, a.wt + a.net.w_off[l], l + 1 < L ? a.wt + a.net.w_off[l + 1] : nullptr,
                                       a.theta + a.net.b_off[l], H1, H1, wave, lane,
                                       keep ? reinterpret_cast<uint16_t*>(tp.act[l]) : nullptr, g8, tp.mask[l], w0, w1);
                __syncthreads();
                uint16_t* tmp = cur; cur = nxt; nxt = tmp;
            }
        } else {
            for (int l = 1; l < L; ++l) {
                const int K = a.net.dims[l], N = a.net.dims[l + 1];
                run_bf16_layer(cur, nxt, ldx, a.wt + a.net.w_off[l], a.theta + a.net.b_off[l], K, N, wave, lane,
                               keep ? reinterpret_cast<uint16_t*>(tp.act[l]) : nullptr, g8, tp.mask[l]);
                __syncthreads();
                uint16_t* tmp = cur; cur = nxt; nxt = tmp;
            }
        }
        // ---- heads: wavefront (tile, quarter) sums one quarter of the last layer for 32 envs ----
        {
            const int l32 = lane & 31, kg = lane >> 5;
            const int tile = wave & 1, kq = wave >> 1, kq_len = HL >> 2;
            f16v acc;
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[r] = 0.0f;
            const uint16_t* xa = cur + (tile * 32 + l32) * ldx + kq * kq_len + 8 * kg;
            const uint16_t* wbs = whs + (l32 & 7) * ldh + kq * kq_len + 8 * kg;
            const bool real = l32 < 8;
            // one base address, recomputed every step, and constant offsets from it: sixteen loop-invariant
            // addresses would otherwise be kept (and spilled) across the time loop
            int hp_base = (kq * BTM + tile * 32 + 4 * kg) * 8 + l32;
            asm volatile("" : "+v"(hp_base));
            for (int k0 = 0; k0 < kq_len; k0 += 16) {
                const bf8 av = *reinterpret_cast<const bf8*>(xa + k0);
                bf8 bvv = *reinterpret_cast<const bf8*>(wbs + k0);
                if (!real) {
#pragma unroll
                    for (int q = 0; q < 8; ++q) bvv[q] = (__bf16)0.0f;
                }
                acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(av, bvv, acc, 0, 0, 0);
            }
            if (real) {
#pragma unroll
                for (int r = 0; r < 16; ++r) hp[hp_base + (8 * (r >> 2) + (r & 3)) * 8] = acc[r];
            }
        }
        __syncthreads();
        if (owner) {
            float hv[8] = {0, 0, 0, 0, 0, 0, 0, 0};
#pragma unroll
            for (int j = 0; j < 8; ++j)
                if (j < NH) {
                    float s = hb[j];
#pragma unroll
                    for (int q = 0; q < 4; ++q) s += hp[(q * BTM + tid) * 8 + j];
                    hv[j] = s;
                }
            float* hd = tp.tr_head + tb * NHP;
            *reinterpret_cast<float4*>(hd) = make_float4(hv[0], hv[1], hv[2], hv[3]);
            if (NHP == 8) *reinterpret_cast<float4*>(hd + 4) = make_float4(hv[4], hv[5], hv[6], hv[7]);
            const float val = last_head(hv[0], hv[1], hv[2], hv[3], hv[4], hv[5], hv[6], hv[7], NH);
            tp.tr_val[tb] = val;
            if (!REPLAY && t < T) {
                const uint2 dr = *reinterpret_cast<const uint2*>(rng + tid * 2);
                float r; int done;
                if (ENV == ENV_PENDULUM) {
                    const float eps = f_from_bits(dr.x);
                    const float act = gaussian_action(hv[0], hv[1], eps);
                    tp.tr_eps[tb] = eps; tp.tr_actf[tb] = act;
                    pendulum_step(a.env, st, act, 0u, 0u, r, done);
                    if (done) {
                        const u32x4 wr = philox(a.seed, (uint32_t)b, a.gstep + (uint64_t)t, DOM_RESET);
                        pendulum_reset(st, wr.x, wr.y);
                    }
                } else {
                    const int act = sample_categorical_any(hv[0], hv[1], hv[2], hv[3], hv[4], hv[5], hv[6], hv[7], a.net.A, u01(dr.x));
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
    if (!REPLAY && owner) {
        tp.s0[b] = st.s0;
        if (ENV == ENV_PENDULUM) { tp.f0[b] = st.f0; tp.f1[b] = st.f1; }
    }
}

// can this net act on the bf16 matrix-core path?
bool rollout_bf16_ok(const NetShape& net, const EnvDims& env, int B)
{
    if (!net.bf16 || B % BTM) return false;
    if (env.kind == ENV_MAZE && (env.rows * env.cols) % 16) return false;   // wall plane in whole 16-cell steps
    for (int l = 1; l <= net.L; ++l) {
        const int n = net.dims[l];
        if (n != 128 && n != 256 && n != 512) return false;     // 1, 2 or 4 tiles of 32 columns per wavefront, 64-input prefetch blocks
    }
    return true;
}

void fill_rollout_args(anakin* h, RolloutArgs& a);

// what: 0 the acting unroll, 1 the actor of a decoupled step (behaviour copies of the parameters, its own prefix
// buffer, no activations kept), 2 the learner's replay of the stored unroll with the current parameters
template <bool REPLAY>
static hipError_t launch_bf16_forward(anakin* h, int what)
{
    RolloutArgs base;
    fill_rollout_args(h, base);
    const Layout& L = h->lay;
    RolloutBf16Args a;
    a.env = base.env; a.net = base.net; a.tp = base.tp; a.theta = base.theta;
    a.w = at<const uint16_t>(h, L.w_bf16); a.wt = at<const uint16_t>(h, L.wt_bf16);
    a.prefix = at<float>(h, L.prefix);
    a.keep_acts = 1;
    if (what == 1) {
        a.theta = at<const float>(h, L.theta_b); a.w = at<const uint16_t>(h, L.w_bf16_b); a.wt = at<const uint16_t>(h, L.wt_bf16_b);
        a.prefix = at<float>(h, L.prefix_b);
        a.keep_acts = 0;
    } else if (what == 2) {
        a.tp.tr_head = at<float>(h, L.head_new); a.tp.tr_val = at<float>(h, L.val_new);
    }
    a.B = h->B; a.T = h->T; a.seed = h->seed; a.gstep = h->gstep;
    int hmax = 0;
    for (int l = 1; l <= h->net.L; ++l) hmax = h->net.dims[l] > hmax ? h->net.dims[l] : hmax;
    a.ldx = hmax + 8;
    const int HL = h->net.dims[h->net.L], H1 = h->net.dims[1];
    const size_t lds = (size_t)2 * BTM * a.ldx * 2 + (size_t)8 * (HL + 8) * 2 + (size_t)4 * BTM * 8 * 4 + (size_t)BTM * (BOBS + 2) * 4;
    auto launch = [&](auto kern) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) return e;
        ProfScope prof(h, REPLAY ? "replay_forward" : "rollout");
        hipLaunchKernelGGL(kern, dim3(h->B / BTM), dim3(BWG), lds, h->stream, a);
        return hipGetLastError();
    };
    bool uni = true;                                             // every hidden layer H1 wide: the weight stream runs across layers
    for (int l = 2; l <= h->net.L; ++l) uni = uni && h->net.dims[l] == H1;
#define ANK_BF16_W(ENVK, W) (uni ? launch(rollout_bf16_kernel<ENVK, W, true, REPLAY>) : launch(rollout_bf16_kernel<ENVK, W, false, REPLAY>))
#define ANK_BF16_CASE(ENVK) (H1 == 128 ? ANK_BF16_W(ENVK, 128) : H1 == 256 ? ANK_BF16_W(ENVK, 256) : ANK_BF16_W(ENVK, 512))
    switch (h->env.kind) {
        case ENV_CATCH:    return ANK_BF16_CASE(ENV_CATCH);
        case ENV_PENDULUM: return ANK_BF16_CASE(ENV_PENDULUM);
        default:           return ANK_BF16_CASE(ENV_MAZE);
    }
#undef ANK_BF16_CASE
#undef ANK_BF16_W
}

hipError_t launch_rollout_bf16(anakin* h) { return launch_bf16_forward<false>(h, 0); }
hipError_t launch_rollout_bf16_behaviour(anakin* h) { return launch_bf16_forward<false>(h, 1); }
hipError_t launch_replay_bf16(anakin* h) { return launch_bf16_forward<true>(h, 2); }

}  // namespace ank
