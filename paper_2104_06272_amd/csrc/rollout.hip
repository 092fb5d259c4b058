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
//
// Kernels: rollout_kernel (weights streamed, vector ALU or matrix cores),
// rollout_resident_kernel (two-layer nets up to 256 wide, W2 in registers),
// rollout_lane_kernel (one hidden layer: one lane per env).  Each has a REPLAY
// form, the learner's forward pass over a stored unroll for decoupled steps.
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
                                            float* __restrict__ Y, int ldx, int tid, float* __restrict__ gout,
                                            const float* w1, const float* b1)
{
    const int N = a.net.dims[1];
    const int CG = N >> 2, tn = tid % CG, m0 = (tid / CG) * RM, c0 = tn << 2;
    const float* wp = w1 + c0;
    float acc[RM][4];
    const float4 b = ld4(b1 + c0);
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
__device__ __forceinline__ void run_first_layer(const RolloutArgs& a, int TM, const uint32_t* obs, float* Y, int tid, float* gout,
                                                const float* w1)
{
    const float* b1 = a.theta + a.net.b_off[0];
    const int RM = TM * a.net.dims[1] / 1024;
    switch (RM) {
        case 1: first_layer<ENV, 1, BF>(a, obs, Y, a.ldx, tid, gout, w1, b1); break;
        case 2: first_layer<ENV, 2, BF>(a, obs, Y, a.ldx, tid, gout, w1, b1); break;
        case 4: first_layer<ENV, 4, BF>(a, obs, Y, a.ldx, tid, gout, w1, b1); break;
        case 8: first_layer<ENV, 8, BF>(a, obs, Y, a.ldx, tid, gout, w1, b1); break;
        default: first_layer<ENV, 16, BF>(a, obs, Y, a.ldx, tid, gout, w1, b1); break;
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


// ---------------------------------------------------------------------------
// Hidden layers on the matrix cores.  On gfx950 the fp32 MFMA instructions add
// their products one k at a time with a fused multiply-add, ascending in k, and
// chain through the accumulator operand -- measured bit-identical to the
// sequential fmaf chain on random, wide-range and integer inputs -- so starting
// the accumulator from the bias and feeding k in ascending order reproduces
// the canonical order exactly while running at matrix-core rate.
//
// Wavefront w owns output columns [w N/4, (w+1) N/4); lane l feeds column
// w N/4 + NT (l % 16|32) + t of tile t, so one vector load of NT consecutive
// weights per k serves all of the lane's tiles and the epilogue stores NT
// consecutive outputs.  The weights of the next block of k are fetched from L2
// into registers while the current block is multiplied.
// ---------------------------------------------------------------------------
typedef float f4v __attribute__((ext_vector_type(4)));
typedef float f16v __attribute__((ext_vector_type(16)));

template <int NT>
__device__ __forceinline__ void load_nt(const float* __restrict__ p, float (&b)[NT])
{
    if (NT == 1) { b[0] = p[0]; }
    else if (NT == 2) { const float2 v = *reinterpret_cast<const float2*>(p); b[0] = v.x; b[1] = v.y; }
    else {
#pragma unroll
        for (int q = 0; q < NT / 4; ++q) {
            const float4 v = *reinterpret_cast<const float4*>(p + 4 * q);
            b[4 * q + 0] = v.x; b[4 * q + 1] = v.y; b[4 * q + 2] = v.z; b[4 * q + 3] = v.w;
        }
    }
}
template <int NT>
__device__ __forceinline__ void store_nt(float* __restrict__ p, const float (&b)[NT])
{
    if (NT == 1) { p[0] = b[0]; }
    else if (NT == 2) { *reinterpret_cast<float2*>(p) = make_float2(b[0], b[1]); }
    else {
#pragma unroll
        for (int q = 0; q < NT / 4; ++q)
            *reinterpret_cast<float4*>(p + 4 * q) = make_float4(b[4 * q + 0], b[4 * q + 1], b[4 * q + 2], b[4 * q + 3]);
    }
}

// 16 envs per workgroup: v_mfma_f32_16x16x4_f32.  Lane l feeds A[row l%16][k l/16] and
// B[k l/16][col l%16]; accumulator register r of lane l is D[row 4*(l/16) + r][col l%16].
template <int NT>
__device__ __forceinline__ void mfma_layer_m16(const float* __restrict__ X, float* __restrict__ Y, int ldx,
                                               const float* __restrict__ W, const float* __restrict__ bias,
                                               int K, int N, int tid, float* __restrict__ gout)
{
    constexpr int U = NT <= 4 ? 8 : (NT == 8 ? 4 : 2);          // k-steps (of 4) per prefetch block
    const int lane = tid & 63, wave = tid >> 6;
    const int col0 = wave * (N >> 2) + NT * (lane & 15), kq = lane >> 4;
    f4v acc[NT];
    {
        float bv[NT];
        load_nt<NT>(bias + col0, bv);
#pragma unroll
        for (int t = 0; t < NT; ++t) { acc[t][0] = bv[t]; acc[t][1] = bv[t]; acc[t][2] = bv[t]; acc[t][3] = bv[t]; }
    }
    const float* wp = W + (size_t)kq * N + col0;
    const float* xp = X + (lane & 15) * ldx + kq;
    float bc[U][NT], bn[U][NT];
#pragma unroll
    for (int u = 0; u < U; ++u) load_nt<NT>(wp + (size_t)(4 * u) * N, bc[u]);
    for (int k0 = 0; k0 < K; k0 += 4 * U) {
        if (k0 + 4 * U < K) {
#pragma unroll
            for (int u = 0; u < U; ++u) load_nt<NT>(wp + (size_t)(k0 + 4 * U + 4 * u) * N, bn[u]);
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const float av = xp[k0 + 4 * u];
#pragma unroll
            for (int t = 0; t < NT; ++t) acc[t] = __builtin_amdgcn_mfma_f32_16x16x4f32(av, bc[u][t], acc[t], 0, 0, 0);
        }
#pragma unroll
        for (int u = 0; u < U; ++u)
#pragma unroll
            for (int t = 0; t < NT; ++t) bc[u][t] = bn[u][t];
    }
#pragma unroll
    for (int r = 0; r < 4; ++r) {
        const int row = 4 * kq + r;
        float o[NT];
#pragma unroll
        for (int t = 0; t < NT; ++t) o[t] = acc[t][r] > 0.0f ? acc[t][r] : 0.0f;
        store_nt<NT>(Y + row * ldx + col0, o);
        if (gout) store_nt<NT>(gout + (size_t)row * N + col0, o);
    }
}

// 32*MT envs per workgroup: v_mfma_f32_32x32x2_f32.  Lane l feeds A[row l%32][k l/32] and
// B[k l/32][col l%32]; accumulator register r is D[row 8*(r/4) + 4*(l/32) + r%4][col l%32].
template <int MT, int NT>
__device__ __forceinline__ void mfma_layer_m32(const float* __restrict__ X, float* __restrict__ Y, int ldx,
                                               const float* __restrict__ W, const float* __restrict__ bias,
                                               int K, int N, int tid, float* __restrict__ gout)
{
    constexpr int U = NT <= 2 ? 8 : (NT == 4 ? 4 : 2);          // k-steps (of 2) per prefetch block
    const int lane = tid & 63, wave = tid >> 6;
    const int col0 = wave * (N >> 2) + NT * (lane & 31), kq = lane >> 5;
    f16v acc[MT][NT];
    {
        float bv[NT];
        load_nt<NT>(bias + col0, bv);
#pragma unroll
        for (int mt = 0; mt < MT; ++mt)
#pragma unroll
            for (int t = 0; t < NT; ++t)
#pragma unroll
                for (int r = 0; r < 16; ++r) acc[mt][t][r] = bv[t];
    }
    const float* wp = W + (size_t)kq * N + col0;
    const float* xp = X + (lane & 31) * ldx + kq;
    float bc[U][NT], bn[U][NT];
#pragma unroll
    for (int u = 0; u < U; ++u) load_nt<NT>(wp + (size_t)(2 * u) * N, bc[u]);
    for (int k0 = 0; k0 < K; k0 += 2 * U) {
        if (k0 + 2 * U < K) {
#pragma unroll
            for (int u = 0; u < U; ++u) load_nt<NT>(wp + (size_t)(k0 + 2 * U + 2 * u) * N, bn[u]);
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
#pragma unroll
            for (int mt = 0; mt < MT; ++mt) {
                const float av = xp[mt * 32 * ldx + k0 + 2 * u];
#pragma unroll
                for (int t = 0; t < NT; ++t)
                    acc[mt][t] = __builtin_amdgcn_mfma_f32_32x32x2f32(av, bc[u][t], acc[mt][t], 0, 0, 0);
            }
        }
#pragma unroll
        for (int u = 0; u < U; ++u)
#pragma unroll
            for (int t = 0; t < NT; ++t) bc[u][t] = bn[u][t];
    }
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const int row = mt * 32 + 8 * (r >> 2) + 4 * kq + (r & 3);
            float o[NT];
#pragma unroll
            for (int t = 0; t < NT; ++t) o[t] = acc[mt][t][r] > 0.0f ? acc[mt][t][r] : 0.0f;
            store_nt<NT>(Y + row * ldx + col0, o);
            if (gout) store_nt<NT>(gout + (size_t)row * N + col0, o);
        }
}

__device__ __forceinline__ void run_mfma_layer(const RolloutArgs& a, int TM, int l, const float* X, float* Y, int tid, float* gout)
{
    const int K = a.net.dims[l], N = a.net.dims[l + 1];
    const float* W = a.theta + a.net.w_off[l];
    const float* bias = a.theta + a.net.b_off[l];
    if (TM == 16) {
        switch (N >> 6) {                                   // tiles per wavefront: N / 4 / 16
            case 1: mfma_layer_m16<1>(X, Y, a.ldx, W, bias, K, N, tid, gout); break;
            case 2: mfma_layer_m16<2>(X, Y, a.ldx, W, bias, K, N, tid, gout); break;
            case 4: mfma_layer_m16<4>(X, Y, a.ldx, W, bias, K, N, tid, gout); break;
            case 8: mfma_layer_m16<8>(X, Y, a.ldx, W, bias, K, N, tid, gout); break;
            default: mfma_layer_m16<16>(X, Y, a.ldx, W, bias, K, N, tid, gout); break;
        }
    } else if (TM == 32) {
        switch (N >> 7) {                                   // N / 4 / 32
            case 1: mfma_layer_m32<1, 1>(X, Y, a.ldx, W, bias, K, N, tid, gout); break;
            case 2: mfma_layer_m32<1, 2>(X, Y, a.ldx, W, bias, K, N, tid, gout); break;
            case 4: mfma_layer_m32<1, 4>(X, Y, a.ldx, W, bias, K, N, tid, gout); break;
            default: mfma_layer_m32<1, 8>(X, Y, a.ldx, W, bias, K, N, tid, gout); break;
        }
    } else {
        switch (N >> 7) {
            case 1: mfma_layer_m32<2, 1>(X, Y, a.ldx, W, bias, K, N, tid, gout); break;
            case 2: mfma_layer_m32<2, 2>(X, Y, a.ldx, W, bias, K, N, tid, gout); break;
            default: mfma_layer_m32<2, 4>(X, Y, a.ldx, W, bias, K, N, tid, gout); break;
        }
    }
}

// Heads: out[m][j] = bh[j] + sum_k X[m][k] Wh[k][j], one sequential fused multiply-add chain
// per (env, head) as the canonical order demands.  The chain is latency-bound, so what matters
// is that its operands are already in registers: lane (m, j) streams row m of X and row j of
// the transposed head matrix (both k-contiguous in LDS, 16-byte reads), 32 k at a time, with
// the next block in flight while the current one is consumed.
// whT: [NH][ldw] in LDS (ldw = HL + 4).
template <int U>
__device__ __forceinline__ void heads_load(const float* __restrict__ x, const float* __restrict__ w, float4 (&xv)[U], float4 (&wv)[U])
{
#pragma unroll
    for (int u = 0; u < U; ++u) { xv[u] = *reinterpret_cast<const float4*>(x + 4 * u); wv[u] = *reinterpret_cast<const float4*>(w + 4 * u); }
}
template <int U>
__device__ __forceinline__ float heads_fma(const float4 (&xv)[U], const float4 (&wv)[U], float acc)
{
#pragma unroll
    for (int u = 0; u < U; ++u) {
        acc = fmaf(xv[u].x, wv[u].x, acc);
        acc = fmaf(xv[u].y, wv[u].y, acc);
        acc = fmaf(xv[u].z, wv[u].z, acc);
        acc = fmaf(xv[u].w, wv[u].w, acc);
    }
    return acc;
}
typedef float f4v_h __attribute__((ext_vector_type(4)));
// The chains on the vector ALU with the operand reads taken off the critical path: lane (m, j)
// keeps a ring of PF blocks of four k (16-byte LDS reads of row m of X and row j of the transposed
// head matrix) and refills each slot, PF blocks ahead, before the four dependent fused multiply-adds
// of the block it just handed over.  HL is a multiple of 4 * PF.
template <int PF, int HL>
__device__ __forceinline__ void heads_pipe(const float* __restrict__ X, int ldx, const float* __restrict__ whT, int ldw,
                                           const float* __restrict__ bhs, float* __restrict__ heads,
                                           int NH, int NHP, int TM, int tid)
{
    constexpr int S = HL >> 2;
    for (int idx = tid; idx < TM * NH; idx += WG) {
        const int m = idx % TM, j = idx / TM;
        const f4v_h* x = reinterpret_cast<const f4v_h*>(X + m * ldx);
        const f4v_h* w = reinterpret_cast<const f4v_h*>(whT + j * ldw);
        f4v_h xr[PF], wr[PF];
#pragma unroll
        for (int u = 0; u < PF; ++u) { xr[u] = x[u]; wr[u] = w[u]; }
        float acc = bhs[j];
#pragma unroll
        for (int s = 0; s < S; ++s) {
            const f4v_h xv = xr[s % PF], wv = wr[s % PF];
            if (s + PF < S) { xr[s % PF] = x[s + PF]; wr[s % PF] = w[s + PF]; }
            __builtin_amdgcn_sched_barrier(0);
            acc = fmaf(xv[0], wv[0], acc);
            acc = fmaf(xv[1], wv[1], acc);
            acc = fmaf(xv[2], wv[2], acc);
            acc = fmaf(xv[3], wv[3], acc);
        }
        heads[m * NHP + j] = acc;
    }
}

// U: float4 per register block (a block covers 4U values of k; HL is a multiple of 4U)
template <int U>
__device__ __forceinline__ void heads_chain(const float* __restrict__ X, int ldx, const float* __restrict__ whT, int ldw,
                                            const float* __restrict__ bhs, float* __restrict__ heads,
                                            int HL, int NH, int NHP, int TM, int tid)
{
    constexpr int KB = 4 * U;
    for (int idx = tid; idx < TM * NH; idx += WG) {
        const int m = idx % TM, j = idx / TM;
        float acc = bhs[j];
        const float* x = X + m * ldx;
        const float* w = whT + j * ldw;
        float4 xa[U], wa[U], xb[U], wb[U];                      // two register blocks, used alternately
        heads_load<U>(x, w, xa, wa);
        for (int k0 = 0; k0 < HL; k0 += 2 * KB) {
            const bool more = k0 + KB < HL;
            if (more) heads_load<U>(x + k0 + KB, w + k0 + KB, xb, wb);
            acc = heads_fma<U>(xa, wa, acc);
            if (more) {
                if (k0 + 2 * KB < HL) heads_load<U>(x + k0 + 2 * KB, w + k0 + 2 * KB, xa, wa);
                acc = heads_fma<U>(xb, wb, acc);
            }
        }
        heads[m * NHP + j] = acc;
    }
}

__device__ __forceinline__ void run_heads(const float* X, int ldx, const float* whT, int ldw, const float* bhs, float* heads,
                                          int HL, int NH, int NHP, int TM, int tid)
{
    switch (HL) {
        case 64: heads_pipe<4, 64>(X, ldx, whT, ldw, bhs, heads, NH, NHP, TM, tid); break;
        case 128: heads_pipe<4, 128>(X, ldx, whT, ldw, bhs, heads, NH, NHP, TM, tid); break;
        case 256: heads_pipe<4, 256>(X, ldx, whT, ldw, bhs, heads, NH, NHP, TM, tid); break;
        case 512: heads_pipe<4, 512>(X, ldx, whT, ldw, bhs, heads, NH, NHP, TM, tid); break;
        default: heads_chain<8>(X, ldx, whT, ldw, bhs, heads, HL, NH, NHP, TM, tid);
    }
}

// REPLAY: the learner's pass over a stored unroll (decoupled acting and learning): the state of
// step t comes from the stored snapshots, the forward pass is the acting one with the parameters
// in a.theta, head outputs and values go to tp.tr_head / tp.tr_val (the caller points them at the
// learner's buffers) and hidden activations to tp.act; nothing is sampled or stepped.
template <int ENV, bool BF, bool MF, bool REPLAY>
__global__ __launch_bounds__(WG) void rollout_kernel(const RolloutArgs a, const int TM)
{
    extern __shared__ float4 smem4[];
    float* smem = reinterpret_cast<float*>(smem4);
    const int ldx = a.ldx, NH = a.net.NH, NHP = a.net.NHP, L = a.net.L, HL = a.net.dims[a.net.L];
    float* bufA = smem;
    float* bufB = bufA + TM * ldx;
    float* whs = bufB + TM * ldx;                 // [8][HL + 4] head weights, transposed
    float* bhs = whs + 8 * (HL + 4);              // [8] head biases
    float* heads = bhs + 8;                       // [TM][NHP]
    uint32_t* obs = reinterpret_cast<uint32_t*>(heads + TM * NHP);   // [TM][OBS_WORDS]
    uint32_t* rng = obs + TM * OBS_WORDS;                            // [TM][4] draws of the current step

    const int tid = threadIdx.x;
    const int b0 = blockIdx.x * TM;
    const int B = a.B, T = a.T;
    const TrajPtrs& tp = a.tp;

    // head weights into LDS once, transposed: whs[j][k], row stride HL + 4
    const int ldw = HL + 4;
    for (int i = tid; i < HL * NH; i += WG) {
        const int k = i / NH, j = i - k * NH;
        float w = a.theta[a.net.wh_off + i];
        if (BF) w = bfr(w);
        whs[j * ldw + k] = w;
    }
    if (tid < 8) bhs[tid] = tid < NH ? a.theta[a.net.bh_off + tid] : 0.0f;

    // env state of this thread's environment (threads 0..TM-1)
    EnvState st{0u, 0.0f, 0.0f};
    const bool owner = tid < TM;
    const int b = b0 + tid;
    if (owner) {
        if (!REPLAY) {
            st.s0 = tp.s0[b];
            if (ENV == ENV_PENDULUM) { st.f0 = tp.f0[b]; st.f1 = tp.f1[b]; }
        }
        if (ENV == ENV_MAZE) {
            for (int w = 0; w < 8; ++w) obs[tid * OBS_WORDS + w] = tp.walls[(size_t)w * B + b];
        }
    }

    for (int t = 0; t <= T; ++t) {
        const size_t tb = (size_t)t * B + b;
        // ---- observe -------------------------------------------------------
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
                obs[tid * OBS_WORDS + 0] = (uint32_t)bc;
                obs[tid * OBS_WORDS + 1] = (uint32_t)pc;
            } else if (ENV == ENV_PENDULUM) {
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
        const bool keep = t < T && a.keep_acts;  // the bootstrap evaluation keeps no activations
        float* g0 = keep ? tp.act[0] + ((size_t)t * B + b0) * a.net.dims[1] : nullptr;
        run_first_layer<ENV, BF>(a, TM, obs, bufA, tid, g0, a.theta + a.net.w_off[0]);
        __syncthreads();
        float* cur = bufA;
        float* nxt = bufB;
        for (int l = 1; l < L; ++l) {
            float* gl = keep ? tp.act[l] + ((size_t)t * B + b0) * a.net.dims[l + 1] : nullptr;
            if (MF) run_mfma_layer(a, TM, l, cur, nxt, tid, gl);
            else run_dense_layer<BF>(a, TM, l, cur, nxt, tid, gl);
            __syncthreads();
            float* tmp = cur; cur = nxt; nxt = tmp;
        }
        run_heads(cur, ldx, whs, ldw, bhs, heads, HL, NH, NHP, TM, tid);
        // the step's random draws do not depend on the network: the last lanes of the workgroup,
        // idle during the head chains, produce them now
        if (!REPLAY && t < T) {
            for (int e = WG - 1 - tid; e < TM; e += WG) {
                const u32x4 w = philox(a.seed, (uint32_t)(b0 + e), a.gstep + (uint64_t)t, DOM_ACTION);
                // the pendulum's noise is ready-made when the heads are: only z and tanh remain on the critical path
                rng[e * 4] = ENV == ENV_PENDULUM ? bits_from_f(gaussian_noise(w.x, w.y)) : w.x;
                rng[e * 4 + 1] = w.y;
            }
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
            const float val = last_head(hv[0], hv[1], hv[2], hv[3], hv[4], hv[5], hv[6], hv[7], NH);
            tp.tr_val[tb] = val;
            if (!REPLAY && t < T) {
                const uint2 dr = *reinterpret_cast<const uint2*>(rng + tid * 4);   // action draw, words 0 and 1
                float r; int done;
                // the reset draw is only needed where an episode ends: the step runs with a placeholder
                // and the few lanes that finished an episode draw and reset afterwards
                if (ENV == ENV_PENDULUM) {
                    const float eps = f_from_bits(dr.x);
                    const float act = gaussian_action(hv[0], hv[1], eps);
                    tp.tr_eps[tb] = eps;
                    tp.tr_actf[tb] = act;
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
    if (!REPLAY && owner) {
        tp.s0[b] = st.s0;
        if (ENV == ENV_PENDULUM) { tp.f0[b] = st.f0; tp.f1[b] = st.f1; }
    }
}


// ---------------------------------------------------------------------------
// Weights resident on chip.  For two-layer nets up to 256 x 256 the whole
// hidden-to-hidden matrix fits the register file of one compute unit: a CU has
// 4 SIMDs x 512 registers x 64 lanes x 4 B = 512 KB, W2 (256 x 256 fp32) is
// 256 KB, i.e. 256 registers per lane at one wavefront per SIMD.  Each lane
// loads, once per launch, exactly the B-operand values it will feed to the
// matrix cores -- W2[k][its columns] for its k phase -- and reuses them for all
// T+1 forward passes, so the acting loop reads no hidden-layer weight from
// memory at all.  The first layer's matrix (gathered by row) and the head
// matrix sit in LDS.  Everything else is as in rollout_kernel, and the
// accumulation order is the same canonical one.
// ---------------------------------------------------------------------------
template <int KS, int NT>
__device__ __forceinline__ void resident_m16(const float (&wreg)[KS][NT], const float* __restrict__ X, float* __restrict__ Y,
                                             int ldx, const float* __restrict__ bias, int N, int tid, float* __restrict__ gout)
{
    const int lane = tid & 63, wave = tid >> 6;
    const int col0 = wave * (N >> 2) + NT * (lane & 15), kq = lane >> 4;
    f4v acc[NT];
    {
        float bv[NT];
        load_nt<NT>(bias + col0, bv);
#pragma unroll
        for (int t = 0; t < NT; ++t) { acc[t][0] = bv[t]; acc[t][1] = bv[t]; acc[t][2] = bv[t]; acc[t][3] = bv[t]; }
    }
    const float* xp = X + (lane & 15) * ldx + kq;
    // the activation operand of step s + PF is read from LDS before the MFMAs of step s are issued: with one
    // wavefront per SIMD nothing else would hide the LDS latency
    constexpr int PF = 4;
    float ap[PF];
#pragma unroll
    for (int u = 0; u < PF; ++u) ap[u] = xp[4 * u];
#pragma unroll
    for (int s = 0; s < KS; ++s) {
        const float av = ap[s % PF];
        ap[s % PF] = xp[4 * (s + PF < KS ? s + PF : 0)];
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int t = 0; t < NT; ++t) acc[t] = __builtin_amdgcn_mfma_f32_16x16x4f32(av, wreg[s][t], acc[t], 0, 0, 0);
    }
#pragma unroll
    for (int r = 0; r < 4; ++r) {
        const int row = 4 * kq + r;
        float o[NT];
#pragma unroll
        for (int t = 0; t < NT; ++t) o[t] = acc[t][r] > 0.0f ? acc[t][r] : 0.0f;
        store_nt<NT>(Y + row * ldx + col0, o);
        if (gout) store_nt<NT>(gout + (size_t)row * N + col0, o);
    }
}

template <int KS, int NT>
__device__ __forceinline__ void resident_m32(const float (&wreg)[KS][NT], const float* __restrict__ X, float* __restrict__ Y,
                                             int ldx, const float* __restrict__ bias, int N, int tid, float* __restrict__ gout)
{
    const int lane = tid & 63, wave = tid >> 6;
    const int col0 = wave * (N >> 2) + NT * (lane & 31), kq = lane >> 5;
    f16v acc[NT];
    {
        float bv[NT];
        load_nt<NT>(bias + col0, bv);
#pragma unroll
        for (int t = 0; t < NT; ++t)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[t][r] = bv[t];
    }
    const float* xp = X + (lane & 31) * ldx + kq;
    constexpr int PF = 4;                                        // LDS reads run this many steps ahead of their MFMAs
    float ap[PF];
#pragma unroll
    for (int u = 0; u < PF; ++u) ap[u] = xp[2 * u];
#pragma unroll
    for (int s = 0; s < KS; ++s) {
        const float av = ap[s % PF];
        ap[s % PF] = xp[2 * (s + PF < KS ? s + PF : 0)];
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int t = 0; t < NT; ++t) acc[t] = __builtin_amdgcn_mfma_f32_32x32x2f32(av, wreg[s][t], acc[t], 0, 0, 0);
    }
#pragma unroll
    for (int r = 0; r < 16; ++r) {
        const int row = 8 * (r >> 2) + 4 * kq + (r & 3);
        float o[NT];
#pragma unroll
        for (int t = 0; t < NT; ++t) o[t] = acc[t][r] > 0.0f ? acc[t][r] : 0.0f;
        store_nt<NT>(Y + row * ldx + col0, o);
        if (gout) store_nt<NT>(gout + (size_t)row * N + col0, o);
    }
}


// RK x RN: shape of the resident hidden-to-hidden layer; M32: 32 envs per workgroup, else 16
template <int ENV, bool M32, int RK, int RN, bool REPLAY>
__global__ __launch_bounds__(WG) void rollout_resident_kernel(const RolloutArgs a)
{
    constexpr int TM = M32 ? 32 : 16;
    constexpr int KS = M32 ? RK / 2 : RK / 4;                      // MFMA k-steps per forward pass
    constexpr int NT = M32 ? RN / 128 : RN / 64;                   // MFMA tiles per wavefront
    constexpr bool W1_IN_LDS = ENV != ENV_MAZE;
    extern __shared__ float4 smem4[];
    float* smem = reinterpret_cast<float*>(smem4);
    constexpr int HL = RN;
    const int ldx = a.ldx, NH = a.net.NH, NHP = a.net.NHP, D = a.net.dims[0];
    float* bufA = smem;
    float* bufB = bufA + TM * ldx;
    float* whs = bufB + TM * ldx;                 // [8][HL + 4] head weights, transposed
    float* bhs = whs + 8 * (HL + 4);              // [8] head biases
    float* heads = bhs + 8;                       // [TM][NHP]
    uint32_t* obs = reinterpret_cast<uint32_t*>(heads + TM * NHP);   // [TM][OBS_WORDS]
    uint32_t* rng = obs + TM * OBS_WORDS;                            // [TM][4] draws of the current step
    float* b1s = reinterpret_cast<float*>(rng + TM * 4);             // [RK], [RN] biases of the two hidden layers
    float* b2s = b1s + RK;
    float* w1s = b2s + RN;                                           // [D][RK] first-layer weights

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int b0 = blockIdx.x * TM;
    const int B = a.B, T = a.T;
    const TrajPtrs& tp = a.tp;

    // The prologue's loads are issued in batches and land while the hidden-to-hidden matrix streams into the
    // registers: one load, one wait, one LDS store at a time would cost a memory round trip per 4 KB.
    constexpr int ldw = HL + 4;
    constexpr int NWH = HL * 8 / WG;                               // head-matrix elements per lane, at most
    constexpr int W1B = 8;                                         // 16-byte pieces of W1 per lane and batch
    static_assert(RK <= WG && RN <= WG, "one bias element per lane");
    const f4v* w1src = reinterpret_cast<const f4v*>(a.theta + a.net.w_off[0]);
    f4v* w1dst = reinterpret_cast<f4v*>(w1s);
    const int n_w1 = W1_IN_LDS ? D * RK / 4 : 0;
    float vwh[NWH];
    f4v vw1[W1B];
#pragma unroll
    for (int u = 0; u < NWH; ++u) {
        const int i = tid + u * WG;
        vwh[u] = a.theta[a.net.wh_off + (i < HL * NH ? i : 0)];     // unconditional: the stores below select
    }
    const float vbh = a.theta[a.net.bh_off + (tid < NH ? tid : 0)];
    const float vb1 = a.theta[a.net.b_off[0] + (tid < RK ? tid : 0)];
    const float vb2 = a.theta[a.net.b_off[1] + (tid < RN ? tid : 0)];
#pragma unroll
    for (int u = 0; u < W1B; ++u) {
        const int i = tid + u * WG;
        if (W1_IN_LDS) vw1[u] = w1src[i < n_w1 ? i : 0];
    }
    __builtin_amdgcn_sched_barrier(0);
    const float* w1 = W1_IN_LDS ? w1s : a.theta + a.net.w_off[0];

    // this lane's share of W2, in matrix-core operand order
    float wreg[KS][NT];
    {
        const float* W2 = a.theta + a.net.w_off[1];
        const int col0 = wave * (RN >> 2) + NT * (M32 ? (lane & 31) : (lane & 15));
        const int kq = M32 ? (lane >> 5) : (lane >> 4);
        constexpr int kstep = M32 ? 2 : 4;
#pragma unroll
        for (int s = 0; s < KS; ++s) load_nt<NT>(W2 + (size_t)(kstep * s + kq) * RN + col0, wreg[s]);
    }
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int u = 0; u < NWH; ++u) {
        const int i = tid + u * WG;
        const int k = i / NH, j = i - k * NH;
        if (i < HL * NH) whs[j * ldw + k] = vwh[u];
    }
    if (tid < 8) bhs[tid] = tid < NH ? vbh : 0.0f;
    if (tid < RK) b1s[tid] = vb1;
    if (tid < RN) b2s[tid] = vb2;
#pragma unroll
    for (int u = 0; u < W1B; ++u) {
        const int i = tid + u * WG;
        if (i < n_w1) w1dst[i] = vw1[u];
    }
    for (int i0 = W1B * WG; i0 < n_w1; i0 += W1B * WG) {
#pragma unroll
        for (int u = 0; u < W1B; ++u) {
            const int i = i0 + tid + u * WG;
            vw1[u] = w1src[i < n_w1 ? i : 0];
        }
#pragma unroll
        for (int u = 0; u < W1B; ++u) {
            const int i = i0 + tid + u * WG;
            if (i < n_w1) w1dst[i] = vw1[u];
        }
    }

    EnvState st{0u, 0.0f, 0.0f};
    const bool owner = tid < TM;
    const int b = b0 + tid;
    if (owner) {
        if (!REPLAY) {
            st.s0 = tp.s0[b];
            if (ENV == ENV_PENDULUM) { st.f0 = tp.f0[b]; st.f1 = tp.f1[b]; }
        }
        if (ENV == ENV_MAZE) {
            for (int w = 0; w < 8; ++w) obs[tid * OBS_WORDS + w] = tp.walls[(size_t)w * B + b];
        }
    }

    // Everything loaded so far (weights, the envs' states) has arrived before the loop starts.  Inside the
    // loop the acting path then only stores to memory, and no step waits for an earlier step's stores: a
    // wait for a load would be a wait for every older store of the wavefront as well.
    if (!REPLAY) __builtin_amdgcn_s_waitcnt(0x0F70);               // vmcnt(0)

    for (int t = 0; t <= T; ++t) {
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
                obs[tid * OBS_WORDS + 0] = (uint32_t)bc;
                obs[tid * OBS_WORDS + 1] = (uint32_t)pc;
            } else if (ENV == ENV_PENDULUM) {
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
        const bool keep = t < T && a.keep_acts;
        float* g0 = keep ? tp.act[0] + ((size_t)t * B + b0) * RK : nullptr;
        first_layer<ENV, TM * RK / 1024, false>(a, obs, bufA, ldx, tid, g0, w1, b1s);
        __syncthreads();
        float* g1 = keep ? tp.act[1] + ((size_t)t * B + b0) * RN : nullptr;
        if (M32) resident_m32<KS, NT>(wreg, bufA, bufB, ldx, b2s, RN, tid, g1);
        else resident_m16<KS, NT>(wreg, bufA, bufB, ldx, b2s, RN, tid, g1);
        __syncthreads();
        heads_pipe<4, HL>(bufB, ldx, whs, ldw, bhs, heads, NH, NHP, TM, tid);
        // the step's random draws do not depend on the network: the last lanes of the workgroup,
        // idle during the head chains, produce them now -- the action draw of every env and the draw
        // that places the next episode, which then costs nothing where an episode ends
        if (!REPLAY && t < T) {
            for (int i = WG - 1 - tid; i < (ENV == ENV_MAZE ? TM : 2 * TM); i += WG) {
                const int e = i < TM ? i : i - TM;
                const u32x4 w = philox(a.seed, (uint32_t)(b0 + e), a.gstep + (uint64_t)t, i < TM ? DOM_ACTION : DOM_RESET);
                // the pendulum's noise is ready-made when the heads are: only z and tanh remain on the critical path
                const uint32_t w0 = (ENV == ENV_PENDULUM && i < TM) ? bits_from_f(gaussian_noise(w.x, w.y)) : w.x;
                *reinterpret_cast<uint2*>(rng + e * 4 + (i < TM ? 0 : 2)) = make_uint2(w0, w.y);
            }
        }
        __syncthreads();
        // the record of the head outputs is written by the second wavefront, which has nothing else to do here:
        // the lanes that sample and step the envs are the critical path of the whole workgroup (handing the rest
        // of the step's record -- state, action, reward, episode end -- to idle lanes through LDS as well was
        // measured: no further gain)
        if (tid >= 64 && tid < 64 + TM) {
            const int e = tid - 64;
            const size_t te = (size_t)t * B + b0 + e;
            const float4 h0 = ld4(heads + e * NHP);
            const float4 h1 = NHP == 8 ? ld4(heads + e * NHP + 4) : make_float4(0.0f, 0.0f, 0.0f, 0.0f);
            float* hd = tp.tr_head + te * NHP;
            *reinterpret_cast<float4*>(hd) = h0;
            if (NHP == 8) *reinterpret_cast<float4*>(hd + 4) = h1;
            tp.tr_val[te] = last_head(h0.x, h0.y, h0.z, h0.w, h1.x, h1.y, h1.z, h1.w, NH);
        }
        if (owner) {
            const float4 h0 = ld4(heads + tid * NHP);
            const float4 h1 = NHP == 8 ? ld4(heads + tid * NHP + 4) : make_float4(0.0f, 0.0f, 0.0f, 0.0f);
            const float hv[8] = {h0.x, h0.y, h0.z, h0.w, h1.x, h1.y, h1.z, h1.w};
            if (!REPLAY && t < T) {
                const uint4 dr = *reinterpret_cast<const uint4*>(rng + tid * 4);   // action draw, reset draw
                float r; int done;
                if (ENV == ENV_PENDULUM) {
                    const float eps = f_from_bits(dr.x);
                    const float act = gaussian_action(hv[0], hv[1], eps);
                    tp.tr_eps[tb] = eps;
                    tp.tr_actf[tb] = act;
                    pendulum_step(a.env, st, act, dr.z, dr.w, r, done);
                } else {
                    const int act = sample_categorical_any(hv[0], hv[1], hv[2], hv[3], hv[4], hv[5], hv[6], hv[7], a.net.A, u01(dr.x));
                    tp.tr_act[tb] = (uint8_t)act;
                    if (ENV == ENV_CATCH) {
                        catch_step(a.env, st, act, dr.z, r, done);
                    } else {
                        const uint32_t* wl = obs + tid * OBS_WORDS;
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

// ---------------------------------------------------------------------------
// One hidden layer of at most 64 units on a Catch board or the pendulum's three features: the
// whole agent fits one lane.  Lane b keeps its env's state and the H hidden activations in
// registers, gathers its two first-layer rows (or takes three fmas per unit) from an LDS copy
// of W1, runs the NH head chains with the head matrix broadcast from LDS, draws its own random
// numbers, samples, steps and records -- no exchange between lanes, so no barrier inside the
// time loop, and every vector instruction works for 64 envs.  The arithmetic per env is the
// same canonical chain as in rollout_kernel.  No hidden activations are kept: the update of
// such nets rebuilds the layer from the state.
// ---------------------------------------------------------------------------
template <int ENV, int H, bool REPLAY>
__global__ __launch_bounds__(WG) void rollout_lane_kernel(const RolloutArgs a)
{
    constexpr int LDW = H + 4;                                    // row stride of W1 in LDS
    extern __shared__ float4 smem4[];
    float* w1s = reinterpret_cast<float*>(smem4);                 // [D][LDW]
    const int D = a.net.dims[0], NH = a.net.NH, NHP = a.net.NHP;
    float* b1s = w1s + D * LDW;                                   // [H]
    float* whs = b1s + H;                                         // [H][8] head weights, k-major, columns >= NH zero
    float* bhs = whs + H * 8;                                     // [8]
    const int tid = threadIdx.x;
    // the parameters come into LDS in batches of eight loads per thread: one load, one wait, one store at a time
    // would be a memory round trip per KB
    {
        const float vb1 = a.theta[a.net.b_off[0] + (tid < H ? tid : 0)];
        const float vbh = a.theta[a.net.bh_off + (tid < NH ? tid : 0)];
        constexpr int NW = (H * 8 + WG - 1) / WG;
        float vwh[NW];
#pragma unroll
        for (int q = 0; q < NW; ++q) {
            const int i = q * WG + tid, k = i >> 3, j = i & 7;
            vwh[q] = a.theta[a.net.wh_off + ((i < H * 8 && j < NH) ? k * NH + j : 0)];
        }
        const float* w1g = a.theta + a.net.w_off[0];
        const int n = D * H;
        for (int i0 = 0; i0 < n; i0 += 8 * WG) {
            float pw[8];
#pragma unroll
            for (int q = 0; q < 8; ++q) { const int i = i0 + q * WG + tid; pw[q] = w1g[i < n ? i : 0]; }
#pragma unroll
            for (int q = 0; q < 8; ++q) { const int i = i0 + q * WG + tid; if (i < n) w1s[(i / H) * LDW + i % H] = pw[q]; }
        }
        if (tid < H) b1s[tid] = vb1;
        if (tid < 8) bhs[tid] = tid < NH ? vbh : 0.0f;
#pragma unroll
        for (int q = 0; q < NW; ++q) {
            const int i = q * WG + tid, j = i & 7;
            if (i < H * 8) whs[i] = j < NH ? vwh[q] : 0.0f;
        }
    }
    __syncthreads();

    const int B = a.B, T = a.T;
    const int b = blockIdx.x * WG + tid;
    if (b >= B) return;
    const TrajPtrs& tp = a.tp;
    EnvState st{0u, 0.0f, 0.0f};
    if (!REPLAY) {
        st.s0 = tp.s0[b];
        if (ENV == ENV_PENDULUM) { st.f0 = tp.f0[b]; st.f1 = tp.f1[b]; }
    }
    for (int t = 0; t <= T; ++t) {
        const size_t tb = (size_t)t * B + b;
        if (REPLAY) {
            st.s0 = tp.tr_s0[tb];
            if (ENV == ENV_PENDULUM) { st.f0 = tp.tr_f0[tb]; st.f1 = tp.tr_f1[tb]; }
        } else {
            tp.tr_s0[tb] = st.s0;
            if (ENV == ENV_PENDULUM) { tp.tr_f0[tb] = st.f0; tp.tr_f1[tb] = st.f1; }
        }
        // the action draw does not depend on the network: issued first, used last
        u32x4 dr{0u, 0u, 0u, 0u};
        if (!REPLAY && t < T) dr = philox(a.seed, (uint32_t)b, a.gstep + (uint64_t)t, DOM_ACTION);
        // ---- first layer -------------------------------------------------------
        float h[H];
        if (ENV == ENV_CATCH) {
            int bc, pc;
            catch_obs_cells(a.env, st.s0, bc, pc);
            const float* r0 = w1s + bc * LDW;
            const float* r1 = w1s + pc * LDW;
#pragma unroll
            for (int j = 0; j < H; j += 4) {
                const float4 bb = ld4(b1s + j), w0 = ld4(r0 + j), w1 = ld4(r1 + j);
                h[j] = (bb.x + w0.x) + w1.x; h[j + 1] = (bb.y + w0.y) + w1.y;
                h[j + 2] = (bb.z + w0.z) + w1.z; h[j + 3] = (bb.w + w0.w) + w1.w;
            }
        } else {
            float sn, cs;
            det_sincos(st.f0, sn, cs);
            const float x[3] = {cs, sn, st.f1};
#pragma unroll
            for (int j = 0; j < H; j += 4) {
                const float4 bb = ld4(b1s + j);
                float v[4] = {bb.x, bb.y, bb.z, bb.w};
#pragma unroll
                for (int k = 0; k < 3; ++k) {
                    const float4 w = ld4(w1s + k * LDW + j);
                    v[0] = fmaf(x[k], w.x, v[0]); v[1] = fmaf(x[k], w.y, v[1]);
                    v[2] = fmaf(x[k], w.z, v[2]); v[3] = fmaf(x[k], w.w, v[3]);
                }
                h[j] = v[0]; h[j + 1] = v[1]; h[j + 2] = v[2]; h[j + 3] = v[3];
            }
        }
        // ---- heads: NH chains over k, ascending --------------------------------
        float hv[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) hv[j] = bhs[j];
#pragma unroll
        for (int k = 0; k < H; ++k) {
            const float x = h[k] > 0.0f ? h[k] : 0.0f;
            const float4 wa = ld4(whs + k * 8);
            hv[0] = fmaf(x, wa.x, hv[0]); hv[1] = fmaf(x, wa.y, hv[1]);
            hv[2] = fmaf(x, wa.z, hv[2]); hv[3] = fmaf(x, wa.w, hv[3]);
            if (NHP == 8) {
                const float4 wb = ld4(whs + k * 8 + 4);
                hv[4] = fmaf(x, wb.x, hv[4]); hv[5] = fmaf(x, wb.y, hv[5]);
                hv[6] = fmaf(x, wb.z, hv[6]); hv[7] = fmaf(x, wb.w, hv[7]);
            }
        }
        float* hd = tp.tr_head + tb * NHP;
        *reinterpret_cast<float4*>(hd) = make_float4(hv[0], hv[1], hv[2], hv[3]);
        if (NHP == 8) *reinterpret_cast<float4*>(hd + 4) = make_float4(hv[4], hv[5], hv[6], hv[7]);
        const float val = last_head(hv[0], hv[1], hv[2], hv[3], hv[4], hv[5], hv[6], hv[7], NH);
        tp.tr_val[tb] = val;
        if (!REPLAY && t < T) {
            float r; int done;
            if (ENV == ENV_PENDULUM) {
                float eps, act;
                sample_gaussian(hv[0], hv[1], dr.x, dr.y, eps, act);
                tp.tr_eps[tb] = eps;
                tp.tr_actf[tb] = act;
                pendulum_step(a.env, st, act, 0u, 0u, r, done);
                if (done) {
                    const u32x4 wr = philox(a.seed, (uint32_t)b, a.gstep + (uint64_t)t, DOM_RESET);
                    pendulum_reset(st, wr.x, wr.y);
                }
            } else {
                const int act = sample_categorical_any(hv[0], hv[1], hv[2], hv[3], hv[4], hv[5], hv[6], hv[7], a.net.A, u01(dr.x));
                tp.tr_act[tb] = (uint8_t)act;
                catch_step(a.env, st, act, 0u, r, done);
                if (done) {
                    const u32x4 wr = philox(a.seed, (uint32_t)b, a.gstep + (uint64_t)t, DOM_RESET);
                    st.s0 = catch_reset(a.env, wr.x);
                }
            }
            tp.tr_rew[tb] = r;
            tp.tr_done[tb] = (uint8_t)done;
        }
    }
    if (!REPLAY) {
        tp.s0[b] = st.s0;
        if (ENV == ENV_PENDULUM) { tp.f0[b] = st.f0; tp.f1[b] = st.f1; }
    }
}

// one-hidden-layer nets the lane kernel takes: width 32 or 64 on Catch or the pendulum, fp32, no kept activations
static int rollout_lane_width(const anakin* h)
{
    const NetShape& n = h->net;
    if (n.bf16 || n.L != 1 || h->env.kind == ENV_MAZE || !one_layer_fused(h)) return 0;
    if (h->mode & (ANAKIN_MODE_CANONICAL_ACTING | ANAKIN_MODE_STREAM_WEIGHTS)) return 0;
    return (n.dims[1] == 32 || n.dims[1] == 64) ? n.dims[1] : 0;
}

template <int ENV, int H, bool REPLAY>
static hipError_t launch_lane(anakin* h, const RolloutArgs& a)
{
    const size_t lds = ((size_t)h->net.dims[0] * (H + 4) + H + H * 8 + 8) * 4;
    ProfScope prof(h, REPLAY ? "replay_forward" : "rollout");
    hipLaunchKernelGGL((rollout_lane_kernel<ENV, H, REPLAY>), dim3((h->B + WG - 1) / WG), dim3(WG), lds, h->stream, a);
    return hipGetLastError();
}

// which resident shape (if any) fits this net: 0 none, else the width (64, 128, 256)
int rollout_resident_width(const NetShape& net)
{
    if (net.bf16 || net.L != 2 || net.dims[1] != net.dims[2]) return 0;
    const int w = net.dims[1];
    return (w == 64 || w == 128 || w == 256) ? w : 0;
}
int rollout_resident_tile(const NetShape& net, int env_kind, int B)
{
    const int w = rollout_resident_width(net);
    if (!w) return 0;
    const int tm = (w >= 128 && B % 32 == 0 && B / 32 >= 256) ? 32 : 16;
    // besides the tile's own buffers the kernel keeps both bias vectors and (Catch, pendulum) the whole first-layer
    // matrix in LDS: a board too large for that runs on the streaming kernels instead
    size_t lds = rollout_lds_bytes(net, EnvDims{}, tm, nullptr) + (size_t)2 * w * 4;
    if (env_kind != ENV_MAZE) lds += (size_t)net.dims[0] * w * 4;
    return lds <= 160 * 1024 ? tm : 0;
}

// can the hidden-to-hidden layers run on the matrix cores with TM envs per workgroup?
static bool mfma_tile_ok(const NetShape& net, int TM)
{
    if (net.bf16 || net.L < 2) return false;
    if (TM != 16 && TM != 32 && TM != 64) return false;
    if (TM * net.dims[1] > 16 * 1024) return false;                 // first-layer register tile
    for (int l = 2; l <= net.L; ++l) {
        const int N = net.dims[l];
        if (TM == 16 ? N < 64 : N < 128) return false;              // at least one MFMA tile per wavefront
        if (TM == 64 && N > 512) return false;                      // accumulator budget
    }
    int hmax = 0;
    for (int l = 1; l <= net.L; ++l) hmax = net.dims[l] > hmax ? net.dims[l] : hmax;
    if ((size_t)2 * TM * (hmax + 4) * 4 > 128 * 1024) return false; // two activation buffers in LDS
    return rollout_lds_bytes(net, EnvDims{}, TM, nullptr) <= 160 * 1024;   // ... and everything else the kernel keeps there
}

int rollout_pick_tile_mfma(const NetShape& net, int B)
{
    int best = 0;
    for (int tm = 16; tm <= 64; tm *= 2) {
        if (B % tm || !mfma_tile_ok(net, tm)) continue;
        if (!best) best = tm;
        if (B / tm >= 256) best = tm;
    }
    return best;
}

size_t rollout_lds_bytes(const NetShape& net, const EnvDims&, int TM, int* ldx_out)
{
    int hmax = 0;
    for (int l = 1; l <= net.L; ++l) hmax = net.dims[l] > hmax ? net.dims[l] : hmax;
    const int ldx = hmax + 4;
    if (ldx_out) *ldx_out = ldx;
    size_t words = (size_t)2 * TM * ldx + (size_t)8 * (net.dims[net.L] + 4) + 8 + (size_t)TM * net.NHP + (size_t)TM * (OBS_WORDS + 4);
    return words * 4;
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
    // a tile also has to fit LDS: two activation buffers of the widest layer plus the transposed head matrix (a
    // 1024-wide last layer with 16 envs is 2 KB over; the caller then gets "no rollout tile fits" at create)
    auto fits = [&](int tm) { return tm >= lo && tm <= hi && B % tm == 0 && rollout_lds_bytes(net, EnvDims{}, tm, nullptr) <= 160 * 1024; };   // what one workgroup can be given on gfx950
    int best = 0;
    for (int tm = 16; tm <= 256; tm *= 2) {
        if (!fits(tm)) continue;
        if (!best) best = tm;                            // smallest valid tile
        if (B / tm >= 2048) best = tm;                   // largest tile that still leaves eight workgroups per CU
    }
    if (best && B / best < 256) {                        // small batches: fill the chip first
        for (int tm = 16; tm <= 256; tm *= 2)
            if (fits(tm) && B / tm >= 256) best = tm;
    }
    return best;
}

template <int ENV, bool BF, bool MF, bool REPLAY>
static hipError_t launch_one(anakin* h, const RolloutArgs& a, int TM)
{
    const size_t lds = rollout_lds_bytes(h->net, h->env, TM, nullptr);
    auto kern = rollout_kernel<ENV, BF, MF, REPLAY>;
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return e;
    ProfScope prof(h, REPLAY ? "replay_forward" : "rollout");
    hipLaunchKernelGGL(kern, dim3(h->B / TM), dim3(WG), lds, h->stream, a, TM);
    return hipGetLastError();
}

void fill_rollout_args(anakin* h, RolloutArgs& a);

template <int ENV, bool M32, int RW, bool REPLAY>
static hipError_t launch_resident(anakin* h, const RolloutArgs& a)
{
    constexpr int TM = M32 ? 32 : 16;
    size_t lds = rollout_lds_bytes(h->net, h->env, TM, nullptr);
    lds += (size_t)2 * RW * 4;                                     // the hidden layers' biases
    if (ENV != ENV_MAZE) lds += (size_t)h->net.dims[0] * RW * 4;
    auto kern = rollout_resident_kernel<ENV, M32, RW, RW, REPLAY>;
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return e;
    ProfScope prof(h, REPLAY ? "replay_forward" : "rollout");
    hipLaunchKernelGGL(kern, dim3(h->B / TM), dim3(WG), lds, h->stream, a);
    return hipGetLastError();
}

template <int ENV, bool REPLAY>
static hipError_t launch_resident_env(anakin* h, const RolloutArgs& a, int width, int tm)
{
    if (width == 256) return tm == 32 ? launch_resident<ENV, true, 256, REPLAY>(h, a) : launch_resident<ENV, false, 256, REPLAY>(h, a);
    if (width == 128) return tm == 32 ? launch_resident<ENV, true, 128, REPLAY>(h, a) : launch_resident<ENV, false, 128, REPLAY>(h, a);
    return launch_resident<ENV, false, 64, REPLAY>(h, a);
}

template <bool REPLAY>
static hipError_t launch_forward(anakin* h, const RolloutArgs& a)
{
    const bool bf = h->net.bf16 != 0;
    if (const int lw = rollout_lane_width(h)) {
        if (a.keep_acts == 0) {
            if (h->env.kind == ENV_CATCH) return lw == 32 ? launch_lane<ENV_CATCH, 32, REPLAY>(h, a) : launch_lane<ENV_CATCH, 64, REPLAY>(h, a);
            return lw == 32 ? launch_lane<ENV_PENDULUM, 32, REPLAY>(h, a) : launch_lane<ENV_PENDULUM, 64, REPLAY>(h, a);
        }
    }
    if (h->TM_res > 0 && !(h->mode & (ANAKIN_MODE_CANONICAL_ACTING | ANAKIN_MODE_STREAM_WEIGHTS))) {
        const int w = rollout_resident_width(h->net);
        switch (h->env.kind) {
            case ENV_CATCH:    return launch_resident_env<ENV_CATCH, REPLAY>(h, a, w, h->TM_res);
            case ENV_PENDULUM: return launch_resident_env<ENV_PENDULUM, REPLAY>(h, a, w, h->TM_res);
            default:           return launch_resident_env<ENV_MAZE, REPLAY>(h, a, w, h->TM_res);
        }
    }
    const bool mf = h->TM_mfma > 0 && !(h->mode & ANAKIN_MODE_CANONICAL_ACTING);
    if (mf) {
        switch (h->env.kind) {
            case ENV_CATCH:    return launch_one<ENV_CATCH, false, true, REPLAY>(h, a, h->TM_mfma);
            case ENV_PENDULUM: return launch_one<ENV_PENDULUM, false, true, REPLAY>(h, a, h->TM_mfma);
            default:           return launch_one<ENV_MAZE, false, true, REPLAY>(h, a, h->TM_mfma);
        }
    }
    switch (h->env.kind) {
        case ENV_CATCH:    return bf ? launch_one<ENV_CATCH, true, false, REPLAY>(h, a, h->TM) : launch_one<ENV_CATCH, false, false, REPLAY>(h, a, h->TM);
        case ENV_PENDULUM: return bf ? launch_one<ENV_PENDULUM, true, false, REPLAY>(h, a, h->TM) : launch_one<ENV_PENDULUM, false, false, REPLAY>(h, a, h->TM);
        default:           return bf ? launch_one<ENV_MAZE, true, false, REPLAY>(h, a, h->TM) : launch_one<ENV_MAZE, false, false, REPLAY>(h, a, h->TM);
    }
}

hipError_t launch_rollout(anakin* h)
{
    RolloutArgs a;
    fill_rollout_args(h, a);
    return launch_forward<false>(h, a);
}

// the actor of a decoupled step: parameters from the behaviour copy, no hidden activations kept
hipError_t launch_rollout_behaviour(anakin* h)
{
    RolloutArgs a;
    fill_rollout_args(h, a);
    a.theta = at<const float>(h, h->lay.theta_b);
    a.keep_acts = 0;
    return launch_forward<false>(h, a);
}

// the learner's forward pass over the stored unroll with the current parameters: hidden activations
// for the backward pass, head outputs and values into the learner's own buffers
hipError_t launch_replay_forward(anakin* h)
{
    RolloutArgs a;
    fill_rollout_args(h, a);
    a.tp.tr_head = at<float>(h, h->lay.head_new);
    a.tp.tr_val = at<float>(h, h->lay.val_new);
    return launch_forward<true>(h, a);
}

}  // namespace ank
