// Matrix-core (MFMA) versions of the dense-layer backward GEMMs for fp32
// networks (paper section 3.1: the update differentiates through the policy
// network; section 3.2: the backward pass is the expensive half).
//
//   gemm_nt_mask_mfma    dX[m][i] = (x[m][i] > 0) * sum_j dY[m][j] W[i][j]
//   gemm_tn_splitk_mfma  partial[s][i][j] = sum_{m in chunk s} x[m][i] dY[m][j]  (+ column sums of dY)
//
// Tiling for CDNA4: a 256-lane workgroup (four 64-wide wavefronts, 2 x 2)
// computes a 128 x 128 output tile; each wavefront owns 64 x 64 of it as 2 x 2
// v_mfma_f32_32x32x2_f32 tiles (64 accumulator registers).  The reduction
// dimension is staged through LDS 16 at a time; the next chunk is fetched into
// registers while the matrix cores work on the current one.
//
// Operand layout of v_mfma_f32_32x32x2_f32 (verified on gfx950): lane l feeds
// A[row l%32][k l/32] and B[k l/32][col l%32]; accumulator register r of lane l
// is D[row 8*(r/4) + 4*(l/32) + r%4][col l%32].
#include "gemm.h"

namespace ank {

typedef float f16v __attribute__((ext_vector_type(16)));

constexpr int BT = 128;     // block tile edge
constexpr int BK = 16;      // reduction chunk

__device__ __forceinline__ f16v mfma32(float a, float b, f16v c)
{
    return __builtin_amdgcn_mfma_f32_32x32x2f32(a, b, c, 0, 0, 0);
}

// ---------------------------------------------------------------------------
// dX = (dY W^T) masked by relu'(x).  Both operands are contiguous along the
// reduction index j, so tiles are stored [row][j] in LDS and every lane fetches
// four consecutive j with one 16-byte read, feeding four MFMA steps (the order
// of the reduction is free here, so step s of a group takes j = 8g + 4 (l/32) + s).
// Row stride 36 floats: eight consecutive rows cover all 32 banks.
// ---------------------------------------------------------------------------
constexpr int NT_BK = 32;
constexpr int NT_LD = NT_BK + 4;

__global__ __launch_bounds__(WG) void gemm_nt_mask_mfma(const GemmNtArgs a)
{
    __shared__ __attribute__((aligned(16))) float As[BT * NT_LD];        // dY tile [m][j]
    __shared__ __attribute__((aligned(16))) float Bs[BT * NT_LD];        // W tile  [i][j]
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1;
    const int m0 = blockIdx.x * BT, i0 = blockIdx.y * BT;
    const int lrow = tid >> 1, lk = (tid & 1) * 16;                // loader: one row, 16 consecutive j
    const bool a_ok = m0 + lrow < a.M, b_ok = i0 + lrow < a.K;
    const float* ap = a.dy + (size_t)(m0 + lrow) * a.N + lk;
    const float* bp = a.w + (size_t)(i0 + lrow) * a.N + lk;
    const float4 zero = make_float4(0, 0, 0, 0);
    float4 ra[4] = {zero, zero, zero, zero}, rb[4] = {zero, zero, zero, zero};
    auto fetch = [&](int j0) {
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            if (a_ok) ra[q] = *reinterpret_cast<const float4*>(ap + j0 + 4 * q);
            if (b_ok) rb[q] = *reinterpret_cast<const float4*>(bp + j0 + 4 * q);
        }
    };
    fetch(0);
    f16v acc[2][2];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.0f;
    const int l32 = lane & 31, lhi = lane >> 5;
    const float* __restrict__ xin = a.x;
    float* __restrict__ dxo = a.dx;
    float xm[4][16];                                               // relu mask source, fetched during the last chunk
    const float* a_rd = As + (wm * 64 + l32) * NT_LD + 4 * lhi;
    const float* b_rd = Bs + (wn * 64 + l32) * NT_LD + 4 * lhi;
    for (int j0 = 0; j0 < a.N; j0 += NT_BK) {
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            *reinterpret_cast<float4*>(&As[lrow * NT_LD + lk + 4 * q]) = ra[q];
            *reinterpret_cast<float4*>(&Bs[lrow * NT_LD + lk + 4 * q]) = rb[q];
        }
        __syncthreads();
        if (j0 + NT_BK < a.N) fetch(j0 + NT_BK);                  // next chunk in flight during the MFMAs
        else {                                                     // last chunk: fetch the relu mask under the MFMAs
#pragma unroll
            for (int t4 = 0; t4 < 4; ++t4) {
                const int i = i0 + wn * 64 + (t4 & 1) * 32 + l32;
                const int mb = m0 + wm * 64 + (t4 >> 1) * 32 + 4 * lhi;
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int m = mb + 8 * (r >> 2) + (r & 3);
                    xm[t4][r] = (m < a.M && i < a.K) ? xin[(size_t)m * a.K + i] : 0.0f;
                }
            }
        }
#pragma unroll
        for (int g = 0; g < NT_BK / 8; ++g) {
            const float4 a0 = *reinterpret_cast<const float4*>(a_rd + 8 * g);
            const float4 a1 = *reinterpret_cast<const float4*>(a_rd + 32 * NT_LD + 8 * g);
            const float4 b0 = *reinterpret_cast<const float4*>(b_rd + 8 * g);
            const float4 b1 = *reinterpret_cast<const float4*>(b_rd + 32 * NT_LD + 8 * g);
            const float a0s[4] = {a0.x, a0.y, a0.z, a0.w}, a1s[4] = {a1.x, a1.y, a1.z, a1.w};
            const float b0s[4] = {b0.x, b0.y, b0.z, b0.w}, b1s[4] = {b1.x, b1.y, b1.z, b1.w};
#pragma unroll
            for (int st = 0; st < 4; ++st) {
                acc[0][0] = mfma32(a0s[st], b0s[st], acc[0][0]);
                acc[0][1] = mfma32(a0s[st], b1s[st], acc[0][1]);
                acc[1][0] = mfma32(a1s[st], b0s[st], acc[1][0]);
                acc[1][1] = mfma32(a1s[st], b1s[st], acc[1][1]);
            }
        }
        __syncthreads();
    }
#pragma unroll
    for (int tr = 0; tr < 2; ++tr)
#pragma unroll
        for (int tc = 0; tc < 2; ++tc) {
            const int i = i0 + wn * 64 + tc * 32 + l32;
            const int mb = m0 + wm * 64 + tr * 32 + 4 * lhi;
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int m = mb + 8 * (r >> 2) + (r & 3);
                if (m < a.M && i < a.K) dxo[(size_t)m * a.K + i] = xm[tr * 2 + tc][r] > 0.0f ? acc[tr][tc][r] : 0.0f;
            }
        }
}

// ---------------------------------------------------------------------------
// dW partials.  Both operands are contiguous along their non-reduced index, so
// tiles are stored [m][i] / [m][j] in LDS and operand reads walk 32 consecutive
// addresses.  OBS: the first layer's x is rebuilt from the state snapshots.
// ---------------------------------------------------------------------------
__device__ __forceinline__ void obs_row8(const ObsSrc& o, int m, int i, int K, float (&e)[8])
{
#pragma unroll
    for (int c = 0; c < 8; ++c) e[c] = 0.0f;
    if (o.kind == ENV_CATCH) {
        int bc, pc;
        catch_obs_cells(o.env, o.s0[m], bc, pc);
#pragma unroll
        for (int c = 0; c < 8; ++c) e[c] = (i + c == bc || i + c == pc) ? 1.0f : 0.0f;
    } else if (o.kind == ENV_PENDULUM) {
        if (i == 0) {
            float sn, cs;
            det_sincos(o.f0[m], sn, cs);
            e[0] = cs; e[1] = sn; e[2] = o.f1[m];
        }
    } else {
        const int n = o.env.rows * o.env.cols;
        const int b = m % o.B, cell = (int)(o.s0[m] & 0xffffu);
#pragma unroll
        for (int c = 0; c < 8; ++c) {
            const int ii = i + c;
            float v = 0.0f;
            if (ii < n) v = (float)((o.walls[(size_t)(ii >> 5) * o.B + b] >> (ii & 31)) & 1u);
            else if (ii < 2 * n) v = (ii - n == cell) ? 1.0f : 0.0f;
            else if (ii < K) v = (ii == 3 * n - 1) ? 1.0f : 0.0f;
            e[c] = v;
        }
    }
#pragma unroll
    for (int c = 0; c < 8; ++c) if (i + c >= K) e[c] = 0.0f;
}

template <bool OBS>
__global__ __launch_bounds__(WG) void gemm_tn_splitk_mfma(const GemmTnArgs a)
{
    __shared__ __attribute__((aligned(16))) float Xs[BK * BT];     // [m][i]
    __shared__ __attribute__((aligned(16))) float Ys[BK * BT];     // [m][j]
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1;
    const int ti = blockIdx.x % a.tiles_i, tj = blockIdx.x / a.tiles_i;
    const int i0 = ti * BT, j0 = tj * BT;
    const int split = blockIdx.y;
    const int m_begin = split * a.rows, m_end = m_begin + a.rows;
    const int lrow = tid >> 4, lc = (tid & 15) * 8;                // loader: one sample row, 8 consecutive columns
    const bool x_ok = i0 + lc < a.K, y_ok = j0 + lc < a.ldy;      // K is a multiple of 8 on the dense path, ldy of 4
    const float4 zero = make_float4(0, 0, 0, 0);
    float4 rx0 = zero, rx1 = zero, ry0 = zero, ry1 = zero;
    auto fetch = [&](int mb) {
        const int m = mb + lrow;
        if (OBS) {
            float e[8];
            obs_row8(a.obs, m, i0 + lc, a.K, e);
            rx0 = make_float4(e[0], e[1], e[2], e[3]); rx1 = make_float4(e[4], e[5], e[6], e[7]);
        } else if (x_ok) {
            const float* p = a.x + (size_t)m * a.K + i0 + lc;
            rx0 = *reinterpret_cast<const float4*>(p); rx1 = *reinterpret_cast<const float4*>(p + 4);
        }
        if (y_ok) {
            const float* p = a.dy + (size_t)m * a.ldy + j0 + lc;
            ry0 = *reinterpret_cast<const float4*>(p);
            if (j0 + lc + 4 < a.ldy) ry1 = *reinterpret_cast<const float4*>(p + 4);
        }
    };
    fetch(m_begin);
    f16v acc[2][2];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.0f;
    float bsum = 0.0f;
    const int l32 = lane & 31, lhi = lane >> 5;
    // a wavefront whose 64 x 64 block lies outside the matrix has nothing to multiply
    const bool live = (i0 + wm * 64 < a.K) && (j0 + wn * 64 < a.N);
    const bool live_i1 = i0 + wm * 64 + 32 < a.K, live_j1 = j0 + wn * 64 + 32 < a.N;
    for (int mb = m_begin; mb < m_end; mb += BK) {
        *reinterpret_cast<float4*>(&Xs[lrow * BT + lc]) = rx0; *reinterpret_cast<float4*>(&Xs[lrow * BT + lc + 4]) = rx1;
        *reinterpret_cast<float4*>(&Ys[lrow * BT + lc]) = ry0; *reinterpret_cast<float4*>(&Ys[lrow * BT + lc + 4]) = ry1;
        __syncthreads();
        if (mb + BK < m_end) fetch(mb + BK);
        if (live) {
#pragma unroll
            for (int ks = 0; ks < BK; ks += 2) {
                const int k = ks + lhi;
                const float a0 = Xs[k * BT + wm * 64 + l32], a1 = Xs[k * BT + wm * 64 + 32 + l32];
                const float b0 = Ys[k * BT + wn * 64 + l32], b1 = Ys[k * BT + wn * 64 + 32 + l32];
                acc[0][0] = mfma32(a0, b0, acc[0][0]);
                if (live_j1) acc[0][1] = mfma32(a0, b1, acc[0][1]);
                if (live_i1) acc[1][0] = mfma32(a1, b0, acc[1][0]);
                if (live_i1 && live_j1) acc[1][1] = mfma32(a1, b1, acc[1][1]);
            }
        }
        if (ti == 0 && tid < BT) {
#pragma unroll
            for (int k = 0; k < BK; ++k) bsum += Ys[k * BT + tid];
        }
        __syncthreads();
    }
    float* out = a.partial + (size_t)split * ((size_t)a.K * a.N + a.N);
    if (live) {
#pragma unroll
        for (int tr = 0; tr < 2; ++tr)
#pragma unroll
            for (int tc = 0; tc < 2; ++tc) {
                const int j = j0 + wn * 64 + tc * 32 + l32;
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int i = i0 + wm * 64 + tr * 32 + 8 * (r >> 2) + 4 * lhi + (r & 3);
                    if (i < a.K && j < a.N) out[(size_t)i * a.N + j] = acc[tr][tc][r];
                }
            }
    }
    if (ti == 0 && tid < BT && j0 + tid < a.N) out[(size_t)a.K * a.N + j0 + tid] = bsum;
}

hipError_t launch_gemm_nt_mfma(const GemmNtArgs& a, hipStream_t s)
{
    hipLaunchKernelGGL(gemm_nt_mask_mfma, dim3((a.M + BT - 1) / BT, (a.K + BT - 1) / BT), dim3(WG), 0, s, a);
    return hipGetLastError();
}

hipError_t launch_gemm_tn_mfma(GemmTnArgs a, hipStream_t s)
{
    a.tiles_i = (a.K + BT - 1) / BT;
    const int tiles_j = (a.N + BT - 1) / BT;
    if (a.use_obs) hipLaunchKernelGGL(gemm_tn_splitk_mfma<true>, dim3(a.tiles_i * tiles_j, a.splits), dim3(WG), 0, s, a);
    else hipLaunchKernelGGL(gemm_tn_splitk_mfma<false>, dim3(a.tiles_i * tiles_j, a.splits), dim3(WG), 0, s, a);
    return hipGetLastError();
}

}  // namespace ank
