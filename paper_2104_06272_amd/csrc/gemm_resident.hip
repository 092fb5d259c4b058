// Backward GEMMs of a 256-wide fp32 hidden layer as one persistent workgroup
// per compute unit (paper section 3.2: the backward pass is the expensive half
// of the update).  With M = B*T samples and 256 x 256 weights the tiled
// kernels in gemm_mfma.hip lose time to tile-count quantisation, to a prologue
// and an epilogue per 128 x 128 tile and to re-reading operands per tile.
// Here a workgroup takes a range of consecutive samples and keeps, for the
// whole launch, the operand that does not depend on the sample in registers:
//
//   gemm_nt_res256   dX = (dY W^T) masked: W lives in registers (wavefront w holds
//                    the 32 output columns 32w.., 128 registers per lane); dY streams
//                    through LDS 32 rows at a time, double buffered
//   gemm_tn_res256   dW partial = X^T dY: the whole 256 x 256 accumulator lives in
//                    registers (eight wavefronts x 128 x 64); X and dY stream through
//                    LDS 32 samples at a time, double buffered; one partial per workgroup
//
// For the top hidden layer both kernels can form dY on the way in from the layer's
// forward activations and the head gradient (HeadFuse), and the dW kernel then also
// sums the head matrix's gradient; the dX kernel of the pendulum's second layer also
// sums the first layer's gradient in its epilogue (FirstFuse).  The two products of
// one layer share a launch (gemm_tn_nt_res256) and run side by side: half the compute
// units take one dW chunk each, the other half one dX row range each, so every unit
// pays one prologue (dX: reading W) or one tail (dW: writing its partial), not both.
//
// Eight wavefronts per workgroup, two per SIMD: while one waits at the barrier
// or for LDS the other feeds the matrix core.  Loads that prefetch past the end
// re-read the last tile instead of branching, so the wait counters the compiler
// places in front of the MFMAs never have to cover a conditional prefetch.
//
// Operand layout of v_mfma_f32_32x32x2_f32: see gemm_mfma.hip.
#include "gemm.h"
#include "detmath.h"

namespace ank {

typedef float f16v_r __attribute__((ext_vector_type(16)));
typedef float f4v_r __attribute__((ext_vector_type(4)));

constexpr int RWG = 512;
constexpr int RT = 32;                  // samples per LDS stage
constexpr int NTR_LD = 256 + 4;         // row stride of the dY stage: eight rows cover all banks for 16-byte reads

__device__ __forceinline__ f16v_r mfma_r(float a, float b, f16v_r c) { return __builtin_amdgcn_mfma_f32_32x32x2f32(a, b, c, 0, 0, 0); }

// ---------------------------------------------------------------------------
// dX[m][i] = (x[m][i] > 0) * sum_j dY[m][j] W[i][j],  N = 256 (reduction), K a multiple of 256.
// The order of the reduction is free: step 4p + e of lane half kg takes j = 8p + 4kg + e, so both
// the resident weights and the LDS operand are fetched 16 bytes at a time.
// ---------------------------------------------------------------------------
// head weights of this thread's four loader columns, and dY formed from the forward activations
struct HeadCols { float w[4][4]; };
__device__ __forceinline__ void load_head_cols(const HeadFuse& hf, int lc, HeadCols& hc)
{
#pragma unroll
    for (int e = 0; e < 4; ++e)
#pragma unroll
        for (int k = 0; k < 4; ++k) hc.w[e][k] = k < hf.NH ? hf.wh[(size_t)(lc + e) * hf.NH + k] : 0.0f;
}
__device__ __forceinline__ f4v_r head_dy(const HeadCols& hc, f4v_r hv, f4v_r d)
{
    f4v_r o;
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        float s = hc.w[e][0] * d[0];
        s = fmaf(hc.w[e][1], d[1], s); s = fmaf(hc.w[e][2], d[2], s); s = fmaf(hc.w[e][3], d[3], s);
        o[e] = hv[e] > 0.0f ? s : 0.0f;
    }
    return o;
}

template <bool HEADS, bool FIRST>
__device__ __forceinline__ void gemm_nt_res256_body(const GemmNtArgs& a, const int rows_per_block, const int bx, const int by)
{
    extern __shared__ float4 smem_r[];
    float* As0 = reinterpret_cast<float*>(smem_r);
    float* As1 = As0 + RT * NTR_LD;
    float* obsS = As1 + RT * NTR_LD;                                 // FIRST: [2][RT][4] features of the stage's samples
    constexpr int N = 256;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, l32 = lane & 31, kg = lane >> 5;
    const int i = by * 256 + wave * 32 + l32;                       // this lane's output column
    const int m_begin = bx * rows_per_block;
    const int m_end = m_begin + rows_per_block < a.M ? m_begin + rows_per_block : a.M;
    if (m_begin >= a.M) return;
    float wreg[128];
#pragma unroll
    for (int p = 0; p < 32; ++p) {
        const float4 v = *reinterpret_cast<const float4*>(a.w + (size_t)i * N + 8 * p + 4 * kg);
        wreg[4 * p] = v.x; wreg[4 * p + 1] = v.y; wreg[4 * p + 2] = v.z; wreg[4 * p + 3] = v.w;
    }
    // loader: 32 rows x 64 pieces of 16 B, four per thread: row 8q + tid/64, piece tid%64
    const int lrow = __builtin_amdgcn_readfirstlane(tid >> 6), lc = (tid & 63) << 2;
    const int m_clamp = m_end - 1;
    f4v_r st[4], dh[HEADS ? 4 : 1];
    HeadCols hc;
    if (HEADS) load_head_cols(a.hf, lc, hc);
    const float* src = HEADS ? a.hf.hl : a.dy;
    auto fetch = [&](int m0) {
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const int m = m0 + 8 * q + lrow;                                                          // uniform in a wavefront
            const int mc = m < m_end ? m : m_clamp;                                                   // rows past the end are never used
            st[q] = *reinterpret_cast<const f4v_r*>(src + (size_t)mc * N + lc);
            if (HEADS) dh[HEADS ? q : 0] = *reinterpret_cast<const f4v_r*>(a.hf.dhead + (size_t)mc * a.hf.NHP);
        }
    };
    auto store_piece = [&](float* buf, int q) {
        *reinterpret_cast<f4v_r*>(buf + (8 * q + lrow) * NTR_LD + lc) = HEADS ? head_dy(hc, st[q], dh[HEADS ? q : 0]) : st[q];
    };
    auto store = [&](float* buf) {
#pragma unroll
        for (int q = 0; q < 4; ++q) store_piece(buf, q);
    };
    // FIRST: the first RT threads work out (cos, sin, thd, 1) of one sample of a stage each; the epilogue of that
    // stage multiplies them into this lane's column of dZ_1
    float gw0 = 0.0f, gw1 = 0.0f, gw2 = 0.0f, gb = 0.0f;
    auto features = [&](int m0, int buf) {
        if (FIRST && tid < RT) {
            const int m = m0 + tid < m_end ? m0 + tid : m_clamp;
            float sn, cs;
            det_sincos(a.ff.f0[m], sn, cs);
            f4v_r o = {cs, sn, a.ff.f1[m], 1.0f};
            *reinterpret_cast<f4v_r*>(obsS + (buf * RT + tid) * 4) = o;
        }
    };
    fetch(m_begin);
    store(As0);
    features(m_begin, 0);
    __syncthreads();
    const uint32_t lane_off = (uint32_t)(4 * kg) * (uint32_t)a.K + (uint32_t)i;
    int t = 0;
    for (int m0 = m_begin; m0 < m_end; m0 += RT, t ^= 1) {
        const float* cur = t ? As1 : As0;
        float* nxt = t ? As0 : As1;
        const bool more = m0 + RT < m_end;
        fetch(more ? m0 + RT : m0);                                 // the last step re-reads its own rows
        // the next stage's features: one wavefront's long sine/cosine chain runs under the other wavefronts' MFMAs
        if (FIRST && m0 + RT < m_end) features(m0 + RT, t ^ 1);
        // rows come in whole groups of eight (M and the rows per workgroup are multiples of 8), so the row
        // part of every address and every bounds check is uniform: scalar base + one 32-bit lane offset
        float xm[16];
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const int mu = m0 + 8 * (r >> 2) + (r & 3);
            xm[r] = (a.x + (size_t)(mu < m_end ? mu : m_begin) * a.K)[lane_off];
        }
        __builtin_amdgcn_sched_barrier(0);
        f16v_r acc;
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[r] = 0.0f;
        const float* a_rd = cur + l32 * NTR_LD + 4 * kg;
        // the LDS read of group p + 2 is issued before the MFMAs of group p: its latency hides under eight MFMAs
        f4v_r av0 = *reinterpret_cast<const f4v_r*>(a_rd), av1 = *reinterpret_cast<const f4v_r*>(a_rd + 8);
#pragma unroll
        for (int p = 0; p < 32; p += 2) {
            const f4v_r nx0 = *reinterpret_cast<const f4v_r*>(a_rd + 8 * (p + 2 < 32 ? p + 2 : 0));
            __builtin_amdgcn_sched_barrier(0);
            acc = mfma_r(av0[0], wreg[4 * p], acc);
            acc = mfma_r(av0[1], wreg[4 * p + 1], acc);
            acc = mfma_r(av0[2], wreg[4 * p + 2], acc);
            acc = mfma_r(av0[3], wreg[4 * p + 3], acc);
            const f4v_r nx1 = *reinterpret_cast<const f4v_r*>(a_rd + 8 * (p + 3 < 32 ? p + 3 : 1));
            __builtin_amdgcn_sched_barrier(0);
            acc = mfma_r(av1[0], wreg[4 * p + 4], acc);
            acc = mfma_r(av1[1], wreg[4 * p + 5], acc);
            acc = mfma_r(av1[2], wreg[4 * p + 6], acc);
            acc = mfma_r(av1[3], wreg[4 * p + 7], acc);
            av0 = nx0; av1 = nx1;
            // the next stage goes to `nxt` a quarter at a time between the MFMAs: each one waits for the one before
            // it (same accumulator), so what is issued in between is free
            if ((p & 6) == 6 && more) store_piece(nxt, p >> 3);
        }
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const int mu = m0 + 8 * (r >> 2) + (r & 3);
            const float o = xm[r] > 0.0f ? acc[r] : 0.0f;
            if (mu < m_end) {
                if (!FIRST) (a.dx + (size_t)mu * a.K)[lane_off] = o;   // FIRST: dZ_1 has no other reader and stays on chip
                if (FIRST) {
                    const f4v_r f = *reinterpret_cast<const f4v_r*>(obsS + (t * RT + 8 * (r >> 2) + 4 * kg + (r & 3)) * 4);
                    gw0 = fmaf(f[0], o, gw0); gw1 = fmaf(f[1], o, gw1); gw2 = fmaf(f[2], o, gw2); gb += o;
                }
            }
        }
        __syncthreads();
    }
    if (FIRST) {
        // the two halves of a wavefront hold the same column for different rows: lower half first
        gw0 += __shfl_xor(gw0, 32, 64); gw1 += __shfl_xor(gw1, 32, 64); gw2 += __shfl_xor(gw2, 32, 64); gb += __shfl_xor(gb, 32, 64);
        if (kg == 0) {
            float* out = a.ff.partial + (size_t)bx * (4 * (size_t)a.K);
            out[i] = gw0; out[(size_t)a.K + i] = gw1; out[2 * (size_t)a.K + i] = gw2; out[3 * (size_t)a.K + i] = gb;
        }
    }
}

// ---------------------------------------------------------------------------
// partial[s][i][j] = sum over the samples of chunk s of x[m][i] dY[m][j], K = N = 256, plus the
// column sums of dY.  Wavefront (wm, wn) owns rows 128 wm.., columns 64 wn.. of the product.
// a.rows is a multiple of 32.
// ---------------------------------------------------------------------------
template <bool HEADS>
__device__ __forceinline__ void gemm_tn_res256_body(const GemmTnArgs& a, const int split)
{
    extern __shared__ float4 smem_r[];
    float* Xs = reinterpret_cast<float*>(smem_r);                    // [2][32][256]
    float* Ys = Xs + 2 * RT * 256;                                   // [2][32][256]
    constexpr int K = 256, N = 256;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, l32 = lane & 31, kg = lane >> 5;
    const int wm = wave >> 2, wn = wave & 3;
    const int m_begin = split * a.rows, m_end = m_begin + a.rows;
    const int lrow = __builtin_amdgcn_readfirstlane(tid >> 6), lc = (tid & 63) << 2;
    f4v_r sx[4], sy[4], dh[HEADS ? 4 : 1];
    f4v_r bsum = {0.0f, 0.0f, 0.0f, 0.0f};
    HeadCols hc;
    float gwh[HEADS ? 4 : 1][4];                                     // head-matrix gradient of this thread's four columns
    f4v_r gbh = {0.0f, 0.0f, 0.0f, 0.0f};                            // head-bias gradient (every thread of a loader row holds the same)
    if (HEADS) {
        load_head_cols(a.hf, lc, hc);
#pragma unroll
        for (int e = 0; e < 4; ++e)
#pragma unroll
            for (int k = 0; k < 4; ++k) gwh[HEADS ? e : 0][k] = 0.0f;
    }
    auto fetch = [&](int m0) {
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const int m = m0 + 8 * q + lrow;                                                          // uniform in a wavefront
            sx[q] = *reinterpret_cast<const f4v_r*>(a.x + (size_t)m * K + lc);
            if (HEADS) {
                sy[q] = *reinterpret_cast<const f4v_r*>(a.hf.hl + (size_t)m * N + lc);
                dh[HEADS ? q : 0] = *reinterpret_cast<const f4v_r*>(a.hf.dhead + (size_t)m * a.hf.NHP);
            } else {
                sy[q] = *reinterpret_cast<const f4v_r*>(a.dy + (size_t)m * a.ldy + lc);
            }
        }
    };
    auto store_piece = [&](int b, int q) {
        {
            *reinterpret_cast<f4v_r*>(Xs + (b * RT + 8 * q + lrow) * 256 + lc) = sx[q];
            if (HEADS) {
                // the head matrix's own gradient: hl^T dhead, from the activations just loaded (zero where the relu cut)
                const f4v_r d = dh[HEADS ? q : 0];
#pragma unroll
                for (int e = 0; e < 4; ++e)
#pragma unroll
                    for (int k = 0; k < 4; ++k) gwh[HEADS ? e : 0][k] = fmaf(sy[q][e], d[k], gwh[HEADS ? e : 0][k]);
                gbh += d;
                sy[q] = head_dy(hc, sy[q], d);
            }
            *reinterpret_cast<f4v_r*>(Ys + (b * RT + 8 * q + lrow) * 256 + lc) = sy[q];
            bsum += sy[q];
        }
    };
    auto store = [&](int b) {
#pragma unroll
        for (int q = 0; q < 4; ++q) store_piece(b, q);
    };
    fetch(m_begin);
    store(0);
    __syncthreads();
    f16v_r acc[4][2];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.0f;
    int t = 0;
    for (int m0 = m_begin; m0 < m_end; m0 += RT, t ^= 1) {
        const bool more = m0 + RT < m_end;
        fetch(more ? m0 + RT : m0);                                 // the last step re-reads its own rows, unused
        __builtin_amdgcn_sched_barrier(0);
        const float* xs = Xs + t * RT * 256 + wm * 128 + l32;
        const float* ys = Ys + t * RT * 256 + wn * 64 + l32;
        // operands of step ks + 2 are read from LDS before the eight MFMAs of step ks are issued
        float av[4], bv[2];
#pragma unroll
        for (int q = 0; q < 4; ++q) av[q] = xs[kg * 256 + 32 * q];
#pragma unroll
        for (int q = 0; q < 2; ++q) bv[q] = ys[kg * 256 + 32 * q];
#pragma unroll
        for (int ks = 0; ks < RT; ks += 2) {
            const int kn = (ks + 2 < RT ? ks + 2 : 0) + kg;
            float an[4], bn[2];
#pragma unroll
            for (int q = 0; q < 4; ++q) an[q] = xs[kn * 256 + 32 * q];
#pragma unroll
            for (int q = 0; q < 2; ++q) bn[q] = ys[kn * 256 + 32 * q];
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j < 2; ++j) acc[i][j] = mfma_r(av[i], bv[j], acc[i][j]);
#pragma unroll
            for (int q = 0; q < 4; ++q) av[q] = an[q];
#pragma unroll
            for (int q = 0; q < 2; ++q) bv[q] = bn[q];
            // the next stage goes to the other half of LDS a quarter at a time between the MFMA steps, so that its
            // stores and the vector work behind them (the head terms) run while the matrix cores are busy
            if ((ks & 6) == 6 && more) store_piece(t ^ 1, ks >> 3);
        }
        __syncthreads();
    }
    float* out = a.partial + (size_t)split * ((size_t)K * N + N);
#pragma unroll
    for (int tr = 0; tr < 4; ++tr)
#pragma unroll
        for (int tc = 0; tc < 2; ++tc) {
            const int j = wn * 64 + tc * 32 + l32;
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int i = wm * 128 + tr * 32 + 8 * (r >> 2) + 4 * kg + (r & 3);
                out[(size_t)i * N + j] = acc[tr][tc][r];
            }
        }
    // column sums: the eight loader rows of a column add up in ascending order
    float* red = Xs;                                                 // [8][256]
    *reinterpret_cast<f4v_r*>(red + lrow * 256 + lc) = bsum;
    __syncthreads();
    if (tid < 256) {
        float s = 0.0f;
#pragma unroll
        for (int g = 0; g < 8; ++g) s += red[g * 256 + tid];
        out[(size_t)K * N + tid] = s;
    }
    if (HEADS) {
        // head-matrix and head-bias gradients: the eight loader rows of a column add up in ascending order
        const int NH = a.hf.NH;
        float* hout = a.hf.head_partial + (size_t)split * ((size_t)N * NH + NH);
        float* red4 = Ys;                                            // [8][256][4]
        __syncthreads();
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            f4v_r v = {gwh[HEADS ? e : 0][0], gwh[HEADS ? e : 0][1], gwh[HEADS ? e : 0][2], gwh[HEADS ? e : 0][3]};
            *reinterpret_cast<f4v_r*>(red4 + ((size_t)lrow * 256 + lc + e) * 4) = v;
        }
        __syncthreads();
        if (tid < 256) {
            f4v_r s4 = {0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
            for (int g = 0; g < 8; ++g) s4 += *reinterpret_cast<const f4v_r*>(red4 + ((size_t)g * 256 + tid) * 4);
            for (int k = 0; k < NH; ++k) hout[(size_t)tid * NH + k] = s4[k];
        }
        __syncthreads();
        // bias: one thread per loader row holds that row's sum (lane 0 of each wavefront)
        if (lane == 0) *reinterpret_cast<f4v_r*>(red4 + lrow * 4) = gbh;
        __syncthreads();
        if (tid < NH) {
            float s = 0.0f;
            for (int g = 0; g < 8; ++g) s += red4[g * 4 + tid];
            hout[(size_t)N * NH + tid] = s;
        }
    }
}

template <bool HEADS, bool FIRST>
__global__ __launch_bounds__(RWG) void gemm_nt_res256(const GemmNtArgs a, const int rows_per_block)
{
    gemm_nt_res256_body<HEADS, FIRST>(a, rows_per_block, (int)blockIdx.x, (int)blockIdx.y);
}
template <bool HEADS>
__global__ __launch_bounds__(RWG) void gemm_tn_res256(const GemmTnArgs a)
{
    gemm_tn_res256_body<HEADS>(a, (int)blockIdx.x);
}
// Both products of one layer in one launch: they read the same operands and do not depend on each other.  The
// dW workgroups come first in the grid; as each retires (its long tail is the write of a 256 KB partial, with the
// matrix cores idle) a dX workgroup takes its compute unit, so the tail of one product overlaps the start of the
// other instead of the two kernels running back to back.
template <bool HEADS, bool FIRST>
__global__ __launch_bounds__(RWG) void gemm_tn_nt_res256(const GemmTnArgs t, const GemmNtArgs n, const int rows_per_block,
                                                         const int tn_blocks, const int nt_bx)
{
    const int b = (int)blockIdx.x;
    if (b < tn_blocks) gemm_tn_res256_body<HEADS>(t, b);
    else gemm_nt_res256_body<HEADS, FIRST>(n, rows_per_block, (b - tn_blocks) % nt_bx, (b - tn_blocks) / nt_bx);
}

bool gemm_nt_res_ok(const GemmNtArgs& a) { return a.N == 256 && a.K % 256 == 0 && a.M >= 8 && a.M % 8 == 0; }
bool gemm_tn_res_ok(const GemmTnArgs& a) { return a.K == 256 && a.N == 256 && !a.use_obs && a.rows % RT == 0 && a.ldy % 4 == 0; }

hipError_t launch_gemm_nt_res(const GemmNtArgs& a, hipStream_t s)
{
    int rows_per_block;
    const int bx = gemm_nt_res_blocks(a.M, 256, &rows_per_block);
    const size_t lds = ((size_t)2 * RT * NTR_LD + (a.ff.f0 ? 2 * RT * 4 : 0)) * sizeof(float);
    auto kern = a.ff.f0 ? (a.hf.hl ? gemm_nt_res256<true, true> : gemm_nt_res256<false, true>)
                        : (a.hf.hl ? gemm_nt_res256<true, false> : gemm_nt_res256<false, false>);
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(kern, dim3(bx, a.K / 256), dim3(RWG), lds, s, a, rows_per_block);
    return hipGetLastError();
}

hipError_t launch_gemm_tn_res(const GemmTnArgs& a, hipStream_t s)
{
    const size_t lds = (size_t)4 * RT * 256 * sizeof(float);
    auto kern = a.hf.hl ? gemm_tn_res256<true> : gemm_tn_res256<false>;
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(kern, dim3(a.splits), dim3(RWG), lds, s, a);
    return hipGetLastError();
}

hipError_t launch_gemm_tn_nt_res(const GemmTnArgs& t, const GemmNtArgs& n, hipStream_t s)
{
    int rows_per_block;
    const int nt_bx = gemm_nt_res_blocks(n.M, gemm_nt_res_cap(t.splits), &rows_per_block), nt_by = n.K / 256;
    const size_t lds_nt = ((size_t)2 * RT * NTR_LD + (n.ff.f0 ? 2 * RT * 4 : 0)) * sizeof(float), lds_tn = (size_t)4 * RT * 256 * sizeof(float);
    const size_t lds = lds_nt > lds_tn ? lds_nt : lds_tn;
    auto kern = n.ff.f0 ? (t.hf.hl ? gemm_tn_nt_res256<true, true> : gemm_tn_nt_res256<false, true>)
                        : (t.hf.hl ? gemm_tn_nt_res256<true, false> : gemm_tn_nt_res256<false, false>);
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(kern, dim3(t.splits + nt_bx * nt_by), dim3(RWG), lds, s, t, n, rows_per_block, t.splits, nt_bx);
    return hipGetLastError();
}

}  // namespace ank
