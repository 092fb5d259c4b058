// The update for bf16 networks on the matrix cores (paper section 3.1: the
// parameter update reuses the forward pass; section 3.2: backward is the
// expensive half).  fp32 master weights and fp32 accumulation; operands of the
// matrix cores are bfloat16.
//
// Data layout.  v_mfma_f32_32x32x16_bf16 wants eight consecutive values of the
// reduction index per lane.  For dX = dY W^T the reduction runs over features,
// so row-major [M][H] operands work.  For dW = X^T dY it runs over the M = B*T
// samples, so X and dY are also kept "sample-packed": P8[M/8][H][8], eight
// consecutive samples of one feature adjacent in memory.  The accumulator
// layout of the MFMA (four consecutive rows per register group) maps directly
// onto that packing, so producers write it with 8-byte stores and consumers
// read whole operands with 16-byte loads, coalesced across lanes.
//
//   head_backward_bf16   dZ_L (row-major + packed), partial dWh / dbh
//   gemm_nt_bf16         dZ_{l-1} = (dZ_l W_l^T) masked by relu'(h_{l-1}), both layouts out
//   gemm_tn_bf16         partial dW_l = h_{l-1}^T dZ_l (+ column sums), split over samples;
//                        for the first layer x is rebuilt from the state snapshots
#include "gemm.h"

namespace ank {

typedef __bf16 bf8 __attribute__((ext_vector_type(8)));
typedef float f16v __attribute__((ext_vector_type(16)));

__device__ __forceinline__ f16v mfma_bf16(bf8 a, bf8 b, f16v c) { return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0); }
__device__ __forceinline__ float bfu(uint16_t h) { return bf16_to_f(h); }

// ---------------------------------------------------------------------------
// heads: thread j walks sample groups of eight; h is packed, dhead fp32 rows
// ---------------------------------------------------------------------------
struct HeadBwdBf16Args {
    int M, H, NH, NHP, rows;                   // rows per workgroup (multiple of 64)
    const uint16_t* hP; const float* dhead; const uint16_t* wh16;   // wh16: bf16 copy of Wh, [H][NH]
    uint16_t* dzR; uint16_t* dzP; float* partial;                    // partial: [blocks over rows][H*NH + NH]
};

__global__ __launch_bounds__(WG) void head_backward_bf16(const HeadBwdBf16Args a)
{
    __shared__ __attribute__((aligned(16))) uint16_t tile[64 * (WG + 8)];   // [64 samples][256 columns] for the row-major copy
    constexpr int LDT = WG + 8;
    const int H = a.H, NH = a.NH, NHP = a.NHP;
    const int jb = blockIdx.y * WG, j = jb + threadIdx.x;
    const bool live = j < H;
    const int m_begin = blockIdx.x * a.rows, m_end = m_begin + a.rows;
    float w[8], dw[8], db[8];
#pragma unroll
    for (int k = 0; k < 8; ++k) { w[k] = (live && k < NH) ? bfu(a.wh16[(size_t)j * NH + k]) : 0.0f; dw[k] = 0.0f; db[k] = 0.0f; }
    for (int m0 = m_begin; m0 < m_end; m0 += 64) {
#pragma unroll 2
        for (int g = 0; g < 8; ++g) {
            const int mg = (m0 >> 3) + g;
            uint4 raw = make_uint4(0, 0, 0, 0);
            if (live) raw = *reinterpret_cast<const uint4*>(a.hP + ((size_t)mg * H + j) * 8);
            const uint32_t rw[4] = {raw.x, raw.y, raw.z, raw.w};
            uint32_t out[4];
#pragma unroll
            for (int q = 0; q < 8; ++q) {
                const float hv = bfu((uint16_t)((rw[q >> 1] >> ((q & 1) * 16)) & 0xffffu));
                const float* dh = a.dhead + (size_t)(mg * 8 + q) * NHP;
                float s = 0.0f;
#pragma unroll
                for (int k = 0; k < 8; ++k) {
                    if (k < NH) {
                        const float d = dh[k];
                        s = fmaf(w[k], d, s);
                        dw[k] = fmaf(hv, d, dw[k]);
                        db[k] += d;
                    }
                }
                const uint16_t o = bf16_bits(hv > 0.0f ? s : 0.0f);
                tile[(g * 8 + q) * LDT + threadIdx.x] = o;
                if (q & 1) out[q >> 1] |= (uint32_t)o << 16; else out[q >> 1] = o;
            }
            if (live) *reinterpret_cast<uint4*>(a.dzP + ((size_t)mg * H + j) * 8) = make_uint4(out[0], out[1], out[2], out[3]);
        }
        __syncthreads();
        // row-major copy: 64 rows x 256 columns, 16-byte pieces
        for (int i = threadIdx.x; i < 64 * (WG / 8); i += WG) {
            const int row = i / (WG / 8), c = (i % (WG / 8)) * 8;
            if (jb + c < H)
                *reinterpret_cast<uint4*>(a.dzR + (size_t)(m0 + row) * H + jb + c) = *reinterpret_cast<const uint4*>(&tile[row * LDT + c]);
        }
        __syncthreads();
    }
    float* out = a.partial + (size_t)blockIdx.x * ((size_t)H * NH + NH);
    if (live) for (int k = 0; k < NH; ++k) out[(size_t)j * NH + k] = dw[k];
    if (j == 0) for (int k = 0; k < NH; ++k) out[(size_t)H * NH + k] = db[k];
}

// ---------------------------------------------------------------------------
// dX = (dY W^T) masked.  dY row-major [M][N], W bf16 [K][N] (row i, reduction j
// contiguous), mask from packed h, output in both layouts.  128 x 128 tile,
// reduction staged through LDS 128 at a time.
// ---------------------------------------------------------------------------
struct GemmNtBf16Args {
    int M, K, N;
    const uint16_t* dyR;      // [M][N]
    const uint16_t* w16;      // [K][N]
    const uint16_t* hP;       // packed h_{l-1}: [M/8][K][8]
    uint16_t* dxR;            // [M][K]
    uint16_t* dxP;            // [M/8][K][8]
};

constexpr int NB_BK = 128;
constexpr int NB_LD = NB_BK + 8;        // row stride in bf16: 272 B, 16-byte aligned, 8 rows spread over all banks

__global__ __launch_bounds__(WG) void gemm_nt_bf16(const GemmNtBf16Args a)
{
    extern __shared__ uint4 smem4[];
    uint16_t* As = reinterpret_cast<uint16_t*>(smem4);          // [128][NB_LD] dY tile
    uint16_t* Bs = As + 128 * NB_LD;                            // [128][NB_LD] W tile
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1, l32 = lane & 31, kg = lane >> 5;
    const int m0 = blockIdx.x * 128, i0 = blockIdx.y * 128;
    // loader: 128 rows x 16 pieces of 16 B = 2048 pieces per matrix, 8 per thread
    uint4 ra[8], rb[8];
    auto fetch = [&](int j0) {
#pragma unroll
        for (int q = 0; q < 8; ++q) {
            const int p = q * WG + tid, row = p >> 4, kc = (p & 15) << 3;
            ra[q] = (m0 + row < a.M) ? *reinterpret_cast<const uint4*>(a.dyR + (size_t)(m0 + row) * a.N + j0 + kc) : make_uint4(0, 0, 0, 0);
            rb[q] = (i0 + row < a.K) ? *reinterpret_cast<const uint4*>(a.w16 + (size_t)(i0 + row) * a.N + j0 + kc) : make_uint4(0, 0, 0, 0);
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
    const uint16_t* a_rd = As + (wm * 64 + l32) * NB_LD + 8 * kg;
    const uint16_t* b_rd = Bs + (wn * 64 + l32) * NB_LD + 8 * kg;
    for (int j0 = 0; j0 < a.N; j0 += NB_BK) {
#pragma unroll
        for (int q = 0; q < 8; ++q) {
            const int p = q * WG + tid, row = p >> 4, kc = (p & 15) << 3;
            *reinterpret_cast<uint4*>(As + row * NB_LD + kc) = ra[q];
            *reinterpret_cast<uint4*>(Bs + row * NB_LD + kc) = rb[q];
        }
        __syncthreads();
        if (j0 + NB_BK < a.N) fetch(j0 + NB_BK);
#pragma unroll
        for (int ks = 0; ks < NB_BK; ks += 16) {
            const bf8 a0 = *reinterpret_cast<const bf8*>(a_rd + ks);
            const bf8 a1 = *reinterpret_cast<const bf8*>(a_rd + 32 * NB_LD + ks);
            const bf8 b0 = *reinterpret_cast<const bf8*>(b_rd + ks);
            const bf8 b1 = *reinterpret_cast<const bf8*>(b_rd + 32 * NB_LD + ks);
            acc[0][0] = mfma_bf16(a0, b0, acc[0][0]);
            acc[0][1] = mfma_bf16(a0, b1, acc[0][1]);
            acc[1][0] = mfma_bf16(a1, b0, acc[1][0]);
            acc[1][1] = mfma_bf16(a1, b1, acc[1][1]);
        }
        __syncthreads();
    }
    // epilogue.  Accumulator register group r/4 of lane (l32, kg) holds rows 8*(r/4) + 4*kg + 0..3 of
    // column l32: exactly half of one packed group of eight samples -> 8-byte mask loads and stores.
    uint16_t* Ts = As;                                           // [128][NB_LD] staging for the row-major copy
#pragma unroll
    for (int tr = 0; tr < 2; ++tr)
#pragma unroll
        for (int tc = 0; tc < 2; ++tc) {
            const int col = wn * 64 + tc * 32 + l32, i = i0 + col;
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                const int rowl = wm * 64 + tr * 32 + 8 * g + 4 * kg;          // first of 4 consecutive rows
                const int m = m0 + rowl;
                uint2 mask = make_uint2(0, 0);
                const bool ok = m < a.M && i < a.K;
                if (ok) mask = *reinterpret_cast<const uint2*>(a.hP + ((size_t)(m >> 3) * a.K + i) * 8 + (m & 7));
                const uint32_t mw[2] = {mask.x, mask.y};
                uint16_t o[4];
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const float hv = bfu((uint16_t)((mw[q >> 1] >> ((q & 1) * 16)) & 0xffffu));
                    o[q] = bf16_bits(hv > 0.0f ? acc[tr][tc][4 * g + q] : 0.0f);
                    Ts[(rowl + q) * NB_LD + col] = o[q];
                }
                if (ok) *reinterpret_cast<uint2*>(a.dxP + ((size_t)(m >> 3) * a.K + i) * 8 + (m & 7)) =
                    make_uint2((uint32_t)o[0] | ((uint32_t)o[1] << 16), (uint32_t)o[2] | ((uint32_t)o[3] << 16));
            }
        }
    __syncthreads();
    for (int p = tid; p < 128 * 16; p += WG) {
        const int row = p >> 4, c = (p & 15) << 3;
        if (m0 + row < a.M && i0 + c < a.K)
            *reinterpret_cast<uint4*>(a.dxR + (size_t)(m0 + row) * a.K + i0 + c) = *reinterpret_cast<const uint4*>(Ts + row * NB_LD + c);
    }
}

// ---------------------------------------------------------------------------
// dW partials from packed operands.  LDS tiles [sample group][column][8]; every
// operand is one 16-byte read.  OBS: the first layer's x comes from the state
// snapshots (walls bit planes, agent cell, goal cell / Catch cells).
// ---------------------------------------------------------------------------
struct GemmTnBf16Args {
    int M, K, N, splits, rows, tiles_i, use_obs;
    const uint16_t* xP;       // packed [M/8][K][8], unused with use_obs
    const uint16_t* dyP;      // packed [M/8][N][8]
    float* partial;           // [splits][K*N + N]
    ObsSrc obs;
};

constexpr int TB_G = 16;      // sample groups (of 8) per LDS stage: 128 samples

__device__ __forceinline__ uint4 obs_piece(const ObsSrc& o, int mg, int i, int K)
{
    // eight consecutive samples (same time step, consecutive envs) of observation feature i
    uint16_t v[8];
#pragma unroll
    for (int q = 0; q < 8; ++q) v[q] = 0;
    if (i < K) {
        const int m = mg * 8;
        if (o.kind == ENV_CATCH) {
#pragma unroll
            for (int q = 0; q < 8; ++q) {
                int bc, pc;
                catch_obs_cells(o.env, o.s0[m + q], bc, pc);
                v[q] = (i == bc || i == pc) ? 0x3f80 : 0;
            }
        } else if (o.kind == ENV_PENDULUM) {
#pragma unroll
            for (int q = 0; q < 8; ++q) {
                float sn, cs;
                det_sincos(o.f0[m + q], sn, cs);
                v[q] = bf16_bits(i == 0 ? cs : (i == 1 ? sn : o.f1[m + q]));
            }
        } else {
            const int n = o.env.rows * o.env.cols;
            if (i < n) {
                const int b = m % o.B;
                const uint4 w0 = *reinterpret_cast<const uint4*>(o.walls + (size_t)(i >> 5) * o.B + b);
                const uint4 w1 = *reinterpret_cast<const uint4*>(o.walls + (size_t)(i >> 5) * o.B + b + 4);
                const uint32_t ws[8] = {w0.x, w0.y, w0.z, w0.w, w1.x, w1.y, w1.z, w1.w};
#pragma unroll
                for (int q = 0; q < 8; ++q) v[q] = ((ws[q] >> (i & 31)) & 1u) ? 0x3f80 : 0;
            } else if (i < 2 * n) {
                const uint4 s0 = *reinterpret_cast<const uint4*>(o.s0 + m);
                const uint4 s1 = *reinterpret_cast<const uint4*>(o.s0 + m + 4);
                const uint32_t ss[8] = {s0.x, s0.y, s0.z, s0.w, s1.x, s1.y, s1.z, s1.w};
#pragma unroll
                for (int q = 0; q < 8; ++q) v[q] = ((int)(ss[q] & 0xffffu) == i - n) ? 0x3f80 : 0;
            } else if (i == 3 * n - 1) {
#pragma unroll
                for (int q = 0; q < 8; ++q) v[q] = 0x3f80;
            }
        }
    }
    return make_uint4((uint32_t)v[0] | ((uint32_t)v[1] << 16), (uint32_t)v[2] | ((uint32_t)v[3] << 16),
                      (uint32_t)v[4] | ((uint32_t)v[5] << 16), (uint32_t)v[6] | ((uint32_t)v[7] << 16));
}

template <bool OBS>
__global__ __launch_bounds__(WG) void gemm_tn_bf16(const GemmTnBf16Args a)
{
    extern __shared__ uint4 smem4[];
    uint4* Xs = smem4;                       // [TB_G][128] pieces of 8 samples
    uint4* Ys = Xs + TB_G * 128;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1, l32 = lane & 31, kg = lane >> 5;
    const int ti = blockIdx.x % a.tiles_i, tj = blockIdx.x / a.tiles_i;
    const int i0 = ti * 128, j0 = tj * 128;
    const int split = blockIdx.y;
    const int g_begin = (split * a.rows) >> 3, g_end = g_begin + (a.rows >> 3);
    // loader: TB_G groups x 128 columns = 2048 pieces per matrix, 8 per thread: piece p -> group p/128, column p%128
    uint4 rx[8], ry[8];
    auto fetch = [&](int g0) {
#pragma unroll
        for (int q = 0; q < 8; ++q) {
            const int p = q * WG + tid, g = g0 + (p >> 7), c = p & 127;
            const bool gok = g < g_end;
            if (OBS) rx[q] = gok ? obs_piece(a.obs, g, i0 + c, a.K) : make_uint4(0, 0, 0, 0);
            else rx[q] = (gok && i0 + c < a.K) ? *reinterpret_cast<const uint4*>(a.xP + ((size_t)g * a.K + i0 + c) * 8) : make_uint4(0, 0, 0, 0);
            ry[q] = (gok && j0 + c < a.N) ? *reinterpret_cast<const uint4*>(a.dyP + ((size_t)g * a.N + j0 + c) * 8) : make_uint4(0, 0, 0, 0);
        }
    };
    fetch(g_begin);
    f16v acc[2][2];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.0f;
    float bsum = 0.0f;
    const bool live = (i0 + wm * 64 < a.K) && (j0 + wn * 64 < a.N);
    for (int g0 = g_begin; g0 < g_end; g0 += TB_G) {
#pragma unroll
        for (int q = 0; q < 8; ++q) { const int p = q * WG + tid; Xs[p] = rx[q]; Ys[p] = ry[q]; }
        __syncthreads();
        if (g0 + TB_G < g_end) fetch(g0 + TB_G);
        if (live) {
#pragma unroll
            for (int ks = 0; ks < TB_G; ks += 2) {                // one MFMA step = 16 samples = 2 groups
                const uint4 xa0 = Xs[(ks + kg) * 128 + wm * 64 + l32], xa1 = Xs[(ks + kg) * 128 + wm * 64 + 32 + l32];
                const uint4 yb0 = Ys[(ks + kg) * 128 + wn * 64 + l32], yb1 = Ys[(ks + kg) * 128 + wn * 64 + 32 + l32];
                const bf8 a0 = *reinterpret_cast<const bf8*>(&xa0), a1 = *reinterpret_cast<const bf8*>(&xa1);
                const bf8 b0 = *reinterpret_cast<const bf8*>(&yb0), b1 = *reinterpret_cast<const bf8*>(&yb1);
                acc[0][0] = mfma_bf16(a0, b0, acc[0][0]);
                acc[0][1] = mfma_bf16(a0, b1, acc[0][1]);
                acc[1][0] = mfma_bf16(a1, b0, acc[1][0]);
                acc[1][1] = mfma_bf16(a1, b1, acc[1][1]);
            }
        }
        if (ti == 0 && tid < 128) {
#pragma unroll 4
            for (int g = 0; g < TB_G; ++g) {
                const uint4 y = Ys[g * 128 + tid];
                const uint32_t yw[4] = {y.x, y.y, y.z, y.w};
#pragma unroll
                for (int q = 0; q < 8; ++q) bsum += bfu((uint16_t)((yw[q >> 1] >> ((q & 1) * 16)) & 0xffffu));
            }
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
                    const int i = i0 + wm * 64 + tr * 32 + 8 * (r >> 2) + 4 * kg + (r & 3);
                    if (i < a.K && j < a.N) out[(size_t)i * a.N + j] = acc[tr][tc][r];
                }
            }
    }
    if (ti == 0 && tid < 128 && j0 + tid < a.N) out[(size_t)a.K * a.N + j0 + tid] = bsum;
}

// ---------------------------------------------------------------------------
// bf16 copies of the parameters the matrix cores read: same indexing (w16) and
// every weight matrix transposed (wt16: layers [N][K], heads [NH][HL]).
// ---------------------------------------------------------------------------
__global__ __launch_bounds__(WG) void refresh_bf16(const float* __restrict__ theta, uint16_t* __restrict__ w16,
                                                   uint16_t* __restrict__ wt16, const NetShape net)
{
    const int i = blockIdx.x * WG + threadIdx.x;
    if (i >= net.P) return;
    const uint16_t v = bf16_bits(theta[i]);
    w16[i] = v;
    wt16[transposed_index(net, i)] = v;
}

hipError_t launch_refresh_bf16(anakin* h)
{
    const Layout& L = h->lay;
    hipLaunchKernelGGL(refresh_bf16, dim3((h->net.P + WG - 1) / WG), dim3(WG), 0, h->stream,
                       at<const float>(h, L.theta), at<uint16_t>(h, L.w_bf16), at<uint16_t>(h, L.wt_bf16), h->net);
    return hipGetLastError();
}

// ---------------------------------------------------------------------------
// backward through all layers for a bf16 network
// ---------------------------------------------------------------------------
hipError_t launch_backward_bf16(anakin* h)
{
    const Layout& L = h->lay;
    const NetShape& n = h->net;
    const int M = h->B * h->T;
    hipError_t e;
    auto dzR = [&](int l) { return at<uint16_t>(h, L.dz[l]); };
    auto dzP = [&](int l) { return at<uint16_t>(h, L.dz[l]) + (size_t)M * n.dims[l + 1]; };
    auto actP = [&](int l) { return at<uint16_t>(h, L.act[l]); };
    {   // heads
        HeadBwdBf16Args a;
        a.M = M; a.H = n.dims[n.L]; a.NH = n.NH; a.NHP = n.NHP;
        const int stage1 = h->splits[n.L] * h->head_fan;
        a.rows = M / stage1;
        a.hP = actP(n.L - 1); a.dhead = at<const float>(h, L.dhead);
        a.wh16 = at<const uint16_t>(h, L.w_bf16) + n.wh_off;
        a.dzR = dzR(n.L - 1); a.dzP = dzP(n.L - 1);
        a.partial = h->head_fan > 1 ? at<float>(h, L.head_stage) : at<float>(h, L.part[n.L]);
        {
            ProfScope prof(h, "head_backward");
            hipLaunchKernelGGL(head_backward_bf16, dim3(stage1, (a.H + WG - 1) / WG), dim3(WG), 0, h->stream, a);
        }
        if ((e = hipGetLastError()) != hipSuccess) return e;
        if (h->head_fan > 1) {
            const int stride = a.H * a.NH + a.NH;
            ProfScope prof(h, "partial_reduce");
            e = launch_partial_reduce(at<const float>(h, L.head_stage), at<float>(h, L.part[n.L]), stride, h->head_fan,
                                      h->splits[n.L], h->stream);
            if (e != hipSuccess) return e;
        }
    }
    for (int l = n.L - 1; l >= 0; --l) {
        GemmTnBf16Args t;
        t.M = M; t.K = n.dims[l]; t.N = n.dims[l + 1];
        t.splits = h->splits[l]; t.rows = M / t.splits;
        t.tiles_i = (t.K + 127) / 128;
        t.use_obs = (l == 0);
        t.xP = l > 0 ? actP(l - 1) : nullptr;
        t.dyP = dzP(l);
        t.partial = at<float>(h, L.part[l]);
        t.obs.kind = h->env.kind; t.obs.env = h->env; t.obs.B = h->B;
        t.obs.s0 = at<const uint32_t>(h, L.tr_s0); t.obs.f0 = at<const float>(h, L.tr_f0);
        t.obs.f1 = at<const float>(h, L.tr_f1); t.obs.walls = at<const uint32_t>(h, L.walls);
        const dim3 grid(t.tiles_i * ((t.N + 127) / 128), t.splits);
        const size_t lds = (size_t)2 * TB_G * 128 * sizeof(uint4);
        e = t.use_obs ? hipFuncSetAttribute(reinterpret_cast<const void*>(gemm_tn_bf16<true>), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds)
                      : hipFuncSetAttribute(reinterpret_cast<const void*>(gemm_tn_bf16<false>), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) return e;
        {
            ProfScope prof(h, l == 0 ? "gemm_tn_obs" : "gemm_tn");
            if (t.use_obs) hipLaunchKernelGGL(gemm_tn_bf16<true>, grid, dim3(WG), lds, h->stream, t);
            else hipLaunchKernelGGL(gemm_tn_bf16<false>, grid, dim3(WG), lds, h->stream, t);
        }
        if ((e = hipGetLastError()) != hipSuccess) return e;
        if (l > 0) {
            GemmNtBf16Args g;
            g.M = M; g.K = n.dims[l]; g.N = n.dims[l + 1];
            g.dyR = dzR(l);
            g.w16 = at<const uint16_t>(h, L.w_bf16) + n.w_off[l];
            g.hP = actP(l - 1);
            g.dxR = dzR(l - 1); g.dxP = dzP(l - 1);
            const size_t lds2 = (size_t)2 * 128 * NB_LD * sizeof(uint16_t);
            auto kern = gemm_nt_bf16;
            e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds2);
            if (e != hipSuccess) return e;
            ProfScope prof(h, "gemm_nt_mask");
            hipLaunchKernelGGL(kern, dim3((g.M + 127) / 128, (g.K + 127) / 128), dim3(WG), lds2, h->stream, g);
            if ((e = hipGetLastError()) != hipSuccess) return e;
        }
    }
    return hipSuccess;
}

}  // namespace ank
