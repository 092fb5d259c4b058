// Dense-layer backward (paper section 3.1: the update differentiates the
// objective through the policy network; section 3.2 notes the backward pass is
// the expensive half).  For a hidden layer y = relu(x W + b) with upstream
// gradient dY (already masked by relu'(y)):
//   gemm_nt_mask    dX[m][i] = (x[m][i] > 0) * sum_j dY[m][j] W[i][j]      (M x K_in, reduce over N_out)
//   gemm_tn_splitk  dW[i][j] = sum_m x[m][i] dY[m][j],  db[j] = sum_m dY[m][j]  (reduce over the M = B*T samples)
// The sample reduction is cut into `splits` row chunks, one partial result per
// chunk; the Adam kernel adds them in ascending order.  The first layer's x is
// the observation, which is never materialised: it is rebuilt from the compact
// state snapshot while the tile is loaded.
//
// This file holds the vector-ALU versions (64x64 tiles, 4x4 per lane); the
// matrix-core versions are in gemm_mfma.hip (tiled) and gemm_resident.hip
// (persistent, 256-wide layers) and share the argument blocks.
#include "gemm.h"

namespace ank {

constexpr int TS = 64;      // tile edge
constexpr int KC = 16;      // reduction chunk staged in LDS

__device__ __forceinline__ float bfq(float x, int bf) { return bf ? bf16_to_f(bf16_bits(x)) : x; }

__global__ __launch_bounds__(WG) void gemm_nt_mask_valu(const GemmNtArgs a)
{
    __shared__ float As[KC][TS + 4];     // dY tile, transposed: [j][m]
    __shared__ float Bs[KC][TS + 4];     // W tile, transposed:  [j][i]
    const int tid = threadIdx.x;
    const int m0 = blockIdx.x * TS, i0 = blockIdx.y * TS;
    const int lr = tid >> 2, lc = (tid & 3) << 2;            // loader: row 0..63, 4 consecutive j
    const int ty = tid >> 4, tx = tid & 15;                   // compute: rows 4ty.., cols 4tx..
    float acc[4][4] = {};
    for (int j0 = 0; j0 < a.N; j0 += KC) {
        float4 va = make_float4(0, 0, 0, 0), vb = make_float4(0, 0, 0, 0);
        if (m0 + lr < a.M) va = *reinterpret_cast<const float4*>(a.dy + (size_t)(m0 + lr) * a.N + j0 + lc);
        if (i0 + lr < a.K) vb = *reinterpret_cast<const float4*>(a.w + (size_t)(i0 + lr) * a.N + j0 + lc);
        As[lc + 0][lr] = va.x; As[lc + 1][lr] = va.y; As[lc + 2][lr] = va.z; As[lc + 3][lr] = va.w;
        Bs[lc + 0][lr] = bfq(vb.x, a.bf16); Bs[lc + 1][lr] = bfq(vb.y, a.bf16);
        Bs[lc + 2][lr] = bfq(vb.z, a.bf16); Bs[lc + 3][lr] = bfq(vb.w, a.bf16);
        __syncthreads();
#pragma unroll
        for (int jj = 0; jj < KC; ++jj) {
            const float4 x = *reinterpret_cast<const float4*>(&As[jj][ty * 4]);
            const float4 y = *reinterpret_cast<const float4*>(&Bs[jj][tx * 4]);
            const float xs[4] = {x.x, x.y, x.z, x.w}, ys[4] = {y.x, y.y, y.z, y.w};
#pragma unroll
            for (int r = 0; r < 4; ++r)
#pragma unroll
                for (int c = 0; c < 4; ++c) acc[r][c] = fmaf(xs[r], ys[c], acc[r][c]);
        }
        __syncthreads();
    }
#pragma unroll
    for (int r = 0; r < 4; ++r) {
        const int m = m0 + ty * 4 + r, i = i0 + tx * 4;
        if (m < a.M && i < a.K) {
            const float4 xv = *reinterpret_cast<const float4*>(a.x + (size_t)m * a.K + i);
            float4 o;
            o.x = xv.x > 0.0f ? acc[r][0] : 0.0f;
            o.y = xv.y > 0.0f ? acc[r][1] : 0.0f;
            o.z = xv.z > 0.0f ? acc[r][2] : 0.0f;
            o.w = xv.w > 0.0f ? acc[r][3] : 0.0f;
            *reinterpret_cast<float4*>(a.dx + (size_t)m * a.K + i) = o;
        }
    }
}

// x[m][i] of the first layer, rebuilt from the state snapshot of sample m
__device__ __forceinline__ float obs_element(const ObsSrc& o, int m, int i)
{
    if (o.kind == ENV_CATCH) {
        int bc, pc;
        catch_obs_cells(o.env, o.s0[m], bc, pc);
        return (i == bc || i == pc) ? 1.0f : 0.0f;
    } else if (o.kind == ENV_PENDULUM) {
        if (i == 2) return o.f1[m];
        float sn, cs;
        det_sincos(o.f0[m], sn, cs);
        return i == 0 ? cs : sn;
    } else {
        const int n = o.env.rows * o.env.cols;
        if (i < n) {
            const int b = m % o.B;
            return (float)((o.walls[(size_t)(i >> 5) * o.B + b] >> (i & 31)) & 1u);
        }
        if (i < 2 * n) return (int)(o.s0[m] & 0xffffu) == i - n ? 1.0f : 0.0f;
        return i == 3 * n - 1 ? 1.0f : 0.0f;
    }
}

template <bool OBS>
__global__ __launch_bounds__(WG) void gemm_tn_splitk_valu(const GemmTnArgs a)
{
    __shared__ float Xs[KC][TS + 4];     // [m][i]
    __shared__ float Ys[KC][TS + 4];     // [m][j]
    const int tid = threadIdx.x;
    const int ti = blockIdx.x % a.tiles_i, tj = blockIdx.x / a.tiles_i;
    const int i0 = ti * TS, j0 = tj * TS;
    const int split = blockIdx.y;
    const int m_begin = split * a.rows, m_end = m_begin + a.rows;
    const int lr = tid >> 4, lc = (tid & 15) << 2;           // loader: row 0..15, 4 consecutive columns
    const int ty = tid >> 4, tx = tid & 15;
    float acc[4][4] = {};
    float bsum = 0.0f;
    for (int mb = m_begin; mb < m_end; mb += KC) {
        const int m = mb + lr;
        float4 vx = make_float4(0, 0, 0, 0), vy = make_float4(0, 0, 0, 0);
        if (OBS) {
            float e[4];
#pragma unroll
            for (int c = 0; c < 4; ++c) e[c] = (i0 + lc + c < a.K) ? obs_element(a.obs, m, i0 + lc + c) : 0.0f;
            vx = make_float4(e[0], e[1], e[2], e[3]);
        } else if (i0 + lc < a.K) {
            vx = *reinterpret_cast<const float4*>(a.x + (size_t)m * a.K + i0 + lc);
        }
        if (j0 + lc < a.ldy) vy = *reinterpret_cast<const float4*>(a.dy + (size_t)m * a.ldy + j0 + lc);
        *reinterpret_cast<float4*>(&Xs[lr][lc]) = vx;
        *reinterpret_cast<float4*>(&Ys[lr][lc]) = vy;
        __syncthreads();
#pragma unroll
        for (int mm = 0; mm < KC; ++mm) {
            const float4 x = *reinterpret_cast<const float4*>(&Xs[mm][ty * 4]);
            const float4 y = *reinterpret_cast<const float4*>(&Ys[mm][tx * 4]);
            const float xs[4] = {x.x, x.y, x.z, x.w}, ys[4] = {y.x, y.y, y.z, y.w};
#pragma unroll
            for (int r = 0; r < 4; ++r)
#pragma unroll
                for (int c = 0; c < 4; ++c) acc[r][c] = fmaf(xs[r], ys[c], acc[r][c]);
        }
        if (ti == 0 && tid < TS) {
#pragma unroll
            for (int mm = 0; mm < KC; ++mm) bsum += Ys[mm][tid];
        }
        __syncthreads();
    }
    float* out = a.partial + (size_t)split * ((size_t)a.K * a.N + a.N);
#pragma unroll
    for (int r = 0; r < 4; ++r) {
        const int i = i0 + ty * 4 + r, j = j0 + tx * 4;
        if (i < a.K && j < a.N)
            *reinterpret_cast<float4*>(out + (size_t)i * a.N + j) = make_float4(acc[r][0], acc[r][1], acc[r][2], acc[r][3]);
    }
    if (ti == 0 && tid < TS && j0 + tid < a.N) out[(size_t)a.K * a.N + j0 + tid] = bsum;
}

hipError_t launch_gemm_nt_valu(const GemmNtArgs& a, hipStream_t s)
{
    hipLaunchKernelGGL(gemm_nt_mask_valu, dim3((a.M + TS - 1) / TS, (a.K + TS - 1) / TS), dim3(WG), 0, s, a);
    return hipGetLastError();
}

hipError_t launch_gemm_tn_valu(GemmTnArgs a, hipStream_t s)
{
    a.tiles_i = (a.K + TS - 1) / TS;
    const int tiles_j = (a.N + TS - 1) / TS;
    if (a.use_obs) hipLaunchKernelGGL(gemm_tn_splitk_valu<true>, dim3(a.tiles_i * tiles_j, a.splits), dim3(WG), 0, s, a);
    else hipLaunchKernelGGL(gemm_tn_splitk_valu<false>, dim3(a.tiles_i * tiles_j, a.splits), dim3(WG), 0, s, a);
    return hipGetLastError();
}

// backward through all hidden layers, last to first (the head kernel has
// already produced dZ of the last hidden layer)
hipError_t launch_head_backward(anakin* h);

hipError_t launch_backward(anakin* h)
{
    const Layout& L = h->lay;
    const NetShape& n = h->net;
    const int M = h->B * h->T;
    hipError_t e;
    // Top hidden layer 256 -> 256 on the matrix cores: its dW and dX products form dZ_L on the way in from the
    // layer's forward activations and the head gradient, and the dW product also sums the head matrix's gradient,
    // so dZ_L is neither written nor read and the head pass is no kernel of its own.
    HeadFuse hf{};
    hf.hl = nullptr;
    {
        const int lt = n.L - 1;
        const bool mfma = !(h->mode & ANAKIN_MODE_VALU_GEMM) && !n.bf16;
        if (mfma && heads_fused_shape(n, M) && h->head_fan == 1 && h->splits[n.L] == h->splits[lt] && (M / h->splits[lt]) % 32 == 0) {
            hf.hl = at<const float>(h, L.act[lt]); hf.dhead = at<const float>(h, L.dhead);
            hf.wh = at<const float>(h, L.w_src) + n.wh_off; hf.NH = n.NH; hf.NHP = n.NHP;
            hf.head_partial = at<float>(h, L.part[n.L]);
        }
    }
    if (!hf.hl) {
        e = launch_head_backward(h);
        if (e != hipSuccess) return e;
    }
    // pendulum: the first layer's gradient is summed in the epilogue of the dX product that forms dZ_1
    const bool first_shape = !(h->mode & ANAKIN_MODE_VALU_GEMM) && first_fused_splits(n, h->env.kind, M, h->splits[1]) > 0;
    bool first_fused = false;
    for (int l = n.L - 1; l >= 0; --l) {
        if (l == 0 && first_fused) continue;
        // one-hot boards (Catch) and the 3-feature pendulum need no GEMM for the first layer
        if (l == 0 && h->env.kind != ENV_MAZE && !(h->mode & ANAKIN_MODE_VALU_GEMM) && (size_t)WG * n.dims[0] * 4 <= 96 * 1024) {
            e = launch_first_layer_grad(h);
            if (e != hipSuccess) return e;
            continue;
        }
        GemmTnArgs t;
        t.M = M; t.K = n.dims[l]; t.N = n.dims[l + 1]; t.ldy = t.N;
        t.splits = h->splits[l]; t.rows = M / t.splits;
        t.dy = at<const float>(h, L.dz[l]);
        t.partial = at<float>(h, L.part[l]);
        t.use_obs = (l == 0);
        t.x = l > 0 ? at<const float>(h, L.act[l - 1]) : nullptr;
        t.obs.kind = h->env.kind; t.obs.env = h->env; t.obs.B = h->B;
        t.obs.s0 = at<const uint32_t>(h, L.tr_s0); t.obs.f0 = at<const float>(h, L.tr_f0);
        t.obs.f1 = at<const float>(h, L.tr_f1); t.obs.walls = at<const uint32_t>(h, L.walls);
        t.bf16 = n.bf16; t.tiles_i = 0;
        t.hf = HeadFuse{}; t.hf.hl = nullptr;
        if (l == n.L - 1 && hf.hl) t.hf = hf;
        const bool mfma = !(h->mode & ANAKIN_MODE_VALU_GEMM) && !n.bf16;
        GemmNtArgs g;
        if (l > 0) {
            g.M = M; g.K = n.dims[l]; g.N = n.dims[l + 1];
            g.dy = at<const float>(h, L.dz[l]);
            g.w = at<const float>(h, L.w_src) + n.w_off[l];
            g.x = at<const float>(h, L.act[l - 1]);
            g.dx = at<float>(h, L.dz[l - 1]);
            g.bf16 = n.bf16;
            g.hf = HeadFuse{}; g.hf.hl = nullptr;
            if (l == n.L - 1 && hf.hl) g.hf = hf;
            g.ff = FirstFuse{nullptr, nullptr, nullptr};
            const bool merged = mfma && gemm_tn_res_ok(t) && gemm_nt_res_ok(g);
            if (l == 1 && first_shape && gemm_nt_res_ok(g)) {
                // the kernel writes one partial per workgroup along the samples: that count has to be the planned one
                int rpb;
                const int bx = gemm_nt_res_blocks(M, merged ? gemm_nt_res_cap(t.splits) : 256, &rpb);
                if (bx == h->splits[0] && (long long)bx * rpb == M) {
                    g.ff.f0 = at<const float>(h, L.tr_f0); g.ff.f1 = at<const float>(h, L.tr_f1);
                    g.ff.partial = at<float>(h, L.part[0]);
                    first_fused = true;
                }
            }
            if (merged) {
                // the layer's two resident products share one launch
                ProfScope prof(h, "gemm_tn_nt");
                e = launch_gemm_tn_nt_res(t, g, h->stream);
                if (e != hipSuccess) return e;
                continue;
            }
        }
        {
            ProfScope prof(h, l == 0 ? "gemm_tn_obs" : "gemm_tn");
            e = !mfma ? launch_gemm_tn_valu(t, h->stream) : gemm_tn_res_ok(t) ? launch_gemm_tn_res(t, h->stream) : launch_gemm_tn_mfma(t, h->stream);
        }
        if (e != hipSuccess) return e;
        if (l > 0) {
            ProfScope prof(h, "gemm_nt_mask");
            e = !mfma ? launch_gemm_nt_valu(g, h->stream) : gemm_nt_res_ok(g) ? launch_gemm_nt_res(g, h->stream) : launch_gemm_nt_mfma(g, h->stream);
            if (e != hipSuccess) return e;
        }
    }
    return hipSuccess;
}

}  // namespace ank
