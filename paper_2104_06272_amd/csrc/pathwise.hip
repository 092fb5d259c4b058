// Pathwise policy gradient through the environment (paper section 3.1: with the environment inside
// the program, the unit of T interactions can be differentiated all the way through).  For the
// pendulum with the tanh-Gaussian policy, L_path = -(1/(B T)) sum r over the stored unroll, seen as
// a function of the parameters with the noise fixed.  This kernel walks every env's unroll
// backwards with the adjoint lambda_t = dL_path/ds_t and writes dL_path/d(mu, log_sigma) per
// sample; the ordinary backward pass then turns head gradients into parameter gradients.
//
// A workgroup owns 16 (or 32) envs for the whole sweep.  Per step: (A) the env's lane turns lambda_{t+1}
// into the gradient of the action and of (mu, log_sigma); (B) dZ2 = relu'(h2) (Wh g); (C)
// dZ1 = relu'(h1) (dZ2 W2^T) on the matrix cores, W2^T resident in registers for the whole sweep
// exactly as the acting kernel keeps W2; (D) g_obs = dZ1 W1^T, three dot products per env; (E)
// lambda_t from the step's and the reward's own derivatives plus g_obs through o = (cos, sin, thd).
// An episode end cuts the adjoint (the next state is a reset state).  The velocity clip is decided
// with the env step's own binary32 expression, so it agrees with what the env did.
#include <type_traits>
#include "internal.h"
#include "detmath.h"

namespace ank {

typedef float f4v_p __attribute__((ext_vector_type(4)));

struct PathArgs {
    const float* theta; int w1_off, w2_off, wh_off;
    const float* tr_f0; const float* tr_f1; const uint8_t* tr_done; const float* tr_actf; const float* tr_eps;
    const float* tr_head; int NH, NHP;
    const float* act0; const float* act1;     // hidden activations of the unroll, [T*B][RW] each
    float* path;                              // [T*B][2]: dL_path / d(mu, log_sigma)
    int B, T;
    float w;                                  // dL_path / dr = -1 / (B T)
};

typedef float f16v_p __attribute__((ext_vector_type(16)));

// M32: 32 envs per workgroup on v_mfma_f32_32x32x2_f32 (for batches of at least 32 envs per compute unit), else 16
// envs on v_mfma_f32_16x16x4_f32; the operand layouts are those of the two acting kernels.
template <int RW, bool M32>
__global__ __launch_bounds__(WG) void pathwise_sweep(const PathArgs a)
{
    constexpr int TM = M32 ? 32 : 16, KS = M32 ? RW / 2 : RW / 4, NT = M32 ? RW / 128 : RW / 64, LDX = RW + 4;
    constexpr int RL = M32 ? 32 : 16;                                  // rows an operand lane indexes
    constexpr int KSTEP = M32 ? 2 : 4;                                 // reduction indices per MFMA
    extern __shared__ float4 smem_p[];
    float* bufA = reinterpret_cast<float*>(smem_p);                    // [TM][LDX] dZ2
    float* bufB = bufA + TM * LDX;                                     // [TM][LDX] dZ1
    float* w1s = bufB + TM * LDX;                                      // first-layer matrix, [3][RW]
    float* whs = w1s + 3 * RW;                                         // head matrix columns of mu and log_sigma, [2][RW]
    float* gh = whs + 2 * RW;                                          // [TM][2]
    float* gobs = gh + TM * 2;                                         // [TM][4]
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int b0 = blockIdx.x * TM, B = a.B, T = a.T;

    for (int i = tid; i < 3 * RW; i += WG) w1s[i] = a.theta[a.w1_off + i];
    for (int i = tid; i < 2 * RW; i += WG) { const int c = i / RW, k = i - c * RW; whs[i] = a.theta[a.wh_off + k * a.NH + c]; }
    // B operand of step s, tile t: W2^T[KSTEP s + kq][col0 + t] = W2[col0 + t][KSTEP s + kq]
    const int col0 = wave * (RW >> 2) + NT * (lane & (RL - 1)), kq = lane / RL;
    float wreg[KS][NT];
    {
        const float* W2 = a.theta + a.w2_off;
#pragma unroll
        for (int s = 0; s < KS; ++s)
#pragma unroll
            for (int t = 0; t < NT; ++t) wreg[s][t] = W2[(size_t)(col0 + t) * RW + KSTEP * s + kq];
    }
    const bool owner = tid < TM;
    const int b = b0 + tid;
    float lam_th = 0.0f, lam_thd = 0.0f, g_th = 0.0f, g_thd = 0.0f, sn = 0.0f, cs = 1.0f;
    // this thread's pieces of h2 for phase (B): loaded one step ahead, while the phases before it run
    constexpr int NQ = TM * RW / 4 / WG;
    f4v_p h2v[NQ];
    auto fetch_h2 = [&](int t) {
        const float* h2 = a.act1 + ((size_t)t * B + b0) * RW;
#pragma unroll
        for (int q = 0; q < NQ; ++q) h2v[q] = *reinterpret_cast<const f4v_p*>(h2 + (size_t)(q * WG + tid) * 4);
    };
    fetch_h2(T - 1);
    __syncthreads();

    for (int t = T - 1; t >= 0; --t) {
        // ---- (A) ------------------------------------------------------------------
        if (owner) {
            const size_t i = (size_t)t * B + b;
            if (a.tr_done[i]) { lam_th = 0.0f; lam_thd = 0.0f; }
            const float th = a.tr_f0[i], thd = a.tr_f1[i], act = a.tr_actf[i], eps = a.tr_eps[i];
            const float ls = a.tr_head[i * a.NHP + 1];
            const bool clamped = ls < -5.0f || ls > 2.0f;
            const float sigma = det_exp(fminf(fmaxf(ls, -5.0f), 2.0f));
            float u = 2.0f * act;
            u = u < -2.0f ? -2.0f : u;
            u = u > 2.0f ? 2.0f : u;
            det_sincos(th, sn, cs);
            const float dt = 0x1.99999ap-5f;
            const float pre = fmaf(fmaf(15.0f, sn, 3.0f * u), dt, thd);          // the env step's expression
            const bool clipped = pre < -8.0f || pre > 8.0f;
            const float g_nthd = fmaf(dt, lam_th, lam_thd);
            const float g_pre = clipped ? 0.0f : g_nthd;
            g_th = lam_th + g_pre * dt * 15.0f * cs + a.w * (-2.0f * th);
            g_thd = g_pre + a.w * (-2.0f * 0x1.99999ap-4f * thd);
            const float g_u = g_pre * dt * 3.0f + a.w * (-2.0f * 0x1.0624dep-10f * u);
            const float g_z = 2.0f * g_u * (1.0f - act * act);
            const float g_ls = clamped ? 0.0f : g_z * sigma * eps;
            gh[tid * 2] = g_z; gh[tid * 2 + 1] = g_ls;
            *reinterpret_cast<float2*>(a.path + i * 2) = make_float2(g_z, g_ls);
        }
        __syncthreads();
        // ---- (B) dZ2[m][j] = (h2 > 0) (Wh[j][mu] g_mu + Wh[j][ls] g_ls) ---------------
#pragma unroll
        for (int qq = 0; qq < NQ; ++qq) {
            const int q = qq * WG + tid;                     // the tile's rows are contiguous: piece q is row q / (RW/4)
            const int m = q / (RW / 4), j = (q - m * (RW / 4)) * 4;
            const f4v_p hv = h2v[qq];
            const f4v_p w0 = *reinterpret_cast<const f4v_p*>(whs + j), w1 = *reinterpret_cast<const f4v_p*>(whs + RW + j);
            const float g0 = gh[m * 2], g1 = gh[m * 2 + 1];
            f4v_p d;
#pragma unroll
            for (int e = 0; e < 4; ++e) d[e] = hv[e] > 0.0f ? fmaf(w1[e], g1, w0[e] * g0) : 0.0f;
            *reinterpret_cast<f4v_p*>(bufA + m * LDX + j) = d;
        }
        __syncthreads();
        // ---- (C) dZ1 = (h1 > 0) (dZ2 W2^T) -------------------------------------------
        {
            typedef typename std::conditional<M32, f16v_p, f4v_p>::type acc_t;
            constexpr int NR_ = M32 ? 16 : 4;                          // accumulator registers per tile
            acc_t acc[NT];
#pragma unroll
            for (int tt = 0; tt < NT; ++tt)
#pragma unroll
                for (int r = 0; r < NR_; ++r) acc[tt][r] = 0.0f;
            // the relu mask of the result: requested before the products so the loads overlap them
            const float* h1 = a.act0 + ((size_t)t * B + b0) * RW;
            float h1v[NR_][NT];
#pragma unroll
            for (int r = 0; r < NR_; ++r) {
                const int row = M32 ? 8 * (r >> 2) + 4 * kq + (r & 3) : 4 * kq + r;
#pragma unroll
                for (int tt = 0; tt < NT; ++tt) h1v[r][tt] = h1[(size_t)row * RW + col0 + tt];
            }
            const float* xp = bufA + (lane & (RL - 1)) * LDX + kq;
            constexpr int PF = 4;
            float ap[PF];
#pragma unroll
            for (int u = 0; u < PF; ++u) ap[u] = xp[KSTEP * u];
#pragma unroll
            for (int s = 0; s < KS; ++s) {
                const float av = ap[s % PF];
                ap[s % PF] = xp[KSTEP * (s + PF < KS ? s + PF : 0)];
                __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                for (int tt = 0; tt < NT; ++tt) {
                    if constexpr (M32) acc[tt] = __builtin_amdgcn_mfma_f32_32x32x2f32(av, wreg[s][tt], acc[tt], 0, 0, 0);
                    else acc[tt] = __builtin_amdgcn_mfma_f32_16x16x4f32(av, wreg[s][tt], acc[tt], 0, 0, 0);
                }
            }
#pragma unroll
            for (int r = 0; r < NR_; ++r) {
                const int row = M32 ? 8 * (r >> 2) + 4 * kq + (r & 3) : 4 * kq + r;
#pragma unroll
                for (int tt = 0; tt < NT; ++tt)
                    bufB[row * LDX + col0 + tt] = h1v[r][tt] > 0.0f ? acc[tt][r] : 0.0f;
            }
        }
        if (t > 0) fetch_h2(t - 1);
        __syncthreads();
        // ---- (D) g_obs[m][c] = sum_i dZ1[m][i] W1[c][i] ----------------------------------
        {
            constexpr int PARTS = WG / TM, SEG = RW / PARTS;          // PARTS lanes share an env's three dot products
            const int m = tid / PARTS, part = tid % PARTS;
            float s0 = 0.0f, s1 = 0.0f, s2 = 0.0f;
#pragma unroll
            for (int e = 0; e < SEG; ++e) {
                const int i = part * SEG + e;
                const float d = bufB[m * LDX + i];
                s0 = fmaf(d, w1s[i], s0); s1 = fmaf(d, w1s[RW + i], s1); s2 = fmaf(d, w1s[2 * RW + i], s2);
            }
#pragma unroll
            for (int off = PARTS / 2; off > 0; off >>= 1) {
                s0 += __shfl_xor(s0, off, PARTS); s1 += __shfl_xor(s1, off, PARTS); s2 += __shfl_xor(s2, off, PARTS);
            }
            if (part == 0) { gobs[m * 4] = s0; gobs[m * 4 + 1] = s1; gobs[m * 4 + 2] = s2; }
        }
        __syncthreads();
        // ---- (E) lambda_t, through o = (cos th, sin th, thd) -----------------------------
        if (owner) {
            lam_th = g_th - sn * gobs[tid * 4] + cs * gobs[tid * 4 + 1];
            lam_thd = g_thd + gobs[tid * 4 + 2];
        }
    }
}

bool pathwise_ok(const anakin* h)
{
    const NetShape& n = h->net;
    if (h->env.kind != ENV_PENDULUM || n.policy != POLICY_TANH_GAUSSIAN || n.bf16 || n.L != 2 || n.dims[1] != n.dims[2]) return false;
    if (n.dims[1] != 64 && n.dims[1] != 128 && n.dims[1] != 256) return false;
    return h->B % 16 == 0;
}

hipError_t launch_pathwise(anakin* h)
{
    const Layout& L = h->lay;
    const NetShape& n = h->net;
    PathArgs a;
    a.theta = at<const float>(h, L.w_src); a.w1_off = n.w_off[0]; a.w2_off = n.w_off[1]; a.wh_off = n.wh_off;
    a.tr_f0 = at<const float>(h, L.tr_f0); a.tr_f1 = at<const float>(h, L.tr_f1); a.tr_done = at<const uint8_t>(h, L.tr_done);
    a.tr_actf = at<const float>(h, L.tr_actf); a.tr_eps = at<const float>(h, L.tr_eps);
    a.tr_head = at<const float>(h, L.tr_head); a.NH = n.NH; a.NHP = n.NHP;
    a.act0 = at<const float>(h, L.act[0]); a.act1 = at<const float>(h, L.act[1]);
    a.path = at<float>(h, L.path);
    a.B = h->B; a.T = h->T; a.w = (float)(-1.0 / ((double)h->B * (double)h->T));
    ProfScope prof(h, "pathwise_sweep");
    // 32 envs per workgroup once that still leaves a workgroup per compute unit (as the acting kernel chooses)
    const bool m32 = n.dims[1] >= 128 && h->B % 32 == 0 && h->B / 32 >= 256;
    const int TM = m32 ? 32 : 16, RW = n.dims[1];
    const dim3 grid(h->B / TM);
    const size_t lds = ((size_t)2 * TM * (RW + 4) + 5 * RW + 6 * TM) * sizeof(float);
    auto go = [&](auto kern) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) return e;
        hipLaunchKernelGGL(kern, grid, dim3(WG), lds, h->stream, a);
        return hipGetLastError();
    };
    switch (RW) {
        case 64:  return go(pathwise_sweep<64, false>);
        case 128: return m32 ? go(pathwise_sweep<128, true>) : go(pathwise_sweep<128, false>);
        default:  return m32 ? go(pathwise_sweep<256, true>) : go(pathwise_sweep<256, false>);
    }
}

}  // namespace ank
