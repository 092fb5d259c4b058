// The update on a stored unroll (paper section 3.1: the parameter update that
// follows the T interactions and reuses the policy's forward pass):
//   returns_scan          reverse scan over t of the lambda-return recursion
//   vtrace_ratio / _scan  off-policy targets for an unroll acted by older parameters (decoupled steps)
//   head_grad             actor-critic loss terms and the gradient w.r.t. head outputs
//   head_backward(_mfma)  gradient of the head matrix, and of the last hidden layer
//   first_layer_grad*     gradient of the first layer from the compact state (Catch, Pendulum)
//   learn_one_layer       the whole backward pass of a one-hidden-layer net
//   adam_reduce(_narrow, _flat)  fixed-order sum of split-K partials fused with Adam
// Hidden-layer GEMMs live in gemm.hip (vector ALU), gemm_mfma.hip (tiled) and
// gemm_resident.hip (persistent, 256-wide layers, which also take over the head
// pass of a 256-wide top layer); the bf16 update in learn_bf16.hip; the reverse
// sweep of the pathwise policy gradient in pathwise.hip.
// No floating-point atomics anywhere: every reduction has a fixed order, so runs
// are reproducible bit for bit.
#include "internal.h"
#include "loss.h"

namespace ank {

// ---------------------------------------------------------------------------
// G_T = V(s_T);  G_t = r + disc ((1-lambda) V_{t+1} + lambda G_{t+1});  A_t = G_t - V_t
// with disc = 0 after an episode end, gamma otherwise.  One lane per env walks
// its column backwards; consecutive lanes touch consecutive addresses of the
// time-major arrays, so every load and store is fully coalesced.
// ---------------------------------------------------------------------------
__global__ __launch_bounds__(WG) void returns_scan(int B, int T, const float* __restrict__ rew,
                                                   const uint8_t* __restrict__ done, const float* __restrict__ val,
                                                   float gamma, float lambda, float* __restrict__ adv,
                                                   float* __restrict__ ret)
{
    const int b = blockIdx.x * WG + threadIdx.x;
    if (b >= B) return;
    const float oml = 1.0f - lambda;
    float G = val[(size_t)T * B + b];
    float vnext = G;
#pragma unroll 4
    for (int t = T - 1; t >= 0; --t) {
        const size_t i = (size_t)t * B + b;
        const float r = rew[i], v = val[i];
        const float disc = done[i] ? 0.0f : gamma;
        const float mix = fmaf(lambda, G, oml * vnext);
        G = fmaf(disc, mix, r);
        ret[i] = G;
        adv[i] = G - v;
        vnext = v;
    }
}

// ---------------------------------------------------------------------------
// Off-policy targets for a stored unroll whose actions came from older parameters (decoupled acting
// and learning, paper section 3.2; the correction is IMPALA's V-trace, which the paper runs on that
// architecture).  head_old: head outputs stored at acting time (the behaviour policy mu); head_new:
// the learner's forward pass over the same states (policy pi and values V).  Per env, backwards in t:
//   w = pi(a|s) / mu(a|s),  rho = min(1, w),  c = lambda min(1, w),  disc = gamma (1 - done)
//   adv_t = rho (r + disc v_{t+1} - V_t)
//   v_t - V_t = rho (r + disc V_{t+1} - V_t) + disc c (v_{t+1} - V_{t+1}),   v_T = V_T
// ret = v, adv = the policy-gradient advantage: the loss kernel then treats them as it treats the
// on-policy return and advantage.  Gaussian policy: the densities are compared at the stored
// pre-squash sample z = mu_old + sigma_old eps_old, and eps_new = (z - mu_new) / sigma_new is
// written for the loss kernel's score function.  The ratios need no order and take a pass of
// their own, one lane per sample; the recursion then walks each env's column as returns_scan does.
// ---------------------------------------------------------------------------
struct VtraceArgs {
    int B, T, A, NH, NHP, policy;
    const float* head_old; const float* head_new; const float* val_new; const uint8_t* act; const float* eps_old;
    const float* rew; const uint8_t* done;
    float gamma, lambda;
    float* adv; float* ret; float* eps_new;
};

__device__ __forceinline__ void load_head(const float* p, int NHP, float (&hv)[8])
{
    const float4 h0 = *reinterpret_cast<const float4*>(p);
    hv[0] = h0.x; hv[1] = h0.y; hv[2] = h0.z; hv[3] = h0.w;
    if (NHP == 8) {
        const float4 h1 = *reinterpret_cast<const float4*>(p + 4);
        hv[4] = h1.x; hv[5] = h1.y; hv[6] = h1.z; hv[7] = h1.w;
    } else { hv[4] = hv[5] = hv[6] = hv[7] = 0.0f; }
}

__device__ __forceinline__ float log_softmax_at(const float (&hv)[8], int A, int act)
{
    float mx = hv[0];
#pragma unroll
    for (int j = 1; j < 8; ++j) if (j < A) mx = fmaxf(mx, hv[j]);
    float Z = 0.0f, ha = hv[0];
#pragma unroll
    for (int j = 0; j < 8; ++j) { if (j < A) Z += det_exp(hv[j] - mx); if (j == act) ha = hv[j]; }
    return ha - mx - det_log(Z);
}

// first pass, one lane per sample, no order: the truncated ratio rho (parked in ret, where the scan
// picks it up before it overwrites the slot with v) and eps_new
__global__ __launch_bounds__(WG) void vtrace_ratio(const VtraceArgs a)
{
    const size_t i = (size_t)blockIdx.x * WG + threadIdx.x;
    if (i >= (size_t)a.B * a.T) return;
    float hn[8], ho[8];
    load_head(a.head_new + i * a.NHP, a.NHP, hn);
    load_head(a.head_old + i * a.NHP, a.NHP, ho);
    float lw;
    if (a.policy == POLICY_CATEGORICAL) {
        const int act = a.act[i];
        lw = log_softmax_at(hn, a.A, act) - log_softmax_at(ho, a.A, act);
    } else {
        const float lso = fminf(fmaxf(ho[1], -5.0f), 2.0f), lsn = fminf(fmaxf(hn[1], -5.0f), 2.0f);
        const float eo = a.eps_old[i];
        const float z = fmaf(det_exp(lso), eo, ho[0]);       // the sampler's own expression
        const float en = (z - hn[0]) / det_exp(lsn);
        a.eps_new[i] = en;
        lw = (-0.5f * en * en - lsn) - (-0.5f * eo * eo - lso);
    }
    if (a.ret) a.ret[i] = fminf(1.0f, det_exp(lw));          // null: only eps_new is wanted
}

// second pass, one lane per env, backwards in t
__global__ __launch_bounds__(WG) void vtrace_scan(const VtraceArgs a)
{
    const int b = blockIdx.x * WG + threadIdx.x;
    if (b >= a.B) return;
    const int B = a.B, T = a.T;
    float Vnext = a.val_new[(size_t)T * B + b];
    float tail = 0.0f;                                       // v_{t+1} - V_{t+1}
#pragma unroll 4
    for (int t = T - 1; t >= 0; --t) {
        const size_t i = (size_t)t * B + b;
        const float rho = a.ret[i], V = a.val_new[i], r = a.rew[i];
        const float c = a.lambda * rho;
        const float disc = a.done[i] ? 0.0f : a.gamma;
        a.adv[i] = rho * (fmaf(disc, Vnext + tail, r) - V);
        tail = fmaf(disc * c, tail, rho * (fmaf(disc, Vnext, r) - V));
        a.ret[i] = V + tail;
        Vnext = V;
    }
}

// ---------------------------------------------------------------------------
// Per sample: l = -A log pi(a|s) + c_v (G - V)^2 - beta H, and d l / d head / M.
// Categorical: d/dlogit_i = -A (1[i=a] - p_i) + beta p_i (log p_i + H).
// Gaussian (score function at the stored noise, log_sigma clamped to [-5,2]):
// d/dmu = -A eps / sigma, d/dlog_sigma = -A (eps^2 - 1) - beta (0 when clamped).
// Also block sums of the loss terms, rewards and episode ends for the metrics.
// ---------------------------------------------------------------------------
struct HeadGradArgs {
    int M, A, NH, NHP, policy;
    const float* head; const uint8_t* act; const float* eps; const float* adv; const float* ret;
    const float* rew; const uint8_t* done;
    float* dhead; float* loss_part;        // [blocks][8]
    float beta, cv, inv_m;
    const float* path;                     // pathwise policy gradient: dL/d(mu, log_sigma) per sample replaces the
                                           // score-function term, and the reported policy loss is minus the mean reward
};

// one sample: its loss terms, and its head gradient to a.dhead.  A_, G_: advantage and return of the sample
__device__ __forceinline__ void head_grad_sample(const HeadGradArgs& a, const int i, float A_, const float G_,
                                                 float& lp_term, float& v_term, float& e_term, float& rsum, float& dcount)
{
    {
        const float* h = a.head + (size_t)i * a.NHP;
        float hv[8];
        const float4 h0 = *reinterpret_cast<const float4*>(h);
        hv[0] = h0.x; hv[1] = h0.y; hv[2] = h0.z; hv[3] = h0.w;
        if (a.NHP == 8) {
            const float4 h1 = *reinterpret_cast<const float4*>(h + 4);
            hv[4] = h1.x; hv[5] = h1.y; hv[6] = h1.z; hv[7] = h1.w;
        } else { hv[4] = hv[5] = hv[6] = hv[7] = 0.0f; }
        if (a.path) A_ = 0.0f;
        float V = hv[0];
#pragma unroll
        for (int j = 1; j < 8; ++j) if (j == a.NH - 1) V = hv[j];
        float d[8] = {0, 0, 0, 0, 0, 0, 0, 0};
        const float dv = G_ - V;
        v_term = a.cv * dv * dv;
        const float gV = -2.0f * a.cv * dv * a.inv_m;
        if (a.policy == POLICY_CATEGORICAL) {
            const int act = a.act[i];
            float mx = hv[0];
#pragma unroll
            for (int j = 1; j < 8; ++j) if (j < a.A) mx = fmaxf(mx, hv[j]);
            float e[8], Z = 0.0f;
#pragma unroll
            for (int j = 0; j < 8; ++j) { e[j] = (j < a.A) ? det_exp(hv[j] - mx) : 0.0f; Z += e[j]; }
            const float logZ = det_log(Z), invZ = 1.0f / Z;
            float H = 0.0f, lpa = 0.0f, p[8], lp[8];
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                lp[j] = hv[j] - mx - logZ;
                p[j] = e[j] * invZ;
                if (j < a.A) H -= p[j] * lp[j];
                if (j == act) lpa = lp[j];
            }
#pragma unroll
            for (int j = 0; j < 8; ++j)
                if (j < a.A) d[j] = (-A_ * ((j == act ? 1.0f : 0.0f) - p[j]) + a.beta * p[j] * (lp[j] + H)) * a.inv_m;
            lp_term = -A_ * lpa;
            e_term = -a.beta * H;
        } else {
            const float ls = hv[1];
            const bool clamped = ls < -5.0f || ls > 2.0f;
            const float lsc = fminf(fmaxf(ls, -5.0f), 2.0f);
            const float sigma = det_exp(lsc), ep = a.eps[i];
            d[0] = (-A_ * ep / sigma) * a.inv_m;
            d[1] = clamped ? 0.0f : (-A_ * (ep * ep - 1.0f) - a.beta) * a.inv_m;
            lp_term = -A_ * (-0.5f * ep * ep - lsc - 0x1.d67f1cp-1f);
            e_term = -a.beta * (lsc + 0x1.6b3f8ep+0f);
        }
#pragma unroll
        for (int j = 0; j < 8; ++j) if (j == a.NH - 1) d[j] = gV;
        if (a.path) {
            const float2 pg = *reinterpret_cast<const float2*>(a.path + (size_t)i * 2);
            d[0] += pg.x; d[1] += pg.y;
            lp_term = -a.rew[i];
        }
        float* o = a.dhead + (size_t)i * a.NHP;
        *reinterpret_cast<float4*>(o) = make_float4(d[0], d[1], d[2], d[3]);
        if (a.NHP == 8) *reinterpret_cast<float4*>(o + 4) = make_float4(d[4], d[5], d[6], d[7]);
        rsum = a.rew[i];
        dcount = a.done[i] ? 1.0f : 0.0f;
    }
}

// fixed-order block reduction of the five loss / metric sums: butterfly inside a wave, then waves in order
__device__ __forceinline__ void loss_block_sums(float lp_term, float v_term, float e_term, float rsum, float dcount,
                                                float (&red)[WG / 64][8], float* __restrict__ loss_part)
{
    float vals[5] = {lp_term, v_term, e_term, rsum, dcount};
#pragma unroll
    for (int k = 0; k < 5; ++k)
        for (int off = 32; off > 0; off >>= 1) vals[k] += __shfl_xor(vals[k], off, 64);
    const int wave = threadIdx.x >> 6;
    if ((threadIdx.x & 63) == 0)
        for (int k = 0; k < 5; ++k) red[wave][k] = vals[k];
    __syncthreads();
    if (threadIdx.x < 8) {
        float s = 0.0f;
        if (threadIdx.x < 5)
            for (int w = 0; w < WG / 64; ++w) s += red[w][threadIdx.x];
        loss_part[(size_t)blockIdx.x * 8 + threadIdx.x] = s;
    }
}

__global__ __launch_bounds__(WG) void head_grad(const HeadGradArgs a)
{
    __shared__ float red[WG / 64][8];
    const int i = blockIdx.x * WG + threadIdx.x;
    float lp_term = 0.0f, v_term = 0.0f, e_term = 0.0f, rsum = 0.0f, dcount = 0.0f;
    if (i < a.M) head_grad_sample(a, i, a.adv[i], a.ret[i], lp_term, v_term, e_term, rsum, dcount);
    loss_block_sums(lp_term, v_term, e_term, rsum, dcount, red, a.loss_part);
}

// ---------------------------------------------------------------------------
// Returns and loss in one launch (the plain on-policy update): a workgroup owns E envs for all T steps (8 or 16:
// 256 samples or fewer where that is possible, so that every thread takes one).  Its
// rewards, values and episode ends come into LDS with every thread loading, the first E lanes then run
// returns_scan's recursion out of LDS (returns and advantages to memory, for the caller to see, and to LDS), and
// every thread takes the samples s, s + 256, ... of the workgroup's T x E through head_grad's arithmetic.
// One launch and no trip of the advantages through memory between the two.
// ---------------------------------------------------------------------------
constexpr int SL_MAXN = 1024;            // samples of a workgroup at most (T x envs)
struct ScanLossArgs {
    HeadGradArgs g;
    int B, T, E;                           // E: envs per workgroup (8 or 16)
    const float* val;                      // [T + 1][B]
    float gamma, lambda;
    float* adv_out; float* ret_out;
};

__global__ __launch_bounds__(WG) void scan_loss(const ScanLossArgs a)
{
    __shared__ float red[WG / 64][8];
    __shared__ float rews[SL_MAXN], vals[SL_MAXN + 16], discs[SL_MAXN];
    __shared__ float advs[SL_MAXN], rets[SL_MAXN];
    const int B = a.B, T = a.T, SL_E = a.E, tid = threadIdx.x;
    const int b0 = blockIdx.x * SL_E;
    const int n = T * SL_E;
    for (int s = tid; s < n + SL_E; s += WG) {
        const int t = s / SL_E, e = s - t * SL_E;
        const size_t i = (size_t)t * B + b0 + e;
        vals[s] = a.val[i];
        if (s < n) { rews[s] = a.g.rew[i]; discs[s] = a.g.done[i] ? 0.0f : a.gamma; }
    }
    __syncthreads();
    if (tid < SL_E) {
        const float oml = 1.0f - a.lambda;
        float G = vals[n + tid], vnext = G;
        for (int t = T - 1; t >= 0; --t) {
            const int s = t * SL_E + tid;
            const float v = vals[s];
            const float mix = fmaf(a.lambda, G, oml * vnext);
            G = fmaf(discs[s], mix, rews[s]);
            rets[s] = G;
            advs[s] = G - v;
            vnext = v;
        }
    }
    __syncthreads();
    float lp_term = 0.0f, v_term = 0.0f, e_term = 0.0f, rsum = 0.0f, dcount = 0.0f;
    for (int s = tid; s < n; s += WG) {
        const int t = s / SL_E, e = s - t * SL_E;
        const int i = t * B + b0 + e;
        const float A_ = advs[s], G_ = rets[s];
        a.adv_out[i] = A_;
        a.ret_out[i] = G_;
        float l0, l1, l2, l3, l4;
        head_grad_sample(a.g, i, A_, G_, l0, l1, l2, l3, l4);
        lp_term += l0; v_term += l1; e_term += l2; rsum += l3; dcount += l4;
    }
    loss_block_sums(lp_term, v_term, e_term, rsum, dcount, red, a.g.loss_part);
}

// ---------------------------------------------------------------------------
// Heads: dWh[j][a] = sum_m h[m][j] dhead[m][a], dbh[a] = sum_m dhead[m][a] (per
// row chunk, as split-K partials) and dZ[m][j] = (h[m][j] > 0) sum_a Wh[j][a]
// dhead[m][a].  K = NH <= 5 is no matrix-core shape: plain vector FMAs, one
// pass over h (read) and dZ (write), both coalesced.
// A workgroup handles `rows` consecutive samples; when the hidden width is
// below 256 several rows are processed side by side and their partial sums are
// combined through LDS in a fixed order.
// ---------------------------------------------------------------------------
struct HeadBwdArgs {
    int M, H, NH, NHP, rows;
    const float* h; const float* dhead; const float* wh;   // wh: theta + wh_off, [H][NH]
    float* dz; float* partial;                             // partial: [splits][H*NH + NH]
    int bf16;
};

// Each lane owns four consecutive hidden units (16-byte loads and stores), H/4 lanes
// cover a row, and 256/(H/4) rows are processed side by side by one workgroup.
__global__ __launch_bounds__(WG) void head_backward(const HeadBwdArgs a)
{
    extern __shared__ float lds[];                          // [groups][H*NH + NH] for the final combine
    const int H = a.H, NH = a.NH, NHP = a.NHP;
    const int hw = H >> 2;                                  // lanes across the hidden dimension (<= 256)
    const int groups = WG / hw;                             // rows processed side by side
    const int g = threadIdx.x / hw, j = (threadIdx.x % hw) << 2;
    const int split = blockIdx.x;
    const int m_begin = split * a.rows, m_end = m_begin + a.rows;
    float w[4][8], dw[4][8], db[8];
#pragma unroll
    for (int c = 0; c < 4; ++c)
#pragma unroll
        for (int k = 0; k < 8; ++k) {
            float x = (k < NH) ? a.wh[(size_t)(j + c) * NH + k] : 0.0f;
            if (a.bf16) x = bf16_to_f(bf16_bits(x));
            w[c][k] = x; dw[c][k] = 0.0f;
        }
#pragma unroll
    for (int k = 0; k < 8; ++k) db[k] = 0.0f;
    const float* __restrict__ hin = a.h;
    const float* __restrict__ dhin = a.dhead;
    float* __restrict__ dzo = a.dz;
    constexpr int RB = 4;                                   // rows in flight per lane
    for (int mb = m_begin + g; mb < m_end; mb += RB * groups) {
        float4 hv4[RB], d0[RB], d1[RB];
#pragma unroll
        for (int u = 0; u < RB; ++u) {
            const int m = mb + u * groups;
            const bool ok = m < m_end;
            hv4[u] = ok ? *reinterpret_cast<const float4*>(hin + (size_t)m * H + j) : make_float4(0, 0, 0, 0);
            d0[u] = ok ? *reinterpret_cast<const float4*>(dhin + (size_t)m * NHP) : make_float4(0, 0, 0, 0);
            d1[u] = (ok && NHP == 8) ? *reinterpret_cast<const float4*>(dhin + (size_t)m * NHP + 4) : make_float4(0, 0, 0, 0);
        }
#pragma unroll
        for (int u = 0; u < RB; ++u) {
            const int m = mb + u * groups;
            if (m >= m_end) break;
            const float d[8] = {d0[u].x, d0[u].y, d0[u].z, d0[u].w, d1[u].x, d1[u].y, d1[u].z, d1[u].w};
            const float hv[4] = {hv4[u].x, hv4[u].y, hv4[u].z, hv4[u].w};
            float o[4];
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                float sacc = 0.0f;
#pragma unroll
                for (int k = 0; k < 8; ++k) {
                    if (k < NH) {
                        sacc = fmaf(w[c][k], d[k], sacc);
                        dw[c][k] = fmaf(hv[c], d[k], dw[c][k]);
                    }
                }
                o[c] = hv[c] > 0.0f ? sacc : 0.0f;
            }
#pragma unroll
            for (int k = 0; k < 8; ++k) if (k < NH) db[k] += d[k];
            *reinterpret_cast<float4*>(dzo + (size_t)m * H + j) = make_float4(o[0], o[1], o[2], o[3]);
        }
    }
    // combine the row groups in ascending group order
    const int stride = H * NH + NH;
    float* out = a.partial + (size_t)split * stride;
    float* mine = lds + (size_t)g * stride;
#pragma unroll
    for (int c = 0; c < 4; ++c)
        for (int k = 0; k < NH; ++k) mine[(j + c) * NH + k] = dw[c][k];
    if (j == 0) for (int k = 0; k < NH; ++k) mine[H * NH + k] = db[k];
    __syncthreads();
    for (int i = threadIdx.x; i < stride; i += WG) {
        float s = 0.0f;
        for (int gg = 0; gg < groups; ++gg) s += lds[(size_t)gg * stride + i];
        out[i] = s;
    }
}

// The same pass on the matrix cores (v_mfma_f32_32x32x2_f32, whose sum over the reduction index is
// the same ascending fma chain the vector kernel uses, so dZ_L is unchanged bit for bit):
//   dZ_L tile [32 samples][32 units] = dhead[32][8] Wh^T[8][32]        4 MFMAs, then the ReLU mask
//   dWh  tile [32 units][heads]     += h^T[32][2 samples] dhead[2][..]  16 MFMAs per 32 samples
// The reduction over samples may take them in any order as long as both operands agree; step (g, q)
// uses sample 8g + 4kg + q for lane half kg, which is the row of the dZ_L accumulator that lane holds,
// so one load of h serves as operand and as mask.  A workgroup walks its rows 32 at a time;
// wavefront w owns units 64w..64w+63 of the 256 the workgroup covers.
typedef float f16v_h __attribute__((ext_vector_type(16)));

__global__ __launch_bounds__(WG) void head_backward_mfma(const HeadBwdArgs a)
{
    __shared__ float Dl[2][32 * 8];                          // head gradients of the current 32 samples, double buffered
    __shared__ float red[WG];
    const int H = a.H, NH = a.NH, NHP = a.NHP;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, l32 = lane & 31, kg = lane >> 5;
    const int jw = blockIdx.y * 256 + wave * 64;             // first unit of this wavefront
    const bool active = jw < H;                              // H is a multiple of 64
    const int split = blockIdx.x;
    const int m_begin = split * a.rows, m_end = m_begin + a.rows;
    // Wh of this lane's unit in both tiles, as B operand of the dZ product: step i takes heads 2i + kg
    float wB[2][4];
#pragma unroll
    for (int t = 0; t < 2; ++t)
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int k = 2 * i + kg;
            float x = (active && k < NH) ? a.wh[(size_t)(jw + 32 * t + l32) * NH + k] : 0.0f;
            if (a.bf16) x = bf16_to_f(bf16_bits(x));
            wB[t][i] = x;
        }
    f16v_h accw[2];
#pragma unroll
    for (int t = 0; t < 2; ++t)
#pragma unroll
        for (int r = 0; r < 16; ++r) accw[t][r] = 0.0f;
    // staging: thread (sample tid / 8, head tid % 8) moves one head gradient per step and keeps its sum
    const int ss = tid >> 3, sk = tid & 7;
    float dsum = 0.0f;
    auto stage = [&](int buf, int m0) {
        const float v = (sk < NH) ? a.dhead[(size_t)(m0 + ss) * NHP + sk] : 0.0f;
        Dl[buf][tid] = v;
        dsum += v;
    };
    const float* __restrict__ hin = a.h + jw + l32;
    float* __restrict__ dzo = a.dz + jw + l32;
    stage(0, m_begin);
    __syncthreads();
    int buf = 0;
    for (int m0 = m_begin; m0 < m_end; m0 += 32, buf ^= 1) {
        if (m0 + 32 < m_end) stage(buf ^ 1, m0 + 32);        // visible after the barrier at the end of this step
        if (active) {
            float hv[2][16];
#pragma unroll
            for (int t = 0; t < 2; ++t)
#pragma unroll
                for (int r = 0; r < 16; ++r)
                    hv[t][r] = hin[(size_t)(m0 + 8 * (r >> 2) + 4 * kg + (r & 3)) * H + 32 * t];
            // dZ product: A = dhead[sample l32][head 2i + kg]
            float dA[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) dA[i] = Dl[buf][l32 * 8 + 2 * i + kg];
            // dWh product: B = dhead[sample 8g + 4kg + q][head l32] for l32 < 8, zero columns beyond
            float dB[16];
#pragma unroll
            for (int r = 0; r < 16; ++r) dB[r] = l32 < 8 ? Dl[buf][(8 * (r >> 2) + 4 * kg + (r & 3)) * 8 + l32] : 0.0f;
#pragma unroll
            for (int t = 0; t < 2; ++t) {
                f16v_h accz;
#pragma unroll
                for (int r = 0; r < 16; ++r) accz[r] = 0.0f;
#pragma unroll
                for (int i = 0; i < 4; ++i) accz = __builtin_amdgcn_mfma_f32_32x32x2f32(dA[i], wB[t][i], accz, 0, 0, 0);
#pragma unroll
                for (int r = 0; r < 16; ++r) accw[t] = __builtin_amdgcn_mfma_f32_32x32x2f32(hv[t][r], dB[r], accw[t], 0, 0, 0);
#pragma unroll
                for (int r = 0; r < 16; ++r)
                    dzo[(size_t)(m0 + 8 * (r >> 2) + 4 * kg + (r & 3)) * H + 32 * t] = hv[t][r] > 0.0f ? accz[r] : 0.0f;
            }
        }
        __syncthreads();
    }
    // dWh: row = unit 8(r/4) + 4kg + r%4 of the tile, column = head l32
    float* out = a.partial + (size_t)split * ((size_t)H * NH + NH);
    if (active && l32 < NH) {
#pragma unroll
        for (int t = 0; t < 2; ++t)
#pragma unroll
            for (int r = 0; r < 16; ++r)
                out[(size_t)(jw + 32 * t + 8 * (r >> 2) + 4 * kg + (r & 3)) * NH + l32] = accw[t][r];
    }
    if (blockIdx.y == 0) {
        red[tid] = dsum;
        __syncthreads();
        if (tid < NH) {
            float sum = 0.0f;
            for (int i = 0; i < 32; ++i) sum += red[i * 8 + tid];
            out[(size_t)H * NH + tid] = sum;
        }
    }
}

// ---------------------------------------------------------------------------
// Second stage of a two-level split-K sum: dst[s][i] = sum_{f < fan} src[s*fan + f][i],
// in ascending f.  Lets a bandwidth-bound producer use many small workgroups while the
// Adam kernel still sees few partials.
// ---------------------------------------------------------------------------
__global__ __launch_bounds__(WG) void partial_reduce(const float* __restrict__ src, float* __restrict__ dst, int count, int fan)
{
    const int i = blockIdx.x * WG + threadIdx.x, s = blockIdx.y;
    if (i >= count) return;
    const float* p = src + (size_t)s * fan * count + i;
    float acc = 0.0f;
#pragma unroll 4
    for (int f = 0; f < fan; ++f) acc += p[(size_t)f * count];
    dst[(size_t)s * count + i] = acc;
}

// ---------------------------------------------------------------------------
// First-layer gradient without a GEMM.  The Catch observation is a 0/1 board
// with exactly two cells set, so dW1 = X^T dZ1 is a scatter: every sample adds
// its dZ1 row into the two weight rows its board selects.  Lane j owns column j
// of an LDS accumulator [cells][columns]; rows of the chunk are visited in
// order, so the sum is deterministic and needs no atomics.  The pendulum's
// three-feature observation is handled by the same kernel with three register
// accumulators per lane.  Column sums (the bias gradient) come for free.
// ---------------------------------------------------------------------------
struct FirstGradArgs {
    int M, K, N, rows;
    const float* dy;          // [M][N] gradient w.r.t. the first layer's pre-activations
    float* partial;           // [splits][K*N + N]
    ObsLite obs;
};

template <int ENV>
__global__ __launch_bounds__(WG) void first_layer_grad(const FirstGradArgs a)
{
    extern __shared__ float accs[];                          // [groups][K][cw]
    const int N = a.N, K = a.K;
    const int cw = N < WG ? N : WG, groups = WG / cw;
    const int g = threadIdx.x / cw, jl = threadIdx.x % cw;
    const int j = blockIdx.y * WG + jl;
    const int split = blockIdx.x;
    const int m_begin = split * a.rows, m_end = m_begin + a.rows;
    float* mine = accs + (size_t)g * K * cw + jl;            // this lane's column, stride cw between cells
    if (ENV == ENV_CATCH) for (int k = 0; k < K; ++k) mine[k * cw] = 0.0f;
    float bsum = 0.0f, r0 = 0.0f, r1 = 0.0f, r2 = 0.0f;
    const float* __restrict__ dyin = a.dy;
    constexpr int RB = 16;                                   // rows in flight per lane
    for (int mb = m_begin + g; mb < m_end; mb += RB * groups) {
        float d[RB], f0[RB], f1[RB];
        uint32_t sw[RB];
#pragma unroll
        for (int u = 0; u < RB; ++u) {
            const int m = mb + u * groups;
            const bool ok = m < m_end;
            d[u] = ok ? dyin[(size_t)m * N + j] : 0.0f;
            if (ENV == ENV_CATCH) sw[u] = ok ? a.obs.s0[m] : 0u;
            else { f0[u] = ok ? a.obs.f0[m] : 0.0f; f1[u] = ok ? a.obs.f1[m] : 0.0f; }
        }
#pragma unroll
        for (int u = 0; u < RB; ++u) {
            if (mb + u * groups >= m_end) break;
            bsum += d[u];
            if (ENV == ENV_CATCH) {
                int bc, pc;
                catch_obs_cells(a.obs.env, sw[u], bc, pc);
                mine[bc * cw] += d[u];
                mine[pc * cw] += d[u];
            } else {
                float sn, cs;
                det_sincos(f0[u], sn, cs);
                r0 = fmaf(cs, d[u], r0); r1 = fmaf(sn, d[u], r1); r2 = fmaf(f1[u], d[u], r2);
            }
        }
    }
    float* out = a.partial + (size_t)split * ((size_t)K * N + N);
    if (ENV != ENV_CATCH) { mine[0] = r0; mine[cw] = r1; mine[2 * cw] = r2; }
    __shared__ float bred[WG];
    bred[threadIdx.x] = bsum;
    __syncthreads();
    // combine the row groups in ascending order
    for (int i = threadIdx.x; i < K * cw; i += WG) {
        const int k = i / cw, c = i % cw;
        float s = 0.0f;
        for (int gg = 0; gg < groups; ++gg) s += accs[((size_t)gg * K + k) * cw + c];
        out[(size_t)k * N + blockIdx.y * WG + c] = s;
    }
    if (threadIdx.x < cw) {
        float s = 0.0f;
        for (int gg = 0; gg < groups; ++gg) s += bred[gg * cw + threadIdx.x];
        out[(size_t)K * N + blockIdx.y * WG + threadIdx.x] = s;
    }
}

// Pendulum first layer for widths that are multiples of 256: the three observation features of a
// row (cos, sin, angular velocity) are computed once per row by one thread and shared through LDS,
// instead of once per row by every column; lane j then walks the rows in ascending order.
__global__ __launch_bounds__(WG) void first_layer_grad_pendulum(const FirstGradArgs a)
{
    __shared__ float feat[3][WG];
    const int N = a.N;
    const int j = blockIdx.y * WG + threadIdx.x;
    const int split = blockIdx.x;
    const int m_begin = split * a.rows, m_end = m_begin + a.rows;
    float bsum = 0.0f, r0 = 0.0f, r1 = 0.0f, r2 = 0.0f;
    const float* __restrict__ dy = a.dy + j;
    for (int mb = m_begin; mb < m_end; mb += WG) {
        const int m = mb + threadIdx.x;
        float sn = 0.0f, cs = 0.0f, td = 0.0f;
        if (m < m_end) { det_sincos(a.obs.f0[m], sn, cs); td = a.obs.f1[m]; }
        __syncthreads();                                     // the previous batch has been consumed
        feat[0][threadIdx.x] = cs; feat[1][threadIdx.x] = sn; feat[2][threadIdx.x] = td;
        __syncthreads();
        const int n = m_end - mb < WG ? m_end - mb : WG;
        constexpr int RB = 16;
        for (int u0 = 0; u0 < n; u0 += RB) {
            float d[RB];
#pragma unroll
            for (int u = 0; u < RB; ++u) d[u] = u0 + u < n ? dy[(size_t)(mb + u0 + u) * N] : 0.0f;
#pragma unroll
            for (int u = 0; u < RB; ++u) {
                if (u0 + u >= n) break;
                bsum += d[u];
                r0 = fmaf(feat[0][u0 + u], d[u], r0); r1 = fmaf(feat[1][u0 + u], d[u], r1); r2 = fmaf(feat[2][u0 + u], d[u], r2);
            }
        }
    }
    float* out = a.partial + (size_t)split * ((size_t)a.K * N + N);
    out[j] = r0; out[(size_t)N + j] = r1; out[(size_t)2 * N + j] = r2;
    out[(size_t)a.K * N + j] = bsum;
}

// The same scatter on the matrix cores for boards of at most 63 cells: dW1 = X^T dZ1 with the 0/1
// board rebuilt from the state word, v_mfma_f32_32x32x2_f32 taking two samples per step.  Row K of
// the padded board is all ones, so the column sums (the bias gradient) fall out of the same product
// and land in the slot after the K weight rows.  The MFMA adds its products in ascending step order,
// which makes the sum as deterministic as the scatter.  A workgroup of eight wavefronts walks its
// samples 64 at a time and reads whole 1 KiB rows of dZ1; wavefront w owns columns 32w..32w+31 and
// both 32-row tiles of the board.  Of each block of 64 samples lane half kg takes sample 32*kg + s at
// step s.  The board operand is the same for all eight wavefronts, so each builds one eighth of it
// (four steps) and shares it through LDS -- vector-ALU work and MFMAs do not overlap well here, and
// this keeps the ALU share small.
typedef float f16v_l __attribute__((ext_vector_type(16)));
typedef float f4v_l __attribute__((ext_vector_type(4)));

typedef __bf16 bf8_l __attribute__((ext_vector_type(8)));
typedef __bf16 bf2_l __attribute__((ext_vector_type(2)));
typedef uint32_t u4v_l __attribute__((ext_vector_type(4)));
__device__ __forceinline__ uint32_t pk_bf16_l(float lo, float hi)
{
    bf2_l v; v[0] = (__bf16)lo; v[1] = (__bf16)hi;               // round to nearest even, one instruction for the pair
    return __builtin_bit_cast(uint32_t, v);
}
// x as three bfloat16 terms whose sum is x (8 + 8 + 8 significand bits): with the 0/1 board as the other operand
// every product is exact and the fp32 accumulation is the one an fp32 matrix instruction would do, at a fifth of
// its matrix-core time (three 8-pass instructions of 16 samples instead of eight 16-pass ones of 2)
__device__ __forceinline__ void split3(const float (&x)[8], u4v_l& hi, u4v_l& mid, u4v_l& lo)
{
    float r[8];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const uint32_t p = pk_bf16_l(x[2 * i], x[2 * i + 1]);
        hi[i] = p;
        r[2 * i] = x[2 * i] - f_from_bits(p << 16);
        r[2 * i + 1] = x[2 * i + 1] - f_from_bits(p & 0xffff0000u);
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const uint32_t p = pk_bf16_l(r[2 * i], r[2 * i + 1]);
        mid[i] = p;
        lo[i] = pk_bf16_l(r[2 * i] - f_from_bits(p << 16), r[2 * i + 1] - f_from_bits(p & 0xffff0000u));
    }
}

__global__ __launch_bounds__(512) void first_layer_grad_mfma(const FirstGradArgs a)
{
    __shared__ u4v_l xs[2][2][4][64];                          // [buffer][tile of 32 cells][step of 16 samples][lane]
    const int N = a.N, K = a.K;
    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6), l32 = lane & 31, kg = lane >> 5;
    const int j = blockIdx.y * 256 + wave * 32 + l32;
    const int split = blockIdx.x;
    const int m_begin = split * a.rows, m_end = m_begin + a.rows;   // a.rows is a multiple of 64, N of 256
    f16v_l acc0, acc1;
#pragma unroll
    for (int r = 0; r < 16; ++r) { acc0[r] = 0.0f; acc1[r] = 0.0f; }
    const uint32_t lane_off = (uint32_t)(32 * kg) * (uint32_t)N + (uint32_t)j;
    // loads of one block of 64 samples: this lane's 32 values of dZ1 (samples 32 kg + 0..31 of column j) and the
    // state word of sample m0 + lane
    auto load = [&](float (&d)[32], uint32_t& sw, int m0) {
        sw = a.obs.s0[m0 + lane];
#pragma unroll
        for (int s = 0; s < 32; ++s) d[s] = (a.dy + (size_t)(m0 + s) * N)[lane_off];
    };
    // The reduction index of step t is k = 8 kg + q for sample 32 kg + 8 t + q of the block: lane (cell l32, half kg)
    // of the board operand holds the 0/1 entries of its cell for those eight samples as bfloat16.  Wavefront w builds
    // the operand of (tile w & 1, step w >> 1) for everybody.
    auto build = [&](uint32_t sw, int buf) {
        int bc, pc;
        catch_obs_cells(a.obs.env, sw, bc, pc);
        const unsigned long long bits = (1ull << bc) | (1ull << pc) | (1ull << K);   // lane l: board of sample l, ones row K
        const uint32_t mine = (wave & 1) ? (uint32_t)(bits >> 32) : (uint32_t)bits;  // the 32 cells of this wavefront's tile
        const int t = wave >> 1;
        u4v_l x;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            uint32_t w2 = 0;
#pragma unroll
            for (int e = 0; e < 2; ++e) {
                const int q = 2 * i + e;
                const uint32_t b0 = (uint32_t)__builtin_amdgcn_readlane((int)mine, 8 * t + q);
                const uint32_t b1 = (uint32_t)__builtin_amdgcn_readlane((int)mine, 32 + 8 * t + q);
                const uint32_t bit = ((kg ? b1 : b0) >> l32) & 1u;
                w2 |= (bit * 0x3f80u) << (16 * e);                 // bfloat16 1.0
            }
            x[i] = w2;
        }
        xs[buf][wave & 1][t][lane] = x;
    };
    auto compute = [&](const float (&d)[32], int buf) {
#pragma unroll
        for (int t = 0; t < 4; ++t) {
            const u4v_l x0 = xs[buf][0][t][lane], x1 = xs[buf][1][t][lane];
            float v[8];
#pragma unroll
            for (int q = 0; q < 8; ++q) v[q] = d[8 * t + q];
            u4v_l hi, mid, lo;
            split3(v, hi, mid, lo);
            const bf8_l a0 = __builtin_bit_cast(bf8_l, x0), a1 = __builtin_bit_cast(bf8_l, x1);
            const bf8_l bh = __builtin_bit_cast(bf8_l, hi), bm = __builtin_bit_cast(bf8_l, mid), bl = __builtin_bit_cast(bf8_l, lo);
            // smallest terms first
            acc0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a0, bl, acc0, 0, 0, 0);
            acc1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a1, bl, acc1, 0, 0, 0);
            acc0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a0, bm, acc0, 0, 0, 0);
            acc1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a1, bm, acc1, 0, 0, 0);
            acc0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a0, bh, acc0, 0, 0, 0);
            acc1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a1, bh, acc1, 0, 0, 0);
        }
    };
    float dA[32], dB[32];
    uint32_t swA, swB;
    // every load is unconditional (past the end it re-reads the last block and the result is dropped), so
    // the wait counters the compiler places before the MFMAs never have to cover the prefetch
    const int m_last = m_end - 64;
    load(dA, swA, m_begin);
    build(swA, 0);
    __syncthreads();
    for (int m0 = m_begin; m0 < m_end; m0 += 128) {
        load(dB, swB, m0 + 64 < m_end ? m0 + 64 : m_last);
        __builtin_amdgcn_sched_barrier(0);
        compute(dA, 0);
        build(swB, 1);
        __syncthreads();
        load(dA, swA, m0 + 128 < m_end ? m0 + 128 : m_last);
        __builtin_amdgcn_sched_barrier(0);
        if (m0 + 64 < m_end) compute(dB, 1);
        build(swA, 0);
        __syncthreads();
    }
    // rows 0..K-1 are dW1, row K the column sums: row i of the padded product goes to out[i*N + j]
    float* out = a.partial + (size_t)split * ((size_t)K * N + N);
#pragma unroll
    for (int r = 0; r < 16; ++r) {
        const int i = 8 * (r >> 2) + 4 * kg + (r & 3);
        if (i <= K) out[(size_t)i * N + j] = acc0[r];
        if (i + 32 <= K) out[(size_t)(i + 32) * N + j] = acc1[r];
    }
}

hipError_t launch_first_layer_grad(anakin* h)
{
    const Layout& L = h->lay;
    const NetShape& n = h->net;
    FirstGradArgs a;
    a.M = h->B * h->T; a.K = n.dims[0]; a.N = n.dims[1];
    a.rows = a.M / h->splits[0];
    a.dy = at<const float>(h, L.dz[0]); a.partial = at<float>(h, L.part[0]);
    a.obs.env = h->env; a.obs.s0 = at<const uint32_t>(h, L.tr_s0);
    a.obs.f0 = at<const float>(h, L.tr_f0); a.obs.f1 = at<const float>(h, L.tr_f1);
    const size_t lds = (size_t)WG * a.K * sizeof(float);
    const dim3 grid(h->splits[0], (a.N + WG - 1) / WG);
    ProfScope prof(h, "first_layer_grad");
    if (h->env.kind == ENV_CATCH && a.K < 64 && a.rows % 64 == 0 && a.N % 256 == 0 && !(h->mode & ANAKIN_MODE_VALU_GEMM)) {
        hipLaunchKernelGGL(first_layer_grad_mfma, dim3(h->splits[0], a.N / 256), dim3(512), 0, h->stream, a);
    } else if (h->env.kind == ENV_CATCH) {
        auto kern = first_layer_grad<ENV_CATCH>;
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) return e;
        hipLaunchKernelGGL(kern, grid, dim3(WG), lds, h->stream, a);
    } else if (a.N % WG == 0 && a.K == 3) {
        hipLaunchKernelGGL(first_layer_grad_pendulum, dim3(h->splits[0], a.N / WG), dim3(WG), 0, h->stream, a);
    } else {
        hipLaunchKernelGGL(first_layer_grad<ENV_PENDULUM>, grid, dim3(WG), lds, h->stream, a);
    }
    return hipGetLastError();
}

// ---------------------------------------------------------------------------
// Whole backward pass of a one-hidden-layer net in one kernel.  Nothing of the
// forward pass is read from HBM: the hidden layer h = relu(b1 + W1[ball] +
// W1[paddle]) (or three fmas for the pendulum) is rebuilt from the 4-byte state
// snapshot with W1 in LDS -- in the acting order, so the bits equal the acting
// ones -- then dZ1 = relu'(h) (Wh dhead), the head-matrix gradient, and the
// scatter of dZ1 into the two selected rows of dW1.  Per sample the kernel
// reads the state word and the dhead row (20 B) and writes nothing; per chunk
// it writes one partial of each parameter region.  Lane j owns hidden unit j.
// ---------------------------------------------------------------------------
struct OneLayerArgs {
    int M, D, H, NH, NHP, rows;
    const float* theta; int w1_off, b1_off, wh_off;
    const float* dhead;
    float* partial0;          // [splits][D*H + H]
    float* partial1;          // [splits][H*NH + NH]
    ObsLite obs;
};

// OLW threads per workgroup: small workgroups keep the LDS accumulators small, so more of them fit a CU
constexpr int OLW = 128;
// NH (number of head outputs) is a template parameter: the per-sample inner loops are the whole cost here
// FULL: the chunk is a whole number of RB x groups sample blocks, so no load needs a bounds check.
// HC: the hidden width when it is known at compile time (index arithmetic by shifts, constant load offsets), else 0.
template <int ENV, int NH, bool FULL, int HC>
__global__ __launch_bounds__(OLW) void learn_one_layer(const OneLayerArgs a)
{
    extern __shared__ float lds[];
    const int H = HC ? HC : a.H, D = a.D;
    constexpr int NHP = NH <= 4 ? 4 : 8;
    const int cw = H < OLW ? H : OLW, groups = OLW / cw;
    float* w1s = lds;                                         // [D][H]
    float* accs = w1s + D * H;                                // [groups][D][cw]
    const int g = threadIdx.x / cw, jl = threadIdx.x % cw;
    const int j = blockIdx.y * OLW + jl;
    for (int i = threadIdx.x; i < D * H; i += OLW) w1s[i] = a.theta[a.w1_off + i];
    float* mine = accs + (size_t)g * D * cw + jl;
    if (ENV == ENV_CATCH) for (int k = 0; k < D; ++k) mine[k * cw] = 0.0f;
    float wh[NH], dwh[NH], dbh[NH];
#pragma unroll
    for (int k = 0; k < NH; ++k) { wh[k] = a.theta[a.wh_off + j * NH + k]; dwh[k] = 0.0f; dbh[k] = 0.0f; }
    const float b1 = a.theta[a.b1_off + j];
    float db1 = 0.0f, r0 = 0.0f, r1 = 0.0f, r2 = 0.0f;
    __syncthreads();
    const int m_begin = blockIdx.x * a.rows, m_end = m_begin + a.rows;
    const float* w1c = w1s + j;
    constexpr int RB = 8;
    for (int mb = m_begin + g; mb < m_end; mb += RB * groups) {
        float4 d0[RB], d1[RB];
        uint32_t sw[RB];
        float f0[RB], f1[RB];
        // one base address per array and trip; the samples of a trip sit at constant distances from it
        const float* dh = a.dhead + (size_t)mb * NHP;
        const uint32_t* sp = a.obs.s0 + mb;
        const float* fp0 = a.obs.f0 + mb;
        const float* fp1 = a.obs.f1 + mb;
#pragma unroll
        for (int u = 0; u < RB; ++u) {
            const int du = u * groups;
            const bool ok = FULL || mb + du < m_end;
            d0[u] = ok ? *reinterpret_cast<const float4*>(dh + du * NHP) : make_float4(0, 0, 0, 0);
            d1[u] = (ok && NHP == 8) ? *reinterpret_cast<const float4*>(dh + du * NHP + 4) : make_float4(0, 0, 0, 0);
            if (ENV == ENV_CATCH) sw[u] = ok ? sp[du] : 0u;
            else { f0[u] = ok ? fp0[du] : 0.0f; f1[u] = ok ? fp1[du] : 0.0f; }
        }
#pragma unroll
        for (int u = 0; u < RB; ++u) {
            if (!FULL && mb + u * groups >= m_end) break;
            const float d[8] = {d0[u].x, d0[u].y, d0[u].z, d0[u].w, d1[u].x, d1[u].y, d1[u].z, d1[u].w};
            float hv, x0 = 0.0f, x1 = 0.0f, x2 = 0.0f;
            int bc = 0, pc = 0;
            if (ENV == ENV_CATCH) {
                catch_obs_cells(a.obs.env, sw[u], bc, pc);
                hv = (b1 + w1c[bc * H]) + w1c[pc * H];
            } else {
                float sn, cs;
                det_sincos(f0[u], sn, cs);
                x0 = cs; x1 = sn; x2 = f1[u];
                hv = fmaf(x2, w1c[2 * H], fmaf(x1, w1c[H], fmaf(x0, w1c[0], b1)));
            }
            hv = hv > 0.0f ? hv : 0.0f;
            float s = 0.0f;
#pragma unroll
            for (int k = 0; k < NH; ++k) { s = fmaf(wh[k], d[k], s); dwh[k] = fmaf(hv, d[k], dwh[k]); dbh[k] += d[k]; }
            const float dz = hv > 0.0f ? s : 0.0f;
            db1 += dz;
            if (ENV == ENV_CATCH) {
                // the ball is never in the paddle's row: two different words, both read before either is stored
                float* pa = mine + bc * cw;
                float* pb = mine + pc * cw;
                const float xa = *pa, xb = *pb;
                *pa = xa + dz;
                *pb = xb + dz;
            }
            else { r0 = fmaf(x0, dz, r0); r1 = fmaf(x1, dz, r1); r2 = fmaf(x2, dz, r2); }
        }
    }
    if (ENV != ENV_CATCH) { mine[0] = r0; mine[cw] = r1; mine[2 * cw] = r2; }
    // per-lane sums of the other regions go through LDS too, then everything is combined group by group
    __shared__ float red[OLW * 10];                            // [10][OLW]: dwh[0..7], db1, (dbh of lane 0 handled below)
#pragma unroll
    for (int k = 0; k < NH; ++k) red[k * OLW + threadIdx.x] = dwh[k];
    red[8 * OLW + threadIdx.x] = db1;
    red[9 * OLW + threadIdx.x] = 0.0f;
    __shared__ float bh_red[8 * 8];                           // [groups <= 8][8]
    if (jl == 0 && blockIdx.y == 0) for (int k = 0; k < NH; ++k) bh_red[g * 8 + k] = dbh[k];
    __syncthreads();
    float* out0 = a.partial0 + (size_t)blockIdx.x * ((size_t)D * H + H);
    float* out1 = a.partial1 + (size_t)blockIdx.x * ((size_t)H * NH + NH);
    for (int i = threadIdx.x; i < D * cw; i += OLW) {
        const int k = i / cw, c = i % cw;
        float s = 0.0f;
        for (int gg = 0; gg < groups; ++gg) s += accs[((size_t)gg * D + k) * cw + c];
        out0[(size_t)k * H + blockIdx.y * OLW + c] = s;
    }
    if (threadIdx.x < cw) {
        const int c = threadIdx.x, col = blockIdx.y * OLW + c;
        float s = 0.0f;
        for (int gg = 0; gg < groups; ++gg) s += red[8 * OLW + gg * cw + c];
        out0[(size_t)D * H + col] = s;
        for (int k = 0; k < NH; ++k) {
            float t = 0.0f;
            for (int gg = 0; gg < groups; ++gg) t += red[k * OLW + gg * cw + c];
            out1[(size_t)col * NH + k] = t;
        }
    }
    if (threadIdx.x < NH && blockIdx.y == 0) {
        float t = 0.0f;
        for (int gg = 0; gg < groups; ++gg) t += bh_red[gg * 8 + threadIdx.x];
        out1[(size_t)H * NH + threadIdx.x] = t;
    }
}

// ---------------------------------------------------------------------------
// Catch with one hidden layer of 32 units (the throughput workload): the WHOLE update up to the
// partial sums in one launch -- returns and advantages, loss and head gradients, and the backward
// pass above -- so that advantages, returns and head gradients never make a round trip through
// HBM (the returns are still written once, for the caller to see) and three launches become one.
// A workgroup of four wavefronts owns a range of envs for all T steps; each wavefront takes 64 of
// them at a time:
//   A1  lane = env: the reverse scan of its column (returns_scan's recursion), adv / ret to HBM
//   A2  lane = env, four time steps at a time: the loss terms and head gradients of its samples
//       (head_grad's arithmetic) into LDS, with the two board cells of the sample as LDS offsets
//   B   lane = (hidden unit, half): each half-wavefront walks every other sample of the chunk:
//       h = relu(b1 + W1[ball] + W1[paddle]) in the acting order, dZ1, the head-matrix sums, and
//       the scatter of dZ1 into the two rows of its own LDS copy of dW1
// All waves run the same trip counts, so workgroup barriers separate A2 from B.
// ---------------------------------------------------------------------------
struct CatchFusedArgs {
    int B, T, D, envs_per_wg;
    EnvDims env;
    const float* theta; int w1_off, b1_off, wh_off;
    const uint32_t* s0; const uint8_t* act; const float* rew; const uint8_t* done; const float* val; const float* head;
    float* adv; float* ret;
    float* partial0;          // [workgroups][D*32 + 32]
    float* partial1;          // [workgroups][32*4 + 4]
    float* loss_part;         // [workgroups][8]
    float gamma, lambda, beta, cv, inv_m;
};

constexpr int CF_WG = 256;              // four wavefronts
constexpr int CF_H = 32;                // hidden units
constexpr int CF_TC = 4;                // time steps per chunk of phases A2 / B

__global__ __launch_bounds__(CF_WG) void learn_catch_fused(const CatchFusedArgs a)
{
    extern __shared__ float lds[];
    const int D = a.D, B = a.B, T = a.T;
    constexpr int H = CF_H;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    float* w1s = lds;                                            // [D][H]
    float* accw = w1s + D * H + (size_t)wave * (2 * D * H + CF_TC * 64 * 4 + CF_TC * 64);
    float* acc = accw;                                           // [2 halves][D][H] this wavefront's dW1 sums
    float4* dh = reinterpret_cast<float4*>(accw + 2 * D * H);    // [CF_TC][64] head gradients of the chunk
    uint32_t* cells = reinterpret_cast<uint32_t*>(dh + CF_TC * 64);   // [CF_TC][64] LDS offsets of the two board cells
    // W1 into LDS in batches of four 16-byte loads per thread (one load, one wait, one store at a time would be a
    // memory round trip per 4 KB); H is a multiple of 4, and so is the offset of W1 in the parameter vector
    {
        const int n4 = D * H / 4;
        const f4v_l* src = reinterpret_cast<const f4v_l*>(a.theta + a.w1_off);
        f4v_l* dst = reinterpret_cast<f4v_l*>(w1s);
        for (int i0 = 0; i0 < n4; i0 += 4 * CF_WG) {
            f4v_l pw[4];
#pragma unroll
            for (int q = 0; q < 4; ++q) { const int i = i0 + q * CF_WG + tid; pw[q] = src[i < n4 ? i : 0]; }
#pragma unroll
            for (int q = 0; q < 4; ++q) { const int i = i0 + q * CF_WG + tid; if (i < n4) dst[i] = pw[q]; }
        }
    }
    for (int i = lane; i < 2 * D * H; i += 64) acc[i] = 0.0f;
    // phase B identity: hidden unit u, half hf (the two halves of a wavefront take alternate samples)
    const int u = lane & 31, hf = lane >> 5;
    float wh[4], dwh[4] = {0, 0, 0, 0};
#pragma unroll
    for (int k = 0; k < 4; ++k) wh[k] = a.theta[a.wh_off + u * 4 + k];
    const float b1 = a.theta[a.b1_off + u];
    float db1 = 0.0f;
    float* mine = acc + (size_t)hf * D * H + u;
    const float* w1c = w1s + u;
    // phase A identity: env e of the wavefront's block; sums of the loss terms and of the head gradients
    float dbh[4] = {0, 0, 0, 0}, sums[5] = {0, 0, 0, 0, 0};
    __syncthreads();
    const float oml = 1.0f - a.lambda;
    const int wg_b0 = blockIdx.x * a.envs_per_wg;
    for (int blk = 0; blk < a.envs_per_wg; blk += CF_WG) {
        const int b = wg_b0 + blk + wave * 64 + lane;
        // ---- A1: returns and advantages of this env, newest step first ----
        {
            float G = a.val[(size_t)T * B + b], vnext = G;
            // eight steps' records are asked for before the first of them is used: the stores of one step and the
            // loads of the next may be the same memory as far as the compiler knows, so step by step every load
            // would wait for its own round trip
            for (int t1 = T; t1 > 0; t1 -= 8) {
                float r8[8], v8[8], d8[8];
#pragma unroll
                for (int u = 0; u < 8; ++u) {
                    const int t = t1 - 1 - u;
                    const size_t i = (size_t)(t >= 0 ? t : 0) * B + b;
                    r8[u] = a.rew[i]; v8[u] = a.val[i]; d8[u] = a.done[i] ? 0.0f : a.gamma;
                }
#pragma unroll
                for (int u = 0; u < 8; ++u) {
                    const int t = t1 - 1 - u;
                    if (t >= 0) {
                        const size_t i = (size_t)t * B + b;
                        const float mix = fmaf(a.lambda, G, oml * vnext);
                        G = fmaf(d8[u], mix, r8[u]);
                        a.ret[i] = G;
                        a.adv[i] = G - v8[u];
                        vnext = v8[u];
                    }
                }
            }
        }
        // the records of a chunk's samples: asked for one chunk ahead, so that they arrive while the chunk before is in
        // phase B (straight after the barrier every load would be a round trip to memory with nothing to hide it)
        f4v_l in_h[CF_TC]; float in_adv[CF_TC], in_ret[CF_TC], in_rew[CF_TC]; uint32_t in_s0[CF_TC]; int in_act[CF_TC], in_done[CF_TC];
        auto fetch_chunk = [&](int t0) {
#pragma unroll
            for (int tt = 0; tt < CF_TC; ++tt) {
                const int t = t0 + tt < T ? t0 + tt : T - 1;         // past the end: re-read the last step, unused
                const size_t i = (size_t)t * B + b;
                in_h[tt] = *reinterpret_cast<const f4v_l*>(a.head + i * 4);
                in_act[tt] = (int)a.act[i]; in_adv[tt] = a.adv[i]; in_ret[tt] = a.ret[i];
                in_rew[tt] = a.rew[i]; in_done[tt] = a.done[i]; in_s0[tt] = a.s0[i];
            }
        };
        fetch_chunk(0);
        for (int t0 = 0; t0 < T; t0 += CF_TC) {
            const int tn = T - t0 < CF_TC ? T - t0 : CF_TC;
            // ---- A2: loss terms and head gradients of (t0 .. t0 + tn - 1, b) ----
#pragma unroll
            for (int tt = 0; tt < CF_TC; ++tt) {
                if (tt < tn) {
                    const float4 hv4 = make_float4(in_h[tt][0], in_h[tt][1], in_h[tt][2], in_h[tt][3]);
                    float d[4], lp_term, v_term, e_term;
                    catch_head_grad(hv4, in_act[tt], in_adv[tt], in_ret[tt], a.beta, a.cv, a.inv_m, d, lp_term, v_term, e_term);
                    sums[0] += lp_term; sums[1] += v_term; sums[2] += e_term; sums[3] += in_rew[tt]; sums[4] += in_done[tt] ? 1.0f : 0.0f;
#pragma unroll
                    for (int k = 0; k < 4; ++k) dbh[k] += d[k];
                    dh[tt * 64 + lane] = make_float4(d[0], d[1], d[2], d[3]);
                    int bc, pc;
                    catch_obs_cells(a.env, in_s0[tt], bc, pc);
                    cells[tt * 64 + lane] = (uint32_t)(bc * H) | ((uint32_t)(pc * H) << 16);
                }
            }
            __syncthreads();
            if (t0 + CF_TC < T) fetch_chunk(t0 + CF_TC);
            // ---- B: half hf takes samples hf, hf + 2, ... of the chunk's tn * 64 ----
            const int ns = tn * 64;
            constexpr int RB = 8;
            for (int s0 = 0; s0 < ns; s0 += 2 * RB) {
                float4 dd[RB];
                uint32_t cc[RB];
#pragma unroll
                for (int q = 0; q < RB; ++q) { dd[q] = dh[s0 + 2 * q + hf]; cc[q] = cells[s0 + 2 * q + hf]; }
                float w0[RB], w1[RB];
#pragma unroll
                for (int q = 0; q < RB; ++q) { w0[q] = w1c[cc[q] & 0xffffu]; w1[q] = w1c[cc[q] >> 16]; }
#pragma unroll
                for (int q = 0; q < RB; ++q) {
                    const float d[4] = {dd[q].x, dd[q].y, dd[q].z, dd[q].w};
                    float hv = (b1 + w0[q]) + w1[q];
                    hv = hv > 0.0f ? hv : 0.0f;
                    float s = 0.0f;
#pragma unroll
                    for (int k = 0; k < 4; ++k) { s = fmaf(wh[k], d[k], s); dwh[k] = fmaf(hv, d[k], dwh[k]); }
                    const float dz = hv > 0.0f ? s : 0.0f;
                    db1 += dz;
                    // the ball is never in the paddle's row, so the two sums are different words: both reads go out
                    // before either store, one LDS round trip per sample instead of two (two samples per round
                    // trip, with the second taking the first's result where they share a word, measured slower)
                    float* pa = mine + (cc[q] & 0xffffu);
                    float* pb = mine + (cc[q] >> 16);
                    const float xa = *pa, xb = *pb;
                    *pa = xa + dz;
                    *pb = xb + dz;
                }
            }
            __syncthreads();
        }
    }
    // ---- sums of the workgroup, in a fixed order: wavefronts ascending, half 0 before half 1 ----
    // every wavefront's dW1 copies are complete (barrier above); the per-lane sums go through the wavefront's
    // head-gradient area, free now: 16 floats per lane
    const size_t ws = (size_t)2 * D * H + CF_TC * 64 * 4 + CF_TC * 64;        // floats per wavefront
    auto red_of = [&](int w, int l) { return w1s + D * H + (size_t)w * ws + 2 * D * H + (size_t)l * 16; };
    {
        float* r = red_of(wave, lane);
#pragma unroll
        for (int k = 0; k < 4; ++k) { r[k] = dwh[k]; r[4 + k] = dbh[k]; }
        r[8] = db1;
#pragma unroll
        for (int k = 0; k < 5; ++k) r[9 + k] = sums[k];
    }
    __syncthreads();
    float* out0 = a.partial0 + (size_t)blockIdx.x * ((size_t)D * H + H);
    float* out1 = a.partial1 + (size_t)blockIdx.x * ((size_t)H * 4 + 4);
    const float* acc_all = w1s + D * H;                          // wavefront w at stride ws
    for (int i = tid; i < D * H; i += CF_WG) {
        float sum = 0.0f;
        for (int w = 0; w < 4; ++w) { sum += acc_all[w * ws + i]; sum += acc_all[w * ws + D * H + i]; }
        out0[i] = sum;
    }
    if (tid < H) {
        float sb = 0.0f, sw[4] = {0, 0, 0, 0};
        for (int w = 0; w < 4; ++w)
            for (int hh = 0; hh < 2; ++hh) {
                const float* r = red_of(w, hh * 32 + tid);
                sb += r[8];
#pragma unroll
                for (int k = 0; k < 4; ++k) sw[k] += r[k];
            }
        out0[(size_t)D * H + tid] = sb;
#pragma unroll
        for (int k = 0; k < 4; ++k) out1[(size_t)tid * 4 + k] = sw[k];
    }
    if (tid < 9) {
        // dbh[0..3] and the five metric sums: over all 256 lanes (envs), ascending
        const int off = tid < 4 ? 4 + tid : 9 + (tid - 4);
        float sum = 0.0f;
        for (int l = 0; l < CF_WG; ++l) sum += red_of(l >> 6, l & 63)[off];
        if (tid < 4) out1[(size_t)H * 4 + tid] = sum;
        else a.loss_part[(size_t)blockIdx.x * 8 + (tid - 4)] = sum;
    }
    if (tid >= 9 && tid < 12) a.loss_part[(size_t)blockIdx.x * 8 + tid - 4] = 0.0f;
}

// whether the fused launch above serves this handle's update (else: scan, loss and one-layer kernels)
bool catch_fused_ok(const anakin* h)
{
    const NetShape& n = h->net;
    return one_layer_fused(h) && h->env.kind == ENV_CATCH && h->env.rows >= 2 && n.dims[1] == CF_H && n.NH == 4 && h->n_updates == 1 &&
           !h->traj_decoupled && !h->pathwise && h->splits[0] > 0 && h->B % (h->splits[0] * CF_WG) == 0 &&
           n.dims[0] * CF_H < 65536 && n.w_off[0] % 4 == 0;           // board-cell offsets are packed into 16 bits; W1 is read 16 bytes at a time
}

hipError_t launch_learn_catch_fused(anakin* h)
{
    const Layout& L = h->lay;
    const NetShape& n = h->net;
    CatchFusedArgs a;
    a.B = h->B; a.T = h->T; a.D = n.dims[0]; a.envs_per_wg = h->B / h->splits[0];
    a.env = h->env;
    a.theta = at<const float>(h, L.w_src); a.w1_off = n.w_off[0]; a.b1_off = n.b_off[0]; a.wh_off = n.wh_off;
    a.s0 = at<const uint32_t>(h, L.tr_s0); a.act = at<const uint8_t>(h, L.tr_act); a.rew = at<const float>(h, L.tr_rew);
    a.done = at<const uint8_t>(h, L.tr_done); a.val = at<const float>(h, L.tr_val); a.head = at<const float>(h, L.tr_head);
    a.adv = at<float>(h, L.adv); a.ret = at<float>(h, L.ret);
    a.partial0 = at<float>(h, L.part[0]); a.partial1 = at<float>(h, L.part[1]); a.loss_part = at<float>(h, L.loss_part);
    a.gamma = h->net_cfg.gamma; a.lambda = h->net_cfg.lambda_; a.beta = h->net_cfg.entropy_coef; a.cv = h->net_cfg.value_coef;
    a.inv_m = (float)(1.0 / ((double)h->B * h->T));
    const size_t lds = ((size_t)a.D * CF_H + 4 * ((size_t)2 * a.D * CF_H + CF_TC * 64 * 4 + CF_TC * 64)) * sizeof(float);
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(learn_catch_fused), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return e;
    h->metric_blocks = h->splits[0];
    ProfScope prof(h, "learn_catch_fused");
    hipLaunchKernelGGL(learn_catch_fused, dim3(h->splits[0]), dim3(CF_WG), lds, h->stream, a);
    return hipGetLastError();
}

hipError_t launch_learn_one_layer(anakin* h)
{
    const Layout& L = h->lay;
    const NetShape& n = h->net;
    OneLayerArgs a;
    a.M = h->B * h->T; a.D = n.dims[0]; a.H = n.dims[1]; a.NH = n.NH; a.NHP = n.NHP;
    a.rows = a.M / h->splits[0];
    a.theta = at<const float>(h, L.w_src); a.w1_off = n.w_off[0]; a.b1_off = n.b_off[0]; a.wh_off = n.wh_off;
    a.dhead = at<const float>(h, L.dhead);
    a.partial0 = at<float>(h, L.part[0]); a.partial1 = at<float>(h, L.part[1]);
    a.obs.env = h->env; a.obs.s0 = at<const uint32_t>(h, L.tr_s0);
    a.obs.f0 = at<const float>(h, L.tr_f0); a.obs.f1 = at<const float>(h, L.tr_f1);
    const size_t lds = ((size_t)a.D * a.H + (size_t)OLW * a.D) * sizeof(float);
    const dim3 grid(h->splits[0], (a.H + OLW - 1) / OLW);
    auto go = [&](auto kern) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) return e;
        ProfScope prof(h, "learn_one_layer");
        hipLaunchKernelGGL(kern, grid, dim3(OLW), lds, h->stream, a);
        return hipGetLastError();
    };
    const int cw = a.H < OLW ? a.H : OLW;
    const bool full = a.rows % (8 * (OLW / cw)) == 0;             // RB x groups samples per loop trip
    if (h->env.kind == ENV_CATCH) {
        if (full && a.H == 32) return go(learn_one_layer<ENV_CATCH, 4, true, 32>);
        return full ? go(learn_one_layer<ENV_CATCH, 4, true, 0>) : go(learn_one_layer<ENV_CATCH, 4, false, 0>);
    }
    return full ? go(learn_one_layer<ENV_PENDULUM, 3, true, 0>) : go(learn_one_layer<ENV_PENDULUM, 3, false, 0>);
}

// ---------------------------------------------------------------------------
// Adam with the gradient reduction fused in: g = sum over split-K partials in
// ascending split order, then m, v, theta.  Streams theta, m, v once in and
// once out (28 bytes per parameter besides the partials).  For bf16 networks
// the rounded copies the matrix-core kernels read are refreshed here too.
// ---------------------------------------------------------------------------
constexpr int ADAM_WAVES = 16;
typedef float f4v_a __attribute__((ext_vector_type(4)));
__device__ __forceinline__ int adam_region_of(const AdamArgs& a, int i)
{
    int r = 0;
#pragma unroll
    for (int k = 1; k < MAX_ADAM_REGIONS; ++k) if (k < a.n_regions && i >= a.reg[k].start) r = k;
    return r;
}
__global__ __launch_bounds__(ADAM_WAVES * 64) void adam_reduce(const AdamArgs a)
{
    // 256 consecutive parameters per workgroup, four per lane; each of the 16 wavefronts adds its share of the
    // split-K partials (splits w, w+16, w+32, ...) with 16-byte loads -- one KiB per wavefront and partial row --
    // then the 16 sums are combined in wave order.  A group of four that straddles two regions, or lies in a
    // region whose rows are not 16-byte aligned, is summed parameter by parameter.
    __shared__ f4v_a red[ADAM_WAVES][64];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int i = (blockIdx.x * 64 + lane) * 4;
    f4v_a g = {0.0f, 0.0f, 0.0f, 0.0f};
    if (i < a.P) {
        const int r = adam_region_of(a, i);
        const Region rg = a.reg[r];
        const int off = i - rg.start;
        if (i + 3 < a.P && off + 3 < rg.count && ((rg.count | off) & 3) == 0) {
            const float* p = rg.partial + off;
#pragma unroll 4
            for (int s = wave; s < rg.splits; s += ADAM_WAVES) g += *reinterpret_cast<const f4v_a*>(p + (size_t)s * rg.count);
        } else {
            // the four parameters side by side, so that their loads overlap as the 16-byte ones do
            const float* pe[4]; size_t cnt[4]; int sp[4], smax = 0;
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const int ie = i + e < a.P ? i + e : i;
                const Region re = a.reg[adam_region_of(a, ie)];
                pe[e] = re.partial + (ie - re.start); cnt[e] = (size_t)re.count;
                sp[e] = i + e < a.P ? re.splits : 0;
                smax = sp[e] > smax ? sp[e] : smax;
            }
#pragma unroll 4
            for (int s = wave; s < smax; s += ADAM_WAVES) {
#pragma unroll
                for (int e = 0; e < 4; ++e) g[e] += s < sp[e] ? pe[e][(size_t)s * cnt[e]] : 0.0f;
            }
        }
    }
    red[wave][lane] = g;
    __syncthreads();
    if (wave != 0 || i >= a.P) return;
    g = red[0][lane];
#pragma unroll
    for (int w = 1; w < ADAM_WAVES; ++w) g += red[w][lane];
    if (i + 3 < a.P) {
        const f4v_a mo = *reinterpret_cast<const f4v_a*>(a.m + i), vo = *reinterpret_cast<const f4v_a*>(a.v + i);
        const f4v_a to = *reinterpret_cast<const f4v_a*>(a.theta + i);
        f4v_a m, v, th;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            m[e] = a.beta1 * mo[e] + (1.0f - a.beta1) * g[e];
            v[e] = a.beta2 * vo[e] + (1.0f - a.beta2) * g[e] * g[e];
            const float mh = m[e] / a.bc1, vh = v[e] / a.bc2;
            th[e] = to[e] - a.lr * mh / (sqrtf(vh) + a.eps);
        }
        *reinterpret_cast<f4v_a*>(a.grad + i) = g;
        *reinterpret_cast<f4v_a*>(a.m + i) = m;
        *reinterpret_cast<f4v_a*>(a.v + i) = v;
        *reinterpret_cast<f4v_a*>(a.theta + i) = th;
        if (a.w_bf16) {
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const uint16_t hb = bf16_bits(th[e]);
                a.w_bf16[i + e] = hb;
                a.wt_bf16[transposed_index(a.net, i + e)] = hb;
            }
        }
        return;
    }
    for (int e = 0; e < 4 && i + e < a.P; ++e) {
        const float m = a.beta1 * a.m[i + e] + (1.0f - a.beta1) * g[e];
        const float v = a.beta2 * a.v[i + e] + (1.0f - a.beta2) * g[e] * g[e];
        const float mh = m / a.bc1, vh = v / a.bc2;
        const float th = a.theta[i + e] - a.lr * mh / (sqrtf(vh) + a.eps);
        a.grad[i + e] = g[e];
        a.m[i + e] = m;
        a.v[i + e] = v;
        a.theta[i + e] = th;
        if (a.w_bf16) {
            const uint16_t hb = bf16_bits(th);
            a.w_bf16[i + e] = hb;
            a.wt_bf16[transposed_index(a.net, i + e)] = hb;
        }
    }
}

// One parameter per lane, 64 per workgroup: four times the workgroups of adam_reduce, which is what small parameter
// vectors (under about 2^18) need to keep every compute unit loading.
__global__ __launch_bounds__(ADAM_WAVES * 64) void adam_reduce_narrow(const AdamArgs a)
{
    // 64 consecutive parameters per workgroup; each of the 16 wavefronts adds its share of the
    // split-K partials (splits w, w+16, w+32, ...), then the 16 sums are combined in wave order
    __shared__ float red[ADAM_WAVES][64];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int i = blockIdx.x * 64 + lane;
    const bool ok = i < a.P;
    float g = 0.0f;
    if (ok) {
        int r = 0;
#pragma unroll
        for (int k = 1; k < MAX_ADAM_REGIONS; ++k) if (k < a.n_regions && i >= a.reg[k].start) r = k;
        const Region rg = a.reg[r];
        const float* p = rg.partial + (i - rg.start);
#pragma unroll 4
        for (int s = wave; s < rg.splits; s += ADAM_WAVES) g += p[(size_t)s * rg.count];
    }
    red[wave][lane] = g;
    __syncthreads();
    if (wave != 0 || !ok) return;
    g = red[0][lane];
#pragma unroll
    for (int w = 1; w < ADAM_WAVES; ++w) g += red[w][lane];
    const float m = a.beta1 * a.m[i] + (1.0f - a.beta1) * g;
    const float v = a.beta2 * a.v[i] + (1.0f - a.beta2) * g * g;
    const float mh = m / a.bc1, vh = v / a.bc2;
    const float th = a.theta[i] - a.lr * mh / (sqrtf(vh) + a.eps);
    a.grad[i] = g;
    a.m[i] = m;
    a.v[i] = v;
    a.theta[i] = th;
    if (a.w_bf16) {
        const uint16_t hb = bf16_bits(th);
        a.w_bf16[i] = hb;
        a.wt_bf16[transposed_index(a.net, i)] = hb;
    }
}

// The same update for parameter regions with few partials (at most 16): one lane per parameter adds its
// partials in ascending order itself, so a wavefront streams 64 consecutive parameters of every array --
// the shape that reaches the HBM roofline when P is large.
__global__ __launch_bounds__(WG) void adam_reduce_flat(const AdamArgs a)
{
    constexpr int UF = 4;                                        // parameters per lane, WG apart: loads of all four in flight
    const int i0 = blockIdx.x * (WG * UF) + threadIdx.x;
    float g[UF], mo[UF], vo[UF], to[UF];
#pragma unroll
    for (int u = 0; u < UF; ++u) {
        const int i = i0 + u * WG;
        g[u] = 0.0f; mo[u] = 0.0f; vo[u] = 0.0f; to[u] = 0.0f;
        if (i < a.P) {
            int r = 0;
#pragma unroll
            for (int k = 1; k < MAX_ADAM_REGIONS; ++k) if (k < a.n_regions && i >= a.reg[k].start) r = k;
            const Region rg = a.reg[r];
            const float* p = rg.partial + (i - rg.start);
            for (int s2 = 0; s2 < rg.splits; ++s2) g[u] += p[(size_t)s2 * rg.count];
            mo[u] = a.m[i]; vo[u] = a.v[i]; to[u] = a.theta[i];
        }
    }
#pragma unroll
    for (int u = 0; u < UF; ++u) {
        const int i = i0 + u * WG;
        if (i >= a.P) continue;
        const float m = a.beta1 * mo[u] + (1.0f - a.beta1) * g[u];
        const float v = a.beta2 * vo[u] + (1.0f - a.beta2) * g[u] * g[u];
        const float mh = m / a.bc1, vh = v / a.bc2;
        const float th = to[u] - a.lr * mh / (sqrtf(vh) + a.eps);
        a.grad[i] = g[u];
        a.m[i] = m;
        a.v[i] = v;
        a.theta[i] = th;
        if (a.w_bf16) {
            const uint16_t hb = bf16_bits(th);
            a.w_bf16[i] = hb;
            a.wt_bf16[transposed_index(a.net, i)] = hb;
        }
    }
}

static void launch_adam_kernel(const AdamArgs& a, hipStream_t s)
{
    int max_splits = 0;
    for (int r = 0; r < a.n_regions; ++r) max_splits = a.reg[r].splits > max_splits ? a.reg[r].splits : max_splits;
    if (max_splits <= 16) hipLaunchKernelGGL(adam_reduce_flat, dim3((a.P + 4 * WG - 1) / (4 * WG)), dim3(WG), 0, s, a);
    else if (a.P >= (1 << 18)) hipLaunchKernelGGL(adam_reduce, dim3((a.P + 255) / 256), dim3(ADAM_WAVES * 64), 0, s, a);
    else hipLaunchKernelGGL(adam_reduce_narrow, dim3((a.P + 63) / 64), dim3(ADAM_WAVES * 64), 0, s, a);
}

// ---------------------------------------------------------------------------
// launchers
// ---------------------------------------------------------------------------
hipError_t launch_returns(anakin* h)
{
    const Layout& L = h->lay;
    ProfScope prof(h, "returns_scan");
    hipLaunchKernelGGL(returns_scan, dim3((h->B + WG - 1) / WG), dim3(WG), 0, h->stream, h->B, h->T,
                       at<const float>(h, L.tr_rew), at<const uint8_t>(h, L.tr_done), at<const float>(h, L.tr_val),
                       h->net_cfg.gamma, h->net_cfg.lambda_, at<float>(h, L.adv), at<float>(h, L.ret));
    return hipGetLastError();
}

hipError_t launch_vtrace(anakin* h)
{
    const Layout& L = h->lay;
    VtraceArgs a;
    a.B = h->B; a.T = h->T; a.A = h->net.A; a.NH = h->net.NH; a.NHP = h->net.NHP; a.policy = h->net.policy;
    a.head_old = at<const float>(h, L.tr_head); a.head_new = at<const float>(h, L.head_new); a.val_new = at<const float>(h, L.val_new);
    a.act = at<const uint8_t>(h, L.tr_act); a.eps_old = at<const float>(h, L.tr_eps);
    a.rew = at<const float>(h, L.tr_rew); a.done = at<const uint8_t>(h, L.tr_done);
    a.gamma = h->net_cfg.gamma; a.lambda = h->net_cfg.lambda_;
    a.adv = at<float>(h, L.adv); a.ret = at<float>(h, L.ret); a.eps_new = at<float>(h, L.eps_new);
    {
        ProfScope prof(h, "vtrace_ratio");
        hipLaunchKernelGGL(vtrace_ratio, dim3((unsigned)(((size_t)h->B * h->T + WG - 1) / WG)), dim3(WG), 0, h->stream, a);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    ProfScope prof(h, "vtrace_scan");
    hipLaunchKernelGGL(vtrace_scan, dim3((h->B + WG - 1) / WG), dim3(WG), 0, h->stream, a);
    return hipGetLastError();
}

// Gaussian policy, forward pass repeated with newer parameters: the noise that reproduces the stored pre-squash
// sample under the new head outputs, eps_new = (z - mu_new) / sigma_new (what the score function is taken at)
hipError_t launch_eps_now(anakin* h)
{
    const Layout& L = h->lay;
    if (h->net.policy == POLICY_CATEGORICAL) return hipSuccess;
    VtraceArgs a;
    a.B = h->B; a.T = h->T; a.A = h->net.A; a.NH = h->net.NH; a.NHP = h->net.NHP; a.policy = h->net.policy;
    a.head_old = at<const float>(h, L.tr_head); a.head_new = at<const float>(h, L.head_new); a.val_new = nullptr;
    a.act = at<const uint8_t>(h, L.tr_act); a.eps_old = at<const float>(h, L.tr_eps);
    a.rew = nullptr; a.done = nullptr; a.gamma = 0.0f; a.lambda = 0.0f;
    a.adv = nullptr; a.ret = nullptr; a.eps_new = at<float>(h, L.eps_new);
    ProfScope prof(h, "eps_now");
    hipLaunchKernelGGL(vtrace_ratio, dim3((unsigned)(((size_t)h->B * h->T + WG - 1) / WG)), dim3(WG), 0, h->stream, a);
    return hipGetLastError();
}

hipError_t launch_head_grad(anakin* h)
{
    const Layout& L = h->lay;
    HeadGradArgs a;
    a.M = h->B * h->T; a.A = h->net.A; a.NH = h->net.NH; a.NHP = h->net.NHP; a.policy = h->net.policy;
    a.head = at<const float>(h, L.tr_head); a.act = at<const uint8_t>(h, L.tr_act); a.eps = at<const float>(h, L.tr_eps);
    a.adv = at<const float>(h, L.adv); a.ret = at<const float>(h, L.ret);
    a.rew = at<const float>(h, L.tr_rew); a.done = at<const uint8_t>(h, L.tr_done);
    a.dhead = at<float>(h, L.dhead); a.loss_part = at<float>(h, L.loss_part);
    a.beta = h->net_cfg.entropy_coef; a.cv = h->net_cfg.value_coef; a.inv_m = (float)(1.0 / (double)a.M);
    a.path = h->pathwise ? at<const float>(h, L.path) : nullptr;
    h->metric_blocks = h->loss_blocks;
    ProfScope prof(h, "head_grad");
    hipLaunchKernelGGL(head_grad, dim3(h->loss_blocks), dim3(WG), 0, h->stream, a);
    return hipGetLastError();
}

// whether returns and loss go out as one launch: the plain update of a whole unroll, and room for one block of loss
// sums per workgroup
// 16 envs per workgroup unless that leaves the second pass over the samples mostly empty (256 < 16 T < 512)
static int scan_loss_envs(const anakin* h) { return (h->T * 16 <= WG || h->T * 16 >= 2 * WG) ? 16 : 8; }
bool scan_loss_ok(const anakin* h)
{
    const int E = scan_loss_envs(h);
    return h->n_updates == 1 && !h->pathwise && !h->traj_decoupled && h->B % E == 0 && h->T * E <= SL_MAXN &&
           h->B / E <= h->loss_blocks;
}

hipError_t launch_scan_loss(anakin* h)
{
    const Layout& L = h->lay;
    ScanLossArgs s;
    HeadGradArgs& a = s.g;
    a.M = h->B * h->T; a.A = h->net.A; a.NH = h->net.NH; a.NHP = h->net.NHP; a.policy = h->net.policy;
    a.head = at<const float>(h, L.tr_head); a.act = at<const uint8_t>(h, L.tr_act); a.eps = at<const float>(h, L.tr_eps);
    a.adv = nullptr; a.ret = nullptr;
    a.rew = at<const float>(h, L.tr_rew); a.done = at<const uint8_t>(h, L.tr_done);
    a.dhead = at<float>(h, L.dhead); a.loss_part = at<float>(h, L.loss_part);
    a.beta = h->net_cfg.entropy_coef; a.cv = h->net_cfg.value_coef; a.inv_m = (float)(1.0 / (double)a.M);
    a.path = nullptr;
    s.B = h->B; s.T = h->T; s.E = scan_loss_envs(h); s.val = at<const float>(h, L.tr_val);
    s.gamma = h->net_cfg.gamma; s.lambda = h->net_cfg.lambda_;
    s.adv_out = at<float>(h, L.adv); s.ret_out = at<float>(h, L.ret);
    h->metric_blocks = h->B / s.E;
    ProfScope prof(h, "scan_loss");
    hipLaunchKernelGGL(scan_loss, dim3(h->B / s.E), dim3(WG), 0, h->stream, s);
    return hipGetLastError();
}

hipError_t launch_partial_reduce(const float* src, float* dst, int count, int fan, int splits, hipStream_t s)
{
    hipLaunchKernelGGL(partial_reduce, dim3((count + WG - 1) / WG, splits), dim3(WG), 0, s, src, dst, count, fan);
    return hipGetLastError();
}

hipError_t launch_head_backward(anakin* h)
{
    const Layout& L = h->lay;
    const NetShape& n = h->net;
    HeadBwdArgs a;
    a.M = h->B * h->T; a.H = n.dims[n.L]; a.NH = n.NH; a.NHP = n.NHP;
    const int splits = h->splits[n.L], fan = h->head_fan;
    const int stage1 = splits * fan;                        // workgroups of the streaming pass
    a.rows = a.M / stage1;
    a.h = at<const float>(h, L.act[n.L - 1]); a.dhead = at<const float>(h, L.dhead);
    a.wh = at<const float>(h, L.w_src) + n.wh_off;
    a.dz = at<float>(h, L.dz[n.L - 1]);
    a.partial = fan > 1 ? at<float>(h, L.head_stage) : at<float>(h, L.part[n.L]);
    a.bf16 = n.bf16;
    const int groups = WG / (a.H >> 2);
    const int stride = a.H * a.NH + a.NH;
    const size_t lds = (size_t)groups * stride * sizeof(float);
    {
        ProfScope prof(h, "head_backward");
        if (a.H % 64 == 0 && a.rows % 32 == 0 && !(h->mode & ANAKIN_MODE_VALU_GEMM))
            hipLaunchKernelGGL(head_backward_mfma, dim3(stage1, (a.H + 255) / 256), dim3(WG), 0, h->stream, a);
        else
            hipLaunchKernelGGL(head_backward, dim3(stage1), dim3(WG), lds, h->stream, a);
    }
    hipError_t e = hipGetLastError();
    if (e != hipSuccess || fan == 1) return e;
    ProfScope prof(h, "partial_reduce");
    hipLaunchKernelGGL(partial_reduce, dim3((stride + WG - 1) / WG, splits), dim3(WG), 0, h->stream,
                       at<const float>(h, L.head_stage), at<float>(h, L.part[n.L]), stride, fan);
    return hipGetLastError();
}

hipError_t launch_adam(anakin* h)
{
    const Layout& L = h->lay;
    const NetShape& n = h->net;
    AdamArgs a;
    a.P = n.P;
    int r = 0;
    for (int l = 0; l < n.L; ++l) {
        if (l == 0 && first_layer_split(h)) {
            // wall rows, agent rows, goal rows (zero but the last, which equals the bias gradient), bias
            const int H1 = n.dims[1], plane = h->env.rows * h->env.cols * H1;
            const float* pw = at<const float>(h, L.part[0]);
            const float* pa = pw + (size_t)plane * h->splits_w;
            const float* pg = pa + (size_t)plane * h->splits[0];
            a.reg[r++] = Region{n.w_off[0], plane, h->splits_w, pw};
            a.reg[r++] = Region{n.w_off[0] + plane, plane, h->splits[0], pa};
            a.reg[r++] = Region{n.w_off[0] + 2 * plane, plane - H1, 0, nullptr};
            a.reg[r++] = Region{n.w_off[0] + 3 * plane - H1, H1, h->splits_w, pg};
            a.reg[r++] = Region{n.b_off[0], H1, h->splits_w, pg};
            continue;
        }
        a.reg[r++] = Region{n.w_off[l], n.dims[l] * n.dims[l + 1] + n.dims[l + 1], h->splits[l], at<const float>(h, L.part[l])};
    }
    a.reg[r++] = Region{n.wh_off, n.dims[n.L] * n.NH + n.NH, h->splits[n.L], at<const float>(h, L.part[n.L])};
    a.n_regions = r;
    for (; r < MAX_ADAM_REGIONS; ++r) a.reg[r] = Region{0x7fffffff, 0, 0, nullptr};
    a.theta = at<float>(h, L.theta); a.grad = at<float>(h, L.grad); a.m = at<float>(h, L.m); a.v = at<float>(h, L.v);
    a.w_bf16 = n.bf16 ? at<uint16_t>(h, L.w_bf16) : nullptr;
    a.wt_bf16 = n.bf16 ? at<uint16_t>(h, L.wt_bf16) : nullptr;
    a.net = n;
    h->adam_t += 1;
    a.lr = h->net_cfg.lr; a.beta1 = h->net_cfg.beta1; a.beta2 = h->net_cfg.beta2; a.eps = h->net_cfg.eps;
    a.bc1 = (float)(1.0 - pow((double)h->net_cfg.beta1, (double)h->adam_t));
    a.bc2 = (float)(1.0 - pow((double)h->net_cfg.beta2, (double)h->adam_t));
    ProfScope prof(h, "adam_reduce");
    launch_adam_kernel(a, h->stream);
    return hipGetLastError();
}

// Adam on a synthetic parameter vector (measurement only): one region, one partial, P parameters laid out
// as theta | grad | m | v | partial in `base`.  Shows the kernel against the HBM roofline at a size that
// does not fit any cache; inside the real workloads P is small and the launch is latency bound.
hipError_t launch_adam_probe(float* base, int P, hipStream_t s)
{
    AdamArgs a;
    a.P = P; a.n_regions = 1;
    a.reg[0] = Region{0, P, 1, base + (size_t)4 * P};
    for (int r = 1; r < MAX_ADAM_REGIONS; ++r) a.reg[r] = Region{0x7fffffff, 0, 0, nullptr};
    a.theta = base; a.grad = base + (size_t)P; a.m = base + (size_t)2 * P; a.v = base + (size_t)3 * P;
    a.w_bf16 = nullptr; a.wt_bf16 = nullptr;
    a.net = NetShape{};
    a.lr = 3e-4f; a.beta1 = 0.9f; a.beta2 = 0.999f; a.eps = 1e-8f; a.bc1 = 0.1f; a.bc2 = 0.001f;
    launch_adam_kernel(a, s);
    return hipGetLastError();
}

}  // namespace ank
