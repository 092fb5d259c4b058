// The whole update of a small Catch agent in ONE launch (paper section 3.1: the unit of T interactions and one
// parameter update is a single device program; for a net and an unroll this small the seven kernels of the
// general update do a few microseconds of work each and the step is bound by their launches).
//
// Shape: Catch, fp32, two hidden layers of 64 units, three actions + value; at most 16 workgroups, each owning
// E envs for all T steps (R = E T <= 112 samples).  Nothing depends on another workgroup's samples until the
// gradient is summed, so every workgroup runs the whole chain on its own rows:
//   scan       returns and advantages of its envs (returns_scan's recursion)
//   loss       loss terms and head gradients of its samples (head_grad's arithmetic)
//   dZ2, dWh   from the stored h2 and the head matrix
//   dZ1        = relu'(h1) (dZ2 W2^T), W2 rows in registers, dZ2 rows broadcast from LDS
//   dW2, db2   = h1^T dZ2
//   dW1, db1   scatter of dZ1 into the two board rows of every sample
// and writes one partial gradient.  The workgroup that arrives last at an integer counter (ordinary vector
// atomic; device-scope fences around it) adds the partials in ascending workgroup order -- so the bytes do not
// depend on which one it was -- and applies Adam.
#include "internal.h"
#include "loss.h"

namespace ank {

constexpr int SF_WG = 256;
constexpr int SF_H = 64;
constexpr int SF_MAX_WG = 16;
constexpr int SF_MAX_R = 112;

struct SmallFusedArgs {
    int B, T, D, E, n_wg, P;
    EnvDims env;
    NetShape net;
    const float* w;            // parameters the unroll was acted with
    const uint32_t* s0; const uint8_t* act; const float* rew; const uint8_t* done; const float* val; const float* head;
    const float* h1; const float* h2;       // [B*T][64] stored activations
    float* adv; float* ret;
    float* part;               // [n_wg][P]
    float* loss_part;          // [n_wg][8]
    unsigned* counter;         // [0] arrivals, [1] departures: both zero between launches
    int max_spin;              // bound on the polls of the rendezvous
    float* theta; float* grad; float* m; float* v;
    float gamma, lambda, beta, cv, inv_m;
    float lr, beta1, beta2, eps, bc1, bc2;
};

typedef float f16v_s __attribute__((ext_vector_type(16)));
typedef float f4_s __attribute__((ext_vector_type(4)));

// sum over the 64 lanes of a wavefront, same value in every lane, fixed order
__device__ __forceinline__ float wave_sum(float v)
{
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, 64);
    return v;
}

__global__ __launch_bounds__(SF_WG) void learn_small_fused(const SmallFusedArgs a)
{
    extern __shared__ float lds[];
    constexpr int H = SF_H, LD = H + 1;                  // row stride 65: a column walk touches every bank once
    const int B = a.B, T = a.T, D = a.D, E = a.E, R = E * T, Rp4 = (R + 3) & ~3, Rpad = (R + 31) & ~31;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, l32 = lane & 31, kg = lane >> 5;
    const int b0 = blockIdx.x * E;
    float* W2s = lds;                                    // [64][LD]
    float* dhk = W2s + H * LD;                           // [4][Rp4] head gradients, one array per head output (4-byte broadcast reads)
    float* advs = dhk + 4 * Rp4;                         // [Rp4]
    float* rets = advs + Rp4;                            // [Rp4]
    float* rews = rets + Rp4;                            // [Rp4] rewards, then (scan) discounts
    float* vals = rews + Rp4;                            // [Rp4 + E rounded up to 4] values of the T + 1 rows
    const int Ep4 = (E + 3) & ~3;
    uint32_t* cells = reinterpret_cast<uint32_t*>(vals + Rp4 + Ep4);   // [Rp4] row offsets of the two board cells
    float* dz1s = reinterpret_cast<float*>(cells + Rp4); // [Rpad][LD]
    float* red = dz1s + Rpad * LD;                       // [4 waves][16] + [256] db1 partials
    float* dwr = red + 64 + SF_WG;                       // [4 groups][64][5] head-matrix and db2 sums of the row groups
    float* un = dwr + 4 * H * 5;                         // dz2s [Rpad][LD], h1s [Rpad][LD]
    float* dz2s = un;
    float* h1s = un + Rpad * LD;
    const NetShape& n = a.net;
    auto sample = [&](int r) { return (size_t)(r / E) * B + b0 + (r % E); };
    const int j = tid & 63, g = tid >> 6;

    // ---- everything this workgroup reads from memory is requested here, before anything is computed: the phases
    //      below then depend on LDS and registers only, not on one round trip to memory after another ----
    float w2v[H * H / SF_WG];
#pragma unroll
    for (int q = 0; q < H * H / SF_WG; ++q) w2v[q] = a.w[n.w_off[1] + q * SF_WG + tid];
    float wh[4];
#pragma unroll
    for (int k = 0; k < 4; ++k) wh[k] = a.w[n.wh_off + j * 4 + k];
    // per-sample records: lane r < R (R <= 112 < 256)
    float4 hv4 = make_float4(0, 0, 0, 0);
    int my_act = 0; uint32_t my_s0 = 0u; float my_rew = 0.0f, my_val = 0.0f, boot = 0.0f; bool my_done = false;
    if (tid < R) {
        const size_t i = sample(tid);
        hv4 = *reinterpret_cast<const float4*>(a.head + i * 4);
        my_act = (int)a.act[i]; my_s0 = a.s0[i]; my_rew = a.rew[i]; my_done = a.done[i] != 0; my_val = a.val[i];
    }
    if (tid < E) boot = a.val[(size_t)T * B + b0 + tid];
    // stored activations of the workgroup's rows: h1 as it is, h2 parked where dZ2 will go; rows from R up to the next
    // multiple of 32 are zero (they are reduction steps of the dW2 product)
    constexpr int NB = (SF_MAX_R + 31) / 32 * 8;             // rows of one lane at most: 32
    float h2v[NB], h1v[NB];
#pragma unroll
    for (int u = 0; u < NB; ++u) {
        const int r = g + 4 * u;
        const bool ok = r < R;
        const size_t i = ok ? sample(r) : 0;
        h2v[u] = ok ? a.h2[i * H + j] : 0.0f;
        h1v[u] = ok ? a.h1[i * H + j] : 0.0f;
    }
    // ... and only now the first use of any of them
#pragma unroll
    for (int q = 0; q < H * H / SF_WG; ++q) { const int i = q * SF_WG + tid; W2s[(i >> 6) * LD + (i & 63)] = w2v[q]; }
    if (tid < R) {
        rews[tid] = my_rew;
        vals[tid] = my_val;
        advs[tid] = my_done ? 0.0f : a.gamma;                // discount of the step, for the scan
    }
    if (tid < E) vals[R + tid] = boot;
#pragma unroll
    for (int u = 0; u < NB; ++u) {
        const int r = g + 4 * u;
        if (r < Rpad) { h1s[r * LD + j] = h1v[u]; dz2s[r * LD + j] = h2v[u]; }
    }
    __syncthreads();
    // ---- scan: one lane per env, all operands in LDS (advs holds the discounts until it is overwritten) ----
    if (tid < E) {
        const float oml = 1.0f - a.lambda;
        float G = vals[R + tid], vnext = G;
        for (int t = T - 1; t >= 0; --t) {
            const int r = t * E + tid;
            const float v = vals[r];
            const float mix = fmaf(a.lambda, G, oml * vnext);
            G = fmaf(advs[r], mix, rews[r]);
            rets[r] = G; advs[r] = G - v;
            vnext = v;
        }
    }
    __syncthreads();
    // ---- loss terms and head gradients: lane r < R ----
    float sums[5] = {0, 0, 0, 0, 0}, dbh[4] = {0, 0, 0, 0};
    if (tid < R) {
        const size_t i = sample(tid);
        a.ret[i] = rets[tid]; a.adv[i] = advs[tid];
        float d[4], lp_term, v_term, e_term;
        catch_head_grad(hv4, my_act, advs[tid], rets[tid], a.beta, a.cv, a.inv_m, d, lp_term, v_term, e_term);
        sums[0] = lp_term; sums[1] = v_term; sums[2] = e_term; sums[3] = my_rew; sums[4] = my_done ? 1.0f : 0.0f;
#pragma unroll
        for (int k = 0; k < 4; ++k) { dbh[k] = d[k]; dhk[k * Rp4 + tid] = d[k]; }
        int bc, pc;
        catch_obs_cells(a.env, my_s0, bc, pc);
        cells[tid] = (uint32_t)(bc * H) | ((uint32_t)(pc * H) << 16);
    }
    __syncthreads();
    // ---- dZ2 (in place of the parked h2) and the head-matrix sums.  Lane (unit j, group g) takes rows g, g + 4, ... ----
    float dwh[4] = {0, 0, 0, 0}, db2 = 0.0f;
    for (int r = g; r < R; r += 4) {
        const float h2r = dz2s[r * LD + j];
        float s = 0.0f;
#pragma unroll
        for (int k = 0; k < 4; ++k) { const float dk = dhk[k * Rp4 + r]; s = fmaf(wh[k], dk, s); dwh[k] = fmaf(h2r, dk, dwh[k]); }
        const float dz = h2r > 0.0f ? s : 0.0f;
        dz2s[r * LD + j] = dz;
        db2 += dz;
    }
    __syncthreads();
    float* out = a.part + (size_t)blockIdx.x * a.P;
    // ---- dZ1 = relu'(h1) (dZ2 W2^T) on the matrix cores (v_mfma_f32_32x32x2_f32: lane (l32, kg) feeds A[row l32][k kg]
    //      and B[k kg][col l32], accumulator register r is D[row 8 (r/4) + 4 kg + r%4][col l32]).  Wavefront w takes the
    //      32 columns 32 (w & 1) .. and the row tiles w >> 1, (w >> 1) + 2; its 32 x 64 block of W2 stays in registers ----
    float db1 = 0.0f;
    {
        const int ct = wave & 1, col = 32 * ct + l32;
        float w2k[H / 2];
#pragma unroll
        for (int q = 0; q < H / 2; ++q) w2k[q] = W2s[col * LD + 2 * q + kg];          // B[k = 2q + kg][col] = W2[col][k]
        for (int rt = wave >> 1; rt * 32 < Rpad; rt += 2) {
            // two accumulators: consecutive matrix instructions do not wait for each other
            f16v_s acc, acc_b;
#pragma unroll
            for (int r = 0; r < 16; ++r) { acc[r] = 0.0f; acc_b[r] = 0.0f; }
            const float* arow = dz2s + (32 * rt + l32) * LD + kg;
#pragma unroll
            for (int q = 0; q < H / 2; q += 2) {
                acc = __builtin_amdgcn_mfma_f32_32x32x2f32(arow[2 * q], w2k[q], acc, 0, 0, 0);
                acc_b = __builtin_amdgcn_mfma_f32_32x32x2f32(arow[2 * q + 2], w2k[q + 1], acc_b, 0, 0, 0);
            }
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[r] += acc_b[r];
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int row = 32 * rt + 8 * (r >> 2) + 4 * kg + (r & 3);
                if (row < R) {
                    const float dz = h1s[row * LD + col] > 0.0f ? acc[r] : 0.0f;
                    dz1s[row * LD + col] = dz;
                    db1 += dz;
                }
            }
        }
    }
    // ---- dW2 = h1^T dZ2: wavefront w owns the 32 x 32 tile (rows i = 32 (w >> 1) .., columns j = 32 (w & 1) ..), the
    //      reduction runs over the rows of the workgroup two at a time (Rpad is a multiple of 32); db2 by the first 64 lanes ----
    {
        const int it = wave >> 1, jt = wave & 1;
        f16v_s acc, acc_b;
#pragma unroll
        for (int r = 0; r < 16; ++r) { acc[r] = 0.0f; acc_b[r] = 0.0f; }
        const float* ap = h1s + kg * LD + 32 * it + l32;
        const float* bp = dz2s + kg * LD + 32 * jt + l32;
        for (int q0 = 0; q0 < Rpad / 2; q0 += 8) {
            float av[8], bv[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) { av[u] = ap[2 * (q0 + u) * LD]; bv[u] = bp[2 * (q0 + u) * LD]; }
#pragma unroll
            for (int u = 0; u < 8; u += 2) {
                acc = __builtin_amdgcn_mfma_f32_32x32x2f32(av[u], bv[u], acc, 0, 0, 0);
                acc_b = __builtin_amdgcn_mfma_f32_32x32x2f32(av[u + 1], bv[u + 1], acc_b, 0, 0, 0);
            }
        }
#pragma unroll
        for (int r = 0; r < 16; ++r)
            out[n.w_off[1] + (32 * it + 8 * (r >> 2) + 4 * kg + (r & 3)) * H + 32 * jt + l32] = acc[r] + acc_b[r];
    }
    // sums over the lanes of every wavefront (butterfly, fixed order), one row of `red` per wavefront
    {
        float q9[9] = {dbh[0], dbh[1], dbh[2], dbh[3], sums[0], sums[1], sums[2], sums[3], sums[4]};
#pragma unroll
        for (int k = 0; k < 9; ++k) q9[k] = wave_sum(q9[k]);
        if (lane < 9) {
            float v = q9[0];
#pragma unroll
            for (int k = 1; k < 9; ++k) if (lane == k) v = q9[k];
            red[wave * 16 + lane] = v;
        }
        red[64 + tid] = db1;
    }
#pragma unroll
    for (int k = 0; k < 4; ++k) dwr[(g * H + j) * 4 + k] = dwh[k];
    dwr[4 * H * 4 + g * H + j] = db2;
    __syncthreads();                                     // dz1s, red and dwr are complete
    // ---- dW1 = X^T dZ1 with X the 0/1 board (two ones per row), on the matrix cores: wavefront w owns board cells
    //      32 (w >> 1) .. (the board has at most 64 here) and columns 32 (w & 1) ..; a product with a one is exact ----
    {
        const int ctile = wave >> 1, jt = wave & 1;
        const uint32_t mycell = (uint32_t)((32 * ctile + l32) * H);           // LDS-offset form, as stored in cells[]
        f16v_s acc, acc_b;
#pragma unroll
        for (int r = 0; r < 16; ++r) { acc[r] = 0.0f; acc_b[r] = 0.0f; }
        const float* bp = dz1s + kg * LD + 32 * jt + l32;
        for (int q0 = 0; q0 < Rpad / 2; q0 += 8) {
            float av[8], bv[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                const int r = 2 * (q0 + u) + kg;
                const uint32_t cc = r < R ? cells[r] : 0xffffffffu;
                av[u] = ((cc & 0xffffu) == mycell || (cc >> 16) == mycell) ? 1.0f : 0.0f;
                bv[u] = r < R ? bp[2 * (q0 + u) * LD] : 0.0f;
            }
#pragma unroll
            for (int u = 0; u < 8; u += 2) {
                acc = __builtin_amdgcn_mfma_f32_32x32x2f32(av[u], bv[u], acc, 0, 0, 0);
                acc_b = __builtin_amdgcn_mfma_f32_32x32x2f32(av[u + 1], bv[u + 1], acc_b, 0, 0, 0);
            }
        }
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const int c = 32 * ctile + 8 * (r >> 2) + 4 * kg + (r & 3);
            if (c < D) out[n.w_off[0] + c * H + 32 * jt + l32] = acc[r] + acc_b[r];
        }
    }
    {
        // Wh: 256 entries, one per lane: entry (unit tid / 4, head tid % 4), groups ascending
        float s = 0.0f;
#pragma unroll
        for (int gg = 0; gg < 4; ++gg) s += dwr[gg * H * 4 + tid];
        out[n.wh_off + tid] = s;
    }
    if (tid >= 128 && tid < 128 + H) {
        const int c = tid - 128;
        out[n.b_off[1] + c] = ((dwr[4 * H * 4 + c] + dwr[4 * H * 4 + H + c]) + dwr[4 * H * 4 + 2 * H + c]) + dwr[4 * H * 4 + 3 * H + c];
    }
    if (tid < H) {
        // db1 of column tid: the lanes (wavefront ct or ct + 2, either half, l32) of its column tile, in that order
        float sb = 0.0f;
        for (int ww = tid >> 5; ww < 4; ww += 2)
            for (int hh = 0; hh < 2; ++hh) sb += red[64 + ww * 64 + hh * 32 + (tid & 31)];
        out[n.b_off[0] + tid] = sb;
    }
    if (tid >= 64 && tid < 73) {
        const int q = tid - 64;
        const float s = ((red[q] + red[16 + q]) + red[32 + q]) + red[48 + q];
        if (q < 4) out[n.bh_off + q] = s;
        else a.loss_part[(size_t)blockIdx.x * 8 + (q - 4)] = s;
    }
    if (tid >= 73 && tid < 76) a.loss_part[(size_t)blockIdx.x * 8 + tid - 68] = 0.0f;
    // ---- rendezvous.  Every workgroup publishes its partial device-wide, takes a ticket, and waits until all
    //      n_wg tickets are out (all workgroups are resident: there are at most 16, one per compute unit).  The wait
    //      is bounded; a workgroup that gives up marks the metrics not-finite and leaves the parameters alone. ----
    __shared__ int go;
    __threadfence();
    __syncthreads();
    if (tid == 0) {
        atomicAdd(a.counter, 1u);
        int ok = 0;
        for (int spin = 0; spin < a.max_spin; ++spin) {
            if (__hip_atomic_load(a.counter, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) >= (unsigned)a.n_wg) { ok = 1; break; }
            __builtin_amdgcn_s_sleep(4);
        }
        go = ok;
    }
    __syncthreads();
    if (go) {
        __threadfence();                                 // the other workgroups' partials, published before their tickets
        // ---- Adam on this workgroup's slice of the parameters: partials added in ascending workgroup order ----
        const int per = (((a.P + a.n_wg - 1) / a.n_wg) + 3) & ~3;
        const int p = blockIdx.x * per + tid * 4;
        if (tid * 4 < per && p < a.P) {                  // P % 4 == 0: whole groups of four
            f4_s pw[SF_MAX_WG];
#pragma unroll
            for (int w = 0; w < SF_MAX_WG; ++w)
                pw[w] = w < a.n_wg ? *reinterpret_cast<const f4_s*>(a.part + (size_t)w * a.P + p) : f4_s{0.0f, 0.0f, 0.0f, 0.0f};
            const f4_s mo = *reinterpret_cast<const f4_s*>(a.m + p), vo = *reinterpret_cast<const f4_s*>(a.v + p);
            const f4_s to = *reinterpret_cast<const f4_s*>(a.theta + p);
            f4_s gs = {0.0f, 0.0f, 0.0f, 0.0f}, mn, vn, tn;
#pragma unroll
            for (int w = 0; w < SF_MAX_WG; ++w) gs += pw[w];         // absent workgroups add zero
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                const float m = a.beta1 * mo[c] + (1.0f - a.beta1) * gs[c];
                const float v = a.beta2 * vo[c] + (1.0f - a.beta2) * gs[c] * gs[c];
                const float mh = m / a.bc1, vh = v / a.bc2;
                mn[c] = m; vn[c] = v; tn[c] = to[c] - a.lr * mh / (sqrtf(vh) + a.eps);
            }
            *reinterpret_cast<f4_s*>(a.grad + p) = gs;
            *reinterpret_cast<f4_s*>(a.m + p) = mn;
            *reinterpret_cast<f4_s*>(a.v + p) = vn;
            *reinterpret_cast<f4_s*>(a.theta + p) = tn;
        }
    } else if (tid == 0) {
        a.loss_part[(size_t)blockIdx.x * 8] = __builtin_nanf("");
    }
    // ---- departure: the last workgroup to leave puts both counters back to zero for the next launch ----
    __syncthreads();
    if (tid == 0) {
        const unsigned d = atomicAdd(a.counter + 1, 1u);
        if (d == (unsigned)a.n_wg - 1u) { a.counter[1] = 0u; a.counter[0] = 0u; }
    }
}

// envs per workgroup for the single-launch update, 0 when the shape does not qualify
int small_fused_envs(const EnvDims& ed, const NetShape& ns, int B, int T)
{
    if (ed.kind != ENV_CATCH || ns.bf16 || ns.L != 2 || ns.dims[1] != SF_H || ns.dims[2] != SF_H || ns.NH != 4) return 0;
    if (ns.dims[0] > 64) return 0;                       // the board's cells are two 32-row tiles of the dW1 product
    for (int E = (B + SF_MAX_WG - 1) / SF_MAX_WG; E <= B && E * T <= SF_MAX_R; ++E)
        if (B % E == 0) return E;
    return 0;
}

size_t small_fused_part_bytes(const EnvDims& ed, const NetShape& ns, int B, int T)
{
    const int E = small_fused_envs(ed, ns, B, T);
    return E ? (size_t)(B / E) * ns.P * sizeof(float) : 0;
}

bool small_fused_ok(const anakin* h)
{
    return small_fused_envs(h->env, h->net, h->B, h->T) > 0 && h->mode == 0 && h->n_updates == 1 && !h->traj_decoupled &&
           !h->pathwise && !h->traj_packed && !h->traj_no_acts;
}

hipError_t launch_learn_small_fused(anakin* h)
{
    const Layout& L = h->lay;
    const NetShape& n = h->net;
    SmallFusedArgs a;
    a.B = h->B; a.T = h->T; a.D = n.dims[0]; a.E = small_fused_envs(h->env, n, h->B, h->T); a.n_wg = h->B / a.E; a.P = n.P;
    a.env = h->env; a.net = n;
    a.w = at<const float>(h, L.w_src);
    a.s0 = at<const uint32_t>(h, L.tr_s0); a.act = at<const uint8_t>(h, L.tr_act); a.rew = at<const float>(h, L.tr_rew);
    a.done = at<const uint8_t>(h, L.tr_done); a.val = at<const float>(h, L.tr_val); a.head = at<const float>(h, L.tr_head);
    a.h1 = at<const float>(h, L.act[0]); a.h2 = at<const float>(h, L.act[1]);
    a.adv = at<float>(h, L.adv); a.ret = at<float>(h, L.ret);
    a.part = at<float>(h, L.small_part); a.loss_part = at<float>(h, L.loss_part);
    a.counter = at<unsigned>(h, L.counters);
    a.max_spin = 1 << 22;                                        // some seconds: only a device that never runs the others gets there
    a.theta = at<float>(h, L.theta); a.grad = at<float>(h, L.grad); a.m = at<float>(h, L.m); a.v = at<float>(h, L.v);
    a.gamma = h->net_cfg.gamma; a.lambda = h->net_cfg.lambda_; a.beta = h->net_cfg.entropy_coef; a.cv = h->net_cfg.value_coef;
    a.inv_m = (float)(1.0 / ((double)h->B * h->T));
    h->adam_t += 1;
    a.lr = h->net_cfg.lr; a.beta1 = h->net_cfg.beta1; a.beta2 = h->net_cfg.beta2; a.eps = h->net_cfg.eps;
    a.bc1 = (float)(1.0 - pow((double)h->net_cfg.beta1, (double)h->adam_t));
    a.bc2 = (float)(1.0 - pow((double)h->net_cfg.beta2, (double)h->adam_t));
    const int R = a.E * a.T, Rp4 = (R + 3) & ~3, Rpad = (R + 31) & ~31, LD = SF_H + 1, Ep4 = (a.E + 3) & ~3;
    const size_t un = (size_t)2 * Rpad * LD;
    const size_t lds = ((size_t)SF_H * LD + (size_t)9 * Rp4 + Ep4 + (size_t)Rpad * LD + 64 + SF_WG + 4 * SF_H * 5 + un) * sizeof(float);
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(learn_small_fused), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return e;
    h->metric_blocks = a.n_wg;
    ProfScope prof(h, "learn_small_fused");
    hipLaunchKernelGGL(learn_small_fused, dim3(a.n_wg), dim3(SF_WG), lds, h->stream, a);
    return hipGetLastError();
}

}  // namespace ank
