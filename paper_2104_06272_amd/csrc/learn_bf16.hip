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
// heads.  Both products run on the matrix cores with the fp32 head gradient
// split into two bfloat16 terms (d = hi + lo, 16 significant bits):
//   dZ_L[m][j] = relu'(h[m][j]) * sum_k d[m][k] Wh[j][k]   one MFMA per 32x32 tile with the
//                reduction index running over (hi_0..7, lo_0..7) against (Wh_0..7, Wh_0..7)
//   dWh[j][k]  = sum_m h[m][j] d[m][k]                      reduction over samples, hi parts in
//                output columns 0..7 and lo parts in 8..15, added at the end
// The reduction over samples may visit them in any order as long as both operands agree; the
// order used here (per lane half kg: samples 4kg..4kg+3 of two consecutive groups of eight) makes
// the 8-byte pieces of packed h that feed it the same ones that mask dZ_L.
// A workgroup walks 64 samples at a time for 256 columns; wavefront w owns columns 64w..64w+63.
// ---------------------------------------------------------------------------
struct HeadBwdBf16Args {
    int M, H, NH, NHP, rows;                   // rows per workgroup (multiple of 64)
    const uint16_t* hP; const float* dhead; const uint16_t* wh16;   // wh16: bf16 copy of Wh, [H][NH]
    uint16_t* dzR; uint16_t* dzP; float* partial;                    // partial: [blocks over rows][H*NH + NH]
};

typedef __bf16 bf2v __attribute__((ext_vector_type(2)));
__device__ __forceinline__ uint32_t cvt_pk_bf16(float lo, float hi)
{
    bf2v v; v[0] = (__bf16)lo; v[1] = (__bf16)hi;
    return __builtin_bit_cast(uint32_t, v);
}

// value r of an accumulator tile where its flag in a ReLU mask word (relu_mask_bit) is set, else +0: the flag is
// spread over the word by a signed one-bit field extract and ANDed onto the value's bits
__device__ __forceinline__ float keep_if(float x, uint32_t mask_word, int r)
{
    const int m = (int)(mask_word << (31 - relu_mask_bit(r))) >> 31;
    return __builtin_bit_cast(float, __builtin_bit_cast(int, x) & m);
}

// two ReLU outputs as bfloat16 in a word (never negative, never -0: relu() returns +0 for every non-positive input)
// -> 0xffff in the halves that are positive, i.e. not zero, and 0 in the others.  Packed 16-bit integer instructions:
// min(h, 1) is 0 or 1, and 0 - that is 0 or 0xffff.
__device__ __forceinline__ uint32_t positive_mask_pk(uint32_t w)
{
    uint32_t r;
    const uint32_t zero = 0u, one = 0x00010001u;
    asm("v_pk_min_u16 %0, %1, %2" : "=v"(r) : "v"(w), "v"(one));
    asm("v_pk_sub_u16 %0, %1, %2" : "=v"(r) : "v"(zero), "v"(r));
    return r;
}

__global__ __launch_bounds__(WG) void head_backward_bf16(const HeadBwdBf16Args a)
{
    constexpr int LDT = WG + 8;
    __shared__ __attribute__((aligned(16))) uint16_t tile[64 * LDT];   // [64 samples][256 columns] for the row-major copy
    __shared__ uint4 Ahl[2][64];                                       // dZ product, A operand per 32-sample tile
    __shared__ uint4 Bhl[2][2][64];                                    // dWh product, B operand per 32-sample tile and 16-sample step
    const int H = a.H, NH = a.NH, NHP = a.NHP;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, l32 = lane & 31, kg = lane >> 5;
    const int jb = blockIdx.y * WG, jw = jb + wave * 64;
    const int m_begin = blockIdx.x * a.rows, m_end = m_begin + a.rows;
    bf8 wB[2];
    bool live[2];
#pragma unroll
    for (int jt = 0; jt < 2; ++jt) {
        const int j = jw + 32 * jt + l32;
        live[jt] = j < H;
        uint16_t w8[8];
#pragma unroll
        for (int k = 0; k < 8; ++k) w8[k] = (live[jt] && k < NH) ? a.wh16[(size_t)j * NH + k] : (uint16_t)0;
        const uint4 wv = make_uint4((uint32_t)w8[0] | ((uint32_t)w8[1] << 16), (uint32_t)w8[2] | ((uint32_t)w8[3] << 16),
                                    (uint32_t)w8[4] | ((uint32_t)w8[5] << 16), (uint32_t)w8[6] | ((uint32_t)w8[7] << 16));
        wB[jt] = *reinterpret_cast<const bf8*>(&wv);
    }
    f16v acc2[2];
#pragma unroll
    for (int jt = 0; jt < 2; ++jt)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc2[jt][r] = 0.0f;
    float db[8] = {0, 0, 0, 0, 0, 0, 0, 0};
    // output columns 16..31 of the dWh product stay zero
    reinterpret_cast<uint4*>(Bhl)[tid] = make_uint4(0, 0, 0, 0);
    __syncthreads();
    for (int m0 = m_begin; m0 < m_end; m0 += 64) {
        // packed h of this wavefront's tiles: group g of 32-sample tile mt, samples 4kg..4kg+3
        uint2 hq[2][2][4];
#pragma unroll
        for (int mt = 0; mt < 2; ++mt)
#pragma unroll
            for (int jt = 0; jt < 2; ++jt)
#pragma unroll
                for (int g = 0; g < 4; ++g) {
                    const size_t G = (size_t)((m0 + 32 * mt) >> 3) + g;
                    hq[mt][jt][g] = live[jt] ? *reinterpret_cast<const uint2*>(a.hP + (G * H + jw + 32 * jt + l32) * 8 + 4 * kg)
                                             : make_uint2(0, 0);
                }
        if (tid < 64) {
            const float* dh = a.dhead + (size_t)(m0 + tid) * NHP;
            float d[8];
            const float4 d0 = *reinterpret_cast<const float4*>(dh);
            d[0] = d0.x; d[1] = d0.y; d[2] = d0.z; d[3] = d0.w;
            if (NHP == 8) { const float4 d1 = *reinterpret_cast<const float4*>(dh + 4); d[4] = d1.x; d[5] = d1.y; d[6] = d1.z; d[7] = d1.w; }
            else { d[4] = d[5] = d[6] = d[7] = 0.0f; }
            uint16_t hi[8], lo[8];
#pragma unroll
            for (int k = 0; k < 8; ++k) {
                if (k >= NH) d[k] = 0.0f;
                db[k] += d[k];
                const uint32_t p = cvt_pk_bf16(d[k], 0.0f);
                hi[k] = (uint16_t)p;
                lo[k] = (uint16_t)cvt_pk_bf16(d[k] - bfu(hi[k]), 0.0f);
            }
            const int mt = tid >> 5, s = tid & 31;
            Ahl[mt][s] = make_uint4((uint32_t)hi[0] | ((uint32_t)hi[1] << 16), (uint32_t)hi[2] | ((uint32_t)hi[3] << 16),
                                    (uint32_t)hi[4] | ((uint32_t)hi[5] << 16), (uint32_t)hi[6] | ((uint32_t)hi[7] << 16));
            Ahl[mt][32 + s] = make_uint4((uint32_t)lo[0] | ((uint32_t)lo[1] << 16), (uint32_t)lo[2] | ((uint32_t)lo[3] << 16),
                                         (uint32_t)lo[4] | ((uint32_t)lo[5] << 16), (uint32_t)lo[6] | ((uint32_t)lo[7] << 16));
            const int g = s >> 3, r = s & 7, kgs = r >> 2, q = (g & 1) * 4 + (r & 3);
            uint16_t* Bp = reinterpret_cast<uint16_t*>(&Bhl[mt][g >> 1][0]);
#pragma unroll
            for (int k = 0; k < 8; ++k) {
                Bp[(kgs * 32 + k) * 8 + q] = hi[k];
                Bp[(kgs * 32 + 8 + k) * 8 + q] = lo[k];
            }
        }
        __syncthreads();
#pragma unroll
        for (int mt = 0; mt < 2; ++mt) {
            const uint4 a1v = Ahl[mt][lane];
            const bf8 a1 = *reinterpret_cast<const bf8*>(&a1v);
            const uint4 b20v = Bhl[mt][0][lane], b21v = Bhl[mt][1][lane];
            const bf8 b20 = *reinterpret_cast<const bf8*>(&b20v), b21 = *reinterpret_cast<const bf8*>(&b21v);
#pragma unroll
            for (int jt = 0; jt < 2; ++jt) {
                const uint4 x0 = make_uint4(hq[mt][jt][0].x, hq[mt][jt][0].y, hq[mt][jt][1].x, hq[mt][jt][1].y);
                const uint4 x1 = make_uint4(hq[mt][jt][2].x, hq[mt][jt][2].y, hq[mt][jt][3].x, hq[mt][jt][3].y);
                acc2[jt] = mfma_bf16(*reinterpret_cast<const bf8*>(&x0), b20, acc2[jt]);
                acc2[jt] = mfma_bf16(*reinterpret_cast<const bf8*>(&x1), b21, acc2[jt]);
                f16v acc1;
#pragma unroll
                for (int r = 0; r < 16; ++r) acc1[r] = 0.0f;
                acc1 = mfma_bf16(a1, wB[jt], acc1);
                const int col = wave * 64 + 32 * jt + l32;
#pragma unroll
                for (int g = 0; g < 4; ++g) {
                    const uint32_t mw[2] = {hq[mt][jt][g].x, hq[mt][jt][g].y};
                    float o[4];
#pragma unroll
                    for (int q = 0; q < 4; ++q) {
                        const float hv = bfu((uint16_t)((mw[q >> 1] >> ((q & 1) * 16)) & 0xffffu));
                        o[q] = hv > 0.0f ? acc1[4 * g + q] : 0.0f;
                    }
                    const uint32_t p01 = cvt_pk_bf16(o[0], o[1]), p23 = cvt_pk_bf16(o[2], o[3]);
                    const int row = 32 * mt + 8 * g + 4 * kg;
                    if (a.dzR) {
                        tile[(row + 0) * LDT + col] = (uint16_t)p01; tile[(row + 1) * LDT + col] = (uint16_t)(p01 >> 16);
                        tile[(row + 2) * LDT + col] = (uint16_t)p23; tile[(row + 3) * LDT + col] = (uint16_t)(p23 >> 16);
                    }
                    if (live[jt]) {
                        const size_t G = (size_t)((m0 + 32 * mt) >> 3) + g;
                        *reinterpret_cast<uint2*>(a.dzP + (G * H + jw + 32 * jt + l32) * 8 + 4 * kg) = make_uint2(p01, p23);
                    }
                }
            }
        }
        __syncthreads();
        // row-major copy (only where the tiled dX kernel reads it): 64 rows x 256 columns, 16-byte pieces
        if (a.dzR)
            for (int i = tid; i < 64 * (WG / 8); i += WG) {
                const int row = i / (WG / 8), c = (i % (WG / 8)) * 8;
                if (jb + c < H)
                    *reinterpret_cast<uint4*>(a.dzR + (size_t)(m0 + row) * H + jb + c) = *reinterpret_cast<const uint4*>(&tile[row * LDT + c]);
            }
    }
    __syncthreads();
    // dWh: rows j of the accumulator, columns k (hi parts) and 8+k (lo parts)
    float* S = reinterpret_cast<float*>(tile);                       // [256 columns j][16]
    if (l32 < 16) {
#pragma unroll
        for (int jt = 0; jt < 2; ++jt)
#pragma unroll
            for (int r = 0; r < 16; ++r)
                S[(wave * 64 + 32 * jt + 8 * (r >> 2) + 4 * kg + (r & 3)) * 16 + l32] = acc2[jt][r];
    }
    __syncthreads();
    float* out = a.partial + (size_t)blockIdx.x * ((size_t)H * NH + NH);
    if (jb + tid < H)
        for (int k = 0; k < NH; ++k) out[(size_t)(jb + tid) * NH + k] = S[tid * 16 + k] + S[tid * 16 + 8 + k];
    if (blockIdx.y == 0) {
        __syncthreads();
        if (tid < 64) for (int k = 0; k < 8; ++k) S[tid * 8 + k] = db[k];
        __syncthreads();
        if (tid < NH) {
            float sum = 0.0f;
            for (int i = 0; i < 64; ++i) sum += S[i * 8 + tid];
            out[(size_t)H * NH + tid] = sum;
        }
    }
}

// ---------------------------------------------------------------------------
// dX = (dY W^T) masked.  dY row-major [M][N], W bf16 [K][N] (row i, reduction j
// contiguous), mask from packed h, output in both layouts.  128 x 128 tile,
// reduction staged through LDS 128 at a time.
// ---------------------------------------------------------------------------
struct GemmNtBf16Args {
    int M, K, N;
    const uint16_t* dyR;      // [M][N] (tiled kernel), or null
    const uint16_t* dyP;      // packed [M/8][N][8] (weights-resident kernel)
    const uint16_t* w16;      // [K][N]
    const uint16_t* hP;       // packed h_{l-1}: [M/8][K][8]
    uint16_t* dxR;            // [M][K], or null when no product below reads the row-major form
    uint16_t* dxP;            // [M/8][K][8]
    // top layer of the weights-resident kernel: dY = dZ_L is not read but formed from the head gradient,
    // dZ_L[m][j] = relu'(hTop[m][j]) * sum_k dhead[m][k] Wh[j][k]
    const uint32_t* maskTop;  // ReLU mask words of h_L (relu_mask_index)
    const uint32_t* maskLo;   // ReLU mask words of h_{l-1}, or null: the mask is then taken from hP
    const float* dhead;       // [M][NHP]
    const uint16_t* wh16;     // bf16 copy of Wh: [N][NH]
    int NH, NHP;
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
    int mt_, it_;
    xcd_map((int)blockIdx.x, (a.M + 127) / 128, (a.K + 127) / 128, mt_, it_);   // the i-tiles of one m-tile share dY
    const int m0 = mt_ * 128, i0 = it_ * 128;
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
        if (a.dxR && m0 + row < a.M && i0 + c < a.K)
            *reinterpret_cast<uint4*>(a.dxR + (size_t)(m0 + row) * a.K + i0 + c) = *reinterpret_cast<const uint4*>(Ts + row * NB_LD + c);
    }
}

// ---------------------------------------------------------------------------
// The same product as a persistent workgroup with the weights in registers: wavefront w of eight
// keeps the 32 output columns 32w.. of a 256-column block of W (NR/4 registers per lane, the B
// operand of every step), dY streams through LDS 32 rows at a time, double buffered, and nothing
// but dY, the mask and the result crosses the memory system.  The kernel is HBM-bound by design:
// about 4 bytes per output element.
// dY is read in its sample-packed form, the one its producer writes for the dW product anyway, and
// turned into rows on the way into LDS: a loader thread takes one 16-byte piece (eight samples of
// one column) and stores its eight values into eight rows.  So dZ_l exists in one layout only, and
// the result is written packed only.  NR: reduction length N (256 or 512); K a multiple of 256; M a
// multiple of 32.
// ---------------------------------------------------------------------------
typedef uint32_t u32x4_l __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2_l __attribute__((ext_vector_type(2)));
constexpr int NRES_WG = 512;
constexpr int NRES_RT = 32;             // rows per stage

template <int NR, bool HEADS>
__global__ __launch_bounds__(NRES_WG) void gemm_nt_bf16_res(const GemmNtBf16Args a, const int rows_per_block)
{
    constexpr int LD = NR + 8;                                   // row stride in bf16: eight rows cover all banks
    constexpr int KS = NR / 16;                                  // MFMA steps
    constexpr int NQ = (NRES_RT / 8) * NR / NRES_WG;             // 16-byte pieces per thread and stage: 4 groups x NR columns
    constexpr int TJ = NR / 256;                                 // HEADS: 32-column tiles of dZ_L a wavefront forms per stage
    extern __shared__ uint4 smem4[];
    uint16_t* As0 = reinterpret_cast<uint16_t*>(smem4);
    uint16_t* As1 = As0 + NRES_RT * LD;
    __shared__ uint4 Ahl[2][64];                                 // HEADS: head gradient of a stage's 32 rows as (hi, lo) bfloat16 terms
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, l32 = lane & 31, kg = lane >> 5;
    int rb_, cb_;
    xcd_map((int)blockIdx.x, (a.M + rows_per_block - 1) / rows_per_block, a.K / 256, rb_, cb_);   // column blocks of the same rows share dY in one L2
    const int i0 = cb_ * 256;
    const int i = i0 + wave * 32 + l32;                          // this lane's output column
    const int m_begin = rb_ * rows_per_block;
    const int m_end = m_begin + rows_per_block < a.M ? m_begin + rows_per_block : a.M;
    if (m_begin >= a.M) return;
    bf8 wreg[KS];
#pragma unroll
    for (int s2 = 0; s2 < KS; ++s2) wreg[s2] = *reinterpret_cast<const bf8*>(a.w16 + (size_t)i * NR + 16 * s2 + 8 * kg);
    // loader: piece p = q * NRES_WG + tid is sample group p / NR of the stage, column p % NR
    // Two register sets of staged pieces: those of stage s + 2 are requested while stage s is computed, so a load
    // has two stage times to come back (one stage is shorter than the memory latency under load, and this kernel
    // lives on the HBM roof).  The relu mask of stage s + 1 is requested one stage ahead for the same reason.
    // HEADS: what is staged is the ReLU mask word of h_L for each 32-column tile jt of the wavefront's columns
    // instead (16 flags, one per accumulator value), and going to LDS means one MFMA per tile, d (hi, lo) against
    // (Wh, Wh), masked by them
    u32x4_l stA[NQ], stB[NQ];
    __shared__ uint4 WhB[HEADS ? NR : 1];                        // row j of Wh, eight entries (zero past NH): the B operand of column j
    if (HEADS) {
        for (int j = tid; j < NR; j += NRES_WG) {
            uint32_t w8[8];
#pragma unroll
            for (int k = 0; k < 8; ++k) w8[k] = k < a.NH ? (uint32_t)a.wh16[(size_t)j * a.NH + k] : 0u;
            WhB[j] = make_uint4(w8[0] | (w8[1] << 16), w8[2] | (w8[3] << 16), w8[4] | (w8[5] << 16), w8[6] | (w8[7] << 16));
        }
    }
    auto fetch = [&](u32x4_l (&st)[NQ], int m0) {
        if (HEADS) {
#pragma unroll
            for (int jt = 0; jt < TJ; ++jt)
                st[0][jt] = a.maskTop[relu_mask_index((size_t)(m0 >> 5), kg, NR, wave * (NR / 8) + 32 * jt + l32)];
            return;
        }
#pragma unroll
        for (int q = 0; q < NQ; ++q) {
            const int p = q * NRES_WG + tid;
            st[q] = *reinterpret_cast<const u32x4_l*>(a.dyP + ((size_t)((m0 >> 3) + p / NR) * NR + p % NR) * 8);
        }
    };
    // par (HEADS): which half of Ahl holds the head gradient of the stage being stored
    auto store = [&](const u32x4_l (&st)[NQ], uint16_t* buf, int par) {
        if (HEADS) {
            const uint4 a1v = Ahl[par][lane];
            const bf8 a1 = *reinterpret_cast<const bf8*>(&a1v);
#pragma unroll
            for (int jt = 0; jt < TJ; ++jt) {
                f16v acc1;
#pragma unroll
                for (int r = 0; r < 16; ++r) acc1[r] = 0.0f;
                const uint4 wv = WhB[wave * (NR / 8) + 32 * jt + l32];
                acc1 = mfma_bf16(a1, *reinterpret_cast<const bf8*>(&wv), acc1);
                uint16_t* dst = buf + (4 * kg) * LD + wave * (NR / 8) + 32 * jt + l32;
                const uint32_t bits = st[0][jt];
#pragma unroll
                for (int g = 0; g < 4; ++g) {
                    const uint32_t p01 = cvt_pk_bf16(keep_if(acc1[4 * g], bits, 4 * g), keep_if(acc1[4 * g + 1], bits, 4 * g + 1));
                    const uint32_t p23 = cvt_pk_bf16(keep_if(acc1[4 * g + 2], bits, 4 * g + 2), keep_if(acc1[4 * g + 3], bits, 4 * g + 3));
                    dst[(8 * g + 0) * LD] = (uint16_t)p01; dst[(8 * g + 1) * LD] = (uint16_t)(p01 >> 16);
                    dst[(8 * g + 2) * LD] = (uint16_t)p23; dst[(8 * g + 3) * LD] = (uint16_t)(p23 >> 16);
                }
            }
            return;
        }
#pragma unroll
        for (int q = 0; q < NQ; ++q) {
            const int p = q * NRES_WG + tid;
            uint16_t* dst = buf + (8 * (p / NR)) * LD + p % NR;
#pragma unroll
            for (int e = 0; e < 8; ++e) dst[e * LD] = (uint16_t)(st[q][e >> 1] >> ((e & 1) * 16));
        }
    };
    // HEADS: the first 256 threads carry one entry (row tid / 8, head output tid % 8) of the head gradient each, two
    // stages ahead
    float dreg = 0.0f;
    auto fetch_d = [&](int m0) {
        if (!HEADS || tid >= 256) return;
        const int k = tid & 7;
        dreg = k < a.NH ? a.dhead[(size_t)(m0 + (tid >> 3)) * a.NHP + k] : 0.0f;
    };
    auto store_d = [&](int par) {
        if (!HEADS || tid >= 256) return;
        const uint32_t hi = cvt_pk_bf16(dreg, 0.0f) & 0xffffu;
        const uint32_t lo = cvt_pk_bf16(dreg - bfu((uint16_t)hi), 0.0f) & 0xffffu;
        uint16_t* A16 = reinterpret_cast<uint16_t*>(&Ahl[par][0]);
        A16[tid] = (uint16_t)hi;                                 // row tid / 8 of the hi half, entry tid % 8
        A16[256 + tid] = (uint16_t)lo;
    };
    const uint32_t lane_off = (uint32_t)i * 8u + 4u * kg;        // inside a packed group of eight samples
    u32x2_l maskA[4], maskB[4];
    auto fetch_mask = [&](u32x2_l (&mk)[4], int m0) {
        if (a.maskLo) { mk[0][0] = a.maskLo[relu_mask_index((size_t)(m0 >> 5), kg, a.K, i)]; return; }
#pragma unroll
        for (int g = 0; g < 4; ++g)
            mk[g] = *reinterpret_cast<const u32x2_l*>(a.hP + ((size_t)((m0 >> 3) + g) * a.K) * 8 + lane_off);
    };
    const int m_lastst = m_end - NRES_RT;                        // loads past the end re-read the last stage, unused
    auto clampm = [&](int m) { return m < m_end ? m : m_lastst; };
    fetch(stA, m_begin);
    if (HEADS) {
        fetch_d(m_begin); store_d(0);
        fetch_d(clampm(m_begin + NRES_RT)); store_d(1);
        __syncthreads();
    }
    store(stA, As0, 0);
    fetch(stA, clampm(m_begin + NRES_RT));                       // stage 1, stored at the end of stage 0
    fetch_mask(maskA, m_begin);
    __syncthreads();
    // one stage (of parity par): MFMAs on `cur` with the KS two-byte stores that put stage s + 1 (`st_next`) into
    // `nxt` spread between them, one per MFMA, so that the LDS writes and the vector work behind them run in the
    // shadow of the matrix cores instead of in a phase of their own (nobody reads `nxt` during this stage; past the
    // end the last stage is formed again, unused); then the epilogue with `mask`; the head gradient of stage s + 2
    // replaces that of stage s
    auto stage = [&](int m0, int par, const uint16_t* cur, uint16_t* nxt, const u32x2_l (&mask)[4],
                     u32x4_l (&st_next)[NQ], u32x4_l (&st_fill)[NQ], u32x2_l (&mask_fill)[4]) {
        fetch(st_fill, clampm(m0 + 2 * NRES_RT));                // two stages ahead
        fetch_d(clampm(m0 + 2 * NRES_RT));
        fetch_mask(mask_fill, clampm(m0 + NRES_RT));             // one stage ahead
        __builtin_amdgcn_sched_barrier(0);
        // the KS values of this lane for the next stage, two per word, and the rows they go to.  HEADS: the tiles of
        // dZ_L stay in their accumulators and every word is masked and rounded right before its two stores, between
        // the MFMAs, instead of all of them ahead of the first one
        uint32_t pk[HEADS ? 1 : KS / 2];
        uint16_t* wbase[HEADS ? TJ : 1];
        f16v accz[HEADS ? TJ : 1];
        uint32_t zbits[HEADS ? TJ : 1];
        if (HEADS) {
            const uint4 a1v = Ahl[par ^ 1][lane];
            const bf8 a1 = *reinterpret_cast<const bf8*>(&a1v);
#pragma unroll
            for (int jt = 0; jt < TJ; ++jt) {
#pragma unroll
                for (int r = 0; r < 16; ++r) accz[jt][r] = 0.0f;
                const uint4 wv = WhB[wave * (NR / 8) + 32 * jt + l32];
                accz[jt] = mfma_bf16(a1, *reinterpret_cast<const bf8*>(&wv), accz[jt]);
                zbits[jt] = st_next[0][jt];
                wbase[jt] = nxt + (4 * kg) * LD + wave * (NR / 8) + 32 * jt + l32;
            }
        } else {
#pragma unroll
            for (int q = 0; q < NQ; ++q)
#pragma unroll
                for (int w = 0; w < 4; ++w) pk[4 * q + w] = st_next[q][w];
            wbase[0] = nxt + (NR == 512 ? tid : 8 * (tid >> 8) * LD + (tid & 255));
        }
        // store k: half k % 2 of word k / 2.  HEADS: word 2g + j of a tile holds rows 8g + 4kg + 2j, + 1 of its
        // column; otherwise piece q = k / 8 is sample group q (NR = 512) or 2q + tid / 256 (NR = 256), sample k % 8
        uint32_t zword = 0u;
        auto put = [&](int k) {
            if (HEADS) {
                const int jt = k >> 4, kk = k & 15;
                if ((kk & 1) == 0)
                    zword = cvt_pk_bf16(keep_if(accz[HEADS ? jt : 0][kk], zbits[HEADS ? jt : 0], kk),
                                        keep_if(accz[HEADS ? jt : 0][kk + 1], zbits[HEADS ? jt : 0], kk + 1));
                wbase[HEADS ? jt : 0][(8 * (kk >> 2) + (kk & 3)) * LD] = (uint16_t)(zword >> ((kk & 1) * 16));
            } else {
                const uint16_t v = (uint16_t)(pk[HEADS ? 0 : k >> 1] >> ((k & 1) * 16));
                wbase[0][((NR == 512 ? 8 : 16) * (k >> 3) + (k & 7)) * LD] = v;
            }
        };
        f16v acc;
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[r] = 0.0f;
        const uint16_t* a_rd = cur + l32 * LD + 8 * kg;
        bf8 av0 = *reinterpret_cast<const bf8*>(a_rd), av1 = *reinterpret_cast<const bf8*>(a_rd + 16);
#pragma unroll
        for (int s2 = 0; s2 < KS; ++s2) {
            const bf8 an = *reinterpret_cast<const bf8*>(a_rd + 16 * (s2 + 2 < KS ? s2 + 2 : 0));
            acc = mfma_bf16(av0, wreg[s2], acc);
            put(s2);
            av0 = av1; av1 = an;
            __builtin_amdgcn_sched_barrier(0);                   // keeps the read / MFMA / store order as written
        }
        // rows 8g + 4kg + q of the stage, column i: half of one packed group per g
#pragma unroll
        for (int g = 0; g < 4; ++g) {
            float o[4];
            if (a.maskLo) {
#pragma unroll
                for (int q = 0; q < 4; ++q) o[q] = keep_if(acc[4 * g + q], mask[0][0], 4 * g + q);
            } else {
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const float hv = bfu((uint16_t)((mask[g][q >> 1] >> ((q & 1) * 16)) & 0xffffu));
                    o[q] = hv > 0.0f ? acc[4 * g + q] : 0.0f;
                }
            }
            u32x2_l pv; pv[0] = cvt_pk_bf16(o[0], o[1]); pv[1] = cvt_pk_bf16(o[2], o[3]);
            *reinterpret_cast<u32x2_l*>(a.dxP + ((size_t)((m0 >> 3) + g) * a.K) * 8 + lane_off) = pv;
        }
        store_d(par);
        __syncthreads();
    };
    for (int m0 = m_begin; m0 < m_end; m0 += 2 * NRES_RT) {
        stage(m0, 0, As0, As1, maskA, stA, stB, maskB);
        if (m0 + NRES_RT < m_end) stage(m0 + NRES_RT, 1, As1, As0, maskB, stB, stA, maskA);
    }
}

// ---------------------------------------------------------------------------
// dW partials from packed operands.  LDS tiles [sample group][column][8]; every
// operand is one 16-byte read.  OBS: the first layer's x comes from the state
// snapshots (walls bit planes, agent cell, goal cell / Catch cells).
// ---------------------------------------------------------------------------
struct GemmTnBf16Args {
    int M, K, N, splits, rows, tiles_i, use_obs;
    int obs_row0;             // with use_obs: row i of this product is observation feature obs_row0 + i
    const uint16_t* xP;       // packed [M/8][K][8], unused with use_obs
    const uint16_t* dyP;      // packed [M/8][N][8]
    float* partial;           // [splits][split_stride]: K x N partial of each split
    size_t split_stride;
    float* bias_out;          // [splits][bias_stride]: N column sums of each split, or null
    size_t bias_stride;
    ObsSrc obs;
    // agent-plane product only: chunks are blocks of env_block environments over all T time steps, and the sum of
    // dY over time is written to sP (two bfloat16 terms per entry) on the way; null: chunks are sample ranges
    uint16_t* sP;
    int T, env_block;
};

constexpr int TB_G = 16;      // sample groups (of 8) per LDS stage: 128 samples

__device__ __forceinline__ uint4 obs_piece(const ObsSrc& o, int mg, int i, bool valid)
{
    // eight consecutive samples (same time step, consecutive envs) of observation feature i
    uint16_t v[8];
#pragma unroll
    for (int q = 0; q < 8; ++q) v[q] = 0;
    if (valid) {
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
            if (OBS) rx[q] = gok ? obs_piece(a.obs, g, a.obs_row0 + i0 + c, i0 + c < a.K) : make_uint4(0, 0, 0, 0);
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
    float* out = a.partial + (size_t)split * a.split_stride;
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
    if (ti == 0 && a.bias_out && tid < 128 && j0 + tid < a.N) a.bias_out[(size_t)split * a.bias_stride + j0 + tid] = bsum;
}

// The same product with a 256 x 256 tile and eight wavefronts (two per SIMD, so one's LDS and
// global traffic overlaps the other's MFMAs): wavefront (wm, wn) owns rows 128*wm.., columns
// 64*wn.. of the tile, eight 32 x 32 accumulators, and every 16-byte read from LDS feeds 2 or 4
// MFMAs.  K and N multiples of 256.
constexpr int BIGWG = 512;
constexpr int TB_BG = 8;      // sample groups (of 8) per LDS stage: 64 samples

// XMODE: where the X operand comes from.  0: packed activations in HBM; 1: the agent plane of the
// maze observation, a one-hot of the agent cell, built from the stage's 64 cell indices which pass
// through LDS one stage ahead; 2: the wall plane of the maze observation (samples are environments,
// rows are cells), built from the stage's 64 x 8 wall words which pass through LDS the same way.
// Pipeline: LDS holds two stages.  While the MFMAs run on stage i, the same wavefronts put stage
// i + 1 into the other half -- its four (X, Y) pieces per thread go between the four MFMA steps, so
// the LDS stores and the vector work behind them (the one-hot, the sums) run in the shadow of the
// matrix cores -- and then ask for stage i + 3 into the registers just emptied: every load has two
// stages to arrive, and there is one barrier per stage.  Chunks are whole pairs of stages of 64
// samples (a.rows % 128 == 0).
template <int XMODE>
__global__ __launch_bounds__(BIGWG) void gemm_tn_bf16_big(const GemmTnBf16Args a)
{
    extern __shared__ uint4 smem4[];         // [2 stages][X | Y][TB_BG][256] pieces of 8 samples
    __shared__ uint32_t posL[2][64];         // XMODE 1: agent cells of the 64 samples of a stage, double buffered
    __shared__ uint32_t wallsL[2][XMODE == 2 ? 8 : 1][64];   // XMODE 2: the eight wall words of the 64 environments of a stage
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 2, wn = wave & 3, l32 = lane & 31, kg = lane >> 5;
    int split, tile;
    xcd_map((int)blockIdx.x, a.splits, a.tiles_i * (a.N / 256), split, tile);   // the tiles of one split share its samples
    const int ti = tile % a.tiles_i, tj = tile / a.tiles_i;
    const int i0 = ti * 256, j0 = tj * 256;
    const int n_stages = a.rows >> 6;
    const bool by_env = XMODE == 1 && a.sP != nullptr;
    // first sample group of stage i of this chunk.  Sample ranges: consecutive stages.  Blocks of environments: the 64
    // environments of one stage at t = 0 .. T-1, then the next 64 (so a thread meets every time step of its samples
    // in order and can add them up)
    auto stage_g0 = [&](int i) -> int {
        if (by_env) {
            const int p = i / a.T, t = i - p * a.T;
            return (t * a.obs.B + split * a.env_block + 64 * p) >> 3;
        }
        return ((split * a.rows) >> 3) + i * TB_BG;
    };
    // loader: thread = (column, parity of the sample group), four groups of the stage each
    const int lc = tid & 255, lg = tid >> 8;
    struct Set { u32x4_l x[TB_BG / 2]; u32x4_l y[TB_BG / 2]; uint32_t pos; };
    Set S0, S1;
    auto fetch = [&](Set& st, int i) {
        if (i >= n_stages) i = n_stages - 1;                     // past the end: re-read the last stage, never used
        const int g0 = stage_g0(i);
        // the cells first: they are needed one step before the rest of the set, and loads complete in issue order
        if (XMODE == 1) st.pos = a.obs.s0[(size_t)g0 * 8 + (tid & 63)];
        // wall words: thread = (environment of the stage, word); a stage never straddles the two halves of the 2B
        // samples (B is a multiple of 64)
        if (XMODE == 2) st.pos = a.obs.walls[(size_t)(tid & 7) * a.obs.B + (g0 * 8) % a.obs.B + (tid >> 3)];
#pragma unroll
        for (int q = 0; q < TB_BG / 2; ++q) {
            const int g = g0 + 2 * q + lg;
            if (XMODE == 0) st.x[q] = *reinterpret_cast<const u32x4_l*>(a.xP + ((size_t)g * a.K + i0 + lc) * 8);
            st.y[q] = *reinterpret_cast<const u32x4_l*>(a.dyP + ((size_t)g * a.N + j0 + lc) * 8);
        }
    };
    float tsum[TB_BG / 2][8];                                    // by_env: sum over time of this thread's dY entries
#pragma unroll
    for (int q = 0; q < TB_BG / 2; ++q)
#pragma unroll
        for (int e = 0; e < 8; ++e) tsum[q][e] = 0.0f;
    float bsum = 0.0f;
    const bool sums = ti == 0 && a.bias_out != nullptr;
    const int cell = a.obs_row0 + i0 + lc - a.obs.env.rows * a.obs.env.cols;   // XMODE 1: the cell this thread's row stands for
    // piece q (sample group 2q + lg) of stage i, held in st, -> half nb of LDS; counted: a real stage (not the
    // repeat of the last one that the last step stores), whose dY entries go into the sums
    auto store_piece = [&](const Set& st, int i, int nb, int q, bool counted) {
        uint4* Xs = smem4 + nb * (2 * TB_BG * 256);
        uint4* Ys = Xs + TB_BG * 256;
        const int gl = 2 * q + lg;
        u32x4_l x;
        if (XMODE == 0) x = st.x[q];
        else if (XMODE == 1) {
            const u32x4_l p0 = *reinterpret_cast<const u32x4_l*>(&posL[i & 1][gl * 8]);
            const u32x4_l p1 = *reinterpret_cast<const u32x4_l*>(&posL[i & 1][gl * 8 + 4]);
            const uint32_t one = 0x3f80u;
            x[0] = ((int)p0[0] == cell ? one : 0u) | ((int)p0[1] == cell ? one << 16 : 0u);
            x[1] = ((int)p0[2] == cell ? one : 0u) | ((int)p0[3] == cell ? one << 16 : 0u);
            x[2] = ((int)p1[0] == cell ? one : 0u) | ((int)p1[1] == cell ? one << 16 : 0u);
            x[3] = ((int)p1[2] == cell ? one : 0u) | ((int)p1[3] == cell ? one << 16 : 0u);
        } else {
            const int c = a.obs_row0 + i0 + lc;                  // this thread's cell: bit c % 32 of wall word c / 32
            const u32x4_l w0 = *reinterpret_cast<const u32x4_l*>(&wallsL[i & 1][XMODE == 2 ? c >> 5 : 0][gl * 8]);
            const u32x4_l w1 = *reinterpret_cast<const u32x4_l*>(&wallsL[i & 1][XMODE == 2 ? c >> 5 : 0][gl * 8 + 4]);
            const uint32_t one = 0x3f80u;
            const int sh = c & 31;
            x[0] = (((w0[0] >> sh) & 1u) * one) | (((w0[1] >> sh) & 1u) * (one << 16));
            x[1] = (((w0[2] >> sh) & 1u) * one) | (((w0[3] >> sh) & 1u) * (one << 16));
            x[2] = (((w1[0] >> sh) & 1u) * one) | (((w1[1] >> sh) & 1u) * (one << 16));
            x[3] = (((w1[2] >> sh) & 1u) * one) | (((w1[3] >> sh) & 1u) * (one << 16));
        }
        *reinterpret_cast<u32x4_l*>(&Xs[gl * 256 + lc]) = x;
        *reinterpret_cast<u32x4_l*>(&Ys[gl * 256 + lc]) = st.y[q];
        // column sums in every workgroup (used only where `sums` holds; the workgroups that need them set the pace
        // anyway, and a branch on `sums` here would split the step into many basic blocks)
        const float keep = counted ? 1.0f : 0.0f;
        if (XMODE != 1) {
            float part = 0.0f;
#pragma unroll
            for (int e = 0; e < 8; ++e) part += bfu((uint16_t)((st.y[q][e >> 1] >> ((e & 1) * 16)) & 0xffffu));
            bsum = fmaf(keep, part, bsum);
        }
        if (by_env) {
#pragma unroll
            for (int e = 0; e < 8; ++e) tsum[q][e] = fmaf(keep, bfu((uint16_t)((st.y[q][e >> 1] >> ((e & 1) * 16)) & 0xffffu)), tsum[q][e]);
        }
    };
    // by_env, after the last time step of a block of 64 environments (stage i): the sums leave as two bfloat16 terms,
    // hi in sample rows 0..B-1 and lo in rows B..2B-1 of a packed matrix with 2B samples
    auto flush_time_sum = [&](int i) {
        const int p = i / a.T;
        const size_t n = (size_t)(a.obs.B >> 3) * a.N;
#pragma unroll
        for (int q = 0; q < TB_BG / 2; ++q) {
            const size_t idx = (size_t)(((split * a.env_block + 64 * p) >> 3) + 2 * q + lg) * a.N + j0 + lc;
            uint32_t hi[4], lo[4];
#pragma unroll
            for (int w = 0; w < 4; ++w) {
                hi[w] = cvt_pk_bf16(tsum[q][2 * w], tsum[q][2 * w + 1]);
                lo[w] = cvt_pk_bf16(tsum[q][2 * w] - bfu((uint16_t)hi[w]), tsum[q][2 * w + 1] - bfu((uint16_t)(hi[w] >> 16)));
            }
            *reinterpret_cast<uint4*>(a.sP + idx * 8) = make_uint4(hi[0], hi[1], hi[2], hi[3]);
            *reinterpret_cast<uint4*>(a.sP + (n + idx) * 8) = make_uint4(lo[0], lo[1], lo[2], lo[3]);
#pragma unroll
            for (int e = 0; e < 8; ++e) tsum[q][e] = 0.0f;
        }
    };
    f16v acc[4][2];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.0f;
    // MFMA step ks (16 samples = groups ks, ks + 1) on half cb of LDS
    auto compute_step = [&](int cb, int ks) {
        const uint4* Xs = smem4 + cb * (2 * TB_BG * 256);
        const uint4* Ys = Xs + TB_BG * 256;
        bf8 av[4], bv[2];
#pragma unroll
        for (int t = 0; t < 4; ++t) av[t] = *reinterpret_cast<const bf8*>(&Xs[(ks + kg) * 256 + wm * 128 + 32 * t + l32]);
#pragma unroll
        for (int t = 0; t < 2; ++t) bv[t] = *reinterpret_cast<const bf8*>(&Ys[(ks + kg) * 256 + wn * 64 + 32 * t + l32]);
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int j = 0; j < 2; ++j) acc[i][j] = mfma_bf16(av[i], bv[j], acc[i][j]);
    };
    // one step: the MFMAs of stage i on half i % 2 of LDS, stage i + 1 (held in `nxt`) into the other half piece by
    // piece between them; then `nxt` is refilled with stage i + 3 and the cells of stage i + 2 (held in `aft`) go to
    // the cell buffer that stage i's one-hot was built from
    auto step = [&](Set& nxt, const Set& aft, int i) {
        const int cb = i & 1;
        const bool counted = i + 1 < n_stages;
#pragma unroll
        for (int q = 0; q < TB_BG / 2; ++q) {
            store_piece(nxt, i + 1, cb ^ 1, q, counted);
            __builtin_amdgcn_sched_barrier(0);
            compute_step(cb, 2 * q);
            __builtin_amdgcn_sched_barrier(0);
        }
        if (by_env && ti == 0 && counted && (i + 2) % a.T == 0) flush_time_sum(i + 1);
        if (XMODE == 1 && tid < 64) posL[cb][tid] = aft.pos & 0xffffu;
        if (XMODE == 2) wallsL[cb][XMODE == 2 ? tid & 7 : 0][tid >> 3] = aft.pos;
        fetch(nxt, i + 3);
        __syncthreads();
    };
    // S0's loads strictly before S1's: the scheduler is otherwise free to issue S1's first, and then the wait-count
    // pass, which merges this state with the loop's own at the loop header, has to wait for every load in flight
    // there on every trip (loads complete in issue order), which would end the look-ahead
    fetch(S0, 0);
    __builtin_amdgcn_sched_barrier(0);
    fetch(S1, 1);
    __builtin_amdgcn_sched_barrier(0);
    if (XMODE == 1) {
        if (tid < 64) { posL[0][tid] = S0.pos & 0xffffu; posL[1][tid] = S1.pos & 0xffffu; }
        __syncthreads();
    }
    if (XMODE == 2) {
        wallsL[0][XMODE == 2 ? tid & 7 : 0][tid >> 3] = S0.pos; wallsL[1][XMODE == 2 ? tid & 7 : 0][tid >> 3] = S1.pos;
        __syncthreads();
    }
#pragma unroll
    for (int q = 0; q < TB_BG / 2; ++q) store_piece(S0, 0, 0, q, true);
    if (by_env && ti == 0 && a.T == 1) flush_time_sum(0);
    __builtin_amdgcn_sched_barrier(0);
    fetch(S0, 2);
    __syncthreads();
    // two steps per trip without a branch between them: with a conditional second step the wait-count pass gives up
    // counting in the same way
    for (int i = 0; i < n_stages; i += 2) {
        step(S1, S0, i);
        step(S0, S1, i + 1);
    }
    float* out = a.partial + (size_t)split * a.split_stride;
#pragma unroll
    for (int tr = 0; tr < 4; ++tr)
#pragma unroll
        for (int tc = 0; tc < 2; ++tc) {
            const int j = j0 + wn * 64 + tc * 32 + l32;
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int i = i0 + wm * 128 + tr * 32 + 8 * (r >> 2) + 4 * kg + (r & 3);
                out[(size_t)i * a.N + j] = acc[tr][tc][r];
            }
        }
    if (sums) {
        // the two threads of a column (even and odd sample groups) add their sums in a fixed order
        float* red = reinterpret_cast<float*>(smem4);
        if (lg == 1) red[lc] = bsum;
        __syncthreads();
        if (lg == 0) a.bias_out[(size_t)split * a.bias_stride + j0 + lc] = bsum + red[lc];
    }
}

// ---------------------------------------------------------------------------
// Top layer with the heads folded in.  dZ_L never reaches memory: this kernel and the dX kernel
// above (HEADS) both form it from the head gradient, stage by stage.  Here the stage's 64 samples
// x 256 columns of dZ_L go to LDS as the Y operand of dW_L = h_{L-1}^T dZ_L: wavefront w forms
// columns 32w.. (two MFMAs, d (hi, lo) against (Wh, Wh), masked by the 8-byte pieces of packed
// h_L it holds in accumulator order).  The workgroups of the first row of tiles also add up
// dWh = h_L^T d for their 256 columns (the same pieces of h_L are the A operand, see
// head_backward_bf16 for the sample order) and, in the first of them, dbh; those of the second
// row the column sums of dZ_L (the layer's bias gradient).  K and N multiples of 256; chunks are
// whole pairs of stages (rows % 128 == 0).
// ---------------------------------------------------------------------------
struct GemmTnTopArgs {
    int M, K, N, splits, rows, tiles_i, NH, NHP;
    const uint16_t* xP;       // packed h_{L-1}: [M/8][K][8]
    const uint16_t* hTop;     // packed h_L: [M/8][N][8]
    const float* dhead;       // [M][NHP]
    const uint16_t* wh16;     // bf16 copy of Wh: [N][NH]
    float* partial;           // [splits][split_stride]: K x N partial, then the N column sums
    size_t split_stride;
    float* head_partial;      // [splits][head_stride]: N x NH partial of dWh, then dbh
    size_t head_stride;
};

__global__ __launch_bounds__(BIGWG) void gemm_tn_bf16_top(const GemmTnTopArgs a)
{
    extern __shared__ uint4 smem4[];         // [2 stages][X | Y][TB_BG][256] pieces of 8 samples
    __shared__ uint4 Ahl[2][2][64];          // [stage parity][32-sample tile]: d as (hi, lo), the A operand of the dZ_L product
    __shared__ uint4 Bhl[2][2][2][64];       // [stage parity][tile][16-sample step]: the same as the B operand of the dWh product
    __shared__ uint4 WhB[256];               // row j0 + c of Wh, eight entries (zero past NH)
    // everything derived from the thread index is worked out again at the start of every step from a value the
    // compiler cannot see through (derive): the dozen loop-invariant addresses it would otherwise keep in registers
    // across the whole loop do not fit beside the accumulators, and a spilled register is reloaded through the same
    // in-order counter as the staged loads, which would end their look-ahead
    int tid = threadIdx.x, lane, wave, wm, wn, l32, kg, lc, lg, col, ds, dk;
    auto derive = [&]() {
        asm volatile("" : "+v"(tid));
        lane = tid & 63; wave = tid >> 6; wm = wave >> 2; wn = wave & 3; l32 = lane & 31; kg = lane >> 5;
        lc = tid & 255; lg = tid >> 8;                           // X loader: (row of the tile, parity of the sample group)
        col = wave * 32 + l32;                                   // dZ_L: this lane's column of the tile
        ds = tid >> 3; dk = tid & 7;                             // head gradient: (sample of the stage, head output)
    };
    derive();
    int split, tile;
    xcd_map((int)blockIdx.x, a.splits, a.tiles_i * (a.N / 256), split, tile);
    const int ti = tile % a.tiles_i, tj = tile / a.tiles_i;
    const int i0 = ti * 256, j0 = tj * 256;
    const int n_stages = a.rows >> 6;
    const int g_first = (split * a.rows) >> 3;
    // extras, one kind per row of tiles so that no workgroup carries both: the first row adds up dWh (and dbh), the
    // second (the first, if there is only one) the column sums of dZ_L
    const bool heads_row = ti == 0, sums_row = ti == (a.tiles_i > 1 ? 1 : 0);
    struct Set { u32x4_l x[TB_BG / 2]; u32x2_l hq[TB_BG]; float d; };
    Set S0, S1;
    auto fetch = [&](Set& st, int i) {
        if (i >= n_stages) i = n_stages - 1;                     // past the end: re-read the last stage, never used
        const int g0 = g_first + i * TB_BG;
        // the head gradient first: it is needed one step before the rest of the set, and loads complete in issue order
        st.d = dk < a.NH ? a.dhead[((size_t)g0 * 8 + ds) * a.NHP + dk] : 0.0f;
#pragma unroll
        for (int q = 0; q < TB_BG / 2; ++q)
            st.x[q] = *reinterpret_cast<const u32x4_l*>(a.xP + ((size_t)(g0 + 2 * q + lg) * a.K + i0 + lc) * 8);
#pragma unroll
        for (int G = 0; G < TB_BG; ++G)
            st.hq[G] = *reinterpret_cast<const u32x2_l*>(a.hTop + ((size_t)(g0 + G) * a.N + j0 + col) * 8 + 4 * kg);
    };
    float bsum = 0.0f, dbsum = 0.0f;
    f16v acc2;
#pragma unroll
    for (int r = 0; r < 16; ++r) acc2[r] = 0.0f;
    // the head gradient of a stage -> both operand forms, into the buffers of parity par
    auto stage_d = [&](const Set& st, int par) {
        const uint16_t hi = (uint16_t)cvt_pk_bf16(st.d, 0.0f);
        const uint16_t lo = (uint16_t)cvt_pk_bf16(st.d - bfu(hi), 0.0f);
        const int mt = ds >> 5, s32 = ds & 31;
        uint16_t* A16 = reinterpret_cast<uint16_t*>(&Ahl[par][mt][0]);
        A16[s32 * 8 + dk] = hi;
        A16[256 + s32 * 8 + dk] = lo;
        const int g = s32 >> 3, r = s32 & 7, kgs = r >> 2, q = (g & 1) * 4 + (r & 3);
        uint16_t* B16 = reinterpret_cast<uint16_t*>(&Bhl[par][mt][g >> 1][0]);
        B16[(kgs * 32 + dk) * 8 + q] = hi;
        B16[(kgs * 32 + 8 + dk) * 8 + q] = lo;
    };
    // part k (0..3) of putting stage i (held in st) into half nb of LDS: X piece k; k even: the dWh MFMAs of 32-sample
    // tile k / 2; k odd: dZ_L of tile k / 2 (one MFMA, masked, to the Y operand).  counted: a real stage, whose
    // values go into the sums (the last step stores the last stage once more)
    auto store_part = [&](const Set& st, int i, int nb, int k, bool counted) {
        uint4* Xs = smem4 + nb * (2 * TB_BG * 256);
        uint4* Ys = Xs + TB_BG * 256;
        const int par = i & 1, mt = k >> 1;
        *reinterpret_cast<u32x4_l*>(&Xs[(2 * k + lg) * 256 + lc]) = st.x[k];
        if ((k & 1) == 0) {
            if (heads_row && counted) {
                const uint4 b0v = Bhl[par][mt][0][lane], b1v = Bhl[par][mt][1][lane];
                u32x4_l x0, x1;
                x0[0] = st.hq[4 * mt][0]; x0[1] = st.hq[4 * mt][1]; x0[2] = st.hq[4 * mt + 1][0]; x0[3] = st.hq[4 * mt + 1][1];
                x1[0] = st.hq[4 * mt + 2][0]; x1[1] = st.hq[4 * mt + 2][1]; x1[2] = st.hq[4 * mt + 3][0]; x1[3] = st.hq[4 * mt + 3][1];
                acc2 = mfma_bf16(*reinterpret_cast<const bf8*>(&x0), *reinterpret_cast<const bf8*>(&b0v), acc2);
                acc2 = mfma_bf16(*reinterpret_cast<const bf8*>(&x1), *reinterpret_cast<const bf8*>(&b1v), acc2);
            }
            return;
        }
        const uint4 wv = WhB[col];
        const uint4 a1v = Ahl[par][mt][lane];
        f16v acc1;
#pragma unroll
        for (int r = 0; r < 16; ++r) acc1[r] = 0.0f;
        acc1 = mfma_bf16(*reinterpret_cast<const bf8*>(&a1v), *reinterpret_cast<const bf8*>(&wv), acc1);
        float part = 0.0f;
#pragma unroll
        for (int g = 0; g < 4; ++g) {
            const int G = 4 * mt + g;
            u32x2_l pv;
            pv[0] = cvt_pk_bf16(acc1[4 * g], acc1[4 * g + 1]) & positive_mask_pk(st.hq[G][0]);
            pv[1] = cvt_pk_bf16(acc1[4 * g + 2], acc1[4 * g + 3]) & positive_mask_pk(st.hq[G][1]);
            *reinterpret_cast<u32x2_l*>(reinterpret_cast<char*>(&Ys[G * 256 + col]) + 8 * kg) = pv;
            if (sums_row) part += (bfu((uint16_t)pv[0]) + bfu((uint16_t)(pv[0] >> 16))) + (bfu((uint16_t)pv[1]) + bfu((uint16_t)(pv[1] >> 16)));
        }
        if (sums_row && counted) bsum += part;
    };
    f16v acc[4][2];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.0f;
    // MFMA step ks (16 samples = groups ks, ks + 1) on half cb of LDS
    auto compute_step = [&](int cb, int ks) {
        const uint4* Xs = smem4 + cb * (2 * TB_BG * 256);
        const uint4* Ys = Xs + TB_BG * 256;
        bf8 bv[2];
#pragma unroll
        for (int t = 0; t < 2; ++t) bv[t] = *reinterpret_cast<const bf8*>(&Ys[(ks + kg) * 256 + wn * 64 + 32 * t + l32]);
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const bf8 av = *reinterpret_cast<const bf8*>(&Xs[(ks + kg) * 256 + wm * 128 + 32 * i + l32]);
#pragma unroll
            for (int j = 0; j < 2; ++j) acc[i][j] = mfma_bf16(av, bv[j], acc[i][j]);
        }
    };
    // one step: the MFMAs of stage i on half i % 2 of LDS with the four parts of stage i + 1 (held in `nxt`) between
    // them; the head gradient of stage i + 2 (held in `aft`) goes to the operand buffers stage i used; then `nxt` is
    // refilled with stage i + 3
    auto step = [&](Set& nxt, const Set& aft, int i) {
        derive();
        const int cb = i & 1;
        const bool counted = i + 1 < n_stages;
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            store_part(nxt, i + 1, cb ^ 1, k, counted);
            __builtin_amdgcn_sched_barrier(0);
            compute_step(cb, 2 * k);
            __builtin_amdgcn_sched_barrier(0);
        }
        stage_d(aft, cb);
        if (i + 2 < n_stages) dbsum += aft.d;
        fetch(nxt, i + 3);
        __syncthreads();
    };
    fetch(S0, 0);                                             // in this order (see gemm_tn_bf16_big)
    __builtin_amdgcn_sched_barrier(0);
    fetch(S1, 1);
    __builtin_amdgcn_sched_barrier(0);
    if (tid < 256) {
        uint32_t w8[8];
#pragma unroll
        for (int k = 0; k < 8; ++k) w8[k] = k < a.NH ? (uint32_t)a.wh16[(size_t)(j0 + tid) * a.NH + k] : 0u;
        WhB[tid] = make_uint4(w8[0] | (w8[1] << 16), w8[2] | (w8[3] << 16), w8[4] | (w8[5] << 16), w8[6] | (w8[7] << 16));
    }
    reinterpret_cast<uint4*>(Bhl)[tid] = make_uint4(0, 0, 0, 0);  // output columns 16..31 of the dWh product stay zero
    __syncthreads();
    stage_d(S0, 0); stage_d(S1, 1);
    dbsum += S0.d + S1.d;
    __syncthreads();
#pragma unroll
    for (int k = 0; k < 4; ++k) store_part(S0, 0, 0, k, true);
    __builtin_amdgcn_sched_barrier(0);
    fetch(S0, 2);
    __syncthreads();
    for (int i = 0; i < n_stages; i += 2) {                   // no branch between the two steps (see gemm_tn_bf16_big)
        step(S1, S0, i);
        step(S0, S1, i + 1);
    }
    float* out = a.partial + (size_t)split * a.split_stride;
#pragma unroll
    for (int tr = 0; tr < 4; ++tr)
#pragma unroll
        for (int tc = 0; tc < 2; ++tc) {
            const int j = j0 + wn * 64 + tc * 32 + l32;
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int i = i0 + wm * 128 + tr * 32 + 8 * (r >> 2) + 4 * kg + (r & 3);
                out[(size_t)i * a.N + j] = acc[tr][tc][r];
            }
        }
    if (!heads_row && !sums_row) return;
    // column sums: the two lanes of a column add up in a fixed order; dWh: accumulator rows are columns j of the
    // tile, accumulator columns k (hi terms) and 8 + k (lo terms)
    float* red = reinterpret_cast<float*>(smem4);               // [256]
    float* Sw = red + 256;                                      // [256 columns][16]
    float* Sd = Sw + 256 * 16;                                  // [64 samples][8]
    if (sums_row && kg == 1) red[col] = bsum;
    if (heads_row) {
        if (l32 < 16) {
#pragma unroll
            for (int r = 0; r < 16; ++r) Sw[(wave * 32 + 8 * (r >> 2) + 4 * kg + (r & 3)) * 16 + l32] = acc2[r];
        }
        Sd[ds * 8 + dk] = dbsum;
    }
    __syncthreads();
    if (sums_row && kg == 0) out[(size_t)a.K * a.N + j0 + col] = bsum + red[col];
    if (!heads_row) return;
    float* hout = a.head_partial + (size_t)split * a.head_stride;
    if (tid < 256)
        for (int k = 0; k < a.NH; ++k) hout[(size_t)(j0 + tid) * a.NH + k] = Sw[tid * 16 + k] + Sw[tid * 16 + 8 + k];
    if (tj == 0 && tid < a.NH) {
        float sum = 0.0f;
        for (int i = 0; i < 64; ++i) sum += Sd[i * 8 + tid];
        hout[(size_t)a.N * a.NH + tid] = sum;
    }
}

// ---------------------------------------------------------------------------
// Maze first layer.  The observation has three one-hot planes (paper section 2.1 style grid
// world: walls, agent, goal) and only the agent plane changes within an unroll, so
//   dW1[wall cell c]  = sum_b walls[b][c] * S[b],   S[b] = sum_t dZ1[t][b]   (B samples, not B*T)
//   dW1[agent cell c] = sum_m [pos_m == c] dZ1[m]                             (the only full-length product)
//   dW1[goal cell]    = db1 = sum_b S[b]  for the one goal cell, zero for the others
// S leaves as two bfloat16 terms (hi rows 0..B-1, lo rows B..2B-1 of a packed matrix with 2B
// samples) and the wall product runs over those 2B samples.  The agent product reads every dZ1
// entry anyway and writes S itself when its chunks are blocks of environments; time_sum_bf16 is
// the separate pass for batch sizes that do not divide that way.
// ---------------------------------------------------------------------------
__global__ __launch_bounds__(WG) void time_sum_bf16(const uint16_t* __restrict__ dzP, uint16_t* __restrict__ sP, int B, int T, int H)
{
    const size_t idx = (size_t)blockIdx.x * WG + threadIdx.x;          // (env group, column)
    const size_t n = (size_t)(B >> 3) * H;
    if (idx >= n) return;
    float s[8] = {0, 0, 0, 0, 0, 0, 0, 0};
#pragma unroll 8
    for (int t = 0; t < T; ++t) {
        const uint4 v = *reinterpret_cast<const uint4*>(dzP + ((size_t)t * n + idx) * 8);
        const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
        for (int e = 0; e < 8; ++e) s[e] += bfu((uint16_t)((w[e >> 1] >> ((e & 1) * 16)) & 0xffffu));
    }
    uint32_t hi[4], lo[4];
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        hi[q] = cvt_pk_bf16(s[2 * q], s[2 * q + 1]);
        lo[q] = cvt_pk_bf16(s[2 * q] - bfu((uint16_t)hi[q]), s[2 * q + 1] - bfu((uint16_t)(hi[q] >> 16)));
    }
    *reinterpret_cast<uint4*>(sP + idx * 8) = make_uint4(hi[0], hi[1], hi[2], hi[3]);
    *reinterpret_cast<uint4*>(sP + (n + idx) * 8) = make_uint4(lo[0], lo[1], lo[2], lo[3]);
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
// Rows of dZ_l (samples) one workgroup of the weights-resident bf16 dX kernel walks, in stages of NRES_RT rows;
// 0 when the layer's shape goes to the tiled kernel instead.  At most 256 row ranges per 256-column block of W.
int bf16_dx_rows_per_workgroup(int M, int K, int N)
{
    if (!((N == 256 || N == 512) && K % 256 == 0 && M % NRES_RT == 0)) return 0;
    const int tiles = M / NRES_RT;
    const int blocks = tiles < 256 ? tiles : 256;
    return ((tiles + blocks - 1) / blocks) * NRES_RT;
}

// Whether the dX product of layer l + 1 (reading dZ_l, l >= 1) runs as the weights-resident kernel.  That kernel reads
// and writes the packed layout only, so it is used only where the product below it (which reads its output) does too.
bool bf16_dx_resident(const NetShape& n, int M, int l)
{
    if (l < 1 || l >= n.L) return false;
    if (bf16_dx_rows_per_workgroup(M, n.dims[l], n.dims[l + 1]) == 0) return false;
    return l == 1 || bf16_dx_resident(n, M, l - 1);
}

// Whether the top layer's products form dZ_L themselves (no head pass, no dZ_L in memory): both sides of the layer
// multiples of 256, the dX product weights-resident, chunks of whole 64-sample stages.
bool bf16_top_fused(const NetShape& n, int M, int splits_top)
{
    if (!n.bf16 || n.L < 2 || n.NH > 8) return false;
    if (n.dims[n.L] % 256 != 0 || n.dims[n.L - 1] % 256 != 0) return false;
    if (!bf16_dx_resident(n, M, n.L - 1)) return false;
    return splits_top > 0 && M % splits_top == 0 && (M / splits_top) % 128 == 0;
}

hipError_t launch_backward_bf16(anakin* h)
{
    const Layout& L = h->lay;
    const NetShape& n = h->net;
    const int M = h->B * h->T;
    hipError_t e;
    auto dzR = [&](int l) { return at<uint16_t>(h, L.dz[l]); };
    auto dzP = [&](int l) { return at<uint16_t>(h, L.dz[l]) + (size_t)M * n.dims[l + 1]; };
    auto actP = [&](int l) { return at<uint16_t>(h, L.act[l]); };
    // dZ_l is kept sample-packed; the row-major copy exists only where the tiled dX kernel of layer l + 1 reads it
    auto needs_rows = [&](int l) { return l >= 1 && !bf16_dx_resident(n, M, l); };
    const bool top_fused = bf16_top_fused(n, M, h->splits[n.L - 1]) && h->splits[n.L] == h->splits[n.L - 1] && h->head_fan == 1;
    if (!top_fused) {   // heads
        HeadBwdBf16Args a;
        a.M = M; a.H = n.dims[n.L]; a.NH = n.NH; a.NHP = n.NHP;
        const int stage1 = h->splits[n.L] * h->head_fan;
        a.rows = M / stage1;
        a.hP = actP(n.L - 1); a.dhead = at<const float>(h, L.dhead);
        a.wh16 = at<const uint16_t>(h, L.w16_src) + n.wh_off;
        a.dzR = needs_rows(n.L - 1) ? dzR(n.L - 1) : nullptr; a.dzP = dzP(n.L - 1);
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
    auto obs_src = [&]() {
        ObsSrc o;
        o.kind = h->env.kind; o.env = h->env; o.B = h->B;
        o.s0 = at<const uint32_t>(h, L.tr_s0); o.f0 = at<const float>(h, L.tr_f0);
        o.f1 = at<const float>(h, L.tr_f1); o.walls = at<const uint32_t>(h, L.walls);
        return o;
    };
    // dW partials of one product; big: 256 x 256 tiles
    auto run_tn = [&](GemmTnBf16Args& t, bool big, const char* name) -> hipError_t {
        const int tile = big ? 256 : 128;
        t.tiles_i = (t.K + tile - 1) / tile;
        const int tiles = t.tiles_i * ((t.N + tile - 1) / tile);
        const dim3 grid = big ? dim3(tiles * t.splits) : dim3(tiles, t.splits);
        const size_t lds = (size_t)2 * (big ? 2 * TB_BG * 256 : TB_G * 128) * sizeof(uint4);   // 256-tile kernel: two stages
        // X operand of the 256-tile kernel: packed activations, the agent plane (one-hot of the cell), or generic rows
        const int cells = h->env.rows * h->env.cols;
        const int xmode = !t.use_obs ? 0 : (h->env.kind == ENV_MAZE && t.obs_row0 == cells && t.K == cells) ? 1 : 2;
        if (big && xmode == 2 && !(h->env.kind == ENV_MAZE && t.obs_row0 == 0 && t.K == cells && h->B % 64 == 0)) return hipErrorInvalidValue;
        const void* fn = big ? (xmode == 0 ? reinterpret_cast<const void*>(gemm_tn_bf16_big<0>) : xmode == 1 ? reinterpret_cast<const void*>(gemm_tn_bf16_big<1>)
                                                                                                              : reinterpret_cast<const void*>(gemm_tn_bf16_big<2>))
                             : (t.use_obs ? reinterpret_cast<const void*>(gemm_tn_bf16<true>) : reinterpret_cast<const void*>(gemm_tn_bf16<false>));
        hipError_t e2 = hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e2 != hipSuccess) return e2;
        ProfScope prof(h, name);
        if (big) {
            if (xmode == 0) hipLaunchKernelGGL(gemm_tn_bf16_big<0>, grid, dim3(BIGWG), lds, h->stream, t);
            else if (xmode == 1) hipLaunchKernelGGL(gemm_tn_bf16_big<1>, grid, dim3(BIGWG), lds, h->stream, t);
            else hipLaunchKernelGGL(gemm_tn_bf16_big<2>, grid, dim3(BIGWG), lds, h->stream, t);
        } else {
            if (t.use_obs) hipLaunchKernelGGL(gemm_tn_bf16<true>, grid, dim3(WG), lds, h->stream, t);
            else hipLaunchKernelGGL(gemm_tn_bf16<false>, grid, dim3(WG), lds, h->stream, t);
        }
        return hipGetLastError();
    };
    for (int l = n.L - 1; l >= 0; --l) {
        if (l == 0 && first_layer_split(h)) {
            const int H1 = n.dims[1], cells = h->env.rows * h->env.cols, plane = cells * H1;
            uint16_t* sP = at<uint16_t>(h, L.prefix);                // B x H1 words, free between unrolls
            float* pw = at<float>(h, L.part[0]);
            float* pa = pw + (size_t)plane * h->splits_w;
            float* pg = pa + (size_t)plane * h->splits[0];
            // the agent product adds dZ1 up over time on its way when its chunks can be blocks of 64 k environments
            const bool sum_in_product = h->B % (64 * h->splits[0]) == 0;
            if (!sum_in_product) {
                ProfScope prof(h, "time_sum");
                hipLaunchKernelGGL(time_sum_bf16, dim3(((h->B >> 3) * H1 + WG - 1) / WG), dim3(WG), 0, h->stream,
                                   dzP(0), sP, h->B, h->T, H1);
                if ((e = hipGetLastError()) != hipSuccess) return e;
            }
            GemmTnBf16Args t;
            t.M = M; t.K = cells; t.N = H1; t.splits = h->splits[0]; t.rows = t.M / t.splits;
            t.use_obs = 1; t.obs_row0 = cells; t.xP = nullptr; t.dyP = dzP(0);
            t.partial = pa; t.split_stride = (size_t)plane; t.bias_out = nullptr; t.bias_stride = 0;
            t.obs = obs_src();
            t.sP = sum_in_product ? sP : nullptr; t.T = h->T; t.env_block = h->B / h->splits[0];
            if ((e = run_tn(t, true, "gemm_tn_agent")) != hipSuccess) return e;
            t.M = 2 * h->B; t.splits = h->splits_w; t.rows = t.M / t.splits;
            t.obs_row0 = 0; t.dyP = sP;
            t.partial = pw; t.bias_out = pg; t.bias_stride = (size_t)H1;
            t.sP = nullptr;
            if ((e = run_tn(t, true, "gemm_tn_walls")) != hipSuccess) return e;
            continue;
        }
        GemmTnBf16Args t;
        t.M = M; t.K = n.dims[l]; t.N = n.dims[l + 1];
        t.splits = h->splits[l]; t.rows = M / t.splits;
        t.use_obs = (l == 0); t.obs_row0 = 0;
        t.xP = l > 0 ? actP(l - 1) : nullptr;
        t.dyP = dzP(l);
        t.partial = at<float>(h, L.part[l]);
        t.split_stride = (size_t)t.K * t.N + t.N;
        t.bias_out = t.partial + (size_t)t.K * t.N; t.bias_stride = t.split_stride;
        t.obs = obs_src();
        t.sP = nullptr; t.T = h->T; t.env_block = 0;
        const bool big = l > 0 && t.K % 256 == 0 && t.N % 256 == 0 && t.M % t.splits == 0 && t.rows % 128 == 0;
        if (l == n.L - 1 && top_fused) {
            GemmTnTopArgs u;
            u.M = M; u.K = t.K; u.N = t.N; u.splits = t.splits; u.rows = t.rows; u.tiles_i = t.K / 256;
            u.NH = n.NH; u.NHP = n.NHP;
            u.xP = t.xP; u.hTop = actP(l); u.dhead = at<const float>(h, L.dhead);
            u.wh16 = at<const uint16_t>(h, L.w16_src) + n.wh_off;
            u.partial = t.partial; u.split_stride = t.split_stride;
            u.head_partial = at<float>(h, L.part[n.L]); u.head_stride = (size_t)t.N * n.NH + n.NH;
            const size_t lds = (size_t)2 * 2 * TB_BG * 256 * sizeof(uint4);   // two stages
            if ((e = hipFuncSetAttribute(reinterpret_cast<const void*>(gemm_tn_bf16_top), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds)) != hipSuccess) return e;
            ProfScope prof(h, "gemm_tn_top");
            hipLaunchKernelGGL(gemm_tn_bf16_top, dim3(u.tiles_i * (u.N / 256) * u.splits), dim3(BIGWG), lds, h->stream, u);
            if ((e = hipGetLastError()) != hipSuccess) return e;
        } else if ((e = run_tn(t, big, l == 0 ? "gemm_tn_obs" : "gemm_tn")) != hipSuccess) return e;
        if (l > 0) {
            GemmNtBf16Args g;
            g.M = M; g.K = n.dims[l]; g.N = n.dims[l + 1];
            g.dyR = needs_rows(l) ? dzR(l) : nullptr;
            g.dyP = dzP(l);
            g.w16 = at<const uint16_t>(h, L.w16_src) + n.w_off[l];
            g.hP = actP(l - 1);
            g.dxR = needs_rows(l - 1) ? dzR(l - 1) : nullptr;
            g.dxP = dzP(l - 1);
            const int rows_per_block = bf16_dx_rows_per_workgroup(g.M, g.K, g.N);
            ProfScope prof(h, "gemm_nt_mask");
            if (bf16_dx_resident(n, M, l)) {
                const size_t lds2 = (size_t)2 * NRES_RT * (g.N + 8) * sizeof(uint16_t);
                const bool top = l == n.L - 1 && top_fused;      // dZ_L comes out of the head gradient inside the kernel
                g.maskTop = at<const uint32_t>(h, L.mask[l]); g.dhead = at<const float>(h, L.dhead);
                // the mask of the layer below as flag words where the acting kernel writes them (every layer it runs
                // on the matrix cores; the first layer only at 512 columns)
                g.maskLo = (l - 1 >= 1 || n.dims[1] == 512) ? at<const uint32_t>(h, L.mask[l - 1]) : nullptr;
                g.wh16 = at<const uint16_t>(h, L.w16_src) + n.wh_off; g.NH = n.NH; g.NHP = n.NHP;
                const void* fn = g.N == 512 ? (top ? reinterpret_cast<const void*>(gemm_nt_bf16_res<512, true>) : reinterpret_cast<const void*>(gemm_nt_bf16_res<512, false>))
                                            : (top ? reinterpret_cast<const void*>(gemm_nt_bf16_res<256, true>) : reinterpret_cast<const void*>(gemm_nt_bf16_res<256, false>));
                e = hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds2);
                if (e != hipSuccess) return e;
                const dim3 grid(((g.M + rows_per_block - 1) / rows_per_block) * (g.K / 256));
                if (g.N == 512 && top) hipLaunchKernelGGL((gemm_nt_bf16_res<512, true>), grid, dim3(NRES_WG), lds2, h->stream, g, rows_per_block);
                else if (g.N == 512) hipLaunchKernelGGL((gemm_nt_bf16_res<512, false>), grid, dim3(NRES_WG), lds2, h->stream, g, rows_per_block);
                else if (top) hipLaunchKernelGGL((gemm_nt_bf16_res<256, true>), grid, dim3(NRES_WG), lds2, h->stream, g, rows_per_block);
                else hipLaunchKernelGGL((gemm_nt_bf16_res<256, false>), grid, dim3(NRES_WG), lds2, h->stream, g, rows_per_block);
            } else {
                const size_t lds2 = (size_t)2 * 128 * NB_LD * sizeof(uint16_t);
                e = hipFuncSetAttribute(reinterpret_cast<const void*>(gemm_nt_bf16), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds2);
                if (e != hipSuccess) return e;
                hipLaunchKernelGGL(gemm_nt_bf16, dim3(((g.M + 127) / 128) * ((g.K + 127) / 128)), dim3(WG), lds2, h->stream, g);
            }
            if ((e = hipGetLastError()) != hipSuccess) return e;
        }
    }
    return hipSuccess;
}

}  // namespace ank
