// Argument blocks of the dense-layer backward kernels (vector-ALU and
// matrix-core versions take the same ones).
#pragma once
#include "internal.h"

namespace ank {

// where the first layer's input comes from: the compact state snapshots
struct ObsSrc {
    int kind, B;
    EnvDims env;
    const uint32_t* s0; const float* f0; const float* f1;   // [T+1][B], row m = t*B + b
    const uint32_t* walls;                                   // [8][B]
};

// dX[m][i] = (x[m][i] > 0) * sum_j dY[m][j] W[i][j];  W is [K][N] row-major (K = inputs, N = outputs)
// heads folded into the top hidden layer's products: dY is not read but formed on the way in,
//   dY[m][j] = (hl[m][j] > 0) * sum_a wh[j][a] dhead[m][a]
// from the layer's own forward activations hl, the per-sample head gradient and the head matrix
struct HeadFuse {
    const float* hl;      // [M][N] activations of the top hidden layer (null: dY is read from memory)
    const float* dhead;   // [M][NHP]
    const float* wh;      // [N][NH]
    int NH, NHP;
    float* head_partial;  // dW product only: [splits][N*NH + NH] partial sums of the head matrix and bias gradients
};

// pendulum first layer folded into the dX product that forms dZ_1: dW_1[c][i] = sum_m o_c(m) dZ_1[m][i] for the three
// observation features o = (cos th, sin th, thd) of sample m, db_1[i] = sum_m dZ_1[m][i], one partial per workgroup
// (dZ_1 itself is then not written: nothing else reads it)
struct FirstFuse {
    const float* f0; const float* f1;   // [M] stored angle and angular velocity (null: not folded)
    float* partial;                     // [workgroups][3*K + K]
};
// workgroups (along the samples) the resident dX kernel is launched with: at most `cap`, whole 32-sample stages each
inline int gemm_nt_res_blocks(int M, int cap, int* rows_per_block_out = nullptr)
{
    const int tiles = (M + 31) / 32;
    const int blocks = tiles < cap ? tiles : cap;
    const int rows_per_block = ((tiles + blocks - 1) / blocks) * 32;
    if (rows_per_block_out) *rows_per_block_out = rows_per_block;
    return (M + rows_per_block - 1) / rows_per_block;
}
// In a launch shared with the dW kernel the two kinds of workgroup run side by side, one per compute unit: the dX
// kernel gets the units the dW chunks leave free.
inline int gemm_nt_res_cap(int tn_splits) { return tn_splits > 0 && tn_splits < 256 ? 256 - tn_splits : 256; }

struct GemmNtArgs {
    int M, K, N, bf16;
    HeadFuse hf;
    FirstFuse ff;
    const float* dy;      // [M][N]
    const float* w;       // [K][N]
    const float* x;       // [M][K] forward activations (relu mask)
    float* dx;            // [M][K]
};

// partial[s][i][j] = sum over rows of chunk s of x[m][i] dY[m][j]; partial[s][K*N + j] = column sums of dY
struct GemmTnArgs {
    int M, K, N, ldy, bf16, splits, rows, tiles_i, use_obs;   // ldy: row stride of dy (>= N)
    HeadFuse hf;
    const float* x;       // [M][K], unused when use_obs
    const float* dy;      // [M][N]
    float* partial;       // [splits][K*N + N]
    ObsSrc obs;
};

hipError_t launch_gemm_nt_valu(const GemmNtArgs& a, hipStream_t s);
hipError_t launch_gemm_tn_valu(GemmTnArgs a, hipStream_t s);
hipError_t launch_gemm_nt_mfma(const GemmNtArgs& a, hipStream_t s);
hipError_t launch_gemm_tn_mfma(GemmTnArgs a, hipStream_t s);
// persistent, operand-resident kernels for 256-wide layers
bool gemm_nt_res_ok(const GemmNtArgs& a);
bool gemm_tn_res_ok(const GemmTnArgs& a);
hipError_t launch_gemm_nt_res(const GemmNtArgs& a, hipStream_t s);
hipError_t launch_gemm_tn_res(const GemmTnArgs& a, hipStream_t s);
hipError_t launch_gemm_tn_nt_res(const GemmTnArgs& t, const GemmNtArgs& n, hipStream_t s);   // both products of a layer, one launch

}  // namespace ank
