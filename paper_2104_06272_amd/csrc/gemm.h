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

struct GemmNtArgs {
    int M, K, N, bf16;
    HeadFuse hf;
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
