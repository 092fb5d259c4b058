// Host-side handle, device workspace layout and kernel argument blocks shared by
// the translation units of libanakin.  Nothing here is part of the public ABI.
#pragma once
#include <stdint.h>
#include <stddef.h>
#include <string>
#include <vector>
#include <hip/hip_runtime.h>
#include "env.h"
#include "../../include/anakin.h"

namespace ank {

constexpr int MAX_LAYERS = 4;
constexpr int MAX_REGIONS = MAX_LAYERS + 1;      // one (W,b) pair per hidden layer + the heads
constexpr int MAX_ADAM_REGIONS = MAX_REGIONS + 4; // the maze first layer of a bf16 net is reduced in five pieces
constexpr int WG = 256;                          // threads per workgroup everywhere

// network shape and parameter offsets (elements into theta)
struct NetShape {
    int D, A, NH, NHP, L;
    int dims[MAX_LAYERS + 2];                    // D, H1..HL
    int w_off[MAX_LAYERS], b_off[MAX_LAYERS], wh_off, bh_off;
    int P;
    int policy, bf16;
};

// trajectory and env-state pointers (device)
struct TrajPtrs {
    uint32_t* s0; float* f0; float* f1; const uint32_t* walls;        // current env state; walls [8][B]
    uint32_t* tr_s0; float* tr_f0; float* tr_f1;                       // [T+1][B] state observed at t
    uint8_t* tr_act; float* tr_eps; float* tr_actf;                    // [T][B]
    float* tr_rew; uint8_t* tr_done;                                   // [T][B]
    float* tr_val;                                                     // [T+1][B]
    float* tr_head;                                                    // [T+1][B][NHP]
    float* act[MAX_LAYERS];                                            // [T*B][H_l] hidden activations
    uint32_t* mask[MAX_LAYERS];                                        // bf16 matrix-core path: which of them are positive, see relu_mask_index
};

// ReLU masks of the bf16 matrix-core path, written by the acting kernels beside the packed activations and read by
// the dX products of the update in place of the activations themselves (1/8 of the bytes).  One 32-bit word per
// (stage of 32 consecutive samples, half kg of the accumulator rows, column): [M/32][2][H].  Lane (column, kg) of a
// 32 x 32 MFMA accumulator tile holds rows 8g + 4kg + q (g, q = 0..3) as value r = 4g + q; bit relu_mask_bit(r) of
// its word says that this activation is positive.  (Values come in packed pairs; pair r/2 puts the flag of its low
// half in bit r/2 and of its high half in bit 16 + r/2, which costs the producer two instructions per pair.)
ANK_HD size_t relu_mask_index(size_t stage, int kg, int H, int col) { return (stage * 2 + (size_t)kg) * (size_t)H + (size_t)col; }
ANK_HD int relu_mask_bit(int r) { return (r >> 1) + 16 * (r & 1); }

struct RolloutArgs {
    EnvDims env;
    NetShape net;
    TrajPtrs tp;
    const float* theta;
    int B, T, ldx;
    int keep_acts;               // store hidden activations for the update (0: the update rebuilds them)
    uint64_t seed, gstep;
};

// position of parameter i in the copy that stores every weight matrix transposed
// (layers [N][K], heads [NH][HL]); biases keep their place
// Layout of the second bf16 copy of the parameters, the one the acting kernel feeds to
// v_mfma_f32_32x32x16_bf16 as the B operand.  A weight matrix W[K][N] with K % 16 == 0 and
// N % 32 == 0 is stored in operand tiles: for every block of 32 output columns and every
// step of 16 inputs, the 64 lanes' 16-byte pieces are adjacent (lane = 32*((k%16)/8) + n%32
// holds k%8 = 0..7), so one wavefront load is one contiguous KiB.  Other layer matrices are
// stored transposed ([N][K]); the head matrix as [NH][HL].
ANK_HD bool mfma_tiled(int K, int N) { return K % 16 == 0 && N % 32 == 0; }
ANK_HD int tiled_offset(int K, int k, int n)
{
    return (((n >> 5) * (K >> 4) + (k >> 4)) << 9) + (((((k & 15) >> 3) << 5) + (n & 31)) << 3) + (k & 7);
}
ANK_HD int transposed_index(const NetShape& n, int i)
{
    for (int l = 0; l < n.L; ++l) {
        const int K = n.dims[l], N = n.dims[l + 1], off = i - n.w_off[l];
        if (off >= 0 && off < K * N)
            return n.w_off[l] + (mfma_tiled(K, N) ? tiled_offset(K, off / N, off % N) : (off % N) * K + off / N);
    }
    const int off = i - n.wh_off, HL = n.dims[n.L];
    if (off >= 0 && off < HL * n.NH) return n.wh_off + (off % n.NH) * HL + off / n.NH;
    return i;
}

// Workgroup L of a 1-D grid runs on XCD L % 8 (round-robin dispatch) and each XCD has its own L2.
// Map L to (outer, inner) so that the n_inner workgroups sharing one `outer` (the same operand
// tile) run back to back on one XCD and the second reader hits in that L2.
__device__ __forceinline__ void xcd_map(int L, int n_outer, int n_inner, int& outer, int& inner)
{
    const int whole = (n_outer >> 3) << 3, full = whole * n_inner;
    if (L < full) { const int q = L >> 3; inner = q % n_inner; outer = (q / n_inner) * 8 + (L & 7); }
    else { const int r = L - full; outer = whole + r / n_inner; inner = r % n_inner; }
}

// state snapshots the first layer's input is rebuilt from (row m = t*B + b of the trajectory)
struct ObsLite { EnvDims env; const uint32_t* s0; const float* f0; const float* f1; };

// split-K partial sums of one parameter region (W_l followed by b_l, or Wh followed by bh)
struct Region { int start, count, splits; const float* partial; };

struct AdamArgs {
    Region reg[MAX_ADAM_REGIONS];
    int n_regions, P;
    float* theta; float* grad; float* m; float* v;
    uint16_t* w_bf16;            // bf16 copy of theta (same indexing), or null
    uint16_t* wt_bf16;           // bf16 copy with every weight matrix transposed, or null
    NetShape net;
    float lr, beta1, beta2, eps, bc1, bc2;
};

struct Layout {
    size_t theta, grad, m, v, w_bf16, wt_bf16;
    size_t theta0, w0_bf16;      // copies of theta / w_bf16 taken before the first of several updates on one unroll
    size_t w_src, w16_src;       // where the backward kernels read weights: theta / w_bf16, or the copies
    size_t s0, f0, f1, walls;
    size_t tr_s0, tr_f0, tr_f1, tr_act, tr_eps, tr_actf, tr_rew, tr_done, tr_val, tr_head;
    size_t adv, ret, dhead;
    size_t act[MAX_LAYERS], dz[MAX_LAYERS];
    size_t mask[MAX_LAYERS];      // bf16 matrix-core path: ReLU masks, inside the unused upper half of act[l]
    size_t part[MAX_REGIONS];
    size_t head_stage;           // first-stage partials of the head gradient
    size_t prefix;               // bf16 acting: per-env first-layer prefix [B][H1] fp32
    size_t loss_part;
    // decoupled acting and learning: the behaviour copy of the parameters the actor runs on, the second set of
    // trajectory records (the actor fills one set while the learner reads the other), and the learner's own
    // forward results on the stored unroll
    size_t theta_b, w_bf16_b, wt_bf16_b, prefix_b;      // bf16 nets: the actor's own rounded copies and first-layer prefix
    size_t alt_tr_s0, alt_tr_f0, alt_tr_f1, alt_tr_act, alt_tr_eps, alt_tr_actf, alt_tr_rew, alt_tr_done, alt_tr_val, alt_tr_head;
    size_t head_new, val_new, eps_new;
    size_t small_part;           // single-launch update of small nets: one whole gradient per workgroup, [workgroups][P]
    size_t counters;             // arrival counters of kernels whose last workgroup finishes the job (zero between launches)
    size_t path;                 // pathwise policy gradient: dL_path / d(mu, log_sigma) per sample, [T*B][2]
    size_t total;
};

}  // namespace ank

struct anakin {
    anakin_env_cfg env_cfg;
    anakin_net_cfg net_cfg;
    ank::EnvDims env;
    ank::NetShape net;
    int B, T;
    uint64_t seed, gstep;
    int adam_t;
    int have_traj;
    int mode;
    char* ws;
    size_t ws_bytes;
    char* scratch;                // base of tagged offsets (see SCRATCH_TAG); null outside anakin_learn_static
    int device;                   // the device the workspace lives on
    hipStream_t stream;
    ank::Layout lay;
    int TM;                       // envs per workgroup in the vector-ALU rollout kernel
    int TM_mfma;                  // envs per workgroup in the matrix-core rollout kernel (0: not applicable)
    int TM_res;                   // envs per workgroup in the weights-resident rollout kernel (0: not applicable)
    int splits[ank::MAX_REGIONS]; // split-K factor per parameter region
    int loss_blocks;
    int metric_blocks;            // blocks of loss partials the last update wrote (0 before the first)
    int head_fan;                 // first-stage workgroups per split of the head-gradient pass
    int chunks_sequential;        // several updates per unroll: chunk k's gradient at the parameters after k updates (else at the acting ones)
    int n_updates;                // Adam updates per unroll (consecutive time chunks of the unroll), 1 by default
    int sub_splits[ank::MAX_REGIONS], sub_splits_w, sub_head_fan, sub_loss_blocks;   // split plan of one chunk
    int splits_w;                 // maze first layer of a bf16 net: split count of the wall-plane product (0: one product
                                  // over all observation rows); splits[0] is then the split count of the agent-plane product
    int bf16_path;                // the bf16 matrix-core kernels support this net
    int traj_packed;              // the stored unroll holds packed bf16 activations
    int traj_no_acts;             // the stored unroll holds no hidden activations (one-layer nets)
    int pathwise;                 // policy gradient through the environment instead of the score function (pendulum)
    int traj_decoupled;           // the stored unroll was collected by a decoupled step: behaviour parameters, no activations
    hipStream_t actor_stream;     // decoupled steps: the actor's stream (the caller's, or created on first use), and the fork/join events
    int actor_stream_owned;       // the library created actor_stream and destroys it
    hipEvent_t ev_fork, ev_join;
    std::string err;
    // optional per-kernel timing with events on the launch stream
    int prof_on;
    struct ProfPending { int name; hipEvent_t start, stop; };
    struct ProfTotal { std::string name; long long calls; double ms; };
    std::vector<ProfPending> prof_pending;
    std::vector<hipEvent_t> prof_pool;
    std::vector<ProfTotal> prof_totals;
};

namespace ank {

// An offset with this bit set is relative to the handle's update-scratch base instead of the workspace base
// (anakin_learn_static points the backward pass's scratch at the library's own static device array).
constexpr size_t SCRATCH_TAG = (size_t)1 << 62;
template <class T> inline T* at(const anakin* h, size_t off)
{
    return reinterpret_cast<T*>((off & SCRATCH_TAG) ? h->scratch + (off & ~SCRATCH_TAG) : h->ws + off);
}

// per-kernel timing: brackets one launch with two events when profiling is on
struct ProfScope {
    anakin* h; int idx;
    ProfScope(anakin* h_, const char* name);
    ~ProfScope();
};
hipError_t prof_resolve(anakin* h);

// kernel launchers (each enqueues on h->stream and returns the HIP status)
hipError_t launch_rollout(anakin* h);
hipError_t launch_rollout_behaviour(anakin* h);
hipError_t launch_replay_forward(anakin* h);
hipError_t launch_vtrace(anakin* h);
hipError_t launch_eps_now(anakin* h);
hipError_t launch_pathwise(anakin* h);
bool pathwise_ok(const anakin* h);
hipError_t launch_returns(anakin* h);
bool scan_loss_ok(const anakin* h);          // returns and loss as one launch
hipError_t launch_scan_loss(anakin* h);
hipError_t launch_head_grad(anakin* h);
hipError_t launch_backward(anakin* h);
hipError_t launch_adam(anakin* h);
hipError_t launch_first_layer_grad(anakin* h);
hipError_t launch_adam_probe(float* base, int P, hipStream_t s);
hipError_t launch_learn_one_layer(anakin* h);
hipError_t launch_learn_catch_fused(anakin* h);
hipError_t launch_learn_small_fused(anakin* h);
bool small_fused_ok(const anakin* h);
size_t small_fused_part_bytes(const EnvDims& ed, const NetShape& ns, int B, int T);
bool catch_fused_ok(const anakin* h);
// single hidden layer on a one-hot or 3-feature observation: the update rebuilds the layer from the state
inline bool one_layer_fused(const anakin* h) { return h->net.L == 1 && h->env.kind != ENV_MAZE && !h->net.bf16 && !(h->mode & ANAKIN_MODE_VALU_GEMM) && h->net.dims[1] <= 128 && (size_t)128 * h->net.dims[0] * 4 + (size_t)h->net.dims[0] * h->net.dims[1] * 4 <= 64 * 1024; }
hipError_t launch_partial_reduce(const float* src, float* dst, int count, int fan, int splits, hipStream_t s);
hipError_t launch_rollout_bf16(anakin* h);
hipError_t launch_rollout_bf16_behaviour(anakin* h);
hipError_t launch_replay_bf16(anakin* h);
hipError_t launch_backward_bf16(anakin* h);
hipError_t launch_refresh_bf16(anakin* h);
int bf16_dx_rows_per_workgroup(int M, int K, int N);
bool bf16_top_fused(const NetShape& n, int M, int splits_top);
bool bf16_dx_resident(const NetShape& n, int M, int l);
bool rollout_bf16_ok(const NetShape& net, const EnvDims& env, int B);
// bf16 network running on the matrix-core path (packed bf16 activations) rather than the fp32 reference path
// the stored unroll was produced by the bf16 matrix-core kernels and the maze first layer is reduced in pieces
inline bool first_layer_split(const anakin* h) { return h->splits_w > 0 && h->traj_packed; }
inline bool bf16_mfma(const anakin* h) { return h->bf16_path && !(h->mode & (ANAKIN_MODE_CANONICAL_ACTING | ANAKIN_MODE_VALU_GEMM)); }
// the head backward pass can ride in the loaders of the top hidden layer's two resident products: a 256 -> 256 top
// layer, at most four head outputs, sample count in whole 32-row stages
inline bool heads_fused_shape(const NetShape& n, int M) { return !n.bf16 && n.L >= 2 && n.NH <= 4 && n.dims[n.L] == 256 && n.dims[n.L - 1] == 256 && M % 32 == 0; }
// the pendulum's first-layer gradient can ride in the epilogue of the resident dX product that forms dZ_1 (second
// layer n x 256 with n a multiple of 256); returns the number of partials that kernel writes (its workgroups along
// the samples, which must cut the samples evenly so that the chunking also serves the other kernels), else 0
inline int first_fused_splits(const NetShape& n, int env_kind, int M, int tn_splits)
{
    if (env_kind != ENV_PENDULUM || n.bf16 || n.L < 2 || n.dims[0] != 3 || n.dims[1] % 256 != 0 || n.dims[2] != 256 || M % 32 != 0) return 0;
    // a 256 -> 256 second layer shares its launch with the dW kernel, which then leaves it only part of the compute units
    const int cap = n.dims[1] == 256 ? (tn_splits > 0 && tn_splits < 256 ? 256 - tn_splits : 256) : 256;
    const int tiles = M / 32, blocks = tiles < cap ? tiles : cap;
    return tiles % blocks == 0 ? blocks : 0;
}
int rollout_pick_tile(const NetShape& net, int B);
int rollout_pick_tile_mfma(const NetShape& net, int B);
int rollout_resident_tile(const NetShape& net, int env_kind, int B);
size_t rollout_lds_bytes(const NetShape& net, const EnvDims& env, int TM, int* ldx);

}  // namespace ank
