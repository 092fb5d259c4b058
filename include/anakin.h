/*
 * anakin.h -- C ABI of the MI355X-native Anakin actor-learner step.
 *
 * Anakin (paper section 3.1, "Online Learning with Anakin", and figure 2 top):
 * the environments live on the accelerator next to the agent; one unit of work
 * is T agent-environment interactions (observation -> action -> reward, paper
 * section 2.1) for a batch of B environments, followed by one parameter update
 * that reuses the policy's forward pass.  The host only schedules (section
 * 3.1); state stays in device memory between calls (section 2.3).
 *
 * All functions return 0 (ANAKIN_OK) or a negative ANAKIN_E_* code; nothing
 * throws across this boundary.  Unless a parameter says "host", pointers named
 * d_* are device pointers and h_* are host pointers.  A handle is not
 * thread-safe; distinct handles are independent.
 *
 * Memory ownership: the caller owns the device workspace and the stream.  The
 * library never allocates device memory; it carves the workspace (256-byte
 * alignment) and owns only the small host-side handle.
 */
#ifndef ANAKIN_H
#define ANAKIN_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum {
    ANAKIN_OK = 0,
    ANAKIN_E_INVALID_ARG = -1,         /* null pointer, wrong length */
    ANAKIN_E_BAD_CONFIG = -2,          /* unsupported env / net / B / T */
    ANAKIN_E_WORKSPACE_TOO_SMALL = -3,
    ANAKIN_E_MISALIGNED = -4,          /* workspace not 256-byte aligned */
    ANAKIN_E_HIP = -5,                 /* a HIP runtime call failed; see anakin_last_error */
    ANAKIN_E_NONFINITE = -6,
    ANAKIN_E_STATE = -7                /* e.g. learn without a stored trajectory */
};

enum { ANAKIN_ENV_CATCH = 0, ANAKIN_ENV_PENDULUM = 1, ANAKIN_ENV_MAZE = 2 };
enum { ANAKIN_POLICY_CATEGORICAL = 0, ANAKIN_POLICY_TANH_GAUSSIAN = 1 };
enum { ANAKIN_DTYPE_FP32 = 0, ANAKIN_DTYPE_BF16 = 1 };

/* anakin_set_mode flags */
enum {
    ANAKIN_MODE_VALU_GEMM = 1,         /* learn-phase GEMMs on vector ALUs instead of matrix cores */
    ANAKIN_MODE_CANONICAL_ACTING = 2,  /* act with the sequential fp32 FMA chain on vector ALUs instead of matrix cores */
    ANAKIN_MODE_STREAM_WEIGHTS = 4     /* acting: stream hidden-layer weights from L2 even when they fit on chip */
};

/* Environment (paper section 3.1: initial_state + step on explicit state).
 * kind CATCH: rows x cols board (max_steps ignored, episodes last rows-1 steps);
 * PENDULUM: rows/cols ignored, max_steps = episode length;
 * MAZE: rows x cols <= 256 cells, p_wall = wall probability, max_steps = step cap. */
typedef struct {
    int32_t kind, rows, cols, max_steps;
    float p_wall;
} anakin_env_cfg;

/* Network, objective and optimiser.  hidden[i] in {32,...,1024}, powers of two.
 * policy CATEGORICAL goes with CATCH and MAZE, TANH_GAUSSIAN with PENDULUM.
 * dtype BF16: bfloat16 weights and activations, fp32 accumulation and fp32
 * master weights.  lambda_ = 1 gives bootstrapped n-step returns. */
typedef struct {
    int32_t n_hidden;
    int32_t hidden[4];
    int32_t policy;
    int32_t dtype;
    float gamma, lambda_, entropy_coef, value_coef, lr, beta1, beta2, eps;
} anakin_net_cfg;

typedef struct anakin anakin_t;

/* Device pointers into the caller's workspace (valid for the handle's life)
 * and their byte offsets from the workspace base.  Time-major: index [t][b].
 * state_* hold the state observed at t (t = 0..T); the rest t = 0..T-1 except
 * value and head (t = 0..T, the last row being the bootstrap evaluation). */
typedef struct {
    int32_t B, T, num_heads, head_stride, n_hidden;
    int32_t hidden[4];
    int32_t act_is_bf16;              /* act[]: 0 fp32 [T*B][H]; 2 bf16 packed [T*B/8][H][8] (8 consecutive samples per
                                         feature); -1 not stored (one-layer nets: the update rebuilds the layer) */
    void* state_s0;  size_t off_state_s0;   /* uint32 [T+1][B] packed state word */
    void* state_f0;  size_t off_state_f0;   /* float  [T+1][B] (pendulum theta) */
    void* state_f1;  size_t off_state_f1;   /* float  [T+1][B] (pendulum theta_dot) */
    void* action;    size_t off_action;     /* uint8  [T][B] categorical action */
    void* eps;       size_t off_eps;        /* float  [T][B] gaussian noise */
    void* action_f;  size_t off_action_f;   /* float  [T][B] squashed gaussian action */
    void* reward;    size_t off_reward;     /* float  [T][B] */
    void* done;      size_t off_done;       /* uint8  [T][B] */
    void* value;     size_t off_value;      /* float  [T+1][B] */
    void* head;      size_t off_head;       /* float  [T+1][B][head_stride] raw head outputs */
    void* adv;       size_t off_adv;        /* float  [T][B] advantages (after learn) */
    void* ret;       size_t off_ret;        /* float  [T][B] returns (after learn) */
    void* act[4];    size_t off_act[4];     /* [T*B][hidden[l]] hidden activations */
} anakin_traj_view;

/* Sums over the last unroll / update.  Filled after synchronising the stream. */
typedef struct {
    double loss, policy_loss, value_loss, entropy_loss;   /* means over B*T (last learn) */
    double reward_sum;                                    /* over the last unroll */
    int64_t episodes;                                     /* episode ends in the last unroll */
    int32_t nonfinite;                                    /* 1 if any of the above is not finite */
} anakin_metrics;

/* Bytes of device workspace needed for this configuration (0 if it is invalid).  The workspace holds everything
 * paper section 2.3 keeps in device memory between executions: parameters and optimiser state, the environment
 * states (section 3.1: explicit state handed from step to step), the stored unroll of figure 2 (top) and the
 * update's scratch. */
size_t anakin_workspace_bytes(const anakin_env_cfg* env, const anakin_net_cfg* net, int32_t B, int32_t T);

/* Create an agent (paper section 3.1: `initial_state` of every environment; section 2.3: the program's inputs
 * are placed in device memory once): B environments in their initial states (drawn from the
 * seed), Glorot-initialised parameters, zero optimiser state -- all written
 * into d_workspace on hip_stream (a hipStream_t, may be null for the default
 * stream).  B must be a multiple of 16.  Synchronises the stream before
 * returning.  On error *out is null and nothing is enqueued. */
int32_t anakin_create(anakin_t** out, const anakin_env_cfg* env, const anakin_net_cfg* net,
                      int32_t B, int32_t T, uint64_t seed,
                      void* d_workspace, size_t workspace_bytes, void* hip_stream);

/* T interactions per env, each: observe, policy/value forward, sample, env
 * step (paper section 2.1 loop; figure 2 top), then the value of the final
 * state.  Fills the trajectory; env state carries over to the next call.
 * Asynchronous: enqueues on the stream and returns. */
int32_t anakin_rollout(anakin_t* h);

/* One update on the stored trajectory: returns/advantages, actor-critic loss,
 * backward pass, Adam (paper section 3.1: "parameter update" reusing the
 * forward pass).  ANAKIN_E_STATE without a preceding rollout.  Asynchronous. */
int32_t anakin_learn(anakin_t* h);

/* anakin_learn for callers that cannot allocate device memory or hand over a larger workspace: code under HIP
 * graph capture, tight serving loops, harnesses that forbid hipMalloc.  The same update on the same stored
 * trajectory with the same result, but the scratch of the backward pass (per-sample head gradients, dZ_l,
 * split-K partial sums) is placed in a static device array of ANAKIN_STATIC_SCRATCH_BYTES that the library holds
 * once per GPU for the life of the process, instead of in the caller's workspace; inputs and outputs (trajectory,
 * parameters, optimiser state, gradient, metrics) stay where anakin_learn has them.  Calls no hipMalloc / hipFree
 * and no allocating routine.  ANAKIN_E_WORKSPACE_TOO_SMALL (with the bytes needed in anakin_last_error) when the
 * configuration's update needs more than the array holds; ANAKIN_E_STATE while per-kernel timing is on (it creates
 * events) or without a stored trajectory.  The array is shared by every handle on a GPU and keeps the last call's
 * contents (nothing in it needs clearing: every byte is written before it is read within one update): calls that
 * overlap in time on one GPU -- different handles on different streams -- race and must be serialised by the
 * caller.  Asynchronous like anakin_learn. */
#define ANAKIN_STATIC_SCRATCH_BYTES (64u << 20)
int32_t anakin_learn_static(anakin_t* h);

/* anakin_rollout followed by anakin_learn: Anakin's minimal unit of computation (paper section 3.1 and
 * figure 2 top: T interactions, then one update), the timed unit.  Asynchronous. */
int32_t anakin_step(anakin_t* h);

/* One decoupled step: acting and learning run side by side on one device (the one-device form of
 * the actor/learner split of paper section 3.2 and figure 3, where the actors run on parameters
 * that lag the learner's).  A copy of the parameters is taken; the actor then unrolls T steps with
 * that copy on a second stream of the library's own, while on the handle's stream the learner
 * applies one update to the unroll the previous decoupled step (or anakin_rollout) stored: a
 * forward pass over its states with the current parameters, V-trace targets (Espeholt et al. 2018;
 * truncation levels 1, trace decay lambda) from the stored behaviour head outputs and the new ones,
 * then the same loss, backward pass and Adam as anakin_learn.  The first call only collects.  The
 * handle's stream waits for the actor before any later work, so the usual stream semantics hold;
 * the result does not depend on how the two streams interleave.  anakin_get_trajectory then shows
 * the unroll just collected (its adv / ret / act fields belong to the update that ran beside it).
 * One update per unroll, score-function gradient: ANAKIN_E_BAD_CONFIG otherwise.  After a decoupled step
 * anakin_learn returns ANAKIN_E_STATE (the stored unroll has no activations); anakin_step and
 * anakin_rollout start a fresh on-policy unroll.  Asynchronous.
 * Streams: this is the one call that uses a second stream.  The caller may hand one over with
 * anakin_set_actor_stream; otherwise the library creates a non-blocking stream of default priority on first use
 * and destroys it in anakin_destroy (the one exception to "the caller owns the streams").
 * Errors: if the learner's half fails, the unroll the actor collected is still stored, the handle's stream is
 * still ordered behind the actor and the error code of the update is returned. */
int32_t anakin_step_decoupled(anakin_t* h);

/* The stream the actor of anakin_step_decoupled runs on: a hipStream_t of the caller's, distinct from the
 * handle's stream and not the null stream, of default priority; it must outlive the handle or be replaced first.
 * Synchronises a previously used actor stream.  ANAKIN_E_INVALID_ARG otherwise. */
int32_t anakin_set_actor_stream(anakin_t* h, void* hip_stream);

/* Frees the host-side handle (never the workspace: paper section 2.3, device memory outlives an execution and
 * here belongs to the caller).  Synchronises the stream. */
int32_t anakin_destroy(anakin_t* h);

/* ---- introspection for parity tests and measurement ----
 * None of these is on the hot path.  Each synchronises the handle's stream and copies between host buffers of the
 * caller and the device workspace; together they expose the explicit, device-resident state that paper sections
 * 2.3 and 3.1 describe (parameters, optimiser state, environment state, the stored unroll), which is also what a
 * checkpoint consists of.  All return ANAKIN_E_INVALID_ARG for a null pointer or a wrong length. */

/* Number of parameters P of the policy/value network (flat vector: W_1, b_1, ..., W_L, b_L, W_heads, b_heads). */
int32_t anakin_param_count(const anakin_t* h, int64_t* out);
/* The parameters the next unroll acts with (section 3.1: the update's output).  n must equal P. */
int32_t anakin_get_params(anakin_t* h, float* h_dst, size_t n);
/* Replaces them (bf16 nets: the rounded copies are refreshed too). */
int32_t anakin_set_params(anakin_t* h, const float* h_src, size_t n);
/* The gradient the last update applied (of the last chunk with several updates per unroll). */
int32_t anakin_get_grads(anakin_t* h, float* h_dst, size_t n);
/* Adam's moments and step count (the optimiser state of the "parameter update" of section 3.1). */
int32_t anakin_get_opt_state(anakin_t* h, float* h_m, float* h_v, int32_t* h_step, size_t n);
int32_t anakin_set_opt_state(anakin_t* h, const float* h_m, const float* h_v, int32_t step, size_t n);
/* The environments' explicit state (section 3.1: `step(state, action)` takes and returns it) as [B][4] int32 +
 * [B][2] float rows: catch (ball_x, ball_y, paddle_x, 0); pendulum (steps,0,0,0) + (theta, theta_dot);
 * maze (cell, steps,0,0).  The setter checks ranges: ANAKIN_E_INVALID_ARG for a state the env cannot be in. */
int32_t anakin_get_env_state(anakin_t* h, int32_t* h_si, float* h_sf);
int32_t anakin_set_env_state(anakin_t* h, const int32_t* h_si, const float* h_sf);
/* The mazes drawn at create, [B][8] words of 32 cells, bit set = wall.  ANAKIN_E_STATE for other envs. */
int32_t anakin_get_walls(anakin_t* h, uint32_t* h_walls);
/* Environment steps taken so far per env (the time coordinate of every random draw: runs are deterministic,
 * paper section 3.1, and a resumed run continues the same streams). */
int32_t anakin_get_global_step(const anakin_t* h, uint64_t* out);
int32_t anakin_set_global_step(anakin_t* h, uint64_t g);
/* Where the stored unroll (figure 2 top) lies in the workspace; see anakin_traj_view. */
int32_t anakin_get_trajectory(anakin_t* h, anakin_traj_view* out);
/* Loss terms of the last update and reward / episode counts of the last unroll.  Returns ANAKIN_E_NONFINITE
 * (with *out filled) if a loss term is not finite; all zero before the first update. */
int32_t anakin_get_metrics(anakin_t* h, anakin_metrics* out);
/* Selects reference implementations (ANAKIN_MODE_* flags) for cross-checks; 0 is the product path.
 * ANAKIN_E_INVALID_ARG for an unknown flag or a combination a bf16 net cannot run. */
int32_t anakin_set_mode(anakin_t* h, int32_t flags);

/* Several Adam updates per unroll (paper section 4, the remark on decoupling the acting batch from
 * the learning batch by splitting the batch on the learner and applying N updates instead of one
 * larger one).  With n_updates = N > 1, anakin_learn cuts the stored unroll into N consecutive
 * chunks of T/N time steps (all B envs each); returns and advantages still come from the whole
 * unroll; chunk k's gradient is that of its own mean loss at the parameters the unroll was acted
 * with (the update reuses the acting forward pass), and the N Adam steps are applied in chunk
 * order.  The metrics then average over the chunks; anakin_get_grads returns the last chunk's
 * gradient.  ANAKIN_E_BAD_CONFIG if T is not a multiple of n_updates or a chunk does not fit the
 * kernels' row granularity; the setting is kept until changed.  Default 1. */
int32_t anakin_set_updates_per_unroll(anakin_t* h, int32_t n_updates);

/* At which parameters the gradient of chunk k of several updates per unroll is taken (the paper's remark in
 * section 4 leaves it open).  ANAKIN_CHUNKS_AT_ACTING_PARAMETERS (default): at the parameters the unroll was acted
 * with -- every chunk reuses the stored forward pass (section 3.1), nothing is recomputed.  ANAKIN_CHUNKS_SEQUENTIAL:
 * at the parameters as they are after the k previous updates, which is what "N smaller updates instead of one
 * larger one" ordinarily means -- before every chunk but the first the forward pass over the stored states is
 * repeated with the current parameters; returns and advantages stay those of the stored unroll, the actions (and
 * for the Gaussian policy the pre-squash samples) stay fixed.  Kept until changed; has no effect with one update
 * per unroll.  ANAKIN_E_INVALID_ARG for an unknown mode. */
enum { ANAKIN_CHUNKS_AT_ACTING_PARAMETERS = 0, ANAKIN_CHUNKS_SEQUENTIAL = 1 };
int32_t anakin_set_update_chunk_mode(anakin_t* h, int32_t mode);

/* Which policy gradient anakin_learn takes.  ANAKIN_PG_SCORE_FUNCTION (default): the actor-critic
 * term -A log pi(a|s).  ANAKIN_PG_PATHWISE: the gradient of minus the mean reward of the stored
 * unroll through the environment's dynamics and the reparameterised policy (paper section 3.1:
 * the unit of T interactions, environment included, can be differentiated all the way through);
 * value and entropy terms stay as they are, the reported policy loss becomes minus the mean
 * reward.  Pendulum with the tanh-Gaussian policy, fp32 net of two equal hidden layers of 64, 128
 * or 256 units, B a multiple of 16, one update per unroll: ANAKIN_E_BAD_CONFIG otherwise (for the
 * last, from anakin_learn).  Kept until changed. */
enum { ANAKIN_PG_SCORE_FUNCTION = 0, ANAKIN_PG_PATHWISE = 1 };
int32_t anakin_set_policy_gradient(anakin_t* h, int32_t kind);

/* How the update of this handle is cut into workgroups (what the parity tests assert their cases reach, and
 * what the benchmark prints).  splits[l], l < n_hidden: chunks of the B*T samples whose partial dW_{l+1} / db_{l+1}
 * sums are written separately and added in a fixed order; splits[n_hidden]: the same for the head matrix;
 * splits_walls: bf16 maze nets whose first layer is reduced plane by plane -- chunks of the 2 B time-summed rows of
 * the wall-plane product (splits[0] then counts the agent-plane product's chunks), else 0;
 * dx_rows[l], 1 <= l < n_hidden: samples one workgroup of the weights-resident bf16 dX kernel of layer l+1 walks
 * (it stages 32 at a time), 0 where another kernel runs; bf16_matrix_path: 1 when acting and update of a bf16
 * net run on the matrix-core kernels (packed activations). */
typedef struct {
    int32_t n_hidden;
    int32_t splits[5];
    int32_t splits_walls;
    int32_t head_fan;
    int32_t dx_rows[4];
    int32_t bf16_matrix_path;
    int32_t updates_per_unroll;
} anakin_plan;
int32_t anakin_get_plan(const anakin_t* h, anakin_plan* out);

/* Per-kernel timing for measurement.  While enabled, every kernel launch is
 * bracketed by two events recorded on the handle's stream (this adds a few
 * microseconds per launch, so throughput is timed with profiling off).
 * anakin_profile(h, 1) clears the totals and starts; anakin_profile(h, 0)
 * stops.  anakin_kernel_times synchronises the stream and writes up to cap
 * entries; *n receives the number of distinct kernels seen. */
typedef struct {
    char name[48];
    int64_t calls;
    double total_ms;
} anakin_kernel_time;
int32_t anakin_profile(anakin_t* h, int32_t enable);
int32_t anakin_kernel_times(anakin_t* h, anakin_kernel_time* out, int32_t cap, int32_t* n);

/* Peak probes for the measurement section (what the GPU delivers for the two rooflines the kernels are
 * priced against).  kind: a register-only loop of fp32 or bf16 MFMAs
 * (no memory traffic) or a streaming copy of scratch_bytes/2 bytes inside the scratch buffer.
 * workgroups: grid size of the probe, 0 for the default (the achieved rate depends on it).
 * scratch: device memory owned by the caller, at least 1 MiB (MFMA probes) or as large as the copy
 * should be (copy probe: first half is read, second half written, ten times; Adam probe: the update
 * kernel on min(scratch_bytes / 20, 2^26) synthetic parameters, five times, 32 bytes per parameter; read
 * probe: the whole buffer but its last workgroups x 1 KiB is read ten times and summed, nothing else is written;
 * L2 probe: every workgroup (512 threads) streams the first MiB of the buffer 200 times in the access pattern of
 * the bf16 acting kernel's weight stream -- the L2-to-CU rate with all units asking at once; needs 1 MiB plus
 * workgroups x 2 KiB).
 * Synchronous: the
 * call enqueues on hip_stream, waits, and returns the work done (*amount: flop, or bytes read +
 * written) and the elapsed time from two events on that stream.  Returns ANAKIN_E_INVALID_ARG for
 * a null pointer, an unknown kind or a scratch buffer that is too small. */
enum { ANAKIN_PROBE_MFMA_F32 = 0, ANAKIN_PROBE_MFMA_BF16 = 1, ANAKIN_PROBE_COPY = 2, ANAKIN_PROBE_ADAM = 3, ANAKIN_PROBE_READ = 4,
       ANAKIN_PROBE_L2_TILES = 5 };
int32_t anakin_peak_probe(int32_t kind, int32_t workgroups, void* scratch, size_t scratch_bytes, void* hip_stream,
                          double* amount, double* milliseconds);

/* Handle-owned message for the last error on this handle (valid until the next
 * call on it); for a null handle, the message of the last failed create. */
const char* anakin_last_error(const anakin_t* h);

#ifdef __cplusplus
}
#endif
#endif /* ANAKIN_H */
