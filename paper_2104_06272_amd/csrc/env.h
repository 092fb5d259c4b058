// The three on-device environments as pure functions of explicit state
// (paper section 3.1: initial_state and step(state, action) -> (state, reward)),
// plus the two action samplers.  One env's state is three 32-bit words:
//   Catch:    s0 = ball_x | ball_y << 8 | paddle_x << 16
//   Pendulum: s0 = steps taken, f0 = theta (kept in [-pi_f, pi_f)), f1 = theta_dot
//   Maze:     s0 = cell | steps << 16; walls: one bit per cell (8 words per env)
#pragma once
#include "detmath.h"

namespace ank {

enum : int { ENV_CATCH = 0, ENV_PENDULUM = 1, ENV_MAZE = 2 };
enum : int { POLICY_CATEGORICAL = 0, POLICY_TANH_GAUSSIAN = 1 };

struct EnvDims { int kind, rows, cols, max_steps; };
struct EnvState { uint32_t s0; float f0, f1; };

// ---- Catch -----------------------------------------------------------------
ANK_HD uint32_t catch_pack(int bx, int by, int px) { return (uint32_t)bx | ((uint32_t)by << 8) | ((uint32_t)px << 16); }
ANK_HD uint32_t catch_reset(const EnvDims& d, uint32_t word) { return catch_pack((int)bounded(word, (uint32_t)d.cols), 0, d.cols / 2); }
// paddle first, then the ball drops; reward and reset when it reaches the last row
ANK_HD void catch_step(const EnvDims& d, EnvState& s, int a, uint32_t reset_word, float& r, int& done)
{
    const int bx = (int)(s.s0 & 0xffu), by = (int)((s.s0 >> 8) & 0xffu) + 1;
    int px = (int)((s.s0 >> 16) & 0xffu) + a - 1;
    px = px < 0 ? 0 : px;
    px = px > d.cols - 1 ? d.cols - 1 : px;
    if (by == d.rows - 1) {
        r = (px == bx) ? 1.0f : -1.0f;
        done = 1;
        s.s0 = catch_reset(d, reset_word);
    } else {
        r = 0.0f;
        done = 0;
        s.s0 = catch_pack(bx, by, px);
    }
}
// the two cells of the board that hold a 1, in ascending index order
ANK_HD void catch_obs_cells(const EnvDims& d, uint32_t s0, int& ball_cell, int& paddle_cell)
{
    ball_cell = (int)((s0 >> 8) & 0xffu) * d.cols + (int)(s0 & 0xffu);
    paddle_cell = (d.rows - 1) * d.cols + (int)((s0 >> 16) & 0xffu);
}

// ---- Pendulum --------------------------------------------------------------
ANK_HD float wrap_angle(float th)
{
    const float pi_f = 0x1.921fb6p+1f;
    if (th >= pi_f)      th = (th - 0x1.921fb6p+2f) - (-0x1.777a5cp-23f);
    else if (th < -pi_f) th = (th + 0x1.921fb6p+2f) + (-0x1.777a5cp-23f);
    return th;
}
ANK_HD void pendulum_reset(EnvState& s, uint32_t w0, uint32_t w1)
{
    s.f0 = wrap_angle(fmaf(0x1.921fb6p+2f, u01(w0), -0x1.921fb6p+1f));
    s.f1 = fmaf(2.0f, u01(w1), -1.0f);
    s.s0 = 0;
}
// reward from the state before the step; semi-implicit Euler; time limit ends the episode
ANK_HD void pendulum_step(const EnvDims& d, EnvState& s, float a, uint32_t w0, uint32_t w1, float& r, int& done)
{
    const float th = s.f0, thd = s.f1;
    float u = 2.0f * a;
    u = u < -2.0f ? -2.0f : u;
    u = u > 2.0f ? 2.0f : u;
    float cost = th * th;
    cost = fmaf(0x1.99999ap-4f, thd * thd, cost);
    cost = fmaf(0x1.0624dep-10f, u * u, cost);
    r = -cost;
    float sn, cs;
    det_sincos(th, sn, cs);
    const float acc = fmaf(15.0f, sn, 3.0f * u);
    float nthd = fmaf(acc, 0x1.99999ap-5f, thd);
    nthd = nthd < -8.0f ? -8.0f : nthd;
    nthd = nthd > 8.0f ? 8.0f : nthd;
    s.f0 = wrap_angle(fmaf(nthd, 0x1.99999ap-5f, th));
    s.f1 = nthd;
    const uint32_t steps = s.s0 + 1u;
    s.s0 = steps;
    // the flag is a value, not a store in either arm of the branch: written as two stores the compiler pairs
    // the arms' zero stores (step count, flag) into one store through a selected address, and the state
    // then lives in scratch memory instead of registers
    done = (int)steps >= d.max_steps ? 1 : 0;
    if (done) pendulum_reset(s, w0, w1);
}

// ---- Maze ------------------------------------------------------------------
// walls are read through a functor so that callers can keep them in registers,
// LDS or global memory: wall(cell) -> bool
template <class WallFn>
ANK_HD void maze_step(const EnvDims& d, EnvState& s, int a, WallFn wall, float& r, int& done)
{
    int cell = (int)(s.s0 & 0xffffu);
    const int steps = (int)(s.s0 >> 16) + 1;
    const int row = cell / d.cols, col = cell - row * d.cols;
    int nr = row, nc = col;
    if (a == 0) nr = row - 1;
    else if (a == 1) nc = col + 1;
    else if (a == 2) nr = row + 1;
    else nc = col - 1;
    if (nr >= 0 && nr < d.rows && nc >= 0 && nc < d.cols) {
        const int cand = nr * d.cols + nc;
        if (!wall(cand)) cell = cand;
    }
    if (cell == d.rows * d.cols - 1) { r = 1.0f; done = 1; }
    else { r = -0x1.47ae14p-7f; done = steps >= d.max_steps ? 1 : 0; }
    s.s0 = done ? 0u : ((uint32_t)cell | ((uint32_t)steps << 16));
}

// ---- Samplers ----------------------------------------------------------------
// inverse CDF over exp(logit - max) with one uniform
template <int MAXA>
ANK_HD int sample_categorical(const float (&logits)[MAXA], int A, float u)
{
    float mx = logits[0];
#pragma unroll
    for (int i = 1; i < MAXA; ++i) if (i < A) mx = logits[i] > mx ? logits[i] : mx;
    float c[MAXA];
    float run = 0.0f;
#pragma unroll
    for (int i = 0; i < MAXA; ++i) {
        if (i < A) {
            const float e = det_exp(logits[i] - mx);
            run = (i == 0) ? e : run + e;
        }
        c[i] = run;
    }
    const float thr = u * run;
    int a = A - 1;
#pragma unroll
    for (int i = MAXA - 1; i >= 0; --i) if (i < A && c[i] > thr) a = i;
    return a;
}

// The same sampler with the usual action counts as constants: the comparisons against A fold away and
// only A exponentials are left in the instruction stream.  Same operations in the same order for every A.
// The heads come in as values: handed over as an array by reference, the branches' loads get merged into one
// load through a selected address and the caller's array ends up in scratch memory.
ANK_HD int sample_categorical_any(float l0, float l1, float l2, float l3, float l4, float l5, float l6, float l7,
                                  int A, float u)
{
    const float lg[8] = {l0, l1, l2, l3, l4, l5, l6, l7};
    if (A == 3) return sample_categorical<8>(lg, 3, u);
    if (A == 4) return sample_categorical<8>(lg, 4, u);
    return sample_categorical<8>(lg, A, u);
}
// the value is the last head
ANK_HD float last_head(float h0, float h1, float h2, float h3, float h4, float h5, float h6, float h7, int NH)
{
    if (NH == 4) return h3;
    if (NH == 5) return h4;
    if (NH == 3) return h2;
    return NH == 8 ? h7 : NH == 7 ? h6 : NH == 6 ? h5 : NH == 2 ? h1 : h0;
}

// Box-Muller noise, z = mu + sigma eps, squashed by tanh; log_sigma clamped to [-5, 2]
// the two halves of the sampler: the noise does not depend on the network, so a kernel can draw it early
ANK_HD float gaussian_noise(uint32_t w0, uint32_t w1)
{
    const float rad = sqrtf(-2.0f * det_log(u01_plus(w0)));
    return rad * det_cos2pi(u01(w1));
}
ANK_HD float gaussian_action(float mu, float log_sigma, float eps)
{
    float ls = log_sigma < -5.0f ? -5.0f : log_sigma;
    ls = ls > 2.0f ? 2.0f : ls;
    const float sigma = det_exp(ls);
    return det_tanh(fmaf(sigma, eps, mu));
}
ANK_HD void sample_gaussian(float mu, float log_sigma, uint32_t w0, uint32_t w1, float& eps, float& act)
{
    eps = gaussian_noise(w0, w1);
    act = gaussian_action(mu, log_sigma, eps);
}

}  // namespace ank
