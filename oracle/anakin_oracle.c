/*
 * anakin_oracle.c -- TEST INFRASTRUCTURE, not product code.
 *
 * A plain, slow, single-threaded CPU statement of what the on-device
 * actor-learner step of the Anakin architecture computes (paper section 3.1,
 * "Online Learning with Anakin"; figure 2 top: T agent-environment
 * interactions followed by one parameter update; section 2.1: the
 * observation/reward -> action loop).  The paper fixes the skeleton only; the
 * concrete environments, network, objective, optimiser and random number
 * generator are the ones this build's workload definitions name, and every
 * place where a choice had to be made is a numbered reading "R-n" in the
 * comments below.
 *
 * Only tests, the smoke check and the benchmark's CPU-baseline leg may call
 * into this file.  It shares no code with the GPU library.
 *
 * Precision: everything that decides an integer (environment transitions,
 * sampled actions) is defined in IEEE binary32 with a fixed operation order,
 * because both sides must take those decisions identically.  Everything that
 * is compared under a tolerance (returns, loss, gradients, Adam) is computed
 * in binary64.
 *
 * Build: gcc -O2 -std=c99 -ffp-contract=off -mfma -shared -fPIC (no fast-math).
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#define ORC_PI 3.14159265358979323846
#define ORC_E  2.71828182845904523536

/* ------------------------------------------------------------------------- */
/* Random numbers: Philox4x32 with 10 rounds (Salmon et al., SC'11).         */
/* Paper section 3.1 asks for self-contained, deterministic experiments; a   */
/* counter-based generator gives that independent of batch layout.           */
/* ------------------------------------------------------------------------- */
void orc_philox4x32_10(const uint32_t ctr[4], const uint32_t key[2], uint32_t out[4])
{
    uint32_t c0 = ctr[0], c1 = ctr[1], c2 = ctr[2], c3 = ctr[3];
    uint32_t k0 = key[0], k1 = key[1];
    for (int round = 0; round < 10; ++round) {
        uint64_t p0 = (uint64_t)0xD2511F53u * c0;
        uint64_t p1 = (uint64_t)0xCD9E8D57u * c2;
        uint32_t n0 = (uint32_t)(p1 >> 32) ^ c1 ^ k0;
        uint32_t n1 = (uint32_t)p1;
        uint32_t n2 = (uint32_t)(p0 >> 32) ^ c3 ^ k1;
        uint32_t n3 = (uint32_t)p0;
        c0 = n0; c1 = n1; c2 = n2; c3 = n3;
        k0 += 0x9E3779B9u;
        k1 += 0xBB67AE85u;
    }
    out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

/* R-1 counter layout: key = seed (low, high word); counter = (index, t_low,
 * t_high, domain).  Domains: 0 action sample (index = env, t = global env-step
 * number), 1 episode reset (same index and t as the step that ended the
 * episode), 2 initial env state (t = 0), 3 parameter init (index = element/4
 * inside an init group, t_low = group id), 4 maze walls (index = env, t_low =
 * attempt, t_high = block of four cells). */
enum { DOM_ACTION = 0, DOM_RESET = 1, DOM_INIT = 2, DOM_PARAM = 3, DOM_MAZE = 4 };

static void draw4(uint64_t seed, uint32_t index, uint64_t t, uint32_t domain, uint32_t w[4])
{
    uint32_t ctr[4] = { index, (uint32_t)t, (uint32_t)(t >> 32), domain };
    uint32_t key[2] = { (uint32_t)seed, (uint32_t)(seed >> 32) };
    orc_philox4x32_10(ctr, key, w);
}

/* R-2: u in [0,1) with 24 bits; u_plus in (0,1] for logarithms. */
float orc_u01(uint32_t x)      { return (float)(x >> 8) * 0x1p-24f; }
float orc_u01_plus(uint32_t x) { return (float)((x >> 8) + 1u) * 0x1p-24f; }
/* R-3: integer in [0,n) by multiply-shift. */
uint32_t orc_bounded(uint32_t x, uint32_t n) { return (uint32_t)(((uint64_t)x * n) >> 32); }

/* ------------------------------------------------------------------------- */
/* R-4 deterministic elementary functions: fixed sequences of binary32       */
/* add/mul/fma/div/sqrt, all correctly rounded, so that a GPU and a CPU give */
/* the same bits.                                                            */
/* ------------------------------------------------------------------------- */
static float bits_to_float(uint32_t u) { float f; memcpy(&f, &u, 4); return f; }
static uint32_t float_to_bits(float f) { uint32_t u; memcpy(&u, &f, 4); return u; }

float orc_exp(float x)
{
    if (x < -87.0f) x = -87.0f;
    if (x > 88.0f) x = 88.0f;
    float n = rintf(x * 0x1.715476p+0f);                 /* x * log2(e), to nearest even */
    float f = fmaf(-n, 0x1.62ep-1f, x);                  /* ln2 high part, 12 significant bits */
    f = fmaf(-n, 0x1.0bfbe8p-15f, f);                    /* ln2 low part */
    float p = 0x1.a01a02p-13f;                           /* 1/7! */
    p = fmaf(p, f, 0x1.6c16c2p-10f);                     /* 1/6! */
    p = fmaf(p, f, 0x1.111112p-7f);                      /* 1/5! */
    p = fmaf(p, f, 0x1.555556p-5f);                      /* 1/4! */
    p = fmaf(p, f, 0x1.555556p-3f);                      /* 1/3! */
    p = fmaf(p, f, 0.5f);
    p = fmaf(p, f, 1.0f);
    p = fmaf(p, f, 1.0f);
    int e = (int)n + 127;                                /* 1..254 after the clamp */
    return p * bits_to_float((uint32_t)e << 23);
}

/* natural log of a positive normal number */
float orc_log(float x)
{
    uint32_t u = float_to_bits(x);
    int e = (int)(u >> 23) - 127;
    float m = bits_to_float((u & 0x007fffffu) | 0x3f800000u);   /* [1,2) */
    if (m > 0x1.6a09e6p+0f) { m = m * 0.5f; e += 1; }           /* (sqrt2/2, sqrt2] */
    float s = (m - 1.0f) / (m + 1.0f);
    float s2 = s * s;
    float p = 0x1.745d18p-4f;                            /* 1/11 */
    p = fmaf(p, s2, 0x1.c71c72p-4f);                     /* 1/9 */
    p = fmaf(p, s2, 0x1.24924ap-3f);                     /* 1/7 */
    p = fmaf(p, s2, 0x1.99999ap-3f);                     /* 1/5 */
    p = fmaf(p, s2, 0x1.555556p-2f);                     /* 1/3 */
    p = fmaf(p, s2, 1.0f);
    float lm = (s + s) * p;                              /* ln m = 2 atanh(s) */
    float fe = (float)e;
    float r = fmaf(fe, 0x1.0bfbe8p-15f, lm);
    return fmaf(fe, 0x1.62ep-1f, r);
}

/* sine and cosine polynomials on |r| <= pi/4 (+ a hair) */
static float sin_poly(float r)
{
    float r2 = r * r;
    float p = 0x1.71de3ap-19f;                           /* 1/9! */
    p = fmaf(p, r2, -0x1.a01a02p-13f);                   /* -1/7! */
    p = fmaf(p, r2, 0x1.111112p-7f);                     /* 1/5! */
    p = fmaf(p, r2, -0x1.555556p-3f);                    /* -1/3! */
    p = p * r2;
    return fmaf(p, r, r);
}
static float cos_poly(float r)
{
    float r2 = r * r;
    float p = -0x1.27e4fcp-22f;                          /* -1/10! */
    p = fmaf(p, r2, 0x1.a01a02p-16f);                    /* 1/8! */
    p = fmaf(p, r2, -0x1.6c16c2p-10f);                   /* -1/6! */
    p = fmaf(p, r2, 0x1.555556p-5f);                     /* 1/4! */
    p = fmaf(p, r2, -0.5f);
    return fmaf(p, r2, 1.0f);
}

/* sin and cos of an angle in [-pi_f, pi_f]; quadrant reduction with a
 * two-constant pi/2. */
void orc_sincos(float th, float* s, float* c)
{
    float q = rintf(th * 0x1.45f306p-1f);                /* th * 2/pi -> -2..2 */
    float r = fmaf(-q, 0x1.92p+0f, th);                  /* pi/2 high */
    r = fmaf(-q, 0x1.fb5444p-12f, r);                    /* pi/2 low */
    float sp = sin_poly(r), cp = cos_poly(r);
    int qi = (int)q & 3;
    if (qi == 0)      { *s = sp;  *c = cp;  }
    else if (qi == 1) { *s = cp;  *c = -sp; }
    else if (qi == 2) { *s = -sp; *c = -cp; }
    else              { *s = -cp; *c = sp;  }
}
float orc_sin(float th) { float s, c; orc_sincos(th, &s, &c); return s; }
float orc_cos(float th) { float s, c; orc_sincos(th, &s, &c); return c; }

/* cos(2 pi u) for u in [0,1): the quadrant split is exact on u itself. */
float orc_cos2pi(float u)
{
    float q = rintf(4.0f * u);                           /* 0..4 */
    float r = fmaf(-0.25f, q, u);                        /* exact, |r| <= 1/8 */
    float a = 0x1.921fb6p+2f * r;                        /* 2 pi r, |a| <= pi/4 */
    int qi = (int)q & 3;
    if (qi == 0) return cos_poly(a);
    if (qi == 1) return -sin_poly(a);
    if (qi == 2) return -cos_poly(a);
    return sin_poly(a);
}

float orc_tanh(float z)
{
    float a = fabsf(z), t;
    if (a < 0.25f) {
        float a2 = a * a;
        float p = -0x1.226e36p-7f;                       /* -1382/155925 */
        p = fmaf(p, a2, 0x1.664f48p-6f);                 /* 62/2835 */
        p = fmaf(p, a2, -0x1.ba1ba2p-5f);                /* -17/315 */
        p = fmaf(p, a2, 0x1.111112p-3f);                 /* 2/15 */
        p = fmaf(p, a2, -0x1.555556p-2f);                /* -1/3 */
        p = p * a2;
        t = fmaf(p, a, a);
    } else if (a > 9.0f) {
        t = 1.0f;
    } else {
        float e = orc_exp(-2.0f * a);
        t = (1.0f - e) / (1.0f + e);
    }
    return copysignf(t, z);
}

/* bfloat16 rounding, to nearest even, of a finite binary32 value */
float orc_bf16_round(float x)
{
    uint32_t u = float_to_bits(x);
    u += 0x7fffu + ((u >> 16) & 1u);
    u &= 0xffff0000u;
    return bits_to_float(u);
}

/* ------------------------------------------------------------------------- */
/* Configuration                                                              */
/* ------------------------------------------------------------------------- */
enum { ENV_CATCH = 0, ENV_PENDULUM = 1, ENV_MAZE = 2 };
enum { POLICY_CATEGORICAL = 0, POLICY_TANH_GAUSSIAN = 1 };

typedef struct {
    int32_t kind, rows, cols, max_steps;
    float p_wall;
} orc_env_cfg;

typedef struct {
    int32_t n_hidden;
    int32_t hidden[4];
    int32_t policy;
    int32_t dtype;                 /* 0: fp32; 1: bf16 layers, fp32 master */
    float gamma, lambda_, entropy_coef, value_coef, lr, beta1, beta2, eps;
} orc_net_cfg;

typedef struct {
    orc_env_cfg env;
    orc_net_cfg net;
    int B, T, D, A, NH, L;
    int dims[6];                   /* D, H1..HL */
    uint64_t seed, gstep;
    size_t P;
    size_t w_off[4], b_off[4], wh_off, bh_off;
    float *theta;
    double *m, *v;                 /* Adam moments (binary64) */
    float *grad;
    int adam_t;
    /* environment state, one row per env */
    int32_t *si;                   /* [B][4] */
    float *sf;                     /* [B][2] */
    uint32_t *walls;               /* [B][8], maze only */
    /* trajectory, time-major */
    int32_t *tr_si;                /* [T+1][B][4] state observed at t */
    float *tr_sf;                  /* [T+1][B][2] */
    int32_t *tr_act;               /* [T][B] categorical action */
    float *tr_actf;                /* [T][B] squashed gaussian action */
    float *tr_eps;                 /* [T][B] gaussian noise */
    float *tr_z;                   /* [T][B] pre-squash gaussian sample */
    float *tr_rew;                 /* [T][B] */
    uint8_t *tr_done;              /* [T][B] */
    float *tr_val;                 /* [T+1][B] */
    float *tr_head;                /* [T+1][B][NH] raw head outputs */
    double *adv, *ret;             /* [T][B] */
    double loss[4];                /* total, policy, value, entropy terms (means) */
    int have_traj;
    double *cur_head;              /* [T+1][B][NH] head outputs of the learner's parameters (off-policy update) */
    double *rho;                   /* [T][B] truncated importance weights of the last off-policy update */
} orc_t;

/* ------------------------------------------------------------------------- */
/* Environments (paper section 3.1: initial_state and step(state, action) -> */
/* (state, reward) as pure functions of explicit state)                       */
/* ------------------------------------------------------------------------- */

/* --- Catch: ball falls one row per step, paddle in the bottom row -------- */
/* state: si = (ball_x, ball_y, paddle_x, 0).  R-5: the paddle starts in the
 * middle column (cols/2) at every reset. */
static void catch_reset(const orc_t* h, uint32_t word, int32_t* si)
{
    si[0] = (int32_t)orc_bounded(word, (uint32_t)h->env.cols);
    si[1] = 0;
    si[2] = h->env.cols / 2;
    si[3] = 0;
}
/* R-6: the paddle moves first (a-1, clamped), then the ball drops a row; the
 * episode ends when the ball reaches the bottom row, with reward +1 if the
 * paddle is under it and -1 otherwise; every other reward is 0.  The reset
 * happens inside the same call (the terminal board is never observed). */
static void catch_step(const orc_t* h, int32_t* si, int a, uint32_t reset_word, float* r, int* done)
{
    int px = si[2] + a - 1;
    if (px < 0) px = 0;
    if (px > h->env.cols - 1) px = h->env.cols - 1;
    si[2] = px;
    si[1] += 1;
    if (si[1] == h->env.rows - 1) {
        *r = (px == si[0]) ? 1.0f : -1.0f;
        *done = 1;
        catch_reset(h, reset_word, si);
    } else {
        *r = 0.0f;
        *done = 0;
    }
}
/* observation: rows*cols board, row-major, 1 at the ball and at the paddle */
static void catch_obs(const orc_t* h, const int32_t* si, float* x)
{
    int n = h->env.rows * h->env.cols;
    for (int i = 0; i < n; ++i) x[i] = 0.0f;
    x[si[1] * h->env.cols + si[0]] = 1.0f;
    x[(h->env.rows - 1) * h->env.cols + si[2]] = 1.0f;
}

/* --- Pendulum swing-up --------------------------------------------------- */
/* state: sf = (theta, theta_dot), si[0] = steps taken in this episode.
 * theta = 0 is upright and the stored angle always lies in [-pi_f, pi_f). */
static float wrap_angle(float th)
{
    const float pi_f = 0x1.921fb6p+1f;
    if (th >= pi_f)      th = (th - 0x1.921fb6p+2f) - (-0x1.777a5cp-23f);
    else if (th < -pi_f) th = (th + 0x1.921fb6p+2f) + (-0x1.777a5cp-23f);
    return th;
}
static void pendulum_reset(uint32_t w0, uint32_t w1, int32_t* si, float* sf)
{
    float th = fmaf(0x1.921fb6p+2f, orc_u01(w0), -0x1.921fb6p+1f);   /* U(-pi, pi) */
    sf[0] = wrap_angle(th);
    sf[1] = fmaf(2.0f, orc_u01(w1), -1.0f);                           /* U(-1, 1) */
    si[0] = 0; si[1] = 0; si[2] = 0; si[3] = 0;
}
/* R-7 torque u = clip(2a, -2, 2) for the squashed action a in [-1,1].
 * R-8 the reward is computed from the state before the step.
 * R-9 semi-implicit Euler: the new (clipped) velocity advances the angle.
 * R-11 reaching max_steps ends the episode like a termination (discount 0). */
static void pendulum_step(const orc_t* h, int32_t* si, float* sf, float a,
                          uint32_t w0, uint32_t w1, float* r, int* done)
{
    float th = sf[0], thd = sf[1];
    float u = 2.0f * a;
    if (u < -2.0f) u = -2.0f;
    if (u > 2.0f) u = 2.0f;
    float cost = th * th;
    cost = fmaf(0x1.99999ap-4f, thd * thd, cost);        /* 0.1 */
    cost = fmaf(0x1.0624dep-10f, u * u, cost);           /* 0.001 */
    *r = -cost;
    float acc = fmaf(15.0f, orc_sin(th), 3.0f * u);      /* 3g/(2l) sin + 3/(m l^2) u */
    float nthd = fmaf(acc, 0x1.99999ap-5f, thd);         /* dt = 0.05 */
    if (nthd < -8.0f) nthd = -8.0f;
    if (nthd > 8.0f) nthd = 8.0f;
    float nth = wrap_angle(fmaf(nthd, 0x1.99999ap-5f, th));
    sf[0] = nth; sf[1] = nthd;
    si[0] += 1;
    if (si[0] >= h->env.max_steps) {
        *done = 1;
        pendulum_reset(w0, w1, si, sf);
    } else {
        *done = 0;
    }
}
static void pendulum_obs(const float* sf, float* x)
{
    float s, c;
    orc_sincos(sf[0], &s, &c);
    x[0] = c; x[1] = s; x[2] = sf[1];
}

/* --- Grid maze ----------------------------------------------------------- */
/* state: si = (cell, steps taken); walls: one bit per cell, bit (cell%32) of
 * word (cell/32), cell = row*cols + col.  R-12 one maze per env for the whole
 * run; R-13 start = cell 0, goal = last cell, both free. */
static int maze_is_wall(const uint32_t* w, int cell) { return (int)((w[cell >> 5] >> (cell & 31)) & 1u); }

static int maze_connected(const orc_t* h, const uint32_t* w)
{
    int R = h->env.rows, C = h->env.cols, n = R * C;
    uint8_t seen[1024];
    int queue[1024];
    memset(seen, 0, sizeof seen);
    int head = 0, tail = 0;
    queue[tail++] = 0; seen[0] = 1;
    while (head < tail) {
        int c = queue[head++];
        if (c == n - 1) return 1;
        int r = c / C, col = c % C;
        int nb[4] = { r > 0 ? c - C : -1, col < C - 1 ? c + 1 : -1, r < R - 1 ? c + C : -1, col > 0 ? c - 1 : -1 };
        for (int i = 0; i < 4; ++i) {
            int d = nb[i];
            if (d >= 0 && !seen[d] && !maze_is_wall(w, d)) { seen[d] = 1; queue[tail++] = d; }
        }
    }
    return 0;
}
/* a cell is a wall iff its Philox word is below floor(p_wall * 2^32); maps are
 * redrawn (attempt + 1) until the goal can be reached from the start */
static int maze_generate(const orc_t* h, int env, uint32_t* w)
{
    int n = h->env.rows * h->env.cols;
    uint32_t thr = (uint32_t)floor((double)h->env.p_wall * 4294967296.0);
    for (uint32_t attempt = 0;; ++attempt) {
        for (int i = 0; i < 8; ++i) w[i] = 0;
        for (int blk = 0; blk * 4 < n; ++blk) {
            uint32_t r4[4];
            draw4(h->seed, (uint32_t)env, (uint64_t)attempt | ((uint64_t)blk << 32), DOM_MAZE, r4);
            for (int i = 0; i < 4 && blk * 4 + i < n; ++i) {
                int cell = blk * 4 + i;
                if (r4[i] < thr) w[cell >> 5] |= 1u << (cell & 31);
            }
        }
        w[0] &= ~1u;
        w[(n - 1) >> 5] &= ~(1u << ((n - 1) & 31));
        if (maze_connected(h, w)) return (int)attempt;
    }
}
/* R-14 actions 0 up, 1 right, 2 down, 3 left; a blocked move leaves the agent
 * in place.  R-15 reward +1 on arriving at the goal, else -0.01.  R-16 the
 * step cap ends the episode with discount 0.  Reset: back to the start. */
static void maze_step(const orc_t* h, int32_t* si, const uint32_t* w, int a, float* r, int* done)
{
    int R = h->env.rows, C = h->env.cols;
    int cell = si[0], row = cell / C, col = cell % C;
    int nr = row, nc = col;
    if (a == 0) nr = row - 1;
    else if (a == 1) nc = col + 1;
    else if (a == 2) nr = row + 1;
    else nc = col - 1;
    if (nr >= 0 && nr < R && nc >= 0 && nc < C && !maze_is_wall(w, nr * C + nc)) cell = nr * C + nc;
    si[0] = cell;
    si[1] += 1;
    if (cell == R * C - 1) { *r = 1.0f; *done = 1; }
    else { *r = -0x1.47ae14p-7f; *done = (si[1] >= h->env.max_steps); }
    if (*done) { si[0] = 0; si[1] = 0; }
}
/* observation: three planes (wall, agent, goal), each rows*cols row-major */
static void maze_obs(const orc_t* h, const int32_t* si, const uint32_t* w, float* x)
{
    int n = h->env.rows * h->env.cols;
    for (int c = 0; c < n; ++c) {
        x[c] = maze_is_wall(w, c) ? 1.0f : 0.0f;
        x[n + c] = (c == si[0]) ? 1.0f : 0.0f;
        x[2 * n + c] = (c == n - 1) ? 1.0f : 0.0f;
    }
}

static void render_obs(const orc_t* h, int b, const int32_t* si, const float* sf, float* x)
{
    if (h->env.kind == ENV_CATCH) catch_obs(h, si, x);
    else if (h->env.kind == ENV_PENDULUM) pendulum_obs(sf, x);
    else maze_obs(h, si, h->walls + (size_t)b * 8, x);
}

/* ------------------------------------------------------------------------- */
/* Network: MLP with ReLU hidden layers and linear heads                      */
/* flat parameter vector: W1 [D][H1], b1, ..., WL, bL, Wh [HL][NH], bh [NH]   */
/* heads: categorical (logit_0..logit_{A-1}, value); gaussian (mu, log_sigma, */
/* value)                                                                     */
/* ------------------------------------------------------------------------- */

/* R-17 Glorot-uniform init: W = a (2u-1), a = sqrt(6/(fan_in+fan_out)); each
 * head (logits / value / mu / log_sigma) is its own group with its own
 * fan_out; biases start at 0.  Element e of a group (row-major over the
 * group's own [in][out] shape) uses word e%4 of the draw with index e/4. */
static void init_group(orc_t* h, uint32_t gid, float* W, int ld, int col0, int fan_in, int fan_out)
{
    float a = (float)sqrt(6.0 / (double)(fan_in + fan_out));
    for (int i = 0; i < fan_in; ++i)
        for (int j = 0; j < fan_out; ++j) {
            uint32_t e = (uint32_t)(i * fan_out + j), w4[4];
            draw4(h->seed, e >> 2, gid, DOM_PARAM, w4);
            float u = orc_u01(w4[e & 3]);
            W[(size_t)i * ld + col0 + j] = a * fmaf(2.0f, u, -1.0f);
        }
}
static void init_params(orc_t* h)
{
    memset(h->theta, 0, h->P * sizeof(float));
    uint32_t gid = 0;
    for (int l = 0; l < h->L; ++l)
        init_group(h, gid++, h->theta + h->w_off[l], h->dims[l + 1], 0, h->dims[l], h->dims[l + 1]);
    float* Wh = h->theta + h->wh_off;
    int HL = h->dims[h->L];
    if (h->net.policy == POLICY_CATEGORICAL) {
        init_group(h, gid++, Wh, h->NH, 0, HL, h->A);
        init_group(h, gid++, Wh, h->NH, h->A, HL, 1);
    } else {
        init_group(h, gid++, Wh, h->NH, 0, HL, 1);
        init_group(h, gid++, Wh, h->NH, 1, HL, 1);
        init_group(h, gid++, Wh, h->NH, 2, HL, 1);
    }
}

/* R-18 acting forward in binary32, canonical order: every output starts from
 * its bias and adds x_k W[k][j] by fused multiply-add for k = 0, 1, 2, ...
 * R-20 with dtype = 1 the weights and every layer input are first rounded to
 * bfloat16 (products are then exact in binary32), the accumulation, bias and
 * ReLU stay binary32, hidden activations are rounded to bfloat16, head
 * outputs are not.  acts (optional) receives the hidden activations. */
static void forward_f32_with(const orc_t* h, const float* theta, int weights_rounded, const float* x, float* head, float* acts)
{
    float bufa[1024], bufb[1024];
    const float* in = x;
    float* out = bufa;
    int bf = h->net.dtype == 1;
    size_t aoff = 0;
    for (int l = 0; l <= h->L; ++l) {
        int K = h->dims[l];
        int N = (l < h->L) ? h->dims[l + 1] : h->NH;
        const float* W = theta + ((l < h->L) ? h->w_off[l] : h->wh_off);
        const float* bias = theta + ((l < h->L) ? h->b_off[l] : h->bh_off);
        float* y = (l < h->L) ? out : head;
        for (int j = 0; j < N; ++j) y[j] = bias[j];
        for (int k = 0; k < K; ++k) {
            float xk = bf ? orc_bf16_round(in[k]) : in[k];
            for (int j = 0; j < N; ++j) {
                float w = W[(size_t)k * N + j];
                if (bf && !weights_rounded) w = orc_bf16_round(w);
                y[j] = fmaf(xk, w, y[j]);
            }
        }
        if (l < h->L) {
            for (int j = 0; j < N; ++j) {
                float v = y[j] > 0.0f ? y[j] : 0.0f;
                y[j] = bf ? orc_bf16_round(v) : v;
            }
            if (acts) { memcpy(acts + aoff, y, (size_t)N * sizeof(float)); aoff += (size_t)N; }
            in = y;
            out = (y == bufa) ? bufb : bufa;
        }
    }
}

/* with the agent's current parameters (weights rounded on the fly when dtype = 1) */
static void forward_f32(const orc_t* h, const float* x, float* head, float* acts)
{
    forward_f32_with(h, h->theta, 0, x, head, acts);
}

/* ------------------------------------------------------------------------- */
/* Action sampling                                                            */
/* ------------------------------------------------------------------------- */
/* R-21 categorical: inverse CDF over unnormalised exp(logit - max), one
 * uniform; first index whose running sum exceeds u * total. */
int orc_sample_categorical(const float* logits, int A, float u)
{
    float mx = logits[0];
    for (int i = 1; i < A; ++i) if (logits[i] > mx) mx = logits[i];
    float c[16];
    float run = 0.0f;
    for (int i = 0; i < A; ++i) {
        float e = orc_exp(logits[i] - mx);
        run = (i == 0) ? e : run + e;
        c[i] = run;
    }
    float thr = u * c[A - 1];
    for (int i = 0; i < A; ++i) if (c[i] > thr) return i;
    return A - 1;
}
/* R-19 log_sigma is clamped to [-5, 2].  R-22 Box-Muller noise from words 0
 * and 1 of the draw; z = mu + sigma eps; squashed action tanh(z). */
void orc_sample_gaussian(float mu, float log_sigma, uint32_t w0, uint32_t w1, float* eps, float* z_out, float* act)
{
    float ls = log_sigma;
    if (ls < -5.0f) ls = -5.0f;
    if (ls > 2.0f) ls = 2.0f;
    float sigma = orc_exp(ls);
    float rad = sqrtf(-2.0f * orc_log(orc_u01_plus(w0)));
    float e = rad * orc_cos2pi(orc_u01(w1));
    float z = fmaf(sigma, e, mu);
    *eps = e;
    *z_out = z;
    *act = orc_tanh(z);
}

/* ------------------------------------------------------------------------- */
/* Handle                                                                     */
/* ------------------------------------------------------------------------- */
static void* zalloc(size_t n) { void* p = calloc(n ? n : 1, 1); return p; }

void orc_destroy(orc_t* h)
{
    if (!h) return;
    free(h->theta); free(h->m); free(h->v); free(h->grad);
    free(h->si); free(h->sf); free(h->walls);
    free(h->tr_si); free(h->tr_sf); free(h->tr_act); free(h->tr_actf); free(h->tr_eps); free(h->tr_z);
    free(h->tr_rew); free(h->tr_done); free(h->tr_val); free(h->tr_head);
    free(h->adv); free(h->ret); free(h->cur_head); free(h->rho);
    free(h);
}

orc_t* orc_create(const orc_env_cfg* env, const orc_net_cfg* net, int B, int T, uint64_t seed)
{
    if (!env || !net || B <= 0 || T <= 0) return NULL;
    if (net->n_hidden < 1 || net->n_hidden > 4) return NULL;
    orc_t* h = (orc_t*)zalloc(sizeof(orc_t));
    h->env = *env; h->net = *net; h->B = B; h->T = T; h->seed = seed; h->gstep = 0;
    if (env->kind == ENV_CATCH) { h->D = env->rows * env->cols; h->A = 3; }
    else if (env->kind == ENV_PENDULUM) { h->D = 3; h->A = 1; }
    else if (env->kind == ENV_MAZE) { h->D = 3 * env->rows * env->cols; h->A = 4; }
    else { free(h); return NULL; }
    if (env->kind == ENV_MAZE && env->rows * env->cols > 256) { free(h); return NULL; }
    if ((net->policy == POLICY_TANH_GAUSSIAN) != (env->kind == ENV_PENDULUM)) { free(h); return NULL; }
    h->NH = (net->policy == POLICY_CATEGORICAL) ? h->A + 1 : 3;
    h->L = net->n_hidden;
    h->dims[0] = h->D;
    for (int l = 0; l < h->L; ++l) {
        if (net->hidden[l] <= 0 || net->hidden[l] > 1024) { free(h); return NULL; }
        h->dims[l + 1] = net->hidden[l];
    }
    if (h->D > 1024) { free(h); return NULL; }
    size_t off = 0;
    for (int l = 0; l < h->L; ++l) {
        h->w_off[l] = off; off += (size_t)h->dims[l] * h->dims[l + 1];
        h->b_off[l] = off; off += (size_t)h->dims[l + 1];
    }
    h->wh_off = off; off += (size_t)h->dims[h->L] * h->NH;
    h->bh_off = off; off += (size_t)h->NH;
    h->P = off;
    h->theta = (float*)zalloc(h->P * sizeof(float));
    h->m = (double*)zalloc(h->P * sizeof(double));
    h->v = (double*)zalloc(h->P * sizeof(double));
    h->grad = (float*)zalloc(h->P * sizeof(float));
    size_t n = (size_t)B, tn = (size_t)T * B, t1n = (size_t)(T + 1) * B;
    h->si = (int32_t*)zalloc(n * 4 * sizeof(int32_t));
    h->sf = (float*)zalloc(n * 2 * sizeof(float));
    h->walls = (uint32_t*)zalloc(n * 8 * sizeof(uint32_t));
    h->tr_si = (int32_t*)zalloc(t1n * 4 * sizeof(int32_t));
    h->tr_sf = (float*)zalloc(t1n * 2 * sizeof(float));
    h->tr_act = (int32_t*)zalloc(tn * sizeof(int32_t));
    h->tr_actf = (float*)zalloc(tn * sizeof(float));
    h->tr_eps = (float*)zalloc(tn * sizeof(float));
    h->tr_z = (float*)zalloc(tn * sizeof(float));
    h->tr_rew = (float*)zalloc(tn * sizeof(float));
    h->tr_done = (uint8_t*)zalloc(tn);
    h->tr_val = (float*)zalloc(t1n * sizeof(float));
    h->tr_head = (float*)zalloc(t1n * h->NH * sizeof(float));
    h->adv = (double*)zalloc(tn * sizeof(double));
    h->ret = (double*)zalloc(tn * sizeof(double));
    h->cur_head = (double*)zalloc(t1n * h->NH * sizeof(double));
    h->rho = (double*)zalloc(tn * sizeof(double));
    init_params(h);
    for (int b = 0; b < B; ++b) {
        uint32_t w4[4];
        draw4(seed, (uint32_t)b, 0, DOM_INIT, w4);
        int32_t* si = h->si + (size_t)b * 4;
        float* sf = h->sf + (size_t)b * 2;
        if (env->kind == ENV_CATCH) catch_reset(h, w4[0], si);
        else if (env->kind == ENV_PENDULUM) pendulum_reset(w4[0], w4[1], si, sf);
        else { maze_generate(h, b, h->walls + (size_t)b * 8); si[0] = 0; si[1] = 0; }
    }
    return h;
}

/* sizes */
int64_t orc_param_count(const orc_t* h) { return (int64_t)h->P; }
int orc_obs_dim(const orc_t* h) { return h->D; }
int orc_num_heads(const orc_t* h) { return h->NH; }
int64_t orc_act_width(const orc_t* h) { int64_t s = 0; for (int l = 1; l <= h->L; ++l) s += h->dims[l]; return s; }
uint64_t orc_global_step(const orc_t* h) { return h->gstep; }
void orc_set_global_step(orc_t* h, uint64_t g) { h->gstep = g; }

/* raw access for the tests */
float* orc_theta(orc_t* h) { return h->theta; }
float* orc_grad(orc_t* h) { return h->grad; }
double* orc_adam_m(orc_t* h) { return h->m; }
double* orc_adam_v(orc_t* h) { return h->v; }
int orc_get_adam_t(const orc_t* h) { return h->adam_t; }
void orc_set_adam_t(orc_t* h, int t) { h->adam_t = t; }
int32_t* orc_state_i(orc_t* h) { return h->si; }
float* orc_state_f(orc_t* h) { return h->sf; }
uint32_t* orc_walls(orc_t* h) { return h->walls; }
int32_t* orc_traj_state_i(orc_t* h) { return h->tr_si; }
float* orc_traj_state_f(orc_t* h) { return h->tr_sf; }
int32_t* orc_traj_action(orc_t* h) { return h->tr_act; }
float* orc_traj_action_f(orc_t* h) { return h->tr_actf; }
float* orc_traj_eps(orc_t* h) { return h->tr_eps; }
float* orc_traj_z(orc_t* h) { return h->tr_z; }
float* orc_traj_reward(orc_t* h) { return h->tr_rew; }
uint8_t* orc_traj_done(orc_t* h) { return h->tr_done; }
float* orc_traj_value(orc_t* h) { return h->tr_val; }
float* orc_traj_head(orc_t* h) { return h->tr_head; }
double* orc_adv(orc_t* h) { return h->adv; }
double* orc_ret(orc_t* h) { return h->ret; }
double* orc_loss(orc_t* h) { return h->loss; }
double* orc_cur_head(orc_t* h) { return h->cur_head; }
double* orc_rho(orc_t* h) { return h->rho; }

/* observation of env b in its current state, and the forward pass on it */
void orc_observe(const orc_t* h, int b, float* x)
{
    render_obs(h, b, h->si + (size_t)b * 4, h->sf + (size_t)b * 2, x);
}
void orc_forward(const orc_t* h, const float* x, float* head, float* acts)
{
    forward_f32(h, x, head, acts);
}

/* one environment step of env b with a given action (tests use this to drive
 * scripted policies); t is the global env-step number for the reset draw */
void orc_env_step(orc_t* h, int b, int action, float action_f, uint64_t t, float* r, int* done)
{
    uint32_t w4[4];
    draw4(h->seed, (uint32_t)b, t, DOM_RESET, w4);
    int32_t* si = h->si + (size_t)b * 4;
    float* sf = h->sf + (size_t)b * 2;
    if (h->env.kind == ENV_CATCH) catch_step(h, si, action, w4[0], r, done);
    else if (h->env.kind == ENV_PENDULUM) pendulum_step(h, si, sf, action_f, w4[0], w4[1], r, done);
    else maze_step(h, si, h->walls + (size_t)b * 8, action, r, done);
}

/* ------------------------------------------------------------------------- */
/* Rollout: T interactions per env, then the value of the state after the    */
/* last one (paper figure 2 top; section 2.3: state stays on the device       */
/* between calls, so envs continue where the previous unroll stopped).       */
/* forced_head (optional, [T+1][B][NH]): use these head outputs instead of    */
/* the oracle's own forward pass -- for acting paths whose accumulation order */
/* a CPU cannot mirror (matrix-core bf16); sampling and env stepping are      */
/* still the oracle's own.                                                    */
/* ------------------------------------------------------------------------- */
/* sel (optional): roll out only the n_sel listed envs -- envs are independent  */
/* and every draw is keyed by (env, step), so any subset replays exactly.      */
void orc_rollout_sel(orc_t* h, const float* forced_head, const int32_t* sel, int n_sel)
{
    int B = h->B, T = h->T, NH = h->NH;
    float x[1024], head[16];
    int count = sel ? n_sel : B;
    for (int ib = 0; ib < count; ++ib) {
        int b = sel ? sel[ib] : ib;
        int32_t* si = h->si + (size_t)b * 4;
        float* sf = h->sf + (size_t)b * 2;
        for (int t = 0; t <= T; ++t) {
            size_t tb = (size_t)t * B + b;
            memcpy(h->tr_si + tb * 4, si, 4 * sizeof(int32_t));
            memcpy(h->tr_sf + tb * 2, sf, 2 * sizeof(float));
            if (forced_head) memcpy(head, forced_head + tb * NH, NH * sizeof(float));
            else { render_obs(h, b, si, sf, x); forward_f32(h, x, head, NULL); }
            memcpy(h->tr_head + tb * NH, head, NH * sizeof(float));
            h->tr_val[tb] = head[NH - 1];
            if (t == T) break;
            uint64_t gt = h->gstep + (uint64_t)t;
            uint32_t wa[4], wr[4];
            draw4(h->seed, (uint32_t)b, gt, DOM_ACTION, wa);
            draw4(h->seed, (uint32_t)b, gt, DOM_RESET, wr);
            float r; int done;
            if (h->net.policy == POLICY_CATEGORICAL) {
                int a = orc_sample_categorical(head, h->A, orc_u01(wa[0]));
                h->tr_act[tb] = a;
                if (h->env.kind == ENV_CATCH) catch_step(h, si, a, wr[0], &r, &done);
                else maze_step(h, si, h->walls + (size_t)b * 8, a, &r, &done);
            } else {
                float eps, z, act;
                orc_sample_gaussian(head[0], head[1], wa[0], wa[1], &eps, &z, &act);
                h->tr_eps[tb] = eps; h->tr_z[tb] = z; h->tr_actf[tb] = act;
                pendulum_step(h, si, sf, act, wr[0], wr[1], &r, &done);
            }
            h->tr_rew[tb] = r;
            h->tr_done[tb] = (uint8_t)done;
        }
    }
    h->gstep += (uint64_t)T;
    h->have_traj = sel ? 0 : 1;
}
void orc_rollout(orc_t* h, const float* forced_head) { orc_rollout_sel(h, forced_head, NULL, 0); }

/* ------------------------------------------------------------------------- */
/* Returns and advantages (binary64).  With disc = gamma (1 - done):          */
/*   G_T = V(s_T);  G_t = r_{t+1} + disc_{t+1} ((1-lambda) V_{t+1} + lambda G_{t+1})
 * and A_t = G_t - V_t.  R-23: "n-step returns" is lambda = 1, every step      */
/* bootstraps from the end of the unroll unless an episode end cuts it.       */
/* ------------------------------------------------------------------------- */
void orc_returns(int T, int B, const float* rew, const uint8_t* done, const float* val,
                 double gamma, double lambda, double* ret, double* adv)
{
    for (int b = 0; b < B; ++b) {
        double G = (double)val[(size_t)T * B + b];
        for (int t = T - 1; t >= 0; --t) {
            size_t tb = (size_t)t * B + b;
            double disc = done[tb] ? 0.0 : gamma;
            double vnext = (double)val[tb + B];
            G = (double)rew[tb] + disc * ((1.0 - lambda) * vnext + lambda * G);
            ret[tb] = G;
            adv[tb] = G - (double)val[tb];
        }
    }
}

/* ------------------------------------------------------------------------- */
/* Objective and its gradient (binary64).  R-24: per sample                   */
/*   l = -A log pi(a|s) + c_v (G - V)^2 - beta H,   L = mean over B*T,        */
/* with A and G constants.  Gaussian policy: score function at the stored     */
/* pre-squash sample z (the tanh Jacobian does not depend on the parameters), */
/* H = log_sigma + 0.5 log(2 pi e) before squashing (R-26).                   */
/* The forward pass is repeated here in binary64 from the stored states with  */
/* the current parameters (same parameters as at acting time, paper section   */
/* 3.1), with the bfloat16 rounding points of R-20 when dtype = 1.            */
/* ------------------------------------------------------------------------- */
static double qround(const orc_t* h, double v)
{
    return h->net.dtype == 1 ? (double)orc_bf16_round((float)v) : v;
}

/* the parameters as the binary64 forward pass sees them (bfloat16-rounded weights when dtype = 1) */
static double* forward_params64(const orc_t* h, const float* theta_src)
{
    int L = h->L, NH = h->NH;
    double* wq = (double*)zalloc(h->P * sizeof(double));
    for (size_t i = 0; i < h->P; ++i) wq[i] = (double)theta_src[i];
    if (h->net.dtype == 1) {
        for (int l = 0; l < L; ++l)
            for (size_t i = 0; i < (size_t)h->dims[l] * h->dims[l + 1]; ++i)
                wq[h->w_off[l] + i] = (double)orc_bf16_round(theta_src[h->w_off[l] + i]);
        for (size_t i = 0; i < (size_t)h->dims[L] * NH; ++i)
            wq[h->wh_off + i] = (double)orc_bf16_round(theta_src[h->wh_off + i]);
    }
    return wq;
}

/* the same values in binary32 (exact: they are binary32 or bfloat16 numbers), for the pass that takes the
 * branch decisions */
static float* forward_params32(const orc_t* h, const double* wq)
{
    float* w32 = (float*)zalloc(h->P * sizeof(float));
    for (size_t i = 0; i < h->P; ++i) w32[i] = (float)wq[i];
    return w32;
}

/* Learn-time forward pass from the stored state of sample tb.  The VALUES are binary64: act[0] the observation,
 * act[l] the output of hidden layer l, head the NH head outputs.  The BRANCHES are those of the pass the update
 * differentiates, which ran in binary32 (paper section 3.1: the update reuses the policy's forward pass): whether
 * a hidden unit is on the active side of its ReLU (on[l][j]) and whether log_sigma is inside its clamp (head32) are
 * read off the binary32 forward pass of R-18 / R-20 with the same parameters, so a pre-activation within rounding
 * of zero takes the same side here as there.  On the active side a unit's value is its binary64 sum (rounded to
 * bfloat16 when dtype = 1), whatever its sign. */
static void forward64(const orc_t* h, const double* wq, const float* w32, size_t tb, double act[5][1024],
                      unsigned char on[5][1024], double* head, float* head32)
{
    int B = h->B, NH = h->NH, L = h->L;
    float xf[1024], acts32[4 * 1024], h32[16];
    int b = (int)(tb % (size_t)B);
    render_obs(h, b, h->tr_si + tb * 4, h->tr_sf + tb * 2, xf);
    forward_f32_with(h, w32, 1, xf, h32, acts32);
    if (head32) memcpy(head32, h32, (size_t)NH * sizeof(float));
    for (int k = 0; k < h->D; ++k) act[0][k] = qround(h, (double)xf[k]);   /* R-20: every layer input, the observation too */
    size_t aoff = 0;
    for (int l = 0; l < L; ++l) {
        int K = h->dims[l], N = h->dims[l + 1];
        const double* W = wq + h->w_off[l];
        const double* bias = wq + h->b_off[l];
        for (int j = 0; j < N; ++j) {
            double s = bias[j];
            for (int k = 0; k < K; ++k) s += act[l][k] * W[(size_t)k * N + j];
            on[l + 1][j] = acts32[aoff + (size_t)j] > 0.0f;
            act[l + 1][j] = on[l + 1][j] ? qround(h, s) : 0.0;
        }
        aoff += (size_t)N;
    }
    int K = h->dims[L];
    const double* W = wq + h->wh_off;
    for (int j = 0; j < NH; ++j) {
        double s = wq[h->bh_off + j];
        for (int k = 0; k < K; ++k) s += act[L][k] * W[(size_t)k * NH + j];
        head[j] = s;
    }
}

/* Backward pass of one sample: given the forward activations, the ReLU sides and the gradient dhead of a scalar
 * with respect to the head outputs, adds that scalar's parameter gradient to g; dobs (optional)
 * receives its gradient with respect to the observation. */
static void backprop_sample(const orc_t* h, const double* wq, double act[5][1024], unsigned char on[5][1024],
                            const double* dhead, double* g, double* dobs)
{
    int NH = h->NH, L = h->L;
    double dz[2][1024];
    {
        int K = h->dims[L];
        double* gW = g + h->wh_off;
        const double* W = wq + h->wh_off;
        for (int j = 0; j < NH; ++j) g[h->bh_off + j] += dhead[j];
        for (int k = 0; k < K; ++k) {
            double s = 0;
            for (int j = 0; j < NH; ++j) { gW[(size_t)k * NH + j] += act[L][k] * dhead[j]; s += W[(size_t)k * NH + j] * dhead[j]; }
            dz[L & 1][k] = on[L][k] ? s : 0.0;
        }
    }
    for (int l = L - 1; l >= 0; --l) {
        int K = h->dims[l], N = h->dims[l + 1];
        double* gW = g + h->w_off[l];
        const double* W = wq + h->w_off[l];
        const double* d = dz[(l + 1) & 1];
        for (int j = 0; j < N; ++j) g[h->b_off[l] + j] += d[j];
        for (int k = 0; k < K; ++k) {
            double xk = act[l][k], s = 0;
            for (int j = 0; j < N; ++j) { gW[(size_t)k * N + j] += xk * d[j]; s += W[(size_t)k * N + j] * d[j]; }
            if (l > 0) dz[l & 1][k] = on[l][k] ? s : 0.0;
            else if (dobs) dobs[k] = s;
        }
    }
}

/* Loss and gradient over the samples tb_begin <= t*B + b < tb_end (mean over    */
/* those samples), with the parameters theta_src.                              */
static void loss_and_grad_range(orc_t* h, const float* theta_src, size_t tb_begin, size_t tb_end)
{
    int NH = h->NH;
    size_t n = tb_end - tb_begin;
    double inv_n = 1.0 / (double)n;
    double beta = (double)h->net.entropy_coef, cv = (double)h->net.value_coef;
    double* g = (double*)zalloc(h->P * sizeof(double));
    double* wq = forward_params64(h, theta_src);             /* parameters as the forward sees them */
    float* w32 = forward_params32(h, wq);
    double act[5][1024], head[16], dhead[16];
    unsigned char on[5][1024];
    float head32[16];
    double Lp = 0, Lv = 0, Le = 0;
    for (size_t tb = tb_begin; tb < tb_end; ++tb) {
        forward64(h, wq, w32, tb, act, on, head, head32);
        double A_ = h->adv[tb], G_ = h->ret[tb];
        double V = head[NH - 1];
        Lv += cv * (G_ - V) * (G_ - V);
        dhead[NH - 1] = -2.0 * cv * (G_ - V) * inv_n;
        if (h->net.policy == POLICY_CATEGORICAL) {
            int A = h->A, a = h->tr_act[tb];
            double mx = head[0];
            for (int i = 1; i < A; ++i) if (head[i] > mx) mx = head[i];
            double Z = 0, p[16] = {0}, lp[16] = {0}, H = 0;
            for (int i = 0; i < A; ++i) Z += exp(head[i] - mx);
            for (int i = 0; i < A; ++i) { lp[i] = head[i] - mx - log(Z); p[i] = exp(lp[i]); H -= p[i] * lp[i]; }
            Lp += -A_ * lp[a];
            Le += -beta * H;
            for (int i = 0; i < A; ++i)
                dhead[i] = (-A_ * ((i == a ? 1.0 : 0.0) - p[i]) + beta * p[i] * (lp[i] + H)) * inv_n;
        } else {
            double mu = head[0], ls = head[1];
            int clamped = (head32[1] < -5.0f) || (head32[1] > 2.0f);   /* side of the clamp: the binary32 pass decides */
            double lsc = ls < -5.0 ? -5.0 : (ls > 2.0 ? 2.0 : ls);
            double sigma = exp(lsc);
            double eps = ((double)h->tr_z[tb] - mu) / sigma;     /* the sample z is the fixed quantity */
            Lp += -A_ * (-0.5 * eps * eps - lsc - 0.5 * log(2.0 * ORC_PI));
            Le += -beta * (lsc + 0.5 * log(2.0 * ORC_PI * ORC_E));
            dhead[0] = (-A_ * eps / sigma) * inv_n;
            dhead[1] = clamped ? 0.0 : (-A_ * (eps * eps - 1.0) - beta) * inv_n;
        }
        backprop_sample(h, wq, act, on, dhead, g, NULL);
    }
    h->loss[1] = Lp * inv_n; h->loss[2] = Lv * inv_n; h->loss[3] = Le * inv_n;
    h->loss[0] = h->loss[1] + h->loss[2] + h->loss[3];
    for (size_t i = 0; i < h->P; ++i) h->grad[i] = (float)g[i];
    free(g); free(wq); free(w32);
}

void orc_loss_and_grad(orc_t* h)
{
    loss_and_grad_range(h, h->theta, 0, (size_t)h->T * h->B);
}

/* the same over the samples begin <= t*B + b < end only (their own mean): lets a test spread the
 * per-sample work of a large update over several oracle instances, one range each */
int orc_loss_and_grad_range(orc_t* h, int64_t begin, int64_t end)
{
    if (begin < 0 || end <= begin || end > (int64_t)h->T * h->B) return -1;
    loss_and_grad_range(h, h->theta, (size_t)begin, (size_t)end);
    return 0;
}

/* ------------------------------------------------------------------------- */
/* Adam (Kingma & Ba), R-27: bias-corrected, epsilon outside the square root, */
/* no weight decay, no clipping.  Binary64 arithmetic on binary32 parameters. */
/* ------------------------------------------------------------------------- */
void orc_adam(int64_t n, float* theta, const float* grad, double* m, double* v, int t,
              double lr, double beta1, double beta2, double eps)
{
    double bc1 = 1.0 - pow(beta1, (double)t), bc2 = 1.0 - pow(beta2, (double)t);
    for (int64_t i = 0; i < n; ++i) {
        double gi = (double)grad[i];
        m[i] = beta1 * m[i] + (1.0 - beta1) * gi;
        v[i] = beta2 * v[i] + (1.0 - beta2) * gi * gi;
        double mh = m[i] / bc1, vh = v[i] / bc2;
        theta[i] = (float)((double)theta[i] - lr * mh / (sqrt(vh) + eps));
    }
}

/* one update on the stored trajectory */
int orc_learn(orc_t* h)
{
    if (!h->have_traj) return -1;
    orc_returns(h->T, h->B, h->tr_rew, h->tr_done, h->tr_val,
                (double)h->net.gamma, (double)h->net.lambda_, h->ret, h->adv);
    orc_loss_and_grad(h);
    h->adam_t += 1;
    orc_adam((int64_t)h->P, h->theta, h->grad, h->m, h->v, h->adam_t,
             (double)h->net.lr, (double)h->net.beta1, (double)h->net.beta2, (double)h->net.eps);
    h->have_traj = 0;
    return 0;
}

/* N updates on one stored trajectory (paper section 4, the remark on decoupling   */
/* the acting batch from the learning batch: split the batch on the learner and  */
/* apply N updates instead of one larger one).  Reading: the T steps are cut     */
/* into N equal, consecutive time chunks; returns and advantages come from the   */
/* whole unroll; chunk k's gradient is that of its own mean loss at the          */
/* parameters the unroll was acted with (the update reuses the acting forward    */
/* pass, paper section 3.1), and the N Adam steps are applied in chunk order.    */
/* loss[] ends up as the mean of the N chunk losses, grad as the last chunk's.   */
static int learn_n(orc_t* h, int n_updates, int sequential)
{
    if (!h->have_traj) return -1;
    if (n_updates < 1 || h->T % n_updates != 0) return -2;
    orc_returns(h->T, h->B, h->tr_rew, h->tr_done, h->tr_val,
                (double)h->net.gamma, (double)h->net.lambda_, h->ret, h->adv);
    float* theta0 = (float*)malloc(h->P * sizeof(float));
    memcpy(theta0, h->theta, h->P * sizeof(float));
    size_t chunk = (size_t)(h->T / n_updates) * h->B;
    double acc[4] = {0, 0, 0, 0};
    for (int k = 0; k < n_updates; ++k) {
        loss_and_grad_range(h, sequential ? h->theta : theta0, (size_t)k * chunk, (size_t)(k + 1) * chunk);
        for (int i = 0; i < 4; ++i) acc[i] += h->loss[i];
        h->adam_t += 1;
        orc_adam((int64_t)h->P, h->theta, h->grad, h->m, h->v, h->adam_t,
                 (double)h->net.lr, (double)h->net.beta1, (double)h->net.beta2, (double)h->net.eps);
    }
    for (int i = 0; i < 4; ++i) h->loss[i] = acc[i] / (double)n_updates;
    free(theta0);
    h->have_traj = 0;
    return 0;
}
int orc_learn_n(orc_t* h, int n_updates) { return learn_n(h, n_updates, 0); }

/* The other reading of the same remark: chunk k's gradient is taken at the parameters as they are after the k
 * previous updates -- N successive smaller updates in the ordinary sense.  Returns and advantages are still those
 * of the stored unroll (acting-time values), actions and pre-squash samples stay fixed; the forward pass of the
 * chunk is that of the current parameters. */
int orc_learn_n_sequential(orc_t* h, int n_updates) { return learn_n(h, n_updates, 1); }

/* ------------------------------------------------------------------------- */
/* Off-policy update (paper section 3.2 and section 4, "Sebulba": acting and   */
/* learning are decoupled, the actor runs on parameters that lag the learner,   */
/* and the agent the paper runs this way is IMPALA's V-trace).  Reading R-32:   */
/* the targets are V-trace (Espeholt et al. 2018, equations 1 and 4) with the   */
/* learner's own value estimates.  With pi the learner's policy, mu the         */
/* behaviour policy that produced the stored action, disc = gamma (1 - done):   */
/*   w_t   = pi(a_t|s_t) / mu(a_t|s_t)                                          */
/*   rho_t = min(rho_bar, w_t),   c_t = lambda min(c_bar, w_t)                  */
/*   delta_t = rho_t (r_t + disc_t V(s_{t+1}) - V(s_t))                          */
/*   v_t - V(s_t) = delta_t + disc_t c_t (v_{t+1} - V(s_{t+1})),   v_T = V(s_T)  */
/*   policy-gradient advantage  rho_t (r_t + disc_t v_{t+1} - V(s_t))            */
/* and the update is the objective of R-24 with G := v and A := that advantage  */
/* (both constants), at the learner's parameters.  mu comes from the head       */
/* outputs stored at acting time, pi and V from a binary64 forward pass of the  */
/* current parameters over the stored states.  For the tanh-Gaussian policy the  */
/* ratio is taken at the stored pre-squash sample z (the squashing Jacobian is   */
/* the same in both densities).  On-policy (w = 1) with lambda = 1 this is the   */
/* update of orc_learn.                                                         */
/* ------------------------------------------------------------------------- */
static double log_prob_of_stored_action(const orc_t* h, const double* head, size_t tb)
{
    if (h->net.policy == POLICY_CATEGORICAL) {
        int A = h->A, a = h->tr_act[tb];
        double mx = head[0], Z = 0;
        for (int i = 1; i < A; ++i) if (head[i] > mx) mx = head[i];
        for (int i = 0; i < A; ++i) Z += exp(head[i] - mx);
        return head[a] - mx - log(Z);
    }
    double mu = head[0], ls = head[1];
    double lsc = ls < -5.0 ? -5.0 : (ls > 2.0 ? 2.0 : ls);
    double eps = ((double)h->tr_z[tb] - mu) / exp(lsc);
    return -0.5 * eps * eps - lsc - 0.5 * log(2.0 * ORC_PI);
}

void orc_vtrace_targets(orc_t* h, double rho_bar, double c_bar)
{
    int B = h->B, T = h->T, NH = h->NH;
    double gamma = (double)h->net.gamma, lambda = (double)h->net.lambda_;
    double* wq = forward_params64(h, h->theta);
    float* w32 = forward_params32(h, wq);
    double act[5][1024];
    unsigned char on[5][1024];
    for (size_t tb = 0; tb < (size_t)(T + 1) * B; ++tb) forward64(h, wq, w32, tb, act, on, h->cur_head + tb * NH, NULL);
    free(wq); free(w32);
    for (int b = 0; b < B; ++b) {
        double tail = 0.0;                                   /* v_{t+1} - V(s_{t+1}) */
        for (int t = T - 1; t >= 0; --t) {
            size_t tb = (size_t)t * B + b;
            double beh[16];
            for (int j = 0; j < NH; ++j) beh[j] = (double)h->tr_head[tb * NH + j];
            double w = exp(log_prob_of_stored_action(h, h->cur_head + tb * NH, tb) - log_prob_of_stored_action(h, beh, tb));
            double rho = w < rho_bar ? w : rho_bar;
            double c = lambda * (w < c_bar ? w : c_bar);
            double disc = h->tr_done[tb] ? 0.0 : gamma;
            double V = h->cur_head[tb * NH + NH - 1], Vn = h->cur_head[(tb + B) * NH + NH - 1];
            double r = (double)h->tr_rew[tb];
            h->rho[tb] = rho;
            h->adv[tb] = rho * (r + disc * (Vn + tail) - V);
            tail = rho * (r + disc * Vn - V) + disc * c * tail;
            h->ret[tb] = V + tail;
        }
    }
}

int orc_learn_vtrace(orc_t* h, double rho_bar, double c_bar)
{
    if (!h->have_traj) return -1;
    orc_vtrace_targets(h, rho_bar, c_bar);
    orc_loss_and_grad(h);
    h->adam_t += 1;
    orc_adam((int64_t)h->P, h->theta, h->grad, h->m, h->v, h->adam_t,
             (double)h->net.lr, (double)h->net.beta1, (double)h->net.beta2, (double)h->net.eps);
    h->have_traj = 0;
    return 0;
}

/* One decoupled step (reading R-33, the one-device form of the actor/learner split of paper
 * section 3.2 and figure 3): the actor unrolls T steps with a copy of the parameters taken at the
 * start of the step, while the learner applies one off-policy update to the trajectory collected
 * by the previous step.  Neither reads what the other writes, so the order below is one of two
 * equivalent ones.  The first step only collects.  Clipping thresholds rho_bar = c_bar = 1. */
void orc_step_decoupled_forced(orc_t* h, const float* forced_head)
{
    float* behaviour = (float*)malloc(h->P * sizeof(float));
    memcpy(behaviour, h->theta, h->P * sizeof(float));
    if (h->have_traj) orc_learn_vtrace(h, 1.0, 1.0);
    float* learner = h->theta;
    h->theta = behaviour;
    orc_rollout(h, forced_head);                            /* forced_head: as in orc_rollout */
    h->theta = learner;
    free(behaviour);
}
void orc_step_decoupled(orc_t* h) { orc_step_decoupled_forced(h, NULL); }

/* ------------------------------------------------------------------------- */
/* Pathwise policy gradient (paper section 3.1: with the environment part of    */
/* the same program, the unit of T interactions can be differentiated all the   */
/* way through).  Reading R-34, pendulum with the tanh-Gaussian policy only      */
/* (its dynamics are differentiable; the board games are not):                   */
/*   L = L_path + L_value + L_entropy,   L_path = -(1/(B T)) sum_{b,t} r_{b,t}    */
/* where the rewards are those of the stored unroll seen as a function of the     */
/* parameters: the noise eps_t is fixed, a_t = tanh(mu(o_t) + sigma(o_t) eps_t),   */
/* u_t = 2 a_t, r_t and s_{t+1} follow the env's step from (s_t, u_t), and the     */
/* state after an episode end is a reset state that does not depend on the        */
/* parameters.  The velocity clip passes no gradient where it is active; angle    */
/* wrapping and the (never active) torque clip pass it unchanged.  L_value and     */
/* L_entropy are the terms of R-24 with the states held fixed.  The gradient of    */
/* L_path is taken by reverse accumulation over t with the adjoint                 */
/* lambda_t = dL_path/ds_t, linearised at the stored binary32 states:              */
/*   through the step   th' = th + dt thd',  thd' = clip(thd + dt (15 sin th + 3u)) */
/*   through the reward r = -(th^2 + 0.1 thd^2 + 0.001 u^2)                          */
/*   through the policy  u = 2 tanh(mu + exp(clamp(ls)) eps),  o = (cos th, sin th, thd) */
/* path_dhead[t][b][0..1] holds dL_path/d(mu, log_sigma) at every sample.          */
/* ------------------------------------------------------------------------- */
void orc_pathwise_grad(orc_t* h, double* g, double* path_dhead)
{
    int B = h->B, T = h->T, NH = h->NH;
    const double dt = (double)0x1.99999ap-5f, c_thd = (double)0x1.99999ap-4f, c_u = (double)0x1.0624dep-10f;
    const double w = -1.0 / ((double)B * (double)T);           /* dL_path / dr */
    double* wq = forward_params64(h, h->theta);
    float* w32 = forward_params32(h, wq);
    double act[5][1024], head[16], dhead[16], dobs[8];
    unsigned char on[5][1024];
    float head32[16];
    for (int b = 0; b < B; ++b) {
        double lam_th = 0.0, lam_thd = 0.0;                       /* adjoint of the state after step t */
        for (int t = T - 1; t >= 0; --t) {
            size_t tb = (size_t)t * B + b;
            if (h->tr_done[tb]) { lam_th = 0.0; lam_thd = 0.0; }   /* the next state is a reset state */
            forward64(h, wq, w32, tb, act, on, head, head32);
            double th = (double)h->tr_sf[tb * 2], thd = (double)h->tr_sf[tb * 2 + 1];
            double mu = head[0], ls = head[1];
            int clamped = (head32[1] < -5.0f) || (head32[1] > 2.0f);
            double sigma = exp(ls < -5.0 ? -5.0 : (ls > 2.0 ? 2.0 : ls));
            double eps = (double)h->tr_eps[tb];
            double a = tanh(mu + sigma * eps), u = 2.0 * a;
            double pre = thd + dt * (15.0 * sin(th) + 3.0 * u);
            int clipped = (pre < -8.0) || (pre > 8.0);
            /* adjoint through th' = th + dt thd' and the clip */
            double g_nthd = lam_thd + dt * lam_th;
            double g_pre = clipped ? 0.0 : g_nthd;
            double g_th = lam_th + g_pre * dt * 15.0 * cos(th) + w * (-2.0 * th);
            double g_thd = g_pre + w * (-2.0 * c_thd * thd);
            double g_u = g_pre * dt * 3.0 + w * (-2.0 * c_u * u);
            double g_z = 2.0 * g_u * (1.0 - a * a);
            for (int j = 0; j < NH; ++j) dhead[j] = 0.0;
            dhead[0] = g_z;
            dhead[1] = clamped ? 0.0 : g_z * sigma * eps;
            if (path_dhead) { path_dhead[tb * 2] = dhead[0]; path_dhead[tb * 2 + 1] = dhead[1]; }
            backprop_sample(h, wq, act, on, dhead, g, dobs);
            /* o = (cos th, sin th, thd) */
            lam_th = g_th - sin(th) * dobs[0] + cos(th) * dobs[1];
            lam_thd = g_thd + dobs[2];
        }
    }
    free(wq); free(w32);
}

/* one update with the objective of R-34 on the stored unroll */
int orc_learn_pathwise(orc_t* h)
{
    if (!h->have_traj) return -1;
    if (h->env.kind != ENV_PENDULUM || h->net.policy != POLICY_TANH_GAUSSIAN) return -2;
    size_t tn = (size_t)h->T * h->B;
    orc_returns(h->T, h->B, h->tr_rew, h->tr_done, h->tr_val,
                (double)h->net.gamma, (double)h->net.lambda_, h->ret, h->adv);
    for (size_t i = 0; i < tn; ++i) h->adv[i] = 0.0;          /* no score-function term */
    orc_loss_and_grad(h);
    double* g = (double*)zalloc(h->P * sizeof(double));
    for (size_t i = 0; i < h->P; ++i) g[i] = (double)h->grad[i];
    orc_pathwise_grad(h, g, NULL);
    for (size_t i = 0; i < h->P; ++i) h->grad[i] = (float)g[i];
    free(g);
    double rs = 0.0;
    for (size_t i = 0; i < tn; ++i) rs += (double)h->tr_rew[i];
    h->loss[1] = -rs / (double)tn;
    h->loss[0] = h->loss[1] + h->loss[2] + h->loss[3];
    h->adam_t += 1;
    orc_adam((int64_t)h->P, h->theta, h->grad, h->m, h->v, h->adam_t,
             (double)h->net.lr, (double)h->net.beta1, (double)h->net.beta2, (double)h->net.eps);
    h->have_traj = 0;
    return 0;
}

/* the surrogate objective only (no gradient, no update): used by the finite-
 * difference pin, which perturbs theta and calls this */
double orc_surrogate_loss(orc_t* h)
{
    float* keep = (float*)malloc(h->P * sizeof(float));
    memcpy(keep, h->grad, h->P * sizeof(float));
    orc_loss_and_grad(h);
    memcpy(h->grad, keep, h->P * sizeof(float));
    free(keep);
    return h->loss[0];
}

void orc_step(orc_t* h) { orc_rollout(h, NULL); orc_learn(h); }
