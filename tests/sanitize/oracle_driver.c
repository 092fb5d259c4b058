/* Runs every entry point of the CPU oracle on small cases of each environment.  Built with
 * -fsanitize=address,undefined by tests/test_oracle_sanitize.py: an out-of-bounds access, a use
 * after free, a leak, a signed overflow or a misaligned access anywhere on these paths ends the
 * run with a non-zero status.  TEST INFRASTRUCTURE: the oracle is included as source, nothing of
 * the GPU path is. */
#include "../../oracle/anakin_oracle.c"

#include <stdio.h>

static orc_net_cfg net(int n_hidden, int h0, int h1, int policy, int dtype)
{
    orc_net_cfg n;
    memset(&n, 0, sizeof n);
    n.n_hidden = n_hidden; n.hidden[0] = h0; n.hidden[1] = h1;
    n.policy = policy; n.dtype = dtype;
    n.gamma = 0.99f; n.lambda_ = 0.95f; n.entropy_coef = 0.01f; n.value_coef = 0.5f;
    n.lr = 1e-3f; n.beta1 = 0.9f; n.beta2 = 0.999f; n.eps = 1e-8f;
    return n;
}

static int run_case(const char* name, orc_env_cfg env, orc_net_cfg nc, int B, int T)
{
    orc_t* h = orc_create(&env, &nc, B, T, 1234u);
    if (!h) { fprintf(stderr, "%s: create failed\n", name); return 1; }
    int bad = 0;
    /* acting and the plain update */
    orc_rollout(h, NULL);
    bad |= orc_learn(h) != 0;
    /* several updates per unroll, both readings */
    orc_rollout(h, NULL);
    bad |= orc_learn_n(h, 2) != 0;
    orc_rollout(h, NULL);
    bad |= orc_learn_n_sequential(h, 2) != 0;
    /* a range of the loss on its own, as the threaded test helper calls it */
    orc_rollout(h, NULL);
    bad |= orc_loss_and_grad_range(h, 0, (int64_t)B * T / 2) != 0;
    orc_loss_and_grad(h);
    /* off-policy: targets, update, decoupled steps */
    orc_rollout(h, NULL);
    orc_vtrace_targets(h, 1.0, 1.0);
    bad |= orc_learn_vtrace(h, 1.0, 1.0) != 0;
    orc_step_decoupled(h);
    orc_step_decoupled(h);
    if (env.kind == ENV_PENDULUM && nc.dtype == 0) {
        orc_rollout(h, NULL);
        bad |= orc_learn_pathwise(h) != 0;
    }
    /* selected environments with forced head outputs */
    {
        const int32_t sel[2] = {0, B - 1};
        float* forced = (float*)calloc((size_t)(T + 1) * B * h->NH, sizeof(float));
        orc_rollout_sel(h, forced, sel, 2);
        free(forced);
    }
    double s = 0.0;
    for (size_t i = 0; i < h->P; ++i) s += h->theta[i];
    if (!(s == s)) { fprintf(stderr, "%s: parameters are not finite\n", name); bad = 1; }
    printf("%s: P=%zu sum(theta)=%.6f %s\n", name, h->P, s, bad ? "FAILED" : "ok");
    orc_destroy(h);
    return bad;
}

int main(void)
{
    int bad = 0;
    orc_env_cfg catch_env = {ENV_CATCH, 10, 5, 0, 0.0f};
    orc_env_cfg pend_env = {ENV_PENDULUM, 0, 0, 20, 0.0f};
    orc_env_cfg maze_env = {ENV_MAZE, 8, 8, 12, 0.2f};
    bad |= run_case("catch 1x32 fp32", catch_env, net(1, 32, 0, POLICY_CATEGORICAL, 0), 6, 4);
    bad |= run_case("catch 64x64 fp32", catch_env, net(2, 64, 64, POLICY_CATEGORICAL, 0), 5, 6);
    bad |= run_case("pendulum 32x32 fp32", pend_env, net(2, 32, 32, POLICY_TANH_GAUSSIAN, 0), 4, 8);
    bad |= run_case("pendulum 32x32 bf16", pend_env, net(2, 32, 32, POLICY_TANH_GAUSSIAN, 1), 4, 4);
    bad |= run_case("maze 32x32 fp32", maze_env, net(2, 32, 32, POLICY_CATEGORICAL, 0), 3, 6);
    bad |= run_case("maze 64x32 bf16", maze_env, net(2, 64, 32, POLICY_CATEGORICAL, 1), 4, 4);
    /* the scalar helpers at their edges */
    volatile float sink = 0.0f;
    const float xs[] = {-200.0f, -87.5f, -1.0f, -0.0f, 0.0f, 1e-30f, 1.0f, 88.0f, 200.0f, 1e30f};
    for (unsigned i = 0; i < sizeof xs / sizeof xs[0]; ++i) {
        sink += orc_exp(xs[i] > 88.0f ? 88.0f : xs[i]) * 0.0f;
        if (xs[i] > 0.0f) sink += orc_log(xs[i]) * 0.0f;
        sink += orc_tanh(xs[i]) + orc_sin(xs[i] > 1e3f ? 1e3f : xs[i]) + orc_cos2pi(0.25f) + orc_bf16_round(xs[i]);
    }
    for (uint32_t n = 1; n < 70; n += 7) sink += (float)orc_bounded(0xfffffff0u + n, n);
    (void)sink;
    return bad;
}
