/* A client of libpql.so written in plain C99 against include/pql.h and the HIP runtime API: no Python,
 * no torch.  It reads one seeded problem from a file, runs the calls of one learner iteration
 * (Algorithms 1-3: push the Actor's steps, sample a batch, critic update, Polyak step, policy update,
 * hard copy into the lagged policy, one Actor step) on device memory it allocates itself, and writes
 * the results to a second file.  tests/test_zy_c_client.py compares them with the Python session's,
 * bit for bit.
 *
 * Input (little endian):  int32 obs_dim, act_dim, num_envs, nstep, n_hidden, hidden[8], batch, rows;
 *                         int64 capacity; uint64 seed; float gamma, lr, beta1, beta2, eps, tau, sigma_min, sigma_max;
 *                         float actor[Pa], critic[2 Pc];
 *                         rows x { float obs[N o], act[N a], rew[N], next_obs[N o], done[N] };
 *                         float act_obs[N o]   (observations of the Actor step)
 * Output:                 int64 idx[batch]; float loss[2], actor_loss; float critic[2 Pc], critic_target[2 Pc],
 *                         actor[Pa], actor_lagged[Pa], actions[N a]
 */
#include <hip/hip_runtime_api.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include "pql.h"

#define CHECK_HIP(x) do { hipError_t e_ = (x); if (e_ != hipSuccess) { \
    fprintf(stderr, "%s:%d: %s\n", __FILE__, __LINE__, hipGetErrorString(e_)); return 2; } } while (0)
#define CHECK_PQL(x) do { int32_t r_ = (x); if (r_ != PQL_OK) { \
    fprintf(stderr, "%s:%d: pql error %d: %s\n", __FILE__, __LINE__, (int)r_, pql_last_error(ctx)); return 3; } } while (0)

static int read_exact(FILE* f, void* dst, size_t bytes) { return fread(dst, 1, bytes, f) == bytes ? 0 : -1; }

static float* dev_floats(size_t n) {
    void* p = NULL;
    if (hipMalloc(&p, (n ? n : 1) * sizeof(float)) != hipSuccess) return NULL;
    return (float*)p;
}

int main(int argc, char** argv) {
    if (argc != 3) { fprintf(stderr, "usage: %s <problem file> <result file>\n", argv[0]); return 1; }
    FILE* in = fopen(argv[1], "rb");
    if (!in) { perror(argv[1]); return 1; }
    int32_t head[15];
    int64_t capacity;
    uint64_t seed;
    float hp[8];
    if (read_exact(in, head, sizeof(head)) || read_exact(in, &capacity, 8) || read_exact(in, &seed, 8) ||
        read_exact(in, hp, sizeof(hp))) { fprintf(stderr, "short header\n"); return 1; }
    pql_config cfg;
    memset(&cfg, 0, sizeof(cfg));
    cfg.obs_dim = head[0]; cfg.act_dim = head[1]; cfg.num_envs = head[2]; cfg.nstep = head[3]; cfg.n_hidden = head[4];
    for (int i = 0; i < PQL_MAX_HIDDEN; ++i) cfg.hidden[i] = head[5 + i];
    const int32_t batch = head[13], rows = head[14];
    cfg.capacity = capacity; cfg.seed = seed; cfg.gamma = hp[0];
    cfg.max_batch = batch > cfg.num_envs ? batch : cfg.num_envs;
    const pql_adam opt = {hp[1], hp[2], hp[3], hp[4], 0.f};
    const float tau = hp[5], sigma_min = hp[6], sigma_max = hp[7];

    pql_ctx* ctx = NULL;
    CHECK_PQL(pql_create(&cfg, &ctx));
    const size_t N = (size_t)cfg.num_envs, o = (size_t)cfg.obs_dim, a = (size_t)cfg.act_dim, B = (size_t)batch;
    const size_t T = (size_t)pql_replay_rows(&cfg);
    const size_t Pa = (size_t)pql_actor_param_count(&cfg), Pc2 = 2 * (size_t)pql_critic_param_count(&cfg);
    const size_t ws_bytes = (size_t)pql_workspace_bytes(&cfg);

    /* device memory: all of it the caller's */
    pql_replay_storage st = {dev_floats(T * N * o), dev_floats(T * N * a), dev_floats(T * N), dev_floats(T * N * o), dev_floats(T * N)};
    pql_batch bt;
    void* idx_dev = NULL;
    CHECK_HIP(hipMalloc(&idx_dev, B * sizeof(int64_t)));
    bt.idx = (int64_t*)idx_dev; bt.obs = dev_floats(B * o); bt.act = dev_floats(B * a); bt.ret = dev_floats(B);
    bt.next_obs = dev_floats(B * o); bt.boot = dev_floats(B);
    float *actor = dev_floats(Pa), *actor_lag = dev_floats(Pa), *a_m = dev_floats(Pa), *a_v = dev_floats(Pa), *a_g = dev_floats(Pa);
    float *critic = dev_floats(Pc2), *critic_t = dev_floats(Pc2), *c_m = dev_floats(Pc2), *c_v = dev_floats(Pc2), *c_g = dev_floats(Pc2);
    float *row_obs = dev_floats(N * o), *row_act = dev_floats(N * a), *row_rew = dev_floats(N), *row_next = dev_floats(N * o),
          *row_done = dev_floats(N), *actions = dev_floats(N * a), *losses = dev_floats(8);
    void* ws = NULL;
    CHECK_HIP(hipMalloc(&ws, ws_bytes));
    if (!st.obs || !st.act || !st.rew || !st.next_obs || !st.done || !bt.obs || !bt.act || !bt.ret || !bt.next_obs || !bt.boot ||
        !actor || !actor_lag || !a_m || !a_v || !a_g || !critic || !critic_t || !c_m || !c_v || !c_g || !row_obs || !row_act ||
        !row_rew || !row_next || !row_done || !actions || !losses) { fprintf(stderr, "hipMalloc failed\n"); return 2; }
    hipStream_t stream;
    CHECK_HIP(hipStreamCreate(&stream));

    /* parameters: targets and the lagged policy start as copies, moments at zero */
    size_t biggest = Pa > Pc2 ? Pa : Pc2;
    if (N * o > biggest) biggest = N * o;
    float* host = (float*)malloc(biggest * sizeof(float));
    if (!host) return 1;
    if (read_exact(in, host, Pa * sizeof(float))) return 1;
    CHECK_HIP(hipMemcpy(actor, host, Pa * sizeof(float), hipMemcpyHostToDevice));
    CHECK_HIP(hipMemcpy(actor_lag, host, Pa * sizeof(float), hipMemcpyHostToDevice));
    if (read_exact(in, host, Pc2 * sizeof(float))) return 1;
    CHECK_HIP(hipMemcpy(critic, host, Pc2 * sizeof(float), hipMemcpyHostToDevice));
    CHECK_HIP(hipMemcpy(critic_t, host, Pc2 * sizeof(float), hipMemcpyHostToDevice));
    CHECK_HIP(hipMemset(a_m, 0, Pa * sizeof(float))); CHECK_HIP(hipMemset(a_v, 0, Pa * sizeof(float)));
    CHECK_HIP(hipMemset(c_m, 0, Pc2 * sizeof(float))); CHECK_HIP(hipMemset(c_v, 0, Pc2 * sizeof(float)));

    /* the Actor's steps go into the ring one row of N transitions at a time */
    for (int32_t r = 0; r < rows; ++r) {
        float* dst[5] = {row_obs, row_act, row_rew, row_next, row_done};
        const size_t len[5] = {N * o, N * a, N, N * o, N};
        for (int k = 0; k < 5; ++k) {
            if (read_exact(in, host, len[k] * sizeof(float))) { fprintf(stderr, "short row %d\n", (int)r); return 1; }
            CHECK_HIP(hipMemcpy(dst[k], host, len[k] * sizeof(float), hipMemcpyHostToDevice));
        }
        CHECK_PQL(pql_replay_push(ctx, st, row_obs, row_act, row_rew, row_next, row_done, stream));
        CHECK_HIP(hipStreamSynchronize(stream));      /* the staging buffers are reused by the next row */
    }
    if (read_exact(in, host, N * o * sizeof(float))) { fprintf(stderr, "short Actor observations\n"); return 1; }
    CHECK_HIP(hipMemcpy(row_obs, host, N * o * sizeof(float), hipMemcpyHostToDevice));
    fclose(in);

    /* one iteration of the learners, then one Actor step */
    CHECK_PQL(pql_sample_nstep(ctx, st, batch, bt, stream));
    CHECK_PQL(pql_critic_update(ctx, critic, critic_t, actor_lag, c_m, c_v, c_g, bt, batch, opt, losses, ws, stream));   /* L_1, L_2, norm */
    CHECK_PQL(pql_soft_update(ctx, critic, critic_t, (int64_t)Pc2, tau, stream));
    CHECK_PQL(pql_actor_update(ctx, actor, critic, a_m, a_v, a_g, bt.obs, batch, opt, losses + 4, ws, stream));   /* J, norm */
    CHECK_PQL(pql_soft_update(ctx, actor, actor_lag, (int64_t)Pa, 1.0f, stream));
    CHECK_PQL(pql_actor_act(ctx, actor, row_obs, cfg.num_envs, sigma_min, sigma_max, actions, ws, stream));
    CHECK_HIP(hipStreamSynchronize(stream));

    FILE* out = fopen(argv[2], "wb");
    if (!out) { perror(argv[2]); return 1; }
    int64_t* idx_host = (int64_t*)malloc(B * sizeof(int64_t));
    float loss_host[8];
    if (!idx_host) return 1;
    CHECK_HIP(hipMemcpy(idx_host, bt.idx, B * sizeof(int64_t), hipMemcpyDeviceToHost));
    CHECK_HIP(hipMemcpy(loss_host, losses, sizeof(loss_host), hipMemcpyDeviceToHost));
    fwrite(idx_host, sizeof(int64_t), B, out);
    fwrite(loss_host, sizeof(float), 2, out);
    fwrite(loss_host + 4, sizeof(float), 1, out);
    const float* vecs[5] = {critic, critic_t, actor, actor_lag, actions};
    const size_t lens[5] = {Pc2, Pc2, Pa, Pa, N * a};
    float* big = (float*)malloc((Pc2 > N * a ? Pc2 : N * a) * sizeof(float) + Pa * sizeof(float));
    if (!big) return 1;
    for (int k = 0; k < 5; ++k) {
        CHECK_HIP(hipMemcpy(big, vecs[k], lens[k] * sizeof(float), hipMemcpyDeviceToHost));
        fwrite(big, sizeof(float), lens[k], out);
    }
    fclose(out);
    int64_t state[8];
    CHECK_PQL(pql_get_state(ctx, state));
    printf("pushes %lld samples %lld acts %lld critic steps %lld policy steps %lld\n", (long long)state[2], (long long)state[3],
           (long long)state[4], (long long)state[5], (long long)state[6]);
    CHECK_PQL(pql_destroy(ctx));
    return 0;
}
