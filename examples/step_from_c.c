/*
 * A caller of the C ABI without Python or PyTorch: plain HIP runtime calls for memory, the
 * library for everything else.  Resets n Craftax-Classic environments, takes a number of steps
 * with a fixed action pattern and prints checksums of the rewards, finished episodes and the
 * last observation.  tests/test_gpu_c_example.py runs it and compares the sums with the
 * same run through the Python binding.  Build: see build_example in paper_2402_16801_amd/build.py.
 *
 *   step_from_c [n] [steps]
 */
#include <hip/hip_runtime_api.h>
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>

#include "../include/craftax.h"

#define CHECK_HIP(call) do { hipError_t e_ = (call); if (e_ != hipSuccess) { fprintf(stderr, "%s: %s\n", #call, hipGetErrorString(e_)); return 2; } } while (0)
#define CHECK_CX(call) do { int r_ = (call); if (r_ != CRAFTAX_OK) { fprintf(stderr, "%s: %d %s\n", #call, r_, craftax_last_error()); return 3; } } while (0)

int main(int argc, char **argv)
{
    const int n = argc > 1 ? atoi(argv[1]) : 1000;
    const int steps = argc > 2 ? atoi(argv[2]) : 50;
    if (n <= 0 || steps <= 0) { fprintf(stderr, "usage: step_from_c [n] [steps]\n"); return 1; }

    craftax_config cfg;
    craftax_default_config(&cfg);
    cfg.max_episode_steps = 20;                       /* short episodes: auto-resets inside the run */
    const size_t state_bytes = craftax_state_bytes(&cfg, n), stride = craftax_obs_bytes(&cfg);
    if (state_bytes == 0) { fprintf(stderr, "bad configuration\n"); return 1; }

    void *state, *obs;
    uint64_t *seeds;
    int32_t *actions;
    float *reward;
    uint8_t *done;
    CHECK_HIP(hipMalloc(&state, state_bytes));
    CHECK_HIP(hipMalloc(&obs, stride * (size_t)n));
    CHECK_HIP(hipMalloc((void **)&seeds, sizeof(uint64_t) * (size_t)n));
    CHECK_HIP(hipMalloc((void **)&actions, sizeof(int32_t) * (size_t)n));
    CHECK_HIP(hipMalloc((void **)&reward, sizeof(float) * (size_t)n));
    CHECK_HIP(hipMalloc((void **)&done, (size_t)n));

    uint64_t *h_seeds = (uint64_t *)malloc(sizeof(uint64_t) * (size_t)n);
    int32_t *h_actions = (int32_t *)malloc(sizeof(int32_t) * (size_t)n);
    float *h_reward = (float *)malloc(sizeof(float) * (size_t)n);
    uint8_t *h_done = (uint8_t *)malloc((size_t)n);
    uint8_t *h_obs = (uint8_t *)malloc(stride * (size_t)n);
    for (int i = 0; i < n; i++) h_seeds[i] = 0x9E3779B97F4A7C15ull * (uint64_t)(i + 1);
    CHECK_HIP(hipMemcpy(seeds, h_seeds, sizeof(uint64_t) * (size_t)n, hipMemcpyHostToDevice));

    CHECK_CX(craftax_state_init(state, &cfg, n, NULL));
    CHECK_CX(craftax_reset(state, seeds, n, NULL));

    long long reward_tenths = 0;                      /* rewards are multiples of 0.1: an exact checksum */
    unsigned long long done_sum = 0, obs_sum = 0;
    for (int t = 0; t < steps; t++) {
        for (int i = 0; i < n; i++) h_actions[i] = (int32_t)((i * 7 + t * 3) % 17);
        CHECK_HIP(hipMemcpy(actions, h_actions, sizeof(int32_t) * (size_t)n, hipMemcpyHostToDevice));
        CHECK_CX(craftax_step(state, actions, obs, reward, done, n, NULL));
        CHECK_HIP(hipMemcpy(h_reward, reward, sizeof(float) * (size_t)n, hipMemcpyDeviceToHost));
        CHECK_HIP(hipMemcpy(h_done, done, (size_t)n, hipMemcpyDeviceToHost));
        for (int i = 0; i < n; i++) { reward_tenths += llround((double)h_reward[i] * 10.0); done_sum += h_done[i]; }
    }
    CHECK_HIP(hipMemcpy(h_obs, obs, stride * (size_t)n, hipMemcpyDeviceToHost));
    for (size_t i = 0; i < stride * (size_t)n; i++) obs_sum += (unsigned long long)h_obs[i] * (unsigned long long)(i % 251 + 1);
    printf("n=%d steps=%d reward_tenths=%lld done_sum=%llu obs_sum=%llu\n", n, steps, reward_tenths, done_sum, obs_sum);

    CHECK_CX(craftax_state_release(state));
    hipFree(state); hipFree(obs); hipFree(seeds); hipFree(actions); hipFree(reward); hipFree(done);
    free(h_seeds); free(h_actions); free(h_reward); free(h_done); free(h_obs);
    return 0;
}
