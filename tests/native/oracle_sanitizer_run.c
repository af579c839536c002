/* Drives every entry point of the CPU oracle under AddressSanitizer and UndefinedBehaviorSanitizer
 * (built and run by tests/test_native_checks.py): resets, steps with all observation layouts,
 * both world generators, both reset modes, the mutations, both variants.  The inputs come from a
 * small counter generator of its own; the point is memory safety, not values.  Exit code 0 and no
 * sanitizer report = clean. */
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include "../../oracle/craftax_oracle.h"
#include "../../oracle/craftax_full.h"

static uint32_t lcg_state = 12345u;
static uint32_t lcg(void) { lcg_state = lcg_state * 1664525u + 1013904223u; return lcg_state >> 8; }

static void classic(int n, int steps, uint32_t worldgen, uint32_t reset_mode, uint32_t cap)
{
    orc_config cfg;
    orc_default_config(&cfg);
    cfg.worldgen = worldgen; cfg.reset_mode = reset_mode; cfg.max_episode_steps = cap;
    orc_env *envs = calloc((size_t)n, sizeof(orc_env));
    uint64_t *seeds = malloc((size_t)n * 8);
    int32_t *actions = malloc((size_t)n * 4);
    float *reward = malloc((size_t)n * 4);
    uint8_t *done = malloc((size_t)n);
    for (int i = 0; i < n; i++) seeds[i] = 1000u + (uint64_t)i * 0x100000001ull;
    orc_reset_batch(envs, &cfg, seeds, NULL, n);
    for (int mode = 0; mode < 4; mode++) {
        uint8_t *obs = malloc(orc_obs_bytes(mode) * (size_t)n);      /* exactly the documented size: overruns are caught */
        for (int s = 0; s < steps; s++) {
            for (int i = 0; i < n; i++) actions[i] = (int32_t)(lcg() % 19u) - 1;     /* includes two ids outside the table */
            if (reset_mode == ORC_RESET_POOL) orc_step_batch_pool(envs, &cfg, actions, mode, obs, reward, done, n, (uint32_t)(mode * steps + s));
            else orc_step_batch(envs, &cfg, actions, mode, obs, reward, done, n);
        }
        orc_observe_batch(envs, &cfg, mode, obs, n);
        free(obs);
    }
    /* players at the four map corners look beyond the map in every renderer */
    for (int i = 0; i < n && i < 4; i++) { envs[i].px = (i & 1) ? 63 : 0; envs[i].py = (i & 2) ? 63 : 0; }
    for (int mode = 0; mode < 4; mode++) {
        uint8_t *obs = malloc(orc_obs_bytes(mode) * (size_t)n);
        orc_observe_batch(envs, &cfg, mode, obs, n);
        for (int i = 0; i < n; i++) actions[i] = 1 + (int32_t)(lcg() % 5u);
        orc_step_batch(envs, &cfg, actions, mode, obs, reward, done, n);
        free(obs);
    }
    for (int i = 0; i < n; i++) {
        orc_mutate_swap(&envs[i], 99, (uint32_t)i, i & 1);
        if (worldgen == ORC_WORLDGEN_PERLIN) {
            uint16_t theta[ORC_THETA_LEN];
            memset(theta, 0, sizeof(theta));
            orc_mutate_noise(&envs[i], &cfg, theta, 7, (uint32_t)i, 511);
            orc_mutate_noise(&envs[i], &cfg, theta, 7, (uint32_t)i + 1u, 0);
        }
    }
    free(envs); free(seeds); free(actions); free(reward); free(done);
}

static void full(int n, int steps, uint32_t worldgen, uint32_t reset_mode, uint32_t cap)
{
    cf_config cfg;
    cf_default_config(&cfg);
    cfg.worldgen = worldgen; cfg.reset_mode = reset_mode; cfg.max_episode_steps = cap;
    cf_env *envs = calloc((size_t)n, sizeof(cf_env));
    uint64_t *seeds = malloc((size_t)n * 8);
    int32_t *actions = malloc((size_t)n * 4);
    float *reward = malloc((size_t)n * 4);
    uint8_t *done = malloc((size_t)n);
    for (int i = 0; i < n; i++) seeds[i] = 5u + (uint64_t)i;
    cf_reset_batch(envs, &cfg, seeds, NULL, n);
    for (int mode = 0; mode < 3; mode++) {
        uint8_t *obs = malloc(cf_obs_bytes(mode) * (size_t)n);
        for (int s = 0; s < steps; s++) {
            for (int i = 0; i < n; i++) actions[i] = (int32_t)(lcg() % 45u) - 1;
            if (reset_mode == 1u) cf_step_batch_pool(envs, &cfg, actions, mode, obs, reward, done, n, (uint32_t)(mode * steps + s));
            else cf_step_batch(envs, &cfg, actions, mode, obs, reward, done, n);
            if (s == steps / 2)      /* move everybody somewhere else: every floor, map corners included */
                for (int i = 0; i < n; i++) {
                    envs[i].floor = (uint8_t)(i % 9);
                    envs[i].px = (uint8_t)((i & 1) ? 47 : (i & 4) ? 24 : 0);
                    envs[i].py = (uint8_t)((i & 2) ? 47 : (i & 4) ? 24 : 0);
                    memset(envs[i].inv, 20, sizeof(envs[i].inv));
                    memset(envs[i].potion, 2, sizeof(envs[i].potion));
                    envs[i].bow = 1; envs[i].book = 2; envs[i].learned_fireball = 1; envs[i].learned_iceball = 1;
                    envs[i].vit[4] = 9;
                }
        }
        cf_observe_batch(envs, &cfg, mode, obs, n);
        free(obs);
    }
    for (int i = 0; i < n; i++) {
        cf_mutate_swap(&envs[i], 3, (uint32_t)i, i & 1);
        if (worldgen == 1u) {
            uint16_t theta[CF_THETA_LEN];
            memset(theta, 0, sizeof(theta));
            cf_mutate_noise(&envs[i], &cfg, theta, 7, (uint32_t)i, 300);
        }
    }
    free(envs); free(seeds); free(actions); free(reward); free(done);
}

int main(void)
{
    classic(24, 100, ORC_WORLDGEN_VALUE, ORC_RESET_EXACT, 40);
    classic(8, 12, ORC_WORLDGEN_PERLIN, ORC_RESET_EXACT, 1);
    classic(33, 30, ORC_WORLDGEN_VALUE, ORC_RESET_POOL, 7);
    full(18, 60, 0u, 0u, 50);
    full(4, 6, 1u, 0u, 1);
    full(17, 14, 0u, 1u, 6);
    printf("oracle_sanitizer_run: ok\n");
    return 0;
}
