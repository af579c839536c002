/*
 * craftax.h - C ABI of the MI355X (gfx950) batched Craftax-Classic simulator.
 *
 * The library implements the environment interface the paper describes in section
 * "RL Environment Interface" (Gymnax-style reset/step with the whole state exposed as one
 * object, 17 discrete actions, symbolic or pixel observations, +1 reward per first-time
 * achievement and +-0.1 per health point) for thousands of independent worlds at once,
 * with the auto-reset of appendix "Optimistic Environment Resets" done exactly (a new
 * world for every finished episode, inside the same step call).
 *
 * Conventions
 *  - Every buffer is owned by the caller.  Pointers marked DEVICE must be HIP device
 *    memory on the current device; pointers marked HOST are ordinary host memory.
 *  - `stream` is a hipStream_t passed as void* (NULL = the default stream).  reset, step,
 *    observe, export and import only enqueue work on it and return without synchronising.
 *  - Return value: 0 on success, negative on error (see CRAFTAX_E_*); the message is
 *    available from craftax_last_error() (thread local).  On error nothing is launched.
 *  - Nothing is allocated by any call except craftax_state_init, which makes one
 *    temporary host staging buffer.
 */
#ifndef CRAFTAX_H
#define CRAFTAX_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define CRAFTAX_ABI_VERSION 1u

enum {
    CRAFTAX_OK = 0,
    CRAFTAX_E_NULL = -1,       /* a required pointer is NULL */
    CRAFTAX_E_ALIGN = -2,      /* state not 256-byte aligned or obs not 16-byte aligned */
    CRAFTAX_E_COUNT = -3,      /* n <= 0, n differs from the state's n, or a range is outside it */
    CRAFTAX_E_STATE = -4,      /* state was not initialised by craftax_state_init in this process */
    CRAFTAX_E_HIP = -5,        /* a HIP call failed */
    CRAFTAX_E_CONFIG = -6      /* unsupported configuration value */
};

enum { CRAFTAX_VARIANT_CLASSIC = 0 };

/* Observation layouts (per environment, stride = craftax_obs_bytes()):
 *  SYM_U8_I8  : bytes [0,1323) 7x9 cells x 21 channels (17-way block one-hot, then zombie,
 *               cow, skeleton, arrow bits), row-major (row, col, channel); int8[22] raw
 *               scalars at byte 1328; stride 1408 (11 cache lines).
 *  SYM_U8_F32 : same cell bytes; float[22] scaled scalars at byte 1328; stride 1536 (12 cache lines).
 *  SYM_F32    : float[1345] = the cell bytes as 0.0/1.0 followed by the 22 scaled scalars
 *               (the flat layout of the paper, section "RL Environment Interface"); stride 5392.
 *  PIXELS_F32 : float[63][63][3] RGB in [0,1]; stride 47632.
 * The 22 scalars: wood, stone, coal, iron, diamond, sapling, wood/stone/iron pickaxe,
 * wood/stone/iron sword, health, food, drink, energy, facing one-hot (left, right, up,
 * down), daylight, sleeping.  Scaled form follows appendix "Observation Space":
 * counts sqrt(n)/10, vitals x/10, flags 0/1.  Unused bytes of the stride are zero. */
enum {
    CRAFTAX_OBS_SYM_U8_I8 = 0,
    CRAFTAX_OBS_SYM_U8_F32 = 1,
    CRAFTAX_OBS_SYM_F32 = 2,
    CRAFTAX_OBS_PIXELS_F32 = 3
};

typedef struct craftax_config {
    uint32_t abi_version;        /* CRAFTAX_ABI_VERSION */
    uint32_t variant;            /* CRAFTAX_VARIANT_CLASSIC */
    uint32_t obs_mode;           /* CRAFTAX_OBS_* */
    uint32_t max_episode_steps;  /* episode is cut (done = 1) when this many steps were taken */
    uint32_t day_length;         /* even, 2..1024 */
    uint32_t cap_zombie, cap_cow, cap_skeleton, cap_arrow;  /* 0..3 each (appendix "Differences
                                    between Craftax-Classic and Crafter": fixed, masked slots) */
    uint32_t cap_plant;          /* 0..10 */
    uint64_t atlas_seed;         /* seed of the synthetic tile atlas (pixel observations) */
} craftax_config;

/* One environment in canonical form, used by export/import (4304 bytes, little endian).
 * Dead mob and plant slots are all zero.  Mob slots: 0-2 zombie, 3-5 cow, 6-8 skeleton,
 * 9-11 arrow. */
typedef struct craftax_mob { uint8_t alive, x, y, dir; int8_t hp; uint8_t cd; uint8_t pad[2]; } craftax_mob;
typedef struct craftax_plant { uint8_t alive, x, y, pad; uint16_t age; } craftax_plant;
typedef struct craftax_env_dump {
    uint8_t map[64 * 64];       /* block ids (appendix "Block Types"), index y*64+x */
    uint8_t px, py, dir, sleeping;
    uint8_t inv[12];
    int8_t vit[4];              /* health, food, drink, energy */
    int16_t cnt[4];             /* hunger, thirst, fatigue, recover */
    uint32_t ach;               /* bit i = achievement id i (appendix "Achievements") */
    uint32_t t, episode;
    uint64_t seed;
    craftax_mob mob[12];
    craftax_plant plant[10];
    uint32_t env;
} craftax_env_dump;

/* Fills *cfg (HOST) with the defaults: Classic, SYM_U8_F32, 10000 steps, day 300, caps 3/3/3/3/10. */
void craftax_default_config(craftax_config *cfg);

/* Bytes of device memory the caller must provide for n environments (0 on a bad config). */
size_t craftax_state_bytes(const craftax_config *cfg, int n);
/* Per-environment observation stride in bytes for cfg->obs_mode (multiple of 16). */
size_t craftax_obs_bytes(const craftax_config *cfg);
/* sizeof(craftax_env_dump). */
size_t craftax_env_dump_bytes(void);

/* Writes the header, lookup tables and tile atlas into `state` (DEVICE, 256-byte aligned,
 * craftax_state_bytes() long) and registers it with the library.  Environments hold no
 * valid world until craftax_reset.  cfg is HOST. */
int craftax_state_init(void *state, const craftax_config *cfg, int n, void *stream);
/* Forgets a state registered by craftax_state_init (the memory stays the caller's). */
int craftax_state_release(void *state);

/* Starts episode 0 of every environment: env i gets seeds[i] (DEVICE, n x uint64) as its
 * Philox key for all later episodes, a generated 64x64 world, full vitals, empty tables. */
int craftax_reset(void *state, const uint64_t *seeds, int n, void *stream);

/* One step of every environment.  actions: DEVICE int32[n]; ids outside 0..16 act as NOOP.
 * Outputs (all DEVICE): obs (n x craftax_obs_bytes(), 16-byte aligned), reward float[n],
 * done uint8[n].  When done[i] = 1 the reward belongs to the episode that just ended and
 * state and obs already hold the first state of the next episode.  obs may be NULL to skip
 * rendering. */
int craftax_step(void *state, const int32_t *actions, void *obs, float *reward, uint8_t *done,
                 int n, void *stream);

/* Renders the current observation of every environment (used after craftax_reset). */
int craftax_observe(void *state, void *obs, int n, void *stream);

/* Copies environments [first, first+count) to / from canonical dumps in DEVICE memory
 * (count x craftax_env_dump).  Import is the state-editing hook: the paper notes that the
 * whole environment state is one object that level editors can modify. */
int craftax_export_envs(const void *state, int first, int count, void *dumps, void *stream);
int craftax_import_envs(void *state, int first, int count, const void *dumps, void *stream);

/* Fills actions (DEVICE int32[steps][n]) with the synthetic action stream used by the
 * benchmark: kind 0 = uniform over 17 actions, kind 1 = half of the draws restricted to
 * ids 1..5.  Input generation only; not part of the simulator. */
int craftax_synth_actions(int32_t *actions, int n, int step0, int steps, uint64_t action_seed,
                          int kind, void *stream);

const char *craftax_last_error(void);

#ifdef __cplusplus
}
#endif
#endif
