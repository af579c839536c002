/*
 * CPU oracle for the Craftax-Classic reset/step/observe path.
 *
 * TEST INFRASTRUCTURE ONLY.  This is a plain, single-threaded, deliberately slow
 * simulator used to check the GPU library.  It shares no code, header, table or
 * constant generator with the HIP implementation, and nothing in the product path
 * may call it.
 *
 * What the paper fixes (and this oracle follows): the 17-entry action table and
 * the 22 achievements with ids 0..21 (appendix "Action Space" / "Achievements"),
 * block ids 2..16 (appendix "Block Types"), creature health/damage (appendix
 * "Creatures": zombie 5/2, skeleton 3/2, cow 3), fixed-capacity masked creature
 * and plant tables (appendix "Differences between Craftax-Classic and Crafter"),
 * a 7x9 symbolic view and a flat length of 1345 (section "RL Environment
 * Interface", appendix "Observation Space"), +1 reward per first-time
 * achievement and +-0.1 per health point (section "RL Environment Interface"),
 * and auto-reset on done (appendix "Optimistic Environment Resets").
 *
 * The paper does not print the game rules themselves ("mimic Crafter").  Every
 * rule below that the paper is silent on is this build's own frozen reading; such
 * functions are marked "parity unpinned" beyond the invariants the tests check.
 */
#ifndef CRAFTAX_ORACLE_H
#define CRAFTAX_ORACLE_H

#include <stdint.h>
#include <stddef.h>

#ifdef __cplusplus
extern "C" {
#endif

#define ORC_MAP 64
#define ORC_NMOB 12   /* slots 0-2 zombie, 3-5 cow, 6-8 skeleton, 9-11 arrow */
#define ORC_NPLANT 10
#define ORC_VIEW_ROWS 7
#define ORC_VIEW_COLS 9
#define ORC_NBLOCK 17
#define ORC_NCHAN 21  /* 17 block channels + zombie, cow, skeleton, arrow */
#define ORC_NVEC 22

typedef struct {
    uint32_t max_episode_steps;
    uint32_t day_length;     /* even, 2..1024 */
    uint32_t cap_zombie, cap_cow, cap_skeleton, cap_arrow; /* each 0..3 */
    uint32_t cap_plant;      /* 0..10 */
    uint64_t atlas_seed;     /* pixel observations only */
    uint32_t worldgen;       /* ORC_WORLDGEN_VALUE (benchmark configurations) or ORC_WORLDGEN_PERLIN (the paper's noise) */
    uint32_t reset_mode;     /* ORC_RESET_EXACT or ORC_RESET_POOL (appendix "Optimistic Environment Resets") */
} orc_config;
enum { ORC_WORLDGEN_VALUE = 0, ORC_WORLDGEN_PERLIN = 1 };

typedef struct {
    uint8_t alive, x, y, dir;
    int8_t hp;
    uint8_t cd;
    uint8_t pad[2];
} orc_mob;

typedef struct {
    uint8_t alive, x, y, pad;
    uint16_t age;
} orc_plant;

/* One environment, canonical layout (4304 bytes, little endian, no hidden padding).
 * Dead mob / plant slots hold all-zero fields. */
typedef struct {
    uint8_t map[ORC_MAP * ORC_MAP];  /* row-major, index y*64+x, block ids */
    uint8_t px, py, dir, sleeping;   /* dir: 1 LEFT 2 RIGHT 3 UP 4 DOWN */
    uint8_t inv[12];  /* wood stone coal iron diamond sapling, wood/stone/iron pickaxe, wood/stone/iron sword */
    int8_t vit[4];    /* health food drink energy */
    int16_t cnt[4];   /* hunger thirst fatigue recover */
    uint32_t ach;     /* bit i = achievement id i */
    uint32_t t;       /* steps taken in this episode */
    uint32_t episode; /* resets since orc_reset */
    uint64_t seed;
    orc_mob mob[ORC_NMOB];
    orc_plant plant[ORC_NPLANT];
    uint32_t env;     /* environment index, part of every Philox counter */
} orc_env;

enum { ORC_OBS_SYM_U8_I8 = 0, ORC_OBS_SYM_U8_F32 = 1, ORC_OBS_SYM_F32 = 2, ORC_OBS_PIXELS_F32 = 3 };

size_t orc_env_bytes(void);
size_t orc_obs_bytes(int obs_mode);

/* Philox4x32-10 (Salmon et al., SC'11). */
void orc_philox4x32_10(const uint32_t ctr[4], const uint32_t key[2], uint32_t out[4]);
/* One inverse round and one forward round, exposed for the bijection test. */
void orc_philox_round(uint32_t c[4], const uint32_t k[2]);
void orc_philox_round_inv(uint32_t c[4], const uint32_t k[2]);
void orc_philox_batch(const uint32_t *ctrs, const uint32_t *keys, uint32_t *out, int n);

void orc_default_config(orc_config *cfg);
void orc_worldgen(uint8_t *map, uint64_t seed, uint32_t env, uint32_t episode);
void orc_worldgen_mode(uint8_t *map, uint64_t seed, uint32_t env, uint32_t episode, uint32_t mode);
uint32_t orc_perlin_noise(const uint16_t *lattice, int width, int spacing, int x, int y);
void orc_reset(orc_env *e, const orc_config *cfg, uint64_t seed, uint32_t env);
/* Rules only: no auto-reset.  Returns reward/done of the step just taken. */
void orc_step_rules(orc_env *e, const orc_config *cfg, int32_t action, float *reward, uint8_t *done);
/* Rules, then auto-reset to a fresh episode if done. */
void orc_step(orc_env *e, const orc_config *cfg, int32_t action, float *reward, uint8_t *done);
void orc_observe(const orc_env *e, const orc_config *cfg, int obs_mode, void *obs);

/* Batched helpers: loop the above over n environments, serially. */
void orc_reset_batch(orc_env *envs, const orc_config *cfg, const uint64_t *seeds,
                     const uint32_t *env_ids, int n);
/* Optimistic resets (appendix "Optimistic Environment Resets"): every step M = max(1, n / 16) new
 * worlds are generated, and the environments that finished take theirs from that pool, sampled
 * without replacement (with repeats only when more than M finish at once).  step_index: number
 * of batch steps taken since the reset; envs[0] must be environment 0 (its seed seeds the pool). */
#define ORC_RESET_EXACT 0u
#define ORC_RESET_POOL 1u
#define ORC_POOL_RATIO 16u
void orc_step_batch_pool(orc_env *envs, const orc_config *cfg, const int32_t *actions, int obs_mode,
                         void *obs, float *reward, uint8_t *done, int n, uint32_t step_index);
uint32_t orc_pool_slot(uint64_t pool_seed, uint32_t step_index, uint32_t rank, uint32_t n);
void orc_step_batch(orc_env *envs, const orc_config *cfg, const int32_t *actions, int obs_mode,
                    void *obs, float *reward, uint8_t *done, int n);
void orc_observe_batch(const orc_env *envs, const orc_config *cfg, int obs_mode, void *obs, int n);

/* UED level mutation (section "Craftax-1B: UED"): swaps two tiles of different type, one inside
 * the central 16x16 area; restricted != 0 keeps to stone <-> ores and grass <-> tree. */
int orc_mutate_swap(orc_env *e, uint64_t mutation_seed, uint32_t round, int restricted);

/* The noise mutation of the same section: the level is the vector of Perlin gradient angles.
 * theta: ORC_THETA_LEN offsets in 1024ths of a turn (in/out); amplitude <= 511. */
#define ORC_THETA_LEN 374
void orc_worldgen_theta(uint8_t *map, uint64_t seed, uint32_t env, uint32_t episode, const uint16_t *theta);
void orc_mutate_noise(orc_env *e, const orc_config *cfg, uint16_t *theta, uint64_t mutation_seed, uint32_t round, uint32_t amplitude);

/* Small accessors for tests. */
float orc_daylight(const orc_config *cfg, uint32_t t);
uint32_t orc_zombie_spawn_threshold(const orc_config *cfg, uint32_t t);
uint32_t orc_step_draw(const orc_env *e, uint32_t block, uint32_t word);
uint32_t orc_value_noise(const uint16_t *lattice, int width, int spacing, int x, int y);

#ifdef __cplusplus
}
#endif
#endif
