/*
 * CPU oracle for the full Craftax environment (9 floors, 43 actions, 67 achievements).
 * TEST INFRASTRUCTURE ONLY: plain single-threaded C, shares nothing with the GPU library.
 *
 * Fixed by the paper and followed here: the action table ids 0..42 (appendix "Action Space"),
 * the achievement table ids 0..66 with rewards 1/3/5/8 summing to 226 (appendix
 * "Achievements", section "Craftax-1B"), block ids 2..36 (appendix "Block Types"), the 19
 * creatures with health / damage / defence / collision type / floor (appendix "Creatures"),
 * 9 floors joined by ladders, an experience point per newly reached floor spendable on
 * dexterity / strength / intelligence, potions whose colour->effect map is re-drawn every
 * episode, enchanting with mana and a gemstone, a bow from a chest on the first dungeon floor,
 * spell books in dungeon chests, dark floors 2, 5, 7, 8 that need torches, a boss floor with
 * waves of every enemy (section "Craftax: An Extension of Crafter ..."), a 9x11 view with
 * per-cell one-hots for block (37), item (5), creature and a light level, dark cells masked,
 * and the inventory vector with its scalings, flat length 8268 (appendix "Observation Space").
 *
 * Everything else (floor generators, mob behaviour, costs, effects, caps) is this build's own
 * frozen reading: the paper does not print it.  Parity unpinned beyond the invariants and
 * hand-traced scenes of the tests.
 */
#ifndef CRAFTAX_FULL_ORACLE_H
#define CRAFTAX_FULL_ORACLE_H

#include <stdint.h>
#include <stddef.h>
#include "craftax_oracle.h"

#ifdef __cplusplus
extern "C" {
#endif

#define CF_FLOORS 9
#define CF_W 48
#define CF_CELLS (CF_W * CF_W)
#define CF_NSLOT 14      /* 0-2 melee, 3-4 ranged, 5-7 passive, 8-10 mob projectiles, 11-13 player projectiles */
#define CF_NPLANT 10
#define CF_NACH 67
#define CF_NACT 43
#define CF_VIEW_ROWS 9
#define CF_VIEW_COLS 11
#define CF_NCHAN 83      /* 37 block + 5 item + 40 creature (5 classes x 8 types) + 1 light */
#define CF_NVEC 51

typedef struct {
    uint32_t max_episode_steps;   /* paper: 100000 */
    uint32_t day_length;
    uint32_t cap_melee, cap_ranged, cap_passive;   /* 3, 2, 3 */
    uint32_t cap_plant;
    uint64_t atlas_seed;          /* seed of the synthetic tile atlas (pixel observations) */
    uint32_t worldgen;            /* ORC_WORLDGEN_VALUE or ORC_WORLDGEN_PERLIN: the noise behind the open floors */
    uint32_t reset_mode;          /* ORC_RESET_EXACT (cf_step_batch) or ORC_RESET_POOL (cf_step_batch_pool) */
} cf_config;

typedef struct {
    uint8_t alive, x, y, dir;
    int8_t hp;
    uint8_t cd;
    uint8_t type;   /* creature index (mobs, mob projectiles: the shooter's), or 0 arrow 1 fireball 2 iceball */
    uint8_t pad;
} cf_mob;

typedef struct {
    uint8_t block[CF_FLOORS][CF_CELLS];
    uint8_t item[CF_FLOORS][CF_CELLS];    /* 0 none 1 torch 2 ladder down 3 ladder up 4 ladder down (blocked) */
    uint8_t light[CF_FLOORS][CF_CELLS];   /* 0..20 */
    uint8_t px, py, dir, floor;
    uint8_t sleeping, resting, learned_fireball, learned_iceball;
    uint8_t inv[10];        /* wood stone coal iron diamond sapphire ruby sapling torch arrow */
    uint8_t potion[6];      /* red green blue pink cyan yellow */
    uint8_t book, pickaxe, sword, sword_ench, bow, bow_ench;   /* levels 0..4; enchant 0 none 1 fire 2 ice */
    uint8_t armour[4], armour_ench[4];
    int8_t vit[5];          /* health food drink energy mana */
    uint8_t xp, dex, str, intel;
    int16_t cnt[5];         /* hunger thirst fatigue recover mana */
    uint8_t potion_effect[6];
    uint8_t kills[CF_FLOORS];
    uint8_t boss_hits, boss_vulnerable;
    uint16_t visited;
    uint8_t ladder_up[CF_FLOORS][2], ladder_down[CF_FLOORS][2];   /* x, y */
    uint32_t ach[3];
    uint32_t t, episode, env;
    uint32_t pad0;
    uint64_t seed;
    cf_mob mob[CF_FLOORS][CF_NSLOT];
    orc_plant plant[CF_NPLANT];
    uint8_t pad1[4];
} cf_env;

enum { CF_OBS_U8_F32 = 0, CF_OBS_F32 = 1, CF_OBS_PIXELS_F32 = 2 };
#define CF_PIX_ROWS 130   /* 9 view rows + 4 inventory rows of 10-pixel tiles */
#define CF_PIX_COLS 110   /* 11 tile columns */

size_t cf_env_bytes(void);
size_t cf_obs_bytes(int mode);
void cf_default_config(cf_config *cfg);
int cf_achievement_reward(int id);
void cf_step_batch_pool(cf_env *envs, const cf_config *cfg, const int32_t *actions, int mode, void *obs, float *reward, uint8_t *done,
                        int n, uint32_t step_index);   /* optimistic resets; step_index = steps since the reset */
void cf_worldgen_floor(cf_env *e, int floor);    /* uses e->seed, e->env, e->episode */
void cf_worldgen_floor_mode(cf_env *e, int floor, uint32_t mode);   /* mode: ORC_WORLDGEN_VALUE or ORC_WORLDGEN_PERLIN */
/* A level as the noise mutation sees it: the angle offsets of every noise lattice, overworld
 * (2 x 4x4 + 4 x 7x7 points) then cave floors 2, 5, 6, 7 (2 x 7x7 each). */
#define CF_THETA_OVERWORLD (2 * 16 + 4 * 49)
#define CF_THETA_CAVE (2 * 49)
#define CF_THETA_LEN (CF_THETA_OVERWORLD + 4 * CF_THETA_CAVE)
void cf_worldgen_floor_theta(cf_env *e, int floor, const uint16_t *theta);   /* Perlin floor of level theta[CF_THETA_LEN] */
void cf_mutate_noise(cf_env *e, const cf_config *cfg, uint16_t *theta, uint64_t mutation_seed, uint32_t round, uint32_t amplitude);
void cf_reset(cf_env *e, const cf_config *cfg, uint64_t seed, uint32_t env);
void cf_step_rules(cf_env *e, const cf_config *cfg, int32_t action, float *reward, uint8_t *done);
void cf_step(cf_env *e, const cf_config *cfg, int32_t action, float *reward, uint8_t *done);
void cf_observe(const cf_env *e, const cf_config *cfg, int mode, void *obs);
void cf_reset_batch(cf_env *envs, const cf_config *cfg, const uint64_t *seeds, const uint32_t *env_ids, int n);
void cf_step_batch(cf_env *envs, const cf_config *cfg, const int32_t *actions, int mode, void *obs,
                   float *reward, uint8_t *done, int n);
void cf_observe_batch(const cf_env *envs, const cf_config *cfg, int mode, void *obs, int n);
uint32_t cf_step_draw(const cf_env *e, uint32_t block, uint32_t word);
/* UED level mutation of the overworld (section "Craftax-1B: UED"), see orc_mutate_swap. */
int cf_mutate_swap(cf_env *e, uint64_t mutation_seed, uint32_t round, int restricted);
/* creature table accessors for tests: field 0 health, 1..3 damage phys/fire/ice, 4..6 defence %, 7 collision */
int cf_creature(int index, int field);

#ifdef __cplusplus
}
#endif
#endif
