/*
 * craftax.h - C ABI of the MI355X (gfx950) batched Craftax-Classic and Craftax simulator.
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
 *  - No call allocates device memory.  craftax_state_init makes one temporary host staging
 *    buffer; craftax_state_init and craftax_state_attach synchronise with the stream they are
 *    given.  No environment variable is read.
 */
#ifndef CRAFTAX_H
#define CRAFTAX_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define CRAFTAX_ABI_VERSION 2u

enum {
    CRAFTAX_OK = 0,
    CRAFTAX_E_NULL = -1,       /* a required pointer is NULL */
    CRAFTAX_E_ALIGN = -2,      /* state not 256-byte aligned or obs not 16-byte aligned */
    CRAFTAX_E_COUNT = -3,      /* n <= 0, n differs from the state's n, or a range is outside it */
    CRAFTAX_E_STATE = -4,      /* state is not registered in this process (craftax_state_init or craftax_state_attach),
                                  or holds no worlds yet (no craftax_reset since craftax_state_init) */
    CRAFTAX_E_HIP = -5,        /* a HIP call failed */
    CRAFTAX_E_CONFIG = -6      /* unsupported configuration value */
};

/* Variants (section "Craftax: An Extension of Crafter ..."): Classic = the Crafter rules on a
 * 64x64 map; CRAFTAX = the full game with nine 48x48 floors, 43 actions, 67 achievements. */
enum { CRAFTAX_VARIANT_CLASSIC = 0, CRAFTAX_VARIANT_CRAFTAX = 1 };

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
 * counts sqrt(n)/10, vitals x/10, flags 0/1.  Unused bytes of the stride are zero.
 *
 * Variant CRAFTAX supports three of the layouts (appendix "Observation Space": 9x11 cells, per
 * cell 37-way block, 5-way item and 40-way creature one-hots plus a light level, cells darker
 * than 0.05 blank; then 51 scalars; 99*83 + 51 = 8268):
 *  SYM_U8_F32 : bytes [0,8217) 9x11 cells x 83 channels, row-major (row, col, channel), channel
 *               82 = light level 0..20; float[51] scalars at byte 8224; stride 8448 (66 lines).
 *  SYM_F32    : float[8268] = the cell bytes as floats (light as level/20) followed by the 51
 *               scalars (the flat layout of the paper); stride 33152.
 *  PIXELS_F32 : float[130][110][3] RGB in [0,1) (section "RL Environment Interface": 110 x 130 x 3;
 *               10-pixel tiles): tile rows 0..8 are the 9x11 view, tile rows 9..12 hold inventory
 *               slot j = 0..43 at row 9 + j/11, column j%11.  Tiles come from an atlas seeded by
 *               cfg->atlas_seed (the paper's textures are not part of this library): a view cell
 *               shows its block tile, overlaid by its item, creature and the player where their
 *               one-bit masks are set, times light level / 20; cells beyond the map edge show
 *               block 1 at full light; slot j shows icon j times min(scalar j, 1).  Stride 171648
 *               (171600 bytes of pixels, zero padding).  craftax_step draws the picture in a
 *               second kernel on the same stream.
 * Channels: 0..36 block id; 37..41 item (none, torch, ladder down, ladder up, blocked ladder
 * down); 42..81 creature = 42 + 8*class + type slot, classes melee, passive, ranged, mob
 * projectile, player projectile; melee and ranged type slot = the floor the creature lives on
 * (appendix "Creatures"), passive cow/snail/bat = 0/1/2, mob projectile plain/fire/ice/both =
 * 0/1/2/3, player projectile arrow/fireball/iceball = 0/1/2.
 * The 51 scalars follow the inventory table of that appendix: wood, stone, coal, iron, diamond,
 * sapphire, ruby, sapling, torch, arrow, 6 potions (sqrt(n)/10); book n/2; pickaxe, sword
 * level/4; sword enchantment; bow; bow enchantment; 4 armour level/2; 4 armour enchantments;
 * health, food, drink, energy, mana, experience, dexterity, strength, intelligence (x/10);
 * facing one-hot; daylight; sleeping; resting; learned fireball; learned iceball; floor/10;
 * floor cleared; boss vulnerable. */
enum {
    CRAFTAX_OBS_SYM_U8_I8 = 0,
    CRAFTAX_OBS_SYM_U8_F32 = 1,
    CRAFTAX_OBS_SYM_F32 = 2,
    CRAFTAX_OBS_PIXELS_F32 = 3
};

typedef struct craftax_config {
    uint32_t abi_version;        /* CRAFTAX_ABI_VERSION */
    uint32_t variant;            /* CRAFTAX_VARIANT_* */
    uint32_t obs_mode;           /* CRAFTAX_OBS_* */
    uint32_t max_episode_steps;  /* episode is cut (done = 1) when this many steps were taken */
    uint32_t day_length;         /* even, 2..1024 */
    uint32_t cap_zombie, cap_cow, cap_skeleton, cap_arrow;  /* 0..3 each (appendix "Differences
                                    between Craftax-Classic and Crafter": fixed, masked slots).
                                    Variant CRAFTAX reads them as the per-floor caps of melee
                                    (cap_zombie, 0..3), passive (cap_cow, 0..3) and ranged
                                    (cap_skeleton, 0..2) creatures; projectiles are always 3+3 */
    uint32_t cap_plant;          /* 0..10 */
    uint64_t atlas_seed;         /* seed of the synthetic tile atlas (pixel observations) */
    uint32_t worldgen;           /* CRAFTAX_WORLDGEN_*: the noise behind the terrain rules */
    uint32_t reset_mode;         /* CRAFTAX_RESET_*: where the world of a new episode comes from */
    uint32_t group_lanes;        /* tuning: lanes of a wavefront that share one environment in the step kernel; 0 = chosen
                                    from n (the default), else 4, 8 or 16 (Classic), 16 or 64 (CRAFTAX).  Results do not
                                    depend on it. */
    uint32_t reserved;           /* must be 0 */
} craftax_config;

/* The noise of world generation.  VALUE: seeded integer value noise (the benchmark
 * configurations).  PERLIN: Perlin gradient noise as in the paper (appendix "World Generation":
 * unit gradients at random lattice angles, corner dot products blended with 6t^5 - 15t^4 + 10t^3),
 * evaluated in integers: 1024 directions, gradients in Q14, fade weights in Q16, every division a
 * floor.  Both feed the same field mix and thresholds.  In variant CRAFTAX the choice applies to the
 * floors drawn from noise fields (the overworld and the four cave floors); the room floors and the
 * boss floor use no noise and are the same in both. */
enum { CRAFTAX_WORLDGEN_VALUE = 0, CRAFTAX_WORLDGEN_PERLIN = 1 };

/* Where the world of a new episode comes from.  EXACT (default): every environment gets a world
 * of its own, a function of (its seed, its number, its episode index), generated one episode
 * ahead.  POOL: the paper's optimistic resets (appendix "Optimistic Environment Resets"), kept as
 * an option for comparison: batch step T (counted from craftax_reset) offers a pool of
 * M = max(1, n / 16) new worlds, world j being the generator run for (seed of environment 0,
 * environment number 2^31 + j, episode T); the environments that finish in that step are taken
 * in increasing number and the r-th of them gets world (shift_T + r) mod M, shift_T being one
 * uniform draw per step: no world twice unless more than M finish at once.  An environment keeps
 * its own seed and counts its episode up, so everything random after the reset still differs
 * between environments that share a world.  The library generates only the pool worlds that are
 * taken.  In variant CRAFTAX a world is all nine floors with their ladders and the potion map.
 * craftax_rollout is not available in this mode. */
enum { CRAFTAX_RESET_EXACT = 0, CRAFTAX_RESET_POOL = 1 };

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

/* One full-Craftax environment in canonical form (63432 bytes, little endian).  Maps are
 * [floor][y][x].  Mob slots per floor: 0-2 melee, 3-4 ranged, 5-7 passive, 8-10 mob
 * projectiles, 11-13 player projectiles; `type` is the creature's row in appendix "Creatures"
 * (0 zombie, 1 skeleton, 2 cow, 3 orc soldier, 4 orc mage, 5 snail, 6 gnome warrior, 7 gnome
 * archer, 8 bat, 9 lizard, 10 kobold, 11 knight, 12 archer, 13 troll, 14 deep thing, 15 pig man,
 * 16 fire elemental, 17 frost troll, 18 ice elemental), for a mob projectile its shooter's, for
 * a player projectile 0 arrow, 1 fireball, 2 iceball.  Dead slots are all zero. */
typedef struct craftax_full_mob { uint8_t alive, x, y, dir; int8_t hp; uint8_t cd, type, pad; } craftax_full_mob;
typedef struct craftax_full_env_dump {
    uint8_t block[9][48 * 48];  /* appendix "Block Types" */
    uint8_t item[9][48 * 48];   /* 0 none, 1 torch, 2 ladder down, 3 ladder up, 4 ladder down (blocked) */
    uint8_t light[9][48 * 48];  /* 0..20 */
    uint8_t px, py, dir, floor;
    uint8_t sleeping, resting, learned_fireball, learned_iceball;
    uint8_t inv[10];            /* wood stone coal iron diamond sapphire ruby sapling torch arrow */
    uint8_t potion[6];          /* red green blue pink cyan yellow */
    uint8_t book, pickaxe, sword, sword_ench, bow, bow_ench;   /* levels 0..4; enchantment 0 none, 1 fire, 2 ice */
    uint8_t armour[4], armour_ench[4];
    int8_t vit[5];              /* health food drink energy mana */
    uint8_t xp, dex, str, intel;
    uint8_t pad_a;
    int16_t cnt[5];             /* hunger thirst fatigue recover mana */
    uint8_t potion_effect[6];   /* colour -> effect of this episode: 0/1 health +/-, 2/3 mana, 4/5 energy */
    uint8_t kills[9];
    uint8_t boss_hits, boss_vulnerable;
    uint8_t pad_b;
    uint16_t visited;           /* bit f = floor f was entered */
    uint8_t ladder_up[9][2], ladder_down[9][2];   /* x, y per floor */
    uint8_t pad_c[2];
    uint32_t ach[3];            /* bit i of word i/32 = achievement id i (appendix "Achievements") */
    uint32_t t, episode, env;
    uint32_t pad0;
    uint64_t seed;
    craftax_full_mob mob[9][14];
    craftax_plant plant[10];
    uint8_t pad1[4];
} craftax_full_env_dump;

/* Fills *cfg (HOST) with the defaults: Classic, SYM_U8_F32, 10000 steps, day 300, caps 3/3/3/3/10. */
void craftax_default_config(craftax_config *cfg);
/* Defaults of a variant: CLASSIC as above; CRAFTAX: SYM_U8_F32, 100000 steps (appendix
 * "Further Environment Details"), day 300, caps melee 3 / passive 3 / ranged 2, 10 plants. */
void craftax_default_config_for(craftax_config *cfg, uint32_t variant);

/* Bytes of device memory the caller must provide for n environments (0 on a bad config).  The
 * paper's interface (section "RL Environment Interface") exposes the whole environment state as
 * one object; here that object is one caller-owned blob of this size for all n environments:
 * header, tables, per-environment records and maps (two map slots each: appendix "Optimistic
 * Environment Resets" is why the next world is kept ready), and the reset bookkeeping. */
size_t craftax_state_bytes(const craftax_config *cfg, int n);
/* Per-environment observation stride in bytes for cfg->obs_mode (multiple of 16): the symbolic
 * and pixel observations of section "RL Environment Interface" / appendix "Observation Space" in
 * the layouts listed above.  0 on a bad config. */
size_t craftax_obs_bytes(const craftax_config *cfg);
/* sizeof(craftax_env_dump). */
size_t craftax_env_dump_bytes(void);
/* Size of one canonical dump for cfg->variant: craftax_env_dump or craftax_full_env_dump. */
size_t craftax_env_dump_bytes_for(const craftax_config *cfg);

/* Prepares the state object of section "RL Environment Interface" for n environments: writes the
 * header, the lookup tables (day/night curve of appendix "Observation Space", scalings of its
 * inventory table, Perlin gradients of appendix "World Generation") and the tile atlas into
 * `state` (DEVICE, 256-byte aligned, craftax_state_bytes() long) and registers the address with
 * the library.  Environments hold no world until craftax_reset: until then step, rollout, observe,
 * export, import and the mutations return CRAFTAX_E_STATE.  cfg is HOST.  Errors: CRAFTAX_E_NULL,
 * CRAFTAX_E_ALIGN, CRAFTAX_E_COUNT (n <= 0), CRAFTAX_E_CONFIG (bad field, or a kernel this
 * configuration would launch needs more LDS or threads per block than the device allows),
 * CRAFTAX_E_HIP. */
int craftax_state_init(void *state, const craftax_config *cfg, int n, void *stream);
/* Checkpoint / resume (the paper's state is one object that can be stored and restored, section
 * "RL Environment Interface").  A state blob is position independent: a byte copy of it, taken
 * while no call on it is in flight (device to device, or through the host or a file and back),
 * continues bit for bit where the original stood once it is attached at its new address.  attach
 * reads the blob's header (DEVICE to HOST, synchronising with `stream`), checks that it was
 * written by this library version for exactly this cfg and n (CRAFTAX_E_STATE if it is no state
 * blob, CRAFTAX_E_CONFIG / CRAFTAX_E_COUNT on a mismatch) and registers the address; nothing in
 * the blob is changed.  The blob must come from a state that had been reset. */
int craftax_state_attach(void *state, const craftax_config *cfg, int n, void *stream);
/* Forgets a state registered by craftax_state_init or craftax_state_attach (the memory stays
 * the caller's). */
int craftax_state_release(void *state);

/* Starts episode 0 of every environment: env i gets seeds[i] (DEVICE, n x uint64) as its
 * Philox key for all later episodes, a generated 64x64 world, full vitals, empty tables. */
int craftax_reset(void *state, const uint64_t *seeds, int n, void *stream);

/* One step of every environment.  actions: DEVICE int32[n]; ids outside the variant's action
 * table (0..16 Classic, 0..42 Craftax: appendix "Action Space") act as NOOP.
 * Outputs (all DEVICE): obs (n x craftax_obs_bytes(), 16-byte aligned), reward float[n],
 * done uint8[n].  When done[i] = 1 the reward belongs to the episode that just ended and
 * state and obs already hold the first state of the next episode.  obs may be NULL to skip
 * rendering. */
int craftax_step(void *state, const int32_t *actions, void *obs, float *reward, uint8_t *done,
                 int n, void *stream);

/* Several steps in one launch, for callers that hold the actions of all of them (a random or
 * scripted policy; the paper's appendix "Optimistic Environment Resets" measures such rollouts):
 * exactly the result of `steps` calls of craftax_step with actions[t] (DEVICE int32[steps][n]),
 * with reward and done of every step (DEVICE float[steps][n], uint8[steps][n]) and the observation
 * written after every step into the same buffer obs (DEVICE, n strides; it ends up holding the
 * observation after the last step; NULL skips rendering).  A thread block keeps its environments
 * on chip for the whole launch and blocks advance independently.  Both variants, symbolic
 * observations and exact resets only (CRAFTAX_E_CONFIG for a pixel mode or reset_mode POOL).
 * Other errors as for craftax_step;
 * CRAFTAX_E_COUNT also for steps <= 0. */
int craftax_rollout(void *state, const int32_t *actions, int steps, void *obs, float *reward,
                    uint8_t *done, int n, void *stream);

/* Renders the current observation of every environment, as the paper's reset returns it (section
 * "RL Environment Interface": symbolic 1345 / 8268 values or 63x63x3 / 110x130x3 pixels, appendix
 * "Observation Space") in the layout of cfg->obs_mode; obs: DEVICE, n x craftax_obs_bytes(),
 * 16-byte aligned.  Used after craftax_reset, an import or a mutation; craftax_step writes the
 * observation itself. */
int craftax_observe(void *state, void *obs, int n, void *stream);

/* Copies environments [first, first+count) to / from canonical dumps in DEVICE memory
 * (count x craftax_env_dump, or craftax_full_env_dump for variant CRAFTAX; 16-byte aligned).
 * Section "RL Environment Interface" exposes the whole environment state as one object so that
 * levels can be inspected and edited (section "Craftax-1B: UED" relies on it); export is the
 * readable form of that object, import the state-editing hook.
 * Import packs the dump into the library's bit fields and accepts exactly the values the rules can
 * reach; anything else is brought into range silently: block ids outside the variant's table
 * (1..16 Classic, 1..36 Craftax) become 1 (out of bounds: solid, never rendered from a tile that
 * does not exist), items above 4 become 0, light is capped at 20; Classic: coordinates are taken
 * modulo 64, counts and vitals modulo 16, the four counters are clamped to -128..127, mob hp and
 * cooldown modulo 16, direction modulo 8; Craftax: see craftax_full_env_dump (coordinates clamped
 * to the 48x48 floor, levels to their maxima).  A dump that holds such values does not come back
 * unchanged from export. */
int craftax_export_envs(const void *state, int first, int count, void *dumps, void *stream);
int craftax_import_envs(void *state, int first, int count, const void *dumps, void *stream);

/* Level mutation for unsupervised environment design (section "Craftax-1B: UED", the "swap" and
 * "restricted swap" operators): in each environment of [first, first+count) two tiles of
 * different type trade places on the current map (variant CRAFTAX: on the overworld, floor 0), one
 * of them inside the central 16x16 area; restricted != 0 only lets stone trade with ores (coal,
 * iron, diamond; sapphire and ruby too in CRAFTAX) and grass with trees.  The paper says no more;
 * this library's reading: up to 32 tries per call, try k drawing Philox block (env, round, 0,
 * MUTATE << 16 | k) keyed by mutation_seed, word 0 -> the central cell ((u * 256) >> 32, row-major
 * in the area), word 1 -> any cell ((u * cells) >> 32, row-major); a try is refused if the two
 * blocks are equal, if a cell holds the player, a live mob, a plant or (CRAFTAX) an item, or,
 * restricted, if the blocks are not of one group; the first try not refused is carried out.
 * tries: DEVICE int32[count] or NULL; receives that try's number + 1, or 0 if all were refused.
 * Nothing but the map changes.  Errors: CRAFTAX_E_COUNT for a range outside the state. */
int craftax_mutate_swap(void *state, int first, int count, uint64_t mutation_seed, uint32_t round,
                        int restricted, int32_t *tries, void *stream);

/* The third operator of the same section, "noise": a level is the vector of angles of the Perlin
 * gradients its world is generated from, and the mutation adds a uniform random number to every
 * element.  theta: DEVICE uint16[count][CRAFTAX_THETA_LEN], in and out, caller-owned (a level
 * buffer keeps one row per level): element i is the offset, in 1024ths of a turn (0..1023), added
 * to the angle of lattice number i of the world generation (the two spacing-16 lattices, then the
 * four spacing-8 ones, each row by row); all zero = the level the seed alone gives.  The call adds
 * to every element an integer uniform in [-amplitude, amplitude] (this library's reading of
 * "uniform random number": ((d * (2 * amplitude + 1)) >> 16) - amplitude with d = u16 number i
 * of Philox stream (env, round, 1, MUTATE << 16 | block) keyed by mutation_seed), modulo a full
 * turn, generates the world of the current episode of each environment of [first, first+count)
 * again from the new angles, and restarts that episode in it (fresh player, empty tables, same
 * episode number; the per-cell draws for trees and ores stay those of the seed).  amplitude 0
 * loads the level theta unchanged.  Variant CRAFTAX: a row has CRAFTAX_FULL_THETA_LEN elements,
 * the lattices of every floor generated from noise: the overworld's two spacing-16 lattices (4x4
 * points) and four spacing-8 ones (7x7), then the two 7x7 lattices of each of the cave floors 2,
 * 5, 6 and 7; the draws count i over the whole row; all nine floors of the current episode are
 * generated again (the room floors and the boss floor come out as they were).  Needs
 * CRAFTAX_WORLDGEN_PERLIN (CRAFTAX_E_CONFIG otherwise); CRAFTAX_E_COUNT for a range outside the
 * state or amplitude > 511; CRAFTAX_E_NULL for theta == NULL. */
#define CRAFTAX_THETA_LEN 374
#define CRAFTAX_FULL_THETA_LEN 620
int craftax_mutate_noise(void *state, int first, int count, uint16_t *theta, uint64_t mutation_seed,
                         uint32_t round, uint32_t amplitude, void *stream);

/* Fills actions (DEVICE int32[steps][n]) with the synthetic action stream used by the
 * benchmark: kind 0 = uniform over 17 actions, kind 1 = half of the draws restricted to
 * ids 1..5, kinds 2 and 3 = the same two over the 43 actions of full Craftax.  Input generation
 * only; not part of the simulator. */
int craftax_synth_actions(int32_t *actions, int n, int step0, int steps, uint64_t action_seed,
                          int kind, void *stream);

/* Per-run metrics (the paper reports achievement success rates and reward as a share of the
 * maximum, section "Craftax-1B"; its appendix "Optimistic Environment Resets" argues from the mean
 * episode length): sums over the n environments.
 *   episodes        episodes finished since craftax_reset
 *   steps           steps taken so far in the episodes now running (sum of t)
 *   achievements[i] environments whose running episode has unlocked achievement i (appendix
 *                   "Achievements": 22 ids for Classic, 67 for Craftax; the rest stay 0)
 *   unlocks[i]      how often achievement i has been unlocked since craftax_reset, counted by the
 *                   step kernels as it happens (an achievement unlocks at most once per episode)
 * Success rate of achievement i over the finished episodes = (unlocks[i] - achievements[i]) /
 * episodes; over a window of steps, the same with the differences of two snapshots.  Mean episode
 * length over a window = n * window / (episodes after - episodes before).  The counters belong to
 * the run, not to the environments: craftax_reset clears them, craftax_import_envs and the
 * mutations leave them alone (an episode restarted by craftax_mutate_noise can unlock again), and
 * they travel with a copy of the state blob.
 * out: DEVICE, one craftax_metrics, 8-byte aligned.  workspace: DEVICE scratch of at least
 * craftax_stats_workspace_bytes(n) bytes, 16-byte aligned, contents irrelevant before and after
 * (each 256 environments leave one partial result there, a second kernel adds them up, so the
 * result does not depend on any order of execution).  Errors: CRAFTAX_E_NULL, CRAFTAX_E_ALIGN,
 * CRAFTAX_E_COUNT (n differs from the state's, or the workspace is too small), CRAFTAX_E_STATE. */
#define CRAFTAX_STATS_ACHIEVEMENTS 96
typedef struct craftax_metrics {
    uint64_t episodes;
    uint64_t steps;
    uint32_t achievements[CRAFTAX_STATS_ACHIEVEMENTS];
    uint32_t n;
    uint32_t pad;
    uint64_t unlocks[CRAFTAX_STATS_ACHIEVEMENTS];
} craftax_metrics;
size_t craftax_stats_workspace_bytes(int n);
int craftax_stats(const void *state, craftax_metrics *out, void *workspace, size_t workspace_bytes, int n, void *stream);

/* craftax_stats for callers that cannot allocate device memory or hand over a workspace: code
 * under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  The partial
 * results go to a buffer inside the library's own device image (2 MiB per GPU, held until the
 * process ends) instead of a workspace; nothing is allocated, by this call or behind it.  Same
 * result as craftax_stats.  Limits: n <= CRAFTAX_STATS_STATIC_MAX_ENVS (CRAFTAX_E_COUNT beyond).
 * All calls on one GPU share that buffer: calls that overlap in time on one GPU (different
 * streams, different states) race and give wrong sums; calls on one stream, or ordered by events,
 * are safe.  The GPU that is current at the call must be the one that holds `state`. */
#define CRAFTAX_STATS_STATIC_MAX_ENVS 524288
int craftax_stats_static(const void *state, craftax_metrics *out, int n, void *stream);

/* Debug build with bounds checks (a build of the same sources with -DCRAFTAX_DEBUG_BOUNDS, shipped
 * as libcraftax_hip_debug.so): every index the kernels form into a map, an LDS window or a staging
 * area is checked on the device; an index outside its range is counted (and replaced by 0, so that
 * nothing faults) instead of being used.  craftax_debug_bounds waits for the device, copies the
 * record to report (HOST: violations so far, then source line, index and limit of the first one),
 * clears it, and returns 1; in the release library it returns 0 and zeroes report.
 * craftax_debug_bounds_selftest runs a kernel that forms one out-of-range index on purpose (it is
 * caught and replaced, nothing faults) and returns 1 if the record then shows exactly that
 * violation, 0 in the release library, a negative CRAFTAX_E_* code on a HIP error. */
int craftax_debug_bounds(uint32_t report[4]);
int craftax_debug_bounds_selftest(void);

const char *craftax_last_error(void);

#ifdef __cplusplus
}
#endif
#endif
