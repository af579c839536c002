/*
 * CPU oracle: Craftax-Classic rules, world generation and observation rendering.
 * TEST INFRASTRUCTURE ONLY (see craftax_oracle.h).  Plain scalar C, one environment
 * at a time, no blocking, no fusion, no tables shared with the GPU library.
 *
 * Citations name the paper's sections/tables.  "reading:" marks a rule the paper
 * does not print and that this build froze itself (parity unpinned beyond the
 * invariants in the tests).
 */
#include "craftax_oracle.h"
#include <string.h>
#include <math.h>

/* ---- ids fixed by the paper --------------------------------------------------------- */
/* appendix "Block Types": ids 2..16.  reading: id 0 = invalid (never on a map),
 * id 1 = out of bounds (what the view shows past the map edge); 17 one-hot channels. */
enum { B_INVALID = 0, B_OOB = 1, B_GRASS = 2, B_WATER = 3, B_STONE = 4, B_TREE = 5, B_WOOD = 6,
       B_PATH = 7, B_COAL = 8, B_IRON = 9, B_DIAMOND = 10, B_TABLE = 11, B_FURNACE = 12,
       B_SAND = 13, B_LAVA = 14, B_PLANT = 15, B_RIPE = 16 };
/* appendix "Action Space", ids 0..16 */
enum { A_NOOP = 0, A_LEFT, A_RIGHT, A_UP, A_DOWN, A_DO, A_SLEEP, A_PLACE_STONE, A_PLACE_TABLE,
       A_PLACE_FURNACE, A_PLACE_PLANT, A_MAKE_WOOD_PICKAXE, A_MAKE_STONE_PICKAXE,
       A_MAKE_IRON_PICKAXE, A_MAKE_WOOD_SWORD, A_MAKE_STONE_SWORD, A_MAKE_IRON_SWORD, A_COUNT };
/* appendix "Achievements", ids 0..21 */
enum { ACH_COLLECT_WOOD = 0, ACH_PLACE_TABLE, ACH_EAT_COW, ACH_COLLECT_SAPLING, ACH_COLLECT_DRINK,
       ACH_MAKE_WOOD_PICKAXE, ACH_MAKE_WOOD_SWORD, ACH_PLACE_PLANT, ACH_DEFEAT_ZOMBIE,
       ACH_COLLECT_STONE, ACH_PLACE_STONE, ACH_EAT_PLANT, ACH_DEFEAT_SKELETON,
       ACH_MAKE_STONE_PICKAXE, ACH_MAKE_STONE_SWORD, ACH_WAKE_UP, ACH_PLACE_FURNACE,
       ACH_COLLECT_COAL, ACH_COLLECT_IRON, ACH_COLLECT_DIAMOND, ACH_MAKE_IRON_PICKAXE,
       ACH_MAKE_IRON_SWORD };

enum { I_WOOD = 0, I_STONE, I_COAL, I_IRON, I_DIAMOND, I_SAPLING, I_WOOD_PICKAXE, I_STONE_PICKAXE,
       I_IRON_PICKAXE, I_WOOD_SWORD, I_STONE_SWORD, I_IRON_SWORD };
enum { V_HEALTH = 0, V_FOOD, V_DRINK, V_ENERGY };
enum { C_HUNGER = 0, C_THIRST, C_FATIGUE, C_RECOVER };
enum { T_ZOMBIE = 0, T_COW = 1, T_SKELETON = 2, T_ARROW = 3 };
enum { DIR_NONE = 0, DIR_LEFT = 1, DIR_RIGHT = 2, DIR_UP = 3, DIR_DOWN = 4 };

/* ---- constants of this build's reading --------------------------------------------- */
#define MAX_COUNT 9              /* inventory counts and vitals saturate at 9 */
#define HP_ZOMBIE 5              /* appendix "Creatures" */
#define HP_COW 3
#define HP_SKELETON 3
#define DMG_ZOMBIE 2
#define DMG_ZOMBIE_SLEEP 7       /* reading */
#define DMG_ARROW 2
#define CD_ZOMBIE 5              /* reading: steps between zombie hits */
#define CD_SKELETON 4            /* reading: steps between shots */
#define CHASE_RANGE 8            /* reading: zombie chases when Chebyshev distance < 8 */
#define SHOOT_RANGE 4            /* reading */
#define DESPAWN_DIST 15          /* reading: Chebyshev distance beyond which a mob vanishes */
#define SPAWN_MIN_DIST 5         /* reading */
#define RIPE_AGE 300             /* reading */
#define FOOD_COW 6
#define FOOD_PLANT 4

#define P_SAPLING 429496730u     /* 10 %  of 2^32 */
#define P_CHASE 52429u           /* 80 %  of 2^16 */
#define P_SHOOT 32768u           /* 50 %  of 2^16 */
#define P_PLANT_EATEN 32u        /* 1/8   of 2^8 */
#define P_COW_SPAWN 128u         /* 1/32  of 2^12 */
#define P_SKELETON_SPAWN 410u    /* 10 %  of 2^12 */

/* Philox counter layout (reading): key = 64-bit seed (low word, high word);
 * counter = (env, a, b, domain<<16 | block).  STEP: a = t, b = episode.
 * WORLDGEN: a = stream, b = episode.  ATLAS: a = stream, b = 0, env = 0. */
enum { DOM_STEP = 0, DOM_WORLDGEN = 1, DOM_ACTIONS = 2, DOM_ATLAS = 3, DOM_MUTATE = 4 };

static uint32_t philox_word(uint64_t seed, uint32_t c0, uint32_t c1, uint32_t c2, uint32_t dom,
                            uint32_t block, uint32_t word)
{
    uint32_t ctr[4] = { c0, c1, c2, (dom << 16) | block };
    uint32_t key[2] = { (uint32_t)seed, (uint32_t)(seed >> 32) };
    uint32_t out[4];
    orc_philox4x32_10(ctr, key, out);
    return out[word];
}

/* Static draw slots of one step (reading): four Philox blocks b = 0..3 of four words each.
 *   block b, word s (s = 0..2): the draws of mob slot k = b + 4 s and of plant slot k (k < 10):
 *       bits 0..15   decision draw, compared with 16-bit thresholds
 *       bits 16..18  movement choice: 0..3 a direction, 4..7 stay
 *       bits 19..26  "eaten" draw of the plant, compared with an 8-bit threshold
 *   block b, word 3: misc[b].  misc[j], j = 0..2, is the spawn attempt of type j (zombie, cow,
 *       skeleton): bits 0..9 and 10..19 pick the x and y offsets as ((v * 31) >> 10) - 15, bits
 *       20..31 are the probability draw (12 bits); misc[3] is the sapling draw of DO on grass
 *       (all 32 bits).
 * A draw is the same number whether or not control flow uses it, so an action whose
 * prerequisites fail equals NOOP exactly. */
uint32_t orc_step_draw(const orc_env *e, uint32_t block, uint32_t word)
{
    return philox_word(e->seed, e->env, e->t, e->episode, DOM_STEP, block, word);
}
static uint32_t slot_draw(const orc_env *e, int k) { return orc_step_draw(e, (uint32_t)(k & 3), (uint32_t)(k >> 2)); }
static uint32_t misc_draw(const orc_env *e, int j) { return orc_step_draw(e, (uint32_t)j, 3); }

static uint32_t choice(uint32_t u, uint32_t n) { return (uint32_t)(((uint64_t)u * n) >> 32); }

static int iabs(int v) { return v < 0 ? -v : v; }
static int imax(int a, int b) { return a > b ? a : b; }
static int imin(int a, int b) { return a < b ? a : b; }
static int inb(int x, int y) { return x >= 0 && x < ORC_MAP && y >= 0 && y < ORC_MAP; }
static void dir_delta(int dir, int *dx, int *dy)
{
    *dx = 0; *dy = 0;
    if (dir == DIR_LEFT) *dx = -1;
    if (dir == DIR_RIGHT) *dx = 1;
    if (dir == DIR_UP) *dy = -1;
    if (dir == DIR_DOWN) *dy = 1;
}

void orc_default_config(orc_config *cfg)
{
    cfg->max_episode_steps = 10000;
    cfg->day_length = 300;
    cfg->cap_zombie = 3; cfg->cap_cow = 3; cfg->cap_skeleton = 3; cfg->cap_arrow = 3;
    cfg->cap_plant = 10;
    cfg->atlas_seed = 0;
    cfg->worldgen = ORC_WORLDGEN_VALUE;
    cfg->reset_mode = ORC_RESET_EXACT;
}

size_t orc_env_bytes(void) { return sizeof(orc_env); }

size_t orc_obs_bytes(int mode)
{
    switch (mode) {
    case ORC_OBS_SYM_U8_I8: return 1408;   /* 11 cache lines of 128 bytes */
    case ORC_OBS_SYM_U8_F32: return 1536;  /* 12 cache lines */
    case ORC_OBS_SYM_F32: return 5392;
    case ORC_OBS_PIXELS_F32: return 47632;
    }
    return 0;
}

/* ---- day / night (reading; the paper only says the observation holds a value in [0,1]) --
 * phase i = t mod L, H = L/2, k = |i - H| = distance of i from midnight (i = H), in [0,H].
 * daylight = smoothstep(k/H) = k^2 (3H - 2k) / H^3: 1 at t = 0 (noon), 0 at t = H.  Pure
 * rational arithmetic: no transcendental is evaluated anywhere. */
static void daylight_ratio(const orc_config *cfg, uint32_t t, uint64_t *num, uint64_t *den)
{
    uint64_t L = cfg->day_length, H = L / 2, i = t % L;
    uint64_t k = i < H ? H - i : i - H;
    *num = k * k * (3 * H - 2 * k);
    *den = H * H * H;
}

float orc_daylight(const orc_config *cfg, uint32_t t)
{
    uint64_t num, den;
    daylight_ratio(cfg, t, &num, &den);
    return (float)((double)num / (double)den);
}

/* darkness in 0..255, then zombie spawn probability threshold (about 1 % by day, 20 % at
 * midnight) */
uint32_t orc_zombie_spawn_threshold(const orc_config *cfg, uint32_t t)
{
    uint64_t num, den;
    daylight_ratio(cfg, t, &num, &den);
    uint32_t dark = 255u - (uint32_t)(255u * num / den);
    return (40u + 3u * dark) << 20;
}

static int light_q7(const orc_config *cfg, uint32_t t)
{
    uint64_t num, den;
    daylight_ratio(cfg, t, &num, &den);
    return (int)(127u * num / den);
}

/* ---- world generation (reading: "seeded value-noise thresholds") --------------------- */
/* Smooth interpolation weights in 1/256 units: smoothstep(k/S)*256. */
static uint32_t smooth_weight(int k, int spacing)
{
    if (spacing == 8) return (uint32_t)(12 * k * k - k * k * k);
    /* spacing 16 */
    return (uint32_t)((24 * k * k - k * k * k + 4) >> 3);
}

/* Bilinear value noise over a lattice of u16 values, result in 0..65535. */
uint32_t orc_value_noise(const uint16_t *lattice, int width, int spacing, int x, int y)
{
    int ix = x / spacing, iy = y / spacing;
    uint32_t wx = smooth_weight(x % spacing, spacing), wy = smooth_weight(y % spacing, spacing);
    uint32_t a = lattice[iy * width + ix], b = lattice[iy * width + ix + 1];
    uint32_t c = lattice[(iy + 1) * width + ix], d = lattice[(iy + 1) * width + ix + 1];
    uint32_t top = a * (256u - wx) + b * wx;
    uint32_t bot = c * (256u - wx) + d * wx;
    return (top * (256u - wy) + bot * wy) >> 16;
}

/* Perlin gradient noise (appendix "World Generation": the paper generates worlds from Perlin
 * noise after the perlin-numpy generator: unit gradients at random angles on a lattice, the four
 * corner dot products blended with the fade curve 6t^5 - 15t^4 + 10t^3, the result times sqrt 2),
 * here in integers so that the GPU can match it bit for bit:
 *   angle index a = lattice u16 >> 6 (1024 directions), gradient (cos, sin)(2 pi a / 1024) in
 *   Q14 (table from the C library, rounded to nearest);
 *   offsets from the four corners in units of 1/S (S = lattice spacing), dot = gx dx + gy dy;
 *   fade weight in Q16: (F 65536 + S^5 / 2) / S^5 with F = k^3 (6 k^2 - 15 k S + 10 S^2);
 *   lerp(p, q, w) = p + floor((q - p) w / 65536), first along x, then along y;
 *   the value n is then in units of 1 / (16384 S); it is returned on the 0..65535 scale of the
 *   terrain thresholds as 32768 + floor(n GAIN / (1024 S)), clamped (reading: the gain makes its
 *   spread about that of the value-noise fields, so that the same thresholds carve the terrain). */
#define PERLIN_GAIN 3900
static int16_t perlin_cos[1024], perlin_sin[1024];
static int perlin_ready = 0;
static void perlin_tables(void)
{
    if (perlin_ready) return;
    for (int a = 0; a < 1024; a++) {
        double th = 6.283185307179586476925286766559 * (double)a / 1024.0;
        perlin_cos[a] = (int16_t)lround(cos(th) * 16384.0);
        perlin_sin[a] = (int16_t)lround(sin(th) * 16384.0);
    }
    perlin_ready = 1;
}
static int64_t floor_div(int64_t v, int64_t d) { return v >= 0 ? v / d : -((-v + d - 1) / d); }
static int64_t perlin_fade(int k, int spacing)
{
    int64_t S = spacing, S5 = S * S * S * S * S;
    int64_t F = (int64_t)k * k * k * (6 * (int64_t)k * k - 15 * (int64_t)k * S + 10 * S * S);
    return (F * 65536 + S5 / 2) / S5;
}
static int64_t perlin_lerp(int64_t p, int64_t q, int64_t w) { return p + floor_div((q - p) * w, 65536); }
uint32_t orc_perlin_noise(const uint16_t *lattice, int width, int spacing, int x, int y)
{
    perlin_tables();
    int ix = x / spacing, iy = y / spacing, kx = x % spacing, ky = y % spacing;
    int64_t dot[2][2];
    for (int cy = 0; cy < 2; cy++)
        for (int cx = 0; cx < 2; cx++) {
            int a = lattice[(iy + cy) * width + ix + cx] >> 6;
            dot[cy][cx] = (int64_t)perlin_cos[a] * (kx - cx * spacing) + (int64_t)perlin_sin[a] * (ky - cy * spacing);
        }
    int64_t wx = perlin_fade(kx, spacing), wy = perlin_fade(ky, spacing);
    int64_t top = perlin_lerp(dot[0][0], dot[0][1], wx), bot = perlin_lerp(dot[1][0], dot[1][1], wx);
    int64_t n = perlin_lerp(top, bot, wy);
    int64_t v = 32768 + floor_div(n * PERLIN_GAIN, 1024 * (int64_t)spacing);
    return (uint32_t)(v < 0 ? 0 : (v > 65535 ? 65535 : v));
}

/* u16 number `idx` of a worldgen stream: numbers are packed two per Philox word, low half
 * first, four words per block. */
static uint16_t worldgen_u16(uint64_t seed, uint32_t env, uint32_t episode, uint32_t stream, uint32_t idx)
{
    uint32_t w = philox_word(seed, env, stream, episode, DOM_WORLDGEN, idx >> 3, (idx >> 1) & 3u);
    return (uint16_t)((idx & 1u) ? (w >> 16) : (w & 0xFFFFu));
}

/* Lattices (stream 0): two at spacing 16 (5x5 points) then four at spacing 8 (9x9). */
#define LAT16_N 25
#define LAT8_N 81
#define LAT_TOTAL (2 * LAT16_N + 4 * LAT8_N)

/* thresholds of the terrain rule, all on 0..65535 scales */
#define TH_MOUNTAIN 39500
#define TH_CAVE_M 41000
#define TH_CAVE_C 43000
#define TH_TUNNEL_CENTER 30000
#define TH_TUNNEL_HALF 1300
#define TH_LAVA_M 43000
#define TH_LAVA_F 44000
#define TH_DIAMOND_M 42000
#define U_DIAMOND 500            /* u < 500: 0.76 % of deep-mountain cells */
#define U_IRON 3000              /* 500 <= u < 3000 where the F field is low */
#define TH_IRON_F 33000
#define U_COAL 8000              /* 3000 <= u < 8000 */
#define TH_WATER 39500
#define TH_SAND 37800
#define TH_FOREST_F 33500
#define U_TREE_FOREST 26000      /* 40 % inside forests */
#define U_TREE_SPARSE 1300       /* 2 % elsewhere */
#define START_CLEAR 2            /* Chebyshev radius of forced grass around the start */
#define START_BIAS_R 10
#define START_BIAS 2500

void orc_worldgen(uint8_t *map, uint64_t seed, uint32_t env, uint32_t episode)
{
    orc_worldgen_mode(map, seed, env, episode, ORC_WORLDGEN_VALUE);
}

/* mode ORC_WORLDGEN_VALUE: the fields are value noise; ORC_WORLDGEN_PERLIN: the same lattices read
 * as gradient angles, the fields are Perlin noise.  Everything else (field mix, thresholds, start
 * area) is shared. */
static void worldgen_fields(uint8_t *map, uint64_t seed, uint32_t env, uint32_t episode, uint32_t mode, const uint16_t *theta);

void orc_worldgen_mode(uint8_t *map, uint64_t seed, uint32_t env, uint32_t episode, uint32_t mode)
{
    worldgen_fields(map, seed, env, episode, mode, NULL);
}

/* The level of the UED experiments (section "Craftax-1B: UED", noise mutation): the angle of every
 * Perlin gradient.  theta[i], in 1024ths of a turn, is added to the angle that lattice number i
 * stands for (order: the two spacing-16 lattices, then the four spacing-8 ones, row by row). */
void orc_worldgen_theta(uint8_t *map, uint64_t seed, uint32_t env, uint32_t episode, const uint16_t *theta)
{
    worldgen_fields(map, seed, env, episode, ORC_WORLDGEN_PERLIN, theta);
}

static void worldgen_fields(uint8_t *map, uint64_t seed, uint32_t env, uint32_t episode, uint32_t mode, const uint16_t *theta)
{
    uint32_t (*noise)(const uint16_t *, int, int, int, int) = mode == ORC_WORLDGEN_PERLIN ? orc_perlin_noise : orc_value_noise;
    uint16_t lat[LAT_TOTAL];
    for (uint32_t i = 0; i < LAT_TOTAL; i++) {
        lat[i] = worldgen_u16(seed, env, episode, 0, i);
        /* the angle is the upper ten bits of the lattice number */
        if (theta) lat[i] = (uint16_t)(lat[i] + ((theta[i] & 1023u) << 6));
    }
    const uint16_t *w16 = lat, *m16 = lat + LAT16_N;
    const uint16_t *w8 = lat + 2 * LAT16_N, *m8 = w8 + LAT8_N, *c8 = m8 + LAT8_N, *f8 = c8 + LAT8_N;

    for (int y = 0; y < ORC_MAP; y++) {
        for (int x = 0; x < ORC_MAP; x++) {
            int W = (int)((3u * noise(w16, 5, 16, x, y) + noise(w8, 9, 8, x, y)) >> 2);
            int M = (int)((3u * noise(m16, 5, 16, x, y) + noise(m8, 9, 8, x, y)) >> 2);
            int C = (int)noise(c8, 9, 8, x, y);
            int F = (int)noise(f8, 9, 8, x, y);
            int u = worldgen_u16(seed, env, episode, 1, (uint32_t)(y * ORC_MAP + x));
            int d = imax(iabs(x - ORC_MAP / 2), iabs(y - ORC_MAP / 2));
            if (d < START_BIAS_R) {  /* keep the start in open country */
                int bias = (START_BIAS_R - d) * START_BIAS;
                W = imax(0, W - bias);
                M = imax(0, M - bias);
            }
            uint8_t b;
            if (d <= START_CLEAR) b = B_GRASS;
            else if (M > TH_MOUNTAIN) {
                if (C > TH_CAVE_C && M > TH_CAVE_M) b = B_PATH;                      /* caves */
                else if (iabs(C - TH_TUNNEL_CENTER) < TH_TUNNEL_HALF) b = B_PATH;     /* tunnels */
                else if (M > TH_LAVA_M && F > TH_LAVA_F) b = B_LAVA;
                else if (M > TH_DIAMOND_M && u < U_DIAMOND) b = B_DIAMOND;
                else if (F < TH_IRON_F && u >= U_DIAMOND && u < U_IRON) b = B_IRON;
                else if (u >= U_IRON && u < U_COAL) b = B_COAL;
                else b = B_STONE;
            } else if (W > TH_WATER) b = B_WATER;
            else if (W > TH_SAND) b = B_SAND;
            else if (F > TH_FOREST_F && u < U_TREE_FOREST) b = B_TREE;
            else if (u < U_TREE_SPARSE) b = B_TREE;
            else b = B_GRASS;
            map[y * ORC_MAP + x] = b;
        }
    }
}

static void reset_episode(orc_env *e, const orc_config *cfg, uint32_t episode)
{
    uint64_t seed = e->seed;
    uint32_t env = e->env;
    memset(e, 0, sizeof(*e));
    e->seed = seed; e->env = env; e->episode = episode;
    orc_worldgen_mode(e->map, seed, env, episode, cfg->worldgen);
    e->px = ORC_MAP / 2; e->py = ORC_MAP / 2;
    e->dir = DIR_DOWN;
    e->vit[V_HEALTH] = e->vit[V_FOOD] = e->vit[V_DRINK] = e->vit[V_ENERGY] = MAX_COUNT;
}

void orc_reset(orc_env *e, const orc_config *cfg, uint64_t seed, uint32_t env)
{
    memset(e, 0, sizeof(*e));
    e->seed = seed; e->env = env;
    reset_episode(e, cfg, 0);
}

/* ---- helpers over the mob table ------------------------------------------------------ */
static int mob_type(int k) { return k / 3; }

static int mob_at(const orc_env *e, int x, int y)
{
    for (int k = 0; k < ORC_NMOB; k++)
        if (e->mob[k].alive && e->mob[k].x == x && e->mob[k].y == y) return k;
    return -1;
}

/* Occupancy (reading): the player and every live mob, arrows included, each own one cell. */
static int occupied(const orc_env *e, int x, int y)
{
    return (e->px == x && e->py == y) || mob_at(e, x, y) >= 0;
}

static void kill_mob(orc_env *e, int k) { memset(&e->mob[k], 0, sizeof(orc_mob)); }

static int walkable_ground(uint8_t b) { return b == B_GRASS || b == B_SAND || b == B_PATH; }
static int arrow_flyable(uint8_t b)
{
    return b == B_GRASS || b == B_SAND || b == B_PATH || b == B_WATER || b == B_LAVA;
}

static void unlock(orc_env *e, int ach) { e->ach |= 1u << ach; }

static int near_block(const orc_env *e, uint8_t b)  /* Chebyshev radius 1 around the player */
{
    for (int dy = -1; dy <= 1; dy++)
        for (int dx = -1; dx <= 1; dx++) {
            int x = e->px + dx, y = e->py + dy;
            if (inb(x, y) && e->map[y * ORC_MAP + x] == b) return 1;
        }
    return 0;
}

static int free_plant_slot(const orc_env *e, const orc_config *cfg)
{
    for (uint32_t k = 0; k < cfg->cap_plant && k < ORC_NPLANT; k++)
        if (!e->plant[k].alive) return (int)k;
    return -1;
}

static int plant_at(const orc_env *e, int x, int y)
{
    for (int k = 0; k < ORC_NPLANT; k++)
        if (e->plant[k].alive && e->plant[k].x == x && e->plant[k].y == y) return k;
    return -1;
}

static int sword_damage(const orc_env *e)  /* reading: 1 bare, 2 wood, 3 stone, 5 iron */
{
    int d = 1;
    if (e->inv[I_WOOD_SWORD]) d = 2;
    if (e->inv[I_STONE_SWORD]) d = 3;
    if (e->inv[I_IRON_SWORD]) d = 5;
    return d;
}

/* ---- phase 1: the player's action (section "RL Environment Interface": every action is
 * legal every step; unmet prerequisites make it a no-op and time still advances) --------- */
static void try_make(orc_env *e, int item, int need_furnace, int wood, int stone, int coal, int iron, int ach)
{
    if (e->inv[item]) return;                       /* reading: tools are flags, made once */
    if (!near_block(e, B_TABLE)) return;
    if (need_furnace && !near_block(e, B_FURNACE)) return;
    if (e->inv[I_WOOD] < wood || e->inv[I_STONE] < stone || e->inv[I_COAL] < coal || e->inv[I_IRON] < iron) return;
    e->inv[I_WOOD] -= wood; e->inv[I_STONE] -= stone; e->inv[I_COAL] -= coal; e->inv[I_IRON] -= iron;
    e->inv[item] = 1;
    unlock(e, ach);
}

static void collect(orc_env *e, int cell, int item, int gate_ok, uint8_t leaves, int ach)
{
    if (!gate_ok || e->inv[item] >= MAX_COUNT) return;
    e->inv[item]++;
    e->map[cell] = leaves;
    unlock(e, ach);
}

static void player_action(orc_env *e, const orc_config *cfg, int a)
{
    int dx, dy;
    if (a >= A_LEFT && a <= A_DOWN) {
        e->dir = (uint8_t)a;                           /* facing changes even when blocked */
        dir_delta(a, &dx, &dy);
        int tx = e->px + dx, ty = e->py + dy;
        if (!inb(tx, ty) || mob_at(e, tx, ty) >= 0) return;
        uint8_t b = e->map[ty * ORC_MAP + tx];
        if (walkable_ground(b)) { e->px = (uint8_t)tx; e->py = (uint8_t)ty; }
        else if (b == B_LAVA) { e->px = (uint8_t)tx; e->py = (uint8_t)ty; e->vit[V_HEALTH] = 0; }
        return;
    }
    dir_delta(e->dir, &dx, &dy);
    int tx = e->px + dx, ty = e->py + dy;
    int t_ok = inb(tx, ty);
    int cell = ty * ORC_MAP + tx;
    switch (a) {
    case A_DO: {
        if (!t_ok) return;
        int k = mob_at(e, tx, ty);
        if (k >= 0) {
            int type = mob_type(k);
            if (type == T_ARROW) return;
            int hp = e->mob[k].hp - sword_damage(e);
            if (hp > 0) { e->mob[k].hp = (int8_t)hp; return; }
            kill_mob(e, k);
            if (type == T_ZOMBIE) unlock(e, ACH_DEFEAT_ZOMBIE);
            if (type == T_SKELETON) unlock(e, ACH_DEFEAT_SKELETON);
            if (type == T_COW) {
                e->vit[V_FOOD] = (int8_t)imin(MAX_COUNT, e->vit[V_FOOD] + FOOD_COW);
                e->cnt[C_HUNGER] = 0;
                unlock(e, ACH_EAT_COW);
            }
            return;
        }
        uint8_t b = e->map[cell];
        switch (b) {
        case B_TREE: collect(e, cell, I_WOOD, 1, B_TREE, ACH_COLLECT_WOOD); break;
        case B_STONE: collect(e, cell, I_STONE, e->inv[I_WOOD_PICKAXE], B_PATH, ACH_COLLECT_STONE); break;
        case B_COAL: collect(e, cell, I_COAL, e->inv[I_WOOD_PICKAXE], B_PATH, ACH_COLLECT_COAL); break;
        case B_IRON: collect(e, cell, I_IRON, e->inv[I_STONE_PICKAXE], B_PATH, ACH_COLLECT_IRON); break;
        case B_DIAMOND: collect(e, cell, I_DIAMOND, e->inv[I_IRON_PICKAXE], B_PATH, ACH_COLLECT_DIAMOND); break;
        case B_WATER:
            e->vit[V_DRINK] = (int8_t)imin(MAX_COUNT, e->vit[V_DRINK] + 1);
            e->cnt[C_THIRST] = 0;
            unlock(e, ACH_COLLECT_DRINK);
            break;
        case B_GRASS:
            if (misc_draw(e, 3) < P_SAPLING)
                collect(e, cell, I_SAPLING, 1, B_GRASS, ACH_COLLECT_SAPLING);
            break;
        case B_RIPE: {
            int p = plant_at(e, tx, ty);
            e->vit[V_FOOD] = (int8_t)imin(MAX_COUNT, e->vit[V_FOOD] + FOOD_PLANT);
            e->cnt[C_HUNGER] = 0;
            e->map[cell] = B_PLANT;                     /* back to a sapling, still tracked */
            if (p >= 0) e->plant[p].age = 0;
            unlock(e, ACH_EAT_PLANT);
            break;
        }
        default: break;
        }
        return;
    }
    case A_SLEEP:
        if (e->vit[V_ENERGY] < MAX_COUNT) e->sleeping = 1;
        return;
    case A_PLACE_STONE: {
        if (!t_ok || mob_at(e, tx, ty) >= 0 || e->inv[I_STONE] < 1) return;
        uint8_t b = e->map[cell];
        if (!(walkable_ground(b) || b == B_WATER || b == B_LAVA)) return;
        e->inv[I_STONE]--; e->map[cell] = B_STONE; unlock(e, ACH_PLACE_STONE);
        return;
    }
    case A_PLACE_TABLE:
        if (!t_ok || mob_at(e, tx, ty) >= 0 || e->inv[I_WOOD] < 1 || !walkable_ground(e->map[cell])) return;
        e->inv[I_WOOD]--; e->map[cell] = B_TABLE; unlock(e, ACH_PLACE_TABLE);
        return;
    case A_PLACE_FURNACE:
        if (!t_ok || mob_at(e, tx, ty) >= 0 || e->inv[I_STONE] < 1 || !walkable_ground(e->map[cell])) return;
        if (!near_block(e, B_TABLE)) return;
        e->inv[I_STONE]--; e->map[cell] = B_FURNACE; unlock(e, ACH_PLACE_FURNACE);
        return;
    case A_PLACE_PLANT: {
        if (!t_ok || mob_at(e, tx, ty) >= 0 || e->inv[I_SAPLING] < 1 || e->map[cell] != B_GRASS) return;
        int s = free_plant_slot(e, cfg);
        if (s < 0) return;
        e->inv[I_SAPLING]--; e->map[cell] = B_PLANT;
        e->plant[s].alive = 1; e->plant[s].x = (uint8_t)tx; e->plant[s].y = (uint8_t)ty; e->plant[s].age = 0;
        unlock(e, ACH_PLACE_PLANT);
        return;
    }
    case A_MAKE_WOOD_PICKAXE: try_make(e, I_WOOD_PICKAXE, 0, 1, 0, 0, 0, ACH_MAKE_WOOD_PICKAXE); return;
    case A_MAKE_STONE_PICKAXE: try_make(e, I_STONE_PICKAXE, 0, 1, 1, 0, 0, ACH_MAKE_STONE_PICKAXE); return;
    case A_MAKE_IRON_PICKAXE: try_make(e, I_IRON_PICKAXE, 1, 1, 0, 1, 1, ACH_MAKE_IRON_PICKAXE); return;
    case A_MAKE_WOOD_SWORD: try_make(e, I_WOOD_SWORD, 0, 1, 0, 0, 0, ACH_MAKE_WOOD_SWORD); return;
    case A_MAKE_STONE_SWORD: try_make(e, I_STONE_SWORD, 0, 1, 1, 0, 0, ACH_MAKE_STONE_SWORD); return;
    case A_MAKE_IRON_SWORD: try_make(e, I_IRON_SWORD, 1, 1, 0, 1, 1, ACH_MAKE_IRON_SWORD); return;
    default: return;
    }
}

/* ---- phase 2: mobs (appendix "Differences ...": every slot is visited every step and
 * unspawned slots are masked).  Visiting order: zombies, cows, arrows, skeletons, so an
 * arrow shot this step first flies on the next one.  Each mob sees all earlier moves. ---- */
static int toward(int dx, int dy)
{
    if (iabs(dx) >= iabs(dy)) return dx < 0 ? DIR_LEFT : DIR_RIGHT;
    return dy < 0 ? DIR_UP : DIR_DOWN;
}

static void try_move(orc_env *e, int k, int dir, int path_only)
{
    if (dir == DIR_NONE) return;
    int dx, dy;
    dir_delta(dir, &dx, &dy);
    int tx = e->mob[k].x + dx, ty = e->mob[k].y + dy;
    if (!inb(tx, ty) || occupied(e, tx, ty)) return;
    uint8_t b = e->map[ty * ORC_MAP + tx];
    if (path_only ? (b != B_PATH) : !walkable_ground(b)) return;
    e->mob[k].x = (uint8_t)tx; e->mob[k].y = (uint8_t)ty;
}

static void mob_update(orc_env *e, const orc_config *cfg, int k, int *damage)
{
    orc_mob *m = &e->mob[k];
    if (!m->alive) return;
    int type = mob_type(k);
    int dx = (int)e->px - m->x, dy = (int)e->py - m->y;
    int adx = iabs(dx), ady = iabs(dy), cheb = imax(adx, ady);
    uint32_t r_act = slot_draw(e, k) & 0xFFFFu;
    uint32_t m8 = (slot_draw(e, k) >> 16) & 7u;     /* 0..3: a direction, 4..7: stay */

    if (type == T_ZOMBIE) {
        if (m->cd > 0) m->cd--;
        if (adx + ady == 1) {            /* orthogonally adjacent: strike when ready, never move */
            if (m->cd == 0) { *damage += e->sleeping ? DMG_ZOMBIE_SLEEP : DMG_ZOMBIE; m->cd = CD_ZOMBIE; }
            return;
        }
        int dir = DIR_NONE;
        if (cheb < CHASE_RANGE && r_act < P_CHASE) dir = toward(dx, dy);
        else if (m8 < 4) dir = (int)m8 + 1;
        try_move(e, k, dir, 0);
    } else if (type == T_COW) {
        try_move(e, k, m8 < 4 ? (int)m8 + 1 : DIR_NONE, 0);
    } else if (type == T_SKELETON) {
        if (m->cd > 0) m->cd--;
        int aligned = (dx == 0 || dy == 0) && cheb <= SHOOT_RANGE;
        if (aligned && m->cd == 0 && r_act < P_SHOOT) {
            int dir = toward(dx, dy), ddx, ddy;
            dir_delta(dir, &ddx, &ddy);
            int tx = m->x + ddx, ty = m->y + ddy;
            m->cd = CD_SKELETON;
            if (tx == e->px && ty == e->py) { *damage += DMG_ARROW; return; }   /* point blank */
            int slot = -1;
            for (uint32_t s = 0; s < cfg->cap_arrow && s < 3; s++)
                if (!e->mob[9 + s].alive) { slot = 9 + (int)s; break; }
            if (slot >= 0 && inb(tx, ty) && arrow_flyable(e->map[ty * ORC_MAP + tx]) && mob_at(e, tx, ty) < 0) {
                orc_mob *a = &e->mob[slot];
                a->alive = 1; a->x = (uint8_t)tx; a->y = (uint8_t)ty; a->dir = (uint8_t)dir; a->hp = 0; a->cd = 0;
            }
            return;
        }
        int dir = DIR_NONE;
        if (m8 < 4) dir = (int)m8 + 1;
        else if (cheb <= SHOOT_RANGE) dir = toward(dx, dy);
        try_move(e, k, dir, 1);          /* skeletons stay on paths */
    } else {                             /* arrow */
        int ddx, ddy;
        dir_delta(m->dir, &ddx, &ddy);
        int tx = m->x + ddx, ty = m->y + ddy;
        if (tx == e->px && ty == e->py) { *damage += DMG_ARROW; kill_mob(e, k); return; }
        if (!inb(tx, ty) || !arrow_flyable(e->map[ty * ORC_MAP + tx]) || mob_at(e, tx, ty) >= 0) { kill_mob(e, k); return; }
        m->x = (uint8_t)tx; m->y = (uint8_t)ty;
    }
}

/* ---- phase 3: despawn far mobs, then one spawn attempt per type -------------------------- */
static void despawn_spawn(orc_env *e, const orc_config *cfg)
{
    for (int k = 0; k < ORC_NMOB; k++) {
        orc_mob *m = &e->mob[k];
        if (m->alive && imax(iabs((int)m->x - e->px), iabs((int)m->y - e->py)) > DESPAWN_DIST) kill_mob(e, k);
    }
    const uint32_t caps[3] = { cfg->cap_zombie, cfg->cap_cow, cfg->cap_skeleton };
    const int8_t hp[3] = { HP_ZOMBIE, HP_COW, HP_SKELETON };
    for (int j = 0; j < 3; j++) {
        uint32_t w = misc_draw(e, j);
        int dx = (int)(((w & 1023u) * 31u) >> 10) - 15;
        int dy = (int)((((w >> 10) & 1023u) * 31u) >> 10) - 15;
        uint32_t rp = w >> 20;
        int slot = -1;
        for (uint32_t s = 0; s < caps[j] && s < 3; s++)
            if (!e->mob[3 * j + s].alive) { slot = 3 * j + (int)s; break; }
        int x = e->px + dx, y = e->py + dy;
        if (slot < 0 || imax(iabs(dx), iabs(dy)) < SPAWN_MIN_DIST || !inb(x, y) || occupied(e, x, y)) continue;
        uint8_t b = e->map[y * ORC_MAP + x];
        uint32_t thr = j == T_ZOMBIE ? orc_zombie_spawn_threshold(cfg, e->t) >> 20   /* its top 12 bits */
                     : j == T_COW ? P_COW_SPAWN : P_SKELETON_SPAWN;
        uint8_t want = j == T_SKELETON ? B_PATH : B_GRASS;
        if (b != want || rp >= thr) continue;
        orc_mob *m = &e->mob[slot];
        m->alive = 1; m->x = (uint8_t)x; m->y = (uint8_t)y; m->dir = 0; m->hp = hp[j]; m->cd = 0;
    }
}

/* ---- phase 4: plants (appendix "Differences ...": up to 10 growing plants are tracked) ---- */
static void plants(orc_env *e)
{
    for (int k = 0; k < ORC_NPLANT; k++) {
        orc_plant *p = &e->plant[k];
        if (!p->alive) continue;
        int cell = p->y * ORC_MAP + p->x;
        if (p->age < 65535) p->age++;
        if (e->map[cell] == B_PLANT && p->age >= RIPE_AGE) e->map[cell] = B_RIPE;
        int zombie_near = 0;
        for (int z = 0; z < 3; z++) {
            const orc_mob *m = &e->mob[z];
            if (m->alive && iabs((int)m->x - p->x) + iabs((int)m->y - p->y) == 1) zombie_near = 1;
        }
        if (zombie_near && ((slot_draw(e, k) >> 19) & 0xFFu) < P_PLANT_EATEN) {
            e->map[cell] = B_GRASS;
            memset(p, 0, sizeof(*p));
        }
    }
}

/* ---- phase 5: hunger, thirst, fatigue, recovery, sleep (reading) -------------------------- */
static void needs(orc_env *e, int damaged)
{
    int asleep = e->sleeping;
    e->cnt[C_HUNGER] += asleep ? 1 : 2;
    if (e->cnt[C_HUNGER] > 50) { e->cnt[C_HUNGER] = 0; e->vit[V_FOOD] = (int8_t)imax(0, e->vit[V_FOOD] - 1); }
    e->cnt[C_THIRST] += asleep ? 1 : 2;
    if (e->cnt[C_THIRST] > 40) { e->cnt[C_THIRST] = 0; e->vit[V_DRINK] = (int8_t)imax(0, e->vit[V_DRINK] - 1); }
    if (asleep) {
        e->cnt[C_FATIGUE]--;
        if (e->cnt[C_FATIGUE] < -10) { e->cnt[C_FATIGUE] = 0; e->vit[V_ENERGY] = (int8_t)imin(MAX_COUNT, e->vit[V_ENERGY] + 1); }
    } else {
        e->cnt[C_FATIGUE]++;
        if (e->cnt[C_FATIGUE] > 30) { e->cnt[C_FATIGUE] = 0; e->vit[V_ENERGY] = (int8_t)imax(0, e->vit[V_ENERGY] - 1); }
    }
    if (e->vit[V_HEALTH] > 0) {           /* the dead neither heal nor starve further */
        int fed = e->vit[V_FOOD] > 0 && e->vit[V_DRINK] > 0 && (e->vit[V_ENERGY] > 0 || asleep);
        e->cnt[C_RECOVER] += fed ? (asleep ? 4 : 2) : (asleep ? -1 : -2);
        if (e->cnt[C_RECOVER] > 50) { e->cnt[C_RECOVER] = 0; e->vit[V_HEALTH] = (int8_t)imin(MAX_COUNT, e->vit[V_HEALTH] + 1); }
        if (e->cnt[C_RECOVER] < -30) { e->cnt[C_RECOVER] = 0; e->vit[V_HEALTH]--; }
    }
    if (asleep && (e->vit[V_ENERGY] >= MAX_COUNT || damaged)) { e->sleeping = 0; unlock(e, ACH_WAKE_UP); }
}

static int popcount32(uint32_t v) { int c = 0; while (v) { c += (int)(v & 1u); v >>= 1; } return c; }

void orc_step_rules(orc_env *e, const orc_config *cfg, int32_t action, float *reward, uint8_t *done)
{
    static const int order[ORC_NMOB] = { 0, 1, 2, 3, 4, 5, 9, 10, 11, 6, 7, 8 };
    int health0 = e->vit[V_HEALTH];
    uint32_t ach0 = e->ach;
    int a = (action < 0 || action >= A_COUNT) ? A_NOOP : (int)action;
    if (e->sleeping) a = A_NOOP;          /* reading: a sleeping player cannot act */

    player_action(e, cfg, a);
    int damage = 0;
    for (int i = 0; i < ORC_NMOB; i++) mob_update(e, cfg, order[i], &damage);
    e->vit[V_HEALTH] = (int8_t)imax(0, e->vit[V_HEALTH] - damage);
    despawn_spawn(e, cfg);
    plants(e);
    needs(e, damage > 0);

    /* section "RL Environment Interface": +1 per achievement first unlocked this episode,
     * +-0.1 per health point; reading: one int->float conversion and one multiply. */
    int gained = popcount32(e->ach & ~ach0);
    *reward = (float)(10 * gained + ((int)e->vit[V_HEALTH] - health0)) * 0.1f;
    e->t++;
    *done = (uint8_t)(e->vit[V_HEALTH] <= 0 || e->t >= cfg->max_episode_steps);
}

/* appendix "Optimistic Environment Resets": a finished episode is replaced by a fresh one
 * within the same call.  Here the reset is exact (a new world per finished episode). */
void orc_step(orc_env *e, const orc_config *cfg, int32_t action, float *reward, uint8_t *done)
{
    orc_step_rules(e, cfg, action, reward, done);
    if (*done) reset_episode(e, cfg, e->episode + 1);
}

/* ---- observations ------------------------------------------------------------------------- */
/* Symbolic (section "RL Environment Interface", appendix "Observation Space"): a 7-row by
 * 9-column window centred on the player; per cell a one-hot over 17 block ids followed by
 * one bit per mob type (zombie, cow, skeleton, arrow); then 22 scalars.  63*21 + 22 = 1345. */
static void symbolic_cells(const orc_env *e, uint8_t *cells /* 1323 */)
{
    memset(cells, 0, ORC_VIEW_ROWS * ORC_VIEW_COLS * ORC_NCHAN);
    for (int r = 0; r < ORC_VIEW_ROWS; r++)
        for (int c = 0; c < ORC_VIEW_COLS; c++) {
            int x = e->px + c - ORC_VIEW_COLS / 2, y = e->py + r - ORC_VIEW_ROWS / 2;
            uint8_t *cell = cells + (r * ORC_VIEW_COLS + c) * ORC_NCHAN;
            uint8_t b = inb(x, y) ? e->map[y * ORC_MAP + x] : B_OOB;
            cell[b] = 1;
            int k = inb(x, y) ? mob_at(e, x, y) : -1;
            if (k >= 0) cell[ORC_NBLOCK + mob_type(k)] = 1;
        }
}

static void vector_raw(const orc_env *e, const orc_config *cfg, int v[ORC_NVEC])
{
    for (int i = 0; i < 12; i++) v[i] = e->inv[i];
    for (int i = 0; i < 4; i++) v[12 + i] = e->vit[i];
    for (int d = 1; d <= 4; d++) v[15 + d] = e->dir == d;
    v[20] = light_q7(cfg, e->t);
    v[21] = e->sleeping;
}

/* appendix "Observation Space", table of inventory observations: counts as sqrt(n)/10,
 * vitals as x/10, indicators as 0/1, day/night in [0,1]. */
static void vector_f32(const orc_env *e, const orc_config *cfg, float v[ORC_NVEC])
{
    for (int i = 0; i < 6; i++) v[i] = (float)(sqrt((double)e->inv[i]) / 10.0);
    for (int i = 6; i < 12; i++) v[i] = (float)e->inv[i];
    for (int i = 0; i < 4; i++) v[12 + i] = (float)((double)e->vit[i] / 10.0);
    for (int d = 1; d <= 4; d++) v[15 + d] = e->dir == d ? 1.0f : 0.0f;
    v[20] = orc_daylight(cfg, e->t);
    v[21] = (float)e->sleeping;
}

/* Pixel observation (reading; the paper's textures are figures that are not available):
 * a 9x9 window of tiles centred on the player, 7x7 pixels per tile, RGB float in [0,1].
 * Tile texels come from a seeded atlas[16][7][7][3], index = block id - 1; an entity
 * (player, zombie, cow, skeleton, arrow) overrides the pixels its 7x7 mask selects with its
 * own texels; every pixel is multiplied once by the daylight value. */
static float atlas_texel(uint64_t seed, uint32_t stream, uint32_t idx)
{
    uint32_t w = philox_word(seed, 0, stream, 0, DOM_ATLAS, idx >> 2, idx & 3u);
    return (float)(w >> 8) * (1.0f / 16777216.0f);
}

static int atlas_mask(uint64_t seed, uint32_t idx)
{
    return (int)(philox_word(seed, 0, 2, 0, DOM_ATLAS, idx >> 2, idx & 3u) >> 31);
}

static void pixels(const orc_env *e, const orc_config *cfg, float *out /* 63*63*3 */)
{
    float light = orc_daylight(cfg, e->t);
    for (int tr = 0; tr < 9; tr++)
        for (int tc = 0; tc < 9; tc++) {
            int x = e->px + tc - 4, y = e->py + tr - 4;
            int b = inb(x, y) ? e->map[y * ORC_MAP + x] : B_OOB;
            int ent = -1;                              /* 0 player, 1 + mob type otherwise */
            if (tr == 4 && tc == 4) ent = 0;
            else if (inb(x, y)) { int k = mob_at(e, x, y); if (k >= 0) ent = 1 + mob_type(k); }
            for (int py = 0; py < 7; py++)
                for (int px = 0; px < 7; px++)
                    for (int ch = 0; ch < 3; ch++) {
                        uint32_t in_tile = (uint32_t)((py * 7 + px) * 3 + ch);
                        float texel = atlas_texel(cfg->atlas_seed, 0, (uint32_t)(b - 1) * 147u + in_tile);
                        if (ent >= 0 && atlas_mask(cfg->atlas_seed, (uint32_t)ent * 49u + (uint32_t)(py * 7 + px)))
                            texel = atlas_texel(cfg->atlas_seed, 1, (uint32_t)ent * 147u + in_tile);
                        out[((tr * 7 + py) * 63 + (tc * 7 + px)) * 3 + ch] = texel * light;
                    }
        }
}

void orc_observe(const orc_env *e, const orc_config *cfg, int mode, void *obs)
{
    uint8_t *o = (uint8_t *)obs;
    memset(o, 0, orc_obs_bytes(mode));
    if (mode == ORC_OBS_PIXELS_F32) { pixels(e, cfg, (float *)obs); return; }
    uint8_t cells[ORC_VIEW_ROWS * ORC_VIEW_COLS * ORC_NCHAN];
    symbolic_cells(e, cells);
    if (mode == ORC_OBS_SYM_U8_I8) {
        int v[ORC_NVEC];
        memcpy(o, cells, sizeof(cells));
        vector_raw(e, cfg, v);
        for (int i = 0; i < ORC_NVEC; i++) ((int8_t *)(o + 1328))[i] = (int8_t)v[i];
    } else if (mode == ORC_OBS_SYM_U8_F32) {
        float v[ORC_NVEC];
        memcpy(o, cells, sizeof(cells));
        vector_f32(e, cfg, v);
        memcpy(o + 1328, v, sizeof(v));
    } else if (mode == ORC_OBS_SYM_F32) {
        float *f = (float *)obs;
        for (size_t i = 0; i < sizeof(cells); i++) f[i] = (float)cells[i];
        vector_f32(e, cfg, f + sizeof(cells));
    }
}

/* ---- batch loops ------------------------------------------------------------------------------ */
void orc_reset_batch(orc_env *envs, const orc_config *cfg, const uint64_t *seeds, const uint32_t *env_ids, int n)
{
    for (int i = 0; i < n; i++) orc_reset(&envs[i], cfg, seeds[i], env_ids ? env_ids[i] : (uint32_t)i);
}

void orc_observe_batch(const orc_env *envs, const orc_config *cfg, int mode, void *obs, int n)
{
    size_t stride = orc_obs_bytes(mode);
    for (int i = 0; i < n; i++) orc_observe(&envs[i], cfg, mode, (uint8_t *)obs + stride * (size_t)i);
}

void orc_step_batch(orc_env *envs, const orc_config *cfg, const int32_t *actions, int mode, void *obs,
                    float *reward, uint8_t *done, int n)
{
    size_t stride = orc_obs_bytes(mode);
    for (int i = 0; i < n; i++) {
        orc_step(&envs[i], cfg, actions[i], &reward[i], &done[i]);
        if (obs) orc_observe(&envs[i], cfg, mode, (uint8_t *)obs + stride * (size_t)i);
    }
}

/* ---- optimistic resets (appendix "Optimistic Environment Resets") ---------------------------------
 * The paper: with N workers only M << N new worlds are generated per step (one per 16 workers);
 * the environments that need a reset sample without replacement from those M, and only if more
 * than M finish in one step do some get the same world.  Readings: world j of the pool of batch
 * step T is the ordinary generator run for (seed of environment 0, environment number 2^31 + j,
 * episode T); the finished environments are taken in increasing number, the r-th of them (r from
 * 0) gets world (shift_T + r) mod M, where shift_T is one uniform draw per step -- distinct worlds
 * for up to M resets, repeats beyond; the environment keeps its own seed and counts its episode
 * up, so everything random after the reset still differs between environments that share a world. */
uint32_t orc_pool_slot(uint64_t pool_seed, uint32_t step_index, uint32_t rank, uint32_t n)
{
    uint32_t m = (uint32_t)n / ORC_POOL_RATIO ? (uint32_t)n / ORC_POOL_RATIO : 1u;
    uint32_t shift = choice(philox_word(pool_seed, 0xFFFFFFFFu, 2, step_index, DOM_WORLDGEN, 0, 0), m);
    return (shift + rank) % m;
}

void orc_step_batch_pool(orc_env *envs, const orc_config *cfg, const int32_t *actions, int mode, void *obs,
                         float *reward, uint8_t *done, int n, uint32_t step_index)
{
    size_t stride = orc_obs_bytes(mode);
    uint64_t pool_seed = envs[0].seed;
    for (int i = 0; i < n; i++) orc_step_rules(&envs[i], cfg, actions[i], &reward[i], &done[i]);
    uint32_t rank = 0;
    for (int i = 0; i < n; i++) {
        if (!done[i]) continue;
        orc_env *e = &envs[i];
        uint32_t slot = orc_pool_slot(pool_seed, step_index, rank++, (uint32_t)n);
        uint64_t seed = e->seed;
        uint32_t env = e->env, episode = e->episode + 1;
        memset(e, 0, sizeof(*e));
        e->seed = seed; e->env = env; e->episode = episode;
        orc_worldgen_mode(e->map, pool_seed, 0x80000000u | slot, step_index, cfg->worldgen);
        e->px = ORC_MAP / 2; e->py = ORC_MAP / 2;
        e->dir = DIR_DOWN;
        e->vit[V_HEALTH] = e->vit[V_FOOD] = e->vit[V_DRINK] = e->vit[V_ENERGY] = MAX_COUNT;
    }
    if (obs)
        for (int i = 0; i < n; i++) orc_observe(&envs[i], cfg, mode, (uint8_t *)obs + stride * (size_t)i);
}

/* ---- level mutations (section "Craftax-1B: UED") ------------------------------------------------
 * "Swap" exchanges two tiles of different type, one of them inside the central 16x16 area of the
 * map; "restricted swap" only exchanges tiles of one group: stone with the ores, grass with
 * trees.  Reading (the paper gives no more than that): up to 32 tries; try k draws Philox block
 * (env, round, 0, MUTATE | k) under the mutation seed: word 0 picks the central cell
 * (choice of 256, row-major inside the area), word 1 the other cell (choice of all cells).  A try
 * is refused if the two blocks are equal, if a cell holds the player or a live mob, if a block is
 * a plant (plants are tracked in a table), or, restricted, if the blocks are not of one group.
 * The first try that is not refused is carried out.  Returns that try's number + 1, or 0. */
static int swap_group(uint8_t b)
{
    if (b == B_STONE || b == B_COAL || b == B_IRON || b == B_DIAMOND) return 1;
    if (b == B_GRASS || b == B_TREE) return 2;
    return 0;
}
int orc_mutate_swap(orc_env *e, uint64_t mutation_seed, uint32_t round, int restricted)
{
    const int c0 = (ORC_MAP - 16) / 2;
    for (uint32_t k = 0; k < 32; k++) {
        uint32_t a = choice(philox_word(mutation_seed, e->env, round, 0, DOM_MUTATE, k, 0), 256);
        uint32_t b = choice(philox_word(mutation_seed, e->env, round, 0, DOM_MUTATE, k, 1), ORC_MAP * ORC_MAP);
        int ax = c0 + (int)(a % 16), ay = c0 + (int)(a / 16), bx = (int)(b % ORC_MAP), by = (int)(b / ORC_MAP);
        uint8_t ba = e->map[ay * ORC_MAP + ax], bb = e->map[by * ORC_MAP + bx];
        if (ba == bb) continue;
        if (occupied(e, ax, ay) || occupied(e, bx, by)) continue;
        if (ba == B_PLANT || ba == B_RIPE || bb == B_PLANT || bb == B_RIPE) continue;
        if (restricted && (swap_group(ba) == 0 || swap_group(ba) != swap_group(bb))) continue;
        e->map[ay * ORC_MAP + ax] = bb;
        e->map[by * ORC_MAP + bx] = ba;
        return (int)k + 1;
    }
    return 0;
}

/* Noise mutation (section "Craftax-1B: UED"): a uniform random number is added to every element
 * of the level's angle vector theta (here an integer in [-amplitude, amplitude], in 1024ths of a
 * turn, element i from u16 number i of a stream of its own), the world of the current episode is
 * generated again from the new angles, and the episode starts over in it. */
void orc_mutate_noise(orc_env *e, const orc_config *cfg, uint16_t *theta, uint64_t mutation_seed, uint32_t round, uint32_t amplitude)
{
    (void)cfg;
    for (uint32_t i = 0; i < LAT_TOTAL; i++) {
        uint32_t w = philox_word(mutation_seed, e->env, round, 1, DOM_MUTATE, i >> 3, (i >> 1) & 3u);
        uint32_t d = (i & 1u) ? (w >> 16) : (w & 0xFFFFu);
        int32_t u = (int32_t)((d * (2u * amplitude + 1u)) >> 16) - (int32_t)amplitude;
        theta[i] = (uint16_t)(((int32_t)(theta[i] & 1023u) + u) & 1023);
    }
    uint64_t seed = e->seed;
    uint32_t env = e->env, episode = e->episode;
    memset(e, 0, sizeof(*e));
    e->seed = seed; e->env = env; e->episode = episode;
    orc_worldgen_theta(e->map, seed, env, episode, theta);
    e->px = ORC_MAP / 2; e->py = ORC_MAP / 2;
    e->dir = DIR_DOWN;
    e->vit[V_HEALTH] = e->vit[V_FOOD] = e->vit[V_DRINK] = e->vit[V_ENERGY] = MAX_COUNT;
}
