/*
 * CPU oracle: full Craftax (see craftax_full.h).  TEST INFRASTRUCTURE ONLY.
 * Plain scalar C, one environment at a time.  "reading:" marks rules the paper does not print.
 */
#include "craftax_full.h"
#include <string.h>
#include <math.h>

/* ---- ids fixed by the paper ---------------------------------------------------------------- */
enum { B_INVALID = 0, B_OOB = 1, B_GRASS = 2, B_WATER = 3, B_STONE = 4, B_TREE = 5, B_WOOD = 6, B_PATH = 7,
       B_COAL = 8, B_IRON = 9, B_DIAMOND = 10, B_TABLE = 11, B_FURNACE = 12, B_SAND = 13, B_LAVA = 14,
       B_PLANT = 15, B_RIPE = 16, B_WALL = 17, B_DARKNESS = 18, B_WALL_MOSS = 19, B_STALAGMITE = 20,
       B_SAPPHIRE = 21, B_RUBY = 22, B_CHEST = 23, B_FOUNTAIN = 24, B_FIRE_GRASS = 25, B_ICE_GRASS = 26,
       B_GRAVEL = 27, B_FIRE_TREE = 28, B_ICE_SHRUB = 29, B_ENCH_FIRE = 30, B_ENCH_ICE = 31,
       B_NECROMANCER = 32, B_GRAVE1 = 33, B_GRAVE2 = 34, B_GRAVE3 = 35, B_NECRO_VULN = 36, B_COUNT = 37 };
enum { IT_NONE = 0, IT_TORCH = 1, IT_LADDER_DOWN = 2, IT_LADDER_UP = 3, IT_LADDER_DOWN_BLOCKED = 4 };
enum { A_NOOP = 0, A_LEFT, A_RIGHT, A_UP, A_DOWN, A_DO, A_SLEEP, A_PLACE_STONE, A_PLACE_TABLE, A_PLACE_FURNACE,
       A_PLACE_PLANT, A_MAKE_WOOD_PICKAXE, A_MAKE_STONE_PICKAXE, A_MAKE_IRON_PICKAXE, A_MAKE_WOOD_SWORD,
       A_MAKE_STONE_SWORD, A_MAKE_IRON_SWORD, A_REST, A_DESCEND, A_ASCEND, A_MAKE_DIAMOND_PICKAXE,
       A_MAKE_DIAMOND_SWORD, A_MAKE_IRON_ARMOUR, A_MAKE_DIAMOND_ARMOUR, A_SHOOT_ARROW, A_MAKE_ARROW,
       A_CAST_FIREBALL, A_CAST_ICEBALL, A_PLACE_TORCH, A_DRINK_POTION_RED, A_DRINK_POTION_GREEN,
       A_DRINK_POTION_BLUE, A_DRINK_POTION_PINK, A_DRINK_POTION_CYAN, A_DRINK_POTION_YELLOW, A_READ_BOOK,
       A_ENCHANT_SWORD, A_ENCHANT_ARMOUR, A_MAKE_TORCH, A_LEVEL_UP_DEXTERITY, A_LEVEL_UP_STRENGTH,
       A_LEVEL_UP_INTELLIGENCE, A_ENCHANT_BOW };
enum { ACH_COLLECT_WOOD = 0, ACH_PLACE_TABLE, ACH_EAT_COW, ACH_COLLECT_SAPLING, ACH_COLLECT_DRINK,
       ACH_MAKE_WOOD_PICKAXE, ACH_MAKE_WOOD_SWORD, ACH_PLACE_PLANT, ACH_DEFEAT_ZOMBIE, ACH_COLLECT_STONE,
       ACH_PLACE_STONE, ACH_EAT_PLANT, ACH_DEFEAT_SKELETON, ACH_MAKE_STONE_PICKAXE, ACH_MAKE_STONE_SWORD,
       ACH_WAKE_UP, ACH_PLACE_FURNACE, ACH_COLLECT_COAL, ACH_COLLECT_IRON, ACH_COLLECT_DIAMOND,
       ACH_MAKE_IRON_PICKAXE, ACH_MAKE_IRON_SWORD, ACH_MAKE_ARROW, ACH_MAKE_TORCH, ACH_PLACE_TORCH,
       ACH_MAKE_DIAMOND_SWORD, ACH_MAKE_IRON_ARMOUR, ACH_MAKE_DIAMOND_ARMOUR, ACH_ENTER_GNOMISH_MINES,
       ACH_ENTER_DUNGEON, ACH_ENTER_SEWERS, ACH_ENTER_VAULT, ACH_ENTER_TROLL_MINES, ACH_ENTER_FIRE_REALM,
       ACH_ENTER_ICE_REALM, ACH_ENTER_GRAVEYARD, ACH_DEFEAT_GNOME_WARRIOR, ACH_DEFEAT_GNOME_ARCHER,
       ACH_DEFEAT_ORC_SOLIDER, ACH_DEFEAT_ORC_MAGE, ACH_DEFEAT_LIZARD, ACH_DEFEAT_KOBOLD, ACH_DEFEAT_TROLL,
       ACH_DEFEAT_DEEP_THING, ACH_DEFEAT_PIGMAN, ACH_DEFEAT_FIRE_ELEMENTAL, ACH_DEFEAT_FROST_TROLL,
       ACH_DEFEAT_ICE_ELEMENTAL, ACH_DAMAGE_NECROMANCER, ACH_DEFEAT_NECROMANCER, ACH_EAT_BAT, ACH_EAT_SNAIL,
       ACH_FIND_BOW, ACH_FIRE_BOW, ACH_COLLECT_SAPPHIRE, ACH_LEARN_FIREBALL, ACH_CAST_FIREBALL,
       ACH_LEARN_ICEBALL, ACH_CAST_ICEBALL, ACH_COLLECT_RUBY, ACH_MAKE_DIAMOND_PICKAXE, ACH_OPEN_CHEST,
       ACH_DRINK_POTION, ACH_ENCHANT_SWORD, ACH_ENCHANT_ARMOUR, ACH_DEFEAT_KNIGHT, ACH_DEFEAT_ARCHER };

/* appendix "Achievements": categories Basic 1, Intermediate 3, Advanced 5, Very Advanced 8 */
int cf_achievement_reward(int id)
{
    static const int8_t r[CF_NACH] = {
        1, 1, 1, 1, 1, 1, 1, 1, 1, 1, 1, 1, 1, 1, 1, 1, 1, 1, 1, 1, 1, 1, 1, 1, 1,   /* 0..24 */
        3, 3, 3, 3, 3,                                                               /* 25..29 */
        5, 5, 5, 8, 8, 8,                                                            /* 30..35 */
        3, 3, 3, 3, 5, 5, 5, 5, 8, 8, 8, 8, 8, 8,                                    /* 36..49 */
        3, 3, 3, 3, 3, 5, 5, 5, 5, 3, 3, 3, 3, 5, 5, 5, 5 };                         /* 50..66 */
    return (id >= 0 && id < CF_NACH) ? r[id] : 0;
}

/* appendix "Creatures".  health, damage (physical, fire, ice), defence % (physical, fire, ice),
 * collision (0 ground, 1 flying, 2 amphibian, 3 aquatic), achievement for defeating / eating.
 * reading: a single defence number is physical defence; a coloured one is that element's. */
enum { C_ZOMBIE = 0, C_SKELETON, C_COW, C_ORC_SOLDIER, C_ORC_MAGE, C_SNAIL, C_GNOME_WARRIOR, C_GNOME_ARCHER,
       C_BAT, C_LIZARD, C_KOBOLD, C_KNIGHT, C_ARCHER, C_TROLL, C_DEEP_THING, C_PIGMAN, C_FIRE_ELEMENTAL,
       C_FROST_TROLL, C_ICE_ELEMENTAL, C_COUNT };
enum { COL_GROUND = 0, COL_FLYING = 1, COL_AMPHIBIAN = 2, COL_AQUATIC = 3 };
static const int16_t CREATURE[C_COUNT][9] = {
    /* hp  dp df di  Dp   Df   Di  col ach */
    { 5,  2, 0, 0,  0,   0,   0, COL_GROUND, ACH_DEFEAT_ZOMBIE },
    { 3,  2, 0, 0,  0,   0,   0, COL_GROUND, ACH_DEFEAT_SKELETON },
    { 3,  0, 0, 0,  0,   0,   0, COL_GROUND, ACH_EAT_COW },
    { 7,  3, 0, 0,  0,   0,   0, COL_GROUND, ACH_DEFEAT_ORC_SOLIDER },
    { 5,  3, 0, 0,  0,   0,   0, COL_GROUND, ACH_DEFEAT_ORC_MAGE },
    { 6,  0, 0, 0,  0,   0,   0, COL_GROUND, ACH_EAT_SNAIL },
    { 9,  4, 0, 0,  0,   0,   0, COL_GROUND, ACH_DEFEAT_GNOME_WARRIOR },
    { 6,  2, 0, 0,  0,   0,   0, COL_GROUND, ACH_DEFEAT_GNOME_ARCHER },
    { 4,  0, 0, 0,  0,   0,   0, COL_FLYING, ACH_EAT_BAT },
    { 11, 5, 0, 0,  0,   0,   0, COL_AMPHIBIAN, ACH_DEFEAT_LIZARD },
    { 8,  4, 0, 0,  0,   0,   0, COL_GROUND, ACH_DEFEAT_KOBOLD },
    { 12, 6, 0, 0,  50,  0,   0, COL_GROUND, ACH_DEFEAT_KNIGHT },
    { 12, 4, 0, 0,  50,  0,   0, COL_GROUND, ACH_DEFEAT_ARCHER },
    { 20, 6, 1, 1,  20,  0,   0, COL_GROUND, ACH_DEFEAT_TROLL },
    { 6,  4, 3, 3,  0,   0,   0, COL_AQUATIC, ACH_DEFEAT_DEEP_THING },
    { 20, 3, 5, 0,  90,  100, 0, COL_GROUND, ACH_DEFEAT_PIGMAN },
    { 14, 3, 5, 0,  90,  100, 0, COL_FLYING, ACH_DEFEAT_FIRE_ELEMENTAL },
    { 24, 4, 0, 5,  90,  0,   100, COL_GROUND, ACH_DEFEAT_FROST_TROLL },
    { 16, 4, 0, 4,  90,  0,   100, COL_FLYING, ACH_DEFEAT_ICE_ELEMENTAL },
};
int cf_creature(int index, int field) { return (index >= 0 && index < C_COUNT && field >= 0 && field < 9) ? CREATURE[index][field] : -1; }

/* which creature lives where (appendix "Creatures", column Floor); floor 8 = boss waves */
static const int8_t MELEE_OF_FLOOR[8] = { C_ZOMBIE, C_ORC_SOLDIER, C_GNOME_WARRIOR, C_LIZARD, C_KNIGHT, C_TROLL, C_PIGMAN, C_FROST_TROLL };
static const int8_t RANGED_OF_FLOOR[8] = { C_SKELETON, C_ORC_MAGE, C_GNOME_ARCHER, C_KOBOLD, C_ARCHER, C_DEEP_THING, C_FIRE_ELEMENTAL, C_ICE_ELEMENTAL };
static const int8_t PASSIVE_OF_FLOOR[8] = { C_COW, C_SNAIL, C_BAT, C_SNAIL, C_SNAIL, C_BAT, C_BAT, -1 };
static const int8_t ENTER_ACH[CF_FLOORS] = { -1, ACH_ENTER_DUNGEON, ACH_ENTER_GNOMISH_MINES, ACH_ENTER_SEWERS, ACH_ENTER_VAULT,
                                             ACH_ENTER_TROLL_MINES, ACH_ENTER_FIRE_REALM, ACH_ENTER_ICE_REALM, ACH_ENTER_GRAVEYARD };
static const uint8_t FLOOR_LIT[CF_FLOORS] = { 1, 1, 0, 1, 1, 0, 1, 0, 0 };   /* section "World Generation": 2, 5, 7, 8 are dark */

enum { I_WOOD = 0, I_STONE, I_COAL, I_IRON, I_DIAMOND, I_SAPPHIRE, I_RUBY, I_SAPLING, I_TORCH, I_ARROW };
enum { V_HEALTH = 0, V_FOOD, V_DRINK, V_ENERGY, V_MANA };
enum { K_HUNGER = 0, K_THIRST, K_FATIGUE, K_RECOVER, K_MANA };
enum { S_MELEE0 = 0, S_RANGED0 = 3, S_PASSIVE0 = 5, S_MPROJ0 = 8, S_PPROJ0 = 11 };
enum { PP_ARROW = 0, PP_FIREBALL = 1, PP_ICEBALL = 2 };

/* ---- constants of this build's reading ---------------------------------------------------- */
#define INV_MAX 99
#define CD_MELEE 5
#define CD_RANGED 4
#define CHASE_RANGE 8
#define SHOOT_RANGE 4
#define DESPAWN_DIST 15
#define SPAWN_MIN_DIST 5
#define RIPE_AGE 300
#define FOOD_MEAT 6
#define FOOD_PLANT 4
#define KILLS_TO_CLEAR 8
#define BOSS_HITS 8
#define MAX_LIGHT 20
#define P_SAPLING 429496730u
#define P_CHASE 3435973836u
#define P_SHOOT 0x80000000u
#define P_PLANT_EATEN 0x20000000u
#define P_PASSIVE_SPAWN 0x08000000u      /* 1/32 */
#define P_RANGED_SPAWN 0x0CCCCCCCu       /* 5 %  */
#define P_MELEE_SPAWN 0x0CCCCCCCu        /* 5 % below the overworld */

enum { DOM_STEP = 0, DOM_WORLDGEN = 1, DOM_MUTATE = 4 };

static uint32_t philox_word(uint64_t seed, uint32_t c0, uint32_t c1, uint32_t c2, uint32_t dom, uint32_t block, uint32_t word)
{
    uint32_t ctr[4] = { c0, c1, c2, (dom << 16) | block };
    uint32_t key[2] = { (uint32_t)seed, (uint32_t)(seed >> 32) };
    uint32_t out[4];
    orc_philox4x32_10(ctr, key, out);
    return out[word];
}
/* Step draws: block k (k = 0..13) = (move draw of slot k, decision draw of slot k, eaten draw of plant
 * k, misc[k]); misc[3j..3j+2] = (x, y, p) of the spawn attempt of class j (melee, ranged, passive);
 * misc[9] sapling, misc[10] and misc[11] chest loot. */
uint32_t cf_step_draw(const cf_env *e, uint32_t block, uint32_t word)
{
    return philox_word(e->seed, e->env, e->t, e->episode, DOM_STEP, block, word);
}
/* World generation: stream = floor*4 + {0 lattice u16s, 1 per-cell u16s, 2 layout words}; stream 63 = potions */
static uint32_t wg_word(const cf_env *e, uint32_t stream, uint32_t idx)
{
    return philox_word(e->seed, e->env, stream, e->episode, DOM_WORLDGEN, idx >> 2, idx & 3u);
}
static uint16_t wg_u16(const cf_env *e, uint32_t stream, uint32_t idx)
{
    uint32_t w = wg_word(e, stream, idx >> 1);
    return (uint16_t)((idx & 1u) ? (w >> 16) : (w & 0xFFFFu));
}
static uint32_t choice(uint32_t u, uint32_t n) { return (uint32_t)(((uint64_t)u * n) >> 32); }
static int iabs(int v) { return v < 0 ? -v : v; }
static int imax(int a, int b) { return a > b ? a : b; }
static int imin(int a, int b) { return a < b ? a : b; }
static int inb(int x, int y) { return x >= 0 && x < CF_W && y >= 0 && y < CF_W; }
static void dir_delta(int dir, int *dx, int *dy)
{
    *dx = dir == 1 ? -1 : (dir == 2 ? 1 : 0);
    *dy = dir == 3 ? -1 : (dir == 4 ? 1 : 0);
}
static int cell(int x, int y) { return y * CF_W + x; }

void cf_default_config(cf_config *cfg)
{
    cfg->max_episode_steps = 100000;   /* appendix "Further Environment Details" */
    cfg->day_length = 300;
    cfg->cap_melee = 3; cfg->cap_ranged = 2; cfg->cap_passive = 3;
    cfg->cap_plant = 10;
    cfg->atlas_seed = 0;
    cfg->worldgen = ORC_WORLDGEN_VALUE;
    cfg->reset_mode = ORC_RESET_EXACT;
}
size_t cf_env_bytes(void) { return sizeof(cf_env); }
size_t cf_obs_bytes(int mode)
{
    if (mode == CF_OBS_U8_F32) return 8448;       /* 66 cache lines */
    if (mode == CF_OBS_F32) return 33152;         /* 259 cache lines */
    return 171648;                                /* 130 x 110 x 3 floats = 171600 bytes, padded to 1341 cache lines */
}

static void unlock(cf_env *e, int a) { e->ach[a >> 5] |= 1u << (a & 31); }

/* terrain classes (reading) */
static int walkable(uint8_t b)
{
    return b == B_GRASS || b == B_SAND || b == B_PATH || b == B_FIRE_GRASS || b == B_ICE_GRASS || b == B_GRAVEL;
}
static int flyable(uint8_t b) { return walkable(b) || b == B_WATER || b == B_LAVA; }
static int passable_for(int collision, uint8_t b)
{
    switch (collision) {
    case COL_GROUND: return walkable(b);
    case COL_FLYING: return flyable(b);
    case COL_AMPHIBIAN: return walkable(b) || b == B_WATER;
    default: return b == B_WATER;
    }
}

/* ---- day / night: same smoothstep curve as the Classic oracle ----------------------------- */
static void daylight_ratio(const cf_config *cfg, uint32_t t, uint64_t *num, uint64_t *den)
{
    uint64_t L = cfg->day_length, H = L / 2, i = t % L;
    uint64_t k = i < H ? H - i : i - H;
    *num = k * k * (3 * H - 2 * k);
    *den = H * H * H;
}
static float daylight(const cf_config *cfg, uint32_t t)
{
    uint64_t n, d; daylight_ratio(cfg, t, &n, &d);
    return (float)((double)n / (double)d);
}
static uint32_t zombie_threshold(const cf_config *cfg, uint32_t t)
{
    uint64_t n, d; daylight_ratio(cfg, t, &n, &d);
    return (40u + 3u * (255u - (uint32_t)(255u * n / d))) << 20;
}

/* ---- world generation (reading: noise thresholds for open floors, rooms + corridors for dungeons) */
static void set_ladders(cf_env *e, int f, int ux, int uy, int dx, int dy)
{
    if (f > 0) { e->block[f][cell(ux, uy)] = B_PATH; e->item[f][cell(ux, uy)] = IT_LADDER_UP; e->ladder_up[f][0] = (uint8_t)ux; e->ladder_up[f][1] = (uint8_t)uy; }
    if (f < CF_FLOORS - 1) {
        e->block[f][cell(dx, dy)] = B_PATH;
        e->item[f][cell(dx, dy)] = f == 0 ? IT_LADDER_DOWN : IT_LADDER_DOWN_BLOCKED;
        e->ladder_down[f][0] = (uint8_t)dx; e->ladder_down[f][1] = (uint8_t)dy;
    }
}

/* The open floors take their fields from value noise (the benchmark configurations) or, as the
 * paper's appendix "World Generation" has it, from Perlin noise over the same lattices. */
typedef uint32_t (*noise_fn)(const uint16_t *, int, int, int, int);
static noise_fn noise_of(uint32_t mode) { return mode == ORC_WORLDGEN_PERLIN ? orc_perlin_noise : orc_value_noise; }

/* theta (may be NULL): the level's angle offsets for this floor's lattices, in 1024ths of a turn;
 * the angle of a lattice point is the upper ten bits of its number (section "Craftax-1B: UED",
 * noise mutation). */
static uint16_t turned(uint16_t number, const uint16_t *theta, uint32_t i)
{
    return theta ? (uint16_t)(number + ((theta[i] & 1023u) << 6)) : number;
}

static void gen_overworld(cf_env *e, uint32_t mode, const uint16_t *theta)
{
    const int f = 0;
    const noise_fn noise = noise_of(mode);
    uint16_t lat[CF_THETA_OVERWORLD];
    for (uint32_t i = 0; i < CF_THETA_OVERWORLD; i++) lat[i] = turned(wg_u16(e, 0, i), theta, i);
    const uint16_t *w16 = lat, *m16 = lat + 16, *w8 = lat + 32, *m8 = w8 + 49, *c8 = m8 + 49, *f8 = c8 + 49;
    for (int y = 0; y < CF_W; y++)
        for (int x = 0; x < CF_W; x++) {
            int W = (int)((3u * noise(w16, 4, 16, x, y) + noise(w8, 7, 8, x, y)) >> 2);
            int M = (int)((3u * noise(m16, 4, 16, x, y) + noise(m8, 7, 8, x, y)) >> 2);
            int C = (int)noise(c8, 7, 8, x, y), F = (int)noise(f8, 7, 8, x, y);
            int u = wg_u16(e, 1, (uint32_t)cell(x, y));
            int d = imax(iabs(x - CF_W / 2), iabs(y - CF_W / 2));
            if (d < 10) { int bias = (10 - d) * 2500; W = imax(0, W - bias); M = imax(0, M - bias); }
            uint8_t b;
            if (d <= 2) b = B_GRASS;
            else if (M > 39500) {
                if (C > 43000 && M > 41000) b = B_PATH;
                else if (iabs(C - 30000) < 1300) b = B_PATH;
                else if (M > 43000 && F > 44000) b = B_LAVA;
                else if (M > 42000 && u < 500) b = B_DIAMOND;
                else if (F < 33000 && u >= 500 && u < 3000) b = B_IRON;
                else if (u >= 3000 && u < 8000) b = B_COAL;
                else b = B_STONE;
            } else if (W > 39500) b = B_WATER;
            else if (W > 37800) b = B_SAND;
            else if (F > 33500 && u < 26000) b = B_TREE;
            else if (u < 1300) b = B_TREE;
            else b = B_GRASS;
            e->block[f][cell(x, y)] = b;
        }
    int dx = (int)choice(wg_word(e, 2, 0), 13) - 6, dy = (int)choice(wg_word(e, 2, 1), 13) - 6;
    if (imax(iabs(dx), iabs(dy)) < 3) dx = 3;
    set_ladders(e, f, 0, 0, CF_W / 2 + dx, CF_W / 2 + dy);
}

static void carve_line(cf_env *e, int f, int x0, int y0, int x1, int y1, uint8_t b)
{
    /* horizontal along y0 from x0 to x1, then vertical along x1 from y0 to y1 */
    for (int x = imin(x0, x1); x <= imax(x0, x1); x++) e->block[f][cell(x, y0)] = b;
    for (int y = imin(y0, y1); y <= imax(y0, y1); y++) e->block[f][cell(x1, y)] = b;
}

static void gen_dungeon(cf_env *e, int f)
{
    const uint8_t wall = f == 3 ? B_WALL_MOSS : B_WALL;
    memset(e->block[f], wall, CF_CELLS);
    int cx[8], cy[8];
    for (int i = 0; i < 8; i++) {
        int w = 5 + (int)choice(wg_word(e, (uint32_t)f * 4 + 2, (uint32_t)(4 * i)), 5);
        int h = 5 + (int)choice(wg_word(e, (uint32_t)f * 4 + 2, (uint32_t)(4 * i + 1)), 5);
        int x = 1 + (int)choice(wg_word(e, (uint32_t)f * 4 + 2, (uint32_t)(4 * i + 2)), (uint32_t)(46 - w));
        int y = 1 + (int)choice(wg_word(e, (uint32_t)f * 4 + 2, (uint32_t)(4 * i + 3)), (uint32_t)(46 - h));
        cx[i] = x + w / 2; cy[i] = y + h / 2;
        for (int yy = y; yy < y + h; yy++)
            for (int xx = x; xx < x + w; xx++) {
                uint8_t b = B_PATH;
                if (f == 3 && wg_u16(e, (uint32_t)f * 4 + 1, (uint32_t)cell(xx, yy)) < 12000) b = B_WATER;   /* sewers */
                e->block[f][cell(xx, yy)] = b;
            }
    }
    for (int i = 1; i <= 6; i++) e->block[f][cell(cx[i] + 1, cy[i] + 1)] = B_CHEST;
    if (f == 1) e->block[f][cell(cx[2] - 1, cy[2] - 1)] = B_FOUNTAIN;
    if (f == 4) { e->block[f][cell(cx[3] - 1, cy[3] - 1)] = B_ENCH_FIRE; e->block[f][cell(cx[4] - 1, cy[4] - 1)] = B_ENCH_ICE; }
    /* corridors last, so that room centre 0 (ladder up) always reaches room centre 7 (ladder down) */
    for (int i = 0; i + 1 < 8; i++) carve_line(e, f, cx[i], cy[i], cx[i + 1], cy[i + 1], B_PATH);
    set_ladders(e, f, cx[0], cy[0], cx[7], cy[7]);
}

static void gen_cave(cf_env *e, int f, uint32_t mode, const uint16_t *theta)
{
    const noise_fn noise = noise_of(mode);
    uint16_t lat[CF_THETA_CAVE];
    for (uint32_t i = 0; i < CF_THETA_CAVE; i++) lat[i] = turned(wg_u16(e, (uint32_t)f * 4, i), theta, i);
    const uint16_t *c8 = lat, *f8 = lat + 49;
    const uint8_t open = f == 6 ? B_FIRE_GRASS : (f == 7 ? B_ICE_GRASS : B_PATH);
    for (int y = 0; y < CF_W; y++)
        for (int x = 0; x < CF_W; x++) {
            int C = (int)noise(c8, 7, 8, x, y), F = (int)noise(f8, 7, 8, x, y);
            int u = wg_u16(e, (uint32_t)f * 4 + 1, (uint32_t)cell(x, y));
            uint8_t b;
            if (C > 31000) {            /* open cave */
                b = open;
                if (f == 2 && u < 1500) b = B_STALAGMITE;
                if (f == 5 && F > 44000) b = B_WATER;
                if (f == 6) { if (F > 43000) b = B_LAVA; else if (u < 3000) b = B_FIRE_TREE; }
                if (f == 7) { if (F > 43000) b = B_WATER; else if (u < 3000) b = B_ICE_SHRUB; }
            } else {                    /* rock with ores */
                b = B_STONE;
                if (f == 2 || f == 5) {
                    if (u < 5000) b = B_COAL;
                    else if (u < 7500) b = B_IRON;
                    else if (u < 8000) b = B_DIAMOND;
                    else if (u < (f == 2 ? 8600 : 9000)) b = B_SAPPHIRE;
                    else if (u < (f == 2 ? 9200 : 10000)) b = B_RUBY;
                } else if (f == 6) { if (u < 2500) b = B_RUBY; else if (u < 6000) b = B_COAL; }
                else { if (u < 2500) b = B_SAPPHIRE; else if (u < 5000) b = B_DIAMOND; }
            }
            e->block[f][cell(x, y)] = b;
        }
    int ux = 10 + (int)choice(wg_word(e, (uint32_t)f * 4 + 2, 0), 6), uy = 10 + (int)choice(wg_word(e, (uint32_t)f * 4 + 2, 1), 6);
    int dx = 32 + (int)choice(wg_word(e, (uint32_t)f * 4 + 2, 2), 6), dy = 32 + (int)choice(wg_word(e, (uint32_t)f * 4 + 2, 3), 6);
    for (int yy = -1; yy <= 1; yy++)
        for (int xx = -1; xx <= 1; xx++) { e->block[f][cell(ux + xx, uy + yy)] = open; e->block[f][cell(dx + xx, dy + yy)] = open; }
    carve_line(e, f, ux, uy, dx, dy, open);     /* the two ladders are always connected */
    set_ladders(e, f, ux, uy, dx, dy);
}

static void gen_graveyard(cf_env *e)
{
    const int f = 8;
    for (int y = 0; y < CF_W; y++)
        for (int x = 0; x < CF_W; x++)
            e->block[f][cell(x, y)] = (x == 0 || y == 0 || x == CF_W - 1 || y == CF_W - 1) ? B_WALL : B_PATH;
    for (int j = 0; j < 3; j++)
        for (int i = 0; i < 5; i++) e->block[f][cell(8 + 8 * i, 12 + 12 * j)] = (uint8_t)(B_GRAVE1 + (i + j) % 3);
    e->block[f][cell(24, 6)] = B_NECRO_VULN;
    set_ladders(e, f, 24, 42, 0, 0);
}

/* Where the angles of floor f stand in a level's vector: the overworld's six lattices first, then
 * the two lattices of each cave floor in floor order; -1 for a floor without noise. */
static int theta_offset(int f)
{
    switch (f) {
    case 0: return 0;
    case 2: return CF_THETA_OVERWORLD;
    case 5: return CF_THETA_OVERWORLD + CF_THETA_CAVE;
    case 6: return CF_THETA_OVERWORLD + 2 * CF_THETA_CAVE;
    case 7: return CF_THETA_OVERWORLD + 3 * CF_THETA_CAVE;
    default: return -1;
    }
}
static void worldgen_floor(cf_env *e, int f, uint32_t mode, const uint16_t *theta)
{
    const uint16_t *th = theta && theta_offset(f) >= 0 ? theta + theta_offset(f) : NULL;
    memset(e->item[f], IT_NONE, CF_CELLS);
    memset(e->light[f], FLOOR_LIT[f] ? MAX_LIGHT : 0, CF_CELLS);
    if (f == 0) gen_overworld(e, mode, th);
    else if (f == 1 || f == 3 || f == 4) gen_dungeon(e, f);
    else if (f == 8) gen_graveyard(e);
    else gen_cave(e, f, mode, th);
}
void cf_worldgen_floor_mode(cf_env *e, int f, uint32_t mode) { worldgen_floor(e, f, mode, NULL); }
void cf_worldgen_floor(cf_env *e, int f) { worldgen_floor(e, f, ORC_WORLDGEN_VALUE, NULL); }
void cf_worldgen_floor_theta(cf_env *e, int f, const uint16_t *theta) { worldgen_floor(e, f, ORC_WORLDGEN_PERLIN, theta); }

static void start_episode(cf_env *e, const cf_config *cfg, uint32_t episode, const uint16_t *theta)
{
    uint64_t seed = e->seed; uint32_t env = e->env;
    memset(e, 0, sizeof(*e));
    e->seed = seed; e->env = env; e->episode = episode;
    for (int f = 0; f < CF_FLOORS; f++) worldgen_floor(e, f, cfg->worldgen, theta);
    e->px = CF_W / 2; e->py = CF_W / 2; e->dir = 4;
    for (int i = 0; i < 5; i++) e->vit[i] = 9;
    e->dex = e->str = e->intel = 1;
    e->boss_vulnerable = 1;
    e->visited = 1;
    /* section "Potions and Enchantments": the colour -> effect map is re-drawn every episode */
    for (int i = 0; i < 6; i++) e->potion_effect[i] = (uint8_t)i;
    for (int i = 5; i >= 1; i--) {
        int j = (int)choice(wg_word(e, 63, (uint32_t)(5 - i)), (uint32_t)(i + 1));
        uint8_t tmp = e->potion_effect[i]; e->potion_effect[i] = e->potion_effect[j]; e->potion_effect[j] = tmp;
    }
}
static void reset_episode(cf_env *e, const cf_config *cfg, uint32_t episode) { start_episode(e, cfg, episode, NULL); }
void cf_reset(cf_env *e, const cf_config *cfg, uint64_t seed, uint32_t env)
{
    memset(e, 0, sizeof(*e));
    e->seed = seed; e->env = env;
    reset_episode(e, cfg, 0);
}

/* ---- helpers ------------------------------------------------------------------------------ */
static int mob_at_floor(const cf_env *e, int f, int x, int y)
{
    const cf_mob *m = e->mob[f];
    for (int k = 0; k < CF_NSLOT; k++) if (m[k].alive && m[k].x == x && m[k].y == y) return k;
    return -1;
}
static int mob_at(const cf_env *e, int x, int y) { return mob_at_floor(e, e->floor, x, y); }
static int occupied(const cf_env *e, int x, int y) { return (e->px == x && e->py == y) || mob_at(e, x, y) >= 0; }
static void kill_mob(cf_env *e, int k) { memset(&e->mob[e->floor][k], 0, sizeof(cf_mob)); }
static int near_block(const cf_env *e, uint8_t b)
{
    for (int dy = -1; dy <= 1; dy++)
        for (int dx = -1; dx <= 1; dx++) {
            int x = e->px + dx, y = e->py + dy;
            if (inb(x, y) && e->block[e->floor][cell(x, y)] == b) return 1;
        }
    return 0;
}
static int cap_health(const cf_env *e) { return 9 + (5 * (e->str - 1)) / 4; }     /* 9, 10, 11, 12, 14 */
static int cap_need(const cf_env *e) { return 9 + 2 * (e->dex - 1); }              /* up to 17 */
static int cap_mana(const cf_env *e) { return 9 + 3 * (e->intel - 1); }            /* up to 21 */
static void add_inv(cf_env *e, int item, int n) { e->inv[item] = (uint8_t)imin(INV_MAX, e->inv[item] + n); }

/* damage = sum over elements of attack * (100 - defence) / 100, integer parts */
static int apply_defence(const int atk[3], const int def[3])
{
    int d = 0;
    for (int i = 0; i < 3; i++) d += atk[i] * (100 - def[i]) / 100;
    return d;
}
static void player_defence(const cf_env *e, int def[3])
{
    def[0] = def[1] = def[2] = 0;
    for (int i = 0; i < 4; i++) {
        def[0] += 10 * e->armour[i];
        if (e->armour_ench[i] == 1) def[1] += 20;
        if (e->armour_ench[i] == 2) def[2] += 20;
    }
}
static int damage_to_player(const cf_env *e, int creature)
{
    int atk[3] = { CREATURE[creature][1], CREATURE[creature][2], CREATURE[creature][3] }, def[3];
    player_defence(e, def);
    int d = apply_defence(atk, def);
    return (e->sleeping || e->resting) ? 2 * d : d;
}
static void melee_attack(const cf_env *e, int atk[3])
{
    static const int base[5] = { 1, 2, 3, 5, 8 };
    atk[0] = base[e->sword] + (e->str - 1); atk[1] = e->sword_ench == 1 ? 4 : 0; atk[2] = e->sword_ench == 2 ? 4 : 0;
}
static void projectile_attack(const cf_env *e, int kind, int atk[3])
{
    atk[0] = atk[1] = atk[2] = 0;
    if (kind == PP_ARROW) { atk[0] = 2 + (e->dex - 1); if (e->bow_ench == 1) atk[1] = 4; if (e->bow_ench == 2) atk[2] = 4; }
    else if (kind == PP_FIREBALL) atk[1] = 4 + 2 * (e->intel - 1);
    else atk[2] = 4 + 2 * (e->intel - 1);
}
/* the player hurts mob slot k with the given attack */
static void hurt_mob(cf_env *e, int k, const int atk[3])
{
    cf_mob *m = &e->mob[e->floor][k];
    if (k >= S_MPROJ0) return;                     /* projectiles cannot be hit */
    int c = m->type;
    int def[3] = { CREATURE[c][4], CREATURE[c][5], CREATURE[c][6] };
    int hp = m->hp - apply_defence(atk, def);
    if (hp > 0) { m->hp = (int8_t)hp; return; }
    kill_mob(e, k);
    unlock(e, CREATURE[c][8]);
    if (k >= S_PASSIVE0) { e->vit[V_FOOD] = (int8_t)imin(cap_need(e), e->vit[V_FOOD] + FOOD_MEAT); e->cnt[K_HUNGER] = 0; }
    else {
        const int f = e->floor;
        if (e->kills[f] < 255) e->kills[f]++;
        /* section "World Generation" of the dungeon floors: the way down opens after enough kills */
        if (f >= 1 && f < CF_FLOORS - 1 && e->kills[f] >= KILLS_TO_CLEAR) {
            int c = cell(e->ladder_down[f][0], e->ladder_down[f][1]);
            if (e->item[f][c] == IT_LADDER_DOWN_BLOCKED) e->item[f][c] = IT_LADDER_DOWN;
        }
    }
}
static int free_slot(const cf_env *e, int first, int count, int cap)
{
    for (int s = 0; s < count && s < cap; s++) if (!e->mob[e->floor][first + s].alive) return first + s;
    return -1;
}

/* a projectile of the player leaves the facing cell (reading) */
static int shoot(cf_env *e, int kind)
{
    int dx, dy; dir_delta(e->dir, &dx, &dy);
    int tx = e->px + dx, ty = e->py + dy;
    if (!inb(tx, ty)) return 0;
    int k = mob_at(e, tx, ty);
    if (k >= 0) {
        if (k >= S_MPROJ0) return 0;
        int atk[3]; projectile_attack(e, kind, atk); hurt_mob(e, k, atk);
        return 1;
    }
    int s = free_slot(e, S_PPROJ0, 3, 3);
    if (s < 0 || !flyable(e->block[e->floor][cell(tx, ty)])) return 0;
    cf_mob *m = &e->mob[e->floor][s];
    m->alive = 1; m->x = (uint8_t)tx; m->y = (uint8_t)ty; m->dir = e->dir; m->hp = 0; m->cd = 0; m->type = (uint8_t)kind;
    return 1;
}

static void place_torch_light(cf_env *e, int x, int y)
{
    for (int dy = -4; dy <= 4; dy++)
        for (int dx = -4; dx <= 4; dx++) {
            int xx = x + dx, yy = y + dy;
            if (!inb(xx, yy)) continue;
            int l = MAX_LIGHT - 4 * imax(iabs(dx), iabs(dy));
            uint8_t *p = &e->light[e->floor][cell(xx, yy)];
            if (l > *p) *p = (uint8_t)l;
        }
}

static void change_floor(cf_env *e, int nf, int x, int y)
{
    if (mob_at_floor(e, nf, x, y) >= 0) return;                /* the far end of the ladder must be free */
    e->floor = (uint8_t)nf; e->px = (uint8_t)x; e->py = (uint8_t)y;
    if (!(e->visited >> nf & 1)) {
        e->visited |= (uint16_t)(1u << nf);
        if (e->xp < 255) e->xp++;                              /* section "Attributes" */
        if (ENTER_ACH[nf] >= 0) unlock(e, ENTER_ACH[nf]);
    }
}

static void open_chest(cf_env *e, int c)
{
    uint32_t r0 = cf_step_draw(e, 10, 3), r1 = cf_step_draw(e, 11, 3);
    e->block[e->floor][c] = B_PATH;
    unlock(e, ACH_OPEN_CHEST);
    if (e->floor == 1 && !e->bow) { e->bow = 1; unlock(e, ACH_FIND_BOW); return; }   /* section "Combat" */
    e->potion[choice(r0, 6)] = (uint8_t)imin(INV_MAX, e->potion[choice(r0, 6)] + 1);
    uint32_t k = choice(r1, 4);
    if (k == 0) add_inv(e, I_ARROW, 4);
    else if (k == 1) add_inv(e, I_TORCH, 4);
    else if (k == 2 && e->book < 2) e->book++;                 /* books live in dungeon chests */
}

static int try_craft(cf_env *e, int need_furnace, int wood, int stone, int coal, int iron, int diamond)
{
    if (!near_block(e, B_TABLE) || (need_furnace && !near_block(e, B_FURNACE))) return 0;
    if (e->inv[I_WOOD] < wood || e->inv[I_STONE] < stone || e->inv[I_COAL] < coal || e->inv[I_IRON] < iron || e->inv[I_DIAMOND] < diamond) return 0;
    e->inv[I_WOOD] -= wood; e->inv[I_STONE] -= stone; e->inv[I_COAL] -= coal; e->inv[I_IRON] -= iron; e->inv[I_DIAMOND] -= diamond;
    return 1;
}

/* ---- phase 1: the player's action ----------------------------------------------------------- */
static void player_action(cf_env *e, const cf_config *cfg, int a)
{
    const int f = e->floor;
    int dx, dy;
    if (a >= A_LEFT && a <= A_DOWN) {
        e->dir = (uint8_t)a;
        dir_delta(a, &dx, &dy);
        int tx = e->px + dx, ty = e->py + dy;
        if (!inb(tx, ty) || mob_at(e, tx, ty) >= 0) return;
        uint8_t b = e->block[f][cell(tx, ty)];
        if (walkable(b)) { e->px = (uint8_t)tx; e->py = (uint8_t)ty; }
        else if (b == B_LAVA) { e->px = (uint8_t)tx; e->py = (uint8_t)ty; e->vit[V_HEALTH] = 0; }
        return;
    }
    dir_delta(e->dir, &dx, &dy);
    const int tx = e->px + dx, ty = e->py + dy, t_ok = inb(tx, ty), c = cell(tx, ty);
    const int here = cell(e->px, e->py);
    switch (a) {
    case A_DO: {
        if (!t_ok) return;
        int k = mob_at(e, tx, ty);
        if (k >= 0) { int atk[3]; melee_attack(e, atk); hurt_mob(e, k, atk); return; }
        uint8_t b = e->block[f][c];
        int item = -1, level = 0, ach = -1; uint8_t leaves = B_PATH;
        switch (b) {
        case B_TREE: item = I_WOOD; ach = ACH_COLLECT_WOOD; leaves = B_TREE; break;
        case B_STONE: item = I_STONE; level = 1; ach = ACH_COLLECT_STONE; break;
        case B_STALAGMITE: item = I_STONE; level = 1; ach = ACH_COLLECT_STONE; break;
        case B_COAL: item = I_COAL; level = 1; ach = ACH_COLLECT_COAL; break;
        case B_IRON: item = I_IRON; level = 2; ach = ACH_COLLECT_IRON; break;
        case B_DIAMOND: item = I_DIAMOND; level = 3; ach = ACH_COLLECT_DIAMOND; break;
        case B_SAPPHIRE: item = I_SAPPHIRE; level = 4; ach = ACH_COLLECT_SAPPHIRE; break;
        case B_RUBY: item = I_RUBY; level = 4; ach = ACH_COLLECT_RUBY; break;
        case B_GRASS:
            if (cf_step_draw(e, 9, 3) < P_SAPLING) { item = I_SAPLING; ach = ACH_COLLECT_SAPLING; leaves = B_GRASS; }
            break;
        case B_WATER: case B_FOUNTAIN:
            e->vit[V_DRINK] = (int8_t)imin(cap_need(e), e->vit[V_DRINK] + 1); e->cnt[K_THIRST] = 0; unlock(e, ACH_COLLECT_DRINK);
            break;
        case B_RIPE:
            e->vit[V_FOOD] = (int8_t)imin(cap_need(e), e->vit[V_FOOD] + FOOD_PLANT); e->cnt[K_HUNGER] = 0;
            e->block[f][c] = B_PLANT;
            for (int p = 0; p < CF_NPLANT; p++) if (e->plant[p].alive && e->plant[p].x == tx && e->plant[p].y == ty) e->plant[p].age = 0;
            unlock(e, ACH_EAT_PLANT);
            break;
        case B_CHEST: open_chest(e, c); break;
        case B_NECRO_VULN:
            /* section "Boss Floor": each hit calls a wave of the next floor's enemies */
            unlock(e, ACH_DAMAGE_NECROMANCER);
            e->boss_hits++;
            if (e->boss_hits >= BOSS_HITS) { unlock(e, ACH_DEFEAT_NECROMANCER); e->block[f][c] = B_PATH; e->boss_vulnerable = 0; }
            else {
                e->block[f][c] = B_NECROMANCER; e->boss_vulnerable = 0;
                const int w = e->boss_hits - 1;
                for (int s = 0; s < 3; s++) {
                    int x = 20 + 4 * s, y = 10;
                    if (!e->mob[f][S_MELEE0 + s].alive && !occupied(e, x, y)) {
                        cf_mob *m = &e->mob[f][S_MELEE0 + s];
                        m->alive = 1; m->x = (uint8_t)x; m->y = (uint8_t)y; m->dir = 0; m->type = (uint8_t)MELEE_OF_FLOOR[w]; m->hp = (int8_t)CREATURE[m->type][0]; m->cd = 0;
                    }
                }
                for (int s = 0; s < 2; s++) {
                    int x = 22 + 4 * s, y = 8;
                    if (!e->mob[f][S_RANGED0 + s].alive && !occupied(e, x, y)) {
                        cf_mob *m = &e->mob[f][S_RANGED0 + s];
                        m->alive = 1; m->x = (uint8_t)x; m->y = (uint8_t)y; m->dir = 0; m->type = (uint8_t)RANGED_OF_FLOOR[w]; m->hp = (int8_t)CREATURE[m->type][0]; m->cd = 0;
                    }
                }
            }
            break;
        default: break;
        }
        if (item >= 0 && e->pickaxe >= level && e->inv[item] < INV_MAX) {
            e->inv[item]++; e->block[f][c] = leaves; unlock(e, ach);
        }
        return;
    }
    case A_SLEEP: if (e->vit[V_ENERGY] < cap_need(e)) e->sleeping = 1; return;
    case A_REST: if (e->vit[V_HEALTH] < cap_health(e)) e->resting = 1; return;
    case A_PLACE_STONE: case A_PLACE_TABLE: case A_PLACE_FURNACE: case A_PLACE_PLANT: case A_PLACE_TORCH: {
        if (!t_ok || mob_at(e, tx, ty) >= 0 || e->item[f][c] != IT_NONE) return;
        uint8_t b = e->block[f][c];
        if (a == A_PLACE_STONE) {
            if (e->inv[I_STONE] < 1 || !(walkable(b) || b == B_WATER || b == B_LAVA)) return;
            e->inv[I_STONE]--; e->block[f][c] = B_STONE; unlock(e, ACH_PLACE_STONE);
        } else if (a == A_PLACE_TABLE) {
            if (e->inv[I_WOOD] < 1 || !walkable(b)) return;
            e->inv[I_WOOD]--; e->block[f][c] = B_TABLE; unlock(e, ACH_PLACE_TABLE);
        } else if (a == A_PLACE_FURNACE) {
            if (e->inv[I_STONE] < 1 || !walkable(b) || !near_block(e, B_TABLE)) return;
            e->inv[I_STONE]--; e->block[f][c] = B_FURNACE; unlock(e, ACH_PLACE_FURNACE);
        } else if (a == A_PLACE_PLANT) {
            if (f != 0 || e->inv[I_SAPLING] < 1 || b != B_GRASS) return;
            int s = -1;
            for (uint32_t p = 0; p < cfg->cap_plant && p < CF_NPLANT; p++) if (!e->plant[p].alive) { s = (int)p; break; }
            if (s < 0) return;
            e->inv[I_SAPLING]--; e->block[f][c] = B_PLANT;
            e->plant[s].alive = 1; e->plant[s].x = (uint8_t)tx; e->plant[s].y = (uint8_t)ty; e->plant[s].age = 0;
            unlock(e, ACH_PLACE_PLANT);
        } else {
            if (e->inv[I_TORCH] < 1 || !walkable(b)) return;
            e->inv[I_TORCH]--; e->item[f][c] = IT_TORCH; place_torch_light(e, tx, ty); unlock(e, ACH_PLACE_TORCH);
        }
        return;
    }
    /* tools are levels: 1 wood, 2 stone, 3 iron, 4 diamond; a MAKE only ever raises the level */
    case A_MAKE_WOOD_PICKAXE: if (e->pickaxe < 1 && try_craft(e, 0, 1, 0, 0, 0, 0)) { e->pickaxe = 1; unlock(e, ACH_MAKE_WOOD_PICKAXE); } return;
    case A_MAKE_STONE_PICKAXE: if (e->pickaxe < 2 && try_craft(e, 0, 1, 1, 0, 0, 0)) { e->pickaxe = 2; unlock(e, ACH_MAKE_STONE_PICKAXE); } return;
    case A_MAKE_IRON_PICKAXE: if (e->pickaxe < 3 && try_craft(e, 1, 1, 0, 1, 1, 0)) { e->pickaxe = 3; unlock(e, ACH_MAKE_IRON_PICKAXE); } return;
    case A_MAKE_DIAMOND_PICKAXE: if (e->pickaxe < 4 && try_craft(e, 1, 1, 0, 0, 0, 3)) { e->pickaxe = 4; unlock(e, ACH_MAKE_DIAMOND_PICKAXE); } return;
    case A_MAKE_WOOD_SWORD: if (e->sword < 1 && try_craft(e, 0, 1, 0, 0, 0, 0)) { e->sword = 1; unlock(e, ACH_MAKE_WOOD_SWORD); } return;
    case A_MAKE_STONE_SWORD: if (e->sword < 2 && try_craft(e, 0, 1, 1, 0, 0, 0)) { e->sword = 2; unlock(e, ACH_MAKE_STONE_SWORD); } return;
    case A_MAKE_IRON_SWORD: if (e->sword < 3 && try_craft(e, 1, 1, 0, 1, 1, 0)) { e->sword = 3; unlock(e, ACH_MAKE_IRON_SWORD); } return;
    case A_MAKE_DIAMOND_SWORD: if (e->sword < 4 && try_craft(e, 1, 1, 0, 0, 0, 2)) { e->sword = 4; unlock(e, ACH_MAKE_DIAMOND_SWORD); } return;
    case A_MAKE_IRON_ARMOUR: case A_MAKE_DIAMOND_ARMOUR: {
        const int lvl = a == A_MAKE_IRON_ARMOUR ? 1 : 2;
        int piece = -1;
        for (int i = 0; i < 4; i++) if (e->armour[i] < lvl) { piece = i; break; }
        if (piece < 0) return;
        if (lvl == 1 ? try_craft(e, 1, 0, 0, 3, 3, 0) : try_craft(e, 1, 0, 0, 0, 0, 3)) {
            e->armour[piece] = (uint8_t)lvl; unlock(e, lvl == 1 ? ACH_MAKE_IRON_ARMOUR : ACH_MAKE_DIAMOND_ARMOUR);
        }
        return;
    }
    case A_MAKE_ARROW: if (try_craft(e, 0, 1, 1, 0, 0, 0)) { add_inv(e, I_ARROW, 2); unlock(e, ACH_MAKE_ARROW); } return;
    case A_MAKE_TORCH: if (try_craft(e, 0, 1, 0, 1, 0, 0)) { add_inv(e, I_TORCH, 4); unlock(e, ACH_MAKE_TORCH); } return;
    case A_SHOOT_ARROW: if (e->bow && e->inv[I_ARROW] >= 1 && shoot(e, PP_ARROW)) { e->inv[I_ARROW]--; unlock(e, ACH_FIRE_BOW); } return;
    case A_CAST_FIREBALL: if (e->learned_fireball && e->vit[V_MANA] >= 2 && shoot(e, PP_FIREBALL)) { e->vit[V_MANA] -= 2; unlock(e, ACH_CAST_FIREBALL); } return;
    case A_CAST_ICEBALL: if (e->learned_iceball && e->vit[V_MANA] >= 2 && shoot(e, PP_ICEBALL)) { e->vit[V_MANA] -= 2; unlock(e, ACH_CAST_ICEBALL); } return;
    case A_DESCEND:
        if (f < CF_FLOORS - 1 && e->item[f][here] == IT_LADDER_DOWN)
            change_floor(e, f + 1, e->ladder_up[f + 1][0], e->ladder_up[f + 1][1]);
        return;
    case A_ASCEND:
        if (f > 0 && e->item[f][here] == IT_LADDER_UP)
            change_floor(e, f - 1, e->ladder_down[f - 1][0], e->ladder_down[f - 1][1]);
        return;
    case A_READ_BOOK:
        if (e->book < 1 || (e->learned_fireball && e->learned_iceball)) return;
        e->book--;
        if (!e->learned_fireball) { e->learned_fireball = 1; unlock(e, ACH_LEARN_FIREBALL); }
        else { e->learned_iceball = 1; unlock(e, ACH_LEARN_ICEBALL); }
        return;
    case A_ENCHANT_SWORD: case A_ENCHANT_ARMOUR: case A_ENCHANT_BOW: {
        /* section "Potions and Enchantments": mana and a gemstone at an enchantment table */
        if (!t_ok) return;
        uint8_t b = e->block[f][c];
        if (b != B_ENCH_FIRE && b != B_ENCH_ICE) return;
        const int elem = b == B_ENCH_FIRE ? 1 : 2, gem = elem == 1 ? I_RUBY : I_SAPPHIRE;
        if (e->vit[V_MANA] < 9 || e->inv[gem] < 1) return;
        if (a == A_ENCHANT_SWORD) { if (e->sword < 1 || e->sword_ench == elem) return; e->sword_ench = (uint8_t)elem; unlock(e, ACH_ENCHANT_SWORD); }
        else if (a == A_ENCHANT_BOW) { if (!e->bow || e->bow_ench == elem) return; e->bow_ench = (uint8_t)elem; }
        else {
            int piece = -1;
            for (int i = 0; i < 4; i++) if (e->armour[i] > 0 && e->armour_ench[i] != elem) { piece = i; break; }
            if (piece < 0) return;
            e->armour_ench[piece] = (uint8_t)elem; unlock(e, ACH_ENCHANT_ARMOUR);
        }
        e->vit[V_MANA] -= 9; e->inv[gem]--;
        return;
    }
    case A_LEVEL_UP_DEXTERITY: if (e->xp >= 1 && e->dex < 5) { e->xp--; e->dex++; } return;
    case A_LEVEL_UP_STRENGTH: if (e->xp >= 1 && e->str < 5) { e->xp--; e->str++; } return;
    case A_LEVEL_UP_INTELLIGENCE: if (e->xp >= 1 && e->intel < 5) { e->xp--; e->intel++; } return;
    default: break;
    }
    if (a >= A_DRINK_POTION_RED && a <= A_DRINK_POTION_YELLOW) {
        const int col = a - A_DRINK_POTION_RED;
        if (e->potion[col] < 1) return;
        e->potion[col]--;
        unlock(e, ACH_DRINK_POTION);
        /* effects (reading): health +8 / -3, mana +8 / -3, energy +8 / -3 */
        const int eff = e->potion_effect[col], which = eff >> 1, delta = (eff & 1) ? -3 : 8;
        const int vit = which == 0 ? V_HEALTH : (which == 1 ? V_MANA : V_ENERGY);
        const int cap = which == 0 ? cap_health(e) : (which == 1 ? cap_mana(e) : cap_need(e));
        e->vit[vit] = (int8_t)imax(0, imin(cap, e->vit[vit] + delta));
    }
}

/* ---- phase 2: mobs of the current floor -------------------------------------------------------- */
static int toward(int dx, int dy)
{
    if (iabs(dx) >= iabs(dy)) return dx < 0 ? 1 : 2;
    return dy < 0 ? 3 : 4;
}
static void try_move(cf_env *e, int k, int dir, int collision)
{
    if (!dir) return;
    cf_mob *m = &e->mob[e->floor][k];
    int dx, dy; dir_delta(dir, &dx, &dy);
    int tx = m->x + dx, ty = m->y + dy;
    if (!inb(tx, ty) || occupied(e, tx, ty) || !passable_for(collision, e->block[e->floor][cell(tx, ty)])) return;
    m->x = (uint8_t)tx; m->y = (uint8_t)ty;
}
static void mob_update(cf_env *e, const cf_config *cfg, int k, int *damage)
{
    (void)cfg;
    cf_mob *m = &e->mob[e->floor][k];
    if (!m->alive) return;
    const int dx = (int)e->px - m->x, dy = (int)e->py - m->y, adx = iabs(dx), ady = iabs(dy), cheb = imax(adx, ady);
    const uint32_t m8 = choice(cf_step_draw(e, (uint32_t)k, 0), 8), r_act = cf_step_draw(e, (uint32_t)k, 1);
    const int wander = m8 < 4 ? (int)m8 + 1 : 0;
    if (k < S_RANGED0) {                                 /* melee */
        if (m->cd > 0) m->cd--;
        if (adx + ady == 1) { if (m->cd == 0) { *damage += damage_to_player(e, m->type); m->cd = CD_MELEE; } return; }
        try_move(e, k, (cheb < CHASE_RANGE && r_act < P_CHASE) ? toward(dx, dy) : wander, CREATURE[m->type][7]);
    } else if (k < S_PASSIVE0) {                         /* ranged */
        if (m->cd > 0) m->cd--;
        const int aligned = (dx == 0 || dy == 0) && cheb <= SHOOT_RANGE;
        if (aligned && m->cd == 0 && r_act < P_SHOOT) {
            int dir = toward(dx, dy), ddx, ddy; dir_delta(dir, &ddx, &ddy);
            int tx = m->x + ddx, ty = m->y + ddy;
            m->cd = CD_RANGED;
            if (tx == e->px && ty == e->py) { *damage += damage_to_player(e, m->type); return; }
            int s = free_slot(e, S_MPROJ0, 3, 3);
            if (s >= 0 && inb(tx, ty) && flyable(e->block[e->floor][cell(tx, ty)]) && mob_at(e, tx, ty) < 0) {
                cf_mob *p = &e->mob[e->floor][s];
                p->alive = 1; p->x = (uint8_t)tx; p->y = (uint8_t)ty; p->dir = (uint8_t)dir; p->hp = 0; p->cd = 0; p->type = m->type;
            }
            return;
        }
        try_move(e, k, wander ? wander : (cheb <= SHOOT_RANGE ? toward(dx, dy) : 0), CREATURE[m->type][7]);
    } else if (k < S_MPROJ0) {                           /* passive */
        try_move(e, k, wander, CREATURE[m->type][7]);
    } else {                                             /* projectiles */
        int ddx, ddy; dir_delta(m->dir, &ddx, &ddy);
        int tx = m->x + ddx, ty = m->y + ddy;
        if (k < S_PPROJ0) {
            if (tx == e->px && ty == e->py) { *damage += damage_to_player(e, m->type); kill_mob(e, k); return; }
            if (!inb(tx, ty) || !flyable(e->block[e->floor][cell(tx, ty)]) || mob_at(e, tx, ty) >= 0) { kill_mob(e, k); return; }
        } else {
            int hit = inb(tx, ty) ? mob_at(e, tx, ty) : -1;
            if (hit >= 0) { int atk[3]; projectile_attack(e, m->type, atk); hurt_mob(e, hit, atk); kill_mob(e, k); return; }
            if (!inb(tx, ty) || (tx == e->px && ty == e->py) || !flyable(e->block[e->floor][cell(tx, ty)])) { kill_mob(e, k); return; }
        }
        m->x = (uint8_t)tx; m->y = (uint8_t)ty;
    }
}

static void despawn_spawn(cf_env *e, const cf_config *cfg)
{
    const int f = e->floor;
    for (int k = 0; k < CF_NSLOT; k++) {
        cf_mob *m = &e->mob[f][k];
        if (m->alive && imax(iabs((int)m->x - e->px), iabs((int)m->y - e->py)) > DESPAWN_DIST) kill_mob(e, k);
    }
    if (f == 8) {
        /* the necromancer can be hit again once its wave is gone */
        int alive = 0;
        for (int k = 0; k < S_PASSIVE0; k++) alive |= e->mob[f][k].alive;
        if (!e->boss_vulnerable && e->boss_hits < BOSS_HITS && !alive) { e->boss_vulnerable = 1; e->block[f][cell(24, 6)] = B_NECRO_VULN; }
        return;
    }
    const int first[3] = { S_MELEE0, S_RANGED0, S_PASSIVE0 }, count[3] = { 3, 2, 3 };
    const uint32_t caps[3] = { cfg->cap_melee, cfg->cap_ranged, cfg->cap_passive };
    const int type[3] = { MELEE_OF_FLOOR[f], RANGED_OF_FLOOR[f], PASSIVE_OF_FLOOR[f] };
    for (int j = 0; j < 3; j++) {
        int dx = (int)choice(cf_step_draw(e, (uint32_t)(3 * j), 3), 31) - 15;
        int dy = (int)choice(cf_step_draw(e, (uint32_t)(3 * j + 1), 3), 31) - 15;
        uint32_t rp = cf_step_draw(e, (uint32_t)(3 * j + 2), 3);
        int slot = free_slot(e, first[j], count[j], (int)caps[j]);
        int x = e->px + dx, y = e->py + dy;
        if (type[j] < 0 || slot < 0 || imax(iabs(dx), iabs(dy)) < SPAWN_MIN_DIST || !inb(x, y) || occupied(e, x, y)) continue;
        uint8_t b = e->block[f][cell(x, y)];
        uint32_t thr; int ok;
        if (f == 0) {          /* overworld as in Craftax-Classic: zombies on grass by darkness, skeletons on paths, cows on grass */
            thr = j == 0 ? zombie_threshold(cfg, e->t) : (j == 1 ? 0x19999999u : P_PASSIVE_SPAWN);
            ok = j == 1 ? b == B_PATH : b == B_GRASS;
        } else {
            thr = j == 0 ? P_MELEE_SPAWN : (j == 1 ? P_RANGED_SPAWN : P_PASSIVE_SPAWN);
            ok = passable_for(CREATURE[type[j]][7], b);
        }
        if (!ok || rp >= thr) continue;
        cf_mob *m = &e->mob[f][slot];
        m->alive = 1; m->x = (uint8_t)x; m->y = (uint8_t)y; m->dir = 0; m->type = (uint8_t)type[j]; m->hp = (int8_t)CREATURE[type[j]][0]; m->cd = 0;
    }
}

static void plants(cf_env *e)
{
    if (e->floor != 0) return;                   /* plants only grow while the player is in the overworld */
    for (int k = 0; k < CF_NPLANT; k++) {
        orc_plant *p = &e->plant[k];
        if (!p->alive) continue;
        int c = cell(p->x, p->y);
        if (p->age < 65535) p->age++;
        if (e->block[0][c] == B_PLANT && p->age >= RIPE_AGE) e->block[0][c] = B_RIPE;
        int near = 0;
        for (int z = 0; z < 3; z++) {
            const cf_mob *m = &e->mob[0][z];
            if (m->alive && iabs((int)m->x - p->x) + iabs((int)m->y - p->y) == 1) near = 1;
        }
        if (near && cf_step_draw(e, (uint32_t)k, 2) < P_PLANT_EATEN) { e->block[0][c] = B_GRASS; memset(p, 0, sizeof(*p)); }
    }
}

static void needs(cf_env *e, int damaged)
{
    const int asleep = e->sleeping, idle = e->sleeping || e->resting;
    e->cnt[K_HUNGER] += asleep ? 1 : 2;
    if (e->cnt[K_HUNGER] > 50) { e->cnt[K_HUNGER] = 0; e->vit[V_FOOD] = (int8_t)imax(0, e->vit[V_FOOD] - 1); }
    e->cnt[K_THIRST] += asleep ? 1 : 2;
    if (e->cnt[K_THIRST] > 40) { e->cnt[K_THIRST] = 0; e->vit[V_DRINK] = (int8_t)imax(0, e->vit[V_DRINK] - 1); }
    if (asleep) {
        e->cnt[K_FATIGUE]--;
        if (e->cnt[K_FATIGUE] < -10) { e->cnt[K_FATIGUE] = 0; e->vit[V_ENERGY] = (int8_t)imin(cap_need(e), e->vit[V_ENERGY] + 1); }
    } else {
        e->cnt[K_FATIGUE]++;
        if (e->cnt[K_FATIGUE] > 30) { e->cnt[K_FATIGUE] = 0; e->vit[V_ENERGY] = (int8_t)imax(0, e->vit[V_ENERGY] - 1); }
    }
    e->cnt[K_MANA] += e->intel;                   /* section "Attributes": intelligence feeds magic */
    if (e->cnt[K_MANA] > 20) { e->cnt[K_MANA] = 0; e->vit[V_MANA] = (int8_t)imin(cap_mana(e), e->vit[V_MANA] + 1); }
    if (e->vit[V_HEALTH] > 0) {
        int fed = e->vit[V_FOOD] > 0 && e->vit[V_DRINK] > 0 && (e->vit[V_ENERGY] > 0 || asleep);
        e->cnt[K_RECOVER] += fed ? (idle ? 4 : 2) : (idle ? -1 : -2);
        if (e->cnt[K_RECOVER] > 50) { e->cnt[K_RECOVER] = 0; e->vit[V_HEALTH] = (int8_t)imin(cap_health(e), e->vit[V_HEALTH] + 1); }
        if (e->cnt[K_RECOVER] < -30) { e->cnt[K_RECOVER] = 0; e->vit[V_HEALTH]--; }
    }
    if (asleep && (e->vit[V_ENERGY] >= cap_need(e) || damaged)) { e->sleeping = 0; unlock(e, ACH_WAKE_UP); }
    if (e->resting && (e->vit[V_HEALTH] >= cap_health(e) || damaged)) e->resting = 0;
}

void cf_step_rules(cf_env *e, const cf_config *cfg, int32_t action, float *reward, uint8_t *done)
{
    /* melee, passive, mob projectiles, player projectiles, then ranged: a shot first flies next step */
    static const int order[CF_NSLOT] = { 0, 1, 2, 5, 6, 7, 8, 9, 10, 11, 12, 13, 3, 4 };
    const int health0 = e->vit[V_HEALTH];
    const uint32_t ach0[3] = { e->ach[0], e->ach[1], e->ach[2] };
    int a = (action < 0 || action >= CF_NACT) ? A_NOOP : (int)action;
    if (e->sleeping || e->resting) a = A_NOOP;
    player_action(e, cfg, a);
    int damage = 0;
    for (int i = 0; i < CF_NSLOT; i++) mob_update(e, cfg, order[i], &damage);
    e->vit[V_HEALTH] = (int8_t)imax(0, e->vit[V_HEALTH] - damage);
    despawn_spawn(e, cfg);
    plants(e);
    needs(e, damage > 0);
    /* section "RL Environment Interface": category reward the first time, +-0.1 per health point */
    int gained = 0;
    for (int i = 0; i < CF_NACH; i++)
        if ((e->ach[i >> 5] >> (i & 31) & 1u) && !(ach0[i >> 5] >> (i & 31) & 1u)) gained += cf_achievement_reward(i);
    *reward = (float)(10 * gained + ((int)e->vit[V_HEALTH] - health0)) * 0.1f;
    e->t++;
    *done = (uint8_t)(e->vit[V_HEALTH] <= 0 || e->t >= cfg->max_episode_steps);
}
void cf_step(cf_env *e, const cf_config *cfg, int32_t action, float *reward, uint8_t *done)
{
    cf_step_rules(e, cfg, action, reward, done);
    if (*done) reset_episode(e, cfg, e->episode + 1);
}

/* ---- observation (appendix "Observation Space") -------------------------------------------------
 * 9 rows x 11 columns; per cell 37 block + 5 item + 40 creature channels (reading: 5 classes -
 * melee, passive, ranged, mob projectile, player projectile - of 8 type slots each) + light; a cell
 * whose light is 0 (< 0.05) is masked entirely.  Then 51 scalars.  99*83 + 51 = 8268. */
static int creature_channel(const cf_env *e, int k)
{
    const cf_mob *m = &e->mob[e->floor][k];
    int cls, slot;
    if (k < S_RANGED0) { cls = 0; slot = 0; for (int i = 0; i < 8; i++) if (MELEE_OF_FLOOR[i] == m->type) slot = i; }
    else if (k < S_PASSIVE0) { cls = 2; slot = 0; for (int i = 0; i < 8; i++) if (RANGED_OF_FLOOR[i] == m->type) slot = i; }
    else if (k < S_MPROJ0) { cls = 1; slot = m->type == C_COW ? 0 : (m->type == C_SNAIL ? 1 : 2); }
    else if (k < S_PPROJ0) { cls = 3; slot = CREATURE[m->type][2] > 0 ? (CREATURE[m->type][3] > 0 ? 3 : 1) : (CREATURE[m->type][3] > 0 ? 2 : 0); }
    else { cls = 4; slot = m->type; }
    return 42 + cls * 8 + slot;
}
static void scalars(const cf_env *e, const cf_config *cfg, float v[CF_NVEC])
{
    int i = 0;
    for (int k = 0; k < 10; k++) v[i++] = (float)(sqrt((double)e->inv[k]) / 10.0);
    for (int k = 0; k < 6; k++) v[i++] = (float)(sqrt((double)e->potion[k]) / 10.0);
    v[i++] = (float)((double)e->book / 2.0);
    v[i++] = (float)((double)e->pickaxe / 4.0);
    v[i++] = (float)((double)e->sword / 4.0);
    v[i++] = (float)e->sword_ench;
    v[i++] = (float)e->bow;
    v[i++] = (float)e->bow_ench;
    for (int k = 0; k < 4; k++) v[i++] = (float)((double)e->armour[k] / 2.0);
    for (int k = 0; k < 4; k++) v[i++] = (float)e->armour_ench[k];
    for (int k = 0; k < 5; k++) v[i++] = (float)((double)e->vit[k] / 10.0);
    v[i++] = (float)((double)e->xp / 10.0);
    v[i++] = (float)((double)e->dex / 10.0);
    v[i++] = (float)((double)e->str / 10.0);
    v[i++] = (float)((double)e->intel / 10.0);
    for (int d = 1; d <= 4; d++) v[i++] = e->dir == d ? 1.0f : 0.0f;
    v[i++] = daylight(cfg, e->t);
    v[i++] = (float)e->sleeping;
    v[i++] = (float)e->resting;
    v[i++] = (float)e->learned_fireball;
    v[i++] = (float)e->learned_iceball;
    v[i++] = (float)((double)e->floor / 10.0);
    v[i++] = (float)(e->floor == 0 || e->kills[e->floor] >= KILLS_TO_CLEAR);
    v[i++] = (float)e->boss_vulnerable;
}
/* ---- pixel observation (section "RL Environment Interface": 110 x 130 x 3 for Craftax, 10-pixel
 * tiles per appendix "Observation Space").  Reading (the paper's textures are not available): the
 * 9 x 11 view as tiles from a seeded atlas, then four rows of 11 inventory slots.
 *   view cell: texel of its block tile; an item, then a creature, then the player (centre cell)
 *   replace the pixels their 10x10 one-bit masks select; the result is multiplied by the cell's
 *   light level / 20 (one multiply); cells of light 0 are black; cells beyond the map edge show
 *   the tile of block 1 at full light.
 *   inventory slot j (0..43), row 9 + j/11, column j%11: icon tile j times min(scalar j of the
 *   symbolic observation, 1).
 * Atlas: texel = (u >> 8) * 2^-24, u = Philox word (key = atlas seed, counter (0, stream, 0,
 * ATLAS | idx/4), word idx%4); streams 8 block tiles [37][10][10][3], 9 item tiles [5], 10
 * creature tiles [40] (by observation channel - 42), 11 the player tile, 12 icon tiles [44],
 * 13 masks (top bit of word tile*100 + pixel; tiles: 5 items, 40 creatures, player). */
enum { DOM_ATLAS = 3 };
static float full_texel(uint64_t seed, uint32_t stream, uint32_t idx)
{
    uint32_t w = philox_word(seed, 0, stream, 0, DOM_ATLAS, idx >> 2, idx & 3u);
    return (float)(w >> 8) * (1.0f / 16777216.0f);
}
static int full_mask(uint64_t seed, uint32_t tile, uint32_t pixel)
{
    uint32_t idx = tile * 100u + pixel;
    return (int)(philox_word(seed, 0, 13, 0, DOM_ATLAS, idx >> 2, idx & 3u) >> 31);
}
static int creature_channel(const cf_env *e, int k);
static void scalars(const cf_env *e, const cf_config *cfg, float v[CF_NVEC]);
static void pixels(const cf_env *e, const cf_config *cfg, float *out)
{
    const int f = e->floor;
    const uint64_t seed = cfg->atlas_seed;
    float v[CF_NVEC];
    scalars(e, cfg, v);
    for (int y = 0; y < CF_PIX_ROWS; y++)
        for (int x = 0; x < CF_PIX_COLS; x++) {
            const int tr = y / 10, tc = x / 10, pix = (y % 10) * 10 + (x % 10);
            for (int c = 0; c < 3; c++) {
                const uint32_t in_tile = (uint32_t)(pix * 3 + c);
                float px;
                if (tr < CF_VIEW_ROWS) {
                    const int mx = e->px + tc - CF_VIEW_COLS / 2, my = e->py + tr - CF_VIEW_ROWS / 2;
                    int block = B_OOB, item = IT_NONE, light = MAX_LIGHT, k = -1;
                    if (inb(mx, my)) {
                        block = e->block[f][cell(mx, my)]; item = e->item[f][cell(mx, my)]; light = e->light[f][cell(mx, my)];
                        k = mob_at(e, mx, my);
                    }
                    float texel = full_texel(seed, 8, (uint32_t)block * 300u + in_tile);
                    if (item != IT_NONE && full_mask(seed, (uint32_t)item, (uint32_t)pix)) texel = full_texel(seed, 9, (uint32_t)item * 300u + in_tile);
                    if (k >= 0) {
                        const uint32_t ch = (uint32_t)creature_channel(e, k) - 42u;
                        if (full_mask(seed, 5u + ch, (uint32_t)pix)) texel = full_texel(seed, 10, ch * 300u + in_tile);
                    }
                    if (mx == e->px && my == e->py && full_mask(seed, 45u, (uint32_t)pix)) texel = full_texel(seed, 11, in_tile);
                    px = light == 0 ? 0.0f : texel * (float)((double)light / 20.0);
                } else {
                    const int j = (tr - CF_VIEW_ROWS) * 11 + tc;
                    px = full_texel(seed, 12, (uint32_t)j * 300u + in_tile) * (v[j] < 1.0f ? v[j] : 1.0f);
                }
                out[(y * CF_PIX_COLS + x) * 3 + c] = px;
            }
        }
}

void cf_observe(const cf_env *e, const cf_config *cfg, int mode, void *obs)
{
    uint8_t *o = (uint8_t *)obs;
    memset(o, 0, cf_obs_bytes(mode));
    if (mode == CF_OBS_PIXELS_F32) { pixels(e, cfg, (float *)obs); return; }
    uint8_t cells[CF_VIEW_ROWS * CF_VIEW_COLS][CF_NCHAN];
    memset(cells, 0, sizeof(cells));
    const int f = e->floor;
    for (int r = 0; r < CF_VIEW_ROWS; r++)
        for (int c = 0; c < CF_VIEW_COLS; c++) {
            int x = e->px + c - CF_VIEW_COLS / 2, y = e->py + r - CF_VIEW_ROWS / 2;
            uint8_t *ch = cells[r * CF_VIEW_COLS + c];
            if (!inb(x, y)) { ch[B_OOB] = 1; ch[37 + IT_NONE] = 1; ch[82] = MAX_LIGHT; continue; }   /* reading: the edge is always visible */
            int l = e->light[f][cell(x, y)];
            if (l == 0) continue;
            ch[e->block[f][cell(x, y)]] = 1;
            ch[37 + e->item[f][cell(x, y)]] = 1;
            int k = mob_at(e, x, y);
            if (k >= 0) ch[creature_channel(e, k)] = 1;
            ch[82] = (uint8_t)l;
        }
    float v[CF_NVEC];
    scalars(e, cfg, v);
    if (mode == CF_OBS_U8_F32) {
        memcpy(o, cells, sizeof(cells));                       /* 8217 bytes, light as its level 0..20 */
        memcpy(o + 8224, v, sizeof(v));
    } else {
        float *fo = (float *)obs;
        for (int i = 0; i < CF_VIEW_ROWS * CF_VIEW_COLS; i++)
            for (int c = 0; c < CF_NCHAN; c++)
                fo[i * CF_NCHAN + c] = c == 82 ? (float)((double)cells[i][c] / 20.0) : (float)cells[i][c];
        memcpy(fo + CF_VIEW_ROWS * CF_VIEW_COLS * CF_NCHAN, v, sizeof(v));
    }
}

void cf_reset_batch(cf_env *envs, const cf_config *cfg, const uint64_t *seeds, const uint32_t *env_ids, int n)
{
    for (int i = 0; i < n; i++) cf_reset(&envs[i], cfg, seeds[i], env_ids ? env_ids[i] : (uint32_t)i);
}
void cf_observe_batch(const cf_env *envs, const cf_config *cfg, int mode, void *obs, int n)
{
    size_t stride = cf_obs_bytes(mode);
    for (int i = 0; i < n; i++) cf_observe(&envs[i], cfg, mode, (uint8_t *)obs + stride * (size_t)i);
}
void cf_step_batch(cf_env *envs, const cf_config *cfg, const int32_t *actions, int mode, void *obs, float *reward, uint8_t *done, int n)
{
    size_t stride = cf_obs_bytes(mode);
    for (int i = 0; i < n; i++) {
        cf_step(&envs[i], cfg, actions[i], &reward[i], &done[i]);
        if (obs) cf_observe(&envs[i], cfg, mode, (uint8_t *)obs + stride * (size_t)i);
    }
}

/* Optimistic resets (appendix "Optimistic Environment Resets"), the reading of the Classic oracle
 * applied to the full game: all environments take the step's rules first; the r-th finished
 * environment (by environment number) then starts its next episode in pool world orc_pool_slot(seed
 * of environment 0, step index, r, n) -- all nine floors, the ladders and the potion map of world
 * (seed of environment 0, environment 2^31 + slot, episode = step index) -- while it keeps its own
 * seed and number and counts its episode up, so every later draw is its own. */
void cf_step_batch_pool(cf_env *envs, const cf_config *cfg, const int32_t *actions, int mode, void *obs, float *reward, uint8_t *done,
                        int n, uint32_t step_index)
{
    size_t stride = cf_obs_bytes(mode);
    uint64_t pool_seed = envs[0].seed;
    for (int i = 0; i < n; i++) cf_step_rules(&envs[i], cfg, actions[i], &reward[i], &done[i]);
    uint32_t rank = 0;
    for (int i = 0; i < n; i++) {
        if (!done[i]) continue;
        cf_env *e = &envs[i];
        uint32_t slot = orc_pool_slot(pool_seed, step_index, rank++, (uint32_t)n);
        uint64_t seed = e->seed;
        uint32_t env = e->env, episode = e->episode + 1;
        e->seed = pool_seed; e->env = 0x80000000u | slot;
        start_episode(e, cfg, step_index, NULL);
        e->seed = seed; e->env = env; e->episode = episode;
    }
    if (obs)
        for (int i = 0; i < n; i++) cf_observe(&envs[i], cfg, mode, (uint8_t *)obs + stride * (size_t)i);
}

/* ---- level mutations (section "Craftax-1B: UED": applied to the overworld) ----------------------
 * Same reading as for Classic, on floor 0: up to 32 tries, try k draws Philox block (env, round, 0,
 * MUTATE | k) under the mutation seed, word 0 the cell inside the central 16x16 area, word 1 any
 * cell; refused if the blocks are equal, a cell holds the player (when on floor 0), a live mob of
 * floor 0 or an item (ladder, torch), a block is a plant, or, restricted, the blocks are not of
 * one group (stone and the ores, gems included; grass and tree).  Returns the try + 1, or 0. */
static int swap_group(uint8_t b)
{
    if (b == B_STONE || b == B_COAL || b == B_IRON || b == B_DIAMOND || b == B_SAPPHIRE || b == B_RUBY) return 1;
    if (b == B_GRASS || b == B_TREE) return 2;
    return 0;
}
int cf_mutate_swap(cf_env *e, uint64_t mutation_seed, uint32_t round, int restricted)
{
    const int c0 = (CF_W - 16) / 2;
    for (uint32_t k = 0; k < 32; k++) {
        uint32_t a = choice(philox_word(mutation_seed, e->env, round, 0, DOM_MUTATE, k, 0), 256);
        uint32_t b = choice(philox_word(mutation_seed, e->env, round, 0, DOM_MUTATE, k, 1), CF_CELLS);
        int ax = c0 + (int)(a % 16), ay = c0 + (int)(a / 16), bx = (int)(b % CF_W), by = (int)(b / CF_W);
        uint8_t ba = e->block[0][cell(ax, ay)], bb = e->block[0][cell(bx, by)];
        if (ba == bb) continue;
        if (e->floor == 0 && ((e->px == ax && e->py == ay) || (e->px == bx && e->py == by))) continue;
        if (mob_at_floor(e, 0, ax, ay) >= 0 || mob_at_floor(e, 0, bx, by) >= 0) continue;
        if (e->item[0][cell(ax, ay)] != IT_NONE || e->item[0][cell(bx, by)] != IT_NONE) continue;
        if (ba == B_PLANT || ba == B_RIPE || bb == B_PLANT || bb == B_RIPE) continue;
        if (restricted && (swap_group(ba) == 0 || swap_group(ba) != swap_group(bb))) continue;
        e->block[0][cell(ax, ay)] = bb;
        e->block[0][cell(bx, by)] = ba;
        return (int)k + 1;
    }
    return 0;
}

/* Noise mutation (section "Craftax-1B: UED"), same reading as for Classic: the level is the vector
 * of the Perlin angles of every noise lattice of the world (theta_offset above gives the order);
 * element i gets a uniform integer offset in [-amplitude, amplitude] (1024ths of a turn) from u16
 * number i of Philox stream (env, round, 1, MUTATE) under the mutation seed; all nine floors of
 * the current episode are generated again from the new angles (the floors without noise come out
 * as they were) and the episode starts over.  Needs cfg->worldgen == PERLIN. */
void cf_mutate_noise(cf_env *e, const cf_config *cfg, uint16_t *theta, uint64_t mutation_seed, uint32_t round, uint32_t amplitude)
{
    for (uint32_t i = 0; i < CF_THETA_LEN; i++) {
        uint32_t w = philox_word(mutation_seed, e->env, round, 1, DOM_MUTATE, i >> 3, (i >> 1) & 3u);
        uint32_t d = (i & 1u) ? (w >> 16) : (w & 0xFFFFu);
        int32_t u = (int32_t)((d * (2u * amplitude + 1u)) >> 16) - (int32_t)amplitude;
        theta[i] = (uint16_t)(((int32_t)(theta[i] & 1023u) + u) & 1023);
    }
    start_episode(e, cfg, e->episode, theta);
}
