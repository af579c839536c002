// Full Craftax on the GPU: ids, constants of the rules, the in-HBM layout and the tables.
// One wavefront owns one environment: everything about the player is wave-uniform (kept in
// scalar registers), lane k < 14 owns mob slot k of the current floor, lane k < 10 plant k.
#pragma once

#include <cstddef>

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "common.hpp"
#include "lookahead.hpp"

namespace cf {

using cx::U4;
using cx::choice;
using cx::philox4x32_10;
using cx::iabs;
using cx::dir_dx;
using cx::dir_dy;

// ---- ids fixed by the paper (appendices "Block Types", "Action Space", "Achievements") ----
enum Block : int { B_INVALID = 0, B_OOB = 1, B_GRASS = 2, B_WATER = 3, B_STONE = 4, B_TREE = 5, B_WOOD = 6, B_PATH = 7,
                   B_COAL = 8, B_IRON = 9, B_DIAMOND = 10, B_TABLE = 11, B_FURNACE = 12, B_SAND = 13, B_LAVA = 14,
                   B_PLANT = 15, B_RIPE = 16, B_WALL = 17, B_DARKNESS = 18, B_WALL_MOSS = 19, B_STALAGMITE = 20,
                   B_SAPPHIRE = 21, B_RUBY = 22, B_CHEST = 23, B_FOUNTAIN = 24, B_FIRE_GRASS = 25, B_ICE_GRASS = 26,
                   B_GRAVEL = 27, B_FIRE_TREE = 28, B_ICE_SHRUB = 29, B_ENCH_FIRE = 30, B_ENCH_ICE = 31,
                   B_NECROMANCER = 32, B_GRAVE1 = 33, B_GRAVE2 = 34, B_GRAVE3 = 35, B_NECRO_VULN = 36, B_COUNT = 37 };
enum Item : int { IT_NONE = 0, IT_TORCH = 1, IT_LADDER_DOWN = 2, IT_LADDER_UP = 3, IT_LADDER_DOWN_BLOCKED = 4, IT_COUNT = 5 };
enum Action : int { A_NOOP = 0, A_LEFT, A_RIGHT, A_UP, A_DOWN, A_DO, A_SLEEP, A_PLACE_STONE, A_PLACE_TABLE,
                    A_PLACE_FURNACE, A_PLACE_PLANT, A_MAKE_WOOD_PICKAXE, A_MAKE_STONE_PICKAXE, A_MAKE_IRON_PICKAXE,
                    A_MAKE_WOOD_SWORD, A_MAKE_STONE_SWORD, A_MAKE_IRON_SWORD, A_REST, A_DESCEND, A_ASCEND,
                    A_MAKE_DIAMOND_PICKAXE, A_MAKE_DIAMOND_SWORD, A_MAKE_IRON_ARMOUR, A_MAKE_DIAMOND_ARMOUR,
                    A_SHOOT_ARROW, A_MAKE_ARROW, A_CAST_FIREBALL, A_CAST_ICEBALL, A_PLACE_TORCH, A_DRINK_POTION_RED,
                    A_DRINK_POTION_GREEN, A_DRINK_POTION_BLUE, A_DRINK_POTION_PINK, A_DRINK_POTION_CYAN,
                    A_DRINK_POTION_YELLOW, A_READ_BOOK, A_ENCHANT_SWORD, A_ENCHANT_ARMOUR, A_MAKE_TORCH,
                    A_LEVEL_UP_DEXTERITY, A_LEVEL_UP_STRENGTH, A_LEVEL_UP_INTELLIGENCE, A_ENCHANT_BOW, A_COUNT = 43 };
enum Ach : int { H_COLLECT_WOOD = 0, H_PLACE_TABLE, H_EAT_COW, H_COLLECT_SAPLING, H_COLLECT_DRINK, H_MAKE_WOOD_PICKAXE,
                 H_MAKE_WOOD_SWORD, H_PLACE_PLANT, H_DEFEAT_ZOMBIE, H_COLLECT_STONE, H_PLACE_STONE, H_EAT_PLANT,
                 H_DEFEAT_SKELETON, H_MAKE_STONE_PICKAXE, H_MAKE_STONE_SWORD, H_WAKE_UP, H_PLACE_FURNACE, H_COLLECT_COAL,
                 H_COLLECT_IRON, H_COLLECT_DIAMOND, H_MAKE_IRON_PICKAXE, H_MAKE_IRON_SWORD, H_MAKE_ARROW, H_MAKE_TORCH,
                 H_PLACE_TORCH, H_MAKE_DIAMOND_SWORD, H_MAKE_IRON_ARMOUR, H_MAKE_DIAMOND_ARMOUR, H_ENTER_GNOMISH_MINES,
                 H_ENTER_DUNGEON, H_ENTER_SEWERS, H_ENTER_VAULT, H_ENTER_TROLL_MINES, H_ENTER_FIRE_REALM,
                 H_ENTER_ICE_REALM, H_ENTER_GRAVEYARD, H_DEFEAT_GNOME_WARRIOR, H_DEFEAT_GNOME_ARCHER,
                 H_DEFEAT_ORC_SOLIDER, H_DEFEAT_ORC_MAGE, H_DEFEAT_LIZARD, H_DEFEAT_KOBOLD, H_DEFEAT_TROLL,
                 H_DEFEAT_DEEP_THING, H_DEFEAT_PIGMAN, H_DEFEAT_FIRE_ELEMENTAL, H_DEFEAT_FROST_TROLL,
                 H_DEFEAT_ICE_ELEMENTAL, H_DAMAGE_NECROMANCER, H_DEFEAT_NECROMANCER, H_EAT_BAT, H_EAT_SNAIL, H_FIND_BOW,
                 H_FIRE_BOW, H_COLLECT_SAPPHIRE, H_LEARN_FIREBALL, H_CAST_FIREBALL, H_LEARN_ICEBALL, H_CAST_ICEBALL,
                 H_COLLECT_RUBY, H_MAKE_DIAMOND_PICKAXE, H_OPEN_CHEST, H_DRINK_POTION, H_ENCHANT_SWORD, H_ENCHANT_ARMOUR,
                 H_DEFEAT_KNIGHT, H_DEFEAT_ARCHER, H_COUNT = 67 };
// Reward categories of appendix "Achievements" (1, 3, 5 or 8 points) as bit masks over the
// three achievement words: ids 0..24 are worth 1; 25..29, 36..39, 50..54, 59..62 are worth 3;
// 30..32, 40..43, 55..58, 63..66 are worth 5; 33..35, 44..49 are worth 8.
constexpr uint32_t CAT1[3] = { 0x01FFFFFFu, 0x00000000u, 0x0u };
constexpr uint32_t CAT3[3] = { 0x3E000000u, 0x787C00F0u, 0x0u };
constexpr uint32_t CAT5[3] = { 0xC0000000u, 0x87800F01u, 0x7u };
constexpr uint32_t CAT8[3] = { 0x00000000u, 0x0003F00Eu, 0x0u };

enum Creature : int { C_ZOMBIE = 0, C_SKELETON, C_COW, C_ORC_SOLDIER, C_ORC_MAGE, C_SNAIL, C_GNOME_WARRIOR,
                      C_GNOME_ARCHER, C_BAT, C_LIZARD, C_KOBOLD, C_KNIGHT, C_ARCHER, C_TROLL, C_DEEP_THING, C_PIGMAN,
                      C_FIRE_ELEMENTAL, C_FROST_TROLL, C_ICE_ELEMENTAL, C_COUNT = 19 };
enum Collision : int { COL_GROUND = 0, COL_FLYING = 1, COL_AMPHIBIAN = 2, COL_AQUATIC = 3 };
enum InvItem : int { I_WOOD = 0, I_STONE, I_COAL, I_IRON, I_DIAMOND, I_SAPPHIRE, I_RUBY, I_SAPLING, I_TORCH, I_ARROW };
enum Vital : int { V_HEALTH = 0, V_FOOD, V_DRINK, V_ENERGY, V_MANA };
enum Counter : int { K_HUNGER = 0, K_THIRST, K_FATIGUE, K_RECOVER, K_MANA };
enum Slot : int { S_MELEE0 = 0, S_RANGED0 = 3, S_PASSIVE0 = 5, S_MPROJ0 = 8, S_PPROJ0 = 11, NSLOT = 14 };
enum Shot : int { PP_ARROW = 0, PP_FIREBALL = 1, PP_ICEBALL = 2 };

// ---- sizes ------------------------------------------------------------------------------------
constexpr int FLOORS = 9, W = 48, CELLS = W * W, NPLANT = 10;
constexpr int VROWS = 9, VCOLS = 11, NCELL = VROWS * VCOLS, NCHAN = 83, NVEC = 51;
constexpr int CELL_BYTES = NCELL * NCHAN;        // 8217
constexpr int VEC_OFFSET = 8224;                 // float[51] of the byte layout
constexpr int STRIDE_U8 = 8448;                  // 66 cache lines
constexpr int STRIDE_F32 = 33152;                // float[8268] padded to 259 cache lines
constexpr int MAX_DAY = cx::MAX_DAY;

// ---- constants of the rules (this library's frozen reading; the paper prints only the
// creature table and the achievement table) ----
constexpr int INV_MAX = 99, CD_MELEE = 5, CD_RANGED = 4, CHASE_RANGE = 8, SHOOT_RANGE = 4, DESPAWN_DIST = 15,
              SPAWN_MIN_DIST = 5, RIPE_AGE = 300, FOOD_MEAT = 6, FOOD_PLANT = 4, KILLS_TO_CLEAR = 8, BOSS_HITS = 8,
              MAX_LIGHT = 20, BOSS_X = 24, BOSS_Y = 6;
constexpr uint32_t P_SAPLING = 429496730u, P_CHASE = 3435973836u, P_SHOOT = 0x80000000u, P_PLANT_EATEN = 0x20000000u,
                   P_PASSIVE_SPAWN = 0x08000000u, P_RANGED_SPAWN = 0x0CCCCCCCu, P_MELEE_SPAWN = 0x0CCCCCCCu,
                   P_SKELETON_SPAWN = 0x19999999u;

// Creature table (appendix "Creatures"): health, damage physical/fire/ice, defence % physical/
// fire/ice, collision type, achievement for defeating (eating) it.  The rows are written out once,
// here; the device reads them from 64-bit constants packed at compile time (creature(type) is a few
// shifts), not from memory: a lookup in memory sat in the middle of every step's chain of
// dependent round trips.
struct CreatureRow { int hp, dp, df, di; int Dp, Df, Di; int col; int ach; };
constexpr int N_CREATURE = 19;
constexpr CreatureRow CREATURE_ROWS[N_CREATURE] = {
    { 5, 2, 0, 0, 0, 0, 0, COL_GROUND, H_DEFEAT_ZOMBIE },          { 3, 2, 0, 0, 0, 0, 0, COL_GROUND, H_DEFEAT_SKELETON },
    { 3, 0, 0, 0, 0, 0, 0, COL_GROUND, H_EAT_COW },                { 7, 3, 0, 0, 0, 0, 0, COL_GROUND, H_DEFEAT_ORC_SOLIDER },
    { 5, 3, 0, 0, 0, 0, 0, COL_GROUND, H_DEFEAT_ORC_MAGE },        { 6, 0, 0, 0, 0, 0, 0, COL_GROUND, H_EAT_SNAIL },
    { 9, 4, 0, 0, 0, 0, 0, COL_GROUND, H_DEFEAT_GNOME_WARRIOR },   { 6, 2, 0, 0, 0, 0, 0, COL_GROUND, H_DEFEAT_GNOME_ARCHER },
    { 4, 0, 0, 0, 0, 0, 0, COL_FLYING, H_EAT_BAT },                { 11, 5, 0, 0, 0, 0, 0, COL_AMPHIBIAN, H_DEFEAT_LIZARD },
    { 8, 4, 0, 0, 0, 0, 0, COL_GROUND, H_DEFEAT_KOBOLD },          { 12, 6, 0, 0, 50, 0, 0, COL_GROUND, H_DEFEAT_KNIGHT },
    { 12, 4, 0, 0, 50, 0, 0, COL_GROUND, H_DEFEAT_ARCHER },        { 20, 6, 1, 1, 20, 0, 0, COL_GROUND, H_DEFEAT_TROLL },
    { 6, 4, 3, 3, 0, 0, 0, COL_AQUATIC, H_DEFEAT_DEEP_THING },     { 20, 3, 5, 0, 90, 100, 0, COL_GROUND, H_DEFEAT_PIGMAN },
    { 14, 3, 5, 0, 90, 100, 0, COL_FLYING, H_DEFEAT_FIRE_ELEMENTAL }, { 24, 4, 0, 5, 90, 0, 100, COL_GROUND, H_DEFEAT_FROST_TROLL },
    { 16, 4, 0, 4, 90, 0, 100, COL_FLYING, H_DEFEAT_ICE_ELEMENTAL },
};
// field f of a row: 0 hp, 1..3 damage, 4 physical defence as a code (0, 20, 50, 90 -> 0..3), 5 and 6 fire
// and ice defence as a flag (0 or 100), 7 collision, 8 achievement
constexpr int creature_field(const CreatureRow& r, int f)
{
    return f == 0 ? r.hp : f == 1 ? r.dp : f == 2 ? r.df : f == 3 ? r.di
         : f == 4 ? (r.Dp == 0 ? 0 : r.Dp == 20 ? 1 : r.Dp == 50 ? 2 : 3) : f == 5 ? (r.Df != 0) : f == 6 ? (r.Di != 0) : f == 7 ? r.col : r.ach;
}
// `count` values of `bits` bits each, from row `first` on
constexpr uint64_t pack_creatures(int f, int bits, int first, int count)
{
    uint64_t v = 0;
    for (int i = 0; i < count && first + i < N_CREATURE; ++i) v |= (uint64_t)creature_field(CREATURE_ROWS[first + i], f) << (bits * i);
    return v;
}
constexpr uint64_t CR_HP[2] = { pack_creatures(0, 5, 0, 12), pack_creatures(0, 5, 12, 12) };
constexpr uint64_t CR_DP = pack_creatures(1, 3, 0, 19), CR_DF = pack_creatures(2, 3, 0, 19), CR_DI = pack_creatures(3, 3, 0, 19);
constexpr uint64_t CR_DEFP = pack_creatures(4, 2, 0, 19), CR_DEFF = pack_creatures(5, 1, 0, 19), CR_DEFI = pack_creatures(6, 1, 0, 19);
constexpr uint64_t CR_COL = pack_creatures(7, 2, 0, 19);
constexpr uint64_t CR_ACH[3] = { pack_creatures(8, 7, 0, 9), pack_creatures(8, 7, 9, 9), pack_creatures(8, 7, 18, 9) };
__host__ __device__ constexpr CreatureRow creature(int type)
{
    const int t = type < N_CREATURE ? type : N_CREATURE - 1;      // a mob word has five bits of type; rows end at 18
    CreatureRow c{};
    c.hp = (int)((t < 12 ? CR_HP[0] >> (5 * t) : CR_HP[1] >> (5 * (t - 12))) & 31u);
    c.dp = (int)((CR_DP >> (3 * t)) & 7u); c.df = (int)((CR_DF >> (3 * t)) & 7u); c.di = (int)((CR_DI >> (3 * t)) & 7u);
    c.Dp = (int)((0x5A321400u >> (8 * (int)((CR_DEFP >> (2 * t)) & 3u))) & 0xFFu);
    c.Df = 100 * (int)((CR_DEFF >> t) & 1u); c.Di = 100 * (int)((CR_DEFI >> t) & 1u);
    c.col = (int)((CR_COL >> (2 * t)) & 3u);
    c.ach = (int)((t < 9 ? CR_ACH[0] >> (7 * t) : t < 18 ? CR_ACH[1] >> (7 * (t - 9)) : CR_ACH[2] >> (7 * (t - 18))) & 127u);
    return c;
}
constexpr bool creature_table_round_trips()
{
    for (int t = 0; t < N_CREATURE; ++t) {
        const CreatureRow a = CREATURE_ROWS[t], b = creature(t);
        if (a.hp != b.hp || a.dp != b.dp || a.df != b.df || a.di != b.di || a.Dp != b.Dp || a.Df != b.Df || a.Di != b.Di || a.col != b.col || a.ach != b.ach)
            return false;
    }
    return true;
}
static_assert(creature_table_round_trips(), "the packed creature table does not decode to its rows");

// Small per-floor and per-type tables, packed the same way (five bits per entry, 31 = none).
template <int N>
constexpr uint64_t pack5(const int (&a)[N])
{
    uint64_t v = 0;
    for (int i = 0; i < N; ++i) v |= (uint64_t)(a[i] < 0 ? 31 : a[i]) << (5 * i);
    return v;
}
constexpr int unpack5(uint64_t packed, int i) { const int v = (int)((packed >> (5 * i)) & 31u); return v == 31 ? -1 : v; }
// who lives on which floor (appendix "Creatures", column Floor); the boss floor calls them as waves
constexpr int MELEE_ROWS[8] = { C_ZOMBIE, C_ORC_SOLDIER, C_GNOME_WARRIOR, C_LIZARD, C_KNIGHT, C_TROLL, C_PIGMAN, C_FROST_TROLL };
constexpr int RANGED_ROWS[8] = { C_SKELETON, C_ORC_MAGE, C_GNOME_ARCHER, C_KOBOLD, C_ARCHER, C_DEEP_THING, C_FIRE_ELEMENTAL, C_ICE_ELEMENTAL };
constexpr int PASSIVE_ROWS[8] = { C_COW, C_SNAIL, C_BAT, C_SNAIL, C_SNAIL, C_BAT, C_BAT, -1 };
__host__ __device__ constexpr int melee_of_floor(int f) { return unpack5(pack5(MELEE_ROWS), f); }
__host__ __device__ constexpr int ranged_of_floor(int f) { return unpack5(pack5(RANGED_ROWS), f); }
__host__ __device__ constexpr int passive_of_floor(int f) { return unpack5(pack5(PASSIVE_ROWS), f); }
static_assert(melee_of_floor(3) == C_LIZARD && ranged_of_floor(7) == C_ICE_ELEMENTAL && passive_of_floor(7) == -1 && passive_of_floor(2) == C_BAT, "floor tables");
// achievement for entering floor f (seven bits per entry, 127 = none)
constexpr int ENTER_ROWS[FLOORS] = { -1, H_ENTER_DUNGEON, H_ENTER_GNOMISH_MINES, H_ENTER_SEWERS, H_ENTER_VAULT,
                                     H_ENTER_TROLL_MINES, H_ENTER_FIRE_REALM, H_ENTER_ICE_REALM, H_ENTER_GRAVEYARD };
constexpr uint64_t pack_enter()
{
    uint64_t v = 0;
    for (int i = 0; i < FLOORS; ++i) v |= (uint64_t)(ENTER_ROWS[i] < 0 ? 127 : ENTER_ROWS[i]) << (7 * i);
    return v;
}
__host__ __device__ constexpr int enter_ach(int f) { const int v = (int)((pack_enter() >> (7 * f)) & 127u); return v == 127 ? -1 : v; }
static_assert(enter_ach(0) == -1 && enter_ach(8) == H_ENTER_GRAVEYARD && enter_ach(4) == H_ENTER_VAULT, "floor achievements");
// Observation channel (42..81) of a creature by slot class: 8 type slots per class, classes in
// the order melee, passive, ranged, mob projectile, player projectile.  The type slot of a melee or
// ranged creature is the floor it lives on.
constexpr int type_slot_of(const int (&rows)[8], int type)
{
    for (int f = 0; f < 8; ++f) if (rows[f] == type) return f;
    return 0;
}
constexpr uint64_t pack_type_slots(const int (&rows)[8])
{
    uint64_t v = 0;
    for (int t = 0; t < N_CREATURE; ++t) v |= (uint64_t)type_slot_of(rows, t) << (3 * t);
    return v;
}
__host__ __device__ constexpr int melee_type_slot(int type) { return (int)((pack_type_slots(MELEE_ROWS) >> (3 * (type < N_CREATURE ? type : 0))) & 7u); }
__host__ __device__ constexpr int ranged_type_slot(int type) { return (int)((pack_type_slots(RANGED_ROWS) >> (3 * (type < N_CREATURE ? type : 0))) & 7u); }
static_assert(melee_type_slot(C_KNIGHT) == 4 && melee_type_slot(C_FROST_TROLL) == 7 && ranged_type_slot(C_ORC_MAGE) == 1 && ranged_type_slot(C_SKELETON) == 0, "type slots");

__device__ inline bool lit_floor(int f) { return (0x05Bu >> f) & 1u; }    // floors 0, 1, 3, 4, 6; dark: 2, 5, 7, 8

// block-id sets as 64-bit masks
constexpr uint64_t bit(int b) { return 1ull << b; }
constexpr uint64_t WALKABLE = bit(B_GRASS) | bit(B_SAND) | bit(B_PATH) | bit(B_FIRE_GRASS) | bit(B_ICE_GRASS) | bit(B_GRAVEL);
constexpr uint64_t FLYABLE = WALKABLE | bit(B_WATER) | bit(B_LAVA);
constexpr uint64_t AMPHIBIAN_OK = WALKABLE | bit(B_WATER);
__device__ inline bool in_set(uint64_t set, int b) { return (set >> b) & 1ull; }
__device__ inline bool passable_for(int col, int b)
{
    const uint64_t set = col == COL_GROUND ? WALKABLE : (col == COL_FLYING ? FLYABLE : (col == COL_AMPHIBIAN ? AMPHIBIAN_OK : bit(B_WATER)));
    return in_set(set, b);
}
__device__ inline bool inb(int x, int y) { return ((unsigned)x < (unsigned)W) & ((unsigned)y < (unsigned)W); }

// ---- in-HBM layout ----------------------------------------------------------------------------
// Per environment: a 1024-byte block = a 64-dword record, nine 16-dword mob tables (one 64-byte
// table per floor, slots 0..13 used) and, from dword 208 on, the ladders and the potion map of
// the world waiting in the spare map slot; and two map slots (the world of episode e in slot
// e & 1, the world of episode e + 1 in the other) of 9 floors x (block map 2304 B + item/light
// map 2304 B), row-major 48-byte rows.  The second map holds item | light << 3 per cell.
//   r0  px | py<<8 | dir<<16 | floor<<24
//   r1  sleeping | resting<<1 | fireball<<2 | iceball<<3 | book<<4 | pickaxe<<6 | sword<<9 | sword_ench<<12 |
//       bow<<14 | bow_ench<<15 | boss_vulnerable<<17 | boss_hits<<18
//   r2  armour 4x2 bits | armour_ench 4x2 bits <<8 | xp<<16 | dex<<20 | str<<23 | int<<26
//   r3..r5  inventory bytes (wood stone coal iron | diamond sapphire ruby sapling | torch arrow potion0 potion1)
//   r6  potion 2..5 bytes      r7  health food drink energy bytes
//   r8  mana | mana counter<<8 (signed byte) | day phase<<16
//   r9  hunger thirst fatigue recover counters (signed bytes)
//   r10 potion colour->effect map 6x3 bits | visited floors<<18
//   r11..r13 kills per floor (bytes)       r14..r22 ladders of floor f: up x | up y<<8 | down x<<16 | down y<<24
//   r23..r25 achievement bits   r26 t   r27 episode   r28,r29 seed   r32..r41 plant slots
// mob word:   alive | x<<1 | y<<7 | dir<<13 | hp<<16 | cd<<21 | type<<25      (0 when the slot is empty)
// plant word: alive | x<<1 | y<<7 | age<<16
constexpr int ENV_DWORDS = 256, REC_DWORDS = 64, MOBTAB_DWORDS = 16;
constexpr int SPARE_LADDER = 208, SPARE_PERM = 217;   // dwords of the environment block describing the spare world
constexpr int NTAG = 9;                               // spare-world tags per environment: one per floor
constexpr int R_POS = 0, R_FLAGS = 1, R_ATTR = 2, R_INV = 3, R_POT = 6, R_VIT = 7, R_MANA = 8, R_CNT = 9, R_PERM = 10,
              R_KILLS = 11, R_LADDER = 14, R_ACH = 23, R_T = 26, R_EPISODE = 27, R_SEED_LO = 28, R_SEED_HI = 29, R_PLANT = 32;
constexpr size_t MAP_BYTES = (size_t)FLOORS * 2 * CELLS;          // 41472 per map slot
__host__ __device__ inline size_t map_offset(uint32_t env, uint32_t episode) { return ((size_t)env * 2 + (episode & 1u)) * MAP_BYTES; }
__device__ inline size_t block_off(int f, int x, int y)
{
    f = CX_IDX(f, FLOORS); x = CX_IDX(x, W); y = CX_IDX(y, W);
    return (size_t)f * (2 * CELLS) + (size_t)(y * W + x);
}
__device__ inline size_t il_off(int f, int x, int y)
{
    f = CX_IDX(f, FLOORS); x = CX_IDX(x, W); y = CX_IDX(y, W);
    return (size_t)f * (2 * CELLS) + CELLS + (size_t)(y * W + x);
}

struct Mob { int alive, x, y, dir, hp, cd, type; };
__host__ __device__ inline Mob unpack_mob(uint32_t w)
{
    Mob m;
    m.alive = w & 1u; m.x = (w >> 1) & 63u; m.y = (w >> 7) & 63u; m.dir = (w >> 13) & 7u;
    m.hp = (w >> 16) & 31u; m.cd = (w >> 21) & 15u; m.type = (w >> 25) & 31u;
    return m;
}
__host__ __device__ inline uint32_t pack_mob(const Mob& m)
{
    return m.alive ? (1u | ((uint32_t)m.x << 1) | ((uint32_t)m.y << 7) | ((uint32_t)m.dir << 13) | ((uint32_t)m.hp << 16) |
                      ((uint32_t)m.cd << 21) | ((uint32_t)m.type << 25)) : 0u;
}

struct Luts {
    float daylight[MAX_DAY];        // smoothstep day/night curve, index t mod day_length
    uint32_t zombie_thr[MAX_DAY];   // zombie spawn threshold per phase
    float sqrt10[100];              // sqrt(n)/10
    float tenth[32];                // x/10
    float light20[32];              // light level / 20
    // pixel observations: 10x10 RGB tiles, texel = (Philox word >> 8) * 2^-24 keyed by the atlas
    // seed.  Tiles 0..36 blocks, 37..41 items, 42..81 creatures (observation channel - 42), 82
    // the player, 83..126 inventory icons.  mask[t][row] bit x: overlay t covers that pixel
    // (t: 0..4 items, 5..44 creatures, 45 the player).
    float atlas[127 * 300];
    uint16_t mask[46][10];
    uint32_t perlin_cs[1024];       // unit gradient of direction a: cos (low half) and sin (high half) in Q14, as int16
};
static_assert(offsetof(Luts, tenth) == offsetof(Luts, sqrt10) + 400 && offsetof(Luts, light20) == offsetof(Luts, tenth) + 128,
              "sqrt10, tenth and light20 are copied to LDS as one run of floats");
constexpr int AT_ITEM = 37, AT_CRE = 42, AT_PLAYER = 82, AT_ICON = 83, AT_TILES = 127;
constexpr int MASK_CRE = 5, MASK_PLAYER = 45;

struct Header {
    uint64_t magic;
    uint32_t version, n;
    uint32_t variant, obs_mode, max_episode_steps, day_length;
    uint32_t cap_melee, cap_ranged, cap_passive, cap_plant;
    uint64_t off_ctrs, off_luts, off_envs, off_maps, off_tags, off_regen0, off_regen1, off_slow, off_unlocks, total;
    uint64_t atlas_seed;
    uint32_t worldgen, reset_mode;
};
static_assert(sizeof(Header) <= cx::HEADER_BYTES, "header outgrew its area");
constexpr uint64_t MAGIC = 0x46554C4C43524158ull;

struct Params {
    int n;
    uint32_t max_episode_steps, day_length;
    uint32_t cap_melee, cap_ranged, cap_passive, cap_plant;
    uint32_t worldgen;              // CRAFTAX_WORLDGEN_*
    uint32_t* unlocks;              // UNLOCK_STRIDE counters per environment (see count_unlocks); null in kernels that do not step
};

// Unlock counters (the paper reports achievement success rates, section "Craftax-1B"): counts[k] =
// how often achievement k has been unlocked in this environment since craftax_reset; an
// achievement unlocks at most once per episode, so the sum over the environments, less the
// running episodes that hold it, is the number of finished episodes that reached it.  Counted in
// the step, from the bits of achievement word w that are new after it; lane l of the environment's
// group takes bits l, l + GW, ...; the adds return nothing, so no wavefront waits for them.
constexpr int UNLOCK_STRIDE = 72;   // dwords per environment: 67 achievements, padded to 288 bytes
template <int GW>
__device__ __forceinline__ void count_unlocks(int l, uint32_t* __restrict__ counts, int w, uint32_t unlocked)
{
    if (unlocked == 0u) return;
#pragma unroll
    for (int b0 = 0; b0 < 32; b0 += GW) {
        const int b = b0 + l;
        if (b < 32 && 32 * w + b < H_COUNT && ((unlocked >> b) & 1u)) atomicAdd(counts + 32 * w + b, 1u);
    }
}

// ---- per-environment LDS area (dword offsets) ----------------------------------------------------
// Window: 11 rows x 13 columns (pitch 16 bytes) of the block map and of the item/light map
// around the player's position at load time, one cell of margin on every side of the 9x11 view
// so that a move of one cell needs no reload.  Cells outside the map read B_OOB / light 20.
constexpr int WIN_ROWS = 11, WIN_COLS = 13, WIN_PITCH = 16;
constexpr int L_REC = 0;                         // 64 dwords
constexpr int L_WB = 64;                         // 44 dwords: block window
constexpr int L_WI = 108;                        // 44 dwords: item/light window
constexpr int L_CRE = 152;                       // 100 dwords: creature channel per view cell
constexpr int L_BITS = 252;                      // 260 dwords: one bit per cell byte of the observation (8217 bits)
constexpr int L_LIGHT = 512;                     // 28 dwords: light level per view cell (bytes)
constexpr int L_VEC = 540;                       // 52 dwords: the 51 scalars and a zero
constexpr int L_SPARE_WB = 592;                  // 44 dwords: block window of the start position of the spare world
constexpr int L_SPARE_WI = 636;                  // 44 dwords: its item/light window
constexpr int L_SPARE_TAG = 680;                 // 54 dwords reserved; the 9 (episode, launch) tags of the spare world use 18
constexpr int L_SPARE_HDR = 734;                 // 10 dwords: ladders and potion map of the spare world
constexpr int L_ENV_DWORDS = 744;
constexpr int ENVS_PER_BLOCK = 4, BLOCK = 256;

__device__ inline void wave_sync()
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}
// wave-uniform value held in a scalar register
__device__ inline int uni(int v) { return __builtin_amdgcn_readfirstlane(v); }
__device__ inline uint32_t uniu(uint32_t v) { return (uint32_t)__builtin_amdgcn_readfirstlane((int)v); }
__device__ inline int lane_get(int v, int lane) { return __builtin_amdgcn_readlane(v, lane); }

// An environment is stepped by GW consecutive lanes of a wavefront: the whole wavefront (GW = 64:
// the player's state lives in scalar registers and the 43-action code runs on the scalar unit), or
// a group of 16 lanes, four environments per wavefront (GW = 16: the player's state is a vector
// register per value, equal in the lanes of a group; the action code runs once per wavefront for
// four environments, and the 14 mob slots fill 14 of 16 lanes instead of 14 of 64).  The step and
// the renderer are written once against these primitives; `lane` below is a lane of the group.
template <int GW> struct Lanes;
template <> struct Lanes<64> {
    __device__ static inline int uni(int v) { return __builtin_amdgcn_readfirstlane(v); }
    __device__ static inline uint32_t uniu(uint32_t v) { return (uint32_t)__builtin_amdgcn_readfirstlane((int)v); }
    __device__ static inline int get(int v, int lane) { return __builtin_amdgcn_readlane(v, lane); }
    __device__ static inline uint32_t ballot(bool pred) { return (uint32_t)__ballot(pred); }      // bit i = lane i, i < 32
};
template <> struct Lanes<16> {
    __device__ static inline int uni(int v) { return v; }
    __device__ static inline uint32_t uniu(uint32_t v) { return v; }
    // value of lane `lane` of the calling lane's group (every lane of the group must be active)
    __device__ static inline int get(int v, int lane) { return __shfl(v, (int)(threadIdx.x & 48u) | lane, 64); }
    // bit i = predicate of lane i of the calling lane's group
    __device__ static inline uint32_t ballot(bool pred)
    {
        const uint64_t m = __ballot(pred);
        const uint32_t lane = threadIdx.x & 63u;
        const uint32_t half = (lane & 32u) ? (uint32_t)(m >> 32) : (uint32_t)m;
        return __builtin_amdgcn_ubfe(half, lane & 16u, 16u);
    }
};

}  // namespace cf
