// Shared definitions of the GPU simulator: ids, constants of the rules, the in-HBM record
// layout, Philox, and the lane-group primitives.  gfx950 only.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace cx {

// ---- ids fixed by the paper (appendices "Block Types", "Action Space", "Achievements") ----
enum Block : int { BK_INVALID = 0, BK_OOB = 1, BK_GRASS = 2, BK_WATER = 3, BK_STONE = 4, BK_TREE = 5,
                   BK_WOOD = 6, BK_PATH = 7, BK_COAL = 8, BK_IRON = 9, BK_DIAMOND = 10, BK_TABLE = 11,
                   BK_FURNACE = 12, BK_SAND = 13, BK_LAVA = 14, BK_PLANT = 15, BK_RIPE = 16 };
enum Action : int { AC_NOOP = 0, AC_LEFT = 1, AC_RIGHT = 2, AC_UP = 3, AC_DOWN = 4, AC_DO = 5, AC_SLEEP = 6,
                    AC_PLACE_STONE = 7, AC_PLACE_TABLE = 8, AC_PLACE_FURNACE = 9, AC_PLACE_PLANT = 10,
                    AC_MAKE_WOOD_PICKAXE = 11, AC_MAKE_STONE_PICKAXE = 12, AC_MAKE_IRON_PICKAXE = 13,
                    AC_MAKE_WOOD_SWORD = 14, AC_MAKE_STONE_SWORD = 15, AC_MAKE_IRON_SWORD = 16, AC_COUNT = 17 };
enum Ach : int { ACH_COLLECT_WOOD = 0, ACH_PLACE_TABLE = 1, ACH_EAT_COW = 2, ACH_COLLECT_SAPLING = 3,
                 ACH_COLLECT_DRINK = 4, ACH_MAKE_WOOD_PICKAXE = 5, ACH_MAKE_WOOD_SWORD = 6, ACH_PLACE_PLANT = 7,
                 ACH_DEFEAT_ZOMBIE = 8, ACH_COLLECT_STONE = 9, ACH_PLACE_STONE = 10, ACH_EAT_PLANT = 11,
                 ACH_DEFEAT_SKELETON = 12, ACH_MAKE_STONE_PICKAXE = 13, ACH_MAKE_STONE_SWORD = 14, ACH_WAKE_UP = 15,
                 ACH_PLACE_FURNACE = 16, ACH_COLLECT_COAL = 17, ACH_COLLECT_IRON = 18, ACH_COLLECT_DIAMOND = 19,
                 ACH_MAKE_IRON_PICKAXE = 20, ACH_MAKE_IRON_SWORD = 21 };
enum Inv : int { IV_WOOD = 0, IV_STONE, IV_COAL, IV_IRON, IV_DIAMOND, IV_SAPLING, IV_WOOD_PICKAXE, IV_STONE_PICKAXE,
                 IV_IRON_PICKAXE, IV_WOOD_SWORD, IV_STONE_SWORD, IV_IRON_SWORD };
enum MobType : int { MT_ZOMBIE = 0, MT_COW = 1, MT_SKELETON = 2, MT_ARROW = 3 };

// ---- constants of the rules (the paper prints creature health/damage in appendix
// "Creatures"; everything else is this library's own frozen reading of "mimic Crafter") ----
constexpr int MAPW = 64;
constexpr int NMOB = 12;          // slots 0-2 zombie, 3-5 cow, 6-8 skeleton, 9-11 arrow
constexpr int NPLANT = 10;
constexpr int MAX_COUNT = 9;
constexpr int HP_ZOMBIE = 5, HP_COW = 3, HP_SKELETON = 3;
constexpr int DMG_ZOMBIE = 2, DMG_ZOMBIE_SLEEP = 7, DMG_ARROW = 2;
constexpr int CD_ZOMBIE = 5, CD_SKELETON = 4;
constexpr int CHASE_RANGE = 8, SHOOT_RANGE = 4, DESPAWN_DIST = 15, SPAWN_MIN_DIST = 5;
constexpr int RIPE_AGE = 300;
constexpr int FOOD_COW = 6, FOOD_PLANT = 4;
constexpr uint32_t P_SAPLING = 429496730u;        // 10 %
constexpr uint32_t P_CHASE = 3435973836u;         // 80 %
constexpr uint32_t P_SHOOT = 0x80000000u;         // 50 %
constexpr uint32_t P_PLANT_EATEN = 0x20000000u;   // 1/8
constexpr uint32_t P_COW_SPAWN = 0x08000000u;     // 1/32
constexpr uint32_t P_SKELETON_SPAWN = 0x19999999u;// 10 %

constexpr int VIEW_ROWS = 7, VIEW_COLS = 9, NCHAN = 21, NVEC = 22;
constexpr int CELL_BYTES = VIEW_ROWS * VIEW_COLS * NCHAN;  // 1323
constexpr int VEC_OFFSET = 1328;
constexpr int MAX_DAY = 1024;

// Philox domains: counter = (env, a, b, domain<<16 | block), key = the env's 64-bit seed.
enum Domain : uint32_t { DOM_STEP = 0, DOM_WORLDGEN = 1, DOM_ACTIONS = 2, DOM_ATLAS = 3 };

// ---- Philox4x32-10 (Salmon et al., SC'11) -------------------------------------------------
struct U4 { uint32_t w[4]; };

__host__ __device__ inline U4 philox4x32_10(uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3,
                                            uint32_t k0, uint32_t k1)
{
#pragma unroll
    for (int r = 0; r < 10; ++r) {
        const uint64_t p0 = (uint64_t)0xD2511F53u * c0;
        const uint64_t p1 = (uint64_t)0xCD9E8D57u * c2;
        const uint32_t n0 = (uint32_t)(p1 >> 32) ^ c1 ^ k0;
        const uint32_t n2 = (uint32_t)(p0 >> 32) ^ c3 ^ k1;
        c1 = (uint32_t)p1;
        c3 = (uint32_t)p0;
        c0 = n0;
        c2 = n2;
        k0 += 0x9E3779B9u;
        k1 += 0xBB67AE85u;
    }
    U4 o;
    o.w[0] = c0; o.w[1] = c1; o.w[2] = c2; o.w[3] = c3;
    return o;
}

__host__ __device__ inline uint32_t choice(uint32_t u, uint32_t n) { return (uint32_t)(((uint64_t)u * n) >> 32); }

// ---- in-HBM layout ----------------------------------------------------------------------------
// One 256-byte record per environment (two 128-byte lines, read and written as 16 x uint4 by
// the 16 lanes that own the environment), plus a 4096-byte row-major map.
struct Mob { uint8_t alive, x, y, dir; int8_t hp; uint8_t cd; uint8_t pad[2]; };          // 8 B
struct Plant { uint8_t alive, x, y, pad; uint16_t age; uint16_t pad2; };                   // 8 B
struct __attribute__((aligned(16))) EnvRec {
    uint8_t px, py, dir, sleeping;   //   0
    uint8_t inv[12];                 //   4
    int8_t vit[4];                   //  16
    int16_t cnt[4];                  //  20
    uint32_t ach;                    //  28
    uint32_t t;                      //  32
    uint32_t episode;                //  36
    uint32_t seed_lo, seed_hi;       //  40
    uint32_t phase;                  //  48  t mod day_length, kept incrementally
    uint32_t pad0[3];                //  52
    Mob mob[NMOB];                   //  64
    Plant plant[NPLANT];             // 160
    uint32_t pad1[4];                // 240
};
static_assert(sizeof(EnvRec) == 256, "record must be 256 bytes");

// Lookup tables built once on the host (craftax_state_init) and kept in the state blob, so
// no float is ever computed on the device beyond single IEEE operations.
struct Luts {
    float daylight[MAX_DAY];        // smoothstep day/night curve, index t mod day_length
    uint32_t zombie_thr[MAX_DAY];   // zombie spawn threshold per phase
    uint8_t light_q7[MAX_DAY];      // daylight in 0..127 for the int8 observation
    float sqrt10[16];               // sqrt(n)/10
    float tenth[16];                // x/10
    float tile[16 * 147];           // tile atlas [block id - 1][7][7][3]
    float ent[5 * 147];             // entity atlas [player, zombie, cow, skeleton, arrow][7][7][3]
    uint8_t ent_mask[256];          // [5][49] 0/1
};

struct Header {
    uint64_t magic;
    uint32_t version, n;
    uint32_t obs_mode, max_episode_steps, day_length;
    uint32_t cap_zombie, cap_cow, cap_skeleton, cap_arrow, cap_plant;
    uint64_t atlas_seed;
    uint64_t off_luts, off_recs, off_maps, total;
};
constexpr uint64_t MAGIC = 0x43524146544158ull;  // "CRAFTAX"

// Scalars every kernel needs, passed by value.
struct Params {
    int n;
    uint32_t max_episode_steps, day_length;
    uint32_t cap_zombie, cap_cow, cap_skeleton, cap_arrow, cap_plant;
};

// ---- lane groups --------------------------------------------------------------------------------
// An environment is owned by G = 16 consecutive lanes of a wavefront (four environments per
// wave64).  Per-environment scalars are held redundantly by all 16 lanes; per-mob and
// per-plant work is spread over lanes 0..11 / 0..9; cross-lane traffic is a ballot or a
// bpermute restricted to the group.
constexpr int G = 16;

__device__ inline uint32_t gballot(bool pred)
{
    const uint64_t m = __ballot(pred);
    const int shift = (threadIdx.x & 63) & ~(G - 1);
    return (uint32_t)(m >> shift) & 0xFFFFu;
}
__device__ inline int gshfl(int v, int src_lane_in_group) { return __shfl(v, src_lane_in_group, G); }

// LDS traffic inside one wave is executed in order, so a group only needs the compiler kept
// from moving LDS accesses across the hand-over point.
__device__ inline void group_sync()
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

__device__ inline bool in_map(int x, int y) { return (unsigned)x < (unsigned)MAPW && (unsigned)y < (unsigned)MAPW; }
__device__ inline bool walkable_ground(int b) { return b == BK_GRASS || b == BK_SAND || b == BK_PATH; }
__device__ inline bool arrow_flyable(int b) { return walkable_ground(b) || b == BK_WATER || b == BK_LAVA; }
__device__ inline int dir_dx(int d) { return d == 1 ? -1 : (d == 2 ? 1 : 0); }
__device__ inline int dir_dy(int d) { return d == 3 ? -1 : (d == 4 ? 1 : 0); }
__device__ inline int iabs(int v) { return v < 0 ? -v : v; }

}  // namespace cx
