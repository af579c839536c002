// Shared definitions of the GPU simulator: ids, constants of the rules, the in-HBM record
// layout, Philox, and the lane-group primitives.  gfx950 only.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace cx {

// ---- bounds checks of the debug build ------------------------------------------------------------
// Built with -DCRAFTAX_DEBUG_BOUNDS, every index into a map, an LDS window or a staging area that
// goes through CX_IDX(index, limit) is checked: an index outside [0, limit) is counted in a
// device-side record (with the source line, the index and the limit of the first one) and 0 is used
// in its place, so that a wrong index is reported without a memory fault.  The release build
// compiles CX_IDX to the bare index.  The record is per translation unit; the host adds them up.
#ifdef CRAFTAX_DEBUG_BOUNDS
static __device__ uint32_t g_bounds[4];   // violations, then line / index / limit of the first one
__device__ inline long long bounds_checked(long long i, long long limit, int line)
{
    if (i >= 0 && i < limit) return i;
    if (atomicAdd(&g_bounds[0], 1u) == 0u) { g_bounds[1] = (uint32_t)line; g_bounds[2] = (uint32_t)i; g_bounds[3] = (uint32_t)limit; }
    return 0;
}
#define CX_IDX(i, limit) ((int)cx::bounds_checked((long long)(i), (long long)(limit), __LINE__))
#else
#define CX_IDX(i, limit) (i)
#endif

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
constexpr uint32_t P_CHASE = 52429u;              // 80 % of 2^16
constexpr uint32_t P_SHOOT = 32768u;              // 50 % of 2^16
constexpr uint32_t P_PLANT_EATEN = 32u;           // 1/8 of 2^8
constexpr uint32_t P_COW_SPAWN = 128u;            // 1/32 of 2^12
constexpr uint32_t P_SKELETON_SPAWN = 410u;       // 10 % of 2^12

constexpr int VIEW_ROWS = 7, VIEW_COLS = 9, NCHAN = 21, NVEC = 22;
constexpr int CELL_BYTES = VIEW_ROWS * VIEW_COLS * NCHAN;  // 1323
constexpr int VEC_OFFSET = 1328;
constexpr int MAX_DAY = 1024;

// Philox domains: counter = (env, a, b, domain<<16 | block), key = the env's 64-bit seed.
enum Domain : uint32_t { DOM_STEP = 0, DOM_WORLDGEN = 1, DOM_ACTIONS = 2, DOM_ATLAS = 3, DOM_MUTATE = 4 };
constexpr int MUTATE_TRIES = 32, MUTATE_AREA = 16;   // swap mutation: tries per call, side of the central area

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
// One 128-byte record (one HBM/L2 line) per environment, 32 dwords, plus two 4096-byte
// tiled maps (see map_index): the world of episode e lives in map slot e & 1, the other slot
// holds (or is being filled with) the world of episode e + 1, generated ahead of time so that
// a finished episode only has to switch slots.  Everything that changes every step lives in
// the record.
//   w0  px | py<<8 | dir<<16 | sleeping<<24
//   w1  six 4-bit item counts (wood stone coal iron diamond sapling) | six tool flags at bit 24
//   w2  four 4-bit vitals (health food drink energy) | phase<<16 (t mod day_length)
//   w3  four signed 8-bit counters (hunger thirst fatigue recover)
//   w4  achievement bits   w5 t   w6 episode   w7,w8 seed   w9 spare
//   w10..w21 mob slots     w22..w31 plant slots
// mob word:   alive | x<<1 | y<<7 | dir<<13 | hp<<16 | cd<<20   (0 when the slot is empty)
// plant word: alive | x<<1 | y<<7 | age<<16                     (0 when the slot is empty)
constexpr int REC_DWORDS = 32;
constexpr int RW_POS = 0, RW_INV = 1, RW_VIT = 2, RW_CNT = 3, RW_ACH = 4, RW_T = 5, RW_EPISODE = 6,
              RW_SEED_LO = 7, RW_SEED_HI = 8, RW_MOB = 10, RW_PLANT = 22;

struct Mob { int alive, x, y, dir, hp, cd; };
struct Plant { int alive, x, y, age; };

__host__ __device__ inline Mob unpack_mob(uint32_t w)
{
    Mob m;
    m.alive = w & 1u; m.x = (w >> 1) & 63u; m.y = (w >> 7) & 63u; m.dir = (w >> 13) & 7u;
    m.hp = (w >> 16) & 15u; m.cd = (w >> 20) & 15u;
    return m;
}
__host__ __device__ inline uint32_t pack_mob(const Mob& m)
{
    return m.alive ? (1u | ((uint32_t)m.x << 1) | ((uint32_t)m.y << 7) | ((uint32_t)m.dir << 13) |
                      ((uint32_t)m.hp << 16) | ((uint32_t)m.cd << 20)) : 0u;
}
__host__ __device__ inline Plant unpack_plant(uint32_t w)
{
    Plant q;
    q.alive = w & 1u; q.x = (w >> 1) & 63u; q.y = (w >> 7) & 63u; q.age = (int)(w >> 16);
    return q;
}
__host__ __device__ inline uint32_t pack_plant(const Plant& q)
{
    return q.alive ? (1u | ((uint32_t)q.x << 1) | ((uint32_t)q.y << 7) | ((uint32_t)q.age << 16)) : 0u;
}

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
    uint32_t perlin_cs[1024];       // unit gradient of direction a: cos (low half) and sin (high half) in Q14, as int16
};

struct Header {
    uint64_t magic;
    uint32_t version, n;
    uint32_t obs_mode, max_episode_steps, day_length;
    uint32_t cap_zombie, cap_cow, cap_skeleton, cap_arrow, cap_plant;
    uint64_t atlas_seed;
    uint64_t off_ctrs, off_luts, off_recs, off_maps, off_tags, off_regen0, off_regen1, off_slow, off_unlocks, total;
    uint32_t variant, worldgen, reset_mode, pad;
};
constexpr uint64_t HEADER_BYTES = 256;   // the header sits alone in the first 256 bytes of the state blob
static_assert(sizeof(Header) <= HEADER_BYTES, "header outgrew its area");
constexpr uint64_t MAGIC = 0x43524146544158ull;  // "CRAFTAX"

// Scalars every kernel needs, passed by value.
struct Params {
    int n;
    uint32_t max_episode_steps, day_length;
    uint32_t cap_zombie, cap_cow, cap_skeleton, cap_arrow, cap_plant;
    uint32_t worldgen;              // CRAFTAX_WORLDGEN_*
    uint32_t reset_mode;            // CRAFTAX_RESET_*
    uint32_t* unlocks;              // UNLOCK_STRIDE counters per environment (see count_unlocks); null in kernels that do not step
};
constexpr uint32_t POOL_RATIO = 16, POOL_ENV = 0x80000000u;   // optimistic resets: environments per pool world; numbering of the pool's worlds

// Unlock counters (the paper reports achievement success rates, section "Craftax-1B": the share of
// episodes in which an achievement was unlocked): counts[k] = how often achievement k has been
// unlocked in this environment since craftax_reset.  An achievement unlocks at most once per
// episode, so the sum over the environments, less the episodes still running that hold it, is the
// number of finished episodes that reached it.  Counted where it happens, in the step: `unlocked`
// = the bits that are new after this step.  The G lanes of the environment's group take the
// achievements l, l + G, ...; the adds return nothing, so no wavefront waits for them, and only
// this group ever touches these words.
constexpr int N_ACHIEVEMENTS = 22, UNLOCK_STRIDE = 24;   // dwords per environment (96 bytes)
template <int G>
__device__ __forceinline__ void count_unlocks(int l, uint32_t* __restrict__ counts, uint32_t unlocked)
{
    if (unlocked == 0u) return;
#pragma unroll
    for (int k0 = 0; k0 < N_ACHIEVEMENTS; k0 += G) {
        const int k = k0 + l;
        if (k < N_ACHIEVEMENTS && ((unlocked >> k) & 1u)) atomicAdd(counts + k, 1u);
    }
}

// ---- lane groups --------------------------------------------------------------------------------
// An environment is owned by G consecutive lanes of a wavefront (G = 4, 8 or 16, so 16, 8 or
// 4 environments per wave64).  Per-environment scalars are held redundantly by all G lanes
// (same inputs, same arithmetic, no exchange needed); mob slot k, plant slot k and Philox
// block k belong to lane k mod G (sub-slot k / G); cross-lane traffic is a ballot or a
// bpermute restricted to the group.  Few lanes per environment amortise the scalar rules
// over more environments per wave (best at tens of thousands of environments); many lanes
// per environment give more waves and shorter per-wave loops (best at a few thousand).
template <int G>
struct Grp {
    static constexpr int EPB = 256 / G;                    // environments per 256-thread block
    static constexpr int NS_MOB = (NMOB + G - 1) / G;      // mob sub-slots per lane
    static constexpr int NS_PLANT = (NPLANT + G - 1) / G;  // plant sub-slots per lane

    // bit i of the result = predicate of lane i of this group
    __device__ static inline uint32_t ballot(bool pred)
    {
        const uint64_t m = __ballot(pred);
        const uint32_t lane = threadIdx.x & 63u;
        const uint32_t half = (lane & 32u) ? (uint32_t)(m >> 32) : (uint32_t)m;
        return __builtin_amdgcn_ubfe(half, lane & 31u & ~(uint32_t)(G - 1), (uint32_t)G);
    }
    // value of lane src_lane_in_group of this group.  Four lanes are a DPP quad: a lane number
    // that the compiler knows (the unrolled loops over slots) turns into one quad-broadcast move
    // instead of a trip through the LDS permute unit.
    __device__ static inline int shfl(int v, int src_lane_in_group)
    {
        if (G == 4 && __builtin_constant_p(src_lane_in_group)) {
            switch (src_lane_in_group) {
            case 0: return __builtin_amdgcn_mov_dpp(v, 0x00, 0xF, 0xF, true);
            case 1: return __builtin_amdgcn_mov_dpp(v, 0x55, 0xF, 0xF, true);
            case 2: return __builtin_amdgcn_mov_dpp(v, 0xAA, 0xF, 0xF, true);
            default: return __builtin_amdgcn_mov_dpp(v, 0xFF, 0xF, 0xF, true);
            }
        }
        return __shfl(v, src_lane_in_group, G);
    }
};

// LDS traffic inside one wave is executed in order, so a group only needs the compiler kept
// from moving LDS accesses across the hand-over point.
__device__ inline void group_sync()
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

// The 64x64 map of an environment is stored as 4x8 tiles of 16 columns x 8 rows; a tile is 128
// bytes = one cache line, rows of a tile are 16 contiguous bytes.  The 9-row, 16-byte-wide
// window the step reads every time then touches 2 to 4 lines instead of 5 to 9.
__device__ inline int map_index(int x, int y)
{
    x = CX_IDX(x, MAPW); y = CX_IDX(y, MAPW);
    return (((y >> 3) << 2) + (x >> 4)) * 128 + ((y & 7) << 4) + (x & 15);
}

// byte offset of the map of `episode` of environment `env` inside the maps area
__host__ __device__ inline size_t map_offset(uint32_t env, uint32_t episode)
{
    return ((size_t)env * 2 + (episode & 1u)) * (size_t)(MAPW * MAPW);
}

__device__ inline bool in_map(int x, int y) { return ((unsigned)x | (unsigned)y) < (unsigned)MAPW; }
// block-id sets as bit masks
constexpr uint32_t WALKABLE_MASK = (1u << BK_GRASS) | (1u << BK_SAND) | (1u << BK_PATH);
constexpr uint32_t FLYABLE_MASK = WALKABLE_MASK | (1u << BK_WATER) | (1u << BK_LAVA);
__device__ inline bool walkable_ground(int b) { return (WALKABLE_MASK >> b) & 1u; }
__device__ inline bool arrow_flyable(int b) { return (FLYABLE_MASK >> b) & 1u; }
__device__ inline int dir_dx(int d) { return d == 1 ? -1 : (d == 2 ? 1 : 0); }
__device__ inline int dir_dy(int d) { return d == 3 ? -1 : (d == 4 ? 1 : 0); }
__device__ inline int iabs(int v) { return v < 0 ? -v : v; }

// Per-environment LDS area: record, map window, one-hot bit staging, scalar vector.
// The window is 9 rows of 16 bytes: row r holds the map bytes of row (py-4+r) from the
// 4-byte-aligned column xa = (px-5) & ~3 on, so it is filled with aligned dword loads; window
// column c (map column px-5+c) sits at byte (px-5 & 3) + c of the row.  Cells outside the map
// read as BK_OOB.  The per-environment stride is 142 dwords: the 4..16 environments of a wave
// start on distinct even banks, so they never collide when they touch the same field.
constexpr int WIN_ROWS = 9, WIN_COLS = 11, WIN_PITCH = 16;
constexpr int WIN_DWORDS = WIN_ROWS * WIN_PITCH / 4;   // 36
constexpr int LDS_REC = 0;                       // 32 dwords
constexpr int LDS_WIN = 32;                      // 36 dwords
constexpr int LDS_BITS = 68;                     // 1328 bits -> 42 dwords
constexpr int LDS_VEC = 110;                     // 24 dwords (22 scalars + padding)
constexpr int LDS_FLAG = 134;                    // 1 = this environment's staged observation is to be written
constexpr int LDS_WINPOS = 135;                  // rollout: bit 31 | py << 8 | px of the position the window was loaded for, or 0
constexpr int LDS_ENV_DWORDS = 142;
static_assert(LDS_VEC + 24 <= LDS_ENV_DWORDS, "per-environment LDS area overflows");
// The layout above keeps the record intact while the observation is staged (the rollout kernel
// carries records from step to step).  The single-step kernel has written its record back before
// it renders, so there the scalar vector takes the record's place: 118 dwords per environment
// (again distinct even banks for the environments of a wave), which lets five blocks of 64
// environments share a compute unit's 160 KB instead of four.
struct KeepLayout { static constexpr int VEC = LDS_VEC, FLAG = LDS_FLAG, STRIDE = LDS_ENV_DWORDS; };
struct StepLayout { static constexpr int VEC = LDS_REC, FLAG = 110, STRIDE = 118; };
static_assert(StepLayout::FLAG >= LDS_BITS + 42 && StepLayout::FLAG < StepLayout::STRIDE && REC_DWORDS >= 24, "single-step LDS layout");

}  // namespace cx
