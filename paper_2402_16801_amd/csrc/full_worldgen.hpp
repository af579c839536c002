// Block-cooperative generation of the nine floors of one full-Craftax world (section "World
// Generation" of the paper's appendix lists the floors: overworld, dungeon, gnomish mines,
// sewers, vault, troll mines, fire realm, ice realm, graveyard).  The paper does not print its
// generators; here every cell of every floor is a pure integer function of (seed, env, episode,
// floor, x, y): value-noise thresholds for the open floors, eight seeded rooms joined by
// L-shaped corridors for the built ones.  One block of 576 threads per (environment, floor),
// each thread owning a run of 4 cells, so that a reset is nine short blocks instead of one long one.
#pragma once

#include "full_common.hpp"

namespace cf {

constexpr int GEN_THREADS = CELLS / 4;                    // 576: one thread per run of 4 cells of a floor
constexpr int LAT0_U16 = 2 * 16 + 4 * 49;                 // overworld lattices: two 4x4 (spacing 16), four 7x7 (spacing 8)
constexpr int LAT0_BLOCKS = (LAT0_U16 + 7) / 8;           // 29
constexpr int LATC_U16 = 2 * 49, LATC_BLOCKS = (LATC_U16 + 7) / 8;   // cave floors: two 7x7 lattices, 13 blocks
constexpr int LAT_STRIDE0 = LAT0_BLOCKS * 8, LAT_STRIDEC = LATC_BLOCKS * 8;
constexpr int LAT_TOTAL = LAT_STRIDE0;                    // a block generates one floor: the largest lattice set

struct Room { int x, y, w, h, cx, cy; };
struct GenLayout {
    Room room[3][8];          // dungeon (floor 1), sewers (3), vault (4)
    int up[FLOORS][2], down[FLOORS][2];
    uint32_t perm;            // potion colour -> effect, 6 x 3 bits
    // The built floor being generated, row by row (bit x = column x), see dungeon_row_masks: cells
    // inside rooms 0..3 and 4..7, cells on corridors 0..3 and 4..6, chest cells; and the five single
    // cells of a floor as x | y << 8: fountain, the two enchantment tables, ladder up, ladder down
    // (0xFFFF: this floor has none).
    uint64_t row_mask[5][W];
    uint32_t spot[5];
};

__device__ inline int cave_index(int f) { return f == 2 ? 0 : (f == 5 ? 1 : (f == 6 ? 2 : 3)); }
__device__ inline int dungeon_index(int f) { return f == 1 ? 0 : (f == 3 ? 1 : 2); }
__device__ inline bool is_dungeon(int f) { return f == 1 || f == 3 || f == 4; }
__device__ inline bool is_cave(int f) { return f == 2 || f == 5 || f == 6 || f == 7; }

__device__ inline bool on_corridor(int x, int y, int x0, int y0, int x1, int y1)
{
    // horizontal along y0 from x0 to x1, then vertical along x1 from y0 to y1
    const bool h = y == y0 && x >= min(x0, x1) && x <= max(x0, x1);
    const bool v = x == x1 && y >= min(y0, y1) && y <= max(y0, y1);
    return h | v;
}

// Noise fields of a run of cells in one row: the two lattice rows are blended once per lattice
// column (vertical weight), then every cell blends two columns (horizontal weight).  The integer
// result equals the row-first bilinear formula ((a(256-wx)+b wx)(256-wy) + (c(256-wx)+d wx) wy) >> 16
// because nothing is rounded before the final shift.  The callers'
// runs of 4 cells start at a multiple of 4, so a run lies inside one lattice cell.
struct Field8 { uint32_t l, r; };
__device__ inline Field8 field8(const uint16_t* lat, int x0, int y)
{
    const uint32_t wy = cx::smooth8(y & 7);
    return { cx::column(lat, 7, x0 >> 3, y >> 3, wy), cx::column(lat, 7, (x0 >> 3) + 1, y >> 3, wy) };
}
__device__ inline Field8 field16(const uint16_t* lat, int x0, int y)
{
    const uint32_t wy = cx::smooth16(y & 15);
    return { cx::column(lat, 4, x0 >> 4, y >> 4, wy), cx::column(lat, 4, (x0 >> 4) + 1, y >> 4, wy) };
}
__device__ inline uint32_t at8(const Field8& f, int x) { return cx::across(f.l, f.r, cx::smooth8(x & 7)); }
__device__ inline uint32_t at16(const Field8& f, int x) { return cx::across(f.l, f.r, cx::smooth16(x & 15)); }

// Cell functions, one per kind of floor: block id | item << 8.
__device__ inline int classify_overworld(const GenLayout& L, int Wn, int Mn, int Cn, int Fn, int x, int y, int u)
{
    const int d = max(iabs(x - W / 2), iabs(y - W / 2));
    if (d < 10) { const int bias = (10 - d) * 2500; Wn = max(0, Wn - bias); Mn = max(0, Mn - bias); }
    int b;
    if (d <= 2) b = B_GRASS;
    else if (Mn > 39500) {
        if (Cn > 43000 && Mn > 41000) b = B_PATH;
        else if (iabs(Cn - 30000) < 1300) b = B_PATH;
        else if (Mn > 43000 && Fn > 44000) b = B_LAVA;
        else if (Mn > 42000 && u < 500) b = B_DIAMOND;
        else if (Fn < 33000 && u >= 500 && u < 3000) b = B_IRON;
        else if (u >= 3000 && u < 8000) b = B_COAL;
        else b = B_STONE;
    } else if (Wn > 39500) b = B_WATER;
    else if (Wn > 37800) b = B_SAND;
    else if (Fn > 33500 && u < 26000) b = B_TREE;
    else if (u < 1300) b = B_TREE;
    else b = B_GRASS;
    if (x == L.down[0][0] && y == L.down[0][1]) return B_PATH | (IT_LADDER_DOWN << 8);
    return b;
}
// The cell of a built floor written out test by test.  The generator uses cell_dungeon_masked below, which
// takes `inside`, `corridor` and the chest test from per-row bit masks; this is what those masks mean.
__device__ inline int cell_dungeon(const GenLayout& L, int f, int x, int y, int u)
{
    const Room* R = L.room[dungeon_index(f)];
    bool inside = false;
#pragma unroll
    for (int i = 0; i < 8; ++i) inside |= (unsigned)(x - R[i].x) < (unsigned)R[i].w && (unsigned)(y - R[i].y) < (unsigned)R[i].h;
    int b = f == 3 ? B_WALL_MOSS : B_WALL;
    if (inside) b = (f == 3 && u < 12000) ? B_WATER : B_PATH;
#pragma unroll
    for (int i = 1; i <= 6; ++i) if (x == R[i].cx + 1 && y == R[i].cy + 1) b = B_CHEST;
    if (f == 1 && x == R[2].cx - 1 && y == R[2].cy - 1) b = B_FOUNTAIN;
    if (f == 4 && x == R[3].cx - 1 && y == R[3].cy - 1) b = B_ENCH_FIRE;
    if (f == 4 && x == R[4].cx - 1 && y == R[4].cy - 1) b = B_ENCH_ICE;
    bool corridor = false;
#pragma unroll
    for (int i = 0; i < 7; ++i) corridor |= on_corridor(x, y, R[i].cx, R[i].cy, R[i + 1].cx, R[i + 1].cy);
    if (corridor) b = B_PATH;       // corridors last: room centre 0 (ladder up) always reaches room centre 7 (ladder down)
    int it = IT_NONE;
    if (x == R[0].cx && y == R[0].cy) { b = B_PATH; it = IT_LADDER_UP; }
    if (x == R[7].cx && y == R[7].cy) { b = B_PATH; it = IT_LADDER_DOWN_BLOCKED; }
    return b | (it << 8);
}
// A built floor as bit masks per row, so that a cell costs a few shifts and tests instead of eight
// room tests, seven corridor tests and nine single-cell tests.  Part p of row y (five parts, so
// that 240 threads share the work): rooms 0..3, rooms 4..7 (`inside` of cell_dungeon), corridors
// 0..3, corridors 4..6 (`corridor`), chests.  The few single cells go to L.spot.
constexpr int M_ROOMS_A = 0, M_ROOMS_B = 1, M_PATH_A = 2, M_PATH_B = 3, M_CHEST = 4, MASK_PARTS = 5;
constexpr int SPOT_FOUNTAIN = 0, SPOT_FIRE = 1, SPOT_ICE = 2, SPOT_UP = 3, SPOT_DOWN = 4;
__device__ inline void dungeon_row_mask(GenLayout& L, int f, int y, int part)
{
    const Room* R = L.room[dungeon_index(f)];
    auto span = [](int a, int b) -> uint64_t { return (~0ull >> (63 - (b - a))) << a; };   // bits a..b, 0 <= a <= b < 64
    uint64_t m = 0ull;
    if (part == M_ROOMS_A || part == M_ROOMS_B) {
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            const Room r = R[4 * (part - M_ROOMS_A) + k];
            if ((unsigned)(y - r.y) < (unsigned)r.h) m |= span(r.x, r.x + r.w - 1);
        }
    } else if (part == M_PATH_A || part == M_PATH_B) {
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            const int i = 4 * (part - M_PATH_A) + k;
            if (i < 7) {
                const int x0 = R[i].cx, y0 = R[i].cy, x1 = R[i + 1].cx, y1 = R[i + 1].cy;
                if (y == y0) m |= span(min(x0, x1), max(x0, x1));
                if (y >= min(y0, y1) && y <= max(y0, y1)) m |= 1ull << x1;
            }
        }
    } else {
#pragma unroll
        for (int i = 1; i <= 6; ++i) if (y == R[i].cy + 1) m |= 1ull << (R[i].cx + 1);
    }
    L.row_mask[CX_IDX(part, MASK_PARTS)][CX_IDX(y, W)] = m;
}
__device__ inline void dungeon_spot(GenLayout& L, int f, int k)
{
    const Room* R = L.room[dungeon_index(f)];
    auto at = [](int x, int y) { return (uint32_t)x | ((uint32_t)y << 8); };
    uint32_t v = 0xFFFFu;
    if (k == SPOT_FOUNTAIN && f == 1) v = at(R[2].cx - 1, R[2].cy - 1);
    if (k == SPOT_FIRE && f == 4) v = at(R[3].cx - 1, R[3].cy - 1);
    if (k == SPOT_ICE && f == 4) v = at(R[4].cx - 1, R[4].cy - 1);
    if (k == SPOT_UP) v = at(R[0].cx, R[0].cy);
    if (k == SPOT_DOWN) v = at(R[7].cx, R[7].cy);
    L.spot[k] = v;
}
// cell_dungeon from the masks of its row (shifted so that bit 0 is this cell) and the single cells:
// the same tests in the same order of precedence.
__device__ inline int cell_dungeon_masked(const GenLayout& L, int f, int x, int y, int u, bool inside, bool corridor, bool chest)
{
    const uint32_t here = (uint32_t)x | ((uint32_t)y << 8);
    int b = f == 3 ? B_WALL_MOSS : B_WALL;
    if (inside) b = (f == 3 && u < 12000) ? B_WATER : B_PATH;
    if (chest) b = B_CHEST;
    if (here == L.spot[SPOT_FOUNTAIN]) b = B_FOUNTAIN;
    if (here == L.spot[SPOT_FIRE]) b = B_ENCH_FIRE;
    if (here == L.spot[SPOT_ICE]) b = B_ENCH_ICE;
    if (corridor) b = B_PATH;
    int it = IT_NONE;
    if (here == L.spot[SPOT_UP]) { b = B_PATH; it = IT_LADDER_UP; }
    if (here == L.spot[SPOT_DOWN]) { b = B_PATH; it = IT_LADDER_DOWN_BLOCKED; }
    return b | (it << 8);
}
__device__ inline int cell_graveyard(int x, int y)
{
    int b = (x == 0 || y == 0 || x == W - 1 || y == W - 1) ? B_WALL : B_PATH;
    if ((x & 7) == 0 && x >= 8 && x <= 40 && (y == 12 || y == 24 || y == 36)) b = B_GRAVE1 + ((x - 8) / 8 + (y - 12) / 12) % 3;
    if (x == BOSS_X && y == BOSS_Y) b = B_NECRO_VULN;
    if (x == 24 && y == 42) return B_PATH | (IT_LADDER_UP << 8);
    return b;
}
// The cell of a cave floor written out test by test.  The generator uses classify_cave_masked below, which takes
// the clearings and the corridor from a per-row bit mask; this is what that mask means.
__device__ inline int classify_cave(const GenLayout& L, int f, int Cn, int Fn, int x, int y, int u)
{
    const int open = f == 6 ? B_FIRE_GRASS : (f == 7 ? B_ICE_GRASS : B_PATH);
    int b;
    if (Cn > 31000) {
        b = open;
        if (f == 2 && u < 1500) b = B_STALAGMITE;
        if (f == 5 && Fn > 44000) b = B_WATER;
        if (f == 6) { if (Fn > 43000) b = B_LAVA; else if (u < 3000) b = B_FIRE_TREE; }
        if (f == 7) { if (Fn > 43000) b = B_WATER; else if (u < 3000) b = B_ICE_SHRUB; }
    } else {
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
    const int ux = L.up[f][0], uy = L.up[f][1], dx = L.down[f][0], dy = L.down[f][1];
    if (max(iabs(x - ux), iabs(y - uy)) <= 1 || max(iabs(x - dx), iabs(y - dy)) <= 1) b = open;
    if (on_corridor(x, y, ux, uy, dx, dy)) b = open;      // the two ladders are always connected
    int it = IT_NONE;
    if (x == ux && y == uy) { b = B_PATH; it = IT_LADDER_UP; }
    if (x == dx && y == dy) { b = B_PATH; it = IT_LADDER_DOWN_BLOCKED; }
    return b | (it << 8);
}

// Row y of a cave floor as one bit mask (L.row_mask[M_CAVE_OPEN]): the cells classify_cave opens whatever
// the noise says, i.e. the 3 x 3 clearings around the two ladders and the L-shaped corridor between
// them; the ladders themselves go to L.spot.  classify_cave_masked is classify_cave with those
// tests taken from the mask: the same rules in the same order.
constexpr int M_CAVE_OPEN = 0;
__device__ inline void cave_row_mask(GenLayout& L, int f, int y)
{
    const int ux = L.up[f][0], uy = L.up[f][1], dx = L.down[f][0], dy = L.down[f][1];
    auto span = [](int a, int b) -> uint64_t { return (~0ull >> (63 - (b - a))) << a; };   // bits a..b, 0 <= a <= b < 64
    uint64_t m = 0ull;
    if (iabs(y - uy) <= 1) m |= span(ux - 1, ux + 1);
    if (iabs(y - dy) <= 1) m |= span(dx - 1, dx + 1);
    if (y == uy) m |= span(min(ux, dx), max(ux, dx));                 // on_corridor: along row uy from ux to dx,
    if (y >= min(uy, dy) && y <= max(uy, dy)) m |= 1ull << dx;        // then along column dx from uy to dy
    L.row_mask[M_CAVE_OPEN][CX_IDX(y, W)] = m;
    if (y == 0) {
        L.spot[SPOT_UP] = (uint32_t)ux | ((uint32_t)uy << 8);
        L.spot[SPOT_DOWN] = (uint32_t)dx | ((uint32_t)dy << 8);
    }
}
__device__ inline int classify_cave_masked(const GenLayout& L, int f, int Cn, int Fn, int x, int y, int u, bool opened)
{
    const int open = f == 6 ? B_FIRE_GRASS : (f == 7 ? B_ICE_GRASS : B_PATH);
    int b;
    if (Cn > 31000) {
        b = open;
        if (f == 2 && u < 1500) b = B_STALAGMITE;
        if (f == 5 && Fn > 44000) b = B_WATER;
        if (f == 6) { if (Fn > 43000) b = B_LAVA; else if (u < 3000) b = B_FIRE_TREE; }
        if (f == 7) { if (Fn > 43000) b = B_WATER; else if (u < 3000) b = B_ICE_SHRUB; }
    } else {
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
    if (opened) b = open;
    const uint32_t here = (uint32_t)x | ((uint32_t)y << 8);
    int it = IT_NONE;
    if (here == L.spot[SPOT_UP]) { b = B_PATH; it = IT_LADDER_UP; }
    if (here == L.spot[SPOT_DOWN]) { b = B_PATH; it = IT_LADDER_DOWN_BLOCKED; }
    return b | (it << 8);
}

// World-generation draws: counter (env, stream, episode, WORLDGEN | block); stream = floor*4 +
// {0 lattices, 1 per-cell u16, 2 layout words}, stream 63 = potion permutation.
__device__ inline U4 wg_block(uint32_t lo, uint32_t hi, uint32_t env, uint32_t episode, uint32_t stream, uint32_t block)
{
    return philox4x32_10(env, stream, episode, (cx::DOM_WORLDGEN << 16) | block, lo, hi);
}

__device__ inline void put_lattice(uint16_t* dst, const U4& r)
{
#pragma unroll
    for (int w = 0; w < 4; ++w) { dst[2 * w] = (uint16_t)(r.w[w] & 0xFFFFu); dst[2 * w + 1] = (uint16_t)(r.w[w] >> 16); }
}
__device__ inline void make_room(GenLayout& L, int f, int i, const U4& r)
{
    Room R;
    R.w = 5 + (int)choice(r.w[0], 5);
    R.h = 5 + (int)choice(r.w[1], 5);
    R.x = 1 + (int)choice(r.w[2], (uint32_t)(46 - R.w));
    R.y = 1 + (int)choice(r.w[3], (uint32_t)(46 - R.h));
    R.cx = R.x + R.w / 2;
    R.cy = R.y + R.h / 2;
    L.room[dungeon_index(f)][i] = R;
    if (i == 0) { L.up[f][0] = R.cx; L.up[f][1] = R.cy; }
    if (i == 7) { L.down[f][0] = R.cx; L.down[f][1] = R.cy; }
}
__device__ inline void make_cave_ladders(GenLayout& L, int f, const U4& r)
{
    L.up[f][0] = 10 + (int)choice(r.w[0], 6); L.up[f][1] = 10 + (int)choice(r.w[1], 6);
    L.down[f][0] = 32 + (int)choice(r.w[2], 6); L.down[f][1] = 32 + (int)choice(r.w[3], 6);
}

// Generates floor f of one environment with the NT threads of the calling block: run t (of 576)
// is the 4 cells [4t, 4t+4) of the floor (row t/12).  The block of floor 0 also derives the
// ladders of every floor and the potion permutation (whole_layout), which the fresh record
// needs, and may drop the cells around the start position into an LDS window (start_wb /
// start_wi, 11 x 16 bytes each) for the first observation.  maps: this environment's 41472
// bytes.  s_lat, L: LDS scratch.  Ends with a block barrier.
// first_run, runs: the part of the floor this call generates (a block of fewer than `runs` threads
// takes several passes).
// perlin_cs (with CAN_PERLIN): the gradient table; the fields of the overworld and of the caves are
// then Perlin noise over the same lattices (appendix "World Generation") instead of value noise.
// A kernel instantiated without CAN_PERLIN carries no code for it.
// theta_f (with CAN_PERLIN; LDS, LAT_TOTAL entries, the same for the whole block): angle offsets in
// 1024ths of a turn added to the upper ten bits of this floor's lattice numbers, the level of the
// noise mutation (section "Craftax-1B: UED").
template <int NT = GEN_THREADS, bool CAN_PERLIN = false>
__device__ __forceinline__ void worldgen_floor_block(uint8_t* __restrict__ maps, uint16_t* s_lat, GenLayout& L, uint32_t lo, uint32_t hi,
                                            uint32_t env, uint32_t episode, int f, uint8_t* start_wb = nullptr,
                                            uint8_t* start_wi = nullptr, int first_run = 0, int runs = GEN_THREADS,
                                            const uint32_t* __restrict__ perlin_cs = nullptr, const uint16_t* theta_f = nullptr)
{
    const bool perlin = CAN_PERLIN && perlin_cs != nullptr;
    static_assert(NT >= 64, "the layout phase uses the first wavefront");
    const int tid0 = threadIdx.x;
    // Layout phase, all in the first wavefront and with one Philox call for the whole wave: every
    // lane picks the (stream, block) of its role, then the roles unpack their words.
    if (tid0 < 64) {
        const int tid = tid0;
        if (f == 0) {
            // lanes 0..28 lattice blocks; 29..52 rooms of floors 1, 3, 4; 53..56 ladders of the caves 2, 5, 6, 7;
            // 57 overworld ladder; 58, 59 potion permutation (section "Potions and Enchantments")
            uint32_t stream = 0u, block = (uint32_t)tid;
            int ff = 0;
            if (tid >= 29 && tid < 53) { const int d = (tid - 29) >> 3; ff = d == 0 ? 1 : (d == 1 ? 3 : 4); stream = (uint32_t)ff * 4u + 2u; block = (uint32_t)((tid - 29) & 7); }
            else if (tid >= 53 && tid < 57) { const int c = tid - 53; ff = c == 0 ? 2 : (c == 1 ? 5 : (c == 2 ? 6 : 7)); stream = (uint32_t)ff * 4u + 2u; block = 0u; }
            else if (tid == 57) { stream = 2u; block = 0u; }
            else if (tid >= 58) { stream = 63u; block = tid == 59 ? 1u : 0u; }
            const U4 r = wg_block(lo, hi, env, episode, stream, block);
            const uint32_t fifth = (uint32_t)__shfl((int)r.w[0], 59);
            if (tid < LAT0_BLOCKS) put_lattice(s_lat + tid * 8, r);
            else if (tid < 53) make_room(L, ff, (tid - 29) & 7, r);
            else if (tid < 57) make_cave_ladders(L, ff, r);
            else if (tid == 57) {
                int dx = (int)choice(r.w[0], 13) - 6;
                const int dy = (int)choice(r.w[1], 13) - 6;
                if (max(iabs(dx), iabs(dy)) < 3) dx = 3;
                L.up[0][0] = 0; L.up[0][1] = 0; L.down[0][0] = W / 2 + dx; L.down[0][1] = W / 2 + dy;
                L.up[8][0] = 24; L.up[8][1] = 42; L.down[8][0] = 0; L.down[8][1] = 0;
            } else if (tid == 58) {
                // a fresh colour -> effect permutation per episode
                const uint32_t draws[5] = { r.w[0], r.w[1], r.w[2], r.w[3], fifth };
                uint32_t perm = 0u;
#pragma unroll
                for (int i = 0; i < 6; ++i) perm |= (uint32_t)i << (3 * i);
#pragma unroll
                for (int i = 5; i >= 1; --i) {
                    const int j = (int)choice(draws[5 - i], (uint32_t)(i + 1));
                    const uint32_t a = (perm >> (3 * i)) & 7u, b = (perm >> (3 * j)) & 7u;
                    perm &= ~((7u << (3 * i)) | (7u << (3 * j)));
                    perm |= (b << (3 * i)) | (a << (3 * j));
                }
                L.perm = perm;
            }
        } else if (is_dungeon(f)) {
            if (tid < 8) make_room(L, f, tid, wg_block(lo, hi, env, episode, (uint32_t)f * 4u + 2u, (uint32_t)tid));
        } else if (is_cave(f)) {
            // lanes 0..12 lattice blocks, lane 13 the ladders
            if (tid <= LATC_BLOCKS) {
                const U4 r = wg_block(lo, hi, env, episode, (uint32_t)f * 4u + (tid == LATC_BLOCKS ? 2u : 0u), tid == LATC_BLOCKS ? 0u : (uint32_t)tid);
                if (tid < LATC_BLOCKS) put_lattice(s_lat + tid * 8, r);
                else make_cave_ladders(L, f, r);
            }
        }
    }
    __syncthreads();
    if (is_dungeon(f)) {                       // the same floor for the whole block
        for (int i = tid0; i < MASK_PARTS * W; i += NT) dungeon_row_mask(L, f, i % W, i / W);
        if (tid0 < 5) dungeon_spot(L, f, tid0);
        __syncthreads();
    } else if (is_cave(f)) {
        if (tid0 < W) cave_row_mask(L, f, tid0);
        __syncthreads();
    }
    if (CAN_PERLIN && theta_f != nullptr) {
        for (int i = tid0; i < LAT_TOTAL; i += NT) s_lat[i] = (uint16_t)(s_lat[i] + ((theta_f[i] & 1023u) << 6));
        __syncthreads();
    }
    // runs of 4 cells, one per thread and pass
#pragma unroll 1
    for (int tid = first_run + tid0; tid < first_run + runs; tid += NT) {
    const int y = tid / 12, x = (tid - y * 12) * 4;
    const bool needs_u = !(f == 1 || f == 4 || f == 8);
    uint32_t rw0 = 0u, rw1 = 0u;
    if (needs_u) {
        // per-cell draws: Philox block (cell / 8) holds eight u16, this thread uses one half of it
        const U4 r = wg_block(lo, hi, env, episode, (uint32_t)f * 4u + 1u, (uint32_t)(tid >> 1));
        rw0 = (tid & 1) ? r.w[2] : r.w[0];
        rw1 = (tid & 1) ? r.w[3] : r.w[1];
    }
    const uint32_t light = lit_floor(f) ? (uint32_t)MAX_LIGHT << 3 : 0u;
    uint32_t pb = 0u, pi = 0u;
    auto put = [&](int j, int cell) {
        pb |= (uint32_t)(cell & 0xFF) << (8 * j);
        pi |= ((uint32_t)(cell >> 8) | light) << (8 * j);
    };
    auto draw = [&](int j) { const uint32_t rw = j < 2 ? rw0 : rw1; return (int)((j & 1) ? (rw >> 16) : (rw & 0xFFFFu)); };
    // the floor is the same for the whole block: one kind of cell function per block
    // (the cells of a run one after the other: side by side they are no faster where many blocks
    // share a compute unit, and they cost the step kernel registers it does not have)
    auto cells = [&](auto&& one) {
#pragma unroll 1
        for (int j = 0; j < 4; ++j) one(j);
    };
    if (CAN_PERLIN && perlin && f == 0) {
        cells([&](int j) {
            const int Wn = (int)((3u * cx::perlin<16>(s_lat, 4, perlin_cs, x + j, y) + cx::perlin<8>(s_lat + 32, 7, perlin_cs, x + j, y)) >> 2);
            const int Mn = (int)((3u * cx::perlin<16>(s_lat + 16, 4, perlin_cs, x + j, y) + cx::perlin<8>(s_lat + 81, 7, perlin_cs, x + j, y)) >> 2);
            put(j, classify_overworld(L, Wn, Mn, (int)cx::perlin<8>(s_lat + 130, 7, perlin_cs, x + j, y),
                                      (int)cx::perlin<8>(s_lat + 179, 7, perlin_cs, x + j, y), x + j, y, draw(j)));
        });
    } else if (CAN_PERLIN && perlin && is_cave(f)) {
        const uint64_t opened = L.row_mask[M_CAVE_OPEN][CX_IDX(y, W)] >> x;   // the run lies in one row
        cells([&](int j) {
            put(j, classify_cave_masked(L, f, (int)cx::perlin<8>(s_lat, 7, perlin_cs, x + j, y), (int)cx::perlin<8>(s_lat + 49, 7, perlin_cs, x + j, y),
                                        x + j, y, draw(j), (opened >> j) & 1ull));
        });
    } else if (f == 0) {
        const Field8 w16 = field16(s_lat, x, y), m16 = field16(s_lat + 16, x, y);
        const Field8 w8 = field8(s_lat + 32, x, y), m8 = field8(s_lat + 81, x, y), c8 = field8(s_lat + 130, x, y), f8 = field8(s_lat + 179, x, y);
        cells([&](int j) {
            const int Wn = (int)((3u * at16(w16, x + j) + at8(w8, x + j)) >> 2), Mn = (int)((3u * at16(m16, x + j) + at8(m8, x + j)) >> 2);
            put(j, classify_overworld(L, Wn, Mn, (int)at8(c8, x + j), (int)at8(f8, x + j), x + j, y, draw(j)));
        });
    } else if (is_dungeon(f)) {
        const int yr = CX_IDX(y, W);                                             // the run lies in one row
        const uint64_t in = (L.row_mask[M_ROOMS_A][yr] | L.row_mask[M_ROOMS_B][yr]) >> x, path = (L.row_mask[M_PATH_A][yr] | L.row_mask[M_PATH_B][yr]) >> x,
                       chest = L.row_mask[M_CHEST][yr] >> x;
        cells([&](int j) { put(j, cell_dungeon_masked(L, f, x + j, y, draw(j), (in >> j) & 1ull, (path >> j) & 1ull, (chest >> j) & 1ull)); });
    } else if (f == 8) {
#pragma unroll
        for (int j = 0; j < 4; ++j) put(j, cell_graveyard(x + j, y));
    } else {
        const Field8 c8 = field8(s_lat, x, y), f8 = field8(s_lat + 49, x, y);
        const uint64_t opened = L.row_mask[M_CAVE_OPEN][CX_IDX(y, W)] >> x;   // the run lies in one row
        cells([&](int j) { put(j, classify_cave_masked(L, f, (int)at8(c8, x + j), (int)at8(f8, x + j), x + j, y, draw(j), (opened >> j) & 1ull)); });
    }
    *reinterpret_cast<uint32_t*>(maps + block_off(f, x, y)) = pb;
    *reinterpret_cast<uint32_t*>(maps + il_off(f, x, y)) = pi;
    if (start_wb != nullptr && f == 0) {
        // window of the start cell (24, 24): rows 19..29, columns 18..30
        const int wr = y - (W / 2 - WIN_ROWS / 2);
        if ((unsigned)wr < (unsigned)WIN_ROWS) {
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const int wc = x + j - (W / 2 - WIN_COLS / 2);
                if ((unsigned)wc < (unsigned)WIN_COLS) {
                    start_wb[wr * WIN_PITCH + wc] = (uint8_t)(pb >> (8 * j));
                    start_wi[wr * WIN_PITCH + wc] = (uint8_t)(pi >> (8 * j));
                }
            }
        }
    }
    }
    __syncthreads();
}

// The ten dwords that describe a generated world beyond its maps: ladders of the nine floors and
// the potion permutation (valid in the block that generated floor 0).
__device__ inline uint32_t layout_word(const GenLayout& L, int i)
{
    if (i < FLOORS) return (uint32_t)L.up[i][0] | ((uint32_t)L.up[i][1] << 8) | ((uint32_t)L.down[i][0] << 16) | ((uint32_t)L.down[i][1] << 24);
    return L.perm;
}

// Word i (0..63) of the record of a fresh episode: player in the middle of the overworld
// facing down, vitals 9, attributes 1, boss vulnerable, floor 0 visited.
// layout: the ten layout_word values of the world.
__device__ inline uint32_t fresh_record_word(int i, const uint32_t* layout, uint32_t lo, uint32_t hi, uint32_t episode)
{
    if (i >= R_LADDER && i < R_LADDER + FLOORS) return layout[i - R_LADDER];
    switch (i) {
    case R_POS: return (uint32_t)(W / 2) | ((uint32_t)(W / 2) << 8) | (4u << 16);
    case R_FLAGS: return 1u << 17;
    case R_ATTR: return (1u << 20) | (1u << 23) | (1u << 26);
    case R_VIT: return 0x09090909u;
    case R_MANA: return 9u;
    case R_PERM: return layout[FLOORS] | (1u << 18);
    case R_EPISODE: return episode;
    case R_SEED_LO: return lo;
    case R_SEED_HI: return hi;
    default: return 0u;
    }
}

}  // namespace cf
