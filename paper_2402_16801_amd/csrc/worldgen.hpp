// Block-cooperative generation of one 64x64 Craftax-Classic world (appendix "World
// Generation" of the paper: noise thresholds carve grassland, forest, lakes, mountains with
// caves, tunnels, ores and lava).  Two noises feed the same rule: seeded integer value noise
// (the benchmark configurations) and Perlin gradient noise as the paper uses, evaluated in
// integers; either way every cell is a pure integer function of (seed, env, episode).
#pragma once

#include "common.hpp"

namespace cx {

constexpr int LAT16_N = 25;   // 5x5 lattice points at spacing 16
constexpr int LAT8_N = 81;    // 9x9 lattice points at spacing 8
constexpr int LAT_TOTAL = 2 * LAT16_N + 4 * LAT8_N;   // 374 u16 values
constexpr int LAT_BLOCKS = (LAT_TOTAL + 7) / 8;       // Philox blocks holding them (8 u16 each)

// terrain thresholds on 0..65535 scales
constexpr int TH_MOUNTAIN = 39500, TH_CAVE_M = 41000, TH_CAVE_C = 43000;
constexpr int TH_TUNNEL_CENTER = 30000, TH_TUNNEL_HALF = 1300;
constexpr int TH_LAVA_M = 43000, TH_LAVA_F = 44000, TH_DIAMOND_M = 42000;
constexpr int U_DIAMOND = 500, U_IRON = 3000, TH_IRON_F = 33000, U_COAL = 8000;
constexpr int TH_WATER = 39500, TH_SAND = 37800, TH_FOREST_F = 33500;
constexpr int U_TREE_FOREST = 26000, U_TREE_SPARSE = 1300;
constexpr int START_CLEAR = 2, START_BIAS_R = 10, START_BIAS = 2500;

// smoothstep(k/S) in 1/256 units for S = 8 and S = 16
__device__ inline uint32_t smooth8(int k) { return (uint32_t)(12 * k * k - k * k * k); }
__device__ inline uint32_t smooth16(int k) { return (uint32_t)((24 * k * k - k * k * k + 4) >> 3); }

// Bilinear value noise, evaluated column-first: the caller blends the two lattice rows once
// per lattice column (vertical weight wy), then every cell of the run blends two columns
// (horizontal weight wx).  The integer result equals the row-first formula
// ((a(256-wx)+b wx)(256-wy) + (c(256-wx)+d wx) wy) >> 16 because nothing is rounded before
// the final shift and every intermediate fits in 32 bits.
__device__ inline uint32_t column(const uint16_t* lat, int width, int ix, int iy, uint32_t wy)
{
    return (uint32_t)lat[CX_IDX(iy * width + ix, width * width)] * (256u - wy) + (uint32_t)lat[CX_IDX((iy + 1) * width + ix, width * width)] * wy;
}
__device__ inline uint32_t across(uint32_t left, uint32_t right, uint32_t wx)
{
    return (left * (256u - wx) + right * wx) >> 16;
}

// Perlin gradient noise (appendix "World Generation"): the lattice numbers are read as one of 1024
// directions (top ten bits); cs[a] holds the unit gradient of direction a in Q14.  S is the
// lattice spacing; offsets from the four corners are in units of 1/S; the fade weight
// 6t^5 - 15t^4 + 10t^3 of t = k/S is (F 65536 + S^5 / 2) / S^5 in Q16 with
// F = k^3 (6 k^2 - 15 k S + 10 S^2); blends are p + floor((q - p) w / 65536), along x then y; the
// value, in units of 1 / (16384 S), lands on the 0..65535 scale of the thresholds as
// 32768 + floor(n * 3900 / (1024 S)), clamped.  All divisors are powers of two: floors are shifts.
constexpr int PERLIN_GAIN = 3900;
template <int S>
__device__ inline int64_t perlin_fade(int k)
{
    const int F = k * k * k * (6 * k * k - 15 * k * S + 10 * S * S);
    return S == 16 ? (int64_t)((F + 8) >> 4) : (int64_t)(2 * F);
}
__device__ inline int64_t perlin_blend(int64_t p, int64_t q, int64_t w) { return p + (((q - p) * w) >> 16); }
template <int S>
__device__ inline uint32_t perlin(const uint16_t* lat, int width, const uint32_t* __restrict__ cs, int x, int y)
{
    static_assert(S == 8 || S == 16, "lattice spacing");
    constexpr int SHIFT = S == 16 ? 4 : 3;
    const int ix = x >> SHIFT, iy = y >> SHIFT, kx = x & (S - 1), ky = y & (S - 1);
    int64_t dot[2][2];
#pragma unroll
    for (int cy = 0; cy < 2; ++cy)
#pragma unroll
        for (int cx = 0; cx < 2; ++cx) {
            const uint32_t g = cs[lat[CX_IDX((iy + cy) * width + ix + cx, width * width)] >> 6];
            dot[cy][cx] = (int64_t)((int)(int16_t)(g & 0xFFFFu) * (kx - cx * S) + (int)(int16_t)(g >> 16) * (ky - cy * S));
        }
    const int64_t wx = perlin_fade<S>(kx), wy = perlin_fade<S>(ky);
    const int64_t n = perlin_blend(perlin_blend(dot[0][0], dot[0][1], wx), perlin_blend(dot[1][0], dot[1][1], wx), wy);
    const int64_t v = 32768 + ((n * PERLIN_GAIN) >> (10 + SHIFT));
    return (uint32_t)(v < 0 ? 0 : (v > 65535 ? 65535 : v));
}

__device__ inline int classify(int W, int M, int C, int F, int x, int y, int u)
{
    const int d = max(iabs(x - MAPW / 2), iabs(y - MAPW / 2));
    if (d < START_BIAS_R) {
        const int bias = (START_BIAS_R - d) * START_BIAS;
        W = max(0, W - bias);
        M = max(0, M - bias);
    }
    if (d <= START_CLEAR) return BK_GRASS;
    if (M > TH_MOUNTAIN) {
        if (C > TH_CAVE_C && M > TH_CAVE_M) return BK_PATH;
        if (iabs(C - TH_TUNNEL_CENTER) < TH_TUNNEL_HALF) return BK_PATH;
        if (M > TH_LAVA_M && F > TH_LAVA_F) return BK_LAVA;
        if (M > TH_DIAMOND_M && u < U_DIAMOND) return BK_DIAMOND;
        if (F < TH_IRON_F && u >= U_DIAMOND && u < U_IRON) return BK_IRON;
        if (u >= U_IRON && u < U_COAL) return BK_COAL;
        return BK_STONE;
    }
    if (W > TH_WATER) return BK_WATER;
    if (W > TH_SAND) return BK_SAND;
    if (F > TH_FOREST_F && u < U_TREE_FOREST) return BK_TREE;
    if (u < U_TREE_SPARSE) return BK_TREE;
    return BK_GRASS;
}

// Generates the map of one environment, or a part of it, with the NT threads of the calling
// block: run t owns the 8 cells [8t, 8t+8) of row t/8, which are exactly one spacing-8
// lattice cell wide (and inside one spacing-16 cell), and whose per-cell uniforms are
// exactly Philox block t of stream 1.  A reset is latency-bound, so the work is cut into
// many short threads and two such blocks fit on a compute unit.
// s_lat: LDS scratch of at least LAT_BLOCKS*8 u16.  Ends with a block barrier, after which
// the map is visible to the whole block.
constexpr int WG_THREADS = 512;

// start_win (may be null): LDS window (9 rows x 4 dwords) of the start position (32, 32); the
// threads that own those cells drop them there, so the first observation of the new episode
// can be rendered without reading the map back.
// first_run, runs: the part of the world this call generates (runs first_run .. first_run + runs - 1
// of the 512; a world may be split over several blocks); runs <= NT.
// PERLIN: the fields are Perlin noise over the same lattices (perlin_cs: the gradient table).
// theta (may be null; LDS or global, LAT_TOTAL values): angle offsets of a mutated level.
// STRIPS: how the runs are dealt to the wavefronts (see below); the rollout kernel, which is short of
// registers, keeps the plain order.
template <int NT = WG_THREADS, bool PERLIN = false, bool STRIPS = true>
__device__ __forceinline__ void worldgen_block(uint8_t* __restrict__ map, uint16_t* s_lat, uint32_t seed_lo, uint32_t seed_hi,
                                      uint32_t env, uint32_t episode, uint32_t* start_win = nullptr, int first_run = 0,
                                      int runs = WG_THREADS, const uint32_t* __restrict__ perlin_cs = nullptr,
                                      const uint16_t* theta = nullptr)
{
    static_assert(WG_THREADS % NT == 0 && NT >= 64, "block size must divide 512");
    // runs is 512 (a world) or 256 (half of one): whole wavefronts, and a number of them that divides the eight runs of a row
    const int tid0 = threadIdx.x;
    const int tid = tid0;
    if (tid < LAT_BLOCKS) {
        const U4 r = philox4x32_10(env, 0u, episode, (DOM_WORLDGEN << 16) | (uint32_t)tid, seed_lo, seed_hi);
#pragma unroll
        for (int w = 0; w < 4; ++w) {
            s_lat[tid * 8 + 2 * w] = (uint16_t)(r.w[w] & 0xFFFFu);
            s_lat[tid * 8 + 2 * w + 1] = (uint16_t)(r.w[w] >> 16);
        }
        // a mutated level (section "Craftax-1B: UED"): every gradient angle, the upper ten bits of its
        // lattice number, turned by theta[i] 1024ths of a turn
        if (theta != nullptr) {
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                const int i = tid * 8 + j;
                if (i < LAT_TOTAL) s_lat[i] = (uint16_t)(s_lat[i] + ((theta[i] & 1023u) << 6));
            }
        }
    }
    __syncthreads();
    // one run of 8 cells per thread (the callers give a block no more runs than it has threads)
    if (tid0 < runs) {
    // Which run a thread takes: a wavefront owns a strip of columns over all rows of the part (one
    // run wide when the part is the whole world, two when it is half of it) rather than eight whole
    // rows.  A strip is all plain or all mountain more often than eight rows across the world, so
    // the terrain rule's branches are skipped more often, and the 16 lanes that fill a map tile are
    // neighbours.  Only the assignment changes: run `tid` is the same cells and draws as ever.
    const int waves = runs >> 6, strip = 8 / waves, wl = tid0 & 63, ww = tid0 >> 6;
    const int tid = first_run + (STRIPS ? (wl / strip) * 8 + ww * strip + (wl % strip) : tid0);
    const U4 r = philox4x32_10(env, 1u, episode, (DOM_WORLDGEN << 16) | (uint32_t)tid, seed_lo, seed_hi);
    const int y = tid >> 3, x0 = (tid & 7) << 3;
    const uint16_t* w16 = s_lat;
    const uint16_t* m16 = s_lat + LAT16_N;
    const uint16_t* w8 = s_lat + 2 * LAT16_N;
    const uint16_t* m8 = w8 + LAT8_N;
    const uint16_t* c8 = m8 + LAT8_N;
    const uint16_t* f8 = c8 + LAT8_N;
    const int iy16 = y >> 4, iy8 = y >> 3, ix16 = x0 >> 4, ix8 = x0 >> 3;
    const uint32_t wy16 = smooth16(y & 15), wy8 = smooth8(y & 7);
    const uint32_t W16a = column(w16, 5, ix16, iy16, wy16), W16b = column(w16, 5, ix16 + 1, iy16, wy16);
    const uint32_t M16a = column(m16, 5, ix16, iy16, wy16), M16b = column(m16, 5, ix16 + 1, iy16, wy16);
    const uint32_t Wl = column(w8, 9, ix8, iy8, wy8), Wr = column(w8, 9, ix8 + 1, iy8, wy8);
    const uint32_t Ml = column(m8, 9, ix8, iy8, wy8), Mr = column(m8, 9, ix8 + 1, iy8, wy8);
    const uint32_t Cl = column(c8, 9, ix8, iy8, wy8), Cr = column(c8, 9, ix8 + 1, iy8, wy8);
    const uint32_t Fl = column(f8, 9, ix8, iy8, wy8), Fr = column(f8, 9, ix8 + 1, iy8, wy8);
    uint32_t packed[2] = { 0u, 0u };
#pragma unroll
    for (int j = 0; j < 8; ++j) {
        const int x = x0 + j;
        const uint32_t rw = r.w[j >> 1];
        const int u = (int)((j & 1) ? (rw >> 16) : (rw & 0xFFFFu));
        int W, M, C, F;
        if (PERLIN) {
            W = (int)((3u * perlin<16>(w16, 5, perlin_cs, x, y) + perlin<8>(w8, 9, perlin_cs, x, y)) >> 2);
            M = (int)((3u * perlin<16>(m16, 5, perlin_cs, x, y) + perlin<8>(m8, 9, perlin_cs, x, y)) >> 2);
            C = (int)perlin<8>(c8, 9, perlin_cs, x, y);
            F = (int)perlin<8>(f8, 9, perlin_cs, x, y);
        } else {
            const uint32_t wx8 = smooth8(j), wx16 = smooth16(x & 15);
            W = (int)((3u * across(W16a, W16b, wx16) + across(Wl, Wr, wx8)) >> 2);
            M = (int)((3u * across(M16a, M16b, wx16) + across(Ml, Mr, wx8)) >> 2);
            C = (int)across(Cl, Cr, wx8);
            F = (int)across(Fl, Fr, wx8);
        }
        packed[j >> 2] |= (uint32_t)classify(W, M, C, F, x, y, u) << (8 * (j & 3));
    }
    *reinterpret_cast<uint2*>(map + map_index(x0, y)) = make_uint2(packed[0], packed[1]);   // 8 cells inside one tile row
    {
        // window of the start cell: rows 28..36, columns 24..39 (aligned start of 32-5)
        constexpr int WY0 = MAPW / 2 - WIN_ROWS / 2, WX0 = (MAPW / 2 - WIN_COLS / 2) & ~3;
        const int wr = y - WY0, wc = x0 - WX0;
        if (start_win != nullptr && (unsigned)wr < (unsigned)WIN_ROWS && (unsigned)wc < (unsigned)WIN_PITCH) {
            start_win[CX_IDX(wr * (WIN_PITCH / 4) + wc / 4, WIN_DWORDS)] = packed[0];
            start_win[CX_IDX(wr * (WIN_PITCH / 4) + wc / 4 + 1, WIN_DWORDS)] = packed[1];
        }
    }
    }
    __syncthreads();
}

// Word i of a fresh record: full vitals, empty tables, player in the middle facing down.
__device__ inline uint32_t fresh_record_word(int i, uint32_t seed_lo, uint32_t seed_hi, uint32_t episode)
{
    switch (i) {
    case RW_POS: return (uint32_t)(MAPW / 2) | ((uint32_t)(MAPW / 2) << 8) | (4u << 16);
    case RW_VIT: return (uint32_t)MAX_COUNT * 0x1111u;
    case RW_EPISODE: return episode;
    case RW_SEED_LO: return seed_lo;
    case RW_SEED_HI: return seed_hi;
    default: return 0u;
    }
}

}  // namespace cx
