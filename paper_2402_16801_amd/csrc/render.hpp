// Observation rendering.
//  - symbolic (section "RL Environment Interface", appendix "Observation Space"): 7x9 cells
//    around the player, per cell a 17-way block one-hot plus one bit per mob type, then 22
//    scalars; flat length 63*21 + 22 = 1345.
//  - pixels: 9x9 tiles of 7x7 RGB texels from a seeded atlas, times the daylight value.
#pragma once

#include "common.hpp"

namespace cx {

// The two byte layouts use strides that are multiples of 128 so that every observation starts on
// a cache-line boundary and can be written as whole lines.
constexpr int OBS_STRIDE_U8_I8 = 1408, OBS_STRIDE_U8_F32 = 1536, OBS_STRIDE_F32 = 5392, OBS_STRIDE_PIXELS = 47632;
constexpr int VEC_CHUNKS_I8 = 2, VEC_CHUNKS_F32 = 6;   // 16-byte chunks that hold the 22 scalars
constexpr int CELL_CHUNKS = VEC_OFFSET / 16;   // 83 sixteen-byte chunks hold the 1323 one-hot bytes (+5 zero)

__host__ __device__ constexpr int obs_stride(int mode)
{
    return mode == 0 ? OBS_STRIDE_U8_I8 : mode == 1 ? OBS_STRIDE_U8_F32 : mode == 2 ? OBS_STRIDE_F32 : OBS_STRIDE_PIXELS;
}

// four bits -> four 0/1 bytes (bit i -> byte i)
__device__ inline uint32_t spread4(uint32_t nibble) { return (nibble * 0x00204081u) & 0x01010101u; }

// Renders one environment's symbolic observation with the G lanes of its group.
// e: the environment's LDS area; its record is current and its window holds the map around
// the window centre, with the player displaced by (mvx, mvy) from that centre and window
// column 0 at byte woff of each 16-byte row.
// The one-hot channels are collected as single bits in LDS (one atomic OR per set channel),
// then each lane expands 16 bits into a 16-byte store, so the HBM write is fully coalesced
// and the staging costs 166 bytes of LDS per environment instead of 1323.
// One 16-byte chunk of a staged observation (byte layouts): chunks 0..82 expand 16 staged bits
// each, the next 2 or 6 hold the scalars, the rest of the stride is zero.
template <int OBS_MODE, class LY = KeepLayout>
__device__ __forceinline__ uint4 staged_chunk(const uint32_t* e, int c)
{
    constexpr int NV = OBS_MODE == 0 ? VEC_CHUNKS_I8 : VEC_CHUNKS_F32;
    if (c < CELL_CHUNKS) {
        const uint32_t h = reinterpret_cast<const uint16_t*>(e + LDS_BITS)[c];
        return make_uint4(spread4(h & 15u), spread4((h >> 4) & 15u), spread4((h >> 8) & 15u), spread4(h >> 12));
    }
    if (c < CELL_CHUNKS + NV) {
        const uint32_t* v = e + LY::VEC + (c - CELL_CHUNKS) * 4;
        return make_uint4(v[0], v[1], v[2], v[3]);
    }
    return make_uint4(0u, 0u, 0u, 0u);
}

// Writes the staged observations of all environments of the calling wave (byte layouts).
// Lanes regroup into runs of max(G, 8): a run writes 128 or 256 contiguous, line-aligned bytes
// of one environment per store instruction, i.e. whole cache lines.  Plain stores: measured
// against streaming (non-temporal) ones they are 5 % faster here, the observation buffer being
// rewritten every step.  With G = 4 a run serves two environments in
// turn.  wave_env: LDS area of the wave's first environment; wave_obs: its observation.
template <int G, int OBS_MODE, class LY = KeepLayout>
__device__ __forceinline__ void flush_wave_observations(uint32_t* wave_env, uint8_t* __restrict__ wave_obs)
{
    constexpr int RUN = G < 8 ? 8 : G, PASSES = RUN / G, STRIDE = obs_stride(OBS_MODE), NCHUNK = STRIDE / 16;
    const int w = threadIdx.x & 63, run = w / RUN, j = w % RUN;
#pragma unroll
    for (int pass = 0; pass < PASSES; ++pass) {
        const int ei = run * PASSES + pass;                       // environment within the wave
        const uint32_t* e = wave_env + ei * LY::STRIDE;
        if (!e[LY::FLAG]) continue;
        uint32_t* out = reinterpret_cast<uint32_t*>(wave_obs + (size_t)ei * STRIDE);
#pragma unroll
        for (int it = 0; it < (NCHUNK + RUN - 1) / RUN; ++it) {
            const int c = it * RUN + j;
            if (c >= NCHUNK) break;
            const uint4 v = staged_chunk<OBS_MODE, LY>(e, c);
            *reinterpret_cast<uint4*>(out + 4 * c) = v;
        }
    }
}

// FILL_VEC = false: the caller has already put the 22 scalars into the LDS vector area.
// FLUSH = false: stop after staging (bits and scalars in LDS); the caller writes them out with
// flush_wave_observations.
// LY: where the scalars are staged.  With StepLayout they overwrite the record, which is read
// completely (position, tables, inventory, vitals) before the first of them is written.
template <int G, int OBS_MODE, bool FILL_VEC = true, bool FLUSH = true, class LY = KeepLayout>
__device__ __forceinline__ void render_symbolic(int l, uint32_t* e, int mvx, int mvy, int woff, const Luts* __restrict__ luts,
                                       uint8_t* __restrict__ obs_out)
{
    const uint32_t* rec = e + LDS_REC;
    const uint8_t* win = reinterpret_cast<const uint8_t*>(e + LDS_WIN);
    uint32_t* bits = e + LDS_BITS;
    static_assert(FILL_VEC || LY::VEC != LDS_REC, "scalars supplied by the caller need an area of their own");
    uint32_t* vec = e + LY::VEC;
#pragma unroll
    for (int it = 0; it < (42 + G - 1) / G; ++it) if (l + it * G < 42) bits[l + it * G] = 0u;
    group_sync();
    const uint32_t w_pos = rec[RW_POS];
    const int px = w_pos & 0xFF, py = (w_pos >> 8) & 0xFF;
    // view cells: lane l takes the columns l, l + G, ... of every row, so that the row and the
    // column group are compile-time constants and a cell costs one LDS read at a fixed offset from
    // the lane's base, one add for its bit number, and the OR
    {
        const uint8_t* cell0 = win + (1 + mvy) * WIN_PITCH + woff + 1 + mvx + l;
        const int bit0 = l * NCHAN;
#pragma unroll
        for (int row = 0; row < VIEW_ROWS; ++row) {
#pragma unroll
            for (int j = 0; j < (VIEW_COLS + G - 1) / G; ++j) {
                if (G * j + G > VIEW_COLS && l + G * j >= VIEW_COLS) continue;
                const int b = win[CX_IDX((int)(cell0 - win) + row * WIN_PITCH + G * j, WIN_ROWS * WIN_PITCH)];
                const int bit = bit0 + (row * VIEW_COLS + G * j) * NCHAN + b;
                atomicOr(&bits[CX_IDX(bit >> 5, 42)], 1u << (bit & 31));
            }
        }
    }
#pragma unroll
    for (int it_k = 0; it_k < ((NMOB) + G - 1) / G; ++it_k) {
        const int k = l + it_k * G;
        if (k >= (NMOB)) break;
        const Mob m = unpack_mob(rec[RW_MOB + k]);
        const int col = m.x - px + VIEW_COLS / 2, row = m.y - py + VIEW_ROWS / 2;
        if (m.alive && (unsigned)col < (unsigned)VIEW_COLS && (unsigned)row < (unsigned)VIEW_ROWS) {
            const int bit = (row * VIEW_COLS + col) * NCHAN + 17 + ((k * 11) >> 5);
            atomicOr(&bits[CX_IDX(bit >> 5, 42)], 1u << (bit & 31));
        }
    }
    // the 22 scalars; int8 flavour packs four per dword
    const uint32_t w_inv = rec[RW_INV], w_vit = rec[RW_VIT];
    const int dir = (w_pos >> 16) & 0xFF, sleeping = (w_pos >> 24) & 0xFF;
    const uint32_t phase = w_vit >> 16;
    auto raw_of = [&](int i) -> int {
        if (i < 6) return (w_inv >> (4 * i)) & 15;
        if (i < 12) return (w_inv >> (18 + i)) & 1;
        if (i < 16) return (w_vit >> (4 * (i - 12))) & 15;
        if (i < 20) return dir == i - 15 ? 1 : 0;
        if (i == 20) return (int)luts->light_q7[phase];
        if (i == 21) return sleeping;
        return 0;
    };
    if (!FILL_VEC) {
    } else if (OBS_MODE == 0) {
#pragma unroll
        for (int it_i = 0; it_i < ((8) + G - 1) / G; ++it_i) {
        const int i = l + it_i * G;
        if (i >= (8)) break;
            uint32_t w = 0;
#pragma unroll
            for (int j = 0; j < 4; ++j) w |= ((uint32_t)raw_of(4 * i + j) & 0xFFu) << (8 * j);
            vec[i] = w;
        }
    } else {
#pragma unroll
        for (int it_i = 0; it_i < ((24) + G - 1) / G; ++it_i) {
        const int i = l + it_i * G;
        if (i >= (24)) break;
            float v = 0.0f;
            if (i < NVEC) {
                const int raw = raw_of(i);
                if (i < 6) v = luts->sqrt10[raw];
                else if (i >= 12 && i < 16) v = luts->tenth[raw];
                else if (i == 20) v = luts->daylight[phase];
                else v = (float)raw;
            }
            vec[i] = __float_as_uint(v);
        }
    }
    group_sync();
    if (!FLUSH) return;
    if (OBS_MODE == 0 || OBS_MODE == 1) {
        uint4* out = reinterpret_cast<uint4*>(obs_out);
#pragma unroll
        for (int it_i = 0; it_i < ((obs_stride(OBS_MODE) / 16) + G - 1) / G; ++it_i) {
            const int i = l + it_i * G;
            if (i >= (obs_stride(OBS_MODE) / 16)) break;
            out[i] = staged_chunk<OBS_MODE, LY>(e, i);
        }
    } else {
        // float[1345]: four values per 16-byte store
        float4* out = reinterpret_cast<float4*>(obs_out);
        for (int it_i = 0; it_i < ((OBS_STRIDE_F32 / 16) + G - 1) / G; ++it_i) {
        const int i = l + it_i * G;
        if (i >= (OBS_STRIDE_F32 / 16)) break;
            float v[4];
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const int idx = 4 * i + j;
                if (idx < CELL_BYTES) v[j] = (float)((bits[idx >> 5] >> (idx & 31)) & 1u);
                else if (idx < CELL_BYTES + NVEC) v[j] = __uint_as_float(vec[idx - CELL_BYTES]);
                else v[j] = 0.0f;
            }
            out[i] = make_float4(v[0], v[1], v[2], v[3]);
        }
    }
    group_sync();   // the staging area may be reused
}

// Pixel observation of one environment by a whole block (256 threads): 63x63x3 floats.
// Each texel is one table value times the daylight value (a single IEEE multiply).
// The picture is walked in linear pixel order, 1024 pixels per block iteration, 256 per wave:
// every lane fetches the three texels of four pixels (the atlas stays in cache), scales them and
// parks them in a wave-private LDS strip, from which every lane writes three aligned 16-byte
// pieces; 12-byte stores at a 12-byte lane stride reach only half the write bandwidth.  The
// fetches of the next group are issued before the stores of the current one.
constexpr int PIX_SIDE = 63, PIX_TILE = 7, PIX_TILE_FLOATS = PIX_TILE * PIX_TILE * 3, PIX_VIEW = 9;
constexpr int PIX_GROUP = 1024, PIX_WAVE = 256, PIX_WAVE_FLOATS = PIX_WAVE * 3;
constexpr int PIX_FULL_GROUPS = OBS_STRIDE_PIXELS / 12 / PIX_GROUP;   // 3 whole groups, then a partial one
static_assert((PIX_FULL_GROUPS + 1) * PIX_GROUP * 12 >= OBS_STRIDE_PIXELS && PIX_FULL_GROUPS * PIX_GROUP <= PIX_SIDE * PIX_SIDE, "pixel groups");

// s_tile, s_ent: 81 ints each; s_strip: 4 * 768 floats, 16-byte aligned.  Writes the whole stride
// (the padding after the picture as zero).
__device__ __forceinline__ void render_pixels_block(const uint32_t* __restrict__ rec, const uint8_t* __restrict__ map,
                                                    const Luts* __restrict__ luts, uint8_t* __restrict__ obs_out,
                                                    int* s_tile, int* s_ent, float* s_strip)
{
    const int tid = threadIdx.x;
    const uint32_t w_pos = rec[RW_POS];
    const int px = w_pos & 0xFF, py = (w_pos >> 8) & 0xFF;
    if (tid < PIX_VIEW * PIX_VIEW) {
        const int tr = tid / PIX_VIEW, tc = tid - tr * PIX_VIEW;
        const int x = px + tc - PIX_VIEW / 2, y = py + tr - PIX_VIEW / 2;
        // ids outside 1..16 would index before or past the atlas: they are drawn as the out-of-bounds tile
        const int b = in_map(x, y) ? (int)map[map_index(x, y)] : (int)BK_OOB;
        s_tile[tid] = (unsigned)(b - 1) < 16u ? b : (int)BK_OOB;
        s_ent[tid] = (tid == PIX_VIEW * PIX_VIEW / 2) ? 0 : -1;
    }
    __syncthreads();
    if (tid < NMOB) {
        const Mob m = unpack_mob(rec[RW_MOB + tid]);
        const int tc = m.x - px + PIX_VIEW / 2, tr = m.y - py + PIX_VIEW / 2;
        if (m.alive && (unsigned)tc < (unsigned)PIX_VIEW && (unsigned)tr < (unsigned)PIX_VIEW) s_ent[tr * PIX_VIEW + tc] = 1 + tid / 3;
    }
    __syncthreads();
    const float light = luts->daylight[rec[RW_VIT] >> 16];
    float4* out = reinterpret_cast<float4*>(obs_out);
    const int w = tid >> 6, l = tid & 63;
    float* strip = s_strip + w * PIX_WAVE_FLOATS;
    float v[4][3], scale[4];
    auto fetch = [&](int g) {
        const int p0 = g * PIX_GROUP + w * PIX_WAVE + l;
        int y = p0 / PIX_SIDE, x = p0 - y * PIX_SIDE;
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            // pixels beyond the picture (the stride's padding) read texel 0 at scale 0
            const bool valid = y < PIX_SIDE;
            const int yy = valid ? y : 0;
            const int tr = yy / PIX_TILE, iy = yy - tr * PIX_TILE, tc = x / PIX_TILE, ix = x - tc * PIX_TILE;
            const int tile = s_tile[CX_IDX(tr * PIX_VIEW + tc, PIX_VIEW * PIX_VIEW)], ent = s_ent[CX_IDX(tr * PIX_VIEW + tc, PIX_VIEW * PIX_VIEW)];
            const int in_tile = (iy * PIX_TILE + ix) * 3;
            const float* src = luts->tile + CX_IDX((tile - 1) * PIX_TILE_FLOATS + in_tile, 16 * PIX_TILE_FLOATS - 2);
            if (ent >= 0 && luts->ent_mask[CX_IDX(ent * (PIX_TILE * PIX_TILE) + iy * PIX_TILE + ix, 5 * PIX_TILE * PIX_TILE)]) src = luts->ent + CX_IDX(ent * PIX_TILE_FLOATS + in_tile, 5 * PIX_TILE_FLOATS - 2);
            v[u][0] = src[0]; v[u][1] = src[1]; v[u][2] = src[2];
            scale[u] = valid ? light : 0.0f;
            x += 64;
            if (x >= PIX_SIDE) { x -= PIX_SIDE; ++y; }
            if (x >= PIX_SIDE) { x -= PIX_SIDE; ++y; }            // 64 pixels on is one row and one pixel further
        }
    };
    float4 piece[3];
    auto turn = [&]() {
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            strip[u * 192 + l * 3] = v[u][0] * scale[u];
            strip[u * 192 + l * 3 + 1] = v[u][1] * scale[u];
            strip[u * 192 + l * 3 + 2] = v[u][2] * scale[u];
        }
        group_sync();
#pragma unroll
        for (int k = 0; k < 3; ++k) piece[k] = *reinterpret_cast<const float4*>(strip + (k * 64 + l) * 4);
        group_sync();
    };
    auto store = [&](int g, bool guarded) {
#pragma unroll
        for (int k = 0; k < 3; ++k) {
            const int q = (g * PIX_GROUP + w * PIX_WAVE) * 3 / 4 + k * 64 + l;
            if (!guarded || q < OBS_STRIDE_PIXELS / 16) {
                __builtin_nontemporal_store(piece[k].x, &out[q].x);
                __builtin_nontemporal_store(piece[k].y, &out[q].y);
                __builtin_nontemporal_store(piece[k].z, &out[q].z);
                __builtin_nontemporal_store(piece[k].w, &out[q].w);
            }
        }
    };
    fetch(0);
    turn();
    fetch(1);
    store(0, false);
#pragma unroll 1
    for (int g = 1; g < PIX_FULL_GROUPS; ++g) {
        turn();
        fetch(g + 1);
        store(g, false);
    }
    turn();
    store(PIX_FULL_GROUPS, true);
}

}  // namespace cx
