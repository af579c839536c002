// Observation rendering.
//  - symbolic (section "RL Environment Interface", appendix "Observation Space"): 7x9 cells
//    around the player, per cell a 17-way block one-hot plus one bit per mob type, then 22
//    scalars; flat length 63*21 + 22 = 1345.
//  - pixels: 9x9 tiles of 7x7 RGB texels from a seeded atlas, times the daylight value.
#pragma once

#include "common.hpp"

namespace cx {

constexpr int OBS_STRIDE_U8_I8 = 1360, OBS_STRIDE_U8_F32 = 1424, OBS_STRIDE_F32 = 5392, OBS_STRIDE_PIXELS = 47632;
constexpr int STAGE_CHUNKS = OBS_STRIDE_U8_F32 / 16;   // 89 uint4 of LDS staging per environment

__host__ __device__ constexpr int obs_stride(int mode)
{
    return mode == 0 ? OBS_STRIDE_U8_I8 : mode == 1 ? OBS_STRIDE_U8_F32 : mode == 2 ? OBS_STRIDE_F32 : OBS_STRIDE_PIXELS;
}

// Renders one environment's symbolic observation with the 16 lanes of its group.
// r: the environment's record in LDS (current).  stage: 89 uint4 of LDS owned by the group.
// The one-hot bytes are assembled in LDS (zero fill, then one byte store per set channel) and
// leave as 16-byte stores, so the HBM write is fully coalesced.
template <int OBS_MODE>
__device__ inline void render_symbolic(int l, const EnvRec* r, const uint8_t* __restrict__ map,
                                       const Luts* __restrict__ luts, uint4* stage, uint8_t* __restrict__ obs_out)
{
    uint8_t* sb = reinterpret_cast<uint8_t*>(stage);
#pragma unroll
    for (int i = l; i < STAGE_CHUNKS; i += G) stage[i] = make_uint4(0, 0, 0, 0);
    group_sync();
    const int px = r->px, py = r->py;
#pragma unroll
    for (int c = l; c < VIEW_ROWS * VIEW_COLS; c += G) {
        const int row = c / VIEW_COLS, col = c - row * VIEW_COLS;
        const int x = px + col - VIEW_COLS / 2, y = py + row - VIEW_ROWS / 2;
        const int b = in_map(x, y) ? (int)map[y * MAPW + x] : (int)BK_OOB;
        sb[c * NCHAN + b] = 1;
    }
    if (l < NMOB) {
        const Mob m = r->mob[l];
        const int col = (int)m.x - px + VIEW_COLS / 2, row = (int)m.y - py + VIEW_ROWS / 2;
        if (m.alive && (unsigned)col < (unsigned)VIEW_COLS && (unsigned)row < (unsigned)VIEW_ROWS)
            sb[(row * VIEW_COLS + col) * NCHAN + 17 + l / 3] = 1;
    }
#pragma unroll
    for (int i = l; i < NVEC; i += G) {
        int raw;
        if (i < 12) raw = r->inv[i];
        else if (i < 16) raw = r->vit[i - 12];
        else if (i < 20) raw = (r->dir == i - 15) ? 1 : 0;
        else if (i == 20) raw = 0;
        else raw = r->sleeping;
        if (OBS_MODE == 0) {
            if (i == 20) raw = luts->light_q7[r->phase];
            reinterpret_cast<int8_t*>(sb + VEC_OFFSET)[i] = (int8_t)raw;
        } else {
            float v;
            if (i < 6) v = luts->sqrt10[raw];
            else if (i < 12) v = (float)raw;
            else if (i < 16) v = luts->tenth[raw];
            else if (i == 20) v = luts->daylight[r->phase];
            else v = (float)raw;
            reinterpret_cast<float*>(sb + VEC_OFFSET)[i] = v;
        }
    }
    group_sync();
    if (OBS_MODE == 0 || OBS_MODE == 1) {
        uint4* out = reinterpret_cast<uint4*>(obs_out);
#pragma unroll
        for (int i = l; i < obs_stride(OBS_MODE) / 16; i += G) out[i] = stage[i];
    } else {
        // float[1345]: expand four staged bytes (or copy four staged floats) per 16-byte store
        float4* out = reinterpret_cast<float4*>(obs_out);
        const float* sv = reinterpret_cast<const float*>(sb + VEC_OFFSET);
        for (int i = l; i < OBS_STRIDE_F32 / 16; i += G) {
            float v[4];
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const int idx = 4 * i + j;
                v[j] = idx < CELL_BYTES ? (float)sb[idx] : (idx < CELL_BYTES + NVEC ? sv[idx - CELL_BYTES] : 0.0f);
            }
            out[i] = make_float4(v[0], v[1], v[2], v[3]);
        }
    }
    group_sync();   // the staging area may be reused
}

// Pixel observation of one environment by a whole block (256 threads): 63x63x3 floats.
// Each texel is one table value times the daylight value (a single IEEE multiply).
__device__ inline void render_pixels_block(const EnvRec* __restrict__ rec, const uint8_t* __restrict__ map,
                                           const Luts* __restrict__ luts, float* __restrict__ out,
                                           int* s_tile /* 81 */, int* s_ent /* 81 */)
{
    const int tid = threadIdx.x;
    const int px = rec->px, py = rec->py;
    if (tid < 81) {
        const int tr = tid / 9, tc = tid - tr * 9;
        const int x = px + tc - 4, y = py + tr - 4;
        s_tile[tid] = in_map(x, y) ? (int)map[y * MAPW + x] : (int)BK_OOB;
        s_ent[tid] = (tid == 40) ? 0 : -1;
    }
    __syncthreads();
    if (tid < NMOB) {
        const Mob m = rec->mob[tid];
        const int tc = (int)m.x - px + 4, tr = (int)m.y - py + 4;
        if (m.alive && (unsigned)tc < 9u && (unsigned)tr < 9u) s_ent[tr * 9 + tc] = 1 + tid / 3;
    }
    __syncthreads();
    const float light = luts->daylight[rec->phase];
    for (int i = tid; i < 63 * 63 * 3; i += 256) {
        const int ch = i % 3, pix = i / 3;
        const int gx = pix % 63, gy = pix / 63;
        const int tc = gx / 7, tr = gy / 7, ix = gx - tc * 7, iy = gy - tr * 7;
        const int tile = s_tile[tr * 9 + tc], ent = s_ent[tr * 9 + tc];
        const int in_tile = (iy * 7 + ix) * 3 + ch;
        float texel = luts->tile[(tile - 1) * 147 + in_tile];
        if (ent >= 0 && luts->ent_mask[ent * 49 + iy * 7 + ix]) texel = luts->ent[ent * 147 + in_tile];
        out[i] = texel * light;
    }
}

}  // namespace cx
