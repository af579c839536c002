// Pixel observation of full Craftax (section "RL Environment Interface": 110 x 130 x 3 floats;
// appendix "Observation Space": 10-pixel tiles).  The paper's textures are not available, so the
// tiles come from a seeded atlas: the 9 x 11 view, one tile per cell, then four rows of eleven
// inventory slots.
//   view cell : block tile; the pixels that the one-bit masks of an item, then of a creature,
//               then of the player (centre cell) select are replaced by those tiles; the texel is
//               multiplied once by light level / 20.  Cells beyond the map edge show block 1 at
//               full light.
//   slot j    : icon tile j times min(scalar j of the symbolic observation, 1), j = 0..43.
// One block per environment.  Thread t < 220 owns pixel column t % 110 of the two image rows an
// iteration covers, so one iteration writes 2640 contiguous bytes and everything that depends on
// the column (tile column, offset inside the tile) is computed once.  The work per pixel is one
// 12-byte atlas read (cache resident: the atlas is 152 KB), three multiplies and one 12-byte
// store; the kernel is bound by its 171,600 bytes of output per environment.
#pragma once

#include "full_render.hpp"

namespace cf {

constexpr int PIX_ROWS = 130, PIX_COLS = 110, TILE_PX = 10, TILE_FLOATS = TILE_PX * TILE_PX * 3;
constexpr int TILE_ROWS = 13, STRIP_SLOTS = 44;
constexpr int STRIDE_PIXELS = 171648;                         // 171,600 bytes of pixels + padding to whole cache lines
constexpr int NO_TILE = 0xFF;

__global__ __launch_bounds__(BLOCK) void kf_pixels(const uint32_t* __restrict__ envs, const uint8_t* __restrict__ maps,
                                                   const Luts* __restrict__ luts, uint8_t* __restrict__ obs)
{
    __shared__ uint32_t s_rec[REC_DWORDS];
    __shared__ uint32_t s_cre[NCELL];
    __shared__ uint32_t s_tile[TILE_ROWS * VCOLS];            // base tile | item tile << 8 | creature tile << 16 | player << 24
    __shared__ float s_scale[TILE_ROWS * VCOLS];
    const int env = blockIdx.x, tid = threadIdx.x;
    const uint32_t* genv = envs + (size_t)env * ENV_DWORDS;
    if (tid < REC_DWORDS) s_rec[tid] = genv[tid];
    else if (tid - REC_DWORDS < NCELL) s_cre[tid - REC_DWORDS] = 0xFFFFFFFFu;
    __syncthreads();
    const uint32_t pos = s_rec[R_POS];
    const int px = pos & 0xFF, py = (pos >> 8) & 0xFF, f = (pos >> 24) & 0xF;
    const uint8_t* m = maps + map_offset((uint32_t)env, s_rec[R_EPISODE]);
    if (tid < NSLOT) {
        const Mob u = unpack_mob(genv[REC_DWORDS + f * MOBTAB_DWORDS + tid]);
        const int vr = (int)u.y - (py - VROWS / 2), vc = (int)u.x - (px - VCOLS / 2);
        if (u.alive && (unsigned)vr < (unsigned)VROWS && (unsigned)vc < (unsigned)VCOLS)
            atomicMin(&s_cre[vr * VCOLS + vc], ((uint32_t)tid << 8) | (uint32_t)(creature_channel(tid, (int)u.type) - 42));   // lowest slot wins
    }
    __syncthreads();
    if (tid < TILE_ROWS * VCOLS) {
        uint32_t info;
        float scale;
        if (tid < NCELL) {
            const int r = tid / VCOLS, c = tid - r * VCOLS;
            const int x = px - VCOLS / 2 + c, y = py - VROWS / 2 + r;
            int block = B_OOB, item = IT_NONE, lv = MAX_LIGHT;
            uint32_t cre = NO_TILE;
            if (inb(x, y)) {
                block = m[block_off(f, x, y)] & 63;
                const int il = m[il_off(f, x, y)];
                item = il & 7; lv = il >> 3;
                const uint32_t cr = s_cre[tid];
                if (cr != 0xFFFFFFFFu) cre = AT_CRE + (cr & 0xFFu);
            }
            info = (uint32_t)block | ((item != IT_NONE ? (uint32_t)(AT_ITEM + item) : (uint32_t)NO_TILE) << 8) | (cre << 16)
                 | ((x == px && y == py) ? 1u << 24 : 0u);
            scale = luts->light20[lv];
        } else {
            const int j = tid - NCELL;
            info = (uint32_t)(AT_ICON + j) | ((uint32_t)NO_TILE << 8) | ((uint32_t)NO_TILE << 16);
            scale = fminf(scalar_value(j, s_rec, luts), 1.0f);
        }
        s_tile[tid] = info;
        s_scale[tid] = scale;
    }
    __syncthreads();
    float* out = reinterpret_cast<float*>(obs + (size_t)env * STRIDE_PIXELS);
    if (tid >= 2 * PIX_COLS) {      // the stride's padding
        if (tid - 2 * PIX_COLS < (STRIDE_PIXELS - PIX_ROWS * PIX_COLS * 12) / 4) out[PIX_ROWS * PIX_COLS * 3 + tid - 2 * PIX_COLS] = 0.0f;
        return;
    }
    const int half = tid >= PIX_COLS ? 1 : 0, x = tid - half * PIX_COLS;
    const int tc = x / TILE_PX, xi = x - tc * TILE_PX;
    const float* atlas = luts->atlas;
#pragma unroll 1
    for (int tr = 0; tr < TILE_ROWS; ++tr) {
        const uint32_t info = s_tile[tr * VCOLS + tc];
        const float scale = s_scale[tr * VCOLS + tc];
        const int base = info & 0xFF;
        const bool plain = (info >> 8) == 0xFFFFu;            // no item, no creature, not the player's cell
#pragma unroll
        for (int k = 0; k < TILE_PX / 2; ++k) {
            const int yi = 2 * k + half;
            int tile = base;
            if (!plain) {
                const int item = (info >> 8) & 0xFF, cre = (info >> 16) & 0xFF;
                if (item != NO_TILE && ((luts->mask[item - AT_ITEM][yi] >> xi) & 1u)) tile = item;
                if (cre != NO_TILE && ((luts->mask[MASK_CRE + cre - AT_CRE][yi] >> xi) & 1u)) tile = cre;
                if ((info >> 24) && ((luts->mask[MASK_PLAYER][yi] >> xi) & 1u)) tile = AT_PLAYER;
            }
            const float* src = atlas + tile * TILE_FLOATS + yi * (TILE_PX * 3) + xi * 3;
            float* dst = out + ((tr * TILE_PX + yi) * PIX_COLS + x) * 3;
            const float r = src[0], g = src[1], b = src[2];
            __builtin_nontemporal_store(r * scale, dst);
            __builtin_nontemporal_store(g * scale, dst + 1);
            __builtin_nontemporal_store(b * scale, dst + 2);
        }
    }
}

}  // namespace cf
