// Pixel observation of full Craftax (section "RL Environment Interface": 110 x 130 x 3 floats;
// appendix "Observation Space": 10-pixel tiles).  The paper's textures are not available, so the
// tiles come from a seeded atlas: the 9 x 11 view, one tile per cell, then four rows of eleven
// inventory slots.
//   view cell : block tile; the pixels that the one-bit masks of an item, then of a creature,
//               then of the player (centre cell) select are replaced by those tiles; the texel is
//               multiplied once by light level / 20.  Cells beyond the map edge show block 1 at
//               full light.
//   slot j    : icon tile j times min(scalar j of the symbolic observation, 1), j = 0..43.
// One block per environment.  The picture is walked in linear pixel order, 1024 pixels (whole
// cache lines) per block iteration, 256 per wave: every lane fetches the three texels of four
// pixels (the atlas is 152 KB and stays in cache), scales them and parks them in a wave-private
// LDS strip, from which every lane writes three aligned 16-byte pieces -- 12-byte stores at a
// 12-byte lane stride reach only half the write bandwidth.  The kernel is bound by its 171,600
// bytes of output per environment.
#pragma once

#include "full_render.hpp"

namespace cf {

constexpr int PIX_ROWS = 130, PIX_COLS = 110, TILE_PX = 10, TILE_FLOATS = TILE_PX * TILE_PX * 3;
constexpr int TILE_ROWS = 13, STRIP_SLOTS = 44;
constexpr int STRIDE_PIXELS = 171648;                         // 171,600 bytes of pixels + padding to whole cache lines
constexpr int NO_TILE = 0xFF;
constexpr int PIX_UNROLL = 4, WAVE_PIXELS = 64 * PIX_UNROLL, GROUP_PIXELS = WAVE_PIXELS * (BLOCK / 64), WAVE_FLOATS = WAVE_PIXELS * 3;
constexpr int FULL_GROUPS = STRIDE_PIXELS / 12 / GROUP_PIXELS;   // 13 whole groups of 1024 pixels, then a partial one
static_assert((FULL_GROUPS + 1) * GROUP_PIXELS * 12 >= STRIDE_PIXELS && FULL_GROUPS * GROUP_PIXELS <= PIX_ROWS * PIX_COLS, "pixel groups");

__global__ __launch_bounds__(BLOCK) void kf_pixels(const uint32_t* __restrict__ envs, const uint8_t* __restrict__ maps,
                                                   const Luts* __restrict__ luts, uint8_t* __restrict__ obs)
{
    __shared__ uint32_t s_rec[REC_DWORDS];
    __shared__ uint32_t s_cre[NCELL];
    __shared__ uint32_t s_tile[TILE_ROWS * VCOLS];            // base tile | item tile << 8 | creature tile << 16 | player << 24
    __shared__ float s_scale[TILE_ROWS * VCOLS];
    __shared__ __attribute__((aligned(4))) uint16_t s_mask[46 * TILE_PX];
    __shared__ __attribute__((aligned(16))) float s_strip[(BLOCK / 64) * WAVE_FLOATS];
    const int env = blockIdx.x, tid = threadIdx.x;
    const uint32_t* genv = envs + (size_t)env * ENV_DWORDS;
    if (tid < REC_DWORDS) s_rec[tid] = genv[tid];
    if (tid < 46 * TILE_PX / 2) reinterpret_cast<uint32_t*>(s_mask)[tid] = reinterpret_cast<const uint32_t*>(&luts->mask[0][0])[tid];
    if (tid < NCELL) s_cre[tid] = 0xFFFFFFFFu;
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
                block = min((int)m[block_off(f, x, y)], (int)B_COUNT - 1);     // ids beyond the table would index past the atlas
                const int il = m[il_off(f, x, y)];
                item = min(il & 7, (int)IT_COUNT - 1); lv = il >> 3;
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
    float4* out = reinterpret_cast<float4*>(obs + (size_t)env * STRIDE_PIXELS);
    const int w = tid >> 6, l = tid & 63;
    const float* atlas = luts->atlas;
    float* strip = s_strip + w * WAVE_FLOATS;
    auto covered = [&](int overlay, int yi, int xi) { return (s_mask[overlay * TILE_PX + yi] >> xi) & 1u; };
    float v[PIX_UNROLL][3], scale[PIX_UNROLL];
    // Group g of the picture is 1024 consecutive pixels, 256 per wave, 4 per lane (64 apart).
    // fetch: the texels of this lane's four pixels of group g.
    auto fetch = [&](int g) {
        const int p0 = g * GROUP_PIXELS + w * WAVE_PIXELS + l;
        int y = p0 / PIX_COLS, x = p0 - y * PIX_COLS;
#pragma unroll
        for (int u = 0; u < PIX_UNROLL; ++u) {
            // pixels beyond the picture (the stride's padding) read texel 0 at scale 0
            const bool valid = y < PIX_ROWS;
            const int yy = valid ? y : 0;
            const int tr = yy / TILE_PX, yi = yy - tr * TILE_PX, tc = x / TILE_PX, xi = x - tc * TILE_PX;
            const uint32_t info = s_tile[tr * VCOLS + tc];
            scale[u] = valid ? s_scale[tr * VCOLS + tc] : 0.0f;
            int tile = info & 0xFF;
            if ((info >> 8) != 0xFFFFu) {                     // an item, a creature or the player on this cell
                const int item = (info >> 8) & 0xFF, cre = (info >> 16) & 0xFF;
                if (item != NO_TILE && covered(item - AT_ITEM, yi, xi)) tile = item;
                if (cre != NO_TILE && covered(MASK_CRE + cre - AT_CRE, yi, xi)) tile = cre;
                if ((info >> 24) && covered(MASK_PLAYER, yi, xi)) tile = AT_PLAYER;
            }
            const float* src = atlas + (uint32_t)(tile * TILE_FLOATS + yi * (TILE_PX * 3) + xi * 3);
            v[u][0] = src[0]; v[u][1] = src[1]; v[u][2] = src[2];
            x += 64;
            if (x >= PIX_COLS) { x -= PIX_COLS; ++y; }
        }
    };
    // turn: scales the fetched texels and regroups the wave's 768 floats through LDS so that
    // lane l holds the 16-byte pieces l, l + 64 and l + 128 of the wave's part of the output
    float4 piece[3];
    auto turn = [&]() {
#pragma unroll
        for (int u = 0; u < PIX_UNROLL; ++u) {
            strip[u * 192 + l * 3] = v[u][0] * scale[u];
            strip[u * 192 + l * 3 + 1] = v[u][1] * scale[u];
            strip[u * 192 + l * 3 + 2] = v[u][2] * scale[u];
        }
        wave_sync();
#pragma unroll
        for (int k = 0; k < 3; ++k) piece[k] = *reinterpret_cast<const float4*>(strip + (k * 64 + l) * 4);
        wave_sync();
    };
    auto store = [&](int g, bool guarded) {
#pragma unroll
        for (int k = 0; k < 3; ++k) {
            const int q = (g * GROUP_PIXELS + w * WAVE_PIXELS) * 3 / 4 + k * 64 + l;
            if (!guarded || q < STRIDE_PIXELS / 16) {
                __builtin_nontemporal_store(piece[k].x, &out[q].x);
                __builtin_nontemporal_store(piece[k].y, &out[q].y);
                __builtin_nontemporal_store(piece[k].z, &out[q].z);
                __builtin_nontemporal_store(piece[k].w, &out[q].w);
            }
        }
    };
    // The fetches of the next group are issued before the stores of this one: the memory
    // operations of a wave complete in order, so neither waits for the other's round trip.  The
    // first group is peeled so that the loop is entered with the same operations in flight as
    // its back edge has, and the last, partial group is stored under a bounds check.
    fetch(0);
    turn();
    fetch(1);
    store(0, false);
#pragma unroll 1
    for (int g = 1; g < FULL_GROUPS; ++g) {
        turn();
        fetch(g + 1);
        store(g, false);
    }
    turn();
    store(FULL_GROUPS, true);
}

}  // namespace cf
