// Symbolic observation of full Craftax (appendix "Observation Space"): 9 x 11 cells around the
// player, per cell one-hot block (37) + item (5) + creature (40: five slot classes of eight
// types) + light; cells darker than 0.05 are blank; then the 51 scalars of the inventory table.
// The wave first builds the byte layout in LDS (zero fill, then a few byte stores per cell),
// then streams it out as whole cache lines, or expands it to floats for the flat layout.
#pragma once

#include "full_common.hpp"

namespace cf {

constexpr int LIGHT_TAG = 0x80;    // marks the light byte of a cell while the float layout is expanded

// Where scalar i of the observation comes from: record word, shift, mask, and how the raw
// integer becomes a float.  Direction, daylight and "floor cleared" are handled apart.
enum Conv : int { CV_SQRT10 = 0, CV_TENTH, CV_HALF, CV_QUARTER, CV_RAW, CV_SPECIAL };
struct ScalarSpec { uint8_t word, shift, mask, conv; };
__device__ __constant__ const ScalarSpec SCALARS[NVEC] = {
    { R_INV, 0, 255, CV_SQRT10 }, { R_INV, 8, 255, CV_SQRT10 }, { R_INV, 16, 255, CV_SQRT10 }, { R_INV, 24, 255, CV_SQRT10 },
    { R_INV + 1, 0, 255, CV_SQRT10 }, { R_INV + 1, 8, 255, CV_SQRT10 }, { R_INV + 1, 16, 255, CV_SQRT10 }, { R_INV + 1, 24, 255, CV_SQRT10 },
    { R_INV + 2, 0, 255, CV_SQRT10 }, { R_INV + 2, 8, 255, CV_SQRT10 },
    { R_INV + 2, 16, 255, CV_SQRT10 }, { R_INV + 2, 24, 255, CV_SQRT10 },                                  // potions 0, 1
    { R_POT, 0, 255, CV_SQRT10 }, { R_POT, 8, 255, CV_SQRT10 }, { R_POT, 16, 255, CV_SQRT10 }, { R_POT, 24, 255, CV_SQRT10 },
    { R_FLAGS, 4, 3, CV_HALF },        // book n/2
    { R_FLAGS, 6, 7, CV_QUARTER },     // pickaxe level/4
    { R_FLAGS, 9, 7, CV_QUARTER },     // sword level/4
    { R_FLAGS, 12, 3, CV_RAW },        // sword enchantment: fire 1, ice 2
    { R_FLAGS, 14, 1, CV_RAW },        // bow
    { R_FLAGS, 15, 3, CV_RAW },        // bow enchantment
    { R_ATTR, 0, 3, CV_HALF }, { R_ATTR, 2, 3, CV_HALF }, { R_ATTR, 4, 3, CV_HALF }, { R_ATTR, 6, 3, CV_HALF },       // armour level/2
    { R_ATTR, 8, 3, CV_RAW }, { R_ATTR, 10, 3, CV_RAW }, { R_ATTR, 12, 3, CV_RAW }, { R_ATTR, 14, 3, CV_RAW },        // armour enchantments
    { R_VIT, 0, 255, CV_TENTH }, { R_VIT, 8, 255, CV_TENTH }, { R_VIT, 16, 255, CV_TENTH }, { R_VIT, 24, 255, CV_TENTH },
    { R_MANA, 0, 255, CV_TENTH },
    { R_ATTR, 16, 15, CV_TENTH },      // experience
    { R_ATTR, 20, 7, CV_TENTH }, { R_ATTR, 23, 7, CV_TENTH }, { R_ATTR, 26, 7, CV_TENTH },                           // dexterity strength intelligence
    { R_POS, 16, 255, CV_SPECIAL }, { R_POS, 16, 255, CV_SPECIAL }, { R_POS, 16, 255, CV_SPECIAL }, { R_POS, 16, 255, CV_SPECIAL },   // facing one-hot
    { R_MANA, 16, 255, CV_SPECIAL },   // daylight
    { R_FLAGS, 0, 1, CV_RAW },         // sleeping
    { R_FLAGS, 1, 1, CV_RAW },         // resting
    { R_FLAGS, 2, 1, CV_RAW },         // learned fireball
    { R_FLAGS, 3, 1, CV_RAW },         // learned iceball
    { R_POS, 24, 15, CV_TENTH },       // floor / 10
    { R_POS, 24, 15, CV_SPECIAL },     // floor cleared
    { R_FLAGS, 17, 1, CV_RAW },        // boss vulnerable
};

// scalar `i` of the observation from the packed record in LDS
__device__ inline float scalar_value(int i, const uint32_t* rec, const Luts* __restrict__ luts)
{
    const ScalarSpec s = SCALARS[i];
    const uint32_t raw = (rec[s.word] >> s.shift) & s.mask;
    if (s.conv == CV_SQRT10) return luts->sqrt10[min(raw, 99u)];
    if (s.conv == CV_TENTH) return luts->tenth[min(raw, 31u)];
    if (s.conv == CV_HALF) return (float)raw * 0.5f;
    if (s.conv == CV_QUARTER) return (float)raw * 0.25f;
    if (s.conv == CV_RAW) return (float)raw;
    if (i >= 39 && i < 43) return (int)raw == i - 38 ? 1.0f : 0.0f;
    if (i == 43) return luts->daylight[rec[R_MANA] >> 16];
    // floor cleared: the overworld always, deeper floors after enough kills
    const int f = (int)raw;
    const int kills = (int)((rec[R_KILLS + (f >> 2)] >> (8 * (f & 3))) & 0xFFu);
    return (f == 0 || kills >= KILLS_TO_CLEAR) ? 1.0f : 0.0f;
}

// Observation channel of the creature in slot k (class by slot range, type slot by creature).
__device__ inline int creature_channel(int k, int type)
{
    if (k < S_RANGED0) return 42 + MELEE_TYPE_SLOT[type];
    if (k < S_PASSIVE0) return 42 + 16 + RANGED_TYPE_SLOT[type];
    if (k < S_MPROJ0) return 42 + 8 + (type == C_COW ? 0 : (type == C_SNAIL ? 1 : 2));
    if (k < S_PPROJ0) {
        const CreatureRow c = CREATURE[type];
        return 42 + 24 + (c.df > 0 ? (c.di > 0 ? 3 : 1) : (c.di > 0 ? 2 : 0));
    }
    return 42 + 32 + type;
}

// e: the wave's LDS area holding the packed record (current), the two windows with origin
// (wx0, wy0) on the current floor; m_*: this lane's mob slot.  F32 = false: writes the
// 8448-byte layout; F32 = true: writes float[8268] (+ zero padding to 33152 bytes).
template <bool F32>
__device__ inline void render_env(const int l, uint32_t* e, const int wx0, const int wy0, const int m_alive, const int m_x,
                                  const int m_y, const int m_type, const Luts* __restrict__ luts, uint8_t* __restrict__ out)
{
    const uint32_t* rec = e + L_REC;
    const uint8_t* wb = reinterpret_cast<const uint8_t*>(e + L_WB);
    const uint8_t* wi = reinterpret_cast<const uint8_t*>(e + L_WI);
    uint32_t* cre = e + L_CRE;
    uint8_t* stage = reinterpret_cast<uint8_t*>(e + L_STAGE);
    const uint32_t pos = uniu(rec[R_POS]);
    const int px = pos & 0xFF, py = (pos >> 8) & 0xFF;
    {
        uint4* z = reinterpret_cast<uint4*>(stage);
#pragma unroll
        for (int it = 0; it < 9; ++it) {
            const int i = l + 64 * it;
            if (i < STRIDE_U8 / 16) z[i] = make_uint4(0u, 0u, 0u, 0u);
        }
        cre[l] = 0xFFFFFFFFu;
        if (l + 64 < NCELL + 1) cre[l + 64] = 0xFFFFFFFFu;
    }
    wave_sync();
    if (l < NSLOT && m_alive) {
        const int vr = m_y - (py - VROWS / 2), vc = m_x - (px - VCOLS / 2);
        if ((unsigned)vr < (unsigned)VROWS && (unsigned)vc < (unsigned)VCOLS)
            atomicMin(&cre[vr * VCOLS + vc], ((uint32_t)l << 8) | (uint32_t)creature_channel(l, m_type));   // lowest slot wins
    }
    if (l < NVEC) reinterpret_cast<float*>(stage + VEC_OFFSET)[l] = scalar_value(l, rec, luts);
    wave_sync();
#pragma unroll
    for (int it = 0; it < 2; ++it) {
        const int cell = l + 64 * it;
        if (cell < NCELL) {
            const int r = cell / VCOLS, c = cell - r * VCOLS;
            const int x = px - VCOLS / 2 + c, y = py - VROWS / 2 + r;
            uint8_t* ch = stage + cell * NCHAN;
            if (!inb(x, y)) {   // beyond the edge of the map: always visible
                ch[B_OOB] = 1; ch[37 + IT_NONE] = 1; ch[82] = (uint8_t)(F32 ? (LIGHT_TAG | MAX_LIGHT) : MAX_LIGHT);
            } else {
                const int il = wi[(y - wy0) * WIN_PITCH + (x - wx0)], light = il >> 3;
                if (light != 0) {
                    ch[wb[(y - wy0) * WIN_PITCH + (x - wx0)]] = 1;
                    ch[37 + (il & 7)] = 1;
                    const uint32_t cr = cre[cell];
                    if (cr != 0xFFFFFFFFu) ch[cr & 0xFFu] = 1;
                    ch[82] = (uint8_t)(F32 ? (LIGHT_TAG | light) : light);
                }
            }
        }
    }
    wave_sync();
    if (!F32) {
        const uint4* src = reinterpret_cast<const uint4*>(stage);
        uint4* dst = reinterpret_cast<uint4*>(out);
#pragma unroll
        for (int it = 0; it < 9; ++it) {
            const int i = l + 64 * it;
            if (i < STRIDE_U8 / 16) {
                const uint4 v = src[i];
                __builtin_nontemporal_store(v.x, &dst[i].x);
                __builtin_nontemporal_store(v.y, &dst[i].y);
                __builtin_nontemporal_store(v.z, &dst[i].z);
                __builtin_nontemporal_store(v.w, &dst[i].w);
            }
        }
    } else {
        const uint32_t* src = reinterpret_cast<const uint32_t*>(stage);
        const float* vec = reinterpret_cast<const float*>(stage + VEC_OFFSET);
        float4* dst = reinterpret_cast<float4*>(out);
#pragma unroll 1
        for (int q = l; q < STRIDE_F32 / 16; q += 64) {
            float v[4];
            if (4 * q + 3 < CELL_BYTES) {
                const uint32_t w = src[q];
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const uint32_t b = (w >> (8 * j)) & 0xFFu;
                    v[j] = (b & LIGHT_TAG) ? luts->light20[b & 31u] : (float)b;
                }
            } else {
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const int idx = 4 * q + j;
                    float f = 0.0f;
                    if (idx < CELL_BYTES) {
                        const uint32_t b = stage[idx];
                        f = (b & LIGHT_TAG) ? luts->light20[b & 31u] : (float)b;
                    } else if (idx < CELL_BYTES + NVEC) f = vec[idx - CELL_BYTES];
                    v[j] = f;
                }
            }
            dst[q] = make_float4(v[0], v[1], v[2], v[3]);
        }
    }
}

}  // namespace cf
