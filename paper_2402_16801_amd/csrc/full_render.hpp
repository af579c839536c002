// Symbolic observation of full Craftax (appendix "Observation Space"): 9 x 11 cells around the
// player, per cell one-hot block (37) + item (5) + creature (40: five slot classes of eight
// types) + light; cells darker than 0.05 are blank; then the 51 scalars of the inventory table.
// The wave stages the one-hot bytes as bits in LDS and expands them while streaming out whole
// cache lines (byte layout) or floats (flat layout).
#pragma once

#include "full_common.hpp"

namespace cf {

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
__device__ __forceinline__ float scalar_value(int i, const uint32_t* rec, const Luts* __restrict__ luts)
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

// What the step kernels fetch ahead of the renderer, so that it waits for no table in memory: the
// specification of the scalars this lane writes (scalar l, l + GW, ...), the small conversion tables
// (sqrt10, tenth, light20, as they lie in Luts) copied to LDS, and the daylight value of the
// observation's phase.
constexpr int LUT_FLOATS = 100 + 32 + 32;
template <int GW>
struct RenderAux {
    uint32_t spec[(NVEC + 1 + GW - 1) / GW];    // ScalarSpec of scalar l + GW * it, as four bytes
    const float* lut;                           // LDS: sqrt10[100], tenth[32], light20[32]
    float day;                                  // daylight[phase of the rendered state]
};
template <int GW>
__device__ __forceinline__ void fetch_scalar_specs(int l, RenderAux<GW>& aux)
{
#pragma unroll
    for (int it = 0; it < (NVEC + 1 + GW - 1) / GW; ++it) {
        const int i = l + GW * it;
        aux.spec[it] = i < NVEC ? *reinterpret_cast<const uint32_t*>(&SCALARS[i]) : 0u;
    }
}
static_assert(sizeof(ScalarSpec) == 4, "a scalar specification travels as one dword");
__device__ __forceinline__ float scalar_value_fast(int i, uint32_t spec, const uint32_t* rec, const float* lut, float day)
{
    const uint32_t word = spec & 0xFFu, shift = (spec >> 8) & 0xFFu, mask = (spec >> 16) & 0xFFu, conv = spec >> 24;
    const uint32_t raw = (rec[word] >> shift) & mask;
    if (conv == CV_SQRT10) return lut[min(raw, 99u)];
    if (conv == CV_TENTH) return lut[100 + min(raw, 31u)];
    if (conv == CV_HALF) return (float)raw * 0.5f;
    if (conv == CV_QUARTER) return (float)raw * 0.25f;
    if (conv == CV_RAW) return (float)raw;
    if (i >= 39 && i < 43) return (int)raw == i - 38 ? 1.0f : 0.0f;
    if (i == 43) return day;
    const int f = (int)raw;
    const int kills = (int)((rec[R_KILLS + (f >> 2)] >> (8 * (f & 3))) & 0xFFu);
    return (f == 0 || kills >= KILLS_TO_CLEAR) ? 1.0f : 0.0f;
}

// Observation channel of the creature in slot k (class by slot range, type slot by creature).
__device__ inline int creature_channel(int k, int type)
{
    if (k < S_RANGED0) return 42 + melee_type_slot(type);
    if (k < S_PASSIVE0) return 42 + 16 + ranged_type_slot(type);
    if (k < S_MPROJ0) return 42 + 8 + (type == C_COW ? 0 : (type == C_SNAIL ? 1 : 2));
    if (k < S_PPROJ0) {
        const CreatureRow c = creature(type);
        return 42 + 24 + (c.df > 0 ? (c.di > 0 ? 3 : 1) : (c.di > 0 ? 2 : 0));
    }
    return 42 + 32 + type;
}

// one-hot nibble -> four bytes of 0/1
__device__ inline uint32_t spread4(uint32_t nibble) { return (nibble * 0x00204081u) & 0x01010101u; }

// e: the wave's LDS area holding the packed record (current), the two windows with origin
// (wx0, wy0) on the current floor; m_*: this lane's mob slot.  F32 = false: writes the
// 8448-byte layout; F32 = true: writes float[8268] (+ zero padding to 33152 bytes).
// The one-hot bytes are staged as single bits (a few LDS atomics per cell) next to a light level
// per cell; every lane then expands 16 bits at a time into one 16-byte piece of the output, so
// that a wavefront writes whole cache lines.
// GW: lanes that render this environment (see Lanes); l: the calling lane's number among them.
template <bool F32, int GW = 64>
__device__ __forceinline__ void render_env(const int l, uint32_t* e, const int wx0, const int wy0, const int m_alive, const int m_x,
                                  const int m_y, const int m_type, const Luts* __restrict__ luts, uint8_t* __restrict__ out,
                                  const RenderAux<GW>* aux = nullptr)
{
    using G = Lanes<GW>;
    const uint32_t* rec = e + L_REC;
    const uint8_t* wb = reinterpret_cast<const uint8_t*>(e + L_WB);
    const uint8_t* wi = reinterpret_cast<const uint8_t*>(e + L_WI);
    uint32_t* cre = e + L_CRE;
    uint32_t* bits = e + L_BITS;
    uint8_t* light = reinterpret_cast<uint8_t*>(e + L_LIGHT);
    float* vec = reinterpret_cast<float*>(e + L_VEC);
    const uint32_t pos = G::uniu(rec[R_POS]);
    const int px = pos & 0xFF, py = (pos >> 8) & 0xFF;
#pragma unroll
    for (int it = 0; it < (260 + GW - 1) / GW; ++it) {
        const int i = l + GW * it;
        if (i < 260) bits[i] = 0u;
    }
#pragma unroll
    for (int it = 0; it < (NCELL + 1 + GW - 1) / GW; ++it) {
        const int i = l + GW * it;
        if (i < NCELL + 1) cre[i] = 0xFFFFFFFFu;
    }
    wave_sync();
    if (l < NSLOT && m_alive) {
        const int vr = m_y - (py - VROWS / 2), vc = m_x - (px - VCOLS / 2);
        if ((unsigned)vr < (unsigned)VROWS && (unsigned)vc < (unsigned)VCOLS)
            atomicMin(&cre[vr * VCOLS + vc], ((uint32_t)l << 8) | (uint32_t)creature_channel(l, m_type));   // lowest slot wins
    }
#pragma unroll
    for (int it = 0; it < (NVEC + 1 + GW - 1) / GW; ++it) {
        const int i = l + GW * it;
        if (i < NVEC + 1) vec[i] = i >= NVEC ? 0.0f : (aux != nullptr ? scalar_value_fast(i, aux->spec[it], rec, aux->lut, aux->day) : scalar_value(i, rec, luts));
    }
    wave_sync();
    auto set_bit = [&](int i) { atomicOr(&bits[CX_IDX(i >> 5, 260)], 1u << (i & 31)); };
#pragma unroll
    for (int it = 0; it < (NCELL + GW - 1) / GW; ++it) {
        const int cell = l + GW * it;
        if (cell < NCELL) {
            const int r = cell / VCOLS, c = cell - r * VCOLS;
            const int x = px - VCOLS / 2 + c, y = py - VROWS / 2 + r;
            int lv = 0;
            if (!inb(x, y)) {   // beyond the edge of the map: always visible
                set_bit(cell * NCHAN + B_OOB); set_bit(cell * NCHAN + 37 + IT_NONE); lv = MAX_LIGHT;
            } else {
                const int il = wi[CX_IDX((y - wy0) * WIN_PITCH + (x - wx0), WIN_ROWS * WIN_PITCH)];
                lv = il >> 3;
                if (lv != 0) {      // cells darker than 0.05 stay blank
                    set_bit(cell * NCHAN + (wb[CX_IDX((y - wy0) * WIN_PITCH + (x - wx0), WIN_ROWS * WIN_PITCH)] & 63));
                    set_bit(cell * NCHAN + 37 + (il & 7));
                    const uint32_t cr = cre[cell];
                    if (cr != 0xFFFFFFFFu) set_bit(cell * NCHAN + (int)(cr & 0xFFu));
                }
            }
            light[cell] = (uint8_t)lv;
        }
    }
    wave_sync();
    // piece j covers bytes [16j, 16j+16) of the cell area; the one light byte inside it (cell c,
    // byte 83c + 82) is patched in
    auto light_in_piece = [&](int j, int* at, int* lv) {
        *at = -1; *lv = 0;
        if (16 * j + 15 >= 82) {
            const int c = (16 * j + 15 - 82) / NCHAN, p = NCHAN * c + 82;
            if (p >= 16 * j && c < NCELL) { *at = p - 16 * j; *lv = light[c]; }
        }
    };
    if (!F32) {
        constexpr int PIECE_UNROLL = GW == 64 ? 9 : 3;
        uint4* dst = reinterpret_cast<uint4*>(out);
#pragma unroll PIECE_UNROLL
        for (int it = 0; it < (STRIDE_U8 / 16 + GW - 1) / GW; ++it) {
            const int j = l + GW * it;
            if (j < STRIDE_U8 / 16) {
                uint32_t v[4] = { 0u, 0u, 0u, 0u };
                if (j < VEC_OFFSET / 16) {
                    const uint32_t b16 = (bits[j >> 1] >> ((j & 1) * 16)) & 0xFFFFu;
#pragma unroll
                    for (int k = 0; k < 4; ++k) v[k] = spread4((b16 >> (4 * k)) & 15u);
                    int at, lv;
                    light_in_piece(j, &at, &lv);
#pragma unroll
                    for (int k = 0; k < 4; ++k) if ((at >> 2) == k) v[k] |= (uint32_t)lv << (8 * (at & 3));
                } else if (j < VEC_OFFSET / 16 + (NVEC + 3) / 4) {
                    const uint4 f = reinterpret_cast<const uint4*>(e + L_VEC)[j - VEC_OFFSET / 16];
                    v[0] = f.x; v[1] = f.y; v[2] = f.z; v[3] = f.w;
                }
                typedef uint32_t piece_t __attribute__((ext_vector_type(4)));
                const piece_t piece = { v[0], v[1], v[2], v[3] };
                __builtin_nontemporal_store(piece, reinterpret_cast<piece_t*>(dst + j));   // one 16-byte streaming store
            }
        }
    } else {
        float4* dst = reinterpret_cast<float4*>(out);
#pragma unroll 1
        for (int j = l; j < STRIDE_F32 / 64; j += GW) {   // 16 floats per piece
            const uint32_t b16 = j < 520 ? (bits[j >> 1] >> ((j & 1) * 16)) & 0xFFFFu : 0u;
            int at, lv;
            light_in_piece(j, &at, &lv);
            const float lf = aux != nullptr ? aux->lut[132 + lv] : luts->light20[lv];
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                float v[4];
#pragma unroll
                for (int k = 0; k < 4; ++k) {
                    const int idx = 16 * j + 4 * q + k;
                    float f = 0.0f;
                    if (idx < CELL_BYTES) f = (4 * q + k == at) ? lf : (float)((b16 >> (4 * q + k)) & 1u);
                    else if (idx < CELL_BYTES + NVEC) f = vec[idx - CELL_BYTES];
                    v[k] = f;
                }
                dst[4 * j + q] = make_float4(v[0], v[1], v[2], v[3]);
            }
        }
    }
}

}  // namespace cf
