// Kernels and host entry points of the full-Craftax variant (nine floors, 43 actions).
#include "full_api.hpp"

#include <hip/hip_runtime.h>

#include <cmath>
#include <cstring>
#include <vector>

#include "worldgen.hpp"
#include "full_common.hpp"
#include "full_render.hpp"
#include "full_step.hpp"
#include "full_worldgen.hpp"

namespace cf {

static_assert(sizeof(craftax_full_env_dump) == 63432, "canonical dump layout");

// a list entry carries what the reset needs: (env, seed low, seed high, next episode index)
struct DoneList { uint32_t* count; uint32_t* finished; uint4* list; };
constexpr int RESET_SLOTS = 64;   // environments regenerated at once by kf_reset_list (nine blocks each)

__device__ inline uint32_t pack_regs(const MobRegs& m)
{
    Mob o;
    o.alive = m.alive; o.x = m.x; o.y = m.y; o.dir = m.dir; o.hp = m.hp; o.cd = m.cd; o.type = m.type;
    return pack_mob(o);
}

// ---------------------------------------------------------------------------------------------
// reset of every environment: one block per (environment, floor); the block of floor 0 also
// writes the fresh record and the empty mob tables
__global__ __launch_bounds__(GEN_THREADS) void kf_reset(uint32_t* __restrict__ envs, uint8_t* __restrict__ maps,
                                                       const uint64_t* __restrict__ seeds, uint32_t* done_count,
                                                       uint32_t* done_finished)
{
    if (blockIdx.x == 0 && threadIdx.x == 0) { *done_count = 0u; *done_finished = 0u; }
    __shared__ uint16_t s_lat[LAT_TOTAL];
    __shared__ GenLayout s_layout;
    const uint32_t env = blockIdx.x / FLOORS;
    const int f = blockIdx.x % FLOORS;
    const uint64_t seed = seeds[env];
    const uint32_t lo = (uint32_t)seed, hi = (uint32_t)(seed >> 32);
    worldgen_floor_block(maps + (size_t)env * MAP_BYTES, s_lat, s_layout, lo, hi, env, 0u, f);
    const int tid = threadIdx.x;
    if (f == 0 && tid < ENV_DWORDS)
        envs[(size_t)env * ENV_DWORDS + tid] = tid < REC_DWORDS ? fresh_record_word(tid, s_layout, lo, hi, 0u) : 0u;
}

// ---------------------------------------------------------------------------------------------
// step: one wavefront per environment, four environments per block.  Finished episodes are not
// written back; they go on the done list that kf_reset_list consumes right after.
template <bool F32>
__global__ __launch_bounds__(BLOCK) void kf_step(uint32_t* __restrict__ envs, uint8_t* __restrict__ maps,
                                                const Luts* __restrict__ luts, const int32_t* __restrict__ actions,
                                                uint8_t* __restrict__ obs, float* __restrict__ reward,
                                                uint8_t* __restrict__ done, DoneList dl, Params p)
{
    __shared__ uint32_t s_env[ENVS_PER_BLOCK * L_ENV_DWORDS];
    const int tid = threadIdx.x, w = tid >> 6, l = tid & 63;
    const int env = blockIdx.x * ENVS_PER_BLOCK + w;
    if (env >= p.n) return;                                     // whole waves leave; the kernel has no block barrier
    uint32_t* e = s_env + w * L_ENV_DWORDS;
    uint32_t* genv = envs + (size_t)env * ENV_DWORDS;
    uint8_t* emaps = maps + (size_t)env * MAP_BYTES;
    e[L_REC + l] = genv[l];
    const int action = uni(actions[env]);
    wave_sync();
    MobRegs m;
    uint32_t qw;
    Player P;
    const StepOut o = step_env(l, (uint32_t)env, e, genv, emaps, luts, action, p, m, qw, P);
    if (l == 0) { reward[env] = o.reward; done[env] = o.done ? 1 : 0; }
    if (o.done) {
        if (l == 0) {
            const uint32_t idx = atomicAdd(dl.count, 1u);
            dl.list[idx] = make_uint4((uint32_t)env, e[L_REC + R_SEED_LO], e[L_REC + R_SEED_HI], P.episode + 1u);
        }
        return;
    }
    if (l == 0) pack_player(e + L_REC, P);
    if (l < NPLANT) e[L_REC + R_PLANT + l] = qw;
    wave_sync();
    genv[l] = e[L_REC + l];
    if (l < MOBTAB_DWORDS) genv[REC_DWORDS + P.floor * MOBTAB_DWORDS + l] = l < NSLOT ? pack_regs(m) : 0u;
    if (obs != nullptr)
        render_env<F32>(l, e, o.wx0, o.wy0, m.alive, m.x, m.y, m.type, luts, obs + (size_t)env * (F32 ? STRIDE_F32 : STRIDE_U8));
}

// Regenerates every environment on the done list, nine blocks (one per floor) each, looping if
// the list is longer than the grid; the block of floor 0 also writes the fresh record and renders
// the first observation.  The last working block clears the list for the next step.
template <bool F32>
__global__ __launch_bounds__(GEN_THREADS) void kf_reset_list(uint32_t* __restrict__ envs, uint8_t* __restrict__ maps,
                                                            const Luts* __restrict__ luts, uint8_t* __restrict__ obs, DoneList dl)
{
    __shared__ uint16_t s_lat[LAT_TOTAL];
    __shared__ GenLayout s_layout;
    __shared__ uint32_t s_env[L_ENV_DWORDS];
    const uint32_t count = *dl.count;
    const uint32_t slot = blockIdx.x / FLOORS, slots = gridDim.x / FLOORS;
    const int f = blockIdx.x % FLOORS;
    if (slot >= count) return;
    const int tid = threadIdx.x;
    // every working block has read the count; the last one to say so clears the list for the
    // next step (entries are only appended by the next step kernel, after this one ends)
    if (tid == 0) {
        const uint32_t workers = (count < slots ? count : slots) * FLOORS;
        if (atomicAdd(dl.finished, 1u) == workers - 1u) { *dl.count = 0u; *dl.finished = 0u; }
    }
    for (uint32_t i = slot; i < count; i += slots) {
        const uint4 entry = dl.list[i];
        const uint32_t env = entry.x, lo = entry.y, hi = entry.z, ep = entry.w;
        worldgen_floor_block(maps + (size_t)env * MAP_BYTES, s_lat, s_layout, lo, hi, env, ep, f,
                             reinterpret_cast<uint8_t*>(s_env + L_WB), reinterpret_cast<uint8_t*>(s_env + L_WI));
        if (f == 0) {
            if (tid < ENV_DWORDS) {
                const uint32_t w = tid < REC_DWORDS ? fresh_record_word(tid, s_layout, lo, hi, ep) : 0u;
                envs[(size_t)env * ENV_DWORDS + tid] = w;
                if (tid < REC_DWORDS) s_env[L_REC + tid] = w;
            }
            __syncthreads();
            if (obs != nullptr && tid < 64)
                render_env<F32>(tid, s_env, W / 2 - WIN_COLS / 2, W / 2 - WIN_ROWS / 2, 0, 0, 0, 0, luts,
                                obs + (size_t)env * (F32 ? STRIDE_F32 : STRIDE_U8));
        }
        __syncthreads();
    }
}

template <bool F32>
__global__ __launch_bounds__(BLOCK) void kf_observe(const uint32_t* __restrict__ envs, const uint8_t* __restrict__ maps,
                                                   const Luts* __restrict__ luts, uint8_t* __restrict__ obs, int n)
{
    __shared__ uint32_t s_env[ENVS_PER_BLOCK * L_ENV_DWORDS];
    const int tid = threadIdx.x, w = tid >> 6, l = tid & 63;
    const int env = blockIdx.x * ENVS_PER_BLOCK + w;
    if (env >= n) return;
    uint32_t* e = s_env + w * L_ENV_DWORDS;
    const uint32_t* genv = envs + (size_t)env * ENV_DWORDS;
    e[L_REC + l] = genv[l];
    wave_sync();
    const uint32_t pos = uniu(e[L_REC + R_POS]);
    const int px = pos & 0xFF, py = (pos >> 8) & 0xFF, f = (pos >> 24) & 0xF;
    const Mob u = unpack_mob(l < NSLOT ? genv[REC_DWORDS + f * MOBTAB_DWORDS + l] : 0u);
    load_window(l, maps + (size_t)env * MAP_BYTES, f, px, py, reinterpret_cast<uint8_t*>(e + L_WB), reinterpret_cast<uint8_t*>(e + L_WI));
    wave_sync();
    render_env<F32>(l, e, px - WIN_COLS / 2, py - WIN_ROWS / 2, u.alive, u.x, u.y, u.type, luts,
                    obs + (size_t)env * (F32 ? STRIDE_F32 : STRIDE_U8));
}

// ---------------------------------------------------------------------------------------------
// canonical dumps: one block per environment
__global__ __launch_bounds__(BLOCK) void kf_export(const uint32_t* __restrict__ envs, const uint8_t* __restrict__ maps,
                                                  craftax_full_env_dump* __restrict__ dumps, int first)
{
    const int env = first + blockIdx.x, tid = threadIdx.x;
    craftax_full_env_dump* d = dumps + blockIdx.x;
    const uint8_t* em = maps + (size_t)env * MAP_BYTES;
    const uint32_t* r = envs + (size_t)env * ENV_DWORDS;
    for (int i = tid; i < FLOORS * CELLS; i += BLOCK) {
        const int f = i / CELLS, c = i - f * CELLS;
        const uint32_t il = em[(size_t)f * 2 * CELLS + CELLS + c];
        d->block[f][c] = em[(size_t)f * 2 * CELLS + c];
        d->item[f][c] = (uint8_t)(il & 7u);
        d->light[f][c] = (uint8_t)(il >> 3);
    }
    if (tid == 0) {
        d->px = r[R_POS] & 0xFF; d->py = (r[R_POS] >> 8) & 0xFF; d->dir = (r[R_POS] >> 16) & 0xFF; d->floor = (r[R_POS] >> 24) & 0xF;
        const uint32_t fl = r[R_FLAGS], at = r[R_ATTR];
        d->sleeping = fl & 1; d->resting = (fl >> 1) & 1; d->learned_fireball = (fl >> 2) & 1; d->learned_iceball = (fl >> 3) & 1;
        d->book = (fl >> 4) & 3; d->pickaxe = (fl >> 6) & 7; d->sword = (fl >> 9) & 7; d->sword_ench = (fl >> 12) & 3;
        d->bow = (fl >> 14) & 1; d->bow_ench = (fl >> 15) & 3; d->boss_vulnerable = (fl >> 17) & 1; d->boss_hits = (fl >> 18) & 15;
        for (int i = 0; i < 4; ++i) { d->armour[i] = (at >> (2 * i)) & 3; d->armour_ench[i] = (at >> (8 + 2 * i)) & 3; }
        d->xp = (at >> 16) & 15; d->dex = (at >> 20) & 7; d->str = (at >> 23) & 7; d->intel = (at >> 26) & 7;
        for (int i = 0; i < 10; ++i) d->inv[i] = (r[R_INV + (i >> 2)] >> (8 * (i & 3))) & 0xFF;
        for (int i = 0; i < 6; ++i) { const int b = 10 + i; d->potion[i] = (r[R_INV + (b >> 2)] >> (8 * (b & 3))) & 0xFF; }
        for (int i = 0; i < 4; ++i) { d->vit[i] = (int8_t)((r[R_VIT] >> (8 * i)) & 0xFF); d->cnt[i] = (int16_t)(int8_t)(r[R_CNT] >> (8 * i)); }
        d->vit[4] = (int8_t)(r[R_MANA] & 0xFF); d->cnt[4] = (int16_t)(int8_t)(r[R_MANA] >> 8);
        for (int i = 0; i < 6; ++i) d->potion_effect[i] = (r[R_PERM] >> (3 * i)) & 7;
        d->visited = (uint16_t)((r[R_PERM] >> 18) & 0x1FF);
        for (int i = 0; i < FLOORS; ++i) {
            d->kills[i] = (r[R_KILLS + (i >> 2)] >> (8 * (i & 3))) & 0xFF;
            const uint32_t lw = r[R_LADDER + i];
            d->ladder_up[i][0] = lw & 0xFF; d->ladder_up[i][1] = (lw >> 8) & 0xFF;
            d->ladder_down[i][0] = (lw >> 16) & 0xFF; d->ladder_down[i][1] = (lw >> 24) & 0xFF;
        }
        d->pad_a = 0; d->pad_b = 0; d->pad_c[0] = d->pad_c[1] = 0; d->pad0 = 0;
        for (int i = 0; i < 4; ++i) d->pad1[i] = 0;
        for (int i = 0; i < 3; ++i) d->ach[i] = r[R_ACH + i];
        d->t = r[R_T]; d->episode = r[R_EPISODE]; d->env = (uint32_t)env;
        d->seed = (uint64_t)r[R_SEED_LO] | ((uint64_t)r[R_SEED_HI] << 32);
    }
    if (tid < FLOORS * NSLOT) {
        const int f = tid / NSLOT, k = tid - f * NSLOT;
        const Mob m = unpack_mob(r[REC_DWORDS + f * MOBTAB_DWORDS + k]);
        craftax_full_mob o;
        o.alive = m.alive; o.x = m.x; o.y = m.y; o.dir = m.dir; o.hp = (int8_t)m.hp; o.cd = m.cd; o.type = m.type; o.pad = 0;
        d->mob[f][k] = o;
    }
    if (tid >= 128 && tid < 128 + NPLANT) {
        const uint32_t q = r[R_PLANT + tid - 128];
        craftax_plant o;
        o.alive = q & 1u; o.x = (q >> 1) & 63u; o.y = (q >> 7) & 63u; o.pad = 0; o.age = (uint16_t)(q >> 16);
        d->plant[tid - 128] = o;
    }
}

// Import packs into the record's bit fields: counts 0..255, counters -128..127, mob hp 0..31,
// cooldown 0..15, experience 0..15, coordinates 0..47, floor 0..8 (every state the rules can
// reach is); values outside are clamped so that no kernel ever indexes beyond its buffers.
__global__ __launch_bounds__(BLOCK) void kf_import(uint32_t* __restrict__ envs, uint8_t* __restrict__ maps,
                                                  const craftax_full_env_dump* __restrict__ dumps, int first, Params p)
{
    const int env = first + blockIdx.x, tid = threadIdx.x;
    const craftax_full_env_dump* d = dumps + blockIdx.x;
    uint8_t* em = maps + (size_t)env * MAP_BYTES;
    uint32_t* r = envs + (size_t)env * ENV_DWORDS;
    for (int i = tid; i < FLOORS * CELLS; i += BLOCK) {
        const int f = i / CELLS, c = i - f * CELLS;
        em[(size_t)f * 2 * CELLS + c] = d->block[f][c];
        em[(size_t)f * 2 * CELLS + CELLS + c] = (uint8_t)((d->item[f][c] & 7u) | ((uint32_t)min((int)d->light[f][c], 31) << 3));
    }
    __shared__ uint32_t s[ENV_DWORDS];
    s[tid] = 0u;
    __syncthreads();
    if (tid == 0) {
        s[R_POS] = (uint32_t)min((int)d->px, W - 1) | ((uint32_t)min((int)d->py, W - 1) << 8) | ((uint32_t)(d->dir & 7) << 16) |
                   ((uint32_t)min((int)d->floor, FLOORS - 1) << 24);
        s[R_FLAGS] = (uint32_t)(d->sleeping & 1) | ((uint32_t)(d->resting & 1) << 1) | ((uint32_t)(d->learned_fireball & 1) << 2) |
                     ((uint32_t)(d->learned_iceball & 1) << 3) | ((uint32_t)(d->book & 3) << 4) | ((uint32_t)(d->pickaxe & 7) << 6) |
                     ((uint32_t)(d->sword & 7) << 9) | ((uint32_t)(d->sword_ench & 3) << 12) | ((uint32_t)(d->bow & 1) << 14) |
                     ((uint32_t)(d->bow_ench & 3) << 15) | ((uint32_t)(d->boss_vulnerable & 1) << 17) | ((uint32_t)(d->boss_hits & 15) << 18);
        uint32_t at = ((uint32_t)(d->xp & 15) << 16) | ((uint32_t)(d->dex & 7) << 20) | ((uint32_t)(d->str & 7) << 23) | ((uint32_t)(d->intel & 7) << 26);
        for (int i = 0; i < 4; ++i) at |= ((uint32_t)(d->armour[i] & 3) << (2 * i)) | ((uint32_t)(d->armour_ench[i] & 3) << (8 + 2 * i));
        s[R_ATTR] = at;
        for (int i = 0; i < 10; ++i) s[R_INV + (i >> 2)] |= (uint32_t)d->inv[i] << (8 * (i & 3));
        for (int i = 0; i < 6; ++i) { const int b = 10 + i; s[R_INV + (b >> 2)] |= (uint32_t)d->potion[i] << (8 * (b & 3)); }
        uint32_t wv = 0, wc = 0;
        for (int i = 0; i < 4; ++i) {
            wv |= (uint32_t)(uint8_t)max(0, (int)d->vit[i]) << (8 * i);
            wc |= (uint32_t)(max(-128, min(127, (int)d->cnt[i])) & 0xFF) << (8 * i);
        }
        s[R_VIT] = wv; s[R_CNT] = wc;
        s[R_MANA] = (uint32_t)(uint8_t)max(0, (int)d->vit[4]) | ((uint32_t)(max(-128, min(127, (int)d->cnt[4])) & 0xFF) << 8) |
                    ((d->t % p.day_length) << 16);
        uint32_t pm = (uint32_t)(d->visited & 0x1FF) << 18;
        for (int i = 0; i < 6; ++i) pm |= (uint32_t)(d->potion_effect[i] & 7) << (3 * i);
        s[R_PERM] = pm;
        for (int i = 0; i < FLOORS; ++i) {
            s[R_KILLS + (i >> 2)] |= (uint32_t)d->kills[i] << (8 * (i & 3));
            s[R_LADDER + i] = (uint32_t)min((int)d->ladder_up[i][0], W - 1) | ((uint32_t)min((int)d->ladder_up[i][1], W - 1) << 8) |
                              ((uint32_t)min((int)d->ladder_down[i][0], W - 1) << 16) | ((uint32_t)min((int)d->ladder_down[i][1], W - 1) << 24);
        }
        for (int i = 0; i < 3; ++i) s[R_ACH + i] = d->ach[i];
        s[R_T] = d->t; s[R_EPISODE] = d->episode;
        s[R_SEED_LO] = (uint32_t)d->seed; s[R_SEED_HI] = (uint32_t)(d->seed >> 32);
    }
    if (tid < FLOORS * NSLOT) {
        const int f = tid / NSLOT, k = tid - f * NSLOT;
        const craftax_full_mob u = d->mob[f][k];
        Mob m;
        m.alive = u.alive & 1; m.x = min((int)u.x, W - 1); m.y = min((int)u.y, W - 1); m.dir = u.dir & 7; m.hp = max(0, min(31, (int)u.hp)); m.cd = min(15, (int)u.cd);
        m.type = u.type & 31;
        s[REC_DWORDS + f * MOBTAB_DWORDS + k] = pack_mob(m);
    }
    if (tid >= 128 && tid < 128 + NPLANT) {
        const craftax_plant u = d->plant[tid - 128];
        s[R_PLANT + tid - 128] = (u.alive & 1) ? (1u | ((uint32_t)min((int)u.x, W - 1) << 1) | ((uint32_t)min((int)u.y, W - 1) << 7) | ((uint32_t)u.age << 16)) : 0u;
    }
    __syncthreads();
    r[tid] = s[tid];
}

// ---------------------------------------------------------------------------------------------
namespace host {

static uint64_t round_up(uint64_t v, uint64_t a) { return (v + a - 1) / a * a; }

bool config_ok(const craftax_config* c, std::string* why)
{
    if (c->abi_version != CRAFTAX_ABI_VERSION) { *why = "abi_version mismatch"; return false; }
    if (c->obs_mode != CRAFTAX_OBS_SYM_U8_F32 && c->obs_mode != CRAFTAX_OBS_SYM_F32) { *why = "the Craftax variant renders SYM_U8_F32 or SYM_F32"; return false; }
    if (c->day_length < 2 || c->day_length > (uint32_t)MAX_DAY || (c->day_length & 1)) { *why = "day_length must be even and in 2..1024"; return false; }
    if (c->cap_zombie > 3 || c->cap_cow > 3 || c->cap_skeleton > 2) { *why = "caps: melee 0..3, passive 0..3, ranged 0..2"; return false; }
    if (c->cap_plant > (uint32_t)NPLANT) { *why = "cap_plant must be 0..10"; return false; }
    if (c->max_episode_steps == 0) { *why = "max_episode_steps must be positive"; return false; }
    return true;
}

static Header make_header(const craftax_config* c, int n)
{
    Header h;
    std::memset(&h, 0, sizeof(h));
    h.magic = MAGIC; h.version = CRAFTAX_ABI_VERSION; h.n = (uint32_t)n; h.variant = c->variant;
    h.obs_mode = c->obs_mode; h.max_episode_steps = c->max_episode_steps; h.day_length = c->day_length;
    h.cap_melee = c->cap_zombie; h.cap_ranged = c->cap_skeleton; h.cap_passive = c->cap_cow; h.cap_plant = c->cap_plant;
    h.off_luts = 256;
    h.off_envs = round_up(h.off_luts + sizeof(Luts), 256);
    h.off_maps = h.off_envs + (uint64_t)n * (ENV_DWORDS * 4);
    h.off_done = round_up(h.off_maps + (uint64_t)n * MAP_BYTES, 256);
    h.total = round_up(h.off_done + (uint64_t)n * 16, 256);
    return h;
}

// Day/night: phase i = t mod L, H = L/2, k = |i - H|, daylight = k^2 (3H - 2k) / H^3 (noon at
// t = 0); the paper only says the observation carries a day/night value in [0,1].
static void build_luts(const craftax_config* c, Luts* L)
{
    std::memset(L, 0, sizeof(*L));
    const uint64_t len = c->day_length, half = len / 2, den = half * half * half;
    for (uint64_t i = 0; i < len; ++i) {
        const uint64_t k = i < half ? half - i : i - half;
        const uint64_t num = k * k * (3 * half - 2 * k);
        L->daylight[i] = (float)((double)num / (double)den);
        L->zombie_thr[i] = (40u + 3u * (255u - (uint32_t)(255u * num / den))) << 20;
    }
    for (int i = 0; i < 100; ++i) L->sqrt10[i] = (float)(std::sqrt((double)i) / 10.0);
    for (int i = 0; i < 32; ++i) L->tenth[i] = (float)((double)i / 10.0);
    for (int i = 0; i < 32; ++i) L->light20[i] = (float)((double)i / 20.0);
}

struct Ptrs { uint32_t* envs; uint8_t* maps; const Luts* luts; DoneList dl; };
static Ptrs pointers(const void* state, const Header& h)
{
    uint8_t* base = const_cast<uint8_t*>(static_cast<const uint8_t*>(state));
    Ptrs q;
    q.luts = reinterpret_cast<const Luts*>(base + h.off_luts);
    q.envs = reinterpret_cast<uint32_t*>(base + h.off_envs);
    q.maps = base + h.off_maps;
    q.dl.count = reinterpret_cast<uint32_t*>(base + cx::DONE_COUNT_OFFSET);
    q.dl.finished = q.dl.count + 1;
    q.dl.list = reinterpret_cast<uint4*>(base + h.off_done);
    return q;
}
static Params make_params(const craftax_config* c, int n)
{
    Params p;
    p.n = n; p.max_episode_steps = c->max_episode_steps; p.day_length = c->day_length;
    p.cap_melee = c->cap_zombie; p.cap_ranged = c->cap_skeleton; p.cap_passive = c->cap_cow; p.cap_plant = c->cap_plant;
    return p;
}
static int check_launch(const char* what, std::string* err)
{
    const hipError_t e = hipGetLastError();
    if (e != hipSuccess) { *err = std::string(what) + ": " + hipGetErrorString(e); return CRAFTAX_E_HIP; }
    return CRAFTAX_OK;
}

size_t state_bytes(const craftax_config* cfg, int n) { return (size_t)make_header(cfg, n).total; }
size_t obs_bytes(const craftax_config* cfg) { return cfg->obs_mode == CRAFTAX_OBS_SYM_F32 ? STRIDE_F32 : STRIDE_U8; }

int state_init(void* state, const craftax_config* cfg, int n, void* stream, std::string* err)
{
    const Header h = make_header(cfg, n);
    std::vector<uint8_t> staging((size_t)h.off_envs, 0);
    std::memcpy(staging.data(), &h, sizeof(Header));
    build_luts(cfg, reinterpret_cast<Luts*>(staging.data() + h.off_luts));
    hipError_t e = hipMemcpyAsync(state, staging.data(), staging.size(), hipMemcpyHostToDevice, (hipStream_t)stream);
    if (e == hipSuccess) e = hipStreamSynchronize((hipStream_t)stream);   // staging dies with this call
    if (e != hipSuccess) { *err = std::string("state_init copy: ") + hipGetErrorString(e); return CRAFTAX_E_HIP; }
    return CRAFTAX_OK;
}

int reset(void* state, const craftax_config* cfg, int n, const uint64_t* seeds, void* stream, std::string* err)
{
    const Ptrs q = pointers(state, make_header(cfg, n));
    hipLaunchKernelGGL(kf_reset, dim3((unsigned)n * FLOORS), dim3(GEN_THREADS), 0, (hipStream_t)stream, q.envs, q.maps, seeds, q.dl.count, q.dl.finished);
    return check_launch("craftax_reset", err);
}

int step(void* state, const craftax_config* cfg, int n, const int32_t* actions, void* obs, float* reward, uint8_t* done,
         void* stream, std::string* err)
{
    const Ptrs q = pointers(state, make_header(cfg, n));
    const Params p = make_params(cfg, n);
    hipStream_t st = (hipStream_t)stream;
    uint8_t* o = static_cast<uint8_t*>(obs);
    const dim3 grid((n + ENVS_PER_BLOCK - 1) / ENVS_PER_BLOCK), rgrid((unsigned)(n < RESET_SLOTS ? n : RESET_SLOTS) * FLOORS);
    if (cfg->obs_mode == CRAFTAX_OBS_SYM_F32) {
        hipLaunchKernelGGL(kf_step<true>, grid, dim3(BLOCK), 0, st, q.envs, q.maps, q.luts, actions, o, reward, done, q.dl, p);
        hipLaunchKernelGGL(kf_reset_list<true>, rgrid, dim3(GEN_THREADS), 0, st, q.envs, q.maps, q.luts, o, q.dl);
    } else {
        hipLaunchKernelGGL(kf_step<false>, grid, dim3(BLOCK), 0, st, q.envs, q.maps, q.luts, actions, o, reward, done, q.dl, p);
        hipLaunchKernelGGL(kf_reset_list<false>, rgrid, dim3(GEN_THREADS), 0, st, q.envs, q.maps, q.luts, o, q.dl);
    }
    return check_launch("craftax_step", err);
}

int observe(void* state, const craftax_config* cfg, int n, void* obs, void* stream, std::string* err)
{
    const Ptrs q = pointers(state, make_header(cfg, n));
    const dim3 grid((n + ENVS_PER_BLOCK - 1) / ENVS_PER_BLOCK);
    uint8_t* o = static_cast<uint8_t*>(obs);
    if (cfg->obs_mode == CRAFTAX_OBS_SYM_F32) hipLaunchKernelGGL(kf_observe<true>, grid, dim3(BLOCK), 0, (hipStream_t)stream, q.envs, q.maps, q.luts, o, n);
    else hipLaunchKernelGGL(kf_observe<false>, grid, dim3(BLOCK), 0, (hipStream_t)stream, q.envs, q.maps, q.luts, o, n);
    return check_launch("craftax_observe", err);
}

int export_envs(const void* state, const craftax_config* cfg, int n, int first, int count, void* dumps, void* stream, std::string* err)
{
    const Ptrs q = pointers(state, make_header(cfg, n));
    hipLaunchKernelGGL(kf_export, dim3(count), dim3(BLOCK), 0, (hipStream_t)stream, q.envs, q.maps,
                       static_cast<craftax_full_env_dump*>(dumps), first);
    return check_launch("craftax_export_envs", err);
}

int import_envs(void* state, const craftax_config* cfg, int n, int first, int count, const void* dumps, void* stream, std::string* err)
{
    const Ptrs q = pointers(state, make_header(cfg, n));
    hipLaunchKernelGGL(kf_import, dim3(count), dim3(BLOCK), 0, (hipStream_t)stream, q.envs, q.maps,
                       static_cast<const craftax_full_env_dump*>(dumps), first, make_params(cfg, n));
    return check_launch("craftax_import_envs", err);
}

}  // namespace host
}  // namespace cf
