// Kernels and the C ABI of the MI355X Craftax-Classic simulator (see include/craftax.h).
#include "../../include/craftax.h"

#include <hip/hip_runtime.h>

#include <cmath>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <mutex>
#include <string>
#include <unordered_map>
#include <vector>

#include "common.hpp"
#include "full_api.hpp"
#include "render.hpp"
#include "step.hpp"
#include "worldgen.hpp"

namespace cx {

constexpr int BLOCK = 256;

// Copies a 128-byte record between HBM (uint4 granules) and an environment's LDS area.
template <int G>
__device__ inline void load_record(int l, const uint4* __restrict__ grec, uint32_t* e)
{
#pragma unroll
    for (int it_c = 0; it_c < ((REC_DWORDS / 4) + G - 1) / G; ++it_c) {
        const int c = l + it_c * G;
        if (c >= (REC_DWORDS / 4)) break;
        const uint4 v = grec[c];
        uint2* d = reinterpret_cast<uint2*>(e + LDS_REC + 4 * c);
        d[0] = make_uint2(v.x, v.y);
        d[1] = make_uint2(v.z, v.w);
    }
}
template <int G>
__device__ inline void store_record(int l, uint4* __restrict__ grec, const uint32_t* e)
{
#pragma unroll
    for (int it_c = 0; it_c < ((REC_DWORDS / 4) + G - 1) / G; ++it_c) {
        const int c = l + it_c * G;
        if (c >= (REC_DWORDS / 4)) break;
        const uint2* d = reinterpret_cast<const uint2*>(e + LDS_REC + 4 * c);
        const uint2 a = d[0], b = d[1];
        grec[c] = make_uint4(a.x, a.y, b.x, b.y);
    }
}

// ---------------------------------------------------------------------------------------------
// reset: one block per environment (appendix "Optimistic Environment Resets" explains why
// world generation is the expensive part; here it is spread over 512 threads).
__global__ __launch_bounds__(WG_THREADS) void k_reset(uint4* __restrict__ recs, uint8_t* __restrict__ maps,
                                                 const uint64_t* __restrict__ seeds, uint32_t* done_count,
                                                 uint32_t* done_finished, Params p)
{
    if (blockIdx.x == 0 && threadIdx.x == 0) { *done_count = 0u; *done_finished = 0u; }
    __shared__ uint16_t s_lat[LAT_BLOCKS * 8];
    const uint32_t env = blockIdx.x;
    const uint64_t seed = seeds[env];
    const uint32_t lo = (uint32_t)seed, hi = (uint32_t)(seed >> 32);
    worldgen_block(maps + (size_t)env * (MAPW * MAPW), s_lat, lo, hi, env, 0u);
    if (threadIdx.x < REC_DWORDS)
        reinterpret_cast<uint32_t*>(recs + (size_t)env * 8)[threadIdx.x] = fresh_record_word(threadIdx.x, lo, hi, 0u);
}

// ---------------------------------------------------------------------------------------------
// step: G lanes per environment, 256/G environments per block.  Environments whose episode
// ended are not written back; their indices are appended to the state's done list, which
// k_reset_list consumes right after (same stream), spreading world generation over the
// whole chip instead of stretching the tail of a few step blocks.
// a list entry carries what the reset needs: (env, seed low, seed high, next episode index)
struct DoneList { uint32_t* count; uint32_t* finished; uint4* list; };

template <int G, int OBS_MODE>
__global__ __launch_bounds__(BLOCK, 4) void k_step(uint4* __restrict__ recs, uint8_t* __restrict__ maps,
                                                   const Luts* __restrict__ luts, const int32_t* __restrict__ actions,
                                                   uint8_t* __restrict__ obs, float* __restrict__ reward,
                                                   uint8_t* __restrict__ done, DoneList dl, Params p)
{
    constexpr int EPB = Grp<G>::EPB;
    __shared__ uint32_t s_env[EPB * LDS_ENV_DWORDS];
    __shared__ int s_ndone;
    __shared__ uint32_t s_base;
    __shared__ uint4 s_list[EPB];

    const int tid = threadIdx.x, g = tid / G, l = tid % G;
    const int env = blockIdx.x * EPB + g;
    const bool active = env < p.n;
    if (tid == 0) s_ndone = 0;
    __syncthreads();
    uint32_t* e = s_env + g * LDS_ENV_DWORDS;
    uint8_t* map = maps + (size_t)(active ? env : 0) * (MAPW * MAPW);
    constexpr bool kSymbolic = OBS_MODE != CRAFTAX_OBS_PIXELS_F32;
    constexpr bool kBytes = OBS_MODE == CRAFTAX_OBS_SYM_U8_I8 || OBS_MODE == CRAFTAX_OBS_SYM_U8_F32;
    bool staged = false;
    if (active) {
        load_record<G>(l, recs + (size_t)env * 8, e);
        group_sync();
        const StepOut o = step_env<G>(l, (uint32_t)env, e, map, luts, actions[env], p);
        if (l == 0) { reward[env] = o.reward; done[env] = o.done ? 1 : 0; }
        if (!o.done) {
            store_record<G>(l, recs + (size_t)env * 8, e);
            if (kSymbolic && obs != nullptr) {
                // byte layouts are staged in LDS here and written by the whole wave below
                render_symbolic<G, OBS_MODE, true, !kBytes>(l, e, o.mvx, o.mvy, o.woff, luts, obs + (size_t)env * obs_stride(OBS_MODE));
                staged = kBytes;
            }
        } else if (l == 0) {
            const uint32_t* rec = e + LDS_REC;   // not written back: still the episode that just ended
            s_list[atomicAdd(&s_ndone, 1)] = make_uint4((uint32_t)env, rec[RW_SEED_LO], rec[RW_SEED_HI], rec[RW_EPISODE] + 1u);
        }
    }
    if (kBytes && obs != nullptr) {
        if (l == 0) e[LDS_FLAG] = staged ? 1u : 0u;
        group_sync();
        const int first = (tid & ~63) / G;                         // first environment of this wave within the block
        flush_wave_observations<G, OBS_MODE>(s_env + first * LDS_ENV_DWORDS,
                                             obs + (size_t)(blockIdx.x * EPB + first) * obs_stride(OBS_MODE));
    }
    __syncthreads();
    const int nd = s_ndone;
    if (nd == 0) return;
    if (tid == 0) s_base = atomicAdd(dl.count, (uint32_t)nd);
    __syncthreads();
    if (tid < nd) dl.list[s_base + tid] = s_list[tid];
}

// Regenerates every environment on the done list (one block each, looping if the list is
// longer than the grid), renders its first observation, and clears the list for the next step.
template <int OBS_MODE>
__global__ __launch_bounds__(WG_THREADS) void k_reset_list(uint4* __restrict__ recs, uint8_t* __restrict__ maps,
                                                      const Luts* __restrict__ luts, uint8_t* __restrict__ obs,
                                                      DoneList dl, Params p)
{
    constexpr int G = 16;
    __shared__ uint16_t s_lat[LAT_BLOCKS * 8];
    __shared__ uint32_t s_env[LDS_ENV_DWORDS];
    uint4 entry = dl.list[blockIdx.x];   // fetched together with the count; ignored if beyond it
    // the scalars of a fresh episode are constants: fetch their table entries before anything else
    const float fresh_tenth = luts->tenth[MAX_COUNT], fresh_day = luts->daylight[0];
    const uint32_t fresh_q7 = luts->light_q7[0];
    const uint32_t count = *dl.count;
    if (blockIdx.x >= count) return;
    const int tid = threadIdx.x;
    // Every working block has now read the count; the last one to say so clears the list for
    // the next step (entries are only appended by the next step kernel, after this one ends).
    if (tid == 0) {
        const uint32_t workers = count < gridDim.x ? count : gridDim.x;
        if (atomicAdd(dl.finished, 1u) == workers - 1u) { *dl.count = 0u; *dl.finished = 0u; }
    }
    constexpr bool kSymbolic = OBS_MODE != CRAFTAX_OBS_PIXELS_F32;
    for (uint32_t i = blockIdx.x; i < count; i += gridDim.x) {
        if (i != blockIdx.x) entry = dl.list[i];
        const uint32_t env = entry.x, lo = entry.y, hi = entry.z, ep = entry.w;
        uint32_t* grec = reinterpret_cast<uint32_t*>(recs + (size_t)env * 8);
        uint8_t* map = maps + (size_t)env * (MAPW * MAPW);
        if (tid >= 64 && tid < 64 + REC_DWORDS) {              // wave 1 writes the record, wave 0 will render
            const uint32_t w = fresh_record_word(tid - 64, lo, hi, ep);
            grec[tid - 64] = w;
            s_env[LDS_REC + tid - 64] = w;
        }
        worldgen_block(map, s_lat, lo, hi, env, ep, s_env + LDS_WIN);   // ends with a block barrier
        if (kSymbolic && obs != nullptr && tid < G) {
            // scalars of a fresh episode: empty inventory, vitals 9, facing down, noon, awake
            uint32_t* vec = s_env + LDS_VEC;
            for (int i = tid; i < 24; i += G) {
                uint32_t w = 0;
                if (OBS_MODE == CRAFTAX_OBS_SYM_U8_I8) {
                    if (i == 3) w = 0x09090909u;                       // bytes 12..15: the four vitals
                    if (i == 4) w = 1u << 24;                          // byte 19: facing down
                    if (i == 5) w = fresh_q7;                          // byte 20: daylight
                } else {
                    if (i >= 12 && i < 16) w = __float_as_uint(fresh_tenth);
                    if (i == 19) w = __float_as_uint(1.0f);
                    if (i == 20) w = __float_as_uint(fresh_day);
                }
                vec[i] = w;
            }
            render_symbolic<G, OBS_MODE, false>(tid, s_env, 0, 0, (MAPW / 2 - WIN_COLS / 2) & 3, luts, obs + (size_t)env * obs_stride(OBS_MODE));
        }
        __syncthreads();
    }
}

template <int OBS_MODE>
__global__ __launch_bounds__(BLOCK) void k_observe(const uint4* __restrict__ recs, const uint8_t* __restrict__ maps,
                                                   const Luts* __restrict__ luts, uint8_t* __restrict__ obs, Params p)
{
    constexpr int G = 16, EPB = Grp<G>::EPB;
    __shared__ uint32_t s_env[EPB * LDS_ENV_DWORDS];
    const int tid = threadIdx.x, g = tid / G, l = tid % G;
    const int env = blockIdx.x * EPB + g;
    if (env >= p.n) return;
    uint32_t* e = s_env + g * LDS_ENV_DWORDS;
    load_record<G>(l, recs + (size_t)env * 8, e);
    group_sync();
    const uint32_t w_pos = e[LDS_REC + RW_POS];
    const int px = w_pos & 0xFF;
    load_window<G>(l, px, (w_pos >> 8) & 0xFF, maps + (size_t)env * (MAPW * MAPW), e + LDS_WIN);
    group_sync();
    render_symbolic<G, OBS_MODE>(l, e, 0, 0, (px - WIN_COLS / 2) & 3, luts, obs + (size_t)env * obs_stride(OBS_MODE));
}

__global__ __launch_bounds__(BLOCK) void k_pixels(const uint4* __restrict__ recs, const uint8_t* __restrict__ maps,
                                                  const Luts* __restrict__ luts, uint8_t* __restrict__ obs, Params p)
{
    __shared__ uint32_t s_rec[REC_DWORDS];
    __shared__ int s_tile[81], s_ent[81];
    const int env = blockIdx.x;
    if (threadIdx.x < REC_DWORDS) s_rec[threadIdx.x] = reinterpret_cast<const uint32_t*>(recs + (size_t)env * 8)[threadIdx.x];
    __syncthreads();
    float* out = reinterpret_cast<float*>(obs + (size_t)env * OBS_STRIDE_PIXELS);
    render_pixels_block(s_rec, maps + (size_t)env * (MAPW * MAPW), luts, out, s_tile, s_ent);
    if (threadIdx.x == 0) out[63 * 63 * 3] = 0.0f;   // the stride's padding word
}

// ---------------------------------------------------------------------------------------------
// canonical dumps: one block per environment
__global__ __launch_bounds__(BLOCK) void k_export(const uint4* __restrict__ recs, const uint8_t* __restrict__ maps,
                                                  craftax_env_dump* __restrict__ dumps, int first)
{
    const int env = first + blockIdx.x, tid = threadIdx.x;
    craftax_env_dump* d = dumps + blockIdx.x;
    {   // 16-byte piece tid of the tiled map = row (tid & 7) of tile (tid >> 3) -> row-major dump
        const int tile = tid >> 3, y = ((tile >> 2) << 3) + (tid & 7), x = (tile & 3) << 4;
        *reinterpret_cast<uint4*>(d->map + y * MAPW + x) = reinterpret_cast<const uint4*>(maps + (size_t)env * (MAPW * MAPW))[tid];
    }
    __shared__ uint32_t r[REC_DWORDS];
    if (tid < REC_DWORDS) r[tid] = reinterpret_cast<const uint32_t*>(recs + (size_t)env * 8)[tid];
    __syncthreads();
    if (tid == 0) {
        d->px = r[RW_POS] & 0xFF; d->py = (r[RW_POS] >> 8) & 0xFF; d->dir = (r[RW_POS] >> 16) & 0xFF; d->sleeping = r[RW_POS] >> 24;
        for (int i = 0; i < 6; ++i) { d->inv[i] = (r[RW_INV] >> (4 * i)) & 15; d->inv[6 + i] = (r[RW_INV] >> (24 + i)) & 1; }
        for (int i = 0; i < 4; ++i) { d->vit[i] = (int8_t)((r[RW_VIT] >> (4 * i)) & 15); d->cnt[i] = (int16_t)(int8_t)(r[RW_CNT] >> (8 * i)); }
        d->ach = r[RW_ACH]; d->t = r[RW_T]; d->episode = r[RW_EPISODE];
        d->seed = (uint64_t)r[RW_SEED_LO] | ((uint64_t)r[RW_SEED_HI] << 32);
        d->env = (uint32_t)env;
    }
    if (tid < NMOB) {
        const Mob m = unpack_mob(r[RW_MOB + tid]);
        craftax_mob o;
        o.alive = m.alive; o.x = m.x; o.y = m.y; o.dir = m.dir; o.hp = (int8_t)m.hp; o.cd = m.cd; o.pad[0] = 0; o.pad[1] = 0;
        d->mob[tid] = o;
    }
    if (tid >= 32 && tid < 32 + NPLANT) {
        const Plant q = unpack_plant(r[RW_PLANT + tid - 32]);
        craftax_plant o;
        o.alive = q.alive; o.x = q.x; o.y = q.y; o.pad = 0; o.age = (uint16_t)q.age;
        d->plant[tid - 32] = o;
    }
}

// Import packs into the record's bit fields: counts and vitals must be 0..15, counters
// -128..127, mob hp and cooldown 0..15, coordinates 0..63 (every state the rules can reach is).
__global__ __launch_bounds__(BLOCK) void k_import(uint4* __restrict__ recs, uint8_t* __restrict__ maps,
                                                  const craftax_env_dump* __restrict__ dumps, int first, Params p)
{
    const int env = first + blockIdx.x, tid = threadIdx.x;
    const craftax_env_dump* d = dumps + blockIdx.x;
    {
        const int tile = tid >> 3, y = ((tile >> 2) << 3) + (tid & 7), x = (tile & 3) << 4;
        reinterpret_cast<uint4*>(maps + (size_t)env * (MAPW * MAPW))[tid] = *reinterpret_cast<const uint4*>(d->map + y * MAPW + x);
    }
    __shared__ uint32_t r[REC_DWORDS];
    if (tid < REC_DWORDS) r[tid] = 0;
    __syncthreads();
    if (tid == 0) {
        r[RW_POS] = (uint32_t)d->px | ((uint32_t)d->py << 8) | ((uint32_t)d->dir << 16) | ((uint32_t)d->sleeping << 24);
        uint32_t wi = 0, wv = 0, wc = 0;
        for (int i = 0; i < 6; ++i) wi |= ((uint32_t)(d->inv[i] & 15) << (4 * i)) | ((uint32_t)(d->inv[6 + i] & 1) << (24 + i));
        for (int i = 0; i < 4; ++i) {
            wv |= (uint32_t)(d->vit[i] & 15) << (4 * i);
            const int c = max(-128, min(127, (int)d->cnt[i]));
            wc |= (uint32_t)(c & 0xFF) << (8 * i);
        }
        r[RW_INV] = wi;
        r[RW_VIT] = wv | ((d->t % p.day_length) << 16);
        r[RW_CNT] = wc;
        r[RW_ACH] = d->ach; r[RW_T] = d->t; r[RW_EPISODE] = d->episode;
        r[RW_SEED_LO] = (uint32_t)d->seed; r[RW_SEED_HI] = (uint32_t)(d->seed >> 32);
    }
    if (tid < NMOB) {
        const craftax_mob s = d->mob[tid];
        Mob m;
        m.alive = s.alive & 1; m.x = s.x & 63; m.y = s.y & 63; m.dir = s.dir & 7; m.hp = s.hp & 15; m.cd = s.cd & 15;
        r[RW_MOB + tid] = pack_mob(m);
    }
    if (tid >= 32 && tid < 32 + NPLANT) {
        const craftax_plant s = d->plant[tid - 32];
        Plant q;
        q.alive = s.alive & 1; q.x = s.x & 63; q.y = s.y & 63; q.age = s.age;
        r[RW_PLANT + tid - 32] = pack_plant(q);
    }
    __syncthreads();
    if (tid < REC_DWORDS) reinterpret_cast<uint32_t*>(recs + (size_t)env * 8)[tid] = r[tid];
}

// synthetic action stream (input generation for benchmarks; not part of the simulator)
__global__ void k_synth_actions(int32_t* __restrict__ actions, int n, int step0, int steps, uint32_t k0, uint32_t k1, int kind)
{
    const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= (size_t)n * (size_t)steps) return;
    const uint32_t s = (uint32_t)(i / (size_t)n), env = (uint32_t)(i % (size_t)n);
    const U4 r = philox4x32_10(env, (uint32_t)step0 + s, 0u, DOM_ACTIONS << 16, k0, k1);
    const uint32_t count = kind >= 2 ? 43u : (uint32_t)AC_COUNT;   // appendix "Action Space": 17 Classic, 43 Craftax
    int a;
    if ((kind & 1) == 0) a = (int)choice(r.w[0], count);
    else a = r.w[0] < 0x80000000u ? 1 + (int)choice(r.w[1], 5) : (int)choice(r.w[1], count);
    actions[i] = a;
}

// ---------------------------------------------------------------------------------------------
// host side
struct HostState {
    craftax_config cfg;
    int n;
    int lanes;   // lanes per environment used by the step kernel
    Header hdr;
};

static std::mutex g_mutex;
static std::unordered_map<const void*, HostState> g_states;
static thread_local std::string g_error;

static int fail(int code, const std::string& msg)
{
    g_error = msg;
    return code;
}

static bool config_ok(const craftax_config* c, std::string* why)
{
    if (c->variant == CRAFTAX_VARIANT_CRAFTAX) return cf::host::config_ok(c, why);
    if (c->abi_version != CRAFTAX_ABI_VERSION) { *why = "abi_version mismatch"; return false; }
    if (c->variant != CRAFTAX_VARIANT_CLASSIC) { *why = "unknown variant"; return false; }
    if (c->obs_mode > CRAFTAX_OBS_PIXELS_F32) { *why = "unknown obs_mode"; return false; }
    if (c->day_length < 2 || c->day_length > MAX_DAY || (c->day_length & 1)) { *why = "day_length must be even and in 2..1024"; return false; }
    if (c->cap_zombie > 3 || c->cap_cow > 3 || c->cap_skeleton > 3 || c->cap_arrow > 3) { *why = "mob caps must be 0..3"; return false; }
    if (c->cap_plant > NPLANT) { *why = "cap_plant must be 0..10"; return false; }
    if (c->max_episode_steps == 0) { *why = "max_episode_steps must be positive"; return false; }
    return true;
}

static uint64_t round_up(uint64_t v, uint64_t a) { return (v + a - 1) / a * a; }

static Header make_header(const craftax_config* c, int n)
{
    Header h;
    std::memset(&h, 0, sizeof(h));
    h.magic = MAGIC; h.version = CRAFTAX_ABI_VERSION; h.n = (uint32_t)n;
    h.obs_mode = c->obs_mode; h.max_episode_steps = c->max_episode_steps; h.day_length = c->day_length;
    h.cap_zombie = c->cap_zombie; h.cap_cow = c->cap_cow; h.cap_skeleton = c->cap_skeleton;
    h.cap_arrow = c->cap_arrow; h.cap_plant = c->cap_plant; h.atlas_seed = c->atlas_seed;
    h.off_luts = 256;
    h.off_recs = round_up(h.off_luts + sizeof(Luts), 256);
    h.off_maps = h.off_recs + (uint64_t)n * (REC_DWORDS * 4);
    h.off_done = h.off_maps + (uint64_t)n * (MAPW * MAPW);
    h.total = round_up(h.off_done + (uint64_t)n * 16, 256);
    return h;
}

// Lookup tables.  Day/night: phase i = t mod L, H = L/2, k = |i - H|, daylight =
// smoothstep(k/H) = k^2 (3H - 2k) / H^3 (noon at t = 0, midnight at t = H): the paper only
// says the observation carries a day/night value in [0,1] (appendix "Observation Space").
static void build_luts(const craftax_config* c, Luts* L)
{
    std::memset(L, 0, sizeof(*L));
    const uint64_t len = c->day_length, half = len / 2, den = half * half * half;
    for (uint64_t i = 0; i < len; ++i) {
        const uint64_t k = i < half ? half - i : i - half;
        const uint64_t num = k * k * (3 * half - 2 * k);
        L->daylight[i] = (float)((double)num / (double)den);
        const uint32_t dark = 255u - (uint32_t)(255u * num / den);
        L->zombie_thr[i] = (40u + 3u * dark) << 20;
        L->light_q7[i] = (uint8_t)(127u * num / den);
    }
    for (int i = 0; i < 16; ++i) {
        L->sqrt10[i] = (float)(std::sqrt((double)i) / 10.0);
        L->tenth[i] = (float)((double)i / 10.0);
    }
    const uint32_t k0 = (uint32_t)c->atlas_seed, k1 = (uint32_t)(c->atlas_seed >> 32);
    auto word = [&](uint32_t stream, uint32_t idx) {
        const U4 r = philox4x32_10(0u, stream, 0u, (DOM_ATLAS << 16) | (idx >> 2), k0, k1);
        return r.w[idx & 3u];
    };
    for (uint32_t i = 0; i < 16 * 147; ++i) L->tile[i] = (float)(word(0, i) >> 8) * (1.0f / 16777216.0f);
    for (uint32_t i = 0; i < 5 * 147; ++i) L->ent[i] = (float)(word(1, i) >> 8) * (1.0f / 16777216.0f);
    for (uint32_t i = 0; i < 5 * 49; ++i) L->ent_mask[i] = (uint8_t)(word(2, i) >> 31);
}

static Params make_params(const HostState& s)
{
    Params p;
    p.n = s.n;
    p.max_episode_steps = s.cfg.max_episode_steps; p.day_length = s.cfg.day_length;
    p.cap_zombie = s.cfg.cap_zombie; p.cap_cow = s.cfg.cap_cow; p.cap_skeleton = s.cfg.cap_skeleton;
    p.cap_arrow = s.cfg.cap_arrow; p.cap_plant = s.cfg.cap_plant;
    return p;
}

static int lookup(const void* state, int n, bool need_n, HostState* out)
{
    if (state == nullptr) return fail(CRAFTAX_E_NULL, "state is NULL");
    std::lock_guard<std::mutex> lock(g_mutex);
    auto it = g_states.find(state);
    if (it == g_states.end()) return fail(CRAFTAX_E_STATE, "state was not initialised by craftax_state_init");
    if (need_n && n != it->second.n) return fail(CRAFTAX_E_COUNT, "n differs from the n given to craftax_state_init");
    *out = it->second;
    return CRAFTAX_OK;
}

static int check_launch(const char* what)
{
    const hipError_t e = hipGetLastError();
    if (e != hipSuccess) return fail(CRAFTAX_E_HIP, std::string(what) + ": " + hipGetErrorString(e));
    return CRAFTAX_OK;
}

struct Ptrs { uint4* recs; uint8_t* maps; const Luts* luts; DoneList dl; };
static Ptrs pointers(const void* state, const HostState& s)
{
    uint8_t* base = const_cast<uint8_t*>(static_cast<const uint8_t*>(state));
    Ptrs q;
    q.luts = reinterpret_cast<const Luts*>(base + s.hdr.off_luts);
    q.recs = reinterpret_cast<uint4*>(base + s.hdr.off_recs);
    q.maps = base + s.hdr.off_maps;
    q.dl.count = reinterpret_cast<uint32_t*>(base + DONE_COUNT_OFFSET);
    q.dl.finished = q.dl.count + 1;
    q.dl.list = reinterpret_cast<uint4*>(base + s.hdr.off_done);
    return q;
}

// Lanes per environment: few lanes amortise the per-environment scalar work over more
// environments per wave and win once there are enough environments to fill the chip; many
// lanes give more, shorter waves and win for small batches.  The environment variable
// CRAFTAX_GROUP_LANES=4|8|16, read by craftax_state_init, overrides the choice (for tuning).
static int group_lanes(int n)
{
    const char* v = std::getenv("CRAFTAX_GROUP_LANES");
    const int g = v ? std::atoi(v) : 0;
    if (g == 4 || g == 8 || g == 16) return g;
    return n >= 32768 ? 4 : (n >= 8192 ? 8 : 16);
}

constexpr int RESET_GRID = 512;   // blocks of k_reset_list; those beyond the list exit at once

template <int OBS_MODE>
static void launch_step(int G, int n, hipStream_t st, const Ptrs& q, const int32_t* actions, uint8_t* o, float* reward,
                        uint8_t* done, const Params& p)
{
    const dim3 block(BLOCK);
    if (G == 4) hipLaunchKernelGGL((k_step<4, OBS_MODE>), dim3((n + 63) / 64), block, 0, st, q.recs, q.maps, q.luts, actions, o, reward, done, q.dl, p);
    else if (G == 8) hipLaunchKernelGGL((k_step<8, OBS_MODE>), dim3((n + 31) / 32), block, 0, st, q.recs, q.maps, q.luts, actions, o, reward, done, q.dl, p);
    else hipLaunchKernelGGL((k_step<16, OBS_MODE>), dim3((n + 15) / 16), block, 0, st, q.recs, q.maps, q.luts, actions, o, reward, done, q.dl, p);
    hipLaunchKernelGGL((k_reset_list<OBS_MODE>), dim3(n < RESET_GRID ? n : RESET_GRID), dim3(WG_THREADS), 0, st, q.recs, q.maps, q.luts, o, q.dl, p);
}

}  // namespace cx

using namespace cx;

extern "C" {

void craftax_default_config_for(craftax_config* cfg, uint32_t variant)
{
    if (!cfg) return;
    std::memset(cfg, 0, sizeof(*cfg));
    cfg->abi_version = CRAFTAX_ABI_VERSION;
    cfg->variant = variant;
    cfg->obs_mode = CRAFTAX_OBS_SYM_U8_F32;
    cfg->max_episode_steps = variant == CRAFTAX_VARIANT_CRAFTAX ? 100000 : 10000;
    cfg->day_length = 300;
    cfg->cap_zombie = cfg->cap_cow = cfg->cap_skeleton = cfg->cap_arrow = 3;
    if (variant == CRAFTAX_VARIANT_CRAFTAX) cfg->cap_skeleton = 2;
    cfg->cap_plant = 10;
    cfg->atlas_seed = 0;
}

void craftax_default_config(craftax_config* cfg) { craftax_default_config_for(cfg, CRAFTAX_VARIANT_CLASSIC); }

size_t craftax_state_bytes(const craftax_config* cfg, int n)
{
    std::string why;
    if (!cfg || n <= 0 || !config_ok(cfg, &why)) return 0;
    if (cfg->variant == CRAFTAX_VARIANT_CRAFTAX) return cf::host::state_bytes(cfg, n);
    return (size_t)make_header(cfg, n).total;
}

size_t craftax_obs_bytes(const craftax_config* cfg)
{
    if (!cfg || cfg->obs_mode > CRAFTAX_OBS_PIXELS_F32) return 0;
    if (cfg->variant == CRAFTAX_VARIANT_CRAFTAX) {
        std::string why;
        return cf::host::config_ok(cfg, &why) ? cf::host::obs_bytes(cfg) : 0;
    }
    return (size_t)obs_stride((int)cfg->obs_mode);
}

size_t craftax_env_dump_bytes(void) { return sizeof(craftax_env_dump); }
size_t craftax_env_dump_bytes_for(const craftax_config* cfg)
{
    if (!cfg) return 0;
    return cfg->variant == CRAFTAX_VARIANT_CRAFTAX ? sizeof(craftax_full_env_dump) : sizeof(craftax_env_dump);
}

int craftax_state_init(void* state, const craftax_config* cfg, int n, void* stream)
{
    if (!state || !cfg) return fail(CRAFTAX_E_NULL, "state or cfg is NULL");
    if ((uintptr_t)state % 256) return fail(CRAFTAX_E_ALIGN, "state must be 256-byte aligned");
    if (n <= 0) return fail(CRAFTAX_E_COUNT, "n must be positive");
    std::string why;
    if (!config_ok(cfg, &why)) return fail(CRAFTAX_E_CONFIG, why);
    HostState s;
    s.cfg = *cfg; s.n = n;
    if (cfg->variant == CRAFTAX_VARIANT_CRAFTAX) {
        std::memset(&s.hdr, 0, sizeof(s.hdr));
        s.lanes = 64;
        std::string err;
        if (int rc = cf::host::state_init(state, cfg, n, stream, &err)) return fail(rc, err);
        std::lock_guard<std::mutex> lock(g_mutex);
        g_states[state] = s;
        return CRAFTAX_OK;
    }
    s.hdr = make_header(cfg, n); s.lanes = group_lanes(n);
    std::vector<uint8_t> staging((size_t)s.hdr.off_recs, 0);
    std::memcpy(staging.data(), &s.hdr, sizeof(Header));
    build_luts(cfg, reinterpret_cast<Luts*>(staging.data() + s.hdr.off_luts));
    hipError_t e = hipMemcpyAsync(state, staging.data(), staging.size(), hipMemcpyHostToDevice, (hipStream_t)stream);
    if (e == hipSuccess) e = hipStreamSynchronize((hipStream_t)stream);   // staging dies with this call
    if (e != hipSuccess) return fail(CRAFTAX_E_HIP, std::string("state_init copy: ") + hipGetErrorString(e));
    std::lock_guard<std::mutex> lock(g_mutex);
    g_states[state] = s;
    return CRAFTAX_OK;
}

int craftax_state_release(void* state)
{
    std::lock_guard<std::mutex> lock(g_mutex);
    return g_states.erase(state) ? CRAFTAX_OK : fail(CRAFTAX_E_STATE, "unknown state");
}

int craftax_reset(void* state, const uint64_t* seeds, int n, void* stream)
{
    HostState s;
    if (int rc = lookup(state, n, true, &s)) return rc;
    if (!seeds) return fail(CRAFTAX_E_NULL, "seeds is NULL");
    if (s.cfg.variant == CRAFTAX_VARIANT_CRAFTAX) {
        std::string err;
        const int rc = cf::host::reset(state, &s.cfg, n, seeds, stream, &err);
        return rc ? fail(rc, err) : rc;
    }
    const Ptrs q = pointers(state, s);
    hipLaunchKernelGGL(k_reset, dim3(n), dim3(WG_THREADS), 0, (hipStream_t)stream, q.recs, q.maps, seeds, q.dl.count, q.dl.finished,
                       make_params(s));
    return check_launch("craftax_reset");
}

int craftax_step(void* state, const int32_t* actions, void* obs, float* reward, uint8_t* done, int n, void* stream)
{
    HostState s;
    if (int rc = lookup(state, n, true, &s)) return rc;
    if (!actions || !reward || !done) return fail(CRAFTAX_E_NULL, "actions, reward or done is NULL");
    if ((uintptr_t)obs % 16) return fail(CRAFTAX_E_ALIGN, "obs must be 16-byte aligned");
    if (s.cfg.variant == CRAFTAX_VARIANT_CRAFTAX) {
        std::string err;
        const int rc = cf::host::step(state, &s.cfg, n, actions, obs, reward, done, stream, &err);
        return rc ? fail(rc, err) : rc;
    }
    const Ptrs q = pointers(state, s);
    const Params p = make_params(s);
    hipStream_t st = (hipStream_t)stream;
    uint8_t* o = static_cast<uint8_t*>(obs);
    const int G = s.lanes;
    switch (s.cfg.obs_mode) {
    case CRAFTAX_OBS_SYM_U8_I8: launch_step<0>(G, n, st, q, actions, o, reward, done, p); break;
    case CRAFTAX_OBS_SYM_U8_F32: launch_step<1>(G, n, st, q, actions, o, reward, done, p); break;
    case CRAFTAX_OBS_SYM_F32: launch_step<2>(G, n, st, q, actions, o, reward, done, p); break;
    default:
        launch_step<3>(G, n, st, q, actions, o, reward, done, p);
        if (o) hipLaunchKernelGGL(k_pixels, dim3(n), dim3(BLOCK), 0, st, q.recs, q.maps, q.luts, o, p);
        break;
    }
    return check_launch("craftax_step");
}

int craftax_observe(void* state, void* obs, int n, void* stream)
{
    HostState s;
    if (int rc = lookup(state, n, true, &s)) return rc;
    if (!obs) return fail(CRAFTAX_E_NULL, "obs is NULL");
    if ((uintptr_t)obs % 16) return fail(CRAFTAX_E_ALIGN, "obs must be 16-byte aligned");
    if (s.cfg.variant == CRAFTAX_VARIANT_CRAFTAX) {
        std::string err;
        const int rc = cf::host::observe(state, &s.cfg, n, obs, stream, &err);
        return rc ? fail(rc, err) : rc;
    }
    const Ptrs q = pointers(state, s);
    const Params p = make_params(s);
    const dim3 grid((n + 15) / 16), block(BLOCK);
    hipStream_t st = (hipStream_t)stream;
    uint8_t* o = static_cast<uint8_t*>(obs);
    switch (s.cfg.obs_mode) {
    case CRAFTAX_OBS_SYM_U8_I8: hipLaunchKernelGGL(k_observe<0>, grid, block, 0, st, q.recs, q.maps, q.luts, o, p); break;
    case CRAFTAX_OBS_SYM_U8_F32: hipLaunchKernelGGL(k_observe<1>, grid, block, 0, st, q.recs, q.maps, q.luts, o, p); break;
    case CRAFTAX_OBS_SYM_F32: hipLaunchKernelGGL(k_observe<2>, grid, block, 0, st, q.recs, q.maps, q.luts, o, p); break;
    default: hipLaunchKernelGGL(k_pixels, dim3(n), block, 0, st, q.recs, q.maps, q.luts, o, p); break;
    }
    return check_launch("craftax_observe");
}

int craftax_export_envs(const void* state, int first, int count, void* dumps, void* stream)
{
    HostState s;
    if (int rc = lookup(state, 0, false, &s)) return rc;
    if (!dumps) return fail(CRAFTAX_E_NULL, "dumps is NULL");
    if (first < 0 || count <= 0 || first + count > s.n) return fail(CRAFTAX_E_COUNT, "range outside the state");
    if ((uintptr_t)dumps % 16) return fail(CRAFTAX_E_ALIGN, "dumps must be 16-byte aligned");
    if (s.cfg.variant == CRAFTAX_VARIANT_CRAFTAX) {
        std::string err;
        const int rc = cf::host::export_envs(state, &s.cfg, s.n, first, count, dumps, stream, &err);
        return rc ? fail(rc, err) : rc;
    }
    const Ptrs q = pointers(state, s);
    hipLaunchKernelGGL(k_export, dim3(count), dim3(BLOCK), 0, (hipStream_t)stream, q.recs, q.maps,
                       static_cast<craftax_env_dump*>(dumps), first);
    return check_launch("craftax_export_envs");
}

int craftax_import_envs(void* state, int first, int count, const void* dumps, void* stream)
{
    HostState s;
    if (int rc = lookup(state, 0, false, &s)) return rc;
    if (!dumps) return fail(CRAFTAX_E_NULL, "dumps is NULL");
    if (first < 0 || count <= 0 || first + count > s.n) return fail(CRAFTAX_E_COUNT, "range outside the state");
    if ((uintptr_t)dumps % 16) return fail(CRAFTAX_E_ALIGN, "dumps must be 16-byte aligned");
    if (s.cfg.variant == CRAFTAX_VARIANT_CRAFTAX) {
        std::string err;
        const int rc = cf::host::import_envs(state, &s.cfg, s.n, first, count, dumps, stream, &err);
        return rc ? fail(rc, err) : rc;
    }
    const Ptrs q = pointers(state, s);
    hipLaunchKernelGGL(k_import, dim3(count), dim3(BLOCK), 0, (hipStream_t)stream, q.recs, q.maps,
                       static_cast<const craftax_env_dump*>(dumps), first, make_params(s));
    return check_launch("craftax_import_envs");
}

int craftax_synth_actions(int32_t* actions, int n, int step0, int steps, uint64_t action_seed, int kind, void* stream)
{
    if (!actions) return fail(CRAFTAX_E_NULL, "actions is NULL");
    if (n <= 0 || steps <= 0 || step0 < 0 || kind < 0 || kind > 3) return fail(CRAFTAX_E_COUNT, "bad n, steps, step0 or kind");
    const size_t total = (size_t)n * (size_t)steps;
    hipLaunchKernelGGL(k_synth_actions, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, (hipStream_t)stream, actions, n,
                       step0, steps, (uint32_t)action_seed, (uint32_t)(action_seed >> 32), kind);
    return check_launch("craftax_synth_actions");
}

const char* craftax_last_error(void) { return g_error.c_str(); }

}  // extern "C"
