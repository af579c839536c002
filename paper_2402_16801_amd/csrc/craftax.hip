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
// Worlds are generated ahead of time (appendix "Optimistic Environment Resets" explains why
// world generation is the expensive part of a reset): map slot e & 1 holds the world of
// episode e, the other slot the world of episode e + 1.  An episode that ends switches slots
// inside the step kernel and puts the environment on a regeneration list; extra blocks of the
// NEXT step launch fill the freed slot with the world after next, in the shadow of the step
// blocks.  Two tags per environment (one per half of the map) say which episode its spare slot holds and which launch wrote
// it; a spare is only trusted when an earlier launch wrote it.  The spare of an episode is
// generated during that episode's first step, so only an episode that ends at its first step
// finds it missing; a fresh episode cannot (full vitals, cleared start area, no mobs) unless the
// episode cap is 1.  Such episodes go on the slow list, which k_reset_list serves right after
// the step kernel; it is launched only for an episode cap of 1.  craftax_reset and
// craftax_import_envs generate the spare themselves.
// A list entry carries what world generation needs: (env, seed low, seed high, episode index);
// env = ENTRY_VOID marks an entry cancelled by an import.
// Each regeneration list is cut into NSUB sub-lists with their own counters (blocks append to
// sub-list blockIdx mod NSUB), so that the appending atomics do not queue up on one address;
// sub_cap is the capacity of a sub-list.
struct Lists { uint32_t* ctr; uint4* regen[2]; uint4* slow; uint2* tags; uint32_t sub_cap; };
__device__ inline uint32_t* counter(const Lists& ls, int i) { return ls.ctr + (size_t)i * CTR_STRIDE; }
constexpr uint32_t TAG_NONE = 0xFFFFFFFFu, ENTRY_VOID = 0xFFFFFFFFu;

// reset: two blocks per environment, for the worlds of episodes 0 and 1
__global__ __launch_bounds__(WG_THREADS) void k_reset(uint4* __restrict__ recs, uint8_t* __restrict__ maps,
                                                 const uint64_t* __restrict__ seeds, Lists ls)
{
    if (blockIdx.x == 0 && threadIdx.x < CT_COUNT) *counter(ls, threadIdx.x) = threadIdx.x == CT_SEQ ? 1u : 0u;
    __shared__ uint16_t s_lat[LAT_BLOCKS * 8];
    const uint32_t env = blockIdx.x >> 1, ep = blockIdx.x & 1u;
    const uint64_t seed = seeds[env];
    const uint32_t lo = (uint32_t)seed, hi = (uint32_t)(seed >> 32);
    worldgen_block(maps + map_offset(env, ep), s_lat, lo, hi, env, ep);
    if (ep == 0) {
        if (threadIdx.x < REC_DWORDS)
            reinterpret_cast<uint32_t*>(recs + (size_t)env * 8)[threadIdx.x] = fresh_record_word(threadIdx.x, lo, hi, 0u);
    } else if (threadIdx.x < 2) ls.tags[2 * env + threadIdx.x] = make_uint2(1u, 0u);
}

// A regeneration block of the step grid: worlds for the episodes after next of the episodes that
// ended in the previous launch.
__device__ __forceinline__ void regeneration_block(uint8_t* __restrict__ maps, const Lists& ls, uint32_t seq, uint32_t count,
                                                   uint32_t rb, uint32_t nrb, uint16_t* s_lat)
{
    const uint32_t which = (seq & 1u) ^ 1u, sub = rb % NSUB;
    const uint4* list = ls.regen[which] + (size_t)sub * ls.sub_cap;
    // two blocks per world, one half each: a regeneration block is then as short as it can be with
    // one run of 8 cells per thread, and the tail it adds to the launch is half as long
    const uint32_t pair = rb / NSUB, half = pair & 1u;
    for (uint32_t i = pair >> 1; i < count; i += nrb / NSUB / 2) {
        const uint4 entry = list[i];
        if (entry.x == ENTRY_VOID) continue;
        worldgen_block<BLOCK>(maps + map_offset(entry.x, entry.w), s_lat, entry.y, entry.z, entry.x, entry.w, nullptr,
                              (int)half * (WG_THREADS / 2), WG_THREADS / 2);
        if (threadIdx.x == 0) ls.tags[2 * entry.x + half] = make_uint2(entry.w, seq);
    }
}

// ---------------------------------------------------------------------------------------------
// step: G lanes per environment, 256/G environments per block, followed in the same grid by
// the regeneration blocks for the episodes that ended in the previous launch.
template <int G, int OBS_MODE>
__global__ __launch_bounds__(BLOCK, 4) void k_step(uint4* __restrict__ recs, uint8_t* __restrict__ maps,
                                                   const Luts* __restrict__ luts, const int32_t* __restrict__ actions,
                                                   uint8_t* __restrict__ obs, float* __restrict__ reward,
                                                   uint8_t* __restrict__ done, Lists ls, Params p, int step_blocks)
{
    constexpr int EPB = Grp<G>::EPB;
    __shared__ uint32_t s_env[EPB * LDS_ENV_DWORDS];
    __shared__ int s_ndone;
    __shared__ uint32_t s_base;
    __shared__ uint4 s_list[EPB];
    const int tid = threadIdx.x;
    // Launch number.  Every block reads it (and, as a regeneration block, the length of its
    // sub-list) and then counts itself in; once all blocks of the launch have done so, one thread
    // advances the number and empties the lists this launch consumes.  Counting is in two levels
    // (NGROUP group counters, then one on top) so that no counter sees more than a few dozen atomics.
    const uint32_t seq = *counter(ls, CT_SEQ);
    const bool regen_role = (int)blockIdx.x >= step_blocks;
    const uint32_t rb = blockIdx.x - (uint32_t)step_blocks, nrb = gridDim.x - (uint32_t)step_blocks;
    uint32_t regen_count = 0u;
    if (regen_role) regen_count = *counter(ls, CT_REGEN + (int)(((seq & 1u) ^ 1u) * NSUB + rb % NSUB));
    const uint32_t gsize = (gridDim.x + NGROUP - 1) / NGROUP, grp = blockIdx.x / gsize;
    uint32_t started = 0u;
    asm volatile("" :: "v"(seq), "v"(regen_count) : "memory");   // both values have arrived before this block counts itself in
    if (tid == 0) started = atomicAdd(counter(ls, CT_GROUP + (int)grp), 1u);
    auto leave = [&]() {
        if (tid != 0) return;
        const uint32_t members = min(gsize, gridDim.x - grp * gsize), ngroups = (gridDim.x + gsize - 1) / gsize;
        if (started != members - 1u) return;
        *counter(ls, CT_GROUP + (int)grp) = 0u;
        if (atomicAdd(counter(ls, CT_TOP), 1u) != ngroups - 1u) return;
        *counter(ls, CT_TOP) = 0u;
        for (int sub = 0; sub < NSUB; ++sub) *counter(ls, CT_REGEN + (int)(((seq & 1u) ^ 1u) * NSUB) + sub) = 0u;
        *counter(ls, CT_SEQ) = seq + 1u;
    };

    if (regen_role) {
        if (rb / NSUB / 2 < regen_count)
            regeneration_block(maps, ls, seq, regen_count, rb, nrb, reinterpret_cast<uint16_t*>(s_env));
        leave();
        return;
    }

    const int g = tid / G, l = tid % G;
    const int env = blockIdx.x * EPB + g;
    const bool active = env < p.n;
    if (tid == 0) s_ndone = 0;
    __syncthreads();
    uint32_t* e = s_env + g * LDS_ENV_DWORDS;
    constexpr bool kSymbolic = OBS_MODE != CRAFTAX_OBS_PIXELS_F32;
    constexpr bool kBytes = OBS_MODE == CRAFTAX_OBS_SYM_U8_I8 || OBS_MODE == CRAFTAX_OBS_SYM_U8_F32;
    bool staged = false;
    if (active) {
        load_record<G>(l, recs + (size_t)env * 8, e);
        group_sync();
        const uint32_t* rec = e + LDS_REC;
        const uint32_t ep = rec[RW_EPISODE], lo = rec[RW_SEED_LO], hi = rec[RW_SEED_HI];
        StepOut o = step_env<G>(l, (uint32_t)env, e, maps + map_offset((uint32_t)env, ep), luts, actions[env], p);
        if (l == 0) { reward[env] = o.reward; done[env] = o.done ? 1 : 0; }
        bool write_back = !o.done;
        if (o.done) {
            // the record in LDS is still the episode that just ended
            const uint4 tag = reinterpret_cast<const uint4*>(ls.tags)[env];   // (episode, launch) of the two halves of the spare world
            if (tag.x == ep + 1u && tag.y < seq && tag.z == ep + 1u && tag.w < seq) {
                // the next world is waiting in the other slot: start the new episode right here
                group_sync();
#pragma unroll
                for (int it = 0; it < (REC_DWORDS + G - 1) / G; ++it) {
                    const int i = l + it * G;
                    if (i < REC_DWORDS) e[LDS_REC + i] = fresh_record_word(i, lo, hi, ep + 1u);
                }
                load_window<G>(l, MAPW / 2, MAPW / 2, maps + map_offset((uint32_t)env, ep + 1u), e + LDS_WIN);
                group_sync();
                o.mvx = 0; o.mvy = 0; o.woff = (MAPW / 2 - WIN_COLS / 2) & 3;
                write_back = true;
                if (l == 0) s_list[atomicAdd(&s_ndone, 1)] = make_uint4((uint32_t)env, lo, hi, ep + 2u);
            } else if (l == 0) {
                ls.slow[atomicAdd(counter(ls, CT_SLOW), 1u)] = make_uint4((uint32_t)env, lo, hi, ep + 1u);
            }
        }
        if (write_back) {
            store_record<G>(l, recs + (size_t)env * 8, e);
            if (kSymbolic && obs != nullptr) {
                // byte layouts are staged in LDS here and written by the whole wave below
                render_symbolic<G, OBS_MODE, true, !kBytes>(l, e, o.mvx, o.mvy, o.woff, luts, obs + (size_t)env * obs_stride(OBS_MODE));
                staged = kBytes;
            }
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
    leave();
    const int nd = s_ndone;
    if (nd == 0) return;
    const uint32_t sub = blockIdx.x % NSUB;
    if (tid == 0) s_base = atomicAdd(counter(ls, CT_REGEN + (int)((seq & 1u) * NSUB + sub)), (uint32_t)nd);
    __syncthreads();
    if (tid < nd) ls.regen[seq & 1u][(size_t)sub * ls.sub_cap + s_base + tid] = s_list[tid];
}

// Serves the slow list: generates the world of the new episode in place (one block each, looping
// if the list is longer than the grid), writes the fresh record, renders the first observation,
// and asks the next step launch to generate the world after it.  Runs after the step kernel (which
// has already advanced the launch number), and only when the episode cap is 1.
template <int OBS_MODE>
__global__ __launch_bounds__(WG_THREADS) void k_reset_list(uint4* __restrict__ recs, uint8_t* __restrict__ maps,
                                                      const Luts* __restrict__ luts, uint8_t* __restrict__ obs,
                                                      Lists ls, Params p, int envs_per_step_block)
{
    constexpr int G = 16;
    __shared__ uint16_t s_lat[LAT_BLOCKS * 8];
    __shared__ uint32_t s_env[LDS_ENV_DWORDS];
    const int tid = threadIdx.x;
    const uint32_t count = *counter(ls, CT_SLOW);
    if (blockIdx.x >= count) return;
    const uint32_t next = (*counter(ls, CT_SEQ) & 1u) ^ 1u;      // the list the next launch's regeneration blocks will read
    // the scalars of a fresh episode are constants: fetch their table entries before anything else
    const float fresh_tenth = luts->tenth[MAX_COUNT], fresh_day = luts->daylight[0];
    const uint32_t fresh_q7 = luts->light_q7[0];
    constexpr bool kSymbolic = OBS_MODE != CRAFTAX_OBS_PIXELS_F32;
    for (uint32_t i = blockIdx.x; i < count; i += gridDim.x) {
        const uint4 entry = ls.slow[i];
        if (entry.x == ENTRY_VOID) continue;
        const uint32_t env = entry.x, lo = entry.y, hi = entry.z, ep = entry.w;
        uint32_t* grec = reinterpret_cast<uint32_t*>(recs + (size_t)env * 8);
        if (tid >= 64 && tid < 64 + REC_DWORDS) {              // wave 1 writes the record, wave 0 will render
            const uint32_t w = fresh_record_word(tid - 64, lo, hi, ep);
            grec[tid - 64] = w;
            s_env[LDS_REC + tid - 64] = w;
        }
        if (tid == 96) {   // same sub-list as the environment's step block uses, so that no sub-list can overflow
            const uint32_t sub = (env / (uint32_t)envs_per_step_block) % NSUB;
            const uint32_t at = atomicAdd(counter(ls, CT_REGEN + (int)(next * NSUB + sub)), 1u);
            ls.regen[next][(size_t)sub * ls.sub_cap + at] = make_uint4(env, lo, hi, ep + 1u);
        }
        worldgen_block(maps + map_offset(env, ep), s_lat, lo, hi, env, ep, s_env + LDS_WIN);   // ends with a block barrier
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
    // the last working block empties the list
    if (tid == 0) {
        const uint32_t workers = count < gridDim.x ? count : gridDim.x;
        if (atomicAdd(counter(ls, CT_SLOW_FINISHED), 1u) == workers - 1u) { *counter(ls, CT_SLOW) = 0u; *counter(ls, CT_SLOW_FINISHED) = 0u; }
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
    load_window<G>(l, px, (w_pos >> 8) & 0xFF, maps + map_offset((uint32_t)env, e[LDS_REC + RW_EPISODE]), e + LDS_WIN);
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
    render_pixels_block(s_rec, maps + map_offset((uint32_t)env, s_rec[RW_EPISODE]), luts, out, s_tile, s_ent);
    if (threadIdx.x == 0) out[63 * 63 * 3] = 0.0f;   // the stride's padding word
}

// ---------------------------------------------------------------------------------------------
// canonical dumps: one block per environment
__global__ __launch_bounds__(BLOCK) void k_export(const uint4* __restrict__ recs, const uint8_t* __restrict__ maps,
                                                  craftax_env_dump* __restrict__ dumps, int first)
{
    const int env = first + blockIdx.x, tid = threadIdx.x;
    craftax_env_dump* d = dumps + blockIdx.x;
    __shared__ uint32_t r[REC_DWORDS];
    if (tid < REC_DWORDS) r[tid] = reinterpret_cast<const uint32_t*>(recs + (size_t)env * 8)[tid];
    __syncthreads();
    {   // 16-byte piece tid of the tiled map = row (tid & 7) of tile (tid >> 3) -> row-major dump
        const int tile = tid >> 3, y = ((tile >> 2) << 3) + (tid & 7), x = (tile & 3) << 4;
        *reinterpret_cast<uint4*>(d->map + y * MAPW + x) = reinterpret_cast<const uint4*>(maps + map_offset((uint32_t)env, r[RW_EPISODE]))[tid];
    }
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
__global__ __launch_bounds__(BLOCK) void k_import(uint4* __restrict__ recs, uint8_t* __restrict__ maps, Lists ls,
                                                  const craftax_env_dump* __restrict__ dumps, int first, Params p)
{
    const int env = first + blockIdx.x, tid = threadIdx.x;
    const craftax_env_dump* d = dumps + blockIdx.x;
    {
        const int tile = tid >> 3, y = ((tile >> 2) << 3) + (tid & 7), x = (tile & 3) << 4;
        reinterpret_cast<uint4*>(maps + map_offset((uint32_t)env, d->episode))[tid] = *reinterpret_cast<const uint4*>(d->map + y * MAPW + x);
    }
    // whatever was queued for this environment belongs to the episode that is being replaced
    for (int li = 0; li < 2 * NSUB + 1; ++li) {
        uint4* list = li < 2 * NSUB ? ls.regen[li / NSUB] + (size_t)(li % NSUB) * ls.sub_cap : ls.slow;
        const uint32_t cnt = *counter(ls, li < 2 * NSUB ? CT_REGEN + li : CT_SLOW);
        for (uint32_t i = tid; i < cnt; i += BLOCK) if (list[i].x == (uint32_t)env) list[i].x = ENTRY_VOID;
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

// after an import: the world of the episode after the imported one, into the spare slot
__global__ __launch_bounds__(WG_THREADS) void k_import_spare(const uint4* __restrict__ recs, uint8_t* __restrict__ maps, Lists ls, int first)
{
    __shared__ uint16_t s_lat[LAT_BLOCKS * 8];
    const uint32_t env = (uint32_t)first + blockIdx.x;
    const uint32_t* r = reinterpret_cast<const uint32_t*>(recs + (size_t)env * 8);
    const uint32_t ep = r[RW_EPISODE] + 1u, lo = r[RW_SEED_LO], hi = r[RW_SEED_HI];
    worldgen_block(maps + map_offset(env, ep), s_lat, lo, hi, env, ep);
    if (threadIdx.x < 2) ls.tags[2 * env + threadIdx.x] = make_uint2(ep, 0u);
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

// Entries a regeneration sub-list must hold: every environment of the step blocks that append to
// it, for the narrowest lane group (most environments per block).
static uint64_t sub_list_capacity(int n)
{
    const uint64_t epb = 64, blocks = ((uint64_t)n + epb - 1) / epb;
    return ((blocks + NSUB - 1) / NSUB) * epb + epb;
}

static Header make_header(const craftax_config* c, int n)
{
    Header h;
    std::memset(&h, 0, sizeof(h));
    h.magic = MAGIC; h.version = CRAFTAX_ABI_VERSION; h.n = (uint32_t)n;
    h.obs_mode = c->obs_mode; h.max_episode_steps = c->max_episode_steps; h.day_length = c->day_length;
    h.cap_zombie = c->cap_zombie; h.cap_cow = c->cap_cow; h.cap_skeleton = c->cap_skeleton;
    h.cap_arrow = c->cap_arrow; h.cap_plant = c->cap_plant; h.atlas_seed = c->atlas_seed;
    h.off_ctrs = 256;
    h.off_luts = h.off_ctrs + (uint64_t)CT_COUNT * CTR_STRIDE * 4;
    h.off_recs = round_up(h.off_luts + sizeof(Luts), 256);
    h.off_maps = h.off_recs + (uint64_t)n * (REC_DWORDS * 4);
    h.off_tags = h.off_maps + (uint64_t)n * 2 * (MAPW * MAPW);     // two map slots per environment
    h.off_regen0 = round_up(h.off_tags + (uint64_t)n * 16, 256);
    const uint64_t list_bytes = (uint64_t)NSUB * sub_list_capacity(n) * 16;
    h.off_regen1 = h.off_regen0 + list_bytes;
    h.off_slow = h.off_regen1 + list_bytes;
    h.total = round_up(h.off_slow + (uint64_t)n * 16, 256);
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

struct Ptrs { uint4* recs; uint8_t* maps; const Luts* luts; Lists ls; };
static Ptrs pointers(const void* state, const HostState& s)
{
    uint8_t* base = const_cast<uint8_t*>(static_cast<const uint8_t*>(state));
    Ptrs q;
    q.luts = reinterpret_cast<const Luts*>(base + s.hdr.off_luts);
    q.recs = reinterpret_cast<uint4*>(base + s.hdr.off_recs);
    q.maps = base + s.hdr.off_maps;
    q.ls.ctr = reinterpret_cast<uint32_t*>(base + s.hdr.off_ctrs);
    q.ls.sub_cap = (uint32_t)sub_list_capacity(s.n);
    q.ls.regen[0] = reinterpret_cast<uint4*>(base + s.hdr.off_regen0);
    q.ls.regen[1] = reinterpret_cast<uint4*>(base + s.hdr.off_regen1);
    q.ls.slow = reinterpret_cast<uint4*>(base + s.hdr.off_slow);
    q.ls.tags = reinterpret_cast<uint2*>(base + s.hdr.off_tags);
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

constexpr int RESET_GRID = 64;    // blocks of k_reset_list (the slow list is nearly always empty); each loops over the list
constexpr int REGEN_BLOCKS = 1024; // regeneration blocks appended to the step grid (two per world); those beyond the list exit at once

template <int OBS_MODE>
static void launch_step(int G, int n, hipStream_t st, const Ptrs& q, const int32_t* actions, uint8_t* o, float* reward,
                        uint8_t* done, const Params& p)
{
    const dim3 block(BLOCK);
    const int regen = ((2 * n < REGEN_BLOCKS ? 2 * n : REGEN_BLOCKS) + 2 * NSUB - 1) / (2 * NSUB) * (2 * NSUB);   // a multiple of twice the sub-list count
    const int sb = (n + 256 / G - 1) / (256 / G);
    if (G == 4) hipLaunchKernelGGL((k_step<4, OBS_MODE>), dim3(sb + regen), block, 0, st, q.recs, q.maps, q.luts, actions, o, reward, done, q.ls, p, sb);
    else if (G == 8) hipLaunchKernelGGL((k_step<8, OBS_MODE>), dim3(sb + regen), block, 0, st, q.recs, q.maps, q.luts, actions, o, reward, done, q.ls, p, sb);
    else hipLaunchKernelGGL((k_step<16, OBS_MODE>), dim3(sb + regen), block, 0, st, q.recs, q.maps, q.luts, actions, o, reward, done, q.ls, p, sb);
    if (p.max_episode_steps == 1u)   // the only way an episode can end before its spare world exists
        hipLaunchKernelGGL((k_reset_list<OBS_MODE>), dim3(n < RESET_GRID ? n : RESET_GRID), dim3(WG_THREADS), 0, st, q.recs, q.maps, q.luts, o, q.ls, p, 256 / G);
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
    hipLaunchKernelGGL(k_reset, dim3(2u * (unsigned)n), dim3(WG_THREADS), 0, (hipStream_t)stream, q.recs, q.maps, seeds, q.ls);
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
    hipLaunchKernelGGL(k_import, dim3(count), dim3(BLOCK), 0, (hipStream_t)stream, q.recs, q.maps, q.ls,
                       static_cast<const craftax_env_dump*>(dumps), first, make_params(s));
    hipLaunchKernelGGL(k_import_spare, dim3(count), dim3(WG_THREADS), 0, (hipStream_t)stream, q.recs, q.maps, q.ls, first);
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
