// Kernels and host entry points of the full-Craftax variant (nine floors, 43 actions).
#include "full_api.hpp"
#include "launch_limits.hpp"

#include <hip/hip_runtime.h>

#include <cmath>
#include <cstring>
#include <vector>

#include "worldgen.hpp"
#include "full_common.hpp"
#include "full_render.hpp"
#include "full_pixels.hpp"
#include "full_step.hpp"
#include "full_worldgen.hpp"

namespace cf {

static_assert(sizeof(craftax_full_env_dump) == 63432, "canonical dump layout");

using la::Lists;
using la::counter;
using la::ENTRY_VOID;
using la::NSUB;

constexpr int EAGER_SPARE_ENVS = 8192;   // up to here a step fetches the spare world's start window in advance (see kf_step)
constexpr int RESET_SLOTS = 64;    // environments served at once by kf_reset_list (nine blocks each)
constexpr int MAX_ENVS_PER_STEP_BLOCK = 16;   // a step block holds 4 environments (a wavefront each) or 16 (16 lanes each)
constexpr int REGEN_BLOCKS = 256;  // regeneration blocks at the head of the step grid: with 1,024 step blocks (4,096 environments) they fill the chip exactly

__device__ inline uint32_t pack_regs(const MobRegs& m)
{
    Mob o;
    o.alive = m.alive; o.x = m.x; o.y = m.y; o.dir = m.dir; o.hp = m.hp; o.cd = m.cd; o.type = m.type;
    return pack_mob(o);
}

// What the block that generated floor 0 of a world leaves behind for the environment: as the
// current world (fresh record, empty mob tables) or as the spare world (its ladders and potion map).
__device__ inline void publish_world(uint32_t* __restrict__ genv, const GenLayout& L, uint32_t lo, uint32_t hi, uint32_t ep,
                                     bool current, uint32_t* s_layout_words)
{
    const int tid = threadIdx.x;
    if (tid < FLOORS + 1) s_layout_words[tid] = layout_word(L, tid);
    __syncthreads();
    if (current) {
        if (tid < SPARE_LADDER) genv[tid] = tid < REC_DWORDS ? fresh_record_word(tid, s_layout_words, lo, hi, ep) : 0u;
    } else if (tid < FLOORS + 1) genv[SPARE_LADDER + tid] = s_layout_words[tid];
}

// ---------------------------------------------------------------------------------------------
// reset of every environment: one block per (environment, episode 0 or 1, floor)
__global__ __launch_bounds__(GEN_THREADS) void kf_reset(uint32_t* __restrict__ envs, uint8_t* __restrict__ maps,
                                                       const uint64_t* __restrict__ seeds, Lists ls, const uint32_t* __restrict__ perlin_cs,
                                                       int pool, uint32_t* __restrict__ unlocks)
{
    if (blockIdx.x == 0) la::reset_counters(ls);
    __shared__ uint16_t s_lat[LAT_TOTAL];
    __shared__ GenLayout s_layout;
    __shared__ uint32_t s_words[FLOORS + 1];
    const uint32_t env = blockIdx.x / (2 * FLOORS), ep = (blockIdx.x / FLOORS) & 1u;
    const int f = blockIdx.x % FLOORS;
    const uint64_t seed = seeds[env];
    const uint32_t lo = (uint32_t)seed, hi = (uint32_t)(seed >> 32);
    worldgen_floor_block<GEN_THREADS, true>(maps + map_offset(env, ep), s_lat, s_layout, lo, hi, env, ep, f, nullptr, nullptr, 0, GEN_THREADS, perlin_cs);
    if (f == 0) publish_world(envs + (size_t)env * ENV_DWORDS, s_layout, lo, hi, ep, ep == 0u, s_words);
    if (f == 0 && ep == 0u && threadIdx.x < UNLOCK_STRIDE) unlocks[(size_t)env * UNLOCK_STRIDE + threadIdx.x] = 0u;
    // With optimistic resets no spare world is ever valid: tag 0 matches no next episode (they count
    // from 1), so the step kernel hands every finished episode to kf_reset_list.
    if (ep == 1u && threadIdx.x == 0) ls.tags[(size_t)env * NTAG + f] = make_uint2(pool ? 0u : 1u, 0u);
}

// The regeneration blocks of the step grid: worlds after next for the episodes that ended in the
// previous launch.  The consumed list is one dense queue of work units, one floor of one world
// each; block rb of nrb takes units rb, rb + nrb, ...  The blocks stand at the head of the grid:
// a step launch holds as many of them as the chip has room for beside the step blocks, so every
// unit starts with the launch and none waits for a block that is scheduled late.
// where a regeneration block keeps its scratch in the step kernel's LDS area (dwords): lattice numbers at 0, the layout at 128
constexpr int REGEN_WORDS_AT = 832, REGEN_PREFIX_AT = 848;
template <bool PERLIN>
__device__ __forceinline__ void regeneration_queue(uint32_t* __restrict__ envs, uint8_t* __restrict__ maps, const Lists& ls,
                                                   uint32_t seq, uint32_t* lds, int regen_blocks, const uint32_t* __restrict__ perlin_cs)
{
    uint16_t* s_lat = reinterpret_cast<uint16_t*>(lds);
    GenLayout& L = *reinterpret_cast<GenLayout*>(lds + 128);
    uint32_t* s_words = lds + REGEN_WORDS_AT;
    const uint32_t* s_prefix = lds + REGEN_PREFIX_AT;
    const uint32_t units = s_prefix[NSUB - 1] * (uint32_t)FLOORS;
    for (uint32_t u = blockIdx.x; u < units; u += (uint32_t)regen_blocks) {
        __syncthreads();   // the previous unit's scratch has been read by everyone
        const uint4 entry = la::queue_entry(ls, seq, s_prefix, u / FLOORS);
        const int f = (int)(u % FLOORS);
        if (entry.x == ENTRY_VOID) continue;
        worldgen_floor_block<BLOCK, PERLIN>(maps + map_offset(entry.x, entry.w), s_lat, L, entry.y, entry.z, entry.x, entry.w, f, nullptr, nullptr,
                                            0, GEN_THREADS, PERLIN ? perlin_cs : nullptr);
        if (f == 0) publish_world(envs + (size_t)entry.x * ENV_DWORDS, L, entry.y, entry.z, entry.w, false, s_words);
        if (threadIdx.x == 0) ls.tags[(size_t)entry.x * NTAG + f] = make_uint2(entry.w, seq);
    }
}
static_assert(LAT_TOTAL * 2 <= 128 * 4 && sizeof(GenLayout) <= (REGEN_WORDS_AT - 128) * 4 && REGEN_WORDS_AT + FLOORS + 1 <= REGEN_PREFIX_AT &&
              REGEN_PREFIX_AT + NSUB <= ENVS_PER_BLOCK * L_ENV_DWORDS, "regeneration scratch overlaps");

// ---------------------------------------------------------------------------------------------
// step: one wavefront per environment, four environments per block; the grid starts with the
// regeneration blocks for the episodes that ended in the previous launch.
// EAGER: the window of the spare world's start position is fetched in every step, with the current
// window, so that an episode that ends switches worlds without a further trip to memory.  With a
// few thousand environments the launch ends when its slowest block ends, and that trip would sit
// on exactly those blocks (+0.7 us per launch at 4,096 environments); with tens of thousands the
// kernel is bound by instruction issue and the hundred instructions per step cost more than the
// rare trip (255 -> 216 us per launch at 65,536 environments).
// PERLIN: the regeneration blocks generate Perlin worlds (a kernel of its own, so that the value-noise
// kernel carries none of that code).
// GW: lanes per environment (see Lanes): 64 = one wavefront per environment, four environments per
// block; 16 = four environments per wavefront, sixteen per block.
template <bool F32, bool EAGER, bool PERLIN, int GW>
__global__ __launch_bounds__(BLOCK, GW == 64 ? 5 : 2) void kf_step(uint32_t* __restrict__ envs, uint8_t* __restrict__ maps,
                                                const Luts* __restrict__ luts, const int32_t* __restrict__ actions,
                                                uint8_t* __restrict__ obs, float* __restrict__ reward,
                                                uint8_t* __restrict__ done, Lists ls, Params p, int regen_blocks)
{
    using G = Lanes<GW>;
    constexpr int EPB = BLOCK / GW;                          // environments per block
    constexpr int REC_IT = REC_DWORDS / GW > 0 ? REC_DWORDS / GW : 1;
    constexpr int WIN_IT = (WIN_ROWS * WIN_COLS + GW - 1) / GW;
    static_assert(REC_DWORDS % GW == 0 || GW > REC_DWORDS, "the record is moved in whole turns of the group");
    static_assert(GW >= MOBTAB_DWORDS && GW >= NTAG && GW >= FLOORS + 1, "a group holds a mob table, the tags and the header in one turn");
    __shared__ uint32_t s_env[EPB * L_ENV_DWORDS];
    __shared__ float s_lut[LUT_FLOATS];
    const int tid = threadIdx.x, w = tid / GW, l = tid % GW;
    if ((int)blockIdx.x < regen_blocks) {
        const la::Ticket ticket = la::enter_launch_queue(ls, s_env + REGEN_PREFIX_AT);
        regeneration_queue<PERLIN>(envs, maps, ls, ticket.seq, s_env, regen_blocks, luts->perlin_cs);
        la::leave_launch(ls, ticket);
        return;
    }
    const uint32_t step_block = blockIdx.x - (uint32_t)regen_blocks;
    const int env = (int)step_block * EPB + w;
    const bool active = env < p.n;
    uint32_t* genv = envs + (size_t)(active ? env : 0) * ENV_DWORDS;
    // Everything that depends on the environment's number alone is fetched before the launch
    // bookkeeping, whose own trip to memory then costs nothing extra: the record, the action, and
    // what a finished episode needs from the spare world (its tags, its ladders and potion map).
    uint32_t rec_word[REC_IT], hdr = 0u;
    int action_raw = 0;
    uint2 tag = make_uint2(0u, 0u);
#pragma unroll
    for (int it = 0; it < REC_IT; ++it) rec_word[it] = 0u;
    // what the renderer looks up in tables: asked for now, used at the end of the step
    RenderAux<GW> aux;
    fetch_scalar_specs<GW>(l, aux);
    aux.lut = s_lut;
    if (tid < LUT_FLOATS) s_lut[tid] = luts->sqrt10[tid];     // sqrt10, tenth and light20 lie one after the other
    if (active) {
#pragma unroll
        for (int it = 0; it < REC_IT; ++it) if (l + GW * it < REC_DWORDS) rec_word[it] = genv[l + GW * it];
        action_raw = actions[env];
        if (l < NTAG) tag = ls.tags[(size_t)env * NTAG + l];
        if (l < FLOORS + 1) hdr = genv[SPARE_LADDER + l];
    }
    const la::Ticket ticket = la::enter_launch(ls, false, 0u);
    const uint32_t seq = ticket.seq;
    __syncthreads();                                          // the conversion tables are in LDS
    if (active) {
        uint32_t* e = s_env + w * L_ENV_DWORDS;
#pragma unroll
        for (int it = 0; it < REC_IT; ++it) if (l + GW * it < REC_DWORDS) e[L_REC + l + GW * it] = rec_word[it];
        const int action = G::uni(action_raw);
        wave_sync();
        const uint32_t ep = G::uniu(e[L_REC + R_EPISODE]), lo = G::uniu(e[L_REC + R_SEED_LO]), hi = G::uniu(e[L_REC + R_SEED_HI]);
        // daylight of the state that will be rendered: the next phase, or phase 0 of a fresh episode
        const uint32_t phase_now = G::uniu(e[L_REC + R_MANA]) >> 16;
        const float day_next = luts->daylight[phase_now + 1u == p.day_length ? 0u : phase_now + 1u], day_fresh = luts->daylight[0];
        MobRegs m;
        uint32_t qw;
        Player P;
        // the window of the spare world's start position comes with the current window
        const uint8_t* spare = maps + map_offset((uint32_t)env, ep + 1u);
        uint32_t sw[WIN_IT];
#pragma unroll
        for (int it = 0; it < WIN_IT; ++it) {
            const int i = l + GW * it;
            sw[it] = 0u;
            if (EAGER && i < WIN_ROWS * WIN_COLS) {
                const int r = i / WIN_COLS, c = i - r * WIN_COLS;
                const int x = W / 2 - WIN_COLS / 2 + c, y = W / 2 - WIN_ROWS / 2 + r;
                sw[it] = (uint32_t)spare[block_off(0, x, y)] | ((uint32_t)spare[il_off(0, x, y)] << 8);
            }
        }
        auto park = [&]() {
            if (l < NTAG) { e[L_SPARE_TAG + 2 * l] = tag.x; e[L_SPARE_TAG + 2 * l + 1] = tag.y; }
            if (l < FLOORS + 1) e[L_SPARE_HDR + l] = hdr;
#pragma unroll
            for (int it = 0; it < WIN_IT; ++it) {
                const int i = l + GW * it;
                if (EAGER && i < WIN_ROWS * WIN_COLS) {
                    const int r = i / WIN_COLS, c = i - r * WIN_COLS;
                    reinterpret_cast<uint8_t*>(e + L_SPARE_WB)[r * WIN_PITCH + c] = (uint8_t)sw[it];
                    reinterpret_cast<uint8_t*>(e + L_SPARE_WI)[r * WIN_PITCH + c] = (uint8_t)(sw[it] >> 8);
                }
            }
        };
        StepOut o = step_env<GW>(l, (uint32_t)env, e, genv, maps + map_offset((uint32_t)env, ep), luts, action, p, m, qw, P, park);
        if (l == 0) { reward[env] = o.reward; done[env] = o.done ? 1 : 0; }
#pragma unroll
        for (int aw = 0; aw < 3; ++aw) count_unlocks<GW>(l, p.unlocks + (size_t)env * UNLOCK_STRIDE, aw, o.unlocked[aw]);
        bool write_back = !o.done, queued = false;
        uint32_t list_at = 0u;
        int floor_now = P.floor;
        if (!o.done) {
            if (l == 0) pack_player(e + L_REC, P);
            if (l < NPLANT) e[L_REC + R_PLANT + l] = qw;
            wave_sync();
        } else {
            // every part of the next world must have been written by an earlier launch
            constexpr uint32_t ALL = (1u << NTAG) - 1u;
            const bool ready = (G::ballot(l < NTAG && e[L_SPARE_TAG + 2 * (l < NTAG ? l : 0)] == ep + 1u &&
                                          e[L_SPARE_TAG + 2 * (l < NTAG ? l : 0) + 1] < seq) & ALL) == ALL;
            if (ready) {
                // start the new episode right here: fresh record from the spare world's ladders and
                // potion map, all mob tables empty, window of the start position from the other slot
                wave_sync();
#pragma unroll
                for (int it = 0; it < REC_IT; ++it)
                    if (l + GW * it < REC_DWORDS) e[L_REC + l + GW * it] = fresh_record_word(l + GW * it, e + L_SPARE_HDR, lo, hi, ep + 1u);
                if (EAGER) {
#pragma unroll
                    for (int it = 0; it < (WIN_ROWS * WIN_PITCH / 4 + GW - 1) / GW; ++it) {
                        const int i = l + GW * it;
                        if (i < WIN_ROWS * WIN_PITCH / 4) { e[L_WB + i] = e[L_SPARE_WB + i]; e[L_WI + i] = e[L_SPARE_WI + i]; }
                    }
                } else {
                    load_window<GW>(l, maps + map_offset((uint32_t)env, ep + 1u), 0, W / 2, W / 2, reinterpret_cast<uint8_t*>(e + L_WB),
                                    reinterpret_cast<uint8_t*>(e + L_WI));
                }
#pragma unroll
                for (int it = 0; it < (FLOORS * MOBTAB_DWORDS + GW - 1) / GW; ++it) {
                    const int i = l + GW * it;
                    if (i < FLOORS * MOBTAB_DWORDS) genv[REC_DWORDS + i] = 0u;
                }
                clear_mob(m);
                floor_now = 0;
                o.wx0 = W / 2 - WIN_COLS / 2; o.wy0 = W / 2 - WIN_ROWS / 2;
                wave_sync();
                write_back = true;
                if (l == 0) list_at = la::claim_entry(ls, seq, step_block);   // the place on the list; the entry follows after the rendering
                queued = true;
            } else if (l == 0) {
                la::append_slow(ls, (uint32_t)p.n, make_uint4((uint32_t)env, lo, hi, ep + 1u));
            }
        }
        if (write_back) {
#pragma unroll
            for (int it = 0; it < REC_IT; ++it) if (l + GW * it < REC_DWORDS) genv[l + GW * it] = e[L_REC + l + GW * it];
            if (l < MOBTAB_DWORDS) genv[REC_DWORDS + floor_now * MOBTAB_DWORDS + l] = l < NSLOT ? pack_regs(m) : 0u;
            if (obs != nullptr) {
                aux.day = o.done ? day_fresh : day_next;
                render_env<F32, GW>(l, e, o.wx0, o.wy0, m.alive, m.x, m.y, m.type, luts, obs + (size_t)env * (F32 ? STRIDE_F32 : STRIDE_U8), &aux);
            }
        }
        if (queued && l == 0) la::commit_entry(ls, seq, step_block, list_at, make_uint4((uint32_t)env, lo, hi, ep + 2u));
    }
    la::leave_launch(ls, ticket);
}

// ---------------------------------------------------------------------------------------------
// rollout: several steps in one launch (see craftax_rollout).  A block keeps the records of its
// four environments in LDS for the whole launch, every wavefront walks its environment through
// the steps, and the block meets at a barrier once per step.  Worlds stay one episode ahead as in
// the step kernel, but the block generates them itself: an environment whose episode ends moves
// into the spare world in its other map slot (ladders and potion map from the header, the start
// window from the map), and the whole block then generates the world after it into the slot that
// was left, floor by floor (the other environments of the block wait those few hundred
// microseconds; nothing is exchanged between blocks, so blocks drift apart and the memory traffic
// of some overlaps the arithmetic of others).  At the end the block writes the records back and
// tags the spare worlds it wrote as written by launch 0, which is what the step kernel expects.
// Before the launch the regeneration lists of the step kernel must be empty (the host runs a
// list-only launch first); a spare world that is missing nonetheless is generated on the spot.
template <bool F32, bool PERLIN>
__global__ __launch_bounds__(BLOCK, 4) void kf_rollout(uint32_t* __restrict__ envs, uint8_t* __restrict__ maps,
                                                       const Luts* __restrict__ luts, const int32_t* __restrict__ actions,
                                                       uint8_t* __restrict__ obs, float* __restrict__ reward,
                                                       uint8_t* __restrict__ done, uint2* __restrict__ tags, Params p, int steps)
{
    __shared__ uint32_t s_env[ENVS_PER_BLOCK * L_ENV_DWORDS];
    __shared__ uint16_t s_lat[LAT_TOTAL];
    __shared__ GenLayout s_layout;
    __shared__ uint32_t s_words[FLOORS + 1];
    __shared__ int s_ended[ENVS_PER_BLOCK];          // this step ended the episode of environment w
    __shared__ int s_spare_ok[ENVS_PER_BLOCK];       // the world of the next episode is complete in the other map slot
    __shared__ int s_changed[ENVS_PER_BLOCK];        // this launch has written a spare world for environment w
    const int tid = threadIdx.x, w = tid >> 6, l = tid & 63;
    const int env = blockIdx.x * ENVS_PER_BLOCK + w;
    const bool active = env < p.n;
    uint32_t* e = s_env + w * L_ENV_DWORDS;
    uint32_t* genv = envs + (size_t)(active ? env : 0) * ENV_DWORDS;
    if (active) e[L_REC + l] = genv[l];
    if (l == 0) { s_ended[w] = 0; s_spare_ok[w] = 0; s_changed[w] = 0; }
    __syncthreads();
    if (active) {
        const uint32_t ep = uniu(e[L_REC + R_EPISODE]);
        uint2 tag = make_uint2(0u, 0u);
        if (l < NTAG) tag = tags[(size_t)env * NTAG + l];
        constexpr uint64_t ALL = (1ull << NTAG) - 1ull;
        const bool complete = (__ballot(l < NTAG && tag.x == ep + 1u) & ALL) == ALL;
        if (l == 0 && complete) s_spare_ok[w] = 1;
    }

    // Generates the world of episode `ep` of block-local environment ww into its map slot, all threads
    // of the block; leaves the ten layout words in s_words.  start: drop the cells around the start
    // position into that environment's LDS windows.
    auto generate = [&](int ww, uint32_t ep, bool start) __attribute__((always_inline)) {
        uint32_t* ew = s_env + ww * L_ENV_DWORDS;
        const uint32_t wenv = (uint32_t)(blockIdx.x * ENVS_PER_BLOCK + ww), lo = ew[L_REC + R_SEED_LO], hi = ew[L_REC + R_SEED_HI];
        uint8_t* slot = maps + map_offset(wenv, ep);
#pragma unroll 1
        for (int f = 0; f < FLOORS; ++f) {
            worldgen_floor_block<BLOCK, PERLIN>(slot, s_lat, s_layout, lo, hi, wenv, ep, f,
                                                start ? reinterpret_cast<uint8_t*>(ew + L_WB) : nullptr,
                                                start ? reinterpret_cast<uint8_t*>(ew + L_WI) : nullptr, 0, GEN_THREADS,
                                                PERLIN ? luts->perlin_cs : nullptr);
            if (f == 0) {                             // the layout of floor 0 describes the whole world
                if (tid < FLOORS + 1) s_words[tid] = layout_word(s_layout, tid);
                __syncthreads();
            }
        }
    };

#pragma unroll 1
    for (int t = 0; t < steps; ++t) {
        // Everything a lane derives from its index is derived again in every turn: the compiler would
        // otherwise keep dozens of such values alive across the whole loop and spill them.
        int tid_t = threadIdx.x;
        uint8_t* obs_t = obs;
        asm volatile("" : "+v"(tid_t));
        asm volatile("" : "+s"(obs_t));
        const int tid = tid_t, w = tid >> 6, l = tid & 63;
        const int env = blockIdx.x * ENVS_PER_BLOCK + w;
        const bool active = env < p.n;
        uint32_t* e = s_env + w * L_ENV_DWORDS;
        uint32_t* genv = envs + (size_t)(active ? env : 0) * ENV_DWORDS;
        uint8_t* obs = obs_t;
        MobRegs m;
        clear_mob(m);
        StepOut o;
        o.done = false; o.reward = 0.0f; o.wx0 = 0; o.wy0 = 0; o.unlocked[0] = o.unlocked[1] = o.unlocked[2] = 0u;
        int floor_now = 0;
        if (active) {
            const int action = uni(actions[(size_t)t * p.n + env]);
            const uint32_t ep = uniu(e[L_REC + R_EPISODE]);
            uint32_t qw;
            Player P;
            o = step_env(l, (uint32_t)env, e, genv, maps + map_offset((uint32_t)env, ep), luts, action, p, m, qw, P, []() {});
            if (l == 0) { reward[(size_t)t * p.n + env] = o.reward; done[(size_t)t * p.n + env] = o.done ? 1 : 0; }
#pragma unroll
            for (int aw = 0; aw < 3; ++aw) count_unlocks<64>(l, p.unlocks + (size_t)env * UNLOCK_STRIDE, aw, o.unlocked[aw]);
            floor_now = P.floor;
            if (!o.done) {
                if (l == 0) pack_player(e + L_REC, P);
                if (l < NPLANT) e[L_REC + R_PLANT + l] = qw;
                wave_sync();
            } else if (l == 0) s_ended[w] = 1;
        }
        __syncthreads();
        // the worlds of the episodes that start now
#pragma unroll 1
        for (int ww = 0; ww < ENVS_PER_BLOCK; ++ww) {
            if (!s_ended[ww]) continue;
            uint32_t* ew = s_env + ww * L_ENV_DWORDS;
            const uint32_t ep1 = ew[L_REC + R_EPISODE] + 1u, lo = ew[L_REC + R_SEED_LO], hi = ew[L_REC + R_SEED_HI];
            const uint32_t wenv = (uint32_t)(blockIdx.x * ENVS_PER_BLOCK + ww);
            uint32_t* wgenv = envs + (size_t)wenv * ENV_DWORDS;
            __syncthreads();
            const bool waiting = s_spare_ok[ww] != 0;
            if (waiting) {
                // the world is waiting in the other slot: its ladders and potion map from the header,
                // the window of its start position from the map
                if (tid < FLOORS + 1) s_words[tid] = wgenv[SPARE_LADDER + tid];
                if (tid >= 64 && tid < 128)
                    load_window(tid - 64, maps + map_offset(wenv, ep1), 0, W / 2, W / 2, reinterpret_cast<uint8_t*>(ew + L_WB),
                                reinterpret_cast<uint8_t*>(ew + L_WI));
                __syncthreads();
            }
            // turn 0 (only if no world was waiting): the world of the new episode, on the spot; turn 1:
            // the world after it, into the slot that has just been left, so that the next end of an
            // episode finds it (and the step kernel after this launch)
#pragma unroll 1
            for (int turn = waiting ? 1 : 0; turn < 2; ++turn) {
                if (turn == 1) {
                    // fresh record in LDS, empty mob tables in memory
                    if (tid < REC_DWORDS) ew[L_REC + tid] = fresh_record_word(tid, s_words, lo, hi, ep1);
                    if (tid < FLOORS * MOBTAB_DWORDS) wgenv[REC_DWORDS + tid] = 0u;
                    __syncthreads();
                }
                generate(ww, ep1 + (uint32_t)turn, turn == 0);
            }
            if (tid < FLOORS + 1) wgenv[SPARE_LADDER + tid] = s_words[tid];
            if (tid == 0) { s_spare_ok[ww] = 1; s_changed[ww] = 1; }
            __syncthreads();
        }
        if (active) {
            if (o.done) {
                clear_mob(m);
                floor_now = 0;
                o.wx0 = W / 2 - WIN_COLS / 2; o.wy0 = W / 2 - WIN_ROWS / 2;
                if (l == 0) s_ended[w] = 0;
            }
            if (l < MOBTAB_DWORDS) genv[REC_DWORDS + floor_now * MOBTAB_DWORDS + l] = l < NSLOT ? pack_regs(m) : 0u;
            if (obs != nullptr)
                render_env<F32>(l, e, o.wx0, o.wy0, m.alive, m.x, m.y, m.type, luts, obs + (size_t)env * (F32 ? STRIDE_F32 : STRIDE_U8));
        }
        __syncthreads();
    }
    // records back; spare worlds for the step kernel
    if (active) genv[l] = e[L_REC + l];
#pragma unroll 1
    for (int ww = 0; ww < ENVS_PER_BLOCK; ++ww) {
        const int wenv = blockIdx.x * ENVS_PER_BLOCK + ww;
        if (wenv >= p.n) continue;
        uint32_t* ew = s_env + ww * L_ENV_DWORDS;
        const uint32_t ep = ew[L_REC + R_EPISODE];
        if (s_spare_ok[ww] && !s_changed[ww]) continue;           // its spare world and tags are as the launch found them
        __syncthreads();
        if (!s_spare_ok[ww]) {
            generate(ww, ep + 1u, false);
            uint32_t* wgenv = envs + (size_t)wenv * ENV_DWORDS;
            if (tid < FLOORS + 1) wgenv[SPARE_LADDER + tid] = s_words[tid];
        }
        if (tid < NTAG) tags[(size_t)wenv * NTAG + tid] = make_uint2(ep + 1u, 0u);
        __syncthreads();
    }
}

// Serves the slow list: generates the world of the new episode in place (nine blocks each, looping
// if the list is longer than the grid); the block of floor 0 writes the fresh record, renders the
// first observation and asks the next step launch for the world after it.  Runs after the step
// kernel, and only when the episode cap is 1.
template <bool F32>
__global__ __launch_bounds__(GEN_THREADS) void kf_reset_list(uint32_t* __restrict__ envs, uint8_t* __restrict__ maps,
                                                            const Luts* __restrict__ luts, uint8_t* __restrict__ obs, Lists ls, int perlin,
                                                            const uint8_t* __restrict__ done, int n, int pool)
{
    __shared__ uint16_t s_lat[LAT_TOTAL];
    __shared__ GenLayout s_layout;
    __shared__ uint32_t s_words[FLOORS + 1];
    __shared__ uint32_t s_env[L_ENV_DWORDS];
    __shared__ uint32_t s_rank[(GEN_THREADS + 63) / 64];
    // Optimistic resets (pool != 0): the world comes from this step's pool.  The step kernel has
    // already advanced the launch number: it is the index of the step just done + 2.  The pool is
    // keyed by the seed of environment 0 (whoever rewrites that record writes the same seed back).
    const uint32_t step_index = pool ? *counter(ls, la::CT_SEQ) - 2u : 0u;
    const uint32_t pool_lo = pool ? envs[R_SEED_LO] : 0u, pool_hi = pool ? envs[R_SEED_HI] : 0u;
    const uint32_t pool_size = (uint32_t)n / cx::POOL_RATIO ? (uint32_t)n / cx::POOL_RATIO : 1u;
    const uint32_t count = la::slow_count(ls, ls.slow_cap);
    const uint32_t slot = blockIdx.x / FLOORS, slots = gridDim.x / FLOORS;
    const int f = blockIdx.x % FLOORS;
    if (slot >= count) return;
    const int tid = threadIdx.x;
    for (uint32_t i = slot; i < count; i += slots) {
        const uint4 entry = ls.slow[i];
        if (entry.x == ENTRY_VOID) continue;
        const uint32_t env = entry.x, lo = entry.y, hi = entry.z, ep = entry.w;
        uint32_t wlo = lo, whi = hi, wenv = env, wep = ep;   // the world's identity: the environment's own ...
        if (pool) {
            // ... or the pool's: rank of this environment among the finished ones = finished environments before it
            uint32_t before = 0u;
            for (uint32_t j = (uint32_t)tid; j < env; j += GEN_THREADS) before += done[j];
            for (int o = 32; o > 0; o >>= 1) before += __shfl_down(before, o);
            __syncthreads();                                  // the previous entry's ranks have been read
            if ((tid & 63) == 0) s_rank[tid >> 6] = before;
            __syncthreads();
            uint32_t rank = 0u;
#pragma unroll
            for (int w = 0; w < (GEN_THREADS + 63) / 64; ++w) rank += s_rank[w];
            const cx::U4 sh = cx::philox4x32_10(0xFFFFFFFFu, 2u, step_index, cx::DOM_WORLDGEN << 16, pool_lo, pool_hi);
            wlo = pool_lo; whi = pool_hi; wenv = cx::POOL_ENV | ((cx::choice(sh.w[0], pool_size) + rank) % pool_size); wep = step_index;
        }
        worldgen_floor_block<GEN_THREADS, true>(maps + map_offset(env, ep), s_lat, s_layout, wlo, whi, wenv, wep, f,
                                                reinterpret_cast<uint8_t*>(s_env + L_WB), reinterpret_cast<uint8_t*>(s_env + L_WI), 0, GEN_THREADS,
                                                perlin ? luts->perlin_cs : nullptr);
        if (f == 0) {
            publish_world(envs + (size_t)env * ENV_DWORDS, s_layout, lo, hi, ep, true, s_words);
            if (tid < REC_DWORDS) s_env[L_REC + tid] = fresh_record_word(tid, s_words, lo, hi, ep);
            if (tid == 96 && !pool) la::append_after_step(ls, env / ENVS_PER_BLOCK, make_uint4(env, lo, hi, ep + 1u));
            __syncthreads();
            if (obs != nullptr && tid < 64)
                render_env<F32>(tid, s_env, W / 2 - WIN_COLS / 2, W / 2 - WIN_ROWS / 2, 0, 0, 0, 0, luts,
                                obs + (size_t)env * (F32 ? STRIDE_F32 : STRIDE_U8));
        }
        __syncthreads();
    }
    // the last working block empties the list (nine blocks per served slot)
    if (tid == 0) {
        const uint32_t workers = (count < slots ? count : slots) * FLOORS;
        if (atomicAdd(counter(ls, la::CT_SLOW_FINISHED), 1u) == workers - 1u) { *counter(ls, la::CT_SLOW) = 0u; *counter(ls, la::CT_SLOW_FINISHED) = 0u; }
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
    const uint32_t pos = uniu(e[L_REC + R_POS]), ep = uniu(e[L_REC + R_EPISODE]);
    const int px = pos & 0xFF, py = (pos >> 8) & 0xFF, f = (pos >> 24) & 0xF;
    const Mob u = unpack_mob(l < NSLOT ? genv[REC_DWORDS + f * MOBTAB_DWORDS + l] : 0u);
    load_window(l, maps + map_offset((uint32_t)env, ep), f, px, py, reinterpret_cast<uint8_t*>(e + L_WB), reinterpret_cast<uint8_t*>(e + L_WI));
    wave_sync();
    render_env<F32>(l, e, px - WIN_COLS / 2, py - WIN_ROWS / 2, u.alive, u.x, u.y, u.type, luts,
                    obs + (size_t)env * (F32 ? STRIDE_F32 : STRIDE_U8));
}

// after an import: the world of the episode after the imported one, into the spare slot
__global__ __launch_bounds__(GEN_THREADS) void kf_import_spare(uint32_t* __restrict__ envs, uint8_t* __restrict__ maps, Lists ls, int first,
                                                                const uint32_t* __restrict__ perlin_cs, int pool)
{
    __shared__ uint16_t s_lat[LAT_TOTAL];
    __shared__ GenLayout s_layout;
    __shared__ uint32_t s_words[FLOORS + 1];
    const uint32_t env = (uint32_t)first + blockIdx.x / FLOORS;
    const int f = blockIdx.x % FLOORS;
    uint32_t* genv = envs + (size_t)env * ENV_DWORDS;
    const uint32_t ep = genv[R_EPISODE] + 1u, lo = genv[R_SEED_LO], hi = genv[R_SEED_HI];
    worldgen_floor_block<GEN_THREADS, true>(maps + map_offset(env, ep), s_lat, s_layout, lo, hi, env, ep, f, nullptr, nullptr, 0, GEN_THREADS, perlin_cs);
    if (f == 0) publish_world(genv, s_layout, lo, hi, ep, false, s_words);
    if (threadIdx.x == 0) ls.tags[(size_t)env * NTAG + f] = make_uint2(pool ? 0u : ep, 0u);
}

// Noise mutation (section "Craftax-1B: UED"): one block per (environment, floor) of the floors
// f0 .. f0 + nf - 1.  The level is the vector of the Perlin angles of every noise lattice: the
// overworld's 228, then 98 for each of the cave floors 2, 5, 6, 7.  The block of a floor adds to its
// own segment a uniform offset in [-amplitude, amplitude] per element (u16 number i of stream
// (round, 1) of the mutation domain, i counted over the whole vector) and generates the floor of
// the current episode again from the turned lattice; the block of floor 0 then starts the episode
// over.  Floor 0 runs in a launch of its own after the others: its block rewrites the record the
// others read their seed and episode from.
__device__ inline int theta_offset(int f)
{
    return f == 0 ? 0 : LAT0_U16 + LATC_U16 * (f == 2 ? 0 : (f == 5 ? 1 : (f == 6 ? 2 : 3)));
}
__global__ __launch_bounds__(GEN_THREADS) void kf_mutate_noise(uint32_t* __restrict__ envs, uint8_t* __restrict__ maps, const Luts* __restrict__ luts,
                                                                uint16_t* __restrict__ theta, int first, int f0, int nf, uint32_t k0, uint32_t k1,
                                                                uint32_t round, uint32_t amplitude)
{
    __shared__ uint16_t s_lat[LAT_TOTAL];
    __shared__ uint16_t s_theta[LAT_TOTAL];
    __shared__ GenLayout s_layout;
    __shared__ uint32_t s_words[FLOORS + 1];
    const int tid = threadIdx.x, slot = blockIdx.x / nf, f = f0 + blockIdx.x % nf;
    const uint32_t env = (uint32_t)first + (uint32_t)slot;
    uint32_t* genv = envs + (size_t)env * ENV_DWORDS;
    const uint32_t ep = genv[R_EPISODE], lo = genv[R_SEED_LO], hi = genv[R_SEED_HI];
    const bool noisy = f == 0 || is_cave(f);
    if (tid < LAT_TOTAL) {
        uint16_t v = 0;
        const int len = f == 0 ? LAT0_U16 : LATC_U16;
        if (noisy && tid < len) {
            const int i = theta_offset(f) + tid;
            uint16_t* th = theta + (size_t)slot * CRAFTAX_FULL_THETA_LEN + i;
            const cx::U4 d = cx::philox4x32_10(env, round, 1u, (cx::DOM_MUTATE << 16) | (uint32_t)(i >> 3), k0, k1);
            const uint32_t w = d.w[(i >> 1) & 3], d16 = (i & 1) ? (w >> 16) : (w & 0xFFFFu);
            const int u = (int)((d16 * (2u * amplitude + 1u)) >> 16) - (int)amplitude;
            v = (uint16_t)(((int)(*th & 1023u) + u) & 1023);
            *th = v;
        }
        s_theta[tid] = v;
    }
    __syncthreads();
    worldgen_floor_block<GEN_THREADS, true>(maps + map_offset(env, ep), s_lat, s_layout, lo, hi, env, ep, f, nullptr, nullptr, 0, GEN_THREADS,
                                            luts->perlin_cs, noisy ? s_theta : nullptr);
    if (f == 0) publish_world(genv, s_layout, lo, hi, ep, true, s_words);
}

// ---------------------------------------------------------------------------------------------
// canonical dumps: one block per environment
__global__ __launch_bounds__(BLOCK) void kf_export(const uint32_t* __restrict__ envs, const uint8_t* __restrict__ maps,
                                                  craftax_full_env_dump* __restrict__ dumps, int first)
{
    const int env = first + blockIdx.x, tid = threadIdx.x;
    craftax_full_env_dump* d = dumps + blockIdx.x;
    const uint32_t* r = envs + (size_t)env * ENV_DWORDS;
    const uint8_t* em = maps + map_offset((uint32_t)env, r[R_EPISODE]);
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

// Import packs into the record's bit fields: counts 0..99, vitals 0..31, counters -128..127, mob
// hp 0..31, cooldown 0..15, creature type 0..18, experience 0..15, coordinates 0..47, floor 0..8,
// block ids 1..36, items 0..4, light 0..20 (every state the rules can reach is); values outside
// are brought into range so that no kernel ever indexes beyond its tables or buffers.
__global__ __launch_bounds__(BLOCK) void kf_import(uint32_t* __restrict__ envs, uint8_t* __restrict__ maps, Lists ls,
                                                  const craftax_full_env_dump* __restrict__ dumps, int first, Params p)
{
    const int env = first + blockIdx.x, tid = threadIdx.x;
    const craftax_full_env_dump* d = dumps + blockIdx.x;
    uint8_t* em = maps + map_offset((uint32_t)env, d->episode);
    la::cancel_entries(ls, (uint32_t)env);   // whatever was queued for this environment belongs to the episode that is being replaced
    uint32_t* r = envs + (size_t)env * ENV_DWORDS;
    for (int i = tid; i < FLOORS * CELLS; i += BLOCK) {
        const int f = i / CELLS, c = i - f * CELLS;
        const uint32_t b = d->block[f][c], it = d->item[f][c];
        em[(size_t)f * 2 * CELLS + c] = (uint8_t)(b - 1u < (uint32_t)(B_COUNT - 1) ? b : (uint32_t)B_OOB);
        em[(size_t)f * 2 * CELLS + CELLS + c] = (uint8_t)((it <= 4u ? it : 0u) | ((uint32_t)min((int)d->light[f][c], 20) << 3));
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
        for (int i = 0; i < 10; ++i) s[R_INV + (i >> 2)] |= (uint32_t)min((int)d->inv[i], 99) << (8 * (i & 3));
        for (int i = 0; i < 6; ++i) { const int b = 10 + i; s[R_INV + (b >> 2)] |= (uint32_t)min((int)d->potion[i], 99) << (8 * (b & 3)); }
        uint32_t wv = 0, wc = 0;
        for (int i = 0; i < 4; ++i) {
            wv |= (uint32_t)max(0, min(31, (int)d->vit[i])) << (8 * i);
            wc |= (uint32_t)(max(-128, min(127, (int)d->cnt[i])) & 0xFF) << (8 * i);
        }
        s[R_VIT] = wv; s[R_CNT] = wc;
        s[R_MANA] = (uint32_t)max(0, min(31, (int)d->vit[4])) | ((uint32_t)(max(-128, min(127, (int)d->cnt[4])) & 0xFF) << 8) |
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
        m.type = min((int)u.type, 18);
        s[REC_DWORDS + f * MOBTAB_DWORDS + k] = pack_mob(m);
    }
    if (tid >= 128 && tid < 128 + NPLANT) {
        const craftax_plant u = d->plant[tid - 128];
        s[R_PLANT + tid - 128] = (u.alive & 1) ? (1u | ((uint32_t)min((int)u.x, W - 1) << 1) | ((uint32_t)min((int)u.y, W - 1) << 7) | ((uint32_t)u.age << 16)) : 0u;
    }
    __syncthreads();
    if (tid < SPARE_LADDER) r[tid] = s[tid];   // the spare world's description is written by kf_import_spare
}

// Level mutation of the overworld (section "Craftax-1B: UED"), as for Classic: up to 32 tries, try
// k drawing Philox block (env, round, 0, MUTATE | k) under the mutation seed; refused if the blocks
// are equal, a cell holds the player (when on floor 0), a live mob of floor 0 or an item, a block
// is a plant, or, restricted, the blocks are not of one group (stone and ores, gems included;
// grass and tree).  One thread per environment.
__device__ inline int swap_group(int b)
{
    if (b == B_STONE || b == B_COAL || b == B_IRON || b == B_DIAMOND || b == B_SAPPHIRE || b == B_RUBY) return 1;
    if (b == B_GRASS || b == B_TREE) return 2;
    return 0;
}
__global__ void kf_mutate_swap(const uint32_t* __restrict__ envs, uint8_t* __restrict__ maps, int first, int count, uint32_t k0,
                               uint32_t k1, uint32_t round, int restricted, int32_t* __restrict__ tries)
{
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= count) return;
    const uint32_t env = (uint32_t)(first + i);
    const uint32_t* genv = envs + (size_t)env * ENV_DWORDS;
    uint8_t* m = maps + map_offset(env, genv[R_EPISODE]);
    const uint32_t pos = genv[R_POS];
    const int px = pos & 0xFF, py = (pos >> 8) & 0xFF, floor = (pos >> 24) & 0xF;
    auto taken = [&](int x, int y) {
        bool t = floor == 0 && x == px && y == py;
        for (int k = 0; k < NSLOT; ++k) {
            const Mob u = unpack_mob(genv[REC_DWORDS + k]);
            t |= u.alive && (int)u.x == x && (int)u.y == y;
        }
        return t || (m[il_off(0, x, y)] & 7) != IT_NONE;
    };
    int done = 0;
    for (int k = 0; k < cx::MUTATE_TRIES && !done; ++k) {
        const cx::U4 d = cx::philox4x32_10(env, round, 0u, (cx::DOM_MUTATE << 16) | (uint32_t)k, k0, k1);
        const int a = (int)cx::choice(d.w[0], cx::MUTATE_AREA * cx::MUTATE_AREA), b = (int)cx::choice(d.w[1], CELLS);
        const int c0 = (W - cx::MUTATE_AREA) / 2;
        const int ax = c0 + a % cx::MUTATE_AREA, ay = c0 + a / cx::MUTATE_AREA, bx = b % W, by = b / W;
        const int ba = m[block_off(0, ax, ay)], bb = m[block_off(0, bx, by)];
        if (ba == bb || taken(ax, ay) || taken(bx, by)) continue;
        if (ba == B_PLANT || ba == B_RIPE || bb == B_PLANT || bb == B_RIPE) continue;
        if (restricted && (swap_group(ba) == 0 || swap_group(ba) != swap_group(bb))) continue;
        m[block_off(0, ax, ay)] = (uint8_t)bb;
        m[block_off(0, bx, by)] = (uint8_t)ba;
        done = k + 1;
    }
    if (tries != nullptr) tries[i] = done;
}

// ---------------------------------------------------------------------------------------------
namespace host {

static uint64_t round_up(uint64_t v, uint64_t a) { return (v + a - 1) / a * a; }

bool config_ok(const craftax_config* c, std::string* why)
{
    if (c->abi_version != CRAFTAX_ABI_VERSION) { *why = "abi_version mismatch"; return false; }
    if (c->obs_mode != CRAFTAX_OBS_SYM_U8_F32 && c->obs_mode != CRAFTAX_OBS_SYM_F32 && c->obs_mode != CRAFTAX_OBS_PIXELS_F32) {
        *why = "the Craftax variant renders SYM_U8_F32, SYM_F32 or PIXELS_F32"; return false;
    }
    if (c->day_length < 2 || c->day_length > (uint32_t)MAX_DAY || (c->day_length & 1)) { *why = "day_length must be even and in 2..1024"; return false; }
    if (c->cap_zombie > 3 || c->cap_cow > 3 || c->cap_skeleton > 2) { *why = "caps: melee 0..3, passive 0..3, ranged 0..2"; return false; }
    if (c->cap_plant > (uint32_t)NPLANT) { *why = "cap_plant must be 0..10"; return false; }
    if (c->max_episode_steps == 0) { *why = "max_episode_steps must be positive"; return false; }
    if (c->reset_mode > CRAFTAX_RESET_POOL) { *why = "unknown reset_mode"; return false; }
    if (c->worldgen > CRAFTAX_WORLDGEN_PERLIN) { *why = "unknown worldgen"; return false; }
    if (c->reserved != 0) { *why = "reserved must be 0"; return false; }
    if (c->group_lanes != 0 && c->group_lanes != 16 && c->group_lanes != 64) { *why = "group_lanes must be 0, 16 or 64"; return false; }
    return true;
}

static Header make_header(const craftax_config* c, int n)
{
    Header h;
    std::memset(&h, 0, sizeof(h));
    h.magic = MAGIC; h.version = CRAFTAX_ABI_VERSION; h.n = (uint32_t)n; h.variant = c->variant;
    h.obs_mode = c->obs_mode; h.max_episode_steps = c->max_episode_steps; h.day_length = c->day_length;
    h.cap_melee = c->cap_zombie; h.cap_ranged = c->cap_skeleton; h.cap_passive = c->cap_cow; h.cap_plant = c->cap_plant;
    h.atlas_seed = c->atlas_seed; h.worldgen = c->worldgen; h.reset_mode = c->reset_mode;
    h.off_ctrs = cx::HEADER_BYTES;
    h.off_luts = h.off_ctrs + la::COUNTER_BYTES;
    h.off_envs = round_up(h.off_luts + sizeof(Luts), 256);
    h.off_maps = h.off_envs + (uint64_t)n * (ENV_DWORDS * 4);
    h.off_tags = round_up(h.off_maps + (uint64_t)n * 2 * MAP_BYTES, 256);     // two map slots per environment
    h.off_regen0 = round_up(h.off_tags + (uint64_t)n * NTAG * 8, 256);
    const uint64_t list_bytes = (uint64_t)NSUB * la::sub_list_capacity((uint64_t)n, MAX_ENVS_PER_STEP_BLOCK) * 16;
    h.off_regen1 = h.off_regen0 + list_bytes;
    h.off_slow = h.off_regen1 + list_bytes;
    h.off_unlocks = round_up(h.off_slow + (uint64_t)n * 16, 256);
    h.total = round_up(h.off_unlocks + (uint64_t)n * UNLOCK_STRIDE * 4, 256);
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
    // unit gradients of the 1024 Perlin directions in Q14, rounded to nearest
    for (int a = 0; a < 1024; ++a) {
        const double turn = 6.283185307179586476925286766559 * (double)a / 1024.0;
        const int16_t c16 = (int16_t)std::lround(std::cos(turn) * 16384.0), s16 = (int16_t)std::lround(std::sin(turn) * 16384.0);
        L->perlin_cs[a] = (uint32_t)(uint16_t)c16 | ((uint32_t)(uint16_t)s16 << 16);
    }
    if (c->obs_mode != CRAFTAX_OBS_PIXELS_F32) return;
    // tile atlas: word idx of stream s is word idx % 4 of Philox block (0, s, 0, ATLAS | idx / 4)
    // under the atlas seed; streams 8 blocks, 9 items, 10 creatures, 11 player, 12 icons, 13 masks
    const uint32_t k0 = (uint32_t)c->atlas_seed, k1 = (uint32_t)(c->atlas_seed >> 32);
    auto fill = [&](uint32_t stream, uint32_t count, float* dst) {
        for (uint32_t i = 0; i < count; i += 4) {
            const cx::U4 r = cx::philox4x32_10(0u, stream, 0u, (cx::DOM_ATLAS << 16) | (i >> 2), k0, k1);
            for (uint32_t k = 0; k < 4 && i + k < count; ++k) dst[i + k] = (float)(r.w[k] >> 8) * (1.0f / 16777216.0f);
        }
    };
    fill(8, 37 * 300, L->atlas);
    fill(9, 5 * 300, L->atlas + AT_ITEM * 300);
    fill(10, 40 * 300, L->atlas + AT_CRE * 300);
    fill(11, 300, L->atlas + AT_PLAYER * 300);
    fill(12, 44 * 300, L->atlas + AT_ICON * 300);
    for (uint32_t i = 0; i < 46 * 100; i += 4) {
        const cx::U4 r = cx::philox4x32_10(0u, 13u, 0u, (cx::DOM_ATLAS << 16) | (i >> 2), k0, k1);
        for (uint32_t k = 0; k < 4; ++k) {
            const uint32_t t = (i + k) / 100, pix = (i + k) % 100;
            if (r.w[k] >> 31) L->mask[t][pix / 10] |= (uint16_t)(1u << (pix % 10));
        }
    }
}

struct Ptrs { uint32_t* envs; uint8_t* maps; const Luts* luts; Lists ls; };
static Ptrs pointers(const void* state, const Header& h)
{
    uint8_t* base = const_cast<uint8_t*>(static_cast<const uint8_t*>(state));
    Ptrs q;
    q.luts = reinterpret_cast<const Luts*>(base + h.off_luts);
    q.envs = reinterpret_cast<uint32_t*>(base + h.off_envs);
    q.maps = base + h.off_maps;
    q.ls.ctr = reinterpret_cast<uint32_t*>(base + h.off_ctrs);
    q.ls.regen[0] = reinterpret_cast<uint4*>(base + h.off_regen0);
    q.ls.regen[1] = reinterpret_cast<uint4*>(base + h.off_regen1);
    q.ls.slow = reinterpret_cast<uint4*>(base + h.off_slow);
    q.ls.tags = reinterpret_cast<uint2*>(base + h.off_tags);
    q.ls.sub_cap = (uint32_t)la::sub_list_capacity((uint64_t)h.n, MAX_ENVS_PER_STEP_BLOCK);
    q.ls.slow_cap = h.n;
    return q;
}
static Params make_params(const void* state, const craftax_config* c, int n)
{
    Params p;
    p.unlocks = reinterpret_cast<uint32_t*>(const_cast<uint8_t*>(static_cast<const uint8_t*>(state)) + make_header(c, n).off_unlocks);
    p.n = n; p.max_episode_steps = c->max_episode_steps; p.day_length = c->day_length;
    p.cap_melee = c->cap_zombie; p.cap_ranged = c->cap_skeleton; p.cap_passive = c->cap_cow; p.cap_plant = c->cap_plant;
    p.worldgen = c->worldgen;
    return p;
}
// the gradient table for the kernels that choose the noise at run time: null = value noise
static const uint32_t* gradients(const craftax_config* c, const Ptrs& q)
{
    return c->worldgen == CRAFTAX_WORLDGEN_PERLIN ? q.luts->perlin_cs : nullptr;
}
static int check_launch(const char* what, std::string* err)
{
    const hipError_t e = hipGetLastError();
    if (e != hipSuccess) { *err = std::string(what) + ": " + hipGetErrorString(e); return CRAFTAX_E_HIP; }
    return CRAFTAX_OK;
}

size_t state_bytes(const craftax_config* cfg, int n) { return (size_t)make_header(cfg, n).total; }
size_t obs_bytes(const craftax_config* cfg)
{
    return cfg->obs_mode == CRAFTAX_OBS_PIXELS_F32 ? STRIDE_PIXELS : cfg->obs_mode == CRAFTAX_OBS_SYM_F32 ? STRIDE_F32 : STRIDE_U8;
}

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

int check_header(const void* header_bytes, const craftax_config* cfg, int n, std::string* err)
{
    Header got;
    std::memcpy(&got, header_bytes, sizeof(got));
    if (got.magic != MAGIC) { *err = "the memory holds no Craftax state blob"; return CRAFTAX_E_STATE; }
    if (got.version != CRAFTAX_ABI_VERSION) { *err = "the state blob was written by another library version"; return CRAFTAX_E_STATE; }
    if (got.n != (uint32_t)n) { *err = "the state blob holds another number of environments"; return CRAFTAX_E_COUNT; }
    const Header want = make_header(cfg, n);
    if (std::memcmp(&got, &want, sizeof(Header)) != 0) { *err = "the state blob was initialised with another configuration"; return CRAFTAX_E_CONFIG; }
    return CRAFTAX_OK;
}

int debug_bounds(uint32_t report[4], std::string* err)
{
#ifdef CRAFTAX_DEBUG_BOUNDS
    uint32_t mine[4] = {0u, 0u, 0u, 0u};
    const uint32_t zero[4] = {0u, 0u, 0u, 0u};
    hipError_t e = hipMemcpyFromSymbol(mine, HIP_SYMBOL(cx::g_bounds), sizeof(mine));
    if (e == hipSuccess) e = hipMemcpyToSymbol(HIP_SYMBOL(cx::g_bounds), zero, sizeof(zero));
    if (e != hipSuccess) { *err = std::string("debug_bounds: ") + hipGetErrorString(e); return CRAFTAX_E_HIP; }
    if (report[0] == 0u && mine[0] != 0u) { report[1] = mine[1]; report[2] = mine[2]; report[3] = mine[3]; }
    report[0] += mine[0];
#else
    (void)report; (void)err;
#endif
    return CRAFTAX_OK;
}

RecordLayout record_layout(const void* state, const craftax_config* cfg, int n)
{
    const Ptrs q = pointers(state, make_header(cfg, n));
    return RecordLayout{q.envs, ENV_DWORDS, R_ACH, 3, R_T, R_EPISODE, make_params(state, cfg, n).unlocks, UNLOCK_STRIDE};
}

int check_kernels(const craftax_config* cfg, std::string* err)
{
    int dev = 0, lds = 0, threads = 0;
    if (hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&lds, hipDeviceAttributeMaxSharedMemoryPerBlock, dev) != hipSuccess ||
        hipDeviceGetAttribute(&threads, hipDeviceAttributeMaxThreadsPerBlock, dev) != hipSuccess) {
        (void)hipGetLastError();
        *err = "no usable HIP device";
        return CRAFTAX_E_HIP;
    }
    const cx::DeviceLimits limits{(size_t)lds, threads};
    auto fits = [&](const char* name, const void* fn, int block) {
        hipFuncAttributes a;
        if (hipFuncGetAttributes(&a, fn) != hipSuccess) { (void)hipGetLastError(); *err = std::string("no attributes for ") + name; return false; }
        return cx::kernel_fits(cx::KernelNeeds{name, a.sharedSizeBytes, a.maxThreadsPerBlock, block}, limits, err);
    };
    const bool perlin = cfg->worldgen == CRAFTAX_WORLDGEN_PERLIN;
    bool ok = true;
    if (cfg->obs_mode == CRAFTAX_OBS_SYM_F32) {
        ok = ok && (perlin ? fits("kf_step", (const void*)kf_step<true, true, true, 64>, BLOCK) : fits("kf_step", (const void*)kf_step<true, true, false, 64>, BLOCK));
        ok = ok && (perlin ? fits("kf_step (16 lanes)", (const void*)kf_step<true, true, true, 16>, BLOCK) : fits("kf_step (16 lanes)", (const void*)kf_step<true, true, false, 16>, BLOCK));
        ok = ok && (perlin ? fits("kf_rollout", (const void*)kf_rollout<true, true>, BLOCK) : fits("kf_rollout", (const void*)kf_rollout<true, false>, BLOCK));
        ok = ok && fits("kf_reset_list", (const void*)kf_reset_list<true>, GEN_THREADS) && fits("kf_observe", (const void*)kf_observe<true>, BLOCK);
    } else {
        ok = ok && (perlin ? fits("kf_step", (const void*)kf_step<false, true, true, 64>, BLOCK) : fits("kf_step", (const void*)kf_step<false, true, false, 64>, BLOCK));
        ok = ok && (perlin ? fits("kf_step (16 lanes)", (const void*)kf_step<false, true, true, 16>, BLOCK) : fits("kf_step (16 lanes)", (const void*)kf_step<false, true, false, 16>, BLOCK));
        ok = ok && (perlin ? fits("kf_rollout", (const void*)kf_rollout<false, true>, BLOCK) : fits("kf_rollout", (const void*)kf_rollout<false, false>, BLOCK));
        ok = ok && fits("kf_reset_list", (const void*)kf_reset_list<false>, GEN_THREADS) && fits("kf_observe", (const void*)kf_observe<false>, BLOCK);
    }
    ok = ok && fits("kf_reset", (const void*)kf_reset, GEN_THREADS) && fits("kf_pixels", (const void*)kf_pixels, BLOCK);
    return ok ? CRAFTAX_OK : CRAFTAX_E_CONFIG;
}

int reset(void* state, const craftax_config* cfg, int n, const uint64_t* seeds, void* stream, std::string* err)
{
    const Ptrs q = pointers(state, make_header(cfg, n));
    hipLaunchKernelGGL(kf_reset, dim3((unsigned)n * 2 * FLOORS), dim3(GEN_THREADS), 0, (hipStream_t)stream, q.envs, q.maps, seeds, q.ls, gradients(cfg, q), cfg->reset_mode == CRAFTAX_RESET_POOL ? 1 : 0,
                       make_params(state, cfg, n).unlocks);
    return check_launch("craftax_reset", err);
}

// Lanes per environment of the step kernel.  A whole wavefront (the default at every batch size)
// keeps the player's state and the 43-action code on the scalar unit, which works beside the vector
// unit.  Sixteen lanes put four environments in a wavefront and fill 14 of 16 lanes with mob slots
// instead of 14 of 64, but the player's code then runs on the vector unit, the kernel needs 210
// vector registers (two wavefronts per SIMD instead of five), and a wavefront renders four
// observations one after the other: measured slower at every size (22.5 against 18.8 us per step at
// 4,096 environments, 243 against 207 us at 65,536).  It stays selectable (cfg->group_lanes = 16)
// and is tested like the default.
static int group_lanes(const craftax_config* cfg, int n)
{
    (void)n;
    return cfg->group_lanes == 16 ? 16 : 64;
}

// one launch of the step kernel: the instance for this spare-world policy, this noise and this group width
template <bool F32>
static void launch_step(int gw, bool eager, bool perlin, dim3 grid, hipStream_t st, const Ptrs& q, const int32_t* actions, uint8_t* o, float* reward,
                        uint8_t* done, const Params& p, int rb)
{
    auto go = [&](auto kernel) { hipLaunchKernelGGL(kernel, grid, dim3(BLOCK), 0, st, q.envs, q.maps, q.luts, actions, o, reward, done, q.ls, p, rb); };
    if (gw == 16) {
        if (perlin) { if (eager) go(kf_step<F32, true, true, 16>); else go(kf_step<F32, false, true, 16>); }
        else { if (eager) go(kf_step<F32, true, false, 16>); else go(kf_step<F32, false, false, 16>); }
    } else {
        if (perlin) { if (eager) go(kf_step<F32, true, true, 64>); else go(kf_step<F32, false, true, 64>); }
        else { if (eager) go(kf_step<F32, true, false, 64>); else go(kf_step<F32, false, false, 64>); }
    }
}

int step(void* state, const craftax_config* cfg, int n, const int32_t* actions, void* obs, float* reward, uint8_t* done,
         bool serve_slow, void* stream, std::string* err)
{
    const Ptrs q = pointers(state, make_header(cfg, n));
    const Params p = make_params(state, cfg, n);
    hipStream_t st = (hipStream_t)stream;
    uint8_t* o = static_cast<uint8_t*>(obs);
    const int gw = group_lanes(cfg, n), epb = BLOCK / gw;
    const int sb = (n + epb - 1) / epb;
    const int rb = FLOORS * n < REGEN_BLOCKS ? FLOORS * n : REGEN_BLOCKS;    // persistent blocks serving a queue: any number works
    const dim3 grid((unsigned)(rb + sb)), rgrid((unsigned)(n < RESET_SLOTS ? n : RESET_SLOTS) * FLOORS);
    const int pool = cfg->reset_mode == CRAFTAX_RESET_POOL ? 1 : 0;
    // kf_reset_list serves the episodes that end before their spare world exists: with exact resets
    // only one-step episodes can, or a fresh episode whose world was edited before its first step
    // (serve_slow: the caller mutated or imported since the last step); with optimistic resets there
    // are no spare worlds and every finished episode is served there, its world depending on who
    // else finished
    const bool slow = p.max_episode_steps == 1u || pool != 0 || serve_slow;
    const bool eager = n <= EAGER_SPARE_ENVS && pool == 0;
    const int perlin = cfg->worldgen == CRAFTAX_WORLDGEN_PERLIN ? 1 : 0;
    if (cfg->obs_mode == CRAFTAX_OBS_PIXELS_F32) {
        // the step runs without rendering; the picture is drawn from the state it leaves
        launch_step<false>(gw, eager, perlin != 0, grid, st, q, actions, nullptr, reward, done, p, rb);
        if (slow) hipLaunchKernelGGL(kf_reset_list<false>, rgrid, dim3(GEN_THREADS), 0, st, q.envs, q.maps, q.luts, (uint8_t*)nullptr, q.ls, perlin, done, n, pool);
        if (o != nullptr) hipLaunchKernelGGL(kf_pixels, dim3((unsigned)n), dim3(BLOCK), 0, st, q.envs, q.maps, q.luts, o);
    } else if (cfg->obs_mode == CRAFTAX_OBS_SYM_F32) {
        launch_step<true>(gw, eager, perlin != 0, grid, st, q, actions, o, reward, done, p, rb);
        if (slow) hipLaunchKernelGGL(kf_reset_list<true>, rgrid, dim3(GEN_THREADS), 0, st, q.envs, q.maps, q.luts, o, q.ls, perlin, done, n, pool);
    } else {
        launch_step<false>(gw, eager, perlin != 0, grid, st, q, actions, o, reward, done, p, rb);
        if (slow) hipLaunchKernelGGL(kf_reset_list<false>, rgrid, dim3(GEN_THREADS), 0, st, q.envs, q.maps, q.luts, o, q.ls, perlin, done, n, pool);
    }
    return check_launch("craftax_step", err);
}

int rollout(void* state, const craftax_config* cfg, int n, const int32_t* actions, int steps, void* obs, float* reward, uint8_t* done,
            void* stream, std::string* err)
{
    if (cfg->obs_mode == CRAFTAX_OBS_PIXELS_F32) { *err = "craftax_rollout needs a symbolic observation"; return CRAFTAX_E_CONFIG; }
    if (cfg->reset_mode != CRAFTAX_RESET_EXACT) { *err = "craftax_rollout needs exact resets"; return CRAFTAX_E_CONFIG; }
    const Ptrs q = pointers(state, make_header(cfg, n));
    const Params p = make_params(state, cfg, n);
    hipStream_t st = (hipStream_t)stream;
    uint8_t* o = static_cast<uint8_t*>(obs);
    const int rb = FLOORS * n < REGEN_BLOCKS ? FLOORS * n : REGEN_BLOCKS;
    const dim3 drain((unsigned)rb), grid((unsigned)((n + ENVS_PER_BLOCK - 1) / ENVS_PER_BLOCK));
    // a launch of regeneration blocks only empties the lists of the step kernel and completes every spare world
    const bool perlin = cfg->worldgen == CRAFTAX_WORLDGEN_PERLIN;
    launch_step<false>(64, false, perlin, drain, st, q, nullptr, nullptr, nullptr, nullptr, p, rb);
    auto go = [&](auto kernel) { hipLaunchKernelGGL(kernel, grid, dim3(BLOCK), 0, st, q.envs, q.maps, q.luts, actions, o, reward, done, q.ls.tags, p, steps); };
    if (cfg->obs_mode == CRAFTAX_OBS_SYM_F32) { if (perlin) go(kf_rollout<true, true>); else go(kf_rollout<true, false>); }
    else { if (perlin) go(kf_rollout<false, true>); else go(kf_rollout<false, false>); }
    return check_launch("craftax_rollout", err);
}

int observe(void* state, const craftax_config* cfg, int n, void* obs, void* stream, std::string* err)
{
    const Ptrs q = pointers(state, make_header(cfg, n));
    const dim3 grid((n + ENVS_PER_BLOCK - 1) / ENVS_PER_BLOCK);
    uint8_t* o = static_cast<uint8_t*>(obs);
    if (cfg->obs_mode == CRAFTAX_OBS_PIXELS_F32) hipLaunchKernelGGL(kf_pixels, dim3((unsigned)n), dim3(BLOCK), 0, (hipStream_t)stream, q.envs, q.maps, q.luts, o);
    else if (cfg->obs_mode == CRAFTAX_OBS_SYM_F32) hipLaunchKernelGGL(kf_observe<true>, grid, dim3(BLOCK), 0, (hipStream_t)stream, q.envs, q.maps, q.luts, o, n);
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
    hipLaunchKernelGGL(kf_import, dim3(count), dim3(BLOCK), 0, (hipStream_t)stream, q.envs, q.maps, q.ls,
                       static_cast<const craftax_full_env_dump*>(dumps), first, make_params(state, cfg, n));
    hipLaunchKernelGGL(kf_import_spare, dim3((unsigned)count * FLOORS), dim3(GEN_THREADS), 0, (hipStream_t)stream, q.envs, q.maps, q.ls, first, gradients(cfg, q), cfg->reset_mode == CRAFTAX_RESET_POOL ? 1 : 0);
    return check_launch("craftax_import_envs", err);
}

int mutate_swap(void* state, const craftax_config* cfg, int n, int first, int count, uint64_t mutation_seed, uint32_t round,
                int restricted, int32_t* tries, void* stream, std::string* err)
{
    const Ptrs q = pointers(state, make_header(cfg, n));
    hipLaunchKernelGGL(kf_mutate_swap, dim3((unsigned)((count + 255) / 256)), dim3(256), 0, (hipStream_t)stream, q.envs, q.maps, first,
                       count, (uint32_t)mutation_seed, (uint32_t)(mutation_seed >> 32), round, restricted != 0 ? 1 : 0, tries);
    return check_launch("craftax_mutate_swap", err);
}

int mutate_noise(void* state, const craftax_config* cfg, int n, int first, int count, uint16_t* theta, uint64_t mutation_seed, uint32_t round,
                 uint32_t amplitude, void* stream, std::string* err)
{
    const Ptrs q = pointers(state, make_header(cfg, n));
    const uint32_t k0 = (uint32_t)mutation_seed, k1 = (uint32_t)(mutation_seed >> 32);
    hipLaunchKernelGGL(kf_mutate_noise, dim3((unsigned)count * (FLOORS - 1)), dim3(GEN_THREADS), 0, (hipStream_t)stream, q.envs, q.maps, q.luts, theta,
                       first, 1, FLOORS - 1, k0, k1, round, amplitude);
    hipLaunchKernelGGL(kf_mutate_noise, dim3((unsigned)count), dim3(GEN_THREADS), 0, (hipStream_t)stream, q.envs, q.maps, q.luts, theta, first, 0, 1,
                       k0, k1, round, amplitude);
    return check_launch("craftax_mutate_noise", err);
}

}  // namespace host
}  // namespace cf
