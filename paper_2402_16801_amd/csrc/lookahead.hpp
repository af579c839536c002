// Worlds generated one episode ahead (shared by the Classic and the full-Craftax kernels).
//
// Appendix "Optimistic Environment Resets" of the paper explains why world generation is the
// expensive part of a reset.  Here every environment owns two map slots: slot e & 1 holds the
// world of episode e, the other slot the world of episode e + 1.  An episode that ends switches
// slots inside the step kernel and puts the environment on a regeneration list; extra blocks of
// the NEXT step launch fill the freed slot with the world after next, in the shadow of the step
// blocks, so that a step is a single kernel launch.  Tags per environment say which episode its
// spare slot holds and which launch wrote it; a spare is only trusted when an earlier launch wrote
// it.  The spare of an episode is generated during that episode's first step, so only an episode
// that ends at its first step finds it missing; a fresh episode cannot (full vitals, cleared
// start area, no mobs) unless the episode cap is 1.  Such episodes go on the slow list, which a
// second kernel serves right after the step kernel; it is launched only for an episode cap of 1.
// Reset and import generate the spare themselves.
//
// A list entry carries what world generation needs: (env, seed low, seed high, episode index);
// env = ENTRY_VOID marks an entry cancelled by an import.  Each of the two regeneration lists
// (filled and consumed in alternate launches) is cut into NSUB sub-lists with their own counters
// (step block b appends to sub-list b mod NSUB), so that the appending atomics do not
// queue up on one address.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace la {

// Device-side counters: one uint32 per 256 bytes (counters hit by atomics from many blocks must
// not share a memory channel), in their own area of the state blob.
//   SEQ     number of step launches so far + 1
//   TOP     groups of blocks of the current step launch that have all started
//   SLOW    entries in the slow list; SLOW_FINISHED: slow-list blocks finished
//   GROUP+g blocks of group g of the current step launch that have started
//   REGEN+p*NSUB+s entries in sub-list s of regeneration list p
constexpr int CTR_STRIDE = 64;   // dwords between counters
constexpr int NGROUP = 64, NSUB = 16;
enum Counter : int { CT_SEQ = 0, CT_TOP = 1, CT_SLOW = 2, CT_SLOW_FINISHED = 3, CT_GROUP = 4, CT_REGEN = CT_GROUP + NGROUP,
                     CT_COUNT = CT_REGEN + 2 * NSUB };
constexpr uint64_t COUNTER_BYTES = (uint64_t)CT_COUNT * CTR_STRIDE * 4;
constexpr uint32_t TAG_NONE = 0xFFFFFFFFu, ENTRY_VOID = 0xFFFFFFFFu;

// sub_cap: capacity of a sub-list; slow_cap: capacity of the slow list (= environments).  tags: (episode, launch) pairs, a fixed number per environment.
struct Lists { uint32_t* ctr; uint4* regen[2]; uint4* slow; uint2* tags; uint32_t sub_cap, slow_cap; };
__device__ inline uint32_t* counter(const Lists& ls, int i) { return ls.ctr + (size_t)i * CTR_STRIDE; }

// Entries a regeneration sub-list must hold: every environment of the step blocks that append to
// it (plus one block of slack for the rounding of the narrower block shapes).
inline uint64_t sub_list_capacity(uint64_t n, uint64_t max_envs_per_block)
{
    const uint64_t blocks = (n + max_envs_per_block - 1) / max_envs_per_block;
    return ((blocks + NSUB - 1) / NSUB) * max_envs_per_block + max_envs_per_block;
}

// first thread block of a reset kernel: all counters to zero, launch number 1
__device__ inline void reset_counters(const Lists& ls)
{
    for (int i = threadIdx.x; i < CT_COUNT; i += blockDim.x) *counter(ls, i) = i == CT_SEQ ? 1u : 0u;
}

// Launch number and the bookkeeping that advances it.  Every block of a step launch reads the
// number (and, as a regeneration block, the length of its sub-list) and then counts itself in;
// once all blocks of the launch have done so, one thread advances the number and empties the
// lists this launch consumes.  Counting is in two levels (NGROUP group counters, then one on
// top) so that no counter sees more than a few dozen atomics.
struct Ticket { uint32_t seq, regen_count, started, gsize, grp; };

// regen_role: this block is one of the nrb regeneration blocks (index rb) at the end of the grid
__device__ inline Ticket enter_launch(const Lists& ls, bool regen_role, uint32_t rb)
{
    Ticket t;
    t.seq = *counter(ls, CT_SEQ);
    t.regen_count = 0u;
    if (regen_role) t.regen_count = min(*counter(ls, CT_REGEN + (int)(((t.seq & 1u) ^ 1u) * NSUB + rb % NSUB)), ls.sub_cap);
    t.gsize = (gridDim.x + NGROUP - 1) / NGROUP;
    t.grp = blockIdx.x / t.gsize;
    t.started = 0u;
    asm volatile("" :: "v"(t.seq), "v"(t.regen_count) : "memory");   // both values have arrived before this block counts itself in
    if (threadIdx.x == 0) t.started = atomicAdd(counter(ls, CT_GROUP + (int)t.grp), 1u);
    return t;
}
__device__ inline void leave_launch(const Lists& ls, const Ticket& t)
{
    if (threadIdx.x != 0) return;
    const uint32_t members = min(t.gsize, gridDim.x - t.grp * t.gsize), ngroups = (gridDim.x + t.gsize - 1) / t.gsize;
    if (t.started != members - 1u) return;
    *counter(ls, CT_GROUP + (int)t.grp) = 0u;
    if (atomicAdd(counter(ls, CT_TOP), 1u) != ngroups - 1u) return;
    *counter(ls, CT_TOP) = 0u;
    for (int sub = 0; sub < NSUB; ++sub) *counter(ls, CT_REGEN + (int)(((t.seq & 1u) ^ 1u) * NSUB) + sub) = 0u;
    *counter(ls, CT_SEQ) = t.seq + 1u;
}

// The same for a block that sees the consumed list as ONE dense queue of entries (full game:
// regeneration block b of B takes the work units b, b + B, ... of that queue, so the work sits on
// the first blocks of the grid and no counter is shared: a few hundred atomics on one address
// would take microseconds).  The lengths of all NSUB sub-lists, as running totals, go to s_prefix
// (LDS, NSUB words; s_prefix[NSUB - 1] = all entries) before the block counts itself in.  All
// threads of the block call; ends with a block barrier.
__device__ inline Ticket enter_launch_queue(const Lists& ls, uint32_t* s_prefix)
{
    Ticket t;
    t.seq = *counter(ls, CT_SEQ);
    t.regen_count = 0u;
    if (threadIdx.x < (unsigned)NSUB) {
        uint32_t c = min(*counter(ls, CT_REGEN + (int)(((t.seq & 1u) ^ 1u) * NSUB + threadIdx.x)), ls.sub_cap);
#pragma unroll
        for (int d = 1; d < NSUB; d <<= 1) {
            const uint32_t below = (uint32_t)__shfl_up((int)c, d, NSUB);
            if ((int)threadIdx.x >= d) c += below;
        }
        s_prefix[threadIdx.x] = c;
    }
    __syncthreads();   // the lengths have arrived (they are in LDS) before this block counts itself in
    t.gsize = (gridDim.x + NGROUP - 1) / NGROUP;
    t.grp = blockIdx.x / t.gsize;
    t.started = 0u;
    asm volatile("" :: "v"(t.seq) : "memory");
    if (threadIdx.x == 0) t.started = atomicAdd(counter(ls, CT_GROUP + (int)t.grp), 1u);
    return t;
}
// Entry number g of the consumed list seen as one queue (g < s_prefix[NSUB - 1]).
__device__ inline uint4 queue_entry(const Lists& ls, uint32_t seq, const uint32_t* s_prefix, uint32_t g)
{
    uint32_t sub = 0u, base = 0u;
#pragma unroll
    for (int k = 0; k < NSUB - 1; ++k) if (g >= s_prefix[k]) { sub = (uint32_t)k + 1u; base = s_prefix[k]; }
    return ls.regen[(seq & 1u) ^ 1u][(size_t)sub * ls.sub_cap + (g - base)];
}
// the sub-list of the list consumed in this launch that regeneration block rb reads
__device__ inline const uint4* consumed_sub_list(const Lists& ls, uint32_t seq, uint32_t rb)
{
    return ls.regen[(seq & 1u) ^ 1u] + (size_t)(rb % NSUB) * ls.sub_cap;
}
// Appends nd entries (staged in LDS by the block) to this launch's list; all threads of the block call.
// step_block: index of the block among the step blocks of the launch.
__device__ inline void append_block_entries(const Lists& ls, uint32_t seq, const uint4* s_list, int nd, uint32_t* s_base, uint32_t step_block)
{
    const uint32_t sub = step_block % NSUB;
    if (threadIdx.x == 0) *s_base = atomicAdd(counter(ls, CT_REGEN + (int)((seq & 1u) * NSUB + sub)), (uint32_t)nd);
    __syncthreads();
    if ((int)threadIdx.x < nd && *s_base + threadIdx.x < ls.sub_cap)   // always true: a sub-list holds every environment of its blocks
        ls.regen[seq & 1u][(size_t)sub * ls.sub_cap + *s_base + threadIdx.x] = s_list[threadIdx.x];
}
// The same for a single entry, in two halves so that the latency of the atomic hides behind whatever
// the caller does in between: claim_entry reserves the place, commit_entry stores the entry there.
__device__ inline uint32_t claim_entry(const Lists& ls, uint32_t seq, uint32_t step_block)
{
    return atomicAdd(counter(ls, CT_REGEN + (int)((seq & 1u) * NSUB + step_block % NSUB)), 1u);
}
__device__ inline void commit_entry(const Lists& ls, uint32_t seq, uint32_t step_block, uint32_t at, uint4 entry)
{
    if (at < ls.sub_cap) ls.regen[seq & 1u][(size_t)(step_block % NSUB) * ls.sub_cap + at] = entry;   // always true: a sub-list holds every environment of its blocks
}
// One entry for the list the NEXT launch consumes, from a kernel that runs after the step kernel
// (which has already advanced the launch number); step_block = index of the step block that owns
// the environment, so that no sub-list can overflow.
__device__ inline void append_after_step(const Lists& ls, uint32_t step_block, uint4 entry)
{
    const uint32_t next = (*counter(ls, CT_SEQ) & 1u) ^ 1u, sub = step_block % NSUB;
    const uint32_t at = atomicAdd(counter(ls, CT_REGEN + (int)(next * NSUB + sub)), 1u);
    if (at < ls.sub_cap) ls.regen[next][(size_t)sub * ls.sub_cap + at] = entry;
}
// One entry for the slow list, which holds at most one entry per environment (capacity n).  The
// kernel that serves the list empties it; should nothing serve it, further entries are dropped
// rather than written past its end.
__device__ inline void append_slow(const Lists& ls, uint32_t capacity, uint4 entry)
{
    const uint32_t at = atomicAdd(counter(ls, CT_SLOW), 1u);
    if (at < capacity) ls.slow[at] = entry;
}
__device__ inline uint32_t slow_count(const Lists& ls, uint32_t capacity) { return min(*counter(ls, CT_SLOW), capacity); }
// Cancels everything queued for `env` (all threads of the block call).
__device__ inline void cancel_entries(const Lists& ls, uint32_t env)
{
    for (int li = 0; li < 2 * NSUB + 1; ++li) {
        uint4* list = li < 2 * NSUB ? ls.regen[li / NSUB] + (size_t)(li % NSUB) * ls.sub_cap : ls.slow;
        const uint32_t cnt = min(*counter(ls, li < 2 * NSUB ? CT_REGEN + li : CT_SLOW), li < 2 * NSUB ? ls.sub_cap : ls.slow_cap);
        for (uint32_t i = threadIdx.x; i < cnt; i += blockDim.x) if (list[i].x == env) list[i].x = ENTRY_VOID;
    }
}
// the last working block of a slow-list kernel empties the slow list
__device__ inline void finish_slow_list(const Lists& ls, uint32_t count)
{
    if (threadIdx.x != 0) return;
    const uint32_t workers = count < gridDim.x ? count : gridDim.x;
    if (atomicAdd(counter(ls, CT_SLOW_FINISHED), 1u) == workers - 1u) { *counter(ls, CT_SLOW) = 0u; *counter(ls, CT_SLOW_FINISHED) = 0u; }
}

}  // namespace la
