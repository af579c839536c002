// Which regeneration units a block of a step launch takes when the step blocks share that work
// (four lanes per environment; see regeneration_share in craftax.hip).  A sub-list of `count`
// entries is 2 * count units (unit u = half u & 1 of entry u >> 1).  Its per_sub regeneration
// blocks take the head, HEAD_ROUNDS rounds of per_sub units; the tail is dealt out in turn to the
// nq step blocks that append to the sub-list and, behind them, to the regeneration blocks again.
// Plain integer arithmetic, usable on the host, so that "every unit is taken exactly once, by a
// block that exists" can be checked without a GPU.
#pragma once

#include <stdint.h>

#if defined(__HIPCC__)
#define CX_UNITS_FN __host__ __device__ inline
#else
#define CX_UNITS_FN inline
#endif

namespace cx {

constexpr uint32_t HEAD_ROUNDS = 2u;

struct UnitWalk {
    uint32_t u;         // the unit to generate now; the walk is over once u >= 2 * count
    uint32_t round;     // units taken so far + 1
};

// helper: step block number `index` among the nq that append to this sub-list; else regeneration
// block number `index` among the sub-list's per_sub.
CX_UNITS_FN UnitWalk first_unit(bool helper, uint32_t index, uint32_t per_sub)
{
    return UnitWalk{ helper ? HEAD_ROUNDS * per_sub + index : index, 1u };
}
CX_UNITS_FN UnitWalk next_unit(UnitWalk w, bool helper, uint32_t index, uint32_t per_sub, uint32_t nq)
{
    const uint32_t head = HEAD_ROUNDS * per_sub, workers = nq + per_sub;
    if (helper) w.u += workers;
    else w.u = w.round < HEAD_ROUNDS ? w.u + per_sub : (w.round == HEAD_ROUNDS ? head + nq + index : w.u + workers);
    ++w.round;
    return w;
}
// the first unit of step block `index`'s share: it has work if this is below 2 * count
CX_UNITS_FN uint32_t first_helper_unit(uint32_t index, uint32_t per_sub) { return HEAD_ROUNDS * per_sub + index; }

}  // namespace cx
