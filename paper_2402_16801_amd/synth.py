"""Seeded synthetic inputs (seeds and action streams) for tests and benchmarks.

This module holds none of the simulator's arithmetic.  It produces the inputs that stand
in for a learner's action stream: the workloads of the paper are a policy driving
thousands of Craftax-Classic workers (section "JAX-Based Environments": up to 4096
workers; appendix "Action Space": 17 actions); here actions are drawn from a counter-based
generator so that any (env, step) entry can be regenerated anywhere.

The generator is Philox4x32-10 (Salmon et al., SC'11), written with numpy uint64 limbs.
"""
from __future__ import annotations

import numpy as np

_M0 = np.uint64(0xD2511F53)
_M1 = np.uint64(0xCD9E8D57)
_W0 = 0x9E3779B9
_W1 = 0xBB67AE85
_MASK = np.uint64(0xFFFFFFFF)
_S32 = np.uint64(32)

DOMAIN_ACTIONS = 2
N_ACTIONS_CLASSIC = 17


def philox4x32_10(c0, c1, c2, c3, k0: int, k1: int):
    """Vectorised Philox4x32-10.  c0..c3: broadcastable integer arrays (values < 2**32);
    k0, k1: python ints.  Returns four uint32 arrays."""
    c0, c1, c2, c3 = np.broadcast_arrays(*[np.asarray(c, dtype=np.uint64) for c in (c0, c1, c2, c3)])
    c0, c1, c2, c3 = c0.copy(), c1.copy(), c2.copy(), c3.copy()
    for r in range(10):
        ka = np.uint64((k0 + r * _W0) & 0xFFFFFFFF)
        kb = np.uint64((k1 + r * _W1) & 0xFFFFFFFF)
        p0 = _M0 * c0  # < 2**64, exact in uint64
        p1 = _M1 * c2
        n0 = (p1 >> _S32) ^ c1 ^ ka
        n1 = p1 & _MASK
        n2 = (p0 >> _S32) ^ c3 ^ kb
        n3 = p0 & _MASK
        c0, c1, c2, c3 = n0, n1, n2, n3
    return tuple(c.astype(np.uint32) for c in (c0, c1, c2, c3))


def choice(u, n: int):
    """Map uint32 draws onto 0..n-1 by the multiply-shift rule."""
    return ((np.asarray(u, dtype=np.uint64) * np.uint64(n)) >> _S32).astype(np.int64)


def seeds_for(n: int, base: int = 0) -> np.ndarray:
    """Per-environment seeds: base + env index."""
    return (np.arange(n, dtype=np.uint64) + np.uint64(base)).astype(np.uint64)


def actions(env_ids, step: int, kind: str = "uniform", action_seed: int = 0,
            n_actions: int = N_ACTIONS_CLASSIC) -> np.ndarray:
    """Actions of the given environments at rollout step `step` (int32 array).

    kind "uniform": iid uniform over the action set.
    kind "skewed":  with probability 1/2 uniform over {LEFT, RIGHT, UP, DOWN, DO} (ids 1..5),
                    otherwise uniform over the whole set.
    """
    env_ids = np.asarray(env_ids, dtype=np.uint64)
    w0, w1, _, _ = philox4x32_10(env_ids, np.uint64(step), np.uint64(0), np.uint64(DOMAIN_ACTIONS << 16),
                                 action_seed & 0xFFFFFFFF, (action_seed >> 32) & 0xFFFFFFFF)
    if kind == "uniform":
        return choice(w0, n_actions).astype(np.int32)
    if kind == "skewed":
        focused = w0 < np.uint32(0x80000000)
        return np.where(focused, 1 + choice(w1, 5), choice(w1, n_actions)).astype(np.int32)
    raise ValueError(f"unknown action kind {kind!r}")


def action_block(n: int, steps: int, kind: str = "uniform", action_seed: int = 0, step0: int = 0,
                 n_actions: int = N_ACTIONS_CLASSIC) -> np.ndarray:
    """int32 array [steps, n] of actions for envs 0..n-1 and rollout steps step0..step0+steps-1."""
    out = np.empty((steps, n), dtype=np.int32)
    env_ids = np.arange(n, dtype=np.uint64)
    for s in range(steps):
        out[s] = actions(env_ids, step0 + s, kind, action_seed, n_actions)
    return out
