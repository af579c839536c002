"""ctypes loader for the CPU oracle (liboracle.so).

TEST INFRASTRUCTURE ONLY: imported by tests/, by the smoke check and by the benchmark's
cpu_baseline leg.  The GPU library never touches this.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SOURCES = ["philox.c", "classic.c", "craftax_full.c"]
_HEADERS = ["craftax_oracle.h", "craftax_full.h"]
LIB_PATH = os.path.join(_HERE, "liboracle.so")

OBS_SYM_U8_I8, OBS_SYM_U8_F32, OBS_SYM_F32, OBS_PIXELS_F32 = 0, 1, 2, 3
OBS_BYTES = {0: 1408, 1: 1536, 2: 5392, 3: 47632}

MOB_DTYPE = np.dtype([("alive", "u1"), ("x", "u1"), ("y", "u1"), ("dir", "u1"), ("hp", "i1"),
                      ("cd", "u1"), ("pad", "u1", (2,))])
PLANT_DTYPE = np.dtype([("alive", "u1"), ("x", "u1"), ("y", "u1"), ("pad", "u1"), ("age", "<u2")])
ENV_DTYPE = np.dtype([
    ("map", "u1", (64, 64)),
    ("px", "u1"), ("py", "u1"), ("dir", "u1"), ("sleeping", "u1"),
    ("inv", "u1", (12,)),
    ("vit", "i1", (4,)),
    ("cnt", "<i2", (4,)),
    ("ach", "<u4"), ("t", "<u4"), ("episode", "<u4"),
    ("seed", "<u8"),
    ("mob", MOB_DTYPE, (12,)),
    ("plant", PLANT_DTYPE, (10,)),
    ("env", "<u4"),
])
assert ENV_DTYPE.itemsize == 4304


# ---- full Craftax ------------------------------------------------------------------------
FULL_OBS_U8_F32, FULL_OBS_F32, FULL_OBS_PIXELS_F32 = 0, 1, 2
FULL_OBS_BYTES = {0: 8448, 1: 33152, 2: 171648}
FULL_MOB_DTYPE = np.dtype([("alive", "u1"), ("x", "u1"), ("y", "u1"), ("dir", "u1"), ("hp", "i1"),
                           ("cd", "u1"), ("type", "u1"), ("pad", "u1")])
FULL_ENV_DTYPE = np.dtype([
    ("block", "u1", (9, 48, 48)), ("item", "u1", (9, 48, 48)), ("light", "u1", (9, 48, 48)),
    ("px", "u1"), ("py", "u1"), ("dir", "u1"), ("floor", "u1"),
    ("sleeping", "u1"), ("resting", "u1"), ("learned_fireball", "u1"), ("learned_iceball", "u1"),
    ("inv", "u1", (10,)), ("potion", "u1", (6,)),
    ("book", "u1"), ("pickaxe", "u1"), ("sword", "u1"), ("sword_ench", "u1"), ("bow", "u1"), ("bow_ench", "u1"),
    ("armour", "u1", (4,)), ("armour_ench", "u1", (4,)),
    ("vit", "i1", (5,)),
    ("xp", "u1"), ("dex", "u1"), ("str", "u1"), ("intel", "u1"),
    ("pad_a", "u1"),
    ("cnt", "<i2", (5,)),
    ("potion_effect", "u1", (6,)), ("kills", "u1", (9,)),
    ("boss_hits", "u1"), ("boss_vulnerable", "u1"),
    ("pad_b", "u1"),
    ("visited", "<u2"),
    ("ladder_up", "u1", (9, 2)), ("ladder_down", "u1", (9, 2)),
    ("pad_c", "u1", (2,)),
    ("ach", "<u4", (3,)),
    ("t", "<u4"), ("episode", "<u4"), ("env", "<u4"), ("pad0", "<u4"),
    ("seed", "<u8"),
    ("mob", FULL_MOB_DTYPE, (9, 14)),
    ("plant", PLANT_DTYPE, (10,)),
    ("pad1", "u1", (4,)),
])
assert FULL_ENV_DTYPE.itemsize == 63432


class FullConfig(ctypes.Structure):
    _fields_ = [("max_episode_steps", ctypes.c_uint32), ("day_length", ctypes.c_uint32),
                ("cap_melee", ctypes.c_uint32), ("cap_ranged", ctypes.c_uint32),
                ("cap_passive", ctypes.c_uint32), ("cap_plant", ctypes.c_uint32), ("atlas_seed", ctypes.c_uint64),
                ("worldgen", ctypes.c_uint32), ("reset_mode", ctypes.c_uint32)]


class Config(ctypes.Structure):
    _fields_ = [("max_episode_steps", ctypes.c_uint32), ("day_length", ctypes.c_uint32),
                ("cap_zombie", ctypes.c_uint32), ("cap_cow", ctypes.c_uint32),
                ("cap_skeleton", ctypes.c_uint32), ("cap_arrow", ctypes.c_uint32),
                ("cap_plant", ctypes.c_uint32), ("atlas_seed", ctypes.c_uint64),
                ("worldgen", ctypes.c_uint32), ("reset_mode", ctypes.c_uint32)]


WORLDGEN_VALUE, WORLDGEN_PERLIN = 0, 1


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (plain C11, contraction off so floats are single IEEE ops)."""
    srcs = [os.path.join(_HERE, s) for s in _SOURCES]
    deps = srcs + [os.path.join(_HERE, h) for h in _HEADERS]
    if not force and os.path.exists(LIB_PATH) and all(
            os.path.getmtime(LIB_PATH) >= os.path.getmtime(d) for d in deps):
        return LIB_PATH
    cmd = ["gcc", "-O2", "-std=c11", "-Wall", "-Wextra", "-ffp-contract=off", "-fPIC", "-shared",
           "-o", LIB_PATH] + srcs + ["-lm"]
    subprocess.run(cmd, check=True)
    return LIB_PATH


_lib = None


def lib() -> ctypes.CDLL:
    global _lib
    if _lib is None:
        build()
        L = ctypes.CDLL(LIB_PATH)
        L.orc_env_bytes.restype = ctypes.c_size_t
        L.orc_obs_bytes.restype = ctypes.c_size_t
        L.orc_daylight.restype = ctypes.c_float
        L.orc_zombie_spawn_threshold.restype = ctypes.c_uint32
        L.orc_step_draw.restype = ctypes.c_uint32
        L.orc_value_noise.restype = ctypes.c_uint32
        L.orc_perlin_noise.restype = ctypes.c_uint32
        assert L.orc_env_bytes() == ENV_DTYPE.itemsize
        L.cf_env_bytes.restype = ctypes.c_size_t
        L.cf_obs_bytes.restype = ctypes.c_size_t
        L.cf_step_draw.restype = ctypes.c_uint32
        assert L.cf_env_bytes() == FULL_ENV_DTYPE.itemsize
        _lib = L
    return _lib


def _p(a: np.ndarray):
    return a.ctypes.data_as(ctypes.c_void_p)


def default_config(**overrides) -> Config:
    cfg = Config()
    lib().orc_default_config(ctypes.byref(cfg))
    for k, v in overrides.items():
        setattr(cfg, k, v)
    return cfg


def philox(ctr, key):
    c = (ctypes.c_uint32 * 4)(*[int(x) for x in ctr])
    k = (ctypes.c_uint32 * 2)(*[int(x) for x in key])
    o = (ctypes.c_uint32 * 4)()
    lib().orc_philox4x32_10(c, k, o)
    return [int(x) for x in o]


def worldgen(seed: int, env: int, episode: int = 0, mode: int = WORLDGEN_VALUE) -> np.ndarray:
    m = np.zeros((64, 64), np.uint8)
    lib().orc_worldgen_mode(_p(m), ctypes.c_uint64(seed), ctypes.c_uint32(env), ctypes.c_uint32(episode), ctypes.c_uint32(mode))
    return m


RESET_EXACT, RESET_POOL = 0, 1
POOL_RATIO = 16
THETA_LEN = 374      # Perlin gradient angles of one Classic world: 2 x 25 + 4 x 81
FULL_THETA_LEN = 620  # of one full-Craftax world: overworld 2 x 16 + 4 x 49, then 2 x 49 for each of the cave floors 2, 5, 6, 7
FULL_THETA_OFFSET = {0: 0, 2: 228, 5: 326, 6: 424, 7: 522}


def worldgen_theta(seed: int, env: int, episode: int, theta: np.ndarray) -> np.ndarray:
    """Perlin world whose gradient angles are turned by theta[i] / 1024 of a turn."""
    th = np.ascontiguousarray(theta, dtype=np.uint16)
    assert th.shape == (THETA_LEN,)
    m = np.zeros((64, 64), np.uint8)
    lib().orc_worldgen_theta(_p(m), ctypes.c_uint64(seed), ctypes.c_uint32(env), ctypes.c_uint32(episode), _p(th))
    return m


def pool_slot(pool_seed: int, step_index: int, rank: int, n: int) -> int:
    L = lib()
    L.orc_pool_slot.restype = ctypes.c_uint32
    return int(L.orc_pool_slot(ctypes.c_uint64(pool_seed), ctypes.c_uint32(step_index), ctypes.c_uint32(rank), ctypes.c_uint32(n)))


def perlin_noise(lattice: np.ndarray, spacing: int, x: int, y: int) -> int:
    """Integer Perlin noise of the oracle over a square u16 lattice, on the 0..65535 scale."""
    lat = np.ascontiguousarray(lattice, dtype=np.uint16)
    return int(lib().orc_perlin_noise(_p(lat), lat.shape[1], spacing, x, y))


def _host_threads() -> int:
    """Worker threads for the batched helpers below: the cores this process may use, 16 at most."""
    try:
        c = len(os.sched_getaffinity(0))
    except AttributeError:
        c = os.cpu_count() or 1
    return max(1, min(16, c))


def _step_many(orc, step_fn, observe_fn, env_bytes, actions, threads, render_last, sample, sample_obs):
    """Harness, no arithmetic: K steps of every environment of `orc`, the environments cut into
    contiguous slices that Python threads advance independently (the C calls release the
    interpreter lock; environments never interact with exact resets).  Inside a slice it is the
    ordinary serial batch call, step after step."""
    from concurrent.futures import ThreadPoolExecutor

    assert orc.cfg.reset_mode == RESET_EXACT, "pool resets couple the environments of a step"
    a = np.ascontiguousarray(actions, dtype=np.int32)
    K, n = a.shape
    assert n == orc.n
    threads = _host_threads() if threads is None else threads
    rew = np.zeros((K, n), np.float32)
    don = np.zeros((K, n), np.uint8)
    stride = orc.obs.shape[1]
    sample = None if sample is None else np.asarray(sample, dtype=np.int64)
    if sample is not None:
        assert sample_obs.shape == (K, len(sample), stride) and sample_obs.dtype == np.uint8 and sample_obs.flags.c_contiguous
    bounds = np.linspace(0, n, min(threads, n) + 1).astype(np.int64)
    cfg = ctypes.byref(orc.cfg)

    def work(w):
        lo, hi = int(bounds[w]), int(bounds[w + 1])
        if hi == lo:
            return
        envs = ctypes.c_void_p(orc.envs.ctypes.data + lo * env_bytes)
        obs = ctypes.c_void_p(orc.obs.ctypes.data + lo * stride)
        mine = [] if sample is None else [(j, int(i)) for j, i in enumerate(sample) if lo <= i < hi]
        for k in range(K):
            step_fn(envs, cfg, ctypes.c_void_p(a.ctypes.data + (k * n + lo) * 4), orc.obs_mode,
                    obs if (render_last and k == K - 1) else None,
                    ctypes.c_void_p(rew.ctypes.data + (k * n + lo) * 4), ctypes.c_void_p(don.ctypes.data + k * n + lo), hi - lo)
            for j, i in mine:
                observe_fn(ctypes.c_void_p(orc.envs.ctypes.data + i * env_bytes), cfg, orc.obs_mode,
                           ctypes.c_void_p(sample_obs.ctypes.data + (k * len(sample) + j) * stride))

    with ThreadPoolExecutor(max_workers=threads) as ex:
        list(ex.map(work, range(len(bounds) - 1)))
    orc.steps += K
    return rew, don


def _reset_many(orc, reset_fn, env_bytes, seeds, threads):
    from concurrent.futures import ThreadPoolExecutor

    seeds = np.ascontiguousarray(seeds, dtype=np.uint64)
    ids = np.arange(orc.n, dtype=np.uint32)
    threads = _host_threads() if threads is None else threads
    bounds = np.linspace(0, orc.n, min(threads, orc.n) + 1).astype(np.int64)
    cfg = ctypes.byref(orc.cfg)

    def work(w):
        lo, hi = int(bounds[w]), int(bounds[w + 1])
        if hi > lo:
            reset_fn(ctypes.c_void_p(orc.envs.ctypes.data + lo * env_bytes), cfg, ctypes.c_void_p(seeds.ctypes.data + lo * 8),
                     ctypes.c_void_p(ids.ctypes.data + lo * 4), hi - lo)

    with ThreadPoolExecutor(max_workers=threads) as ex:
        list(ex.map(work, range(len(bounds) - 1)))
    orc.steps = 0


class Oracle:
    """n independent environments stepped serially on the host."""

    def __init__(self, n: int, cfg: Config | None = None, obs_mode: int = OBS_SYM_U8_F32):
        self.n = n
        self.cfg = cfg if cfg is not None else default_config()
        self.obs_mode = obs_mode
        self.steps = 0
        self.envs = np.zeros(n, dtype=ENV_DTYPE)
        self.obs = np.zeros((n, OBS_BYTES[obs_mode]), np.uint8)
        self.reward = np.zeros(n, np.float32)
        self.done = np.zeros(n, np.uint8)

    def reset(self, seeds, env_ids=None):
        seeds = np.ascontiguousarray(seeds, dtype=np.uint64)
        ids = None if env_ids is None else np.ascontiguousarray(env_ids, dtype=np.uint32)
        self.steps = 0                      # batch steps since the reset (names the pool of the optimistic resets)
        lib().orc_reset_batch(_p(self.envs), ctypes.byref(self.cfg), _p(seeds),
                              None if ids is None else _p(ids), self.n)
        return self.observe()

    def observe(self):
        lib().orc_observe_batch(_p(self.envs), ctypes.byref(self.cfg), self.obs_mode, _p(self.obs), self.n)
        return self.obs

    def step(self, actions, render: bool = True):
        a = np.ascontiguousarray(actions, dtype=np.int32)
        assert a.shape == (self.n,)
        if self.cfg.reset_mode == RESET_POOL:
            lib().orc_step_batch_pool(_p(self.envs), ctypes.byref(self.cfg), _p(a), self.obs_mode,
                                      _p(self.obs) if render else None, _p(self.reward), _p(self.done), self.n,
                                      ctypes.c_uint32(self.steps))
        else:
            lib().orc_step_batch(_p(self.envs), ctypes.byref(self.cfg), _p(a), self.obs_mode,
                                 _p(self.obs) if render else None, _p(self.reward), _p(self.done), self.n)
        self.steps += 1
        return self.obs, self.reward, self.done

    def step_many(self, actions, threads=None, render_last=True, sample=None, sample_obs=None):
        """K = len(actions) steps of all environments on several host threads (slices of
        environments; see _step_many).  Returns reward [K, n] and done [K, n]; self.obs holds the
        observation after the last step if render_last; the observations of the environments in
        `sample` after every step go to sample_obs [K, len(sample), stride]."""
        return _step_many(self, lib().orc_step_batch, lib().orc_observe, ENV_DTYPE.itemsize, actions, threads, render_last,
                          sample, sample_obs)

    def reset_many(self, seeds, threads=None):
        """reset() of all environments (numbered 0..n-1) on several host threads; no rendering."""
        _reset_many(self, lib().orc_reset_batch, ENV_DTYPE.itemsize, seeds, threads)

    def step_rules_one(self, i: int, action: int):
        """Rules without auto-reset on environment i; returns (reward, done)."""
        r = ctypes.c_float()
        d = ctypes.c_uint8()
        ptr = ctypes.c_void_p(self.envs.ctypes.data + i * ENV_DTYPE.itemsize)
        lib().orc_step_rules(ptr, ctypes.byref(self.cfg), ctypes.c_int32(action), ctypes.byref(r), ctypes.byref(d))
        return r.value, d.value

    def observe_one(self, i: int, mode: int | None = None) -> np.ndarray:
        mode = self.obs_mode if mode is None else mode
        out = np.zeros(OBS_BYTES[mode], np.uint8)
        ptr = ctypes.c_void_p(self.envs.ctypes.data + i * ENV_DTYPE.itemsize)
        lib().orc_observe(ptr, ctypes.byref(self.cfg), mode, _p(out))
        return out

    def draw(self, i: int, block: int, word: int) -> int:
        ptr = ctypes.c_void_p(self.envs.ctypes.data + i * ENV_DTYPE.itemsize)
        return int(lib().orc_step_draw(ptr, ctypes.c_uint32(block), ctypes.c_uint32(word)))

    def mutate_swap(self, mutation_seed: int, round_: int, restricted: bool) -> np.ndarray:
        """Swap mutation on every environment; returns the accepted try + 1 (0: no swap) per env."""
        out = np.zeros(self.n, np.int32)
        for i in range(self.n):
            ptr = ctypes.c_void_p(self.envs.ctypes.data + i * ENV_DTYPE.itemsize)
            out[i] = lib().orc_mutate_swap(ptr, ctypes.c_uint64(mutation_seed), ctypes.c_uint32(round_), int(restricted))
        return out

    def mutate_noise(self, theta: np.ndarray, mutation_seed: int, round_: int, amplitude: int) -> None:
        """Noise mutation on every environment; theta (uint16 [n][THETA_LEN]) is updated in place."""
        assert theta.dtype == np.uint16 and theta.shape == (self.n, THETA_LEN) and theta.flags.c_contiguous
        for i in range(self.n):
            ptr = ctypes.c_void_p(self.envs.ctypes.data + i * ENV_DTYPE.itemsize)
            lib().orc_mutate_noise(ptr, ctypes.byref(self.cfg), ctypes.c_void_p(theta.ctypes.data + i * THETA_LEN * 2),
                                   ctypes.c_uint64(mutation_seed), ctypes.c_uint32(round_), ctypes.c_uint32(amplitude))


def full_default_config(**overrides) -> FullConfig:
    cfg = FullConfig()
    lib().cf_default_config(ctypes.byref(cfg))
    for k, v in overrides.items():
        setattr(cfg, k, v)
    return cfg


class FullOracle:
    """n independent full-Craftax environments stepped serially on the host."""

    def __init__(self, n: int, cfg: FullConfig | None = None, obs_mode: int = FULL_OBS_U8_F32):
        self.n = n
        self.cfg = cfg if cfg is not None else full_default_config()
        self.obs_mode = obs_mode
        self.envs = np.zeros(n, dtype=FULL_ENV_DTYPE)
        self.steps = 0                      # batch steps since the reset (names the pool of the optimistic resets)
        self.obs = np.zeros((n, FULL_OBS_BYTES[obs_mode]), np.uint8)
        self.reward = np.zeros(n, np.float32)
        self.done = np.zeros(n, np.uint8)

    def _ptr(self, i: int):
        return ctypes.c_void_p(self.envs.ctypes.data + i * FULL_ENV_DTYPE.itemsize)

    def reset(self, seeds, env_ids=None):
        seeds = np.ascontiguousarray(seeds, dtype=np.uint64)
        ids = None if env_ids is None else np.ascontiguousarray(env_ids, dtype=np.uint32)
        lib().cf_reset_batch(_p(self.envs), ctypes.byref(self.cfg), _p(seeds),
                             None if ids is None else _p(ids), self.n)
        self.steps = 0
        return self.observe()

    def observe(self):
        lib().cf_observe_batch(_p(self.envs), ctypes.byref(self.cfg), self.obs_mode, _p(self.obs), self.n)
        return self.obs

    def step(self, actions, render: bool = True):
        a = np.ascontiguousarray(actions, dtype=np.int32)
        assert a.shape == (self.n,)
        if self.cfg.reset_mode == RESET_POOL:
            lib().cf_step_batch_pool(_p(self.envs), ctypes.byref(self.cfg), _p(a), self.obs_mode,
                                     _p(self.obs) if render else None, _p(self.reward), _p(self.done), self.n,
                                     ctypes.c_uint32(self.steps))
        else:
            lib().cf_step_batch(_p(self.envs), ctypes.byref(self.cfg), _p(a), self.obs_mode,
                                _p(self.obs) if render else None, _p(self.reward), _p(self.done), self.n)
        self.steps += 1
        return self.obs, self.reward, self.done

    def step_many(self, actions, threads=None, render_last=True, sample=None, sample_obs=None):
        """As Oracle.step_many, for the full game."""
        return _step_many(self, lib().cf_step_batch, lib().cf_observe, FULL_ENV_DTYPE.itemsize, actions, threads, render_last,
                          sample, sample_obs)

    def reset_many(self, seeds, threads=None):
        _reset_many(self, lib().cf_reset_batch, FULL_ENV_DTYPE.itemsize, seeds, threads)

    def step_rules_one(self, i: int, action: int):
        r = ctypes.c_float()
        d = ctypes.c_uint8()
        lib().cf_step_rules(self._ptr(i), ctypes.byref(self.cfg), ctypes.c_int32(action),
                            ctypes.byref(r), ctypes.byref(d))
        return r.value, d.value

    def observe_one(self, i: int, mode: int | None = None) -> np.ndarray:
        mode = self.obs_mode if mode is None else mode
        out = np.zeros(FULL_OBS_BYTES[mode], np.uint8)
        lib().cf_observe(self._ptr(i), ctypes.byref(self.cfg), mode, _p(out))
        return out

    def draw(self, i: int, block: int, word: int) -> int:
        return int(lib().cf_step_draw(self._ptr(i), ctypes.c_uint32(block), ctypes.c_uint32(word)))

    def mutate_noise(self, theta: np.ndarray, mutation_seed: int, round_: int, amplitude: int) -> None:
        """Noise mutation on every environment; theta (uint16 [n][FULL_THETA_LEN]) is updated in place."""
        assert theta.dtype == np.uint16 and theta.shape == (self.n, FULL_THETA_LEN) and theta.flags.c_contiguous
        for i in range(self.n):
            lib().cf_mutate_noise(self._ptr(i), ctypes.byref(self.cfg), ctypes.c_void_p(theta.ctypes.data + i * FULL_THETA_LEN * 2),
                                  ctypes.c_uint64(mutation_seed), ctypes.c_uint32(round_), ctypes.c_uint32(amplitude))

    def worldgen_floor_theta(self, i: int, f: int, theta: np.ndarray) -> None:
        """Regenerates floor f of environment i as the Perlin floor of level theta."""
        assert theta.dtype == np.uint16 and theta.shape == (FULL_THETA_LEN,) and theta.flags.c_contiguous
        lib().cf_worldgen_floor_theta(self._ptr(i), f, _p(theta))

    def mutate_swap(self, mutation_seed: int, round_: int, restricted: bool) -> np.ndarray:
        """Swap mutation of the overworld of every environment; returns the accepted try + 1 per env."""
        out = np.zeros(self.n, np.int32)
        for i in range(self.n):
            out[i] = lib().cf_mutate_swap(self._ptr(i), ctypes.c_uint64(mutation_seed), ctypes.c_uint32(round_), int(restricted))
        return out
