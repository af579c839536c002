"""Thin ctypes binding of libcraftax_hip.so (see include/craftax.h).

Argument marshalling only: every step of the simulator runs in the HIP kernels.  PyTorch is
used for device memory and streams.  There is no CPU fallback: if the library is missing or
no GPU is present the calls raise.
"""
from __future__ import annotations

import ctypes
import os

import numpy as np

_PKG = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_PKG, "libcraftax_hip.so")
DEBUG_LIB_PATH = os.path.join(_PKG, "libcraftax_hip_debug.so")     # the same sources built with bounds checks

OBS_SYM_U8_I8, OBS_SYM_U8_F32, OBS_SYM_F32, OBS_PIXELS_F32 = 0, 1, 2, 3
WORLDGEN_VALUE, WORLDGEN_PERLIN = 0, 1
VARIANT_CLASSIC, VARIANT_CRAFTAX = 0, 1

EXPORTS = [
    "craftax_default_config", "craftax_default_config_for", "craftax_state_bytes", "craftax_obs_bytes",
    "craftax_env_dump_bytes", "craftax_env_dump_bytes_for",
    "craftax_state_init", "craftax_state_attach", "craftax_state_release", "craftax_reset", "craftax_step", "craftax_observe",
    "craftax_rollout", "craftax_export_envs", "craftax_import_envs", "craftax_mutate_swap", "craftax_mutate_noise", "craftax_synth_actions", "craftax_last_error",
    "craftax_stats_workspace_bytes", "craftax_stats", "craftax_stats_static",
    "craftax_debug_bounds", "craftax_debug_bounds_selftest",
]


THETA_LEN = 374      # angle offsets per Classic level (craftax_mutate_noise)
FULL_THETA_LEN = 620  # per full-Craftax level
RESET_EXACT, RESET_POOL = 0, 1


class Config(ctypes.Structure):
    _fields_ = [("abi_version", ctypes.c_uint32), ("variant", ctypes.c_uint32), ("obs_mode", ctypes.c_uint32),
                ("max_episode_steps", ctypes.c_uint32), ("day_length", ctypes.c_uint32),
                ("cap_zombie", ctypes.c_uint32), ("cap_cow", ctypes.c_uint32), ("cap_skeleton", ctypes.c_uint32),
                ("cap_arrow", ctypes.c_uint32), ("cap_plant", ctypes.c_uint32), ("atlas_seed", ctypes.c_uint64),
                ("worldgen", ctypes.c_uint32), ("reset_mode", ctypes.c_uint32),
                ("group_lanes", ctypes.c_uint32), ("reserved", ctypes.c_uint32)]


# numpy views of the canonical dumps declared in include/craftax.h
_MOB = np.dtype([("alive", "u1"), ("x", "u1"), ("y", "u1"), ("dir", "u1"), ("hp", "i1"), ("cd", "u1"), ("pad", "u1", (2,))])
_PLANT = np.dtype([("alive", "u1"), ("x", "u1"), ("y", "u1"), ("pad", "u1"), ("age", "<u2")])
ENV_DUMP_DTYPE = np.dtype([
    ("map", "u1", (64, 64)), ("px", "u1"), ("py", "u1"), ("dir", "u1"), ("sleeping", "u1"), ("inv", "u1", (12,)),
    ("vit", "i1", (4,)), ("cnt", "<i2", (4,)), ("ach", "<u4"), ("t", "<u4"), ("episode", "<u4"), ("seed", "<u8"),
    ("mob", _MOB, (12,)), ("plant", _PLANT, (10,)), ("env", "<u4")])
_FULL_MOB = np.dtype([("alive", "u1"), ("x", "u1"), ("y", "u1"), ("dir", "u1"), ("hp", "i1"), ("cd", "u1"), ("type", "u1"), ("pad", "u1")])
FULL_ENV_DUMP_DTYPE = np.dtype([
    ("block", "u1", (9, 48, 48)), ("item", "u1", (9, 48, 48)), ("light", "u1", (9, 48, 48)),
    ("px", "u1"), ("py", "u1"), ("dir", "u1"), ("floor", "u1"),
    ("sleeping", "u1"), ("resting", "u1"), ("learned_fireball", "u1"), ("learned_iceball", "u1"),
    ("inv", "u1", (10,)), ("potion", "u1", (6,)),
    ("book", "u1"), ("pickaxe", "u1"), ("sword", "u1"), ("sword_ench", "u1"), ("bow", "u1"), ("bow_ench", "u1"),
    ("armour", "u1", (4,)), ("armour_ench", "u1", (4,)), ("vit", "i1", (5,)),
    ("xp", "u1"), ("dex", "u1"), ("str", "u1"), ("intel", "u1"), ("pad_a", "u1"), ("cnt", "<i2", (5,)),
    ("potion_effect", "u1", (6,)), ("kills", "u1", (9,)), ("boss_hits", "u1"), ("boss_vulnerable", "u1"), ("pad_b", "u1"),
    ("visited", "<u2"), ("ladder_up", "u1", (9, 2)), ("ladder_down", "u1", (9, 2)), ("pad_c", "u1", (2,)),
    ("ach", "<u4", (3,)), ("t", "<u4"), ("episode", "<u4"), ("env", "<u4"), ("pad0", "<u4"), ("seed", "<u8"),
    ("mob", _FULL_MOB, (9, 14)), ("plant", _PLANT, (10,)), ("pad1", "u1", (4,))])
assert ENV_DUMP_DTYPE.itemsize == 4304 and FULL_ENV_DUMP_DTYPE.itemsize == 63432


STATS_ACHIEVEMENTS = 96
STATS_DTYPE = np.dtype([("episodes", "<u8"), ("steps", "<u8"), ("achievements", "<u4", (STATS_ACHIEVEMENTS,)), ("n", "<u4"), ("pad", "<u4"),
                        ("unlocks", "<u8", (STATS_ACHIEVEMENTS,))])
assert STATS_DTYPE.itemsize == 408 + 8 * STATS_ACHIEVEMENTS


class CraftaxError(RuntimeError):
    pass


_lib = None


def use_library(path: str):
    """Switches every later call of this module to the library at `path` (LIB_PATH or
    DEBUG_LIB_PATH).  States made with one library are not known to the other."""
    global _lib, LIB_PATH
    LIB_PATH = path
    _lib = None


def craftax_debug_bounds():
    """(checks built in, [violations, line, index, limit]) of the loaded library; clears the record."""
    rep = (ctypes.c_uint32 * 4)()
    rc = load().craftax_debug_bounds(rep)
    if rc < 0:
        raise CraftaxError(f"craftax_debug_bounds failed ({rc}): {load().craftax_last_error().decode()}")
    return bool(rc), [int(x) for x in rep]


def load() -> ctypes.CDLL:
    """Loads the built library; raises if it has not been built (run __graft_entry__.build())."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise CraftaxError(f"{LIB_PATH} is missing: build it first (python -c 'import __graft_entry__ as g; g.build()')")
    # PyTorch ships its own HIP runtime; import it first so that this library binds to the
    # same runtime instance (same SONAME) instead of bringing a second one into the process.
    import torch  # noqa: F401

    L = ctypes.CDLL(LIB_PATH)
    vp, i32, u64 = ctypes.c_void_p, ctypes.c_int, ctypes.c_uint64
    L.craftax_default_config.argtypes = [ctypes.POINTER(Config)]
    L.craftax_default_config.restype = None
    L.craftax_default_config_for.argtypes = [ctypes.POINTER(Config), ctypes.c_uint32]
    L.craftax_default_config_for.restype = None
    L.craftax_env_dump_bytes_for.argtypes = [ctypes.POINTER(Config)]
    L.craftax_env_dump_bytes_for.restype = ctypes.c_size_t
    L.craftax_state_bytes.argtypes = [ctypes.POINTER(Config), i32]
    L.craftax_state_bytes.restype = ctypes.c_size_t
    L.craftax_obs_bytes.argtypes = [ctypes.POINTER(Config)]
    L.craftax_obs_bytes.restype = ctypes.c_size_t
    L.craftax_env_dump_bytes.argtypes = []
    L.craftax_env_dump_bytes.restype = ctypes.c_size_t
    L.craftax_state_init.argtypes = [vp, ctypes.POINTER(Config), i32, vp]
    L.craftax_state_attach.argtypes = [vp, ctypes.POINTER(Config), i32, vp]
    L.craftax_state_release.argtypes = [vp]
    L.craftax_reset.argtypes = [vp, vp, i32, vp]
    L.craftax_step.argtypes = [vp, vp, vp, vp, vp, i32, vp]
    L.craftax_observe.argtypes = [vp, vp, i32, vp]
    L.craftax_export_envs.argtypes = [vp, i32, i32, vp, vp]
    L.craftax_import_envs.argtypes = [vp, i32, i32, vp, vp]
    L.craftax_rollout.argtypes = [vp, vp, i32, vp, vp, vp, i32, vp]
    L.craftax_mutate_swap.argtypes = [vp, i32, i32, u64, ctypes.c_uint32, i32, vp, vp]
    L.craftax_mutate_noise.argtypes = [vp, i32, i32, vp, u64, ctypes.c_uint32, ctypes.c_uint32, vp]
    L.craftax_synth_actions.argtypes = [vp, i32, i32, i32, u64, i32, vp]
    L.craftax_stats_workspace_bytes.argtypes = [i32]
    L.craftax_stats_workspace_bytes.restype = ctypes.c_size_t
    L.craftax_stats.argtypes = [vp, vp, vp, ctypes.c_size_t, i32, vp]
    L.craftax_stats_static.argtypes = [vp, vp, i32, vp]
    L.craftax_debug_bounds.argtypes = [ctypes.POINTER(ctypes.c_uint32 * 4)]
    L.craftax_debug_bounds_selftest.argtypes = []
    L.craftax_last_error.argtypes = []
    L.craftax_last_error.restype = ctypes.c_char_p
    _lib = L
    return L


def _check(rc: int, what: str):
    if rc != 0:
        raise CraftaxError(f"{what} failed ({rc}): {load().craftax_last_error().decode()}")


def default_config(variant: int = VARIANT_CLASSIC, **overrides) -> Config:
    cfg = Config()
    load().craftax_default_config_for(ctypes.byref(cfg), variant)
    for k, v in overrides.items():
        setattr(cfg, k, v)
    return cfg


def craftax_state_bytes(cfg: Config, n: int) -> int:
    return int(load().craftax_state_bytes(ctypes.byref(cfg), n))


def craftax_obs_bytes(cfg: Config) -> int:
    return int(load().craftax_obs_bytes(ctypes.byref(cfg)))


def craftax_env_dump_bytes() -> int:
    return int(load().craftax_env_dump_bytes())


def craftax_env_dump_bytes_for(cfg: Config) -> int:
    return int(load().craftax_env_dump_bytes_for(ctypes.byref(cfg)))


def _stream_ptr(stream) -> int:
    return 0 if stream is None else int(stream.cuda_stream)


def craftax_state_init(state, cfg: Config, n: int, stream=None):
    _check(load().craftax_state_init(state.data_ptr(), ctypes.byref(cfg), n, _stream_ptr(stream)), "craftax_state_init")


def craftax_state_attach(state, cfg: Config, n: int, stream=None):
    _check(load().craftax_state_attach(state.data_ptr(), ctypes.byref(cfg), n, _stream_ptr(stream)), "craftax_state_attach")


def craftax_state_release(state):
    load().craftax_state_release(state.data_ptr())


def craftax_reset(state, seeds, n: int, stream=None):
    _check(load().craftax_reset(state.data_ptr(), seeds.data_ptr(), n, _stream_ptr(stream)), "craftax_reset")


def craftax_step(state, actions, obs, reward, done, n: int, stream=None):
    _check(load().craftax_step(state.data_ptr(), actions.data_ptr(), 0 if obs is None else obs.data_ptr(),
                               reward.data_ptr(), done.data_ptr(), n, _stream_ptr(stream)), "craftax_step")


def craftax_rollout(state, actions, steps: int, obs, reward, done, n: int, stream=None):
    _check(load().craftax_rollout(state.data_ptr(), actions.data_ptr(), steps, 0 if obs is None else obs.data_ptr(),
                                  reward.data_ptr(), done.data_ptr(), n, _stream_ptr(stream)), "craftax_rollout")


def craftax_observe(state, obs, n: int, stream=None):
    _check(load().craftax_observe(state.data_ptr(), obs.data_ptr(), n, _stream_ptr(stream)), "craftax_observe")


def craftax_export_envs(state, first: int, count: int, dumps, stream=None):
    _check(load().craftax_export_envs(state.data_ptr(), first, count, dumps.data_ptr(), _stream_ptr(stream)),
           "craftax_export_envs")


def craftax_import_envs(state, first: int, count: int, dumps, stream=None):
    _check(load().craftax_import_envs(state.data_ptr(), first, count, dumps.data_ptr(), _stream_ptr(stream)),
           "craftax_import_envs")


def craftax_mutate_swap(state, first: int, count: int, mutation_seed: int, round_: int, restricted: bool, tries=None, stream=None):
    _check(load().craftax_mutate_swap(state.data_ptr(), first, count, mutation_seed, round_, int(bool(restricted)),
                                      None if tries is None else tries.data_ptr(), _stream_ptr(stream)), "craftax_mutate_swap")


def craftax_mutate_noise(state, first: int, count: int, theta, mutation_seed: int, round_: int, amplitude: int, stream=None):
    _check(load().craftax_mutate_noise(state.data_ptr(), first, count, None if theta is None else theta.data_ptr(), mutation_seed,
                                       round_, amplitude, _stream_ptr(stream)), "craftax_mutate_noise")


def craftax_stats_workspace_bytes(n: int) -> int:
    return int(load().craftax_stats_workspace_bytes(n))


def craftax_stats(state, out, workspace, n: int, stream=None):
    _check(load().craftax_stats(state.data_ptr(), out.data_ptr(), workspace.data_ptr(), workspace.numel() * workspace.element_size(),
                                n, _stream_ptr(stream)), "craftax_stats")


def craftax_stats_static(state, out, n: int, stream=None):
    _check(load().craftax_stats_static(state.data_ptr(), out.data_ptr(), n, _stream_ptr(stream)), "craftax_stats_static")


STATS_STATIC_MAX_ENVS = 524288


def craftax_synth_actions(actions, n: int, step0: int, steps: int, action_seed: int, kind: int, stream=None):
    _check(load().craftax_synth_actions(actions.data_ptr(), n, step0, steps, action_seed, kind, _stream_ptr(stream)),
           "craftax_synth_actions")


class Craftax:
    """Owns the device buffers of n environments and forwards to the C ABI."""

    def __init__(self, n: int, cfg: Config | None = None, device: str = "cuda:0"):
        import torch

        if not torch.cuda.is_available():
            raise CraftaxError("no GPU visible: the simulator has no CPU path")
        self.torch = torch
        self.n = n
        self.cfg = cfg if cfg is not None else default_config()
        self.device = torch.device(device)
        nbytes = craftax_state_bytes(self.cfg, n)
        if nbytes == 0:
            raise CraftaxError("invalid configuration")
        self.obs_bytes = craftax_obs_bytes(self.cfg)
        self.state = torch.empty(nbytes, dtype=torch.uint8, device=self.device)
        self.obs = torch.zeros((n, self.obs_bytes), dtype=torch.uint8, device=self.device)
        self.reward = torch.zeros(n, dtype=torch.float32, device=self.device)
        self.done = torch.zeros(n, dtype=torch.uint8, device=self.device)
        self.stream = torch.cuda.current_stream(self.device)
        craftax_state_init(self.state, self.cfg, n, self.stream)

    def close(self):
        if self.state is not None:
            craftax_state_release(self.state)
            self.state = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def reset(self, seeds):
        torch = self.torch
        s = torch.as_tensor(np.ascontiguousarray(seeds, dtype=np.uint64).view(np.int64), device=self.device)
        craftax_reset(self.state, s, self.n, self.stream)
        craftax_observe(self.state, self.obs, self.n, self.stream)
        return self.obs

    def step(self, actions):
        """actions: int32 device tensor [n]."""
        craftax_step(self.state, actions, self.obs, self.reward, self.done, self.n, self.stream)
        return self.obs, self.reward, self.done

    @property
    def dump_dtype(self) -> np.dtype:
        return FULL_ENV_DUMP_DTYPE if self.cfg.variant == VARIANT_CRAFTAX else ENV_DUMP_DTYPE

    def export_envs(self, first: int = 0, count: int | None = None) -> np.ndarray:
        torch = self.torch
        count = self.n - first if count is None else count
        size = craftax_env_dump_bytes_for(self.cfg)
        buf = torch.empty((count, size), dtype=torch.uint8, device=self.device)
        craftax_export_envs(self.state, first, count, buf, self.stream)
        return buf.cpu().numpy()

    def import_envs(self, dumps: np.ndarray, first: int = 0):
        torch = self.torch
        raw = np.ascontiguousarray(dumps).view(np.uint8).reshape(-1, craftax_env_dump_bytes_for(self.cfg))
        buf = torch.as_tensor(raw, device=self.device)
        craftax_import_envs(self.state, first, raw.shape[0], buf, self.stream)
        self.torch.cuda.synchronize(self.device)

    def stats(self) -> np.ndarray:
        """Metrics snapshot (craftax_stats) as a numpy record of STATS_DTYPE."""
        torch = self.torch
        out = torch.zeros(STATS_DTYPE.itemsize, dtype=torch.uint8, device=self.device)
        work = torch.empty(craftax_stats_workspace_bytes(self.n), dtype=torch.uint8, device=self.device)
        craftax_stats(self.state, out, work, self.n, self.stream)
        return out.cpu().numpy().view(STATS_DTYPE)[0]

    def mutate_swap(self, mutation_seed: int, round_: int, restricted: bool, first: int = 0, count: int | None = None) -> np.ndarray:
        """Swap mutation of the current maps; returns the accepted try + 1 (0: none) per environment."""
        count = self.n - first if count is None else count
        tries = self.torch.zeros(count, dtype=self.torch.int32, device=self.device)
        craftax_mutate_swap(self.state, first, count, mutation_seed, round_, restricted, tries, self.stream)
        return tries.cpu().numpy()

    def mutate_noise(self, theta, mutation_seed: int, round_: int, amplitude: int, first: int = 0):
        """Noise mutation; theta: device int16 tensor [count][THETA_LEN] (FULL_THETA_LEN for the full game)
        holding the angle offsets, updated in place."""
        row = FULL_THETA_LEN if self.cfg.variant == VARIANT_CRAFTAX else THETA_LEN
        assert theta.dtype == self.torch.int16 and theta.is_contiguous() and theta.shape[1] == row
        craftax_mutate_noise(self.state, first, theta.shape[0], theta, mutation_seed, round_, amplitude, self.stream)
