"""Host-only checks of the C ABI: the library loads, exports every symbol the header
declares, and its size queries agree with the documented layouts.  No kernel is launched."""
import ctypes
import os
import re

import pytest

from paper_2402_16801_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(binding.LIB_PATH):
        import __graft_entry__ as g
        g.build()
    return binding.load()


def test_every_declared_symbol_is_exported(lib):
    header = open(os.path.join(ROOT, "include", "craftax.h")).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    declared = set(re.findall(r"\b(craftax_[a-z_]+)\s*\(", header))
    assert declared == set(binding.EXPORTS)
    for name in declared:
        assert getattr(lib, name) is not None


def test_sizes_and_defaults(lib):
    cfg = binding.default_config()
    assert (cfg.abi_version, cfg.variant, cfg.obs_mode) == (2, 0, 1)
    assert (cfg.max_episode_steps, cfg.day_length) == (10000, 300)
    assert (cfg.cap_zombie, cfg.cap_cow, cfg.cap_skeleton, cfg.cap_arrow, cfg.cap_plant) == (3, 3, 3, 3, 10)
    assert binding.craftax_env_dump_bytes() == 4304
    strides = {0: 1408, 1: 1536, 2: 5392, 3: 47632}
    for mode, stride in strides.items():
        cfg.obs_mode = mode
        assert binding.craftax_obs_bytes(cfg) == stride and stride % 16 == 0
    assert 1345 * 4 <= strides[2] and 63 * 63 * 3 * 4 <= strides[3]
    cfg.obs_mode = 1
    b1, b2 = binding.craftax_state_bytes(cfg, 1), binding.craftax_state_bytes(cfg, 1001)
    per_env = 2 * 4096 + 128 + 16 + 3 * 16         # two map slots, record, two spare tags, three list entries
    assert abs((b2 - b1) - 1000 * per_env) < 70000 and b1 % 256 == 0   # sub-lists round their capacity up
    assert binding.craftax_state_bytes(cfg, 0) == 0 and binding.craftax_state_bytes(cfg, -3) == 0
    cfg.day_length = 7
    assert binding.craftax_state_bytes(cfg, 4) == 0


def test_full_variant_sizes_and_defaults(lib):
    cfg = binding.default_config(binding.VARIANT_CRAFTAX)
    assert (cfg.abi_version, cfg.variant, cfg.obs_mode) == (2, 1, 1)
    assert (cfg.max_episode_steps, cfg.day_length) == (100000, 300)
    assert (cfg.cap_zombie, cfg.cap_cow, cfg.cap_skeleton, cfg.cap_plant) == (3, 3, 2, 10)
    assert binding.craftax_env_dump_bytes_for(cfg) == 63432
    assert binding.craftax_env_dump_bytes_for(binding.default_config()) == 4304
    assert binding.craftax_obs_bytes(cfg) == 8448 >= 99 * 83 + 51 * 4
    cfg.obs_mode = binding.OBS_SYM_F32
    assert binding.craftax_obs_bytes(cfg) == 33152 >= 8268 * 4
    cfg.obs_mode = binding.OBS_PIXELS_F32
    assert binding.craftax_obs_bytes(cfg) == 171648 >= 130 * 110 * 3 * 4
    for bad in (binding.OBS_SYM_U8_I8, 4):
        cfg.obs_mode = bad
        assert binding.craftax_obs_bytes(cfg) == 0 and binding.craftax_state_bytes(cfg, 8) == 0
    cfg.obs_mode = binding.OBS_SYM_U8_F32
    b1, b2 = binding.craftax_state_bytes(cfg, 1), binding.craftax_state_bytes(cfg, 1001)
    # per environment: 1024-byte record + mob tables, two slots of 9 floors x 2 maps x 2304 bytes, 9 spare-world
    # tags, three list entries (the sub-lists round their capacity up), 72 unlock counters
    assert abs((b2 - b1) - 1000 * (1024 + 2 * 9 * 2 * 2304 + 9 * 8 + 3 * 16 + 72 * 4)) < 8192 and b1 % 256 == 0
    cfg.cap_skeleton = 3
    assert binding.craftax_state_bytes(cfg, 8) == 0


def test_host_side_argument_errors(lib):
    cfg = binding.default_config()
    assert lib.craftax_state_init(None, ctypes.byref(cfg), 4, None) == -1
    assert lib.craftax_step(None, None, None, None, None, 4, None) == -1
    assert lib.craftax_step(ctypes.c_void_p(4096), None, None, None, None, 4, None) == -4
    assert lib.craftax_last_error() != b""
    assert lib.craftax_state_release(ctypes.c_void_p(4096)) == -4


def test_header_constants_match_their_python_mirrors():
    """The binding (and, separately, the oracle's wrapper) restate the header's numbers; a change on
    one side only would shift every array row."""
    from oracle import pyoracle as po
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    text = open(os.path.join(root, "include", "craftax.h")).read()
    defines = {k: int(v) for k, v in re.findall(r"#define\s+(CRAFTAX_\w+)\s+(\d+)\s*$", text, re.M)}
    enums = {k: int(v) for k, v in re.findall(r"(CRAFTAX_\w+)\s*=\s*(\d+)", text)}
    assert defines["CRAFTAX_THETA_LEN"] == binding.THETA_LEN == po.THETA_LEN == 2 * 25 + 4 * 81
    assert defines["CRAFTAX_FULL_THETA_LEN"] == binding.FULL_THETA_LEN == po.FULL_THETA_LEN == 2 * 16 + 4 * 49 + 4 * 2 * 49
    assert enums["CRAFTAX_WORLDGEN_VALUE"] == binding.WORLDGEN_VALUE == po.WORLDGEN_VALUE
    assert enums["CRAFTAX_WORLDGEN_PERLIN"] == binding.WORLDGEN_PERLIN == po.WORLDGEN_PERLIN
    assert enums["CRAFTAX_RESET_EXACT"] == binding.RESET_EXACT == po.RESET_EXACT
    assert enums["CRAFTAX_RESET_POOL"] == binding.RESET_POOL == po.RESET_POOL
    assert enums["CRAFTAX_VARIANT_CLASSIC"] == binding.VARIANT_CLASSIC and enums["CRAFTAX_VARIANT_CRAFTAX"] == binding.VARIANT_CRAFTAX
    assert defines["CRAFTAX_STATS_ACHIEVEMENTS"] == binding.STATS_ACHIEVEMENTS >= 67
    assert defines["CRAFTAX_STATS_STATIC_MAX_ENVS"] == binding.STATS_STATIC_MAX_ENVS and binding.STATS_STATIC_MAX_ENVS % 256 == 0
    assert binding.STATS_DTYPE.itemsize == 8 + 8 + 4 * 96 + 8 + 8 * 96
    assert binding.craftax_stats_workspace_bytes(1) == 1024 and binding.craftax_stats_workspace_bytes(257) == 2048
    assert binding.craftax_stats_workspace_bytes(0) == 0
