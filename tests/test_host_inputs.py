"""CPU-side checks of what surrounds the kernels: the seeded input generators (they serve both the
GPU tests and the oracle, and hold none of the method's arithmetic) and the host-side argument
checks of the newer entry points, which must refuse bad calls before anything is launched."""
import ctypes

import numpy as np
import pytest

from oracle import pyoracle as po
from paper_2402_16801_amd import binding, synth


@pytest.fixture(scope="module")
def lib():
    return binding.load()


def test_action_streams_are_pure_functions_with_the_stated_distributions():
    ids = np.arange(20000)
    a = synth.actions(ids, 3, "uniform", 5)
    assert a.dtype == np.int32 and a.min() == 0 and a.max() == 16
    assert np.array_equal(a, synth.actions(ids, 3, "uniform", 5))                  # pure in (env, step, seed)
    assert np.array_equal(a[[7, 19000]], synth.actions(np.array([7, 19000]), 3, "uniform", 5))   # any entry on its own
    assert not np.array_equal(a, synth.actions(ids, 4, "uniform", 5)) and not np.array_equal(a, synth.actions(ids, 3, "uniform", 6))
    hist = np.bincount(a, minlength=17) / len(a)
    assert np.all(np.abs(hist - 1 / 17) < 0.01)
    s = synth.actions(ids, 3, "skewed", 5)
    frac_move_do = np.isin(s, [1, 2, 3, 4, 5]).mean()
    assert abs(frac_move_do - (0.5 + 0.5 * 5 / 17)) < 0.015                        # half the draws go to LEFT..DO
    full = synth.actions(ids, 9, "uniform", 1, 43)
    assert full.max() == 42 and np.all(np.abs(np.bincount(full, minlength=43) / len(full) - 1 / 43) < 0.006)
    # the generator behind it is the same Philox the oracle was tested against
    c = synth.philox4x32_10(np.array([5]), np.array([6]), np.array([7]), np.array([8]), 0x1234, 0x9876)
    assert [int(x[0]) for x in c] == po.philox([5, 6, 7, 8], [0x1234, 0x9876])
    assert np.array_equal(synth.seeds_for(4, 10), np.array([10, 11, 12, 13], np.uint64))


def test_new_entry_points_refuse_bad_calls_on_the_host(lib):
    bogus = ctypes.c_void_p(4096)                      # aligned, but never registered
    buf = ctypes.c_void_p(8192)
    # unregistered state
    assert lib.craftax_rollout(bogus, buf, 4, buf, buf, buf, 4, None) == -4
    assert lib.craftax_observe(bogus, buf, 4, None) == -4
    assert lib.craftax_export_envs(bogus, 0, 1, buf, None) == -4
    assert lib.craftax_import_envs(bogus, 0, 1, buf, None) == -4
    assert lib.craftax_mutate_swap(bogus, 0, 1, 1, 0, 0, None, None) == -4
    assert lib.craftax_mutate_noise(bogus, 0, 1, buf, 1, 0, 5, None) == -4
    assert lib.craftax_reset(bogus, buf, 4, None) == -4
    # no state at all
    assert lib.craftax_rollout(None, buf, 4, buf, buf, buf, 4, None) == -1
    assert lib.craftax_mutate_noise(None, 0, 1, buf, 1, 0, 5, None) == -1
    # the synthetic action generator checks its own arguments
    assert lib.craftax_synth_actions(None, 4, 0, 1, 0, 0, None) == -1
    assert lib.craftax_synth_actions(buf, 0, 0, 1, 0, 0, None) == -3
    assert lib.craftax_synth_actions(buf, 4, 0, 0, 0, 0, None) == -3
    assert lib.craftax_synth_actions(buf, 4, -1, 1, 0, 0, None) == -3
    assert lib.craftax_synth_actions(buf, 4, 0, 1, 0, 4, None) == -3
    assert lib.craftax_last_error() != b""


@pytest.mark.parametrize("field,value", [("reset_mode", 2), ("worldgen", 2), ("day_length", 301), ("day_length", 0), ("day_length", 2048),
                                         ("cap_zombie", 4), ("cap_plant", 11), ("max_episode_steps", 0), ("obs_mode", 4),
                                         ("abi_version", 7), ("abi_version", 1), ("variant", 2), ("group_lanes", 2), ("group_lanes", 32),
                                         ("reserved", 1)])
def test_bad_configurations_get_no_state(lib, field, value):
    cfg = binding.default_config(**{field: value})
    assert binding.craftax_state_bytes(cfg, 64) == 0
    assert lib.craftax_state_init(ctypes.c_void_p(4096), ctypes.byref(cfg), 64, None) == -6


def test_full_game_accepts_only_its_own_options(lib):
    ok = binding.default_config(binding.VARIANT_CRAFTAX)
    assert binding.craftax_state_bytes(ok, 8) > 0
    assert binding.craftax_state_bytes(binding.default_config(binding.VARIANT_CRAFTAX, worldgen=binding.WORLDGEN_PERLIN), 8) > 0
    assert binding.craftax_state_bytes(binding.default_config(binding.VARIANT_CRAFTAX, reset_mode=binding.RESET_POOL), 8) > 0
    for field, value in [("worldgen", 2), ("reset_mode", 2), ("obs_mode", binding.OBS_SYM_U8_I8)]:
        assert binding.craftax_state_bytes(binding.default_config(binding.VARIANT_CRAFTAX, **{field: value}), 8) == 0
    # the state grows linearly and stays 256-byte aligned
    sizes = [binding.craftax_state_bytes(ok, n) for n in (1, 2, 64, 4096)]
    assert all(s % 256 == 0 for s in sizes) and sizes == sorted(sizes)


def test_bench_refuses_more_than_one_gpu():
    """One GPU is all this build measures: any other count ends with a message, before anything touches a GPU."""
    import os, subprocess, sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    res = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"], capture_output=True, text=True, timeout=120)
    assert res.returncode != 0 and "ONE GPU" in (res.stderr + res.stdout) and "{" not in res.stdout
