"""The debug build of the library (the same sources with a bounds check on every index the kernels
form into a map, an LDS window or a staging area) run through busy scenarios of both variants: it
must report no index out of range, and it must compute what the oracle computes.  A wrong index
would be counted and replaced, never dereferenced, so nothing here can fault."""
import numpy as np
import pytest

from oracle import pyoracle as po
from paper_2402_16801_amd import synth

pytestmark = pytest.mark.gpu


@pytest.fixture()
def dbg():
    import torch
    from paper_2402_16801_amd import binding
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    release = binding.LIB_PATH
    binding.use_library(binding.DEBUG_LIB_PATH)
    try:
        built_in, _ = binding.craftax_debug_bounds()
        assert built_in, "libcraftax_hip_debug.so was built without the checks"
        yield binding
    finally:
        binding.use_library(release)


def _clean(cx, what):
    built_in, report = cx.craftax_debug_bounds()
    assert built_in and report[0] == 0, f"{what}: {report[0]} indices out of range, first at source line {report[1]}: index {report[2]}, limit {report[3]}"


def test_the_check_itself_reports_a_planted_index(dbg):
    assert dbg.load().craftax_debug_bounds_selftest() == 1, dbg.load().craftax_last_error()
    _clean(dbg, "after the self-test")


def test_release_library_has_no_checks():
    from paper_2402_16801_amd import binding
    built_in, report = binding.craftax_debug_bounds()
    assert not built_in and report == [0, 0, 0, 0]
    assert binding.load().craftax_debug_bounds_selftest() == 0


@pytest.mark.parametrize("lanes", [4, 8, 16])
def test_classic_runs_without_an_index_out_of_range(dbg, lanes):
    import torch
    cx = dbg
    n, cap = 300, 45
    for obs_mode, omode in ((cx.OBS_SYM_U8_F32, po.OBS_SYM_U8_F32), (cx.OBS_SYM_F32, po.OBS_SYM_F32), (cx.OBS_PIXELS_F32, po.OBS_PIXELS_F32)):
        sim = cx.Craftax(n, cx.default_config(obs_mode=obs_mode, max_episode_steps=cap, group_lanes=lanes))
        orc = po.Oracle(n, po.default_config(max_episode_steps=cap), omode)
        seeds = synth.seeds_for(n, 31)
        sim.reset(seeds); orc.reset(seeds)
        # players at the map corners and edges look beyond the map in every renderer and rule
        e = orc.envs
        e["px"][:8] = [0, 63, 0, 63, 0, 63, 31, 32]
        e["py"][:8] = [0, 0, 63, 63, 31, 32, 0, 63]
        for i in range(8):
            e["map"][i, e["py"][i], e["px"][i]] = 2
        sim.import_envs(e)
        for s in range(100 if obs_mode != cx.OBS_PIXELS_F32 else 30):
            a = synth.actions(np.arange(n), s, "skewed", 4)
            obs, rew, done = sim.step(torch.as_tensor(a, device=sim.device))
            oobs, orew, odone = orc.step(a)
            assert np.array_equal(done.cpu().numpy(), odone) and np.array_equal(obs.cpu().numpy(), oobs), (obs_mode, s)
        if obs_mode == cx.OBS_SYM_U8_F32:
            sim.mutate_swap(5, 0, False); orc.mutate_swap(5, 0, False)
            acts = torch.as_tensor(synth.action_block(n, 60, "uniform", 8, 200), device=sim.device)
            rew = torch.empty((60, n), dtype=torch.float32, device=sim.device)
            done = torch.empty((60, n), dtype=torch.uint8, device=sim.device)
            cx.craftax_rollout(sim.state, acts, 60, sim.obs, rew, done, n, sim.stream)
            for s in range(60):
                orc.step(acts[s].cpu().numpy(), render=(s == 59))
            assert np.array_equal(sim.obs.cpu().numpy(), orc.obs)
            assert int(sim.stats()["n"]) == n
        assert sim.export_envs().tobytes() == orc.envs.tobytes()
        sim.close()
        _clean(cx, f"Classic, {lanes} lanes, observation layout {obs_mode}")


def test_classic_perlin_pool_and_noise_without_an_index_out_of_range(dbg):
    import torch
    cx = dbg
    n = 200
    sim = cx.Craftax(n, cx.default_config(worldgen=cx.WORLDGEN_PERLIN, reset_mode=cx.RESET_POOL, max_episode_steps=20))
    orc = po.Oracle(n, po.default_config(worldgen=po.WORLDGEN_PERLIN, reset_mode=po.RESET_POOL, max_episode_steps=20))
    seeds = synth.seeds_for(n, 2)
    sim.reset(seeds); orc.reset(seeds)
    theta = torch.zeros((n, cx.THETA_LEN), dtype=torch.int16, device=sim.device)
    sim.mutate_noise(theta, 9, 0, 300)
    th = np.zeros((n, po.THETA_LEN), np.uint16)
    orc.mutate_noise(th, 9, 0, 300)
    for s in range(70):
        a = synth.actions(np.arange(n), s, "uniform", 6)
        obs, _, done = sim.step(torch.as_tensor(a, device=sim.device))
        oobs, _, odone = orc.step(a)
        assert np.array_equal(done.cpu().numpy(), odone) and np.array_equal(obs.cpu().numpy(), oobs), s
    sim.close()
    _clean(cx, "Classic, Perlin worlds, pool resets, noise mutation")


@pytest.mark.parametrize("lanes", [64, 16])
def test_full_game_runs_without_an_index_out_of_range(dbg, lanes):
    import torch
    from test_gpu_full_parity import rich_scene
    cx = dbg
    n, cap = 72, 60
    for obs_mode, omode in ((cx.OBS_SYM_U8_F32, po.FULL_OBS_U8_F32), (cx.OBS_PIXELS_F32, po.FULL_OBS_PIXELS_F32)):
        sim = cx.Craftax(n, cx.default_config(cx.VARIANT_CRAFTAX, obs_mode=obs_mode, max_episode_steps=cap, group_lanes=lanes))
        orc = po.FullOracle(n, po.full_default_config(max_episode_steps=cap), omode)
        seeds = synth.seeds_for(n, 17)
        sim.reset(seeds); orc.reset(seeds)
        rich_scene(orc.envs)                          # every floor, gear, spells, chests, the boss
        # some players in map corners as well
        for i, (x, y) in enumerate(((0, 0), (47, 0), (0, 47), (47, 47))):
            e = orc.envs[9 + i]
            f = int(e["floor"])
            e["px"], e["py"] = x, y
            e["block"][f, y, x] = 7
            e["item"][f, y, x] = 0
        sim.import_envs(orc.envs)
        steps = 150 if obs_mode == cx.OBS_SYM_U8_F32 else 25
        for s in range(steps):
            a = synth.actions(np.arange(n), s, "uniform", 12, 43)
            obs, rew, done = sim.step(torch.as_tensor(a, device=sim.device))
            oobs, orew, odone = orc.step(a)
            assert np.array_equal(done.cpu().numpy(), odone) and np.array_equal(obs.cpu().numpy(), oobs), (obs_mode, s)
        if obs_mode == cx.OBS_SYM_U8_F32:
            acts = torch.as_tensor(synth.action_block(n, 80, "uniform", 13, 300, 43), device=sim.device)
            rew = torch.empty((80, n), dtype=torch.float32, device=sim.device)
            done = torch.empty((80, n), dtype=torch.uint8, device=sim.device)
            cx.craftax_rollout(sim.state, acts, 80, sim.obs, rew, done, n, sim.stream)
            for s in range(80):
                orc.step(acts[s].cpu().numpy(), render=(s == 79))
            assert np.array_equal(sim.obs.cpu().numpy(), orc.obs)
            sim.mutate_swap(3, 1, True); orc.mutate_swap(3, 1, True)
        assert sim.export_envs().tobytes() == orc.envs.tobytes()
        sim.close()
        _clean(cx, f"Craftax, {lanes} lanes, observation layout {obs_mode}")
