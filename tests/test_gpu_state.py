"""GPU tests of the state object itself: checkpoint / resume through a byte copy and
craftax_state_attach, calls before the first reset, imports of out-of-range dumps, and the one
way an edited world can end an episode before its spare world exists.  All against the CPU oracle,
tolerance 0."""
import ctypes

import numpy as np
import pytest

from oracle import pyoracle as po
from paper_2402_16801_amd import synth

pytestmark = pytest.mark.gpu

LAVA, GRASS = 14, 2


@pytest.fixture(scope="module")
def cx():
    import torch
    from paper_2402_16801_amd import binding
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    binding.load()
    return binding


def _pair(cx, variant, n, **kw):
    """A GPU simulator and an oracle of the same configuration."""
    if variant == "classic":
        gcfg = cx.default_config(obs_mode=cx.OBS_SYM_U8_F32, **kw)
        return cx.Craftax(n, gcfg), po.Oracle(n, po.default_config(**kw), po.OBS_SYM_U8_F32), 17
    gcfg = cx.default_config(cx.VARIANT_CRAFTAX, **kw)
    ocfg = po.full_default_config(**kw)
    return cx.Craftax(n, gcfg), po.FullOracle(n, ocfg, po.FULL_OBS_U8_F32), 43


def _step_both(sim, orc, a, what):
    import torch
    obs, rew, done = sim.step(torch.as_tensor(a, device=sim.device))
    oobs, orew, odone = orc.step(a)
    assert np.array_equal(done.cpu().numpy(), odone), f"done, {what}"
    assert np.array_equal(rew.cpu().numpy().view(np.uint32), orew.view(np.uint32)), f"reward, {what}"
    assert np.array_equal(obs.cpu().numpy(), oobs), f"observation, {what}"
    return odone


@pytest.mark.parametrize("variant,n,cap", [("classic", 300, 37), ("classic", 4200, 23), ("craftax", 70, 29)])
def test_checkpoint_by_byte_copy_and_attach(cx, variant, n, cap):
    """T steps, a byte copy of the state blob into a second allocation (once through host memory),
    attach, T more steps on the copy: bit-exact with the oracle's uninterrupted 2T steps and with
    the original continuing on its own.  The episode cap makes many episodes end right after the
    restore, the first of them on the first step after it."""
    import torch
    sim, orc, n_actions = _pair(cx, variant, n, max_episode_steps=cap)
    seeds = synth.seeds_for(n, 77)
    sim.reset(seeds)
    orc.reset(seeds)
    T = 2 * cap - 1                       # the step after the restore ends the second episode of every survivor
    for s in range(T):
        _step_both(sim, orc, synth.actions(np.arange(n), s, "skewed", 5, n_actions), f"step {s}")
    torch.cuda.synchronize()
    # checkpoint: the blob goes to the host and comes back at another address
    saved = sim.state.cpu()
    copy = cx.Craftax.__new__(cx.Craftax)
    copy.__dict__.update(sim.__dict__)
    copy.state = torch.empty_like(sim.state)
    copy.state.copy_(saved)
    copy.obs, copy.reward, copy.done = torch.zeros_like(sim.obs), torch.zeros_like(sim.reward), torch.zeros_like(sim.done)
    assert copy.state.data_ptr() != sim.state.data_ptr()
    lib = cx.load()
    assert lib.craftax_step(copy.state.data_ptr(), 0, 0, 0, 0, n, None) == -4, "a blob is unusable before it is attached"
    cx.craftax_state_attach(copy.state, copy.cfg, n, copy.stream)
    assert copy.export_envs().tobytes() == orc.envs.tobytes()
    ended = 0
    for s in range(T, 2 * T):
        a = synth.actions(np.arange(n), s, "skewed", 5, n_actions)
        d = _step_both(copy, orc, a, f"restored, step {s}")
        ended += int(d.sum())
        if s == T:
            assert d.sum() > n // 2, "most episodes were to end on the first step after the restore"
        sim.step(torch.as_tensor(a, device=sim.device))            # the original goes on as well
        assert torch.equal(sim.obs, copy.obs) and torch.equal(sim.reward, copy.reward) and torch.equal(sim.done, copy.done)
    assert ended > n
    assert copy.export_envs().tobytes() == orc.envs.tobytes() == sim.export_envs().tobytes()
    # a second restore of the same checkpoint replays the same future
    again = torch.empty_like(sim.state)
    again.copy_(saved)
    third = cx.Craftax.__new__(cx.Craftax)
    third.__dict__.update(copy.__dict__)
    third.state = again
    cx.craftax_state_attach(again, third.cfg, n, third.stream)
    ref = type(orc)(n, orc.cfg, orc.obs_mode)
    ref.reset(seeds)
    for s in range(T + 3):
        a = synth.actions(np.arange(n), s, "skewed", 5, n_actions)
        if s < T:
            ref.step(a, render=False)
        else:
            _step_both(third, ref, a, f"second restore, step {s}")
    cx.craftax_state_release(again)
    copy.close()
    sim.close()


def test_attach_refuses_what_is_not_its_blob(cx):
    import torch
    n = 40
    cfg = cx.default_config()
    sim = cx.Craftax(n, cfg)
    sim.reset(synth.seeds_for(n))
    lib = cx.load()
    blob = torch.empty_like(sim.state)
    blob.copy_(sim.state)
    junk = torch.zeros(4096, dtype=torch.uint8, device=sim.device)
    assert lib.craftax_state_attach(junk.data_ptr(), ctypes.byref(cfg), n, None) == -4          # no magic
    assert lib.craftax_state_attach(blob.data_ptr(), ctypes.byref(cfg), n + 1, None) == -3       # another n
    other = cx.default_config(day_length=200)
    assert lib.craftax_state_attach(blob.data_ptr(), ctypes.byref(other), n, None) == -6         # another configuration
    pool = cx.default_config(reset_mode=cx.RESET_POOL)
    assert lib.craftax_state_attach(blob.data_ptr(), ctypes.byref(pool), n, None) == -6
    full = cx.default_config(cx.VARIANT_CRAFTAX)
    assert lib.craftax_state_attach(blob.data_ptr(), ctypes.byref(full), n, None) == -4          # a Classic blob is no Craftax blob
    assert lib.craftax_state_attach(blob.data_ptr() + 16, ctypes.byref(cfg), n, None) == -2
    assert lib.craftax_state_attach(None, ctypes.byref(cfg), n, None) == -1
    # group_lanes is tuning only: a blob may be attached with another width
    wide = cx.default_config(group_lanes=16)
    assert lib.craftax_state_attach(blob.data_ptr(), ctypes.byref(wide), n, None) == 0
    assert lib.craftax_state_release(blob.data_ptr()) == 0
    sim.close()


@pytest.mark.parametrize("variant", ["classic", "craftax"])
def test_calls_before_the_first_reset_are_refused(cx, variant):
    """A state that was initialised but never reset holds no records, maps or tags: every call that
    would read them returns CRAFTAX_E_STATE and launches nothing."""
    import torch
    n = 8
    sim, _, _ = _pair(cx, variant, n)
    lib = cx.load()
    st, buf = sim.state.data_ptr(), sim.obs.data_ptr()
    a = torch.zeros((4, n), dtype=torch.int32, device=sim.device)
    assert lib.craftax_step(st, a.data_ptr(), buf, sim.reward.data_ptr(), sim.done.data_ptr(), n, None) == -4
    assert b"craftax_reset" in lib.craftax_last_error()
    assert lib.craftax_rollout(st, a.data_ptr(), 4, buf, sim.reward.data_ptr(), sim.done.data_ptr(), n, None) == -4
    assert lib.craftax_observe(st, buf, n, None) == -4
    dumps = torch.zeros((n, cx.craftax_env_dump_bytes_for(sim.cfg)), dtype=torch.uint8, device=sim.device)
    assert lib.craftax_export_envs(st, 0, n, dumps.data_ptr(), None) == -4
    assert lib.craftax_import_envs(st, 0, n, dumps.data_ptr(), None) == -4
    assert lib.craftax_mutate_swap(st, 0, n, 1, 0, 0, None, None) == -4
    sim.reset(synth.seeds_for(n))
    assert lib.craftax_observe(st, buf, n, None) == 0
    assert lib.craftax_export_envs(st, 0, n, dumps.data_ptr(), None) == 0
    torch.cuda.synchronize()
    sim.close()


def test_import_brings_out_of_range_values_into_range(cx):
    """Edited dumps with block ids, coordinates and counts outside their tables: the import maps
    them into range (checked through export, nothing is rendered from the raw values), and the
    simulator then runs on as the oracle does from the same, cleaned state."""
    n = 24
    sim, orc, _ = _pair(cx, "classic", n)
    seeds = synth.seeds_for(n, 5)
    sim.reset(seeds); orc.reset(seeds)
    bad = orc.envs.copy()
    bad["map"][:, 10, 10] = 17
    bad["map"][:, 11, 10] = 200
    bad["map"][:, 30, 33] = 0            # inside the first view
    bad["map"][:, 31, 34] = 255
    bad["px"][::2] = 64 + 32             # taken modulo 64
    bad["dir"][1::2] = 8 + 4
    bad["inv"][:, 0] = 16 + 3
    bad["vit"][:, 1] = 16 + 5
    bad["cnt"][:, 0] = 300
    bad["mob"][:, 2] = (3, 64 + 20, 64 + 21, 8 + 2, 16 + 4, 16 + 1, (0, 0))
    sim.import_envs(bad)
    want = orc.envs.copy()
    for y, x in ((10, 10), (11, 10), (30, 33), (31, 34)):
        want["map"][:, y, x] = 1
    want["dir"][1::2] = 4
    want["inv"][:, 0] = 3
    want["vit"][:, 1] = 5
    want["cnt"][:, 0] = 127
    want["mob"][:, 2] = (1, 20, 21, 2, 4, 1, (0, 0))
    got = sim.export_envs().view(po.ENV_DTYPE).reshape(-1)
    for name in po.ENV_DTYPE.names:
        assert np.array_equal(got[name], want[name]), name
    orc.envs[:] = want
    cx.craftax_observe(sim.state, sim.obs, n, sim.stream)
    assert np.array_equal(sim.obs.cpu().numpy(), orc.observe())
    for s in range(30):
        _step_both(sim, orc, synth.actions(np.arange(n), s, "uniform", 9), f"step {s}")
    sim.close()


def test_full_import_brings_out_of_range_values_into_range(cx):
    n = 12
    sim, orc, _ = _pair(cx, "craftax", n)
    seeds = synth.seeds_for(n, 6)
    sim.reset(seeds); orc.reset(seeds)
    bad = orc.envs.copy()
    bad["block"][:, 0, 5, 5] = 37
    bad["block"][:, 3, 7, 9] = 0
    bad["block"][:, 0, 23, 25] = 250     # inside the first view
    bad["item"][:, 0, 6, 6] = 5
    bad["item"][:, 0, 7, 7] = 9          # low three bits 1 would read as a torch
    bad["light"][:, 0, 8, 8] = 31
    bad["inv"][:, 2] = 200
    bad["potion"][:, 1] = 150
    bad["vit"][:, 4] = 90
    bad["mob"][:, 0, 1] = (1, 20, 20, 0, 3, 0, 25, 0)
    sim.import_envs(bad)
    want = orc.envs.copy()
    want["block"][:, 0, 5, 5] = 1
    want["block"][:, 3, 7, 9] = 1
    want["block"][:, 0, 23, 25] = 1
    want["light"][:, 0, 8, 8] = 20
    want["inv"][:, 2] = 99
    want["potion"][:, 1] = 99
    want["vit"][:, 4] = 31
    want["mob"][:, 0, 1] = (1, 20, 20, 0, 3, 0, 18, 0)
    got = sim.export_envs().view(po.FULL_ENV_DTYPE).reshape(-1)
    for name in po.FULL_ENV_DTYPE.names:
        assert np.array_equal(got[name], want[name]), name
    sim.close()


@pytest.mark.parametrize("variant,n,lanes", [("classic", 6000, 0), ("classic", 6000, 4), ("craftax", 3000, 0)])
def test_death_on_the_first_step_after_an_auto_reset_and_a_swap(cx, variant, n, lanes):
    """Every environment resets in the same step (equal caps); right after that step the swap
    mutation runs until some worlds have lava next to the start; the next action walks into it.
    Those episodes end on their first step, before the step kernel could trust their spare world:
    the library has to serve them at once, as the oracle does."""
    import torch
    cap = 5
    kw = {"max_episode_steps": cap}
    sim, orc, n_actions = _pair(cx, variant, n, **kw)
    if variant == "classic" and lanes:
        sim.close()
        gcfg = cx.default_config(obs_mode=cx.OBS_SYM_U8_F32, group_lanes=lanes, **kw)
        sim = cx.Craftax(n, gcfg)
    seeds = synth.seeds_for(n, 900)
    sim.reset(seeds); orc.reset(seeds)
    for s in range(cap):                                  # step cap-1 ends every episode: all worlds are fresh now
        d = _step_both(sim, orc, synth.actions(np.arange(n), s, "uniform", 3, n_actions), f"step {s}")
    assert d.all()
    centre = 32 if variant == "classic" else 24
    grid = (lambda e: e["map"]) if variant == "classic" else (lambda e: e["block"][:, 0])
    rounds = 0
    while True:
        g_tries = sim.mutate_swap(11, rounds, False)
        o_tries = orc.mutate_swap(11, rounds, False)
        assert np.array_equal(g_tries, o_tries)
        rounds += 1
        m = grid(orc.envs)
        near = np.stack([m[:, centre, centre - 1], m[:, centre, centre + 1], m[:, centre - 1, centre], m[:, centre + 1, centre]], 1) == LAVA
        if near.any(axis=1).sum() >= 3 or rounds >= 400:
            break
    doomed = near.any(axis=1)
    assert doomed.sum() >= 1, "no swap put lava next to a start: raise n or the number of rounds"
    a = np.where(doomed, 1 + near.argmax(axis=1), 0).astype(np.int32)     # LEFT, RIGHT, UP, DOWN into the lava; others wait
    d = _step_both(sim, orc, a, "the step into the lava")
    assert np.array_equal(d.astype(bool), doomed), "exactly the doomed episodes end on their first step"
    assert sim.export_envs().tobytes() == orc.envs.tobytes()
    for s in range(cap, 4 * cap):
        _step_both(sim, orc, synth.actions(np.arange(n), s, "uniform", 3, n_actions), f"step {s}")
    assert sim.export_envs().tobytes() == orc.envs.tobytes()
    sim.close()


def _bit_counts(words, n_ach):
    """How many rows of the achievement words (n x W uint32) have bit i set, for i < n_ach, in 96 slots."""
    w = words.reshape(len(words), -1).astype(np.uint64)
    out = np.zeros(96, np.int64)
    for i in range(n_ach):
        out[i] = int(((w[:, i // 32] >> np.uint64(i % 32)) & np.uint64(1)).sum())
    return out


def _unlocked_this_step(orc, before, actions, odone, n_ach):
    """Achievement bits that the step just taken by `orc` switched on, counted per achievement.  For an
    environment whose episode went on they are the difference of its achievement words; one whose
    episode ended has been reset already, so its last step is taken again from the copy made before
    the step, by the oracle's rules alone (no reset)."""
    after = orc.envs["ach"].reshape(orc.n, -1)
    prev = before["ach"].reshape(orc.n, -1)
    new = np.where(odone[:, None] == 1, 0, after & ~prev).astype(np.uint32)
    ended = np.nonzero(odone)[0]
    if len(ended):
        shadow = type(orc)(len(ended), orc.cfg, orc.obs_mode)
        shadow.envs[:] = before[ended]
        for j, i in enumerate(ended):
            shadow.step_rules_one(j, int(actions[i]))
        new[ended] = shadow.envs["ach"].reshape(len(ended), -1) & ~prev[ended]
    return _bit_counts(new, n_ach)


@pytest.mark.parametrize("variant,n,lanes", [("classic", 1000, 0), ("classic", 257, 4), ("classic", 70, 8), ("craftax", 300, 0), ("craftax", 70, 16)])
def test_metrics_match_the_oracle(cx, variant, n, lanes):
    """craftax_stats (episodes finished, steps into the running episodes, achievements held by the
    running episodes, unlock events since the reset) against the same sums over the oracle's
    environments, at several points of a run of single steps and rollouts; then the success rates
    over the finished episodes that follow from them, and a reset that clears the counters."""
    import torch
    sim, orc, n_actions = _pair(cx, variant, n, max_episode_steps=60)
    if lanes:                                   # another shape of the step kernel
        sim.close()
        cfg = cx.default_config(cx.VARIANT_CRAFTAX if variant == "craftax" else cx.VARIANT_CLASSIC, obs_mode=cx.OBS_SYM_U8_F32,
                                max_episode_steps=60, group_lanes=lanes)
        sim = cx.Craftax(n, cfg)
    seeds = synth.seeds_for(n, 21)
    sim.reset(seeds); orc.reset(seeds)
    n_ach = 22 if variant == "classic" else 67
    seen = np.zeros(96, np.int64)
    unlocks = np.zeros(96, np.int64)
    finished_with = np.zeros(96, np.int64)      # finished episodes that had unlocked achievement i
    s = 0
    while s < 170:
        if s in (40, 100):                      # a rollout of 25 steps in between: the same counters
            T = 25
            acts = np.stack([synth.actions(np.arange(n), s + k, "skewed", 2, n_actions) for k in range(T)])
            rew = torch.empty((T, n), dtype=torch.float32, device=sim.device)
            dn = torch.empty((T, n), dtype=torch.uint8, device=sim.device)
            cx.craftax_rollout(sim.state, torch.as_tensor(acts, device=sim.device), T, None, rew, dn, n, sim.stream)
            for k in range(T):
                before = orc.envs.copy()
                _, _, odone = orc.step(acts[k], render=False)
                step_new = _unlocked_this_step(orc, before, acts[k], odone, n_ach)
                unlocks += step_new
                assert np.array_equal(dn[k].cpu().numpy(), odone)
            s += T
        else:
            a = synth.actions(np.arange(n), s, "skewed", 2, n_actions)
            before = orc.envs.copy()
            odone = _step_both(sim, orc, a, f"step {s}")
            unlocks += _unlocked_this_step(orc, before, a, odone, n_ach)
            s += 1
        if s % 30 == 0 or s < 3:
            got = sim.stats()
            e = orc.envs
            bits = _bit_counts(e["ach"], n_ach)
            assert (int(got["episodes"]), int(got["steps"]), int(got["n"])) == (int(e["episode"].astype(np.int64).sum()), int(e["t"].astype(np.int64).sum()), n)
            assert np.array_equal(got["achievements"].astype(np.int64), bits), f"running episodes, step {s}"
            assert np.array_equal(got["unlocks"].astype(np.int64), unlocks), f"unlock events, step {s}"
            seen = np.maximum(seen, bits)
    assert int(got["episodes"]) >= 2 * n and (seen > 0).sum() >= 3, "the run was to finish episodes and unlock achievements"
    # success rate over the finished episodes: every unlock belongs to a finished or to a running episode
    finished_with = got["unlocks"].astype(np.int64) - got["achievements"].astype(np.int64)
    assert (finished_with >= 0).all() and (finished_with <= int(got["episodes"])).all() and finished_with.sum() > 0
    sim.reset(seeds)
    again = sim.stats()
    assert int(again["episodes"]) == 0 and not again["unlocks"].any() and not again["achievements"].any()
    sim.close()
