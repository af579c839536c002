"""Whole-population parity at the benchmark sizes: every environment of the GPU batch is followed
by the CPU oracle (slices of environments on the host's cores), not a sample of them.

Compared, all with tolerance 0:
  * reward (as bit patterns) and done of every environment after every step;
  * the observation of every environment at the end of every chunk of steps, and after every
    single step for a sample of environments taken at a stride coprime to every block shape of
    the kernels (so the sample visits every lane position);
  * the whole exported state of every environment at the steps listed in `state_at`.
The oracle's inputs come from the seeded generators of `synth` only; the same host-made action
blocks are uploaded to the GPU.
"""
import numpy as np

from oracle import pyoracle as po
from paper_2402_16801_amd import synth


def coprime_sample(n, stride):
    ids = np.arange(stride // 3, n, stride)
    ids = np.unique(np.concatenate([ids, [0, n - 1]]))
    assert len(set((ids % 64).tolist())) == min(64, n), "the sample must visit every position inside a block"
    return ids


def first_difference(got, want, dtype, what):
    g, w = got.view(dtype).reshape(-1), want.view(dtype).reshape(-1)
    for name in dtype.names:
        if not np.array_equal(g[name], w[name]):
            bad = [i for i in range(len(g)) if not np.array_equal(g[name][i], w[name][i])]
            raise AssertionError(f"state field {name!r} differs at {what}, envs {bad[:8]} ({len(bad)} in all)")
    raise AssertionError(f"state bytes differ at {what}")


def run_population(cx, sim, orc, T, kind, n_actions, chunk, stride, state_at, dump_dtype, action_seed=0, seed_base=0,
                   progress=True):
    """sim: binding.Craftax with n environments; orc: Oracle / FullOracle with the same n, same
    configuration and observation layout.  Returns the number of episodes that finished."""
    import torch

    n = sim.n
    assert orc.n == n
    sample = coprime_sample(n, stride)
    idx_dev = torch.as_tensor(sample, device=sim.device, dtype=torch.long)
    seeds = synth.seeds_for(n, seed_base)
    obs = sim.reset(seeds)
    orc.reset_many(seeds)
    assert np.array_equal(obs.cpu().numpy(), orc.observe()), "reset observation"
    ostride = sim.obs_bytes
    finished = 0
    for s0 in range(0, T, chunk):
        K = min(chunk, T - s0)
        acts = synth.action_block(n, K, kind, action_seed, s0, n_actions)
        acts_dev = torch.as_tensor(acts, device=sim.device)
        rew_dev = torch.empty((K, n), dtype=torch.float32, device=sim.device)
        done_dev = torch.empty((K, n), dtype=torch.uint8, device=sim.device)
        sobs_dev = torch.empty((K, len(sample), ostride), dtype=torch.uint8, device=sim.device)
        cuts = [s for s in state_at if s0 < s <= s0 + K]          # a state comparison ends a sub-chunk
        k0 = 0
        for k1 in sorted(set(cuts + [s0 + K])):
            k1 -= s0
            for k in range(k0, k1):
                sim.step(acts_dev[k])
                rew_dev[k].copy_(sim.reward)
                done_dev[k].copy_(sim.done)
                torch.index_select(sim.obs, 0, idx_dev, out=sobs_dev[k])
            sobs = np.zeros((k1 - k0, len(sample), ostride), np.uint8)
            orew, odone = orc.step_many(acts[k0:k1], sample=sample, sample_obs=sobs)
            g_rew, g_done = rew_dev[k0:k1].cpu().numpy(), done_dev[k0:k1].cpu().numpy()
            if not np.array_equal(g_done, odone):
                k, i = np.argwhere(g_done != odone)[0]
                raise AssertionError(f"done differs at step {s0 + k0 + k}, env {i}")
            if not np.array_equal(g_rew.view(np.uint32), orew.view(np.uint32)):
                k, i = np.argwhere(g_rew.view(np.uint32) != orew.view(np.uint32))[0]
                raise AssertionError(f"reward differs at step {s0 + k0 + k}, env {i}: {g_rew[k, i]} vs {orew[k, i]}")
            g_sobs = sobs_dev[k0:k1].cpu().numpy()
            if not np.array_equal(g_sobs, sobs):
                k, j = np.argwhere((g_sobs != sobs).any(axis=2))[0]
                raise AssertionError(f"observation differs at step {s0 + k0 + k}, env {sample[j]}")
            g_obs = sim.obs.cpu().numpy()
            if not np.array_equal(g_obs, orc.obs):
                bad = np.nonzero((g_obs != orc.obs).any(axis=1))[0]
                raise AssertionError(f"observation differs after step {s0 + k1 - 1}, envs {bad[:8]} ({len(bad)} in all)")
            finished += int(odone.sum())
            if s0 + k1 in state_at:
                dumps = sim.export_envs()
                if not np.array_equal(dumps.reshape(-1), orc.envs.view(np.uint8).reshape(-1)):
                    first_difference(dumps, orc.envs, dump_dtype, f"step {s0 + k1}")
            k0 = k1
        if progress:
            print(f"  step {s0 + K}/{T} ok: all {n} environments, episodes finished {finished}", flush=True)
    return finished
