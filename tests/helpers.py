"""Shared test helpers: small CPU-checker set-ups and golden-file reading."""
import math
import os

import numpy as np

from oracle.ref import RefEnv
from paper_2602_01665_amd import inputs as I

GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")


def golden_table(name):
    """Reads `key value...` lines of a golden text file (lines with # are comments)."""
    out = {}
    with open(os.path.join(GOLDEN, name)) as f:
        for line in f:
            line = line.split("#", 1)[0].strip()
            if not line:
                continue
            parts = line.split()
            out[parts[0]] = [float(v) for v in parts[1:]]
    return out


def unit(name, team, x, y, theta=0.0, **kw):
    return dict(unit=name, team=team, x=x, y=y, theta=theta, **kw)


def make_ref(units, map_size=32.0, grid=0, terrain=None, zone_desc=None, max_zones=0,
             **param_override):
    sc = I.custom_scenario(units, map_size, grid, terrain, zone_desc)
    p = I.custom_params(len(units), map_size, grid, max_zones, **param_override)
    env = RefEnv(p, sc)
    env.reset()
    return env


def acts(*a):
    return np.array([a], np.uint8)


def other_slot(D_row, i, j):
    """The 16-float block of unit j inside agent i's observation row."""
    k = j if j < i else j - 1
    return D_row[16 + 16 * k: 16 + 16 * (k + 1)]


def vis_bit(vis, e, i, j):
    return int((int(vis[e, i, j >> 6]) >> (j & 63)) & 1)


class ShardedRef:
    """The checker on a large batch: the envs are dealt to `threads` sub-batches, each stepped
    by its own RefEnv on its own host thread (envs share nothing; the checker's calls release
    the interpreter lock).  `fields()` gives the whole batch's arrays again."""

    def __init__(self, w, params_of, scenario, threads=16):
        from concurrent.futures import ThreadPoolExecutor
        E = w.num_envs
        self.bounds = [E * k // threads for k in range(threads + 1)]
        # (every sub-batch knows its envs' indices in the whole batch: the random draws of the
        # heuristic policy are keyed by them)
        self.parts = [RefEnv(dict(params_of(self.bounds[k + 1] - self.bounds[k]),
                                  env_ids=np.arange(self.bounds[k], self.bounds[k + 1], dtype=np.int32)),
                             I.take_envs(scenario, slice(self.bounds[k], self.bounds[k + 1])))
                      for k in range(threads)]
        self.pool = ThreadPoolExecutor(threads)
        self.N, self.D = self.parts[0].N, self.parts[0].D
        # one observation array for the whole batch; every sub-batch writes its slice of it
        self.obs = np.zeros((E, self.N, self.D), np.float32)
        for k, r in enumerate(self.parts):
            r.obs = self.obs[self.bounds[k]:self.bounds[k + 1]]

    def _each(self, fn):
        list(self.pool.map(fn, range(len(self.parts))))

    def reset(self):
        self._each(lambda k: self.parts[k].reset())

    def tick(self, actions):
        def run(k):
            self.parts[k].step(actions[self.bounds[k]:self.bounds[k + 1]])
            self.parts[k].observe()
        self._each(run)

    def scripted_tick(self, policy, controlled, actions):
        """Decide-then-step: the controlled units' entries of `actions` ([E, N], in place) are
        chosen by the heuristic policy on the current state, then the tick runs.  Returns the
        memory flags as they stand after the decisions."""
        flags = [None] * len(self.parts)

        def run(k):
            lo, hi = self.bounds[k], self.bounds[k + 1]
            r = self.parts[k]
            part = np.ascontiguousarray(actions[lo:hi])
            r.heuristic_actions(policy, controlled[lo:hi], part)
            flags[k] = r.mem["mem_valid"].copy()
            actions[lo:hi] = part
            r.step(part)
            r.mem["mem_valid"][r.dones.astype(bool)] = 0
            r.observe()
        self._each(run)
        return np.concatenate(flags)

    def state(self, name):
        return np.concatenate([r.st[name] for r in self.parts])

    def output(self, name):
        return np.concatenate([getattr(r, name) for r in self.parts])

    def global_state(self):
        return np.concatenate([r.global_state() for r in self.parts])
