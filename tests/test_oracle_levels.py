"""Pins of the CPU checker's level bank: the configuration of an env is applied when an
episode starts (Sec. 4.1; App. A "Environment Parameters"), here as a row of a bank of
levels that is re-drawn at every reset and auto-reset."""
import math

import numpy as np

from oracle import ref
from paper_2602_01665_amd import inputs as I
from tests.helpers import unit, vis_bit


def bank(*scenarios):
    """Stacks single-row scenarios into a bank of levels."""
    out = {}
    for k in scenarios[0]:
        vals = [s[k] for s in scenarios]
        out[k] = None if vals[0] is None else np.concatenate(vals, axis=0)
    return out


def two_level_env(E=1, **over):
    """Level 0: farmers far apart.  Level 1: a mammoth facing an archer at spear distance."""
    l0 = I.custom_scenario([unit("farmer", 0, 4, 4, 0.0), unit("farmer", 1, 28, 28, math.pi)])
    l1 = I.custom_scenario([unit("mammoth", 0, 10, 16, 0.0), unit("archer", 1, 12, 16, math.pi)])
    p = I.custom_params(2, num_envs=E, num_levels=2, level_seed=9, **over)
    env = ref.RefEnv(p, bank(l0, l1))
    return env


def test_reset_takes_the_queued_level_and_refills_the_queue():
    env = two_level_env(E=3)
    env.st["next_level"][:] = [1, 0, 1]
    env.reset()
    assert env.st["level"].tolist() == [1, 0, 1]
    assert env.st["hp"][:, 0].tolist() == [685.0, 60.0, 685.0]        # mammoth / farmer / mammoth
    assert env.st["x"][:, 1].tolist() == [12.0, 28.0, 12.0]
    h = ref.lib().tabx_ref_hash
    assert env.st["next_level"].tolist() == [h(9, e, 0, 0, 3) % 2 for e in range(3)]
    assert env.st["level_draws"].tolist() == [1, 1, 1]
    # a masked reset advances only the chosen envs
    queued = env.st["next_level"].copy()
    env.reset(np.array([0, 1, 0], np.uint8))
    assert env.st["level"].tolist() == [1, int(queued[1]), 1]
    assert env.st["level_draws"].tolist() == [1, 2, 1]
    assert env.st["next_level"][1] == h(9, 1, 0, 1, 3) % 2


def test_queued_level_is_folded_into_range():
    env = two_level_env(E=2)
    env.st["next_level"][:] = [-1, 5]          # as unsigned: 4294967295 % 2 = 1, 5 % 2 = 1
    env.reset()
    assert env.st["level"].tolist() == [1, 1]


def test_auto_reset_switches_level_and_everything_follows_it():
    # level 1: the archer (40 health) dies to two mammoth hits?  no: make it quick with max_steps
    env = two_level_env(E=1, max_steps=3)
    env.st["next_level"][:] = [0]
    env.reset()
    assert env.st["level"][0] == 0
    env.st["next_level"][:] = [1]              # the caller's choice for the next episode
    idle = np.zeros((1, 2), np.uint8)
    for _ in range(3):
        env.step(idle)
    assert env.dones[0] == 1 and env.st["level"][0] == 1
    assert env.st["hp"][0].tolist() == [685.0, 40.0] and env.st["t"][0] == 0
    obs, vis, amask = env.observe()
    # the observation carries the new level's specs: own block = hp, ratio, x, y, theta, range, dmg
    assert obs[0, 0, :7].tolist() == [685.0, 1.0, 10.0, 16.0, 0.0, 3.0, 20.0]
    assert vis_bit(vis, 0, 0, 1) == 1 and vis_bit(vis, 0, 1, 0) == 1
    # and combat uses them: the mammoth (damage 20) strikes the archer in front of it
    env.step(np.array([[I.ACT_ATTACK, I.ACT_NOOP]], np.uint8))
    assert env.st["hp"][0, 1] == 20.0
    assert env.st["cd"][0, 0] == np.float32(6.5)


def test_teams_and_enabled_flags_come_from_the_level():
    # level 0: 1 ally vs 2 adversaries.  level 1: 2 allies vs 1 adversary, one unit disabled
    l0 = I.custom_scenario([unit("farmer", 0, 4, 4), unit("farmer", 1, 20, 20), unit("farmer", 1, 24, 24)])
    l1 = I.custom_scenario([unit("farmer", 0, 4, 4), unit("farmer", 0, 8, 8, enabled=0),
                            unit("farmer", 1, 24, 24)])
    p = I.custom_params(3, num_envs=1, num_levels=2, max_steps=2)
    env = ref.RefEnv(p, bank(l0, l1))
    env.st["next_level"][:] = [0]
    env.reset()
    env.st["next_level"][:] = [1]
    hp = env.st["hp"].copy()
    hp[0, 1] = 30.0                            # adversaries' mean ratio 0.75 under level 0
    env.set_state(hp=hp)
    idle = np.zeros((1, 3), np.uint8)
    env.step(idle)
    assert env.st["phi_prev"][0] == np.float32(1.0 - 0.75)
    env.step(idle)                             # truncation: reset into level 1
    assert env.st["level"][0] == 1
    assert env.st["alive"][0].tolist() == [1, 0, 1]
    assert env.st["phi_prev"][0] == 0.0        # 1/1 allies (the disabled one does not count) - 1/1
    hp = env.st["hp"].copy()
    hp[0, 2] = 15.0
    env.set_state(hp=hp)
    rew, _ = env.step(idle)
    assert rew[0].tolist() == [0.75, 0.0, -0.75]       # disabled unit: no reward


def test_team_of_an_enabled_unit_differs_between_levels():
    # the same two farmers, sides swapped in level 1
    l0 = I.custom_scenario([unit("farmer", 0, 4, 4), unit("farmer", 1, 24, 24)])
    l1 = I.custom_scenario([unit("farmer", 1, 4, 4), unit("farmer", 0, 24, 24)])
    p = I.custom_params(2, num_envs=2, num_levels=2)
    env = ref.RefEnv(p, bank(l0, l1))
    env.st["next_level"][:] = [0, 1]
    env.reset()
    hp = env.st["hp"].copy()
    hp[:, 0] = 30.0                             # unit 0 at half health in both envs
    env.set_state(hp=hp)
    rew, _ = env.step(np.zeros((2, 2), np.uint8))
    assert rew[0].tolist() == [-0.5, 0.5]       # level 0: unit 0 is the ally that suffers
    assert rew[1].tolist() == [-0.5, 0.5]       # level 1: it is the adversary; its own team loses
    assert env.st["phi_prev"].tolist() == [-0.5, 0.5]
    obs, _, _ = env.observe()
    assert obs[:, :, 15].tolist() == [[0.0, 1.0], [1.0, 0.0]]


def test_terrain_and_zone_slots_come_from_the_level():
    g0 = np.zeros((1, 8, 8), np.int8)
    g1 = np.zeros((1, 8, 8), np.int8)
    g1[0, 2, 5] = I.ZONE_BUSH                   # cell size 4: x in [20,24), y in [8,12)
    units = [unit("farmer", 0, 14, 10, 0.0), unit("farmer", 1, 22, 10, math.pi)]
    zd0 = np.zeros((1, 1, 6), np.float32)
    zd1 = np.array([[[I.ZONE_BUSH, 22.0, 10.0, 2.0, 2.0, 0.0]]], np.float32)
    l0 = I.custom_scenario(units, grid=8, terrain=g0, zone_desc=zd0)
    l1 = I.custom_scenario(units, grid=8, terrain=g1, zone_desc=zd1)
    p = I.custom_params(2, grid=8, max_zones=1, num_envs=2, num_levels=2)
    env = ref.RefEnv(p, bank(l0, l1))
    env.st["next_level"][:] = [0, 1]
    env.reset()
    obs, vis, _ = env.observe()
    assert vis_bit(vis, 0, 0, 1) == 1           # open ground
    assert vis_bit(vis, 1, 0, 1) == 0           # same pose, but this env's level has a bush there
    assert obs[0, 0, 32:].tolist() == [0.0] * 6
    assert obs[1, 0, 32:].tolist() == [float(I.ZONE_BUSH), 8.0, 0.0, 2.0, 2.0, 0.0]
    assert obs[1, 1, 14] == float(I.ZONE_BUSH)  # zone type under the hidden unit


def test_identity_bank_equals_no_bank():
    """A bank with one level per env, each env pinned to its own row, is the plain scenario."""
    w = I.WORKLOADS["c2_4096env_5v5"]
    E = 12
    p, sc = I.make_params(w, E, max_steps=40), I.make_scenario(w, E)
    plain = ref.RefEnv(p, sc)
    banked = ref.RefEnv(dict(p, num_levels=E, level_seed=3), sc)
    plain.reset()
    banked.reset()                               # next_level starts as e % L = e
    for s in range(120):
        a = I.actions_for_step(w.seed, s, E, w.num_units)
        banked.st["next_level"][:] = np.arange(E)
        r0, d0 = plain.step(a)
        r1, d1 = banked.step(a)
        assert np.array_equal(r0, r1) and np.array_equal(d0, d1)
        for k in plain.st:
            assert np.array_equal(plain.st[k], banked.st[k]), (s, k)
    assert np.array_equal(plain.observe()[0], banked.observe()[0])
    assert np.array_equal(plain.global_state(), banked.global_state())
    assert plain.st["ep_count"].sum() > 0


def test_level_draws_are_uniform_and_reproducible():
    w = I.WORKLOADS["c2_4096env_5v5"]
    E, L = 64, 7
    p = I.make_params(w, E, max_steps=4, num_levels=L, level_seed=21)
    sc = I.make_scenario(w, L)
    def run():
        env = ref.RefEnv(p, sc)
        env.reset()
        seen = []
        idle = np.zeros((E, w.num_units), np.uint8)
        for s in range(4 * 60):
            env.step(idle)
            if (s + 1) % 4 == 0:
                assert env.dones.all()
                seen.append(env.st["level"].copy())
        return np.array(seen), env
    a, env = run()
    b, _ = run()
    assert np.array_equal(a, b)
    assert env.st["level_draws"].tolist() == [61] * E
    cnt = np.bincount(a.ravel(), minlength=L).astype(float)
    exp = a.size / L
    assert ((cnt - exp) ** 2 / exp).sum() < 22.5          # chi-square, 6 dof, 0.999 quantile
    # envs do not move in step with each other
    assert len({tuple(a[:, e]) for e in range(E)}) == E
    # the first reset queued draw 0, which the first auto-reset took: the episode after the
    # k-th auto-reset (k from 0) plays draw k
    h = ref.lib().tabx_ref_hash
    assert all(a[k, e] == h(21, e, 0, k, 3) % L for k in (0, 5, 59) for e in (0, 3, 63))


def test_a_sample_of_the_batch_replays_with_its_env_ids():
    """Draws are keyed by the env's index: a sub-batch given the original indices reproduces
    its envs of the full batch tick for tick (level draws and the heuristic policy alike)."""
    w = I.WORKLOADS["c2_4096env_5v5"]
    E, L, N = 24, 5, w.num_units
    sc = I.make_scenario(w, L)
    p = I.make_params(w, E, max_steps=6, num_levels=L, level_seed=17)
    rows = np.array([2, 3, 11, 23])
    full = ref.RefEnv(p, sc)
    part = ref.RefEnv(dict(p, num_envs=len(rows), env_ids=rows), sc)
    full.reset()
    part.st["next_level"][:] = full.st["level"][rows]      # both start from the same levels
    part.reset()
    part.st["next_level"][:] = full.st["next_level"][rows]
    part.st["level_draws"][:] = full.st["level_draws"][rows]
    pol = I.policy("medium", 8)
    ctl_f = np.ones((E, N), np.uint8)
    ctl_p = np.ones((len(rows), N), np.uint8)
    for s in range(60):
        af = np.zeros((E, N), np.uint8)
        ap = np.zeros((len(rows), N), np.uint8)
        full.policy_step(pol, ctl_f, af)
        part.policy_step(pol, ctl_p, ap)
        assert np.array_equal(af[rows], ap), s
        for k in full.st:
            assert np.array_equal(full.st[k][rows], part.st[k]), (s, k)
    assert full.st["ep_count"].sum() > E
