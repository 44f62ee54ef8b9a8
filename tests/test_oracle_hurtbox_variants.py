"""Pins of the two hurtbox variants of the CPU checker: every valid body in the hurtbox is
struck (the reading of Sec. 4's "units positioned within this region are affected"), and the
hurtbox bounded laterally by the field of view (App. A "Attack range geometry")."""
import math

import numpy as np
import pytest

from paper_2602_01665_amd import inputs as I
from tests.helpers import acts, make_ref, other_slot, unit

A = I


def test_strike_lands_on_every_body_in_the_hurtbox():
    units = [unit("farmer", 0, 10, 10, 0.0), unit("farmer", 1, 11.5, 10.0),
             unit("farmer", 1, 12.5, 10.5), unit("farmer", 1, 10.0, 14.0),
             unit("farmer", 0, 12.0, 9.5)]
    hit = acts(A.ACT_ATTACK, 0, 0, 0, 0)
    env = make_ref(units)
    env.step(hit)
    assert env.st["hp"][0].tolist() == [60.0, 46.0, 60.0, 60.0, 60.0]      # the closest only
    env = make_ref(units, hit_all=1)
    env.step(hit)
    # both enemies in the box, not the one beside it, never the ally standing in it
    assert env.st["hp"][0].tolist() == [60.0, 46.0, 46.0, 60.0, 60.0]
    assert env.st["cd"][0, 0] == np.float32(2.5)


def test_every_striker_counts_and_sums_in_index_order():
    units = [unit("farmer", 0, 10, 10, 0.0), unit("assassin", 0, 10, 10.5, 0.0),
             unit("farmer", 1, 11.5, 10.0), unit("farmer", 1, 12.0, 10.5)]
    env = make_ref(units, hit_all=1)
    env.step(acts(A.ACT_ATTACK, A.ACT_ATTACK, 0, 0))
    assert env.st["hp"][0].tolist() == [60.0, 70.0, 60.0 - 14.0 - 22.0, 60.0 - 14.0 - 22.0]


def test_heal_reaches_every_ally_in_the_box_and_no_enemy():
    units = [unit("healer", 0, 10, 10, 0.0), unit("farmer", 0, 13, 10), unit("farmer", 0, 16, 10.5),
             unit("farmer", 1, 14, 9.5)]
    env = make_ref(units, hit_all=1)
    env.set_state(hp=np.array([[25.0, 10.0, 58.0, 33.0]], np.float32))
    env.step(acts(A.ACT_ATTACK, 0, 0, 0))
    assert env.st["hp"][0].tolist() == [25.0, 17.0, 60.0, 33.0]            # second one clamps at 60


def test_every_struck_unit_is_revealed():
    g = np.zeros((8, 8), np.int8)
    g[2, 3] = I.ZONE_BUSH | (1 << 2)            # cell size 4: x in [12,16), y in [8,12)
    units = [unit("archer", 0, 4, 10, 0.0), unit("farmer", 1, 13, 10), unit("farmer", 1, 15, 10.5)]
    env = make_ref(units, grid=8, terrain=g, hit_all=1)
    env.step(acts(A.ACT_ATTACK, 0, 0))
    assert env.st["reveal"][0].tolist() == [1.0, 1.0, 1.0]
    env = make_ref(units, grid=8, terrain=g)
    env.step(acts(A.ACT_ATTACK, 0, 0))
    assert env.st["reveal"][0].tolist() == [1.0, 1.0, 0.0]


@pytest.mark.parametrize("pos,rect,cone", [
    ((11.0, 12.5), True, False),     # in the wide box, 68 degrees off the heading: outside a 60-degree cone
    ((14.0, 11.5), True, True),      # 20.6 degrees off
    ((10.5, 10.8), True, False),     # close and 58 degrees off
    ((16.5, 10.0), False, False),    # beyond the range either way
])
def test_hurtbox_bounded_by_the_field_of_view(pos, rect, cone):
    wide = dict(hurt_halfwidth=3.0, range=5.0, sight_angle=math.pi / 3)
    units = [unit("farmer", 0, 10, 10, 0.0, **wide), unit("farmer", 1, pos[0], pos[1])]
    for flag, expect in ((0, rect), (1, cone)):
        env = make_ref(units, hurtbox_cone=flag)
        env.step(acts(A.ACT_ATTACK, 0))
        assert (env.st["hp"][0, 1] == 46.0) == expect, (flag, pos)
        # the observation's attackable feature agrees wherever the unit is seen at all
        env = make_ref(units, hurtbox_cone=flag)
        obs, vis, _ = env.observe()
        if vis[0, 0, 0] & 2:
            assert other_slot(obs[0, 0], 0, 1)[14] == float(expect)


def test_full_circle_cone_changes_nothing():
    w = I.Workload("cone360", 16, 4, 24.0, 24, "iid", 0.7, "iid", steps=150, seed=313)
    from oracle.ref import RefEnv
    sc = I.make_scenario(w, 16)
    sc["sight_cos_half"][...] = -1.0
    sc["sight_angle"][...] = np.float32(2 * math.pi)
    a_env = RefEnv(I.make_params(w, 16, max_steps=48), sc)
    b_env = RefEnv(I.make_params(w, 16, max_steps=48, hurtbox_cone=1), sc)
    a_env.reset()
    b_env.reset()
    for s in range(150):
        a = I.actions_for_step(w.seed, s, 16, w.num_units)
        a_env.step(a)
        b_env.step(a)
        for k in a_env.st:
            assert np.array_equal(a_env.st[k], b_env.st[k]), (s, k)
    assert a_env.st["ep_count"].sum() > 0
