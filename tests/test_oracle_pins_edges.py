"""Further pins of the CPU checker (no GPU): cases that tell the checker from a copy with one
plausible slip which the pins of test_oracle_pins.py let through (tests/oracle_mutants.py lists
the slips; tests/test_oracle_mutations.py shows that every one of them now fails a pin).

Citations as in test_oracle_pins.py: App. A "Movement and kinematic update", "Attack range
geometry and target selection", "Zones", "Observation and Global State", "Additional
Performance Metrics"; the closed hurtbox boundary and the per-unit sight range are this
build's readings of them.
"""
import math

import numpy as np

from paper_2602_01665_amd import inputs as I
from tests.helpers import acts, make_ref, other_slot, unit, vis_bit

A = I


def test_arena_that_is_not_square():
    # 32 wide, 16 high: y is clipped to the height, x to the width, each with the penalty
    env = make_ref([unit("assassin", 0, 31.9, 8.0), unit("assassin", 1, 20.0, 15.9)], map_h=16.0)
    for _ in range(3):
        env.step(acts(A.ACT_XP, A.ACT_YP))
    assert env.st["x"][0, 0] == 32.0 and env.st["y"][0, 0] == 8.0
    assert env.st["x"][0, 1] == 20.0 and env.st["y"][0, 1] == 16.0
    assert env.st["hp"][0, 0] < 70.0 and env.st["hp"][0, 1] < 70.0
    # y = 20 would be inside a 32 x 32 arena
    env = make_ref([unit("assassin", 0, 5.0, 5.0), unit("assassin", 1, 20.0, 20.0)])
    env.step(acts(A.ACT_NOOP, A.ACT_NOOP))
    assert env.st["y"][0, 1] == 20.0 and env.st["hp"][0, 1] == 70.0


def _strike(target):
    env = make_ref([unit("assassin", 0, 10.0, 10.0, 0.0), target])
    env.step(acts(A.ACT_ATTACK, A.ACT_NOOP))
    return env.st["hp"][0, 1] < 70.0


def test_hurtbox_gap_is_compared_with_the_body_radius_squared():
    # rectangle ends at x = 12.5; gap 0.6 against a body of radius 0.5: 0.36 > 0.25, a miss
    assert not _strike(unit("assassin", 1, 13.1, 10.0, radius=0.5))
    assert _strike(unit("assassin", 1, 12.9, 10.0, radius=0.5))
    # gap 1.8 against radius 2: 3.24 <= 4, a hit
    assert _strike(unit("assassin", 1, 14.3, 10.0, radius=2.0))
    assert not _strike(unit("assassin", 1, 14.6, 10.0, radius=2.0))


def test_hurtbox_boundary_is_closed():
    # heading 0 has cosine 1 and sine 0 exactly; the body of radius 1 at x = 13.5 touches the
    # far edge x = 12.5 in one point, laterally at y = 12 the edge y = 11: both count
    assert _strike(unit("assassin", 1, 13.5, 10.0))
    assert _strike(unit("assassin", 1, 11.0, 12.0))
    assert not _strike(unit("assassin", 1, float(np.nextafter(np.float32(13.5), np.float32(14))), 10.0))


def test_swamp_slows_from_the_tick_a_unit_stands_in_it():
    g = np.zeros((8, 8), np.int8)
    g[1, 5] = I.ZONE_SWAMP                  # x in [20, 24), y in [4, 8)
    env = make_ref([unit("archer", 0, 22.0, 6.0), unit("archer", 0, 19.9, 6.0),
                    unit("archer", 1, 5.0, 25.0)], grid=8, terrain=g)
    assert list(env.st["cur_speed"][0]) == [0.5, 1.0, 1.0]
    xs = [env.st["x"][0].copy()]
    for _ in range(4):
        env.step(acts(A.ACT_XP, A.ACT_XP, A.ACT_NOOP))
        xs.append(env.st["x"][0].copy())
        # the own block of the observation shows the current speed
        env.observe()
        assert env.obs[0, 0, 13] == env.st["cur_speed"][0, 0]
        assert env.obs[0, 1, 13] == env.st["cur_speed"][0, 1]
    d = np.diff(np.array(xs), axis=0)
    # unit 0 stays in the swamp: every move is 0.5 * dt, and its speed stays halved
    assert list(d[1:, 0]) == [0.125, 0.125, 0.125] and env.st["cur_speed"][0, 0] == 0.5
    # unit 1 walks in: the first move (1.0 * dt) carries it to 20.15, inside the swamp; the
    # velocity of the next tick was set before the zone took effect, then it is slowed
    assert list(d[1:, 1]) == [0.25, 0.25, 0.125] and env.st["cur_speed"][0, 1] == 0.5
    assert env.obs[0, 1, 13] == 0.5 and env.obs[0, 1, 14] == float(I.ZONE_SWAMP)


def test_first_kill_is_kept_for_the_rest_of_the_episode():
    # tick 1: the lone adversary archer 2 dies (kill code 1); later an ally burns in lava
    g = np.zeros((8, 8), np.int8)
    g[1, 1] = I.ZONE_LAVA
    env = make_ref([unit("assassin", 0, 10.0, 20.0, 0.0), unit("healer", 0, 6.0, 6.0),
                    unit("archer", 1, 12.0, 20.0), unit("mammoth", 1, 28.0, 28.0)],
                   grid=8, terrain=g)
    env.set_state(hp=np.array([[70.0, 25.0, 5.0, 685.0]], np.float32))
    env.step(acts(A.ACT_ATTACK, A.ACT_NOOP, A.ACT_NOOP, A.ACT_NOOP))
    assert env.st["alive"][0, 2] == 0 and env.st["kill_run"][0] == 1
    for _ in range(30):
        env.step(acts(A.ACT_NOOP, A.ACT_NOOP, A.ACT_NOOP, A.ACT_NOOP))
    assert env.st["alive"][0, 1] == 0 and env.st["kill_run"][0] == 1
    assert env.st["ep_count"][0] == 0


def test_sight_range_is_the_observers():
    # facing each other 12 apart; unit 0 sees 15 far, unit 1 only 8
    env = make_ref([unit("farmer", 0, 8.0, 16.0, 0.0, sight_range=15.0),
                    unit("farmer", 1, 20.0, 16.0, math.pi, sight_range=8.0)])
    env.observe()
    assert vis_bit(env.vis, 0, 0, 1) == 1 and vis_bit(env.vis, 0, 1, 0) == 0
    assert other_slot(env.obs[0, 0], 0, 1)[12] == 1.0
    assert not other_slot(env.obs[0, 1], 1, 0).any()
