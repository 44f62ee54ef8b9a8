"""Pins of the heuristic policy on units that hold several roles at once, one hand-placed scene
per statement of App. A "Role-Appropriate Heuristic Policy Mechanism" (the classes are not
mutually exclusive: a fast long-range unit is both Ranger and Assassin).

Every expected action below is worked out from the passage's sentences and this build's readings
of what it leaves open (Healer rules before Assassin rules; half-range standoff), on the scene's
geometry, not from the checker's code: sight cone 120 degrees, sight range 16, reach = attack
range + target body radius, moves along the larger component of the offset.  No GPU.
"""
import math

import numpy as np
import pytest

from paper_2602_01665_amd import inputs as I
from tests.helpers import make_ref, unit
from tests.test_oracle_policy import A, GREEDY, decide

FAST = 1.6          # >= the Assassin speed of every tier (1.4)
ONLY0 = np.array([[1, 0, 0, 0, 0, 0]], np.uint8)


def _first(n):
    return np.array([[1] + [0] * (n - 1)], np.uint8)


def test_a_fast_long_range_unit_selects_its_target_as_an_assassin():
    """Target selection: Assassins take the visible enemy of lowest maximum health; the others
    the nearest.  Both enemies are in view of the unit at (4,16) heading +x: the Mammoth (685
    health) 8 away, the Farmer (60) 12.2 away."""
    def scene(speed):
        return make_ref([unit("archer", 0, 4, 16, 0.0, speed=speed), unit("mammoth", 1, 12, 16, 0.0),
                         unit("farmer", 1, 16, 18, 0.0)])
    env = scene(FAST)
    decide(env, controlled=_first(3))
    assert (env.mem["mem_x"][0, 0], env.mem["mem_y"][0, 0]) == (16.0, 18.0)     # the Farmer
    env = scene(1.0)
    decide(env, controlled=_first(3))
    assert (env.mem["mem_x"][0, 0], env.mem["mem_y"][0, 0]) == (12.0, 16.0)     # the nearest


def test_it_turns_to_its_own_selected_target_before_it_kites():
    """Priority 2 (rotate if that would bring the SELECTED target into the engagement region)
    comes before the Rangers' kiting.  Cooldown running.  The Mammoth dead ahead is in the
    hurtbox and inside the kiting distance (8 < 0.7 * 27); the Farmer, up to the left at (12,22),
    is within reach but outside the box.  The Ranger-and-Assassin has selected the Farmer: it
    turns left.  The plain Ranger has selected the Mammoth, which is already in its box: nothing to
    turn to, so it kites, away from the Mammoth (-x)."""
    def scene(speed):
        env = make_ref([unit("archer", 0, 4, 16, 0.0, speed=speed), unit("mammoth", 1, 12, 16, 0.0),
                        unit("farmer", 1, 12, 22, 0.0)])
        env.set_state(cd=np.array([[3.0, 0.0, 0.0]], np.float32))
        return env
    assert decide(scene(FAST), controlled=_first(3))[0, 0] == A["left"]
    assert decide(scene(1.0), controlled=_first(3))[0, 0] == A["xm"]
    # with the shot ready both strike: something worth a strike is in the engagement region
    env = scene(FAST)
    env.set_state(cd=np.zeros((1, 3), np.float32))
    assert decide(env, controlled=_first(3))[0, 0] == A["attack"]


def test_it_kites_as_a_ranger_even_though_assassins_close_in():
    """Threat mitigation: a Ranger retreats when an opponent is nearer than xi * attack range,
    and this comes before navigation.  The lone Farmer 10 away is in the box (nothing to turn
    to), the shot is cooling down: expert tier (0.7 * 27 = 18.9) retreats along -x; with
    xi = 0.3 (8.1) nothing threatens and the unit, aligned, waits."""
    env = make_ref([unit("archer", 0, 16, 16, 0.0, speed=FAST), unit("farmer", 1, 26, 16, math.pi)])
    env.set_state(cd=np.array([[3.0, 0.0]], np.float32))
    assert decide(env, controlled=_first(2))[0, 0] == A["xm"]
    assert decide(env, dict(GREEDY, xi=0.3), controlled=_first(2))[0, 0] == A["noop"]
    # a fast short-range unit (Assassin only) in the same place never retreats
    env = make_ref([unit("farmer", 0, 16, 16, 0.0, speed=FAST), unit("farmer", 1, 18, 16, math.pi)])
    env.set_state(cd=np.array([[3.0, 0.0]], np.float32))
    assert decide(env, controlled=_first(2))[0, 0] == A["noop"]


def test_it_navigates_behind_the_target_as_an_assassin():
    """Spatial positioning: Assassins go behind the target, the others in front of it.  A unit of
    attack range 10 (a Ranger) at (10,10) heading 45 degrees sees a Farmer at (19,19) that faces
    +x, 12.7 away: beyond reach 11 and beyond the kiting distance 7.  Behind it is (14,19):
    offset (4,9), move +y.  In front of it is (24,19): offset (14,9), move +x."""
    tgt = unit("farmer", 1, 19, 19, 0.0)
    fast = make_ref([unit("farmer", 0, 10, 10, math.pi / 4, range=10.0, speed=FAST), tgt])
    slow = make_ref([unit("farmer", 0, 10, 10, math.pi / 4, range=10.0), tgt])
    assert decide(fast, controlled=_first(2))[0, 0] == A["yp"]
    assert decide(slow, controlled=_first(2))[0, 0] == A["xp"]
    # the target turned to face -y: behind is (19,24), offset (9,14): +y; in front (19,14): +x
    tgt = unit("farmer", 1, 19, 19, 3 * math.pi / 2)
    fast = make_ref([unit("farmer", 0, 10, 10, math.pi / 4, range=10.0, speed=FAST), tgt])
    slow = make_ref([unit("farmer", 0, 10, 10, math.pi / 4, range=10.0), tgt])
    assert decide(fast, controlled=_first(2))[0, 0] == A["yp"]
    assert decide(slow, controlled=_first(2))[0, 0] == A["xp"]


def test_with_nothing_in_sight_it_seeks_a_bush_as_a_ranger():
    """No visible and no remembered target: Rangers first walk to a nearby bush zone and search
    there; other units search at once, however fast they are."""
    zd = [[I.ZONE_BUSH, 26.0, 14.0, 2.0, 2.0, 0.0], [I.ZONE_BUSH, 8.0, 22.0, 2.0, 2.0, 0.0]]

    def build(name, x, y, **kw):
        return make_ref([unit(name, 0, x, y, 0.0, **kw), unit("farmer", 1, 2, 2, 0.0)],
                        zone_desc=zd, max_zones=2, zone_shapes=1)
    # (10,12): the second bush is 10.2 away, the first 16.1: offset (-2,10): +y
    assert decide(build("archer", 10, 12, speed=FAST), controlled=_first(2))[0, 0] == A["yp"]
    assert decide(build("archer", 8.5, 21.5, speed=FAST), controlled=_first(2))[0, 0] in (A["left"], A["right"])
    assert decide(build("farmer", 10, 12, speed=FAST), controlled=_first(2))[0, 0] in (A["left"], A["right"])


def test_a_fast_healer_selects_its_target_as_a_healer():
    """Healers take the nearest injured ally, else the nearest ally; a unit whose strike heals
    cannot harm an opponent, so the Healer rule goes before the Assassin rule.  In view of the
    fast Healer at (4,16): a healthy ally 4 away, an injured ally at (14,17), an enemy Farmer of
    low maximum health at (12,14)."""
    env = make_ref([unit("healer", 0, 4, 16, 0.0, speed=FAST), unit("farmer", 0, 8, 16, 0.0),
                    unit("farmer", 0, 14, 17, 0.0), unit("farmer", 1, 12, 14, 0.0)])
    hp = env.st["hp"].copy()
    hp[0, 2] = 30.0
    env.set_state(hp=hp)
    decide(env, controlled=_first(4))
    assert (env.mem["mem_x"][0, 0], env.mem["mem_y"][0, 0]) == (14.0, 17.0)
    # nobody injured: the nearest ally, still no opponent
    hp[0, 2] = 60.0
    env.set_state(hp=hp)
    env.mem["mem_valid"][...] = 0
    decide(env, controlled=_first(4))
    assert (env.mem["mem_x"][0, 0], env.mem["mem_y"][0, 0]) == (8.0, 16.0)


@pytest.mark.parametrize("heading", [0.0, math.pi / 2])
def test_a_fast_healer_goes_to_its_target_itself(heading):
    """Healers minimise the distance to their target: neither behind it (heading +y: (19,15),
    offset (9,5), +x) nor in front of it (heading +x: (24,20), offset (14,10), +x).  The injured
    ally is at (19,20), 13.5 away and beyond reach 11: offset (9,10), move +y, whatever it faces."""
    env = make_ref([unit("healer", 0, 10, 10, math.pi / 4, speed=FAST), unit("farmer", 0, 19, 20, heading),
                    unit("farmer", 1, 30, 1, 0.0)])
    hp = env.st["hp"].copy()
    hp[0, 1] = 30.0
    env.set_state(hp=hp)
    assert decide(env, controlled=_first(3))[0, 0] == A["yp"]


def test_a_long_range_healer_kites_from_a_near_opponent():
    """The Healer of the unit table has attack range 10, the Ranger threshold: the
    distance-maintenance protocol applies to it.  Its injured ally is 12 ahead (beyond reach),
    an opponent 5 ahead (inside 0.7 * 10): it retreats along -x; with range 9.9 it is no Ranger
    and walks on to its ally (+x)."""
    def scene(rng):
        env = make_ref([unit("healer", 0, 12, 16, 0.0, range=rng), unit("farmer", 0, 24, 16, 0.0),
                        unit("farmer", 1, 17, 16.5, 0.0)])
        hp = env.st["hp"].copy()
        hp[0, 1] = 30.0
        env.set_state(hp=hp, cd=np.array([[1.0, 0.0, 0.0]], np.float32))
        return env
    assert decide(scene(10.0), controlled=_first(3))[0, 0] == A["xm"]
    assert decide(scene(9.9), controlled=_first(3))[0, 0] == A["xp"]
