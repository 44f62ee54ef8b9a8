"""Seeded synthetic inputs for the TABX batched step: scenarios, parameters, actions.

This module holds no part of the environment's arithmetic.  It only draws the
numbers that both the GPU library and the CPU checker take as inputs (numpy
arrays), so that the two can be run on identical bytes.  The unit statistics are
the rows of the paper's "Default unit statistics" table (App. A, Unit
Specifications); the five workloads are synthetic stand-ins shaped like the
paper's battle scenarios (the paper's own scenario files are not available).
"""
from __future__ import annotations

from dataclasses import dataclass, field
import math

import numpy as np

# --------------------------------------------------------------------------
# Paper data: App. A "Unit Specifications", table "Default unit statistics".
# columns: health, body radius, body weight, speed, attack damage, attack range,
#          attack cooldown, space occupied.  Negative damage = healing.
# --------------------------------------------------------------------------
ROSTER = {
    "farmer":   (60.0, 1.0, 1.0, 1.1, 14.0, 2.5, 2.5, 1),
    "assassin": (70.0, 1.0, 1.0, 1.4, 22.0, 2.5, 1.5, 1),
    "theking":  (346.0, 1.47, 10.0, 1.2, 46.0, 3.2, 2.5, 1),
    "mammoth":  (685.0, 4.25, 50.0, 1.2, 20.0, 3.0, 6.5, 4),
    "archer":   (40.0, 1.0, 1.0, 1.0, 28.0, 27.0, 8.0, 1),
    "cannon":   (100.0, 1.0, 5.2, 0.5, 80.0, 40.0, 10.0, 1),
    "deadeye":  (40.0, 1.0, 1.0, 1.1, 25.0, 20.0, 8.0, 1),
    "healer":   (25.0, 1.0, 1.0, 1.0, -7.0, 10.0, 2.0, 1),
    "paladin":  (220.0, 1.32, 8.5, 1.2, -6.0, 7.5, 2.0, 1),
}
# Role classes of Sec. 4.2 mapped to one roster row each: Ranger = range >= 10
# (Archer), Assassin = speed >= 1.4 (Assassin), Healer = negative damage (Healer).
ROLE_UNIT = ("archer", "assassin", "healer")      # role id 0, 1, 2
ROLE_RANGER, ROLE_ASSASSIN, ROLE_HEALER = 0, 1, 2

# Terrain cell encoding: low two bits = zone type, upper bits = zone id.
ZONE_OPEN, ZONE_LAVA, ZONE_BUSH, ZONE_SWAMP = 0, 1, 2, 3

# Discrete actions (Sec. 4 and App. A "Action Space").
ACT_NOOP, ACT_XP, ACT_YP, ACT_XM, ACT_YM, ACT_ATTACK, ACT_ROT_L, ACT_ROT_R = range(8)
NUM_ACTIONS = 8

# Physics / zone constants the paper leaves as free parameters.
DEFAULTS = dict(
    dt=0.25,
    turn_rate=math.pi / 2.0,      # rad per time unit  (pi/8 per step)
    max_steps=256,
    lava_dps=4.0,
    swamp_mult=0.5,
    reveal_time=1.0,
    boundary_frac=0.1,            # App. A "Movement and kinematic update"
    sight_angle=2.0 * math.pi / 3.0,
    sight_range=16.0,
    collision_alpha=0.0,          # the benchmark tick has no body collisions; tests use 0.8
    collision_slop=0.01,
)

# Paper data: App. A table "Heuristic policy parameters across all difficulty tier":
# stochasticity of action (epsilon), aggressive threshold (xi), Assassin speed, Ranger range.
POLICY_TIERS = {
    "random":   dict(epsilon=1.0,  xi=0.0, assassin_speed=1.4, ranger_range=10.0),
    "novice":   dict(epsilon=0.5,  xi=0.1, assassin_speed=1.4, ranger_range=10.0),
    "medium":   dict(epsilon=0.2,  xi=0.3, assassin_speed=1.4, ranger_range=10.0),
    "advanced": dict(epsilon=0.1,  xi=0.5, assassin_speed=1.4, ranger_range=10.0),
    "expert":   dict(epsilon=0.01, xi=0.7, assassin_speed=1.4, ranger_range=10.0),
}


def policy(tier: str, seed: int = 1) -> dict:
    return dict(POLICY_TIERS[tier], seed=int(seed))


FLOAT_UNIT_FIELDS = (
    "init_x", "init_y", "init_theta", "hmax", "radius", "mass", "speed", "dmg",
    "range", "cooldown", "sight_angle", "sight_cos_half", "sight_range",
    "hurt_halfwidth",
)
BYTE_UNIT_FIELDS = ("team", "enabled")


@dataclass(frozen=True)
class Workload:
    """One synthetic workload (the five of them mirror the benchmark configs)."""
    name: str
    num_envs: int
    team_size: int                 # units per team; N = 2 * team_size
    map_size: float
    grid: int                      # terrain cells per side, 0 = no terrain
    terrain: str                   # "none" | "iid" | "rects" (cell grids) | "ellipses" (no grid)
    p_open: float
    roles: str                     # "one_each" | "iid" | "ratio"
    role_counts: tuple = ()        # per team, for "ratio"
    spawn: str = "halves"          # "halves" | "clusters"
    max_zones: int = 0
    steps: int = 100
    seed: int = 0
    extra: dict = field(default_factory=dict)

    @property
    def num_units(self) -> int:
        return 2 * self.team_size


WORKLOADS = {
    "c1_16env_3v3": Workload("c1_16env_3v3", 16, 3, 32.0, 0, "none", 1.0, "one_each",
                             steps=100, seed=20260201),
    "c2_4096env_5v5": Workload("c2_4096env_5v5", 4096, 5, 64.0, 64, "iid", 0.7, "iid",
                               steps=500, seed=20260202),
    "c3_16384env_10v10": Workload("c3_16384env_10v10", 16384, 10, 64.0, 64, "rects", 1.0,
                                  "ratio", role_counts=(4, 3, 3), max_zones=8,
                                  steps=1000, seed=20260203),
    "c4_65536env_5v5": Workload("c4_65536env_5v5", 65536, 5, 48.0, 0, "none", 1.0, "iid",
                                steps=1000, seed=20260204),
    "c5_1024env_64v64": Workload("c5_1024env_64v64", 1024, 64, 128.0, 128, "iid", 0.6,
                                 "ratio", role_counts=(22, 21, 21), spawn="clusters",
                                 steps=500, seed=20260205),
}
# the headline shape with the paper's zone geometry (ellipses with their own effect magnitudes)
# instead of the benchmark's cell grid; not one of the five benchmark configurations
WORKLOADS["c3e_16384env_10v10_ellipses"] = Workload(
    "c3e_16384env_10v10_ellipses", 16384, 10, 64.0, 0, "ellipses", 1.0, "ratio",
    role_counts=(4, 3, 3), max_zones=8, steps=1000, seed=20260213)
# shapes that launch four wavefronts per env group (32 and more units per env, one-wavefront
# envs): the headline's terrain and zones with larger teams, sized to about the same 0.45 GB of
# observation rows per tick; not benchmark configurations either
WORKLOADS["n32_6144env_16v16"] = Workload(
    "n32_6144env_16v16", 6144, 16, 64.0, 64, "rects", 1.0, "ratio", role_counts=(6, 5, 5),
    max_zones=8, steps=500, seed=20260216)
WORKLOADS["n64_1536env_32v32"] = Workload(
    "n64_1536env_32v32", 1536, 32, 64.0, 64, "rects", 1.0, "ratio", role_counts=(12, 10, 10),
    max_zones=8, steps=500, seed=20260232)
HEADLINE = "c3_16384env_10v10"


def obs_dim(num_units: int, max_zones: int) -> int:
    """Floats per agent observation: N unit blocks of 16 (own first) + zone slots of 6."""
    return 16 * num_units + 6 * max_zones


def make_params(w: Workload, num_envs: int | None = None, **override) -> dict:
    p = dict(
        num_envs=int(w.num_envs if num_envs is None else num_envs),
        num_units=w.num_units,
        grid_w=w.grid, grid_h=w.grid,
        max_zones=w.max_zones,
        max_steps=DEFAULTS["max_steps"],
        map_w=float(w.map_size), map_h=float(w.map_size),
        cell_size=float(w.map_size / w.grid) if w.grid else 1.0,
        dt=DEFAULTS["dt"], turn_rate=DEFAULTS["turn_rate"],
        lava_dps=DEFAULTS["lava_dps"], swamp_mult=DEFAULTS["swamp_mult"],
        reveal_time=DEFAULTS["reveal_time"], boundary_frac=DEFAULTS["boundary_frac"],
        collision_alpha=DEFAULTS["collision_alpha"], collision_slop=DEFAULTS["collision_slop"],
        zone_shapes=1 if w.terrain == "ellipses" else 0,
        num_levels=0, level_seed=0, hurtbox_cone=0, hit_all=0, env_id_offset=0,
    )
    p.update(override)
    return p


def _spec_arrays(role: np.ndarray) -> dict:
    """Per-unit spec arrays from an integer role array of any shape."""
    table = np.array([ROSTER[name][:7] for name in ROLE_UNIT], dtype=np.float32)
    s = table[role]                                   # [..., 7]
    out = dict(hmax=s[..., 0], radius=s[..., 1], mass=s[..., 2], speed=s[..., 3],
               dmg=s[..., 4], range=s[..., 5], cooldown=s[..., 6])
    shape = role.shape
    out["sight_angle"] = np.full(shape, DEFAULTS["sight_angle"], np.float32)
    out["sight_cos_half"] = np.full(
        shape, np.float32(math.cos(DEFAULTS["sight_angle"] / 2.0)), np.float32)
    out["sight_range"] = np.full(shape, DEFAULTS["sight_range"], np.float32)
    out["hurt_halfwidth"] = out["radius"].copy()
    return {k: np.ascontiguousarray(v, dtype=np.float32) for k, v in out.items()}


def _draw_roles(w: Workload, rng: np.random.Generator, E: int) -> np.ndarray:
    n = w.team_size
    if w.roles == "one_each":
        assert n == 3
        team = np.tile(np.array([0, 1, 2], np.int64), (E, 1))
        return np.concatenate([team, team], axis=1)
    if w.roles == "iid":
        return rng.integers(0, 3, size=(E, 2 * n))
    if w.roles == "ratio":
        assert sum(w.role_counts) == n
        team = np.repeat(np.arange(3), w.role_counts)
        return np.tile(np.concatenate([team, team]), (E, 1))
    raise ValueError(w.roles)


def _draw_terrain(w: Workload, rng: np.random.Generator, E: int, Z: int):
    """Returns (terrain int8 [E,G,G] or None, zone_desc float32 [E,Z,6] or None)."""
    G = w.grid
    if w.terrain == "ellipses":
        # App. A "Zones": type, centre, two semi-axes, effect magnitude; 4..Z active slots
        assert Z >= 4 and G == 0
        desc = np.zeros((E, Z, 6), np.float32)
        count = rng.integers(4, Z + 1, size=E)
        kind = rng.integers(1, 4, size=(E, Z))
        desc[..., 0] = kind
        desc[..., 1] = rng.uniform(0.0, w.map_size, size=(E, Z))
        desc[..., 2] = rng.uniform(0.0, w.map_size, size=(E, Z))
        desc[..., 3] = rng.uniform(2.0, 9.0, size=(E, Z))
        desc[..., 4] = rng.uniform(2.0, 9.0, size=(E, Z))
        effect = np.where(kind == ZONE_LAVA, rng.uniform(2.0, 6.0, size=(E, Z)),
                          np.where(kind == ZONE_SWAMP, rng.uniform(0.3, 0.8, size=(E, Z)), 0.0))
        desc[..., 5] = effect
        desc[np.arange(Z)[None, :] >= count[:, None]] = 0.0
        return None, desc
    if w.terrain == "none" or G == 0:
        return None, (np.zeros((E, Z, 6), np.float32) if Z else None)
    cell = w.map_size / G
    if w.terrain == "iid":
        is_open = rng.random((E, G, G)) < w.p_open
        kind = rng.integers(1, 4, size=(E, G, G)).astype(np.int8)
        terrain = np.where(is_open, np.int8(0), kind).astype(np.int8)
        return terrain, (np.zeros((E, Z, 6), np.float32) if Z else None)
    if w.terrain == "rects":
        assert Z >= 8
        terrain = np.zeros((E, G, G), np.int8)
        desc = np.zeros((E, Z, 6), np.float32)
        count = rng.integers(4, 9, size=E)
        ys = np.arange(G)[None, :, None]
        xs = np.arange(G)[None, None, :]
        effect = np.array([0.0, DEFAULTS["lava_dps"], 0.0, DEFAULTS["swamp_mult"]],
                          np.float32)
        for r in range(8):
            kind = rng.integers(1, 4, size=E)
            wx = rng.integers(4, 17, size=E)
            wy = rng.integers(4, 17, size=E)
            x0 = (rng.random(E) * (G - wx + 1)).astype(np.int64)
            y0 = (rng.random(E) * (G - wy + 1)).astype(np.int64)
            active = r < count
            inside = ((xs >= x0[:, None, None]) & (xs < (x0 + wx)[:, None, None]) &
                      (ys >= y0[:, None, None]) & (ys < (y0 + wy)[:, None, None]) &
                      active[:, None, None])
            code = (kind | (r << 2)).astype(np.int8)
            terrain = np.where(inside, code[:, None, None], terrain)
            d = np.stack([kind.astype(np.float32),
                          ((x0 + 0.5 * wx) * cell).astype(np.float32),
                          ((y0 + 0.5 * wy) * cell).astype(np.float32),
                          (0.5 * wx * cell).astype(np.float32),
                          (0.5 * wy * cell).astype(np.float32),
                          effect[kind]], axis=1)
            desc[:, r, :] = np.where(active[:, None], d, 0.0)
        return np.ascontiguousarray(terrain), desc
    raise ValueError(w.terrain)


def make_scenario(w: Workload, num_envs: int | None = None, seed: int | None = None,
                  env_offset: int = 0) -> dict:
    """Draws a scenario: dict of numpy arrays, per-unit arrays shaped [E, N].

    `env_offset` is mixed into the seed so that independent sub-batches differ.
    """
    E = int(w.num_envs if num_envs is None else num_envs)
    n, N = w.team_size, w.num_units
    rng = np.random.default_rng([w.seed if seed is None else seed, env_offset])
    W = np.float32(w.map_size)
    half = np.float32(w.map_size / 2.0)

    role = _draw_roles(w, rng, E)
    sc = _spec_arrays(role)
    sc["role"] = role.astype(np.uint8)                # bookkeeping only, not an input
    team = np.concatenate([np.zeros(n, np.uint8), np.ones(n, np.uint8)])
    sc["team"] = np.ascontiguousarray(np.tile(team, (E, 1)))
    sc["enabled"] = np.ones((E, N), np.uint8)

    if w.spawn == "halves":
        x = rng.random((E, N), dtype=np.float32) * half
        x[:, n:] += half
        y = rng.random((E, N), dtype=np.float32) * W
    elif w.spawn == "clusters":
        K, margin, sigma = 4, 12.0, 6.0
        cx = margin + rng.random((E, 2, K)) * (w.map_size / 2.0 - 2 * margin)
        cx[:, 1, :] += w.map_size / 2.0
        cy = margin + rng.random((E, 2, K)) * (w.map_size - 2 * margin)
        pick = rng.integers(0, K, size=(E, N))
        t = np.tile(team.astype(np.int64), (E, 1))
        e_idx = np.arange(E)[:, None]
        x = cx[e_idx, t, pick] + sigma * rng.standard_normal((E, N))
        y = cy[e_idx, t, pick] + sigma * rng.standard_normal((E, N))
        x = np.clip(x, 0.0, w.map_size).astype(np.float32)
        y = np.clip(y, 0.0, w.map_size).astype(np.float32)
    else:
        raise ValueError(w.spawn)
    two_pi = np.float32(2.0 * math.pi)
    theta = rng.random((E, N), dtype=np.float32) * two_pi
    theta = np.minimum(theta, np.nextafter(two_pi, np.float32(0.0)))
    sc["init_x"] = np.ascontiguousarray(x, np.float32)
    sc["init_y"] = np.ascontiguousarray(y, np.float32)
    sc["init_theta"] = np.ascontiguousarray(theta, np.float32)

    terrain, desc = _draw_terrain(w, rng, E, w.max_zones)
    sc["terrain"] = terrain
    sc["zone_desc"] = desc
    return sc


def take_envs(sc: dict, idx) -> dict:
    """Sub-batch of a scenario (rows `idx` of every per-env array)."""
    out = {}
    for k, v in sc.items():
        out[k] = None if v is None else np.ascontiguousarray(v[idx])
    return out


def actions_for_step(seed: int, step: int, num_envs: int, num_units: int) -> np.ndarray:
    """uint8 [E, N] actions uniform over the discrete action set, keyed by (seed, step)."""
    rng = np.random.default_rng([seed + 1000, step])
    return rng.integers(0, NUM_ACTIONS, size=(num_envs, num_units), dtype=np.uint8)


def custom_scenario(units, map_size=32.0, grid=0, terrain=None, zone_desc=None) -> dict:
    """Hand-built single-env scenario for worked examples.

    `units`: list of dicts with keys unit (roster name), team, x, y, theta and
    optional overrides of any float spec field / enabled.
    """
    N = len(units)
    sc = {k: np.zeros((1, N), np.float32) for k in FLOAT_UNIT_FIELDS}
    sc["team"] = np.zeros((1, N), np.uint8)
    sc["enabled"] = np.ones((1, N), np.uint8)
    for u, d in enumerate(units):
        row = ROSTER[d.get("unit", "farmer")]
        vals = dict(hmax=row[0], radius=row[1], mass=row[2], speed=row[3], dmg=row[4],
                    range=row[5], cooldown=row[6],
                    sight_angle=DEFAULTS["sight_angle"], sight_range=DEFAULTS["sight_range"],
                    init_x=d["x"], init_y=d["y"], init_theta=d.get("theta", 0.0))
        vals["hurt_halfwidth"] = vals["radius"]
        for k in FLOAT_UNIT_FIELDS:
            if k in d:
                vals[k] = d[k]
        if "sight_cos_half" not in d:
            vals["sight_cos_half"] = math.cos(vals["sight_angle"] / 2.0)
        for k in FLOAT_UNIT_FIELDS:
            sc[k][0, u] = np.float32(vals[k])
        sc["team"][0, u] = d["team"]
        sc["enabled"][0, u] = d.get("enabled", 1)
    sc["terrain"] = None if terrain is None else np.ascontiguousarray(
        np.asarray(terrain, np.int8).reshape(1, grid, grid))
    sc["zone_desc"] = None if zone_desc is None else np.ascontiguousarray(
        np.asarray(zone_desc, np.float32).reshape(1, -1, 6))
    return sc


def custom_params(num_units, map_size=32.0, grid=0, max_zones=0, **override) -> dict:
    p = dict(num_envs=1, num_units=num_units, grid_w=grid, grid_h=grid, max_zones=max_zones,
             max_steps=DEFAULTS["max_steps"], map_w=float(map_size), map_h=float(map_size),
             cell_size=float(map_size / grid) if grid else 1.0,
             dt=DEFAULTS["dt"], turn_rate=DEFAULTS["turn_rate"],
             lava_dps=DEFAULTS["lava_dps"], swamp_mult=DEFAULTS["swamp_mult"],
             reveal_time=DEFAULTS["reveal_time"], boundary_frac=DEFAULTS["boundary_frac"],
             collision_alpha=DEFAULTS["collision_alpha"], collision_slop=DEFAULTS["collision_slop"],
             zone_shapes=0, num_levels=0, level_seed=0, hurtbox_cone=0, hit_all=0,
             env_id_offset=0)
    p.update(override)
    return p
