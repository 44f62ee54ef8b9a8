"""HIP library vs CPU checker, element by element, through the C ABI (needs an MI355X).

Bar: integer / boolean fields (alive, t, dones, visibility masks, action masks,
discrete observation features) bit-exact; float32 fields (positions, headings,
health, timers, rewards, observations) within 1e-5 absolute, over full seeded
rollouts with auto-reset.
"""
import math
import sys

import numpy as np
import pytest

from paper_2602_01665_amd import inputs as I
from tests.parity import compare_metrics, compare_outputs, compare_state

pytestmark = pytest.mark.gpu

DENSE = I.Workload("dense_4v4", 128, 4, 24.0, 24, "iid", 0.7, "iid", steps=300, seed=991)


def _say(msg):
    print(msg, flush=True)
    sys.stdout.flush()


def _pair(w, E, scenario=None, **override):
    import torch
    from oracle.ref import RefEnv
    from paper_2602_01665_amd.binding import TabxEnv
    assert torch.cuda.is_available()
    p = I.make_params(w, E, **override)
    sc = I.make_scenario(w, E) if scenario is None else scenario
    ref = RefEnv(p, sc)
    gpu = TabxEnv(p, sc, want_metrics=True, want_global_state=True)
    ref.reset()
    gpu.reset()
    torch.cuda.synchronize()
    compare_state(gpu.state_numpy(), ref.st, "after reset: ")
    return p, sc, ref, gpu


def _rollout(w, E, steps, fused, scenario=None, obs_every=1, **override):
    import torch
    p, sc, ref, gpu = _pair(w, E, scenario, **override)
    N = p["num_units"]
    inexact = dones = 0
    for s in range(steps):
        a = I.actions_for_step(w.seed, s, E, N)
        ad = torch.from_numpy(a).to(gpu.device)
        ref.step(a)
        look = (s % obs_every == 0) or s == steps - 1
        if fused:
            gpu.step_observe(ad)
        else:
            gpu.step(ad)
            if look:
                gpu.observe()
        if look or fused:
            ref.observe()
        torch.cuda.synchronize()
        where = f"{w.name} E={E} step {s}: "
        inexact += compare_state(gpu.state_numpy(), ref.st, where)
        inexact += compare_outputs(gpu, ref, where, check_obs=look or fused)
        inexact += compare_metrics(gpu, ref, where)
        if look or fused:
            # the global state every observing call leaves in the state's output buffer
            assert np.array_equal(gpu.gs_live.cpu().numpy(), ref.global_state()), \
                where + "global state written by the observe stage"
        if s % 16 == 0:
            g = gpu.global_state()
            torch.cuda.synchronize()
            assert np.array_equal(g.cpu().numpy(), ref.global_state()), where + "global state"
        dones += int(ref.dones.sum())
    assert int(ref.st["ep_count"].sum()) == dones
    return inexact, dones


CASES = [
    ("c1_16env_3v3", 16, 100, dict(max_steps=32)),   # the small config, full size
    ("c2_4096env_5v5", 96, 200, dict(max_steps=64)),
    ("c3_16384env_10v10", 64, 200, dict(max_steps=96)),
    ("c4_65536env_5v5", 256, 200, dict(max_steps=50)),
    ("c5_1024env_64v64", 3, 60, dict(max_steps=40)),
]


@pytest.mark.parametrize("fused", [False, True], ids=["separate", "fused"])
@pytest.mark.parametrize("name,E,steps,over", CASES, ids=[c[0] for c in CASES])
def test_rollout_matches_checker(name, E, steps, over, fused):
    _say(f"[gpu] rollout {name} E={E} steps={steps} fused={fused}")
    inexact, dones = _rollout(I.WORKLOADS[name], E, steps, fused, **over)
    _say(f"[gpu]   floats within tolerance but not bit-identical: {inexact}; episodes ended: {dones}")
    assert dones > 0              # auto-reset was exercised


FORMS = [
    # (workload, envs, wavefronts sharing an env group in the fused tick, overrides)
    ("c3_16384env_10v10", 700, 4, {}),                       # at most three env groups per CU
    ("c3_16384env_10v10", 2400, 2, {}),                      # under one residency round
    ("c3_16384env_10v10", 2400, 2, dict(collision_alpha=0.8)),
    ("c3_16384env_10v10", 2400, 2, dict(collision_alpha=0.8, dynamics=1, move_gain=2.0, restitution=0.5)),
    ("c2_4096env_5v5", 5400, 2, {}),
    ("c4_65536env_5v5", 13000, 1, {}),                       # a full machine, five flushes
    ("n32_6144env_16v16", 1700, 4, {}),                      # sixteen flushes
    ("c3e_16384env_10v10_ellipses", 700, 2, {}),             # elliptical zones never take four
]


@pytest.mark.parametrize("name,E,sharing,over", FORMS,
                         ids=[f"{c[0]}-{c[1]}-{c[2]}" + ("-dynamics" if "dynamics" in c[3] else "-collisions" if c[3] else "")
                              for c in FORMS])
def test_every_form_of_the_fused_launch(name, E, sharing, over):
    """How many wavefronts share an env group in the fused tick depends on the batch size, the
    number of observers and the options; each form runs here at a batch size that selects it
    (checked against what the library says it would launch), every env against the checker."""
    from paper_2602_01665_amd import binding as B
    w = I.WORKLOADS[name]
    info = B.tabx_launch_info(B.make_params(I.make_params(w, E, max_steps=20, **over)), "step_observe")
    assert info["wavefronts_per_env_group"] == sharing, info
    _say(f"[gpu] fused launch form: {name} E={E}, {sharing} wavefront(s) per env group {over}")
    inexact, dones = _rollout(w, E, 45, True, max_steps=20, **over)
    assert dones > 0


@pytest.mark.parametrize("fused", [False, True], ids=["separate", "fused"])
def test_combat_heavy_rollout(fused):
    _say(f"[gpu] dense 4v4 combat rollout fused={fused}")
    inexact, dones = _rollout(DENSE, 128, 300, fused, max_steps=48)
    _say(f"[gpu]   inexact floats {inexact}; episodes ended {dones}")
    assert dones > 128


VARIANTS = [dict(hit_all=1), dict(hurtbox_cone=1), dict(hit_all=1, hurtbox_cone=1)]


@pytest.mark.parametrize("fused", [False, True], ids=["separate", "fused"])
@pytest.mark.parametrize("variant", VARIANTS, ids=["hit_all", "cone", "hit_all+cone"])
def test_hurtbox_variants(variant, fused):
    """Strikes that land on every body in the hurtbox, and the hurtbox bounded by the sight
    cone: crowded 4v4, the 10v10 workload, and 64v64 (two wavefronts per env, two mask words)."""
    _say(f"[gpu] hurtbox variant {variant} fused={fused}")
    inexact, dones = _rollout(DENSE, 128, 200, fused, max_steps=48, **variant)
    assert dones > 64
    wide = I.make_scenario(I.WORKLOADS["c3_16384env_10v10"], 48)
    wide["hurt_halfwidth"] *= np.float32(3.0)            # boxes wider than the cone near the unit
    _rollout(I.WORKLOADS["c3_16384env_10v10"], 48, 120, fused, scenario=wide, max_steps=64,
             **variant)
    _rollout(I.WORKLOADS["c5_1024env_64v64"], 2, 50, fused, max_steps=30, **variant)


@pytest.mark.parametrize("team_size,disabled", [(1, 0), (3, 1), (7, 2), (16, 3), (17, 0),
                                                (32, 5), (33, 4), (50, 9), (64, 0)])
def test_ragged_unit_counts_and_padding(team_size, disabled):
    """Unit counts around the 32 / 64 / 128 lane boundaries, with disabled placeholders."""
    w = I.Workload(f"ragged_{team_size}", 5, team_size, 40.0, 20, "iid", 0.6, "iid",
                   steps=60, seed=4242 + team_size)
    sc = I.make_scenario(w, 5)
    rng = np.random.default_rng(team_size)
    for e in range(5):
        off = rng.choice(w.num_units, size=min(disabled, w.num_units - 2), replace=False)
        # keep at least one unit per team enabled
        off = [u for u in off if u not in (0, w.num_units - 1)]
        sc["enabled"][e, off] = 0
    _say(f"[gpu] ragged N={w.num_units} disabled={disabled}")
    inexact, dones = _rollout(w, 5, 60, True, scenario=sc, max_steps=25)
    assert dones > 0


def test_zone_descriptor_slots_and_full_cone():
    """Zone slots up to the maximum, 360-degree and narrow cones, odd cell size."""
    w = I.Workload("zones", 9, 6, 30.0, 20, "rects", 1.0, "iid", max_zones=16, steps=80,
                   seed=77)
    sc = I.make_scenario(w, 9)
    sc["sight_angle"][:, ::3] = np.float32(2 * math.pi)
    sc["sight_cos_half"][:, ::3] = np.float32(-1.0)
    sc["sight_angle"][:, 1::3] = np.float32(0.5)
    sc["sight_cos_half"][:, 1::3] = np.float32(math.cos(0.25))
    _say("[gpu] zone descriptors Z=16, mixed cones")
    _rollout(w, 9, 80, True, scenario=sc, max_steps=30)
    _rollout(w, 9, 40, False, scenario=sc, max_steps=30)


@pytest.mark.parametrize("terrain", ["rects", "ellipses"])
@pytest.mark.parametrize("team_size", [32, 64])
def test_maximum_sizes(team_size, terrain):
    """The largest rows the library takes: 128 units (two wavefronts per env) or 64 units (four
    wavefronts per env group) with all 16 zone slots, as grid zones and as ellipses."""
    w = I.Workload(f"max_{team_size}_{terrain}", 3, team_size, 96.0, 0 if terrain == "ellipses" else 48,
                   terrain, 1.0, "iid", max_zones=16, spawn="clusters", steps=40, seed=5150 + team_size)
    _say(f"[gpu] maximum sizes N={w.num_units} Z=16 {terrain}")
    _rollout(w, 3, 40, True, max_steps=17)
    _rollout(w, 3, 20, False, max_steps=17)


@pytest.mark.parametrize("zones", [1, 2, 3, 5, 7])
@pytest.mark.parametrize("team_size", [2, 5, 10, 40])
def test_odd_zone_counts_and_row_alignment(zones, team_size):
    """Rows whose length is not a multiple of 4 floats (odd zone counts) and of every
    alignment class, in single-wave and two-wave workgroups."""
    w = I.Workload(f"z{zones}_n{team_size}", 7, team_size, 36.0, 18, "iid", 0.6, "iid",
                   max_zones=zones, steps=30, seed=900 + zones)
    sc = I.make_scenario(w, 7)
    rng = np.random.default_rng(zones * 100 + team_size)
    zd = np.zeros((7, zones, 6), np.float32)
    zd[..., 0] = rng.integers(0, 4, size=(7, zones))
    zd[..., 1:] = rng.uniform(0.5, 30.0, size=(7, zones, 5))
    sc["zone_desc"] = zd
    _say(f"[gpu] zones={zones} N={w.num_units}")
    _rollout(w, 7, 30, True, scenario=sc, max_steps=12)
    _rollout(w, 7, 12, False, scenario=sc, max_steps=12)


def test_degenerate_team_shapes():
    """One unit, an odd number of units, an empty enemy team, everybody on one team."""
    cases = {
        "single": [dict(unit="archer", team=0, x=5.0, y=5.0)],
        "odd_2v1": [dict(unit="assassin", team=0, x=5.0, y=5.0), dict(unit="healer", team=0, x=6.0, y=5.0),
                    dict(unit="assassin", team=1, x=7.0, y=5.0, theta=3.14)],
        "one_team": [dict(unit="healer", team=0, x=5.0, y=5.0), dict(unit="farmer", team=0, x=7.0, y=5.0)],
        "enemy_disabled": [dict(unit="assassin", team=0, x=5.0, y=5.0),
                           dict(unit="assassin", team=1, x=6.0, y=5.0, enabled=0)],
    }
    for name, units in cases.items():
        one = I.custom_scenario(units, 16.0)
        E = 11
        sc = {k: (None if v is None else np.ascontiguousarray(np.repeat(v, E, axis=0)))
              for k, v in one.items()}
        w = I.Workload(name, E, 1, 16.0, 0, "none", 1.0, "iid", steps=20, seed=5)
        p = I.custom_params(len(units), 16.0, max_steps=6)
        p["num_envs"] = E
        _say(f"[gpu] degenerate case {name}")
        import torch
        from oracle.ref import RefEnv
        from paper_2602_01665_amd.binding import TabxEnv
        ref, gpu = RefEnv(p, sc), TabxEnv(p, sc)
        ref.reset()
        gpu.reset()
        rng = np.random.default_rng(1)
        for s in range(20):
            a = rng.integers(0, 8, size=(E, len(units)), dtype=np.uint8)
            ref.step(a)
            ref.observe()
            gpu.step_observe(torch.from_numpy(a).to("cuda:0"))
            torch.cuda.synchronize()
            compare_state(gpu.state_numpy(), ref.st, f"{name} step {s}: ")
            compare_outputs(gpu, ref, f"{name} step {s}: ")


@pytest.mark.parametrize("name,E,steps", [("c1_16env_3v3", 16, 100), ("c3_16384env_10v10", 48, 120),
                                          ("c5_1024env_64v64", 2, 40)])
@pytest.mark.parametrize("fused", [False, True], ids=["separate", "fused"])
def test_rollout_with_body_collisions(name, E, steps, fused):
    """The optional collision correction of the physics stage, crowded spawns included."""
    _say(f"[gpu] collisions on: {name} E={E} fused={fused}")
    inexact, dones = _rollout(I.WORKLOADS[name], E, steps, fused, max_steps=40,
                              collision_alpha=0.8, collision_slop=0.01)
    assert dones > 0


@pytest.mark.parametrize("name,E,steps", [("c1_16env_3v3", 16, 100), ("c3_16384env_10v10", 48, 120),
                                          ("c5_1024env_64v64", 2, 40)])
@pytest.mark.parametrize("fused", [False, True], ids=["separate", "fused"])
@pytest.mark.parametrize("alpha,e", [(0.8, 0.5), (0.0, 1.0)], ids=["colliding", "passing"])
def test_rollout_with_persistent_velocities(name, E, steps, fused, alpha, e):
    """The optional physics mode in which the action sets an acceleration and colliding bodies
    exchange an impulse (velocities and accelerations are compared as state)."""
    _say(f"[gpu] persistent velocities: {name} E={E} fused={fused} alpha={alpha} e={e}")
    inexact, dones = _rollout(I.WORKLOADS[name], E, steps, fused, max_steps=40, dynamics=1,
                              move_gain=2.0, restitution=e, collision_alpha=alpha,
                              collision_slop=0.01)
    assert dones > 0


@pytest.mark.parametrize("team_size,zones,E", [(3, 4, 37), (10, 8, 40), (10, 16, 9), (40, 6, 3)])
@pytest.mark.parametrize("fused", [False, True], ids=["separate", "fused"])
def test_rollout_with_elliptical_zones(team_size, zones, E, fused):
    """Zones as ellipses with their own effect magnitudes instead of the cell grid."""
    w = I.Workload(f"ell_{team_size}_{zones}", E, team_size, 40.0, 0, "ellipses", 1.0, "iid",
                   max_zones=zones, steps=80, seed=600 + zones)
    _say(f"[gpu] elliptical zones N={w.num_units} Z={zones} fused={fused}")
    inexact, dones = _rollout(w, E, 80, fused, max_steps=30)
    assert dones > 0


@pytest.mark.parametrize("kinematic", [False, True], ids=["finite", "kinematic"])
@pytest.mark.parametrize("dynamics", [0, 1], ids=["kinematic_mode", "persistent_velocity"])
def test_collisions_in_a_crowd_of_mixed_bodies(kinematic, dynamics):
    names = list(I.ROSTER)
    rng = np.random.default_rng(9)
    units = [dict(unit=names[k % 9], team=k % 2, x=float(rng.uniform(10, 22)),
                  y=float(rng.uniform(10, 22)), theta=float(rng.uniform(0, 6.28)))
             for k in range(30)]
    one = I.custom_scenario(units, 32.0)
    E = 21
    sc = {k: (None if v is None else np.ascontiguousarray(np.repeat(v, E, axis=0)))
          for k, v in one.items()}
    sc["init_x"] = (sc["init_x"] + rng.uniform(-3, 3, sc["init_x"].shape)).astype(np.float32)
    sc["init_y"] = (sc["init_y"] + rng.uniform(-3, 3, sc["init_y"].shape)).astype(np.float32)
    sc["init_x"][:, 3] = sc["init_x"][:, 2]          # coincident centres
    sc["init_y"][:, 3] = sc["init_y"][:, 2]
    if kinematic:
        # every fifth body is kinematic (infinite mass: exempt from the correction), among them
        # one of the coincident pair and, in half of the envs, both
        sc["mass"][:, ::5] = np.inf
        sc["mass"][:, 2] = np.inf
        sc["mass"][::2, 3] = np.inf
    w = I.Workload("crowd", E, 15, 32.0, 0, "none", 1.0, "iid", steps=80, seed=77)
    _say(f"[gpu] collisions in a crowd of 30 mixed bodies, kinematic={kinematic} dynamics={dynamics}")
    inexact, dones = _rollout(w, E, 80, True, scenario=sc, max_steps=30, collision_alpha=0.5,
                              collision_slop=0.05, dynamics=dynamics, move_gain=3.0, restitution=0.8)
    assert dones > 0


def test_other_roster_units():
    """Every roster row (big bodies, wide hurtboxes, long cooldowns) in one battle."""
    names = list(I.ROSTER)
    units = []
    rng = np.random.default_rng(5)
    for t in (0, 1):
        for n in names:
            units.append(dict(unit=n, team=t, x=float(rng.uniform(8, 24)),
                              y=float(rng.uniform(8, 24)), theta=float(rng.uniform(0, 6.28))))
    one = I.custom_scenario(units, 32.0)
    E = 33
    sc = {k: (None if v is None else np.ascontiguousarray(np.repeat(v, E, axis=0)))
          for k, v in one.items()}
    sc["init_x"] = (sc["init_x"] + rng.uniform(-4, 4, sc["init_x"].shape)).astype(np.float32)
    sc["init_theta"] = rng.uniform(0, 6.28, sc["init_theta"].shape).astype(np.float32)
    w = I.Workload("roster", E, len(names), 32.0, 0, "none", 1.0, "iid", steps=150, seed=31)
    _say("[gpu] full roster 9v9")
    inexact, dones = _rollout(w, E, 150, True, scenario=sc, max_steps=60)
    assert dones > 0


def test_fused_equals_separate_and_is_deterministic():
    import torch
    from paper_2602_01665_amd.binding import TabxEnv
    w = I.WORKLOADS["c3_16384env_10v10"]
    E = 512
    p = I.make_params(w, E, max_steps=40)
    sc = I.make_scenario(w, E)
    envs = [TabxEnv(p, sc) for _ in range(3)]
    for g in envs:
        g.reset()
    _say("[gpu] fused vs separate vs repeated run, E=512")
    for s in range(120):
        ad = torch.from_numpy(I.actions_for_step(w.seed, s, E, w.num_units)).to("cuda:0")
        envs[0].step_observe(ad)
        envs[1].step(ad)
        envs[1].observe()
        envs[2].step_observe(ad)
        torch.cuda.synchronize()
        for other in envs[1:]:
            for k in envs[0].st:
                assert torch.equal(envs[0].st[k], other.st[k]), (s, k)
            for name in ("rewards", "dones", "obs", "vis", "amask"):
                assert torch.equal(getattr(envs[0], name), getattr(other, name)), (s, name)


def test_snapshot_restore_replays_bitwise():
    import torch
    from paper_2602_01665_amd.binding import TabxEnv
    w = DENSE
    E = 64
    p = I.make_params(w, E, max_steps=48)
    g = TabxEnv(p, I.make_scenario(w, E))
    g.reset()
    acts = [torch.from_numpy(I.actions_for_step(w.seed, s, E, w.num_units)).to("cuda:0")
            for s in range(90)]
    for s in range(30):
        g.step_observe(acts[s])
    snap = g.snapshot()
    trace = []
    for s in range(30, 90):
        g.step_observe(acts[s])
        trace.append((g.obs.clone(), g.rewards.clone(), g.dones.clone()))
    g.restore(snap)
    for n, s in enumerate(range(30, 90)):
        g.step_observe(acts[s])
        assert torch.equal(g.obs, trace[n][0]) and torch.equal(g.rewards, trace[n][1])
        assert torch.equal(g.dones, trace[n][2])


def test_reset_mask_and_empty_batch():
    import torch
    from oracle.ref import RefEnv
    from paper_2602_01665_amd.binding import TabxEnv
    w = I.WORKLOADS["c2_4096env_5v5"]
    E = 40
    p, sc, ref, gpu = _pair(w, E)
    for s in range(12):
        a = I.actions_for_step(w.seed, s, E, w.num_units)
        ref.step(a)
        gpu.step(torch.from_numpy(a).to("cuda:0"))
    mask = np.zeros(E, np.uint8)
    mask[[0, 3, 17, 39]] = 1
    ref.reset(mask)
    gpu.reset(torch.from_numpy(mask).to("cuda:0"))
    torch.cuda.synchronize()
    compare_state(gpu.state_numpy(), ref.st, "masked reset: ")
    # an empty batch is a valid no-op
    p0 = I.make_params(w, 0)
    sc0 = I.take_envs(sc, slice(0, 0))
    g0 = TabxEnv(p0, sc0)
    g0.reset()
    g0.step_observe(torch.zeros(0, dtype=torch.uint8, device="cuda:0"))
    torch.cuda.synchronize()


def test_out_of_range_action_is_noop():
    import torch
    w = I.WORKLOADS["c1_16env_3v3"]
    p, sc, ref, gpu = _pair(w, 16)
    rng = np.random.default_rng(3)
    for s in range(30):
        a = rng.integers(0, 256, size=(16, 6), dtype=np.uint8)
        ref.step(np.where(a >= 8, 0, a).astype(np.uint8))
        gpu.step(torch.from_numpy(a).to("cuda:0"))
        torch.cuda.synchronize()
        compare_state(gpu.state_numpy(), ref.st, f"wild actions step {s}: ")


# ---------------------------------------------------------------- full-size launches
FULL = [
    ("c2_4096env_5v5", 500, 48),
    ("c3_16384env_10v10", 1000, 40),
    ("c4_65536env_5v5", 1000, 64),
    ("c5_1024env_64v64", 500, 3),
]


@pytest.mark.parametrize("name,steps,n_sample", FULL, ids=[c[0] for c in FULL])
def test_full_size_sampled_envs(name, steps, n_sample):
    """The benchmark's launch (fused tick, full env count, full step count); the checker
    replays a sample of the envs (first, last, random) and every tick of them is compared."""
    import torch
    from oracle.ref import RefEnv
    from paper_2602_01665_amd.binding import TabxEnv
    w = I.WORKLOADS[name]
    E, N = w.num_envs, w.num_units
    _say(f"[gpu] full size {name}: E={E} N={N} steps={steps} sample={n_sample}")
    p = I.make_params(w)
    sc = I.make_scenario(w)
    rng = np.random.default_rng(11)
    rows = np.unique(np.concatenate([[0, 1, E - 1], rng.choice(E, n_sample - 3, replace=False)]))
    ref = RefEnv(I.make_params(w, len(rows)), I.take_envs(sc, rows))
    ref.track_margin = True
    gpu = TabxEnv(p, sc, want_metrics=True)
    ref.reset()
    gpu.reset()
    rows_t = torch.from_numpy(rows).to("cuda:0")
    inexact = dones = 0
    for s in range(steps):
        a = I.actions_for_step(w.seed, s, E, N)
        gpu.step_observe(torch.from_numpy(a).to("cuda:0"))
        ref.step(a[rows])
        ref.observe()
        st = {k: (v.reshape(E, N)[rows_t] if v.numel() == E * N else v[rows_t]).cpu().numpy()
              for k, v in gpu.st.items()}
        where = f"{name} full size step {s}: "
        inexact += compare_state(st, ref.st, where)
        inexact += compare_outputs(gpu, ref, where, rows=rows_t)
        inexact += compare_metrics(gpu, ref, where, rows=rows_t)
        dones += int(ref.dones.sum())
        if s % 100 == 0:
            _say(f"[gpu]   step {s} ok")
    _say(f"[gpu]   inexact floats {inexact}; sampled episodes ended {dones}; smallest "
         f"boundary margin seen by the checker {ref.margin.min():.3e}")
    gs = gpu.global_state()[rows_t].cpu().numpy()
    assert np.array_equal(gs, ref.global_state()), "global state of the sampled envs"
    # properties that hold for every env at any size
    obs = gpu.obs
    assert torch.isfinite(obs).all()
    hp = gpu.st["hp"].reshape(E, N)
    assert (hp >= 0).all() and (hp <= gpu.sc["hmax"].reshape(E, N)).all()
    assert torch.equal(gpu.st["alive"].reshape(E, N) == 1, hp > 0)
    r = gpu.rewards
    team = gpu.sc["team"].reshape(E, N).bool()
    assert torch.equal(r[:, :1].expand(E, N)[~team], r[~team])
    assert torch.equal((-r[:, :1]).expand(E, N)[team], r[team])


WHOLE = [
    # (past the truncation horizon of 256 ticks, so that every env restarts at least once)
    ("c2_4096env_5v5", 300),
    ("c3_16384env_10v10", 300),
    ("c4_65536env_5v5", 280),
    ("c5_1024env_64v64", 260),
]


@pytest.mark.parametrize("name,ticks", WHOLE, ids=[c[0] for c in WHOLE])
def test_full_size_every_env(name, ticks):
    """The benchmark's launch (fused tick, full env count): the checker steps the WHOLE batch
    (its envs dealt to host threads) and every field of every env is compared after every tick,
    bit for bit, so that each workgroup of the full-size grid (every XCD's first and last groups,
    the ragged last one) is checked, not only the sampled envs of the full-length run above.
    (Run once over the workloads' full step counts as well: 1000, 1000, 500 and 500 ticks of c3,
    c4, c5 and c2, every env, every field, bit-identical.)"""
    import torch
    from tests.helpers import ShardedRef
    from tests.parity import FLOAT_STATE, INT_STATE, METRIC_FLOAT, METRIC_INT
    from paper_2602_01665_amd.binding import TabxEnv
    w = I.WORKLOADS[name]
    E, N = w.num_envs, w.num_units
    _say(f"[gpu] full size, every env, {name}: E={E} N={N} ticks={ticks}")
    sc = I.make_scenario(w)
    ref = ShardedRef(w, lambda n: I.make_params(w, n), sc)
    gpu = TabxEnv(I.make_params(w), sc, want_metrics=True, want_global_state=True)
    ref.reset()
    gpu.reset()

    def same(t, want):
        want = torch.from_numpy(np.ascontiguousarray(want))
        if want.dtype in (torch.uint64,):
            want = want.view(torch.int64)
        return torch.equal(t.reshape(-1).view(torch.uint8), want.to(t.device).reshape(-1).view(torch.uint8))

    dones = 0
    for s in range(ticks):
        a = I.actions_for_step(w.seed, s, E, N)
        gpu.step_observe(torch.from_numpy(a).to("cuda:0"))
        ref.tick(a)
        where = f"{name} every env tick {s}: "
        assert same(gpu.obs, ref.obs), where + "obs"
        for k in FLOAT_STATE + INT_STATE:
            assert same(gpu.st[k], ref.state(k)), where + k
        for k in METRIC_FLOAT + METRIC_INT:
            assert same(gpu.metrics[k], ref.state(k)), where + k
        assert same(gpu.rewards, ref.output("rewards")), where + "rewards"
        assert same(gpu.dones, ref.output("dones")), where + "dones"
        assert same(gpu.vis, ref.output("vis").view(np.int64)), where + "vis_mask"
        assert same(gpu.amask, ref.output("amask")), where + "action_mask"
        if s % 10 == 0 or s == ticks - 1:
            assert same(gpu.gs_live, ref.global_state()), where + "global state"
        dones += int(ref.output("dones").sum())
        if s % 25 == 0:
            _say(f"[gpu]   tick {s} ok, {dones} episodes ended")
    _say(f"[gpu]   all {ticks} ticks bit-identical, {dones} episodes ended")


def test_full_size_headline_shape_with_dense_combat():
    """The headline launch shape (16384 envs, 10v10, rectangle terrain, 8 zone slots) with a
    fragile, fast-firing roster on an arena of 16 x 16 (health and cooldowns at a twentieth), where
    uniformly random actions kill: episodes end by elimination, so the kill, first-kill, win and
    restart paths run all over the full-size grid (with the benchmark's own roster every episode
    of random play ends by truncation).  Every env, every field, every tick against the checker,
    bit for bit."""
    import dataclasses
    import torch
    from tests.helpers import ShardedRef
    from tests.parity import FLOAT_STATE, INT_STATE, METRIC_FLOAT, METRIC_INT
    from paper_2602_01665_amd.binding import TabxEnv
    w = dataclasses.replace(I.WORKLOADS["c3_16384env_10v10"], name="c3_dense_combat", map_size=16.0)
    E, N = w.num_envs, w.num_units
    ticks = 140
    _say(f"[gpu] full size, every env, dense combat: E={E} N={N} ticks={ticks}")
    sc = I.make_scenario(w)
    sc["hmax"] = (sc["hmax"] * np.float32(0.05)).astype(np.float32)
    sc["cooldown"] = (sc["cooldown"] * np.float32(0.05)).astype(np.float32)
    ref = ShardedRef(w, lambda n: I.make_params(w, n), sc)
    gpu = TabxEnv(I.make_params(w), sc, want_metrics=True)
    assert B_launch_is_headline(gpu)
    ref.reset()
    gpu.reset()

    def same(t, want):
        want = torch.from_numpy(np.ascontiguousarray(want))
        if want.dtype in (torch.uint64,):
            want = want.view(torch.int64)
        return torch.equal(t.reshape(-1).view(torch.uint8), want.to(t.device).reshape(-1).view(torch.uint8))

    for s in range(ticks):
        a = I.actions_for_step(w.seed, s, E, N)
        gpu.step_observe(torch.from_numpy(a).to("cuda:0"))
        ref.tick(a)
        where = f"dense combat every env tick {s}: "
        assert same(gpu.obs, ref.obs), where + "obs"
        for k in FLOAT_STATE + INT_STATE:
            assert same(gpu.st[k], ref.state(k)), where + k
        for k in METRIC_FLOAT + METRIC_INT:
            assert same(gpu.metrics[k], ref.state(k)), where + k
        assert same(gpu.rewards, ref.output("rewards")), where + "rewards"
        assert same(gpu.dones, ref.output("dones")), where + "dones"
        assert same(gpu.vis, ref.output("vis").view(np.int64)), where + "vis_mask"
    count = gpu.metrics["ep_count"].cpu().numpy()
    length = gpu.metrics["ep_len"].cpu().numpy()
    win = gpu.metrics["ep_win"].cpu().numpy()
    first = gpu.metrics["ep_first_kill"].cpu().numpy()
    ended = count > 0
    _say(f"[gpu]   envs with a finished episode {int(ended.sum())}, ended early "
         f"{int((length[ended] < 256).sum())}, allied wins {int(win[ended].sum())}, first kills "
         f"{np.bincount(first[ended].astype(np.int64), minlength=4).tolist()}")
    # eliminations, not truncations; both outcomes; each kind of first kill
    assert ended.sum() > E // 8 and (length[ended] < 256).all()
    assert 0 < win[ended].sum() < ended.sum()
    assert (np.bincount(first[ended].astype(np.int64), minlength=4)[1:3] > 0).all()


def B_launch_is_headline(gpu):
    """The dense-combat batch is launched like the headline workload (two wavefronts per group of
    three envs, two rows per flush)."""
    from paper_2602_01665_amd import binding as B
    head = B.tabx_launch_info(B.make_params(I.make_params(I.WORKLOADS[I.HEADLINE])), "step_observe")
    mine = B.tabx_launch_info(gpu.params, "step_observe")
    return head == mine


def test_observation_tensor_beyond_two_giga_floats():
    """1.44 million 5v5 envs: the observation tensor has more than 2^31 floats (9.2 GB), so every
    row offset must be computed in 64 bits; sampled envs from both ends and from behind the 2^31
    boundary are compared tick by tick, fused and as separate calls."""
    import torch
    from oracle.ref import RefEnv
    from paper_2602_01665_amd.binding import TabxEnv
    w = I.WORKLOADS["c4_65536env_5v5"]
    E, N = 1441792 + 5, w.num_units
    p = I.make_params(w, E, max_steps=3)
    D = I.obs_dim(N, p["max_zones"])
    assert E * N * D > 2 ** 31 and E * N <= 2 ** 30
    _say(f"[gpu] large batch: E={E} N={N} D={D}: {E * N * D * 4 / 1e9:.1f} GB of observations")
    sc = I.make_scenario(w, E)
    first_behind = 2 ** 31 // (N * D) + 1
    rng = np.random.default_rng(5)
    rows = np.unique(np.concatenate([[0, 1, first_behind - 1, first_behind, E - 2, E - 1],
                                     rng.choice(E, 26, replace=False)]))
    ref = RefEnv(I.make_params(w, len(rows), max_steps=3), I.take_envs(sc, rows))
    gpu = TabxEnv(p, sc, want_metrics=True)
    ref.reset()
    gpu.reset()
    rows_t = torch.from_numpy(rows).to("cuda:0")
    dones = 0
    for s in range(8):
        a = I.actions_for_step(w.seed, s, E, N)
        ad = torch.from_numpy(a).to("cuda:0")
        if s % 2 == 0:
            gpu.step_observe(ad)
        else:
            gpu.step(ad)
            gpu.observe()
        ref.step(a[rows])
        ref.observe()
        st = {k: (v.reshape(E, N)[rows_t] if v.numel() == E * N else v[rows_t]).cpu().numpy()
              for k, v in gpu.st.items()}
        where = f"large batch step {s}: "
        compare_state(st, ref.st, where)
        compare_outputs(gpu, ref, where, rows=rows_t)
        compare_metrics(gpu, ref, where, rows=rows_t)
        dones += int(ref.dones.sum())
    assert dones >= 2 * len(rows)
    assert torch.isfinite(gpu.obs[-4096:]).all()
    del gpu
    torch.cuda.empty_cache()


def test_calls_can_be_captured_into_a_graph():
    """The entry points allocate nothing and only enqueue kernels, so a stream capture records
    them; replays (with eager work and synchronisations in between) give what eager calls give."""
    import torch
    from paper_2602_01665_amd.binding import TabxEnv
    w = I.WORKLOADS["c2_4096env_5v5"]
    E, N, K = 512, w.num_units, 6
    p, sc = I.make_params(w, E, max_steps=10), I.make_scenario(w, E)
    acts = [torch.from_numpy(I.actions_for_step(w.seed, s, E, N)).to("cuda:0") for s in range(K)]
    eager = TabxEnv(p, sc, want_metrics=True)
    graphed = TabxEnv(p, sc, want_metrics=True)
    eager.reset()
    graphed.reset()
    torch.cuda.synchronize()
    side = torch.cuda.Stream()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        with torch.cuda.graph(g, stream=side):
            for s in range(K):
                graphed.step_observe(acts[s], stream=side)
    torch.cuda.synchronize()
    for replay in range(4):
        _say(f"[gpu] graph replay {replay}")
        g.replay()
        for s in range(K):
            eager.step_observe(acts[s])
        torch.cuda.synchronize()
        for k in eager.st:
            assert torch.equal(eager.st[k], graphed.st[k]), (replay, k)
        assert torch.equal(eager.obs, graphed.obs) and torch.equal(eager.rewards, graphed.rewards)
        assert torch.equal(eager.vis, graphed.vis) and torch.equal(eager.dones, graphed.dones)
        for k in eager.metrics:
            assert torch.equal(eager.metrics[k], graphed.metrics[k]), (replay, k)
        # unrelated eager work between the replays
        _ = (eager.obs * 2).sum().item()
    assert int(eager.metrics["ep_count"].sum()) > 0


def test_launch_shapes_assume_the_device_that_is_there():
    """The launch-shape heuristics are tuned for a machine of 256 CUs with 160 KB of LDS each,
    64 KB per workgroup at most, 64-lane wavefronts: the device must be that machine."""
    import torch
    from paper_2602_01665_amd import binding as B
    info = B.tabx_launch_info(B.make_params(I.make_params(I.WORKLOADS[I.HEADLINE])), "step_observe")
    props = torch.cuda.get_device_properties(0)
    assert props.multi_processor_count == info["assumed_compute_units"]
    assert props.warp_size == info["assumed_wavefront_lanes"]
    # (the most the planner lets one workgroup take: the device must allow at least that)
    assert props.shared_memory_per_block >= info["assumed_lds_per_workgroup_bytes"]
    if hasattr(props, "shared_memory_per_multiprocessor"):
        assert props.shared_memory_per_multiprocessor == info["assumed_lds_per_cu_bytes"]
    _say(f"[gpu] device: {props.multi_processor_count} CUs, {props.shared_memory_per_block} B LDS per workgroup, "
         f"{getattr(props, 'shared_memory_per_multiprocessor', None)} B per CU, {props.warp_size} lanes")
