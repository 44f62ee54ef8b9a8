"""Seeded random configurations: unit counts, batch sizes, terrain kinds, zone slots, optional
stages and launch forms drawn at random (all valid), each rolled out against the checker.
The point is the combinations: several wavefronts per env group with a level bank and elliptical zones, the
scripted tick with collisions and strikes on everybody, ragged counts with each of them."""
import sys

import numpy as np
import pytest

from paper_2602_01665_amd import inputs as I
from tests.parity import compare_metrics, compare_outputs, compare_state

pytestmark = pytest.mark.gpu


def _say(msg):
    print(msg, flush=True)
    sys.stdout.flush()


def _draw_config(seed):
    rng = np.random.default_rng([4711, seed])
    team = int(rng.choice([2, 3, 4, 5, 6, 8, 10, 12, 16, 21, 32, 40]))
    terrain = str(rng.choice(["none", "iid", "rects", "ellipses"]))
    grid = 0 if terrain in ("none", "ellipses") else int(rng.choice([16, 24, 32]))
    zones = {"none": int(rng.choice([0, 0, 3])), "iid": int(rng.choice([0, 2, 5])),
             "rects": int(rng.choice([8, 11])), "ellipses": int(rng.choice([4, 8, 13]))}[terrain]
    w = I.Workload(f"random_{seed}", 1, team, float(rng.choice([24.0, 40.0, 48.0])), grid, terrain,
                   0.65, str(rng.choice(["iid", "one_each"])) if team == 3 else "iid",
                   max_zones=zones, steps=60, seed=9000 + seed)
    G = max(1, 64 // (2 * team))
    E = int(rng.choice([1, G, G + 1, 3 * G + 2, 37]))
    over = dict(max_steps=int(rng.choice([9, 17, 30])),
                hit_all=int(rng.random() < 0.3), hurtbox_cone=int(rng.random() < 0.3),
                collision_alpha=float(rng.choice([0.0, 0.0, 0.8])))
    # (a stream of its own, so that the configurations drawn above stay what they were)
    rng2 = np.random.default_rng([4712, seed])
    if rng2.random() < 0.35:           # persistent velocities, with whatever collision setting was drawn
        over.update(dynamics=1, move_gain=float(rng2.choice([1.0, 2.0, 4.0])),
                    restitution=float(rng2.choice([0.0, 0.5, 1.0])))
        if rng2.random() < 0.5:
            over["collision_alpha"] = 0.8
    levels = int(rng.choice([0, 0, 3, 7]))
    form = str(rng.choice(["fused", "separate", "scripted"]))
    return w, E, over, levels, form


@pytest.mark.parametrize("seed", range(64))
def test_random_configuration(seed):
    import torch
    from oracle.ref import RefEnv
    from paper_2602_01665_amd.binding import TabxEnv
    w, E, over, L, form = _draw_config(seed)
    N = w.num_units
    _say(f"[gpu] random config {seed}: N={N} E={E} terrain={w.terrain} grid={w.grid} "
         f"zones={w.max_zones} levels={L} form={form} {over}")
    p = I.make_params(w, E, num_levels=L, level_seed=seed, **over)
    sc = I.make_scenario(w, L if L else E)
    ref = RefEnv(p, sc)
    gpu = TabxEnv(p, sc, want_metrics=True, want_global_state=True)
    ref.reset()
    gpu.reset()
    pol = I.policy("advanced", seed)
    if form == "scripted":
        gpu.prime_scripted(pol, None)
    ctl = np.ones((E, N), np.uint8)
    for s in range(w.steps):
        where = f"random config {seed} step {s}: "
        a = I.actions_for_step(w.seed, s, E, N)
        ad = torch.from_numpy(a).to(gpu.device)
        if form == "scripted":
            ref.policy_step(pol, ctl, a)
            gpu.scripted_step_observe(pol, None, ad)
            torch.cuda.synchronize()
            assert np.array_equal(ad.cpu().numpy(), a), where + "actions"
        else:
            ref.step(a)
            if form == "fused":
                gpu.step_observe(ad)
            else:
                gpu.step(ad)
                gpu.observe()
        ref.observe()
        torch.cuda.synchronize()
        compare_state(gpu.state_numpy(), ref.st, where)
        compare_outputs(gpu, ref, where)
        compare_metrics(gpu, ref, where)
        assert np.array_equal(gpu.gs_live.cpu().numpy(), ref.global_state()), \
            where + "global state written by the observe stage"
        if s % 10 == 0:
            g = gpu.global_state()
            torch.cuda.synchronize()
            assert np.array_equal(g.cpu().numpy(), ref.global_state()), where + "global state"
    assert int(ref.st["ep_count"].sum()) > 0
