"""Level bank (per-episode reconfiguration): HIP library vs CPU checker through the C ABI.

Same bar as the other parity tests; the level arrays (level, next_level, level_draws) are
integer state and must match exactly."""
import sys

import numpy as np
import pytest

from paper_2602_01665_amd import inputs as I
from tests.parity import compare_metrics, compare_outputs, compare_state

pytestmark = pytest.mark.gpu


def _say(msg):
    print(msg, flush=True)
    sys.stdout.flush()


def _bank(w, L, seed=0, vary_teams=True):
    """L levels drawn like the workload's scenario; some levels get disabled placeholders and
    reshuffled teams so that counts per team differ between levels."""
    sc = I.make_scenario(w, L, seed=w.seed + 77 + seed)
    rng = np.random.default_rng(seed + 5)
    N = w.num_units
    if vary_teams and N >= 4:
        for lv in range(L):
            if lv % 3 == 1:
                off = rng.choice(np.arange(1, N - 1), size=max(1, N // 5), replace=False)
                sc["enabled"][lv, off] = 0
            if lv % 3 == 2:
                flip = rng.choice(np.arange(1, N - 1), size=max(1, N // 4), replace=False)
                sc["team"][lv, flip] ^= 1
    return sc


def _rollout(w, E, L, steps, fused, policy=None, curriculum=False, **override):
    import torch
    from oracle.ref import RefEnv
    from paper_2602_01665_amd.binding import TabxEnv
    p = I.make_params(w, E, num_levels=L, level_seed=w.seed, **override)
    sc = _bank(w, L)
    ref = RefEnv(p, sc)
    gpu = TabxEnv(p, sc, want_metrics=True)
    ref.reset()
    gpu.reset()
    torch.cuda.synchronize()
    compare_state(gpu.state_numpy(), ref.st, "after reset: ")
    N = w.num_units
    team = None
    dones = 0
    seen = set()
    ctl = np.ones((E, N), np.uint8)
    for s in range(steps):
        where = f"{w.name} E={E} L={L} step {s}: "
        a = I.actions_for_step(w.seed, s, E, N)
        ad = torch.from_numpy(a).to(gpu.device)
        if curriculum and s % 7 == 3:
            # the caller's own choice for the next episodes of some envs
            pick = (np.arange(E) * 3 + s) % L
            mask = np.arange(E) % 2 == 0
            ref.st["next_level"][mask] = pick[mask]
            gpu.st["next_level"][torch.from_numpy(mask).to(gpu.device)] = \
                torch.from_numpy(pick[mask].astype(np.int32)).to(gpu.device)
        if policy:
            ref.policy_step(policy, ctl, a)
            if fused:
                gpu.policy_step_observe(policy, None, ad)
            else:
                gpu.heuristic_actions(policy, None, ad)
                gpu.step(ad)
                torch.cuda.synchronize()
                done = torch.from_numpy(ref.dones.astype(bool)).to(gpu.device)
                gpu.mem["mem_valid"].view(E, N)[done] = 0
                gpu.observe()
            torch.cuda.synchronize()
            assert np.array_equal(ad.cpu().numpy(), a), where + "actions"
        else:
            ref.step(a)
            if fused:
                gpu.step_observe(ad)
            else:
                gpu.step(ad)
                gpu.observe()
        ref.observe()
        torch.cuda.synchronize()
        compare_state(gpu.state_numpy(), ref.st, where)
        compare_outputs(gpu, ref, where)
        compare_metrics(gpu, ref, where)
        if s % 8 == 0:
            g = gpu.global_state()
            torch.cuda.synchronize()
            assert np.array_equal(g.cpu().numpy(), ref.global_state()), where + "global state"
        dones += int(ref.dones.sum())
        seen.update(ref.st["level"].tolist())
    return dones, seen


@pytest.mark.parametrize("fused", [False, True], ids=["separate", "fused"])
@pytest.mark.parametrize("name,E,L,steps,over", [
    ("c1_16env_3v3", 16, 4, 120, dict(max_steps=12)),
    ("c2_4096env_5v5", 61, 9, 150, dict(max_steps=20)),
    ("c3_16384env_10v10", 40, 6, 120, dict(max_steps=16)),
    ("c3e_16384env_10v10_ellipses", 40, 6, 120, dict(max_steps=16)),
    ("c5_1024env_64v64", 3, 4, 60, dict(max_steps=9)),
    # batch sizes at which the fused tick runs two wavefronts per env group, and one
    ("c3_16384env_10v10", 2400, 6, 50, dict(max_steps=16)),
    ("c4_65536env_5v5", 13000, 9, 50, dict(max_steps=16)),
], ids=lambda v: v if isinstance(v, str) else None)
def test_level_bank_rollouts(name, E, L, steps, over, fused):
    _say(f"[gpu] level bank {name} E={E} L={L} fused={fused}")
    dones, seen = _rollout(I.WORKLOADS[name], E, L, steps, fused, **over)
    _say(f"[gpu]   episodes ended {dones}, levels played {sorted(seen)}")
    assert dones > E and len(seen) == L


@pytest.mark.parametrize("team_size", [16, 23, 32])
def test_level_bank_with_large_teams(team_size):
    """32 to 64 units per env: the rows of an env group are written by four wavefronts, all of
    which follow the level switch."""
    import dataclasses
    third = team_size // 3
    w = dataclasses.replace(I.WORKLOADS["c3_16384env_10v10"], name=f"levels_{team_size}v{team_size}",
                            team_size=team_size, role_counts=(team_size - 2 * third, third, third))
    _say(f"[gpu] level bank {w.name}")
    dones, seen = _rollout(w, 7, 5, 80, True, max_steps=11)
    assert dones > 7 and len(seen) == 5


def test_curriculum_overrides_the_draws():
    _say("[gpu] level bank with caller-chosen next levels")
    dones, seen = _rollout(I.WORKLOADS["c2_4096env_5v5"], 50, 11, 140, True, curriculum=True,
                           max_steps=10)
    assert dones > 50 and len(seen) == 11


@pytest.mark.parametrize("fused", [False, True], ids=["separate", "fused"])
def test_level_bank_with_scripted_units(fused):
    _say(f"[gpu] level bank + heuristic policy fused={fused}")
    for name in ("c3_16384env_10v10", "c3e_16384env_10v10_ellipses"):
        dones, seen = _rollout(I.WORKLOADS[name], 30, 5, 120, fused,
                               policy=I.policy("advanced", 4), max_steps=24)
        assert dones > 30


def test_more_levels_than_envs_and_a_single_level():
    _say("[gpu] level bank: L > E and L = 1")
    w = I.WORKLOADS["c2_4096env_5v5"]
    dones, seen = _rollout(w, 7, 40, 160, True, max_steps=5)
    assert len(seen) > 20
    dones, seen = _rollout(w, 33, 1, 40, True, max_steps=8)
    assert seen == {0}


def test_missing_level_arrays_are_refused():
    import torch
    from paper_2602_01665_amd import binding as B
    w = I.WORKLOADS["c2_4096env_5v5"]
    p = I.make_params(w, 8, num_levels=3)
    env = B.TabxEnv(p, _bank(w, 3))
    st = dict(env.st)
    del st["next_level"]
    bad = B.TabxEnv._state_struct(st, {})
    with pytest.raises(B.TabxError):
        B.tabx_reset(env.params, env.scenario, bad, None)
    with pytest.raises(B.TabxError):
        B.tabx_reset(B.make_params(dict(p, num_levels=-1)), env.scenario, env.state, None)
