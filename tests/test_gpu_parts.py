"""A batch processed as several parts (TabxParams.env_id_offset, TabxEnv.parts) gives bit for bit
what the whole batch gives: state, outputs, metrics, global state, the level bank's draws and the
heuristic policy's decisions, with the parts on streams of their own."""
import sys

import numpy as np
import pytest

from paper_2602_01665_amd import inputs as I

pytestmark = pytest.mark.gpu


def _say(msg):
    print(msg, flush=True)
    sys.stdout.flush()


def _same(a, b, what):
    import torch
    assert torch.equal(a, b), what


@pytest.mark.parametrize("name,E,k,levels", [
    ("c3_16384env_10v10", 50, 3, 4),          # ragged parts, level bank, scripted adversaries
    ("c3e_16384env_10v10_ellipses", 37, 2, 0),
    ("c2_4096env_5v5", 4096, 2, 0),           # parts larger than one residency round
    ("c5_1024env_64v64", 6, 2, 3),
])
def test_parts_equal_the_whole_batch(name, E, k, levels):
    import torch
    from paper_2602_01665_amd.binding import TabxEnv
    w = I.WORKLOADS[name]
    N = w.num_units
    _say(f"[gpu] parts: {name} E={E} k={k} levels={levels}")
    p = I.make_params(w, E, max_steps=13, num_levels=levels, level_seed=5)
    sc = I.make_scenario(w, levels if levels else E)
    whole = TabxEnv(p, sc, want_metrics=True, want_global_state=True)
    split = TabxEnv(p, sc, want_metrics=True, want_global_state=True)
    parts = split.parts(k)
    assert sum(q.E for q in parts) == E and [q.first_env for q in parts] == sorted(q.first_env for q in parts)
    streams = [torch.cuda.Stream() for _ in parts]
    pol = I.policy("medium", 9)
    team = torch.from_numpy(np.ascontiguousarray(
        I.make_scenario(w, E)["team"] if not levels else np.tile(np.arange(N) >= N // 2, (E, 1)),
        np.uint8)).to("cuda:0")
    whole.reset()
    whole.prime_scripted(pol, team)
    for q, st in zip(parts, streams):
        sl = slice(q.first_env, q.first_env + q.E)
        q.reset(stream=st)
        q.prime_scripted(pol, team[sl], st)
    torch.cuda.synchronize()
    for s in range(40):
        a = torch.from_numpy(I.actions_for_step(w.seed, s, E, N)).to("cuda:0")
        a2 = a.clone()
        whole.scripted_step_observe(pol, team, a)
        for q, st in zip(parts, streams):
            sl = slice(q.first_env, q.first_env + q.E)
            q.scripted_step_observe(pol, team[sl], a2[sl], st)
        torch.cuda.synchronize()
        where = f"{name} tick {s}: "
        _same(a, a2, where + "actions written back")
        for n in whole.st:
            _same(whole.st[n], split.st[n], where + n)
        for n in whole.metrics:
            _same(whole.metrics[n], split.metrics[n], where + n)
        for n in whole.mem:
            _same(whole.mem[n], split.mem[n], where + n)
        _same(whole.obs, split.obs, where + "obs")
        _same(whole.rewards, split.rewards, where + "rewards")
        _same(whole.dones, split.dones, where + "dones")
        _same(whole.vis, split.vis, where + "vis_mask")
        _same(whole.amask, split.amask, where + "action_mask")
        _same(whole.gs_live, split.gs_live, where + "global state")
    assert int(whole.metrics["ep_count"].sum()) >= E        # episodes ended, levels were drawn


def test_a_part_matches_the_checker_under_its_original_env_indices():
    """The second part of a batch (env_id_offset = its first env) against the CPU checker that
    replays those envs with their original indices: level draws and scripted decisions agree."""
    import torch
    from oracle.ref import RefEnv
    from paper_2602_01665_amd.binding import TabxEnv
    from tests.parity import compare_metrics, compare_outputs, compare_state
    w = I.WORKLOADS["c3_16384env_10v10"]
    E, N, L = 40, w.num_units, 5
    p = I.make_params(w, E, max_steps=15, num_levels=L, level_seed=11)
    sc = I.make_scenario(w, L)
    batch = TabxEnv(p, sc, want_metrics=True, want_global_state=True)
    part = batch.parts(2)[1]
    rows = np.arange(part.first_env, part.first_env + part.E)
    _say(f"[gpu] part [{rows[0]}, {rows[-1]}] of {E} envs against the checker")
    ref = RefEnv(dict(p, num_envs=len(rows), env_ids=rows), sc)
    ref.st["next_level"][:] = rows % L
    ref.reset()
    part.reset()
    pol = I.policy("advanced", 2)
    assert (sc["team"] == sc["team"][0]).all()
    ctl = np.broadcast_to(sc["team"][0], (len(rows), N)).astype(np.uint8)
    ctl_d = torch.from_numpy(np.ascontiguousarray(ctl)).to("cuda:0")
    dones = 0
    for s in range(60):
        a = np.ascontiguousarray(I.actions_for_step(w.seed, s, E, N)[rows])
        ad = torch.from_numpy(a).to("cuda:0")
        part.policy_step_observe(pol, ctl_d, ad)
        ref.policy_step(pol, ctl, a)
        ref.observe()
        torch.cuda.synchronize()
        where = f"part tick {s}: "
        assert np.array_equal(ad.cpu().numpy(), a), where + "actions"
        compare_state(part.state_numpy(), ref.st, where)
        compare_outputs(part, ref, where)
        compare_metrics(part, ref, where)
        assert np.array_equal(part.mem["mem_valid"].view(len(rows), N).cpu().numpy(),
                              ref.mem["mem_valid"]), where + "mem_valid"
        dones += int(ref.dones.sum())
    assert dones > len(rows)
    # the first part's envs were never touched
    assert float(batch.obs[:part.first_env].abs().sum()) == 0.0
