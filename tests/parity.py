"""Element-by-element comparison of the HIP library with the CPU checker."""
import numpy as np

FLOAT_STATE = ("x", "y", "vx", "vy", "theta", "hp", "cd", "reveal", "cur_speed", "phi_prev")
INT_STATE = ("alive", "t")
LEVEL_STATE = ("level", "next_level", "level_draws")
FLOAT_TOL = 1e-5          # absolute, float32 fields (positions, headings, HP, rewards, obs)


def _cmp_float(name, got, want, where=""):
    got = np.asarray(got)
    want = np.asarray(want)
    assert got.shape == want.shape, (name, got.shape, want.shape)
    # (equal values are equal, infinities included: a kinematic body's mass is +inf)
    with np.errstate(invalid="ignore"):
        bad = ~((got == want) | (np.abs(got.astype(np.float64) - want.astype(np.float64)) <= FLOAT_TOL))
    if bad.any():
        idx = np.argwhere(bad)[0]
        raise AssertionError(f"{where}{name}: {int(bad.sum())} floats differ by more than "
                             f"{FLOAT_TOL}; first at {tuple(idx)}: gpu {got[tuple(idx)]!r} "
                             f"cpu {want[tuple(idx)]!r}")
    return int((got != want).sum())


def _cmp_int(name, got, want, where=""):
    got = np.asarray(got)
    want = np.asarray(want)
    assert got.shape == want.shape, (name, got.shape, want.shape)
    if not np.array_equal(got, want):
        idx = np.argwhere(got != want)[0]
        raise AssertionError(f"{where}{name}: {int((got != want).sum())} entries differ; first at "
                             f"{tuple(idx)}: gpu {got[tuple(idx)]!r} cpu {want[tuple(idx)]!r}")


def compare_state(gpu_state: dict, ref_state: dict, where="", rows=None):
    """gpu_state: numpy dict from TabxEnv.state_numpy(); rows: env indices of the GPU batch
    that correspond to the checker's envs (None = all)."""
    inexact = 0
    for k in FLOAT_STATE + tuple(k for k in ("ax", "ay") if k in ref_state):
        g = gpu_state[k] if rows is None else gpu_state[k][rows]
        inexact += _cmp_float(k, g, ref_state[k], where)
    for k in INT_STATE + tuple(k for k in LEVEL_STATE if k in ref_state):
        g = gpu_state[k] if rows is None else gpu_state[k][rows]
        _cmp_int(k, g, ref_state[k], where)
    return inexact


METRIC_FLOAT = ("ret_run", "ep_return")
METRIC_INT = ("kill_run", "ep_count", "ep_len", "ep_win", "ep_first_kill")


def compare_metrics(gpu, ref, where="", rows=None):
    """Episode metrics of a TabxEnv built with want_metrics=True against the checker's."""
    inexact = 0
    for k in METRIC_FLOAT + METRIC_INT:
        g = gpu.metrics[k] if rows is None else gpu.metrics[k][rows]
        g = g.cpu().numpy()
        if k in METRIC_FLOAT:
            inexact += _cmp_float(k, g, ref.st[k], where)
        else:
            _cmp_int(k, g, ref.st[k], where)
    return inexact


def compare_outputs(gpu, ref, where="", rows=None, check_obs=True):
    """gpu: TabxEnv (torch tensors), ref: RefEnv.  Returns the number of float entries that
    are within tolerance but not bit-identical."""
    def g(t):
        t = t if rows is None else t[rows]
        return t.cpu().numpy()
    inexact = 0
    inexact += _cmp_float("rewards", g(gpu.rewards), ref.rewards, where)
    _cmp_int("dones", g(gpu.dones), ref.dones, where)
    if check_obs:
        inexact += _cmp_float("obs", g(gpu.obs), ref.obs, where)
        _cmp_int("vis_mask", g(gpu.vis).view(np.uint64), ref.vis, where)
        _cmp_int("action_mask", g(gpu.amask), ref.amask, where)
        # discrete-valued observation features must agree exactly
        go, ro = g(gpu.obs), ref.obs
        N = ref.N
        cols = [12, 14, 15] + [16 + 16 * s + f for s in range(N - 1) for f in (12, 13, 14)]
        _cmp_int("obs discrete features", go[..., cols], ro[..., cols], where)
    return inexact
