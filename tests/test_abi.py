"""The C-ABI library loads and exports what include/tabx.h declares; host-side argument
validation returns the documented error codes without touching a GPU."""
import ctypes as C
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "tabx.h")


@pytest.fixture(scope="module")
def B():
    from paper_2602_01665_amd import build
    if build.is_stale():
        build.build()
    from paper_2602_01665_amd import binding
    return binding


def _declared():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(tabx_[a-z_]+)\s*\(", text)))


def test_every_declared_symbol_is_exported(B):
    names = _declared()
    assert set(names) == set(B.EXPORTS)
    lib = C.CDLL(B.LIB_PATH)
    for n in names:
        assert getattr(lib, n) is not None, n


def _params(B, **kw):
    base = dict(num_envs=4, num_units=20, grid_w=0, grid_h=0, max_zones=8, max_steps=10,
                map_w=8.0, map_h=8.0, cell_size=1.0, dt=0.25, turn_rate=1.0, lava_dps=1.0,
                swamp_mult=0.5, reveal_time=1.0, boundary_frac=0.1, collision_alpha=0.0,
                collision_slop=0.01, zone_shapes=0)
    base.update(kw)
    return B.TabxParams(**base)


def test_obs_dim_and_shape_errors(B):
    lib = B._lib
    assert lib.tabx_num_actions() == 8
    assert lib.tabx_obs_dim(C.byref(_params(B))) == 16 * 20 + 6 * 8
    assert lib.tabx_obs_dim(C.byref(_params(B, num_units=128, max_zones=0))) == 16 * 128
    assert lib.tabx_obs_dim(None) == -1
    for bad in (dict(num_units=0), dict(num_units=129), dict(max_zones=17), dict(max_zones=-1),
                dict(num_envs=-1), dict(grid_w=4), dict(max_steps=0), dict(zone_shapes=2),
                dict(zone_shapes=1, max_zones=0), dict(zone_shapes=1, grid_w=4, grid_h=4)):
        assert lib.tabx_obs_dim(C.byref(_params(B, **bad))) == -2, bad
    # per-unit arrays hold at most 2^30 elements (the kernels address them with 32-bit offsets)
    assert lib.tabx_obs_dim(C.byref(_params(B, num_envs=(1 << 30) // 20, num_units=20))) > 0
    assert lib.tabx_obs_dim(C.byref(_params(B, num_envs=(1 << 30) // 20 + 1, num_units=20))) == -2
    assert lib.tabx_obs_dim(C.byref(_params(B, num_levels=(1 << 30) // 20 + 1, num_units=20))) == -2
    assert lib.tabx_obs_dim(C.byref(_params(B, env_id_offset=-1))) == -2
    assert lib.tabx_obs_dim(C.byref(_params(B, env_id_offset=2 ** 31 - 5))) > 0
    assert lib.tabx_obs_dim(C.byref(_params(B, env_id_offset=2 ** 31 - 4))) == -2
    for bad in (dict(dt=0.0), dict(cell_size=-1.0), dict(map_w=float("nan")),
                dict(lava_dps=float("inf"))):
        assert lib.tabx_obs_dim(C.byref(_params(B, **bad))) == -5, bad
    for code in (0, -1, -2, -3, -4, -5, -99):
        assert len(lib.tabx_strerror(code)) > 0


def test_null_and_alignment_errors_come_back_before_any_launch(B):
    lib = B._lib
    p = _params(B, max_zones=0)
    sc, st = B.TabxScenario(), B.TabxState()
    assert lib.tabx_reset(C.byref(p), None, C.byref(st), None, None) == -1
    assert lib.tabx_reset(C.byref(p), C.byref(sc), C.byref(st), None, None) == -1
    # fake but non-null addresses: validation only inspects them, nothing is launched
    fake = 0x1000
    for k, _ in B.TabxScenario._fields_:
        if k not in ("terrain", "zone_desc"):
            setattr(sc, k, C.cast(C.c_void_p(fake), dict(B.TabxScenario._fields_)[k]))
    assert lib.tabx_reset(C.byref(p), C.byref(sc), None, None, None) == -1
    for k, typ in B.TabxState._fields_:
        setattr(st, k, C.cast(C.c_void_p(fake), typ))
    assert lib.tabx_step(C.byref(p), C.byref(sc), C.byref(st), None, None, None, None) == -1
    st.hp = C.cast(C.c_void_p(fake + 2), B._F)
    assert lib.tabx_reset(C.byref(p), C.byref(sc), C.byref(st), None, None) == -3
    st.hp = C.cast(C.c_void_p(fake), B._F)
    assert lib.tabx_observe(C.byref(p), C.byref(sc), C.byref(st), C.c_void_p(fake + 4), None,
                            None, None) == -3
    # terrain pointer must be present exactly when there is a grid
    pg = _params(B, max_zones=0, grid_w=4, grid_h=4)
    assert lib.tabx_reset(C.byref(pg), C.byref(sc), C.byref(st), None, None) == -1
    # an empty batch is a no-op that needs no buffers
    p0 = _params(B, num_envs=0)
    assert lib.tabx_step(C.byref(p0), None, None, None, None, None, None) == 0


def test_policy_level_and_variant_arguments_are_validated(B):
    lib = B._lib
    for bad in (dict(num_levels=-1), dict(hit_all=2), dict(hurtbox_cone=-1)):
        assert lib.tabx_obs_dim(C.byref(_params(B, **bad))) == -2, bad
    p = _params(B, max_zones=0)
    sc, st = B.TabxScenario(), B.TabxState()
    fake = 0x1000
    for k, typ in B.TabxScenario._fields_:
        if k not in ("terrain", "zone_desc"):
            setattr(sc, k, C.cast(C.c_void_p(fake), typ))
    for k, typ in B.TabxState._fields_:
        setattr(st, k, C.cast(C.c_void_p(fake), typ))
    pol = B.TabxPolicy(epsilon=0.1, xi=0.3, assassin_speed=1.4, ranger_range=10.0, seed=1)
    mem = B.TabxPolicyMemory()
    acts = C.c_void_p(fake)
    heur = lib.tabx_heuristic_actions
    # no policy, no memory struct, empty memory struct, no output
    assert heur(C.byref(p), C.byref(sc), C.byref(st), None, C.byref(mem), None, acts, None) == -1
    assert heur(C.byref(p), C.byref(sc), C.byref(st), C.byref(pol), None, None, acts, None) == -1
    assert heur(C.byref(p), C.byref(sc), C.byref(st), C.byref(pol), C.byref(mem), None, acts, None) == -1
    for k, typ in B.TabxPolicyMemory._fields_:
        if k != "next_action":
            setattr(mem, k, C.cast(C.c_void_p(fake), typ))
    assert heur(C.byref(p), C.byref(sc), C.byref(st), C.byref(pol), C.byref(mem), None, None, None) == -1
    bad_pol = B.TabxPolicy(epsilon=float("nan"), xi=0.3, assassin_speed=1.4, ranger_range=10.0, seed=1)
    assert heur(C.byref(p), C.byref(sc), C.byref(st), C.byref(bad_pol), C.byref(mem), None, acts, None) == -5
    # the scripted tick needs the buffer its decisions wait in
    assert lib.tabx_scripted_step_observe(C.byref(p), C.byref(sc), C.byref(st), C.byref(pol),
                                          C.byref(mem), None, acts, acts, acts, acts, None, None,
                                          None) == -1
    # a level bank needs its three per-env arrays
    pl = _params(B, max_zones=0, num_levels=3)
    st.next_level = C.cast(None, B._I32)
    assert lib.tabx_reset(C.byref(pl), C.byref(sc), C.byref(st), None, None) == -1
    st.next_level = C.cast(C.c_void_p(fake + 1), B._I32)
    assert lib.tabx_reset(C.byref(pl), C.byref(sc), C.byref(st), None, None) == -3


def test_part_structs_advance_every_pointer(B):
    """tabx_part is host arithmetic: per-unit pointers advance by first_env * N elements, per-env
    pointers by first_env, terrain / zone slots by first_env rows, NULL stays NULL, a bank of
    levels is left alone, env_id_offset accumulates."""
    lib = B._lib
    N, Z, gw, gh = 20, 8, 6, 5
    p = _params(B, num_envs=64, num_units=N, max_zones=Z, grid_w=gw, grid_h=gh, env_id_offset=7)
    base = 1 << 20

    def fake(struct):
        out = struct()
        for k, (name, typ) in enumerate(struct._fields_):
            setattr(out, name, C.cast(C.c_void_p(base * (k + 1)), typ))
        return out

    def addr(struct_obj, name):
        return C.cast(getattr(struct_obj, name), C.c_void_p).value or 0

    sc, st = fake(B.TabxScenario), fake(B.TabxState)
    st.kill_run = C.cast(None, type(st.kill_run))
    pp, psc, pst = B.tabx_part(p, sc, st, 12, 16)
    assert (pp.num_envs, pp.env_id_offset, pp.num_units) == (16, 19, N)
    for name, typ in B.TabxScenario._fields_:
        step = {"team": 1, "enabled": 1, "terrain": gw * gh, "zone_desc": 4 * 6 * Z}.get(name, 4 * N)
        if name in ("terrain", "zone_desc"):
            assert addr(psc, name) - addr(sc, name) == 12 * step, name
        else:
            assert addr(psc, name) - addr(sc, name) == 12 * N * (step // N if step >= N else step), name
    unit4 = {"x", "y", "vx", "vy", "theta", "hp", "cd", "reveal", "cur_speed", "ax", "ay"}
    size = {"alive": N, "t": 4, "phi_prev": 4, "ret_run": 4, "ep_count": 4, "ep_len": 4,
            "ep_return": 4, "ep_win": 1, "ep_first_kill": 1, "level": 4, "next_level": 4,
            "level_draws": 4, "global_state": 4 * (16 * N + 6 * Z)}
    for name, typ in B.TabxState._fields_:
        if name == "kill_run":
            assert addr(pst, name) == 0
            continue
        want = 12 * (4 * N if name in unit4 else size[name])
        assert addr(pst, name) - addr(st, name) == want, name
    # a bank of levels: the scenario arrays are shared by all parts
    pl = _params(B, num_envs=64, num_units=N, max_zones=Z, grid_w=gw, grid_h=gh, num_levels=3)
    _, psc, _ = B.tabx_part(pl, sc, st, 12, 16)
    for name, _ in B.TabxScenario._fields_:
        assert addr(psc, name) == addr(sc, name), name
    for first, count in ((-1, 4), (60, 5), (0, -1)):
        with pytest.raises(B.TabxError):
            B.tabx_part(p, sc, st, first, count)


def test_plain_c_client_compiles_and_links():
    """include/tabx.h is valid C11 and a C program links against the library with gcc alone
    (the program itself needs a GPU: tests/test_gpu_c_client.py runs it)."""
    import os
    from oracle import ref
    from tests import c_client
    ref.build()
    binary = c_client.build()
    assert os.access(binary, os.X_OK)


def test_launch_info_reports_the_layout_without_a_gpu(B):
    """tabx_launch_info is host-only: the shapes of the five workloads' fused ticks, and its errors."""
    from paper_2602_01665_amd import inputs as I
    want = {"c1_16env_3v3": (10, 4, 256), "c2_4096env_5v5": (6, 4, 256),
            "c3_16384env_10v10": (3, 2, 128), "c4_65536env_5v5": (6, 1, 64),
            "c5_1024env_64v64": (1, 2, 128)}
    for name, (envs, waves, threads) in want.items():
        w = I.WORKLOADS[name]
        p = B.make_params(I.make_params(w))
        info = B.tabx_launch_info(p, "step_observe")
        assert (info["envs_per_workgroup"], info["wavefronts_per_env_group"],
                info["threads_per_workgroup"]) == (envs, waves, threads), (name, info)
        groups = -(-w.num_envs // envs)
        assert groups <= info["workgroups"] < groups + 8          # rounded up to the eight XCDs
        assert 0 < info["dynamic_lds_bytes"] <= 64 * 1024
        assert B.tabx_launch_info(p, "reset")["dynamic_lds_bytes"] == 0
        # a stand-alone observe spreads an env group's observers over several workgroups
        # (one-wave envs: about four flushes of two rows each per workgroup)
        split = {"c1_16env_3v3": 2, "c2_4096env_5v5": 3, "c3_16384env_10v10": 3,
                 "c4_65536env_5v5": 3, "c5_1024env_64v64": 1}[name]
        assert B.tabx_launch_info(p, "observe")["workgroups"] == split * info["workgroups"]
    p = B.make_params(I.make_params(I.WORKLOADS["c1_16env_3v3"]))
    info = B.TabxLaunchInfo()
    import ctypes as C
    assert B._lib.tabx_launch_info(C.byref(p), 7, C.byref(info)) == -2       # unknown call
    assert B._lib.tabx_launch_info(C.byref(p), 3, None) == -1                # NULL
    assert B._lib.tabx_launch_info(None, 3, C.byref(info)) == -1
