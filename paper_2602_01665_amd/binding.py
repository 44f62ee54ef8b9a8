"""Thin Python binding of libtabx.so (the C ABI declared in include/tabx.h).

Argument marshalling only: every stage of the environment tick runs inside the
HIP kernels.  PyTorch owns the device memory and the stream; this module turns
tensors into the pointer structs the library takes.  There is no CPU fallback:
if the library has not been built, importing fails loudly.
"""
from __future__ import annotations

import ctypes as C
import os

import torch

_PKG = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_PKG, "libtabx.so")

_F = C.POINTER(C.c_float)
_U8 = C.POINTER(C.c_uint8)

SCENARIO_FLOAT = ("init_x", "init_y", "init_theta", "hmax", "radius", "mass", "speed", "dmg",
                  "range", "cooldown", "sight_angle", "sight_cos_half", "sight_range",
                  "hurt_halfwidth")
STATE_FLOAT = ("x", "y", "vx", "vy", "theta", "hp", "cd", "reveal", "cur_speed")

EXPORTS = ("tabx_obs_dim", "tabx_num_actions", "tabx_reset", "tabx_step", "tabx_observe",
           "tabx_step_observe", "tabx_global_state", "tabx_heuristic_actions",
           "tabx_policy_step_observe", "tabx_scripted_step_observe", "tabx_part", "tabx_launch_info",
           "tabx_strerror")

_I8 = C.POINTER(C.c_int8)
_I32 = C.POINTER(C.c_int32)
METRICS = (("ret_run", _F, torch.float32), ("kill_run", _I8, torch.int8),
           ("ep_count", _I32, torch.int32), ("ep_len", _I32, torch.int32),
           ("ep_return", _F, torch.float32), ("ep_win", _I8, torch.int8),
           ("ep_first_kill", _I8, torch.int8))


LEVELS = ("level", "next_level", "level_draws")


class TabxParams(C.Structure):
    _fields_ = [(n, C.c_int32) for n in
                ("num_envs", "num_units", "grid_w", "grid_h", "max_zones", "max_steps")] + \
               [(n, C.c_float) for n in
                ("map_w", "map_h", "cell_size", "dt", "turn_rate", "lava_dps", "swamp_mult",
                 "reveal_time", "boundary_frac", "collision_alpha", "collision_slop")] + \
               [("zone_shapes", C.c_int32), ("num_levels", C.c_int32), ("level_seed", C.c_uint32),
                ("hurtbox_cone", C.c_int32), ("hit_all", C.c_int32),
                ("env_id_offset", C.c_int32), ("dynamics", C.c_int32),
                ("move_gain", C.c_float), ("restitution", C.c_float)]


class TabxScenario(C.Structure):
    _fields_ = [(n, _F) for n in SCENARIO_FLOAT] + \
               [("team", _U8), ("enabled", _U8), ("terrain", C.POINTER(C.c_int8)),
                ("zone_desc", _F)]


class TabxState(C.Structure):
    _fields_ = [(n, _F) for n in STATE_FLOAT] + \
               [("alive", _U8), ("t", C.POINTER(C.c_int32)), ("phi_prev", _F)] + \
               [(n, t) for n, t, _ in METRICS] + \
               [(n, _I32) for n in LEVELS] + [("global_state", _F), ("ax", _F), ("ay", _F)]


class TabxError(RuntimeError):
    pass


class TabxPolicy(C.Structure):
    _fields_ = [("epsilon", C.c_float), ("xi", C.c_float), ("assassin_speed", C.c_float),
                ("ranger_range", C.c_float), ("seed", C.c_uint32)]


class TabxPolicyMemory(C.Structure):
    _fields_ = [("mem_x", _F), ("mem_y", _F), ("mem_valid", _U8), ("next_action", _U8)]


def load_library(path: str = LIB_PATH) -> C.CDLL:
    if not os.path.exists(path):
        raise ImportError(
            f"{path} is missing: build it with `python -m paper_2602_01665_amd.build` "
            "(hipcc, gfx950).  There is no fallback path.")
    lib = C.CDLL(path)
    P, S, T, V = C.POINTER(TabxParams), C.POINTER(TabxScenario), C.POINTER(TabxState), C.c_void_p
    lib.tabx_obs_dim.argtypes = [P]
    lib.tabx_num_actions.argtypes = []
    lib.tabx_reset.argtypes = [P, S, T, V, V]
    lib.tabx_step.argtypes = [P, S, T, V, V, V, V]
    lib.tabx_observe.argtypes = [P, S, T, V, V, V, V]
    lib.tabx_step_observe.argtypes = [P, S, T, V, V, V, V, V, V, V]
    lib.tabx_global_state.argtypes = [P, S, T, V, V]
    lib.tabx_heuristic_actions.argtypes = [P, S, T, C.POINTER(TabxPolicy),
                                           C.POINTER(TabxPolicyMemory), V, V, V]
    lib.tabx_policy_step_observe.argtypes = [P, S, T, C.POINTER(TabxPolicy),
                                             C.POINTER(TabxPolicyMemory)] + [V] * 8
    lib.tabx_scripted_step_observe.argtypes = lib.tabx_policy_step_observe.argtypes
    lib.tabx_strerror.argtypes = [C.c_int]
    lib.tabx_strerror.restype = C.c_char_p
    for name in EXPORTS[:-1]:
        getattr(lib, name).restype = C.c_int
    return lib


_lib = load_library()


def _check(rc: int, what: str):
    if rc != 0:
        raise TabxError(f"{what}: {_lib.tabx_strerror(rc).decode()} ({rc})")


def _ptr(t):
    return None if t is None else C.c_void_p(t.data_ptr())


def _cast(t, typ):
    return C.cast(C.c_void_p(t.data_ptr()), typ) if t is not None else C.cast(None, typ)


def make_params(p: dict) -> TabxParams:
    return TabxParams(**{k: p.get(k, 0) for k, _ in TabxParams._fields_})


def tabx_obs_dim(params: TabxParams) -> int:
    d = _lib.tabx_obs_dim(C.byref(params))
    if d < 0:
        _check(d, "tabx_obs_dim")
    return d


def tabx_part(params: TabxParams, scenario: TabxScenario, state: TabxState, first_env: int,
              count: int):
    """The structs of the envs [first_env, first_env + count) of a batch."""
    pp, psc, pst = TabxParams(), TabxScenario(), TabxState()
    _check(_lib.tabx_part(C.byref(params), C.byref(scenario), C.byref(state), int(first_env),
                          int(count), C.byref(pp), C.byref(psc), C.byref(pst)), "tabx_part")
    return pp, psc, pst


class TabxLaunchInfo(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("workgroups", "threads_per_workgroup", "envs_per_workgroup",
                                          "wavefronts_per_env_group", "rows_per_flush",
                                          "dynamic_lds_bytes", "assumed_compute_units",
                                          "assumed_lds_per_cu_bytes",
                                          "assumed_lds_per_workgroup_bytes",
                                          "assumed_wavefront_lanes")]


CALLS = {"reset": 0, "step": 1, "observe": 2, "step_observe": 3, "heuristic_actions": 4,
         "policy_step_observe": 5, "scripted_step_observe": 6}


def tabx_launch_info(params: TabxParams, call: str) -> dict:
    """How the library would lay the call out (host only, nothing is enqueued)."""
    info = TabxLaunchInfo()
    _check(_lib.tabx_launch_info(C.byref(params), CALLS[call], C.byref(info)), "tabx_launch_info")
    return {n: getattr(info, n) for n, _ in TabxLaunchInfo._fields_}


def tabx_num_actions() -> int:
    return _lib.tabx_num_actions()


def _stream_ptr(stream):
    if stream is None:
        stream = torch.cuda.current_stream()
    return C.c_void_p(stream.cuda_stream)


def tabx_reset(params, scenario, state, env_mask=None, stream=None):
    _check(_lib.tabx_reset(C.byref(params), C.byref(scenario), C.byref(state), _ptr(env_mask),
                           _stream_ptr(stream)), "tabx_reset")


def tabx_step(params, scenario, state, actions, rewards, dones, stream=None):
    _check(_lib.tabx_step(C.byref(params), C.byref(scenario), C.byref(state), _ptr(actions),
                          _ptr(rewards), _ptr(dones), _stream_ptr(stream)), "tabx_step")


def tabx_observe(params, scenario, state, obs, vis_mask=None, action_mask=None, stream=None):
    _check(_lib.tabx_observe(C.byref(params), C.byref(scenario), C.byref(state), _ptr(obs),
                             _ptr(vis_mask), _ptr(action_mask), _stream_ptr(stream)),
           "tabx_observe")


def tabx_step_observe(params, scenario, state, actions, rewards, dones, obs, vis_mask=None,
                      action_mask=None, stream=None):
    _check(_lib.tabx_step_observe(C.byref(params), C.byref(scenario), C.byref(state),
                                  _ptr(actions), _ptr(rewards), _ptr(dones), _ptr(obs),
                                  _ptr(vis_mask), _ptr(action_mask), _stream_ptr(stream)),
           "tabx_step_observe")


def tabx_global_state(params, scenario, state, out, stream=None):
    _check(_lib.tabx_global_state(C.byref(params), C.byref(scenario), C.byref(state), _ptr(out),
                                  _stream_ptr(stream)), "tabx_global_state")


def tabx_heuristic_actions(params, scenario, state, policy, memory, controlled, actions,
                           stream=None):
    _check(_lib.tabx_heuristic_actions(C.byref(params), C.byref(scenario), C.byref(state),
                                       C.byref(policy), C.byref(memory), _ptr(controlled),
                                       _ptr(actions), _stream_ptr(stream)),
           "tabx_heuristic_actions")


def tabx_policy_step_observe(params, scenario, state, policy, memory, controlled, actions,
                             rewards, dones, obs, vis_mask=None, action_mask=None, stream=None):
    _check(_lib.tabx_policy_step_observe(C.byref(params), C.byref(scenario), C.byref(state),
                                         C.byref(policy), C.byref(memory), _ptr(controlled),
                                         _ptr(actions), _ptr(rewards), _ptr(dones), _ptr(obs),
                                         _ptr(vis_mask), _ptr(action_mask), _stream_ptr(stream)),
           "tabx_policy_step_observe")


def tabx_scripted_step_observe(params, scenario, state, policy, memory, controlled, actions,
                               rewards, dones, obs, vis_mask=None, action_mask=None, stream=None):
    _check(_lib.tabx_scripted_step_observe(C.byref(params), C.byref(scenario), C.byref(state),
                                           C.byref(policy), C.byref(memory), _ptr(controlled),
                                           _ptr(actions), _ptr(rewards), _ptr(dones), _ptr(obs),
                                           _ptr(vis_mask), _ptr(action_mask),
                                           _stream_ptr(stream)),
           "tabx_scripted_step_observe")


class TabxEnv:
    """Device buffers of one batch of environments plus the calls on them."""

    def __init__(self, params: dict, scenario: dict, device="cuda:0", want_vis=True,
                 want_action_mask=True, want_metrics=False, want_global_state=False):
        self.device = torch.device(device)
        self.p = dict(params)
        self.params = make_params(self.p)
        E, N = self.p["num_envs"], self.p["num_units"]
        self.E, self.N = E, N
        L = self.p.get("num_levels", 0)
        rows = L if L > 0 else E           # scenario rows: a bank of levels, or one per env
        self.D = tabx_obs_dim(self.params)
        self.words = (N + 63) // 64
        dev = self.device

        def up(a, dtype):
            return torch.as_tensor(a, dtype=dtype).contiguous().to(dev)

        self.sc = {k: up(scenario[k], torch.float32).reshape(rows * N) for k in SCENARIO_FLOAT}
        self.sc["team"] = up(scenario["team"], torch.uint8).reshape(rows * N)
        self.sc["enabled"] = up(scenario["enabled"], torch.uint8).reshape(rows * N)
        ter = scenario.get("terrain")
        self.sc["terrain"] = None if ter is None else up(ter, torch.int8)
        zd = scenario.get("zone_desc") if self.p["max_zones"] > 0 else None
        self.sc["zone_desc"] = None if zd is None else up(zd, torch.float32)
        self.scenario = TabxScenario(
            **{k: _cast(self.sc[k], _F) for k in SCENARIO_FLOAT},
            team=_cast(self.sc["team"], _U8), enabled=_cast(self.sc["enabled"], _U8),
            terrain=_cast(self.sc["terrain"], C.POINTER(C.c_int8)),
            zone_desc=_cast(self.sc["zone_desc"], _F))

        self.st = {k: torch.zeros(E * N, dtype=torch.float32, device=dev) for k in STATE_FLOAT}
        self.st["alive"] = torch.zeros(E * N, dtype=torch.uint8, device=dev)
        self.st["t"] = torch.zeros(E, dtype=torch.int32, device=dev)
        self.st["phi_prev"] = torch.zeros(E, dtype=torch.float32, device=dev)
        self.metrics = {}
        if want_metrics:
            self.metrics = {n: torch.zeros(E, dtype=dt, device=dev) for n, _, dt in METRICS}
        if L > 0:
            self.st["level"] = torch.zeros(E, dtype=torch.int32, device=dev)
            self.st["next_level"] = (torch.arange(E, device=dev) % L).to(torch.int32)
            self.st["level_draws"] = torch.zeros(E, dtype=torch.int32, device=dev)
        if self.p.get("dynamics", 0) == 1:     # persistent velocities: the acceleration is state
            self.st["ax"] = torch.zeros(E * N, dtype=torch.float32, device=dev)
            self.st["ay"] = torch.zeros(E * N, dtype=torch.float32, device=dev)
        # global state written by every observing call (else only by global_state())
        self.gs_live = (torch.zeros(E, self.D, dtype=torch.float32, device=dev)
                        if want_global_state else None)
        self.state = self._state_struct(self.st, self.metrics, self.gs_live)
        self.gstate = None
        self.memory = None

        self.rewards = torch.zeros(E, N, dtype=torch.float32, device=dev)
        self.dones = torch.zeros(E, dtype=torch.uint8, device=dev)
        self.obs = torch.zeros(E, N, self.D, dtype=torch.float32, device=dev)
        self.vis = (torch.zeros(E, N, self.words, dtype=torch.int64, device=dev)
                    if want_vis else None)
        self.amask = (torch.zeros(E, N, dtype=torch.uint8, device=dev)
                      if want_action_mask else None)

    @staticmethod
    def _state_struct(st: dict, metrics: dict, global_state=None) -> TabxState:
        return TabxState(**{k: _cast(st[k], _F) for k in STATE_FLOAT},
                         alive=_cast(st["alive"], _U8),
                         t=_cast(st["t"], C.POINTER(C.c_int32)),
                         phi_prev=_cast(st["phi_prev"], _F),
                         **{n: _cast(metrics[n], t) for n, t, _ in METRICS if n in metrics},
                         **{n: _cast(st[n], _I32) for n in LEVELS if n in st},
                         **{n: _cast(st[n], _F) for n in ("ax", "ay") if n in st},
                         global_state=_cast(global_state, _F))

    def parts(self, k: int):
        """This batch as k consecutive parts that share its device tensors (views, nothing is
        copied): each part is a TabxEnv of its own with `env_id_offset` set, so calls on the
        parts compute exactly what the same calls on the whole batch would.  Launching the
        parts on different streams lets one part's launch fill the start and the end of
        another's.  Part boundaries are multiples of four envs (pointer alignment)."""
        E, N = self.E, self.N
        L = self.p.get("num_levels", 0)
        self._policy_memory()
        cuts = [min(E, (j * E // k + 3) // 4 * 4) for j in range(k)] + [E]
        out = []
        for start, stop in zip(cuts[:-1], cuts[1:]):
            count = stop - start
            if count <= 0:
                continue

            def unit(t):
                return t[start * N:stop * N]

            def env(t):
                return None if t is None else t[start:stop]

            v = object.__new__(TabxEnv)
            v.device, v.N, v.D, v.words, v.E = self.device, N, self.D, self.words, count
            v.p = dict(self.p, num_envs=count,
                       env_id_offset=self.p.get("env_id_offset", 0) + start)
            v.params, v.scenario, v.state = tabx_part(self.params, self.scenario, self.state,
                                                      start, count)
            names = list(SCENARIO_FLOAT) + ["team", "enabled"]
            v.sc = {n: (self.sc[n] if L > 0 else unit(self.sc[n])) for n in names}
            v.sc["terrain"] = self.sc["terrain"] if L > 0 else env(self.sc["terrain"])
            v.sc["zone_desc"] = self.sc["zone_desc"] if L > 0 else env(self.sc["zone_desc"])
            v.st = {n: (unit(t) if t.numel() == E * N else env(t)) for n, t in self.st.items()}
            v.metrics = {n: env(t) for n, t in self.metrics.items()}
            v.gs_live = env(self.gs_live)
            v.gstate = env(self.gstate)
            v.mem = {n: unit(t) for n, t in self.mem.items()}
            v.memory = TabxPolicyMemory(mem_x=_cast(v.mem["mem_x"], _F),
                                        mem_y=_cast(v.mem["mem_y"], _F),
                                        mem_valid=_cast(v.mem["mem_valid"], _U8),
                                        next_action=_cast(v.mem["next_action"], _U8))
            v.rewards, v.dones, v.obs = env(self.rewards), env(self.dones), env(self.obs)
            v.vis, v.amask = env(self.vis), env(self.amask)
            v.first_env = start
            out.append(v)
        return out

    def global_state(self, stream=None):
        if self.gstate is None:
            self.gstate = torch.zeros(self.E, 16 * self.N + 6 * self.p["max_zones"],
                                      dtype=torch.float32, device=self.device)
        tabx_global_state(self.params, self.scenario, self.state, self.gstate, stream)
        return self.gstate

    def _policy_memory(self):
        if self.memory is None:
            n = self.E * self.N
            self.mem = {"mem_x": torch.zeros(n, dtype=torch.float32, device=self.device),
                        "mem_y": torch.zeros(n, dtype=torch.float32, device=self.device),
                        "mem_valid": torch.zeros(n, dtype=torch.uint8, device=self.device),
                        "next_action": torch.zeros(n, dtype=torch.uint8, device=self.device)}
            self.memory = TabxPolicyMemory(mem_x=_cast(self.mem["mem_x"], _F),
                                           mem_y=_cast(self.mem["mem_y"], _F),
                                           mem_valid=_cast(self.mem["mem_valid"], _U8),
                                           next_action=_cast(self.mem["next_action"], _U8))
        return self.memory

    def heuristic_actions(self, policy: dict, controlled, actions, stream=None):
        """Fills `actions` (uint8 [E, N] on the device, in place) for the controlled units."""
        self._policy_memory()
        tabx_heuristic_actions(self.params, self.scenario, self.state, TabxPolicy(**policy),
                               self.memory, controlled, actions, stream)
        return actions

    def policy_step_observe(self, policy: dict, controlled, actions, stream=None):
        tabx_policy_step_observe(self.params, self.scenario, self.state, TabxPolicy(**policy),
                                 self._policy_memory(), controlled, actions, self.rewards,
                                 self.dones, self.obs, self.vis, self.amask, stream)

    def prime_scripted(self, policy: dict, controlled, stream=None):
        """Decides the scripted units' first actions (after a reset or any outside change)."""
        self._policy_memory()
        tabx_heuristic_actions(self.params, self.scenario, self.state, TabxPolicy(**policy),
                               self.memory, controlled, self.mem["next_action"], stream)

    def scripted_step_observe(self, policy: dict, controlled, actions, stream=None):
        tabx_scripted_step_observe(self.params, self.scenario, self.state, TabxPolicy(**policy),
                                   self._policy_memory(), controlled, actions, self.rewards,
                                   self.dones, self.obs, self.vis, self.amask, stream)

    def reset(self, env_mask=None, stream=None):
        tabx_reset(self.params, self.scenario, self.state, env_mask, stream)

    def step(self, actions, stream=None):
        tabx_step(self.params, self.scenario, self.state, actions, self.rewards, self.dones,
                  stream)

    def observe(self, stream=None):
        tabx_observe(self.params, self.scenario, self.state, self.obs, self.vis, self.amask,
                     stream)

    def step_observe(self, actions, stream=None):
        tabx_step_observe(self.params, self.scenario, self.state, actions, self.rewards,
                          self.dones, self.obs, self.vis, self.amask, stream)

    def snapshot(self) -> dict:
        return {k: v.clone() for k, v in self.st.items()}

    def restore(self, snap: dict):
        for k, v in snap.items():
            self.st[k].copy_(v)

    def state_numpy(self) -> dict:
        out = {}
        for k, v in self.st.items():
            a = v.cpu().numpy()
            per_env = k in ("t", "phi_prev") or k in LEVELS
            out[k] = a if per_env else a.reshape(self.E, self.N)
        return out
