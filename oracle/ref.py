"""ctypes/numpy front end of the CPU checker (oracle/tabx_ref.cpp).

TEST INFRASTRUCTURE ONLY: imported by tests/, the smoke check and the
benchmark's CPU-baseline leg.  It never touches the GPU library.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "tabx_ref.cpp")
_LIB = os.path.join(_HERE, "libtabx_ref.so")
# A test may point the front end at another build of the checker (tests/test_oracle_mutations.py
# runs the pins against copies with planted mistakes); such a library is used as it is.
_OVERRIDE = os.environ.get("TABX_REF_LIB")

_F = C.POINTER(C.c_float)
_B = C.POINTER(C.c_ubyte)


_I8 = C.POINTER(C.c_byte)
_I32 = C.POINTER(C.c_int)


class RefParams(C.Structure):
    _fields_ = [(n, C.c_int) for n in
                ("num_envs", "num_units", "grid_w", "grid_h", "max_zones", "max_steps")] + \
               [(n, C.c_float) for n in
                ("map_w", "map_h", "cell_size", "dt", "turn_rate", "lava_dps", "swamp_mult",
                 "reveal_time", "boundary_frac", "collision_alpha", "collision_slop")] + \
               [("zone_shapes", C.c_int), ("num_levels", C.c_int), ("level_seed", C.c_uint),
                ("hurtbox_cone", C.c_int), ("hit_all", C.c_int), ("dynamics", C.c_int),
                ("move_gain", C.c_float), ("restitution", C.c_float), ("env_ids", _I32)]


_SC_FLOAT = ("init_x", "init_y", "init_theta", "hmax", "radius", "mass", "speed", "dmg",
             "range", "cooldown", "sight_angle", "sight_cos_half", "sight_range",
             "hurt_halfwidth")
_ST_FLOAT = ("x", "y", "vx", "vy", "theta", "hp", "cd", "reveal", "cur_speed")


class RefScenario(C.Structure):
    _fields_ = [(n, _F) for n in _SC_FLOAT] + [("team", _B), ("enabled", _B),
                                                ("terrain", C.POINTER(C.c_byte)),
                                                ("zone_desc", _F)]


_METRICS = (("ret_run", _F, np.float32), ("kill_run", _I8, np.int8), ("ep_count", _I32, np.int32),
            ("ep_len", _I32, np.int32), ("ep_return", _F, np.float32), ("ep_win", _I8, np.int8),
            ("ep_first_kill", _I8, np.int8))


_LEVELS = ("level", "next_level", "level_draws")


class RefState(C.Structure):
    _fields_ = [(n, _F) for n in _ST_FLOAT] + [("alive", _B), ("t", C.POINTER(C.c_int)),
                                                ("phi_prev", _F)] + \
               [(n, t) for n, t, _ in _METRICS] + \
               [(n, _I32) for n in _LEVELS] + [("ax", _F), ("ay", _F)]


class RefPolicy(C.Structure):
    _fields_ = [("epsilon", C.c_float), ("xi", C.c_float), ("assassin_speed", C.c_float),
                ("ranger_range", C.c_float), ("seed", C.c_uint)]


class RefPolicyMemory(C.Structure):
    _fields_ = [("mem_x", _F), ("mem_y", _F), ("mem_valid", _B)]


def build(force: bool = False) -> str:
    """Compiles the checker with g++ (no contraction, no fast-math)."""
    if force or not os.path.exists(_LIB) or \
            os.path.getmtime(_LIB) < max(os.path.getmtime(_SRC),
                                         os.path.getmtime(os.path.join(_HERE, "tabx_ref.h"))):
        cmd = ["g++", "-O2", "-std=c++17", "-ffp-contract=off", "-fno-fast-math",
               "-Wall", "-Wextra", "-shared", "-fPIC", _SRC, "-o", _LIB]
        subprocess.run(cmd, check=True)
    return _LIB


_lib = None


def lib():
    global _lib
    if _lib is None:
        if _OVERRIDE:
            _lib = C.CDLL(_OVERRIDE)
        else:
            build()
            _lib = C.CDLL(_LIB)
        _lib.tabx_ref_obs_dim.restype = C.c_int
        _lib.tabx_ref_sincos.argtypes = [C.c_float, _F, _F]
        _lib.tabx_ref_sincos_n.argtypes = [_F, C.c_int, _F, _F]
        _lib.tabx_ref_hash.restype = C.c_uint
        _lib.tabx_ref_hash.argtypes = [C.c_uint] * 5
        _lib.tabx_ref_heuristic_actions.restype = None
        for fn in (_lib.tabx_ref_reset, _lib.tabx_ref_step, _lib.tabx_ref_observe,
                   _lib.tabx_ref_sincos, _lib.tabx_ref_sincos_n, _lib.tabx_ref_global_state):
            fn.restype = None
    return _lib


def ref_sincos(theta: float):
    s, c = C.c_float(), C.c_float()
    lib().tabx_ref_sincos(C.c_float(float(np.float32(theta))), C.byref(s), C.byref(c))
    return np.float32(s.value), np.float32(c.value)


def ref_sincos_n(theta):
    th = np.ascontiguousarray(theta, np.float32)
    s = np.empty_like(th)
    c = np.empty_like(th)
    lib().tabx_ref_sincos_n(th.ctypes.data_as(_F), th.size, s.ctypes.data_as(_F),
                            c.ctypes.data_as(_F))
    return s, c


def _ptr(a, typ):
    return None if a is None else a.ctypes.data_as(typ)


class RefEnv:
    """Batched CPU environment: numpy state, calls into the checker per tick."""

    def __init__(self, params: dict, scenario: dict, metrics: bool = True):
        self.p = dict(params)
        self.metrics = metrics
        E, N = self.p["num_envs"], self.p["num_units"]
        self.E, self.N = E, N
        L = self.p.get("num_levels", 0)
        rows = L if L > 0 else E            # scenario rows: a bank of levels, or one per env
        self.sc = {}
        for k in _SC_FLOAT:
            a = np.ascontiguousarray(scenario[k], np.float32)
            assert a.shape == (rows, N), (k, a.shape)
            self.sc[k] = a
        for k in ("team", "enabled"):
            a = np.ascontiguousarray(scenario[k], np.uint8)
            assert a.shape == (rows, N)
            self.sc[k] = a
        ter = scenario.get("terrain")
        if ter is not None:
            ter = np.ascontiguousarray(ter, np.int8)
            assert ter.shape == (rows, self.p["grid_h"], self.p["grid_w"])
        self.sc["terrain"] = ter
        zd = scenario.get("zone_desc")
        if zd is not None and self.p["max_zones"] > 0:
            zd = np.ascontiguousarray(zd, np.float32)
            assert zd.shape == (rows, self.p["max_zones"], 6)
        else:
            zd = None
        self.sc["zone_desc"] = zd

        self.env_ids = None
        if self.p.get("env_ids") is not None:
            self.env_ids = np.ascontiguousarray(self.p["env_ids"], np.int32)
            assert self.env_ids.shape == (E,)
        self.cp = RefParams(**{k: self.p.get(k, 0) for k, _ in RefParams._fields_
                               if k != "env_ids"}, env_ids=_ptr(self.env_ids, _I32))
        self.csc = RefScenario(**{k: _ptr(self.sc[k], _F) for k in _SC_FLOAT},
                               team=_ptr(self.sc["team"], _B),
                               enabled=_ptr(self.sc["enabled"], _B),
                               terrain=_ptr(ter, C.POINTER(C.c_byte)),
                               zone_desc=_ptr(zd, _F))
        self.D = int(lib().tabx_ref_obs_dim(C.byref(self.cp)))
        self.words = (N + 63) // 64
        self.st = {k: np.zeros((E, N), np.float32) for k in _ST_FLOAT}
        self.st["alive"] = np.zeros((E, N), np.uint8)
        self.st["t"] = np.zeros(E, np.int32)
        self.st["phi_prev"] = np.zeros(E, np.float32)
        if metrics:
            for n, _, dt in _METRICS:
                self.st[n] = np.zeros(E, dt)
        if L > 0:
            self.st["level"] = np.zeros(E, np.int32)
            self.st["next_level"] = (np.arange(E) % L).astype(np.int32)   # first episodes
            self.st["level_draws"] = np.zeros(E, np.int32)
        if self.p.get("dynamics", 0) == 1:            # persistent velocities: the acceleration is state
            self.st["ax"] = np.zeros((E, N), np.float32)
            self.st["ay"] = np.zeros((E, N), np.float32)
        self._bind_state()
        self.gstate = np.zeros((E, 16 * N + 6 * self.p["max_zones"]), np.float32)
        self.rewards = np.zeros((E, N), np.float32)
        self.dones = np.zeros(E, np.uint8)
        self.obs = np.zeros((E, N, self.D), np.float32)
        self.vis = np.zeros((E, N, self.words), np.uint64)
        self.amask = np.zeros((E, N), np.uint8)
        self.margin = np.full(E, np.inf, np.float64)
        self.track_margin = False

    def _bind_state(self):
        self.cst = RefState(**{k: _ptr(self.st[k], _F) for k in _ST_FLOAT},
                            alive=_ptr(self.st["alive"], _B),
                            t=_ptr(self.st["t"], C.POINTER(C.c_int)),
                            phi_prev=_ptr(self.st["phi_prev"], _F),
                            **({n: _ptr(self.st[n], t) for n, t, _ in _METRICS}
                               if self.metrics else {}),
                            **({n: _ptr(self.st[n], _I32) for n in _LEVELS}
                               if "level" in self.st else {}),
                            **({n: _ptr(self.st[n], _F) for n in ("ax", "ay")}
                               if "ax" in self.st else {}))

    def set_state(self, **arrays):
        """Overwrites state fields in place (hand-worked cases)."""
        for k, v in arrays.items():
            self.st[k][...] = v

    def snapshot(self) -> dict:
        return {k: v.copy() for k, v in self.st.items()}

    def restore(self, snap: dict):
        for k, v in snap.items():
            self.st[k][...] = v

    def _mm(self):
        return _ptr(self.margin, C.POINTER(C.c_double)) if self.track_margin else None

    def reset(self, env_mask=None):
        m = None if env_mask is None else np.ascontiguousarray(env_mask, np.uint8)
        lib().tabx_ref_reset(C.byref(self.cp), C.byref(self.csc), C.byref(self.cst),
                             _ptr(m, _B))

    def step(self, actions):
        a = np.ascontiguousarray(actions, np.uint8)
        assert a.shape == (self.E, self.N)
        lib().tabx_ref_step(C.byref(self.cp), C.byref(self.csc), C.byref(self.cst),
                            _ptr(a, _B), _ptr(self.rewards, _F), _ptr(self.dones, _B),
                            self._mm())
        return self.rewards, self.dones

    def observe(self):
        lib().tabx_ref_observe(C.byref(self.cp), C.byref(self.csc), C.byref(self.cst),
                               _ptr(self.obs, _F),
                               _ptr(self.vis, C.POINTER(C.c_ulonglong)),
                               _ptr(self.amask, _B), self._mm())
        return self.obs, self.vis, self.amask

    def global_state(self):
        lib().tabx_ref_global_state(C.byref(self.cp), C.byref(self.csc), C.byref(self.cst),
                                    _ptr(self.gstate, _F))
        return self.gstate

    def heuristic_actions(self, policy: dict, controlled, actions):
        """Fills `actions` (uint8 [E, N], in place) for the controlled, alive units."""
        if not hasattr(self, "mem"):
            self.mem = {"mem_x": np.zeros((self.E, self.N), np.float32),
                        "mem_y": np.zeros((self.E, self.N), np.float32),
                        "mem_valid": np.zeros((self.E, self.N), np.uint8)}
            self.cmem = RefPolicyMemory(mem_x=_ptr(self.mem["mem_x"], _F),
                                        mem_y=_ptr(self.mem["mem_y"], _F),
                                        mem_valid=_ptr(self.mem["mem_valid"], _B))
        pol = RefPolicy(**policy)
        ctl = np.ascontiguousarray(controlled, np.uint8)
        assert actions.dtype == np.uint8 and actions.flags["C_CONTIGUOUS"]
        lib().tabx_ref_heuristic_actions(C.byref(self.cp), C.byref(self.csc), C.byref(self.cst),
                                         C.byref(pol), C.byref(self.cmem), _ptr(ctl, _B),
                                         _ptr(actions, _B))
        return actions

    def policy_step(self, policy: dict, controlled, actions):
        """heuristic_actions, then step, then the units of finished envs forget their targets:
        what the library's fused policy tick computes."""
        self.heuristic_actions(policy, controlled, actions)
        out = self.step(actions)
        self.mem["mem_valid"][self.dones.astype(bool)] = 0
        return out
