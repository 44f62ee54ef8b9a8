"""Shared test helpers: small CPU-checker set-ups and golden-file reading."""
import math
import os

import numpy as np

from oracle.ref import RefEnv
from paper_2602_01665_amd import inputs as I

GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")


def golden_table(name):
    """Reads `key value...` lines of a golden text file (lines with # are comments)."""
    out = {}
    with open(os.path.join(GOLDEN, name)) as f:
        for line in f:
            line = line.split("#", 1)[0].strip()
            if not line:
                continue
            parts = line.split()
            out[parts[0]] = [float(v) for v in parts[1:]]
    return out


def unit(name, team, x, y, theta=0.0, **kw):
    return dict(unit=name, team=team, x=x, y=y, theta=theta, **kw)


def make_ref(units, map_size=32.0, grid=0, terrain=None, zone_desc=None, max_zones=0,
             **param_override):
    sc = I.custom_scenario(units, map_size, grid, terrain, zone_desc)
    p = I.custom_params(len(units), map_size, grid, max_zones, **param_override)
    env = RefEnv(p, sc)
    env.reset()
    return env


def acts(*a):
    return np.array([a], np.uint8)


def other_slot(D_row, i, j):
    """The 16-float block of unit j inside agent i's observation row."""
    k = j if j < i else j - 1
    return D_row[16 + 16 * k: 16 + 16 * (k + 1)]


def vis_bit(vis, e, i, j):
    return int((int(vis[e, i, j >> 6]) >> (j & 63)) & 1)
