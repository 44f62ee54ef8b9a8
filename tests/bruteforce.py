"""Independent float64 formulations used to pin the CPU checker (no shared code).

Visibility uses an atan2 angle difference and hypot; the hurtbox test uses the
Minkowski-sum decomposition of "circle meets rectangle" (two slabs plus four
corner discs) with libm sin/cos, instead of the checker's closest-point clamp
and its polynomial sin/cos.  Each routine also returns how far every pair is
from a decision boundary, so that comparisons can skip pairs whose outcome a
float32 rounding could legitimately flip.
"""
import math

import numpy as np

ZONE_BUSH = 2


def cell_codes(p, terrain_e, x, y):
    if terrain_e is None or p["grid_w"] == 0:
        return np.zeros(len(x), np.int64)
    cx = np.minimum((x.astype(np.float64) / p["cell_size"]).astype(np.int64), p["grid_w"] - 1)
    cy = np.minimum((y.astype(np.float64) / p["cell_size"]).astype(np.int64), p["grid_h"] - 1)
    return terrain_e[cy, cx].astype(np.int64)


def hurtbox_matrix(x, y, theta, rng_, hw, radius):
    """hit[i, j] and margin[i, j]: does unit j's body meet unit i's hurtbox."""
    n = len(x)
    hit = np.zeros((n, n), bool)
    margin = np.full((n, n), np.inf)
    for i in range(n):
        c, s = math.cos(float(theta[i])), math.sin(float(theta[i]))
        L, w = float(rng_[i]), float(hw[i])
        for j in range(n):
            if i == j:
                continue
            dx, dy = float(x[j]) - float(x[i]), float(y[j]) - float(y[i])
            lx, ly = dx * c + dy * s, -dx * s + dy * c
            r = float(radius[j])
            in_slab_a = (0.0 <= lx <= L) and (abs(ly) <= w + r)
            in_slab_b = (-r <= lx <= L + r) and (abs(ly) <= w)
            in_corner = any(math.hypot(lx - cx, ly - cy) <= r
                            for cx in (0.0, L) for cy in (-w, w))
            hit[i, j] = in_slab_a or in_slab_b or in_corner
            # signed distance of the centre from the rounded rectangle's outline
            qx = max(-lx, lx - L, 0.0)
            qy = max(abs(ly) - w, 0.0)
            outside = math.hypot(qx, qy)
            if outside > 0.0:
                margin[i, j] = abs(outside - r)
            else:
                inside_depth = min(lx, L - lx, w - abs(ly))
                margin[i, j] = inside_depth + r
    return hit, margin


def visibility_matrix(p, terrain_e, x, y, theta, alive, team, reveal, sight_angle,
                      sight_range):
    n = len(x)
    code = cell_codes(p, terrain_e, x, y)
    vis = np.zeros((n, n), bool)
    margin = np.full((n, n), np.inf)
    for i in range(n):
        for j in range(n):
            if i == j or not alive[i] or not alive[j]:
                continue
            dx, dy = float(x[j]) - float(x[i]), float(y[j]) - float(y[i])
            dist = math.hypot(dx, dy)
            m = abs(dist - float(sight_range[i]))
            in_range = dist <= float(sight_range[i])
            if dist > 0.0:
                diff = math.atan2(dy, dx) - float(theta[i])
                diff = (diff + math.pi) % (2 * math.pi) - math.pi
                half = float(sight_angle[i]) / 2.0
                in_cone = abs(diff) <= half
                if in_range:
                    m = min(m, abs(abs(diff) - half) * max(dist, 1e-3))
            else:
                in_cone = True
            bush_j = (code[j] & 3) == ZONE_BUSH
            hidden = (bush_j and team[i] != team[j] and not (code[i] == code[j])
                      and not reveal[j] > 0.0)
            vis[i, j] = in_range and in_cone and not hidden
            margin[i, j] = m
    return vis, margin


def step_health(p, terrain_e, sc_e, st_e, act):
    """One tick's positions, headings and health from scratch, in float64.

    sc_e / st_e: per-unit 1-D arrays of one env.  Returns (x, y, theta, hp, min_margin).
    """
    n = len(act)
    dt = p["dt"]
    alive = st_e["alive"].astype(bool)
    en = sc_e["enabled"].astype(bool)
    x = st_e["x"].astype(np.float64).copy()
    y = st_e["y"].astype(np.float64).copy()
    th = st_e["theta"].astype(np.float64).copy()
    hp = st_e["hp"].astype(np.float64).copy()
    cd = np.maximum(st_e["cd"].astype(np.float64) - dt, 0.0)
    bdmg = np.zeros(n)
    min_margin = np.inf
    for u in range(n):
        if not alive[u]:
            continue
        x[u] += float(st_e["vx"][u]) * dt
        y[u] += float(st_e["vy"][u]) * dt
        # closeness to an arena edge or a terrain cell edge (exact hits are safe:
        # the float32 sum is then exact as well)
        for v, hi in ((x[u], p["map_w"]), (y[u], p["map_h"])):
            for edge in (0.0, hi):
                if v != edge:
                    min_margin = min(min_margin, abs(v - edge))
            if p["grid_w"]:
                f = (v / p["cell_size"]) % 1.0
                if f != 0.0:
                    min_margin = min(min_margin, min(f, 1.0 - f) * p["cell_size"])
        if x[u] < 0 or x[u] > p["map_w"] or y[u] < 0 or y[u] > p["map_h"]:
            bdmg[u] = 0.1 * float(sc_e["hmax"][u]) * dt
        x[u] = min(max(x[u], 0.0), p["map_w"])
        y[u] = min(max(y[u], 0.0), p["map_h"])
        if act[u] == 6:
            th[u] = (th[u] + p["turn_rate"] * dt) % (2 * math.pi)
        elif act[u] == 7:
            th[u] = (th[u] - p["turn_rate"] * dt) % (2 * math.pi)
    hit, margin = hurtbox_matrix(x, y, th, sc_e["range"], sc_e["hurt_halfwidth"],
                                 sc_e["radius"])
    delta = np.zeros(n)
    for i in range(n):
        if not alive[i] or act[i] != 5 or cd[i] > 0.0:
            continue
        best, best_d = -1, np.inf
        hit_d = []
        struck = []
        for j in range(n):
            if j == i or not alive[j]:
                continue
            heal = sc_e["dmg"][i] < 0
            if heal != (sc_e["team"][i] == sc_e["team"][j]):
                continue
            min_margin = min(min_margin, margin[i, j])
            d = math.hypot(x[j] - x[i], y[j] - y[i])
            inside = bool(hit[i, j])
            if inside and p.get("hurtbox_cone", 0) and d > 0.0:
                # the body's centre must also lie within the angle of the sight cone
                off = math.atan2(y[j] - y[i], x[j] - x[i]) - th[i]
                off = abs((off + math.pi) % (2 * math.pi) - math.pi)
                half = float(sc_e["sight_angle"][i]) / 2.0
                min_margin = min(min_margin, abs(off - half) * d)
                inside = off <= half
            if inside:
                hit_d.append(d)
                struck.append(j)
            if inside and d < best_d:
                best, best_d = j, d
        if p.get("hit_all", 0):
            for j in struck:            # every valid body in the hurtbox
                delta[j] += float(sc_e["dmg"][i])
        elif best >= 0:
            delta[best] += float(sc_e["dmg"][i])
            hit_d.sort()
            if len(hit_d) > 1:          # a near tie for "closest" may flip in float32
                min_margin = min(min_margin, hit_d[1] - hit_d[0])
    code = cell_codes(p, terrain_e, x.astype(np.float32), y.astype(np.float32))
    for u in range(n):
        if not alive[u]:
            continue
        hp[u] = min(max(hp[u] - delta[u] - bdmg[u], 0.0), float(sc_e["hmax"][u]))
        if (code[u] & 3) == 1:
            hp[u] = max(hp[u] - p["lava_dps"] * dt, 0.0)
    hp[~en] = 0.0
    return x, y, th, hp, min_margin
