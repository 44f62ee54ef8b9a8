/*
 * tabx_ref.cpp -- CPU checker for the TABX batched environment step.
 *
 * TEST INFRASTRUCTURE ONLY (see tabx_ref.h).  One env at a time, one unit at a
 * time, one pair at a time; nothing is blocked, fused or reordered.  Build with
 *   g++ -O2 -std=c++17 -ffp-contract=off -fno-fast-math -shared -fPIC
 * so that every float expression below is evaluated exactly as written.
 *
 * Stage order follows App. A "Interaction Dynamics": (1) physics update,
 * (2) action application (movement / rotation / combat), (3) post-processing
 * (zone effects, alive flags, reward, termination).
 */
#include "tabx_ref.h"

#include <cmath>
#include <vector>

namespace {

enum { ACT_NOOP = 0, ACT_XP = 1, ACT_YP = 2, ACT_XM = 3, ACT_YM = 4,
       ACT_ATTACK = 5, ACT_ROT_L = 6, ACT_ROT_R = 7 };
enum { ZONE_OPEN = 0, ZONE_LAVA = 1, ZONE_BUSH = 2, ZONE_SWAMP = 3 };

const float TWO_PI_F = 6.28318530717958647692f;

/* ---- sine / cosine of a heading in [0, 2*pi] -------------------------------
 * Quadrant reduction n = trunc(theta * 2/pi + 1/2), remainder by a two-term
 * split of pi/2, then Taylor polynomials of degree 9 (sin) and 8 (cos) in
 * Horner form with explicit fused multiply-adds.  |r| <= pi/4 so the series
 * remainders are below 3e-8.  No libm transcendental is involved, so the
 * value is a fixed function of the float input on any IEEE machine. */
void sincos_spec(float theta, float *s_out, float *c_out)
{
    const float TWO_OVER_PI = 0.63661977236758134308f;
    const float PIO2_HI = 1.57079637050628662109375f;      /* float(pi/2)      */
    const float PIO2_LO = -4.37113882867379435e-8f;        /* pi/2 - PIO2_HI   */
    const float S1 = -1.0f / 6.0f, S2 = 1.0f / 120.0f, S3 = -1.0f / 5040.0f,
                S4 = 1.0f / 362880.0f;
    const float C1 = -0.5f, C2 = 1.0f / 24.0f, C3 = -1.0f / 720.0f,
                C4 = 1.0f / 40320.0f;

    float q = theta * TWO_OVER_PI;
    q = q + 0.5f;
    int   n  = (int)q;
    float fn = (float)n;
    float r  = std::fmaf(-fn, PIO2_HI, theta);
    r        = std::fmaf(-fn, PIO2_LO, r);
    float r2 = r * r;

    float ps = std::fmaf(r2, S4, S3);
    ps       = std::fmaf(r2, ps, S2);
    ps       = std::fmaf(r2, ps, S1);
    float r3 = r * r2;
    float sr = std::fmaf(r3, ps, r);

    float pc = std::fmaf(r2, C4, C3);
    pc       = std::fmaf(r2, pc, C2);
    pc       = std::fmaf(r2, pc, C1);
    float cr = std::fmaf(r2, pc, 1.0f);

    switch (n & 3) {
    case 0:  *s_out = sr;  *c_out = cr;  break;
    case 1:  *s_out = cr;  *c_out = -sr; break;
    case 2:  *s_out = -sr; *c_out = -cr; break;
    default: *s_out = -cr; *c_out = sr;  break;
    }
}

inline float clampf(float v, float lo, float hi)
{
    return v < lo ? lo : (v > hi ? hi : v);
}

/* The env's index for the counter-based random draws. */
unsigned env_id(const RefParams &P, int e)
{
    return (unsigned)(P.env_ids ? P.env_ids[e] : e);
}

/* Which row of the scenario arrays configures env e: its own (no level bank) or the level it
 * currently plays (the configuration is applied at reset, Sec. 4.1; App. A "Environment
 * Parameters"). */
int level_of(const RefParams &P, const RefState &st, int e)
{
    return P.num_levels > 0 ? st.level[e] : e;
}

/* The scenario as env e sees it: every pointer moved to the row of its level, so that the
 * per-env code below indexes unit arrays by unit, `terrain` by cell and `zone_desc` by slot. */
RefScenario level_slice(const RefParams &P, const RefScenario &bank, const RefState &st, int e)
{
    const long row = level_of(P, st, e);
    const long N = P.num_units;
    RefScenario S = bank;
    S.init_x += row * N;       S.init_y += row * N;       S.init_theta += row * N;
    S.hmax += row * N;         S.radius += row * N;       S.mass += row * N;
    S.speed += row * N;        S.dmg += row * N;          S.range += row * N;
    S.cooldown += row * N;     S.sight_angle += row * N;  S.sight_cos_half += row * N;
    S.sight_range += row * N;  S.hurt_halfwidth += row * N;
    S.team += row * N;         S.enabled += row * N;
    if (S.terrain) S.terrain += row * P.grid_h * P.grid_w;
    if (S.zone_desc) S.zone_desc += row * P.max_zones * 6;
    return S;
}

/* An episode of env e is about to start: it takes the level queued in next_level (any int is
 * folded into [0, num_levels)), and the queue is refilled with a uniform draw, the
 * counter-based hash of (level_seed, env, number of draws so far); the caller may overwrite
 * the queued level at any time before the episode ends. */
unsigned hash32(unsigned seed, unsigned env, unsigned unit, unsigned tick, unsigned draw);
void advance_level(const RefParams &P, RefState &st, int e)
{
    if (P.num_levels <= 0) return;
    const unsigned L = (unsigned)P.num_levels;
    st.level[e] = (int)((unsigned)st.next_level[e] % L);
    const unsigned n = (unsigned)st.level_draws[e];
    st.next_level[e] = (int)(hash32(P.level_seed, env_id(P, e), 0u, n, 3u) % L);
    st.level_draws[e] = (int)(n + 1u);
}

/* Zone code under a position: low two bits = zone type, upper bits = zone identity; 0 = open.
 * Cell-grid zones: the code stored in the cell.  Elliptical zones (App. A "Zones": type,
 * centre, two axes, effect magnitude): the last listed active zone whose ellipse
 * (x-cx)^2/hx^2 + (y-cy)^2/hy^2 <= 1 holds the point, tested without division as
 * (dx^2)*hy^2 + (dy^2)*hx^2 <= hx^2*hy^2; identity = slot index + 1. */
int cell_code(const RefParams &P, const RefScenario &S, float x, float y)
{
    if (P.zone_shapes == 1) {
        int code = 0;
        for (int z = 0; z < P.max_zones && S.zone_desc; ++z) {
            const float *d = S.zone_desc + (long)z * 6;
            if (d[0] == 0.0f) continue;
            float dx = x - d[1];
            float dy = y - d[2];
            float hx2 = d[3] * d[3];
            float hy2 = d[4] * d[4];
            bool inside = ((dx * dx) * hy2) + ((dy * dy) * hx2) <= hx2 * hy2;
            if (inside) code = ((int)d[0] & 3) | ((z + 1) << 2);
        }
        return code;
    }
    if (!S.terrain || P.grid_w <= 0 || P.grid_h <= 0) return 0;
    int cx = (int)(x / P.cell_size);
    int cy = (int)(y / P.cell_size);
    if (cx > P.grid_w - 1) cx = P.grid_w - 1;
    if (cy > P.grid_h - 1) cy = P.grid_h - 1;
    if (cx < 0) cx = 0;
    if (cy < 0) cy = 0;
    return (int)S.terrain[(long)cy * P.grid_w + cx];
}

/* Effect magnitude of the zone a code names: the zone's own (elliptical zones) or the
 * global parameter (cell grid). */
float zone_effect(const RefParams &P, const RefScenario &S, int code, float global_value)
{
    if (P.zone_shapes == 1 && (code >> 2) > 0)
        return S.zone_desc[(long)((code >> 2) - 1) * 6 + 5];
    return global_value;
}

/* Mean health ratio of one team over its enabled units, ascending index
 * (the bracketed means of Eq. 1).  A team with no enabled unit has ratio 0. */
float team_ratio(const RefParams &P, const RefScenario &S, const RefState &st,
                 int e, int team)
{
    const int N = P.num_units, b = e * N;
    float sum = 0.0f;
    int   cnt = 0;
    for (int u = 0; u < N; ++u) {
        if (!S.enabled[u] || S.team[u] != team) continue;
        sum = sum + st.hp[b + u] / S.hmax[u];
        cnt += 1;
    }
    return cnt > 0 ? sum / (float)cnt : 0.0f;
}

void reset_env(const RefParams &P, const RefScenario &S, RefState &st, int e)
{
    const int N = P.num_units, b = e * N;
    for (int u = 0; u < N; ++u) {
        const int k = b + u;
        st.x[k] = S.init_x[u];
        st.y[k] = S.init_y[u];
        st.theta[k] = S.init_theta[u];
        st.vx[k] = 0.0f;
        st.vy[k] = 0.0f;
        if (P.dynamics == 1) {
            st.ax[k] = 0.0f;
            st.ay[k] = 0.0f;
        }
        st.hp[k] = S.enabled[u] ? S.hmax[u] : 0.0f;
        st.cd[k] = 0.0f;
        st.reveal[k] = 0.0f;
        st.alive[k] = S.enabled[u] ? 1 : 0;
        const int code = cell_code(P, S, st.x[k], st.y[k]);
        st.cur_speed[k] = ((code & 3) == ZONE_SWAMP)
                              ? S.speed[u] * zone_effect(P, S, code, P.swamp_mult) : S.speed[u];
    }
    st.t[e] = 0;
    st.phi_prev[e] = team_ratio(P, S, st, e, 0) - team_ratio(P, S, st, e, 1);
    if (st.ret_run) st.ret_run[e] = 0.0f;
    if (st.kill_run) st.kill_run[e] = 0;
}

/* Hurtbox test (App. A "Attack range geometry"): the attacker's forward
 * rectangle x in [0, L], y in [-hw, hw] (attacker frame) against the target's
 * body circle; closed boundary.  Returns the overlap flag, the squared
 * centre distance in *d2 and, if margin is given, |gap - r_j| in doubles. */
bool hurtbox_hit(float xi, float yi, float ci, float si, float L, float hw,
                 float xj, float yj, float rj, float *d2, double *margin)
{
    float dx = xj - xi;
    float dy = yj - yi;
    float lx = (dx * ci) + (dy * si);
    float ly = (dy * ci) - (dx * si);
    float ex = lx - clampf(lx, 0.0f, L);
    float ey = ly - clampf(ly, -hw, hw);
    float g2 = (ex * ex) + (ey * ey);
    *d2 = (dx * dx) + (dy * dy);
    if (margin) *margin = std::fabs(std::sqrt((double)g2) - (double)rj);
    return g2 <= rj * rj;
}

/* Angular part of the field of view: the offset (dx, dy) lies within the cone of half-angle
 * acos(cos_half) around the heading (ci, si); a zero offset counts as inside. */
bool within_cone_angle(float dx, float dy, float ci, float si, float cos_half)
{
    float d2 = (dx * dx) + (dy * dy);
    float dot = (dx * ci) + (dy * si);
    return (d2 == 0.0f) || (dot >= cos_half * std::sqrt(d2));
}

/* Role filter: damage dealers reach enemies only, healers (negative damage)
 * allies only. */
inline bool role_allows(float dmg_i, int team_i, int team_j)
{
    return dmg_i < 0.0f ? (team_i == team_j) : (team_i != team_j);
}

/* Contact of two circular bodies (App. A "Collision detection and resolution", circle to
 * circle): penetration depth pen = r_i + r_j - |p_j - p_i| and the normal from i to j;
 * coincident centres separate along x, the lower index to the left. */
struct Contact { float nx, ny, pen; };
Contact body_contact(const RefScenario &S, const std::vector<float> &px, const std::vector<float> &py,
                     int i, int j)
{
    Contact c;
    float dx = px[j] - px[i];
    float dy = py[j] - py[i];
    float dist = std::sqrt((dx * dx) + (dy * dy));
    c.pen = (S.radius[i] + S.radius[j]) - dist;
    if (dist > 0.0f) {
        c.nx = dx / dist;
        c.ny = dy / dist;
    } else {               /* coincident centres: separate along x by index */
        c.nx = (i < j) ? 1.0f : -1.0f;
        c.ny = 0.0f;
    }
    return c;
}

void step_env(const RefParams &P, const RefScenario &bank, RefState &st, int e,
              const unsigned char *act, float *rewards, unsigned char *dones,
              double *min_margin)
{
    const RefScenario S = level_slice(P, bank, st, e);
    const int N = P.num_units, b = e * N;
    std::vector<unsigned char> alive0(N);
    std::vector<float> bdmg(N, 0.0f), c(N), s(N);
    std::vector<int> target(N, -1);
    std::vector<unsigned char> landed(N, 0);
    std::vector<unsigned char> inbox((size_t)N * N, 0);   /* attackable matrix: i may strike j */

    for (int u = 0; u < N; ++u) alive0[u] = st.alive[b + u];

    /* ---- stage 1: physics --------------------------------------------------- */
    for (int u = 0; u < N; ++u) {
        const int k = b + u;
        if (!S.enabled[u]) continue;
        float v = st.cd[k] - P.dt;
        st.cd[k] = v > 0.0f ? v : 0.0f;
        v = st.reveal[k] - P.dt;
        st.reveal[k] = v > 0.0f ? v : 0.0f;
        if (!alive0[u]) continue;
        if (P.dynamics == 1) {
            /* explicit Euler, in the passage's order: the velocity from the current
             * acceleration first, then the position from that velocity */
            st.vx[k] = st.vx[k] + st.ax[k] * P.dt;
            st.vy[k] = st.vy[k] + st.ay[k] * P.dt;
        }
        float x = st.x[k] + st.vx[k] * P.dt;
        float y = st.y[k] + st.vy[k] * P.dt;
        bool oob = (x < 0.0f) || (x > P.map_w) || (y < 0.0f) || (y > P.map_h);
        if (oob) bdmg[u] = (P.boundary_frac * S.hmax[u]) * P.dt;
        st.x[k] = clampf(x, 0.0f, P.map_w);
        st.y[k] = clampf(y, 0.0f, P.map_h);
    }

    /* ---- stage 1b: overlapping bodies are pushed apart (App. A "Collision detection and
     * resolution").  Circle against circle: penetration depth pen = r_i + r_j - |p_j - p_i|
     * along the normal n = (p_j - p_i) / |p_j - p_i|; what exceeds the slop is corrected by
     * the fraction alpha, split by inverse mass (unit i takes m_j / (m_i + m_j) of it).
     * All pairs are evaluated on the positions after the kinematic update and each unit
     * adds its corrections in ascending partner index (Jacobi style), then is clipped to
     * the arena again.  Dead bodies collide like live ones; disabled placeholders do not
     * exist.  A kinematic body (same passage: exempt from the response) is one whose mass is
     * +infinity: it gives way to nobody, a body of finite mass gives way to it for the whole
     * corrected depth, and two kinematic bodies leave each other alone.  The impulse part of
     * the paper's response changes velocities only; in the kinematic mode the action stage
     * rewrites every velocity later in the same tick, so it is evaluated only with persistent
     * velocities (dynamics = 1, below). */
    if (P.collision_alpha > 0.0f) {
        std::vector<float> px(N), py(N), ax(N, 0.0f), ay(N, 0.0f);
        for (int u = 0; u < N; ++u) {
            px[u] = st.x[b + u];
            py[u] = st.y[b + u];
        }
        /* Impulse response (same passage; only with persistent velocities, dynamics = 1): for
         * every pair that interpenetrates (depth > 0, the slop applies to the position
         * correction only) the relative velocity v_j - v_i is projected onto the normal n
         * (from i to j).  A pair that is already separating (projection > 0) gets no impulse.
         * Otherwise the impulse magnitude is (1 + e) * (-v_rel.n) / (1/m_i + 1/m_j) and unit i's
         * velocity changes by it times 1/m_i, away from j.  A kinematic body (infinite mass,
         * inverse mass 0) is exempt; its partner bounces off it as off a wall.  Jacobi style
         * like the correction: all pairs on the velocities after the kinematic update, unit i
         * adding its changes in ascending partner index. */
        if (P.dynamics == 1) {
            std::vector<float> pvx(N), pvy(N), dvx(N, 0.0f), dvy(N, 0.0f);
            for (int u = 0; u < N; ++u) {
                pvx[u] = st.vx[b + u];
                pvy[u] = st.vy[b + u];
            }
            for (int i = 0; i < N; ++i) {
                if (!S.enabled[i]) continue;
                const float inv_i = 1.0f / S.mass[i];          /* 0 for a kinematic body */
                if (inv_i == 0.0f) continue;
                for (int j = 0; j < N; ++j) {
                    if (j == i || !S.enabled[j]) continue;
                    const Contact ct = body_contact(S, px, py, i, j);
                    if (!(ct.pen > 0.0f)) continue;
                    const float nx = ct.nx, ny = ct.ny;
                    float rvx = pvx[j] - pvx[i];
                    float rvy = pvy[j] - pvy[i];
                    float vn = (rvx * nx) + (rvy * ny);
                    if (vn > 0.0f) continue;                   /* separating: correction only */
                    const float inv_j = 1.0f / S.mass[j];
                    float jimp = ((1.0f + P.restitution) * (0.0f - vn)) / (inv_i + inv_j);
                    dvx[i] = dvx[i] - ((jimp * inv_i) * nx);
                    dvy[i] = dvy[i] - ((jimp * inv_i) * ny);
                }
            }
            for (int u = 0; u < N; ++u) {
                if (!S.enabled[u]) continue;
                st.vx[b + u] = pvx[u] + dvx[u];
                st.vy[b + u] = pvy[u] + dvy[u];
            }
        }
        for (int i = 0; i < N; ++i) {
            if (!S.enabled[i]) continue;
            for (int j = 0; j < N; ++j) {
                if (j == i || !S.enabled[j]) continue;
                const Contact ct = body_contact(S, px, py, i, j);
                const float pen = ct.pen, nx = ct.nx, ny = ct.ny;
                if (!(pen > P.collision_slop)) continue;
                const bool kinematic_i = std::isinf(S.mass[i]);
                const bool kinematic_j = std::isinf(S.mass[j]);
                float share;
                if (kinematic_i) share = 0.0f;
                else if (kinematic_j) share = 1.0f;
                else share = S.mass[j] / (S.mass[i] + S.mass[j]);
                float c = ((pen - P.collision_slop) * P.collision_alpha) * share;
                ax[i] = ax[i] - (c * nx);
                ay[i] = ay[i] - (c * ny);
            }
        }
        for (int u = 0; u < N; ++u) {
            if (!S.enabled[u]) continue;
            st.x[b + u] = clampf(px[u] + ax[u], 0.0f, P.map_w);
            st.y[b + u] = clampf(py[u] + ay[u], 0.0f, P.map_h);
        }
    }

    /* ---- stage 2: actions ---------------------------------------------------- */
    const float dtheta = P.turn_rate * P.dt;
    for (int u = 0; u < N; ++u) {
        const int k = b + u;
        /* the velocity the unit wants: its current speed along a move action, else none */
        float wx = 0.0f, wy = 0.0f;
        if (alive0[u]) {
            const int a = act[k];
            const float sp = st.cur_speed[k];
            if (a == ACT_XP) wx = sp;
            else if (a == ACT_YP) wy = sp;
            else if (a == ACT_XM) wx = -sp;
            else if (a == ACT_YM) wy = -sp;
        }
        if (P.dynamics == 1) {
            /* persistent velocity: the action sets the acceleration the next physics stage
             * integrates; what is not alive neither moves nor accelerates */
            if (alive0[u]) {
                st.ax[k] = (wx - st.vx[k]) * P.move_gain;
                st.ay[k] = (wy - st.vy[k]) * P.move_gain;
            } else {
                st.vx[k] = 0.0f;
                st.vy[k] = 0.0f;
                st.ax[k] = 0.0f;
                st.ay[k] = 0.0f;
            }
        } else {
            st.vx[k] = wx;
            st.vy[k] = wy;
        }
        if (alive0[u]) {
            const int a = act[k];
            if (a == ACT_ROT_L) {
                float th = st.theta[k] + dtheta;
                if (th >= TWO_PI_F) th = th - TWO_PI_F;
                st.theta[k] = th;
            } else if (a == ACT_ROT_R) {
                float th = st.theta[k] - dtheta;
                if (th < 0.0f) th = th + TWO_PI_F;
                st.theta[k] = th;
            }
        }
        sincos_spec(st.theta[k], &s[u], &c[u]);
    }

    /* attackable matrix row by row, closest valid target (ties: lowest index) */
    for (int i = 0; i < N; ++i) {
        if (!alive0[i]) continue;
        const int ki = b + i;
        float best = 0.0f;
        for (int j = 0; j < N; ++j) {
            if (j == i || !alive0[j]) continue;
            const int kj = b + j;
            if (!role_allows(S.dmg[i], S.team[i], S.team[j])) continue;
            float d2;
            double m;
            bool hit = hurtbox_hit(st.x[ki], st.y[ki], c[i], s[i], S.range[i],
                                   S.hurt_halfwidth[i], st.x[kj], st.y[kj],
                                   S.radius[j], &d2, min_margin ? &m : nullptr);
            if (min_margin && m < min_margin[e]) min_margin[e] = m;
            if (hit && P.hurtbox_cone)
                hit = within_cone_angle(st.x[kj] - st.x[ki], st.y[kj] - st.y[ki], c[i], s[i],
                                        S.sight_cos_half[i]);
            if (hit) inbox[i * N + j] = 1;
            if (hit && (target[i] < 0 || d2 < best)) {
                target[i] = j;
                best = d2;
            }
        }
    }

    /* eligibility: chose the combat action with the cooldown elapsed; the
     * cooldown restarts whether or not a target is in the hurtbox */
    for (int i = 0; i < N; ++i) {
        const int ki = b + i;
        bool elig = alive0[i] && act[ki] == ACT_ATTACK && st.cd[ki] <= 0.0f;
        if (elig) st.cd[ki] = S.cooldown[i];
        landed[i] = (elig && target[i] >= 0) ? 1 : 0;
    }

    /* victim-side application: every victim sums the damage (heals negative)
     * of the attackers that designated it, ascending attacker index, then
     * subtracts once together with the boundary penalty and clamps */
    for (int j = 0; j < N; ++j) {
        if (!alive0[j]) continue;
        const int kj = b + j;
        float acc = 0.0f;
        for (int i = 0; i < N; ++i) {
            const bool strikes_j = P.hit_all ? inbox[i * N + j] != 0 : target[i] == j;
            if (landed[i] && strikes_j) acc = acc + S.dmg[i];
        }
        float h = (st.hp[kj] - acc) - bdmg[j];
        st.hp[kj] = clampf(h, 0.0f, S.hmax[j]);
    }
    /* combat reveal (bush rule): a landed damaging attack exposes both ends */
    for (int i = 0; i < N; ++i) {
        if (landed[i] && S.dmg[i] > 0.0f) {
            st.reveal[b + i] = P.reveal_time;
            for (int j = 0; j < N; ++j) {
                const bool strikes_j = P.hit_all ? inbox[i * N + j] != 0 : target[i] == j;
                if (strikes_j) st.reveal[b + j] = P.reveal_time;
            }
        }
    }

    /* ---- stage 3: zone effects, alive flags, reward, termination -------------- */
    for (int u = 0; u < N; ++u) {
        const int k = b + u;
        if (!S.enabled[u]) { st.alive[k] = 0; continue; }
        const int code = cell_code(P, S, st.x[k], st.y[k]);
        const int zone = code & 3;
        if (alive0[u] && zone == ZONE_LAVA) {
            float h = st.hp[k] - (zone_effect(P, S, code, P.lava_dps) * P.dt);
            st.hp[k] = h > 0.0f ? h : 0.0f;
        }
        st.cur_speed[k] = (zone == ZONE_SWAMP)
                              ? S.speed[u] * zone_effect(P, S, code, P.swamp_mult) : S.speed[u];
        st.alive[k] = st.hp[k] > 0.0f ? 1 : 0;
    }
    st.t[e] += 1;

    const float ratio0 = team_ratio(P, S, st, e, 0);
    const float ratio1 = team_ratio(P, S, st, e, 1);
    const float phi = ratio0 - ratio1;
    const float dense = phi - st.phi_prev[e];
    float r0 = dense, r1 = -dense;

    int alive_cnt[2] = {0, 0}, before_cnt[2] = {0, 0};
    for (int u = 0; u < N; ++u) {
        if (st.alive[b + u]) alive_cnt[S.team[u] ? 1 : 0] += 1;
        if (alive0[u]) before_cnt[S.team[u] ? 1 : 0] += 1;
    }
    const bool done = alive_cnt[0] == 0 || alive_cnt[1] == 0 || st.t[e] >= P.max_steps;
    if (done) {
        /* one rule for wipe-out and truncation: the allies win only with a
         * strictly larger mean health ratio (equal ratios: allies lose) */
        const bool ally_win = ratio0 > ratio1;
        r0 = r0 + (ally_win ? 1.0f : -1.0f);
        r1 = r1 + (ally_win ? -1.0f : 1.0f);
    }
    for (int u = 0; u < N; ++u) {
        const int k = b + u;
        rewards[k] = S.enabled[u] ? (S.team[u] ? r1 : r0) : 0.0f;
    }
    dones[e] = done ? 1 : 0;

    /* episode metrics: first loss of a unit, running allied return, summary at the end */
    if (st.kill_run && st.kill_run[e] == 0) {
        const bool enemy_died = alive_cnt[1] < before_cnt[1];
        const bool ally_died = alive_cnt[0] < before_cnt[0];
        st.kill_run[e] = (signed char)((enemy_died ? 1 : 0) | (ally_died ? 2 : 0));
    }
    if (st.ret_run) st.ret_run[e] = st.ret_run[e] + r0;
    if (done) {
        if (st.ep_count) st.ep_count[e] += 1;
        if (st.ep_len) st.ep_len[e] = st.t[e];
        if (st.ep_return && st.ret_run) st.ep_return[e] = st.ret_run[e];
        if (st.ep_win) st.ep_win[e] = (ratio0 > ratio1) ? 1 : 0;
        if (st.ep_first_kill && st.kill_run) st.ep_first_kill[e] = st.kill_run[e];
    }
    if (done) {
        advance_level(P, st, e);
        reset_env(P, level_slice(P, bank, st, e), st, e);
    }
    else st.phi_prev[e] = phi;
}

/* The 16 own-unit features of App. A "Own-unit features" (+ zone type underfoot, team). */
void own_block(const RefParams &P, const RefScenario &S, const RefState &st, int e, int u,
               int code, float *row)
{
    const int k = e * P.num_units + u;
    row[0] = st.hp[k];
    row[1] = st.hp[k] / S.hmax[u];
    row[2] = st.x[k];
    row[3] = st.y[k];
    row[4] = st.theta[k];
    row[5] = S.range[u];
    row[6] = S.dmg[u];
    row[7] = st.cd[k];
    row[8] = S.cooldown[u] != 0.0f ? st.cd[k] / S.cooldown[u] : 0.0f;
    row[9] = S.radius[u];
    row[10] = S.mass[u];
    row[11] = S.sight_angle[u];
    row[12] = st.alive[k] ? 1.0f : 0.0f;
    row[13] = st.cur_speed[k];
    row[14] = (float)(code & 3);
    row[15] = (float)S.team[u];
}

void global_state_env(const RefParams &P, const RefScenario &S, const RefState &st, int e,
                      float *out)
{
    const int N = P.num_units, Z = P.max_zones;
    for (int o = 0; o < 16 * N + 6 * Z; ++o) out[o] = 0.0f;
    for (int u = 0; u < N; ++u) {
        const int k = e * N + u;
        if (!S.enabled[u]) continue;
        own_block(P, S, st, e, u, cell_code(P, S, st.x[k], st.y[k]), out + 16 * u);
    }
    for (int z = 0; z < Z && S.zone_desc; ++z) {
        const float *d = S.zone_desc + (long)z * 6;
        if (d[0] == 0.0f) continue;
        for (int c = 0; c < 6; ++c) out[16 * N + 6 * z + c] = d[c];
    }
}

/* What unit i (alive, heading cosine / sine ci, si, zone code code_i) perceives of unit j
 * (alive): the offset, whether j is visible to i (fan-shaped field of view and the bush
 * rule) and whether i's combat action could reach j (hurtbox and role filter).  `margin`,
 * if given, is lowered to the distance of the geometric tests from their boundaries. */
struct PairView {
    float dx, dy, d2;
    bool visible, same_team, attackable;
};

PairView pair_view(const RefParams &P, const RefScenario &S, const RefState &st, int e, int i,
                   int j, float ci, float si, int code_i, int code_j, double *margin)
{
    const int N = P.num_units, ki = e * N + i, kj = e * N + j;
    PairView V;
    V.dx = st.x[kj] - st.x[ki];
    V.dy = st.y[kj] - st.y[ki];
    V.d2 = (V.dx * V.dx) + (V.dy * V.dy);
    float R = S.sight_range[i];
    bool in_range = V.d2 <= R * R;
    float dot = (V.dx * ci) + (V.dy * si);
    float dist = std::sqrt(V.d2);
    bool in_cone = (V.d2 == 0.0f) || (dot >= S.sight_cos_half[i] * dist);
    if (margin) {
        double m = std::fabs((double)dist - (double)R);
        if (m < *margin) *margin = m;
        if (dist > 0.0f) {
            double cosang = (double)dot / (double)dist;
            if (cosang > 1.0) cosang = 1.0;
            if (cosang < -1.0) cosang = -1.0;
            double half = std::acos((double)S.sight_cos_half[i]);
            m = std::fabs(std::acos(cosang) - half);
            if (in_range && m < *margin) *margin = m;
        }
    }
    V.same_team = S.team[i] == S.team[j];
    bool bush_j = (code_j & 3) == ZONE_BUSH;
    bool same_bush = bush_j && (code_i & 3) == ZONE_BUSH && code_i == code_j;
    bool concealed = bush_j && !V.same_team && !same_bush && !(st.reveal[kj] > 0.0f);
    V.visible = in_range && in_cone && !concealed;

    float d2h;
    double mh;
    bool overlap = hurtbox_hit(st.x[ki], st.y[ki], ci, si, S.range[i], S.hurt_halfwidth[i],
                               st.x[kj], st.y[kj], S.radius[j], &d2h, margin ? &mh : nullptr);
    bool allowed = role_allows(S.dmg[i], S.team[i], S.team[j]);
    if (margin && allowed && mh < *margin) *margin = mh;
    if (P.hurtbox_cone) overlap = overlap && in_cone;
    V.attackable = overlap && allowed;
    return V;
}

void observe_env(const RefParams &P, const RefScenario &S, const RefState &st, int e,
                 float *obs, unsigned long long *vis_mask, unsigned char *action_mask,
                 double *min_margin)
{
    const int N = P.num_units, Z = P.max_zones, b = e * N;
    const int D = tabx_ref_obs_dim(&P);
    const int words = (N + 63) / 64;
    std::vector<float> c(N), s(N);
    std::vector<int> code(N);
    for (int u = 0; u < N; ++u) {
        sincos_spec(st.theta[b + u], &s[u], &c[u]);
        code[u] = cell_code(P, S, st.x[b + u], st.y[b + u]);
    }

    for (int i = 0; i < N; ++i) {
        const int ki = b + i;
        float *row = obs + ((long)ki) * D;
        for (int o = 0; o < D; ++o) row[o] = 0.0f;
        if (vis_mask)
            for (int w = 0; w < words; ++w) vis_mask[(long)ki * words + w] = 0ull;
        if (action_mask)
            action_mask[ki] = (st.alive[ki] && st.cd[ki] <= 0.0f) ? 1 : 0;
        if (!S.enabled[i]) continue;

        /* own block */
        own_block(P, S, st, e, i, code[i], row);

        /* other units, ascending index, self skipped */
        int slot = 0;
        for (int j = 0; j < N; ++j) {
            if (j == i) continue;
            const int kj = b + j;
            float *o = row + 16 + 16 * slot;
            slot += 1;
            if (!st.alive[ki] || !st.alive[kj]) continue;

            const PairView V = pair_view(P, S, st, e, i, j, c[i], s[i], code[i], code[j],
                                         min_margin ? &min_margin[e] : nullptr);
            const float dx = V.dx, dy = V.dy;
            const bool visible = V.visible, same_team = V.same_team, attackable = V.attackable;

            if (!visible) continue;
            if (vis_mask) vis_mask[(long)ki * words + (j >> 6)] |= 1ull << (j & 63);
            o[0] = st.hp[kj];
            o[1] = st.hp[kj] / S.hmax[j];
            o[2] = dx;
            o[3] = dy;
            o[4] = st.theta[kj];
            o[5] = S.range[j];
            o[6] = S.dmg[j];
            o[7] = st.cd[kj];
            o[8] = S.cooldown[j] != 0.0f ? st.cd[kj] / S.cooldown[j] : 0.0f;
            o[9] = S.radius[j];
            o[10] = S.mass[j];
            o[11] = S.sight_angle[j];
            o[12] = 1.0f;
            o[13] = same_team ? 1.0f : 0.0f;
            o[14] = attackable ? 1.0f : 0.0f;
            o[15] = st.cur_speed[kj];
        }

        /* zone descriptor slots; an inactive slot (type 0) stays zero */
        for (int z = 0; z < Z; ++z) {
            if (!S.zone_desc) break;
            const float *d = S.zone_desc + (long)z * 6;
            float *o = row + 16 * N + 6 * z;
            if (d[0] == 0.0f) continue;
            o[0] = d[0];
            o[1] = d[1] - st.x[ki];
            o[2] = d[2] - st.y[ki];
            o[3] = d[3];
            o[4] = d[4];
            o[5] = d[5];
        }
    }
}

/* ---- heuristic opponent ---------------------------------------------------------------
 * Counter-based random numbers: a 32-bit integer hash (two multiply / xor-shift rounds) of
 * (seed, env, unit, tick, draw index); the same function is written out in the GPU library. */
unsigned hash32(unsigned seed, unsigned env, unsigned unit, unsigned tick, unsigned draw)
{
    unsigned x = seed;
    x ^= env * 0x9E3779B9u;
    x ^= unit * 0x85EBCA6Bu;
    x ^= tick * 0xC2B2AE35u;
    x ^= draw * 0x27D4EB2Fu;
    x ^= x >> 16;
    x *= 0x7FEB352Du;
    x ^= x >> 15;
    x *= 0x846CA68Bu;
    x ^= x >> 16;
    return x;
}

/* The cardinal move that closes most of the offset (gx, gy); idle if there is none. */
int move_along(float gx, float gy)
{
    float ax = gx < 0.0f ? -gx : gx;
    float ay = gy < 0.0f ? -gy : gy;
    if (ax >= ay) return gx > 0.0f ? ACT_XP : (gx < 0.0f ? ACT_XM : ACT_NOOP);
    return gy > 0.0f ? ACT_YP : ACT_YM;
}

/* One unit's decision, in the priority order of App. A "Role-Appropriate Heuristic Policy
 * Mechanism": attack; rotate to bring the chosen target into the hurtbox; Rangers keep their
 * distance; navigate to the role's position at the target; pursue the last known position;
 * search (Rangers head for a bush first).  An epsilon-greedy override comes last. */
int policy_unit(const RefParams &P, const RefScenario &S, const RefState &st,
                const RefPolicy &pol, RefPolicyMemory &mem, int e, int i,
                const std::vector<float> &c, const std::vector<float> &s,
                const std::vector<int> &code)
{
    const int N = P.num_units, b = e * N, ki = b + i;
    const bool healer = S.dmg[i] < 0.0f;
    const bool assassin = S.speed[i] >= pol.assassin_speed;
    const bool ranger = S.range[i] >= pol.ranger_range;

    /* target selection among the visible units; nearest visible enemy; anything in reach */
    int tgt = -1, near_enemy = -1;
    float tgt_d2 = 0.0f, tgt_h = 0.0f, near_d2 = 0.0f;
    bool tgt_injured = false, can_hit = false, tgt_in_box = false;
    for (int j = 0; j < N; ++j) {
        if (j == i || !st.alive[b + j]) continue;
        const PairView V = pair_view(P, S, st, e, i, j, c[i], s[i], code[i], code[j], nullptr);
        if (!V.visible) continue;
        /* the combat action is worth taking: an enemy in the hurtbox, or for a healer an
         * ally there that is below its maximum health */
        if (V.attackable && (!healer || st.hp[b + j] < S.hmax[j])) can_hit = true;
        if (!V.same_team && (near_enemy < 0 || V.d2 < near_d2)) {
            near_enemy = j;
            near_d2 = V.d2;
        }
        bool better = false;
        if (healer) {          /* nearest injured ally, else nearest ally */
            if (V.same_team) {
                const bool injured = st.hp[b + j] < S.hmax[j];
                better = tgt < 0 || (injured && !tgt_injured) ||
                         (injured == tgt_injured && V.d2 < tgt_d2);
                if (better) tgt_injured = injured;
            }
        } else if (assassin) { /* lowest maximum health, then nearest */
            if (!V.same_team)
                better = tgt < 0 || S.hmax[j] < tgt_h ||
                         (S.hmax[j] == tgt_h && V.d2 < tgt_d2);
        } else {               /* nearest enemy */
            if (!V.same_team) better = tgt < 0 || V.d2 < tgt_d2;
        }
        if (better) {
            tgt = j;
            tgt_d2 = V.d2;
            tgt_h = S.hmax[j];
            tgt_in_box = V.attackable;
        }
    }

    const unsigned tick = (unsigned)st.t[e];
    const unsigned coin = hash32(pol.seed, env_id(P, e), (unsigned)i, tick, 2u) & 1u;
    const int search_turn = coin ? ACT_ROT_L : ACT_ROT_R;
    int act = ACT_NOOP;
    if (tgt >= 0) {
        const int kt = b + tgt;
        mem.mem_x[ki] = st.x[kt];
        mem.mem_y[ki] = st.y[kt];
        mem.mem_valid[ki] = 1;
        const float tdx = st.x[kt] - st.x[ki];
        const float tdy = st.y[kt] - st.y[ki];
        const float reach = S.range[i] + S.radius[tgt];
        const bool within = tgt_d2 <= reach * reach;
        const float kite = pol.xi * S.range[i];
        if (can_hit && st.cd[ki] <= 0.0f) {
            act = ACT_ATTACK;
        } else if (within && !tgt_in_box) {
            /* turn towards the side the target is on */
            const float lx = (tdx * c[i]) + (tdy * s[i]);
            const float ly = (tdy * c[i]) - (tdx * s[i]);
            act = ly > 0.0f ? ACT_ROT_L : (ly < 0.0f ? ACT_ROT_R : (lx < 0.0f ? ACT_ROT_L : ACT_NOOP));
        } else if (ranger && near_enemy >= 0 && near_d2 < kite * kite) {
            act = move_along(st.x[ki] - st.x[b + near_enemy], st.y[ki] - st.y[b + near_enemy]);
        } else if (tgt_in_box) {
            act = ACT_NOOP;            /* aligned, waiting for the cooldown */
        } else {
            /* Assassins go behind the target, Healers to it, the rest in front of it */
            float ct, st_;
            sincos_spec(st.theta[kt], &st_, &ct);
            const float standoff = 0.5f * S.range[i];
            float gx = st.x[kt], gy = st.y[kt];
            if (!healer) {
                if (assassin) {
                    gx = gx - (ct * standoff);
                    gy = gy - (st_ * standoff);
                } else {
                    gx = gx + (ct * standoff);
                    gy = gy + (st_ * standoff);
                }
            }
            act = move_along(gx - st.x[ki], gy - st.y[ki]);
        }
    } else if (mem.mem_valid[ki]) {
        const float gx = mem.mem_x[ki] - st.x[ki];
        const float gy = mem.mem_y[ki] - st.y[ki];
        if ((gx * gx) + (gy * gy) <= 1.0f) {
            mem.mem_valid[ki] = 0;
            act = search_turn;
        } else {
            act = move_along(gx, gy);
        }
    } else {
        /* Rangers outside a bush walk to the nearest bush zone they know of, then search */
        int bush = -1;
        float bush_d2 = 0.0f, bx = 0.0f, by = 0.0f;
        if (ranger && (code[i] & 3) != ZONE_BUSH && S.zone_desc) {
            for (int z = 0; z < P.max_zones; ++z) {
                const float *d = S.zone_desc + (long)z * 6;
                if ((int)d[0] != ZONE_BUSH) continue;
                const float zx = d[1] - st.x[ki];
                const float zy = d[2] - st.y[ki];
                const float d2 = (zx * zx) + (zy * zy);
                if (bush < 0 || d2 < bush_d2) {
                    bush = z;
                    bush_d2 = d2;
                    bx = zx;
                    by = zy;
                }
            }
        }
        act = bush >= 0 ? move_along(bx, by) : search_turn;
    }

    /* epsilon-greedy override */
    const unsigned h0 = hash32(pol.seed, env_id(P, e), (unsigned)i, tick, 0u);
    const float u0 = (float)(h0 >> 8) * (1.0f / 16777216.0f);
    if (u0 < pol.epsilon) act = (int)(hash32(pol.seed, env_id(P, e), (unsigned)i, tick, 1u) & 7u);
    return act;
}

void policy_env(const RefParams &P, const RefScenario &S, const RefState &st,
                const RefPolicy &pol, RefPolicyMemory &mem, int e,
                const unsigned char *controlled, unsigned char *actions)
{
    const int N = P.num_units, b = e * N;
    std::vector<float> c(N), s(N);
    std::vector<int> code(N);
    for (int u = 0; u < N; ++u) {
        sincos_spec(st.theta[b + u], &s[u], &c[u]);
        code[u] = cell_code(P, S, st.x[b + u], st.y[b + u]);
    }
    for (int i = 0; i < N; ++i) {
        const int ki = b + i;
        if (!controlled[ki] || !S.enabled[i] || !st.alive[ki]) continue;
        actions[ki] = (unsigned char)policy_unit(P, S, st, pol, mem, e, i, c, s, code);
    }
}

} /* namespace */

extern "C" {

unsigned tabx_ref_hash(unsigned seed, unsigned env, unsigned unit, unsigned tick, unsigned draw)
{
    return hash32(seed, env, unit, tick, draw);
}

void tabx_ref_heuristic_actions(const RefParams *p, const RefScenario *sc, const RefState *st,
                                const RefPolicy *pol, RefPolicyMemory *mem,
                                const unsigned char *controlled, unsigned char *actions)
{
    for (int e = 0; e < p->num_envs; ++e)
        policy_env(*p, level_slice(*p, *sc, *st, e), *st, *pol, *mem, e, controlled, actions);
}


int tabx_ref_obs_dim(const RefParams *p)
{
    return 16 * p->num_units + 6 * p->max_zones;
}

void tabx_ref_sincos(float theta, float *s, float *c) { sincos_spec(theta, s, c); }

void tabx_ref_sincos_n(const float *theta, int n, float *s, float *c)
{
    for (int k = 0; k < n; ++k) sincos_spec(theta[k], &s[k], &c[k]);
}

void tabx_ref_reset(const RefParams *p, const RefScenario *sc, RefState *st,
                    const unsigned char *env_mask)
{
    for (int e = 0; e < p->num_envs; ++e)
        if (!env_mask || env_mask[e]) {
            advance_level(*p, *st, e);
            reset_env(*p, level_slice(*p, *sc, *st, e), *st, e);
        }
}

void tabx_ref_step(const RefParams *p, const RefScenario *sc, RefState *st,
                   const unsigned char *actions, float *rewards, unsigned char *dones,
                   double *min_margin)
{
    for (int e = 0; e < p->num_envs; ++e)
        step_env(*p, *sc, *st, e, actions, rewards, dones, min_margin);
}

void tabx_ref_observe(const RefParams *p, const RefScenario *sc, const RefState *st,
                      float *obs, unsigned long long *vis_mask,
                      unsigned char *action_mask, double *min_margin)
{
    for (int e = 0; e < p->num_envs; ++e)
        observe_env(*p, level_slice(*p, *sc, *st, e), *st, e, obs, vis_mask, action_mask, min_margin);
}

void tabx_ref_global_state(const RefParams *p, const RefScenario *sc, const RefState *st,
                           float *out)
{
    const long Dg = 16 * p->num_units + 6 * p->max_zones;
    for (int e = 0; e < p->num_envs; ++e) global_state_env(*p, level_slice(*p, *sc, *st, e), *st, e, out + e * Dg);
}

} /* extern "C" */
