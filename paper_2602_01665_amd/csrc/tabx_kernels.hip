// TABX batched battle-environment step and observation for MI355X (gfx950).
//
// One workgroup advances one environment.  Lane u owns unit u during the
// per-unit stages (state and specification live in its registers); the unit
// data other lanes need is published in LDS and read back as broadcasts in the
// all-pairs loops (hurtbox, visibility).  The observation tensor, which is
// almost all of the HBM traffic, is written row by row with one lane per output
// float so that every store instruction covers 256 contiguous bytes.
//
// The rules follow the paper's App. A ("Interaction Dynamics", "Reward",
// "Observation and Global State", "Zones").  All arithmetic is float32 with one
// rounding per written operation: the file is compiled with -ffp-contract=off
// and uses fmaf only where it is spelled out.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "tabx.h"

#pragma clang fp contract(off)

namespace tabx {

struct KArgs {
    TabxParams   p;
    TabxScenario sc;
    TabxState    st;
    const uint8_t *actions;
    const uint8_t *env_mask;
    float    *rewards;
    uint8_t  *dones;
    float    *obs;
    uint64_t *vis_mask;
    uint8_t  *action_mask;
    int       obs_dim;
};

constexpr float kTwoPi = 6.28318530717958647692f;

// Sine and cosine of a heading in [0, 2*pi]: quadrant index n = trunc(theta *
// 2/pi + 1/2), remainder through a two-term split of pi/2, degree-9 / degree-8
// Taylor polynomials in Horner form with explicit fused multiply-adds.
__device__ __forceinline__ void heading_sincos(float theta, float &s, float &c)
{
    float q = theta * 0.63661977236758134308f;
    q = q + 0.5f;
    const int   n  = (int)q;
    const float fn = (float)n;
    float r = __builtin_fmaf(-fn, 1.57079637050628662109375f, theta);
    r       = __builtin_fmaf(-fn, -4.37113882867379435e-8f, r);
    const float r2 = r * r;
    float ps = __builtin_fmaf(r2, 1.0f / 362880.0f, -1.0f / 5040.0f);
    ps       = __builtin_fmaf(r2, ps, 1.0f / 120.0f);
    ps       = __builtin_fmaf(r2, ps, -1.0f / 6.0f);
    const float r3 = r * r2;
    const float sr = __builtin_fmaf(r3, ps, r);
    float pc = __builtin_fmaf(r2, 1.0f / 40320.0f, -1.0f / 720.0f);
    pc       = __builtin_fmaf(r2, pc, 1.0f / 24.0f);
    pc       = __builtin_fmaf(r2, pc, -0.5f);
    const float cr = __builtin_fmaf(r2, pc, 1.0f);
    const int quad = n & 3;
    const float a = (quad & 1) ? cr : sr;          // |sin| source
    const float b = (quad & 1) ? sr : cr;          // |cos| source
    s = (quad & 2) ? -a : a;
    c = (quad == 1 || quad == 2) ? -b : b;
}

__device__ __forceinline__ float clamp_between(float v, float lo, float hi)
{
    return v < lo ? lo : (v > hi ? hi : v);
}

// Registers of one unit: mutable state, then read-only specification.
struct Unit {
    float x, y, vx, vy, theta, hp, cd, reveal, cur_speed;
    int   alive;
    float hmax, radius, mass, speed, dmg, range, cooldown;
    float sight_angle, cos_half, sight_range, hurt_hw;
    int   team, enabled;
};

template <int NMAX>
struct EnvShared {
    float x[NMAX], y[NMAX], c[NMAX], s[NMAX], radius[NMAX];
    float dealt[NMAX];            // damage parameter of a unit whose attack landed
    int   target[NMAX];           // designated victim or -1
    float ratio[NMAX];            // hp / hmax of enabled units, else 0
    int   code[NMAX];             // terrain cell code under the unit
    uint8_t alive[NMAX], team[NMAX], enabled[NMAX], hidden[NMAX];
    float tab[NMAX][16];          // per-unit observation features
    uint64_t vis[NMAX][(NMAX + 63) / 64];
    uint64_t att[NMAX][(NMAX + 63) / 64];
    float zone[TABX_Z_MAX][6];
};

__device__ __forceinline__ int terrain_code(const KArgs &a, int e, float x, float y)
{
    if (a.sc.terrain == nullptr) return 0;
    int cx = (int)(x / a.p.cell_size);
    int cy = (int)(y / a.p.cell_size);
    cx = cx > a.p.grid_w - 1 ? a.p.grid_w - 1 : cx;
    cy = cy > a.p.grid_h - 1 ? a.p.grid_h - 1 : cy;
    cx = cx < 0 ? 0 : cx;
    cy = cy < 0 ? 0 : cy;
    return (int)a.sc.terrain[((size_t)e * a.p.grid_h + cy) * a.p.grid_w + cx];
}

__device__ __forceinline__ void load_spec(const KArgs &a, size_t k, Unit &U)
{
    U.hmax = a.sc.hmax[k];
    U.radius = a.sc.radius[k];
    U.mass = a.sc.mass[k];
    U.speed = a.sc.speed[k];
    U.dmg = a.sc.dmg[k];
    U.range = a.sc.range[k];
    U.cooldown = a.sc.cooldown[k];
    U.sight_angle = a.sc.sight_angle[k];
    U.cos_half = a.sc.sight_cos_half[k];
    U.sight_range = a.sc.sight_range[k];
    U.hurt_hw = a.sc.hurt_halfwidth[k];
    U.team = a.sc.team[k];
    U.enabled = a.sc.enabled[k];
}

__device__ __forceinline__ void load_state(const KArgs &a, size_t k, Unit &U)
{
    U.x = a.st.x[k];
    U.y = a.st.y[k];
    U.vx = a.st.vx[k];
    U.vy = a.st.vy[k];
    U.theta = a.st.theta[k];
    U.hp = a.st.hp[k];
    U.cd = a.st.cd[k];
    U.reveal = a.st.reveal[k];
    U.cur_speed = a.st.cur_speed[k];
    U.alive = a.st.alive[k];
}

__device__ __forceinline__ void store_state(const KArgs &a, size_t k, const Unit &U)
{
    a.st.x[k] = U.x;
    a.st.y[k] = U.y;
    a.st.vx[k] = U.vx;
    a.st.vy[k] = U.vy;
    a.st.theta[k] = U.theta;
    a.st.hp[k] = U.hp;
    a.st.cd[k] = U.cd;
    a.st.reveal[k] = U.reveal;
    a.st.cur_speed[k] = U.cur_speed;
    a.st.alive[k] = (uint8_t)U.alive;
}

// Episode start for one unit: spawn pose, full health, timers cleared.
__device__ __forceinline__ void spawn_unit(const KArgs &a, int e, size_t k, Unit &U)
{
    U.x = a.sc.init_x[k];
    U.y = a.sc.init_y[k];
    U.theta = a.sc.init_theta[k];
    U.vx = 0.0f;
    U.vy = 0.0f;
    U.hp = U.enabled ? U.hmax : 0.0f;
    U.cd = 0.0f;
    U.reveal = 0.0f;
    U.alive = U.enabled ? 1 : 0;
    const int zone = terrain_code(a, e, U.x, U.y) & 3;
    U.cur_speed = zone == TABX_ZONE_SWAMP ? U.speed * a.p.swamp_mult : U.speed;
}

// Mean health ratios of both teams from the ratios published in LDS, summed in
// ascending unit index (Eq. 1), and the per-team alive counts.  Every lane runs
// the same loop over broadcast reads and ends up with the same values.
template <int NMAX>
__device__ __forceinline__ void team_means(const EnvShared<NMAX> &sh, int N, float &m0,
                                           float &m1, int &alive0, int &alive1)
{
    float s0 = 0.0f, s1 = 0.0f;
    int c0 = 0, c1 = 0;
    alive0 = 0;
    alive1 = 0;
    for (int u = 0; u < N; ++u) {
        const bool en = sh.enabled[u] != 0;
        const bool t1 = sh.team[u] != 0;
        const float q = sh.ratio[u];
        // adding +0.0f leaves a finite sum unchanged, so the selects are exact
        s0 = s0 + ((en && !t1) ? q : 0.0f);
        s1 = s1 + ((en && t1) ? q : 0.0f);
        c0 += (en && !t1) ? 1 : 0;
        c1 += (en && t1) ? 1 : 0;
        alive0 += (sh.alive[u] && !t1) ? 1 : 0;
        alive1 += (sh.alive[u] && t1) ? 1 : 0;
    }
    m0 = c0 > 0 ? s0 / (float)c0 : 0.0f;
    m1 = c1 > 0 ? s1 / (float)c1 : 0.0f;
}

// Hurtbox overlap: attacker i's forward rectangle [0, L] x [-hw, hw] against
// the body circle of j (closest point of the rectangle to the circle centre).
__device__ __forceinline__ bool hurtbox_overlap(float dx, float dy, float ci, float si,
                                                float L, float hw, float rj)
{
    const float lx = (dx * ci) + (dy * si);
    const float ly = (dy * ci) - (dx * si);
    const float ex = lx - clamp_between(lx, 0.0f, L);
    const float ey = ly - clamp_between(ly, -hw, hw);
    return (ex * ex) + (ey * ey) <= rj * rj;
}

template <int NMAX>
__device__ __forceinline__ void step_env(const KArgs &a, EnvShared<NMAX> &sh, int e, int u,
                                         bool has, size_t k, Unit &U)
{
    const int N = a.p.num_units;
    const float dt = a.p.dt;
    const int alive0 = has ? U.alive : 0;
    const int act = has ? (int)a.actions[k] : 0;
    float bdmg = 0.0f;

    // stage 1: cooldown / reveal timers, explicit Euler move, arena penalty + clip
    if (has && U.enabled) {
        float v = U.cd - dt;
        U.cd = v > 0.0f ? v : 0.0f;
        v = U.reveal - dt;
        U.reveal = v > 0.0f ? v : 0.0f;
        if (alive0) {
            const float nx = U.x + U.vx * dt;
            const float ny = U.y + U.vy * dt;
            const bool oob = (nx < 0.0f) || (nx > a.p.map_w) || (ny < 0.0f) || (ny > a.p.map_h);
            if (oob) bdmg = (a.p.boundary_frac * U.hmax) * dt;
            U.x = clamp_between(nx, 0.0f, a.p.map_w);
            U.y = clamp_between(ny, 0.0f, a.p.map_h);
        }
    }

    // stage 2a: movement sets next tick's velocity, rotation turns the heading now
    float cu = 1.0f, su = 0.0f;
    if (has) {
        U.vx = 0.0f;
        U.vy = 0.0f;
        if (alive0) {
            const float sp = U.cur_speed;
            if (act == TABX_ACT_MOVE_XP) U.vx = sp;
            else if (act == TABX_ACT_MOVE_YP) U.vy = sp;
            else if (act == TABX_ACT_MOVE_XM) U.vx = -sp;
            else if (act == TABX_ACT_MOVE_YM) U.vy = -sp;
            else if (act == TABX_ACT_ROT_LEFT) {
                float th = U.theta + (a.p.turn_rate * dt);
                if (th >= kTwoPi) th = th - kTwoPi;
                U.theta = th;
            } else if (act == TABX_ACT_ROT_RIGHT) {
                float th = U.theta - (a.p.turn_rate * dt);
                if (th < 0.0f) th = th + kTwoPi;
                U.theta = th;
            }
        }
        heading_sincos(U.theta, su, cu);
        sh.x[u] = U.x;
        sh.y[u] = U.y;
        sh.radius[u] = U.radius;
        sh.alive[u] = (uint8_t)alive0;
        sh.team[u] = (uint8_t)U.team;
        sh.enabled[u] = (uint8_t)U.enabled;
    }
    __syncthreads();

    // stage 2b: attackable row of unit u, closest valid target (ties: lowest index)
    int target = -1;
    if (has && alive0) {
        float best = 0.0f;
        const bool heals = U.dmg < 0.0f;
        for (int j = 0; j < N; ++j) {
            const bool allowed = heals ? (sh.team[j] == U.team) : (sh.team[j] != U.team);
            const float dx = sh.x[j] - U.x;
            const float dy = sh.y[j] - U.y;
            const bool hit = hurtbox_overlap(dx, dy, cu, su, U.range, U.hurt_hw, sh.radius[j]);
            const float d2 = (dx * dx) + (dy * dy);
            const bool ok = (j != u) && sh.alive[j] && allowed && hit;
            if (ok && (target < 0 || d2 < best)) {
                target = j;
                best = d2;
            }
        }
    }
    const bool eligible = has && alive0 && act == TABX_ACT_ATTACK && U.cd <= 0.0f;
    if (eligible) U.cd = U.cooldown;
    const bool landed = eligible && target >= 0;
    if (has) {
        sh.target[u] = landed ? target : -1;
        sh.dealt[u] = U.dmg;
    }
    __syncthreads();

    // stage 2c: victim side.  Sum what the attackers that designated this unit
    // deal, ascending attacker index; subtract once with the arena penalty; clamp.
    if (has && alive0) {
        float acc = 0.0f;
        bool struck = landed && U.dmg > 0.0f;
        for (int i = 0; i < N; ++i) {
            const bool mine = sh.target[i] == u;
            const float d = sh.dealt[i];
            acc = acc + (mine ? d : 0.0f);
            struck = struck || (mine && d > 0.0f);
        }
        const float h = (U.hp - acc) - bdmg;
        U.hp = clamp_between(h, 0.0f, U.hmax);
        if (struck) U.reveal = a.p.reveal_time;
    }

    // stage 3: zone effects at the new position, alive flag
    if (has) {
        if (U.enabled) {
            const int zone = terrain_code(a, e, U.x, U.y) & 3;
            if (alive0 && zone == TABX_ZONE_LAVA) {
                const float h = U.hp - (a.p.lava_dps * dt);
                U.hp = h > 0.0f ? h : 0.0f;
            }
            U.cur_speed = zone == TABX_ZONE_SWAMP ? U.speed * a.p.swamp_mult : U.speed;
            U.alive = U.hp > 0.0f ? 1 : 0;
        } else {
            U.alive = 0;
        }
        sh.ratio[u] = U.enabled ? U.hp / U.hmax : 0.0f;
    }
    __syncthreads();           // everyone is done reading sh.alive as "alive at entry"
    if (has) sh.alive[u] = (uint8_t)U.alive;
    __syncthreads();

    // reward (Eq. 1), termination, terminal bonus
    float m0, m1;
    int n0, n1;
    team_means(sh, N, m0, m1, n0, n1);
    const int t_new = a.st.t[e] + 1;
    const float phi = m0 - m1;
    const float dense = phi - a.st.phi_prev[e];
    float r0 = dense, r1 = -dense;
    const bool done = n0 == 0 || n1 == 0 || t_new >= a.p.max_steps;
    if (done) {
        const bool ally_win = m0 > m1;
        r0 = r0 + (ally_win ? 1.0f : -1.0f);
        r1 = r1 + (ally_win ? -1.0f : 1.0f);
    }
    if (has) a.rewards[k] = U.enabled ? (U.team ? r1 : r0) : 0.0f;
    __syncthreads();           // all lanes have read t / phi_prev before lane 0 rewrites them

    float phi_next = phi;
    if (done) {                // uniform over the workgroup
        if (has) {
            spawn_unit(a, e, k, U);
            sh.ratio[u] = U.enabled ? U.hp / U.hmax : 0.0f;
            sh.alive[u] = (uint8_t)U.alive;
        }
        __syncthreads();
        team_means(sh, N, m0, m1, n0, n1);
        phi_next = m0 - m1;
    }
    if (u == 0) {
        a.st.t[e] = done ? 0 : t_new;
        a.st.phi_prev[e] = phi_next;
        a.dones[e] = done ? 1 : 0;
    }
    if (has) store_state(a, k, U);
}

template <int LPE, int NMAX>
__device__ __forceinline__ void observe_env(const KArgs &a, EnvShared<NMAX> &sh, int e, int u,
                                            bool has, size_t k, const Unit &U)
{
    constexpr int W = (NMAX + 63) / 64;
    const int N = a.p.num_units;
    const int Z = a.p.max_zones;
    const int D = a.obs_dim;

    float cu = 1.0f, su = 0.0f;
    int code_u = 0;
    __syncthreads();           // LDS may still be read by the step stage of slower waves
    if (has) {
        heading_sincos(U.theta, su, cu);
        code_u = terrain_code(a, e, U.x, U.y);
        sh.x[u] = U.x;
        sh.y[u] = U.y;
        sh.radius[u] = U.radius;
        sh.alive[u] = (uint8_t)U.alive;
        sh.team[u] = (uint8_t)U.team;
        sh.enabled[u] = (uint8_t)U.enabled;
        sh.code[u] = code_u;
        sh.hidden[u] = ((code_u & 3) == TABX_ZONE_BUSH && !(U.reveal > 0.0f)) ? 1 : 0;
        float *t = sh.tab[u];
        t[0] = U.hp;
        t[1] = U.hp / U.hmax;
        t[2] = U.x;
        t[3] = U.y;
        t[4] = U.theta;
        t[5] = U.range;
        t[6] = U.dmg;
        t[7] = U.cd;
        t[8] = U.cooldown != 0.0f ? U.cd / U.cooldown : 0.0f;
        t[9] = U.radius;
        t[10] = U.mass;
        t[11] = U.sight_angle;
        t[12] = U.alive ? 1.0f : 0.0f;
        t[13] = U.cur_speed;
        t[14] = (float)(code_u & 3);
        t[15] = U.cur_speed;
        if (a.action_mask) a.action_mask[k] = (U.alive && U.cd <= 0.0f) ? 1 : 0;
    }
    for (int q = u; q < Z * 6; q += LPE)
        (&sh.zone[0][0])[q] = a.sc.zone_desc[(size_t)e * Z * 6 + q];
    __syncthreads();

    // visibility row and attackable row of unit u over all j
    if (has) {
        uint64_t vis[W], att[W];
#pragma unroll
        for (int w = 0; w < W; ++w) { vis[w] = 0; att[w] = 0; }
        if (U.alive) {
            const bool heals = U.dmg < 0.0f;
            const bool in_bush = (code_u & 3) == TABX_ZONE_BUSH;
            const float R2 = U.sight_range * U.sight_range;
            for (int j = 0; j < N; ++j) {
                const float dx = sh.x[j] - U.x;
                const float dy = sh.y[j] - U.y;
                const float d2 = (dx * dx) + (dy * dy);
                const float dot = (dx * cu) + (dy * su);
                const bool in_range = d2 <= R2;
                const bool in_cone = (d2 == 0.0f) || (dot >= U.cos_half * __builtin_sqrtf(d2));
                const bool same_team = sh.team[j] == U.team;
                const bool same_bush = in_bush && sh.code[j] == code_u;
                const bool concealed = sh.hidden[j] && !same_team && !same_bush;
                const bool pair = (j != u) && sh.alive[j];
                const bool v = pair && in_range && in_cone && !concealed;
                const bool allowed = heals ? same_team : !same_team;
                const bool hit = hurtbox_overlap(dx, dy, cu, su, U.range, U.hurt_hw, sh.radius[j]);
                const bool at = pair && allowed && hit;
                if (W == 1) {
                    vis[0] |= (uint64_t)v << j;
                    att[0] |= (uint64_t)at << j;
                } else {
#pragma unroll
                    for (int w = 0; w < W; ++w) {
                        if ((j >> 6) == w) {
                            vis[w] |= (uint64_t)v << (j & 63);
                            att[w] |= (uint64_t)at << (j & 63);
                        }
                    }
                }
            }
        }
        const int words = (N + 63) >> 6;
#pragma unroll
        for (int w = 0; w < W; ++w) {
            sh.vis[u][w] = vis[w];
            sh.att[u][w] = att[w];
            if (a.vis_mask && w < words) a.vis_mask[k * words + w] = vis[w];
        }
    }
    __syncthreads();

    // observation rows: wave `wv` writes rows wv, wv + waves, ...; lane = output float
    const int lane = u & 63;
    const int wv = u >> 6;
    constexpr int WAVES = LPE / 64;
    const int zone_start = 15 + 16 * (N - 1);
    for (int i = wv; i < N; i += WAVES) {
        float *row = a.obs + ((size_t)e * N + i) * D;
        const bool en = sh.enabled[i] != 0;
        const float xi = sh.x[i], yi = sh.y[i];
        const int team_i = sh.team[i];
        for (int o = lane; o < D; o += 64) {
            float v;
            if (o < 15) {
                v = sh.tab[i][o];
            } else if (o < zone_start) {
                const int q = o - 15;
                const int slot = q >> 4;
                const int f = q & 15;
                const int j = slot + (slot >= i ? 1 : 0);
                const bool seen = (sh.vis[i][j >> 6] >> (j & 63)) & 1;
                float t = sh.tab[j][f];
                if (f == 2) t = t - xi;
                if (f == 3) t = t - yi;
                if (f == 13) t = sh.team[j] == team_i ? 1.0f : 0.0f;
                if (f == 14) t = ((sh.att[i][j >> 6] >> (j & 63)) & 1) ? 1.0f : 0.0f;
                v = seen ? t : 0.0f;
            } else {
                const int q = o - zone_start;
                const int z = q / 6;
                const int g = q - 6 * z;
                float t = sh.zone[z][g];
                if (g == 1) t = t - xi;
                if (g == 2) t = t - yi;
                v = sh.zone[z][0] != 0.0f ? t : 0.0f;
            }
            row[o] = en ? v : 0.0f;
        }
    }
}

template <int LPE, int NMAX, bool DO_STEP, bool DO_OBS>
__global__ __launch_bounds__(LPE) void tabx_kernel(const KArgs a)
{
    __shared__ EnvShared<NMAX> sh;
    const int e = blockIdx.x;
    const int u = threadIdx.x;
    const bool has = u < a.p.num_units;
    const size_t k = (size_t)e * a.p.num_units + u;
    Unit U = {};
    if (has) {
        load_spec(a, k, U);
        load_state(a, k, U);
    }
    if (DO_STEP) step_env<NMAX>(a, sh, e, u, has, k, U);
    if (DO_OBS) observe_env<LPE, NMAX>(a, sh, e, u, has, k, U);
}

template <int LPE, int NMAX>
__global__ __launch_bounds__(LPE) void tabx_reset_kernel(const KArgs a)
{
    __shared__ EnvShared<NMAX> sh;
    const int e = blockIdx.x;
    const int u = threadIdx.x;
    if (a.env_mask && a.env_mask[e] == 0) return;      // uniform over the workgroup
    const int N = a.p.num_units;
    const bool has = u < N;
    const size_t k = (size_t)e * N + u;
    Unit U = {};
    if (has) {
        load_spec(a, k, U);
        spawn_unit(a, e, k, U);
        sh.ratio[u] = U.enabled ? U.hp / U.hmax : 0.0f;
        sh.alive[u] = (uint8_t)U.alive;
        sh.team[u] = (uint8_t)U.team;
        sh.enabled[u] = (uint8_t)U.enabled;
        store_state(a, k, U);
    }
    __syncthreads();
    float m0, m1;
    int n0, n1;
    team_means(sh, N, m0, m1, n0, n1);
    if (u == 0) {
        a.st.t[e] = 0;
        a.st.phi_prev[e] = m0 - m1;
    }
}

// ------------------------------------------------------------------ host side

enum Mode { MODE_RESET, MODE_STEP, MODE_OBSERVE, MODE_STEP_OBSERVE };

static bool aligned(const void *p, size_t n) { return ((uintptr_t)p % n) == 0; }

static int check_params(const TabxParams *p)
{
    if (!p) return TABX_ERR_NULL;
    if (p->num_envs < 0 || p->num_units < 1 || p->num_units > TABX_N_MAX) return TABX_ERR_SHAPE;
    if (p->max_zones < 0 || p->max_zones > TABX_Z_MAX) return TABX_ERR_SHAPE;
    if (p->grid_w < 0 || p->grid_h < 0 || ((p->grid_w == 0) != (p->grid_h == 0)))
        return TABX_ERR_SHAPE;
    if (p->max_steps < 1) return TABX_ERR_SHAPE;
    if ((int64_t)p->num_envs * p->num_units > (int64_t)1 << 30) return TABX_ERR_SHAPE;
    const float pos[] = {p->map_w, p->map_h, p->cell_size, p->dt};
    for (float v : pos)
        if (!(v > 0.0f) || !(v < 3.0e38f)) return TABX_ERR_PARAM;
    const float fin[] = {p->turn_rate, p->lava_dps, p->swamp_mult, p->reveal_time,
                         p->boundary_frac};
    for (float v : fin)
        if (!(v > -3.0e38f && v < 3.0e38f)) return TABX_ERR_PARAM;
    return TABX_OK;
}

static int check_scenario(const TabxParams *p, const TabxScenario *s)
{
    if (!s) return TABX_ERR_NULL;
    const float *f[] = {s->init_x, s->init_y, s->init_theta, s->hmax, s->radius, s->mass,
                        s->speed, s->dmg, s->range, s->cooldown, s->sight_angle,
                        s->sight_cos_half, s->sight_range, s->hurt_halfwidth};
    for (const float *q : f) {
        if (!q) return TABX_ERR_NULL;
        if (!aligned(q, 4)) return TABX_ERR_ALIGN;
    }
    if (!s->team || !s->enabled) return TABX_ERR_NULL;
    if ((p->grid_w > 0) != (s->terrain != nullptr)) return TABX_ERR_NULL;
    if ((p->max_zones > 0) != (s->zone_desc != nullptr)) return TABX_ERR_NULL;
    if (s->zone_desc && !aligned(s->zone_desc, 4)) return TABX_ERR_ALIGN;
    return TABX_OK;
}

static int check_state(const TabxState *s)
{
    if (!s) return TABX_ERR_NULL;
    const float *f[] = {s->x, s->y, s->vx, s->vy, s->theta, s->hp, s->cd, s->reveal,
                        s->cur_speed, s->phi_prev};
    for (const float *q : f) {
        if (!q) return TABX_ERR_NULL;
        if (!aligned(q, 4)) return TABX_ERR_ALIGN;
    }
    if (!s->alive || !s->t) return TABX_ERR_NULL;
    if (!aligned(s->t, 4)) return TABX_ERR_ALIGN;
    return TABX_OK;
}

template <int LPE, int NMAX>
static void launch_mode(Mode mode, const KArgs &a, hipStream_t stream)
{
    const dim3 grid((unsigned)a.p.num_envs), block(LPE);
    switch (mode) {
    case MODE_RESET:
        hipLaunchKernelGGL((tabx_reset_kernel<LPE, NMAX>), grid, block, 0, stream, a);
        break;
    case MODE_STEP:
        hipLaunchKernelGGL((tabx_kernel<LPE, NMAX, true, false>), grid, block, 0, stream, a);
        break;
    case MODE_OBSERVE:
        hipLaunchKernelGGL((tabx_kernel<LPE, NMAX, false, true>), grid, block, 0, stream, a);
        break;
    case MODE_STEP_OBSERVE:
        hipLaunchKernelGGL((tabx_kernel<LPE, NMAX, true, true>), grid, block, 0, stream, a);
        break;
    }
}

static int run(Mode mode, const TabxParams *p, const TabxScenario *sc, const TabxState *st,
               const uint8_t *actions, const uint8_t *env_mask, float *rewards,
               uint8_t *dones, float *obs, uint64_t *vis_mask, uint8_t *action_mask,
               void *stream)
{
    int rc = check_params(p);
    if (rc) return rc;
    if (p->num_envs == 0) return TABX_OK;          // empty batch: nothing to validate or do
    if ((rc = check_scenario(p, sc))) return rc;
    if ((rc = check_state(st))) return rc;
    const bool stepping = mode == MODE_STEP || mode == MODE_STEP_OBSERVE;
    const bool observing = mode == MODE_OBSERVE || mode == MODE_STEP_OBSERVE;
    if (stepping) {
        if (!actions || !rewards || !dones) return TABX_ERR_NULL;
        if (!aligned(rewards, 4)) return TABX_ERR_ALIGN;
    }
    if (observing) {
        if (!obs) return TABX_ERR_NULL;
        if (!aligned(obs, 16) || (vis_mask && !aligned(vis_mask, 16))) return TABX_ERR_ALIGN;
    }
    KArgs a;
    a.p = *p;
    a.sc = *sc;
    a.st = *st;
    a.actions = actions;
    a.env_mask = env_mask;
    a.rewards = rewards;
    a.dones = dones;
    a.obs = obs;
    a.vis_mask = vis_mask;
    a.action_mask = action_mask;
    a.obs_dim = 15 + 16 * (p->num_units - 1) + 6 * p->max_zones;

    hipStream_t s = (hipStream_t)stream;
    (void)hipGetLastError();
    if (p->num_units <= 32) launch_mode<64, 32>(mode, a, s);
    else if (p->num_units <= 64) launch_mode<64, 64>(mode, a, s);
    else launch_mode<128, 128>(mode, a, s);
    return hipGetLastError() == hipSuccess ? TABX_OK : TABX_ERR_LAUNCH;
}

} // namespace tabx

extern "C" {

int tabx_obs_dim(const TabxParams *p)
{
    const int rc = tabx::check_params(p);
    if (rc) return rc;
    return 15 + 16 * (p->num_units - 1) + 6 * p->max_zones;
}

int tabx_num_actions(void) { return TABX_NUM_ACTIONS; }

int tabx_reset(const TabxParams *p, const TabxScenario *sc, const TabxState *st,
               const uint8_t *env_mask, void *stream)
{
    return tabx::run(tabx::MODE_RESET, p, sc, st, nullptr, env_mask, nullptr, nullptr, nullptr,
                     nullptr, nullptr, stream);
}

int tabx_step(const TabxParams *p, const TabxScenario *sc, const TabxState *st,
              const uint8_t *actions, float *rewards, uint8_t *dones, void *stream)
{
    return tabx::run(tabx::MODE_STEP, p, sc, st, actions, nullptr, rewards, dones, nullptr,
                     nullptr, nullptr, stream);
}

int tabx_observe(const TabxParams *p, const TabxScenario *sc, const TabxState *st, float *obs,
                 uint64_t *vis_mask, uint8_t *action_mask, void *stream)
{
    return tabx::run(tabx::MODE_OBSERVE, p, sc, st, nullptr, nullptr, nullptr, nullptr, obs,
                     vis_mask, action_mask, stream);
}

int tabx_step_observe(const TabxParams *p, const TabxScenario *sc, const TabxState *st,
                      const uint8_t *actions, float *rewards, uint8_t *dones, float *obs,
                      uint64_t *vis_mask, uint8_t *action_mask, void *stream)
{
    return tabx::run(tabx::MODE_STEP_OBSERVE, p, sc, st, actions, nullptr, rewards, dones, obs,
                     vis_mask, action_mask, stream);
}

const char *tabx_strerror(int code)
{
    switch (code) {
    case TABX_OK: return "ok";
    case TABX_ERR_NULL: return "a required pointer is NULL (or an optional one does not match the shape)";
    case TABX_ERR_SHAPE: return "unsupported shape (num_units, max_zones, grid, max_steps or num_envs)";
    case TABX_ERR_ALIGN: return "a pointer is not aligned as required";
    case TABX_ERR_LAUNCH: return "the HIP runtime refused the kernel launch";
    case TABX_ERR_PARAM: return "a physics constant is not finite or not positive";
    default: return "unknown error code";
    }
}

} // extern "C"
