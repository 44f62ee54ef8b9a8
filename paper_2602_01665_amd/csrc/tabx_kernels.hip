// TABX batched battle-environment step and observation for MI355X (gfx950).
//
// Work layout.  A 64-lane wavefront advances G = floor(64 / N) whole environments
// at once (N = units per env): lane l owns unit l % N of env slot l / N, so the
// struct-of-arrays state of the G envs is one contiguous, coalesced run of G*N
// elements per field.  For 64 < N <= 128 a workgroup of two wavefronts owns one
// env.  The per-unit stages run in registers; what other lanes need is published
// in LDS and read back as broadcasts inside the all-pairs loops (hurtbox,
// visibility), which every lane runs over the units of its own env.
//
// The observation tensor is almost all of the HBM traffic.  Its other-unit
// blocks are written by a flat loop over (row, slot) pairs with four lanes per
// 16-float block (one 16-byte store each, 1 KB contiguous per wave instruction);
// the own blocks and zone slots are written by two smaller loops.
//
// Kernel time is bounded by VALU issue, not by HBM, unless the instruction count
// per env is kept low; hence: boolean pair predicates are combined as scalar
// lane masks, per-row visibility is pre-shifted into slot order so that the
// writer needs one bit-field extract per block, and counts come from ballots.
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
    int       envs_per_block;      // G
    int       rows_per_group;      // observation rows staged in LDS per pass
    int       stage_floats;        // staging floats per wave (multiple of 4)
    int       stage_offset;        // staging offset in dynamic LDS, floats (multiple of 4)
};

typedef float f4u __attribute__((ext_vector_type(4), aligned(4)));   // 16-byte store, 4-byte aligned

constexpr float kTwoPi = 6.28318530717958647692f;
constexpr float kInf = __builtin_huge_valf();

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

// Same value as clamp_between for finite inputs with lo <= hi (the sign of a zero
// result may differ, which the callers square away); one instruction.
__device__ __forceinline__ float median3(float v, float lo, float hi)
{
    return __builtin_amdgcn_fmed3f(v, lo, hi);
}

// Registers of one unit: mutable state, then read-only specification.
struct Unit {
    float x, y, vx, vy, theta, hp, cd, reveal, cur_speed;
    int   alive;
    float hmax, radius, mass, speed, dmg, range, cooldown;
    float sight_angle, cos_half, sight_range, hurt_hw;
    int   team, enabled;
};

// Where a lane sits: env slot g of the workgroup, unit u of that env, `base` =
// workgroup lane of the env's unit 0, e = env index, k = e * N + u.
struct Place {
    int l, g, u, base, e;
    bool has;
    size_t k;
};

template <int WAVES, int NW>
struct Shared {
    static constexpr int L = 64 * WAVES;
    float4   pj[L];           // pair-loop record of a unit: x, y, r^2, flags
    int2     hitrec[L];       // {designated victim (local index) or -1, damage bits}
    float2   share[L];        // this unit's term in the team-0 / team-1 ratio sums
    float    tab[L][16];      // observation features of a unit
    float4   row[L];          // observer record: x, y, info bits
    uint32_t V[L][NW];        // visible, by slot (self bit dropped)
    uint32_t A[L][NW];        // attackable, by slot
    uint32_t T[L][NW];        // same team, by slot
    uint64_t ballots[WAVES][4];
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

// Episode start for one unit: spawn pose, full health, timers cleared.  Returns
// the terrain cell code under the spawn point.
__device__ __forceinline__ int spawn_unit(const KArgs &a, int e, size_t k, Unit &U)
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
    const int code = terrain_code(a, e, U.x, U.y);
    U.cur_speed = (code & 3) == TABX_ZONE_SWAMP ? U.speed * a.p.swamp_mult : U.speed;
    return code;
}

template <int WAVES>
__device__ __forceinline__ Place locate(const KArgs &a)
{
    Place P;
    const int N = a.p.num_units;
    P.l = threadIdx.x;
    if (WAVES == 1) {
        P.g = P.l / N;
        P.u = P.l - P.g * N;
    } else {
        P.g = 0;
        P.u = P.l;
    }
    P.e = blockIdx.x * a.envs_per_block + P.g;
    P.has = P.g < a.envs_per_block && P.u < N && P.e < a.p.num_envs;
    P.base = P.has ? P.l - P.u : 0;
    P.k = (size_t)P.e * N + P.u;
    return P;
}

// How many lanes of the caller's env satisfy each of four predicates.
template <int WAVES, int NW>
__device__ __forceinline__ void env_counts(Shared<WAVES, NW> &sh, const Place &P, int N,
                                           const bool (&pred)[4], int (&cnt)[4])
{
    if (WAVES == 1) {
        const uint64_t range = (N >= 64 ? ~0ull : ((1ull << N) - 1ull)) << P.base;
#pragma unroll
        for (int q = 0; q < 4; ++q) cnt[q] = __popcll(__ballot(pred[q]) & range);
    } else {
        const int wv = P.l >> 6;
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const uint64_t b = __ballot(pred[q]);
            if ((P.l & 63) == 0) sh.ballots[wv][q] = b;
        }
        __syncthreads();
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            cnt[q] = 0;
#pragma unroll
            for (int w = 0; w < WAVES; ++w) cnt[q] += __popcll(sh.ballots[w][q]);
        }
        __syncthreads();
    }
}

// Mean health ratio of both teams over their enabled units (the bracketed means of
// Eq. 1): the terms published in sh.share are added in ascending unit index; a term
// of +0.0f (unit of the other team, or disabled) leaves a finite sum unchanged.
template <int WAVES, int NW>
__device__ __forceinline__ void team_means(const Shared<WAVES, NW> &sh, const Place &P, int N,
                                           int c0, int c1, float &m0, float &m1)
{
    float s0 = 0.0f, s1 = 0.0f;
    for (int jj = 0; jj < N; ++jj) {
        const float2 q = sh.share[P.base + jj];
        s0 = s0 + q.x;
        s1 = s1 + q.y;
    }
    m0 = c0 > 0 ? s0 / (float)c0 : 0.0f;
    m1 = c1 > 0 ? s1 / (float)c1 : 0.0f;
}

// Squared gap between attacker i's forward rectangle [0, L] x [-hw, hw] and the
// centre of j (closest point of the rectangle), from j's offset (dx, dy);
// `along` returns the offset's component along i's heading.
__device__ __forceinline__ float hurtbox_gap2(float dx, float dy, float ci, float si, float L,
                                              float hw, float neg_hw, float &along)
{
    const float lx = (dx * ci) + (dy * si);
    const float ly = (dy * ci) - (dx * si);
    const float ex = lx - median3(lx, 0.0f, L);
    const float ey = ly - median3(ly, neg_hw, hw);
    along = lx;
    return (ex * ex) + (ey * ey);
}

template <int WAVES, int NW>
__device__ __forceinline__ void step_env(const KArgs &a, Shared<WAVES, NW> &sh, const Place &P,
                                         Unit &U, int &code_u)
{
    const int N = a.p.num_units;
    const float dt = a.p.dt;
    const bool has = P.has;
    const int alive0 = has ? U.alive : 0;
    const int act = has ? (int)a.actions[P.k] : 0;
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
    }
    // flags: team of a unit alive at entry, 2 for anything that cannot be a target
    sh.pj[P.l] = make_float4(U.x, U.y, U.radius * U.radius,
                             __int_as_float(alive0 ? U.team : 2));
    __syncthreads();

    // stage 2b: attackable row of this unit over its env, closest valid target
    // (strict "<" keeps the lowest index on ties)
    int target = -1;
    {
        const int want = (U.dmg < 0.0f) ? U.team : 1 - U.team;   // healers reach allies only
        const float neg_hw = -U.hurt_hw;
        float best = kInf;
        for (int jj = 0; jj < N; ++jj) {
            const float4 J = sh.pj[P.base + jj];
            const float dx = J.x - U.x;
            const float dy = J.y - U.y;
            float along;
            const float g2 = hurtbox_gap2(dx, dy, cu, su, U.range, U.hurt_hw, neg_hw, along);
            const float d2 = (dx * dx) + (dy * dy);
            const bool ok = (g2 <= J.z) && (__float_as_int(J.w) == want) && (jj != P.u);
            const bool take = ok && (d2 < best);
            best = take ? d2 : best;
            target = take ? jj : target;
        }
    }
    const bool eligible = has && alive0 && act == TABX_ACT_ATTACK && U.cd <= 0.0f;
    if (eligible) U.cd = U.cooldown;
    const bool landed = eligible && target >= 0;
    sh.hitrec[P.l] = make_int2(landed ? target : -1, __float_as_int(U.dmg));
    __syncthreads();

    // stage 2c: victim side.  Sum what the attackers that designated this unit
    // deal, ascending attacker index; subtract once with the arena penalty; clamp.
    {
        float acc = 0.0f;
        bool struck = landed && U.dmg > 0.0f;
        for (int ii = 0; ii < N; ++ii) {
            const int2 h = sh.hitrec[P.base + ii];
            const bool mine = h.x == P.u;
            const float d = __int_as_float(h.y);
            acc = acc + (mine ? d : 0.0f);
            struck = struck || (mine && d > 0.0f);
        }
        if (has && alive0) {
            const float h = (U.hp - acc) - bdmg;
            U.hp = clamp_between(h, 0.0f, U.hmax);
            if (struck) U.reveal = a.p.reveal_time;
        }
    }

    // stage 3: zone effects at the new position, alive flag
    float ratio = 0.0f;
    if (has) {
        if (U.enabled) {
            code_u = terrain_code(a, P.e, U.x, U.y);
            const int zone = code_u & 3;
            if (alive0 && zone == TABX_ZONE_LAVA) {
                const float h = U.hp - (a.p.lava_dps * dt);
                U.hp = h > 0.0f ? h : 0.0f;
            }
            U.cur_speed = zone == TABX_ZONE_SWAMP ? U.speed * a.p.swamp_mult : U.speed;
            U.alive = U.hp > 0.0f ? 1 : 0;
            ratio = U.hp / U.hmax;
        } else {
            U.alive = 0;
        }
    }
    const bool en = has && U.enabled;
    sh.share[P.l] = make_float2((en && U.team == 0) ? ratio : 0.0f,
                                (en && U.team != 0) ? ratio : 0.0f);
    const bool pred[4] = {en && U.team == 0, en && U.team != 0,
                          has && U.alive && U.team == 0, has && U.alive && U.team != 0};
    int cnt[4];
    env_counts(sh, P, N, pred, cnt);
    __syncthreads();

    // reward (Eq. 1), termination, terminal bonus
    float m0, m1;
    team_means(sh, P, N, cnt[0], cnt[1], m0, m1);
    const int t_new = has ? a.st.t[P.e] + 1 : 0;
    const float phi_prev = has ? a.st.phi_prev[P.e] : 0.0f;
    const float phi = m0 - m1;
    const float dense = phi - phi_prev;
    float r0 = dense, r1 = -dense;
    const bool done = has && (cnt[2] == 0 || cnt[3] == 0 || t_new >= a.p.max_steps);
    if (done) {
        const bool ally_win = m0 > m1;
        r0 = r0 + (ally_win ? 1.0f : -1.0f);
        r1 = r1 + (ally_win ? -1.0f : 1.0f);
    }
    if (has) a.rewards[P.k] = U.enabled ? (U.team ? r1 : r0) : 0.0f;

    // auto-reset of finished envs; the potential of the fresh state seeds phi_prev
    float phi_next = phi;
    if (__syncthreads_or(done ? 1 : 0)) {
        if (done) {
            code_u = spawn_unit(a, P.e, P.k, U);
            ratio = U.enabled ? U.hp / U.hmax : 0.0f;
        }
        sh.share[P.l] = make_float2((en && U.team == 0) ? ratio : 0.0f,
                                    (en && U.team != 0) ? ratio : 0.0f);
        __syncthreads();
        float f0, f1;
        team_means(sh, P, N, cnt[0], cnt[1], f0, f1);
        if (done) phi_next = f0 - f1;
    }
    if (has && P.u == 0) {
        a.st.t[P.e] = done ? 0 : t_new;
        a.st.phi_prev[P.e] = phi_next;
        a.dones[P.e] = done ? 1 : 0;
    }
    if (has) store_state(a, P.k, U);
}

// Removes bit i from a multi-word mask, moving the bits above it down by one.
template <int NW>
__device__ __forceinline__ void drop_bit(const uint32_t (&m)[NW], int i, uint32_t (&out)[NW])
{
#pragma unroll
    for (int w = 0; w < NW; ++w) {
        const int lo = i - 32 * w;          // bits of this word below `lo` keep their place
        const uint32_t keep = lo >= 32 ? 0xffffffffu : (lo <= 0 ? 0u : ((1u << lo) - 1u));
        const uint32_t next = (w + 1 < NW) ? m[w + 1] : 0u;
        const uint32_t shifted = (m[w] >> 1) | (next << 31);
        out[w] = (m[w] & keep) | (shifted & ~keep);
    }
}

template <int WAVES, int NW>
__device__ __forceinline__ void observe_env(const KArgs &a, Shared<WAVES, NW> &sh,
                                            float *zone_lds, const Place &P, const Unit &U,
                                            int code_u)
{
    constexpr int LANES = 64 * WAVES;
    const int N = a.p.num_units;
    const int G = a.envs_per_block;
    const int D = a.obs_dim;
    const int zlen = 6 * a.p.max_zones;
    const bool has = P.has;

    __syncthreads();                 // LDS of the step stage is free to reuse
    float cu = 1.0f, su = 0.0f;
    {
        const bool in_bush = (code_u & 3) == TABX_ZONE_BUSH;
        const int alive = has ? U.alive : 0;
        const int hidden = (in_bush && !(U.reveal > 0.0f)) ? 1 : 0;
        const int flags = alive | (U.team << 1) | (hidden << 2) | ((code_u & 0xff) << 8);
        sh.pj[P.l] = make_float4(U.x, U.y, U.radius * U.radius, __int_as_float(flags));
        const int info = P.u | (P.base << 8) | ((has && U.enabled) ? (1 << 16) : 0) | (P.g << 24);
        sh.row[P.l] = make_float4(U.x, U.y, __int_as_float(info), 0.0f);
        if (has) {
            heading_sincos(U.theta, su, cu);
            float4 *t = reinterpret_cast<float4 *>(sh.tab[P.l]);
            t[0] = make_float4(U.hp, U.hp / U.hmax, U.x, U.y);
            t[1] = make_float4(U.theta, U.range, U.dmg, U.cd);
            t[2] = make_float4(U.cooldown != 0.0f ? U.cd / U.cooldown : 0.0f, U.radius, U.mass,
                               U.sight_angle);
            // own block ends with (alive, speed, zone); other-unit blocks read the
            // speed from the last column and get columns 13, 14 from the masks
            t[3] = make_float4(U.alive ? 1.0f : 0.0f, U.cur_speed, (float)(code_u & 3),
                               U.cur_speed);
            if (a.action_mask) a.action_mask[P.k] = (U.alive && U.cd <= 0.0f) ? 1 : 0;
        }
    }
    // zone slots of each env slot: value (zero if the slot is inactive) and which
    // own coordinate to subtract (centre x / y of an active slot)
    float    *zv = zone_lds;
    uint32_t *zmx = reinterpret_cast<uint32_t *>(zone_lds + G * zlen);
    uint32_t *zmy = zmx + G * zlen;
    for (int q = P.l; q < G * zlen; q += LANES) {
        const int g = q / zlen;
        const int e = blockIdx.x * G + g;
        float v = 0.0f;
        uint32_t mx = 0, my = 0;
        if (e < a.p.num_envs) {
            const int zz = q - g * zlen;
            const int comp = zz % 6;
            const float *d = a.sc.zone_desc + (size_t)e * zlen;
            const bool active = d[zz - comp] != 0.0f;
            v = active ? d[zz] : 0.0f;
            mx = (active && comp == 1) ? 0xffffffffu : 0u;
            my = (active && comp == 2) ? 0xffffffffu : 0u;
        }
        zv[q] = v;
        zmx[q] = mx;
        zmy[q] = my;
    }
    __syncthreads();

    // visibility / attackable / same-team rows of this unit over its env
    uint32_t vis[NW], att[NW], same[NW];
    {
        const bool heals = U.dmg < 0.0f;
        const bool seer = has && U.alive;
        const float R2 = U.sight_range * U.sight_range;
        const float neg_hw = -U.hurt_hw;
        const int bush_key = ((code_u & 3) == TABX_ZONE_BUSH) ? (code_u & 0xff) : -1;
#pragma unroll
        for (int w = 0; w < NW; ++w) {
            uint32_t v = 0, t = 0, s = 0;
            const int jend = (N - 32 * w) < 32 ? (N - 32 * w) : 32;
            for (int b = 0; b < jend; ++b) {
                const int jj = 32 * w + b;
                const float4 J = sh.pj[P.base + jj];
                const int fj = __float_as_int(J.w);
                const float dx = J.x - U.x;
                const float dy = J.y - U.y;
                float dot;
                const float g2 = hurtbox_gap2(dx, dy, cu, su, U.range, U.hurt_hw, neg_hw, dot);
                const float d2 = (dx * dx) + (dy * dy);
                const bool in_range = d2 <= R2;
                const bool in_cone = (d2 == 0.0f) || (dot >= U.cos_half * __builtin_sqrtf(d2));
                const bool same_team = ((fj >> 1) & 1) == U.team;
                const bool same_bush = (fj >> 8) == bush_key;
                const bool concealed = (fj & 4) && !same_team && !same_bush;
                const bool pair = seer && (fj & 1) && (jj != P.u);
                const bool seen = pair && in_range && in_cone && !concealed;
                const bool hit = pair && (heals == same_team) && (g2 <= J.z);
                const uint32_t bit = 1u << b;
                v |= seen ? bit : 0u;
                t |= hit ? bit : 0u;
                s |= same_team ? bit : 0u;
            }
            vis[w] = v;
            att[w] = t;
            same[w] = s;
        }
    }
    if (has && a.vis_mask) {
        const int words = (N + 63) >> 6;
#pragma unroll
        for (int w = 0; w < (NW + 1) / 2; ++w) {
            const uint64_t lo = vis[2 * w];
            const uint64_t hi = (2 * w + 1 < NW) ? vis[2 * w + 1] : 0u;
            if (w < words) a.vis_mask[P.k * words + w] = lo | (hi << 32);
        }
    }
    {
        uint32_t sv[NW], sa[NW], st[NW];
        drop_bit<NW>(vis, P.u, sv);
        drop_bit<NW>(att, P.u, sa);
        drop_bit<NW>(same, P.u, st);
#pragma unroll
        for (int w = 0; w < NW; ++w) {
            sh.V[P.l][w] = sv[w];
            sh.A[P.l][w] = sa[w];
            sh.T[P.l][w] = st[w];
        }
    }
    __syncthreads();

    // ---- writer.  Rows are the units of this workgroup's envs in lane order.  Each wave
    // builds a group of whole rows in its LDS staging area (other-unit blocks, own
    // blocks, zone slots) and then streams the group to HBM front to back, 1 KB per
    // store instruction, so that every cache line is completed by consecutive stores;
    // rows written piecemeal leave partly written lines behind and cost twice the time.
    const int envs_here = (a.p.num_envs - blockIdx.x * G) < G ? (a.p.num_envs - blockIdx.x * G) : G;
    const int rows = envs_here * N;
    float *out = a.obs + (size_t)blockIdx.x * G * N * D;
    const int lane = P.l & 63;
    const int wv = P.l >> 6;
    const int RG = a.rows_per_group;
    float *stg = zone_lds + a.stage_offset + wv * a.stage_floats;
    const int n1 = N - 1;
    const int zoff = 15 + 16 * n1;
    const int grp = lane & 3;
    const bool first = grp == 0, last = grp == 3;
    // (row, slot) pair of this lane in the first pass over a group; a pass covers 16 pairs
    const int sp0 = lane >> 2;
    const int rl0 = n1 > 0 ? sp0 / n1 : 0;
    const int s0 = sp0 - rl0 * n1;
    const int wraps = n1 > 0 ? (16 + n1 - 1) / n1 : 0;
    // (row, zone float) of this lane in the first pass over a group's zone slots
    const int rlz0 = zlen > 0 ? lane / zlen : 0;
    const int zz0 = lane - rlz0 * zlen;
    const int wraps_z = zlen > 0 ? (64 + zlen - 1) / zlen : 0;

    for (int r0 = wv * RG; r0 < rows; r0 += WAVES * RG) {
        const int nr = (rows - r0) < RG ? (rows - r0) : RG;
        // other-unit blocks: four lanes per 16-float block
        {
            const int total = nr * n1;
            int rl = rl0, s = s0;
            for (int sp = sp0; sp < total; sp += 16) {
                const int r = r0 + rl;
                const float4 R = sh.row[r];
                const int info = __float_as_int(R.z);
                const int i = info & 0xff;
                const int rbase = (info >> 8) & 0xff;
                const int j = s + (s >= i ? 1 : 0);
                float4 t = *reinterpret_cast<const float4 *>(&sh.tab[rbase + j][grp * 4]);
                const int ws = (NW == 1) ? 0 : (s >> 5);
                const int seen = __builtin_amdgcn_sbfe((int)sh.V[r][ws], s & 31, 1);   // 0 or -1
                const int atk = __builtin_amdgcn_sbfe((int)sh.A[r][ws], s & 31, 1);
                const int ally = __builtin_amdgcn_sbfe((int)sh.T[r][ws], s & 31, 1);
                // relative position (first quarter), team / attackable flags (last quarter)
                t.z = t.z - (first ? R.x : 0.0f);
                t.w = t.w - (first ? R.y : 0.0f);
                const float one = 1.0f;
                t.y = last ? __int_as_float(ally & __float_as_int(one)) : t.y;
                t.z = last ? __int_as_float(atk & __float_as_int(one)) : t.z;
                float *d = stg + (rl * D + 15 + s * 16 + grp * 4);
                d[0] = __int_as_float(__float_as_int(t.x) & seen);
                d[1] = __int_as_float(__float_as_int(t.y) & seen);
                d[2] = __int_as_float(__float_as_int(t.z) & seen);
                d[3] = __int_as_float(__float_as_int(t.w) & seen);
                s += 16;
                for (int w = 0; w < wraps; ++w) {
                    const bool wrap = s >= n1;
                    s = wrap ? s - n1 : s;
                    rl = wrap ? rl + 1 : rl;
                }
            }
        }
        // own blocks: 16 lanes per row, 15 of them store
        {
            const int c = lane & 15;
            for (int rl = lane >> 4; rl < nr; rl += 4) {
                const int r = r0 + rl;
                const int info = __float_as_int(sh.row[r].z);
                const float v = sh.tab[r][c];
                if (c < 15) stg[rl * D + c] = (info & (1 << 16)) ? v : 0.0f;
            }
        }
        // zone slots: lane per float over the group's rows
        if (zlen > 0) {
            const int total = nr * zlen;
            int rl = rlz0, zz = zz0;
            for (int t = lane; t < total; t += 64) {
                const float4 R = sh.row[r0 + rl];
                const int info = __float_as_int(R.z);
                const int q = ((info >> 24) & 0xff) * zlen + zz;
                const uint32_t shift = (__float_as_int(R.x) & zmx[q]) | (__float_as_int(R.y) & zmy[q]);
                const float v = zv[q] - __int_as_float((int)shift);
                stg[rl * D + zoff + zz] = (info & (1 << 16)) ? v : 0.0f;
                zz += 64;
                for (int w = 0; w < wraps_z; ++w) {
                    const bool wrap = zz >= zlen;
                    zz = wrap ? zz - zlen : zz;
                    rl = wrap ? rl + 1 : rl;
                }
            }
        }
        // LDS operations of one wave execute in order; the barrier only pins the code order
        __builtin_amdgcn_wave_barrier();
        const int nfl = nr * D;
        float *dst = out + r0 * D;
        for (int i = lane * 4; i < nfl; i += 256) {
            const float4 v = *reinterpret_cast<const float4 *>(stg + i);
            if (i + 3 < nfl) {
                f4u o = {v.x, v.y, v.z, v.w};
                *reinterpret_cast<f4u *>(dst + i) = o;
            } else {
                dst[i] = v.x;
                if (i + 1 < nfl) dst[i + 1] = v.y;
                if (i + 2 < nfl) dst[i + 2] = v.z;
            }
        }
        __builtin_amdgcn_wave_barrier();
    }
}

template <int WAVES, int NW, bool DO_STEP, bool DO_OBS>
__global__ __launch_bounds__(64 * WAVES) void tabx_tick_kernel(const KArgs a)
{
    __shared__ Shared<WAVES, NW> sh;
    extern __shared__ __attribute__((aligned(16))) float zone_lds[];
    const Place P = locate<WAVES>(a);
    Unit U = {};
    int code_u = 0;
    if (P.has) {
        load_spec(a, P.k, U);
        load_state(a, P.k, U);
    }
    if (DO_STEP) step_env<WAVES, NW>(a, sh, P, U, code_u);
    else if (P.has) code_u = terrain_code(a, P.e, U.x, U.y);
    if (DO_OBS) observe_env<WAVES, NW>(a, sh, zone_lds, P, U, code_u);
}

template <int WAVES, int NW>
__global__ __launch_bounds__(64 * WAVES) void tabx_reset_kernel(const KArgs a)
{
    __shared__ Shared<WAVES, NW> sh;
    const Place P = locate<WAVES>(a);
    const int N = a.p.num_units;
    const bool go = P.has && !(a.env_mask && a.env_mask[P.e] == 0);
    Unit U = {};
    float ratio = 0.0f;
    if (go) {
        load_spec(a, P.k, U);
        spawn_unit(a, P.e, P.k, U);
        ratio = U.enabled ? U.hp / U.hmax : 0.0f;
        store_state(a, P.k, U);
    }
    const bool en = go && U.enabled;
    sh.share[P.l] = make_float2((en && U.team == 0) ? ratio : 0.0f,
                                (en && U.team != 0) ? ratio : 0.0f);
    const bool pred[4] = {en && U.team == 0, en && U.team != 0, false, false};
    int cnt[4];
    env_counts(sh, P, N, pred, cnt);
    __syncthreads();
    float m0, m1;
    team_means(sh, P, N, cnt[0], cnt[1], m0, m1);
    if (go && P.u == 0) {
        a.st.t[P.e] = 0;
        a.st.phi_prev[P.e] = m0 - m1;
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

template <int WAVES, int NW>
static void launch_mode(Mode mode, const KArgs &a, hipStream_t stream)
{
    const int G = a.envs_per_block;
    const dim3 grid((unsigned)((a.p.num_envs + G - 1) / G)), block(64 * WAVES);
    const size_t zone_bytes = ((size_t)a.stage_offset + (size_t)WAVES * a.stage_floats) * sizeof(float);
    switch (mode) {
    case MODE_RESET:
        hipLaunchKernelGGL((tabx_reset_kernel<WAVES, NW>), grid, block, 0, stream, a);
        break;
    case MODE_STEP:
        hipLaunchKernelGGL((tabx_tick_kernel<WAVES, NW, true, false>), grid, block, 0, stream, a);
        break;
    case MODE_OBSERVE:
        hipLaunchKernelGGL((tabx_tick_kernel<WAVES, NW, false, true>), grid, block, zone_bytes,
                           stream, a);
        break;
    case MODE_STEP_OBSERVE:
        hipLaunchKernelGGL((tabx_tick_kernel<WAVES, NW, true, true>), grid, block, zone_bytes,
                           stream, a);
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
    // N <= 64: one wavefront per workgroup, floor(64 / N) envs packed into it;
    // 64 < N <= 128: two wavefronts per env
    a.envs_per_block = p->num_units <= 64 ? 64 / p->num_units : 1;
    // observation rows are staged in LDS in groups of about 6 KB per wave
    a.rows_per_group = 1536 / a.obs_dim > 0 ? 1536 / a.obs_dim : 1;
    a.stage_floats = (a.rows_per_group * a.obs_dim + 3) & ~3;
    a.stage_offset = (3 * a.envs_per_block * 6 * p->max_zones + 3) & ~3;
    if (p->num_units <= 32) launch_mode<1, 1>(mode, a, s);
    else if (p->num_units <= 64) launch_mode<1, 2>(mode, a, s);
    else launch_mode<2, 4>(mode, a, s);
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
