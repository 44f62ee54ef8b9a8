// TABX batched battle-environment step and observation for MI355X (gfx950).
//
// Work layout.  A 64-lane wavefront advances G = floor(64 / N) whole environments
// at once (N = units per env): lane l owns unit l % N of env slot l / N, so the
// struct-of-arrays state of the G envs is one contiguous, coalesced run of G*N
// elements per field.  For 64 < N <= 128 a workgroup of two wavefronts owns one
// env.  The per-unit stages run in registers; what other lanes need is published
// in LDS and read back as broadcasts inside the all-pairs loops.
//
// The observation tensor is almost all of the HBM traffic, and HBM only takes it
// at full rate when every cache line is completed by consecutive stores.  The
// observe stage therefore loops over the observers i of an env; in pass i every
// lane tests "does observer i see / reach my unit" and writes its unit's 16-float
// block, taken from its own registers, into an LDS image of observer i's row;
// the finished rows (one per packed env) are then streamed to HBM front to back,
// 16 bytes per lane and 1 KB per store instruction.  Own blocks and zone slots
// join the same stream.
//
// The rules follow the paper's App. A ("Interaction Dynamics", "Reward",
// "Observation and Global State", "Zones").  All arithmetic is float32 with one
// rounding per written operation: the file is compiled with -ffp-contract=off
// and uses fmaf only where it is spelled out.
#include <hip/hip_runtime.h>
#include <math.h>
#include <stdint.h>

#include "tabx.h"

#pragma clang fp contract(off)

namespace tabx {

constexpr int kMaxPasses = 10;     // store passes that stream one set of staged rows

struct PolicyArgs {
    TabxPolicy       pol;
    TabxPolicyMemory mem;          // mem_valid == nullptr: no policy in this launch
    const uint8_t   *controlled;
    uint8_t         *actions_out;
};

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
    int       obs_dim;             // D
    int       envs_per_block;      // G
    int       row_pitch;           // floats between staged rows: D rounded up to 4
    int       copy_passes;         // ceil(G * R * row_pitch / 4 / lanes), <= kMaxPasses
    int       rows_per_flush;      // R: consecutive rows of an env staged before they are stored
    int       num_groups;          // workgroups that have envs to process
    int       zdesc_offset;        // elliptical zones: descriptor copy in dynamic LDS, floats
    int       mask_offset;         // hit-all strikes: per-lane victim masks in dynamic LDS, floats
    int       groups_per_xcd;      // ceil(num_groups / 8)
    float     inv_cell;            // 1 / cell_size, used only when that is exact (power of two)
    int       cell_pow2;
    PolicyArgs pa;
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

// What the step stage already knows about a unit and the observe stage needs again.
struct Carry {
    float cu, su;      // cosine / sine of the heading
    float ratio;       // hp / hmax
};

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
    int grp;           // which run of G envs this workgroup owns
    int l, g, u, base, e;
    bool has;
    size_t k;
    int row;           // row of the scenario arrays that configures env e (its level, or e itself)
    size_t ks;         // row * N + u
};

template <int WAVES>
struct Shared {
    static constexpr int L = 64 * WAVES;
    union {
        struct {                  // step stage
            float4 pj[L];         // pair-loop record of a unit: x, y, r^2, flags
            int2   hitrec[L];     // {designated victim (local index) or -1, damage bits}
            float2 share[L];      // this unit's term in the team-0 / team-1 ratio sums
        } st;
        struct {                  // policy stage: what a deciding unit needs of the others
            float4 pose[L];       // x, y, cos(theta), sin(theta)
            float4 body[L];       // radius, max health, health, -
        } po;
        struct {                  // observe stage: what an observer's row needs
            float4 pose[L];       // x, y, cos(theta), sin(theta)
            float4 reach[L];      // attack range, hurtbox half-width, sight range^2, cos(cone / 2)
        } ob;
    };
    int      seer[L];             // observer flags: alive | team<<1 | heals<<2 | enabled<<3 | bush key<<8
                                  // (policy stage: alive | team<<1 | concealable<<2 | bush key<<8)
    uint64_t rowbits[WAVES == 1 ? 1 : L][WAVES];   // two-wave workgroups: ballots of "observer i sees lane"
    uint64_t ballots[WAVES][4];
    int      rows[WAVES == 1 ? 64 : 1];   // level bank: the row an env slot has just switched to, or -1
};

// Orders LDS traffic between the lanes of a workgroup without waiting for global
// stores in flight (a full __syncthreads would drain them).  One wavefront executes
// its LDS operations in order, so a single-wave workgroup only pins the code order.
template <int WAVES>
__device__ __forceinline__ void lds_barrier()
{
    if (WAVES == 1) {
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    } else {
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
        __builtin_amdgcn_s_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
    }
}

// Zone code under a position: low two bits = zone type, upper bits = zone identity; 0 = open.
// Cell-grid zones: the code stored in the cell.  Elliptical zones (App. A "Zones"): the last
// listed active zone whose ellipse holds the point, tested without division as
// (dx^2)*hy^2 + (dy^2)*hx^2 <= hx^2*hy^2; identity = slot index + 1, and `own_effect` returns
// that zone's effect magnitude.  `zd` = the env's zone descriptors (LDS or global), `row` = its
// row of the scenario arrays.
__device__ __forceinline__ int zone_at(const KArgs &a, const float *zd, int row, float x, float y,
                                       float &own_effect)
{
    if (a.p.zone_shapes == 1) {
        int code = 0;
        for (int z = 0; z < a.p.max_zones; ++z) {
            const float *d = zd + 6 * z;
            const float kind = d[0];
            const float dx = x - d[1];
            const float dy = y - d[2];
            const float hx2 = d[3] * d[3];
            const float hy2 = d[4] * d[4];
            const bool inside = (kind != 0.0f) && (((dx * dx) * hy2) + ((dy * dy) * hx2) <= hx2 * hy2);
            code = inside ? (((int)kind & 3) | ((z + 1) << 2)) : code;
            own_effect = inside ? d[5] : own_effect;
        }
        return code;
    }
    if (a.sc.terrain == nullptr) return 0;
    // dividing by a power of two and multiplying by its reciprocal round identically
    int cx = a.cell_pow2 ? (int)(x * a.inv_cell) : (int)(x / a.p.cell_size);
    int cy = a.cell_pow2 ? (int)(y * a.inv_cell) : (int)(y / a.p.cell_size);
    cx = cx > a.p.grid_w - 1 ? a.p.grid_w - 1 : cx;
    cy = cy > a.p.grid_h - 1 ? a.p.grid_h - 1 : cy;
    cx = cx < 0 ? 0 : cx;
    cy = cy < 0 ? 0 : cy;
    return (int)a.sc.terrain[((size_t)row * a.p.grid_h + cy) * a.p.grid_w + cx];
}

// Effect magnitude that applies in the zone just found: its own (elliptical zones) or the
// global parameter (cell grid).
__device__ __forceinline__ float zone_magnitude(const KArgs &a, float own_effect, float global_value)
{
    return a.p.zone_shapes == 1 ? own_effect : global_value;
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
__device__ __forceinline__ int spawn_unit(const KArgs &a, const float *zd, int row, size_t ks,
                                          Unit &U, float &zeff)
{
    U.x = a.sc.init_x[ks];
    U.y = a.sc.init_y[ks];
    U.theta = a.sc.init_theta[ks];
    U.vx = 0.0f;
    U.vy = 0.0f;
    U.hp = U.enabled ? U.hmax : 0.0f;
    U.cd = 0.0f;
    U.reveal = 0.0f;
    U.alive = U.enabled ? 1 : 0;
    const int code = zone_at(a, zd, row, U.x, U.y, zeff);
    U.cur_speed = (code & 3) == TABX_ZONE_SWAMP
                      ? U.speed * zone_magnitude(a, zeff, a.p.swamp_mult) : U.speed;
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
    // Workgroups are dealt to the 8 XCDs round robin; give each XCD one contiguous eighth of
    // the env range, so that neighbouring env groups, which share the cache lines at the ends
    // of their SoA segments, meet in the same L2.
    P.grp = (int)(blockIdx.x & 7) * a.groups_per_xcd + (int)(blockIdx.x >> 3);
    P.e = P.grp * a.envs_per_block + P.g;
    P.has = P.grp < a.num_groups && P.g < a.envs_per_block && P.u < N && P.e < a.p.num_envs;
    P.base = P.has ? P.l - P.u : 0;
    P.k = (size_t)P.e * N + P.u;
    P.row = P.e;
    if (a.p.num_levels > 0) {      // folded into the bank whatever the array holds
        const int lv = P.has ? a.st.level[P.e] : 0;
        P.row = lv < 0 ? 0 : (lv >= a.p.num_levels ? a.p.num_levels - 1 : lv);
    }
    P.ks = (size_t)P.row * N + P.u;
    return P;
}

// How many lanes of the caller's env satisfy each of four predicates.
template <int WAVES>
__device__ __forceinline__ void env_counts(Shared<WAVES> &sh, const Place &P, int N,
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
        lds_barrier<WAVES>();
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            cnt[q] = 0;
#pragma unroll
            for (int w = 0; w < WAVES; ++w) cnt[q] += __popcll(sh.ballots[w][q]);
        }
        lds_barrier<WAVES>();
    }
}

// Mean health ratio of both teams over their enabled units (the bracketed means of
// Eq. 1): the terms published in sh.share are added in ascending unit index; a term
// of +0.0f (unit of the other team, or disabled) leaves a finite sum unchanged.
template <int WAVES>
__device__ __forceinline__ void team_means(const Shared<WAVES> &sh, const Place &P, int N,
                                           int c0, int c1, float &m0, float &m1)
{
    float s0 = 0.0f, s1 = 0.0f;
    for (int jj = 0; jj < N; ++jj) {
        const float2 q = sh.st.share[P.base + jj];
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

// ------------------------------------------------------------------ heuristic policy
//
// Role-appropriate heuristic policy (Sec. 4.2; App. A "Role-Appropriate Heuristic Policy
// Mechanism" and the table of tier parameters).  Lane = deciding unit; the units of its env
// are scanned through records in LDS.  Visibility and reach are the tests of the observation
// (fan-shaped field of view, bush rule, hurtbox, role filter), from the observer's side.

// Counter-based random numbers: two multiply / xor-shift rounds over the draw's coordinates.
__device__ __forceinline__ uint32_t policy_hash(uint32_t seed, uint32_t env, uint32_t unit,
                                                uint32_t tick, uint32_t draw)
{
    uint32_t x = seed;
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

// The cardinal move that closes most of the offset (gx, gy); idle if there is none.
__device__ __forceinline__ int move_along(float gx, float gy)
{
    const float ax = __builtin_fabsf(gx), ay = __builtin_fabsf(gy);
    const int along_x = gx > 0.0f ? TABX_ACT_MOVE_XP : (gx < 0.0f ? TABX_ACT_MOVE_XM : TABX_ACT_NOOP);
    const int along_y = gy > 0.0f ? TABX_ACT_MOVE_YP : TABX_ACT_MOVE_YM;
    return ax >= ay ? along_x : along_y;
}

// Decides for the lane's unit from the state in U (heading cosine / sine cu, su, zone code
// code_u under it); returns the action, or -1 if the unit is not the policy's to move.  Writes
// the action and the remembered target position.  All lanes of the workgroup call it.
template <int WAVES>
__device__ __forceinline__ int policy_env(const KArgs &a, Shared<WAVES> &sh, const Place &P,
                                          const Unit &U, int code_u, float cu, float su)
{
    const PolicyArgs &pa = a.pa;
    const int N = a.p.num_units;
    const bool in_bush = (code_u & 3) == TABX_ZONE_BUSH;
    const int my_key = in_bush ? (code_u & 0xff) : 0x100;          // 0x100 matches no cell code
    const bool concealable = in_bush && !(U.reveal > 0.0f);
    sh.po.pose[P.l] = make_float4(U.x, U.y, cu, su);
    sh.po.body[P.l] = make_float4(U.radius, U.hmax, U.hp, 0.0f);
    sh.seer[P.l] = (P.has ? U.alive : 0) | (U.team << 1) | (concealable ? 4 : 0) | (my_key << 8);
    // per-env tick counter and the unit's memory, requested before the scan
    const bool decide = P.has && U.enabled && U.alive && (!pa.controlled || pa.controlled[P.k]);
    const uint32_t tick = decide ? (uint32_t)a.st.t[P.e] : 0u;
    const int remembered = decide ? pa.mem.mem_valid[P.k] : 0;
    const float mx = decide ? pa.mem.mem_x[P.k] : 0.0f;
    const float my = decide ? pa.mem.mem_y[P.k] : 0.0f;
    lds_barrier<WAVES>();

    const bool healer = U.dmg < 0.0f;
    const bool assassin = U.speed >= pa.pol.assassin_speed;
    const bool ranger = U.range >= pa.pol.ranger_range;
    const float sight2 = U.sight_range * U.sight_range;
    const float neg_hw = -U.hurt_hw;

    // One scan, no divergent branches: the target by role (Healer: injured allies first, then
    // nearest; Assassin: lowest maximum health, then nearest; others: nearest enemy; a strict
    // "better" keeps the lower index on ties), the nearest visible enemy, and whether
    // anything worth a strike is in the hurtbox.
    int tgt = -1;
    bool any_enemy = false, can_hit = false, tgt_in_box = false;
    float tgt_d2 = 0.0f, tgt_key = 0.0f, near_d2 = 0.0f, near_dx = 0.0f, near_dy = 0.0f;
    for (int j = 0; j < N; ++j) {
        const int fj = sh.seer[P.base + j];
        const float4 A = sh.po.pose[P.base + j];
        const float4 B = sh.po.body[P.base + j];
        const float dx = A.x - U.x;
        const float dy = A.y - U.y;
        float dot;
        const float g2 = hurtbox_gap2(dx, dy, cu, su, U.range, U.hurt_hw, neg_hw, dot);
        const float d2 = (dx * dx) + (dy * dy);
        const bool in_range = d2 <= sight2;
        const bool in_cone = (d2 == 0.0f) || (dot >= U.cos_half * __builtin_sqrtf(d2));
        const bool same_team = ((fj >> 1) & 1) == U.team;
        const bool same_bush = (fj >> 8) == my_key;
        const bool concealed = (fj & 4) && !same_team && !same_bush;
        const bool seen = (j != P.u) && (fj & 1) && in_range && in_cone && !concealed;
        // (a seen unit is inside the cone, so a cone-bounded hurtbox needs no further test)
        const bool attackable = seen && (healer == same_team) && (g2 <= B.x * B.x);
        const bool injured = B.z < B.y;
        can_hit = can_hit || (attackable && (!healer || injured));
        const bool enemy = seen && !same_team;
        const bool nearer = enemy && (!any_enemy || d2 < near_d2);
        any_enemy = any_enemy || enemy;
        near_d2 = nearer ? d2 : near_d2;
        near_dx = nearer ? dx : near_dx;
        near_dy = nearer ? dy : near_dy;
        const bool candidate = seen && (healer == same_team);
        const float key = healer ? (injured ? 0.0f : 1.0f) : (assassin ? B.y : 0.0f);
        const bool better = candidate && (tgt < 0 || key < tgt_key || (key == tgt_key && d2 < tgt_d2));
        tgt = better ? j : tgt;
        tgt_d2 = better ? d2 : tgt_d2;
        tgt_key = better ? key : tgt_key;
        tgt_in_box = better ? attackable : tgt_in_box;
    }

    int act = -1;
    if (decide) {
        const uint32_t coin = policy_hash(pa.pol.seed, (uint32_t)P.e, (uint32_t)P.u, tick, 2u) & 1u;
        const int search_turn = coin ? TABX_ACT_ROT_LEFT : TABX_ACT_ROT_RIGHT;
        if (tgt >= 0) {
            const float4 T = sh.po.pose[P.base + tgt];
            const float tr = sh.po.body[P.base + tgt].x;
            pa.mem.mem_x[P.k] = T.x;
            pa.mem.mem_y[P.k] = T.y;
            if (!remembered) pa.mem.mem_valid[P.k] = 1;
            const float tdx = T.x - U.x;
            const float tdy = T.y - U.y;
            const float reach = U.range + tr;
            const bool within = tgt_d2 <= reach * reach;
            const float kite = pa.pol.xi * U.range;
            // turning towards the side the target is on
            const float lx = (tdx * cu) + (tdy * su);
            const float ly = (tdy * cu) - (tdx * su);
            const int turn = ly > 0.0f ? TABX_ACT_ROT_LEFT
                                       : (ly < 0.0f ? TABX_ACT_ROT_RIGHT
                                                    : (lx < 0.0f ? TABX_ACT_ROT_LEFT : TABX_ACT_NOOP));
            // Assassins go behind the target, Healers to it, the rest in front of it
            const float standoff = 0.5f * U.range;
            const float ox = T.z * standoff, oy = T.w * standoff;
            const float gx = healer ? T.x : (assassin ? T.x - ox : T.x + ox);
            const float gy = healer ? T.y : (assassin ? T.y - oy : T.y + oy);
            const int approach = move_along(gx - U.x, gy - U.y);
            const int retreat = move_along(-near_dx, -near_dy);
            act = (can_hit && U.cd <= 0.0f) ? (int)TABX_ACT_ATTACK
                  : (within && !tgt_in_box) ? turn
                  : (ranger && any_enemy && near_d2 < kite * kite) ? retreat
                  : tgt_in_box ? (int)TABX_ACT_NOOP            // aligned, waiting for the cooldown
                               : approach;
        } else if (remembered) {
            const float gx = mx - U.x;
            const float gy = my - U.y;
            const bool arrived = (gx * gx) + (gy * gy) <= 1.0f;
            if (arrived) pa.mem.mem_valid[P.k] = 0;
            act = arrived ? search_turn : move_along(gx, gy);
        } else {
            // Rangers outside a bush walk to the nearest bush zone they know of, then search
            int bush = -1;
            float bush_d2 = 0.0f, bx = 0.0f, by = 0.0f;
            if (ranger && !in_bush && a.sc.zone_desc) {
                const float *zd = a.sc.zone_desc + (size_t)P.row * 6 * a.p.max_zones;
                for (int z = 0; z < a.p.max_zones; ++z) {
                    const float *d = zd + 6 * z;
                    if ((int)d[0] != TABX_ZONE_BUSH) continue;
                    const float zx = d[1] - U.x;
                    const float zy = d[2] - U.y;
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
        // epsilon-greedy override
        const uint32_t h0 = policy_hash(pa.pol.seed, (uint32_t)P.e, (uint32_t)P.u, tick, 0u);
        const float u0 = (float)(h0 >> 8) * (1.0f / 16777216.0f);
        if (u0 < pa.pol.epsilon)
            act = (int)(policy_hash(pa.pol.seed, (uint32_t)P.e, (uint32_t)P.u, tick, 1u) & 7u);
        pa.actions_out[P.k] = (uint8_t)act;
    }
    lds_barrier<WAVES>();          // the records may be overwritten by the next stage
    return act;
}

// Level bank: an episode of the lane's env is about to start (`take`, uniform over the env's
// lanes).  Unit 0 takes the queued level (folded into [0, num_levels)), refills the queue with
// a uniform draw, the hash of (level_seed, env, draws so far), and tells the env's other lanes
// through LDS.  Returns the env's new row, or -1 if it keeps its level.  All lanes call it.
template <int WAVES>
__device__ __forceinline__ int advance_level(const KArgs &a, Shared<WAVES> &sh, const Place &P,
                                             bool take)
{
    if (P.has && P.u == 0) {
        int row = -1;
        if (take) {
            const uint32_t L = (uint32_t)a.p.num_levels;
            row = (int)((uint32_t)a.st.next_level[P.e] % L);
            const uint32_t n = (uint32_t)a.st.level_draws[P.e];
            a.st.level[P.e] = row;
            a.st.next_level[P.e] = (int)(policy_hash(a.p.level_seed, (uint32_t)P.e, 0u, n, 3u) % L);
            a.st.level_draws[P.e] = (int)(n + 1u);
        }
        sh.rows[P.g] = row;
    }
    lds_barrier<WAVES>();
    return P.has ? sh.rows[P.g] : -1;
}

// `forced` >= 0 replaces the unit's entry of the action array (the policy stage chose it).
// `zd`: the env's zone descriptors in LDS (elliptical zones), rewritten when the env changes
// level.  Returns whether any env of the workgroup restarted.
template <int WAVES>
__device__ __forceinline__ bool step_env(const KArgs &a, Shared<WAVES> &sh, float *zd,
                                         uint64_t *masks, Place &P, Unit &U, int &code_u,
                                         Carry &C, int forced)
{
    float zeff = 0.0f;             // effect magnitude of the zone under the unit (elliptical zones)
    const int N = a.p.num_units;
    const float dt = a.p.dt;
    const bool has = P.has;
    const int alive0 = has ? U.alive : 0;
    const int act = forced >= 0 ? forced : (has ? (int)a.actions[P.k] : 0);
    // per-env scalars, requested early: they are needed only after three LDS exchanges
    const int t_new = has ? a.st.t[P.e] + 1 : 0;
    const float phi_prev = has ? a.st.phi_prev[P.e] : 0.0f;
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

    // stage 1b: overlapping bodies are pushed apart.  Every unit sums, over its partners in
    // ascending index, the share of each overlap it has to give way for; all pairs are taken
    // on the positions after the kinematic update; then the unit is clipped again.
    if (a.p.collision_alpha > 0.0f) {
        // partner record: x, y, radius, mass (negative mass: not a body)
        sh.st.pj[P.l] = make_float4(U.x, U.y, U.radius, (has && U.enabled) ? U.mass : -1.0f);
        lds_barrier<WAVES>();
        float ax = 0.0f, ay = 0.0f;
        for (int jj = 0; jj < N; ++jj) {
            const float4 J = sh.st.pj[P.base + jj];
            const float dx = J.x - U.x;
            const float dy = J.y - U.y;
            const float dist = __builtin_sqrtf((dx * dx) + (dy * dy));
            const float pen = (U.radius + J.z) - dist;
            const bool apart = dist > 0.0f;
            // coincident centres separate along x, the lower index to the left
            const float nx = apart ? dx / dist : (P.u < jj ? 1.0f : -1.0f);
            const float ny = apart ? dy / dist : 0.0f;
            const float share = J.w / (U.mass + J.w);
            const float c = ((pen - a.p.collision_slop) * a.p.collision_alpha) * share;
            const bool push = (pen > a.p.collision_slop) && (jj != P.u) && (J.w >= 0.0f);
            // subtracting a zero product leaves the finite sum unchanged
            const float ce = push ? c : 0.0f;
            ax = ax - (ce * nx);
            ay = ay - (ce * ny);
        }
        if (has && U.enabled) {
            U.x = clamp_between(U.x + ax, 0.0f, a.p.map_w);
            U.y = clamp_between(U.y + ay, 0.0f, a.p.map_h);
        }
        lds_barrier<WAVES>();          // the partner records are rewritten for the combat stage
    }

    // the position is final for this tick: fetch the terrain cell under it now, the zone
    // effects of stage 3 use it after the combat exchange
    if (has && U.enabled) code_u = zone_at(a, zd, P.row, U.x, U.y, zeff);

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
    sh.st.pj[P.l] = make_float4(U.x, U.y, U.radius * U.radius,
                             __int_as_float(alive0 ? U.team : 2));
    lds_barrier<WAVES>();

    // stage 2b: attackable row of this unit over its env, closest valid target
    // (strict "<" keeps the lowest index on ties).  Variants: the hurtbox also bounded by the
    // sight cone's angle; the whole row kept as a bit mask when a strike lands on everybody.
    const bool cone_bound = a.p.hurtbox_cone != 0;
    const bool hit_all = a.p.hit_all != 0;
    int target = -1;
    {
        const int want = (U.dmg < 0.0f) ? U.team : 1 - U.team;   // healers reach allies only
        const float neg_hw = -U.hurt_hw;
        float best = kInf;
        if (!cone_bound && !hit_all) {
            for (int jj = 0; jj < N; ++jj) {
                const float4 J = sh.st.pj[P.base + jj];
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
        } else {
            uint64_t row[WAVES] = {};
            for (int jj = 0; jj < N; ++jj) {
                const float4 J = sh.st.pj[P.base + jj];
                const float dx = J.x - U.x;
                const float dy = J.y - U.y;
                float along;
                const float g2 = hurtbox_gap2(dx, dy, cu, su, U.range, U.hurt_hw, neg_hw, along);
                const float d2 = (dx * dx) + (dy * dy);
                bool ok = (g2 <= J.z) && (__float_as_int(J.w) == want) && (jj != P.u);
                if (cone_bound)
                    ok = ok && ((d2 == 0.0f) || (along >= U.cos_half * __builtin_sqrtf(d2)));
                const bool take = ok && (d2 < best);
                best = take ? d2 : best;
                target = take ? jj : target;
                const uint64_t bit = (uint64_t)(ok ? 1 : 0) << (jj & 63);
                row[0] |= (WAVES == 1 || jj < 64) ? bit : 0ull;
                if (WAVES == 2) row[WAVES - 1] |= jj >= 64 ? bit : 0ull;
            }
            if (hit_all) {
#pragma unroll
                for (int w = 0; w < WAVES; ++w) masks[P.l * WAVES + w] = row[w];
            }
        }
    }
    const bool eligible = has && alive0 && act == TABX_ACT_ATTACK && U.cd <= 0.0f;
    if (eligible) U.cd = U.cooldown;
    const bool landed = eligible && target >= 0;
    // designated victim; -2: everybody in this unit's mask
    sh.st.hitrec[P.l] = make_int2(landed ? (hit_all ? -2 : target) : -1, __float_as_int(U.dmg));
    lds_barrier<WAVES>();

    // stage 2c: victim side.  Sum what the attackers that designated this unit
    // deal, ascending attacker index; subtract once with the arena penalty; clamp.
    {
        float acc = 0.0f;
        bool struck = landed && U.dmg > 0.0f;
        if (!hit_all) {
            for (int ii = 0; ii < N; ++ii) {
                const int2 h = sh.st.hitrec[P.base + ii];
                const bool mine = h.x == P.u;
                const float d = __int_as_float(h.y);
                acc = acc + (mine ? d : 0.0f);
                struck = struck || (mine && d > 0.0f);
            }
        } else {
            const int word = WAVES == 1 ? 0 : (P.u >> 6);
            for (int ii = 0; ii < N; ++ii) {
                const int2 h = sh.st.hitrec[P.base + ii];
                const uint64_t row = masks[(P.base + ii) * WAVES + word];
                const bool mine = h.x == -2 && ((row >> (P.u & 63)) & 1ull);
                const float d = __int_as_float(h.y);
                acc = acc + (mine ? d : 0.0f);
                struck = struck || (mine && d > 0.0f);
            }
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
            const int zone = code_u & 3;
            if (alive0 && zone == TABX_ZONE_LAVA) {
                const float h = U.hp - (zone_magnitude(a, zeff, a.p.lava_dps) * dt);
                U.hp = h > 0.0f ? h : 0.0f;
            }
            U.cur_speed = zone == TABX_ZONE_SWAMP
                              ? U.speed * zone_magnitude(a, zeff, a.p.swamp_mult) : U.speed;
            U.alive = U.hp > 0.0f ? 1 : 0;
            ratio = U.hp / U.hmax;
        } else {
            U.alive = 0;
        }
    }
    const bool en = has && U.enabled;
    sh.st.share[P.l] = make_float2((en && U.team == 0) ? ratio : 0.0f,
                                (en && U.team != 0) ? ratio : 0.0f);
    const bool pred[4] = {en && U.team == 0, en && U.team != 0,
                          has && U.alive && U.team == 0, has && U.alive && U.team != 0};
    int cnt[4];
    env_counts(sh, P, N, pred, cnt);
    // episode metrics need the alive counts at entry as well (first loss of a unit)
    const bool want_kills = a.st.kill_run != nullptr;
    int before[4] = {0, 0, 0, 0};
    if (want_kills) {
        const bool pred0[4] = {alive0 && U.team == 0, alive0 && U.team != 0, false, false};
        env_counts(sh, P, N, pred0, before);
    }
    lds_barrier<WAVES>();

    // reward (Eq. 1), termination, terminal bonus
    float m0, m1;
    team_means(sh, P, N, cnt[0], cnt[1], m0, m1);
    const float phi = m0 - m1;
    const float dense = phi - phi_prev;
    float r0 = dense, r1 = -dense;
    const bool done = has && (cnt[2] == 0 || cnt[3] == 0 || t_new >= a.p.max_steps);
    // does any env of this workgroup restart?  (one env per workgroup when WAVES == 2:
    // the flag is already uniform there, up to the idle lanes)
    bool any_done;
    if (WAVES == 1) {
        any_done = __ballot(done) != 0ull;
    } else {
        const uint64_t b = __ballot(done);
        if ((P.l & 63) == 0) sh.ballots[P.l >> 6][0] = b;
        lds_barrier<WAVES>();
        any_done = (sh.ballots[0][0] | sh.ballots[WAVES - 1][0]) != 0ull;
    }
    if (done) {
        const bool ally_win = m0 > m1;
        r0 = r0 + (ally_win ? 1.0f : -1.0f);
        r1 = r1 + (ally_win ? -1.0f : 1.0f);
    }
    if (has) a.rewards[P.k] = U.enabled ? (U.team ? r1 : r0) : 0.0f;

    // auto-reset of finished envs; the potential of the fresh state seeds phi_prev
    float phi_next = phi;
    lds_barrier<WAVES>();          // everyone has read the ratio terms of the finished tick
    if (any_done) {
        bool en_next = en;
        if (a.p.num_levels > 0) {
            // the finished envs move to their queued level: new specifications, new zones
            const int row = advance_level<WAVES>(a, sh, P, done);
            if (row >= 0) {
                P.row = row;
                P.ks = (size_t)row * N + P.u;
                load_spec(a, P.ks, U);
                en_next = U.enabled != 0;
                if (a.p.zone_shapes == 1) {
                    const int zlen = 6 * a.p.max_zones;
                    for (int q = P.u; q < zlen; q += N) zd[q] = a.sc.zone_desc[(size_t)row * zlen + q];
                }
            }
            if (a.p.zone_shapes == 1) lds_barrier<WAVES>();
        }
        if (done) {
            if (a.pa.mem.mem_valid) a.pa.mem.mem_valid[P.k] = 0;   // a new episode remembers nothing
            code_u = spawn_unit(a, zd, P.row, P.ks, U, zeff);
            ratio = U.enabled ? U.hp / U.hmax : 0.0f;
            heading_sincos(U.theta, su, cu);
        }
        int c0 = cnt[0], c1 = cnt[1];
        if (a.p.num_levels > 0) {
            // teams and placeholders may differ in the new level
            const bool pred1[4] = {en_next && U.team == 0, en_next && U.team != 0, false, false};
            int fresh[4];
            env_counts(sh, P, N, pred1, fresh);
            c0 = fresh[0];
            c1 = fresh[1];
        }
        sh.st.share[P.l] = make_float2((en_next && U.team == 0) ? ratio : 0.0f,
                                    (en_next && U.team != 0) ? ratio : 0.0f);
        lds_barrier<WAVES>();
        float f0, f1;
        team_means(sh, P, N, c0, c1, f0, f1);
        if (done) phi_next = f0 - f1;
    }
    if (has && P.u == 0) {
        a.st.t[P.e] = done ? 0 : t_new;
        a.st.phi_prev[P.e] = phi_next;
        a.dones[P.e] = done ? 1 : 0;
        // episode metrics: first loss of a unit, running allied return, summary at the end
        int kills = 0;
        if (want_kills) {
            kills = a.st.kill_run[P.e];
            if (kills == 0) kills = (cnt[3] < before[1] ? 1 : 0) | (cnt[2] < before[0] ? 2 : 0);
            a.st.kill_run[P.e] = (int8_t)(done ? 0 : kills);
        }
        float ret = 0.0f;
        if (a.st.ret_run) {
            ret = a.st.ret_run[P.e] + r0;
            a.st.ret_run[P.e] = done ? 0.0f : ret;
        }
        if (done) {
            if (a.st.ep_count) a.st.ep_count[P.e] += 1;
            if (a.st.ep_len) a.st.ep_len[P.e] = t_new;
            if (a.st.ep_return && a.st.ret_run) a.st.ep_return[P.e] = ret;
            if (a.st.ep_win) a.st.ep_win[P.e] = (m0 > m1) ? 1 : 0;
            if (a.st.ep_first_kill && want_kills) a.st.ep_first_kill[P.e] = (int8_t)kills;
        }
    }
    if (has) store_state(a, P.k, U);
    C.cu = cu;
    C.su = su;
    C.ratio = ratio;
    return any_done;
}

// Observation rows of every unit of the workgroup's envs, visibility masks, action masks.
//
// A row is N blocks of 16 floats (the observer's own block first, then the other units in
// ascending index) followed by the zone slots.  The rows of pass i (observer i of every env
// packed in the workgroup) are assembled in LDS as exact images of the HBM rows, pitch
// row_pitch = D rounded up to 4 floats, and then go out in 16-byte chunks, chunk t of the
// staged rows handled by lane t % lanes of store pass t / lanes.
// Zone slots of the observation rows: lane (env slot zg, 16-byte chunk zc of the zone part)
// keeps its four zone floats in registers for the whole launch: the value (zero if the slot
// is inactive) and which observer coordinate to subtract (centre x / y of an active slot).
struct ZoneRegs {
    bool  lane;
    int   zg, zc;
    float val[4];
    int   sx[4], sy[4];
};

// Issued at the top of the kernel so that the descriptor loads are long done when the
// observe stage needs them.
// Row of the scenario arrays that configures env `env`.
__device__ __forceinline__ int row_of(const KArgs &a, int env)
{
    if (a.p.num_levels <= 0) return env;
    const int lv = a.st.level[env];
    return lv < 0 ? 0 : (lv >= a.p.num_levels ? a.p.num_levels - 1 : lv);
}

template <int WAVES>
__device__ __forceinline__ ZoneRegs load_zone_regs(const KArgs &a, const Place &P, int row_override = -1)
{
    ZoneRegs Z = {};
    const int G = a.envs_per_block;
    const int zlen = 6 * a.p.max_zones;
    const int ZC = (zlen + 3) >> 2;
    const int envs_left = P.grp < a.num_groups ? a.p.num_envs - P.grp * G : 0;
    Z.zg = ZC > 0 ? P.l / ZC : 0;
    Z.zc = P.l - Z.zg * ZC;
    Z.lane = ZC > 0 && Z.zg < (envs_left < G ? envs_left : G);
    if (Z.lane) {
        const int row = row_override >= 0 ? row_override : row_of(a, P.grp * G + Z.zg);
        const float *d = a.sc.zone_desc + (size_t)row * zlen;
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            const int zz = 4 * Z.zc + k;
            if (zz < zlen) {
                const int comp = zz % 6;
                const bool active = d[zz - comp] != 0.0f;
                Z.val[k] = active ? d[zz] : 0.0f;
                Z.sx[k] = (active && comp == 1) ? -1 : 0;
                Z.sy[k] = (active && comp == 2) ? -1 : 0;
            }
        }
    }
    return Z;
}

// Where 16-byte chunk c of the staged row images lives in LDS.
__device__ __forceinline__ int staged_chunk(int c) { return c + (c >> 4); }

template <int WAVES, bool CARRIED>
__device__ __forceinline__ void observe_env(const KArgs &a, Shared<WAVES> &sh, float *stg,
                                            const Place &P, const Unit &U, int code_u,
                                            const Carry &C, const ZoneRegs &Zr)
{
    constexpr int LANES = 64 * WAVES;
    const int N = a.p.num_units;
    const int G = a.envs_per_block;
    const int D = a.obs_dim;
    const int Dp = a.row_pitch;
    const int CPR = Dp >> 2;                     // 16-byte chunks per staged row
    const int zlen = 6 * a.p.max_zones;
    const bool has = P.has;
    const int lane = P.l & 63;
    const int wv = P.l >> 6;
    const int envs_left = P.grp < a.num_groups ? a.p.num_envs - P.grp * G : 0;
    const int envs_here = envs_left < G ? envs_left : G;

    // Blocks of 16 floats written by neighbouring lanes are 64 bytes apart, which would put every
    // fourth lane on the same LDS banks; one spare 16-byte chunk after every 16 spreads them.
    float4 *stage = reinterpret_cast<float4 *>(stg);
    const bool blocks_aligned = (Dp & 15) == 0;  // every block then lies within one group of 16 chunks

    lds_barrier<WAVES>();                        // the step stage is done with the LDS union

    // ---- publish this unit as an observer
    float cu = 1.0f, su = 0.0f;
    const int alive = has ? U.alive : 0;
    const bool enabled = has && U.enabled;
    const bool in_bush = (code_u & 3) == TABX_ZONE_BUSH;
    const int my_code = code_u & 0xff;
    const bool hidden = in_bush && !(U.reveal > 0.0f);
    const float ratio = CARRIED ? C.ratio : U.hp / U.hmax;   // disabled units: masked below
    const float cd_ratio = U.cooldown != 0.0f ? U.cd / U.cooldown : 0.0f;
    const float r2_me = U.radius * U.radius;
    {
        if (CARRIED) {
            cu = C.cu;
            su = C.su;
        } else if (has) {
            heading_sincos(U.theta, su, cu);
        }
        const int key = in_bush ? my_code : 0x100;         // 0x100 matches no cell code
        sh.ob.pose[P.l] = make_float4(U.x, U.y, cu, su);
        sh.ob.reach[P.l] = make_float4(U.range, U.hurt_hw, U.sight_range * U.sight_range, U.cos_half);
        sh.seer[P.l] = alive | (U.team << 1) | (U.dmg < 0.0f ? 4 : 0) | (enabled ? 8 : 0) | (key << 8);
        if (has && a.action_mask) a.action_mask[P.k] = (alive && U.cd <= 0.0f) ? 1 : 0;
    }
    // what differs between a unit's block in its own row and in another unit's row
    const int own_mask = enabled ? -1 : 0;
    const float own_alive = alive ? 1.0f : 0.0f;
    const float own_zone = (float)(code_u & 3);
    const float own_team = (float)U.team;

    // ---- zone chunks: lane (env slot zg, chunk zc) holds its four zone floats in registers
    const int zg = Zr.zg, zc = Zr.zc;
    const bool zone_lane = Zr.lane;
    const float (&zval)[4] = Zr.val;
    const int (&zsx)[4] = Zr.sx;
    const int (&zsy)[4] = Zr.sy;
    const int zone_seer0 = (WAVES == 1) ? zg * N : 0;     // lane of observer 0 of the zone lane's env
    const bool cone_free = a.p.hurtbox_cone == 0;          // the hurtbox is the plain rectangle
    const int R = a.rows_per_flush;
    const int zone_dst0 = ((WAVES == 1) ? zg * R * Dp : 0) + 16 * N + 4 * zc;

    // ---- store passes: chunk t = p * LANES + l of the staged rows -> (row slot, chunk in row)
    unsigned dst_off[kMaxPasses];
    int valid[kMaxPasses];
    {
        const int RC = R * CPR;                    // chunks per env slot and flush
        int tg = P.l / RC;                         // env slot of chunk t
        int q = P.l - tg * RC;                     // chunk within the env's R staged rows
#pragma unroll
        for (int p = 0; p < kMaxPasses; ++p) {
            int vm = 0;                            // R > 1 only when D is a multiple of 4
#pragma unroll
            for (int k = 0; k < 4; ++k) vm |= (R > 1 || 4 * q + k < D) ? (1 << k) : 0;
            valid[p] = (p < a.copy_passes && tg < envs_here) ? vm : 0;
            dst_off[p] = (unsigned)(tg * N * D + 4 * q);
            q += LANES;                            // chunk t + LANES of the next pass
            while (q >= RC) {
                q -= RC;
                tg += 1;
            }
        }
    }

    lds_barrier<WAVES>();

    // ---- one pass per observer index i: every lane's unit seen from observer i of its env
    float *out = a.obs + (size_t)P.grp * G * N * D;
    uint64_t my_row = 0;
    const int blk_row0 = (WAVES == 1) ? P.g * R * Dp : 0;
    for (int i0 = 0; i0 < N; i0 += R) {
    for (int rr = 0; rr < R; ++rr) {
        const int i = i0 + rr;
        const int oi = P.base + i;
        const float4 A = sh.ob.pose[oi];
        const float4 B = sh.ob.reach[oi];
        const int fi = sh.seer[oi];
        const int buf = (WAVES == 1) ? rr * Dp : (i & 1) * Dp;
        // offset of this unit from the observer; `dot` is its component along the heading
        const float dx = U.x - A.x;
        const float dy = U.y - A.y;
        float dot;
        const float g2 = hurtbox_gap2(dx, dy, A.z, A.w, B.x, B.y, -B.y, dot);
        const float d2 = (dx * dx) + (dy * dy);
        const bool in_range = d2 <= B.z;
        const bool in_cone = (d2 == 0.0f) || (dot >= B.w * __builtin_sqrtf(d2));
        const bool same_team = ((fi >> 1) & 1) == U.team;
        const bool same_bush = (fi >> 8) == my_code;
        const bool concealed = hidden && !same_team && !same_bush;
        const bool self = i == P.u;
        const bool pair = alive && (fi & 1) && !self;
        const bool seen = pair && in_range && in_cone && !concealed;
        const bool hit = pair && ((((fi >> 2) & 1) != 0) == same_team) && (g2 <= r2_me) &&
                         (in_cone || cone_free);
        if (a.vis_mask) {
            // the ballot over the lanes is observer i's row; its own lane keeps it
            const uint64_t b = __ballot(seen);
            if (WAVES == 1) my_row = self ? b : my_row;
            else if (lane == 0) sh.rowbits[i][wv] = b;
        }
        if (has) {
            // block position in the row: own block first, then the others in index order
            const int blk = self ? 0 : (P.u < i ? P.u + 1 : P.u);
            const int m = self ? own_mask : (seen ? -1 : 0);
            const float c2 = self ? U.x : dx;
            const float c3 = self ? U.y : dy;
            const float c12 = self ? own_alive : 1.0f;
            const float c13 = self ? U.cur_speed : (same_team ? 1.0f : 0.0f);
            const float c14 = self ? own_zone : (hit ? 1.0f : 0.0f);
            const float c15 = self ? own_team : U.cur_speed;
            const float4 q0 = make_float4(__int_as_float(__float_as_int(U.hp) & m),
                                          __int_as_float(__float_as_int(ratio) & m),
                                          __int_as_float(__float_as_int(c2) & m),
                                          __int_as_float(__float_as_int(c3) & m));
            const float4 q1 = make_float4(__int_as_float(__float_as_int(U.theta) & m),
                                          __int_as_float(__float_as_int(U.range) & m),
                                          __int_as_float(__float_as_int(U.dmg) & m),
                                          __int_as_float(__float_as_int(U.cd) & m));
            const float4 q2 = make_float4(__int_as_float(__float_as_int(cd_ratio) & m),
                                          __int_as_float(__float_as_int(U.radius) & m),
                                          __int_as_float(__float_as_int(U.mass) & m),
                                          __int_as_float(__float_as_int(U.sight_angle) & m));
            const float4 q3 = make_float4(__int_as_float(__float_as_int(c12) & m),
                                          __int_as_float(__float_as_int(c13) & m),
                                          __int_as_float(__float_as_int(c14) & m),
                                          __int_as_float(__float_as_int(c15) & m));
            const int cb = (buf + blk_row0 + 16 * blk) >> 2;       // first 16-byte chunk of the block
            if (blocks_aligned) {
                float4 *d = stage + staged_chunk(cb);
                d[0] = q0;
                d[1] = q1;
                d[2] = q2;
                d[3] = q3;
            } else {
                stage[staged_chunk(cb)] = q0;
                stage[staged_chunk(cb + 1)] = q1;
                stage[staged_chunk(cb + 2)] = q2;
                stage[staged_chunk(cb + 3)] = q3;
            }
        }
        if (zone_lane) {
            const float4 Z = sh.ob.pose[zone_seer0 + i];
            const int en = (sh.seer[zone_seer0 + i] & 8) ? -1 : 0;
            const int xb = __float_as_int(Z.x), yb = __float_as_int(Z.y);
            float zo[4];
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                const float shift = __int_as_float((xb & zsx[k]) | (yb & zsy[k]));
                zo[k] = __int_as_float(__float_as_int(zval[k] - shift) & en);
            }
            stage[staged_chunk((buf + zone_dst0) >> 2)] = make_float4(zo[0], zo[1], zo[2], zo[3]);
        }
    }
        lds_barrier<WAVES>();

        // stream the finished rows: LDS chunk -> one 16-byte store, row order, 1 KB per instruction
        const int buf = (WAVES == 1) ? 0 : (i0 & 1) * Dp;
        float *row = out + i0 * D;
        // chunk t = p * LANES + lane of the staged rows sits at staged_chunk(t): LANES is a
        // multiple of 16, so the passes are a constant stride apart
        const float4 *src = stage + staged_chunk((buf >> 2) + P.l);
        constexpr int PASS_STRIDE = LANES + LANES / 16;
        if (D == Dp) {
            // every chunk is whole: fetch all passes from LDS first, then issue the stores
            float4 v[kMaxPasses];
#pragma unroll
            for (int p = 0; p < kMaxPasses; ++p)
                if (p < a.copy_passes)
                    v[p] = src[p * PASS_STRIDE];
#pragma unroll
            for (int p = 0; p < kMaxPasses; ++p) {
                if (p < a.copy_passes && valid[p] != 0) {
                    // single-wave workgroups stream with the non-temporal hint: the rows are
                    // never read back by the kernel, and the hint measurably raises the store
                    // rate there (it lowers it for the two-wave, 8 KB-row case)
                    f4u o = {v[p].x, v[p].y, v[p].z, v[p].w};
                    f4u *dp = reinterpret_cast<f4u *>(row + dst_off[p]);
                    if (WAVES == 1) __builtin_nontemporal_store(o, dp);
                    else *dp = o;
                }
            }
        } else {
            // rows that are not a multiple of 16 bytes end in a partial chunk
#pragma unroll
            for (int p = 0; p < kMaxPasses; ++p) {
                const int vm = valid[p];
                if (p < a.copy_passes && vm != 0) {
                    const float4 v = src[p * PASS_STRIDE];
                    float *dp = row + dst_off[p];
                    if (vm == 15) {
                        f4u o = {v.x, v.y, v.z, v.w};
                        *reinterpret_cast<f4u *>(dp) = o;
                    } else {
                        if (vm & 1) dp[0] = v.x;
                        if (vm & 2) dp[1] = v.y;
                        if (vm & 4) dp[2] = v.z;
                        if (vm & 8) dp[3] = v.w;
                    }
                }
            }
        }
        if (WAVES == 1) lds_barrier<WAVES>();    // two waves alternate between two staging buffers
    }

    if (a.vis_mask) {
        lds_barrier<WAVES>();
        if (has) {
            if (WAVES == 1) {
                const uint64_t range = N >= 64 ? ~0ull : ((1ull << N) - 1ull);
                a.vis_mask[P.k] = (my_row >> P.base) & range;
            } else {
                const int words = (N + 63) >> 6;
                for (int w = 0; w < words; ++w) a.vis_mask[P.k * words + w] = sh.rowbits[P.u][w];
            }
        }
    }
}

template <int WAVES, bool DO_POLICY, bool DO_STEP, bool DO_OBS>
__global__ __launch_bounds__(64 * WAVES) void tabx_tick_kernel(const KArgs a)
{
    __shared__ Shared<WAVES> sh;
    extern __shared__ __attribute__((aligned(16))) float dyn_lds[];
    Place P = locate<WAVES>(a);
    Unit U = {};
    int code_u = 0;
    if (P.has) {
        load_spec(a, P.ks, U);
        load_state(a, P.k, U);
    }
    ZoneRegs Zr = {};
    if (DO_OBS) Zr = load_zone_regs<WAVES>(a, P);
    // elliptical zones: the descriptors of the workgroup's envs sit in LDS for the lookups
    const int zlen = 6 * a.p.max_zones;
    float *zdesc = dyn_lds + a.zdesc_offset;
    if (a.p.zone_shapes == 1) {
        const int G = a.envs_per_block;
        for (int q = P.l; q < G * zlen; q += 64 * WAVES) {
            const int g = q / zlen;
            const int env = P.grp * G + g;
            const bool live = P.grp < a.num_groups && env < a.p.num_envs;
            zdesc[q] = live ? a.sc.zone_desc[(size_t)row_of(a, env) * zlen + (q - g * zlen)] : 0.0f;
        }
        lds_barrier<WAVES>();
    }
    float *zd = zdesc + (P.has ? P.g : 0) * zlen;
    Carry C = {1.0f, 0.0f, 0.0f};
    float zeff_unused = 0.0f;
    int forced = -1;
    if (DO_POLICY) {
        float cu = 1.0f, su = 0.0f;
        if (P.has) {
            code_u = zone_at(a, zd, P.row, U.x, U.y, zeff_unused);
            heading_sincos(U.theta, su, cu);
        }
        forced = policy_env<WAVES>(a, sh, P, U, code_u, cu, su);
    }
    bool restarted = false;
    uint64_t *masks = reinterpret_cast<uint64_t *>(dyn_lds + a.mask_offset);
    if (DO_STEP) restarted = step_env<WAVES>(a, sh, zd, masks, P, U, code_u, C, forced);
    else if (P.has && !DO_POLICY) code_u = zone_at(a, zd, P.row, U.x, U.y, zeff_unused);
    if (DO_STEP && DO_OBS && a.p.num_levels > 0 && restarted) {
        // zone slots of the envs that changed level
        const int row = Zr.lane ? sh.rows[Zr.zg] : -1;
        if (row >= 0) Zr = load_zone_regs<WAVES>(a, P, row);
    }
    if (DO_OBS) observe_env<WAVES, DO_STEP>(a, sh, dyn_lds, P, U, code_u, C, Zr);
}

template <int WAVES>
__global__ __launch_bounds__(64 * WAVES) void tabx_reset_kernel(const KArgs a)
{
    __shared__ Shared<WAVES> sh;
    Place P = locate<WAVES>(a);
    const int N = a.p.num_units;
    const bool go = P.has && !(a.env_mask && a.env_mask[P.e] == 0);
    if (a.p.num_levels > 0) {
        const int row = advance_level<WAVES>(a, sh, P, go);
        if (row >= 0) {
            P.row = row;
            P.ks = (size_t)row * N + P.u;
        }
    }
    Unit U = {};
    float ratio = 0.0f;
    if (go) {
        load_spec(a, P.ks, U);
        float zeff = 0.0f;
        spawn_unit(a, a.sc.zone_desc + (size_t)P.row * 6 * a.p.max_zones, P.row, P.ks, U, zeff);
        ratio = U.enabled ? U.hp / U.hmax : 0.0f;
        store_state(a, P.k, U);
    }
    const bool en = go && U.enabled;
    sh.st.share[P.l] = make_float2((en && U.team == 0) ? ratio : 0.0f,
                                   (en && U.team != 0) ? ratio : 0.0f);
    const bool pred[4] = {en && U.team == 0, en && U.team != 0, false, false};
    int cnt[4];
    env_counts(sh, P, N, pred, cnt);
    lds_barrier<WAVES>();
    float m0, m1;
    team_means(sh, P, N, cnt[0], cnt[1], m0, m1);
    if (go && P.u == 0) {
        a.st.t[P.e] = 0;
        a.st.phi_prev[P.e] = m0 - m1;
        if (a.st.ret_run) a.st.ret_run[P.e] = 0.0f;
        if (a.st.kill_run) a.st.kill_run[P.e] = 0;
    }
}

// Global state: every enabled unit's own block, then the zone slots with absolute centres.
// One thread per unit (16 floats, four 16-byte stores) or per zone chunk.
__global__ __launch_bounds__(256) void tabx_global_state_kernel(const KArgs a, float *out)
{
    const int N = a.p.num_units;
    const int zlen = 6 * a.p.max_zones;
    const int Dg = 16 * N + zlen;
    const size_t units = (size_t)a.p.num_envs * N;
    const size_t tid = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (tid < units) {
        const int e = (int)(tid / N);
        const int u = (int)(tid - (size_t)e * N);
        const int row = row_of(a, e);
        Unit U = {};
        load_spec(a, (size_t)row * N + u, U);
        load_state(a, tid, U);
        float4 q[4];
        if (U.enabled) {
            float zeff = 0.0f;
            const int code = zone_at(a, a.sc.zone_desc + (size_t)row * zlen, row, U.x, U.y, zeff);
            q[0] = make_float4(U.hp, U.hp / U.hmax, U.x, U.y);
            q[1] = make_float4(U.theta, U.range, U.dmg, U.cd);
            q[2] = make_float4(U.cooldown != 0.0f ? U.cd / U.cooldown : 0.0f, U.radius, U.mass,
                               U.sight_angle);
            q[3] = make_float4(U.alive ? 1.0f : 0.0f, U.cur_speed, (float)(code & 3), (float)U.team);
        } else {
            q[0] = q[1] = q[2] = q[3] = make_float4(0.0f, 0.0f, 0.0f, 0.0f);
        }
        float *d = out + (size_t)e * Dg + 16 * u;       // Dg may be 2 mod 4: 8-byte aligned rows
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            f4u o = {q[k].x, q[k].y, q[k].z, q[k].w};
            *reinterpret_cast<f4u *>(d + 4 * k) = o;
        }
    }
    // zone floats: one thread per float, after the unit threads
    const size_t zt = tid;
    const size_t zones = (size_t)a.p.num_envs * zlen;
    if (zlen > 0 && zt < zones) {
        const int e = (int)(zt / zlen);
        const int zz = (int)(zt - (size_t)e * zlen);
        const float *d = a.sc.zone_desc + (size_t)row_of(a, e) * zlen;
        const int comp = zz % 6;
        out[(size_t)e * Dg + 16 * N + zz] = d[zz - comp] != 0.0f ? d[zz] : 0.0f;
    }
}

// ------------------------------------------------------------------ host side

enum Mode { MODE_RESET, MODE_STEP, MODE_OBSERVE, MODE_STEP_OBSERVE, MODE_POLICY,
            MODE_POLICY_STEP_OBSERVE };

static bool aligned(const void *p, size_t n) { return ((uintptr_t)p % n) == 0; }

static int check_params(const TabxParams *p)
{
    if (!p) return TABX_ERR_NULL;
    if (p->num_envs < 0 || p->num_units < 1 || p->num_units > TABX_N_MAX) return TABX_ERR_SHAPE;
    if (p->max_zones < 0 || p->max_zones > TABX_Z_MAX) return TABX_ERR_SHAPE;
    if (p->grid_w < 0 || p->grid_h < 0 || ((p->grid_w == 0) != (p->grid_h == 0)))
        return TABX_ERR_SHAPE;
    if (p->max_steps < 1) return TABX_ERR_SHAPE;
    if (p->zone_shapes != 0 && p->zone_shapes != 1) return TABX_ERR_SHAPE;
    if (p->zone_shapes == 1 && (p->grid_w != 0 || p->max_zones < 1)) return TABX_ERR_SHAPE;
    if (p->num_levels < 0) return TABX_ERR_SHAPE;
    if ((p->hurtbox_cone | p->hit_all) & ~1) return TABX_ERR_SHAPE;
    if ((int64_t)p->num_levels * p->num_units > (int64_t)1 << 30) return TABX_ERR_SHAPE;
    if ((int64_t)p->num_envs * p->num_units > (int64_t)1 << 30) return TABX_ERR_SHAPE;
    const float pos[] = {p->map_w, p->map_h, p->cell_size, p->dt};
    for (float v : pos)
        if (!(v > 0.0f) || !(v < 3.0e38f)) return TABX_ERR_PARAM;
    const float fin[] = {p->turn_rate, p->lava_dps, p->swamp_mult, p->reveal_time,
                         p->boundary_frac, p->collision_alpha, p->collision_slop};
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

static int check_state(const TabxParams *p, const TabxState *s)
{
    if (!s) return TABX_ERR_NULL;
    if (p->num_levels > 0) {
        const void *lv[] = {s->level, s->next_level, s->level_draws};
        for (const void *q : lv) {
            if (!q) return TABX_ERR_NULL;
            if (!aligned(q, 4)) return TABX_ERR_ALIGN;
        }
    }
    const float *f[] = {s->x, s->y, s->vx, s->vy, s->theta, s->hp, s->cd, s->reveal,
                        s->cur_speed, s->phi_prev};
    for (const float *q : f) {
        if (!q) return TABX_ERR_NULL;
        if (!aligned(q, 4)) return TABX_ERR_ALIGN;
    }
    if (!s->alive || !s->t) return TABX_ERR_NULL;
    if (!aligned(s->t, 4)) return TABX_ERR_ALIGN;
    const void *m4[] = {s->ret_run, s->ep_count, s->ep_len, s->ep_return};
    for (const void *q : m4)
        if (q && !aligned(q, 4)) return TABX_ERR_ALIGN;
    return TABX_OK;
}

template <int WAVES>
static void launch_mode(Mode mode, KArgs a, hipStream_t stream)
{
    const dim3 grid((unsigned)(8 * a.groups_per_xcd)), block(64 * WAVES);
    // dynamic LDS: the staged rows (G rows for a single wavefront, two alternating one-row
    // buffers for a two-wave workgroup)
    const size_t rows_staged = WAVES == 1 ? (size_t)a.envs_per_block * a.rows_per_flush : 2;
    // ... rounded up to whole store passes, which read their 16 bytes per lane unconditionally
    size_t dyn_floats = rows_staged * a.row_pitch;
    const size_t pass_floats = (size_t)a.copy_passes * 64 * WAVES * 4 + (WAVES == 2 ? a.row_pitch : 0);
    if (dyn_floats < pass_floats) dyn_floats = pass_floats;
    // ... with one spare 16-byte chunk after every 16 (see staged_chunk)
    dyn_floats = 4 * ((dyn_floats + 3) / 4 + (dyn_floats + 3) / 64 + 1);
    // ... followed, for elliptical zones, by the zone descriptors of the workgroup's envs
    const size_t zdesc_floats = a.p.zone_shapes == 1 ? (size_t)a.envs_per_block * 6 * a.p.max_zones : 0;
    // ... and, when a strike lands on everybody in the hurtbox, one victim mask per lane
    const size_t zdesc_even = (zdesc_floats + 1) & ~(size_t)1;
    const size_t mask_floats = a.p.hit_all ? (size_t)64 * WAVES * WAVES * 2 : 0;
    const size_t dyn_bytes = (dyn_floats + zdesc_even + mask_floats) * sizeof(float);
    const size_t step_bytes = (zdesc_even + mask_floats) * sizeof(float);
    a.zdesc_offset = (mode == MODE_STEP || mode == MODE_POLICY) ? 0 : (int)dyn_floats;
    a.mask_offset = a.zdesc_offset + (int)zdesc_even;
    switch (mode) {
    case MODE_RESET:
        hipLaunchKernelGGL((tabx_reset_kernel<WAVES>), grid, block, 0, stream, a);
        break;
    case MODE_STEP:
        hipLaunchKernelGGL((tabx_tick_kernel<WAVES, false, true, false>), grid, block, step_bytes,
                           stream, a);
        break;
    case MODE_OBSERVE:
        hipLaunchKernelGGL((tabx_tick_kernel<WAVES, false, false, true>), grid, block, dyn_bytes,
                           stream, a);
        break;
    case MODE_STEP_OBSERVE:
        hipLaunchKernelGGL((tabx_tick_kernel<WAVES, false, true, true>), grid, block, dyn_bytes,
                           stream, a);
        break;
    case MODE_POLICY:
        hipLaunchKernelGGL((tabx_tick_kernel<WAVES, true, false, false>), grid, block, step_bytes,
                           stream, a);
        break;
    case MODE_POLICY_STEP_OBSERVE:
        hipLaunchKernelGGL((tabx_tick_kernel<WAVES, true, true, true>), grid, block, dyn_bytes,
                           stream, a);
        break;
    }
}

static int run(Mode mode, const TabxParams *p, const TabxScenario *sc, const TabxState *st,
               const uint8_t *actions, const uint8_t *env_mask, float *rewards,
               uint8_t *dones, float *obs, uint64_t *vis_mask, uint8_t *action_mask,
               void *stream, const TabxPolicy *policy = nullptr,
               const TabxPolicyMemory *memory = nullptr, const uint8_t *controlled = nullptr,
               uint8_t *actions_out = nullptr)
{
    int rc = check_params(p);
    if (rc) return rc;
    if (p->num_envs == 0) return TABX_OK;          // empty batch: nothing to validate or do
    if ((rc = check_scenario(p, sc))) return rc;
    if ((rc = check_state(p, st))) return rc;
    const bool deciding = mode == MODE_POLICY || mode == MODE_POLICY_STEP_OBSERVE;
    const bool stepping = mode == MODE_STEP || mode == MODE_STEP_OBSERVE ||
                          mode == MODE_POLICY_STEP_OBSERVE;
    const bool observing = mode == MODE_OBSERVE || mode == MODE_STEP_OBSERVE ||
                           mode == MODE_POLICY_STEP_OBSERVE;
    if (deciding) {
        if (!policy || !memory || !actions_out) return TABX_ERR_NULL;
        if (!memory->mem_x || !memory->mem_y || !memory->mem_valid) return TABX_ERR_NULL;
        if (!aligned(memory->mem_x, 4) || !aligned(memory->mem_y, 4)) return TABX_ERR_ALIGN;
        const float fin[] = {policy->epsilon, policy->xi, policy->assassin_speed, policy->ranger_range};
        for (float v : fin)
            if (!(v > -3.0e38f && v < 3.0e38f)) return TABX_ERR_PARAM;
    }
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
    a.obs_dim = 16 * p->num_units + 6 * p->max_zones;
    a.pa = {};
    if (deciding) {
        a.pa.pol = *policy;
        a.pa.mem = *memory;
        a.pa.controlled = controlled;
        a.pa.actions_out = actions_out;
    }

    hipStream_t s = (hipStream_t)stream;
    (void)hipGetLastError();
    // N <= 64: one wavefront per workgroup with G whole envs packed into it; G is floor(64 / N)
    // unless the staged rows of G envs would need more than kMaxPasses store passes or more
    // zone chunks than lanes.  64 < N <= 128: two wavefronts per env.
    const int N = p->num_units;
    const int waves = N <= 64 ? 1 : 2;
    a.row_pitch = (a.obs_dim + 3) & ~3;
    const int cpr = a.row_pitch / 4;
    const int zc = (6 * p->max_zones + 3) / 4;
    int G = 1;
    if (waves == 1) {
        G = 64 / N;
        const int by_passes = kMaxPasses * 64 / cpr;
        if (G > by_passes) G = by_passes;
        if (zc > 0 && G > 64 / zc) G = 64 / zc;
        if (G < 1) G = 1;
    }
    a.envs_per_block = G;
    // two rows per flush: longer contiguous runs per env, and whole 128-byte lines where a
    // single row ends on half a line
    int R = 1;
    if (waves == 1 && a.obs_dim % 4 == 0 && N % 2 == 0 && (2 * G * cpr + 63) / 64 <= kMaxPasses)
        R = 2;
    a.rows_per_flush = R;
    a.num_groups = (p->num_envs + G - 1) / G;
    a.groups_per_xcd = (a.num_groups + 7) / 8;
    {
        int ex = 0;
        const float mant = frexpf(p->cell_size, &ex);
        a.cell_pow2 = (mant == 0.5f && ex > -100 && ex < 100) ? 1 : 0;
        a.inv_cell = 1.0f / p->cell_size;
    }
    a.copy_passes = (G * R * cpr + 64 * waves - 1) / (64 * waves);
    if (a.copy_passes > kMaxPasses) return TABX_ERR_SHAPE;
    if (waves == 1) launch_mode<1>(mode, a, s);
    else launch_mode<2>(mode, a, s);
    return hipGetLastError() == hipSuccess ? TABX_OK : TABX_ERR_LAUNCH;
}

} // namespace tabx

extern "C" {

int tabx_obs_dim(const TabxParams *p)
{
    const int rc = tabx::check_params(p);
    if (rc) return rc;
    return 16 * p->num_units + 6 * p->max_zones;
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

int tabx_global_state(const TabxParams *p, const TabxScenario *sc, const TabxState *st,
                      float *out, void *stream)
{
    int rc = tabx::check_params(p);
    if (rc) return rc;
    if (p->num_envs == 0) return TABX_OK;
    if ((rc = tabx::check_scenario(p, sc))) return rc;
    if ((rc = tabx::check_state(p, st))) return rc;
    if (!out) return TABX_ERR_NULL;
    if (!tabx::aligned(out, 16)) return TABX_ERR_ALIGN;
    tabx::KArgs a = {};
    a.p = *p;
    a.sc = *sc;
    a.st = *st;
    {
        int ex = 0;
        const float mant = frexpf(p->cell_size, &ex);
        a.cell_pow2 = (mant == 0.5f && ex > -100 && ex < 100) ? 1 : 0;
        a.inv_cell = 1.0f / p->cell_size;
    }
    const size_t units = (size_t)p->num_envs * p->num_units;
    const size_t zones = (size_t)p->num_envs * 6 * p->max_zones;
    const size_t threads = units > zones ? units : zones;
    (void)hipGetLastError();
    hipLaunchKernelGGL(tabx::tabx_global_state_kernel, dim3((unsigned)((threads + 255) / 256)),
                       dim3(256), 0, (hipStream_t)stream, a, out);
    return hipGetLastError() == hipSuccess ? TABX_OK : TABX_ERR_LAUNCH;
}

int tabx_heuristic_actions(const TabxParams *p, const TabxScenario *sc, const TabxState *st,
                           const TabxPolicy *policy, const TabxPolicyMemory *memory,
                           const uint8_t *controlled, uint8_t *actions, void *stream)
{
    return tabx::run(tabx::MODE_POLICY, p, sc, st, nullptr, nullptr, nullptr, nullptr, nullptr,
                     nullptr, nullptr, stream, policy, memory, controlled, actions);
}

int tabx_policy_step_observe(const TabxParams *p, const TabxScenario *sc, const TabxState *st,
                             const TabxPolicy *policy, const TabxPolicyMemory *memory,
                             const uint8_t *controlled, uint8_t *actions, float *rewards,
                             uint8_t *dones, float *obs, uint64_t *vis_mask,
                             uint8_t *action_mask, void *stream)
{
    return tabx::run(tabx::MODE_POLICY_STEP_OBSERVE, p, sc, st, actions, nullptr, rewards, dones,
                     obs, vis_mask, action_mask, stream, policy, memory, controlled, actions);
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
