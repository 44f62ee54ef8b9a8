// Shared device-side definitions of the TABX kernels: launch arguments, per-lane registers,
// the LDS exchange area, the float32 helpers whose rounding both sides of the parity tests
// agree on, zone lookup, state load / store and the lane-to-unit mapping.
#pragma once
#include <hip/hip_runtime.h>
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
    uint8_t         *next_action;  // scripted tick: decided at the end of one call, applied by the next
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
    int       zdesc_offset;        // copy of the zone descriptors in dynamic LDS, floats (from the wavefront's
                                   //    area; from the start if the workgroup keeps one copy, see the kernel)
    int       zdesc_staged;        // ... which exists for elliptical zones and for deciding units
    int       script_offset;       // scripted units deciding in the observe stage: their LDS, floats
    int       groups_per_xcd;      // ceil(num_groups / 8)
    int       twin;                // 2 or 4: that many wavefronts of a workgroup own the same env
                                   //    group and share its observers (chunk = wavefront index)
    int       dyn_stride;          // floats of dynamic LDS per wavefront (when several share an env group)
    int       obs_chunks;          // workgroups that share the observers of one env group (>= 1)
    int       obs_per_chunk;       // observers per such workgroup (a multiple of rows_per_flush)
    float     inv_cell;            // 1 / cell_size, used only when that is exact (power of two)
    int       cell_pow2;
    PolicyArgs pa;
};

// Per-wavefront time stamps of an instrumented build (-DTABX_TRACE; compiled out of the product):
// slot 0 kernel entry, 6 before the step stage, 1 after it (or after the hand-over), 2 / 3 / 4
// observer loop start / first rows stored / loop end, 5 kernel end, 7 hardware ids.
#ifdef TABX_TRACE
__device__ unsigned long long g_trace[1 << 21];
#define TABX_STAMP(slot)                                                                          \
    do {                                                                                          \
        if ((threadIdx.x & 63) == 0)                                                              \
            g_trace[(((size_t)blockIdx.x * 4 + (threadIdx.x >> 6)) * 8 + (slot)) & ((1 << 21) - 1)] = \
                wall_clock64();                                                                   \
    } while (0)
#else
#define TABX_STAMP(slot) do { } while (0)
#endif

typedef float f4u __attribute__((ext_vector_type(4), aligned(4)));   // 16-byte store, 4-byte aligned

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
    int   tick;        // the env's tick counter after the step
    bool  restarted;   // the env's episode ended in this step
    int   warm;        // a byte loaded only to bring its cache line in (see step_env)
    // scripted units: the remembered target position as it was at the start of the call
    // (loaded with the state: at the end of the wavefront a load would queue behind its stores)
    int   mem_valid;
    float mem_x, mem_y;
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
    int chunk;         // which share of the observers of these envs it writes (observe stage)
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
            union {
                float4 pj[L];     // collision partners: x, y, radius, mass
                float4 aim0[L];   // combat, a striker's pose: x, y, cos(theta), sin(theta)
                float2 share[L];  // afterwards: this unit's term in the team-0 / team-1 ratio sums
            };
            float4 aim1[L];       // ... its hurtbox: range | target team in the sign bit,
                                  //     half-width, damage, cos(cone / 2)
            unsigned long long best[L];   // ... the closest body in it: (distance^2 bits, index)
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
};

// Several wavefronts of one workgroup may share an env group (fused tick): the first one runs
// the step stage and alone touches the state; the others take the stepped units over through
// LDS and each writes the rows of its share of the observers.  What they all see sits here
// (one per workgroup, whether or not its wavefronts share a group).
struct TwinShared {
    int rows[64];      // level bank: the row an env slot has just switched to, or -1
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
        // four slots per round, their descriptors fetched together (a slot beyond the last one
        // re-reads the last and is masked out), so that the fetch latency is paid once per round
        const int Z = a.p.max_zones;
        for (int z0 = 0; z0 < Z; z0 += 4) {
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                const int z = z0 + k;
                const float *d = zd + 6 * (z < Z ? z : Z - 1);
                const float kind = d[0];
                const float dx = x - d[1];
                const float dy = y - d[2];
                const float hx2 = d[3] * d[3];
                const float hy2 = d[4] * d[4];
                const bool inside = (z < Z) && (kind != 0.0f) &&
                                    (((dx * dx) * hy2) + ((dy * dy) * hx2) <= hx2 * hy2);
                code = inside ? (((int)kind & 3) | ((z + 1) << 2)) : code;
                own_effect = inside ? d[5] : own_effect;
            }
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

// The launch arguments where the kernel-argument segment holds them.  The kernels have more
// argument words than scalar registers; fields that are needed once, late or rarely (episode
// metrics, level bank, masks written at the end) are read through this pointer at the point of
// use instead of sitting in registers, or spilled, from the first instruction on.
typedef const __attribute__((address_space(4))) KArgs *LateArgs;
__device__ __forceinline__ LateArgs late_args()
{
    return (LateArgs)__builtin_amdgcn_kernarg_segment_ptr();
}

// Element k of a per-unit array (at most 2^30 elements: its byte offset fits 32 bits, so the
// access is "uniform base + 32-bit lane offset" and needs no 64-bit address arithmetic per lane).
template <class T>
__device__ __forceinline__ const T &at32(const T *base, size_t k)
{
    return *reinterpret_cast<const T *>(reinterpret_cast<const char *>(base) +
                                        (uint32_t)(k * sizeof(T)));
}

__device__ __forceinline__ void load_spec(const KArgs &a, size_t k, Unit &U)
{
    U.hmax = at32(a.sc.hmax, k);
    U.radius = at32(a.sc.radius, k);
    U.mass = at32(a.sc.mass, k);
    U.speed = at32(a.sc.speed, k);
    U.dmg = at32(a.sc.dmg, k);
    U.range = at32(a.sc.range, k);
    U.cooldown = at32(a.sc.cooldown, k);
    U.sight_angle = at32(a.sc.sight_angle, k);
    U.cos_half = at32(a.sc.sight_cos_half, k);
    U.sight_range = at32(a.sc.sight_range, k);
    U.hurt_hw = at32(a.sc.hurt_halfwidth, k);
    U.team = ((int)at32(a.sc.team, k) + 255) >> 8;    // 0 or 1: any non-zero byte means the adversaries
    U.enabled = at32(a.sc.enabled, k);
}

__device__ __forceinline__ void load_state(const KArgs &a, size_t k, Unit &U)
{
    U.x = at32(a.st.x, k);
    U.y = at32(a.st.y, k);
    U.vx = at32(a.st.vx, k);
    U.vy = at32(a.st.vy, k);
    U.theta = at32(a.st.theta, k);
    U.hp = at32(a.st.hp, k);
    U.cd = at32(a.st.cd, k);
    U.reveal = at32(a.st.reveal, k);
    U.cur_speed = at32(a.st.cur_speed, k);
    U.alive = at32(a.st.alive, k);
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
    P.l = a.twin ? (int)(threadIdx.x & 63) : (int)threadIdx.x;
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
    const int slot = (int)(blockIdx.x >> 3);
    const int in_xcd = a.obs_chunks > 1 ? slot / a.obs_chunks : slot;
    P.chunk = a.twin ? (int)(threadIdx.x >> 6) : slot - in_xcd * a.obs_chunks;
    P.grp = in_xcd < a.groups_per_xcd ? (int)(blockIdx.x & 7) * a.groups_per_xcd + in_xcd : a.num_groups;
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

} // namespace tabx
