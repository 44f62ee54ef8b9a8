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
// Files: tabx_device.h (launch arguments, registers, LDS exchange area, helpers),
// tabx_policy.h (heuristic policy: scan stage and rule cascade), tabx_step.h
// (step stage), tabx_observe.h (observe stage, where scripted units also decide),
// this file (kernels, argument checks, launches, the C entry points).
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

#include "tabx_device.h"
#include "tabx_policy.h"
#include "tabx_step.h"
#include "tabx_observe.h"

namespace tabx {

template <int WAVES, bool DO_POLICY, bool DO_STEP, bool DO_OBS, bool SCRIPT = false,
          int TWIN = 0>
__global__ __launch_bounds__(64 * WAVES * (TWIN ? TWIN : 1)) void tabx_tick_kernel(const KArgs a)
{
    __shared__ Shared<WAVES> sh_all[TWIN ? TWIN : 1];
    __shared__ TwinShared twin;
    extern __shared__ __attribute__((aligned(16))) float dyn_all[];
    const int half = TWIN ? (int)(threadIdx.x >> 6) : 0;
    Shared<WAVES> &sh = sh_all[half];
    float *dyn_lds = dyn_all + half * a.dyn_stride;
    int *rows = twin.rows;                      // TWIN: 0, or how many wavefronts share an env group
    TABX_STAMP(0);
#ifdef TABX_TRACE
    if ((threadIdx.x & 63) == 0) {
        unsigned hw = 0, xcc = 0;
        asm volatile("s_getreg_b32 %0, hwreg(HW_REG_HW_ID)" : "=s"(hw));
        asm volatile("s_getreg_b32 %0, hwreg(HW_REG_XCC_ID)" : "=s"(xcc));
        g_trace[(((size_t)blockIdx.x * 4 + (threadIdx.x >> 6)) * 8 + 7) & ((1 << 21) - 1)] =
            ((unsigned long long)xcc << 32) | hw;
    }
#endif
    Place P = locate<WAVES>(a);
    Unit U = {};
    int code_u = 0;
    // TWIN: the first wavefront of the workgroup runs the step stage; the others, which only
    // write their share of the observers' rows afterwards, take its result over through LDS
    const bool lead = !TWIN || half == 0;
    if (P.has) {
        load_spec(a, P.ks, U);
        if (lead) load_state(a, P.k, U);
    }
    ZoneRegs Zr = {};
    if (DO_OBS) Zr = load_zone_regs<WAVES>(a, P);
    // elliptical zones, deciding units: the descriptors of the workgroup's envs sit in LDS for
    // the zone lookups and the bush search
    const int zlen = 6 * a.p.max_zones;
    // (wavefronts that only write rows never look at them: then the workgroup keeps one copy,
    // behind the wavefronts' areas, and only the first wavefront fills it)
    constexpr bool ZSHARED = TWIN != 0 && !SCRIPT;
    float *zdesc = (ZSHARED ? dyn_all : dyn_lds) + a.zdesc_offset;
    if (a.zdesc_staged && (lead || !ZSHARED)) {
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
    Carry C = {1.0f, 0.0f, 0.0f, 0, false, 0, 0, 0.0f, 0.0f};
    float zeff_unused = 0.0f;
    int forced = -1;
    if (SCRIPT) {
        // the action this unit decided on at the end of the previous call
        // (a wavefront that does not step has no alive flags yet: it loads the memories of
        // all the units the policy may move)
        const bool decides = P.has && U.enabled && (U.alive || !lead) &&
                             (!a.pa.controlled || at32(a.pa.controlled, P.k));
        if (decides) {
            if (lead) {
                forced = at32(a.pa.next_action, P.k);
                a.pa.actions_out[P.k] = (uint8_t)forced;
            }
            C.mem_valid = at32(a.pa.mem.mem_valid, P.k);
            C.mem_x = at32(a.pa.mem.mem_x, P.k);
            C.mem_y = at32(a.pa.mem.mem_y, P.k);
        }
    }
    if (DO_POLICY) {
        float cu = 1.0f, su = 0.0f;
        if (P.has) {
            code_u = zone_at(a, zd, P.row, U.x, U.y, zeff_unused);
            heading_sincos(U.theta, su, cu);
        }
        forced = policy_env<WAVES>(a, sh, P, U, code_u, cu, su, zd);
    }
    bool restarted = false;
    TABX_STAMP(6);
    if (DO_STEP && lead) {
        restarted = step_env<WAVES, TWIN != 0>(a, sh, zd, rows, P, U, code_u, C, forced);
        if (TWIN) {
            // hand the stepped units to the other wavefronts: three 16-byte records per lane in
            // each one's row staging area, which it does not use before it has read them
            const float4 r0 = make_float4(U.x, U.y, U.theta, U.hp);
            const float4 r1 = make_float4(U.cd, U.reveal, U.cur_speed, __int_as_float(C.tick));
            const float4 r2 = make_float4(C.cu, C.su, __int_as_float(code_u),
                                          __int_as_float(U.alive | (C.restarted ? 2 : 0)));
            for (int w = 1; w < TWIN; ++w) {
                float4 *box = reinterpret_cast<float4 *>(dyn_all + w * a.dyn_stride);
                box[P.l] = r0;
                box[64 + P.l] = r1;
                box[128 + P.l] = r2;
            }
            lds_barrier<2>();
        }
    } else if (DO_STEP) {
        lds_barrier<2>();
        const float4 *box = reinterpret_cast<const float4 *>(dyn_lds);
        const float4 r0 = box[P.l], r1 = box[64 + P.l], r2 = box[128 + P.l];
        U.x = r0.x; U.y = r0.y; U.theta = r0.z; U.hp = r0.w;
        U.cd = r1.x; U.reveal = r1.y; U.cur_speed = r1.z; C.tick = __float_as_int(r1.w);
        C.cu = r2.x; C.su = r2.y; code_u = __float_as_int(r2.z);
        const int flags = __float_as_int(r2.w);
        U.alive = flags & 1;
        C.restarted = (flags & 2) != 0;
        restarted = __ballot(C.restarted) != 0ull;
        lds_barrier<1>();          // the records are read: the staging area may take rows now
        if (SCRIPT && P.has && C.restarted) {
            // a new episode remembers nothing: the wavefront that decides for a unit clears its flag
            const int first = P.chunk * a.obs_per_chunk;
            if (P.u >= first && P.u < first + a.obs_per_chunk) a.pa.mem.mem_valid[P.k] = 0;
        }
        if (a.p.num_levels > 0 && restarted) {
            // envs that moved to another level: their specifications and elliptical zones
            const int row = (P.has && C.restarted) ? rows[P.g] : -1;
            if (row >= 0) {
                P.row = row;
                P.ks = (size_t)row * a.p.num_units + P.u;
                load_spec(a, P.ks, U);
                if (a.zdesc_staged && !ZSHARED)
                    for (int q = P.u; q < zlen; q += a.p.num_units)
                        zd[q] = a.sc.zone_desc[(size_t)row * zlen + q];
            }
            if (a.zdesc_staged && !ZSHARED) lds_barrier<1>();
        }
        // the unit's health ratio, as the step stage leaves it (same operands, same rounding)
        C.ratio = (P.has && U.enabled) ? U.hp / U.hmax : 0.0f;
    } else if (P.has && !DO_POLICY) {
        code_u = zone_at(a, zd, P.row, U.x, U.y, zeff_unused);
    }
    if (DO_STEP && DO_OBS && a.p.num_levels > 0 && restarted) {
        // zone slots of the envs that changed level
        const int row = Zr.lane ? rows[Zr.zg] : -1;
        if (row >= 0) Zr = load_zone_regs<WAVES>(a, P, row);
    }
    TABX_STAMP(1);
    if (SCRIPT && !DO_STEP && P.has) C.tick = a.st.t[P.e];
    ScriptLds<WAVES> *script = reinterpret_cast<ScriptLds<WAVES> *>(dyn_lds + a.script_offset);
    if (DO_OBS) observe_env<WAVES, DO_STEP, SCRIPT>(a, sh, dyn_lds, P, U, code_u, C, Zr, script, zd);
    if (DO_STEP) asm volatile("" ::"v"(C.warm));    // keeps the cache-warming load of step_env
    TABX_STAMP(5);
}

template <int WAVES>
__global__ __launch_bounds__(64 * WAVES) void tabx_reset_kernel(const KArgs a)
{
    __shared__ Shared<WAVES> sh;
    __shared__ int level_rows[64];      // level bank: the row an env slot has just switched to
    Place P = locate<WAVES>(a);
    const int N = a.p.num_units;
    const bool go = P.has && !(a.env_mask && a.env_mask[P.e] == 0);
    if (a.p.num_levels > 0) {
        const int row = advance_level<WAVES>(a, sh, P, go, level_rows);
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
        if (a.p.dynamics == 1) {
            a.st.ax[P.k] = 0.0f;
            a.st.ay[P.k] = 0.0f;
        }
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

// The machine the launch shapes below are tuned for (MI355X, gfx950).  tabx_launch_info reports
// them, so that a caller, or a test that runs on the device, can hold them against the
// properties the device itself reports.
constexpr int kComputeUnits = 256;
constexpr int kLdsPerCuBytes = 160 * 1024;          // a CU's LDS, shared by its resident workgroups
constexpr int kLdsPerWorkgroupBytes = 64 * 1024;    // the most one workgroup may take
constexpr int kWavefrontLanes = 64;

enum Mode { MODE_RESET, MODE_STEP, MODE_OBSERVE, MODE_STEP_OBSERVE, MODE_POLICY,
            MODE_POLICY_STEP_OBSERVE, MODE_SCRIPTED_STEP_OBSERVE };

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
    if ((p->hurtbox_cone | p->hit_all | p->dynamics) & ~1) return TABX_ERR_SHAPE;
    if (p->env_id_offset < 0 || (int64_t)p->env_id_offset + p->num_envs > INT32_MAX)
        return TABX_ERR_SHAPE;
    if ((int64_t)p->num_levels * p->num_units > (int64_t)1 << 30) return TABX_ERR_SHAPE;
    if ((int64_t)p->num_envs * p->num_units > (int64_t)1 << 30) return TABX_ERR_SHAPE;
    const float pos[] = {p->map_w, p->map_h, p->cell_size, p->dt};
    for (float v : pos)
        if (!(v > 0.0f) || !(v < 3.0e38f)) return TABX_ERR_PARAM;
    const float fin[] = {p->turn_rate, p->lava_dps, p->swamp_mult, p->reveal_time,
                         p->boundary_frac, p->collision_alpha, p->collision_slop,
                         p->move_gain, p->restitution};
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
    if (p->dynamics == 1 && (!s->ax || !s->ay)) return TABX_ERR_NULL;
    const void *m4[] = {s->ret_run, s->ep_count, s->ep_len, s->ep_return, s->global_state,
                        s->ax, s->ay};
    for (const void *q : m4)
        if (q && !aligned(q, 4)) return TABX_ERR_ALIGN;
    return TABX_OK;
}

// Dynamic LDS of a launch and where its parts lie (fills the offsets in `a`).
struct LdsPlan { size_t dyn_bytes, step_bytes; };
template <int WAVES>
static LdsPlan plan_lds(Mode mode, KArgs &a)
{
    // dynamic LDS: the staged rows (G rows for a single wavefront, two alternating one-row
    // buffers for a two-wave workgroup)
    const size_t rows_staged = WAVES == 1 ? (size_t)a.envs_per_block * a.rows_per_flush : 2;
    // (the two alternating buffers of a two-wave workgroup are whole 64-byte groups apart)
    const size_t pitch = WAVES == 1 ? (size_t)a.row_pitch : (size_t)((a.row_pitch + 15) / 16 * 16);
    // ... rounded up to whole store passes, which read their 16 bytes per lane unconditionally
    size_t dyn_floats = rows_staged * pitch;
    const size_t pass_floats = (size_t)a.copy_passes * 64 * WAVES * 4 + (WAVES == 2 ? pitch : 0);
    if (dyn_floats < pass_floats) dyn_floats = pass_floats;
    // (wavefronts that take over another one's step receive three 16-byte records per lane here)
    if (a.twin && dyn_floats < 3 * 64 * 4) dyn_floats = 3 * 64 * 4;
    // ... in whole 64-byte groups (staged_chunk permutes the chunks of a group among themselves)
    dyn_floats = (dyn_floats + 15) / 16 * 16;
    // ... followed, for elliptical zones, by the zone descriptors of the workgroup's envs
    const size_t zdesc_floats = a.zdesc_staged ? (size_t)a.envs_per_block * 6 * a.p.max_zones : 0;
    // ... and by the bidding area of scripted units that decide in the observe stage
    const size_t zdesc_even = (zdesc_floats + 1) & ~(size_t)1;
    const size_t script_floats = mode == MODE_SCRIPTED_STEP_OBSERVE ? sizeof(ScriptLds<WAVES>) / 4 : 0;
    // (wavefronts sharing an env group: one such area each; the zone descriptors only once, behind
    // the areas, unless the wavefronts decide for scripted units and each look zones up: a
    // workgroup of two wavefronts on c3 takes 23.8 KB, and six of them must fit a CU's 160 KB)
    const int sharers = a.twin ? a.twin : 1;
    const bool zshared = a.twin && mode != MODE_SCRIPTED_STEP_OBSERVE;   // the kernels' ZSHARED
    a.dyn_stride = (int)((dyn_floats + (zshared ? 0 : zdesc_even) + script_floats + 3) & ~(size_t)3);
    const size_t dyn_bytes = ((size_t)a.dyn_stride * sharers + (zshared ? zdesc_even : 0)) * sizeof(float);
    const size_t step_bytes = zdesc_floats * sizeof(float);
    a.zdesc_offset = (mode == MODE_STEP || mode == MODE_POLICY) ? 0
                     : zshared ? a.dyn_stride * sharers : (int)dyn_floats;
    a.script_offset = zshared ? (int)dyn_floats : a.zdesc_offset + (int)zdesc_even;
    return {dyn_bytes, step_bytes};
}

// Enqueues one kernel and returns the status of THIS launch (the runtime's sticky "last error"
// is neither read nor cleared: an error the caller's own earlier work left pending stays theirs).
template <class Kernel, class Arg0>
static hipError_t enqueue(Kernel kernel, dim3 grid, dim3 block, size_t lds_bytes, hipStream_t stream,
                          Arg0 &a0)
{
    void *args[] = {(void *)&a0};
    return hipLaunchKernel((const void *)kernel, grid, block, args, lds_bytes, stream);
}

template <int WAVES>
static hipError_t launch_mode(Mode mode, KArgs a, hipStream_t stream)
{
    const dim3 grid((unsigned)(8 * a.groups_per_xcd * a.obs_chunks));
    const dim3 block(64 * WAVES * (a.twin ? a.twin : 1));
    const LdsPlan lds = plan_lds<WAVES>(mode, a);
    const size_t dyn_bytes = lds.dyn_bytes, step_bytes = lds.step_bytes;
    switch (mode) {
    case MODE_RESET:
        return enqueue(tabx_reset_kernel<WAVES>, grid, block, 0, stream, a);
    case MODE_STEP:
        return enqueue(tabx_tick_kernel<WAVES, false, true, false>, grid, block, step_bytes, stream, a);
    case MODE_OBSERVE:
        return enqueue(tabx_tick_kernel<WAVES, false, false, true>, grid, block, dyn_bytes, stream, a);
    case MODE_STEP_OBSERVE:
        if (WAVES == 1 && a.twin > 2)
            return enqueue(tabx_tick_kernel<1, false, true, true, false, 4>, grid, block, dyn_bytes,
                           stream, a);
        if (WAVES == 1 && a.twin)
            return enqueue(tabx_tick_kernel<1, false, true, true, false, 2>, grid, block, dyn_bytes,
                           stream, a);
        return enqueue(tabx_tick_kernel<WAVES, false, true, true>, grid, block, dyn_bytes, stream, a);
    case MODE_POLICY:
        return enqueue(tabx_tick_kernel<WAVES, true, false, false>, grid, block, step_bytes, stream, a);
    case MODE_POLICY_STEP_OBSERVE:
        return enqueue(tabx_tick_kernel<WAVES, true, true, true>, grid, block, dyn_bytes, stream, a);
    case MODE_SCRIPTED_STEP_OBSERVE:
        if (WAVES == 1 && a.twin)
            return enqueue(tabx_tick_kernel<1, false, true, true, true, 2>, grid, block, dyn_bytes,
                           stream, a);
        return enqueue(tabx_tick_kernel<WAVES, false, true, true, true>, grid, block, dyn_bytes,
                       stream, a);
    }
    return hipErrorInvalidValue;
}

// How a call is laid out on the machine: envs per workgroup, rows per flush, wavefronts per env
// group, store passes (all written into `a`; needs a.obs_dim and a.p).  Returns the wavefronts
// an env takes (1 or 2).
static int plan_shape(Mode mode, const TabxParams *p, KArgs &a)
{
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
    // Long-lived wavefronts make a long tail at the end of the launch, and a wavefront's chain
    // of flushes is the latency floor of a small batch.  Where that matters the observers of an
    // env group are split between several wavefronts:
    //  - a stand-alone observe uses several workgroups per group (each loads the group's units
    //    and writes its share of the rows): up to -14 % on the packed-env kernels (below), +5 %
    //    with two-wave envs, which therefore do not split;
    //  - a launch that also steps cannot (the second workgroup would need the state after the
    //    first one's step), but the wavefronts of ONE workgroup can: the first one runs the step
    //    stage and hands the stepped units to the others through LDS (see the kernel); all of
    //    them load the specifications meanwhile and then write their share of the rows.
    //    Measured: c3 107 -> 99.5 us, c2 15.8 -> 14.0 us, but c4 (10 observers, five flushes per
    //    wavefront, a full machine) 87 -> 102 us; with a longer step stage the wavefronts that
    //    wait for it cost more than the shorter chains save:
    //    body collisions 111.9 -> 114.0 us, the scripted c3 tick 117.0 -> 129.0 us; hence the
    //    conditions below.  Three or four wavefronts per group: 120 us and more on c3, but a
    //    gain from 32 units per env on (below).
    a.obs_chunks = 1;
    a.obs_per_chunk = N;
    a.twin = 0;
    if (waves == 1 && N >= 4) {
        const int per = ((N + 1) / 2 + R - 1) / R * R;
        const int num_groups = (p->num_envs + G - 1) / G;
        // under one residency round (eight single-wavefront workgroups per CU)
        const bool small_batch = num_groups <= 8 * kComputeUnits;
        // eight or more flushes, and a short step stage
        const bool long_chain = N >= 16 * R / 2 && !(p->collision_alpha > 0.0f);
        if (per < N && mode == MODE_OBSERVE) {
            // about four flushes per workgroup, one workgroup more for short chains (c3: ten
            // flushes over 3 workgroups 91.7 us, over 2: 95.3, 5: 100.3, one: 106.4; c4: five
            // flushes over 3: 73.6 us, 2: 76.8, one: 84.4; 16v16: sixteen over 4: 85 us, 2: 92.7,
            // 8: 89.4; 32v32: thirty-two over 8: 80.7 us, 4: 88, 2: 92.8); at most two with zone
            // descriptors to stage per workgroup (elliptical zones: 95.2 us with 2, 96.9 with 3)
            const int flushes = (N + R - 1) / R;
            int share = (flushes + 3) / 4 + (flushes < 8 ? 1 : 0);
            if (share > 8) share = 8;
            if (share > 2 && p->zone_shapes == 1) share = 2;
            a.obs_per_chunk = ((N + share - 1) / share + R - 1) / R * R;
            a.obs_chunks = (N + a.obs_per_chunk - 1) / a.obs_per_chunk;
        } else if (per < N && ((mode == MODE_STEP_OBSERVE && (small_batch || long_chain)) ||
                               (mode == MODE_SCRIPTED_STEP_OBSERVE && small_batch))) {
            a.obs_per_chunk = per;
            a.twin = 2;
            // 16 or more flushes: four wavefronts (N = 32: 99.6 -> 96.8 us, N = 64: 97.4 ->
            // 91.7 us at 0.45 GB of rows per tick; fewer than four flushes each costs more than
            // it saves: N = 16 with four, 92 -> 124 us)
            // (as long as four staging areas fit the 64 KB of LDS a workgroup may take)
            const size_t staged = (size_t)G * R * a.row_pitch * sizeof(float) + 64;
            const size_t lds4 = 4 * (staged + sizeof(Shared<1>)) + sizeof(TwinShared);
            // ... or a batch of at most three env groups per CU, whose launch is one wavefront's
            // chain from the first load to the last store (3v3 x 16 envs 9.8 -> 8.8 us, 5v5 x
            // 4096 13.0 -> 12.2 us, 10v10 x 1024 18.8 -> 15.4 us; from five groups per CU on it
            // costs: 5v5 x 8192 18.5 -> 21.9 us, 10v10 x 4096 33.4 -> 35.8 us)
            const bool tiny_batch = num_groups <= 3 * kComputeUnits && N > 2 * R;
            if (mode == MODE_STEP_OBSERVE && (N >= 16 * R || tiny_batch) && p->zone_shapes == 0 &&
                lds4 <= kLdsPerWorkgroupBytes - 4 * 1024) {
                a.twin = 4;
                a.obs_per_chunk = ((N + 3) / 4 + R - 1) / R * R;
            }
        }
    }
    // (two-wave envs: each wavefront streams one half of a row, both halves whole 64-byte groups)
    const int half = ((cpr / 2) + 3) & ~3, rest = ((cpr + 3) & ~3) - half;
    a.copy_passes = waves == 1 ? (G * R * cpr + 63) / 64 : ((half > rest ? half : rest) + 63) / 64;
    return waves;
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
    const bool deciding = mode == MODE_POLICY || mode == MODE_POLICY_STEP_OBSERVE ||
                          mode == MODE_SCRIPTED_STEP_OBSERVE;
    const bool stepping = mode == MODE_STEP || mode == MODE_STEP_OBSERVE ||
                          mode == MODE_POLICY_STEP_OBSERVE || mode == MODE_SCRIPTED_STEP_OBSERVE;
    const bool observing = mode == MODE_OBSERVE || mode == MODE_STEP_OBSERVE ||
                           mode == MODE_POLICY_STEP_OBSERVE || mode == MODE_SCRIPTED_STEP_OBSERVE;
    if (deciding) {
        if (!policy || !memory || !actions_out) return TABX_ERR_NULL;
        if (!memory->mem_x || !memory->mem_y || !memory->mem_valid) return TABX_ERR_NULL;
        if (!aligned(memory->mem_x, 4) || !aligned(memory->mem_y, 4)) return TABX_ERR_ALIGN;
        if (mode == MODE_SCRIPTED_STEP_OBSERVE && !memory->next_action) return TABX_ERR_NULL;
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
    a.zdesc_staged = (p->zone_shapes == 1 || (deciding && p->max_zones > 0)) ? 1 : 0;
    if (deciding) {
        a.pa.pol = *policy;
        a.pa.mem = *memory;
        a.pa.controlled = controlled;
        a.pa.actions_out = actions_out;
        a.pa.next_action = memory->next_action;
    }

    hipStream_t s = (hipStream_t)stream;
    const int waves = plan_shape(mode, p, a);
    if (a.copy_passes > kMaxPasses) return TABX_ERR_SHAPE;
    const hipError_t err = waves == 1 ? launch_mode<1>(mode, a, s) : launch_mode<2>(mode, a, s);
    return err == hipSuccess ? TABX_OK : TABX_ERR_LAUNCH;
}

} // namespace tabx

#ifdef TABX_TRACE
// Instrumented builds only: copies the first n time stamps to the host / clears them.
extern "C" int tabx_dbg_read(void *dst, int n)
{
    if (hipDeviceSynchronize() != hipSuccess) return -1;
    return hipMemcpyFromSymbol(dst, HIP_SYMBOL(tabx::g_trace), (size_t)n * 8) == hipSuccess ? 0 : -1;
}
extern "C" int tabx_dbg_clear(void)
{
    void *p = nullptr;
    if (hipGetSymbolAddress(&p, HIP_SYMBOL(tabx::g_trace)) != hipSuccess) return -1;
    return hipMemset(p, 0, sizeof(tabx::g_trace)) == hipSuccess ? 0 : -1;
}
#endif

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
    void *args[] = {(void *)&a, (void *)&out};
    const hipError_t err = hipLaunchKernel((const void *)tabx::tabx_global_state_kernel,
                                           dim3((unsigned)((threads + 255) / 256)), dim3(256), args,
                                           0, (hipStream_t)stream);
    return err == hipSuccess ? TABX_OK : TABX_ERR_LAUNCH;
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

int tabx_scripted_step_observe(const TabxParams *p, const TabxScenario *sc, const TabxState *st,
                               const TabxPolicy *policy, const TabxPolicyMemory *memory,
                               const uint8_t *controlled, uint8_t *actions, float *rewards,
                               uint8_t *dones, float *obs, uint64_t *vis_mask,
                               uint8_t *action_mask, void *stream)
{
    return tabx::run(tabx::MODE_SCRIPTED_STEP_OBSERVE, p, sc, st, actions, nullptr, rewards,
                     dones, obs, vis_mask, action_mask, stream, policy, memory, controlled,
                     actions);
}

int tabx_part(const TabxParams *p, const TabxScenario *sc, const TabxState *st, int32_t first_env,
              int32_t count, TabxParams *pp, TabxScenario *psc, TabxState *pst)
{
    int rc = tabx::check_params(p);
    if (rc) return rc;
    if (!sc || !st || !pp || !psc || !pst) return TABX_ERR_NULL;
    if (first_env < 0 || count < 0 || (int64_t)first_env + count > p->num_envs) return TABX_ERR_SHAPE;
    const size_t N = (size_t)p->num_units;
    const size_t e0 = (size_t)first_env, u0 = e0 * N;
    *pp = *p;
    pp->num_envs = count;
    pp->env_id_offset = p->env_id_offset + first_env;
    *psc = *sc;
    if (p->num_levels == 0) {          // one scenario row per env: the part starts at its own
        const float **f[] = {&psc->init_x, &psc->init_y, &psc->init_theta, &psc->hmax, &psc->radius,
                             &psc->mass, &psc->speed, &psc->dmg, &psc->range, &psc->cooldown,
                             &psc->sight_angle, &psc->sight_cos_half, &psc->sight_range,
                             &psc->hurt_halfwidth};
        for (const float **q : f)
            if (*q) *q += u0;
        if (psc->team) psc->team += u0;
        if (psc->enabled) psc->enabled += u0;
        if (psc->terrain) psc->terrain += e0 * (size_t)p->grid_h * (size_t)p->grid_w;
        if (psc->zone_desc) psc->zone_desc += e0 * 6 * (size_t)p->max_zones;
    }
    *pst = *st;
    float **uf[] = {&pst->x, &pst->y, &pst->vx, &pst->vy, &pst->theta, &pst->hp, &pst->cd,
                    &pst->reveal, &pst->cur_speed};
    for (float **q : uf)
        if (*q) *q += u0;
    if (pst->alive) pst->alive += u0;
    if (pst->t) pst->t += e0;
    if (pst->phi_prev) pst->phi_prev += e0;
    if (pst->ret_run) pst->ret_run += e0;
    if (pst->kill_run) pst->kill_run += e0;
    if (pst->ep_count) pst->ep_count += e0;
    if (pst->ep_len) pst->ep_len += e0;
    if (pst->ep_return) pst->ep_return += e0;
    if (pst->ep_win) pst->ep_win += e0;
    if (pst->ep_first_kill) pst->ep_first_kill += e0;
    if (pst->level) pst->level += e0;
    if (pst->next_level) pst->next_level += e0;
    if (pst->level_draws) pst->level_draws += e0;
    if (pst->global_state)
        pst->global_state += e0 * (16 * N + 6 * (size_t)p->max_zones);
    if (pst->ax) pst->ax += u0;
    if (pst->ay) pst->ay += u0;
    return TABX_OK;
}

int tabx_launch_info(const TabxParams *p, int call, TabxLaunchInfo *info)
{
    using namespace tabx;
    const int rc = check_params(p);
    if (rc) return rc;
    if (!info) return TABX_ERR_NULL;
    if (call < TABX_CALL_RESET || call > TABX_CALL_SCRIPTED_STEP_OBSERVE) return TABX_ERR_SHAPE;
    static const Mode modes[] = {MODE_RESET, MODE_STEP, MODE_OBSERVE, MODE_STEP_OBSERVE, MODE_POLICY,
                                 MODE_POLICY_STEP_OBSERVE, MODE_SCRIPTED_STEP_OBSERVE};
    const Mode mode = modes[call];
    const bool deciding = mode == MODE_POLICY || mode == MODE_POLICY_STEP_OBSERVE ||
                          mode == MODE_SCRIPTED_STEP_OBSERVE;
    KArgs a = {};
    a.p = *p;
    a.obs_dim = 16 * p->num_units + 6 * p->max_zones;
    a.zdesc_staged = (p->zone_shapes == 1 || (deciding && p->max_zones > 0)) ? 1 : 0;
    const int waves = plan_shape(mode, p, a);
    if (a.copy_passes > kMaxPasses) return TABX_ERR_SHAPE;
    const LdsPlan lds = waves == 1 ? plan_lds<1>(mode, a) : plan_lds<2>(mode, a);
    const bool staged = mode != MODE_RESET && mode != MODE_STEP && mode != MODE_POLICY;
    info->workgroups = 8 * a.groups_per_xcd * a.obs_chunks;
    info->threads_per_workgroup = 64 * waves * (a.twin ? a.twin : 1);
    info->envs_per_workgroup = a.envs_per_block;
    info->wavefronts_per_env_group = waves * (a.twin ? a.twin : 1);
    info->rows_per_flush = a.rows_per_flush;
    info->dynamic_lds_bytes = mode == MODE_RESET ? 0 : (int32_t)(staged ? lds.dyn_bytes : lds.step_bytes);
    info->assumed_compute_units = kComputeUnits;
    info->assumed_lds_per_cu_bytes = kLdsPerCuBytes;
    info->assumed_lds_per_workgroup_bytes = kLdsPerWorkgroupBytes;
    info->assumed_wavefront_lanes = kWavefrontLanes;
    return TABX_OK;
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
