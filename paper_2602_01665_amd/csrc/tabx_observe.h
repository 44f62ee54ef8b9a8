// Observe stage of the TABX tick (App. A "Observation and Global State").
#pragma once
#include "tabx_device.h"
#include "tabx_policy.h"   // the scripted units' rule cascade

#pragma clang fp contract(off)

namespace tabx {

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

// Where 16-byte chunk c of a set of staged row images lives in LDS (c counts from the start of
// the set): the four chunks of every aligned 64-byte group are permuted by the group's index
// (XOR with bits 3..4 of c).  Measured on gfx950 (SQ_LDS_BANK_CONFLICT / SQ_LDS_IDX_ACTIVE of
// one-pattern kernels): a 16-byte write of 64 lanes takes 8 cycles when every 8 consecutive lanes
// hit 8 different 16-byte slots modulo 128 bytes; the unit blocks that neighbouring lanes write
// are 64 bytes apart, which unpermuted puts every other lane on the same slot (32 cycles; 16
// with one spare chunk per 16; 8 with this permutation).  A 16-byte read takes 4 cycles only
// if lane t reads chunk base + t, 8 as soon as a spare chunk interrupts the run and 12 if the
// lanes of a group read it in permuted order.  So the store passes read the physical chunks in
// lane order and undo the permutation on the way out: lane t's chunk goes to the place of
// logical chunk staged_chunk(t) in HBM, which is in the same 64-byte group, so every store
// instruction still writes whole lines.  The map is its own inverse, and staged_chunk(c + 32 k)
// = staged_chunk(c) + 32 k.
__device__ __forceinline__ int staged_chunk(int c) { return c ^ ((c >> 3) & 3); }

// LDS of the scripted units that decide their next action inside the observe stage: per
// deciding unit the smallest bids for "target" and "nearest enemy" and the "something to
// strike" flag, per unit what a bidder or a decider needs beyond the observe-stage records.
template <int WAVES>
struct ScriptLds {
    static constexpr int L = 64 * WAVES;
    unsigned long long tkey[L];   // role key << 40 | bits(distance^2) << 8 | index << 1 | in hurtbox
    unsigned long long nkey[L];   // bits(distance^2) << 32 | index
    int                canhit[L];
    float2             extra[L];  // body radius, max health
};

// SCRIPT: the units the heuristic policy moves decide their next action here, from the very
// pair tests the observation rows are made of (App. A "Role-Appropriate Heuristic Policy
// Mechanism": a unit acts on what it sees and can reach).  While observer i's pass runs,
// every unit it sees bids with LDS atomic minima for "i's target" (key: the role's order,
// then distance, then index, with "in i's hurtbox" riding in the lowest bit) and for "i's
// nearest enemy"; afterwards each deciding unit reads its winners and runs the rule cascade.
template <int WAVES, bool CARRIED, bool SCRIPT>
__device__ __forceinline__ void observe_env(const KArgs &a, Shared<WAVES> &sh, float *stg,
                                            const Place &P, const Unit &U, int code_u,
                                            const Carry &C, const ZoneRegs &Zr,
                                            ScriptLds<WAVES> *script, const float *zd)
{
    constexpr int LANES = 64 * WAVES;
    const int N = a.p.num_units;
    const int G = a.envs_per_block;
    const int D = a.obs_dim;
    const int Dp = a.row_pitch;
    const int CPR = Dp >> 2;                     // 16-byte chunks per staged row
    const int zlen = 6 * a.p.max_zones;
    const bool has = P.has;
    const bool want_vis = late_args()->vis_mask != nullptr;
    const bool want_gs = late_args()->st.global_state != nullptr;
    const int lane = P.l & 63;
    const int wv = P.l >> 6;
    const int envs_left = P.grp < a.num_groups ? a.p.num_envs - P.grp * G : 0;
    const int envs_here = envs_left < G ? envs_left : G;

    float4 *stage = reinterpret_cast<float4 *>(stg);
    const bool blocks_aligned = (Dp & 15) == 0;  // every block is then one aligned 64-byte group

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
        int role = 0;
        if (SCRIPT) {
            const bool decides = enabled && alive && (!a.pa.controlled || at32(a.pa.controlled, P.k));
            role = (U.speed >= a.pa.pol.assassin_speed ? 0x10 : 0) | (decides ? 0x20 : 0);
            script->tkey[P.l] = ~0ull;
            script->nkey[P.l] = ~0ull;
            script->canhit[P.l] = 0;
            script->extra[P.l] = make_float2(U.radius, has ? U.hmax : 0.0f);
        }
        sh.seer[P.l] = alive | (U.team << 1) | (U.dmg < 0.0f ? 4 : 0) | (enabled ? 8 : 0) | role |
                       (key << 8);
        uint8_t *const action_mask = late_args()->action_mask;
        if (has && action_mask && P.chunk == 0)
            action_mask[P.k] = (alive && U.cd <= 0.0f) ? 1 : 0;
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
    // two-wave workgroups (one env, one row per flush): each wavefront streams one contiguous half
    // of the row, 64 chunks per pass
    // (both halves are whole 64-byte groups, so that the permutation stays within a half)
    const int half_row = ((CPR >> 1) + 3) & ~3;
    const int row_chunks = (CPR + 3) & ~3;         // pitch of the two alternating row buffers
    // the PHYSICAL chunk the lane reads in pass 0; it holds logical chunk staged_chunk(first_chunk)
    const int first_chunk = WAVES == 2 ? wv * half_row + lane : P.l;
    if (WAVES == 2) {
        const bool whole = (D & 3) == 0;
        const int end = wv == 0 ? half_row : row_chunks;
        int phys = first_chunk;
        int q = staged_chunk(first_chunk);
#pragma unroll
        for (int p = 0; p < kMaxPasses; ++p) {
            const int left = D - 4 * q;
            const int vm = (whole || left >= 4) ? 15 : ((1 << (left > 0 ? left : 0)) - 1);
            valid[p] = (phys < end && q < CPR && envs_here > 0) ? vm : 0;
            dst_off[p] = (unsigned)(4 * q);
            q += 64;
            phys += 64;
        }
    } else {
        const int RC = R * CPR;                    // chunks per env slot and flush
        const bool whole = (D & 3) == 0;           // no row ends inside a chunk (always so if R > 1)
        int tg = 0;                                // env slot of chunk t
        int q = staged_chunk(P.l);                 // chunk within the env's R staged rows
        while (q >= RC) {                          // (RC >= 64 for all but tiny rows)
            q -= RC;
            tg += 1;
        }
#pragma unroll
        for (int p = 0; p < kMaxPasses; ++p) {
            // which of the chunk's four floats belong to the row
            const int left = D - 4 * q;
            const int vm = (whole || left >= 4) ? 15 : ((1 << (left > 0 ? left : 0)) - 1);
            // (a pass beyond copy_passes holds only chunks of env slots >= G >= envs_here)
            valid[p] = tg < envs_here ? vm : 0;
            dst_off[p] = (unsigned)(tg * N * D + 4 * q);
            q += LANES;                            // chunk t + LANES of the next pass
            if (RC >= LANES) {                     // at most one env slot further
                const bool next_slot = q >= RC;
                q = next_slot ? q - RC : q;
                tg = next_slot ? tg + 1 : tg;
            } else {
                while (q >= RC) {
                    q -= RC;
                    tg += 1;
                }
            }
        }
    }

    lds_barrier<WAVES>();

    // scripted deciders: what this unit contributes to a bid, whoever the observer is
    bool injured_me = false;
    unsigned rank_me = 0;          // how many units of the env have a smaller maximum health
    unsigned order_heal = 0, key_tail = 0;
    if (SCRIPT) {
        injured_me = U.hp < U.hmax;
        order_heal = injured_me ? 0u : 1u;
        key_tail = (unsigned)P.u << 1;
        for (int jj = 0; jj < N; ++jj) rank_me += script->extra[P.base + jj].y < U.hmax ? 1u : 0u;
    }

    // ---- one pass per observer index i: every lane's unit seen from observer i of its env
    float *out = a.obs + (size_t)P.grp * G * N * D;
    uint64_t my_row = 0;
    const int blk_row0 = (WAVES == 1) ? P.g * R * Dp : 0;
    // the observers this workgroup writes the rows of: all of them, or its share when the rows
    // of an env group are spread over several short-lived workgroups
    const int i_begin = P.chunk * a.obs_per_chunk;
    const int i_end = (i_begin + a.obs_per_chunk < N) ? i_begin + a.obs_per_chunk : N;
    TABX_STAMP(2);
    for (int i0 = i_begin; i0 < i_end; i0 += R) {
    for (int rr = 0; rr < R; ++rr) {
        const int i = i0 + rr;
        const int oi = P.base + i;
        const float4 A = sh.ob.pose[oi];
        const float4 B = sh.ob.reach[oi];
        const int fi = sh.seer[oi];
        // two-wave workgroups alternate between two row buffers; a single wavefront stages R rows
        const int base = (WAVES == 1) ? 0 : (i & 1) * row_chunks;
        const int buf = (WAVES == 1) ? rr * Dp : 0;
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
        if (SCRIPT) {
            // observer i decides its next action: this unit bids if i sees it (nothing to do
            // in a pass whose observers decide nothing or see nobody)
            const bool vis = seen && (fi & 0x20);
            if (__ballot(vis) != 0ull) {
                const bool i_heals = (fi & 4) != 0;
                const unsigned d2b = (unsigned)__float_as_int(d2);
                if (vis && hit && (!i_heals || injured_me)) atomicOr(&script->canhit[oi], 1);
                if (vis && !same_team)
                    atomicMin(&script->nkey[oi], ((unsigned long long)d2b << 32) | (unsigned)P.u);
                if (vis && (i_heals == same_team)) {
                    // Healer: injured allies first; Assassin: lowest maximum health first
                    const unsigned order = i_heals ? order_heal : ((fi & 0x10) ? rank_me : 0u);
                    const unsigned hi = (order << 8) | (d2b >> 24);
                    const unsigned lo = (d2b << 8) | key_tail | (hit ? 1u : 0u);
                    atomicMin(&script->tkey[oi], ((unsigned long long)hi << 32) | lo);
                }
            }
        }
        if (want_vis) {
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
            if (self && want_gs) {
                // the own block with its absolute position is the unit's block of the global state
                f4u *gs = reinterpret_cast<f4u *>(late_args()->st.global_state + (size_t)P.e * D + 16 * P.u);
                gs[0] = f4u{q0.x, q0.y, q0.z, q0.w};
                gs[1] = f4u{q1.x, q1.y, q1.z, q1.w};
                gs[2] = f4u{q2.x, q2.y, q2.z, q2.w};
                gs[3] = f4u{q3.x, q3.y, q3.z, q3.w};
            }
            const int cb = (buf + blk_row0 + 16 * blk) >> 2;       // first 16-byte chunk of the block
            // (written as 128-bit vector values: as four-member structs the last chunk has been
            // seen to go out as four separate dwords, each a many-way bank conflict)
            typedef float v4 __attribute__((ext_vector_type(4)));
            v4 *vstage = reinterpret_cast<v4 *>(stg);
            const v4 w0 = {q0.x, q0.y, q0.z, q0.w}, w1 = {q1.x, q1.y, q1.z, q1.w};
            const v4 w2 = {q2.x, q2.y, q2.z, q2.w}, w3 = {q3.x, q3.y, q3.z, q3.w};
            if (blocks_aligned) {
                // (cb is a multiple of 4: the block's chunks are permuted among themselves)
                v4 *d = vstage + base + cb;
                const int sw = (cb >> 3) & 3;
                d[sw] = w0;
                d[1 ^ sw] = w1;
                d[2 ^ sw] = w2;
                d[3 ^ sw] = w3;
            } else {
                vstage[base + staged_chunk(cb)] = w0;
                vstage[base + staged_chunk(cb + 1)] = w1;
                vstage[base + staged_chunk(cb + 2)] = w2;
                vstage[base + staged_chunk(cb + 3)] = w3;
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
            stage[base + staged_chunk((buf + zone_dst0) >> 2)] = make_float4(zo[0], zo[1], zo[2], zo[3]);
            if (want_gs && i == 0) {
                // ... and the zone slots with absolute centres are its tail
                float *gz = late_args()->st.global_state + (size_t)(P.grp * G + zg) * D + 16 * N + 4 * zc;
                const int left = zlen - 4 * zc;
                if (left >= 4) {
                    *reinterpret_cast<f4u *>(gz) = f4u{zval[0], zval[1], zval[2], zval[3]};
                } else {
                    // (constant indices: a runtime index would move the zone registers to
                    // scratch memory for the whole kernel)
#pragma unroll
                    for (int k = 0; k < 3; ++k)
                        if (k < left) gz[k] = zval[k];
                }
            }
        }
    }
        lds_barrier<WAVES>();

        // stream the finished rows: LDS chunk -> one 16-byte store, row order, 1 KB per instruction
        float *row = out + i0 * D;
        // the lane reads physical chunk first_chunk + 64 p in pass p: whole runs, in lane order
        const float4 *src = stage + ((WAVES == 1) ? 0 : (i0 & 1) * row_chunks) + first_chunk;
        constexpr int PASS_STRIDE = 64;
        if (D == Dp) {
            // every chunk is whole: fetch all passes from LDS first, then issue the stores
            float4 v[kMaxPasses];
#pragma unroll
            for (int p = 0; p < kMaxPasses; ++p)
                if (p < a.copy_passes)
                    v[p] = src[p * PASS_STRIDE];
#pragma unroll
            for (int p = 0; p < kMaxPasses; ++p) {
                // (the mask is made opaque here: as a loop invariant its tests would be hoisted
                // out of the observer loop as forty lane masks, most of them spilled)
                int vm = valid[p];
                asm volatile("" : "+v"(vm));
                if (p < a.copy_passes && vm != 0) {
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
                int vm = valid[p];
                asm volatile("" : "+v"(vm));
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
        // Two-wave envs (one workgroup per env for the whole launch): the wavefront lets its row
        // stores land before it goes on.  Without this the XCDs drain at different rates and the
        // launch lasts as long as the slowest (ends of the eight between 163 and 216 us on 64v64);
        // with at most one row per wavefront in flight they stay together (191 ... 209 us) and the
        // launch is 3 % shorter.  Waiting before the next row's stores instead, or allowing two
        // or four stores to stay in flight, gains less; the packed-env kernels gain nothing.
        if (WAVES == 2) asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        if (i0 == i_begin) TABX_STAMP(3);
    }
    TABX_STAMP(4);

    if (want_vis) {
        uint64_t *const vis_mask = late_args()->vis_mask;
        lds_barrier<WAVES>();
        if (has && P.u >= i_begin && P.u < i_end) {
            if (WAVES == 1) {
                const uint64_t range = N >= 64 ? ~0ull : ((1ull << N) - 1ull);
                vis_mask[P.k] = (my_row >> P.base) & range;
            } else {
                const int words = (N + 63) >> 6;
                for (int w = 0; w < words; ++w) vis_mask[P.k * words + w] = sh.rowbits[P.u][w];
            }
        }
    }

    if (SCRIPT) {
        lds_barrier<WAVES>();      // all bids are in
        // (wavefronts sharing an env group: the one that ran the unit's pass as observer holds its bids)
        const bool decides = (sh.seer[P.l] & 0x20) != 0 && P.u >= i_begin && P.u < i_end;
        if (decides) {
            const unsigned long long tk = script->tkey[P.l];
            const unsigned long long nk = script->nkey[P.l];
            Sighting S;
            S.tgt = tk == ~0ull ? -1 : (int)((tk >> 1) & 0x7f);
            S.tgt_d2 = __int_as_float((int)(unsigned)(tk >> 8));
            S.tgt_in_box = (tk & 1ull) != 0ull;
            const int tl = P.base + (S.tgt >= 0 ? S.tgt : 0);
            S.T = sh.ob.pose[tl];
            S.tr = script->extra[tl].x;
            S.any_enemy = nk != ~0ull;
            S.near_d2 = __int_as_float((int)(unsigned)(nk >> 32));
            const float4 E = sh.ob.pose[P.base + (S.any_enemy ? (int)(nk & 0x7f) : 0)];
            S.near_dx = E.x - U.x;
            S.near_dy = E.y - U.y;
            S.can_hit = script->canhit[P.l] != 0;
            const int remembered = C.restarted ? 0 : C.mem_valid;
            const float mx = C.mem_x;
            const float my = C.mem_y;
            policy_cascade(a, P, U, cu, su, in_bush, S, (uint32_t)C.tick, remembered, mx, my, zd,
                           a.pa.next_action);
        }
    }
}

} // namespace tabx
