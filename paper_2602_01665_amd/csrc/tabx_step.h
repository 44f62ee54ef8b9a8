// Step stage of the TABX tick (App. A "Interaction Dynamics", "Reward", "Zones"): timers,
// kinematics, actions, hurtbox combat, zone effects, rewards, termination and auto-reset.
#pragma once
#include "tabx_device.h"
#include "tabx_policy.h"   // policy_hash draws the levels

#pragma clang fp contract(off)

namespace tabx {

// Level bank: an episode of the lane's env is about to start (`take`, uniform over the env's
// lanes).  Unit 0 takes the queued level (folded into [0, num_levels)), refills the queue with
// a uniform draw, the hash of (level_seed, env, draws so far), and tells the env's other lanes
// through LDS (`rows`: one slot per env of the workgroup).  Returns the env's new row, or -1
// if it keeps its level.  All lanes call it.
template <int WAVES>
__device__ __forceinline__ int advance_level(const KArgs &a, Shared<WAVES> &sh, const Place &P,
                                             bool take, int *rows)
{
    if (P.has && P.u == 0 && P.chunk == 0) {
        int row = -1;
        if (take) {
            const LateArgs late = late_args();
            int32_t *const level = late->st.level, *const next_level = late->st.next_level;
            int32_t *const level_draws = late->st.level_draws;
            const uint32_t L = (uint32_t)a.p.num_levels;
            row = (int)((uint32_t)next_level[P.e] % L);
            const uint32_t n = (uint32_t)level_draws[P.e];
            level[P.e] = row;
            next_level[P.e] = (int)(policy_hash(a.p.level_seed, (uint32_t)(P.e + a.p.env_id_offset), 0u, n, 3u) % L);
            level_draws[P.e] = (int)(n + 1u);
        }
        rows[P.g] = row;
    }
    lds_barrier<WAVES>();
    return P.has ? rows[P.g] : -1;
}

// `forced` >= 0 replaces the unit's entry of the action array (the policy stage chose it).
// `zd`: the env's zone descriptors in LDS (elliptical zones), rewritten when the env changes
// level.  Returns whether any env of the workgroup restarted.
// SHARED: further wavefronts of the workgroup take the stepped units over and decide for some of them.
template <int WAVES, bool SHARED = false>
__device__ __forceinline__ bool step_env(const KArgs &a, Shared<WAVES> &sh, float *zd,
                                         int *rows, Place &P, Unit &U, int &code_u, Carry &C,
                                         int forced)
{
    float zeff = 0.0f;             // effect magnitude of the zone under the unit (elliptical zones)
    const int N = a.p.num_units;
    const float dt = a.p.dt;
    const bool has = P.has;
    const int alive0 = has ? U.alive : 0;
    const int act = forced >= 0 ? forced : (has ? (int)at32(a.actions, P.k) : 0);
    // per-env scalars, requested early: they are needed only after three LDS exchanges
    const int t_new = has ? at32(a.st.t, (size_t)P.e) + 1 : 0;
    const float phi_prev = has ? at32(a.st.phi_prev, (size_t)P.e) : 0.0f;
    // ... and the running episode metrics, if kept: loaded where they are used, at the end of the
    // stage, they would queue behind the observation stores of the other wavefronts
    const LateArgs late = late_args();
    int8_t *const kill_run_p = late->st.kill_run;
    float *const ret_run_p = late->st.ret_run;
    const bool want_kills = kill_run_p != nullptr;
    const int kills_run = (want_kills && has) ? at32(kill_run_p, (size_t)P.e) : 0;
    const float ret_run = (ret_run_p && has) ? at32(ret_run_p, (size_t)P.e) : 0.0f;
    float bdmg = 0.0f;
    const bool writer = P.chunk == 0;      // (always: only a group's first wavefront steps)
    // persistent velocities: the acceleration the last action stage set is part of the state
    const bool dynamic = late->p.dynamics == 1;
    float acx = 0.0f, acy = 0.0f;
    if (dynamic && has) {
        acx = at32(late->st.ax, P.k);
        acy = at32(late->st.ay, P.k);
    }

    // stage 1: cooldown / reveal timers, explicit Euler move, arena penalty + clip
    if (has && U.enabled) {
        float v = U.cd - dt;
        U.cd = v > 0.0f ? v : 0.0f;
        v = U.reveal - dt;
        U.reveal = v > 0.0f ? v : 0.0f;
        if (alive0) {
            if (dynamic) {             // the velocity from the acceleration first, then the position
                U.vx = U.vx + acx * dt;
                U.vy = U.vy + acy * dt;
            }
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
        // (with persistent velocities the partners' velocities travel in the next array, which
        // the combat stage rewrites only after the barrier that ends this stage)
        if (dynamic) sh.st.aim1[P.l] = make_float4(U.vx, U.vy, 0.0f, 0.0f);
        lds_barrier<WAVES>();
        float ax = 0.0f, ay = 0.0f;
        float dvx = 0.0f, dvy = 0.0f;
        const float inv_i = 1.0f / U.mass;             // 0 for a kinematic body, which takes no impulse
        const bool bounces = dynamic && has && U.enabled && inv_i != 0.0f;
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
            if (dynamic) {
                // impulse along the normal from the relative velocity, unless the pair is
                // already separating; split by inverse mass (the slop gates the correction only)
                const float4 V = sh.st.aim1[P.base + jj];
                const float rvx = V.x - U.vx;
                const float rvy = V.y - U.vy;
                const float vn = (rvx * nx) + (rvy * ny);
                const float inv_j = 1.0f / J.w;
                const float jimp = ((1.0f + late->p.restitution) * (0.0f - vn)) / (inv_i + inv_j);
                const bool hit = bounces && (pen > 0.0f) && (jj != P.u) && (J.w >= 0.0f) && !(vn > 0.0f);
                // (subtracting a zero product leaves the finite sum unchanged)
                const float je = hit ? jimp * inv_i : 0.0f;
                dvx = dvx - (je * nx);
                dvy = dvy - (je * ny);
            }
            // a kinematic body (infinite mass) gives way to nobody; a body of finite mass
            // gives way to it for the whole corrected depth
            const float inf = __builtin_inff();
            const float share = U.mass == inf ? 0.0f : (J.w == inf ? 1.0f : J.w / (U.mass + J.w));
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
            if (dynamic) {
                U.vx = U.vx + dvx;
                U.vy = U.vy + dvy;
            }
        }
        lds_barrier<WAVES>();          // the partner records are rewritten for the combat stage
    }

    // the position is final for this tick: fetch the terrain cell under it now, the zone
    // effects of stage 3 use it after the combat exchange
    if (has && U.enabled) code_u = zone_at(a, zd, P.row, U.x, U.y, zeff);
    // The action array is the one input that is new in every tick, so its lines come from HBM,
    // where a read queues behind the observation stores for microseconds once those are
    // flowing, and every wavefront's step stage waits for its action bytes.  The first
    // wavefronts of each XCD, which start while HBM is still idle, therefore touch every line of
    // their XCD's share of the array (lane l of the j-th wavefront: line 64 j + l); the later
    // generations find them in the cache.  Measured with a fresh action batch per tick:
    // c3 108.6 -> 102.5 us, c4 95.4 -> 89.7 us (101 / 88 us with actions that are cached anyway).
    if (writer) {
        const size_t span = (size_t)a.groups_per_xcd * a.envs_per_block * N;   // units per XCD
        const size_t first = (size_t)(blockIdx.x & 7) * span;
        const size_t off = ((size_t)(blockIdx.x >> 3) * 64 + (size_t)(threadIdx.x & 63)) * 128;
        if (off < span && first + off < (size_t)a.p.num_envs * N) C.warm = at32(a.actions, first + off);
    }

    // stage 2a: movement sets next tick's velocity, rotation turns the heading now
    float cu = 1.0f, su = 0.0f;
    if (has) {
        // the velocity the unit wants: its current speed along a move action, else none
        float wx = 0.0f, wy = 0.0f;
        if (alive0) {
            const float sp = U.cur_speed;
            if (act == TABX_ACT_MOVE_XP) wx = sp;
            else if (act == TABX_ACT_MOVE_YP) wy = sp;
            else if (act == TABX_ACT_MOVE_XM) wx = -sp;
            else if (act == TABX_ACT_MOVE_YM) wy = -sp;
        }
        if (dynamic) {
            // the acceleration for the next tick's physics stage; what is not alive holds neither
            acx = alive0 ? (wx - U.vx) * late->p.move_gain : 0.0f;
            acy = alive0 ? (wy - U.vy) * late->p.move_gain : 0.0f;
            U.vx = alive0 ? U.vx : 0.0f;
            U.vy = alive0 ? U.vy : 0.0f;
        } else {
            U.vx = wx;
            U.vy = wy;
        }
        if (alive0) {
            if (act == TABX_ACT_ROT_LEFT) {
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
    // stage 2b: combat, seen from the victims.  Few units strike in a tick (the cooldowns see to
    // that), so instead of every unit scanning its env for targets, every unit tests itself
    // against the strikers of its env only.  A striker publishes its pose and hurtbox; each unit
    // in that hurtbox (body circle against the forward rectangle, role filter, optionally the
    // sight cone's angle) bids for "closest" with an LDS atomic minimum over the 64-bit key
    // (squared distance bits, unit index): the smallest key is the closest valid body, the
    // lowest index among equally distant ones.
    const bool cone_bound = a.p.hurtbox_cone != 0;
    const bool hit_all = a.p.hit_all != 0;
    const bool eligible = has && alive0 && act == TABX_ACT_ATTACK && U.cd <= 0.0f;
    if (eligible) U.cd = U.cooldown;
    {
        const int want = (U.dmg < 0.0f) ? U.team : 1 - U.team;   // healers reach allies only
        // the attack range is never negative: its sign bit carries the team the strike is for
        const float range_want = __int_as_float(__float_as_int(U.range) | (want << 31));
        sh.st.aim0[P.l] = make_float4(U.x, U.y, cu, su);
        sh.st.aim1[P.l] = make_float4(range_want, U.hurt_hw, U.dmg, U.cos_half);
        sh.st.best[P.l] = ~0ull;
    }
    // the strikers of this lane's env, as bit masks over its unit indices
    uint64_t strikers[WAVES];
    {
        const uint64_t b = __ballot(eligible);
        if (WAVES == 1) {
            strikers[0] = (b >> P.base) & (N >= 64 ? ~0ull : ((1ull << N) - 1ull));
        } else if ((P.l & 63) == 0) {
            sh.ballots[P.l >> 6][0] = b;
        }
    }
    lds_barrier<WAVES>();
    if (WAVES == 2) {
#pragma unroll
        for (int w = 0; w < WAVES; ++w) strikers[w] = sh.ballots[w][0];
    }

    float acc = 0.0f;              // what lands on this unit, strikers in ascending index
    bool struck = false;           // ... and whether any of it was damage
    {
        const float r2 = U.radius * U.radius;
#pragma unroll
        for (int w = 0; w < WAVES; ++w) {
            uint64_t m = strikers[w];
            while (m != 0ull) {
                const int s_u = 64 * w + __builtin_ctzll(m);
                m &= m - 1ull;
                const float4 A0 = sh.st.aim0[P.base + s_u];
                const float4 A1 = sh.st.aim1[P.base + s_u];
                const int rb = __float_as_int(A1.x);
                const float range = __int_as_float(rb & 0x7fffffff);
                const int want = (rb >> 31) & 1;
                const float dx = U.x - A0.x;
                const float dy = U.y - A0.y;
                float along;
                const float g2 = hurtbox_gap2(dx, dy, A0.z, A0.w, range, A1.y, -A1.y, along);
                const float d2 = (dx * dx) + (dy * dy);
                bool ok = alive0 && (U.team == want) && (s_u != P.u) && (g2 <= r2);
                if (cone_bound) ok = ok && ((d2 == 0.0f) || (along >= A1.w * __builtin_sqrtf(d2)));
                if (ok) {
                    const unsigned long long key =
                        ((unsigned long long)(unsigned)__float_as_int(d2) << 32) | (unsigned)P.u;
                    atomicMin(&sh.st.best[P.base + s_u], key);
                    if (hit_all) {             // a strike lands on everybody in the hurtbox
                        acc = acc + A1.z;
                        struck = struck || (A1.z > 0.0f);
                    }
                }
            }
        }
    }
    lds_barrier<WAVES>();

    // stage 2c: a strike has landed if anybody bid; unless everybody in the hurtbox is struck,
    // the victims now look up which striker designated them
    const bool landed = eligible && sh.st.best[P.l] != ~0ull;
    if (!hit_all) {
#pragma unroll
        for (int w = 0; w < WAVES; ++w) {
            uint64_t m = strikers[w];
            while (m != 0ull) {
                const int s_u = 64 * w + __builtin_ctzll(m);
                m &= m - 1ull;
                const bool mine = (unsigned)sh.st.best[P.base + s_u] == (unsigned)P.u;
                const float d = sh.st.aim1[P.base + s_u].z;
                acc = acc + (mine ? d : 0.0f);
                struck = struck || (mine && d > 0.0f);
            }
        }
    }
    struck = struck || (landed && U.dmg > 0.0f);
    if (has && alive0) {
        // subtract once, together with the arena penalty; clamp
        const float h = (U.hp - acc) - bdmg;
        U.hp = clamp_between(h, 0.0f, U.hmax);
        if (struck) U.reveal = a.p.reveal_time;
    }
    // (the ratio terms written next share LDS with the strikers' poses, which nobody reads any
    // more: the bids above were the last use, and a barrier has passed since)

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
    if (has && writer) a.rewards[P.k] = U.enabled ? (U.team ? r1 : r0) : 0.0f;

    // auto-reset of finished envs; the potential of the fresh state seeds phi_prev
    float phi_next = phi;
    lds_barrier<WAVES>();          // everyone has read the ratio terms of the finished tick
    if (any_done) {
        bool en_next = en;
        if (a.p.num_levels > 0) {
            // the finished envs move to their queued level: new specifications, new zones
            const int row = advance_level<WAVES>(a, sh, P, done, rows);
            if (row >= 0) {
                P.row = row;
                P.ks = (size_t)row * N + P.u;
                load_spec(a, P.ks, U);
                en_next = U.enabled != 0;
                if (a.zdesc_staged) {
                    const int zlen = 6 * a.p.max_zones;
                    for (int q = P.u; q < zlen; q += N) zd[q] = a.sc.zone_desc[(size_t)row * zlen + q];
                }
            }
            if (a.zdesc_staged) lds_barrier<WAVES>();
        }
        if (done) {
            // a new episode remembers nothing.  Where several wavefronts share the env group, the
            // wavefront that later decides for the unit clears its flag itself (it may set it again
            // at once, and two wavefronts' stores to one byte have no order between them)
            uint8_t *const mem_valid = late->pa.mem.mem_valid;
            if (mem_valid && writer && (!SHARED || P.u < a.obs_per_chunk)) mem_valid[P.k] = 0;
            code_u = spawn_unit(a, zd, P.row, P.ks, U, zeff);
            acx = 0.0f;
            acy = 0.0f;
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
    if (has && P.u == 0 && writer) {
        a.st.t[P.e] = done ? 0 : t_new;
        a.st.phi_prev[P.e] = phi_next;
        a.dones[P.e] = done ? 1 : 0;
        // episode metrics: first loss of a unit, running allied return, summary at the end
        int kills = 0;
        if (want_kills) {
            kills = kills_run;
            if (kills == 0) kills = (cnt[3] < before[1] ? 1 : 0) | (cnt[2] < before[0] ? 2 : 0);
            late->st.kill_run[P.e] = (int8_t)(done ? 0 : kills);
        }
        float ret = 0.0f;
        if (late->st.ret_run) {
            ret = ret_run + r0;
            late->st.ret_run[P.e] = done ? 0.0f : ret;
        }
        if (done) {
            if (late->st.ep_count) late->st.ep_count[P.e] += 1;
            if (late->st.ep_len) late->st.ep_len[P.e] = t_new;
            if (late->st.ep_return && late->st.ret_run) late->st.ep_return[P.e] = ret;
            if (late->st.ep_win) late->st.ep_win[P.e] = (m0 > m1) ? 1 : 0;
            if (late->st.ep_first_kill && want_kills) late->st.ep_first_kill[P.e] = (int8_t)kills;
        }
    }
    if (has && writer) store_state(a, P.k, U);
    if (dynamic && has && writer) {
        late->st.ax[P.k] = acx;
        late->st.ay[P.k] = acy;
    }
    C.cu = cu;
    C.su = su;
    C.ratio = ratio;
    C.tick = done ? 0 : t_new;
    C.restarted = done;
    return any_done;
}

} // namespace tabx
