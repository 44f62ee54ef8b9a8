// Heuristic policy stage of the TABX tick (Sec. 4.2; App. A "Role-Appropriate Heuristic
// Policy Mechanism").
#pragma once
#include "tabx_device.h"

#pragma clang fp contract(off)

namespace tabx {

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

// What a deciding unit has made out of the units it sees.
struct Sighting {
    int    tgt;            // selected target (unit index in the env) or -1
    float  tgt_d2;         // its squared distance
    bool   tgt_in_box;     // ... and whether the unit's combat action would reach it
    float4 T;              // its x, y, cos(theta), sin(theta)
    float  tr;             // its body radius
    bool   any_enemy;      // nearest visible enemy: exists,
    float  near_d2, near_dx, near_dy;   // squared distance and offset
    bool   can_hit;        // something worth a strike is in the hurtbox
};

// The rule cascade of the policy for one deciding unit (state in U, heading cosine / sine
// cu, su): first rule that applies, then the epsilon-greedy override.  Updates the unit's
// remembered target position and writes the action to out[k].
__device__ __forceinline__ int policy_cascade(const KArgs &a, const Place &P, const Unit &U,
                                              float cu, float su, bool in_bush, const Sighting &S,
                                              uint32_t tick, int remembered, float mx, float my,
                                              const float *zd, uint8_t *out)
{
    const PolicyArgs &pa = a.pa;
    const bool healer = U.dmg < 0.0f;
    const bool assassin = U.speed >= pa.pol.assassin_speed;
    const bool ranger = U.range >= pa.pol.ranger_range;
    int act;
    const uint32_t env_id = (uint32_t)(P.e + a.p.env_id_offset);     // the env's index in the whole batch
    const uint32_t coin = policy_hash(pa.pol.seed, env_id, (uint32_t)P.u, tick, 2u) & 1u;
    const int search_turn = coin ? TABX_ACT_ROT_LEFT : TABX_ACT_ROT_RIGHT;
    if (S.tgt >= 0) {
        const float4 T = S.T;
        pa.mem.mem_x[P.k] = T.x;
        pa.mem.mem_y[P.k] = T.y;
        if (!remembered) pa.mem.mem_valid[P.k] = 1;
        const float tdx = T.x - U.x;
        const float tdy = T.y - U.y;
        const float reach = U.range + S.tr;
        const bool within = S.tgt_d2 <= reach * reach;
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
        const int retreat = move_along(-S.near_dx, -S.near_dy);
        act = (S.can_hit && U.cd <= 0.0f) ? (int)TABX_ACT_ATTACK
              : (within && !S.tgt_in_box) ? turn
              : (ranger && S.any_enemy && S.near_d2 < kite * kite) ? retreat
              : S.tgt_in_box ? (int)TABX_ACT_NOOP            // aligned, waiting for the cooldown
                             : approach;
    } else if (remembered) {
        const float gx = mx - U.x;
        const float gy = my - U.y;
        const bool arrived = (gx * gx) + (gy * gy) <= 1.0f;
        if (arrived) pa.mem.mem_valid[P.k] = 0;
        act = arrived ? search_turn : move_along(gx, gy);
    } else {
        // Rangers outside a bush walk to the nearest bush zone they know of, then search
        // (`zd`: the env's zone descriptors in LDS)
        bool found = false;
        float bush_d2 = 0.0f, bx = 0.0f, by = 0.0f;
        if (ranger && !in_bush) {
            for (int z = 0; z < a.p.max_zones; ++z) {
                const float *d = zd + 6 * z;
                const float zx = d[1] - U.x;
                const float zy = d[2] - U.y;
                const float d2 = (zx * zx) + (zy * zy);
                const bool take = ((int)d[0] == TABX_ZONE_BUSH) && (!found || d2 < bush_d2);
                found = found || take;
                bush_d2 = take ? d2 : bush_d2;
                bx = take ? zx : bx;
                by = take ? zy : by;
            }
        }
        act = found ? move_along(bx, by) : search_turn;
    }
    // epsilon-greedy override
    const uint32_t h0 = policy_hash(pa.pol.seed, env_id, (uint32_t)P.u, tick, 0u);
    const float u0 = (float)(h0 >> 8) * (1.0f / 16777216.0f);
    if (u0 < pa.pol.epsilon)
        act = (int)(policy_hash(pa.pol.seed, env_id, (uint32_t)P.u, tick, 1u) & 7u);
    out[P.k] = (uint8_t)act;
    return act;
}

// Decides for the lane's unit from the state in U (heading cosine / sine cu, su, zone code
// code_u under it); returns the action, or -1 if the unit is not the policy's to move.  Writes
// the action and the remembered target position.  All lanes of the workgroup call it.
template <int WAVES>
__device__ __forceinline__ int policy_env(const KArgs &a, Shared<WAVES> &sh, const Place &P,
                                          const Unit &U, int code_u, float cu, float su,
                                          const float *zd)
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
    const bool decide = P.has && U.enabled && U.alive && (!pa.controlled || at32(pa.controlled, P.k));
    const uint32_t tick = decide ? (uint32_t)a.st.t[P.e] : 0u;
    const int remembered = decide ? pa.mem.mem_valid[P.k] : 0;
    const float mx = decide ? pa.mem.mem_x[P.k] : 0.0f;
    const float my = decide ? pa.mem.mem_y[P.k] : 0.0f;
    lds_barrier<WAVES>();

    const bool healer = U.dmg < 0.0f;
    const bool assassin = U.speed >= pa.pol.assassin_speed;
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
        Sighting S;
        S.tgt = tgt;
        S.tgt_d2 = tgt_d2;
        S.tgt_in_box = tgt_in_box;
        S.T = sh.po.pose[P.base + (tgt >= 0 ? tgt : 0)];
        S.tr = sh.po.body[P.base + (tgt >= 0 ? tgt : 0)].x;
        S.any_enemy = any_enemy;
        S.near_d2 = near_d2;
        S.near_dx = near_dx;
        S.near_dy = near_dy;
        S.can_hit = can_hit;
        act = policy_cascade(a, P, U, cu, su, in_bush, S, tick, remembered, mx, my, zd,
                             pa.actions_out);
    }
    lds_barrier<WAVES>();          // the records may be overwritten by the next stage
    return act;
}

} // namespace tabx
