/*
 * tabx.h -- C ABI of the MI355X (gfx950) TABX batched battle-environment library.
 *
 * The library advances thousands of independent battle instances per call:
 * unit movement and facing, hurtbox combat (attack / heal), terrain zones,
 * health and alive flags, team rewards, termination with auto-reset, and the
 * per-agent partial observations, as the paper defines them in App. A
 * ("Observation and Global State", "Action Space", "Interaction Dynamics",
 * "Reward", "Zones") and Sec. 4.
 *
 * Conventions
 *  - E = num_envs, N = num_units per env (allies first or in any order; `team`
 *    says which), D = tabx_obs_dim().  E * N (and num_levels * N) may not exceed 2^30:
 *    TABX_ERR_SHAPE otherwise.
 *  - Every pointer inside TabxScenario / TabxState and every array argument is a
 *    DEVICE pointer into memory owned by the caller.  The library allocates and
 *    frees nothing and keeps no global state; it borrows the pointers until the
 *    enqueued work has finished on `stream`.
 *  - Per-unit arrays are struct-of-arrays, one array per field, indexed
 *    [e * N + u] (scenario arrays: [row * N + u] with row = e, or the env's level when a
 *    level bank is used, see TabxParams.num_levels).  float arrays must be 4-byte aligned, `obs` and `vis_mask`
 *    16-byte aligned.
 *  - `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *    Calls validate their arguments on the host, enqueue kernels and return
 *    without synchronising; they allocate nothing and enqueue no memsets or
 *    copies, so a stream capture can record them into a graph.
 *  - Every entry point returns TABX_OK (0) or a negative TabxError; on error
 *    nothing has been enqueued.  num_envs == 0 is a valid no-op.
 *  - An action id >= TABX_NUM_ACTIONS acts as TABX_ACT_NOOP.
 */
#ifndef TABX_H
#define TABX_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define TABX_N_MAX 128        /* largest supported num_units            */
#define TABX_Z_MAX 16         /* largest supported max_zones            */
#define TABX_NUM_ACTIONS 8

/* Discrete actions (Sec. 4; App. A "Action Space"): idle, four world-frame
 * moves, the combat action (attack, or heal for units with negative damage),
 * rotate left (counter-clockwise) and right. */
enum TabxAction {
    TABX_ACT_NOOP = 0, TABX_ACT_MOVE_XP = 1, TABX_ACT_MOVE_YP = 2, TABX_ACT_MOVE_XM = 3,
    TABX_ACT_MOVE_YM = 4, TABX_ACT_ATTACK = 5, TABX_ACT_ROT_LEFT = 6, TABX_ACT_ROT_RIGHT = 7
};

/* Terrain cell code (App. A "Zones"): low two bits = zone type, upper bits =
 * zone id (two bush cells belong to the same bush iff their codes are equal). */
enum TabxZone { TABX_ZONE_OPEN = 0, TABX_ZONE_LAVA = 1, TABX_ZONE_BUSH = 2, TABX_ZONE_SWAMP = 3 };

enum TabxError {
    TABX_OK = 0,
    TABX_ERR_NULL = -1,      /* a required pointer is NULL                          */
    TABX_ERR_SHAPE = -2,     /* sizes out of range (N, zones, grid, negative E ...) */
    TABX_ERR_ALIGN = -3,     /* a pointer is not aligned as required                */
    TABX_ERR_LAUNCH = -4,    /* the HIP runtime refused the launch                  */
    TABX_ERR_PARAM = -5      /* a physics constant is not finite / not positive     */
};

/* Physics and shape constants (App. A "Environment Parameters": the physics
 * axis of the configuration).  Plain values, passed by pointer from the host. */
typedef struct TabxParams {
    int32_t num_envs, num_units;
    int32_t grid_w, grid_h;       /* terrain cells; both 0 = no terrain              */
    int32_t max_zones;            /* zone-descriptor slots per env in the obs (>= 0) */
    int32_t max_steps;            /* truncation horizon (> 0)                        */
    float   map_w, map_h;         /* arena is [0, map_w] x [0, map_h]                */
    float   cell_size;            /* world units per terrain cell (> 0)              */
    float   dt;                   /* time step                                       */
    float   turn_rate;            /* heading change per time unit for a rotation     */
    float   lava_dps;             /* lava health loss per time unit                  */
    float   swamp_mult;           /* speed multiplier inside a swamp                 */
    float   reveal_time;          /* how long combat exposes a unit hidden in a bush */
    float   boundary_frac;        /* out-of-arena damage = boundary_frac*hmax*dt     */
    /* Body collisions (App. A "Collision detection and resolution"): after the kinematic
     * update overlapping body circles are pushed apart: of the penetration depth beyond
     * collision_slop the fraction collision_alpha is corrected per tick, split by inverse
     * mass (needs mass > 0; mass = +infinity marks a kinematic body, which is exempt: it gives
     * way to nobody and a finite partner gives way for the whole corrected depth), every unit
     * summing its corrections over its partners in
     * ascending index on the pre-correction positions, then clipped to the arena.  Dead
     * bodies collide, disabled placeholders do not.  collision_alpha = 0 switches it off. */
    float   collision_alpha;
    float   collision_slop;
    /* Zone geometry.  0: zones are the cells of `terrain` (codes as in TabxZone) and the lava /
     * swamp magnitudes are lava_dps / swamp_mult.  1: zones are the ellipses of zone_desc
     * (App. A "Zones": type, centre, two semi-axes, own effect magnitude: lava loss per time
     * unit or swamp speed multiplier); needs grid_w = grid_h = 0 and max_zones >= 1; a point
     * belongs to the last listed active zone with (dx^2)*hy^2 + (dy^2)*hx^2 <= hx^2*hy^2, and
     * two units share a bush iff they are in the same slot. */
    int32_t zone_shapes;
    /* Per-episode reconfiguration (Sec. 4.1, App. A "Environment Parameters": the configuration
     * is applied when an episode starts, without rebuilding anything).  0: row e of the scenario
     * arrays configures env e for good.  L > 0: the scenario arrays are a bank of L levels
     * ([L * N] per unit field, terrain [L][grid_h][grid_w], zone_desc [L][max_zones][6]) and env e
     * plays row state->level[e].  Whenever an episode of env e starts (tabx_reset, or the
     * auto-reset inside a step) it takes level (uint32) next_level[e] mod L, and next_level[e]
     * is refilled with a uniform draw: hash32(level_seed, e, 0, level_draws[e]++, 3) mod L, the
     * hash of tabx_heuristic_actions.  The caller may overwrite next_level between calls (a
     * curriculum) or leave the draws alone (domain randomisation). */
    int32_t  num_levels;
    uint32_t level_seed;
    /* Hurtbox variants (App. A "Attack range geometry and target selection"; Sec. 4), both 0 or 1.
     * hurtbox_cone = 1: the rectangle is also bounded by the unit's field of view: a body in it
     * counts only if its centre lies within the angle of the sight cone (sight_cos_half), at any
     * distance.  hit_all = 1: a strike lands on every valid body in the hurtbox instead of the
     * closest one (each victim still sums its strikers in ascending index; every struck unit of
     * a damaging strike is revealed). */
    int32_t  hurtbox_cone;
    int32_t  hit_all;
    /* A batch may be processed as several calls on parts of it (every pointer advanced to the
     * part's first env, num_envs = the part's size), for instance on two streams so that one
     * part's launch fills the start and the end of the other's.  env_id_offset = index of the
     * part's first env in the whole batch (>= 0): it is added to the env index in the keys of
     * the random draws (level bank, heuristic policy), so the parts draw what the whole batch
     * would.  Nothing else depends on it. */
    int32_t  env_id_offset;
    /* Physics mode (App. A "Movement and kinematic update": explicit Euler, the velocity from
     * the current acceleration, then the position; "Collision detection and resolution": impulse
     * response).  0 (default): kinematic: a move action sets the velocity outright, any other
     * action zeroes it, and a collision only corrects positions.  1: persistent velocity: the
     * action stage sets the acceleration move_gain * (wanted velocity - velocity), where the
     * wanted velocity is the unit's current speed along a move action and zero otherwise; the
     * next tick's physics stage integrates it (v += a * dt, then p += v * dt); with body
     * collisions on, every interpenetrating pair (depth > 0, whatever the slop) whose relative
     * velocity along the normal n (from i to j) is not separating (v_rel.n <= 0) exchanges the
     * impulse (1 + restitution) * (-v_rel.n) / (1/m_i + 1/m_j) along n, unit i's velocity
     * changing by it times 1/m_i; a kinematic body (mass = +infinity) takes none.  All pairs are
     * resolved on the velocities after the kinematic update, each unit adding its changes in
     * ascending partner index.  Units that are not alive hold no velocity or acceleration.
     * Needs TabxState.ax / ay. */
    int32_t  dynamics;
    float    move_gain;           /* per time unit; move_gain * dt in (0, 1] is sensible       */
    float    restitution;         /* coefficient of restitution e, normally in [0, 1]          */
} TabxParams;

/* The scenario: unit specifications and zones (the unit and zone axes of the
 * configuration).  Read-only for the library.  All [E * N] unless noted. */
typedef struct TabxScenario {
    const float *init_x, *init_y, *init_theta;     /* spawn pose; theta in [0, 2*pi) */
    const float *hmax, *radius, *mass, *speed;     /* hmax > 0 for enabled units     */
    const float *dmg, *range, *cooldown;           /* dmg < 0 heals allies           */
    const float *sight_angle;                      /* full cone width, rad (obs only) */
    const float *sight_cos_half;                   /* cos(sight_angle / 2)           */
    const float *sight_range;                      /* cone radius                    */
    const float *hurt_halfwidth;                   /* lateral half-width of hurtbox  */
    const uint8_t *team;                           /* 0 = allies, 1 = adversaries (must be 0 or 1:
                                                      any other non-zero byte is read as 1) */
    const uint8_t *enabled;                        /* 0 = padding placeholder        */
    const int8_t  *terrain;    /* [E][grid_h][grid_w] cell codes, NULL iff no grid   */
    const float   *zone_desc;  /* [E][max_zones][6] = type, cx, cy, hx, hy, effect;
                                  NULL iff max_zones == 0                            */
} TabxScenario;

/* Mutable environment state.  [E * N] unless noted.  A snapshot is a copy of
 * these arrays. */
typedef struct TabxState {
    float *x, *y, *vx, *vy, *theta, *hp, *cd, *reveal, *cur_speed;
    uint8_t *alive;
    int32_t *t;          /* [E] ticks since the episode began                 */
    float   *phi_prev;   /* [E] health-ratio potential after the previous tick */
    /* Episode metrics (the paper's appendix "Additional Performance Metrics": episode
     * return, episode length, first kill, win).  All [E]; each may be NULL, but the
     * summaries need their running counterpart (ep_return needs ret_run, ep_first_kill
     * needs kill_run).  tabx_reset clears the running ones. */
    float   *ret_run;        /* allied return accumulated in the running episode        */
    int8_t  *kill_run;       /* which team lost a unit first in the running episode:
                                0 nobody yet, 1 adversaries, 2 allies, 3 both, same tick */
    int32_t *ep_count;       /* episodes finished so far (incremented, never cleared)   */
    int32_t *ep_len;         /* length of the last finished episode                     */
    float   *ep_return;      /* allied return of the last finished episode              */
    int8_t  *ep_win;         /* 1 if the allies won it                                  */
    int8_t  *ep_first_kill;  /* kill_run at its end                                     */
    /* Level bank, required iff params->num_levels > 0, all [E] (see TabxParams.num_levels).
     * The caller initialises next_level (and level_draws, normally to 0) before the first
     * tabx_reset; `level` is written by the library. */
    int32_t *level;          /* the level the env is playing                            */
    int32_t *next_level;     /* the level its next episode will take                    */
    int32_t *level_draws;    /* how many uniform draws the env has made                 */
    /* Optional output, [E][16 * N + 6 * max_zones] f32, 4-byte aligned: if not NULL, every call
     * that produces observations (tabx_observe, tabx_step_observe and the policy / scripted
     * ticks) also writes the global state of tabx_global_state here, for centralised critics
     * that want it every tick; it costs its bytes and no second launch. */
    float   *global_state;
    /* Required iff params->dynamics == 1, [E * N] f32: the acceleration the last action stage set
     * (TabxParams.dynamics); tabx_reset clears it. */
    float   *ax, *ay;
} TabxState;

/* Floats per agent observation: 16 * N + 6 * max_zones.
 * Negative TabxError if the shape is unsupported. */
int tabx_obs_dim(const TabxParams *params);
int tabx_num_actions(void);

/* Starts episodes (App. A "Environment Parameters": configuration applied at
 * reset).  env_mask: device [E] bytes, non-zero = reset that env; NULL = all. */
int tabx_reset(const TabxParams *params, const TabxScenario *scenario,
               const TabxState *state, const uint8_t *env_mask, void *stream);

/* One tick for every env (App. A "Interaction Dynamics", "Reward"):
 * physics -> actions (move / rotate / combat) -> zone effects, alive flags,
 * rewards, termination; a finished env is reset in place and reports done = 1.
 *   actions [E][N] u8 (in), rewards [E][N] f32 (out), dones [E] u8 (out). */
int tabx_step(const TabxParams *params, const TabxScenario *scenario,
              const TabxState *state, const uint8_t *actions,
              float *rewards, uint8_t *dones, void *stream);

/* Per-agent observations of the current state (App. A "Observation and Global
 * State", "Action Space" for the mask).
 *   obs [E][N][D] f32 (out): own block (16 floats), other-unit blocks (16 each,
 *     ascending unit index without self, all zero unless visible), zone slots (6 each);
 *     own = health, health / max, x, y, heading, attack range, damage, cooldown left,
 *           cooldown left / cooldown, body radius, mass, sight angle, alive, current
 *           speed, zone type underfoot, team;
 *     other = health, health / max, x - own x, y - own y, heading, attack range, damage,
 *           cooldown left, cooldown ratio, body radius, mass, sight angle, alive (1),
 *           same team, attackable by the observer, current speed;
 *     zone = type, centre x - own x, centre y - own y, half extent x, half extent y,
 *           effect magnitude (all zero for a slot of type 0);
 *     a disabled unit's row is all zero;
 *   vis_mask [E][N][ceil(N/64)] u64 (out, NULL to skip): bit j of row i = i sees j;
 *   action_mask [E][N] u8 (out, NULL to skip): 1 = the combat action is available. */
int tabx_observe(const TabxParams *params, const TabxScenario *scenario,
                 const TabxState *state, float *obs, uint64_t *vis_mask,
                 uint8_t *action_mask, void *stream);

/* tabx_step followed by tabx_observe in one launch; results identical to the
 * two separate calls. */
int tabx_step_observe(const TabxParams *params, const TabxScenario *scenario,
                      const TabxState *state, const uint8_t *actions,
                      float *rewards, uint8_t *dones, float *obs,
                      uint64_t *vis_mask, uint8_t *action_mask, void *stream);

/* Global state for centralised critics (App. A "Global state"): all unit features without
 * visibility masking plus the zone slots.
 *   out [E][16 * N + 6 * max_zones] f32: unit u's own block (as in its observation row,
 *   absolute position; zero if disabled) at floats [16 u, 16 u + 16), then the zone slots
 *   with absolute centres (zero for type 0).  16-byte aligned. */
int tabx_global_state(const TabxParams *params, const TabxScenario *scenario,
                      const TabxState *state, float *out, void *stream);

/* Role-appropriate heuristic policy for scripted units (Sec. 4.2; App. A "Role-Appropriate
 * Heuristic Policy Mechanism"; tier values in the table "Heuristic policy parameters across
 * all difficulty tier": epsilon / xi = 1.0/0.0 random, 0.5/0.1 novice, 0.2/0.3 medium,
 * 0.1/0.5 advanced, 0.01/0.7 expert; Assassin speed 1.4, Ranger range 10.0 in all of them). */
typedef struct TabxPolicy {
    float    epsilon;          /* probability of a uniformly random action                  */
    float    xi;               /* Rangers retreat from enemies nearer than xi * attack range */
    float    assassin_speed;   /* speed >= this: Assassin                                   */
    float    ranger_range;     /* attack range >= this: Ranger                              */
    uint32_t seed;             /* of the counter-based random numbers                       */
} TabxPolicy;

/* Last known target position per unit, device [E * N]; the caller zeroes mem_valid when an
 * episode of that env starts (or leaves stale memories in, as it prefers). */
typedef struct TabxPolicyMemory {
    float   *mem_x, *mem_y;
    uint8_t *mem_valid;
    uint8_t *next_action;      /* [E * N], only for tabx_scripted_step_observe (else may be NULL) */
} TabxPolicyMemory;

/* Chooses actions[e * N + u] for every enabled, living unit with controlled[e * N + u] != 0
 * (controlled == NULL: all of them) from the current state; other entries of `actions` are
 * not written.  Roles: Healer = negative damage, Assassin and Ranger by the two thresholds;
 * a unit can have several.  Of the units it sees (field of view and bush rule of
 * tabx_observe) a Healer selects the nearest injured ally, else the nearest ally; an Assassin
 * the enemy of lowest maximum health, nearer first among equals; any other unit the nearest
 * enemy; remaining ties go to the lower index.  Then, first rule that applies:
 *   1. combat action, if the cooldown has elapsed and a visible unit it may strike is in the
 *      hurtbox (for a Healer: an ally below maximum health);
 *   2. rotate towards the target's side if it is within range + its body radius of the unit
 *      but not in the hurtbox;
 *   3. Ranger: step away (along the larger axis of the offset) from the nearest visible enemy
 *      if it is nearer than xi * range;
 *   4. idle if the target is in the hurtbox (waiting for the cooldown);
 *   5. move along the larger axis of the offset to the role's goal: behind the target by half
 *      the own range (Assassin), the target itself (Healer), in front of it by half the range
 *      (others); the target's position is remembered;
 *   6. no target: move to the remembered position; within distance 1 of it, forget it and
 *      search;
 *   7. nothing remembered: a Ranger outside bushes moves to the nearest bush-type zone slot
 *      centre; otherwise search = rotate left or right by a random bit.
 * Finally with probability epsilon the action is replaced by one uniform over all eight.
 * Random numbers are a 32-bit hash of (seed, env, unit, tick t, draw index): reproducible and
 * independent of launch shape.  Same stream rules and errors as the other calls. */
int tabx_heuristic_actions(const TabxParams *params, const TabxScenario *scenario,
                           const TabxState *state, const TabxPolicy *policy,
                           const TabxPolicyMemory *memory, const uint8_t *controlled,
                           uint8_t *actions, void *stream);

/* tabx_heuristic_actions followed by tabx_step_observe in one launch: the scripted units'
 * actions are chosen from the state at entry, written into `actions` (in / out: the entries
 * of the other units are read) and applied in the same tick.  An env that finishes also has
 * the mem_valid flags of its units cleared, so the new episode starts without memories (the
 * separate calls leave that to the caller, who sees `dones`).  Otherwise the results are
 * identical to the two calls. */
int tabx_policy_step_observe(const TabxParams *params, const TabxScenario *scenario,
                             const TabxState *state, const TabxPolicy *policy,
                             const TabxPolicyMemory *memory, const uint8_t *controlled,
                             uint8_t *actions, float *rewards, uint8_t *dones, float *obs,
                             uint64_t *vis_mask, uint8_t *action_mask, void *stream);

/* The tick for training against scripted units: same results as tabx_policy_step_observe, but
 * the scripted units decide at the END of the call, on the state the call leaves behind, from
 * the pair tests its observation rows are made of anyway (so the policy costs a few atomics
 * instead of a second all-pairs scan); the decision waits in memory->next_action and the next
 * call applies it (and copies it into `actions`).  The caller primes memory->next_action with
 *     tabx_heuristic_actions(..., controlled, memory->next_action)
 * after tabx_reset and after anything else that changes the state, the policy or `controlled`
 * behind the library's back (a restored snapshot, another tier).  Between such events the
 * sequence of states, actions, memories and observations is identical to the one
 * tabx_policy_step_observe produces. */
int tabx_scripted_step_observe(const TabxParams *params, const TabxScenario *scenario,
                               const TabxState *state, const TabxPolicy *policy,
                               const TabxPolicyMemory *memory, const uint8_t *controlled,
                               uint8_t *actions, float *rewards, uint8_t *dones, float *obs,
                               uint64_t *vis_mask, uint8_t *action_mask, void *stream);

/* Host-only helper for processing a batch in parts (see TabxParams.env_id_offset): fills
 * part_params / part_scenario / part_state with the structs of the envs [first_env,
 * first_env + count) of the given batch: num_envs = count, env_id_offset advanced, every
 * per-unit pointer advanced by first_env * N elements, every per-env pointer by first_env,
 * terrain and zone_desc by first_env rows (scenario arrays are left alone when they are a bank
 * of levels); NULL pointers stay NULL.  The caller advances the other arrays the same way:
 * actions, rewards, action_mask, controlled and the policy memory by first_env * N, dones by
 * first_env, obs by first_env * N * D floats, vis_mask by first_env * N * ceil(N/64) words.
 * obs and vis_mask must stay 16-byte aligned: choose first_env accordingly (a multiple of 4
 * always does).  TABX_ERR_SHAPE if the range does not lie inside the batch. */
int tabx_part(const TabxParams *params, const TabxScenario *scenario, const TabxState *state,
              int32_t first_env, int32_t count, TabxParams *part_params,
              TabxScenario *part_scenario, TabxState *part_state);

/* Host-only: how the library would lay a call out on the machine, without enqueuing anything
 * (for occupancy checks and tuning: on gfx950 a CU keeps as many workgroups resident as its
 * 160 KB of LDS and its registers allow, and the launches are sized against that).  `call` names
 * the entry point; the policy calls count as deciding.  dynamic_lds_bytes is what the launch
 * requests on top of the kernel's static LDS.  TABX_ERR_SHAPE for an unknown call. */
enum TabxCall {
    TABX_CALL_RESET = 0, TABX_CALL_STEP = 1, TABX_CALL_OBSERVE = 2, TABX_CALL_STEP_OBSERVE = 3,
    TABX_CALL_HEURISTIC_ACTIONS = 4, TABX_CALL_POLICY_STEP_OBSERVE = 5,
    TABX_CALL_SCRIPTED_STEP_OBSERVE = 6
};
typedef struct TabxLaunchInfo {
    int32_t workgroups;              /* grid size                                             */
    int32_t threads_per_workgroup;
    int32_t envs_per_workgroup;      /* envs packed into a workgroup                          */
    int32_t wavefronts_per_env_group;/* wavefronts that share those envs (1, 2 or 4)          */
    int32_t rows_per_flush;          /* observation rows of an env staged before a flush      */
    int32_t dynamic_lds_bytes;
    /* the machine the launch shapes are tuned for: compare with the device's own properties */
    int32_t assumed_compute_units;            /* 256                                         */
    int32_t assumed_lds_per_cu_bytes;         /* 160 KB                                      */
    int32_t assumed_lds_per_workgroup_bytes;  /* 64 KB: the most a launch takes per workgroup */
    int32_t assumed_wavefront_lanes;          /* 64                                          */
} TabxLaunchInfo;
int tabx_launch_info(const TabxParams *params, int call, TabxLaunchInfo *info);

const char *tabx_strerror(int code);

#ifdef __cplusplus
}
#endif
#endif /* TABX_H */
