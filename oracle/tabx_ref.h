/*
 * tabx_ref.h -- CPU checker for the TABX batched environment step.
 *
 * TEST INFRASTRUCTURE ONLY.  A plain, slow, single-threaded implementation of
 * the environment rules of the paper's App. A (observation, action space,
 * interaction dynamics, reward, zones), used by the tests, the smoke check and
 * the benchmark's CPU-baseline leg to judge the GPU library.  It shares no code
 * with the GPU library; the product never calls it.
 *
 * All pointers are host pointers owned by the caller.  Per-unit arrays are laid
 * out [E][N] (env-major), float32 state as the workloads prescribe.
 *
 * Arithmetic: every float operation is a single correctly rounded IEEE float32
 * operation (+ - * / sqrt, comparisons) or an explicit fmaf, evaluated in the
 * order written in tabx_ref.cpp; sums over units run in ascending unit index.
 *
 * Parity pins (tests/test_oracle_*.py): hand-worked combat, heal, cooldown,
 * boundary, terrain and reward cases derived from the paper's unit table and
 * formulas; invariants; brute-force visibility/attackability with an
 * independent double-precision atan2/hypot formulation; sincos against libm;
 * the heuristic policy branch by branch on hand-placed units, its tier table
 * against the paper's; the level bank's queue semantics and an identity bank
 * against the plain scenario; the hurtbox variants by hand and by a float64
 * brute force of one tick's health; the collision correction and, with
 * persistent velocities, the relaxation towards the wanted velocity and the
 * restitution impulse against closed forms (equal masses head-on, 50 : 1
 * masses, a kinematic partner, a separating pair) and conserved momentum; the
 * policy again from its passage with units that hold several roles at once;
 * tests/test_oracle_mutations.py plants 196
 * one-line mistakes in copies of this checker and requires the pins to fail on
 * each.  The heuristic's numbers the paper does
 * not give (half-range standoff, arrival radius, the hash behind its random
 * draws) are this build's readings: "parity unpinned" against the authors'.
 * The free parameters the paper does not print (time step, turn rate, sight
 * cone, reveal duration, zone magnitudes) are inputs; their default values are
 * "parity unpinned" with respect to the authors' own code, which is not
 * available.
 */
#ifndef TABX_REF_H
#define TABX_REF_H

#ifdef __cplusplus
extern "C" {
#endif

typedef struct RefParams {
    int   num_envs, num_units;
    int   grid_w, grid_h;       /* terrain cells; 0 = no terrain */
    int   max_zones;            /* zone descriptor slots per env in the observation */
    int   max_steps;            /* truncation horizon */
    float map_w, map_h, cell_size;
    float dt, turn_rate;
    float lava_dps, swamp_mult, reveal_time, boundary_frac;
    float collision_alpha;      /* fraction of an overlap corrected per tick; 0 = bodies pass through */
    float collision_slop;       /* overlap tolerated without correction */
    int   zone_shapes;          /* 0: zones are the cells of `terrain`; 1: zones are the ellipses of
                                   zone_desc (centre, semi-axes, own effect magnitude)           */
    int   num_levels;           /* 0: row e of the scenario arrays configures env e.  L > 0: the
                                   scenario arrays are a bank of L levels and env e plays row
                                   level[e], re-drawn whenever one of its episodes starts        */
    unsigned level_seed;        /* of the uniform level draws                                    */
    int   hurtbox_cone;         /* 1: the hurtbox is also bounded by the unit's field of view: a
                                   body in the rectangle counts only if its centre lies within
                                   the sight cone's angle (any distance)                         */
    int   hit_all;              /* 0: a strike lands on the closest valid body in the hurtbox;
                                   1: on every valid body in it                                  */
    int   dynamics;             /* 0: kinematic (a move sets the velocity outright, everything else
                                   zeroes it).  1: persistent velocity: the action stage sets an
                                   acceleration (move_gain * (wanted velocity - velocity)), the physics
                                   stage integrates it (velocity first, then position), and colliding
                                   bodies exchange an impulse with restitution                    */
    float move_gain;            /* dynamics = 1: how fast the velocity follows the wanted one, per time unit */
    float restitution;          /* dynamics = 1: coefficient of restitution e of the collision impulse       */
    const int *env_ids;         /* NULL, or [E]: the index each env has in the batch it was taken
                                   from; the random draws (level draws, heuristic policy) are
                                   keyed by it, so a sample of a large batch replays exactly     */
} RefParams;

typedef struct RefScenario {
    const float *init_x, *init_y, *init_theta;
    const float *hmax, *radius, *mass, *speed, *dmg, *range, *cooldown;
    const float *sight_angle, *sight_cos_half, *sight_range, *hurt_halfwidth;
    const unsigned char *team, *enabled;
    const signed char   *terrain;    /* [rows][grid_h][grid_w] or NULL */
    const float         *zone_desc;  /* [rows][max_zones][6] or NULL   */
} RefScenario;

typedef struct RefState {
    float *x, *y, *vx, *vy, *theta, *hp, *cd, *reveal, *cur_speed;
    unsigned char *alive;
    int   *t;          /* [E] */
    float *phi_prev;   /* [E] */
    /* episode metrics (the paper's "Additional Performance Metrics": return, length,
     * first kill, win); all [E], all optional (NULL) */
    float *ret_run;          /* allied return accumulated in the running episode       */
    signed char *kill_run;   /* which team lost a unit first in the running episode:
                                0 nobody yet, 1 adversaries, 2 allies, 3 both same tick */
    int   *ep_count;         /* episodes finished so far                               */
    int   *ep_len;           /* length of the last finished episode                    */
    float *ep_return;        /* allied return of the last finished episode             */
    signed char *ep_win;     /* 1 if the allies won it                                 */
    signed char *ep_first_kill; /* kill_run at its end                                 */
    /* level bank (num_levels > 0), all [E]: the level being played, the level the next
     * episode will take (refilled with a uniform draw when it is taken; the caller may
     * overwrite it), and how many draws the env has made */
    int   *level, *next_level, *level_draws;
    /* dynamics = 1: the acceleration the last action stage set, [E][N] (NULL otherwise) */
    float *ax, *ay;
} RefState;

int  tabx_ref_obs_dim(const RefParams *p);
void tabx_ref_sincos(float theta, float *s, float *c);
void tabx_ref_sincos_n(const float *theta, int n, float *s, float *c);

/* env_mask: [E] bytes, non-zero = reset that env; NULL = all. */
void tabx_ref_reset(const RefParams *p, const RefScenario *sc, RefState *st,
                    const unsigned char *env_mask);

/* actions [E][N] u8; rewards [E][N] f32; dones [E] u8.
 * min_margin: [E] doubles or NULL; each entry is lowered to the smallest
 * distance (world units or radians) of any tested pair from a hurtbox boundary
 * seen in this call (diagnostic, never feeds back into the results). */
void tabx_ref_step(const RefParams *p, const RefScenario *sc, RefState *st,
                   const unsigned char *actions, float *rewards,
                   unsigned char *dones, double *min_margin);

/* obs [E][N][D]; vis_mask [E][N][ceil(N/64)] u64 or NULL; action_mask [E][N] or NULL.
 * min_margin as above, for the sight-range, sight-angle and hurtbox tests. */
void tabx_ref_observe(const RefParams *p, const RefScenario *sc, const RefState *st,
                      float *obs, unsigned long long *vis_mask,
                      unsigned char *action_mask, double *min_margin);

/* Role-appropriate heuristic policy (Sec. 4.2, App. A "Role-Appropriate Heuristic Policy
 * Mechanism", table "Heuristic policy parameters"). */
typedef struct RefPolicy {
    float epsilon;          /* probability of a uniformly random action instead of the intended one */
    float xi;               /* Rangers retreat from enemies closer than xi * attack range          */
    float assassin_speed;   /* speed >= this: Assassin class (1.4 in every tier of the table)      */
    float ranger_range;     /* attack range >= this: Ranger class (10.0)                           */
    unsigned seed;          /* of the counter-based random numbers                                 */
} RefPolicy;

typedef struct RefPolicyMemory {   /* last known target position per unit, [E*N] */
    float *mem_x, *mem_y;
    unsigned char *mem_valid;
} RefPolicyMemory;

/* Writes actions[e*N+u] for every unit with controlled[e*N+u] != 0 that is enabled and alive;
 * other entries are left alone. */
void tabx_ref_heuristic_actions(const RefParams *p, const RefScenario *sc, const RefState *st,
                                const RefPolicy *pol, RefPolicyMemory *mem,
                                const unsigned char *controlled, unsigned char *actions);
unsigned tabx_ref_hash(unsigned seed, unsigned env, unsigned unit, unsigned tick, unsigned draw);

/* Global state (App. A "Global state"): out [E][16 * N + 6 * Z]: every unit's own block
 * (as in its observation row, absolute position, zero if disabled), then the zone slots
 * with absolute centres (zero for type 0).  No visibility masking. */
void tabx_ref_global_state(const RefParams *p, const RefScenario *sc, const RefState *st,
                           float *out);

#ifdef __cplusplus
}
#endif
#endif
