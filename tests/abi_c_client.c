/*
 * A plain C program that drives the HIP library through include/tabx.h alone (no Python, no
 * torch: hipMalloc / hipMemcpy for the device memory) and checks every tick against the CPU
 * checker, bit for bit.  Test infrastructure: built by tests/c_client.py, run by
 * tests/test_gpu_c_client.py on a GPU machine.  Inputs: a seeded 3v3 batch with a cell grid, two zone
 * slots, a short truncation horizon (so that episodes restart) and a ragged env count.
 *
 * Exit status 0 and a line "abi_c_client: PASS ..." on success; 1 with the first difference
 * otherwise.
 */
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include <hip/hip_runtime_api.h>

#include "tabx.h"
#include "tabx_ref.h"

enum { E = 37, N = 6, GRID = 16, ZONES = 2, TICKS = 80 };
#define EN (E * N)

static uint32_t rng_state = 20260201u;
static uint32_t rnd(void)
{
    rng_state = rng_state * 1664525u + 1013904223u;
    return rng_state >> 8;
}
static float uniform(float lo, float hi) { return lo + (hi - lo) * ((float)rnd() / 16777216.0f); }

#define HIP_OK(call)                                                                        \
    do {                                                                                    \
        hipError_t err_ = (call);                                                           \
        if (err_ != hipSuccess) {                                                           \
            printf("abi_c_client: %s failed: %s\n", #call, hipGetErrorString(err_));        \
            exit(1);                                                                        \
        }                                                                                   \
    } while (0)
#define TABX_OK_OR_DIE(call)                                                                \
    do {                                                                                    \
        int rc_ = (call);                                                                   \
        if (rc_ != TABX_OK) {                                                               \
            printf("abi_c_client: %s returned %d (%s)\n", #call, rc_, tabx_strerror(rc_));  \
            exit(1);                                                                        \
        }                                                                                   \
    } while (0)

static void *to_device(const void *host, size_t bytes)
{
    void *d = NULL;
    HIP_OK(hipMalloc(&d, bytes));
    HIP_OK(hipMemcpy(d, host, bytes, hipMemcpyHostToDevice));
    return d;
}

static void *device_zeros(size_t bytes)
{
    void *d = NULL;
    HIP_OK(hipMalloc(&d, bytes));
    HIP_OK(hipMemset(d, 0, bytes));
    return d;
}

/* Device array against the checker's host array; floats may differ by 1e-5, the rest not at all. */
static int same(const char *name, int tick, const void *dev, const void *host, size_t bytes,
                int is_float, long *inexact)
{
    void *got = malloc(bytes);
    HIP_OK(hipMemcpy(got, dev, bytes, hipMemcpyDeviceToHost));
    int ok = 1;
    if (memcmp(got, host, bytes) != 0) {
        if (!is_float) {
            ok = 0;
        } else {
            const float *g = (const float *)got, *h = (const float *)host;
            for (size_t k = 0; k < bytes / 4; ++k) {
                if (!(fabs((double)g[k] - (double)h[k]) <= 1e-5)) ok = 0;
                else if (g[k] != h[k]) ++*inexact;
            }
        }
        if (!ok) printf("abi_c_client: tick %d: %s differs from the checker\n", tick, name);
    }
    free(got);
    return ok;
}

int main(void)
{
    /* ---- scenario (host) */
    static float init_x[EN], init_y[EN], init_theta[EN], hmax[EN], radius[EN], mass[EN], speed[EN];
    static float dmg[EN], range[EN], cooldown[EN], sight_angle[EN], cos_half[EN], sight_range[EN];
    static float hurt_hw[EN], zone_desc[E * ZONES * 6];
    static uint8_t team[EN], enabled[EN];
    static int8_t terrain[E * GRID * GRID];
    const float map = 16.0f;
    for (int e = 0; e < E; ++e) {
        for (int u = 0; u < N; ++u) {
            const int k = e * N + u, kind = u % 3, side = u / 3;
            team[k] = (uint8_t)side;
            enabled[k] = 1;
            init_x[k] = uniform(side ? 8.0f : 0.5f, side ? 15.5f : 8.0f);
            init_y[k] = uniform(0.5f, 15.5f);
            init_theta[k] = uniform(0.0f, 6.28f);
            /* a striker, a long-range shooter and a healer (negative damage heals allies) */
            hmax[k] = kind == 0 ? 80.0f : (kind == 1 ? 50.0f : 40.0f);
            radius[k] = 0.75f;
            mass[k] = 1.0f;
            speed[k] = kind == 0 ? 1.5f : 1.0f;
            dmg[k] = kind == 0 ? 20.0f : (kind == 1 ? 12.0f : -10.0f);
            range[k] = kind == 1 ? 9.0f : 3.0f;
            cooldown[k] = kind == 0 ? 1.0f : 2.0f;
            sight_angle[k] = 2.5f;
            cos_half[k] = cosf(0.5f * sight_angle[k]);
            sight_range[k] = 11.0f;
            hurt_hw[k] = 1.25f;
        }
        for (int c = 0; c < GRID * GRID; ++c) {
            const uint32_t r = rnd() % 10u;
            terrain[e * GRID * GRID + c] = (int8_t)(r < 7u ? TABX_ZONE_OPEN : (int)(r - 6u));
        }
        for (int z = 0; z < ZONES; ++z) {
            float *d = zone_desc + (e * ZONES + z) * 6;
            d[0] = (float)(z == 0 ? TABX_ZONE_LAVA : (e % 2 ? TABX_ZONE_BUSH : TABX_ZONE_OPEN));
            d[1] = uniform(2.0f, 14.0f);
            d[2] = uniform(2.0f, 14.0f);
            d[3] = uniform(1.0f, 3.0f);
            d[4] = uniform(1.0f, 3.0f);
            d[5] = d[0] == (float)TABX_ZONE_LAVA ? 4.0f : 0.0f;
        }
    }

    TabxParams p;
    memset(&p, 0, sizeof p);
    p.num_envs = E; p.num_units = N; p.grid_w = GRID; p.grid_h = GRID; p.max_zones = ZONES;
    p.max_steps = 25; p.map_w = map; p.map_h = map; p.cell_size = map / GRID; p.dt = 0.25f;
    p.turn_rate = 2.0f; p.lava_dps = 4.0f; p.swamp_mult = 0.5f; p.reveal_time = 1.0f;
    p.boundary_frac = 0.1f;
    RefParams rp;
    memset(&rp, 0, sizeof rp);
    rp.num_envs = E; rp.num_units = N; rp.grid_w = GRID; rp.grid_h = GRID; rp.max_zones = ZONES;
    rp.max_steps = p.max_steps; rp.map_w = map; rp.map_h = map; rp.cell_size = p.cell_size;
    rp.dt = p.dt; rp.turn_rate = p.turn_rate; rp.lava_dps = p.lava_dps;
    rp.swamp_mult = p.swamp_mult; rp.reveal_time = p.reveal_time; rp.boundary_frac = p.boundary_frac;

    const int D = tabx_obs_dim(&p);
    if (D != 16 * N + 6 * ZONES || D != tabx_ref_obs_dim(&rp) || tabx_num_actions() != 8) {
        printf("abi_c_client: observation width %d / action count %d unexpected\n", D, tabx_num_actions());
        return 1;
    }

    /* ---- checker side (host arrays) */
    static float hx[EN], hy[EN], hvx[EN], hvy[EN], hth[EN], hhp[EN], hcd[EN], hrev[EN], hcs[EN], hphi[E];
    static uint8_t halive[EN], hdones[E], hamask[EN], actions[EN];
    static int32_t ht[E];
    static float hrew[EN];
    static unsigned long long hvis[EN];
    float *hobs = (float *)calloc((size_t)EN * D, sizeof(float));
    float *hgs = (float *)calloc((size_t)E * D, sizeof(float));
    RefScenario rsc = {init_x, init_y, init_theta, hmax, radius, mass, speed, dmg, range, cooldown,
                       sight_angle, cos_half, sight_range, hurt_hw, team, enabled,
                       (const signed char *)terrain, zone_desc};
    RefState rst;
    memset(&rst, 0, sizeof rst);
    rst.x = hx; rst.y = hy; rst.vx = hvx; rst.vy = hvy; rst.theta = hth; rst.hp = hhp; rst.cd = hcd;
    rst.reveal = hrev; rst.cur_speed = hcs; rst.alive = halive; rst.t = ht; rst.phi_prev = hphi;

    /* ---- library side (device arrays) */
    TabxScenario sc;
    sc.init_x = to_device(init_x, sizeof init_x);       sc.init_y = to_device(init_y, sizeof init_y);
    sc.init_theta = to_device(init_theta, sizeof init_theta);
    sc.hmax = to_device(hmax, sizeof hmax);             sc.radius = to_device(radius, sizeof radius);
    sc.mass = to_device(mass, sizeof mass);             sc.speed = to_device(speed, sizeof speed);
    sc.dmg = to_device(dmg, sizeof dmg);                sc.range = to_device(range, sizeof range);
    sc.cooldown = to_device(cooldown, sizeof cooldown);
    sc.sight_angle = to_device(sight_angle, sizeof sight_angle);
    sc.sight_cos_half = to_device(cos_half, sizeof cos_half);
    sc.sight_range = to_device(sight_range, sizeof sight_range);
    sc.hurt_halfwidth = to_device(hurt_hw, sizeof hurt_hw);
    sc.team = to_device(team, sizeof team);             sc.enabled = to_device(enabled, sizeof enabled);
    sc.terrain = to_device(terrain, sizeof terrain);    sc.zone_desc = to_device(zone_desc, sizeof zone_desc);
    TabxState st;
    memset(&st, 0, sizeof st);
    float **fields[9] = {&st.x, &st.y, &st.vx, &st.vy, &st.theta, &st.hp, &st.cd, &st.reveal, &st.cur_speed};
    for (int f = 0; f < 9; ++f) *fields[f] = device_zeros(EN * sizeof(float));
    st.alive = device_zeros(EN);
    st.t = device_zeros(E * sizeof(int32_t));
    st.phi_prev = device_zeros(E * sizeof(float));
    st.global_state = device_zeros((size_t)E * D * sizeof(float));
    uint8_t *d_actions = device_zeros(EN), *d_dones = device_zeros(E), *d_amask = device_zeros(EN);
    float *d_rew = device_zeros(EN * sizeof(float));
    float *d_obs = device_zeros((size_t)EN * D * sizeof(float));
    uint64_t *d_vis = device_zeros(EN * sizeof(uint64_t));
    hipStream_t stream;
    HIP_OK(hipStreamCreate(&stream));

    TABX_OK_OR_DIE(tabx_reset(&p, &sc, &st, NULL, stream));
    tabx_ref_reset(&rp, &rsc, &rst, NULL);

    long inexact = 0, episodes = 0;
    for (int tick = 0; tick < TICKS; ++tick) {
        for (int k = 0; k < EN; ++k) actions[k] = (uint8_t)(rnd() % 8u);
        HIP_OK(hipMemcpyAsync(d_actions, actions, EN, hipMemcpyHostToDevice, stream));
        if (tick % 2 == 0) {
            TABX_OK_OR_DIE(tabx_step_observe(&p, &sc, &st, d_actions, d_rew, d_dones, d_obs, d_vis,
                                             d_amask, stream));
        } else {
            TABX_OK_OR_DIE(tabx_step(&p, &sc, &st, d_actions, d_rew, d_dones, stream));
            TABX_OK_OR_DIE(tabx_observe(&p, &sc, &st, d_obs, d_vis, d_amask, stream));
        }
        HIP_OK(hipStreamSynchronize(stream));
        tabx_ref_step(&rp, &rsc, &rst, actions, hrew, hdones, NULL);
        tabx_ref_observe(&rp, &rsc, &rst, hobs, hvis, hamask, NULL);
        tabx_ref_global_state(&rp, &rsc, &rst, hgs);
        int ok = 1;
        ok &= same("x", tick, st.x, hx, sizeof hx, 1, &inexact);
        ok &= same("y", tick, st.y, hy, sizeof hy, 1, &inexact);
        ok &= same("vx", tick, st.vx, hvx, sizeof hvx, 1, &inexact);
        ok &= same("vy", tick, st.vy, hvy, sizeof hvy, 1, &inexact);
        ok &= same("theta", tick, st.theta, hth, sizeof hth, 1, &inexact);
        ok &= same("hp", tick, st.hp, hhp, sizeof hhp, 1, &inexact);
        ok &= same("cd", tick, st.cd, hcd, sizeof hcd, 1, &inexact);
        ok &= same("reveal", tick, st.reveal, hrev, sizeof hrev, 1, &inexact);
        ok &= same("cur_speed", tick, st.cur_speed, hcs, sizeof hcs, 1, &inexact);
        ok &= same("phi_prev", tick, st.phi_prev, hphi, sizeof hphi, 1, &inexact);
        ok &= same("alive", tick, st.alive, halive, sizeof halive, 0, &inexact);
        ok &= same("t", tick, st.t, ht, sizeof ht, 0, &inexact);
        ok &= same("rewards", tick, d_rew, hrew, sizeof hrew, 1, &inexact);
        ok &= same("dones", tick, d_dones, hdones, sizeof hdones, 0, &inexact);
        ok &= same("obs", tick, d_obs, hobs, (size_t)EN * D * sizeof(float), 1, &inexact);
        ok &= same("vis_mask", tick, d_vis, hvis, sizeof hvis, 0, &inexact);
        ok &= same("action_mask", tick, d_amask, hamask, sizeof hamask, 0, &inexact);
        ok &= same("global_state", tick, st.global_state, hgs, (size_t)E * D * sizeof(float), 1, &inexact);
        if (!ok) return 1;
        for (int e = 0; e < E; ++e) episodes += hdones[e];
    }
    if (episodes == 0) {
        printf("abi_c_client: no episode ended, auto-reset was not exercised\n");
        return 1;
    }
    /* an argument error comes back as a code, before any launch */
    TabxParams bad = p;
    bad.num_units = TABX_N_MAX + 1;
    if (tabx_step(&bad, &sc, &st, d_actions, d_rew, d_dones, stream) != TABX_ERR_SHAPE ||
        tabx_step(&p, &sc, &st, NULL, d_rew, d_dones, stream) != TABX_ERR_NULL) {
        printf("abi_c_client: invalid arguments were not refused\n");
        return 1;
    }
    HIP_OK(hipStreamDestroy(stream));
    printf("abi_c_client: PASS (%d envs, %d units, %d ticks, %ld episodes ended, %ld floats within "
           "tolerance but not bit-identical)\n", E, N, TICKS, episodes, inexact);
    return 0;
}
