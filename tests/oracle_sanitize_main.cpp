// Host-side sanitizer run of the CPU checker: random scenarios of several shapes, all features
// on, a few hundred ticks each, under AddressSanitizer and UndefinedBehaviorSanitizer.
// Built and run by tests/test_oracle_sanitizers.py; prints "ok" when it got through.
#include "../oracle/tabx_ref.h"

#include <cstdio>
#include <cstdlib>
#include <random>
#include <vector>

int main()
{
    std::mt19937 rng(12345);
    auto uni = [&](float lo, float hi) { return std::uniform_real_distribution<float>(lo, hi)(rng); };
    const int shapes[][3] = {{5, 1, 0}, {7, 6, 3}, {3, 20, 8}, {2, 33, 5}, {1, 128, 2}};
    for (auto &sh : shapes) {
        for (int ellipses = 0; ellipses < 2; ++ellipses) {
            const int E = sh[0], N = sh[1], Z = sh[2];
            if (ellipses && Z == 0) continue;
            const int G = ellipses ? 0 : 12;
            RefParams p = {};
            p.num_envs = E; p.num_units = N; p.grid_w = p.grid_h = G; p.max_zones = Z;
            p.max_steps = 17; p.map_w = p.map_h = 24.0f; p.cell_size = 2.0f; p.dt = 0.25f;
            p.turn_rate = 1.5f; p.lava_dps = 4.0f; p.swamp_mult = 0.5f; p.reveal_time = 1.0f;
            p.boundary_frac = 0.1f; p.collision_alpha = 0.7f; p.collision_slop = 0.01f;
            p.zone_shapes = ellipses;
            const size_t n = (size_t)E * N;
            std::vector<std::vector<float>> f(14, std::vector<float>(n));
            for (size_t k = 0; k < n; ++k) {
                f[0][k] = uni(0, 24); f[1][k] = uni(0, 24); f[2][k] = uni(0, 6.28f);
                f[3][k] = uni(20, 100); f[4][k] = uni(0.5f, 2); f[5][k] = uni(1, 10);
                f[6][k] = uni(0.5f, 1.5f); f[7][k] = uni(-10, 30); f[8][k] = uni(1, 20);
                f[9][k] = uni(0, 3); f[10][k] = 2.0f; f[11][k] = 0.54f; f[12][k] = 12.0f;
                f[13][k] = f[4][k];
            }
            std::vector<unsigned char> team(n), enabled(n);
            for (size_t k = 0; k < n; ++k) { team[k] = (k % N) >= (size_t)(N + 1) / 2; enabled[k] = rng() % 9 != 0; }
            std::vector<signed char> terrain((size_t)E * G * G);
            for (auto &c : terrain) c = (signed char)((rng() % 3 == 0) ? (rng() % 4) | ((rng() % 3) << 2) : 0);
            std::vector<float> zd((size_t)E * Z * 6);
            for (size_t k = 0; k < zd.size(); k += 6) {
                zd[k] = (float)(rng() % 4); zd[k + 1] = uni(0, 24); zd[k + 2] = uni(0, 24);
                zd[k + 3] = uni(1, 6); zd[k + 4] = uni(1, 6); zd[k + 5] = uni(0.2f, 5);
            }
            RefScenario sc = {f[0].data(), f[1].data(), f[2].data(), f[3].data(), f[4].data(),
                              f[5].data(), f[6].data(), f[7].data(), f[8].data(), f[9].data(),
                              f[10].data(), f[11].data(), f[12].data(), f[13].data(),
                              team.data(), enabled.data(), G ? terrain.data() : nullptr,
                              Z ? zd.data() : nullptr};
            std::vector<std::vector<float>> s(9, std::vector<float>(n));
            std::vector<unsigned char> alive(n);
            std::vector<int> t(E), epc(E), epl(E);
            std::vector<float> phi(E), ret(E), epr(E);
            std::vector<signed char> kr(E), epw(E), epk(E);
            RefState st = {s[0].data(), s[1].data(), s[2].data(), s[3].data(), s[4].data(),
                           s[5].data(), s[6].data(), s[7].data(), s[8].data(), alive.data(),
                           t.data(), phi.data(), ret.data(), kr.data(), epc.data(), epl.data(),
                           epr.data(), epw.data(), epk.data()};
            const int D = tabx_ref_obs_dim(&p);
            std::vector<float> obs(n * D), rew(n), gs((size_t)E * D);
            std::vector<unsigned long long> vis(n * ((N + 63) / 64));
            std::vector<unsigned char> am(n), done(E), act(n);
            std::vector<double> margin(E, 1e30);
            tabx_ref_reset(&p, &sc, &st, nullptr);
            for (int tick = 0; tick < 120; ++tick) {
                for (auto &a : act) a = (unsigned char)(rng() % 10);      // ids 8, 9: treated as idle
                tabx_ref_step(&p, &sc, &st, act.data(), rew.data(), done.data(), margin.data());
                tabx_ref_observe(&p, &sc, &st, obs.data(), vis.data(), am.data(), margin.data());
                tabx_ref_global_state(&p, &sc, &st, gs.data());
            }
        }
    }
    std::puts("ok");
    return 0;
}
