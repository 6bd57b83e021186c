// Random update streams, valid and broken, through the host planner, and random
// iteration times through the mode selector.  Built with the address and
// undefined-behaviour sanitizers by test_host_logic.py (host code only, no HIP):
// every call must return a status without tripping either.
// usage: host_fuzz <planner iterations> <selector iterations>
#include <cstdio>
#include <algorithm>
#include <cmath>
#include <cstdlib>
#include <random>
#include <vector>
#include "star_plan.h"
int main(int argc, char** argv) {
    const long n_plan = argc > 1 ? atol(argv[1]) : 20000, n_sel = argc > 2 ? atol(argv[2]) : 10000;
    std::mt19937_64 rng(1234);
    long ok = 0, bad = 0;
    for (long it = 0; it < n_plan; ++it) {
        int W = 1 + rng() % 32;
        int U = rng() % 40;
        std::vector<int32_t> off(1, 0), mem, st;
        std::vector<float> cf, lr;
        for (int u = 0; u < U; ++u) {
            int y = (rng() % 16 == 0) ? 0 : 1 + rng() % W;
            if (rng() % 64 == 0) y = W + 1 + rng() % 3;
            std::vector<int> ids(W); for (int i = 0; i < W; ++i) ids[i] = i;
            std::shuffle(ids.begin(), ids.end(), rng);
            for (int k = 0; k < y; ++k) {
                int id = ids[k % W];
                if (rng() % 500 == 0) id = (int)(rng() % 70) - 3;
                mem.push_back(id); st.push_back((int)(rng() % 6) - (rng() % 300 == 0));
                float c = (float)((rng() % 2001) / 1000.0 - (rng() % 4 == 0 ? 1.0 : 0.0));
                if (rng() % 2000 == 0) c = NAN;
                cf.push_back(c);
            }
            off.push_back((int32_t)mem.size());
            lr.push_back((float)((rng() % 1000) / 1e4));
        }
        if (rng() % 200 == 0 && off.size() > 2) std::swap(off[1], off[2]);
        star_updates up{};
        up.U = U; up.offsets = off.data(); up.members = mem.data();
        int wm = rng() % 3;
        up.staleness = (wm == 1 || rng() % 4 == 0) ? st.data() : nullptr;
        up.coeff = (wm == 2 || rng() % 4 == 0) ? cf.data() : nullptr;
        up.lr = rng() % 2 ? lr.data() : nullptr;
        star_hparams hp{};
        hp.lr = 0.05f; hp.momentum = (rng() % 10) / 10.0f; hp.weight_decay = (rng() % 3) * 1e-4f;
        hp.wmode = (decltype(hp.wmode))wm; hp.scale_lr_by_group = rng() % 2;
        star::Plan pl; std::string err;
        bool norms = rng() % 2;
        star_status s = rng() % 3 ? star::build_plan(W, &up, &hp, 0, norms, &pl, &err)
                                  : star::build_plan(W, &up, nullptr, wm, true, &pl, &err);
        if (s == STAR_OK) { ++ok; (void)star::choose_route(pl, rng() % 2 ? 4 : 2, rng() % 4); } else ++bad;
    }
    printf("plans accepted %ld rejected %ld\n", ok, bad);
    if (ok == 0 || bad == 0) return 1;  // the generator must exercise both sides
    long sel = 0;
    for (long it = 0; it < n_sel; ++it) {
        int N = 1 + rng() % 32;
        std::vector<double> t(N), ct(N), ts(N), waits(1 + rng() % 6), table;
        for (auto& x : t) x = 0.05 + (rng() % 1000) / 500.0;
        for (auto& x : ct) x = 0.05 + (rng() % 1000) / 400.0;
        for (auto& x : waits) x = (rng() % 300) / 1000.0;
        std::vector<int32_t> go(N + 1), gm(N), strag(N);
        star_mode_choice ch; double td;
        if (star_select_mode_ps(N, t.data(), (rng() % 5000) / 10.0, 128.0 * N, 0.2, (rng() % 50) / 100.0 + 0.01, &ch,
                                ts.data(), &td, go.data(), gm.data(), strag.data()) == STAR_OK) ++sel;
        table.assign(1 + (size_t)N * waits.size(), 0);
        int32_t rem; double w, ta;
        if (star_select_mode_ar(N, t.data(), ct.data(), (rng() % 5000) / 10.0, 128.0 * N, 0.2, (int)waits.size(),
                                waits.data(), &rem, &w, &ta, table.data()) == STAR_OK) ++sel;
    }
    printf("selector calls accepted %ld\n", sel);
    return sel == 2 * n_sel ? 0 : 1;
}
