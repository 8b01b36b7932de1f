// Host-side driver for the sanitizer tier (AddressSanitizer + UndefinedBehaviorSanitizer on the host code of
// libplora; no GPU is touched).  It walks seeded random descriptions - valid ones and ones broken in every way the
// validator names - through every host-only entry point and through the argument checks of the device entry points
// (each call is made to fail its last check, so everything in front of the first launch runs and nothing is enqueued),
// and random planner instances through the planner.  It checks a few structural facts itself; what it is for is that
// the sanitizers see all of that code run.  Prints "ok <calls>" and exits 0.
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <atomic>
#include <random>
#include <thread>
#include <vector>

#include "plora.h"
#include "plora_debug.h"
#include "plora_plan.h"

#define REQUIRE(c) do { if (!(c)) { std::fprintf(stderr, "driver check failed: %s (line %d)\n", #c, __LINE__); std::exit(2); } } while (0)

struct Desc {
    std::vector<int32_t> off, ad, rank;
    std::vector<float> scale;
    plora_desc d{};
    void bind()
    {
        d.n_seg = (int32_t)ad.size(); d.n_adapters = (int32_t)rank.size();
        d.seg_off = off.data(); d.seg_adapter = ad.data();
        d.rank = rank.empty() ? nullptr : rank.data(); d.scale = scale.empty() ? nullptr : scale.data();
    }
};

static Desc random_desc(std::mt19937 &g, bool big)
{
    Desc x;
    auto u = [&](int lo, int hi) { return (int)(lo + g() % (unsigned)(hi - lo + 1)); };
    const int n_ad = u(0, big ? 200 : 6), n_seg = u(n_ad ? 1 : 0, big ? 300 : 9);
    x.off.push_back(0);
    for (int s = 0; s < n_seg; ++s) {
        x.off.push_back(x.off.back() + (u(0, 4) == 0 ? 0 : u(1, big ? 700 : 300)));
        x.ad.push_back(n_ad ? u(-1, n_ad - 1) : -1);
    }
    for (int k = 0; k < n_ad; ++k) { x.rank.push_back(u(1, PLORA_MAX_RANK)); x.scale.push_back(0.25f * (float)u(1, 16)); }
    x.d.T = x.off.back(); x.d.d_in = 8 * u(1, 600); x.d.d_out = 8 * u(1, 600);
    x.d.dtype = u(0, 3) ? PLORA_BF16 : PLORA_F32; x.d.w_layout = u(0, 1);
    x.bind();
    return x;
}

static std::atomic<long> calls{0};

static void host_calls(const Desc &x, std::mt19937 &g)
{
    const plora_desc *d = &x.d;
    const plora_status st = plora_validate(d); ++calls;
    REQUIRE(plora_status_string(st) != nullptr);
    const size_t ws = plora_workspace_bytes(d), wl = plora_lora_workspace_bytes(d), wq = plora_nf4_workspace_bytes(d);
    calls += 3;
    REQUIRE((st == PLORA_OK) == (ws != 0));
    if (st != PLORA_OK) { REQUIRE(wl == 0 && wq == 0 && plora_h_elems(d) == 0); return; }
    REQUIRE(wl >= 256);
    std::vector<int64_t> h_off((size_t)d->n_seg + 1);
    const int32_t br = 1 + (int32_t)(g() % 300);
    const int64_t nb = plora_build_metadata(d, br, h_off.data(), nullptr, 0); ++calls;
    REQUIRE(nb >= 0 && (size_t)h_off.back() == plora_h_elems(d));
    std::vector<int32_t> blocks((size_t)nb * 4 + 4);
    REQUIRE(plora_build_metadata(d, br, nullptr, blocks.data(), nb) == nb); ++calls;
    REQUIRE(plora_build_metadata(d, br, nullptr, blocks.data(), nb / 2) == nb); ++calls;      // short buffer: count still right
    plora_debug_info info;
    std::memset(&info, 0, sizeof info);
    const int need = plora_debug_metadata(d, &info, nullptr, 0); ++calls;
    if (need >= 0 && info.table_bytes > 0) {
        std::vector<char> tables((size_t)info.table_bytes);
        REQUIRE(plora_debug_metadata(d, &info, tables.data(), tables.size()) >= 0); ++calls;
    }
    // device entry points, each made to fail its last check: everything in front of the first launch runs
    std::vector<const void *> tab((size_t)d->n_adapters + 1, reinterpret_cast<const void *>(uintptr_t(0x10000)));
    std::vector<float *> gtab((size_t)d->n_adapters + 1, reinterpret_cast<float *>(uintptr_t(0x20000)));
    void *fake = reinterpret_cast<void *>(uintptr_t(0x40000));
    const size_t lots = size_t(1) << 50;
    if (d->T > 0) {
        REQUIRE(plora_linear_fwd(d, fake, fake, tab.data(), tab.data(), nullptr, nullptr, fake, lots, nullptr) == PLORA_ERR_NULL);
        REQUIRE(plora_linear_bwd(d, fake, fake, tab.data(), tab.data(), nullptr, nullptr, fake, gtab.data(), gtab.data(), fake, lots, nullptr) == PLORA_ERR_NULL);
        REQUIRE(plora_lora_fwd(d, fake, tab.data(), tab.data(), nullptr, nullptr, fake, lots, nullptr) == PLORA_ERR_NULL);
        REQUIRE(plora_linear_fwd_noalloc(d, fake, fake, tab.data(), tab.data(), nullptr, nullptr, nullptr) != PLORA_OK);
        calls += 4;
    }
    REQUIRE(plora_linear_fwd(d, fake, fake, tab.data(), tab.data(), fake, nullptr, fake, ws - 1, nullptr) == PLORA_ERR_WORKSPACE); ++calls;
    // groups of 1 to 4 projections on this packing (own widths and ranks)
    const int n_proj = 1 + (int)(g() % PLORA_MAX_GROUP);
    std::vector<Desc> ps((size_t)n_proj, x);
    std::vector<plora_desc> pd;
    for (int p = 0; p < n_proj; ++p) {
        ps[p].d.d_out = 8 * (1 + (int64_t)(g() % 300));
        for (auto &r : ps[p].rank) r = 1 + (int32_t)(g() % PLORA_MAX_RANK);
        ps[p].bind();
    }
    for (int p = 0; p < n_proj; ++p) pd.push_back(ps[p].d);
    plora_group grp{n_proj, pd.data()};
    const size_t gw = plora_group_workspace_bytes(&grp); ++calls;
    size_t sum = 0;
    for (int p = 0; p < n_proj; ++p) sum += plora_workspace_bytes(&pd[p]);
    REQUIRE(gw >= sum);
    if (d->T > 0) {
        std::vector<const void *> arr((size_t)n_proj, fake);
        std::vector<const void *const *> tabs((size_t)n_proj, tab.data());
        std::vector<void *> ys((size_t)n_proj, fake);
        ys.back() = nullptr;                                                        // the last projection's y is missing
        REQUIRE(plora_group_fwd(&grp, fake, arr.data(), tabs.data(), tabs.data(), ys.data(), nullptr, fake, lots, nullptr) == PLORA_ERR_NULL);
        ++calls;
    }
    pd.back().T += 1;                                                               // a projection that disagrees
    REQUIRE(plora_group_workspace_bytes(&grp) == 0 || n_proj == 1); ++calls;
}

static void break_desc(Desc x, std::mt19937 &g)
{
    switch (g() % 8) {
    case 0: x.d.d_in += 4; break;
    case 1: if (!x.off.empty()) x.off.back() += 1; break;
    case 2: if (!x.ad.empty()) x.ad[g() % x.ad.size()] = (int32_t)x.rank.size(); break;
    case 3: if (!x.rank.empty()) x.rank[g() % x.rank.size()] = PLORA_MAX_RANK + 1; break;
    case 4: x.d.dtype = 9; break;
    case 5: x.d.w_layout = 2; break;
    case 6: x.d.T = -1; break;
    default: if (x.off.size() > 2) std::swap(x.off[1], x.off.back()); break;
    }
    x.bind();
    (void)plora_validate(&x.d); (void)plora_workspace_bytes(&x.d); (void)plora_h_elems(&x.d);
    (void)plora_build_metadata(&x.d, 64, nullptr, nullptr, 0);
    plora_group grp{1, &x.d};
    (void)plora_group_workspace_bytes(&grp);
    calls += 5;
}

static void planner_calls(std::mt19937 &g)
{
    const int n = 1 + (int)(g() % 40), n_deg = 1 + (int)(g() % 4), gpus = 1 + (int)(g() % 9);
    std::uniform_real_distribution<double> u01(0.0, 1.0);
    std::vector<int32_t> rank((size_t)n);
    std::vector<double> mem((size_t)n), t_base((size_t)n_deg), t_cfg((size_t)n * n_deg);
    const int32_t choices[5] = {8, 16, 32, 64, 128};
    for (int k = 0; k < n; ++k) {
        rank[k] = choices[g() % 5];
        mem[k] = (g() % 3 == 0) ? (double)rank[k] : rank[k] * (0.8 + 0.4 * u01(g));   // ties on purpose, one time in three
    }
    for (int i = 0; i < n_deg; ++i) {
        t_base[i] = 30.0 / (1 << i);
        for (int k = 0; k < n; ++k) t_cfg[(size_t)i * n + k] = rank[k] * (0.05 + 0.1 * u01(g)) / (1 << i);
    }
    plora_plan_problem p{n, n_deg, rank.data(), mem.data(), 40.0 + 100.0 * u01(g), 150.0 + 400.0 * u01(g), 0.9, t_base.data(), t_cfg.data()};
    std::vector<int32_t> cfg((size_t)n);
    std::vector<uint8_t> avail((size_t)n);
    for (auto &a : avail) a = g() % 4 != 0;
    plora_plan_job job;
    REQUIRE(plora_plan_pack(&p, (int32_t)(g() % n_deg), avail.data(), cfg.data(), &job) == PLORA_OK);
    for (int i = 0; i < job.count; ++i) REQUIRE(avail[cfg[i]] && (i == 0 || cfg[i] > cfg[i - 1]));
    std::vector<plora_plan_job> jobs((size_t)n + 16);
    int32_t nj = 0;
    REQUIRE(plora_plan_dtm(&p, gpus, nullptr, jobs.data(), (int32_t)jobs.size(), &nj, cfg.data()) == PLORA_OK);
    int used = 0;
    for (int j = 0; j < nj; ++j) used += jobs[j].gpus;
    REQUIRE(used <= gpus);
    plora_plan_summary s;
    REQUIRE(plora_plan_schedule(&p, gpus, jobs.data(), (int32_t)jobs.size(), cfg.data(), &s) == PLORA_OK);
    std::vector<int> seen((size_t)n, 0);
    for (int k = 0; k < n; ++k) { REQUIRE(cfg[k] >= 0 && cfg[k] < n); seen[cfg[k]] += 1; }
    for (int k = 0; k < n; ++k) REQUIRE(seen[k] == 1);                                 // every configuration exactly once
    REQUIRE(s.makespan * (1.0 + 1e-12) >= s.gpu_work / gpus && s.tail_bound >= 1.0);
    REQUIRE(plora_plan_schedule(&p, gpus, jobs.data(), 0, cfg.data(), &s) == (s.n_jobs ? PLORA_ERR_WORKSPACE : PLORA_OK));
    plora_plan_model m{32, 4096, 1024, 14336, 2.0, 3.0};
    plora_plan_lora c{(int32_t)rank[0], 1 + (int32_t)(g() % 8), 512, (uint32_t)(g() % 128)};
    plora_plan_sharding sh{(int32_t)(g() % 4), 1 << (g() % 3), 1 << (g() % 2), 1 << (g() % 4)};
    REQUIRE(plora_plan_lora_bytes(&m, &c, &sh) >= 0.0 && plora_plan_lora_bytes(&m, &c, nullptr) >= 0.0);
    calls += 6;
}

// Several host threads on the same and on different descriptions at once (the library's only shared state is the
// cache of derived metadata): for the thread sanitizer.
static void threaded(int rounds)
{
    std::vector<std::thread> th;
    for (int t = 0; t < 8; ++t)
        th.emplace_back([t, rounds]() {
            std::mt19937 g(77u + (unsigned)(t % 3));          // threads 0, 3, 6 (and so on) walk the same descriptions
            for (int i = 0; i < rounds; ++i) {
                Desc x = random_desc(g, false);
                host_calls(x, g);
                planner_calls(g);
            }
        });
    for (auto &t : th) t.join();
}

int main(int argc, char **argv)
{
    const int rounds = argc > 1 ? std::atoi(argv[1]) : 300;
    if (argc > 2 && std::strcmp(argv[2], "threads") == 0) {
        threaded(rounds);
        std::printf("ok %ld\n", calls.load());
        return 0;
    }
    std::mt19937 g(20250802u);
    for (int i = 0; i < rounds; ++i) {
        Desc x = random_desc(g, i % 10 == 9);
        host_calls(x, g);
        break_desc(x, g);
        planner_calls(g);
    }
    REQUIRE(plora_validate(nullptr) == PLORA_ERR_NULL && plora_workspace_bytes(nullptr) == 0 && plora_group_workspace_bytes(nullptr) == 0);
    std::printf("ok %ld\n", calls.load());
    return 0;
}
