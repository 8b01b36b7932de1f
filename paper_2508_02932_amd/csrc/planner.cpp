// Packing planner of libplora (host only): the memory model of appendix B, F(D, K) of section 3.2 solved exactly,
// DTM (Alg. 1), the job planner (Alg. 2) and the tail bound of appendix D.  Declared in include/plora_plan.h.
//
// F(D, K) maximises a ratio of two sums over 0-1 variables under one knapsack constraint.  Parametric search over the
// ratio: for a trial value L the best subset for  sum (r_k - L t_k) H_k  is a 0-1 knapsack; if that subset's own ratio
// beats L it becomes the next trial value, otherwise L is the optimum (every step strictly raises L, and there are
// finitely many subsets).  The knapsack is solved by depth-first branch and bound with the fractional bound;
// configurations that are interchangeable (same profit, same memory) are never branched on twice.
#include "plora_plan.h"

#include <algorithm>
#include <cmath>
#include <cstdint>
#include <new>
#include <vector>

namespace {

constexpr int64_t kNodeLimit = int64_t(1) << 26;

bool valid(const plora_plan_problem *p)
{
    if (!p || !p->rank || !p->mem || !p->t_base || !p->t_config) return false;
    return true;
}

plora_status check(const plora_plan_problem *p)
{
    if (!valid(p)) return PLORA_ERR_NULL;
    if (p->n_configs < 1 || p->n_configs > PLORA_PLAN_MAX_CONFIGS) return PLORA_ERR_SHAPE;
    if (p->n_degrees < 1 || p->n_degrees > PLORA_PLAN_MAX_DEGREES) return PLORA_ERR_SHAPE;
    if (!(p->mem_base >= 0.0) || !(p->mem_gpu > 0.0) || !(p->load > 0.0) || !(p->load <= 1.0)) return PLORA_ERR_SHAPE;
    for (int k = 0; k < p->n_configs; ++k)
        if (p->rank[k] < 1 || !(p->mem[k] >= 0.0) || !std::isfinite(p->mem[k])) return PLORA_ERR_SHAPE;
    for (int i = 0; i < p->n_degrees; ++i) {
        if (!(p->t_base[i] >= 0.0) || !std::isfinite(p->t_base[i])) return PLORA_ERR_SHAPE;
        for (int k = 0; k < p->n_configs; ++k) {
            const double t = p->t_config[(size_t)i * p->n_configs + k];
            if (!(t > 0.0) || !std::isfinite(t)) return PLORA_ERR_SHAPE;
        }
    }
    return PLORA_OK;
}

// T(H, d) and the rank sum of a set given in increasing order (the sums are formed in that order).
double duration_of(const plora_plan_problem *p, int deg, const int32_t *cfg, int n)
{
    double s = 0.0;
    for (int i = 0; i < n; ++i) s += p->t_config[(size_t)deg * p->n_configs + cfg[i]];
    return p->t_base[deg] + s;
}

double ratio_of(const plora_plan_problem *p, int deg, const int32_t *cfg, int n)
{
    int64_t r = 0;
    for (int i = 0; i < n; ++i) r += p->rank[cfg[i]];
    return (double)r / duration_of(p, deg, cfg, n);
}

// ---- 0-1 knapsack: maximise the profit of a subset whose weight stays within cap --------------------------------
struct Item { int k; double p, m; };

struct Knapsack {
    std::vector<Item> it;             // sorted by profit per weight, best first; weightless items in front
    std::vector<double> pre_p, pre_m; // prefix sums
    double cap = 0.0, best = -1.0;
    std::vector<char> take, best_take;
    int64_t nodes = 0;
    bool cut = false;

    // fractional bound of what items i.. can add with `room` left
    double bound(int i, double room) const
    {
        const int n = (int)it.size();
        // largest j with pre_m[j] - pre_m[i] <= room
        int lo = i, hi = n;
        while (lo < hi) {
            const int mid = (lo + hi + 1) / 2;
            if (pre_m[mid] - pre_m[i] <= room) lo = mid; else hi = mid - 1;
        }
        double b = pre_p[lo] - pre_p[i];
        if (lo < n) {
            const double left = room - (pre_m[lo] - pre_m[i]);
            if (it[lo].m > 0.0) b += it[lo].p * (left / it[lo].m);
        }
        return b;
    }

    void dfs(int i, double cur_p, double cur_m)
    {
        if (++nodes > kNodeLimit) { cut = true; return; }
        const int n = (int)it.size();
        if (cur_p > best) { best = cur_p; best_take = take; }
        if (i >= n) return;
        // a tiny relative slack keeps the proof sound when the bound and the incumbent differ by rounding only
        if (cur_p + bound(i, cap - cur_m) <= best * (1.0 + 1e-15)) return;
        if (cur_m + it[i].m <= cap) {
            take[i] = 1;
            dfs(i + 1, cur_p + it[i].p, cur_m + it[i].m);
            take[i] = 0;
            if (cut) return;
        }
        int j = i + 1;                 // leaving i out: its twins stay out as well
        while (j < n && it[j].p == it[i].p && it[j].m == it[i].m) ++j;
        dfs(j, cur_p, cur_m);
    }

    // returns the chosen configurations (any order); empty if no item has a positive profit
    std::vector<int> solve(std::vector<Item> items, double capacity)
    {
        cap = capacity;
        it.clear();
        for (const Item &x : items)
            if (x.p > 0.0 && x.m <= cap) it.push_back(x);
        std::sort(it.begin(), it.end(), [](const Item &a, const Item &b) {
            const bool az = a.m == 0.0, bz = b.m == 0.0;
            if (az != bz) return az;
            if (!az) {
                const double ra = a.p / a.m, rb = b.p / b.m;
                if (ra != rb) return ra > rb;
            }
            if (a.p != b.p) return a.p > b.p;
            if (a.m != b.m) return a.m < b.m;
            return a.k < b.k;
        });
        const int n = (int)it.size();
        pre_p.assign(n + 1, 0.0); pre_m.assign(n + 1, 0.0);
        for (int i = 0; i < n; ++i) { pre_p[i + 1] = pre_p[i] + it[i].p; pre_m[i + 1] = pre_m[i] + it[i].m; }
        take.assign(n, 0); best_take.assign(n, 0);
        best = 0.0; nodes = 0; cut = false;
        if (n) dfs(0, 0.0, 0.0);
        std::vector<int> out;
        for (int i = 0; i < n; ++i)
            if (best_take[i]) out.push_back(it[i].k);
        return out;
    }
};

// F(D, K): fills cfg (increasing order) and job; count 0 if nothing fits.
void pack_one(const plora_plan_problem *p, int deg, const uint8_t *avail, int32_t *cfg, plora_plan_job *job)
{
    const int n = p->n_configs;
    const double cap = p->load * p->mem_gpu * (double)(1 << deg) - p->mem_base;
    const double t0 = p->t_base[deg];
    const double *t = p->t_config + (size_t)deg * n;
    job->first = 0; job->count = 0; job->gpus = 1 << deg; job->proved = 1; job->value = 0.0; job->start = 0.0; job->end = 0.0;

    std::vector<int> cand;
    for (int k = 0; k < n; ++k)
        if ((!avail || avail[k]) && p->mem[k] <= cap) cand.push_back(k);
    if (cand.empty()) return;
    // start from the best single configuration
    std::vector<int> cur(1, cand[0]);
    double lam = -1.0;
    for (int k : cand) {
        const double v = (double)p->rank[k] / (t0 + t[k]);
        if (v > lam) { lam = v; cur[0] = k; }
    }
    Knapsack ks;
    for (int iter = 0; iter < 200; ++iter) {
        std::vector<Item> items;
        items.reserve(cand.size());
        for (int k : cand) items.push_back(Item{k, (double)p->rank[k] - lam * t[k], p->mem[k]});
        std::vector<int> s = ks.solve(items, cap);
        if (ks.cut) job->proved = 0;
        if (s.empty()) break;
        std::sort(s.begin(), s.end());
        std::vector<int32_t> s32(s.begin(), s.end());
        const double v = ratio_of(p, deg, s32.data(), (int)s32.size());
        if (!(v > lam)) break;                    // no subset beats the trial ratio: it is the optimum
        lam = v; cur = s;
    }
    std::sort(cur.begin(), cur.end());
    job->count = (int32_t)cur.size();
    for (size_t i = 0; i < cur.size(); ++i) cfg[i] = cur[i];
    job->value = ratio_of(p, deg, cfg, job->count);
}

struct Cand {
    std::vector<plora_plan_job> jobs;
    std::vector<std::vector<int32_t>> cfgs;
    double total() const { double s = 0.0; for (const auto &j : jobs) s += j.value; return s; }
};

void dtm_rec(const plora_plan_problem *p, int g, std::vector<uint8_t> &avail, int n_avail, Cand &tmp, Cand &best, double &best_v, bool &have)
{
    auto leaf = [&]() {
        const double v = tmp.total();
        if (!have || v > best_v) { best = tmp; best_v = v; have = true; }
    };
    if (g <= 0 || n_avail == 0) { leaf(); return; }
    int top = 0;
    while ((2 << top) <= g) ++top;                 // g' = 2^top = 2^floor(log2 g)
    if (top > p->n_degrees - 1) top = p->n_degrees - 1;
    bool went = false;
    std::vector<int32_t> cfg((size_t)p->n_configs);
    for (int deg = top; deg >= 0; --deg) {
        plora_plan_job job;
        pack_one(p, deg, avail.data(), cfg.data(), &job);
        if (job.count == 0) continue;
        went = true;
        std::vector<int32_t> mine(cfg.begin(), cfg.begin() + job.count);
        for (int32_t k : mine) avail[k] = 0;
        tmp.jobs.push_back(job); tmp.cfgs.push_back(mine);
        dtm_rec(p, g - (1 << deg), avail, n_avail - job.count, tmp, best, best_v, have);
        tmp.jobs.pop_back(); tmp.cfgs.pop_back();
        for (int32_t k : mine) avail[k] = 1;
    }
    if (!went) leaf();                              // nothing fits on what is left
}

Cand dtm(const plora_plan_problem *p, int g, std::vector<uint8_t> &avail)
{
    int n_avail = 0;
    for (uint8_t a : avail) n_avail += a != 0;
    Cand tmp, best;
    double best_v = -1.0;
    bool have = false;
    dtm_rec(p, g, avail, n_avail, tmp, best, best_v, have);
    return best;
}

template <class F> plora_status guarded(F f)
{
    try { return f(); }
    catch (const std::bad_alloc &) { return PLORA_ERR_INTERNAL; }
    catch (...) { return PLORA_ERR_INTERNAL; }
}

}  // namespace

extern "C" {

double plora_plan_lora_bytes(const plora_plan_model *m, const plora_plan_lora *c, const plora_plan_sharding *s)
{
    if (!m || !c) return -1.0;
    if (m->n_layers < 1 || m->hidden < 1 || m->kv_hidden < 1 || m->inter < 1 || !(m->c_prec > 0.0) || !(m->c_grad >= 1.0)) return -1.0;
    if (c->rank < 1 || c->batch < 1 || c->seq < 1 || c->targets >= (1u << 7)) return -1.0;
    int zero = 0;
    double tp = 1.0, pp = 1.0, fsdp = 1.0;
    if (s) {
        if (s->zero_level < 0 || s->zero_level > 3 || s->d_tp < 1 || s->d_pp < 1 || s->d_fsdp < 1) return -1.0;
        zero = s->zero_level; tp = s->d_tp; pp = s->d_pp; fsdp = s->d_fsdp;
    }
    const double h = (double)m->hidden, kv = (double)m->kv_hidden, in = (double)m->inter;
    const double h_in[7] = {h, h, h, h, h, h, in}, h_out[7] = {h, kv, kv, h, in, in, h};
    double param = 0.0;
    int n_target = 0;
    for (int i = 0; i < 7; ++i)
        if (c->targets & (1u << i)) {
            param += m->n_layers * (h_in[i] * c->rank + h_out[i] * c->rank) * m->c_prec;
            ++n_target;
        }
    param /= tp * pp;
    const double grad = param, opt = (m->c_grad - 1.0) * param;
    const double act = (double)m->n_layers * n_target * c->batch * c->seq * c->rank * m->c_prec;
    switch (zero) {
    case 0: return param + grad + opt + act;
    case 1: return grad + param + opt / fsdp + act;
    case 2: return param + (grad + opt) / fsdp + act;
    default: return (param + grad + opt) / fsdp + act;
    }
}

plora_status plora_plan_pack(const plora_plan_problem *p, int32_t degree_index, const uint8_t *avail, int32_t *configs_out,
                             plora_plan_job *job_out)
{
    return guarded([&]() -> plora_status {
        plora_status st = check(p);
        if (st != PLORA_OK) return st;
        if (!configs_out || !job_out) return PLORA_ERR_NULL;
        if (degree_index < 0 || degree_index >= p->n_degrees) return PLORA_ERR_SHAPE;
        pack_one(p, degree_index, avail, configs_out, job_out);
        return PLORA_OK;
    });
}

plora_status plora_plan_dtm(const plora_plan_problem *p, int32_t gpus, const uint8_t *avail, plora_plan_job *jobs_out,
                            int32_t jobs_cap, int32_t *n_jobs_out, int32_t *configs_out)
{
    return guarded([&]() -> plora_status {
        plora_status st = check(p);
        if (st != PLORA_OK) return st;
        if (!jobs_out || !n_jobs_out || !configs_out) return PLORA_ERR_NULL;
        if (gpus < 1 || gpus > (1 << (PLORA_PLAN_MAX_DEGREES - 1)) * 8) return PLORA_ERR_SHAPE;
        std::vector<uint8_t> av((size_t)p->n_configs, 1);
        if (avail)
            for (int k = 0; k < p->n_configs; ++k) av[k] = avail[k] ? 1 : 0;
        const Cand c = dtm(p, gpus, av);
        if ((int)c.jobs.size() > jobs_cap) return PLORA_ERR_WORKSPACE;
        int32_t pos = 0;
        for (size_t j = 0; j < c.jobs.size(); ++j) {
            jobs_out[j] = c.jobs[j];
            jobs_out[j].first = pos;
            for (int32_t k : c.cfgs[j]) configs_out[pos++] = k;
        }
        *n_jobs_out = (int32_t)c.jobs.size();
        return PLORA_OK;
    });
}

plora_status plora_plan_schedule(const plora_plan_problem *p, int32_t gpus, plora_plan_job *jobs_out, int32_t jobs_cap,
                                 int32_t *configs_out, plora_plan_summary *out)
{
    return guarded([&]() -> plora_status {
        plora_status st = check(p);
        if (st != PLORA_OK) return st;
        if (!jobs_out || !configs_out || !out) return PLORA_ERR_NULL;
        if (gpus < 1 || gpus > (1 << (PLORA_PLAN_MAX_DEGREES - 1)) * 8) return PLORA_ERR_SHAPE;
        const int n = p->n_configs;
        std::vector<uint8_t> left((size_t)n, 1);
        int n_left = n, g_avail = gpus;
        std::vector<plora_plan_job> jobs;
        std::vector<int> running;                       // indices into jobs
        std::vector<int32_t> cfg_all;
        double now = 0.0;
        while (n_left > 0) {
            if (g_avail > 0) {
                const Cand c = dtm(p, g_avail, left);
                for (size_t j = 0; j < c.jobs.size(); ++j) {
                    plora_plan_job job = c.jobs[j];
                    int deg = 0;
                    while ((1 << deg) < job.gpus) ++deg;
                    job.first = (int32_t)cfg_all.size();
                    job.start = now;
                    job.end = now + duration_of(p, deg, c.cfgs[j].data(), job.count);
                    for (int32_t k : c.cfgs[j]) { cfg_all.push_back(k); left[k] = 0; }
                    n_left -= job.count;
                    g_avail -= job.gpus;
                    running.push_back((int)jobs.size());
                    jobs.push_back(job);
                }
            }
            if (n_left == 0 || running.empty()) break;  // done, or nothing runs and nothing could be started
            now = jobs[running[0]].end;
            for (int j : running) now = std::min(now, jobs[j].end);
            std::vector<int> still;
            for (int j : running) {
                if (jobs[j].end == now) g_avail += jobs[j].gpus; else still.push_back(j);
            }
            running.swap(still);
        }
        if ((int)jobs.size() > jobs_cap) return PLORA_ERR_WORKSPACE;
        plora_plan_summary s;
        s.makespan = 0.0; s.gpu_work = 0.0; s.tail_bound = 1.0; s.n_jobs = (int32_t)jobs.size(); s.n_unscheduled = n_left; s.all_proved = 1;
        int last = -1;
        for (size_t j = 0; j < jobs.size(); ++j) {
            jobs_out[j] = jobs[j];
            s.gpu_work += jobs[j].gpus * (jobs[j].end - jobs[j].start);
            if (last < 0 || jobs[j].end > jobs[last].end) last = (int)j;
            if (!jobs[j].proved) s.all_proved = 0;
        }
        if (last >= 0) {
            s.makespan = jobs[last].end;
            const double t_last = jobs[last].end - jobs[last].start;
            s.tail_bound = s.makespan / (s.makespan - t_last * (double)(gpus - jobs[last].gpus) / (double)gpus);
        }
        size_t pos = 0;
        for (int32_t k : cfg_all) configs_out[pos++] = k;
        for (int k = 0; k < n; ++k)
            if (left[k]) configs_out[pos++] = k;
        *out = s;
        return PLORA_OK;
    });
}

}  // extern "C"
