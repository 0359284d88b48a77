// Discrete-event simulator of MarsRL's agentic rollout scheduling (host code; the model is stated in mars_sched.h).
//
// Layout: flat structure-of-arrays item and group tables that grow in creation order, a FIFO of waiting sequences and a
// compact array of running ones; per (problem, role) a counter of groups still out.  One pass over the running set per
// stage; everything a stage completes is resolved in group-creation order, which makes the run independent of container
// iteration order.  Random draws are hashes of what they are for, never of when they are made.
#include <algorithm>
#include <cmath>
#include <cstdint>
#include <deque>
#include <vector>

#include "mars_sched.h"

namespace {

constexpr int kRoles = 5;
enum Purpose { kLenClass = 0, kLen = 1, kOutcome = 2, kPick = 3 };

inline uint64_t mix(uint64_t z) {
    z += 0x9E3779B97F4A7C15ull;
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    return z ^ (z >> 31);
}

struct Sim {
    const mars_sched_config_t &c;
    uint64_t seed_mix;
    // items
    std::vector<int32_t> problem, role, group, member, parent, length, left, value, reward;
    std::vector<int64_t> t_done;
    // groups
    std::vector<int32_t> g_problem, g_role, g_index, g_parent, g_left;
    std::vector<int64_t> g_submit, g_done;
    std::vector<std::vector<int32_t>> by_agent;      // [problem * kRoles + role] -> group ids
    std::vector<int32_t> out_groups;                 // [problem * kRoles + role] -> groups not yet back
    std::vector<int64_t> end_time;
    std::deque<int32_t> waiting;
    std::vector<int32_t> running;
    int32_t early_stop[kRoles] = {0, 0, 0, 0, 0};

    explicit Sim(const mars_sched_config_t &cfg) : c(cfg), seed_mix(mix(cfg.seed)) {
        by_agent.resize((size_t)c.problems * kRoles);
        out_groups.assign((size_t)c.problems * kRoles, 0);
        end_time.assign(c.problems, -1);
    }

    uint64_t draw(int p, int r, int g, int m, int purpose) const {
        const uint64_t key = ((((uint64_t)p * 8 + r) * 4 + g) * 64 + m) * 8 + purpose;
        return mix(seed_mix ^ key);
    }
    static bool holds(uint64_t u, int32_t p24) { return (int64_t)(u >> 40) < (int64_t)p24; }
    static bool verifier(int r) { return r == 1 || r == 3; }

    void submit(int p, int r, const std::vector<int32_t> &parents, int64_t now) {
        for (size_t gi = 0; gi < parents.size(); ++gi) {
            const int32_t gid = (int32_t)g_problem.size();
            g_problem.push_back(p); g_role.push_back(r); g_index.push_back((int32_t)gi); g_parent.push_back(parents[gi]);
            g_left.push_back(c.group_size); g_submit.push_back(now); g_done.push_back(-1);
            by_agent[(size_t)p * kRoles + r].push_back(gid);
            for (int m = 0; m < c.group_size; ++m) {
                const bool is_long = holds(draw(p, r, (int)gi, m, kLenClass), c.p_long[r]);
                const int64_t lo = is_long ? c.short_hi[r] : c.short_lo[r], hi = is_long ? c.long_hi[r] : c.short_hi[r];
                const int32_t len = (int32_t)(lo + (int64_t)((draw(p, r, (int)gi, m, kLen) >> 11) % (uint64_t)(hi - lo + 1)));
                const uint64_t w = draw(p, r, (int)gi, m, kOutcome);
                int32_t val, rew;
                if (verifier(r)) {
                    const bool wrong = value[parents[gi]] == 0;
                    val = holds(w, wrong ? c.p_flag_wrong[r] : c.p_flag_right[r]) ? 1 : 0;
                    rew = (val == (wrong ? 1 : 0)) ? 1 : 0;
                } else {
                    const bool was_right = r != 0 && value[parent[parents[gi]]] == 1;
                    val = holds(w, was_right ? c.p_keep[r] : c.p_correct[r]) ? 1 : 0;
                    rew = val;
                }
                const int32_t id = (int32_t)problem.size();
                problem.push_back(p); role.push_back(r); group.push_back(gid); member.push_back(m); parent.push_back(parents[gi]);
                length.push_back(len); left.push_back(len); value.push_back(val); reward.push_back(rew); t_done.push_back(-1);
                waiting.push_back(id);
            }
        }
        out_groups[(size_t)p * kRoles + r] = (int32_t)parents.size();
    }

    // up to m distinct elements of `from`, appended to `to`: partial Fisher-Yates, draw j keyed by (list, j)
    void pick(std::vector<int32_t> from, int m, int p, int r, int list, std::vector<int32_t> &to) const {
        const int n = (int)from.size();
        for (int j = 0; j < m && j < n; ++j) {
            const int i = j + (int)((draw(p, r, 3, list * 8 + j, kPick) >> 11) % (uint64_t)(n - j));
            std::swap(from[j], from[i]);
            to.push_back(from[j]);
        }
    }

    std::vector<int32_t> choose(const std::vector<int32_t> &cands, int p, int r) const {
        std::vector<int32_t> sel, pos, neg;
        for (int32_t i : cands) (reward[i] == 1 ? pos : neg).push_back(i);
        const int n = c.n_select;
        if (c.strategy == 0) {
            pick(cands, n, p, r, 0, sel);
        } else if (c.strategy == 1) {
            pick(pos, n / 2, p, r, 1, sel);
            pick(neg, n - n / 2, p, r, 2, sel);
            std::vector<int32_t> rest;
            for (int32_t i : cands)
                if (std::find(sel.begin(), sel.end(), i) == sel.end()) rest.push_back(i);
            pick(rest, n - (int)sel.size(), p, r, 3, sel);
        } else {
            const bool v = verifier(r);
            pick(v ? neg : pos, n, p, r, 1, sel);
            pick(v ? pos : neg, n - (int)sel.size(), p, r, 2, sel);
        }
        return sel;
    }

    void agent_done(int p, int r, int64_t now) {
        if (r == kRoles - 1) { end_time[p] = now; return; }
        std::vector<int32_t> cands;
        for (int32_t gid : by_agent[(size_t)p * kRoles + r])
            for (int m = 0; m < c.group_size; ++m) {
                const int32_t id = first_item(gid) + m;
                if (verifier(r + 1) || value[id] == 1) cands.push_back(id);
            }
        const std::vector<int32_t> sel = choose(cands, p, r + 1);
        if (sel.empty()) { end_time[p] = now; ++early_stop[r + 1]; return; }
        submit(p, r + 1, sel, now);
    }
    int32_t first_item(int32_t gid) const { return gid * c.group_size; }      // groups and their items are created together

    int64_t now = 0, tokens = 0;
    void run() {
        for (int p = 0; p < c.problems; ++p) submit(p, 0, std::vector<int32_t>{-1}, 0);
        std::vector<int32_t> back;
        while (!waiting.empty() || !running.empty()) {
            while (!waiting.empty() && (c.capacity == 0 || (int)running.size() < c.capacity)) {
                running.push_back(waiting.front());
                waiting.pop_front();
            }
            int32_t step = 0;
            for (int32_t id : running) step = std::max(step, std::min(c.segment, left[id]));
            now += step;
            back.clear();
            size_t keep = 0;
            for (size_t k = 0; k < running.size(); ++k) {
                const int32_t id = running[k];
                const int32_t d = std::min(c.segment, left[id]);
                left[id] -= d;
                tokens += d;
                if (left[id] == 0) {
                    t_done[id] = now;
                    if (--g_left[group[id]] == 0) back.push_back(group[id]);
                } else {
                    running[keep++] = id;
                }
            }
            running.resize(keep);
            std::sort(back.begin(), back.end());
            for (int32_t gid : back) {
                g_done[gid] = now;
                const size_t a = (size_t)g_problem[gid] * kRoles + g_role[gid];
                if (--out_groups[a] == 0) agent_done(g_problem[gid], g_role[gid], now);
            }
        }
    }
};

int check(const mars_sched_config_t *c) {
    if (!c) return 1;
    if (c->problems < 1 || c->group_size < 1 || c->group_size > 64 || c->n_select < 1 || c->n_select > 8 || c->segment < 1 ||
        c->capacity < 0 || c->strategy < 0 || c->strategy > 2)
        return 2;
    for (int r = 0; r < kRoles; ++r) {
        if (c->short_lo[r] < 1 || c->short_hi[r] < c->short_lo[r] || c->long_hi[r] < c->short_hi[r]) return 2;
        const int32_t ps[5] = {c->p_long[r], c->p_correct[r], c->p_keep[r], c->p_flag_wrong[r], c->p_flag_right[r]};
        for (int32_t p : ps)
            if (p < 0 || p > (1 << 24)) return 2;
    }
    return 0;
}

}  // namespace

extern "C" {

int mars_sched_bounds(const mars_sched_config_t *cfg, int64_t *max_items, int64_t *max_groups) {
    const int st = check(cfg);
    if (st) return st;
    if (!max_items || !max_groups) return 1;
    *max_groups = (int64_t)cfg->problems * (1 + 4 * cfg->n_select);
    *max_items = *max_groups * cfg->group_size;
    return 0;
}

int mars_sched_simulate(const mars_sched_config_t *cfg, mars_sched_summary_t *summary, const mars_sched_arrays_t *out,
                        int64_t cap_items, int64_t cap_groups) {
    const int st = check(cfg);
    if (st) return st;
    if (!summary) return 1;
    Sim s(*cfg);
    s.run();
    const int64_t ni = (int64_t)s.problem.size(), ng = (int64_t)s.g_problem.size();
    const int G = cfg->group_size;
    if (out && (ni > cap_items || ng > cap_groups)) return 3;
    summary->makespan = s.now;
    summary->tokens = s.tokens;
    summary->n_items = (int32_t)ni;
    summary->n_groups = (int32_t)ng;
    for (int r = 0; r < kRoles; ++r) summary->early_stop[r] = s.early_stop[r];
    int64_t sum_train = 0, sum_wait = 0;
    for (int64_t g = 0; g < ng; ++g) {
        const int64_t t_train = cfg->pipeline ? s.g_done[g] : s.end_time[s.g_problem[g]];
        sum_train += t_train;
        sum_wait += t_train - s.g_submit[g];
        if (!out) continue;
        if (out->group_problem) out->group_problem[g] = s.g_problem[g];
        if (out->group_role) out->group_role[g] = s.g_role[g];
        if (out->group_index) out->group_index[g] = s.g_index[g];
        if (out->group_parent) out->group_parent[g] = s.g_parent[g];
        if (out->group_t_submit) out->group_t_submit[g] = s.g_submit[g];
        if (out->group_t_group) out->group_t_group[g] = s.g_done[g];
        if (out->group_t_train) out->group_t_train[g] = t_train;
        if (out->group_adv) {
            int k = 0;
            for (int m = 0; m < G; ++m) k += s.reward[g * G + m];
            const double mean = (double)k / (double)G;
            const double sd = std::sqrt((double)((int64_t)k * (G - k)) / (double)((int64_t)G * G));
            for (int m = 0; m < G; ++m) out->group_adv[g * G + m] = ((double)s.reward[g * G + m] - mean) / (sd + cfg->adv_eps);
        }
    }
    summary->sum_t_train = sum_train;
    summary->sum_wait = sum_wait;
    if (out) {
        for (int64_t i = 0; i < ni; ++i) {
            if (out->item_problem) out->item_problem[i] = s.problem[i];
            if (out->item_role) out->item_role[i] = s.role[i];
            if (out->item_group) out->item_group[i] = s.group[i];
            if (out->item_member) out->item_member[i] = s.member[i];
            if (out->item_parent) out->item_parent[i] = s.parent[i];
            if (out->item_length) out->item_length[i] = s.length[i];
            if (out->item_value) out->item_value[i] = s.value[i];
            if (out->item_reward) out->item_reward[i] = s.reward[i];
            if (out->item_t_done) out->item_t_done[i] = s.t_done[i];
        }
    }
    return 0;
}

}  // extern "C"
