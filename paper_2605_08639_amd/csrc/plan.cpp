// relibra_plan: host-side load-balancing solver (paper Sections 4 and 5.2).
//
// Stage 1 (per training batch) reorders experts across ranks: greedy LPT as the starting
// state, then steepest descent over the pair-swap neighbourhood of Algorithm 1 with O(1)
// incremental evaluation of a swap (Section 4.2, "incremental state update").
// Stage 2 (per micro-batch, per node) is Algorithm 2: replicate the heaviest expert of the
// bottleneck rank onto the least-loaded rank of the node that can take it, then re-solve the
// token split; repeated until no slot helps.  One worker thread per micro-batch (Section 6).
//
// All arithmetic is integer; every choice has a fixed tie-break, so the plan is a pure
// function of the histograms.
#include "../../include/relibra.h"

#include <algorithm>
#include <cstdint>
#include <cstring>
#include <iterator>
#include <numeric>
#include <thread>
#include <vector>

namespace {

using i64 = long long;
using u128 = unsigned __int128;

struct Cost {
    i64 peak;
    u128 sq;
    bool operator<(const Cost &o) const { return peak < o.peak || (peak == o.peak && sq < o.sq); }
};

// ---------------------------------------------------------------- stage 1
std::vector<int> lpt_start(const std::vector<i64> &load_of, int EP)
{
    const int E = (int)load_of.size(), M = E / EP;
    std::vector<int> by_load(E);
    std::iota(by_load.begin(), by_load.end(), 0);
    std::stable_sort(by_load.begin(), by_load.end(),
                     [&](int a, int b) { return load_of[a] > load_of[b]; });
    std::vector<i64> L(EP, 0);
    std::vector<int> room(EP, M), where(E, 0);
    for (int e : by_load) {
        int pick = -1;
        for (int g = 0; g < EP; ++g)
            if (room[g] > 0 && (pick < 0 || L[g] < L[pick])) pick = g;
        where[e] = pick;
        L[pick] += load_of[e];
        --room[pick];
    }
    return where;
}

// Three largest rank loads with their ranks, so that "max over the ranks a swap does not
// touch" is a constant-time lookup.
struct Top3 {
    i64 v[3];
    int g[3];
    void build(const std::vector<i64> &L)
    {
        for (int i = 0; i < 3; ++i) { v[i] = -1; g[i] = -1; }
        for (int x = 0; x < (int)L.size(); ++x) {
            i64 val = L[x];
            int idx = x;
            for (int i = 0; i < 3; ++i)
                if (val > v[i]) { std::swap(val, v[i]); std::swap(idx, g[i]); }
        }
    }
    i64 max_excluding(int a, int b) const
    {
        for (int i = 0; i < 3; ++i)
            if (g[i] != a && g[i] != b) return v[i] < 0 ? 0 : v[i];
        return 0;
    }
};

Cost cost_of(const std::vector<i64> &L)
{
    Cost c{0, 0};
    for (i64 x : L) { c.peak = std::max(c.peak, x); c.sq += (u128)x * (u128)x; }
    return c;
}

// Steepest descent over pair swaps: in every step the swap with the smallest resulting
// (peak, sum of squares), ties to the smallest (a, b), applied while it lowers the cost.
// A swap of a (rank p) and b (rank q) moves d = l_b - l_a tokens from q to p: the sum of squares
// changes by 2 d (L_p - L_q + d), so candidates are compared by (new peak, that change).  Over
// all integer d the change is at least -floor((L_p - L_q)^2 / 4): a pair of ranks that cannot
// lower the peak and whose bound cannot reach the best change found so far is skipped whole,
// which leaves a handful of rank pairs to enumerate once the loads are nearly level.
// D = the integer type of the change: 64 bits when the loads are small enough, else 128.
template <class D>
Cost swap_descent_t(const std::vector<i64> &load_of, int EP, std::vector<int> &where)
{
    const int E = (int)load_of.size();
    std::vector<i64> L(EP, 0);
    for (int e = 0; e < E; ++e) L[where[e]] += load_of[e];
    std::vector<std::vector<int>> on(EP);
    for (int e = 0; e < E; ++e) on[where[e]].push_back(e);
    struct RankPair { int p, q; i64 gap; };
    std::vector<RankPair> pairs;
    Top3 top;
    for (;;) {
        const Cost cur = cost_of(L);
        top.build(L);
        pairs.clear();
        for (int p = 0; p < EP; ++p)
            for (int q = p + 1; q < EP; ++q) pairs.push_back({p, q, L[p] > L[q] ? L[p] - L[q] : L[q] - L[p]});
        std::stable_sort(pairs.begin(), pairs.end(), [](const RankPair &x, const RankPair &y) { return x.gap > y.gap; });
        bool have = false;
        i64 best_peak = 0;
        D best_delta = 0;
        int pa = -1, pb = -1;
        for (const RankPair &rp : pairs) {
            const bool touches_peak = L[rp.p] == cur.peak || L[rp.q] == cur.peak;
            if (have && !touches_peak) {
                if (best_peak < cur.peak) continue;                          // cannot lower the peak, the best one does
                const D bound = -((D)(rp.gap / 2) * (D)(rp.gap - rp.gap / 2));
                if (bound > best_delta) continue;                            // cannot reach the best change
            }
            const i64 rest = top.max_excluding(rp.p, rp.q);
            for (int x : on[rp.p])
                for (int y : on[rp.q]) {
                    const int a = x < y ? x : y, b = x < y ? y : x;
                    const int ga = x < y ? rp.p : rp.q, gb = x < y ? rp.q : rp.p;
                    const i64 d = load_of[b] - load_of[a];                  // rank ga gains d, rank gb loses d
                    const i64 peak = std::max(std::max(L[ga] + d, L[gb] - d), rest);
                    if (have && peak > best_peak) continue;
                    const D delta = (D)d * (D)(L[ga] - L[gb] + d);           // half the change of the sum of squares
                    const bool better = !have || peak < best_peak || delta < best_delta ||
                                        (delta == best_delta && (a < pa || (a == pa && b < pb)));
                    if (better) { have = true; best_peak = peak; best_delta = delta; pa = a; pb = b; }
                }
        }
        if (!have || !(best_peak < cur.peak || (best_peak == cur.peak && best_delta < 0))) return cur;
        const int ga = where[pa], gb = where[pb];
        const i64 d = load_of[pb] - load_of[pa];
        L[ga] += d;
        L[gb] -= d;
        where[pa] = gb;
        where[pb] = ga;
        std::replace(on[ga].begin(), on[ga].end(), pa, pb);
        std::replace(on[gb].begin(), on[gb].end(), pb, pa);
    }
}

Cost swap_descent(const std::vector<i64> &load_of, int EP, std::vector<int> &where)
{
    i64 total = 0;
    for (i64 x : load_of) total += x;
    if (total < ((i64)1 << 30)) return swap_descent_t<i64>(load_of, EP, where);
    return swap_descent_t<__int128>(load_of, EP, where);
}

// ---------------------------------------------------------------- stage 2
// One node: n ranks, experts listed in ascending global id.
struct Node {
    int n = 0, r = 0;
    std::vector<i64> cnt;                  // tokens of each expert in this micro-batch
    std::vector<int> home;                 // local home rank
    std::vector<uint32_t> allowed;         // bit g set: expert may be served on local rank g
    std::vector<std::vector<i64>> share;   // share[e][g]: tokens of e served on g
    std::vector<i64> L;                    // rank loads

    void recompute_loads()
    {
        std::fill(L.begin(), L.end(), 0);
        for (size_t e = 0; e < cnt.size(); ++e)
            for (int g = 0; g < n; ++g) L[g] += share[e][g];
    }

    // Token split for the current placement: move tokens along chains of ranks from a
    // heavier rank to a lighter one while some chain joins two ranks whose loads differ by
    // two or more.  The end state minimises the largest load (it is an optimum of the
    // split LP of Section 5.2) and the sum of squares.  Order of moves: source = ranks by
    // descending load, lower id first; breadth-first chains, neighbours in ascending rank,
    // lowest expert id per hop; sink = lightest reached rank, lower id first.
    void balance()
    {
        const int ne = (int)cnt.size();
        std::vector<int> by_load(n), parent(n), via(n), bfs;
        bfs.reserve(n);
        for (;;) {
            recompute_loads();
            std::iota(by_load.begin(), by_load.end(), 0);
            std::stable_sort(by_load.begin(), by_load.end(), [&](int a, int b) { return L[a] > L[b]; });
            bool moved = false;
            for (int u : by_load) {
                uint32_t seen = 1u << u;
                parent[u] = -1;
                bfs.clear();
                bfs.push_back(u);
                for (size_t head = 0; head < bfs.size(); ++head) {
                    const int w = bfs[head];
                    uint32_t fresh = 0;
                    for (int e = 0; e < ne; ++e) {        // ascending id: first hit = lowest expert
                        if (share[e][w] <= 0) continue;
                        uint32_t reach = allowed[e] & ~seen;
                        while (reach) {
                            const int v = __builtin_ctz(reach);
                            reach &= reach - 1;
                            seen |= 1u << v;
                            fresh |= 1u << v;
                            parent[v] = w;
                            via[v] = e;
                        }
                    }
                    while (fresh) {                        // neighbours join the queue in ascending rank
                        bfs.push_back(__builtin_ctz(fresh));
                        fresh &= fresh - 1;
                    }
                }
                int sink = -1;
                for (int g = 0; g < n; ++g)
                    if (g != u && (seen >> g & 1) && (sink < 0 || L[g] < L[sink])) sink = g;
                if (sink < 0 || L[sink] + 2 > L[u]) continue;
                i64 d = (L[u] - L[sink]) / 2;
                for (int x = sink; parent[x] >= 0; x = parent[x]) d = std::min(d, share[via[x]][parent[x]]);
                for (int x = sink; parent[x] >= 0; x = parent[x]) {
                    share[via[x]][parent[x]] -= d;
                    share[via[x]][x] += d;
                }
                moved = true;
                break;
            }
            if (!moved) return;
        }
    }

    i64 solve()
    {
        const int ne = (int)cnt.size();
        share.assign(ne, std::vector<i64>(n, 0));
        allowed.assign(ne, 0);
        L.assign(n, 0);
        i64 total = 0;
        for (int e = 0; e < ne; ++e) {
            allowed[e] = 1u << home[e];
            share[e][home[e]] = cnt[e];
            total += cnt[e];
        }
        const i64 floor_load = (total + n - 1) / n;
        std::vector<int> slots_used(n, 0);
        std::vector<int> cand;
        for (;;) {
            recompute_loads();
            const int gb = (int)(std::max_element(L.begin(), L.end()) - L.begin());   // first max
            if (L[gb] <= floor_load) break;
            cand.clear();
            for (int e = 0; e < ne; ++e)
                if (share[e][gb] > 0) cand.push_back(e);
            std::stable_sort(cand.begin(), cand.end(),
                             [&](int a, int b) { return share[a][gb] > share[b][gb]; });
            int e_pick = -1, g_pick = -1;
            for (int e : cand) {
                for (int g = 0; g < n; ++g) {
                    if ((allowed[e] >> g & 1) || slots_used[g] >= r) continue;
                    if (g_pick < 0 || L[g] < L[g_pick]) g_pick = g;
                }
                if (g_pick >= 0) { e_pick = e; break; }
            }
            if (e_pick < 0) break;
            allowed[e_pick] |= 1u << g_pick;
            ++slots_used[g_pick];
            balance();
        }
        for (int e = 0; e < ne; ++e)                       // drop replicas that got no tokens
            for (int g = 0; g < n; ++g)
                if (g != home[e] && (allowed[e] >> g & 1) && share[e][g] == 0) allowed[e] &= ~(1u << g);
        recompute_loads();
        return *std::max_element(L.begin(), L.end());
    }
};

// Result of stage 2 for one micro-batch under a given placement.
struct MbPlan {
    i64 peak = 0;
    std::vector<std::vector<std::pair<int, i64>>> inst;   // per expert: (rank, rows), ascending rank
};

MbPlan replicate_microbatch(const int32_t *cnt, const std::vector<int> &where, int E, int EP, int rpn, int r)
{
    MbPlan out;
    out.inst.resize(E);
    for (int base = 0; base < EP; base += rpn) {
        Node nd;
        nd.n = rpn;
        nd.r = r;
        std::vector<int> members;
        for (int e = 0; e < E; ++e)
            if (where[e] >= base && where[e] < base + rpn) {
                members.push_back(e);
                nd.cnt.push_back(cnt[e]);
                nd.home.push_back(where[e] - base);
            }
        out.peak = std::max(out.peak, nd.solve());
        for (size_t i = 0; i < members.size(); ++i)
            for (int g = 0; g < rpn; ++g)
                if (nd.allowed[i] >> g & 1) out.inst[members[i]].push_back({base + g, nd.share[i][g]});
    }
    return out;
}

std::vector<MbPlan> replicate_batch(const int32_t *counts, int n_mb, const std::vector<int> &where,
                                    int E, int EP, int rpn, int r)
{
    std::vector<MbPlan> plans(n_mb);
    unsigned hw = std::thread::hardware_concurrency();
    int workers = (int)std::min<unsigned>(hw ? hw : 1u, (unsigned)n_mb);
    workers = std::min(workers, 16);
    if (workers <= 1) {
        for (int mb = 0; mb < n_mb; ++mb)
            plans[mb] = replicate_microbatch(counts + (size_t)mb * E, where, E, EP, rpn, r);
        return plans;
    }
    std::vector<std::thread> pool;
    for (int w = 0; w < workers; ++w)
        pool.emplace_back([&, w]() {
            for (int mb = w; mb < n_mb; mb += workers)
                plans[mb] = replicate_microbatch(counts + (size_t)mb * E, where, E, EP, rpn, r);
        });
    for (auto &t : pool) t.join();
    return plans;
}

// Stage 2 with the execution time of Section 4.1 as objective (Algorithm 2 as printed: bottleneck
// and target GPU by T_MoE,g = T_g^comp + T_g^comm), one micro-batch, all nodes at once.  A state's
// time: every expert's instances take their sources by relibra_assign_sources, loads and times
// follow Eq. 1-6 (relibra_moe_time_split).  A replica is kept if (T_MoE, sum_g T_g^2) gets
// lexicographically smaller; the candidates are the bottleneck GPU's experts, most tokens first.
struct TimedState {
    const int64_t *x;
    const relibra_cost_model *model;
    int E, EP, rpn;
    const std::vector<int> &where;
    std::vector<Node> &nodes;
    std::vector<int> local;                 // index of expert e inside its node
    std::vector<int32_t> ptr, rank, rows, first, y, ybase;
    std::vector<int64_t> loads;

    TimedState(const int64_t *x_, const relibra_cost_model *m, int E_, const std::vector<int> &w, std::vector<Node> &n)
        : x(x_), model(m), E(E_), EP(m->EP), rpn(m->ranks_per_node), where(w), nodes(n), local(E_), ptr(E_ + 1),
          first((size_t)m->EP * E_), loads(5 * (size_t)m->EP)
    {
    }

    // T_MoE of the current state; per[g] = T_g
    double time(std::vector<double> &per)
    {
        rank.clear();
        rows.clear();
        for (int e = 0; e < E; ++e) {
            ptr[e] = (int32_t)rank.size();
            const Node &nd = nodes[where[e] / rpn];
            const int base = where[e] / rpn * rpn, i = local[e];
            for (int g = 0; g < rpn; ++g)
                if (nd.allowed[i] >> g & 1) {
                    rank.push_back(base + g);
                    rows.push_back((int32_t)nd.share[i][g]);
                }
        }
        ptr[E] = (int32_t)rank.size();
        const size_t cells = rank.size() * (size_t)EP;
        y.resize(cells);
        ybase.resize(cells);
        double out3[3] = {0, 0, 0};
        relibra_assign_sources(x, E, EP, rpn, ptr.data(), rank.data(), rows.data(), first.data(), y.data(), ybase.data());
        relibra_moe_time_split(y.data(), (int)rank.size(), rank.data(), model, out3, loads.data());
        const int64_t *comp = loads.data(), *itx = comp + EP, *irx = comp + 2 * EP, *rtx = comp + 3 * EP, *rrx = comp + 4 * EP;
        for (int g = 0; g < EP; ++g) {
            const double intra = model->sec_per_token_intra * (double)std::max(itx[g], irx[g]);
            const double rdma = model->sec_per_token_inter * (double)std::max(rtx[g], rrx[g]);
            per[g] = model->sec_per_token_comp * (double)comp[g] + std::max(intra, rdma);
        }
        return out3[0];
    }
};

MbPlan replicate_microbatch_timed(const int64_t *x, const relibra_cost_model *model, const std::vector<int> &where,
                                  int E, int r, double &t_before, double &t_after)
{
    const int EP = model->EP, rpn = model->ranks_per_node;
    std::vector<Node> nodes(EP / rpn);
    std::vector<std::vector<int>> members(EP / rpn);
    TimedState st(x, model, E, where, nodes);
    for (int e = 0; e < E; ++e) {
        Node &nd = nodes[where[e] / rpn];
        i64 tokens = 0;
        for (int j = 0; j < EP; ++j) tokens += x[(size_t)j * E + e];
        st.local[e] = (int)nd.cnt.size();
        members[where[e] / rpn].push_back(e);
        nd.cnt.push_back(tokens);
        nd.home.push_back(where[e] % rpn);
    }
    for (Node &nd : nodes) {
        nd.n = rpn;
        nd.r = r;
        const int ne = (int)nd.cnt.size();
        nd.share.assign(ne, std::vector<i64>(rpn, 0));
        nd.allowed.assign(ne, 0);
        nd.L.assign(rpn, 0);
        for (int i = 0; i < ne; ++i) {
            nd.allowed[i] = 1u << nd.home[i];
            nd.share[i][nd.home[i]] = nd.cnt[i];
        }
    }
    auto squares = [](const std::vector<double> &v) {
        double s = 0;
        for (double t : v) s += t * t;
        return s;
    };
    std::vector<double> per(EP), per_try(EP);
    std::vector<int> slots_used(EP, 0), cand;
    double T = st.time(per), S = squares(per);
    t_before = T;
    for (;;) {
        const int gb = (int)(std::max_element(per.begin(), per.end()) - per.begin());      // first maximum
        Node &nd = nodes[gb / rpn];
        const int base = gb / rpn * rpn, lb = gb - base, ne = (int)nd.cnt.size();
        cand.clear();
        for (int i = 0; i < ne; ++i)
            if (nd.share[i][lb] > 0) cand.push_back(i);
        std::stable_sort(cand.begin(), cand.end(), [&](int a, int b) { return nd.share[a][lb] > nd.share[b][lb]; });
        bool kept = false;
        for (int i : cand) {
            int gt = -1;
            for (int g = 0; g < rpn; ++g) {
                if ((nd.allowed[i] >> g & 1) || slots_used[base + g] >= r) continue;
                if (gt < 0 || per[base + g] < per[base + gt]) gt = g;
            }
            if (gt < 0) continue;
            const std::vector<std::vector<i64>> share_before = nd.share;
            nd.allowed[i] |= 1u << gt;
            nd.balance();
            const double T_try = st.time(per_try), S_try = squares(per_try);
            if (T_try < T || (T_try == T && S_try < S)) {
                T = T_try;
                S = S_try;
                per.swap(per_try);
                ++slots_used[base + gt];
                kept = true;
                break;
            }
            nd.allowed[i] &= ~(1u << gt);
            nd.share = share_before;
        }
        if (!kept) break;
    }
    MbPlan out;
    out.inst.resize(E);
    for (size_t n = 0; n < nodes.size(); ++n) {
        Node &nd = nodes[n];
        for (size_t i = 0; i < members[n].size(); ++i)
            for (int g = 0; g < rpn; ++g) {
                if (g != nd.home[i] && (nd.allowed[i] >> g & 1) && nd.share[i][g] == 0) nd.allowed[i] &= ~(1u << g);
                if (nd.allowed[i] >> g & 1) out.inst[members[n][i]].push_back({(int)n * rpn + g, nd.share[i][g]});
            }
        nd.recompute_loads();
        out.peak = std::max(out.peak, *std::max_element(nd.L.begin(), nd.L.end()));
    }
    t_after = st.time(per);
    return out;
}

}  // namespace

static void write_tables(const int32_t *counts, int n_mb, int E, int EP, int r, const std::vector<int> &where,
                         const std::vector<MbPlan> &plans,
                         int32_t *expert_to_slot, int32_t *replica_expert,
                         int32_t *inst_ptr, int32_t *inst_rank, int32_t *inst_rows, int32_t *inst_group,
                         int32_t *group_expert, int32_t *group_offset, int32_t *group_dw_slot,
                         int64_t *max_load_before, int64_t *max_load_after);

// Both entry points.  placed = nullptr: stage 1 chooses the placement; otherwise the caller's
// placement (rank per expert, exactly M per rank) is taken as it is and only stage 2 runs.
static int plan_impl(const int32_t *counts, int n_mb, int E, int k, int EP, int rpn, int r, const int32_t *placed,
                     int32_t *expert_to_slot, int32_t *replica_expert,
                     int32_t *inst_ptr, int32_t *inst_rank, int32_t *inst_rows, int32_t *inst_group,
                     int32_t *group_expert, int32_t *group_offset, int32_t *group_dw_slot,
                     int64_t *max_load_before, int64_t *max_load_after)
{
    if (!counts || !expert_to_slot || !inst_ptr || !inst_rank || !inst_rows || !inst_group ||
        !group_expert || !group_offset || !group_dw_slot || !max_load_before || !max_load_after)
        return RELIBRA_EINVAL;
    if (n_mb < 1 || E < 1 || EP < 1 || E % EP || rpn < 1 || rpn > 32 || EP % rpn || r < 0 || k < 1 || k > E)
        return RELIBRA_EINVAL;
    if (r > 0 && !replica_expert) return RELIBRA_EINVAL;
    const int M = E / EP;

    std::vector<i64> batch_load(E, 0);
    for (int mb = 0; mb < n_mb; ++mb)
        for (int e = 0; e < E; ++e) {
            const int32_t c = counts[(size_t)mb * E + e];
            if (c < 0) return RELIBRA_ERANGE;
            batch_load[e] += c;
        }

    std::vector<int> unplanned(E);
    for (int e = 0; e < E; ++e) unplanned[e] = e / M;
    std::vector<int> chosen;
    std::vector<MbPlan> chosen_plans;
    if (placed) {
        std::vector<int> held(EP, 0);
        chosen.resize(E);
        for (int e = 0; e < E; ++e) {
            if (placed[e] < 0 || placed[e] >= EP || ++held[placed[e]] > M) return RELIBRA_ERANGE;
            chosen[e] = placed[e];
        }
        chosen_plans = replicate_batch(counts, n_mb, chosen, E, EP, rpn, r);
    } else {
        // stage 1: descent from the unplanned layout and from LPT; ties keep the unplanned one
        std::vector<int> from_id = unplanned, from_lpt = lpt_start(batch_load, EP);
        Cost c_id{0, 0};
        std::thread other([&]() { c_id = swap_descent(batch_load, EP, from_id); });     // the two starts are independent
        const Cost c_lpt = swap_descent(batch_load, EP, from_lpt);
        other.join();
        const std::vector<int> &reordered = (c_lpt < c_id) ? from_lpt : from_id;
        // stage 2 under both placements; the reordering must pay for itself over the batch
        chosen = unplanned;
        chosen_plans = replicate_batch(counts, n_mb, unplanned, E, EP, rpn, r);
        if (reordered != unplanned) {
            std::vector<MbPlan> with_new = replicate_batch(counts, n_mb, reordered, E, EP, rpn, r);
            i64 j_id = 0, j_new = 0;
            for (int mb = 0; mb < n_mb; ++mb) { j_id += chosen_plans[mb].peak; j_new += with_new[mb].peak; }
            if (j_new < j_id) {
                chosen = reordered;
                chosen_plans.swap(with_new);
            }
        }
    }
    write_tables(counts, n_mb, E, EP, r, chosen, chosen_plans, expert_to_slot, replica_expert, inst_ptr, inst_rank, inst_rows,
                 inst_group, group_expert, group_offset, group_dw_slot, max_load_before, max_load_after);
    return RELIBRA_OK;
}

// The plan tables of a placement and its per-micro-batch replication (layout: relibra_plan).
static void write_tables(const int32_t *counts, int n_mb, int E, int EP, int r, const std::vector<int> &where,
                         const std::vector<MbPlan> &plans,
                         int32_t *expert_to_slot, int32_t *replica_expert,
                         int32_t *inst_ptr, int32_t *inst_rank, int32_t *inst_rows, int32_t *inst_group,
                         int32_t *group_expert, int32_t *group_offset, int32_t *group_dw_slot,
                         int64_t *max_load_before, int64_t *max_load_after)
{
    const int M = E / EP, S = M + r, G = EP * S, inst_cap = E + EP * r;
    std::vector<int> filled(EP, 0);
    for (int e = 0; e < E; ++e) expert_to_slot[e] = where[e] * M + filled[where[e]]++;

    for (int mb = 0; mb < n_mb; ++mb) {
        const MbPlan &P = plans[mb];
        int32_t *gexp = group_expert + (size_t)mb * G;
        int32_t *goff = group_offset + (size_t)mb * (G + 1);
        int32_t *gslot = group_dw_slot + (size_t)mb * G;
        int32_t *rep = r ? replica_expert + (size_t)mb * EP * r : nullptr;
        int32_t *iptr = inst_ptr + (size_t)mb * (E + 1);
        int32_t *irank = inst_rank + (size_t)mb * inst_cap;
        int32_t *irows = inst_rows + (size_t)mb * inst_cap;
        int32_t *igrp = inst_group + (size_t)mb * inst_cap;
        std::vector<i64> rows(G, 0);
        std::fill(gexp, gexp + G, -1);
        for (int g = 0; g < G; ++g) gslot[g] = (g % S < M) ? -1 : E + (g / S) * r + (g % S - M);
        if (rep) std::fill(rep, rep + (size_t)EP * r, -1);
        std::fill(irank, irank + inst_cap, -1);
        std::fill(irows, irows + inst_cap, 0);
        std::fill(igrp, igrp + inst_cap, -1);
        std::vector<int> next_rep(EP, 0);
        int p = 0;
        for (int e = 0; e < E; ++e) {                      // ascending e fills replica slots in id order
            iptr[e] = p;
            for (const auto &ir : P.inst[e]) {
                const int rk = ir.first;
                int grp;
                if (rk == where[e]) {
                    grp = rk * S + expert_to_slot[e] % M;
                    gslot[grp] = e;
                } else {
                    const int j = next_rep[rk]++;
                    grp = rk * S + M + j;
                    rep[rk * r + j] = e;
                }
                gexp[grp] = e;
                rows[grp] = ir.second;
                irank[p] = rk;
                irows[p] = (int32_t)ir.second;
                igrp[p] = grp;
                ++p;
            }
        }
        iptr[E] = p;
        goff[0] = 0;
        for (int g = 0; g < G; ++g) goff[g + 1] = goff[g] + (int32_t)rows[g];
        i64 worst = 0;
        for (int g = 0; g < EP; ++g) {
            i64 s = 0;
            for (int e = g * M; e < (g + 1) * M; ++e) s += counts[(size_t)mb * E + e];
            worst = std::max(worst, s);
        }
        max_load_before[mb] = worst;
        max_load_after[mb] = P.peak;
    }
}

extern "C" int relibra_plan(const int32_t *counts, int n_mb, int E, int k, int EP, int rpn, int r,
                            int32_t *expert_to_slot, int32_t *replica_expert,
                            int32_t *inst_ptr, int32_t *inst_rank, int32_t *inst_rows, int32_t *inst_group,
                            int32_t *group_expert, int32_t *group_offset, int32_t *group_dw_slot,
                            int64_t *max_load_before, int64_t *max_load_after)
{
    return plan_impl(counts, n_mb, E, k, EP, rpn, r, nullptr, expert_to_slot, replica_expert, inst_ptr, inst_rank,
                     inst_rows, inst_group, group_expert, group_offset, group_dw_slot, max_load_before, max_load_after);
}

extern "C" int relibra_plan_placed(const int32_t *counts, int n_mb, int E, int k, int EP, int rpn, int r,
                                   const int32_t *expert_rank,
                                   int32_t *expert_to_slot, int32_t *replica_expert,
                                   int32_t *inst_ptr, int32_t *inst_rank, int32_t *inst_rows, int32_t *inst_group,
                                   int32_t *group_expert, int32_t *group_offset, int32_t *group_dw_slot,
                                   int64_t *max_load_before, int64_t *max_load_after)
{
    if (!expert_rank) return RELIBRA_EINVAL;
    return plan_impl(counts, n_mb, E, k, EP, rpn, r, expert_rank, expert_to_slot, replica_expert, inst_ptr, inst_rank,
                     inst_rows, inst_group, group_expert, group_offset, group_dw_slot, max_load_before, max_load_after);
}

extern "C" int relibra_plan_timed(const int64_t *x_host, int n_mb, int E, int k, const relibra_cost_model *model, int r,
                                  const int32_t *expert_rank,
                                  int32_t *expert_to_slot, int32_t *replica_expert,
                                  int32_t *inst_ptr, int32_t *inst_rank, int32_t *inst_rows, int32_t *inst_group,
                                  int32_t *group_expert, int32_t *group_offset, int32_t *group_dw_slot,
                                  int64_t *max_load_before, int64_t *max_load_after, double *t_before, double *t_after)
{
    if (!x_host || !model || !expert_rank || !expert_to_slot || !inst_ptr || !inst_rank || !inst_rows || !inst_group ||
        !group_expert || !group_offset || !group_dw_slot || !max_load_before || !max_load_after || !t_before || !t_after)
        return RELIBRA_EINVAL;
    const int EP = model->EP, rpn = model->ranks_per_node;
    if (n_mb < 1 || E < 1 || EP < 1 || E % EP || rpn < 1 || rpn > 32 || EP % rpn || r < 0 || k < 1 || k > E)
        return RELIBRA_EINVAL;
    if (model->sec_per_token_comp < 0 || model->sec_per_token_intra < 0 || model->sec_per_token_inter < 0) return RELIBRA_EINVAL;
    if (r > 0 && !replica_expert) return RELIBRA_EINVAL;
    const int M = E / EP;
    std::vector<int> where(E), held(EP, 0);
    for (int e = 0; e < E; ++e) {
        if (expert_rank[e] < 0 || expert_rank[e] >= EP || ++held[expert_rank[e]] > M) return RELIBRA_ERANGE;
        where[e] = expert_rank[e];
    }
    std::vector<int32_t> counts((size_t)n_mb * E);
    for (int mb = 0; mb < n_mb; ++mb)
        for (int e = 0; e < E; ++e) {
            i64 tokens = 0;
            for (int j = 0; j < EP; ++j) {
                const int64_t v = x_host[((size_t)mb * EP + j) * E + e];
                if (v < 0 || v > 0x7fffffffLL) return RELIBRA_ERANGE;
                tokens += v;
            }
            if (tokens > 0x7fffffffLL) return RELIBRA_ERANGE;
            counts[(size_t)mb * E + e] = (int32_t)tokens;
        }
    std::vector<MbPlan> plans(n_mb);
    {
        unsigned hw = std::thread::hardware_concurrency();
        const int workers = std::max(1, std::min({(int)(hw ? hw : 1u), n_mb, 16}));
        std::vector<std::thread> pool;
        for (int w = 0; w < workers; ++w)
            pool.emplace_back([&, w]() {
                for (int mb = w; mb < n_mb; mb += workers)
                    plans[mb] = replicate_microbatch_timed(x_host + (size_t)mb * EP * E, model, where, E, r, t_before[mb], t_after[mb]);
            });
        for (auto &t : pool) t.join();
    }
    write_tables(counts.data(), n_mb, E, EP, r, where, plans, expert_to_slot, replica_expert, inst_ptr, inst_rank, inst_rows,
                 inst_group, group_expert, group_offset, group_dw_slot, max_load_before, max_load_after);
    return RELIBRA_OK;
}

// Imbalance diagnostics of Section 2.2.
extern "C" int relibra_load_stats(const int32_t *counts, int n_mb, int E, int top,
                                  double *skewness, double *intersection)
{
    if (!counts || !skewness || n_mb < 1 || E < 1 || top < 1 || top > E) return RELIBRA_EINVAL;
    if (n_mb > 1 && !intersection) return RELIBRA_EINVAL;
    std::vector<std::vector<int>> hot(n_mb);
    for (int mb = 0; mb < n_mb; ++mb) {
        const int32_t *c = counts + (size_t)mb * E;
        i64 sum = 0, peak = 0;
        for (int e = 0; e < E; ++e) {
            if (c[e] < 0) return RELIBRA_ERANGE;
            sum += c[e];
            peak = std::max<i64>(peak, c[e]);
        }
        skewness[mb] = sum > 0 ? (double)peak * E / (double)sum : 1.0;
        std::vector<int> order(E);
        std::iota(order.begin(), order.end(), 0);
        std::stable_sort(order.begin(), order.end(), [&](int a, int b) { return c[a] > c[b]; });   // ties: lower id
        hot[mb].assign(order.begin(), order.begin() + top);
        std::sort(hot[mb].begin(), hot[mb].end());
    }
    for (int mb = 0; mb + 1 < n_mb; ++mb) {
        std::vector<int> both;
        std::set_intersection(hot[mb].begin(), hot[mb].end(), hot[mb + 1].begin(), hot[mb + 1].end(), std::back_inserter(both));
        intersection[mb] = (double)both.size() / top;
    }
    return RELIBRA_OK;
}
