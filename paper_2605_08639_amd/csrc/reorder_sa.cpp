// Communication-aware cost model of the MoE module (paper Section 4.1, Eq. 1-6) and the
// swap-based simulated annealing of Algorithm 1 (Section 4.2), host side.
//
// Loads are integers (tokens): computation load per rank, intra-node-link and RDMA send /
// receive loads per rank, derived from the per-source routing histogram x[j][e] and the
// source-destination type of (source rank, rank hosting the expert) on a rail-optimised
// cluster.  A swap of two experts touches the two hosting ranks' receive side and every
// source's send side: the state update is O(|G|) (Section 4.2, "incremental state update");
// the smoothed objective (log-sum-exp in place of every max) is then re-evaluated from the
// O(|G|) loads.  One thread per seed (Section 6).
//
// Readings: the acceptance test is the Metropolis rule exp(-(T' - T)/theta) (the printed
// exponent has the opposite sign and would accept every worsening move); times are divided by
// the starting state's exact T_MoE before smoothing so that beta = 20 acts on numbers of order
// one; the random draws come from splitmix64, three per iteration (e_a, e_b, u).
#include "../../include/relibra.h"

#include <algorithm>
#include <cmath>
#include <cstdint>
#include <numeric>
#include <thread>
#include <vector>

namespace {

using i64 = long long;

enum { LOC = 0, NV = 1, SR = 2, CR = 3 };

inline int link_type(int src, int dst, int rpn)
{
    if (src == dst) return LOC;
    if (src / rpn == dst / rpn) return NV;
    return (src % rpn == dst % rpn) ? SR : CR;
}

struct Loads {
    int EP = 0;
    std::vector<i64> comp, nv_tx, nv_rx, rd_tx, rd_rx;
    explicit Loads(int ep) : EP(ep), comp(ep, 0), nv_tx(ep, 0), nv_rx(ep, 0), rd_tx(ep, 0), rd_rx(ep, 0) {}
};

struct Problem {
    const int64_t *x;       // [EP][E]
    int E, EP, rpn;
    double per_comp, per_intra, per_inter;   // seconds per token
    double beta, t_ref;

    // expert e served on rank g: add (sign = +1) or remove (-1) its tokens from every load
    void place(Loads &L, int e, int g, i64 sign) const
    {
        for (int j = 0; j < EP; ++j) {
            const i64 n = sign * (i64)x[(size_t)j * E + e];
            if (n == 0) continue;
            L.comp[g] += n;
            switch (link_type(j, g, rpn)) {
            case NV: L.nv_tx[j] += n; L.nv_rx[g] += n; break;
            case SR: L.rd_tx[j] += n; L.rd_rx[g] += n; break;
            case CR: L.nv_tx[j] += n; L.nv_rx[g] += n; L.rd_tx[j] += n; L.rd_rx[g] += n; break;
            default: break;
            }
        }
    }

    Loads loads_of(const std::vector<int> &rank_of) const
    {
        Loads L(EP);
        for (int e = 0; e < E; ++e) place(L, e, rank_of[e], +1);
        return L;
    }

    static double soft_max(const double *z, int n, double beta)
    {
        double top = z[0];
        for (int i = 1; i < n; ++i) top = std::max(top, z[i]);
        double sum = 0.0;
        for (int i = 0; i < n; ++i) sum += std::exp(beta * (z[i] - top));
        return top + std::log(sum) / beta;
    }

    // exact: T_MoE = max comp time + max comm time (Eq. 6); out3 = {T, max comp, max comm}
    void exact(const Loads &L, double *out3) const
    {
        double mc = 0.0, mm = 0.0;
        for (int g = 0; g < EP; ++g) {
            mc = std::max(mc, (double)L.comp[g] * per_comp);
            const double link = std::max((double)L.nv_tx[g] * per_intra, (double)L.nv_rx[g] * per_intra);
            const double rdma = std::max((double)L.rd_tx[g] * per_inter, (double)L.rd_rx[g] * per_inter);
            mm = std::max(mm, std::max(link, rdma));
        }
        out3[0] = mc + mm;
        out3[1] = mc;
        out3[2] = mm;
    }

    // smoothed objective on times / t_ref, inner max of Eq. 5 smoothed as well
    double smooth(const Loads &L, std::vector<double> &zc, std::vector<double> &zm) const
    {
        for (int g = 0; g < EP; ++g) {
            zc[g] = ((double)L.comp[g] * per_comp) / t_ref;
            const double four[4] = {((double)L.nv_tx[g] * per_intra) / t_ref, ((double)L.nv_rx[g] * per_intra) / t_ref,
                                    ((double)L.rd_tx[g] * per_inter) / t_ref, ((double)L.rd_rx[g] * per_inter) / t_ref};
            zm[g] = soft_max(four, 4, beta);
        }
        return soft_max(zc.data(), EP, beta) + soft_max(zm.data(), EP, beta);
    }
};

// greedy LPT with M experts per rank (Section 4.2): heaviest first (ties: lower id), onto the
// least-loaded rank that still has room (ties: lower rank)
std::vector<int> lpt(const std::vector<i64> &load, int EP)
{
    const int E = (int)load.size(), M = E / EP;
    std::vector<int> order(E);
    std::iota(order.begin(), order.end(), 0);
    std::stable_sort(order.begin(), order.end(), [&](int a, int b) { return load[a] > load[b]; });
    std::vector<i64> sum(EP, 0);
    std::vector<int> held(EP, 0), rank_of(E, 0);
    for (int e : order) {
        int pick = -1;
        for (int g = 0; g < EP; ++g)
            if (held[g] < M && (pick < 0 || sum[g] < sum[pick])) pick = g;
        rank_of[e] = pick;
        sum[pick] += load[e];
        ++held[pick];
    }
    return rank_of;
}

struct SplitMix64 {
    uint64_t state;
    uint64_t next()
    {
        uint64_t z = (state += 0x9E3779B97F4A7C15ull);
        z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
        z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
        return z ^ (z >> 31);
    }
};

struct SeedResult {
    std::vector<int> rank_of;
    double exact_T = 0.0, smooth_T = 0.0;
    i64 iterations = 0;
};

// trace (optional): the first trace_cap iterations as moves[i] = {e_a, e_b, accepted}, vals[i] = {u, T', theta}
struct Trace {
    int cap = 0;
    int32_t *moves = nullptr;
    double *vals = nullptr;
};

SeedResult anneal(const Problem &P, const std::vector<int> &start, double smooth_start, double gamma, double eps,
                  uint64_t rng_state, const Trace &trace = Trace{})
{
    SplitMix64 rng{rng_state};
    std::vector<int> cur = start;
    SeedResult res;
    res.rank_of = start;
    Loads L = P.loads_of(cur);
    std::vector<double> zc(P.EP), zm(P.EP);
    double T = smooth_start, T_best = smooth_start, theta = smooth_start;
    while (theta > eps) {
        const int ea = (int)(rng.next() % (uint64_t)P.E);
        const int eb = (int)(rng.next() % (uint64_t)P.E);
        const double u = (double)(rng.next() >> 11) * (1.0 / 9007199254740992.0);
        const int ra = cur[ea], rb = cur[eb];
        double Tn = T;
        if (ra != rb) {
            P.place(L, ea, ra, -1); P.place(L, ea, rb, +1);
            P.place(L, eb, rb, -1); P.place(L, eb, ra, +1);
            Tn = P.smooth(L, zc, zm);
        }
        const bool accept = Tn < T || u < std::exp(-(Tn - T) / theta);
        if (res.iterations < trace.cap) {
            int32_t *mv = trace.moves + 3 * res.iterations;
            double *vl = trace.vals + 3 * res.iterations;
            mv[0] = ea; mv[1] = eb; mv[2] = accept ? 1 : 0;
            vl[0] = u; vl[1] = Tn; vl[2] = theta;
        }
        if (accept) {
            T = Tn;
            cur[ea] = rb;
            cur[eb] = ra;
        } else if (ra != rb) {
            P.place(L, ea, rb, -1); P.place(L, ea, ra, +1);
            P.place(L, eb, ra, -1); P.place(L, eb, rb, +1);
        }
        if (T < T_best) {
            T_best = T;
            res.rank_of = cur;
        }
        theta *= gamma;
        ++res.iterations;
    }
    const Loads Lb = P.loads_of(res.rank_of);
    double ex[3];
    P.exact(Lb, ex);
    res.exact_T = ex[0];
    res.smooth_T = P.smooth(Lb, zc, zm);
    return res;
}

int check_model(const int64_t *x, int E, const relibra_cost_model *m)
{
    if (!x || !m || E < 1 || m->EP < 1 || E % m->EP || m->ranks_per_node < 1 || m->EP % m->ranks_per_node) return RELIBRA_EINVAL;
    if (!(m->sec_per_token_comp >= 0.0) || !(m->sec_per_token_intra >= 0.0) || !(m->sec_per_token_inter >= 0.0)) return RELIBRA_EINVAL;
    for (size_t i = 0; i < (size_t)m->EP * E; ++i)
        if (x[i] < 0 || x[i] > ((int64_t)1 << 40)) return RELIBRA_ERANGE;
    return RELIBRA_OK;
}

Problem make_problem(const int64_t *x, int E, const relibra_cost_model *m, double beta, double t_ref)
{
    return Problem{x, E, m->EP, m->ranks_per_node, m->sec_per_token_comp, m->sec_per_token_intra,
                   m->sec_per_token_inter, beta, t_ref};
}

}  // namespace

extern "C" int relibra_moe_time(const int64_t *x_host, int E, const relibra_cost_model *model,
                                const int32_t *expert_rank, double beta, double t_ref,
                                double *out4, int64_t *loads_out)
{
    if (int rc = check_model(x_host, E, model)) return rc;
    if (!expert_rank || !out4 || !(beta > 0.0) || !(t_ref > 0.0)) return RELIBRA_EINVAL;
    std::vector<int> rank_of(E);
    for (int e = 0; e < E; ++e) {
        if (expert_rank[e] < 0 || expert_rank[e] >= model->EP) return RELIBRA_ERANGE;
        rank_of[e] = expert_rank[e];
    }
    const Problem P = make_problem(x_host, E, model, beta, t_ref);
    const Loads L = P.loads_of(rank_of);
    std::vector<double> zc(P.EP), zm(P.EP);
    P.exact(L, out4);
    out4[3] = P.smooth(L, zc, zm);
    if (loads_out) {
        const std::vector<i64> *rows[5] = {&L.comp, &L.nv_tx, &L.nv_rx, &L.rd_tx, &L.rd_rx};
        for (int i = 0; i < 5; ++i)
            for (int g = 0; g < P.EP; ++g) loads_out[(size_t)i * P.EP + g] = (*rows[i])[g];
    }
    return RELIBRA_OK;
}

extern "C" int relibra_cost_model_init(relibra_cost_model *model, int EP, int ranks_per_node, int h, int hff,
                                       double F, double B_intra, double B_inter, int bytes_per_value)
{
    if (!model || EP < 1 || ranks_per_node < 1 || EP % ranks_per_node || h < 1 || hff < 1 || bytes_per_value < 1 ||
        !(F > 0.0) || !(B_intra > 0.0) || !(B_inter > 0.0))
        return RELIBRA_EINVAL;
    model->EP = EP;
    model->ranks_per_node = ranks_per_node;
    model->sec_per_token_comp = 6.0 * (double)h * (double)hff / F;                 // three GEMMs of 2 h h' flops (Eq. 4)
    model->sec_per_token_intra = (double)bytes_per_value * (double)h / B_intra;    // one token's hidden vector (Eq. 5)
    model->sec_per_token_inter = (double)bytes_per_value * (double)h / B_inter;
    return RELIBRA_OK;
}

namespace {

// Greedy-LPT start of Algorithm 1 and the normalisation it fixes: P.t_ref = the start's exact T_MoE.
struct SaStart {
    std::vector<int> rank_of;
    double exact_T, smooth_T;
};
SaStart sa_start(Problem &P)
{
    std::vector<i64> load(P.E, 0);
    for (int j = 0; j < P.EP; ++j)
        for (int e = 0; e < P.E; ++e) load[e] += P.x[(size_t)j * P.E + e];
    SaStart st{lpt(load, P.EP), 0.0, 0.0};
    P.t_ref = 1.0;
    const Loads L0 = P.loads_of(st.rank_of);
    double ex0[3];
    P.exact(L0, ex0);
    st.exact_T = ex0[0];
    P.t_ref = ex0[0] > 0.0 ? ex0[0] : 1.0;
    std::vector<double> zc(P.EP), zm(P.EP);
    st.smooth_T = P.smooth(L0, zc, zm);
    return st;
}

}  // namespace

extern "C" long long relibra_reorder_sa_trace(const int64_t *x_host, int E, const relibra_cost_model *model,
                                              double beta, double gamma, double eps, uint64_t seed,
                                              int trace_cap, int32_t *moves_out, double *vals_out,
                                              int32_t *start_rank_out, int32_t *expert_rank_out, double *stats2)
{
    if (int rc = check_model(x_host, E, model)) return rc;
    if (!expert_rank_out || !start_rank_out || !stats2 || !(beta > 0.0) || !(gamma > 0.0 && gamma < 1.0) || !(eps > 0.0) ||
        trace_cap < 0 || (trace_cap > 0 && (!moves_out || !vals_out)))
        return RELIBRA_EINVAL;
    Problem P = make_problem(x_host, E, model, beta, 1.0);
    const SaStart st = sa_start(P);
    const SeedResult res = anneal(P, st.rank_of, st.smooth_T, gamma, eps, seed, Trace{trace_cap, moves_out, vals_out});
    for (int e = 0; e < E; ++e) {
        start_rank_out[e] = st.rank_of[e];
        expert_rank_out[e] = res.rank_of[e];
    }
    stats2[0] = P.t_ref;
    stats2[1] = st.smooth_T;
    return res.iterations;
}

extern "C" int relibra_reorder_sa(const int64_t *x_host, int E, const relibra_cost_model *model,
                                  double beta, double gamma, double eps, int n_seeds, uint64_t seed,
                                  int32_t *expert_rank_out, double *stats5)
{
    if (int rc = check_model(x_host, E, model)) return rc;
    if (!expert_rank_out || !stats5 || !(beta > 0.0) || !(gamma > 0.0 && gamma < 1.0) || !(eps > 0.0) ||
        n_seeds < 1 || n_seeds > 4096)
        return RELIBRA_EINVAL;
    const int EP = model->EP;
    Problem P = make_problem(x_host, E, model, beta, 1.0);
    const SaStart st0 = sa_start(P);
    const std::vector<int> &start = st0.rank_of;
    const double ex0[1] = {st0.exact_T};
    const double smooth0 = st0.smooth_T;
    (void)EP;

    std::vector<SeedResult> results(n_seeds);
    unsigned hw = std::thread::hardware_concurrency();
    const int workers = std::max(1, std::min<int>({n_seeds, (int)(hw ? hw : 1u), 64}));
    auto work = [&](int w) {
        for (int s = w; s < n_seeds; s += workers)
            results[s] = anneal(P, start, smooth0, gamma, eps, seed + (uint64_t)s * 0xD1342543DE82EF95ull);
    };
    if (workers == 1) {
        work(0);
    } else {
        std::vector<std::thread> pool;
        for (int w = 0; w < workers; ++w) pool.emplace_back(work, w);
        for (auto &t : pool) t.join();
    }
    int best = 0;
    for (int s = 1; s < n_seeds; ++s)
        if (results[s].exact_T < results[best].exact_T) best = s;
    for (int e = 0; e < E; ++e) expert_rank_out[e] = results[best].rank_of[e];
    stats5[0] = ex0[0];
    stats5[1] = results[best].exact_T;
    stats5[2] = smooth0;
    stats5[3] = results[best].smooth_T;
    stats5[4] = (double)results[n_seeds - 1].iterations;
    return RELIBRA_OK;
}
