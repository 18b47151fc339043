/*
 * CPU oracle for the replay-guided MoE expert-layer path.  TEST INFRASTRUCTURE ONLY:
 * it is called by the tests, by the smoke check and by the benchmark's CPU-baseline
 * leg, never by the product path, and it shares no code with the HIP library.
 *
 * Plain loops, integers for everything that is counted, double precision for
 * everything that is floating point (inputs are bf16 bit patterns, widened exactly).
 * Each function names the passage of the paper it follows.
 *
 * Parity pins live in tests/test_oracle_*.py; every function is pinned.  The randomized
 * annealing of Algorithm 1 (oracle_reorder_sa) depends on constants the paper does not
 * publish (cooling rate, threshold, seed set, random generator): they are arguments, the
 * generator is splitmix64 (pinned against its published outputs), and the acceptance
 * rule, cooling and draw order are pinned by a hand-worked three-step run; its cost
 * model, smoothed objective and invariants are pinned separately.
 */
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#include <math.h>

#ifdef _OPENMP
#include <omp.h>
#endif

typedef long long i64;
typedef unsigned __int128 u128;

/* ------------------------------------------------------------------------- */
/* Per-expert load (Eq. 1: l_e = number of routed tokens of expert e).        */
/* counts[mb][e]; total[e] = sum over micro-batches (Section 4.1: the         */
/* inter-batch problem balances the load accumulated over the whole batch).   */
/* returns 0, or -2 if an id is outside [0,E).                                */
int oracle_route_hist(const int32_t *ids, int n_mb, int T, int k, int E,
                      int32_t *counts, i64 *total)
{
    for (int i = 0; i < n_mb * E; ++i) counts[i] = 0;
    for (int e = 0; e < E; ++e) total[e] = 0;
    for (int mb = 0; mb < n_mb; ++mb)
        for (int t = 0; t < T; ++t)
            for (int s = 0; s < k; ++s) {
                int e = ids[((size_t)mb * T + t) * k + s];
                if (e < 0 || e >= E) return -2;
                counts[mb * E + e] += 1;
                total[e] += 1;
            }
    return 0;
}

/* ------------------------------------------------------------------------- */
/* Stage 1: inter-batch expert reordering (Section 4, Algorithm 1 made        */
/* deterministic: steepest swap descent over the same swap neighbourhood).    */

/* Greedy LPT with a per-rank capacity of M experts (Section 4.2): experts in  */
/* descending load (ties: lower id first), each onto the rank that still has   */
/* room and has the smallest load so far (ties: lower rank).                   */
void oracle_lpt(const i64 *l, int E, int EP, int32_t *rank_of)
{
    int M = E / EP;
    int *order = (int *)malloc(sizeof(int) * E);
    for (int e = 0; e < E; ++e) order[e] = e;
    /* insertion sort: descending load, ascending id */
    for (int i = 1; i < E; ++i) {
        int x = order[i], j = i - 1;
        while (j >= 0 && (l[order[j]] < l[x] || (l[order[j]] == l[x] && order[j] > x))) {
            order[j + 1] = order[j];
            --j;
        }
        order[j + 1] = x;
    }
    i64 *load = (i64 *)calloc(EP, sizeof(i64));
    int *held = (int *)calloc(EP, sizeof(int));
    for (int i = 0; i < E; ++i) {
        int e = order[i], best = -1;
        for (int g = 0; g < EP; ++g) {
            if (held[g] >= M) continue;
            if (best < 0 || load[g] < load[best]) best = g;
        }
        rank_of[e] = best;
        load[best] += l[e];
        held[best] += 1;
    }
    free(order); free(load); free(held);
}

/* State cost: (max_g L_g, sum_g L_g^2), compared lexicographically.  The second  */
/* component does the job of the paper's log-sum-exp smoothing (Section 4.2,      */
/* "objective smoothing"): it still moves when the maximum sits on a plateau.     */
static void phi_of(const i64 *load, int EP, i64 *mx, u128 *sq)
{
    i64 m = 0; u128 s = 0;
    for (int g = 0; g < EP; ++g) {
        if (load[g] > m) m = load[g];
        s += (u128)load[g] * (u128)load[g];
    }
    *mx = m; *sq = s;
}
static int phi_less(i64 m1, u128 s1, i64 m2, u128 s2)
{
    return m1 < m2 || (m1 == m2 && s1 < s2);
}

/* Steepest swap descent from the placement in rank_of (updated in place).       */
/* Every pair of experts on different ranks is tried; the swap with the smallest  */
/* resulting cost wins (ties: smallest (e_a, e_b)); it is applied only if it      */
/* strictly lowers the cost.                                                      */
void oracle_swap_descent(const i64 *l, int E, int EP, int32_t *rank_of)
{
    i64 *load = (i64 *)calloc(EP, sizeof(i64));
    for (int e = 0; e < E; ++e) load[rank_of[e]] += l[e];
    i64 cur_m; u128 cur_s;
    phi_of(load, EP, &cur_m, &cur_s);
    for (;;) {
        int ba = -1, bb = -1; i64 bm = 0; u128 bs = 0;
        for (int a = 0; a < E; ++a)
            for (int b = a + 1; b < E; ++b) {
                int ga = rank_of[a], gb = rank_of[b];
                if (ga == gb) continue;
                /* only the two ranks involved change (Section 4.2, incremental update) */
                load[ga] += l[b] - l[a];
                load[gb] += l[a] - l[b];
                i64 m; u128 s;
                phi_of(load, EP, &m, &s);
                load[ga] -= l[b] - l[a];
                load[gb] -= l[a] - l[b];
                if (ba < 0 || phi_less(m, s, bm, bs)) { ba = a; bb = b; bm = m; bs = s; }
            }
        if (ba < 0 || !phi_less(bm, bs, cur_m, cur_s)) break;
        int ga = rank_of[ba], gb = rank_of[bb];
        load[ga] += l[bb] - l[ba];
        load[gb] += l[ba] - l[bb];
        rank_of[ba] = gb; rank_of[bb] = ga;
        cur_m = bm; cur_s = bs;
    }
    free(load);
}

/* Reordering without the batch-level guard: descent from the unplanned layout    */
/* (expert e on rank e / M) and from LPT; the better final cost wins, ties keep    */
/* the unplanned start.                                                            */
void oracle_reorder(const i64 *l, int E, int EP, int32_t *rank_of)
{
    int M = E / EP;
    int32_t *p_id = (int32_t *)malloc(sizeof(int32_t) * E);
    int32_t *p_lpt = (int32_t *)malloc(sizeof(int32_t) * E);
    for (int e = 0; e < E; ++e) p_id[e] = e / M;
    oracle_lpt(l, E, EP, p_lpt);
    oracle_swap_descent(l, E, EP, p_id);
    oracle_swap_descent(l, E, EP, p_lpt);
    i64 *load = (i64 *)malloc(sizeof(i64) * EP);
    i64 m1, m2; u128 s1, s2;
    for (int g = 0; g < EP; ++g) load[g] = 0;
    for (int e = 0; e < E; ++e) load[p_id[e]] += l[e];
    phi_of(load, EP, &m1, &s1);
    for (int g = 0; g < EP; ++g) load[g] = 0;
    for (int e = 0; e < E; ++e) load[p_lpt[e]] += l[e];
    phi_of(load, EP, &m2, &s2);
    free(load);
    int lpt_better = phi_less(m2, s2, m1, s1);
    memcpy(rank_of, lpt_better ? p_lpt : p_id, sizeof(int32_t) * E);
    free(p_id); free(p_lpt);
}

/* ------------------------------------------------------------------------- */
/* Imbalance diagnostics (Section 2.2): load skewness of a micro-batch = largest */
/* expert load over the mean expert load; intersection ratio of the `top`        */
/* highest-load experts (ties: lower id) between adjacent micro-batches.         */
void oracle_load_stats(const int32_t *counts, int n_mb, int E, int top, double *skew, double *inter)
{
    uint8_t *hot = (uint8_t *)calloc((size_t)n_mb * E, 1);
    for (int mb = 0; mb < n_mb; ++mb) {
        const int32_t *c = counts + (size_t)mb * E;
        i64 sum = 0, peak = 0;
        for (int e = 0; e < E; ++e) { sum += c[e]; if (c[e] > peak) peak = c[e]; }
        skew[mb] = sum > 0 ? (double)peak / ((double)sum / E) : 1.0;
        for (int pick = 0; pick < top; ++pick) {          /* selection: largest not yet taken, lowest id on ties */
            int best = -1;
            for (int e = 0; e < E; ++e)
                if (!hot[(size_t)mb * E + e] && (best < 0 || c[e] > c[best])) best = e;
            hot[(size_t)mb * E + best] = 1;
        }
    }
    for (int mb = 0; mb + 1 < n_mb; ++mb) {
        int both = 0;
        for (int e = 0; e < E; ++e) both += hot[(size_t)mb * E + e] && hot[(size_t)(mb + 1) * E + e];
        inter[mb] = (double)both / top;
    }
    free(hot);
}

/* ------------------------------------------------------------------------- */
/* Communication-aware cost model of the MoE module (Section 4.1, Eq. 1-6)    */
/* and Algorithm 1 as printed (swap-based simulated annealing, Section 4.2).  */

/* x[j][e]: tokens that sit on source rank j and are routed to expert e.       */
/* Tokens of a micro-batch are dealt to the EP ranks in equal contiguous runs  */
/* (data-parallel attention): token t sits on rank t / (T / EP).               */
int oracle_route_hist_src(const int32_t *ids, int T, int k, int E, int EP, i64 *x)
{
    if (EP < 1 || T % EP) return -1;
    for (int i = 0; i < EP * E; ++i) x[i] = 0;
    for (int t = 0; t < T; ++t)
        for (int s = 0; s < k; ++s) {
            int e = ids[(size_t)t * k + s];
            if (e < 0 || e >= E) return -2;
            x[(size_t)(t / (T / EP)) * E + e] += 1;
        }
    return 0;
}

/* Source-destination type on a rail-optimised cluster of rpn-GPU nodes        */
/* (Section 4.1): 0 local copy, 1 intra-node link, 2 inter-node same rail      */
/* (GPUs with the same index inside their nodes), 3 inter-node cross rail.     */
int oracle_tau(int j, int g, int rpn)
{
    if (j == g) return 0;
    if (j / rpn == g / rpn) return 1;
    if (j % rpn == g % rpn) return 2;
    return 3;
}

/* Loads in tokens under placement rank_of (Eq. 1-3): computation load of g,   */
/* intra-node link send/receive load (types nv and cr) and RDMA send/receive   */
/* load (types sr and cr) during dispatch.                                     */
void oracle_loads(const i64 *x, int E, int EP, int rpn, const int32_t *rank_of,
                  i64 *comp, i64 *nv_tx, i64 *nv_rx, i64 *rd_tx, i64 *rd_rx)
{
    for (int g = 0; g < EP; ++g) comp[g] = nv_tx[g] = nv_rx[g] = rd_tx[g] = rd_rx[g] = 0;
    for (int e = 0; e < E; ++e) {
        int g = rank_of[e];
        for (int j = 0; j < EP; ++j) {
            i64 n = x[(size_t)j * E + e];
            int tau = oracle_tau(j, g, rpn);
            comp[g] += n;
            if (tau == 1 || tau == 3) { nv_tx[j] += n; nv_rx[g] += n; }
            if (tau == 2 || tau == 3) { rd_tx[j] += n; rd_rx[g] += n; }
        }
    }
}

/* LSE_beta(z) = log(sum exp(beta z)) / beta (Section 4.2, objective smoothing), */
/* evaluated around the maximum.                                                */
double oracle_lse(const double *z, int n, double beta)
{
    double m = z[0];
    for (int i = 1; i < n; ++i) if (z[i] > m) m = z[i];
    double acc = 0.0;
    for (int i = 0; i < n; ++i) acc += exp(beta * (z[i] - m));
    return m + log(acc) / beta;
}

/* model[0..4] = seconds per token of computation (6hh'/F, Eq. 4), seconds per  */
/* token over the intra-node link and over RDMA (bytes per token / bandwidth,  */
/* Eq. 5), then unused.  out[0] = T_MoE (Eq. 6) in seconds, out[1] = max_g      */
/* T_comp, out[2] = max_g T_comm, out[3] = smoothed objective with every time   */
/* divided by t_ref (so that beta acts on numbers of order one).               */
void oracle_moe_time(const i64 *x, int E, int EP, int rpn, const int32_t *rank_of,
                     const double *model, double beta, double t_ref, double *out)
{
    i64 *L = (i64 *)malloc(sizeof(i64) * 5 * EP);
    i64 *comp = L, *nv_tx = L + EP, *nv_rx = L + 2 * EP, *rd_tx = L + 3 * EP, *rd_rx = L + 4 * EP;
    double *zc = (double *)malloc(sizeof(double) * 2 * EP), *zm = zc + EP;
    oracle_loads(x, E, EP, rpn, rank_of, comp, nv_tx, nv_rx, rd_tx, rd_rx);
    double max_comp = 0.0, max_comm = 0.0;
    for (int g = 0; g < EP; ++g) {
        double tc = (double)comp[g] * model[0];
        double t4[4] = {(double)nv_tx[g] * model[1], (double)nv_rx[g] * model[1],
                        (double)rd_tx[g] * model[2], (double)rd_rx[g] * model[2]};
        double tm = t4[0];
        for (int i = 1; i < 4; ++i) if (t4[i] > tm) tm = t4[i];
        if (tc > max_comp) max_comp = tc;
        if (tm > max_comm) max_comm = tm;
        for (int i = 0; i < 4; ++i) t4[i] /= t_ref;
        zc[g] = tc / t_ref;
        zm[g] = oracle_lse(t4, 4, beta);
    }
    out[0] = max_comp + max_comm;
    out[1] = max_comp;
    out[2] = max_comm;
    out[3] = oracle_lse(zc, EP, beta) + oracle_lse(zm, EP, beta);
    free(L);
    free(zc);
}

/* splitmix64 (Steele, Lea, Flood 2014): the counter-based generator both the  */
/* oracle and the library implement for the annealing's random draws.          */
static uint64_t sm64_next(uint64_t *state)
{
    uint64_t z = (*state += 0x9E3779B97F4A7C15ull);
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    return z ^ (z >> 31);
}

/* Algorithm 1.  Start: greedy LPT on l_e = sum_j x[j][e].  Per seed: repeat   */
/* {draw two experts, swap their ranks, evaluate the smoothed objective, accept */
/* if better or with probability exp(-(T' - T)/theta), remember the best,       */
/* theta *= gamma} while theta > eps; theta starts at the start's objective.    */
/* (The printed acceptance exponent has the opposite sign, which would accept   */
/* every worsening move; read as the Metropolis rule.)  The seeds' best states  */
/* are compared by the exact T_MoE; ties keep the lower seed.  Every time is    */
/* divided by the start's exact T_MoE before smoothing.  Three draws per        */
/* iteration in the order e_a, e_b, u; seed s starts its generator at           */
/* seed + s * 0xD1342543DE82EF95.  stats[0] = exact T of the start, [1] = exact */
/* T of the result, [2] = smoothed start, [3] = smoothed result, [4] = iterations per seed. */
/* first n outputs of the generator started at state `seed` (for the pin against the    */
/* published test vectors)                                                             */
void oracle_splitmix64(uint64_t seed, int n, uint64_t *out)
{
    for (int i = 0; i < n; ++i) out[i] = sm64_next(&seed);
}

/* One seed of Algorithm 1 from `start` (generator state rng).  best receives the seed's */
/* best placement, *T_best_out its smoothed objective; returns the iterations.  With    */
/* trace_cap > 0 the first trace_cap iterations are recorded: moves[i] = {e_a, e_b,      */
/* accepted (0/1)}, vals[i] = {u, T' (smoothed objective of the swapped state), theta}. */
static i64 sa_one_seed(const i64 *x, int E, int EP, int rpn, const double *model, double beta,
                       double t_ref, double gamma, double eps, uint64_t rng,
                       const int32_t *start, double smooth0, int32_t *cur, int32_t *best,
                       int trace_cap, int32_t *moves, double *vals)
{
    double o[4];
    memcpy(cur, start, sizeof(int32_t) * E);
    memcpy(best, start, sizeof(int32_t) * E);
    double T = smooth0, T_best = smooth0, theta = smooth0;
    i64 iters = 0;
    while (theta > eps) {
        int ea = (int)(sm64_next(&rng) % (uint64_t)E);
        int eb = (int)(sm64_next(&rng) % (uint64_t)E);
        double u = (double)(sm64_next(&rng) >> 11) * (1.0 / 9007199254740992.0);
        int32_t ra = cur[ea], rb = cur[eb];
        cur[ea] = rb;
        cur[eb] = ra;
        oracle_moe_time(x, E, EP, rpn, cur, model, beta, t_ref, o);
        double Tn = o[3];
        int accepted = 0;
        if (Tn < T || u < exp(-(Tn - T) / theta)) {
            T = Tn;
            accepted = 1;
        } else {
            cur[ea] = ra;
            cur[eb] = rb;
        }
        if (T < T_best) {
            T_best = T;
            memcpy(best, cur, sizeof(int32_t) * E);
        }
        if (iters < trace_cap) {
            moves[3 * iters] = ea; moves[3 * iters + 1] = eb; moves[3 * iters + 2] = accepted;
            vals[3 * iters] = u; vals[3 * iters + 1] = Tn; vals[3 * iters + 2] = theta;
        }
        theta *= gamma;
        ++iters;
    }
    return iters;
}

int oracle_reorder_sa(const i64 *x, int E, int EP, int rpn, const double *model,
                      double beta, double gamma, double eps, int n_seeds, uint64_t seed,
                      int32_t *rank_out, double *stats)
{
    if (E % EP || n_seeds < 1 || !(gamma > 0.0 && gamma < 1.0) || !(eps > 0.0)) return -1;
    i64 *l = (i64 *)calloc(E, sizeof(i64));
    for (int j = 0; j < EP; ++j)
        for (int e = 0; e < E; ++e) l[e] += x[(size_t)j * E + e];
    int32_t *start = (int32_t *)malloc(sizeof(int32_t) * E);
    int32_t *cur = (int32_t *)malloc(sizeof(int32_t) * E);
    int32_t *best = (int32_t *)malloc(sizeof(int32_t) * E);
    oracle_lpt(l, E, EP, start);
    double o[4];
    oracle_moe_time(x, E, EP, rpn, start, model, beta, 1.0, o);
    const double t_ref = o[0] > 0.0 ? o[0] : 1.0;
    oracle_moe_time(x, E, EP, rpn, start, model, beta, t_ref, o);
    const double exact0 = o[0], smooth0 = o[3];
    double best_exact = 0.0, best_smooth = 0.0;
    i64 iters = 0;
    for (int s = 0; s < n_seeds; ++s) {
        iters = sa_one_seed(x, E, EP, rpn, model, beta, t_ref, gamma, eps, seed + (uint64_t)s * 0xD1342543DE82EF95ull,
                            start, smooth0, cur, best, 0, NULL, NULL);
        oracle_moe_time(x, E, EP, rpn, best, model, beta, t_ref, o);
        if (s == 0 || o[0] < best_exact) {
            best_exact = o[0];
            best_smooth = o[3];
            memcpy(rank_out, best, sizeof(int32_t) * E);
        }
    }
    stats[0] = exact0;
    stats[1] = best_exact;
    stats[2] = smooth0;
    stats[3] = best_smooth;
    stats[4] = (double)iters;
    free(l);
    free(start);
    free(cur);
    free(best);
    return 0;
}

/* The first seed's run of oracle_reorder_sa with its trajectory written out (see    */
/* sa_one_seed); rank_out = that seed's best placement, start_out = the LPT start,   */
/* stats[0] = t_ref (the start's exact T_MoE), stats[1] = smoothed start.  Returns   */
/* the iterations, or -1.                                                           */
long long oracle_reorder_sa_trace(const i64 *x, int E, int EP, int rpn, const double *model,
                                  double beta, double gamma, double eps, uint64_t seed,
                                  int trace_cap, int32_t *moves, double *vals,
                                  int32_t *start_out, int32_t *rank_out, double *stats)
{
    if (E % EP || !(gamma > 0.0 && gamma < 1.0) || !(eps > 0.0)) return -1;
    i64 *l = (i64 *)calloc(E, sizeof(i64));
    for (int j = 0; j < EP; ++j)
        for (int e = 0; e < E; ++e) l[e] += x[(size_t)j * E + e];
    int32_t *cur = (int32_t *)malloc(sizeof(int32_t) * E);
    oracle_lpt(l, E, EP, start_out);
    double o[4];
    oracle_moe_time(x, E, EP, rpn, start_out, model, beta, 1.0, o);
    const double t_ref = o[0] > 0.0 ? o[0] : 1.0;
    oracle_moe_time(x, E, EP, rpn, start_out, model, beta, t_ref, o);
    stats[0] = t_ref;
    stats[1] = o[3];
    i64 iters = sa_one_seed(x, E, EP, rpn, model, beta, t_ref, gamma, eps, seed, start_out, o[3], cur, rank_out,
                            trace_cap, moves, vals);
    free(l);
    free(cur);
    return iters;
}

/* ------------------------------------------------------------------------- */
/* Stage 2: intra-batch replication for one node (Section 5.2, Algorithm 2,   */
/* computation-only objective: the time of a rank is its load in tokens).     */
/*                                                                            */
/* A node has n ranks (local ids 0..n-1) and ne experts (local ids 0..ne-1,    */
/* listed in ascending global expert id).  home[e] is the local rank of e.     */
/* z[e*n+g] = 1 iff tokens of e may be served on g (Eq. 8-11); a[e*n+g] is the  */
/* integer number of tokens of e served on g (the split y scaled by x).        */

/* Token split for a given placement z (Section 5.2, SolveTokenSplitLP, restricted   */
/* to the computation term).  Among the splits that minimise the largest rank load   */
/* the linear program leaves the choice open; the one taken here also minimises the   */
/* sum of squared rank loads, reached by repeatedly moving tokens along a chain of    */
/* ranks from a heavier rank u to a lighter rank v whenever load(v) <= load(u) - 2:    */
/*   - ranks are tried as u in descending load (ties: lower id);                       */
/*   - breadth-first search from u over ranks: u' -> v' if some expert with tokens on  */
/*     u' may also be served on v' (v' scanned ascending; the lowest such expert is    */
/*     the one that moves along that edge);                                            */
/*   - v = the reached rank of smallest load (ties: lower id); if load(v) <= load(u)-2  */
/*     move d = min(floor((load(u)-load(v))/2), tokens available on each edge of the    */
/*     path) and start over; if no u has such a v the split is final.                  */
/* When no such chain is left the split is optimal for every convex cost of the loads  */
/* at once, the maximum included.  The split continues from the one in a (warm start).  */
void oracle_balance_split(const uint8_t *z, int ne, int n, i64 *a)
{
    i64 *load = (i64 *)malloc(sizeof(i64) * n);
    int *par = (int *)malloc(sizeof(int) * n);
    int *par_e = (int *)malloc(sizeof(int) * n);
    int *queue = (int *)malloc(sizeof(int) * n);
    int *order = (int *)malloc(sizeof(int) * n);
    for (;;) {
        for (int g = 0; g < n; ++g) {
            load[g] = 0;
            for (int e = 0; e < ne; ++e) load[g] += a[e * n + g];
            order[g] = g;
        }
        for (int i = 1; i < n; ++i) {            /* descending load, ascending id */
            int x = order[i], j = i - 1;
            while (j >= 0 && load[order[j]] < load[x]) { order[j + 1] = order[j]; --j; }
            order[j + 1] = x;
        }
        int moved = 0;
        for (int oi = 0; oi < n && !moved; ++oi) {
            int u = order[oi];
            for (int g = 0; g < n; ++g) par[g] = -2;
            par[u] = -1;
            int qh = 0, qt = 0;
            queue[qt++] = u;
            while (qh < qt) {
                int w = queue[qh++];
                for (int v = 0; v < n; ++v) {
                    if (par[v] != -2) continue;
                    int via = -1;
                    for (int e = 0; e < ne; ++e)
                        if (a[e * n + w] > 0 && z[e * n + v]) { via = e; break; }
                    if (via < 0) continue;
                    par[v] = w; par_e[v] = via;
                    queue[qt++] = v;
                }
            }
            int v = -1;
            for (int g = 0; g < n; ++g)
                if (g != u && par[g] != -2 && (v < 0 || load[g] < load[v])) v = g;
            if (v < 0 || load[v] > load[u] - 2) continue;
            i64 d = (load[u] - load[v]) / 2;
            for (int x = v; par[x] >= 0; x = par[x])
                if (a[par_e[x] * n + par[x]] < d) d = a[par_e[x] * n + par[x]];
            for (int x = v; par[x] >= 0; x = par[x]) {
                a[par_e[x] * n + par[x]] -= d;
                a[par_e[x] * n + x] += d;
            }
            moved = 1;
        }
        if (!moved) break;
    }
    free(load); free(par); free(par_e); free(queue); free(order);
}

/* Algorithm 2 on one node.  Outputs z and a (ne*n each); returns the node's max   */
/* rank load after replication.                                                    */
i64 oracle_replicate_node(const i64 *cnt, const int32_t *home, int ne, int n, int r,
                          uint8_t *z, i64 *a)
{
    int *used = (int *)calloc(n, sizeof(int));
    i64 *load = (i64 *)calloc(n, sizeof(i64));
    i64 total = 0;
    for (int i = 0; i < ne * n; ++i) { z[i] = 0; a[i] = 0; }
    for (int e = 0; e < ne; ++e) {           /* no replica: everything at home */
        z[e * n + home[e]] = 1;
        a[e * n + home[e]] = cnt[e];
        total += cnt[e];
    }
    i64 floor_cap = (total + n - 1) / n;     /* no split can beat the node average */
    for (;;) {
        for (int g = 0; g < n; ++g) {
            load[g] = 0;
            for (int e = 0; e < ne; ++e) load[g] += a[e * n + g];
        }
        int gb = 0;                          /* bottleneck rank */
        for (int g = 1; g < n; ++g) if (load[g] > load[gb]) gb = g;
        if (load[gb] <= floor_cap) break;
        /* experts served on gb with a positive share, heaviest share first; the first  */
        /* one that some rank can still take a replica of is replicated                  */
        int picked_e = -1, picked_g = -1;
        uint8_t *tried = (uint8_t *)calloc(ne, 1);
        for (;;) {
            int e_star = -1;
            for (int e = 0; e < ne; ++e) {
                if (tried[e] || a[e * n + gb] <= 0) continue;
                if (e_star < 0 || a[e * n + gb] > a[e_star * n + gb]) e_star = e;
            }
            if (e_star < 0) break;
            tried[e_star] = 1;
            int gt = -1;                     /* least-loaded rank that can take a replica */
            for (int g = 0; g < n; ++g) {
                if (z[e_star * n + g] || used[g] >= r) continue;
                if (gt < 0 || load[g] < load[gt]) gt = g;
            }
            if (gt >= 0) { picked_e = e_star; picked_g = gt; break; }
        }
        free(tried);
        if (picked_e < 0) break;
        z[picked_e * n + picked_g] = 1;
        used[picked_g] += 1;
        oracle_balance_split(z, ne, n, a);
    }
    /* a replica that ended up with no tokens is not materialised */
    for (int e = 0; e < ne; ++e)
        for (int g = 0; g < n; ++g)
            if (g != home[e] && z[e * n + g] && a[e * n + g] == 0) z[e * n + g] = 0;
    i64 mx = 0;
    for (int g = 0; g < n; ++g) {
        i64 s = 0;
        for (int e = 0; e < ne; ++e) s += a[e * n + g];
        if (s > mx) mx = s;
    }
    free(used); free(load);
    return mx;
}

/* Replication of one micro-batch over all nodes under placement rank_of.          */
/* zz, aa: [E][EP] (global ids).  Returns the micro-batch's max rank load.          */
static i64 replicate_mb(const int32_t *cnt_mb, const int32_t *rank_of, int E, int EP, int rpn,
                        int r, uint8_t *zz, i64 *aa)
{
    int nodes = EP / rpn;
    i64 worst = 0;
    memset(zz, 0, (size_t)E * EP);
    memset(aa, 0, sizeof(i64) * (size_t)E * EP);
    int *ex = (int *)malloc(sizeof(int) * E);
    for (int nd = 0; nd < nodes; ++nd) {
        int ne = 0;
        for (int e = 0; e < E; ++e)
            if (rank_of[e] / rpn == nd) ex[ne++] = e;
        i64 *cnt = (i64 *)malloc(sizeof(i64) * (ne ? ne : 1));
        int32_t *home = (int32_t *)malloc(sizeof(int32_t) * (ne ? ne : 1));
        uint8_t *z = (uint8_t *)malloc((size_t)(ne ? ne : 1) * rpn);
        i64 *a = (i64 *)malloc(sizeof(i64) * (size_t)(ne ? ne : 1) * rpn);
        for (int i = 0; i < ne; ++i) { cnt[i] = cnt_mb[ex[i]]; home[i] = rank_of[ex[i]] - nd * rpn; }
        i64 mx = oracle_replicate_node(cnt, home, ne, rpn, r, z, a);
        if (mx > worst) worst = mx;
        for (int i = 0; i < ne; ++i)
            for (int g = 0; g < rpn; ++g) {
                zz[(size_t)ex[i] * EP + nd * rpn + g] = z[i * rpn + g];
                aa[(size_t)ex[i] * EP + nd * rpn + g] = a[i * rpn + g];
            }
        free(cnt); free(home); free(z); free(a);
    }
    free(ex);
    return worst;
}

/* ------------------------------------------------------------------------- */
/* Algorithm 2 with the execution time of Section 4.1 as its objective          */
/* (Section 5.2: bottleneck GPU and least-loaded GPU by T_MoE,g, computation     */
/* plus communication).  One micro-batch, whole EP group.                        */
/*                                                                              */
/* The state is z[e][g] / a[e][g] as above.  Its time: the instances of every    */
/* expert (ranks with z = 1, ascending) get their sources from                   */
/* oracle_assign_sources, the loads and times follow Eq. 1-6                     */
/* (oracle_moe_time_split); T_g = T_g^comp + T_g^comm per GPU.                   */
/* Loop: g_b = GPU of largest T_g (lowest id on ties); its experts with tokens   */
/* served there, most tokens first (lower id on ties), are tried in turn: the    */
/* target is the GPU of g_b's node without a copy of the expert and with a free  */
/* slot whose T_g is smallest (lowest id); the copy is placed, the node's tokens */
/* are split again (oracle_balance_split, warm start) and the move is kept if    */
/* (T_MoE of Eq. 6, sum_g T_g^2) got lexicographically smaller (the second       */
/* component moves when the maximum sits on a plateau, as in stage 1), otherwise */
/* undone and the next expert is tried.  The loop ends when no expert of the     */
/* bottleneck GPU gives a gain.                                                  */
/* Copies that end with no tokens are dropped.  T2[0], T2[1] = T_MoE before and  */
/* after; returns the largest computation load after.                            */
int oracle_assign_sources(const i64 *x, int E, int EP, int rpn, const int32_t *inst_ptr,
                          const int32_t *inst_rank, const int32_t *inst_rows, i64 *y);
void oracle_moe_time_split(const i64 *y, int n_inst, int EP, int rpn, const int32_t *inst_rank,
                           const double *model, double *out, i64 *loads);

static double eval_state(const i64 *x, int E, int EP, int rpn, const uint8_t *z, const i64 *a,
                         const double *model, double *tg, i64 *max_comp)
{
    int cap = E * EP;
    int32_t *ptr = (int32_t *)malloc(sizeof(int32_t) * (E + 1));
    int32_t *rank = (int32_t *)malloc(sizeof(int32_t) * cap);
    int32_t *rows = (int32_t *)malloc(sizeof(int32_t) * cap);
    int p = 0;
    for (int e = 0; e < E; ++e) {
        ptr[e] = p;
        for (int g = 0; g < EP; ++g)
            if (z[(size_t)e * EP + g]) { rank[p] = g; rows[p] = (int32_t)a[(size_t)e * EP + g]; ++p; }
    }
    ptr[E] = p;
    i64 *y = (i64 *)malloc(sizeof(i64) * (size_t)(p ? p : 1) * EP);
    i64 *loads = (i64 *)malloc(sizeof(i64) * 5 * EP);
    double out[3];
    oracle_assign_sources(x, E, EP, rpn, ptr, rank, rows, y);
    oracle_moe_time_split(y, p, EP, rpn, rank, model, out, loads);
    i64 mc = 0;
    for (int g = 0; g < EP; ++g) {
        double nv = model[1] * (double)(loads[EP + g] > loads[2 * EP + g] ? loads[EP + g] : loads[2 * EP + g]);
        double rd = model[2] * (double)(loads[3 * EP + g] > loads[4 * EP + g] ? loads[3 * EP + g] : loads[4 * EP + g]);
        tg[g] = model[0] * (double)loads[g] + (nv > rd ? nv : rd);
        if (loads[g] > mc) mc = loads[g];
    }
    if (max_comp) *max_comp = mc;
    free(ptr); free(rank); free(rows); free(y); free(loads);
    return out[0];
}

/* the balanced split of oracle_balance_split applied to the experts of one node */
static void node_split(int nd, const int32_t *rank_of, int E, int EP, int rpn, const uint8_t *z, i64 *a)
{
    int *ex = (int *)malloc(sizeof(int) * E), ne = 0;
    for (int e = 0; e < E; ++e) if (rank_of[e] / rpn == nd) ex[ne++] = e;
    uint8_t *zn = (uint8_t *)malloc((size_t)(ne ? ne : 1) * rpn);
    i64 *an = (i64 *)malloc(sizeof(i64) * (size_t)(ne ? ne : 1) * rpn);
    for (int i = 0; i < ne; ++i)
        for (int g = 0; g < rpn; ++g) {
            zn[i * rpn + g] = z[(size_t)ex[i] * EP + nd * rpn + g];
            an[i * rpn + g] = a[(size_t)ex[i] * EP + nd * rpn + g];
        }
    oracle_balance_split(zn, ne, rpn, an);
    for (int i = 0; i < ne; ++i)
        for (int g = 0; g < rpn; ++g) a[(size_t)ex[i] * EP + nd * rpn + g] = an[i * rpn + g];
    free(ex); free(zn); free(an);
}

i64 oracle_replicate_comm(const i64 *x, const int32_t *rank_of, int E, int EP, int rpn, int r,
                          const double *model, uint8_t *z, i64 *a, double *T2)
{
    size_t zsz = (size_t)E * EP;
    memset(z, 0, zsz);
    memset(a, 0, sizeof(i64) * zsz);
    for (int e = 0; e < E; ++e) {
        i64 l = 0;
        for (int j = 0; j < EP; ++j) l += x[(size_t)j * E + e];
        z[(size_t)e * EP + rank_of[e]] = 1;
        a[(size_t)e * EP + rank_of[e]] = l;
    }
    int *used = (int *)calloc(EP, sizeof(int));
    double *tg = (double *)malloc(sizeof(double) * EP), *tg_try = (double *)malloc(sizeof(double) * EP);
    i64 *a_keep = (i64 *)malloc(sizeof(i64) * zsz);
    uint8_t *tried = (uint8_t *)malloc(E);
    double T = eval_state(x, E, EP, rpn, z, a, model, tg, NULL);
    double S = 0;
    for (int g = 0; g < EP; ++g) S += tg[g] * tg[g];
    T2[0] = T;
    for (;;) {
        int gb = 0;
        for (int g = 1; g < EP; ++g) if (tg[g] > tg[gb]) gb = g;
        int nd = gb / rpn, accepted = 0;
        memset(tried, 0, E);
        for (;;) {
            int e_star = -1;
            for (int e = 0; e < E; ++e) {
                if (tried[e] || a[(size_t)e * EP + gb] <= 0) continue;
                if (e_star < 0 || a[(size_t)e * EP + gb] > a[(size_t)e_star * EP + gb]) e_star = e;
            }
            if (e_star < 0) break;
            tried[e_star] = 1;
            int gt = -1;
            for (int g = nd * rpn; g < (nd + 1) * rpn; ++g) {
                if (z[(size_t)e_star * EP + g] || used[g] >= r) continue;
                if (gt < 0 || tg[g] < tg[gt]) gt = g;
            }
            if (gt < 0) continue;
            memcpy(a_keep, a, sizeof(i64) * zsz);
            z[(size_t)e_star * EP + gt] = 1;
            node_split(nd, rank_of, E, EP, rpn, z, a);
            double T_try = eval_state(x, E, EP, rpn, z, a, model, tg_try, NULL);
            double S_try = 0;
            for (int g = 0; g < EP; ++g) S_try += tg_try[g] * tg_try[g];
            if (T_try < T || (T_try == T && S_try < S)) {
                T = T_try;
                S = S_try;
                memcpy(tg, tg_try, sizeof(double) * EP);
                used[gt] += 1;
                accepted = 1;
                break;
            }
            z[(size_t)e_star * EP + gt] = 0;
            memcpy(a, a_keep, sizeof(i64) * zsz);
        }
        if (!accepted) break;
    }
    for (int e = 0; e < E; ++e)
        for (int g = 0; g < EP; ++g)
            if (g != rank_of[e] && z[(size_t)e * EP + g] && a[(size_t)e * EP + g] == 0) z[(size_t)e * EP + g] = 0;
    i64 mc = 0;
    T2[1] = eval_state(x, E, EP, rpn, z, a, model, tg, &mc);
    free(used); free(tg); free(tg_try); free(a_keep); free(tried);
    return mc;
}

/* Plan tables from a placement and, per micro-batch, the placement bits zz[mb][e][g] and the   */
/* token shares aa[mb][e][g] (table layout: see oracle_plan_ex).                              */
static void emit_tables(const int32_t *counts, int n_mb, int E, int EP, int r, const int32_t *rank_of,
                        const uint8_t *zz, const i64 *aa, const i64 *mx,
                        int32_t *expert_to_slot, int32_t *replica_expert,
                        int32_t *inst_ptr, int32_t *inst_rank, int32_t *inst_rows, int32_t *inst_group,
                        int32_t *group_expert, int32_t *group_offset, i64 *max_before, i64 *max_after)
{
    int M = E / EP, G = EP * (M + r), cap_inst = E + EP * r;
    size_t zsz = (size_t)E * EP;
    /* local slots: ascending expert id within a rank */
    int *next_local = (int *)calloc(EP, sizeof(int));
    for (int e = 0; e < E; ++e) expert_to_slot[e] = rank_of[e] * M + next_local[rank_of[e]]++;
    free(next_local);

    for (int mb = 0; mb < n_mb; ++mb) {
        const uint8_t *z = zz + zsz * mb;
        const i64 *a = aa + zsz * mb;
        int32_t *rep = replica_expert + (size_t)mb * EP * r;
        int32_t *gexp = group_expert + (size_t)mb * G;
        int32_t *goff = group_offset + (size_t)mb * (G + 1);
        i64 *grow = (i64 *)calloc(G, sizeof(i64));
        for (int g = 0; g < G; ++g) gexp[g] = -1;
        for (int i = 0; i < EP * r; ++i) rep[i] = -1;
        for (int e = 0; e < E; ++e) {
            int slot = expert_to_slot[e];
            int grp = (slot / M) * (M + r) + slot % M;
            gexp[grp] = e;
            grow[grp] = a[(size_t)e * EP + rank_of[e]];
        }
        for (int g = 0; g < EP; ++g) {
            int j = 0;
            for (int e = 0; e < E; ++e)          /* ascending id fills slots in order */
                if (rank_of[e] != g && z[(size_t)e * EP + g]) {
                    rep[g * r + j] = e;
                    gexp[g * (M + r) + M + j] = e;
                    grow[g * (M + r) + M + j] = a[(size_t)e * EP + g];
                    ++j;
                }
        }
        goff[0] = 0;
        for (int g = 0; g < G; ++g) goff[g + 1] = goff[g] + (int32_t)grow[g];
        /* instances of each expert, ascending rank */
        int32_t *ip = inst_ptr + (size_t)mb * (E + 1);
        int32_t *ir = inst_rank + (size_t)mb * cap_inst;
        int32_t *iw = inst_rows + (size_t)mb * cap_inst;
        int32_t *ig = inst_group + (size_t)mb * cap_inst;
        for (int i = 0; i < cap_inst; ++i) { ir[i] = -1; iw[i] = 0; ig[i] = -1; }
        int p = 0;
        for (int e = 0; e < E; ++e) {
            ip[e] = p;
            for (int g = 0; g < EP; ++g) {
                if (!z[(size_t)e * EP + g]) continue;
                int grp = -1;
                if (g == rank_of[e]) grp = g * (M + r) + expert_to_slot[e] % M;
                else for (int j = 0; j < r; ++j) if (rep[g * r + j] == e) grp = g * (M + r) + M + j;
                ir[p] = g; iw[p] = (int32_t)a[(size_t)e * EP + g]; ig[p] = grp;
                ++p;
            }
        }
        ip[E] = p;
        free(grow);
        /* unplanned: expert e on rank e / M, no replicas */
        i64 worst = 0;
        for (int g = 0; g < EP; ++g) {
            i64 s = 0;
            for (int e = g * M; e < (g + 1) * M; ++e) s += counts[(size_t)mb * E + e];
            if (s > worst) worst = s;
        }
        max_before[mb] = worst;
        max_after[mb] = mx[mb];
    }
}

/* Whole plan (Sections 4 and 5): reorder once per batch, replicate per micro-batch, */
/* and keep the reordering only if it lowers J = sum over micro-batches of the max    */
/* rank load after replication (ties keep the unplanned layout, which moves no        */
/* expert).  Output tables:                                                           */
/*   expert_to_slot[E]           rank*M + local slot (local slots by ascending id)     */
/*   replica_expert[n_mb][EP][r] expert in each replica slot (ascending id), -1 empty  */
/*   inst_ptr[n_mb][E+1], inst_rank/rows/group[n_mb][E+EP*r]                           */
/*                               instances of each expert, ascending rank; the home    */
/*                               instance is always listed                             */
/*   group_expert[n_mb][G], group_offset[n_mb][G+1], G = EP*(M+r), rank-major:         */
/*                               M home slots then r replica slots per rank            */
/*   max_before[n_mb]            max rank load, unplanned layout, no replicas          */
/*   max_after[n_mb]             max rank load under the plan                          */
/* placed != NULL: that placement (rank per expert, M per rank) is used as it is   */
/* and only the per-micro-batch replication runs (a placement found under another */
/* objective, e.g. by the annealing of Algorithm 1).                              */
int oracle_plan_ex(const int32_t *counts, int n_mb, int E, int EP, int rpn, int r, const int32_t *placed,
                   int32_t *expert_to_slot, int32_t *replica_expert,
                   int32_t *inst_ptr, int32_t *inst_rank, int32_t *inst_rows, int32_t *inst_group,
                   int32_t *group_expert, int32_t *group_offset,
                   i64 *max_before, i64 *max_after)
{
    if (E <= 0 || EP <= 0 || E % EP || rpn <= 0 || EP % rpn || r < 0 || n_mb <= 0) return -1;
    int M = E / EP, G = EP * (M + r), cap_inst = E + EP * r;
    i64 *l = (i64 *)calloc(E, sizeof(i64));
    for (int mb = 0; mb < n_mb; ++mb)
        for (int e = 0; e < E; ++e) {
            if (counts[mb * E + e] < 0) { free(l); return -1; }
            l[e] += counts[mb * E + e];
        }
    int32_t *p_id = (int32_t *)malloc(sizeof(int32_t) * E);
    int32_t *p_new = (int32_t *)malloc(sizeof(int32_t) * E);
    for (int e = 0; e < E; ++e) p_id[e] = e / M;
    if (placed) memcpy(p_new, placed, sizeof(int32_t) * E);
    else oracle_reorder(l, E, EP, p_new);

    size_t zsz = (size_t)E * EP;
    uint8_t *z_id = (uint8_t *)malloc(zsz * n_mb), *z_new = (uint8_t *)malloc(zsz * n_mb);
    i64 *a_id = (i64 *)malloc(sizeof(i64) * zsz * n_mb), *a_new = (i64 *)malloc(sizeof(i64) * zsz * n_mb);
    i64 *mx_id = (i64 *)malloc(sizeof(i64) * n_mb), *mx_new = (i64 *)malloc(sizeof(i64) * n_mb);
    i64 J_id = 0, J_new = 0;
    for (int mb = 0; mb < n_mb; ++mb) {
        mx_id[mb] = replicate_mb(counts + (size_t)mb * E, p_id, E, EP, rpn, r, z_id + zsz * mb, a_id + zsz * mb);
        mx_new[mb] = replicate_mb(counts + (size_t)mb * E, p_new, E, EP, rpn, r, z_new + zsz * mb, a_new + zsz * mb);
        J_id += mx_id[mb]; J_new += mx_new[mb];
    }
    int use_new = placed ? 1 : (J_new < J_id);
    const int32_t *rank_of = use_new ? p_new : p_id;
    const uint8_t *zz = use_new ? z_new : z_id;
    const i64 *aa = use_new ? a_new : a_id;
    const i64 *mx = use_new ? mx_new : mx_id;

    emit_tables(counts, n_mb, E, EP, r, rank_of, zz, aa, mx, expert_to_slot, replica_expert, inst_ptr, inst_rank,
                inst_rows, inst_group, group_expert, group_offset, max_before, max_after);
    free(l); free(p_id); free(p_new); free(z_id); free(z_new); free(a_id); free(a_new);
    free(mx_id); free(mx_new);
    return 0;
}

/* Plan under a given placement with the time-aware replication above: x[mb][j][e] per-source */
/* histograms, placed[e] the rank of every expert (M per rank).  Tables as oracle_plan_ex;    */
/* t_before / t_after [n_mb]: T_MoE (Eq. 6) of every micro-batch without and with replicas.    */
int oracle_plan_comm(const i64 *x, int n_mb, int E, int EP, int rpn, int r, const int32_t *placed,
                     const double *model,
                     int32_t *expert_to_slot, int32_t *replica_expert,
                     int32_t *inst_ptr, int32_t *inst_rank, int32_t *inst_rows, int32_t *inst_group,
                     int32_t *group_expert, int32_t *group_offset,
                     i64 *max_before, i64 *max_after, double *t_before, double *t_after)
{
    if (E <= 0 || EP <= 0 || E % EP || rpn <= 0 || EP % rpn || r < 0 || n_mb <= 0 || !placed) return -1;
    size_t zsz = (size_t)E * EP;
    uint8_t *zz = (uint8_t *)malloc(zsz * n_mb);
    i64 *aa = (i64 *)malloc(sizeof(i64) * zsz * n_mb);
    i64 *mx = (i64 *)malloc(sizeof(i64) * n_mb);
    int32_t *counts = (int32_t *)malloc(sizeof(int32_t) * (size_t)n_mb * E);
    for (int mb = 0; mb < n_mb; ++mb) {
        const i64 *xm = x + (size_t)mb * EP * E;
        for (int e = 0; e < E; ++e) {
            i64 l = 0;
            for (int j = 0; j < EP; ++j) l += xm[(size_t)j * E + e];
            counts[(size_t)mb * E + e] = (int32_t)l;
        }
        double T2[2];
        mx[mb] = oracle_replicate_comm(xm, placed, E, EP, rpn, r, model, zz + zsz * mb, aa + zsz * mb, T2);
        t_before[mb] = T2[0];
        t_after[mb] = T2[1];
    }
    emit_tables(counts, n_mb, E, EP, r, placed, zz, aa, mx, expert_to_slot, replica_expert, inst_ptr, inst_rank,
                inst_rows, inst_group, group_expert, group_offset, max_before, max_after);
    free(zz); free(aa); free(mx); free(counts);
    return 0;
}

/* ------------------------------------------------------------------------- */
/* Permutation (Section 5.2, token splitting): assignment a = t*k + s of       */
/* expert e has ordinal q among the assignments of e (in ascending a); the      */
/* instances of e, in ascending rank, take consecutive runs of ordinals of the   */
/* lengths the plan gave them.  row_of[a] is the row in the group-ordered        */
/* buffer; src_of is its inverse.                                                */
int oracle_permute(const int32_t *ids, int T, int k, int E,
                   const int32_t *inst_ptr, const int32_t *inst_rows, const int32_t *inst_group,
                   const int32_t *group_offset, int32_t *row_of, int32_t *src_of)
{
    int N = T * k;
    int32_t *seen = (int32_t *)calloc(E, sizeof(int32_t));
    for (int a = 0; a < N; ++a) {
        int e = ids[a];
        if (e < 0 || e >= E) { free(seen); return -2; }
        int q = seen[e]++;
        int i = inst_ptr[e], before = 0;
        while (i < inst_ptr[e + 1] && q >= before + inst_rows[i]) { before += inst_rows[i]; ++i; }
        if (i >= inst_ptr[e + 1]) { free(seen); return -3; }   /* plan does not cover this token */
        int row = group_offset[inst_group[i]] + (q - before);
        row_of[a] = row;
        src_of[row] = a;
    }
    free(seen);
    return 0;
}

/* ------------------------------------------------------------------------- */
/* Source-aware token split (Section 5.2: y_{j,e,g}, the share of source GPU   */
/* j's tokens of expert e that GPU g serves; Section 4.1 for the link types).   */
/* The plan fixes how many tokens each instance of an expert serves (the        */
/* computation split).  Which SOURCES fill an instance is still free, and it    */
/* decides the traffic: all instances of e sit in one node, so for source j     */
/* exactly one rank of that node is "aligned" with j (j itself inside the node, */
/* the rank with j's index inside its node otherwise); a token served there     */
/* is a local copy or a same-rail transfer, served anywhere else in the node    */
/* it crosses the intra-node link once more.  RDMA volume does not depend on    */
/* the choice.  Per expert:                                                     */
/*   1. every instance takes tokens of its own rank (local copies);             */
/*   2. every instance, ascending, takes tokens of the other sources aligned    */
/*      with it, ascending source;                                              */
/*   3. what is left goes source by source (ascending) to the instances that    */
/*      still have room (ascending).                                            */
/* Steps 1-2 give every instance min(room, aligned tokens): the aligned sets of  */
/* different instances are disjoint, so the number of tokens that cross the      */
/* intra-node link is the smallest any split with these instance sizes can have. */
/* y[i*EP + j] = tokens of source j served by instance i (CSR order of the plan). */
/* returns 0, or -3 if an expert's instance sizes do not add up to its tokens.   */
int oracle_assign_sources(const i64 *x, int E, int EP, int rpn, const int32_t *inst_ptr,
                          const int32_t *inst_rank, const int32_t *inst_rows, i64 *y)
{
    i64 *left = (i64 *)malloc(sizeof(i64) * EP);
    for (int e = 0; e < E; ++e) {
        int lo = inst_ptr[e], hi = inst_ptr[e + 1];
        i64 have = 0, want = 0;
        for (int j = 0; j < EP; ++j) { left[j] = x[(size_t)j * E + e]; have += left[j]; }
        for (int i = lo; i < hi; ++i) {
            want += inst_rows[i];
            for (int j = 0; j < EP; ++j) y[(size_t)i * EP + j] = 0;
        }
        if (have != want) { free(left); return -3; }
        i64 *room = (i64 *)malloc(sizeof(i64) * (hi - lo + 1));
        for (int i = lo; i < hi; ++i) room[i - lo] = inst_rows[i];
        for (int i = lo; i < hi; ++i) {                      /* 1: local copies */
            int j = inst_rank[i];
            i64 m = left[j] < room[i - lo] ? left[j] : room[i - lo];
            y[(size_t)i * EP + j] += m; left[j] -= m; room[i - lo] -= m;
        }
        for (int i = lo; i < hi; ++i)                        /* 2: same rail, other nodes */
            for (int j = 0; j < EP; ++j) {
                if (oracle_tau(j, inst_rank[i], rpn) != 2) continue;
                i64 m = left[j] < room[i - lo] ? left[j] : room[i - lo];
                y[(size_t)i * EP + j] += m; left[j] -= m; room[i - lo] -= m;
            }
        for (int j = 0; j < EP; ++j)                         /* 3: the rest */
            for (int i = lo; i < hi; ++i) {
                i64 m = left[j] < room[i - lo] ? left[j] : room[i - lo];
                y[(size_t)i * EP + j] += m; left[j] -= m; room[i - lo] -= m;
            }
        free(room);
    }
    free(left);
    return 0;
}

/* Loads (Eq. 1-3) and times (Eq. 4-6) of a micro-batch under a split y: instance i  */
/* on rank inst_rank[i] serves y[i][j] tokens of source j.  model as in             */
/* oracle_moe_time; out[0] = T_MoE, out[1] = max T_comp, out[2] = max T_comm;        */
/* loads[5][EP] = computation, intra-node send, receive, RDMA send, receive (tokens). */
void oracle_moe_time_split(const i64 *y, int n_inst, int EP, int rpn, const int32_t *inst_rank,
                           const double *model, double *out, i64 *loads)
{
    i64 *comp = loads, *nv_tx = loads + EP, *nv_rx = loads + 2 * EP, *rd_tx = loads + 3 * EP, *rd_rx = loads + 4 * EP;
    for (int g = 0; g < 5 * EP; ++g) loads[g] = 0;
    for (int i = 0; i < n_inst; ++i) {
        int g = inst_rank[i];
        if (g < 0) continue;
        for (int j = 0; j < EP; ++j) {
            i64 n = y[(size_t)i * EP + j];
            int tau = oracle_tau(j, g, rpn);
            comp[g] += n;
            if (tau == 1 || tau == 3) { nv_tx[j] += n; nv_rx[g] += n; }
            if (tau == 2 || tau == 3) { rd_tx[j] += n; rd_rx[g] += n; }
        }
    }
    double tc = 0, tm = 0;
    for (int g = 0; g < EP; ++g) {
        double c = model[0] * (double)comp[g];
        double nv = model[1] * (double)(nv_tx[g] > nv_rx[g] ? nv_tx[g] : nv_rx[g]);
        double rd = model[2] * (double)(rd_tx[g] > rd_rx[g] ? rd_tx[g] : rd_rx[g]);
        double m = nv > rd ? nv : rd;
        if (c > tc) tc = c;
        if (m > tm) tm = m;
    }
    out[0] = tc + tm; out[1] = tc; out[2] = tm;
}

/* Permutation under a source-aware split: assignment a = t*k + s, token t on source  */
/* j = t / (T/EP), expert e, ordinal q among the assignments of (j, e) in ascending a. */
/* The instances of e (CSR order) take runs of y[i][j] ordinals of source j; inside   */
/* instance i the rows are laid out source after source.                              */
int oracle_permute_src(const int32_t *ids, int T, int k, int E, int EP,
                       const int32_t *inst_ptr, const int32_t *inst_group, const int32_t *group_offset,
                       const i64 *y, int32_t *row_of, int32_t *src_of)
{
    int N = T * k;
    if (EP < 1 || T % EP) return -1;
    int per = T / EP;
    int32_t *seen = (int32_t *)calloc((size_t)EP * E, sizeof(int32_t));
    for (int a = 0; a < N; ++a) {
        int e = ids[a], j = (a / k) / per;
        if (e < 0 || e >= E) { free(seen); return -2; }
        int q = seen[(size_t)j * E + e]++;
        int i = inst_ptr[e];
        i64 before = 0;
        while (i < inst_ptr[e + 1] && q >= before + y[(size_t)i * EP + j]) { before += y[(size_t)i * EP + j]; ++i; }
        if (i >= inst_ptr[e + 1]) { free(seen); return -3; }
        i64 base = 0;
        for (int jj = 0; jj < j; ++jj) base += y[(size_t)i * EP + jj];
        int row = group_offset[inst_group[i]] + (int)(base + (q - before));
        row_of[a] = row;
        src_of[row] = a;
    }
    free(seen);
    return 0;
}

/* ------------------------------------------------------------------------- */
/* Floating point.  bf16 bit patterns widen exactly to double.                */
static inline double bf(uint16_t b)
{
    uint32_t u = (uint32_t)b << 16; float f; memcpy(&f, &u, 4); return (double)f;
}
static inline double sigmoid(double x) { return 1.0 / (1.0 + exp(-x)); }

/* Gather of token rows into group order: Xrows[row] = X[src_of[row] / k] (bit copy). */
void oracle_gather_rows(const uint16_t *X, const int32_t *src_of, int N, int k, int h, uint16_t *Xrows)
{
    for (int row = 0; row < N; ++row)
        memcpy(Xrows + (size_t)row * h, X + (size_t)(src_of[row] / k) * h, sizeof(uint16_t) * h);
}

/* Layer-shared replica buffer, forward push (Section 5.1): W holds n_home + n_slots parameter   */
/* blocks of block_elems bf16 values; slot s with replica_expert[s] = e >= 0 receives a copy of  */
/* block e at block n_home + s; empty slots (-1) keep whatever they held.                        */
void oracle_replica_push(uint16_t *W, const int32_t *replica_expert, int n_home, int n_slots, size_t block_elems)
{
    for (int s = 0; s < n_slots; ++s) {
        int e = replica_expert[s];
        if (e < 0) continue;
        for (size_t i = 0; i < block_elems; ++i)
            W[(size_t)(n_home + s) * block_elems + i] = W[(size_t)e * block_elems + i];
    }
}

/* Expert FFN forward over groups [g_begin, g_end) (Section 4.1: three GEMMs of   */
/* 2hh' flops per token).  For a row x of a group whose expert is e:              */
/*   Gt = Wg_e x, U = Wu_e x, A = silu(Gt) * U, y = Wd_e A.                        */
/* Wg, Wu: [E][h'][h]; Wd: [E][h][h'].  Outputs are double, no rounding between.   */
void oracle_ffn_fwd(const uint16_t *Xrows, const int32_t *group_offset, const int32_t *group_expert,
                    int g_begin, int g_end, const uint16_t *Wg, const uint16_t *Wu, const uint16_t *Wd,
                    int h, int hff, double *Gt, double *U, double *A, double *Y)
{
    for (int g = g_begin; g < g_end; ++g) {
        int e = group_expert[g];
        if (e < 0) continue;
        const uint16_t *wg = Wg + (size_t)e * hff * h, *wu = Wu + (size_t)e * hff * h;
        const uint16_t *wd = Wd + (size_t)e * h * hff;
        #pragma omp parallel for schedule(static)
        for (int row = group_offset[g]; row < group_offset[g + 1]; ++row) {
            const uint16_t *x = Xrows + (size_t)row * h;
            for (int j = 0; j < hff; ++j) {
                double sg = 0.0, su = 0.0;
                for (int i = 0; i < h; ++i) {
                    double xi = bf(x[i]);
                    sg += xi * bf(wg[(size_t)j * h + i]);
                    su += xi * bf(wu[(size_t)j * h + i]);
                }
                Gt[(size_t)row * hff + j] = sg;
                U[(size_t)row * hff + j] = su;
                A[(size_t)row * hff + j] = sg * sigmoid(sg) * su;
            }
            for (int i = 0; i < h; ++i) {
                double s = 0.0;
                for (int j = 0; j < hff; ++j) s += A[(size_t)row * hff + j] * bf(wd[(size_t)i * hff + j]);
                Y[(size_t)row * h + i] = s;
            }
        }
    }
}

/* Expert FFN backward over groups [g_begin, g_end).  With dy the upstream         */
/* gradient of a row:                                                              */
/*   dA = Wd_e^T dy;  dGt = dA * U * silu'(Gt);  dU = dA * silu(Gt);                */
/*   dx = Wg_e^T dGt + Wu_e^T dU;                                                   */
/*   dWd_e += dy A^T;  dWg_e += dGt x^T;  dWu_e += dU x^T                            */
/* summed over every group (home or replica) of expert e in the range (Section 5.1:  */
/* replica gradients are pushed back and accumulated on the home copy).              */
/* dWg, dWu: [E][h'][h]; dWd: [E][h][h']; all zeroed here first.                     */
void oracle_ffn_bwd(const uint16_t *Xrows, const uint16_t *dYrows,
                    const int32_t *group_offset, const int32_t *group_expert,
                    int g_begin, int g_end, int E,
                    const uint16_t *Wg, const uint16_t *Wu, const uint16_t *Wd, int h, int hff,
                    double *dXrows, double *dWg, double *dWu, double *dWd)
{
    size_t wsz = (size_t)E * h * hff;
    memset(dWg, 0, sizeof(double) * wsz);
    memset(dWu, 0, sizeof(double) * wsz);
    memset(dWd, 0, sizeof(double) * wsz);
    for (int g = g_begin; g < g_end; ++g) {
        int e = group_expert[g];
        if (e < 0) continue;
        int r0 = group_offset[g], n = group_offset[g + 1] - r0;
        if (n <= 0) continue;
        const uint16_t *wg = Wg + (size_t)e * hff * h, *wu = Wu + (size_t)e * hff * h;
        const uint16_t *wd = Wd + (size_t)e * h * hff;
        double *Gt = (double *)malloc(sizeof(double) * (size_t)n * hff);
        double *U = (double *)malloc(sizeof(double) * (size_t)n * hff);
        double *Aa = (double *)malloc(sizeof(double) * (size_t)n * hff);
        double *dGt = (double *)malloc(sizeof(double) * (size_t)n * hff);
        double *dU = (double *)malloc(sizeof(double) * (size_t)n * hff);
        #pragma omp parallel for schedule(static)
        for (int q = 0; q < n; ++q) {
            const uint16_t *x = Xrows + (size_t)(r0 + q) * h;
            const uint16_t *dy = dYrows + (size_t)(r0 + q) * h;
            for (int j = 0; j < hff; ++j) {
                double sg = 0.0, su = 0.0, da = 0.0;
                for (int i = 0; i < h; ++i) {
                    double xi = bf(x[i]);
                    sg += xi * bf(wg[(size_t)j * h + i]);
                    su += xi * bf(wu[(size_t)j * h + i]);
                    da += bf(dy[i]) * bf(wd[(size_t)i * hff + j]);
                }
                double sig = sigmoid(sg);
                size_t o = (size_t)q * hff + j;
                Gt[o] = sg; U[o] = su; Aa[o] = sg * sig * su;
                dGt[o] = da * su * (sig * (1.0 + sg * (1.0 - sig)));
                dU[o] = da * (sg * sig);
            }
            for (int i = 0; i < h; ++i) {
                double s = 0.0;
                for (int j = 0; j < hff; ++j)
                    s += dGt[(size_t)q * hff + j] * bf(wg[(size_t)j * h + i])
                       + dU[(size_t)q * hff + j] * bf(wu[(size_t)j * h + i]);
                dXrows[(size_t)(r0 + q) * h + i] = s;
            }
        }
        double *gg = dWg + (size_t)e * hff * h, *gu = dWu + (size_t)e * hff * h;
        double *gd = dWd + (size_t)e * h * hff;
        #pragma omp parallel for schedule(static)
        for (int j = 0; j < hff; ++j)
            for (int i = 0; i < h; ++i) {
                double s1 = 0.0, s2 = 0.0;
                for (int q = 0; q < n; ++q) {
                    double xi = bf(Xrows[(size_t)(r0 + q) * h + i]);
                    s1 += dGt[(size_t)q * hff + j] * xi;
                    s2 += dU[(size_t)q * hff + j] * xi;
                }
                gg[(size_t)j * h + i] += s1;
                gu[(size_t)j * h + i] += s2;
            }
        #pragma omp parallel for schedule(static)
        for (int i = 0; i < h; ++i)
            for (int j = 0; j < hff; ++j) {
                double s = 0.0;
                for (int q = 0; q < n; ++q)
                    s += bf(dYrows[(size_t)(r0 + q) * h + i]) * Aa[(size_t)q * hff + j];
                gd[(size_t)i * hff + j] += s;
            }
        free(Gt); free(U); free(Aa); free(dGt); free(dU);
    }
}

/* Unpermute + gate-weighted combine (Section 2.1: the outputs of a token's selected */
/* experts are combined): Out[t] = sum_s gate[t][s] * Yrows[row_of[t*k+s]].           */
/* gates == NULL means every gate is 1 (the backward of the row gather).              */
void oracle_combine_fwd(const double *Yrows, const float *gates, const int32_t *row_of,
                        int T, int k, int h, double *Out)
{
    for (int t = 0; t < T; ++t)
        for (int i = 0; i < h; ++i) {
            double s = 0.0;
            for (int j = 0; j < k; ++j) {
                double gt = gates ? (double)gates[t * k + j] : 1.0;
                s += gt * Yrows[(size_t)row_of[t * k + j] * h + i];
            }
            Out[(size_t)t * h + i] = s;
        }
}

/* Backward of the combine: dYrows[row] = gate * dOut[t]; dgate[t][s] = <dOut[t], Yrows[row]>. */
void oracle_combine_bwd(const double *dOut, const double *Yrows, const float *gates,
                        const int32_t *row_of, int T, int k, int h, double *dYrows, double *dgate)
{
    for (int t = 0; t < T; ++t)
        for (int j = 0; j < k; ++j) {
            size_t row = (size_t)row_of[t * k + j];
            double gt = (double)gates[t * k + j], dot = 0.0;
            for (int i = 0; i < h; ++i) {
                dYrows[row * h + i] = gt * dOut[(size_t)t * h + i];
                dot += dOut[(size_t)t * h + i] * Yrows[row * h + i];
            }
            dgate[t * k + j] = dot;
        }
}

/* Threads the row loops above run on (for reporting beside timings). */
int oracle_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* The plan with stage 1 run by the oracle itself. */
int oracle_plan(const int32_t *counts, int n_mb, int E, int EP, int rpn, int r,
                int32_t *expert_to_slot, int32_t *replica_expert,
                int32_t *inst_ptr, int32_t *inst_rank, int32_t *inst_rows, int32_t *inst_group,
                int32_t *group_expert, int32_t *group_offset,
                i64 *max_before, i64 *max_after)
{
    return oracle_plan_ex(counts, n_mb, E, EP, rpn, r, NULL, expert_to_slot, replica_expert, inst_ptr, inst_rank,
                          inst_rows, inst_group, group_expert, group_offset, max_before, max_after);
}
