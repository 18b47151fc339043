// Source-aware token split (paper Section 5.2: y_{j,e,g}, the share of source rank j's tokens
// of expert e that rank g serves) and the cost model of Section 4.1 (Eq. 1-6) evaluated on a
// split, host side.
//
// The plan fixes the size of every instance of an expert; this file decides which SOURCES fill
// which instance.  All instances of an expert sit in one node.  Seen from a source rank j,
// exactly one rank of that node is cheap: j itself when j is in the node (local copy, no link),
// otherwise the rank with j's index inside its node (same rail: RDMA only).  Any other instance
// costs one more crossing of the intra-node link; the RDMA volume is the same either way.  So an
// instance first takes what its own rank holds, then what the other sources on its rail hold,
// and only the remainder is dealt out in source order.  Because the cheap sources of different
// instances do not overlap, this reaches the smallest intra-node volume any split with the same
// instance sizes can have.
#include "../../include/relibra.h"

#include <algorithm>
#include <cstdint>
#include <vector>

namespace {

using i64 = long long;

struct Topology {
    int EP, rpn;
    bool local(int src, int dst) const { return src == dst; }
    bool same_node(int src, int dst) const { return src / rpn == dst / rpn; }
    bool same_rail(int src, int dst) const { return src % rpn == dst % rpn; }
    bool uses_intra(int src, int dst) const { return src != dst && (same_node(src, dst) || !same_rail(src, dst)); }
    bool uses_rdma(int src, int dst) const { return !same_node(src, dst); }
};

bool model_ok(const relibra_cost_model *m)
{
    return m && m->EP >= 1 && m->ranks_per_node >= 1 && m->EP % m->ranks_per_node == 0 &&
           m->sec_per_token_comp >= 0 && m->sec_per_token_intra >= 0 && m->sec_per_token_inter >= 0;
}

}  // namespace

extern "C" int relibra_assign_sources(const int64_t *x_host, int E, int EP, int ranks_per_node,
                                      const int32_t *inst_ptr, const int32_t *inst_rank, const int32_t *inst_rows,
                                      int32_t *src_first, int32_t *inst_src_rows, int32_t *inst_src_base)
{
    if (E < 1 || EP < 1 || ranks_per_node < 1 || EP % ranks_per_node) return RELIBRA_EINVAL;
    if (!x_host || !inst_ptr || !inst_rank || !inst_rows || !src_first || !inst_src_rows || !inst_src_base)
        return RELIBRA_EINVAL;
    const Topology topo{EP, ranks_per_node};
    if (inst_ptr[0] != 0) return RELIBRA_ERANGE;
    std::vector<i64> left(EP), room;
    for (int e = 0; e < E; ++e) {
        const int lo = inst_ptr[e], hi = inst_ptr[e + 1];
        if (hi < lo) return RELIBRA_ERANGE;
        i64 have = 0, want = 0;
        for (int j = 0; j < EP; ++j) {
            left[j] = x_host[(size_t)j * E + e];
            if (left[j] < 0 || have + left[j] > 0x7fffffffLL) return RELIBRA_ERANGE;
            src_first[(size_t)j * E + e] = (int32_t)have;       // ordinal of source j's first token of e
            have += left[j];
        }
        room.assign(hi - lo, 0);
        for (int i = lo; i < hi; ++i) {
            if (inst_rows[i] < 0 || inst_rank[i] < 0 || inst_rank[i] >= EP) return RELIBRA_ERANGE;
            room[i - lo] = inst_rows[i];
            want += inst_rows[i];
            std::fill(inst_src_rows + (size_t)i * EP, inst_src_rows + (size_t)(i + 1) * EP, 0);
        }
        if (have != want) return RELIBRA_ERANGE;
        auto take = [&](int i, int j) {
            const i64 m = std::min(left[j], room[i - lo]);
            inst_src_rows[(size_t)i * EP + j] += (int32_t)m;
            left[j] -= m;
            room[i - lo] -= m;
        };
        for (int i = lo; i < hi; ++i) take(i, inst_rank[i]);                     // its own rank's tokens
        for (int i = lo; i < hi; ++i)                                            // its rail in the other nodes
            for (int j = inst_rank[i] % ranks_per_node; j < EP; j += ranks_per_node)
                if (!topo.same_node(j, inst_rank[i])) take(i, j);
        for (int j = 0; j < EP; ++j)                                             // the remainder, in source order
            for (int i = lo; i < hi && left[j] > 0; ++i) take(i, j);
        for (int i = lo; i < hi; ++i) {
            int32_t run = 0;
            for (int j = 0; j < EP; ++j) {
                inst_src_base[(size_t)i * EP + j] = run;
                run += inst_src_rows[(size_t)i * EP + j];
            }
        }
    }
    return RELIBRA_OK;
}

extern "C" int relibra_moe_time_split(const int32_t *inst_src_rows, int n_inst, const int32_t *inst_rank,
                                      const relibra_cost_model *model, double *out3, int64_t *loads_out)
{
    if (!model_ok(model) || n_inst < 0 || !out3 || (n_inst > 0 && (!inst_src_rows || !inst_rank))) return RELIBRA_EINVAL;
    const int EP = model->EP;
    const Topology topo{EP, model->ranks_per_node};
    std::vector<i64> load(5 * (size_t)EP, 0);
    i64 *comp = load.data(), *intra_tx = comp + EP, *intra_rx = comp + 2 * EP, *rdma_tx = comp + 3 * EP, *rdma_rx = comp + 4 * EP;
    for (int i = 0; i < n_inst; ++i) {
        const int g = inst_rank[i];
        if (g < 0) continue;                                   // unused tail of the instance table
        if (g >= EP) return RELIBRA_ERANGE;
        for (int j = 0; j < EP; ++j) {
            const i64 n = inst_src_rows[(size_t)i * EP + j];
            if (n < 0) return RELIBRA_ERANGE;
            comp[g] += n;
            if (topo.uses_intra(j, g)) { intra_tx[j] += n; intra_rx[g] += n; }
            if (topo.uses_rdma(j, g)) { rdma_tx[j] += n; rdma_rx[g] += n; }
        }
    }
    double t_comp = 0, t_comm = 0;
    for (int g = 0; g < EP; ++g) {
        t_comp = std::max(t_comp, model->sec_per_token_comp * (double)comp[g]);
        const double intra = model->sec_per_token_intra * (double)std::max(intra_tx[g], intra_rx[g]);
        const double rdma = model->sec_per_token_inter * (double)std::max(rdma_tx[g], rdma_rx[g]);
        t_comm = std::max(t_comm, std::max(intra, rdma));
    }
    out3[0] = t_comp + t_comm;
    out3[1] = t_comp;
    out3[2] = t_comm;
    if (loads_out) std::copy(load.begin(), load.end(), loads_out);
    return RELIBRA_OK;
}
