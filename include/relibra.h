/*
 * relibra.h -- C ABI of the replay-guided MoE expert-layer path for one AMD MI355X (gfx950).
 *
 * The path: replayed top-k routing ids -> per-expert load histogram -> inter-batch expert
 * reordering + intra-batch expert replication plan -> token permutation into
 * expert/replica-grouped rows -> SwiGLU expert FFN forward / backward as grouped bf16 MFMA
 * GEMMs -> unpermute + gate-weighted combine.  "Simulated EP": the groups of every
 * expert-parallel rank live on the one GPU; a [g_begin, g_end) range selects one rank's share.
 *
 * Conventions
 *  - Every pointer is marked "dev" (device memory, the caller's allocation) or "host".
 *    The library allocates no device memory and keeps no state between calls that affects
 *    results (process-wide and set once, thread-safely: the kernels' LDS size attributes; the
 *    optional launch timing of relibra_prof_* is process-global and not thread-safe).
 *  - Device work is enqueued on `stream` (a hipStream_t) and not waited for.  Only
 *    relibra_plan is synchronous: it is host code with host inputs and outputs.
 *  - bf16 tensors are passed as `void*` to 2-byte elements, row-major, last index contiguous.
 *  - Return value: RELIBRA_OK or a negative status.  Bad contents of device tables are
 *    found by the kernels themselves: they skip the offending work (no out-of-bounds access)
 *    and OR a bit into *err_flag_dev, which the caller zeroes beforehand and reads back when
 *    it next synchronises.
 *  - Notation follows the paper: E experts, top-k, T tokens per micro-batch, N = T*k routed
 *    rows, EP ranks, M = E/EP home experts per rank, r replica slots per rank,
 *    G = EP*(M+r) groups (rank-major: M home slots then r replica slots per rank),
 *    h hidden size, hff = h' expert intermediate size.
 */
#ifndef RELIBRA_H
#define RELIBRA_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef void *relibra_stream;

enum {
    RELIBRA_OK = 0,
    RELIBRA_EINVAL = -1,      /* a size or pointer argument is unusable                   */
    RELIBRA_ERANGE = -2,      /* a host table holds a value outside its range             */
    RELIBRA_EWORKSPACE = -3,  /* workspace_bytes is below relibra_workspace_bytes(...)    */
    RELIBRA_EHIP = -4,        /* a HIP runtime call failed                                */
    RELIBRA_EUNSUPPORTED = -5 /* shape outside what the kernels are built for             */
};

/* bits OR-ed into *err_flag_dev by kernels */
enum {
    RELIBRA_ERR_ID_RANGE = 1,    /* an expert id outside [0,E)                               */
    RELIBRA_ERR_PLAN_COVER = 2,  /* plan tables do not cover an assignment (permute)         */
    RELIBRA_ERR_GROUP_TABLE = 4  /* group_offset / group_expert / dw_slot tables inconsistent */
};

/* which = */
enum { RELIBRA_WS_PERMUTE = 0, RELIBRA_WS_FFN_FWD = 1, RELIBRA_WS_FFN_BWD = 2, RELIBRA_WS_WGRAD_BATCHED = 3,
       RELIBRA_WS_DGATE = 4 };

/* flags of relibra_moe_ffn_bwd */
enum {
    RELIBRA_BWD_ACCUMULATE = 1,     /* home dW += this micro-batch's gradient (else overwrite) */
    RELIBRA_BWD_NO_REPLICA_SUM = 2, /* leave replica-slot dW where it is (partial group range) */
    RELIBRA_BWD_REPLICA_WEIGHTS = 4, /* a group reads its parameters from slot group_dw_slot[g] of
                                       Wg/Wu/Wd [n_dw_slots, ...] (filled by relibra_replica_push) */
    RELIBRA_BWD_DEFER_WGRAD = 8,    /* data gradients only: dW untouched (dW and Xrows may be NULL);
                                       dGt, dU stay in the workspace for relibra_moe_ffn_wgrad_batched */
    RELIBRA_BWD_TRANSPOSED_WEIGHTS = 16 /* Wg, Wu are given as [., h, hff] and Wd as [., hff, h]:
                                       transposed copies (relibra_transpose_experts), which put the
                                       data gradients' contraction index contiguous in memory */
};

/* modes of relibra_unpermute_combine */
enum { RELIBRA_COMBINE_FWD = 0, RELIBRA_COMBINE_BWD = 1, RELIBRA_COMBINE_SUM = 2 };

/*
 * Per-expert load histogram (paper Eq. 1: l_e = tokens routed to expert e), one histogram per
 * micro-batch in a single launch.
 *   ids_dev    [n_mb, T, k] int32, dev, in   replayed top-k expert ids (Section 2.3)
 *   counts_dev [n_mb, E]    int32, dev, out  overwritten
 *   err_flag_dev            int32, dev, in/out  RELIBRA_ERR_ID_RANGE on an id outside [0,E);
 *                                              such ids are not counted
 * One workgroup per micro-batch counts in LDS and stores the finished histogram (no zero-fill pass,
 * no global atomics); the launch is bandwidth-bound when it covers many micro-batches, e.g. the
 * replayed routing of every layer, ids [layers * n_mb, T, k], in one call.
 * Limits: 1 <= E <= 4096, 1 <= k <= E.  Empty input (n_mb*T == 0) is a no-op on counts of size 0,
 * or zeroes counts when only T == 0.
 */
int relibra_route_hist(const int32_t *ids_dev, int n_mb, int T, int k, int E,
                       int32_t *counts_dev, int32_t *err_flag_dev, relibra_stream stream);

/*
 * Load-balancing plan (paper Section 4: inter-batch expert reordering, Algorithm 1 with a
 * deterministic steepest swap descent in place of random annealing moves; Section 5.2:
 * intra-batch expert replication, Algorithm 2, with the token-split LP solved exactly in
 * integers).  Objective: computation load only (Eq. 1), i.e. the largest number of routed rows
 * any rank serves.  All pointers are HOST memory; the call is synchronous and deterministic.
 *
 *   counts_host      [n_mb, E] int32  in   histograms of one training batch
 *   ranks_per_node                    in   replicas stay inside a node (Section 5.2, G(e))
 *   r                                 in   replica slots per rank (Eq. 11)
 *   expert_to_slot   [E]              out  rank*M + local slot (local slots by ascending id);
 *                                          the same for every micro-batch of the batch
 *   replica_expert   [n_mb, EP, r]    out  expert held by each replica slot (ascending id), -1 empty
 *   inst_ptr         [n_mb, E+1]      out  CSR over experts into the three inst_* tables
 *   inst_rank/rows/group [n_mb, E+EP*r] out instances of each expert in ascending rank: rank,
 *                                          rows served (the integer token split), group index;
 *                                          the home instance is always listed; unused tail = -1/0/-1
 *   group_expert     [n_mb, G]        out  expert of each group, -1 for an empty replica slot
 *   group_offset     [n_mb, G+1]      out  exclusive prefix sum of rows per group; [G] = T*k
 *   group_dw_slot    [n_mb, G]        out  weight-gradient slot of the group: e for a home group,
 *                                          E + rank*r + j for replica slot j of a rank
 *   max_load_before  [n_mb] int64     out  largest rank load, unplanned layout (e on rank e/M)
 *   max_load_after   [n_mb] int64     out  largest rank load under the plan
 * The reordering is kept only if it lowers sum_mb max_load_after; otherwise experts stay put.
 * Errors: RELIBRA_EINVAL unless E % EP == 0, EP % ranks_per_node == 0, 1 <= k <= E, r >= 0,
 * n_mb >= 1; RELIBRA_ERANGE on a negative count.
 */
int relibra_plan(const int32_t *counts_host, int n_mb, int E, int k, int EP, int ranks_per_node, int r,
                 int32_t *expert_to_slot, int32_t *replica_expert,
                 int32_t *inst_ptr, int32_t *inst_rank, int32_t *inst_rows, int32_t *inst_group,
                 int32_t *group_expert, int32_t *group_offset, int32_t *group_dw_slot,
                 int64_t *max_load_before, int64_t *max_load_after);

/*
 * The same plan with the expert placement given by the caller: stage 1 is skipped, stage 2
 * (Algorithm 2, per micro-batch) runs under expert_rank.  For placements found with another
 * objective, e.g. relibra_reorder_sa.
 *   expert_rank [E] int32 host in: rank of each expert, exactly E/EP experts per rank
 *                                  (else RELIBRA_ERANGE)
 * Everything else as relibra_plan.
 */
int relibra_plan_placed(const int32_t *counts_host, int n_mb, int E, int k, int EP, int ranks_per_node, int r,
                        const int32_t *expert_rank,
                        int32_t *expert_to_slot, int32_t *replica_expert,
                        int32_t *inst_ptr, int32_t *inst_rank, int32_t *inst_rows, int32_t *inst_group,
                        int32_t *group_expert, int32_t *group_offset, int32_t *group_dw_slot,
                        int64_t *max_load_before, int64_t *max_load_after);

/*
 * Imbalance diagnostics of Section 2.2, from the per-micro-batch histograms (all pointers HOST):
 *   skewness[mb]     = largest expert load / mean expert load of the micro-batch (1 when empty)
 *   intersection[mb] = |H_mb ∩ H_mb+1| / top, H = the `top` highest-load experts (ties: lower id),
 *                      for mb = 0 .. n_mb-2 (may be NULL when n_mb == 1)
 * For several layers pass their histograms one after the other (relibra_route_hist takes
 * ids of [layers * n_mb, T, k] in one launch) and read the ratios within each layer's block.
 */
int relibra_load_stats(const int32_t *counts_host, int n_mb, int E, int top,
                       double *skewness, double *intersection);

/*
 * Cost model of the MoE module on a rail-optimised cluster (Section 4.1).  A token on source
 * rank j routed to an expert on rank g is a local copy (j == g), crosses the intra-node link
 * (same node), RDMA on the same rail (other node, same index inside the node) or both
 * (cross rail: relayed over the intra-node link first).  Times per routed token:
 *   sec_per_token_comp  = 6 h h' / F                      (Eq. 4)
 *   sec_per_token_intra = bytes per token / B_intra-node  (Eq. 5; 2h bytes for bf16)
 *   sec_per_token_inter = bytes per token / B_rdma
 */
typedef struct relibra_cost_model {
    int EP, ranks_per_node;
    double sec_per_token_comp, sec_per_token_intra, sec_per_token_inter;
} relibra_cost_model;

/*
 * Fill the model from the quantities of Eq. 4-5: h, hff = h', F = effective FLOP/s of the expert
 * GEMMs, B_intra / B_inter = bytes per second of the intra-node link and of RDMA, bytes_per_value
 * = 2 for bf16 activations.  RELIBRA_EINVAL on a non-positive argument or EP % ranks_per_node != 0.
 */
int relibra_cost_model_init(relibra_cost_model *model_host, int EP, int ranks_per_node, int h, int hff,
                            double F, double B_intra, double B_inter, int bytes_per_value);

/*
 * Evaluate the model for one placement (Eq. 1-6).  All pointers HOST.
 *   x_host      [EP, E] int64 in   tokens on source rank j routed to expert e (token t of a
 *                                  micro-batch sits on rank t / (T/EP): relibra_route_hist on
 *                                  ids viewed as [n_mb*EP, T/EP, k] yields it)
 *   expert_rank [E] int32 in       rank hosting each expert
 *   out4        [4] double out     T_MoE = max comp + max comm (Eq. 6), max_g T_comp (Eq. 4),
 *                                  max_g T_comm (Eq. 5), and the smoothed objective of Section 4.2
 *                                  (every max replaced by LSE_beta, times divided by t_ref)
 *   loads_out   [5, EP] int64 out or NULL: computation load (Eq. 1), intra-node send, receive
 *                                  (Eq. 2-3), RDMA send, receive, in tokens
 */
int relibra_moe_time(const int64_t *x_host, int E, const relibra_cost_model *model,
                     const int32_t *expert_rank, double beta, double t_ref,
                     double *out4, int64_t *loads_out);

/*
 * Algorithm 1: swap-based simulated annealing from the greedy-LPT placement under the smoothed
 * objective (Section 4.2), n_seeds independent runs in parallel threads, best final placement by
 * the exact T_MoE (ties: lower seed).  The paper does not publish gamma, epsilon, the seed set or
 * the generator: gamma, eps (on the smoothed objective, whose scale is the start's T_MoE = 1),
 * n_seeds and seed are arguments; draws come from splitmix64 started at
 * seed + s * 0xD1342543DE82EF95 for seed index s, three per iteration (e_a, e_b, u); a worse
 * state is accepted with probability exp(-(T' - T)/theta).  Deterministic for given arguments.
 *   expert_rank_out [E] int32 out; stats5 [5] double out: exact T_MoE of the start, of the
 *   result, smoothed objective of the start, of the result, iterations per seed.
 */
int relibra_reorder_sa(const int64_t *x_host, int E, const relibra_cost_model *model,
                       double beta, double gamma, double eps, int n_seeds, uint64_t seed,
                       int32_t *expert_rank_out, double *stats5);

/*
 * One seed's run of Algorithm 1 (generator started at `seed`: what relibra_reorder_sa runs for seed
 * index 0) with its trajectory written out, for checking the acceptance rule, the cooling and the
 * order of the random draws step by step.  All pointers HOST.
 *   moves_out [trace_cap, 3] int32: e_a, e_b, accepted (0/1) of the first trace_cap iterations
 *   vals_out  [trace_cap, 3] double: u, the smoothed objective T' of the swapped state, theta
 *   start_rank_out [E]: the greedy-LPT start; expert_rank_out [E]: the run's best placement
 *   stats2 [2]: the start's exact T_MoE (every time is divided by it before smoothing), its
 *   smoothed objective (= the first theta)
 * Returns the number of iterations (>= 0) or a negative status.
 */
long long relibra_reorder_sa_trace(const int64_t *x_host, int E, const relibra_cost_model *model,
                                   double beta, double gamma, double eps, uint64_t seed,
                                   int trace_cap, int32_t *moves_out, double *vals_out,
                                   int32_t *start_rank_out, int32_t *expert_rank_out, double *stats2);

/*
 * Token permutation of one micro-batch (Section 5.2, token splitting; the local half of the
 * dispatch all-to-all, Section 2.1).  Assignment a = t*k + s with expert e = ids[a] has
 * ordinal q among e's assignments in ascending a; the instances of e, in ascending rank, take
 * consecutive runs of ordinals of inst_rows length; the assignment lands on row
 * group_offset[inst_group[i]] + (q - rows of earlier instances).
 *   ids_dev [T,k]; inst_ptr_dev [E+1]; inst_rows_dev, inst_group_dev [>= inst_ptr[E]];
 *   group_offset_dev [G+1]: one micro-batch's slices of the plan tables, dev, in
 *   X_dev      [T, h] bf16, dev, in  (may be NULL together with Xrows_dev: indices only)
 *   row_of_dev [N] int32, dev, out   assignment -> row
 *   src_of_dev [N] int32, dev, out   row -> assignment (inverse)
 *   Xrows_dev  [N, h] bf16, dev, out Xrows[row] = X[src_of[row] / k]
 *   workspace_dev: relibra_workspace_bytes(RELIBRA_WS_PERMUTE, ...) bytes, dev, scratch
 * Limits: E <= 4096, h % 8 == 0, 16-byte aligned X / Xrows.
 */
int relibra_permute(const int32_t *ids_dev, const int32_t *inst_ptr_dev, const int32_t *inst_rows_dev,
                    const int32_t *inst_group_dev, const int32_t *group_offset_dev,
                    const void *X_dev, int T, int k, int E, int G, int h,
                    int32_t *row_of_dev, int32_t *src_of_dev, void *Xrows_dev,
                    void *workspace_dev, size_t workspace_bytes,
                    int32_t *err_flag_dev, relibra_stream stream);

/*
 * relibra_permute for callers that cannot allocate device memory or pass a workspace (code under
 * HIP graph capture, tight serving loops, harnesses that forbid hipMalloc): the same kernels with
 * their scratch (the per-unit count matrix, relibra_workspace_bytes(RELIBRA_WS_PERMUTE, ...) bytes)
 * in a static device array of RELIBRA_PERMUTE_STATIC_BYTES that each GPU the library runs on holds
 * until the process ends.  Sizes that need more return RELIBRA_EWORKSPACE; a failed lookup of the
 * array's device address returns RELIBRA_EHIP.  The call allocates and frees nothing.  Every call on
 * a GPU uses that GPU's one array: calls that overlap on one GPU (different streams) race and must
 * be ordered by the caller; calls in sequence need no clearing in between.  All other arguments,
 * results and error flags as relibra_permute.
 */
#define RELIBRA_PERMUTE_STATIC_BYTES (4u << 20)
int relibra_permute_static(const int32_t *ids_dev, const int32_t *inst_ptr_dev, const int32_t *inst_rows_dev,
                           const int32_t *inst_group_dev, const int32_t *group_offset_dev,
                           const void *X_dev, int T, int k, int E, int G, int h,
                           int32_t *row_of_dev, int32_t *src_of_dev, void *Xrows_dev,
                           int32_t *err_flag_dev, relibra_stream stream);

/*
 * Source-aware token split (Section 5.2: y_{j,e,g}, the share of source rank j's tokens of
 * expert e served by rank g; Section 4.1 for the link types).  The plan fixes how many tokens
 * every instance of an expert serves; which sources fill an instance decides the traffic.  Per
 * expert, every instance first takes the tokens that sit on its own rank (local copies), then
 * those of the sources on its rail in the other nodes (ascending rank; RDMA without a relay
 * hop), and the remainder is dealt out source by source to the instances that still have room
 * (both ascending).  No split with the same instance sizes moves fewer tokens over the
 * intra-node link; the RDMA volume does not depend on the split.  All pointers HOST.
 *   x_host [EP, E] int64 in          tokens of source rank j routed to expert e (token t of a
 *                                    micro-batch sits on rank t / (T/EP))
 *   inst_ptr [E+1], inst_rank, inst_rows [>= inst_ptr[E]] int32 in: one micro-batch's plan tables
 *   src_first     [EP, E] int32 out          sum of x over the sources before j
 *   inst_src_rows [inst_ptr[E], EP] int32 out  tokens of source j served by instance i
 *   inst_src_base [inst_ptr[E], EP] int32 out  exclusive prefix sum of inst_src_rows over j
 * Errors: RELIBRA_EINVAL on bad sizes or null pointers; RELIBRA_ERANGE when an expert's instance
 * sizes do not add up to its tokens, or on a negative or out-of-range table entry.
 */
int relibra_assign_sources(const int64_t *x_host, int E, int EP, int ranks_per_node,
                           const int32_t *inst_ptr, const int32_t *inst_rank, const int32_t *inst_rows,
                           int32_t *src_first, int32_t *inst_src_rows, int32_t *inst_src_base);

/*
 * The cost model of Section 4.1 (Eq. 1-6) on a split: instance i on rank inst_rank[i] (negative:
 * unused entry) serves inst_src_rows[i][j] tokens of source j.  All pointers HOST.
 *   out3 [3] double out: T_MoE (Eq. 6), max_g T_comp (Eq. 4), max_g T_comm (Eq. 5), seconds
 *   loads_out [5, EP] int64 out or NULL: computation load, intra-node send, receive, RDMA send,
 *   receive, in tokens (Eq. 1-3)
 */
int relibra_moe_time_split(const int32_t *inst_src_rows, int n_inst, const int32_t *inst_rank,
                           const relibra_cost_model *model, double *out3, int64_t *loads_out);

/*
 * Plan under a given placement with Algorithm 2 as printed in Section 5.2: the bottleneck GPU and
 * the GPU that receives a replica are chosen by T_MoE,g = T_g^comp + T_g^comm (Section 4.1)
 * instead of by load alone.  Per micro-batch, over the whole EP group: the GPU of largest T_g
 * (lowest id on ties) is the bottleneck; its experts with tokens served there are tried, most
 * tokens first (lower id on ties); the replica goes to the GPU of the same node without a copy
 * and with a free slot whose T_g is smallest; tokens are split again (the computation split of
 * relibra_plan, then the sources of relibra_assign_sources) and the replica is kept if
 * (T_MoE of Eq. 6, sum_g T_g^2) got lexicographically smaller, else the next expert is tried;
 * the loop ends when no expert of the bottleneck GPU gives a gain.  All pointers HOST.
 *   x_host [n_mb, EP, E] int64 in   per-source histograms (model->EP, model->ranks_per_node)
 *   expert_rank [E] int32 in        placement, exactly E/EP experts per rank (e.g. relibra_reorder_sa)
 *   t_before, t_after [n_mb] double out  T_MoE of every micro-batch without and with the replicas
 * Tables and the other outputs as relibra_plan_placed.  Deterministic.
 */
int relibra_plan_timed(const int64_t *x_host, int n_mb, int E, int k, const relibra_cost_model *model, int r,
                       const int32_t *expert_rank,
                       int32_t *expert_to_slot, int32_t *replica_expert,
                       int32_t *inst_ptr, int32_t *inst_rank, int32_t *inst_rows, int32_t *inst_group,
                       int32_t *group_expert, int32_t *group_offset, int32_t *group_dw_slot,
                       int64_t *max_load_before, int64_t *max_load_after, double *t_before, double *t_after);

/*
 * relibra_permute under a source-aware split.  Assignment a = t*k + s of token t (source rank
 * j = t / (T/EP)) and expert e has ordinal q among the assignments of (j, e) in ascending a;
 * the instances of e, in the plan's order, take runs of inst_src_rows[i][j] such ordinals; the
 * rows of an instance are laid out source after source:
 *   row = group_offset[inst_group[i]] + inst_src_base[i][j] + (q - tokens of j on earlier instances).
 * The three split tables (device copies of relibra_assign_sources' outputs) replace inst_rows;
 * everything else, the error flags included, as relibra_permute.  T % EP == 0.
 */
int relibra_permute_src(const int32_t *ids_dev, const int32_t *inst_ptr_dev,
                        const int32_t *inst_group_dev, const int32_t *group_offset_dev,
                        int EP, const int32_t *src_first_dev, const int32_t *inst_src_rows_dev,
                        const int32_t *inst_src_base_dev,
                        const void *X_dev, int T, int k, int E, int G, int h,
                        int32_t *row_of_dev, int32_t *src_of_dev, void *Xrows_dev,
                        void *workspace_dev, size_t workspace_bytes,
                        int32_t *err_flag_dev, relibra_stream stream);

/*
 * Expert FFN forward over groups [g_begin, g_end) (Section 4.1: three GEMMs, 6hh' flops per row).
 * For every row x of a group whose expert is e:
 *   Gt = Wg_e x,  U = Wu_e x,  A = silu(Gt) * U,  y = Wd_e A
 * with bf16 operands, fp32 accumulation, and one rounding to bf16 of each stored tensor.
 *   Xrows [n_rows, h] bf16 in;  Wg, Wu [E, hff, h] bf16 in;  Wd [E, h, hff] bf16 in
 *   group_offset_dev [G+1], group_expert_dev [G] int32 in (groups with expert -1 or no rows are skipped)
 *   Gt_save, U_save, A_save [n_rows, hff] bf16 out (kept for the backward pass)
 *   Yrows [n_rows, h] bf16 out.  Rows of groups outside the range are left untouched.
 *   n_rows: capacity of the row buffers; offsets beyond it raise RELIBRA_ERR_GROUP_TABLE.
 * group_expert[g] is the index of the group's parameter block in Wg/Wu/Wd and E their number of
 * blocks: with a physical replica buffer (relibra_replica_push) pass the plan's group_dw_slot
 * table and E + EP*r here, and replica groups read their own copy.
 * flags: 0, or RELIBRA_FWD_TRANSPOSED_WEIGHTS: Wg, Wu, Wd point to transposed copies
 * ([E, h, hff], [E, h, hff], [E, hff, h], made by relibra_transpose_experts); the results are
 * identical bit for bit.  The weight operand is then read along full cache lines through the
 * transposing LDS reads, which measures a few percent faster; the copies cost one pass over the
 * weights per optimizer step.  Other flag bits: RELIBRA_EINVAL.
 * Limits: h % 64 == 0, hff % 64 == 0, g_end - g_begin <= 8192 (RELIBRA_EUNSUPPORTED beyond), 16-byte
 *   aligned tensors.
 */
#define RELIBRA_FWD_TRANSPOSED_WEIGHTS 1
int relibra_moe_ffn_fwd(const void *Xrows_dev, int n_rows,
                        const int32_t *group_offset_dev, const int32_t *group_expert_dev,
                        int G, int g_begin, int g_end, int E,
                        const void *Wg_dev, const void *Wu_dev, const void *Wd_dev, int h, int hff,
                        void *Gt_save_dev, void *U_save_dev, void *A_save_dev, void *Yrows_dev, int flags,
                        void *workspace_dev, size_t workspace_bytes,
                        int32_t *err_flag_dev, relibra_stream stream);

/*
 * The permutation's row gather fused into the GEMMs that read the gathered rows (instead of
 * materialising Xrows with relibra_permute and reading it back).  relibra_row_tokens turns the
 * permutation's src_of into the token of every row, row_tok[row] = src_of[row] / k (entries
 * outside [0, T*k) become token 0 and raise RELIBRA_ERR_PLAN_COVER).  relibra_moe_ffn_fwd_gather
 * is relibra_moe_ffn_fwd reading row `row` of its input as X[row_tok[row]]: X [T, h] bf16 is the
 * token tensor, row_tok [n_rows] int32; values are clamped into [0, T).  Results are identical to
 * the two-step form bit for bit.  (The batched weight gradients take the same pair, see
 * relibra_wgrad_mb.)
 */
int relibra_row_tokens(const int32_t *src_of_dev, int N, int k, int T, int32_t *row_tok_dev,
                       int32_t *err_flag_dev, relibra_stream stream);
int relibra_moe_ffn_fwd_gather(const void *X_dev, int T, const int32_t *row_tok_dev, int n_rows,
                               const int32_t *group_offset_dev, const int32_t *group_expert_dev,
                               int G, int g_begin, int g_end, int E,
                               const void *Wg_dev, const void *Wu_dev, const void *Wd_dev, int h, int hff,
                               void *Gt_save_dev, void *U_save_dev, void *A_save_dev, void *Yrows_dev, int flags,
                               void *workspace_dev, size_t workspace_bytes,
                               int32_t *err_flag_dev, relibra_stream stream);

/*
 * Gate-side fusion (a restructuring of this build, not of the paper: the combine of Section 2.1,
 * a gate-weighted sum of the selected experts' outputs, is linear, so its backward can move into
 * the expert backward).  With row_gate[r] = the gate of the assignment row r serves
 * (relibra_row_gates: gates_dev [T*k] fp32 indexed by src_of):
 *   forward (relibra_moe_ffn_fwd_gated): relibra_moe_ffn_fwd_gather that also stores
 *       Ag_save [n_rows, hff] bf16 = row_gate * A, the right operand of dWd below; all other
 *       outputs are unchanged (Yrows stays ungated: relibra_unpermute_combine applies the gates).
 *       With Ag_save_dev == A_save_dev the gated activations take the plain ones' place (one tensor
 *       less to write): the down projection then yields gate-scaled rows, and the combine is
 *       RELIBRA_COMBINE_SUM (rounding differs from gating afterwards; within the tolerance);
 *   backward (relibra_moe_ffn_bwd_gated): takes dOut [T, h] bf16, the gradient of the combined
 *       output, instead of dYrows = gate * dOut[token] (no combine-backward pass, no dYrows
 *       buffer).  With dA' = Wd_e^T dOut[tok(r)]:
 *         dGt = gate * dA' * U * silu'(Gt);  dU = gate * dA' * silu(Gt);  dx as in relibra_moe_ffn_bwd;
 *         dgate[r] = sum_n dA'[n] * (silu(Gt) * U)[n]   (= <dOut[tok(r)], Yrows[r]> up to rounding)
 *       dgate_dev fp32: [n_rows] by row, or, with src_of_dev != NULL, written at src_of[r]: the
 *       gates' own [T*k] layout.  Rows outside the groups' range are left alone.  Always defers
 *       the weight gradients (dGt, dU stay in workspace_dev for relibra_moe_ffn_wgrad_batched,
 *       which takes dOut_dev and Ag_save in relibra_wgrad_mb); flags: RELIBRA_BWD_REPLICA_WEIGHTS,
 *       RELIBRA_BWD_TRANSPOSED_WEIGHTS.  dgate_scratch_dev: relibra_workspace_bytes(RELIBRA_WS_DGATE,
 *       ...) bytes (partial row sums, added in a fixed order: results are reproducible bit for bit).
 * Errors as in the ungated calls; a src_of entry outside [0, n_rows) is skipped and flagged
 * RELIBRA_ERR_PLAN_COVER.
 */
int relibra_row_gates(const int32_t *src_of_dev, const float *gates_dev, int N, float *row_gate_dev,
                      int32_t *err_flag_dev, relibra_stream stream);
int relibra_moe_ffn_fwd_gated(const void *X_dev, int T, const int32_t *row_tok_dev, const float *row_gate_dev, int n_rows,
                              const int32_t *group_offset_dev, const int32_t *group_expert_dev,
                              int G, int g_begin, int g_end, int E,
                              const void *Wg_dev, const void *Wu_dev, const void *Wd_dev, int h, int hff,
                              void *Gt_save_dev, void *U_save_dev, void *A_save_dev, void *Ag_save_dev, void *Yrows_dev,
                              int flags, void *workspace_dev, size_t workspace_bytes,
                              int32_t *err_flag_dev, relibra_stream stream);
int relibra_moe_ffn_bwd_gated(const void *dOut_dev, int T, const int32_t *row_tok_dev, const float *row_gate_dev,
                              const int32_t *src_of_dev,
                              const void *Gt_save_dev, const void *U_save_dev, int n_rows,
                              const int32_t *group_offset_dev, const int32_t *group_expert_dev,
                              const int32_t *group_dw_slot_dev,
                              int G, int g_begin, int g_end, int E, int n_dw_slots,
                              const void *Wg_dev, const void *Wu_dev, const void *Wd_dev, int h, int hff,
                              void *dXrows_dev, float *dgate_dev, int flags,
                              void *workspace_dev, size_t workspace_bytes,
                              void *dgate_scratch_dev, size_t dgate_scratch_bytes,
                              int32_t *err_flag_dev, relibra_stream stream);

/*
 * Expert FFN backward over groups [g_begin, g_end).  With dy the upstream gradient of a row:
 *   dA = Wd_e^T dy;  dGt = dA * U * silu'(Gt);  dU = dA * silu(Gt);  dx = Wg_e^T dGt + Wu_e^T dU
 *   dWd += dy A^T;   dWg += dGt x^T;   dWu += dU x^T          (contraction over the group's rows)
 * Each group writes the weight-gradient slot group_dw_slot[g]; slots >= E are replica slots,
 * whose gradients are then added into the home expert's slot in ascending slot order
 * (Section 5.1: replica gradients are pushed back and accumulated on the source GPU), unless
 * RELIBRA_BWD_NO_REPLICA_SUM.  Home slots are overwritten, or added to with
 * RELIBRA_BWD_ACCUMULATE (gradient accumulation over micro-batches, Section 2.1); a home group
 * with no rows writes zeros (overwrite) or nothing (accumulate).  No float atomics: results
 * are bit-reproducible.
 *   dYrows, Xrows [n_rows,h]; Gt_save, U_save, A_save [n_rows,hff] bf16 in
 *   dXrows [n_rows, h] bf16 out
 *   dWg, dWu [n_dw_slots, hff, h], dWd [n_dw_slots, h, hff] fp32 in/out, n_dw_slots >= E
 *   workspace_dev: relibra_workspace_bytes(RELIBRA_WS_FFN_BWD, ...) bytes (holds dGt, dU)
 */
int relibra_moe_ffn_bwd(const void *dYrows_dev, const void *Xrows_dev,
                        const void *Gt_save_dev, const void *U_save_dev, const void *A_save_dev, int n_rows,
                        const int32_t *group_offset_dev, const int32_t *group_expert_dev,
                        const int32_t *group_dw_slot_dev,
                        int G, int g_begin, int g_end, int E, int n_dw_slots,
                        const void *Wg_dev, const void *Wu_dev, const void *Wd_dev, int h, int hff,
                        void *dXrows_dev, float *dWg_dev, float *dWu_dev, float *dWd_dev, int flags,
                        void *workspace_dev, size_t workspace_bytes,
                        int32_t *err_flag_dev, relibra_stream stream);

/*
 * Transposed copy of per-expert matrices: out[e][j][i] = in[e][i][j], bf16, e < n_blocks.
 * A GEMM reads its weight operand with the contraction index contiguous or strided in memory,
 * depending on the layout it is given: the forward GEMMs find it contiguous in the stored layout,
 * the data gradients strided.  The strided form (whole cache lines per load, transposing LDS
 * reads) measures 6-10 % faster per kernel, so the forward pass can be handed transposed copies
 * (RELIBRA_FWD_TRANSPOSED_WEIGHTS); RELIBRA_BWD_TRANSPOSED_WEIGHTS does the opposite for the data
 * gradients.  Parameters change once per optimizer step, so the copies are made once per step
 * (2x the weights' bytes of traffic) and serve every micro-batch; 288 GB of HBM hold both layouts.
 *   in_dev [n_blocks, rows, cols], out_dev [n_blocks, cols, rows] bf16, dev; must not overlap.
 * Limits: rows % 8 == 0, cols % 8 == 0, n_blocks <= 65535, 16-byte aligned.
 */
int relibra_transpose_experts(const void *in_dev, int n_blocks, int rows, int cols, void *out_dev,
                              relibra_stream stream);

/*
 * Weight gradients of a whole training batch in one pass (the gradient accumulation over
 * micro-batches of Section 2.1, done in registers instead of in memory).  The per-micro-batch
 * form adds each micro-batch's contribution into fp32 dW in HBM: 24 h h' bytes of traffic per
 * live expert and micro-batch, which outweighs the GEMM itself for groups below ~1000 rows.
 * With 288 GB of HBM every micro-batch's activations can stay resident instead, so that one
 * kernel contracts over ALL rows an expert received in the batch (every micro-batch, home and
 * replica instances alike) and writes dW once:
 *   dWd[e] (+)= sum dy A^T,  dWg[e] (+)= sum dGt x^T,  dWu[e] (+)= sum dU x^T.
 * The sum runs over micro-batches in ascending order and, inside one, over the expert's
 * instances in the order of the plan's instance table: fixed order, no atomics.
 * Usage: run relibra_moe_ffn_bwd of every micro-batch with RELIBRA_BWD_DEFER_WGRAD over all
 * groups (g_begin = 0, g_end = G), each with its OWN row buffers and workspace, keep them,
 * then call this once.  On several GPUs a rank would contract its own instances this way and
 * push the partial dW of replicated experts to their home rank once per batch.
 *   mbs_host [n_mb] host in: per micro-batch device pointers
 *       dYrows, Xrows [n_rows,h] (or X, row_tok: see the struct), A_save [n_rows,hff] bf16;
 *       bwd_workspace = the workspace that
 *       micro-batch's deferred backward call used (same n_rows, G, hff);
 *       inst_ptr [E+1], inst_group [inst_cap], group_offset [G+1] int32: the plan's tables
 *   dWg, dWu [E,hff,h], dWd [E,h,hff] fp32 dev: overwritten, or added to with RELIBRA_WGRAD_ACCUMULATE
 *   flags: RELIBRA_WGRAD_ACCUMULATE, and optionally one of RELIBRA_WGRAD_TILE_NARROW / _WIDE to fix the
 *       output tile (256 x 128 with four waves, two workgroups per compute unit, or 256 x 256 with
 *       eight waves, one): by default the wide tile wherever the output is at least 256 wide,
 *       except for dWd when hff < 1024 and an expert averages fewer than 16384 rows over the
 *       batch (n_rows * n_mb / E).  Same sums in the same order either way: results are identical
 *       bit for bit.  Other bits: RELIBRA_EINVAL.
 *   workspace_dev: relibra_workspace_bytes(RELIBRA_WS_WGRAD_BATCHED, ...) bytes
 * Table entries out of range are skipped and flagged RELIBRA_ERR_GROUP_TABLE.
 * Limits: 1 <= n_mb <= RELIBRA_MAX_WGRAD_MB, h % 64 == 0, hff % 64 == 0, 16-byte aligned tensors.
 */
#define RELIBRA_MAX_WGRAD_MB 48
enum { RELIBRA_WGRAD_ACCUMULATE = 1, RELIBRA_WGRAD_TILE_NARROW = 2, RELIBRA_WGRAD_TILE_WIDE = 4 };
typedef struct relibra_wgrad_mb {
    const void *dYrows_dev, *Xrows_dev, *A_save_dev;
    const void *bwd_workspace_dev;
    const int32_t *inst_ptr_dev, *inst_group_dev, *group_offset_dev;
    /* fused row gather: with Xrows_dev == NULL, row r of the micro-batch is X_dev[row_tok_dev[r]]
       (X_dev [n_tokens, h] bf16 token tensor, row_tok_dev [n_rows] from relibra_row_tokens) */
    const void *X_dev;
    const int32_t *row_tok_dev;
    int n_tokens;
    /* gate-fused backward (relibra_moe_ffn_bwd_gated): with dYrows_dev == NULL, the upstream gradient
       of row r is dOut_dev[row_tok_dev[r]] (dOut_dev [n_tokens, h] bf16) and A_save_dev must hold the
       gate-scaled activations Ag_save of relibra_moe_ffn_fwd_gated; needs the fused row gather
       (Xrows_dev == NULL) */
    const void *dOut_dev;
} relibra_wgrad_mb;

int relibra_moe_ffn_wgrad_batched(const relibra_wgrad_mb *mbs_host, int n_mb, int n_rows,
                                  int G, int inst_cap, int E, int h, int hff,
                                  float *dWg_dev, float *dWu_dev, float *dWd_dev, int flags,
                                  void *workspace_dev, size_t workspace_bytes,
                                  int32_t *err_flag_dev, relibra_stream stream);

/*
 * Layer-shared replica buffer, forward push (Section 5.1: before a layer's expert computation
 * every GPU pushes the experts that are replicated in this micro-batch into the replica slots
 * of their target GPUs; the r slots per GPU are reused by every layer and micro-batch).
 * On one GPU the parameter arrays hold the EP*r replica slots behind the E home blocks:
 *   Wg, Wu [E + EP*r, hff, h], Wd [E + EP*r, h, hff] bf16, dev, in/out
 *   replica_expert_dev [EP*r] int32, dev, in: the plan's table for this micro-batch
 *                      (slot s = rank*r + j holds expert replica_expert[s], -1 = empty)
 * and the call copies block e to block E + s for every live slot.  n_workgroups (>= 1) bounds
 * the compute units the copy may occupy, so that it can run beside other kernels on a second
 * stream (the paper overlaps it with attention and gives it few SMs).  Values >= E in the
 * table are skipped and flagged RELIBRA_ERR_ID_RANGE.
 * Limits: h*hff % 8 == 0, 16-byte aligned tensors.
 */
int relibra_replica_push(void *Wg_dev, void *Wu_dev, void *Wd_dev,
                         const int32_t *replica_expert_dev, int E, int EP, int r, int h, int hff,
                         int n_workgroups, int32_t *err_flag_dev, relibra_stream stream);

/*
 * Layer-shared replica buffer, gradient return (Section 5.1: in the backward pass the gradients
 * produced by the replicas of a micro-batch are pushed back and accumulated on the source GPUs;
 * the gradient buffer has the replica buffer's size and is reused the same way).  The reverse of
 * relibra_replica_push on the gradient arrays
 *   dWg, dWu [E + EP*r, hff, h], dWd [E + EP*r, h, hff] fp32, dev, in/out:
 * for every live slot s (replica_expert[s] = e >= 0), in ascending slot order, block E + s is
 * added into block e.  relibra_moe_ffn_bwd does the same sum in line unless it is given
 * RELIBRA_BWD_NO_REPLICA_SUM; this call makes it a kernel of its own with a caller-bounded number
 * of workgroups (n_workgroups >= 1), to run on a second stream beside other work.  The order of
 * every element's additions is the in-line sum's: results are identical bit for bit.  The slots
 * keep their contents (the next backward call overwrites them).  Entries >= E: skipped, flagged
 * RELIBRA_ERR_ID_RANGE.  Limits: h*hff % 4 == 0, 16-byte aligned tensors.
 */
int relibra_replica_pull(float *dWg_dev, float *dWu_dev, float *dWd_dev,
                         const int32_t *replica_expert_dev, int E, int EP, int r, int h, int hff,
                         int n_workgroups, int32_t *err_flag_dev, relibra_stream stream);

/*
 * Unpermute + gate-weighted combine and its backward (Section 2.1: the outputs of a token's
 * selected experts are combined; the local half of the combine all-to-all).
 *  mode RELIBRA_COMBINE_FWD: out_tok[t] = sum_s gates[t,s] * rows[row_of[t*k+s]]   (fp32 sum in
 *        slot order, one rounding to bf16)
 *  mode RELIBRA_COMBINE_SUM: same with every gate = 1 (backward of the row gather); gates unused
 *  mode RELIBRA_COMBINE_BWD: out_rows[row_of[t*k+s]] = gates[t,s] * tok[t]  (bf16) and
 *        dgate[t,s] = <tok[t], rows[row_of[t*k+s]]>  (fp32); tok = dOut, rows = Yrows
 *   rows_dev [N,h] bf16 in; tok_dev [T,h] bf16 in (BWD only); gates_dev [T,k] fp32 in;
 *   row_of_dev [N] int32 in; out_tok_dev [T,h] bf16 out (FWD, SUM); out_rows_dev [N,h] bf16 out
 *   and dgate_dev [T,k] fp32 out (BWD).  Rows referenced must lie in [0, N): others are skipped
 *   and flagged RELIBRA_ERR_PLAN_COVER.
 * Limits: h % 8 == 0, 1 <= k <= 64.
 */
int relibra_unpermute_combine(int mode, const void *rows_dev, const void *tok_dev,
                              const float *gates_dev, const int32_t *row_of_dev,
                              int T, int k, int h,
                              void *out_tok_dev, void *out_rows_dev, float *dgate_dev,
                              int32_t *err_flag_dev, relibra_stream stream);

/*
 * Per-kernel timing for benchmarks (not part of the method).  Between relibra_prof_start and
 * relibra_prof_stop every kernel launch of the chosen level is bracketed by two HIP events on
 * its launch stream: level 1 = the six grouped-GEMM kernels, level 2 = every kernel, 0 = off.
 * At most max_records launches are recorded (events are created in relibra_prof_start, host
 * side only).  relibra_prof_stop waits for the recorded events and returns, per kernel id
 * (RELIBRA_K_*), the summed milliseconds and the launch count in two host arrays of
 * RELIBRA_K_COUNT entries.  Process-global, not thread-safe.
 */
enum {
    RELIBRA_K_HIST = 0, RELIBRA_K_PERM_COUNT, RELIBRA_K_PERM_SCAN, RELIBRA_K_PERM_RANK,
    RELIBRA_K_GATHER, RELIBRA_K_COMBINE_FWD, RELIBRA_K_COMBINE_BWD, RELIBRA_K_COMBINE_SUM, RELIBRA_K_SCHED,
    RELIBRA_K_FWD_GATE_UP, RELIBRA_K_FWD_DOWN, RELIBRA_K_BWD_ACT, RELIBRA_K_BWD_DX,
    RELIBRA_K_WGRAD_DOWN, RELIBRA_K_WGRAD_GATE_UP, RELIBRA_K_REPLICA_SUM, RELIBRA_K_REPLICA_PUSH,
    RELIBRA_K_WGRAD_ORDER, RELIBRA_K_TRANSPOSE, RELIBRA_K_ROW_TOKENS, RELIBRA_K_ROW_GATES, RELIBRA_K_DGATE_REDUCE,
    RELIBRA_K_REPLICA_PULL, RELIBRA_K_COUNT
};
int relibra_prof_start(int level, int max_records);
int relibra_prof_stop(double *ms_by_kernel_host, int64_t *launches_by_kernel_host);

/* Bytes of device scratch each call needs (0 on unusable sizes). */
size_t relibra_workspace_bytes(int which, int T, int k, int E, int G, int h, int hff);

/* Text for a status code (static storage). */
const char *relibra_status_string(int status);

#ifdef __cplusplus
}
#endif
#endif
