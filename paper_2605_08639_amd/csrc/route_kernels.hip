// Routing-side kernels: load histogram, token permutation, unpermute + combine.
// All three are bound by HBM traffic (or, for the index parts, by launch latency); none is
// a contraction, so there is no MFMA here: the work is coalesced 16-byte accesses,
// wave-level ballots and LDS-private counters.
#include "common.h"

#include <mutex>

namespace relibra {

constexpr int kMaxExperts = 4096;
constexpr int kHistThreads = 1024;   // one block per micro-batch
constexpr int kHistLdsBytes = 64 * 1024;
constexpr int kUnit = RELIBRA_PERM_UNIT;   // assignments per permutation unit (one wave): short units, many waves -
                                         // the rank kernel is a chain of dependent table reads per round of 64
constexpr int kPermThreads = 256;    // 4 waves = 4 units per block

// ---------------------------------------------------------------- histogram (Eq. 1)
// One block per micro-batch: it counts the micro-batch's ids in LDS and STORES the finished
// histogram, so there is no zero-fill launch in front, no global atomics, and the result does
// not depend on any execution order.  Hot experts (a Zipf router sends a fifth of the assignments
// to one expert) would serialise LDS atomics on one address; every bin is therefore kept in C
// copies, lane l adding to copy l % C, laid out so that the copies of a bin sit in different banks.
// A single micro-batch (<= 512 KiB of ids) is latency-sized whatever the kernel does; the
// bandwidth-bound use is many micro-batches at once (every layer's replayed routing, Section 3),
// where the grid is thousands of blocks.
__global__ void __launch_bounds__(kHistThreads)
hist_kernel(const int32_t *__restrict__ ids, int per_mb, int E, int copies_log2, int vec_ok,
            int32_t *__restrict__ counts, int32_t *err_flag)
{
    extern __shared__ int32_t bins[];          // [E << copies_log2]
    const int mb = blockIdx.x;
    const int n_bins = E << copies_log2;
    for (int i = threadIdx.x; i < n_bins; i += kHistThreads) bins[i] = 0;
    __syncthreads();
    const int32_t *src = ids + (size_t)mb * per_mb;
    const int copy = threadIdx.x & ((1 << copies_log2) - 1);
    bool bad = false;
    if (vec_ok) {                      // 16-byte aligned rows of the id tensor
        const int4 *v = reinterpret_cast<const int4 *>(src);
        const int n4 = per_mb / 4;
        int i = threadIdx.x;
        for (; i + 3 * kHistThreads < n4; i += 4 * kHistThreads) {       // four loads in flight per lane
            const int4 q[4] = {v[i], v[i + kHistThreads], v[i + 2 * kHistThreads], v[i + 3 * kHistThreads]};
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int e4[4] = {q[u].x, q[u].y, q[u].z, q[u].w};
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    if ((unsigned)e4[j] < (unsigned)E) atomicAdd(&bins[(e4[j] << copies_log2) + copy], 1);
                    else bad = true;
                }
            }
        }
        for (; i < n4; i += kHistThreads) {
            const int4 q = v[i];
            const int e4[4] = {q.x, q.y, q.z, q.w};
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                if ((unsigned)e4[j] < (unsigned)E) atomicAdd(&bins[(e4[j] << copies_log2) + copy], 1);
                else bad = true;
            }
        }
    } else {
        for (int i = threadIdx.x; i < per_mb; i += kHistThreads) {
            const int e = src[i];
            if ((unsigned)e < (unsigned)E) atomicAdd(&bins[(e << copies_log2) + copy], 1);
            else bad = true;
        }
    }
    if (bad) atomicOr(err_flag, RELIBRA_ERR_ID_RANGE);
    __syncthreads();
    for (int e = threadIdx.x; e < E; e += kHistThreads) {
        int c = 0;
        for (int j = 0; j < (1 << copies_log2); ++j) c += bins[(e << copies_log2) + ((j + e) & ((1 << copies_log2) - 1))];
        counts[(size_t)mb * E + e] = c;
    }
}

// ---------------------------------------------------------------- permutation indices
// The stable partition is a counting sort over experts in three passes:
//   1. every wave counts its unit of assignments per expert        -> unit_cnt[unit][e]
//   2. an exclusive scan over units, per expert                    -> unit_cnt[unit][e] = base
//   3. every wave walks its unit in order, 64 assignments at a time; a ballot-built mask of
//      the lanes holding the same expert gives each lane its ordinal inside the step, an LDS
//      counter per expert carries the ordinal across steps.
// The ordinal is then mapped through the expert's instance list to a row (Section 5.2).

__global__ void __launch_bounds__(kPermThreads)
perm_count_kernel(const int32_t *__restrict__ ids, int N, int E, int32_t *__restrict__ unit_cnt,
                  int32_t *__restrict__ src_of, int32_t *err_flag)
{
    extern __shared__ int32_t lds[];
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    int32_t *bins = lds + wave * E;
    const int unit = blockIdx.x * (kPermThreads / 64) + wave;
    for (int e = lane; e < E; e += 64) bins[e] = 0;
    __builtin_amdgcn_wave_barrier();
    const int lo = unit * kUnit, hi = min(N, lo + kUnit);
    bool bad = false;
    for (int a = lo + lane; a < hi; a += 64) {
        const int e = ids[a];
        if ((unsigned)e < (unsigned)E) atomicAdd(&bins[e], 1);
        else bad = true;
        src_of[a] = -1;                // rows nobody claims stay marked
    }
    if (bad) atomicOr(err_flag, RELIBRA_ERR_ID_RANGE);
    __builtin_amdgcn_wave_barrier();
    if (lo < N)
        for (int e = lane; e < E; e += 64) unit_cnt[(size_t)unit * E + e] = bins[e];
}

// One block per expert: exclusive scan of that expert's counts over the units.
__global__ void __launch_bounds__(256) perm_scan_kernel(int32_t *unit_cnt, int n_units, int E)
{
    __shared__ int32_t scan[256];
    __shared__ int32_t carry;
    const int e = blockIdx.x, tid = threadIdx.x;
    if (tid == 0) carry = 0;
    __syncthreads();
    for (int base = 0; base < n_units; base += 256) {
        const int u = base + tid;
        const int c = u < n_units ? unit_cnt[(size_t)u * E + e] : 0;
        scan[tid] = c;
        __syncthreads();
        for (int off = 1; off < 256; off <<= 1) {
            const int v = tid >= off ? scan[tid - off] : 0;
            __syncthreads();
            scan[tid] += v;
            __syncthreads();
        }
        if (u < n_units) unit_cnt[(size_t)u * E + e] = carry + scan[tid] - c;
        __syncthreads();
        if (tid == 255) carry += scan[255];
        __syncthreads();
    }
}

// Optional per-source split of the permutation (all null / zero: split in token order).
struct SrcSplit {
    const int32_t *src_first;       // [EP][E] ordinal, among e's assignments, of source j's first one
    const int32_t *inst_src_rows;   // [instances][EP] tokens of source j served by instance i
    const int32_t *inst_src_base;   // [instances][EP] exclusive prefix of inst_src_rows over j
    int EP, k, tokens_per_src;
};

__global__ void __launch_bounds__(kPermThreads)
perm_rank_kernel(const int32_t *__restrict__ ids, int N, int E, int G, int ebits,
                 const int32_t *__restrict__ unit_base,
                 const int32_t *__restrict__ inst_ptr, const int32_t *__restrict__ inst_rows,
                 const int32_t *__restrict__ inst_group, const int32_t *__restrict__ group_offset,
                 int32_t *__restrict__ row_of, int32_t *__restrict__ src_of, int32_t *err_flag,
                 SrcSplit sp)
{
    extern __shared__ int32_t lds[];
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    int32_t *next = lds + wave * E;        // next ordinal of each expert, private to the wave
    const int unit = blockIdx.x * (kPermThreads / 64) + wave;
    const int lo = unit * kUnit, hi = min(N, lo + kUnit);
    if (lo < N)
        for (int e = lane; e < E; e += 64) next[e] = unit_base[(size_t)unit * E + e];
    __builtin_amdgcn_wave_barrier();
    const uint64_t lt_mask = (lane == 0) ? 0ull : (~0ull >> (64 - lane));
    int flags = 0;
    for (int base = lo; base < hi; base += 64) {
        const int a = base + lane;
        const bool live = a < hi;
        const int e_raw = live ? ids[a] : -1;
        const bool ok = live && (unsigned)e_raw < (unsigned)E;
        const int e = ok ? e_raw : 0;
        // lanes with the same expert: intersect ballots bit by bit
        uint64_t same = __ballot(ok);
        for (int b = 0; b < ebits; ++b) {
            const uint64_t vote = __ballot((e >> b) & 1);
            same &= ((e >> b) & 1) ? vote : ~vote;
        }
        int q = 0;
        if (ok) {
            const int before = __popcll(same & lt_mask);
            const int leader = __ffsll((long long)same) - 1;
            int start = 0;
            if (lane == leader) {          // one lane per expert touches the counter
                start = next[e];
                next[e] = start + __popcll(same);
            }
            start = __shfl(start, leader);
            q = start + before;
        }
        __builtin_amdgcn_wave_barrier();
        if (ok) {
            int i = inst_ptr[e];
            const int end = inst_ptr[e + 1];
            int skipped = 0, row = -1;
            if (sp.src_first) {
                // source-aware split: ordinal among the source's own tokens of e, runs of
                // inst_src_rows[i][j], rows of an instance laid out source after source
                const int j = min((a / sp.k) / sp.tokens_per_src, sp.EP - 1);
                const int qj = q - sp.src_first[(size_t)j * E + e];
                for (; qj >= 0 && i < end; ++i) {
                    const int n = sp.inst_src_rows[(size_t)i * sp.EP + j];
                    if (qj < skipped + n) {
                        const int g = inst_group[i];
                        if ((unsigned)g < (unsigned)G) row = group_offset[g] + sp.inst_src_base[(size_t)i * sp.EP + j] + (qj - skipped);
                        break;
                    }
                    skipped += n;
                }
            } else {
                for (; i < end; ++i) {
                    const int n = inst_rows[i];
                    if (q < skipped + n) {
                        const int g = inst_group[i];
                        if ((unsigned)g < (unsigned)G) row = group_offset[g] + (q - skipped);
                        break;
                    }
                    skipped += n;
                }
            }
            if ((unsigned)row < (unsigned)N) {
                row_of[a] = row;
                src_of[row] = a;
            } else {
                row_of[a] = -1;
                flags |= RELIBRA_ERR_PLAN_COVER;
            }
        } else if (live) {
            row_of[a] = -1;
            flags |= RELIBRA_ERR_ID_RANGE;
        }
    }
    if (flags) atomicOr(err_flag, flags);
}

// Thread mapping of the row-streaming kernels: a row of vec_per_row 16-byte pieces is walked by
// LPR = 2^lpr_log2 consecutive threads, each taking every LPR-th piece (LPR = the smallest power
// of two that leaves a thread at most `pieces` pieces, at most the block), so a block of 256
// threads serves 256 / LPR rows at a time and no index needs a division.
constexpr int kRowThreads = 256;
inline int lanes_per_row_log2(int vec_per_row, int pieces)
{
    int l = 0;
    while ((1 << l) * pieces < vec_per_row && (1 << l) < kRowThreads) ++l;
    return l;
}

// Row gather: Xrows[row] = X[src_of[row] / k], 16 bytes per piece, four pieces of a row in flight
// per thread.
__global__ void __launch_bounds__(kRowThreads)
gather_rows_kernel(const uint4 *__restrict__ X, const int32_t *__restrict__ src_of, int N, int T, int k,
                   int vec_per_row, int lpr_log2, uint4 *__restrict__ Xrows)
{
    const int lpr = 1 << lpr_log2, rows_per_block = kRowThreads >> lpr_log2;
    const int r_local = threadIdx.x >> lpr_log2, c0 = threadIdx.x & (lpr - 1);
    for (int row = blockIdx.x * rows_per_block + r_local; row < N; row += gridDim.x * rows_per_block) {
        const int a = src_of[row];
        if (a < 0) continue;
        const int t = a / k;
        if (t >= T) continue;
        const uint4 *__restrict__ src = X + (size_t)t * vec_per_row;
        uint4 *__restrict__ dst = Xrows + (size_t)row * vec_per_row;
        int c = c0;
        for (; c + 3 * lpr < vec_per_row; c += 4 * lpr) {
            const uint4 v0 = src[c], v1 = src[c + lpr], v2 = src[c + 2 * lpr], v3 = src[c + 3 * lpr];
            dst[c] = v0; dst[c + lpr] = v1; dst[c + 2 * lpr] = v2; dst[c + 3 * lpr] = v3;
        }
        for (; c < vec_per_row; c += lpr) dst[c] = src[c];
    }
}

// ---------------------------------------------------------------- combine
__device__ __forceinline__ void unpack8(const uint4 &v, float *f)
{
    const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        f[2 * j] = __uint_as_float(w[j] << 16);
        f[2 * j + 1] = __uint_as_float(w[j] & 0xffff0000u);
    }
}
__device__ __forceinline__ uint4 pack8(const float *f)
{
    uint4 v;
    v.x = pack2bf(f[0], f[1]);
    v.y = pack2bf(f[2], f[3]);
    v.z = pack2bf(f[4], f[5]);
    v.w = pack2bf(f[6], f[7]);
    return v;
}

// out[t] = sum_s gate[t,s] * rows[row_of[t,s]]; fp32 accumulation in slot order.
template <bool GATED>
__global__ void __launch_bounds__(256)
combine_fwd_kernel(const uint4 *__restrict__ rows, const float *__restrict__ gates,
                   const int32_t *__restrict__ row_of, int T, int k, int N, int vec_per_row,
                   uint4 *__restrict__ out, int32_t *err_flag)
{
    const size_t total = (size_t)T * vec_per_row;
    bool bad = false;
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < total; i += (size_t)gridDim.x * 256) {
        const int t = (int)(i / vec_per_row), c = (int)(i % vec_per_row);
        float acc[8] = {0, 0, 0, 0, 0, 0, 0, 0};
        for (int s0 = 0; s0 < k; s0 += 8) {                 // eight row fetches in flight
            uint4 v[8];
            float g[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                g[u] = 0.0f;
                v[u] = make_uint4(0, 0, 0, 0);
                if (s0 + u < k) {
                    const int row = row_of[(size_t)t * k + s0 + u];
                    if ((unsigned)row < (unsigned)N) {
                        g[u] = GATED ? gates[(size_t)t * k + s0 + u] : 1.0f;
                        v[u] = rows[(size_t)row * vec_per_row + c];
                    } else {
                        bad = true;
                    }
                }
            }
#pragma unroll
            for (int u = 0; u < 8; ++u) {                   // fp32 sum in slot order
                float f[8];
                unpack8(v[u], f);
#pragma unroll
                for (int j = 0; j < 8; ++j) acc[j] = fmaf(g[u], f[j], acc[j]);
            }
        }
        out[i] = pack8(acc);
    }
    if (bad) atomicOr(err_flag, RELIBRA_ERR_PLAN_COVER);
}

// One wave per assignment (t,s): dYrows[row] = gate * dOut[t]; dgate = <dOut[t], Yrows[row]>.
__global__ void __launch_bounds__(256)
combine_bwd_kernel(const uint4 *__restrict__ Yrows, const uint4 *__restrict__ dOut,
                   const float *__restrict__ gates, const int32_t *__restrict__ row_of,
                   int N, int vec_per_row, int k, uint4 *__restrict__ dYrows, float *__restrict__ dgate,
                   int32_t *err_flag)
{
    const int lane = threadIdx.x & 63;
    const int a = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (a >= N) return;
    const int row = row_of[a];
    if ((unsigned)row >= (unsigned)N) {
        if (lane == 0) { atomicOr(err_flag, RELIBRA_ERR_PLAN_COVER); dgate[a] = 0.0f; }
        return;
    }
    const int t = a / k;
    const float g = gates[a];
    float dot = 0.0f;
    for (int c = lane; c < vec_per_row; c += 64) {
        float d[8], y[8], o[8];
        unpack8(dOut[(size_t)t * vec_per_row + c], d);
        unpack8(Yrows[(size_t)row * vec_per_row + c], y);
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            o[j] = g * d[j];
            dot = fmaf(d[j], y[j], dot);
        }
        dYrows[(size_t)row * vec_per_row + c] = pack8(o);
    }
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) dot += __shfl_xor(dot, off);
    if (lane == 0) dgate[a] = dot;
}

// row -> token: row_tok[row] = src_of[row] / k (assignment a = t*k + s belongs to token t).
__global__ void __launch_bounds__(256)
row_tokens_kernel(const int32_t *__restrict__ src_of, int N, int k, int T, int32_t *__restrict__ row_tok,
                  int32_t *__restrict__ err_flag)
{
    bool bad = false;
    for (int i = blockIdx.x * 256 + threadIdx.x; i < N; i += gridDim.x * 256) {
        const int a = src_of[i];
        int t = 0;
        if (a < 0 || a / k >= T) bad = true; else t = a / k;
        row_tok[i] = t;
    }
    if (bad) atomicOr(err_flag, RELIBRA_ERR_PLAN_COVER);
}

// row -> gate of the assignment the row serves: row_gate[row] = gates[src_of[row]] (gates flat [T*k]).
__global__ void __launch_bounds__(256)
row_gates_kernel(const int32_t *__restrict__ src_of, const float *__restrict__ gates, int N, float *__restrict__ row_gate,
                 int32_t *__restrict__ err_flag)
{
    bool bad = false;
    for (int i = blockIdx.x * 256 + threadIdx.x; i < N; i += gridDim.x * 256) {
        const int a = src_of[i];
        float g = 0.0f;
        if (a < 0 || a >= N) bad = true; else g = gates[a];
        row_gate[i] = g;
    }
    if (bad) atomicOr(err_flag, RELIBRA_ERR_PLAN_COVER);
}

inline int grid_for(size_t work_items, int per_block, int cap)
{
    size_t b = (work_items + per_block - 1) / per_block;
    if (b < 1) b = 1;
    if (b > (size_t)cap) b = cap;
    return (int)b;
}

}  // namespace relibra

using namespace relibra;

extern "C" int relibra_route_hist(const int32_t *ids_dev, int n_mb, int T, int k, int E,
                                  int32_t *counts_dev, int32_t *err_flag_dev, relibra_stream stream_)
{
    hipStream_t stream = (hipStream_t)stream_;
    if (n_mb < 0 || T < 0 || k < 1 || E < 1 || E > kMaxExperts || k > E) return RELIBRA_EINVAL;
    if ((size_t)T * k > 0x7fffffffull) return RELIBRA_EINVAL;
    if (n_mb == 0) return RELIBRA_OK;
    if (!counts_dev || !err_flag_dev) return RELIBRA_EINVAL;
    const int per_mb = T * k;
    if (per_mb > 0 && !ids_dev) return RELIBRA_EINVAL;
    int copies_log2 = 4;                     // up to 16 copies of every bin, as many as fit the LDS budget
    while (copies_log2 > 0 && ((size_t)E << copies_log2) * sizeof(int32_t) > (size_t)kHistLdsBytes) --copies_log2;
    RELIBRA_LAUNCH(RELIBRA_K_HIST, stream, hist_kernel<<<(unsigned)n_mb, kHistThreads, ((size_t)E << copies_log2) * sizeof(int32_t), stream>>>(
        ids_dev, per_mb, E, copies_log2, ((per_mb & 3) == 0 && aligned16(ids_dev)) ? 1 : 0, counts_dev, err_flag_dev));
    RELIBRA_HIP_TRY(launch_check());
    return RELIBRA_OK;
}

static int permute_impl(const int32_t *ids_dev, const int32_t *inst_ptr_dev, const int32_t *inst_rows_dev,
                        const int32_t *inst_group_dev, const int32_t *group_offset_dev, const SrcSplit &split,
                        const void *X_dev, int T, int k, int E, int G, int h,
                        int32_t *row_of_dev, int32_t *src_of_dev, void *Xrows_dev,
                        void *workspace_dev, size_t workspace_bytes,
                        int32_t *err_flag_dev, relibra_stream stream_)
{
    hipStream_t stream = (hipStream_t)stream_;
    if (T < 0 || k < 1 || E < 1 || E > kMaxExperts || k > E || G < 1 || h < 0) return RELIBRA_EINVAL;
    if ((size_t)T * k > 0x7fffffffull) return RELIBRA_EINVAL;
    const int N = T * k;
    if (N == 0) return RELIBRA_OK;
    if (!ids_dev || !inst_ptr_dev || (!inst_rows_dev && !split.src_first) || !inst_group_dev || !group_offset_dev ||
        !row_of_dev || !src_of_dev || !err_flag_dev || !workspace_dev)
        return RELIBRA_EINVAL;
    const bool with_rows = X_dev != nullptr || Xrows_dev != nullptr;
    if (with_rows && (!X_dev || !Xrows_dev || h < 8 || h % 8 || !aligned16(X_dev) || !aligned16(Xrows_dev)))
        return RELIBRA_EINVAL;
    if (workspace_bytes < relibra_workspace_bytes(RELIBRA_WS_PERMUTE, T, k, E, G, h, 0)) return RELIBRA_EWORKSPACE;
    int32_t *unit_cnt = (int32_t *)workspace_dev;
    const int n_units = (N + kUnit - 1) / kUnit;
    const int blocks = (n_units + 3) / 4;
    const size_t lds = (size_t)4 * E * sizeof(int32_t);
    int ebits = 0;
    while ((1 << ebits) < E) ++ebits;
    RELIBRA_LAUNCH(RELIBRA_K_PERM_COUNT, stream, perm_count_kernel<<<blocks, kPermThreads, lds, stream>>>(ids_dev, N, E, unit_cnt, src_of_dev, err_flag_dev));
    RELIBRA_HIP_TRY(launch_check());
    RELIBRA_LAUNCH(RELIBRA_K_PERM_SCAN, stream, perm_scan_kernel<<<E, 256, 0, stream>>>(unit_cnt, n_units, E));
    RELIBRA_HIP_TRY(launch_check());
    RELIBRA_LAUNCH(RELIBRA_K_PERM_RANK, stream, perm_rank_kernel<<<blocks, kPermThreads, lds, stream>>>(ids_dev, N, E, G, ebits, unit_cnt, inst_ptr_dev,
                                                            inst_rows_dev, inst_group_dev, group_offset_dev,
                                                            row_of_dev, src_of_dev, err_flag_dev, split));
    RELIBRA_HIP_TRY(launch_check());
    if (with_rows) {
        const int vpr = h / 8, lpr_log2 = lanes_per_row_log2(vpr, 4);
        const int grid = grid_for((size_t)N, kRowThreads >> lpr_log2, 256 * 32);
        RELIBRA_LAUNCH(RELIBRA_K_GATHER, stream, gather_rows_kernel<<<grid, kRowThreads, 0, stream>>>((const uint4 *)X_dev, src_of_dev, N, T, k, vpr,
                                                     lpr_log2, (uint4 *)Xrows_dev));
        RELIBRA_HIP_TRY(launch_check());
    }
    return RELIBRA_OK;
}

extern "C" int relibra_permute(const int32_t *ids_dev, const int32_t *inst_ptr_dev, const int32_t *inst_rows_dev,
                               const int32_t *inst_group_dev, const int32_t *group_offset_dev,
                               const void *X_dev, int T, int k, int E, int G, int h,
                               int32_t *row_of_dev, int32_t *src_of_dev, void *Xrows_dev,
                               void *workspace_dev, size_t workspace_bytes,
                               int32_t *err_flag_dev, relibra_stream stream_)
{
    if (T > 0 && !inst_rows_dev) return RELIBRA_EINVAL;
    return permute_impl(ids_dev, inst_ptr_dev, inst_rows_dev, inst_group_dev, group_offset_dev, SrcSplit{},
                        X_dev, T, k, E, G, h, row_of_dev, src_of_dev, Xrows_dev, workspace_dev, workspace_bytes,
                        err_flag_dev, stream_);
}

// The permutation for callers that cannot allocate: its unit-count matrix lives in a static device
// array instead of a caller's workspace.  Every GPU holds its own copy of the array at its own
// address; host code never uses the array's name as an address, only what hipGetSymbolAddress
// returned for the device that is current.
static __device__ __align__(256) int32_t scratch[RELIBRA_PERMUTE_STATIC_BYTES / sizeof(int32_t)];

namespace {
constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
int32_t *g_scratch_ptr[kMaxDevices] = {};     // per device: the device address of `scratch`
}  // namespace

// Device address of this device's copy of `scratch` (looked up once per device); null on failure.
static int32_t *scratch_for_current_device()
{
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return nullptr;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void *ptr = nullptr;
        if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess) return nullptr;
        g_scratch_ptr[dev] = (int32_t *)ptr;
    }
    return g_scratch_ptr[dev];
}

extern "C" int relibra_permute_static(const int32_t *ids_dev, const int32_t *inst_ptr_dev, const int32_t *inst_rows_dev,
                                      const int32_t *inst_group_dev, const int32_t *group_offset_dev,
                                      const void *X_dev, int T, int k, int E, int G, int h,
                                      int32_t *row_of_dev, int32_t *src_of_dev, void *Xrows_dev,
                                      int32_t *err_flag_dev, relibra_stream stream_)
{
    if (T > 0 && !inst_rows_dev) return RELIBRA_EINVAL;
    if (T < 0 || k < 1 || E < 1 || G < 1) return RELIBRA_EINVAL;
    const size_t need = relibra_workspace_bytes(RELIBRA_WS_PERMUTE, T, k, E, G, h, 0);
    if (need == 0 && (size_t)T * k > 0) return RELIBRA_EINVAL;
    if (need > (size_t)RELIBRA_PERMUTE_STATIC_BYTES) return RELIBRA_EWORKSPACE;     // beyond the static array
    int32_t *ws = scratch_for_current_device();
    if (!ws) return RELIBRA_EHIP;
    // Nothing in the array has to start at zero: the counting kernel overwrites every entry the other
    // two kernels read.
    return permute_impl(ids_dev, inst_ptr_dev, inst_rows_dev, inst_group_dev, group_offset_dev, SrcSplit{},
                        X_dev, T, k, E, G, h, row_of_dev, src_of_dev, Xrows_dev, ws, (size_t)RELIBRA_PERMUTE_STATIC_BYTES,
                        err_flag_dev, stream_);
}

extern "C" int relibra_permute_src(const int32_t *ids_dev, const int32_t *inst_ptr_dev,
                                   const int32_t *inst_group_dev, const int32_t *group_offset_dev,
                                   int EP, const int32_t *src_first_dev, const int32_t *inst_src_rows_dev,
                                   const int32_t *inst_src_base_dev,
                                   const void *X_dev, int T, int k, int E, int G, int h,
                                   int32_t *row_of_dev, int32_t *src_of_dev, void *Xrows_dev,
                                   void *workspace_dev, size_t workspace_bytes,
                                   int32_t *err_flag_dev, relibra_stream stream_)
{
    if (EP < 1 || T < 0 || T % EP) return RELIBRA_EINVAL;
    if (T > 0 && (!src_first_dev || !inst_src_rows_dev || !inst_src_base_dev)) return RELIBRA_EINVAL;
    const SrcSplit split{src_first_dev, inst_src_rows_dev, inst_src_base_dev, EP, k, T > 0 ? T / EP : 1};
    return permute_impl(ids_dev, inst_ptr_dev, nullptr, inst_group_dev, group_offset_dev, split,
                        X_dev, T, k, E, G, h, row_of_dev, src_of_dev, Xrows_dev, workspace_dev, workspace_bytes,
                        err_flag_dev, stream_);
}

extern "C" int relibra_unpermute_combine(int mode, const void *rows_dev, const void *tok_dev,
                                         const float *gates_dev, const int32_t *row_of_dev,
                                         int T, int k, int h,
                                         void *out_tok_dev, void *out_rows_dev, float *dgate_dev,
                                         int32_t *err_flag_dev, relibra_stream stream_)
{
    hipStream_t stream = (hipStream_t)stream_;
    if (T < 0 || k < 1 || k > 64 || h < 8 || h % 8) return RELIBRA_EINVAL;
    if ((size_t)T * k > 0x7fffffffull) return RELIBRA_EINVAL;
    if (mode != RELIBRA_COMBINE_FWD && mode != RELIBRA_COMBINE_BWD && mode != RELIBRA_COMBINE_SUM)
        return RELIBRA_EINVAL;
    if (T == 0) return RELIBRA_OK;
    if (!rows_dev || !row_of_dev || !err_flag_dev || !aligned16(rows_dev)) return RELIBRA_EINVAL;
    const int N = T * k, vpr = h / 8;
    if (mode == RELIBRA_COMBINE_BWD) {
        if (!tok_dev || !gates_dev || !out_rows_dev || !dgate_dev || !aligned16(tok_dev) || !aligned16(out_rows_dev))
            return RELIBRA_EINVAL;
        RELIBRA_LAUNCH(RELIBRA_K_COMBINE_BWD, stream, combine_bwd_kernel<<<(N + 3) / 4, 256, 0, stream>>>((const uint4 *)rows_dev, (const uint4 *)tok_dev,
                                                            gates_dev, row_of_dev, N, vpr, k,
                                                            (uint4 *)out_rows_dev, dgate_dev, err_flag_dev));
    } else {
        if (!out_tok_dev || !aligned16(out_tok_dev)) return RELIBRA_EINVAL;
        const int grid = grid_for((size_t)T * vpr, 256, 256 * 64);
        if (mode == RELIBRA_COMBINE_FWD) {
            if (!gates_dev) return RELIBRA_EINVAL;
            RELIBRA_LAUNCH(RELIBRA_K_COMBINE_FWD, stream, combine_fwd_kernel<true><<<grid, 256, 0, stream>>>((const uint4 *)rows_dev, gates_dev, row_of_dev,
                                                               T, k, N, vpr, (uint4 *)out_tok_dev, err_flag_dev));
        } else {
            RELIBRA_LAUNCH(RELIBRA_K_COMBINE_SUM, stream, combine_fwd_kernel<false><<<grid, 256, 0, stream>>>((const uint4 *)rows_dev, nullptr, row_of_dev,
                                                                T, k, N, vpr, (uint4 *)out_tok_dev, err_flag_dev));
        }
    }
    RELIBRA_HIP_TRY(launch_check());
    return RELIBRA_OK;
}

extern "C" int relibra_row_tokens(const int32_t *src_of_dev, int N, int k, int T, int32_t *row_tok_dev,
                                  int32_t *err_flag_dev, relibra_stream stream_)
{
    hipStream_t stream = (hipStream_t)stream_;
    if (N < 0 || k < 1 || T < 1) return RELIBRA_EINVAL;
    if (N == 0) return RELIBRA_OK;
    if (!src_of_dev || !row_tok_dev || !err_flag_dev) return RELIBRA_EINVAL;
    RELIBRA_LAUNCH(RELIBRA_K_ROW_TOKENS, stream, row_tokens_kernel<<<grid_for((size_t)N, 256, 1024), 256, 0, stream>>>(
        src_of_dev, N, k, T, row_tok_dev, err_flag_dev));
    RELIBRA_HIP_TRY(launch_check());
    return RELIBRA_OK;
}

extern "C" int relibra_row_gates(const int32_t *src_of_dev, const float *gates_dev, int N, float *row_gate_dev,
                                 int32_t *err_flag_dev, relibra_stream stream_)
{
    hipStream_t stream = (hipStream_t)stream_;
    if (N < 0) return RELIBRA_EINVAL;
    if (N == 0) return RELIBRA_OK;
    if (!src_of_dev || !gates_dev || !row_gate_dev || !err_flag_dev) return RELIBRA_EINVAL;
    RELIBRA_LAUNCH(RELIBRA_K_ROW_GATES, stream, row_gates_kernel<<<grid_for((size_t)N, 256, 1024), 256, 0, stream>>>(
        src_of_dev, gates_dev, N, row_gate_dev, err_flag_dev));
    RELIBRA_HIP_TRY(launch_check());
    return RELIBRA_OK;
}

extern "C" const char *relibra_status_string(int status)
{
    switch (status) {
    case RELIBRA_OK: return "ok";
    case RELIBRA_EINVAL: return "invalid argument";
    case RELIBRA_ERANGE: return "table value out of range";
    case RELIBRA_EWORKSPACE: return "workspace too small";
    case RELIBRA_EHIP: return "HIP runtime error";
    case RELIBRA_EUNSUPPORTED: return "unsupported shape";
    default: return "unknown status";
    }
}
