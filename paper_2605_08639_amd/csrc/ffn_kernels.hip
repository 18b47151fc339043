// Expert FFN forward / backward as grouped bf16 MFMA GEMMs (gfx950, v_mfma_f32_32x32x16_bf16).
//
// One workgroup (4 wavefronts of 64 lanes, 2x2) owns a 128x128 output tile; a wavefront owns
// 64x64 of it as 2x2 MFMA tiles with fp32 accumulators.  Operand tiles are staged through
// LDS in [row][k] order with a 16-byte pad per row, so that every MFMA fragment is one
// conflict-free 16-byte LDS read.  Global loads of the next k-slab are issued before the
// MFMAs of the current one.
//
// Three operand situations occur (rows = the non-contracted index of an operand):
//   k-contiguous in memory  (X, A, dY, dGt, dU as left operands; Wg, Wu, Wd in the forward)
//   k-strided in memory     (weights in the data-gradient GEMMs; both operands of the
//                            weight-gradient GEMMs, whose contraction runs over a group's rows)
// The ragged dimension is always clamped (reads) and masked (writes); a ragged contraction
// (weight gradients) is zero-filled.
#include "common.h"

namespace relibra {

typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef float f32x16_t __attribute__((ext_vector_type(16)));

constexpr int BM = 128, BN = 128, BK = 64;
constexpr int LDK = BK + 8;                 // padded LDS row, in elements
constexpr int THREADS = 256;
constexpr int TM = 2, TN = 2;               // MFMA tiles per wave, 32x32 each
constexpr int CHUNKS = BM * BK / 8 / THREADS;   // 16-byte pieces per thread per operand tile (= 4)

static_assert(BM == BN, "operand tiles share one loader");

// ---------------------------------------------------------------- schedule tables
// Sanitised copies of the caller's group tables plus the list of row tiles, built on the
// device so that no host synchronisation is needed.
struct Sched {
    int32_t *hdr;          // [0] row tiles, [1] replica pairs
    int32_t *grp_row0, *grp_rows, *grp_expert, *grp_slot;   // [Gr]
    int32_t *tile_prefix;  // [Gr+1]
    int32_t *tile_group, *tile_row0, *tile_rows;            // [Rmax]
    int32_t *pair_slot, *pair_expert;                       // [Gr]
    bf16_t *dGt, *dU;      // [n_rows, hff] (backward only)
};

inline size_t round256(size_t x) { return (x + 255) & ~(size_t)255; }
inline int max_row_tiles(int n_rows, int Gr) { return (n_rows + BM - 1) / BM + Gr; }
inline size_t sched_ints(int n_rows, int Gr) { return 8 + 4 * (size_t)Gr + (Gr + 1) + 3 * (size_t)max_row_tiles(n_rows, Gr) + 2 * (size_t)Gr; }
inline size_t ffn_ws_bytes(int n_rows, int Gr, int hff, bool bwd)
{
    size_t b = round256(sched_ints(n_rows, Gr) * sizeof(int32_t));
    if (bwd) b += 2 * round256((size_t)n_rows * hff * sizeof(bf16_t));
    return b;
}
inline Sched carve(void *ws, int n_rows, int Gr, int hff, bool bwd)
{
    Sched s;
    int32_t *p = (int32_t *)ws;
    const int R = max_row_tiles(n_rows, Gr);
    s.hdr = p; p += 8;
    s.grp_row0 = p; p += Gr;
    s.grp_rows = p; p += Gr;
    s.grp_expert = p; p += Gr;
    s.grp_slot = p; p += Gr;
    s.tile_prefix = p; p += Gr + 1;
    s.tile_group = p; p += R;
    s.tile_row0 = p; p += R;
    s.tile_rows = p; p += R;
    s.pair_slot = p; p += Gr;
    s.pair_expert = p; p += Gr;
    char *q = (char *)ws + round256(sched_ints(n_rows, Gr) * sizeof(int32_t));
    s.dGt = s.dU = nullptr;
    if (bwd) {
        s.dGt = (bf16_t *)q;
        s.dU = (bf16_t *)(q + round256((size_t)n_rows * hff * sizeof(bf16_t)));
    }
    return s;
}

// One block.  Validates the group tables of [g_begin, g_end) (bad groups become empty and raise
// the flag), lists the row tiles group by group, and lists the live replica slots.
__global__ void __launch_bounds__(256)
sched_kernel(const int32_t *__restrict__ group_offset, const int32_t *__restrict__ group_expert,
             const int32_t *__restrict__ group_dw_slot, int g_begin, int Gr, int n_rows, int E, int n_dw_slots,
             Sched s, int32_t *err_flag)
{
    __shared__ int32_t scan[256];
    __shared__ int32_t carry;
    const int tid = threadIdx.x;
    if (tid == 0) { carry = 0; s.tile_prefix[0] = 0; }
    __syncthreads();
    bool bad_any = false;
    for (int base = 0; base < Gr; base += 256) {
        const int i = base + tid;
        int tiles = 0;
        if (i < Gr) {
            const int g = g_begin + i;
            int lo = group_offset[g], hi = group_offset[g + 1], e = group_expert[g];
            int slot = group_dw_slot ? group_dw_slot[g] : 0;
            bool bad = lo < 0 || hi < lo || hi > n_rows || e < -1 || e >= E;
            if (group_dw_slot && e >= 0 && (slot < 0 || slot >= n_dw_slots)) bad = true;
            if (bad) { bad_any = true; lo = hi = 0; e = -1; }
            if (e < 0) hi = lo;
            s.grp_row0[i] = lo;
            s.grp_rows[i] = hi - lo;
            s.grp_expert[i] = e;
            s.grp_slot[i] = slot;
            tiles = (hi - lo + BM - 1) / BM;
        }
        scan[tid] = tiles;
        __syncthreads();
        for (int off = 1; off < 256; off <<= 1) {
            const int v = tid >= off ? scan[tid - off] : 0;
            __syncthreads();
            scan[tid] += v;
            __syncthreads();
        }
        if (i < Gr) s.tile_prefix[i + 1] = carry + scan[tid];
        __syncthreads();
        if (tid == 255) carry += scan[255];
        __syncthreads();
    }
    if (bad_any) atomicOr(err_flag, RELIBRA_ERR_GROUP_TABLE);
    const int total = carry;
    if (tid == 0) s.hdr[0] = total;
    __threadfence_block();
    __syncthreads();
    for (int t = tid; t < total; t += 256) {
        int lo = 0, hi = Gr;                 // last group whose prefix <= t
        while (hi - lo > 1) {
            const int mid = (lo + hi) >> 1;
            if (s.tile_prefix[mid] <= t) lo = mid; else hi = mid;
        }
        const int j = t - s.tile_prefix[lo];
        s.tile_group[t] = lo;
        s.tile_row0[t] = s.grp_row0[lo] + j * BM;
        s.tile_rows[t] = min(BM, s.grp_rows[lo] - j * BM);
    }
    if (tid == 0) {
        int n = 0;
        if (group_dw_slot)
            for (int i = 0; i < Gr; ++i)
                if (s.grp_expert[i] >= 0 && s.grp_slot[i] >= E) {
                    s.pair_slot[n] = s.grp_slot[i];
                    s.pair_expert[n] = s.grp_expert[i];
                    ++n;
                }
        s.hdr[1] = n;
    }
}

// ---------------------------------------------------------------- operand tiles
struct Operand {
    const bf16_t *base;   // element (row, k): base[row*ld + k] (k-contiguous) or base[k*ld + row] (k-strided)
    int ld;
    int row0;             // first row of the tile
    int row_last;         // last valid row (reads of rows beyond it are clamped onto it)
};

struct Frag4 { uint4 v[CHUNKS]; };

template <bool KS>
__device__ __forceinline__ Frag4 load_tile(const Operand &op, int k0, int k_valid, int tid)
{
    Frag4 f;
#pragma unroll
    for (int i = 0; i < CHUNKS; ++i) {
        const int c = tid + i * THREADS;
        if (!KS) {
            const int row = min(op.row0 + c / (BK / 8), op.row_last);
            f.v[i] = *reinterpret_cast<const uint4 *>(op.base + (size_t)row * op.ld + k0 + (c % (BK / 8)) * 8);
        } else {
            const int kk = k0 + c / (BM / 8);
            int r8 = op.row0 + (c % (BM / 8)) * 8;
            if (r8 > op.row_last) r8 = op.row_last - 7;      // whole piece out of range: masked at the store
            if (kk < k_valid)
                f.v[i] = *reinterpret_cast<const uint4 *>(op.base + (size_t)kk * op.ld + r8);
            else
                f.v[i] = make_uint4(0, 0, 0, 0);
        }
    }
    return f;
}

template <bool KS>
__device__ __forceinline__ void store_tile(bf16_t (*s)[LDK], const Frag4 &f, int tid)
{
#pragma unroll
    for (int i = 0; i < CHUNKS; ++i) {
        const int c = tid + i * THREADS;
        if (!KS) {
            *reinterpret_cast<uint4 *>(&s[c / (BK / 8)][(c % (BK / 8)) * 8]) = f.v[i];
        } else {
            const int kk = c / (BM / 8), r8 = (c % (BM / 8)) * 8;
            const uint32_t w[4] = {f.v[i].x, f.v[i].y, f.v[i].z, f.v[i].w};
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                s[r8 + 2 * j][kk] = (bf16_t)(w[j] & 0xffffu);
                s[r8 + 2 * j + 1][kk] = (bf16_t)(w[j] >> 16);
            }
        }
    }
}

struct Smem {
    bf16_t t[3][BM][LDK];     // left operands first, then right operands (at most three in all)
};

// acc[a*NB+b][i][j] += A_a(tile) * B_b(tile)^T over k in [k_begin, k_end).
template <int NA, int NB, bool A_KS, bool B_KS>
__device__ __forceinline__ void mainloop(f32x16_t (&acc)[NA * NB][TM][TN], const Operand (&A)[NA],
                                         const Operand (&B)[NB], int k_begin, int k_end, int k_valid,
                                         Smem &sm, int tid)
{
    const int lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1;
    Frag4 ra[NA], rb[NB];
#pragma unroll
    for (int a = 0; a < NA; ++a) ra[a] = load_tile<A_KS>(A[a], k_begin, k_valid, tid);
#pragma unroll
    for (int b = 0; b < NB; ++b) rb[b] = load_tile<B_KS>(B[b], k_begin, k_valid, tid);
    for (int k0 = k_begin; k0 < k_end; k0 += BK) {
        __syncthreads();
#pragma unroll
        for (int a = 0; a < NA; ++a) store_tile<A_KS>(sm.t[a], ra[a], tid);
#pragma unroll
        for (int b = 0; b < NB; ++b) store_tile<B_KS>(sm.t[NA + b], rb[b], tid);
        __syncthreads();
        if (k0 + BK < k_end) {
#pragma unroll
            for (int a = 0; a < NA; ++a) ra[a] = load_tile<A_KS>(A[a], k0 + BK, k_valid, tid);
#pragma unroll
            for (int b = 0; b < NB; ++b) rb[b] = load_tile<B_KS>(B[b], k0 + BK, k_valid, tid);
        }
#pragma unroll
        for (int kk = 0; kk < BK; kk += 16) {
            const int kofs = kk + (lane >> 5) * 8;
            bf16x8_t fa[NA][TM], fb[NB][TN];
#pragma unroll
            for (int a = 0; a < NA; ++a)
#pragma unroll
                for (int i = 0; i < TM; ++i)
                    fa[a][i] = *reinterpret_cast<const bf16x8_t *>(&sm.t[a][wm * 64 + i * 32 + (lane & 31)][kofs]);
#pragma unroll
            for (int b = 0; b < NB; ++b)
#pragma unroll
                for (int j = 0; j < TN; ++j)
                    fb[b][j] = *reinterpret_cast<const bf16x8_t *>(&sm.t[NA + b][wn * 64 + j * 32 + (lane & 31)][kofs]);
#pragma unroll
            for (int a = 0; a < NA; ++a)
#pragma unroll
                for (int b = 0; b < NB; ++b)
#pragma unroll
                    for (int i = 0; i < TM; ++i)
#pragma unroll
                        for (int j = 0; j < TN; ++j)
                            acc[a * NB + b][i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(
                                fa[a][i], fb[b][j], acc[a * NB + b][i][j], 0, 0, 0);
        }
    }
}

template <int N>
__device__ __forceinline__ void zero_acc(f32x16_t (&acc)[N][TM][TN])
{
#pragma unroll
    for (int n = 0; n < N; ++n)
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j)
#pragma unroll
                for (int v = 0; v < 16; ++v) acc[n][i][j][v] = 0.0f;
}

// Visit every accumulator element of this lane: f(r, c, i, j, v) with (r, c) inside the 128x128 tile.
template <typename F>
__device__ __forceinline__ void for_each_acc(int tid, F f)
{
    const int lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1;
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int r = wm * 64 + i * 32 + 8 * (v >> 2) + 4 * (lane >> 5) + (v & 3);
                const int c = wn * 64 + j * 32 + (lane & 31);
                f(r, c, i, j, v);
            }
}

__device__ __forceinline__ float sigmoidf_(float x) { return 1.0f / (1.0f + __expf(-x)); }

// ---------------------------------------------------------------- forward kernels
// Gt = X Wg^T, U = X Wu^T (one pass over X), A = silu(Gt) * U.
__global__ void __launch_bounds__(THREADS)
fwd_gate_up_kernel(Sched s, const bf16_t *__restrict__ X, const bf16_t *__restrict__ Wg,
                   const bf16_t *__restrict__ Wu, int h, int hff, int n_col_tiles,
                   bf16_t *__restrict__ Gt, bf16_t *__restrict__ U, bf16_t *__restrict__ Aout)
{
    __shared__ Smem sm;
    const int rt = blockIdx.x / n_col_tiles, ct = blockIdx.x % n_col_tiles;
    if (rt >= s.hdr[0]) return;
    const int tid = threadIdx.x;
    const int g = s.tile_group[rt], row0 = s.tile_row0[rt], rows = s.tile_rows[rt];
    const int e = s.grp_expert[g];
    const size_t wofs = (size_t)e * hff * h;
    const int col0 = ct * BN, cols = min(BN, hff - col0);
    Operand A[1] = {{X, h, row0, row0 + rows - 1}};
    Operand B[2] = {{Wg + wofs, h, col0, hff - 1}, {Wu + wofs, h, col0, hff - 1}};
    f32x16_t acc[2][TM][TN];
    zero_acc(acc);
    mainloop<1, 2, false, false>(acc, A, B, 0, h, h, sm, tid);
    for_each_acc(tid, [&](int r, int c, int i, int j, int v) {
        if (r < rows && c < cols) {
            const float gt = acc[0][i][j][v], u = acc[1][i][j][v];
            const size_t o = (size_t)(row0 + r) * hff + col0 + c;
            Gt[o] = f2bf(gt);
            U[o] = f2bf(u);
            Aout[o] = f2bf(gt * sigmoidf_(gt) * u);
        }
    });
}

// Y = A Wd^T.
__global__ void __launch_bounds__(THREADS)
fwd_down_kernel(Sched s, const bf16_t *__restrict__ Ain, const bf16_t *__restrict__ Wd, int h, int hff,
                int n_col_tiles, bf16_t *__restrict__ Y)
{
    __shared__ Smem sm;
    const int rt = blockIdx.x / n_col_tiles, ct = blockIdx.x % n_col_tiles;
    if (rt >= s.hdr[0]) return;
    const int tid = threadIdx.x;
    const int g = s.tile_group[rt], row0 = s.tile_row0[rt], rows = s.tile_rows[rt];
    const int e = s.grp_expert[g];
    const int col0 = ct * BN, cols = min(BN, h - col0);
    Operand A[1] = {{Ain, hff, row0, row0 + rows - 1}};
    Operand B[1] = {{Wd + (size_t)e * h * hff, hff, col0, h - 1}};
    f32x16_t acc[1][TM][TN];
    zero_acc(acc);
    mainloop<1, 1, false, false>(acc, A, B, 0, hff, hff, sm, tid);
    for_each_acc(tid, [&](int r, int c, int i, int j, int v) {
        if (r < rows && c < cols) Y[(size_t)(row0 + r) * h + col0 + c] = f2bf(acc[0][i][j][v]);
    });
}

// ---------------------------------------------------------------- backward kernels
// dA = dY Wd, then dGt = dA * U * silu'(Gt), dU = dA * silu(Gt).
__global__ void __launch_bounds__(THREADS)
bwd_act_kernel(Sched s, const bf16_t *__restrict__ dY, const bf16_t *__restrict__ Wd,
               const bf16_t *__restrict__ Gt, const bf16_t *__restrict__ U, int h, int hff, int n_col_tiles)
{
    __shared__ Smem sm;
    const int rt = blockIdx.x / n_col_tiles, ct = blockIdx.x % n_col_tiles;
    if (rt >= s.hdr[0]) return;
    const int tid = threadIdx.x;
    const int g = s.tile_group[rt], row0 = s.tile_row0[rt], rows = s.tile_rows[rt];
    const int e = s.grp_expert[g];
    const int col0 = ct * BN, cols = min(BN, hff - col0);
    Operand A[1] = {{dY, h, row0, row0 + rows - 1}};
    Operand B[1] = {{Wd + (size_t)e * h * hff, hff, col0, hff - 1}};     // (n in hff, k in h) at [k*hff + n]
    f32x16_t acc[1][TM][TN];
    zero_acc(acc);
    mainloop<1, 1, false, true>(acc, A, B, 0, h, h, sm, tid);
    for_each_acc(tid, [&](int r, int c, int i, int j, int v) {
        if (r < rows && c < cols) {
            const size_t o = (size_t)(row0 + r) * hff + col0 + c;
            const float da = acc[0][i][j][v], gt = bf2f(Gt[o]), u = bf2f(U[o]);
            const float sg = sigmoidf_(gt);
            s.dGt[o] = f2bf(da * u * (sg * (1.0f + gt * (1.0f - sg))));
            s.dU[o] = f2bf(da * (gt * sg));
        }
    });
}

// dX = dGt Wg + dU Wu (one accumulator, the contraction runs over both products).
__global__ void __launch_bounds__(THREADS)
bwd_dx_kernel(Sched s, const bf16_t *__restrict__ Wg, const bf16_t *__restrict__ Wu, int h, int hff,
              int n_col_tiles, bf16_t *__restrict__ dX)
{
    __shared__ Smem sm;
    const int rt = blockIdx.x / n_col_tiles, ct = blockIdx.x % n_col_tiles;
    if (rt >= s.hdr[0]) return;
    const int tid = threadIdx.x;
    const int g = s.tile_group[rt], row0 = s.tile_row0[rt], rows = s.tile_rows[rt];
    const int e = s.grp_expert[g];
    const size_t wofs = (size_t)e * hff * h;
    const int col0 = ct * BN, cols = min(BN, h - col0);
    f32x16_t acc[1][TM][TN];
    zero_acc(acc);
    {
        Operand A[1] = {{s.dGt, hff, row0, row0 + rows - 1}};
        Operand B[1] = {{Wg + wofs, h, col0, h - 1}};                    // (n in h, k in hff) at [k*h + n]
        mainloop<1, 1, false, true>(acc, A, B, 0, hff, hff, sm, tid);
    }
    {
        Operand A[1] = {{s.dU, hff, row0, row0 + rows - 1}};
        Operand B[1] = {{Wu + wofs, h, col0, h - 1}};
        mainloop<1, 1, false, true>(acc, A, B, 0, hff, hff, sm, tid);
    }
    for_each_acc(tid, [&](int r, int c, int i, int j, int v) {
        if (r < rows && c < cols) dX[(size_t)(row0 + r) * h + col0 + c] = f2bf(acc[0][i][j][v]);
    });
}

// Weight gradients: out[slot][m][n] (+)= sum over the group's rows of L[row][m] * R[row][n].
// NA = 2 computes two left operands against one right operand (dGt and dU against X).
template <int NA>
__global__ void __launch_bounds__(THREADS)
wgrad_kernel(Sched s, const bf16_t *__restrict__ L0, const bf16_t *__restrict__ L1,
             const bf16_t *__restrict__ R, int m_dim, int n_dim, int E, int accumulate,
             float *__restrict__ out0, float *__restrict__ out1)
{
    __shared__ Smem sm;
    const int n_nt = (n_dim + BN - 1) / BN, n_mt = (m_dim + BM - 1) / BM;
    const int per_group = n_nt * n_mt;
    const int gi = blockIdx.x / per_group, rem = blockIdx.x % per_group;
    const int e = s.grp_expert[gi];
    if (e < 0) return;
    const int slot = s.grp_slot[gi];
    const bool add = accumulate && slot < E;
    const int row0 = s.grp_row0[gi], rows = s.grp_rows[gi];
    if (rows == 0 && add) return;
    const int tid = threadIdx.x;
    const int m0 = (rem / n_nt) * BM, n0 = (rem % n_nt) * BN;
    Operand A[NA];
    A[0] = {L0 + (size_t)row0 * m_dim, m_dim, m0, m_dim - 1};
    if (NA == 2) A[NA - 1] = {L1 + (size_t)row0 * m_dim, m_dim, m0, m_dim - 1};
    Operand B[1] = {{R + (size_t)row0 * n_dim, n_dim, n0, n_dim - 1}};
    f32x16_t acc[NA][TM][TN];
    zero_acc(acc);
    const int k_end = (rows + BK - 1) / BK * BK;
    mainloop<NA, 1, true, true>(acc, A, B, 0, k_end, rows, sm, tid);
    const size_t base = (size_t)slot * m_dim * n_dim;
    const int mv = min(BM, m_dim - m0), nv = min(BN, n_dim - n0);
    for_each_acc(tid, [&](int r, int c, int i, int j, int v) {
        if (r < mv && c < nv) {
            const size_t o = base + (size_t)(m0 + r) * n_dim + n0 + c;
            if (add) {
                out0[o] += acc[0][i][j][v];
                if (NA == 2) out1[o] += acc[NA - 1][i][j][v];
            } else {
                out0[o] = acc[0][i][j][v];
                if (NA == 2) out1[o] = acc[NA - 1][i][j][v];
            }
        }
    });
}

// Replica gradients return to the home copy (Section 5.1).  A thread owns element positions
// and walks the live replica slots in ascending slot order, so the sum has a fixed order.
__global__ void __launch_bounds__(256)
replica_sum_kernel(Sched s, size_t per_expert_vec4, float4 *__restrict__ dW)
{
    const int n_pairs = s.hdr[1];
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < per_expert_vec4; i += (size_t)gridDim.x * 256)
        for (int p = 0; p < n_pairs; ++p) {
            const float4 src = dW[(size_t)s.pair_slot[p] * per_expert_vec4 + i];
            float4 *dst = &dW[(size_t)s.pair_expert[p] * per_expert_vec4 + i];
            float4 d = *dst;
            d.x += src.x; d.y += src.y; d.z += src.z; d.w += src.w;
            *dst = d;
        }
}

struct FfnArgs {
    int n_rows, G, g_begin, g_end, E, h, hff;
};

inline int check_ffn_args(const FfnArgs &a)
{
    if (a.n_rows < 0 || a.G < 1 || a.g_begin < 0 || a.g_end > a.G || a.g_begin > a.g_end || a.E < 1) return RELIBRA_EINVAL;
    if (a.h < 64 || a.hff < 64 || a.h % 64 || a.hff % 64) return RELIBRA_EUNSUPPORTED;
    if ((size_t)a.n_rows * (size_t)(a.h > a.hff ? a.h : a.hff) > ((size_t)1 << 40)) return RELIBRA_EUNSUPPORTED;
    return RELIBRA_OK;
}

}  // namespace relibra

using namespace relibra;

extern "C" size_t relibra_workspace_bytes(int which, int T, int k, int E, int G, int h, int hff)
{
    if (T < 0 || k < 1 || E < 1 || G < 1 || (size_t)T * k > 0x7fffffffull) return 0;
    const int N = T * k;
    switch (which) {
    case RELIBRA_WS_PERMUTE: return round256((size_t)((N + 511) / 512 + 4) * E * sizeof(int32_t));
    case RELIBRA_WS_FFN_FWD: return ffn_ws_bytes(N, G, hff, false);
    case RELIBRA_WS_FFN_BWD: return ffn_ws_bytes(N, G, hff, true);
    default: return 0;
    }
    (void)h;
}

extern "C" int relibra_moe_ffn_fwd(const void *Xrows, int n_rows,
                                   const int32_t *group_offset, const int32_t *group_expert,
                                   int G, int g_begin, int g_end, int E,
                                   const void *Wg, const void *Wu, const void *Wd, int h, int hff,
                                   void *Gt_save, void *U_save, void *A_save, void *Yrows,
                                   void *ws, size_t ws_bytes, int32_t *err_flag, relibra_stream stream_)
{
    hipStream_t stream = (hipStream_t)stream_;
    const FfnArgs a{n_rows, G, g_begin, g_end, E, h, hff};
    if (int rc = check_ffn_args(a)) return rc;
    const int Gr = g_end - g_begin;
    if (Gr == 0 || n_rows == 0) return RELIBRA_OK;
    if (!Xrows || !group_offset || !group_expert || !Wg || !Wu || !Wd || !Gt_save || !U_save || !A_save ||
        !Yrows || !ws || !err_flag)
        return RELIBRA_EINVAL;
    if (!aligned16(Xrows) || !aligned16(Wg) || !aligned16(Wu) || !aligned16(Wd) || !aligned16(A_save) ||
        !aligned16(ws))
        return RELIBRA_EINVAL;
    if (ws_bytes < ffn_ws_bytes(n_rows, Gr, hff, false)) return RELIBRA_EWORKSPACE;
    Sched s = carve(ws, n_rows, Gr, hff, false);
    RELIBRA_LAUNCH(RELIBRA_K_SCHED, stream, sched_kernel<<<1, 256, 0, stream>>>(group_offset, group_expert, nullptr, g_begin, Gr, n_rows, E, 0, s, err_flag));
    RELIBRA_HIP_TRY(launch_check());
    const int R = max_row_tiles(n_rows, Gr);
    const int ct1 = (hff + BN - 1) / BN, ct2 = (h + BN - 1) / BN;
    RELIBRA_LAUNCH(RELIBRA_K_FWD_GATE_UP, stream, fwd_gate_up_kernel<<<(unsigned)(R * ct1), THREADS, 0, stream>>>(
        s, (const bf16_t *)Xrows, (const bf16_t *)Wg, (const bf16_t *)Wu, h, hff, ct1,
        (bf16_t *)Gt_save, (bf16_t *)U_save, (bf16_t *)A_save));
    RELIBRA_HIP_TRY(launch_check());
    RELIBRA_LAUNCH(RELIBRA_K_FWD_DOWN, stream, fwd_down_kernel<<<(unsigned)(R * ct2), THREADS, 0, stream>>>(
        s, (const bf16_t *)A_save, (const bf16_t *)Wd, h, hff, ct2, (bf16_t *)Yrows));
    RELIBRA_HIP_TRY(launch_check());
    return RELIBRA_OK;
}

extern "C" int relibra_moe_ffn_bwd(const void *dYrows, const void *Xrows,
                                   const void *Gt_save, const void *U_save, const void *A_save, int n_rows,
                                   const int32_t *group_offset, const int32_t *group_expert,
                                   const int32_t *group_dw_slot,
                                   int G, int g_begin, int g_end, int E, int n_dw_slots,
                                   const void *Wg, const void *Wu, const void *Wd, int h, int hff,
                                   void *dXrows, float *dWg, float *dWu, float *dWd, int flags,
                                   void *ws, size_t ws_bytes, int32_t *err_flag, relibra_stream stream_)
{
    hipStream_t stream = (hipStream_t)stream_;
    const FfnArgs a{n_rows, G, g_begin, g_end, E, h, hff};
    if (int rc = check_ffn_args(a)) return rc;
    if (n_dw_slots < E) return RELIBRA_EINVAL;
    const int Gr = g_end - g_begin;
    if (Gr == 0) return RELIBRA_OK;
    if (!dYrows || !Xrows || !Gt_save || !U_save || !A_save || !group_offset || !group_expert || !group_dw_slot ||
        !Wg || !Wu || !Wd || !dXrows || !dWg || !dWu || !dWd || !ws || !err_flag)
        return RELIBRA_EINVAL;
    if (!aligned16(dYrows) || !aligned16(Xrows) || !aligned16(A_save) || !aligned16(Wg) || !aligned16(Wu) ||
        !aligned16(Wd) || !aligned16(dWg) || !aligned16(dWu) || !aligned16(dWd) || !aligned16(ws))
        return RELIBRA_EINVAL;
    if (ws_bytes < ffn_ws_bytes(n_rows, Gr, hff, true)) return RELIBRA_EWORKSPACE;
    Sched s = carve(ws, n_rows, Gr, hff, true);
    RELIBRA_LAUNCH(RELIBRA_K_SCHED, stream, sched_kernel<<<1, 256, 0, stream>>>(group_offset, group_expert, group_dw_slot, g_begin, Gr, n_rows, E,
                                        n_dw_slots, s, err_flag));
    RELIBRA_HIP_TRY(launch_check());
    const int R = max_row_tiles(n_rows, Gr);
    const int ct_ff = (hff + BN - 1) / BN, ct_h = (h + BN - 1) / BN;
    const int accumulate = (flags & RELIBRA_BWD_ACCUMULATE) ? 1 : 0;
    if (n_rows > 0) {
        RELIBRA_LAUNCH(RELIBRA_K_BWD_ACT, stream, bwd_act_kernel<<<(unsigned)(R * ct_ff), THREADS, 0, stream>>>(
            s, (const bf16_t *)dYrows, (const bf16_t *)Wd, (const bf16_t *)Gt_save, (const bf16_t *)U_save,
            h, hff, ct_ff));
        RELIBRA_HIP_TRY(launch_check());
        RELIBRA_LAUNCH(RELIBRA_K_BWD_DX, stream, bwd_dx_kernel<<<(unsigned)(R * ct_h), THREADS, 0, stream>>>(
            s, (const bf16_t *)Wg, (const bf16_t *)Wu, h, hff, ct_h, (bf16_t *)dXrows));
        RELIBRA_HIP_TRY(launch_check());
    }
    const int tiles = ct_ff * ct_h;
    RELIBRA_LAUNCH(RELIBRA_K_WGRAD_DOWN, stream, wgrad_kernel<1><<<(unsigned)(Gr * tiles), THREADS, 0, stream>>>(
        s, (const bf16_t *)dYrows, nullptr, (const bf16_t *)A_save, h, hff, E, accumulate, dWd, nullptr));
    RELIBRA_HIP_TRY(launch_check());
    RELIBRA_LAUNCH(RELIBRA_K_WGRAD_GATE_UP, stream, wgrad_kernel<2><<<(unsigned)(Gr * tiles), THREADS, 0, stream>>>(
        s, s.dGt, s.dU, (const bf16_t *)Xrows, hff, h, E, accumulate, dWg, dWu));
    RELIBRA_HIP_TRY(launch_check());
    if (!(flags & RELIBRA_BWD_NO_REPLICA_SUM) && n_dw_slots > E) {
        const size_t vec4 = (size_t)h * hff / 4;
        const int grid = (int)((vec4 + 255) / 256 < 4096 ? (vec4 + 255) / 256 : 4096);
        RELIBRA_LAUNCH(RELIBRA_K_REPLICA_SUM, stream, replica_sum_kernel<<<grid, 256, 0, stream>>>(s, vec4, (float4 *)dWg));
        RELIBRA_LAUNCH(RELIBRA_K_REPLICA_SUM, stream, replica_sum_kernel<<<grid, 256, 0, stream>>>(s, vec4, (float4 *)dWu));
        RELIBRA_LAUNCH(RELIBRA_K_REPLICA_SUM, stream, replica_sum_kernel<<<grid, 256, 0, stream>>>(s, vec4, (float4 *)dWd));
        RELIBRA_HIP_TRY(launch_check());
    }
    return RELIBRA_OK;
}
