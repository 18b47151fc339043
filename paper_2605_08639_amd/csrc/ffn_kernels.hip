// Expert FFN forward / backward as grouped bf16 MFMA GEMMs (gfx950, v_mfma_f32_32x32x16_bf16).
//
// A wavefront always owns 64 rows x 128 columns of the output as 2 x 4 MFMA tiles with fp32
// accumulators, two wavefronts per SIMD.  Row-tiled kernels (forward, data gradients) come in two
// workgroup shapes: narrow, 4 waves = 128 rows x 256 columns, 72 KiB of LDS, two workgroups per
// compute unit; wide, 8 waves = 128 rows x 512 columns (gate/up: 2 x 256), one workgroup per
// compute unit, used where the wide tile divides the output width (the rows' slab is loaded once
// for twice the columns).  A group's tail of at most 64 rows runs as a 64-row tile.  Operand slabs
// of 32 k-values go global -> LDS directly (global_load_lds, 16 bytes per lane) through a ring of
// three slabs (four in the wide weight-gradient tile); the wide row tiles stage their rows 64
// k-values deep (full 128-byte lines) in a ring of their own, 144 KiB of LDS in all; see gemm_tile.h
// for the tile layouts and the pipeline.
//
// MFMA operand roles: the lanes carry the index that is contiguous in the output's memory
// only for the fp32 weight gradients (128-byte runs per store); for the bf16 row tensors the
// lanes carry the row index and each lane holds 4 consecutive columns, re-laid through per-wave
// LDS staging so that global accesses are 16 bytes per lane along rows.
// The ragged dimension is always clamped (reads) and masked (writes); a ragged contraction
// (weight gradients) is masked to zero in the fragments.
//
// Block index -> tile: XCD x (blockIdx % 8) takes the x-th eighth of the ordered tile list, so
// that operand tiles shared by neighbouring tiles are served by one L2.
//
// Weight gradients exist in two forms: per micro-batch (read-add-write of fp32 dW, replica slots
// summed into the home slot) and once per batch over every resident micro-batch, contracted in
// registers (wgrad_batched_kernel), which avoids the dW traffic that dominates short groups.
#include "gemm_tile.h"

#include <mutex>
#include <type_traits>

namespace relibra {

// Tile geometry: 4 waves, 128-row x 256-column tiles, three LDS slabs, two workgroups per
// compute unit (one group's prologue and epilogue overlap the other's MFMAs).
constexpr int BM = 128;                     // rows of a full row tile
constexpr int NWAVES = BM / 32;
constexpr int THREADS = NWAVES * 64;
constexpr int NSTAGES = 3;
constexpr int WGN = BM;                     // output columns of a weight-gradient tile

// ---------------------------------------------------------------- schedule tables
// Sanitised copies of the caller's group tables plus the list of row tiles, built on the
// device so that no host synchronisation is needed.
struct Sched {
    int32_t *hdr;          // [0] row tiles, [1] replica pairs
    int32_t *grp_row0, *grp_rows, *grp_expert, *grp_slot;   // [Gr]
    int32_t *tile_prefix;  // [Gr+1]
    int32_t *tile_group, *tile_row0, *tile_rows;            // [Rmax]
    int32_t *tile_band;    // [Rmax] band of the row tile: first row tile | number of row tiles << 24
    int32_t *pair_slot, *pair_expert;                       // [Gr]
    bf16_t *dGt, *dU;      // [n_rows, hff] (backward only)
};

inline size_t round256(size_t x) { return (x + 255) & ~(size_t)255; }
inline int max_row_tiles(int n_rows, int Gr) { return (n_rows + BM - 1) / BM + Gr; }
constexpr int kLdsBytes = NSTAGES * (256 + BM) * BK * 2;   // NSTAGES slabs of 256 + BM operand rows
// The row-tiled GEMMs also come with a tile twice as wide (512 columns, or 2 x 256 for gate and up)
// run by eight waves, one workgroup per compute unit: the same 128 x 64 per wave and two waves
// per SIMD, but the rows' slab is loaded once for twice the columns (five load instructions per
// wave and slab instead of six, one of them instead of two on the half-line k-contiguous rows);
// measured on dense problems of these shapes: 17-20 % faster.
constexpr int kWideRowWaves = 8;
// In the wide tiles the rows (the k-contiguous operand) are staged 64 k-values deep, in full 128-byte
// lines, through a ring of their own (KLoop, deep B side): three slabs of 512 weight rows plus three
// 64-deep tiles of 128 rows.
constexpr int kRowDepthWide = 2 * BK;
constexpr int kLdsBytesWide = NSTAGES * 512 * BK * 2 + ((NSTAGES + 3) / 2) * BM * kRowDepthWide * 2;
static_assert(kLdsBytesWide >= NSTAGES * (512 + BM) * BK * 2 && kLdsBytesWide >= 8 * 64 * 128 * 2 && kLdsBytesWide <= 160 * 1024,
              "slabs and the epilogue's staging (8 waves x 64 x 128 bf16) fit");
constexpr int kDgateParts = 4;                 // partial gate-gradient sums per row and 256-column tile (one per wave column at most)
inline size_t dgate_scratch_bytes(int n_rows, int hff) { return round256((size_t)kDgateParts * ((hff + 255) / 256) * n_rows * sizeof(float)); }
inline size_t sched_ints(int n_rows, int Gr) { return 8 + 4 * (size_t)Gr + (Gr + 1) + 4 * (size_t)max_row_tiles(n_rows, Gr) + 2 * (size_t)Gr; }
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
    s.tile_band = p; p += R;
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

// Order of the tiles.  A group's row tiles are cut into bands of kBand; the tiles of a band run
// column tile by column tile, the band's row tiles innermost, so that the tiles a set of compute
// units works on at one time share weight column tiles as well as row tiles.  Against row-major
// order over the group this takes 15 to 27 % off the HBM reads of the forward gate/up and the
// dX kernels (measured, bands of 8) and about 1 % off their time: the L2 misses are not what
// bounds them.
constexpr int kBand = 8;
constexpr int kMaxSchedGroups = 8192;          // groups of one call (g_end - g_begin)

// One block.  Validates the group tables of [g_begin, g_end) (bad groups become empty and raise
// the flag), lists the row tiles group by group, and lists the live replica slots.
__global__ void __launch_bounds__(256)
sched_kernel(const int32_t *__restrict__ group_offset, const int32_t *__restrict__ group_expert,
             const int32_t *__restrict__ group_dw_slot, int g_begin, int Gr, int n_rows, int E, int n_dw_slots,
             Sched s, int32_t *err_flag)
{
    extern __shared__ int32_t prefix[];        // [Gr + 1] tile_prefix, kept in LDS for the searches below
    __shared__ int32_t scan[256];
    __shared__ int32_t carry;
    const int tid = threadIdx.x;
    if (tid == 0) { carry = 0; s.tile_prefix[0] = 0; prefix[0] = 0; }
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
        if (i < Gr) s.tile_prefix[i + 1] = prefix[i + 1] = carry + scan[tid];
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
            if (prefix[mid] <= t) lo = mid; else hi = mid;
        }
        const int j = t - prefix[lo];
        s.tile_group[t] = lo;
        s.tile_row0[t] = s.grp_row0[lo] + j * BM;
        s.tile_rows[t] = min(BM, s.grp_rows[lo] - j * BM);
        const int m = prefix[lo + 1] - prefix[lo], b0 = j / kBand * kBand;
        s.tile_band[t] = (prefix[lo] + b0) | (min(kBand, m - b0) << 24);
    }
    // live replica slots, in group order (256 groups at a time; a running count in LDS)
    if (tid == 0) carry = 0;
    __syncthreads();
    if (group_dw_slot) {
        for (int base = 0; base < Gr; base += 256) {
            const int i = base + tid;
            const bool live = i < Gr && s.grp_expert[i] >= 0 && s.grp_slot[i] >= E;
            scan[tid] = live ? 1 : 0;
            __syncthreads();
            for (int off = 1; off < 256; off <<= 1) {
                const int v = tid >= off ? scan[tid - off] : 0;
                __syncthreads();
                scan[tid] += v;
                __syncthreads();
            }
            if (live) {
                const int at = carry + scan[tid] - 1;
                s.pair_slot[at] = s.grp_slot[i];
                s.pair_expert[at] = s.grp_expert[i];
            }
            __syncthreads();
            if (tid == 255) carry += scan[255];
            __syncthreads();
        }
    }
    if (tid == 0) s.hdr[1] = carry;
}

// ---------------------------------------------------------------- tile lookup
struct RowTile {
    int group, row0, rows, expert, col0;
    bool valid;
};

// Order of the tiles of an n_r x n_c grid (weight gradients): bands of kGridBand rows; inside a
// band column by column, the band's rows innermost.  The ~64 tiles a set of compute units works
// on at one time then form a roughly square patch (8 x 8), which shares 8 + 8 operand tiles
// instead of 1 + 64.
constexpr int kGridBand = 8;
__device__ __forceinline__ void band_order(int idx, int n_r, int n_c, int &r, int &c)
{
    const int band = idx / (kGridBand * n_c), within = idx - band * (kGridBand * n_c);
    const int rows_here = min(kGridBand, n_r - band * kGridBand);
    c = within / rows_here;
    r = band * kGridBand + within - c * rows_here;
}

// Physical block -> tile.  The hardware deals blocks to the 8 XCDs round-robin (blockIdx % 8);
// XCD x takes the x-th eighth of the ordered tile list, so neighbouring tiles share one L2.
__device__ __forceinline__ RowTile find_row_tile(const Sched &s, int n_col_tiles, int col_tile_width, bool w_from_slot = false)
{
    RowTile t;
    const int n_rt = s.hdr[0];
    const int total = n_rt * n_col_tiles;
    const int per_xcd = (total + 7) >> 3;
    const int logical = (blockIdx.x & 7) * per_xcd + (blockIdx.x >> 3);
    t.valid = logical < total && (int)(blockIdx.x >> 3) < per_xcd;
    if (!t.valid) return t;
    // the band that holds row tile logical / n_col_tiles holds tile `logical`
    const int band = s.tile_band[logical / n_col_tiles];
    const int first = band & 0xffffff, rows_here = band >> 24;
    const int within = logical - first * n_col_tiles;
    const int ct = within / rows_here, rt = first + within - ct * rows_here;
    t.group = s.tile_group[rt];
    t.row0 = s.tile_row0[rt];
    t.rows = s.tile_rows[rt];
    t.expert = w_from_slot ? s.grp_slot[t.group] : s.grp_expert[t.group];   // index of the parameter block
    t.col0 = ct * col_tile_width;
    return t;
}

// 1 / (1 + e^-x) with the hardware reciprocal (1 ulp; the result is rounded to bf16 anyway): a
// plain division expands to the ten-instruction IEEE sequence, 128 times per lane and tile.
__device__ __forceinline__ float sigmoidf_(float x) { return __builtin_amdgcn_rcpf(1.0f + __expf(-x)); }

__device__ __forceinline__ uint2 pack4bf(float a, float b, float c, float d)
{
    uint2 w;
    w.x = pack2bf(a, b);
    w.y = pack2bf(c, d);
    return w;
}
__device__ __forceinline__ void unpack4bf(uint2 w, float (&f)[4])
{
    f[0] = __uint_as_float(w.x << 16);
    f[1] = __uint_as_float(w.x & 0xffff0000u);
    f[2] = __uint_as_float(w.y << 16);
    f[3] = __uint_as_float(w.y & 0xffff0000u);
}

// Per-wave LDS staging between the accumulator layout (a lane holds 4 consecutive columns of
// its row) and the row-major layout (a row's columns spread over consecutive lanes), so that
// global accesses of the epilogue are 16 bytes per lane along rows: full cache lines.
// A wave stages 64 rows x NCOLS bf16; 16-byte pieces of a row are XOR-ed with the row number.
template <int NCOLS>
struct WaveStage {
    static constexpr int PIECES = NCOLS / 8;
    static constexpr int BYTES = 64 * NCOLS * 2;
    static constexpr int ROWS_PER_PASS = 64 / PIECES;
    static constexpr int PASSES = 64 / ROWS_PER_PASS;

    // accumulator side: 8 bytes = columns col..col+3 (col % 4 == 0) of `row`
    static __device__ __forceinline__ int acc_addr(int row, int col)
    {
        return row * (NCOLS * 2) + ((((col >> 3) ^ row) & (PIECES - 1)) << 4) + ((col >> 2) & 1) * 8;
    }
    static __device__ __forceinline__ void put(char *buf, int row, int col, uint2 v) { *reinterpret_cast<uint2 *>(buf + acc_addr(row, col)) = v; }
    static __device__ __forceinline__ uint2 get(const char *buf, int row, int col) { return *reinterpret_cast<const uint2 *>(buf + acc_addr(row, col)); }

    // row-major side: stage -> global, rows grow0.. of a tensor with leading dimension ld.
    // All LDS reads first, then the (predicated) stores: left to itself the compiler moves every
    // read into the branch of its store, and each store then waits for its own read in turn.
    static __device__ __forceinline__ void flush(const char *buf, bf16_t *out, int ld, int grow0, int row_end,
                                                 int gcol0, int n_dim, int lane)
    {
        uint4 v[PASSES];
#pragma unroll
        for (int p = 0; p < PASSES; ++p) {
            const int r = p * ROWS_PER_PASS + lane / PIECES, piece = lane % PIECES;
            v[p] = *reinterpret_cast<const uint4 *>(buf + r * (NCOLS * 2) + (((piece ^ r) & (PIECES - 1)) << 4));
        }
#pragma unroll
        for (int p = 0; p < PASSES; ++p)          // the values are needed here: the reads stay above
            asm volatile("" : "+v"(v[p].x), "+v"(v[p].y), "+v"(v[p].z), "+v"(v[p].w));
#pragma unroll
        for (int p = 0; p < PASSES; ++p) {
            const int r = p * ROWS_PER_PASS + lane / PIECES, piece = lane % PIECES;
            if (grow0 + r < row_end && gcol0 + piece * 8 < n_dim)
                *reinterpret_cast<uint4 *>(out + (size_t)(grow0 + r) * ld + gcol0 + piece * 8) = v[p];
        }
    }
    // global -> stage.  Rows and columns beyond the tensor are read from clamped (valid) addresses
    // instead of being skipped: what lands in their places is never stored by flush, and without
    // the predicates all loads of the fill are in flight together (predicated, every load was
    // waited for before the next one went out: one memory round trip per pass).
    // Needs grow0 < row_end and n_dim >= 8.
    // two tensors of the same shape into two staging areas, all loads in flight together
    static __device__ __forceinline__ void fill2(char *buf0, char *buf1, const bf16_t *in0, const bf16_t *in1, int ld, int grow0,
                                                 int row_end, int gcol0, int n_dim, int lane)
    {
        uint4 v0[PASSES], v1[PASSES];
#pragma unroll
        for (int p = 0; p < PASSES; ++p) {
            const int r = p * ROWS_PER_PASS + lane / PIECES, piece = lane % PIECES;
            const size_t at = (size_t)min(grow0 + r, row_end - 1) * ld + min(gcol0 + piece * 8, n_dim - 8);
            v0[p] = *reinterpret_cast<const uint4 *>(in0 + at);
            v1[p] = *reinterpret_cast<const uint4 *>(in1 + at);
        }
#pragma unroll
        for (int p = 0; p < PASSES; ++p) {
            const int r = p * ROWS_PER_PASS + lane / PIECES, piece = lane % PIECES;
            const int at = r * (NCOLS * 2) + (((piece ^ r) & (PIECES - 1)) << 4);
            *reinterpret_cast<uint4 *>(buf0 + at) = v0[p];
            *reinterpret_cast<uint4 *>(buf1 + at) = v1[p];
        }
    }
    static __device__ __forceinline__ void fill(char *buf, const bf16_t *in, int ld, int grow0, int row_end,
                                                int gcol0, int n_dim, int lane)
    {
        uint4 v[PASSES];
#pragma unroll
        for (int p = 0; p < PASSES; ++p) {
            const int r = p * ROWS_PER_PASS + lane / PIECES, piece = lane % PIECES;
            const int gr = min(grow0 + r, row_end - 1), gc = min(gcol0 + piece * 8, n_dim - 8);
            v[p] = *reinterpret_cast<const uint4 *>(in + (size_t)gr * ld + gc);
        }
#pragma unroll
        for (int p = 0; p < PASSES; ++p) {
            const int r = p * ROWS_PER_PASS + lane / PIECES, piece = lane % PIECES;
            *reinterpret_cast<uint4 *>(buf + r * (NCOLS * 2) + (((piece ^ r) & (PIECES - 1)) << 4)) = v[p];
        }
    }
};

// LDS operations of one wave execute in order; this keeps the compiler from moving them across
// the hand-over between the two layouts and waits for the data.
__device__ __forceinline__ void wave_lds_fence()
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_s_waitcnt(0xC07F);          // lgkmcnt(0)
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

// The k-loops issue a slab's loads one by one between the MFMAs of a slab period instead of in one
// burst behind the barrier (gemm_tile.h); needs a ring of at least three slabs to pay.
constexpr bool kSpreadLoads = true;

// Wave layouts: every wave owns 64 rows; the waves left over split the columns.
template <int BB, int NWV = NWAVES> struct Waves { static constexpr int B = BB / 64, A = NWV / B; };

// ---------------------------------------------------------------- forward
// Gt = X Wg^T, U = X Wu^T (one pass over X), A = silu(Gt) * U.   Column tile: 128 of h'.
template <int BB, bool WT, int AW = 128>
__device__ __forceinline__ void fwd_gate_up_body(const RowTile &t, const bf16_t *X, const int32_t *row_tok, int tok_last,
                                                 const bf16_t *Wg, const bf16_t *Wu,
                                                 int h, int hff, bf16_t *Gt, bf16_t *U, bf16_t *Aout,
                                                 const float *row_gate, bf16_t *Agout, char *lds)
{
    constexpr int NWV = AW == 128 ? NWAVES : kWideRowWaves;
    using WV = Waves<BB, NWV>;
    using WTile = typename std::conditional<WT, KsTile<AW>, KcTile<AW>>::type;
    using KL = KLoop<WTile, KcTile<BB, (AW == 128 ? BK : kRowDepthWide)>, 2, 1, AW, BB, WV::A, WV::B, 1, false, NSTAGES, kSpreadLoads>;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const size_t wofs = (size_t)t.expert * hff * h;
    const int ldw = WT ? hff : h;                             // (n in h', k in h) at [n*h + k], or at [k*h' + n]
    const Operand A[1][2] = {{{Wg + wofs, ldw, t.col0, hff - 1}, {Wu + wofs, ldw, t.col0, hff - 1}}};
    // rows of the group: a gathered copy (row_tok == nullptr), or token rows fetched through row_tok
    const Operand B[1][1] = {{{X, h, t.row0, t.row0 + t.rows - 1, row_tok, tok_last}}};
    typename KL::Acc acc;
    KL::zero(acc);
    KL::run(acc, A, B, h / BK, h, lds, tid);
    // epilogue: three tensors, one after the other through this wave's staging area
    constexpr int WCOLS = AW / WV::A;                         // columns of this wave per tensor
    using ST = WaveStage<WCOLS>;
    static_assert(KL::TB == 2, "a wave owns 64 rows");
    __syncthreads();                                          // every wave is done with the operand slabs
    char *buf = lds + wave * ST::BYTES;
    const int wrow0 = t.row0 + (wave % WV::B) * 64, row_end = t.row0 + t.rows;
    const int wcol0 = t.col0 + (wave / WV::B) * WCOLS;
    // With row gates: the activations scaled by the gate of the row's assignment, as a fourth tensor
    // (Agout) or, with Agout == Aout, in place of the plain ones (the down projection then yields
    // gated rows and the combine is a plain sum).
    const bool gated = row_gate != nullptr, in_place = gated && Agout == Aout;
    float gate[KL::TB];
#pragma unroll
    for (int tb = 0; tb < KL::TB; ++tb) gate[tb] = gated ? row_gate[min(wrow0 + tb * 32 + (lane & 31), row_end - 1)] : 0.0f;
#pragma unroll
    for (int which = 0; which < 4; ++which) {
        if (which == 3 && !gated) break;
        if (which == 2 && in_place) continue;                 // the fourth pass writes A's place
#pragma unroll
        for (int tb = 0; tb < KL::TB; ++tb)
#pragma unroll
            for (int ta = 0; ta < KL::TA; ++ta)
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    float v[4];
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        const float g = acc[0][ta][tb][q * 4 + e], u = acc[1][ta][tb][q * 4 + e];
                        v[e] = which == 0 ? g : which == 1 ? u : which == 2 ? g * sigmoidf_(g) * u : gate[tb] * (g * sigmoidf_(g) * u);
                    }
                    ST::put(buf, tb * 32 + (lane & 31), ta * 32 + q * 8 + (lane >> 5) * 4, pack4bf(v[0], v[1], v[2], v[3]));
                }
        wave_lds_fence();
        ST::flush(buf, which == 0 ? Gt : which == 1 ? U : which == 2 ? Aout : Agout, hff, wrow0, row_end, wcol0, hff, lane);
        wave_lds_fence();
    }
}

// WT: Wg, Wu given as transposed copies [h][h'] (contraction index strided, transposing LDS reads).
template <bool WT, int AW = 128>
__global__ void __launch_bounds__(AW == 128 ? THREADS : kWideRowWaves * 64, AW == 128 ? 2 : 1)
fwd_gate_up_kernel(Sched s, const bf16_t *__restrict__ X, const int32_t *__restrict__ row_tok, int tok_last,
                   const bf16_t *__restrict__ Wg, const bf16_t *__restrict__ Wu, int h, int hff, int n_col_tiles,
                   bf16_t *__restrict__ Gt, bf16_t *__restrict__ U, bf16_t *__restrict__ Aout,
                   const float *__restrict__ row_gate, bf16_t *__restrict__ Agout)
{
    extern __shared__ __attribute__((aligned(1024))) char lds[];
    const RowTile t = find_row_tile(s, n_col_tiles, AW);
    if (!t.valid) return;
    if (t.rows > BM / 2) fwd_gate_up_body<BM, WT, AW>(t, X, row_tok, tok_last, Wg, Wu, h, hff, Gt, U, Aout, row_gate, Agout, lds);
    else fwd_gate_up_body<BM / 2, WT, AW>(t, X, row_tok, tok_last, Wg, Wu, h, hff, Gt, U, Aout, row_gate, Agout, lds);
}

// Gate-side fusion of the activation backward (EPI = 2).  With the upstream gradient of row r
// taken straight from the token tensor, dY'[r] = dOut[tok(r)] (the combine's gate left out), the
// accumulators hold dA' = dY' Wd, and
//   dGt = gate * dA' * U * silu'(Gt),  dU = gate * dA' * silu(Gt),  dgate[r] = sum_n dA'[r][n] * A[r][n]
// with A = silu(Gt) * U recomputed in place: the same values as scaling dOut by the gate first
// and reducing dOut against the down projection's output, without either pass over the rows.
struct GateFusion {
    const int32_t *row_tok = nullptr;   // [n_rows] row -> token (null: P0 holds group-ordered rows)
    int tok_last = 0;
    const float *row_gate = nullptr;    // [n_rows]
    float *dgate_part = nullptr;        // [kDgateParts * column tiles][n_rows] partial row sums, summed later in slot order
    int n_rows = 0;
};

// Shared body of the three single-accumulator row-tiled GEMMs.  EPI: 0 = store bf16 (Y, dX);
// 1 = dA -> dGt, dU (needs Gt, U); 2 = the same with the gate fused in (GateFusion).
// W_KS: weights k-strided (data gradients).  NPH = 2 sums two products (dX = dGt Wg + dU Wu).
template <int BB, bool W_KS, int NPH, int EPI, int AW = 256>
__device__ __forceinline__ void row_gemm_body(const RowTile &t, const bf16_t *P0, const bf16_t *P1, int ldp,
                                              const bf16_t *W0, const bf16_t *W1, int ldw, int n_dim, int k_dim,
                                              bf16_t *out0, bf16_t *out1, const bf16_t *Gt, const bf16_t *U, char *lds,
                                              const GateFusion &gf = GateFusion{})
{
    constexpr int NWV = AW == 256 ? NWAVES : kWideRowWaves;
    using WV = Waves<BB, NWV>;
    using WT = typename std::conditional<W_KS, KsTile<AW>, KcTile<AW>>::type;
    using KL = KLoop<WT, KcTile<BB, (AW == 256 ? BK : kRowDepthWide)>, 1, 1, AW, BB, WV::A, WV::B, NPH, false, NSTAGES, kSpreadLoads>;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    Operand A[NPH][1], B[NPH][1];
    A[0][0] = {W0, ldw, t.col0, n_dim - 1};
    B[0][0] = {P0, ldp, t.row0, t.row0 + t.rows - 1};
    if (EPI == 2 && gf.row_tok) B[0][0] = {P0, ldp, t.row0, t.row0 + t.rows - 1, gf.row_tok, gf.tok_last};
    if (NPH == 2) {
        A[NPH - 1][0] = {W1, ldw, t.col0, n_dim - 1};
        B[NPH - 1][0] = {P1, ldp, t.row0, t.row0 + t.rows - 1};
    }
    typename KL::Acc acc;
    KL::zero(acc);
    KL::run(acc, A, B, k_dim / BK, k_dim, lds, tid);
    constexpr int WCOLS = AW / WV::A;
    using ST = WaveStage<WCOLS>;
    static_assert(KL::TB == 2, "a wave owns 64 rows");
    __syncthreads();                                          // every wave is done with the operand slabs
    char *buf = lds + wave * ST::BYTES;
    const int wrow0 = t.row0 + (wave % WV::B) * 64, row_end = t.row0 + t.rows;
    const int wcol0 = t.col0 + (wave / WV::B) * WCOLS;
    if (EPI == 0) {
#pragma unroll
        for (int tb = 0; tb < KL::TB; ++tb)
#pragma unroll
            for (int ta = 0; ta < KL::TA; ++ta)
#pragma unroll
                for (int q = 0; q < 4; ++q)
                    ST::put(buf, tb * 32 + (lane & 31), ta * 32 + q * 8 + (lane >> 5) * 4,
                            pack4bf(acc[0][ta][tb][q * 4], acc[0][ta][tb][q * 4 + 1], acc[0][ta][tb][q * 4 + 2],
                                    acc[0][ta][tb][q * 4 + 3]));
        wave_lds_fence();
        ST::flush(buf, out0, n_dim, wrow0, row_end, wcol0, n_dim, lane);
    } else {
        // dA (in the accumulators) -> dGt, dU, half of the wave's columns at a time: Gt and U come
        // in through two staging areas and are overwritten in place by dGt and dU.
        using SH = WaveStage<WCOLS / 2>;
        constexpr int TAH = KL::TA / 2;
        static_assert(TAH >= 1, "at least 64 columns per wave");
        char *buf_g = buf, *buf_u = buf + SH::BYTES;
        float gate[KL::TB], dsum[KL::TB];
#pragma unroll
        for (int tb = 0; tb < KL::TB; ++tb) {
            gate[tb] = EPI == 2 ? gf.row_gate[min(wrow0 + tb * 32 + (lane & 31), row_end - 1)] : 1.0f;
            dsum[tb] = 0.0f;
        }
#pragma unroll
        for (int half = 0; half < 2; ++half) {
            const int hcol0 = wcol0 + half * (WCOLS / 2);
            SH::fill2(buf_g, buf_u, Gt, U, n_dim, wrow0, row_end, hcol0, n_dim, lane);
            wave_lds_fence();
            // this half's share of the row sums; a half (32 or 64 columns, n_dim % 64 == 0) lies inside
            // the tensor or outside it as a whole, and outside it holds clamped copies
            float hsum[KL::TB];
#pragma unroll
            for (int tb = 0; tb < KL::TB; ++tb) hsum[tb] = 0.0f;
#pragma unroll
            for (int tb = 0; tb < KL::TB; ++tb)
#pragma unroll
                for (int th = 0; th < TAH; ++th)
#pragma unroll
                    for (int q = 0; q < 4; ++q) {
                        const int ta = half * TAH + th;
                        const int row = tb * 32 + (lane & 31), col = th * 32 + q * 8 + (lane >> 5) * 4;
                        float g[4], u[4], dg[4], du[4], pa[4];
                        unpack4bf(SH::get(buf_g, row, col), g);
                        unpack4bf(SH::get(buf_u, row, col), u);
#pragma unroll
                        for (int e = 0; e < 4; ++e) {
                            const float da = acc[0][ta][tb][q * 4 + e];
                            const float sg = sigmoidf_(g[e]);
                            if (EPI == 2) {
                                pa[e] = da * (g[e] * sg * u[e]);
                                const float dag = gate[tb] * da;
                                dg[e] = dag * u[e] * (sg * (1.0f + g[e] * (1.0f - sg)));
                                du[e] = dag * (g[e] * sg);
                            } else {
                                dg[e] = da * u[e] * (sg * (1.0f + g[e] * (1.0f - sg)));
                                du[e] = da * (g[e] * sg);
                            }
                        }
                        SH::put(buf_g, row, col, pack4bf(dg[0], dg[1], dg[2], dg[3]));
                        SH::put(buf_u, row, col, pack4bf(du[0], du[1], du[2], du[3]));
                        // The running sum is needed only after the loop, and the compiler would sink all
                        // of its arithmetic down there, parking every operand in scratch memory on the
                        // way; an assembly statement that "uses" the sum keeps each add where it is.
                        if (EPI == 2) {
                            hsum[tb] += (pa[0] + pa[1]) + (pa[2] + pa[3]);
                            asm volatile("" : "+v"(hsum[tb]));
                        }
                    }
            wave_lds_fence();
            SH::flush(buf_g, out0, n_dim, wrow0, row_end, hcol0, n_dim, lane);
            SH::flush(buf_u, out1, n_dim, wrow0, row_end, hcol0, n_dim, lane);
            wave_lds_fence();
            if (EPI == 2 && hcol0 < n_dim) {
#pragma unroll
                for (int tb = 0; tb < KL::TB; ++tb) dsum[tb] += hsum[tb];
            }
        }
        if (EPI == 2) {
            // a row's columns lie on lanes l and l + 32; one partial sum per row and wave column, in the
            // slot of its 256 columns (kDgateParts slots each; a wave column is 64 or 128 wide)
            constexpr int PER = 256 / WCOLS;
            static_assert(PER >= 1 && PER <= kDgateParts, "wave columns per 256 columns");
            const int slot = (wcol0 / 256) * kDgateParts + (wcol0 % 256) / WCOLS;
#pragma unroll
            for (int tb = 0; tb < KL::TB; ++tb) {
                const float total = dsum[tb] + __shfl_xor(dsum[tb], 32);
                const int r = wrow0 + tb * 32 + (lane & 31);
                if (lane < 32 && r < row_end) {
                    gf.dgate_part[(size_t)slot * gf.n_rows + r] = total;
#pragma unroll
                    for (int extra = PER; extra < kDgateParts; extra += PER)      // the slots this tile shape does not fill
                        gf.dgate_part[(size_t)(slot + extra) * gf.n_rows + r] = 0.0f;
                }
            }
        }
    }
}

// Y = A Wd^T.  WT: Wd given as a transposed copy [h'][h].
template <bool WT, int AW = 256>
__global__ void __launch_bounds__(AW == 256 ? THREADS : kWideRowWaves * 64, AW == 256 ? 2 : 1)
fwd_down_kernel(Sched s, const bf16_t *__restrict__ Ain, const bf16_t *__restrict__ Wd, int h, int hff,
                int n_col_tiles, bf16_t *__restrict__ Y)
{
    extern __shared__ __attribute__((aligned(1024))) char lds[];
    const RowTile t = find_row_tile(s, n_col_tiles, AW);
    if (!t.valid) return;
    const bf16_t *W = Wd + (size_t)t.expert * h * hff;
    const int ldw = WT ? h : hff;                             // (n in h, k in h') at [n*h' + k], or at [k*h + n]
    if (t.rows > BM / 2) row_gemm_body<BM, WT, 1, 0, AW>(t, Ain, nullptr, hff, W, nullptr, ldw, h, hff, Y, nullptr, nullptr, nullptr, lds);
    else row_gemm_body<BM / 2, WT, 1, 0, AW>(t, Ain, nullptr, hff, W, nullptr, ldw, h, hff, Y, nullptr, nullptr, nullptr, lds);
}

// ---------------------------------------------------------------- backward
// dA = dY Wd, then dGt = dA * U * silu'(Gt), dU = dA * silu(Gt).
// WT = false: Wd as the forward pass holds it, [h][h'], contraction index strided (transposing
// LDS reads, full-line loads: the faster operand path).  WT = true: a transposed copy [h'][h],
// contraction index contiguous.
template <bool WT, bool GATED = false, int AW = 256>
__global__ void __launch_bounds__(AW == 256 ? THREADS : kWideRowWaves * 64, AW == 256 ? 2 : 1)
bwd_act_kernel(Sched s, const bf16_t *__restrict__ dY, const bf16_t *__restrict__ Wd,
               const bf16_t *__restrict__ Gt, const bf16_t *__restrict__ U, int h, int hff, int n_col_tiles,
               int w_from_slot, GateFusion gf)
{
    extern __shared__ __attribute__((aligned(1024))) char lds[];
    const RowTile t = find_row_tile(s, n_col_tiles, AW, w_from_slot != 0);
    if (!t.valid) return;
    const bf16_t *W = Wd + (size_t)t.expert * h * hff;      // (n in h', k in h) at [k*h' + n], or at [n*h + k]
    const int ldw = WT ? h : hff;
    constexpr int EPI = GATED ? 2 : 1;
    if (t.rows > BM / 2) row_gemm_body<BM, !WT, 1, EPI, AW>(t, dY, nullptr, h, W, nullptr, ldw, hff, h, s.dGt, s.dU, Gt, U, lds, gf);
    else row_gemm_body<BM / 2, !WT, 1, EPI, AW>(t, dY, nullptr, h, W, nullptr, ldw, hff, h, s.dGt, s.dU, Gt, U, lds, gf);
}

// dgate of the gate-fused backward: the partial row sums of the activation backward added up in
// slot order (fixed order: bit-reproducible), written per row or, with src_of, at the assignment
// the row serves (the [T,k] layout of the gates).  Rows outside [group_offset[g_begin],
// group_offset[g_end]) were not computed and are left alone.
__global__ void __launch_bounds__(256)
dgate_reduce_kernel(const float *__restrict__ part, int n_slots, int n_rows, const int32_t *__restrict__ group_offset,
                    int g_begin, int g_end, const int32_t *__restrict__ src_of, float *__restrict__ dgate,
                    int32_t *__restrict__ err_flag)
{
    const int lo = max(0, min(group_offset[g_begin], n_rows)), hi = max(lo, min(group_offset[g_end], n_rows));
    bool bad = false;
    for (int r = lo + blockIdx.x * 256 + threadIdx.x; r < hi; r += gridDim.x * 256) {
        float sum = 0.0f;
        for (int p = 0; p < n_slots; ++p) sum += part[(size_t)p * n_rows + r];
        int at = r;
        if (src_of) {
            at = src_of[r];
            if (at < 0 || at >= n_rows) { bad = true; continue; }
        }
        dgate[at] = sum;
    }
    if (bad) atomicOr(err_flag, RELIBRA_ERR_PLAN_COVER);
}

// dX = dGt Wg + dU Wu (one accumulator, the contraction runs over both products).
// WT as above: Wg, Wu [h'][h] as the forward pass holds them, or transposed copies [h][h'].
template <bool WT, int AW = 256>
__global__ void __launch_bounds__(AW == 256 ? THREADS : kWideRowWaves * 64, AW == 256 ? 2 : 1)
bwd_dx_kernel(Sched s, const bf16_t *__restrict__ Wg, const bf16_t *__restrict__ Wu, int h, int hff,
              int n_col_tiles, int w_from_slot, bf16_t *__restrict__ dX)
{
    extern __shared__ __attribute__((aligned(1024))) char lds[];
    const RowTile t = find_row_tile(s, n_col_tiles, AW, w_from_slot != 0);
    if (!t.valid) return;
    const size_t wofs = (size_t)t.expert * hff * h;         // (n in h, k in h') at [k*h + n], or at [n*h' + k]
    const int ldw = WT ? hff : h;
    if (t.rows > BM / 2) row_gemm_body<BM, !WT, 2, 0, AW>(t, s.dGt, s.dU, hff, Wg + wofs, Wu + wofs, ldw, h, hff, dX, nullptr, nullptr, nullptr, lds);
    else row_gemm_body<BM / 2, !WT, 2, 0, AW>(t, s.dGt, s.dU, hff, Wg + wofs, Wu + wofs, ldw, h, hff, dX, nullptr, nullptr, nullptr, lds);
}

// Transposed copy of per-expert matrices, out[e][j][i] = in[e][i][j]: 64 x 64 tiles through LDS,
// 16-byte accesses on both sides.
__global__ void __launch_bounds__(256)
transpose_experts_kernel(const bf16_t *__restrict__ in, int rows, int cols, bf16_t *__restrict__ out)
{
    __shared__ bf16_t tile[64][64 + 8];
    const size_t base = (size_t)blockIdx.z * rows * cols;
    const int r0 = blockIdx.y * 64, c0 = blockIdx.x * 64, tid = threadIdx.x;
#pragma unroll
    for (int i = 0; i < 2; ++i) {
        const int r = (tid >> 3) + i * 32, c = (tid & 7) * 8;
        uint4 v = make_uint4(0, 0, 0, 0);
        if (r0 + r < rows && c0 + c < cols) v = *reinterpret_cast<const uint4 *>(in + base + (size_t)(r0 + r) * cols + c0 + c);
        *reinterpret_cast<uint4 *>(&tile[r][c]) = v;
    }
    __syncthreads();
#pragma unroll
    for (int i = 0; i < 2; ++i) {
        const int c = (tid >> 3) + i * 32, r = (tid & 7) * 8;        // output row c0 + c, output columns r0 + r ..
        if (c0 + c < cols && r0 + r < rows) {
            uint32_t w[4];
#pragma unroll
            for (int j = 0; j < 4; ++j) w[j] = (uint32_t)tile[r + 2 * j][c] | ((uint32_t)tile[r + 2 * j + 1][c] << 16);
            *reinterpret_cast<uint4 *>(out + base + (size_t)(c0 + c) * rows + r0 + r) = make_uint4(w[0], w[1], w[2], w[3]);
        }
    }
}

// Weight-gradient epilogue.  The accumulators hold, per lane, one column n and 16 rows m of each
// MFMA tile; each 32 x 64 fp32 block of the wave goes through this wave's 8 KiB of LDS and
// leaves as 16 bytes per lane along n: 1 KiB per store (or load-add-store) instruction.
template <class KL, int NA, int BA, int NWV = NWAVES>
__device__ __forceinline__ void wgrad_epilogue(typename KL::Acc &acc, char *lds, float *out0, float *out1, size_t base,
                                               int m0, int n0, int m_dim, int n_dim, bool add, int wave, int lane)
{
    static_assert(KL::TB % 2 == 0, "a wave owns a multiple of 64 columns");
    __syncthreads();                                          // every wave is done with the operand slabs
    float *buf = reinterpret_cast<float *>(lds + wave * 8192);
    const int wm0 = m0 + (wave / (NWV / 2)) * (BA / 2);
    const int col4 = lane & 15;
#pragma unroll
    for (int half = 0; half < KL::TB / 2; ++half)             // 64 columns of the wave at a time
#pragma unroll
    for (int a = 0; a < NA; ++a)
#pragma unroll
        for (int ta = 0; ta < KL::TA; ++ta) {
            const int wn0 = n0 + (wave % (NWV / 2)) * (KL::TB * 32) + half * 64, gcol = wn0 + col4 * 4;
#pragma unroll
            for (int tb = 0; tb < 2; ++tb)
#pragma unroll
                for (int v = 0; v < 16; ++v)
                    buf[(8 * (v >> 2) + 4 * (lane >> 5) + (v & 3)) * 64 + tb * 32 + (lane & 31)] = acc[a][ta][half * 2 + tb][v];
            wave_lds_fence();
            float *out = (a == 0 ? out0 : out1) + base;
            float4 val[8];
#pragma unroll
            for (int p = 0; p < 8; ++p) val[p] = *reinterpret_cast<const float4 *>(buf + (p * 4 + (lane >> 4)) * 64 + col4 * 4);
            if (add) {
                float4 old[8];
#pragma unroll
                for (int p = 0; p < 8; ++p) {
                    const int r = wm0 + ta * 32 + p * 4 + (lane >> 4);
                    old[p] = make_float4(0.f, 0.f, 0.f, 0.f);
                    if (r < m_dim && gcol < n_dim) old[p] = *reinterpret_cast<const float4 *>(out + (size_t)r * n_dim + gcol);
                }
#pragma unroll
                for (int p = 0; p < 8; ++p) {
                    val[p].x += old[p].x; val[p].y += old[p].y; val[p].z += old[p].z; val[p].w += old[p].w;
                }
            }
#pragma unroll
            for (int p = 0; p < 8; ++p) {
                const int r = wm0 + ta * 32 + p * 4 + (lane >> 4);
                if (r < m_dim && gcol < n_dim) *reinterpret_cast<float4 *>(out + (size_t)r * n_dim + gcol) = val[p];
            }
            wave_lds_fence();
        }
}

// Weight gradients: out[slot][m][n] (+)= sum over the group's rows of L[row][m] * R[row][n].
// NA = 2 computes two left operands against one right operand (dGt and dU against X).
// Tile: (NA x BA) x WGN with BA = WGM / NA.  Two geometries: WGM = 256 (three slabs, two
// workgroups per compute unit) for long groups, where the MFMA rate matters, and WGM = 128 (two
// slabs, four workgroups per compute unit) for short groups, where the kernel is a stream of
// fp32 read-add-writes and more waves in flight mean more HBM bandwidth.
template <int WGM> struct WgradCfg {
    static constexpr int STAGES = WGM == 256 ? NSTAGES : 2;
    static constexpr int OCC = WGM == 256 ? 2 : 4;                  // waves per SIMD aimed at
    static constexpr int SLABS = STAGES * (WGM + WGN) * BK * 2;
    static constexpr int LDS = SLABS > NWAVES * 8192 ? SLABS : NWAVES * 8192;
};
template <int NA, int WGM>
__global__ void __launch_bounds__(THREADS, WgradCfg<WGM>::OCC)
wgrad_kernel(Sched s, const bf16_t *__restrict__ L0, const bf16_t *__restrict__ L1,
             const bf16_t *__restrict__ R, int m_dim, int n_dim, int E, int accumulate, int total,
             float *__restrict__ out0, float *__restrict__ out1)
{
    constexpr int BA = WGM / NA;
    using KL = KLoop<KsTile<BA>, KsTile<WGN>, NA, 1, BA, WGN, 2, NWAVES / 2, 1, true, WgradCfg<WGM>::STAGES, (kSpreadLoads && WgradCfg<WGM>::STAGES >= 3)>;
    extern __shared__ __attribute__((aligned(1024))) char lds[];
    const int n_nt = (n_dim + WGN - 1) / WGN, n_mt = (m_dim + BA - 1) / BA;
    const int per_group = n_nt * n_mt;
    const int per_xcd = (total + 7) >> 3;
    const int logical = (blockIdx.x & 7) * per_xcd + (blockIdx.x >> 3);
    if (logical >= total) return;
    const int gi = logical / per_group, rem = logical % per_group;
    const int e = s.grp_expert[gi];
    if (e < 0) return;
    const int slot = s.grp_slot[gi];
    const bool add = accumulate && slot < E;
    const int row0 = s.grp_row0[gi], rows = s.grp_rows[gi];
    if (rows == 0 && add) return;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    int mt, nt;
    band_order(rem, n_mt, n_nt, mt, nt);
    const int m0 = mt * BA, n0 = nt * WGN;
    Operand A[1][NA], B[1][1];
    A[0][0] = {L0 + (size_t)row0 * m_dim, m_dim, m0, m_dim - 1};
    if (NA == 2) A[0][NA - 1] = {L1 + (size_t)row0 * m_dim, m_dim, m0, m_dim - 1};
    B[0][0] = {R + (size_t)row0 * n_dim, n_dim, n0, n_dim - 1};
    typename KL::Acc acc;
    KL::zero(acc);
    KL::run(acc, A, B, (rows + BK - 1) / BK, rows, lds, tid);
    wgrad_epilogue<KL, NA, BA>(acc, lds, out0, out1, (size_t)slot * m_dim * n_dim, m0, n0, m_dim, n_dim, add, wave, lane);
}

// ---------------------------------------------------------------- batched weight gradients
// One pass over every micro-batch of a training batch: the tile of expert e contracts over all
// rows e received, instance by instance, micro-batch by micro-batch, in registers, and writes
// dW once.  Per-micro-batch device pointers travel as a kernel argument of the ordering kernel,
// which turns them into one record per piece for the GEMM kernels.
constexpr int kMaxWgradMb = RELIBRA_MAX_WGRAD_MB;
constexpr int kWgradChunk = 64;
struct MbTable {
    const bf16_t *dY[kMaxWgradMb], *X[kMaxWgradMb], *A[kMaxWgradMb], *dGt[kMaxWgradMb], *dU[kMaxWgradMb];
    const int32_t *iptr[kMaxWgradMb], *igrp[kMaxWgradMb], *goff[kMaxWgradMb];
    const int32_t *rtok[kMaxWgradMb];      // null: X holds group-ordered rows; else X holds tokens and row r is X[rtok[r]]
    int tok_last[kMaxWgradMb];
    unsigned long long dy_tokens;          // bit mb set: dY[mb] is the token tensor dOut and row r is dOut[rtok[r]]
};

// Instance range of expert e in micro-batch mb, sanitised: [p0, p1) inside the instance table.
__device__ __forceinline__ bool inst_range(const MbTable &tb, int mb, int e, int inst_cap, int &p0, int &p1)
{
    p0 = tb.iptr[mb][e];
    p1 = tb.iptr[mb][e + 1];
    if (p0 < 0 || p1 < p0 || p1 > inst_cap) { p0 = p1 = 0; return false; }
    return true;
}
// Row range of instance p of micro-batch mb, sanitised: rows = 0 when a table entry is bad.
__device__ __forceinline__ bool inst_rows(const MbTable &tb, int mb, int p, int G, int n_rows, int &row0, int &rows)
{
    row0 = rows = 0;
    const int g = tb.igrp[mb][p];
    if (g < 0 || g >= G) return false;
    const int lo = tb.goff[mb][g], hi = tb.goff[mb][g + 1];
    if (lo < 0 || hi < lo || hi > n_rows) return false;
    row0 = lo;
    rows = hi - lo;
    return true;
}

// Workspace of the batched weight gradients.
struct WgradPlan {
    int32_t *exp_rows;     // [E] rows of the expert over the whole batch
    int32_t *exp_slabs;    // [E] k-loop slabs: sum over its pieces of ceil(rows / BK)
    int32_t *exp_order;    // [E] experts in descending order of rows (ties: lower id)
    int32_t *piece_ptr;    // [E+1] CSR over experts into the piece arrays
    int32_t *piece_mb, *piece_row0, *piece_rows;   // [S] micro-batch, first row, rows (> 0) of a piece
    // [S] what a tile's k-loop needs of a piece, as one record each (one wide scalar load per switch
    // of piece instead of a chain of single ones): operand addresses at the piece's first row, the
    // row table (0: none), rows, last token.  64-byte aligned.
    int32_t *rec_down, *rec_gu;
};
constexpr int kRecDownInts = 8, kRecGuInts = 16;
struct PieceRecDown { unsigned long long L, R, gather; int32_t rows, tok_last; };
struct PieceRecGu { unsigned long long L0, L1, R, gather; int32_t rows, tok_last; int32_t pad[6]; };
static_assert(sizeof(PieceRecDown) == kRecDownInts * 4 && sizeof(PieceRecGu) == kRecGuInts * 4, "record sizes");
inline size_t wgrad_plan_ints(int E, int G)
{
    const size_t S = (size_t)kMaxWgradMb * ((size_t)E + G);
    return 4 * (size_t)E + 1 + 3 * S + 16 + (kRecDownInts + kRecGuInts) * S;
}
inline WgradPlan carve_wgrad(void *ws, int E, int G)
{
    WgradPlan w;
    int32_t *p = (int32_t *)ws;
    const size_t S = (size_t)kMaxWgradMb * ((size_t)E + G);
    w.exp_rows = p; p += E;
    w.exp_slabs = p; p += E;
    w.exp_order = p; p += E;
    w.piece_ptr = p; p += E + 1;
    w.piece_mb = p; p += S;
    w.piece_row0 = p; p += S;
    w.piece_rows = p; p += S;
    p += (16 - ((p - (int32_t *)ws) & 15)) & 15;             // records: 64-byte aligned (the workspace is 256-byte aligned)
    w.rec_down = p; p += kRecDownInts * S;
    w.rec_gu = p;
    return w;
}

// One block.  Lists, per expert, the pieces of its contraction: every instance with rows, micro-
// batch by micro-batch in the order of the plan's instance table (entries out of range are left
// out and flagged), and ranks the experts by rows so that the tiles run heaviest first.
__global__ void __launch_bounds__(256)
wgrad_order_kernel(MbTable tb, int n_mb, int G, int inst_cap, int n_rows, int E, int h, int hff, WgradPlan w, int32_t *err_flag)
{
    extern __shared__ int32_t rows_of[];       // [E]
    __shared__ int32_t scan[256];
    __shared__ int32_t carry;
    const int tid = threadIdx.x;
    bool bad = false;
    if (tid == 0) { carry = 0; w.piece_ptr[0] = 0; }
    __syncthreads();
    // The piece arrays hold S entries: enough for every instance of every micro-batch of a well-formed
    // (monotone) instance table.  A corrupted table whose ranges overlap could list more; pieces
    // beyond S are left out (and flagged), so that nothing is written past the arrays.
    const int S = kMaxWgradMb * (E + G);
    for (int base = 0; base < E; base += 256) {
        const int e = base + tid;
        int pieces = 0;
        if (e < E) {
            for (int mb = 0; mb < n_mb; ++mb) {
                int p0, p1;
                if (!inst_range(tb, mb, e, inst_cap, p0, p1)) bad = true;
                for (int p = p0; p < p1; ++p) {
                    int row0, rows;
                    if (!inst_rows(tb, mb, p, G, n_rows, row0, rows)) bad = true;
                    if (rows > 0) ++pieces;
                }
            }
        }
        pieces = min(pieces, S + 1);                 // saturate: the sums below stay inside an int
        scan[tid] = pieces;
        __syncthreads();
        for (int off = 1; off < 256; off <<= 1) {
            const int v = tid >= off ? scan[tid - off] : 0;
            __syncthreads();
            scan[tid] += v;
            __syncthreads();
        }
        if (e < E) {
            int at = min(carry + scan[tid] - pieces, S);
            const int end = min(carry + scan[tid], S);
            if (carry + scan[tid] > S) bad = true;
            w.piece_ptr[e + 1] = end;
            long long total = 0, slabs = 0;
            for (int mb = 0; mb < n_mb && at < end; ++mb) {
                int p0, p1;
                inst_range(tb, mb, e, inst_cap, p0, p1);
                for (int p = p0; p < p1 && at < end; ++p) {
                    int row0, rows;
                    inst_rows(tb, mb, p, G, n_rows, row0, rows);
                    if (rows > 0) {
                        total += rows;
                        slabs += (rows + BK - 1) / BK;
                        w.piece_mb[at] = mb; w.piece_row0[at] = row0; w.piece_rows[at] = rows;
                        const bool dy_tok = (tb.dy_tokens >> mb) & 1, x_tok = tb.rtok[mb] != nullptr;
                        const unsigned long long table = (unsigned long long)(uintptr_t)(tb.rtok[mb] + row0);
                        PieceRecDown d;     // dWd: L = dY rows (or dOut tokens through the table), R = A rows
                        d.L = (unsigned long long)(uintptr_t)(dy_tok ? tb.dY[mb] : tb.dY[mb] + (size_t)row0 * h);
                        d.R = (unsigned long long)(uintptr_t)(tb.A[mb] + (size_t)row0 * hff);
                        d.gather = dy_tok ? table : 0ull;
                        d.rows = rows;
                        d.tok_last = tb.tok_last[mb];
                        ((PieceRecDown *)w.rec_down)[at] = d;
                        PieceRecGu u;       // dWg, dWu: L = dGt, dU rows; R = X rows (or tokens through the table)
                        u.L0 = (unsigned long long)(uintptr_t)(tb.dGt[mb] + (size_t)row0 * hff);
                        u.L1 = (unsigned long long)(uintptr_t)(tb.dU[mb] + (size_t)row0 * hff);
                        u.R = (unsigned long long)(uintptr_t)(x_tok ? tb.X[mb] : tb.X[mb] + (size_t)row0 * h);
                        u.gather = x_tok ? table : 0ull;
                        u.rows = rows;
                        u.tok_last = tb.tok_last[mb];
                        for (int z = 0; z < 6; ++z) u.pad[z] = 0;
                        ((PieceRecGu *)w.rec_gu)[at] = u;
                        ++at;
                    }
                }
            }
            rows_of[e] = (int32_t)(total > 0x7fffffffLL ? 0x7fffffffLL : total);
            w.exp_rows[e] = rows_of[e];
            w.exp_slabs[e] = (int32_t)(slabs > 0x7fffffffLL ? 0x7fffffffLL : slabs);
        }
        __syncthreads();
        if (tid == 255) carry = min(carry + scan[255], S + 1);
        __syncthreads();
    }
    if (bad) atomicOr(err_flag, RELIBRA_ERR_GROUP_TABLE);
    __syncthreads();
    for (int e = tid; e < E; e += 256) {
        const int mine = rows_of[e];
        int rank = 0;
        for (int o = 0; o < E; ++o) rank += (rows_of[o] > mine || (rows_of[o] == mine && o < e)) ? 1 : 0;
        w.exp_order[rank] = e;
    }
}

// The pieces of one expert's contraction as the k-loop sees them: one record per piece, written
// by the ordering kernel (an earlier launch, the same for every lane: read as scalars).
template <int NA>
struct WgradPieces {
    const_i32_ptr rows;                    // this expert's slice of the piece rows
    const_i32_ptr recs;                    // and of the records
    int m_dim, n_dim, m0, n0;
    __device__ __forceinline__ int valid(int i) const { return rows[i]; }
    __device__ __forceinline__ void piece(int i, Operand (&A)[1][NA], Operand (&B)[1][1], int &k_valid) const
    {
        constexpr int RI = NA == 1 ? kRecDownInts : kRecGuInts;
        typedef int32_t rec_vec __attribute__((ext_vector_type(RI)));
        typedef const __attribute__((address_space(4))) rec_vec *rec_ptr;
        const rec_vec r = *(rec_ptr)(recs + (size_t)i * RI);
        auto ptr = [&](int at) { return (const bf16_t *)(uintptr_t)(((unsigned long long)(uint32_t)r[at + 1] << 32) | (uint32_t)r[at]); };
        if (NA == 1) {
            const int32_t *table = (const int32_t *)ptr(4);
            k_valid = r[6];
            A[0][0] = {ptr(0), m_dim, m0, m_dim - 1, table, r[7]};
            B[0][0] = {ptr(2), n_dim, n0, n_dim - 1};
        } else {
            const int32_t *table = (const int32_t *)ptr(6);
            k_valid = r[8];
            A[0][0] = {ptr(0), m_dim, m0, m_dim - 1};
            A[0][NA - 1] = {ptr(2), m_dim, m0, m_dim - 1};
            B[0][0] = {ptr(4), n_dim, n0, n_dim - 1, table, r[9]};
        }
    }
};

// NA = 1: dWd.  NA = 2: dWg, dWu.  WN: columns of a tile.  128: four waves, three slabs, two
// workgroups per compute unit.  256: eight waves of 128 x 64 each, one workgroup per compute unit,
// four slabs: two thirds of the operand bytes (and load instructions) per flop, the same two
// waves per SIMD.  (Four waves of 128 x 128 on that tile, one per SIMD, were 5-10 % slower.)
constexpr int kWideWaves = 8;
template <int WN> struct WgradWide {
    static constexpr int STAGES = WN == 256 ? 4 : WgradCfg<256>::STAGES;
    static constexpr int OCC = WN == 256 ? 1 : WgradCfg<256>::OCC;
    static constexpr int SLABS = STAGES * (256 + WN) * BK * 2;
    static constexpr int LDS = SLABS > 8 * 8192 ? SLABS : 8 * 8192;
};
template <int NA, int WN, int NWV = NWAVES>
__global__ void __launch_bounds__(NWV * 64, WgradWide<WN>::OCC)
wgrad_batched_kernel(int E, int m_dim, int n_dim, WgradPlan w, int accumulate,
                     float *__restrict__ out0, float *__restrict__ out1)
{
    constexpr int WGM = 256, BA = WGM / NA;
    // NA = 1: the A side (dY) may be gathered; its loads go last in the window (see KLoop)
    // the operand that may come through a row table: dY of dWd (A side), X of dWg, dWu (B side)
    using KL = KLoop<KsTile<BA, BK, NA == 1>, KsTile<WN, BK, NA == 2>, NA, 1, BA, WN, 2, NWV / 2, 1, true, WgradWide<WN>::STAGES, kSpreadLoads, NA == 1>;
    extern __shared__ __attribute__((aligned(1024))) char lds[];
    const int n_nt = (n_dim + WN - 1) / WN, n_mt = (m_dim + BA - 1) / BA;
    const int per_expert = n_nt * n_mt;
    // Tile list: experts in descending order of rows, each expert's tiles in band order, cut into
    // chunks of kWgradChunk tiles (an 8 x 8 patch sharing operand tiles).  The chunks are dealt to
    // the XCDs back and forth (0..7, 7..0, ...), so every L2 gets near-equal work, heaviest first.
    const int x = blockIdx.x & 7, t = blockIdx.x >> 3;
    const int q = t / kWgradChunk;
    const long long tile = ((long long)q * 8 + ((q & 1) ? 7 - x : x)) * kWgradChunk + t % kWgradChunk;
    if (tile >= (long long)E * per_expert) return;
    const int e = w.exp_order[tile / per_expert];
    if ((unsigned)e >= (unsigned)E) return;
    const bool add = accumulate != 0;
    if (w.exp_rows[e] == 0 && add) return;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    int mt, nt;
    band_order((int)(tile % per_expert), n_mt, n_nt, mt, nt);
    const int m0 = mt * BA, n0 = nt * WN;
    typename KL::Acc acc;
    KL::zero(acc);
    const int s0 = w.piece_ptr[e];
    const WgradPieces<NA> src{(const_i32_ptr)(uintptr_t)(w.piece_rows + s0),
                              (const_i32_ptr)(uintptr_t)((NA == 1 ? w.rec_down + (size_t)s0 * kRecDownInts : w.rec_gu + (size_t)s0 * kRecGuInts)),
                              m_dim, n_dim, m0, n0};
    KL::run_pieces(acc, src, w.piece_ptr[e + 1] - s0, w.exp_slabs[e], lds, tid);
    wgrad_epilogue<KL, NA, BA, NWV>(acc, lds, out0, out1, (size_t)e * m_dim * n_dim, m0, n0, m_dim, n_dim, add, wave, lane);
}

// Replica gradients return to the home copy (Section 5.1).  A thread owns element positions
// and walks the live replica slots in ascending slot order, so the sum has a fixed order.
// blockIdx.y selects the tensor (all three have h * h' elements per expert).
__global__ void __launch_bounds__(256)
replica_sum_kernel(Sched s, size_t per_expert_vec4, float4 *__restrict__ dWg, float4 *__restrict__ dWu,
                   float4 *__restrict__ dWd)
{
    const int n_pairs = s.hdr[1];
    float4 *__restrict__ dW = blockIdx.y == 0 ? dWg : blockIdx.y == 1 ? dWu : dWd;
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
    if (a.g_end - a.g_begin > kMaxSchedGroups) return RELIBRA_EUNSUPPORTED;   // the schedule kernel keeps a prefix per group in LDS
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
    case RELIBRA_WS_PERMUTE: return round256((size_t)((N + RELIBRA_PERM_UNIT - 1) / RELIBRA_PERM_UNIT + 4) * E * sizeof(int32_t));
    case RELIBRA_WS_FFN_FWD: return ffn_ws_bytes(N, G, hff, false);
    case RELIBRA_WS_FFN_BWD: return ffn_ws_bytes(N, G, hff, true);
    case RELIBRA_WS_WGRAD_BATCHED: return round256(wgrad_plan_ints(E, G) * sizeof(int32_t));
    case RELIBRA_WS_DGATE: return dgate_scratch_bytes(N, hff);
    default: return 0;
    }
    (void)h;
}

// Kernels use more than 64 KiB of dynamic LDS: raise the per-kernel limit (an attribute of the
// loaded kernel, not of a call) once per process, whichever thread calls first.
static int set_lds_limits()
{
    RELIBRA_HIP_TRY(hipFuncSetAttribute((const void *)fwd_gate_up_kernel<false>, hipFuncAttributeMaxDynamicSharedMemorySize, kLdsBytes));
    RELIBRA_HIP_TRY(hipFuncSetAttribute((const void *)fwd_gate_up_kernel<true>, hipFuncAttributeMaxDynamicSharedMemorySize, kLdsBytes));
    RELIBRA_HIP_TRY(hipFuncSetAttribute((const void *)fwd_down_kernel<false>, hipFuncAttributeMaxDynamicSharedMemorySize, kLdsBytes));
    RELIBRA_HIP_TRY(hipFuncSetAttribute((const void *)fwd_down_kernel<true>, hipFuncAttributeMaxDynamicSharedMemorySize, kLdsBytes));
    RELIBRA_HIP_TRY(hipFuncSetAttribute((const void *)bwd_act_kernel<false>, hipFuncAttributeMaxDynamicSharedMemorySize, kLdsBytes));
    RELIBRA_HIP_TRY(hipFuncSetAttribute((const void *)bwd_act_kernel<true>, hipFuncAttributeMaxDynamicSharedMemorySize, kLdsBytes));
    RELIBRA_HIP_TRY(hipFuncSetAttribute((const void *)bwd_act_kernel<false, true>, hipFuncAttributeMaxDynamicSharedMemorySize, kLdsBytes));
    RELIBRA_HIP_TRY(hipFuncSetAttribute((const void *)bwd_act_kernel<true, true>, hipFuncAttributeMaxDynamicSharedMemorySize, kLdsBytes));
    RELIBRA_HIP_TRY(hipFuncSetAttribute((const void *)bwd_act_kernel<false, false, 512>, hipFuncAttributeMaxDynamicSharedMemorySize, kLdsBytesWide));
    RELIBRA_HIP_TRY(hipFuncSetAttribute((const void *)bwd_act_kernel<true, false, 512>, hipFuncAttributeMaxDynamicSharedMemorySize, kLdsBytesWide));
    RELIBRA_HIP_TRY(hipFuncSetAttribute((const void *)bwd_act_kernel<false, true, 512>, hipFuncAttributeMaxDynamicSharedMemorySize, kLdsBytesWide));
    RELIBRA_HIP_TRY(hipFuncSetAttribute((const void *)bwd_act_kernel<true, true, 512>, hipFuncAttributeMaxDynamicSharedMemorySize, kLdsBytesWide));
    RELIBRA_HIP_TRY(hipFuncSetAttribute((const void *)bwd_dx_kernel<false>, hipFuncAttributeMaxDynamicSharedMemorySize, kLdsBytes));
    RELIBRA_HIP_TRY(hipFuncSetAttribute((const void *)bwd_dx_kernel<true>, hipFuncAttributeMaxDynamicSharedMemorySize, kLdsBytes));
    RELIBRA_HIP_TRY(hipFuncSetAttribute((const void *)fwd_gate_up_kernel<false, 256>, hipFuncAttributeMaxDynamicSharedMemorySize, kLdsBytesWide));
    RELIBRA_HIP_TRY(hipFuncSetAttribute((const void *)fwd_gate_up_kernel<true, 256>, hipFuncAttributeMaxDynamicSharedMemorySize, kLdsBytesWide));
    RELIBRA_HIP_TRY(hipFuncSetAttribute((const void *)fwd_down_kernel<false, 512>, hipFuncAttributeMaxDynamicSharedMemorySize, kLdsBytesWide));
    RELIBRA_HIP_TRY(hipFuncSetAttribute((const void *)fwd_down_kernel<true, 512>, hipFuncAttributeMaxDynamicSharedMemorySize, kLdsBytesWide));
    RELIBRA_HIP_TRY(hipFuncSetAttribute((const void *)bwd_dx_kernel<false, 512>, hipFuncAttributeMaxDynamicSharedMemorySize, kLdsBytesWide));
    RELIBRA_HIP_TRY(hipFuncSetAttribute((const void *)bwd_dx_kernel<true, 512>, hipFuncAttributeMaxDynamicSharedMemorySize, kLdsBytesWide));
    RELIBRA_HIP_TRY(hipFuncSetAttribute((const void *)wgrad_kernel<1, 256>, hipFuncAttributeMaxDynamicSharedMemorySize, WgradCfg<256>::LDS));
    RELIBRA_HIP_TRY(hipFuncSetAttribute((const void *)wgrad_kernel<2, 256>, hipFuncAttributeMaxDynamicSharedMemorySize, WgradCfg<256>::LDS));
    RELIBRA_HIP_TRY(hipFuncSetAttribute((const void *)wgrad_batched_kernel<1, 128>, hipFuncAttributeMaxDynamicSharedMemorySize, WgradWide<128>::LDS));
    RELIBRA_HIP_TRY(hipFuncSetAttribute((const void *)wgrad_batched_kernel<2, 128>, hipFuncAttributeMaxDynamicSharedMemorySize, WgradWide<128>::LDS));
    RELIBRA_HIP_TRY(hipFuncSetAttribute((const void *)wgrad_batched_kernel<1, 256, kWideWaves>, hipFuncAttributeMaxDynamicSharedMemorySize, WgradWide<256>::LDS));
    RELIBRA_HIP_TRY(hipFuncSetAttribute((const void *)wgrad_batched_kernel<2, 256, kWideWaves>, hipFuncAttributeMaxDynamicSharedMemorySize, WgradWide<256>::LDS));
    RELIBRA_HIP_TRY(hipFuncSetAttribute((const void *)wgrad_kernel<1, 128>, hipFuncAttributeMaxDynamicSharedMemorySize, WgradCfg<128>::LDS));
    RELIBRA_HIP_TRY(hipFuncSetAttribute((const void *)wgrad_kernel<2, 128>, hipFuncAttributeMaxDynamicSharedMemorySize, WgradCfg<128>::LDS));
    return RELIBRA_OK;
}
static int ensure_lds_limits()
{
    static std::once_flag once;
    static int status = RELIBRA_OK;
    std::call_once(once, [] { status = set_lds_limits(); });
    return status;
}

static inline unsigned grid8(long long tiles) { return (unsigned)((tiles + 7) / 8 * 8); }

// The wide column tiles are taken where they divide the output (a ragged last tile of that width
// would idle half a workgroup).
static inline bool row_tiles_wide(int n_dim, int width) { return n_dim % width == 0; }

// Launch of a row-tiled GEMM kernel template <bool WT, int AW>: narrow (four waves, two workgroups
// per compute unit) or wide (eight waves, one) column tiles.
#define RELIBRA_ROW_LAUNCH(kid, kern, wt_, wide_, AWN, AWW, tiles, ...)                                                      \
    do {                                                                                                                      \
        if (wide_) {                                                                                                          \
            if (wt_) RELIBRA_LAUNCH(kid, stream, (kern<true, AWW><<<grid8(tiles), kWideRowWaves * 64, kLdsBytesWide, stream>>>(__VA_ARGS__)));  \
            else RELIBRA_LAUNCH(kid, stream, (kern<false, AWW><<<grid8(tiles), kWideRowWaves * 64, kLdsBytesWide, stream>>>(__VA_ARGS__)));    \
        } else {                                                                                                              \
            if (wt_) RELIBRA_LAUNCH(kid, stream, (kern<true, AWN><<<grid8(tiles), THREADS, kLdsBytes, stream>>>(__VA_ARGS__)));   \
            else RELIBRA_LAUNCH(kid, stream, (kern<false, AWN><<<grid8(tiles), THREADS, kLdsBytes, stream>>>(__VA_ARGS__)));     \
        }                                                                                                                     \
    } while (0)


// Xrows: the group-ordered rows, or (row_tok != nullptr) the token tensor [T, h] they are gathered from.
static int ffn_fwd_impl(const void *Xrows, const int32_t *row_tok, int T, int n_rows,
                                   const int32_t *group_offset, const int32_t *group_expert,
                                   int G, int g_begin, int g_end, int E,
                                   const void *Wg, const void *Wu, const void *Wd, int h, int hff,
                                   void *Gt_save, void *U_save, void *A_save, void *Yrows, int flags,
                                   void *ws, size_t ws_bytes, int32_t *err_flag, relibra_stream stream_,
                                   const float *row_gate = nullptr, void *Ag_save = nullptr)
{
    hipStream_t stream = (hipStream_t)stream_;
    if (flags & ~RELIBRA_FWD_TRANSPOSED_WEIGHTS) return RELIBRA_EINVAL;
    if ((row_gate == nullptr) != (Ag_save == nullptr) || !aligned16(Ag_save)) return RELIBRA_EINVAL;   // Ag_save == A_save: gated in place
    const bool wt = (flags & RELIBRA_FWD_TRANSPOSED_WEIGHTS) != 0;
    const FfnArgs a{n_rows, G, g_begin, g_end, E, h, hff};
    if (int rc = check_ffn_args(a)) return rc;
    const int Gr = g_end - g_begin;
    if (Gr == 0 || n_rows == 0) return RELIBRA_OK;
    if (!Xrows || !group_offset || !group_expert || !Wg || !Wu || !Wd || !Gt_save || !U_save || !A_save ||
        !Yrows || !ws || !err_flag)
        return RELIBRA_EINVAL;
    if (!aligned16(Xrows) || !aligned16(Wg) || !aligned16(Wu) || !aligned16(Wd) || !aligned16(A_save) ||
        !aligned16(Gt_save) || !aligned16(U_save) || !aligned16(Yrows) || !aligned16(ws))
        return RELIBRA_EINVAL;
    if (ws_bytes < ffn_ws_bytes(n_rows, Gr, hff, false)) return RELIBRA_EWORKSPACE;
    if (int rc = ensure_lds_limits()) return rc;
    Sched s = carve(ws, n_rows, Gr, hff, false);
    RELIBRA_LAUNCH(RELIBRA_K_SCHED, stream, sched_kernel<<<1, 256, (size_t)(Gr + 1) * sizeof(int32_t), stream>>>(group_offset, group_expert, nullptr, g_begin, Gr, n_rows, E, 0, s, err_flag));
    RELIBRA_HIP_TRY(launch_check());
    const long long R = max_row_tiles(n_rows, Gr);
    // column tiles: the wide ones where they divide the output
    const bool wide1 = row_tiles_wide(hff, 256), wide2 = row_tiles_wide(h, 512);
    const int ct1 = wide1 ? hff / 256 : (hff + 127) / 128, ct2 = wide2 ? h / 512 : (h + 255) / 256;
    RELIBRA_ROW_LAUNCH(RELIBRA_K_FWD_GATE_UP, fwd_gate_up_kernel, wt, wide1, 128, 256, R * ct1,
                       s, (const bf16_t *)Xrows, row_tok, T - 1, (const bf16_t *)Wg, (const bf16_t *)Wu, h, hff, ct1,
                       (bf16_t *)Gt_save, (bf16_t *)U_save, (bf16_t *)A_save, row_gate, (bf16_t *)Ag_save);
    RELIBRA_HIP_TRY(launch_check());
    RELIBRA_ROW_LAUNCH(RELIBRA_K_FWD_DOWN, fwd_down_kernel, wt, wide2, 256, 512, R * ct2,
                       s, (const bf16_t *)A_save, (const bf16_t *)Wd, h, hff, ct2, (bf16_t *)Yrows);
    RELIBRA_HIP_TRY(launch_check());
    return RELIBRA_OK;
}

extern "C" int relibra_moe_ffn_fwd(const void *Xrows, int n_rows,
                                   const int32_t *group_offset, const int32_t *group_expert,
                                   int G, int g_begin, int g_end, int E,
                                   const void *Wg, const void *Wu, const void *Wd, int h, int hff,
                                   void *Gt_save, void *U_save, void *A_save, void *Yrows, int flags,
                                   void *ws, size_t ws_bytes, int32_t *err_flag, relibra_stream stream_)
{
    return ffn_fwd_impl(Xrows, nullptr, 1, n_rows, group_offset, group_expert, G, g_begin, g_end, E, Wg, Wu, Wd, h, hff,
                        Gt_save, U_save, A_save, Yrows, flags, ws, ws_bytes, err_flag, stream_);
}

extern "C" int relibra_moe_ffn_fwd_gather(const void *X, int T, const int32_t *row_tok, int n_rows,
                                          const int32_t *group_offset, const int32_t *group_expert,
                                          int G, int g_begin, int g_end, int E,
                                          const void *Wg, const void *Wu, const void *Wd, int h, int hff,
                                          void *Gt_save, void *U_save, void *A_save, void *Yrows, int flags,
                                          void *ws, size_t ws_bytes, int32_t *err_flag, relibra_stream stream_)
{
    if (T < 1 || !row_tok) return RELIBRA_EINVAL;
    return ffn_fwd_impl(X, row_tok, T, n_rows, group_offset, group_expert, G, g_begin, g_end, E, Wg, Wu, Wd, h, hff,
                        Gt_save, U_save, A_save, Yrows, flags, ws, ws_bytes, err_flag, stream_);
}

extern "C" int relibra_moe_ffn_fwd_gated(const void *X, int T, const int32_t *row_tok, const float *row_gate, int n_rows,
                                         const int32_t *group_offset, const int32_t *group_expert,
                                         int G, int g_begin, int g_end, int E,
                                         const void *Wg, const void *Wu, const void *Wd, int h, int hff,
                                         void *Gt_save, void *U_save, void *A_save, void *Ag_save, void *Yrows, int flags,
                                         void *ws, size_t ws_bytes, int32_t *err_flag, relibra_stream stream_)
{
    if (T < 1 || !row_tok || !row_gate || !Ag_save) return RELIBRA_EINVAL;
    return ffn_fwd_impl(X, row_tok, T, n_rows, group_offset, group_expert, G, g_begin, g_end, E, Wg, Wu, Wd, h, hff,
                        Gt_save, U_save, A_save, Yrows, flags, ws, ws_bytes, err_flag, stream_, row_gate, Ag_save);
}

// Gate-fused form of the backward call: the upstream gradient comes from the token tensor.
struct GatedBwd {
    const void *dOut;
    int T;
    const int32_t *row_tok;
    const float *row_gate;
    const int32_t *src_of;   // optional
    float *dgate;
    void *scratch;
    size_t scratch_bytes;
};

static int ffn_bwd_impl(const void *dYrows, const void *Xrows,
                                   const void *Gt_save, const void *U_save, const void *A_save, int n_rows,
                                   const int32_t *group_offset, const int32_t *group_expert,
                                   const int32_t *group_dw_slot,
                                   int G, int g_begin, int g_end, int E, int n_dw_slots,
                                   const void *Wg, const void *Wu, const void *Wd, int h, int hff,
                                   void *dXrows, float *dWg, float *dWu, float *dWd, int flags,
                                   void *ws, size_t ws_bytes, int32_t *err_flag, relibra_stream stream_,
                                   const GatedBwd *gb)
{
    hipStream_t stream = (hipStream_t)stream_;
    const FfnArgs a{n_rows, G, g_begin, g_end, E, h, hff};
    if (int rc = check_ffn_args(a)) return rc;
    if (n_dw_slots < E) return RELIBRA_EINVAL;
    if (gb) {
        if (!(flags & RELIBRA_BWD_DEFER_WGRAD) || gb->T < 1 || !gb->dOut || !gb->row_tok || !gb->row_gate || !gb->dgate ||
            !gb->scratch || !aligned16(gb->dOut) || !aligned16(gb->scratch))
            return RELIBRA_EINVAL;
        if (gb->scratch_bytes < dgate_scratch_bytes(n_rows, hff)) return RELIBRA_EWORKSPACE;
        dYrows = gb->dOut;                       // the argument checks below see the tensor the kernels read
    }
    const int Gr = g_end - g_begin;
    if (Gr == 0) return RELIBRA_OK;
    const bool defer = (flags & RELIBRA_BWD_DEFER_WGRAD) != 0;    // then dW is not touched and may be null
    // Xrows is an operand of the weight gradients only
    if (!dYrows || !Gt_save || !U_save || !A_save || !group_offset || !group_expert || !group_dw_slot ||
        !Wg || !Wu || !Wd || !dXrows || !ws || !err_flag || (!defer && (!Xrows || !dWg || !dWu || !dWd)))
        return RELIBRA_EINVAL;
    if (!aligned16(dYrows) || !aligned16(Xrows) || !aligned16(A_save) || !aligned16(Gt_save) || !aligned16(U_save) ||
        !aligned16(Wg) || !aligned16(Wu) || !aligned16(Wd) || !aligned16(dXrows) || !aligned16(dWg) ||
        !aligned16(dWu) || !aligned16(dWd) || !aligned16(ws))
        return RELIBRA_EINVAL;
    if (ws_bytes < ffn_ws_bytes(n_rows, Gr, hff, true)) return RELIBRA_EWORKSPACE;
    if (int rc = ensure_lds_limits()) return rc;
    Sched s = carve(ws, n_rows, Gr, hff, true);
    // the slot table matters only to kernels that write dW or read replica parameters
    const int32_t *slot_table = (defer && !(flags & RELIBRA_BWD_REPLICA_WEIGHTS)) ? nullptr : group_dw_slot;
    RELIBRA_LAUNCH(RELIBRA_K_SCHED, stream, sched_kernel<<<1, 256, (size_t)(Gr + 1) * sizeof(int32_t), stream>>>(group_offset, group_expert, slot_table, g_begin, Gr, n_rows, E,
                                        n_dw_slots, s, err_flag));
    RELIBRA_HIP_TRY(launch_check());
    const long long R = max_row_tiles(n_rows, Gr);
    const bool wide_h = row_tiles_wide(h, 512);
    const bool wide_ff = row_tiles_wide(hff, 512);
    const int ct_ff = wide_ff ? hff / 512 : (hff + 255) / 256, ct_h = wide_h ? h / 512 : (h + 255) / 256;
    const int accumulate = (flags & RELIBRA_BWD_ACCUMULATE) ? 1 : 0;
    const int w_from_slot = (flags & RELIBRA_BWD_REPLICA_WEIGHTS) ? 1 : 0;
    if (n_rows > 0) {
        const bf16_t *wd = (const bf16_t *)Wd, *wg = (const bf16_t *)Wg, *wu = (const bf16_t *)Wu;
        const bf16_t *dy = (const bf16_t *)dYrows, *gt = (const bf16_t *)Gt_save, *us = (const bf16_t *)U_save;
        const bool wt = (flags & RELIBRA_BWD_TRANSPOSED_WEIGHTS) != 0;
        GateFusion gf;
        gf.n_rows = n_rows;
        if (gb) {
            gf.row_tok = gb->row_tok;
            gf.tok_last = gb->T - 1;
            gf.row_gate = gb->row_gate;
            gf.dgate_part = (float *)gb->scratch;
        }
#define RELIBRA_BWD_ACT(WT_, GATED_)                                                                                              \
    do {                                                                                                                          \
        if (wide_ff) RELIBRA_LAUNCH(RELIBRA_K_BWD_ACT, stream, (bwd_act_kernel<WT_, GATED_, 512><<<grid8(R * ct_ff), kWideRowWaves * 64, kLdsBytesWide, stream>>>( \
            s, dy, wd, gt, us, h, hff, ct_ff, w_from_slot, gf)));                                                                 \
        else RELIBRA_LAUNCH(RELIBRA_K_BWD_ACT, stream, (bwd_act_kernel<WT_, GATED_, 256><<<grid8(R * ct_ff), THREADS, kLdsBytes, stream>>>(         \
            s, dy, wd, gt, us, h, hff, ct_ff, w_from_slot, gf)));                                                                 \
    } while (0)
        if (wt) { if (gb) RELIBRA_BWD_ACT(true, true); else RELIBRA_BWD_ACT(true, false); }
        else { if (gb) RELIBRA_BWD_ACT(false, true); else RELIBRA_BWD_ACT(false, false); }
#undef RELIBRA_BWD_ACT
        RELIBRA_HIP_TRY(launch_check());
        if (wt) RELIBRA_ROW_LAUNCH(RELIBRA_K_BWD_DX, bwd_dx_kernel, true, wide_h, 256, 512, R * ct_h,
                                   s, wg, wu, h, hff, ct_h, w_from_slot, (bf16_t *)dXrows);
        else RELIBRA_ROW_LAUNCH(RELIBRA_K_BWD_DX, bwd_dx_kernel, false, wide_h, 256, 512, R * ct_h,
                                s, wg, wu, h, hff, ct_h, w_from_slot, (bf16_t *)dXrows);
        RELIBRA_HIP_TRY(launch_check());
        if (gb) {
            RELIBRA_LAUNCH(RELIBRA_K_DGATE_REDUCE, stream, dgate_reduce_kernel<<<std::min(1024, (n_rows + 255) / 256), 256, 0, stream>>>(
                (const float *)gb->scratch, kDgateParts * ((hff + 255) / 256), n_rows, group_offset, g_begin, g_end, gb->src_of, gb->dgate, err_flag));
            RELIBRA_HIP_TRY(launch_check());
        }
    }
    if (defer) return RELIBRA_OK;                                  // dGt, dU stay in the workspace
    // short groups (few rows per group on average): the small, high-occupancy geometry
    const bool small_tiles = (long long)n_rows < 512LL * Gr;
    const int wgm = small_tiles ? 128 : 256;
    const long long t_down = (long long)Gr * ((h + wgm - 1) / wgm) * ((hff + WGN - 1) / WGN);              // dWd: m in h, n in h'
    const long long t_gu = (long long)Gr * ((hff + wgm / 2 - 1) / (wgm / 2)) * ((h + WGN - 1) / WGN);      // dWg, dWu: m in h', n in h
    if (small_tiles) {
        RELIBRA_LAUNCH(RELIBRA_K_WGRAD_DOWN, stream, wgrad_kernel<1, 128><<<grid8(t_down), THREADS, WgradCfg<128>::LDS, stream>>>(
            s, (const bf16_t *)dYrows, nullptr, (const bf16_t *)A_save, h, hff, E, accumulate, (int)t_down, dWd, nullptr));
        RELIBRA_HIP_TRY(launch_check());
        RELIBRA_LAUNCH(RELIBRA_K_WGRAD_GATE_UP, stream, wgrad_kernel<2, 128><<<grid8(t_gu), THREADS, WgradCfg<128>::LDS, stream>>>(
            s, s.dGt, s.dU, (const bf16_t *)Xrows, hff, h, E, accumulate, (int)t_gu, dWg, dWu));
        RELIBRA_HIP_TRY(launch_check());
    } else {
        RELIBRA_LAUNCH(RELIBRA_K_WGRAD_DOWN, stream, wgrad_kernel<1, 256><<<grid8(t_down), THREADS, WgradCfg<256>::LDS, stream>>>(
            s, (const bf16_t *)dYrows, nullptr, (const bf16_t *)A_save, h, hff, E, accumulate, (int)t_down, dWd, nullptr));
        RELIBRA_HIP_TRY(launch_check());
        RELIBRA_LAUNCH(RELIBRA_K_WGRAD_GATE_UP, stream, wgrad_kernel<2, 256><<<grid8(t_gu), THREADS, WgradCfg<256>::LDS, stream>>>(
            s, s.dGt, s.dU, (const bf16_t *)Xrows, hff, h, E, accumulate, (int)t_gu, dWg, dWu));
        RELIBRA_HIP_TRY(launch_check());
    }
    if (!(flags & RELIBRA_BWD_NO_REPLICA_SUM) && n_dw_slots > E) {
        const size_t vec4 = (size_t)h * hff / 4;
        const int grid = (int)((vec4 + 255) / 256 < 4096 ? (vec4 + 255) / 256 : 4096);
        RELIBRA_LAUNCH(RELIBRA_K_REPLICA_SUM, stream, replica_sum_kernel<<<dim3(grid, 3), 256, 0, stream>>>(
            s, vec4, (float4 *)dWg, (float4 *)dWu, (float4 *)dWd));
        RELIBRA_HIP_TRY(launch_check());
    }
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
    return ffn_bwd_impl(dYrows, Xrows, Gt_save, U_save, A_save, n_rows, group_offset, group_expert, group_dw_slot, G, g_begin,
                        g_end, E, n_dw_slots, Wg, Wu, Wd, h, hff, dXrows, dWg, dWu, dWd, flags, ws, ws_bytes, err_flag, stream_,
                        nullptr);
}

extern "C" int relibra_moe_ffn_bwd_gated(const void *dOut, int T, const int32_t *row_tok, const float *row_gate,
                                         const int32_t *src_of,
                                         const void *Gt_save, const void *U_save, int n_rows,
                                         const int32_t *group_offset, const int32_t *group_expert,
                                         const int32_t *group_dw_slot,
                                         int G, int g_begin, int g_end, int E, int n_dw_slots,
                                         const void *Wg, const void *Wu, const void *Wd, int h, int hff,
                                         void *dXrows, float *dgate, int flags,
                                         void *ws, size_t ws_bytes, void *dgate_scratch, size_t dgate_scratch_bytes_,
                                         int32_t *err_flag, relibra_stream stream_)
{
    if (flags & ~(RELIBRA_BWD_REPLICA_WEIGHTS | RELIBRA_BWD_TRANSPOSED_WEIGHTS | RELIBRA_BWD_DEFER_WGRAD)) return RELIBRA_EINVAL;
    const GatedBwd gb{dOut, T, row_tok, row_gate, src_of, dgate, dgate_scratch, dgate_scratch_bytes_};
    // the saved activations are an operand of the weight gradients only: Gt stands in for the pointer check
    return ffn_bwd_impl(nullptr, nullptr, Gt_save, U_save, Gt_save, n_rows, group_offset, group_expert, group_dw_slot, G, g_begin,
                        g_end, E, n_dw_slots, Wg, Wu, Wd, h, hff, dXrows, nullptr, nullptr, nullptr,
                        flags | RELIBRA_BWD_DEFER_WGRAD, ws, ws_bytes, err_flag, stream_, &gb);
}

extern "C" int relibra_moe_ffn_wgrad_batched(const relibra_wgrad_mb *mbs, int n_mb, int n_rows,
                                             int G, int inst_cap, int E, int h, int hff,
                                             float *dWg, float *dWu, float *dWd, int flags,
                                             void *ws, size_t ws_bytes, int32_t *err_flag, relibra_stream stream_)
{
    hipStream_t stream = (hipStream_t)stream_;
    if (flags & ~(RELIBRA_WGRAD_ACCUMULATE | RELIBRA_WGRAD_TILE_NARROW | RELIBRA_WGRAD_TILE_WIDE)) return RELIBRA_EINVAL;
    if ((flags & RELIBRA_WGRAD_TILE_NARROW) && (flags & RELIBRA_WGRAD_TILE_WIDE)) return RELIBRA_EINVAL;
    const int accumulate = (flags & RELIBRA_WGRAD_ACCUMULATE) ? 1 : 0;
    const FfnArgs a{n_rows, G, 0, G, E, h, hff};
    if (int rc = check_ffn_args(a)) return rc;
    if (!mbs || n_mb < 1 || n_mb > kMaxWgradMb || inst_cap < 1 || E > 4096) return RELIBRA_EINVAL;
    if (!dWg || !dWu || !dWd || !ws || !err_flag || !aligned16(dWg) || !aligned16(dWu) || !aligned16(dWd) || !aligned16(ws))
        return RELIBRA_EINVAL;
    if (ws_bytes < relibra_workspace_bytes(RELIBRA_WS_WGRAD_BATCHED, 0, 1, E, G, h, hff)) return RELIBRA_EWORKSPACE;
    MbTable tb;
    tb.dy_tokens = 0;
    for (int mb = 0; mb < kMaxWgradMb; ++mb) {
        const relibra_wgrad_mb &m = mbs[mb < n_mb ? mb : 0];
        if (mb < n_mb) {
            const bool gathered = m.Xrows_dev == nullptr;
            if (!m.dYrows_dev && (!m.dOut_dev || !gathered || !aligned16(m.dOut_dev))) return RELIBRA_EINVAL;
            if (!m.A_save_dev || !m.bwd_workspace_dev || !m.inst_ptr_dev || !m.inst_group_dev ||
                !m.group_offset_dev || (gathered && (!m.X_dev || !m.row_tok_dev || m.n_tokens < 1)))
                return RELIBRA_EINVAL;
            if (!aligned16(m.dYrows_dev) || !aligned16(gathered ? m.X_dev : m.Xrows_dev) || !aligned16(m.A_save_dev) ||
                !aligned16(m.bwd_workspace_dev))
                return RELIBRA_EINVAL;
        }
        const Sched s = carve(const_cast<void *>(m.bwd_workspace_dev), n_rows, G, hff, true);
        tb.dY[mb] = (const bf16_t *)(m.dYrows_dev ? m.dYrows_dev : m.dOut_dev);
        if (!m.dYrows_dev) tb.dy_tokens |= 1ull << mb;
        tb.X[mb] = (const bf16_t *)(m.Xrows_dev ? m.Xrows_dev : m.X_dev);
        tb.rtok[mb] = m.Xrows_dev ? nullptr : m.row_tok_dev;
        tb.tok_last[mb] = m.Xrows_dev ? 0 : m.n_tokens - 1;
        tb.A[mb] = (const bf16_t *)m.A_save_dev;
        tb.dGt[mb] = s.dGt;
        tb.dU[mb] = s.dU;
        tb.iptr[mb] = m.inst_ptr_dev;
        tb.igrp[mb] = m.inst_group_dev;
        tb.goff[mb] = m.group_offset_dev;
    }
    if (int rc = ensure_lds_limits()) return rc;
    if (inst_cap > E + G) return RELIBRA_EINVAL;               // an instance is a group: at most G of them
    const WgradPlan w = carve_wgrad(ws, E, G);
    RELIBRA_LAUNCH(RELIBRA_K_WGRAD_ORDER, stream, wgrad_order_kernel<<<1, 256, E * sizeof(int32_t), stream>>>(
        tb, n_mb, G, inst_cap, n_rows, E, h, hff, w, err_flag));
    RELIBRA_HIP_TRY(launch_check());
    auto grid_of = [&](long long tiles_per_expert) {          // blocks: 8 XCDs x chunks per XCD x tiles per chunk
        const long long chunks = ((long long)E * tiles_per_expert + kWgradChunk - 1) / kWgradChunk;
        return (unsigned)(8 * ((chunks + 7) / 8) * kWgradChunk);
    };
    // Tile width.  The 256-column tile moves two thirds of the operand bytes per flop and is the
    // default wherever the output is at least that wide (measured on every workload shape: 3-10 %
    // faster), with one exception: dWd with a narrow h' and a short contraction, where its three
    // tile columns lose to the narrow tile's six (h' = 768, 8 k rows per expert: 3.76 against 3.62 ms).
    const bool long_k = (long long)n_rows * n_mb >= (long long)16384 * E;
    const bool forced = (flags & (RELIBRA_WGRAD_TILE_NARROW | RELIBRA_WGRAD_TILE_WIDE)) != 0;
    const bool want_wide = (flags & RELIBRA_WGRAD_TILE_WIDE) != 0;
    const bool wide_down = forced ? want_wide : (hff >= 1024 || (long_k && hff >= 256));
    const bool wide_gu = forced ? want_wide : h >= 256;
    const int wn_down = wide_down ? 256 : 128, wn_gu = wide_gu ? 256 : 128;
    const unsigned g_down = grid_of((long long)((h + 255) / 256) * ((hff + wn_down - 1) / wn_down));  // dWd: m in h, n in h'
    const unsigned g_gu = grid_of((long long)((hff + 127) / 128) * ((h + wn_gu - 1) / wn_gu));        // dWg, dWu: m in h', n in h
    if (wide_down) {
        RELIBRA_LAUNCH(RELIBRA_K_WGRAD_DOWN, stream, (wgrad_batched_kernel<1, 256, kWideWaves><<<g_down, kWideWaves * 64, WgradWide<256>::LDS, stream>>>(
            E, h, hff, w, accumulate, dWd, nullptr)));
    } else {
        RELIBRA_LAUNCH(RELIBRA_K_WGRAD_DOWN, stream, wgrad_batched_kernel<1, 128><<<g_down, THREADS, WgradWide<128>::LDS, stream>>>(
            E, h, hff, w, accumulate, dWd, nullptr));
    }
    RELIBRA_HIP_TRY(launch_check());
    if (wide_gu) {
        RELIBRA_LAUNCH(RELIBRA_K_WGRAD_GATE_UP, stream, (wgrad_batched_kernel<2, 256, kWideWaves><<<g_gu, kWideWaves * 64, WgradWide<256>::LDS, stream>>>(
            E, hff, h, w, accumulate, dWg, dWu)));
    } else {
        RELIBRA_LAUNCH(RELIBRA_K_WGRAD_GATE_UP, stream, wgrad_batched_kernel<2, 128><<<g_gu, THREADS, WgradWide<128>::LDS, stream>>>(
            E, hff, h, w, accumulate, dWg, dWu));
    }
    RELIBRA_HIP_TRY(launch_check());
    return RELIBRA_OK;
}

extern "C" int relibra_transpose_experts(const void *in_dev, int n_blocks, int rows, int cols, void *out_dev,
                                         relibra_stream stream_)
{
    hipStream_t stream = (hipStream_t)stream_;
    if (n_blocks < 0 || rows < 8 || cols < 8 || rows % 8 || cols % 8 || n_blocks > 65535) return RELIBRA_EINVAL;
    if (n_blocks == 0) return RELIBRA_OK;
    if (!in_dev || !out_dev || in_dev == out_dev || !aligned16(in_dev) || !aligned16(out_dev)) return RELIBRA_EINVAL;
    if ((rows + 63) / 64 > 65535) return RELIBRA_EUNSUPPORTED;
    const dim3 grid((cols + 63) / 64, (rows + 63) / 64, n_blocks);
    RELIBRA_LAUNCH(RELIBRA_K_TRANSPOSE, stream, transpose_experts_kernel<<<grid, 256, 0, stream>>>(
        (const bf16_t *)in_dev, rows, cols, (bf16_t *)out_dev));
    RELIBRA_HIP_TRY(launch_check());
    return RELIBRA_OK;
}
