// Building blocks of the grouped bf16 MFMA GEMMs (gfx950): LDS operand tiles filled by
// direct global->LDS loads, MFMA fragment reads, and a k-loop pipelined over a ring of LDS slabs.
//
// An operand tile covers ROWS rows of the non-contracted index and BKT (32 or 64) values of the
// contracted index k.  Two memory situations:
//   KcTile: k contiguous in memory (element (row,k) at base[row*ld + k]).  LDS holds [row][BKT],
//           64 or 128 bytes per row, 16-byte pieces XOR-swizzled by the row so that the 16-byte
//           fragment reads of 32 consecutive rows spread over all banks.  With BKT = 64 a row
//           is one full 128-byte line per load: the L1's outstanding requests, which bound the
//           L2 -> LDS rate, carry twice the bytes (measured 17 against 12 TB/s, loads alone).
//   KsTile: k strided in memory (element (row,k) at base[k*ld + row]).  LDS holds [k][ROWS] as
//           it lies in memory; fragments are read with the transposing LDS read
//           (ds_read_b64_tr_b16), 16-byte pieces XOR-swizzled by k.
// global_load_lds writes 64 lanes x 16 bytes to 1 KiB of consecutive LDS; which global address
// a lane fetches is free, so the swizzle is applied on the global side.
#pragma once
#include "common.h"
#include <type_traits>

namespace relibra {

typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef float f32x16_t __attribute__((ext_vector_type(16)));
typedef short s16x4_t __attribute__((ext_vector_type(4)));
typedef short s16x8_t __attribute__((ext_vector_type(8)));

constexpr int BK = 32;                      // default contraction slab per pipeline stage (two k16 MFMA steps)

// Uniform loads through this type are scalar loads (tracked by lgkmcnt, not by the vmcnt the
// pipeline counts by hand); the memory must not change while the kernel runs.
typedef const __attribute__((address_space(4))) int32_t *const_i32_ptr;
// C consecutive table entries as one scalar load (the table is only 4-byte aligned)
template <int C> struct ScalarRun {
    typedef int32_t vec __attribute__((ext_vector_type(C)));
    typedef vec unaligned __attribute__((aligned(4)));
    typedef const __attribute__((address_space(4))) unaligned *ptr;
};

#define RELIBRA_LDS(p) ((__attribute__((address_space(3))) void *)(p))
#define RELIBRA_GLB(p) ((const __attribute__((address_space(1))) void *)(p))

// s_waitcnt vmcnt(N) lgkmcnt(0) (gfx9 encoding; expcnt = 7 means "do not wait")
template <int N>
__device__ __forceinline__ void wait_vm_lgkm0()
{
    __builtin_amdgcn_s_waitcnt((N & 15) | (7 << 4) | ((N >> 4) << 14));
}

// One direct global->LDS load: 64 lanes x 16 bytes from the lanes' addresses g to the 1 KiB at the
// wave-uniform LDS address block.  Written as assembly so that the compiler keeps no record of
// LDS being filled behind its back: with the builtin it puts a wait for ALL of the wave's
// outstanding loads in front of every transposing LDS read, which empties the ring of slabs in
// flight; the k-loop counts vmcnt by hand anyway.  M0 carries the LDS address (one wait state
// between its write and the load).
// (M0 is a reserved register that the compiler does not otherwise use in these kernels; naming it
// as clobbered draws a warning that says so.)
#pragma clang diagnostic push
#pragma clang diagnostic ignored "-Winline-asm"
__device__ __forceinline__ void load_lds16(const bf16_t *g, char *block)
{
    const uint32_t m = (uint32_t)(uintptr_t)RELIBRA_LDS(block);
    asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off" : : "v"(g), "s"(m) : "memory", "m0");
}
// The same load with the address split into a wave-uniform base (scalar register pair) and a
// 32-bit per-lane byte offset: when only the uniform part changes from slab to slab, the k-loop
// spends no vector instruction on addresses.
__device__ __forceinline__ void load_lds16_sv(const bf16_t *uniform_base, uint32_t lane_byte_off, char *block)
{
    const uint32_t m = (uint32_t)(uintptr_t)RELIBRA_LDS(block);
    asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1" : : "v"(lane_byte_off), "s"(uniform_base), "s"(m) : "memory", "m0");
}
#pragma clang diagnostic pop

struct Operand {
    const bf16_t *base;   // see KcTile / KsTile for the addressing
    int ld;               // leading dimension in elements
    int row0;             // first row of the tile
    int row_last;         // last valid row; rows beyond are clamped onto valid ones (masked later)
    // Row gather (optional): row r of the operand is row gather[r] of `base` (clamped into
    // [0, gather_last]), so that rows of a token tensor are fetched in group order without a
    // gathered copy.  KcTile: r = the tile row.  KsTile: r = the contraction index.
    const int32_t *gather = nullptr;
    int gather_last = 0;
};

// k-contiguous operand: LDS [row][BKT].
// BKT = 32: 64 bytes per row, 16 rows per 1 KiB load block; piece c of row r sits at piece
//   c ^ g(r), g(r) = ((r>>1)&3) ^ ((r>>3)&1).
// BKT = 64: 128 bytes per row, 8 rows per block; g(r) = (r&7) ^ ((r>>3)&1).
// Either way the 16-byte reads of any 8 (or 16) consecutive rows at one k offset fall into
// distinct 16-byte bank groups.
template <int ROWS, int BKT = BK>
struct KcTile {
    static_assert(BKT == 32 || BKT == 64, "slab depth");
    static constexpr int DEPTH = BKT;
    static constexpr int ROW_BYTES = BKT * 2;
    static constexpr int PIECES = BKT / 8;            // 16-byte pieces per row
    static constexpr int RPB = 64 / PIECES;           // rows per 1 KiB block
    static constexpr int BYTES = ROWS * ROW_BYTES;
    static constexpr int BLOCKS = ROWS / RPB;
    static constexpr int READS = 1;                   // LDS read instructions per fragment
    // Load blocks per wave and slab.  A tile with fewer blocks than waves has every block loaded
    // by NW / BLOCKS waves (the same bytes to the same place), so that all waves issue the same
    // number of loads and count them alike.
    template <int NW>
    static constexpr int per_wave() { return BLOCKS >= NW ? BLOCKS / NW : 1; }

    static __device__ __forceinline__ int swz(int r)
    {
        return BKT == 32 ? (((r >> 1) & 3) ^ ((r >> 3) & 1)) : ((r & 7) ^ ((r >> 3) & 1));
    }

    // Per-lane source addresses (at k = 0) of the load blocks this wave issues for every slab: they
    // do not change along k, and a gathered row costs its index lookup once per tile.
    template <int NW>
    struct Lanes {
        const bf16_t *p[per_wave<NW>()];
    };
    template <int NW>
    static __device__ __forceinline__ Lanes<NW> prepare(const Operand &op, int wave, int lane)
    {
        static_assert(BLOCKS % NW == 0 || NW % BLOCKS == 0, "rows must split evenly over the waves");
        Lanes<NW> ln;
#pragma unroll
        for (int i = 0; i < per_wave<NW>(); ++i) {
            const int j = (wave + i * NW) % BLOCKS;
            const int r = j * RPB + lane / PIECES;
            const int c = (lane % PIECES) ^ swz(r);
            int grow = min(op.row0 + r, op.row_last);
            if (op.gather) grow = min(max(op.gather[grow], 0), op.gather_last);
            ln.p[i] = op.base + (size_t)grow * op.ld + c * 8;
        }
        return ln;
    }
    template <int NW>
    struct Idx {};                                     // nothing to look up per slab
    template <int NW>
    static __device__ __forceinline__ void fetch(Idx<NW> &, const Lanes<NW> &, int, int, int) {}
    // load block number i (0 .. BLOCKS/NW - 1) of this wave's share of a slab (the same in the steady state)
    template <int NW, bool STEADY = false>
    static __device__ __forceinline__ void load_one(char *lds, const Lanes<NW> &ln, const Idx<NW> &, int k0, int /*k_last*/, int wave,
                                                    int /*lane*/, int i)
    {
        load_lds16(ln.p[i] + k0, lds + ((wave + i * NW) % BLOCKS) * 1024);
    }
    template <int NW>
    static __device__ __forceinline__ void load(char *lds, const Lanes<NW> &ln, const Idx<NW> &ix, int k0, int k_last, int wave,
                                                int lane)
    {
#pragma unroll
        for (int i = 0; i < per_wave<NW>(); ++i) load_one<NW>(lds, ln, ix, k0, k_last, wave, lane, i);
    }

    // fragment of rows r0..r0+31 (r0 % 32 == 0), k = kk*16 + (lane/32)*8 .. +7
    static __device__ __forceinline__ bf16x8_t frag(const char *lds, int r0, int kk, int lane)
    {
        const int r = r0 + (lane & 31);
        const int c = (kk * 2 + (lane >> 5)) ^ swz(lane & 31);
        return *reinterpret_cast<const bf16x8_t *>(lds + r * ROW_BYTES + c * 16);
    }

    // Loading the tile in two halves (the load blocks of rows 0 .. ROWS/2-1, then the rest), for a
    // k-loop whose slabs are half as deep as this tile (KLoop, "deep B side"): one half per slab
    // period keeps the number of loads per wave and period constant while every request is a full
    // 128-byte line (BKT = 64).
    template <int NW>
    static constexpr int per_wave_half() { return BLOCKS / 2 >= NW ? BLOCKS / 2 / NW : 1; }
    template <int NW>
    struct LanesHalf {
        const bf16_t *p[2][per_wave_half<NW>()];
    };
    template <int NW>
    static __device__ __forceinline__ LanesHalf<NW> prepare_half(const Operand &op, int wave, int lane)
    {
        static_assert(BLOCKS % 2 == 0 && ((BLOCKS / 2) % NW == 0 || NW % (BLOCKS / 2) == 0), "rows must split evenly over the waves");
        LanesHalf<NW> ln;
#pragma unroll
        for (int half = 0; half < 2; ++half)
#pragma unroll
            for (int i = 0; i < per_wave_half<NW>(); ++i) {
                const int j = half * (BLOCKS / 2) + (wave + i * NW) % (BLOCKS / 2);
                const int r = j * RPB + lane / PIECES;
                const int c = (lane % PIECES) ^ swz(r);
                int grow = min(op.row0 + r, op.row_last);
                if (op.gather) grow = min(max(op.gather[grow], 0), op.gather_last);
                ln.p[half][i] = op.base + (size_t)grow * op.ld + c * 8;
            }
        return ln;
    }
    // load block number i of this wave's share of half `half` (uniform) of the tile whose first k is k0
    template <int NW>
    static __device__ __forceinline__ void load_half_one(char *lds, const LanesHalf<NW> &ln, int k0, int wave, int half, int i)
    {
        // both pointers are read with constant indices and blended by a mask: a select between the two
        // array elements would be turned into a dynamically indexed load, i.e. the array into scratch
        // memory, whose loads would also disturb the k-loop's hand-counted vmcnt
        const uintptr_t a0 = (uintptr_t)ln.p[0][i], a1 = (uintptr_t)ln.p[1][i];
        const uintptr_t m = (uintptr_t)0 - (uintptr_t)(half & 1);
        const bf16_t *src = (const bf16_t *)((a0 & ~m) | (a1 & m));
        load_lds16(src + k0, lds + (half * (BLOCKS / 2) + (wave + i * NW) % (BLOCKS / 2)) * 1024);
    }
};

// k-strided operand: LDS [k][ROWS] as in memory; 16-byte pieces of a k-row XOR-ed with fk(k) so
// that the 8-byte transposing reads of 4 k-rows x 16 (or 32) rows hit distinct banks.
// MAY_GATHER: the operand may carry a row table (Operand::gather); without it the lookup code is
// not compiled in (even unused it cost the weight-gradient kernels 4-5 %: selects and scalar
// registers in every load).
template <int ROWS, int BKT = BK, bool MAY_GATHER = false>
struct KsTile {
    static constexpr int DEPTH = BKT;
    static constexpr int BYTES = ROWS * BKT * 2;
    static constexpr int SPR = ROWS / 8;              // 16-byte pieces per k-row
    static constexpr int KPB = 64 / SPR;              // k-rows per 1 KiB block
    static constexpr int BLOCKS = BKT / KPB;
    static constexpr int READS = 2;                   // LDS read instructions per fragment
    static_assert(ROWS >= 64 && ROWS <= 512, "tile height");
    template <int NW>
    static constexpr int per_wave() { return BLOCKS / NW; }
    // i-th load block of a wave.  An operand that may be gathered gives a wave consecutive blocks,
    // so that the rows it looks up per slab are consecutive table entries (one wide scalar load).
    template <int NW>
    static __device__ __forceinline__ int block_of(int wave, int i)
    {
        return MAY_GATHER ? wave * (BLOCKS / NW) + i : wave + i * NW;
    }

    static __device__ __forceinline__ int fk(int k) { return (((k & 1) * 10) ^ (((k >> 1) & 1) * 4)) & (SPR - 1); }

    // The piece of a k-row a lane loads is XOR-ed with fk(k), which depends on k mod 4 only; with
    // the blocks dealt to the waves round robin and a number of waves divisible by four, k mod 4 of
    // a lane's k-row is the same in every block the wave loads, so the lane-dependent part of the
    // address is ONE constant: lane_off, in bytes from the first element of the block's first k-row.
    template <int NW>
    static constexpr bool steady_ok() { return !MAY_GATHER && NW % 4 == 0 && (KPB == 1 || KPB == 2 || KPB % 4 == 0); }
    template <int NW>
    struct Lanes {
        Operand op;
        uint32_t lane_off;
    };
    template <int NW>
    static __device__ __forceinline__ Lanes<NW> prepare(const Operand &op, int wave, int lane)
    {
        const int kq = lane / SPR;
        const int s = (lane % SPR) ^ fk(block_of<NW>(wave, 0) * KPB + kq);
        int grow = op.row0 + s * 8;
        if (grow > op.row_last) grow = op.row_last - 7;
        return Lanes<NW>{op, (uint32_t)(((long long)kq * op.ld + grow) * 2)};
    }

    // A gathered operand (contraction index -> row of `base`) needs, per slab, the rows of the KPB
    // k-rows of each of this wave's load blocks: fetched as scalars (fetch) ahead of the loads, in
    // one wide scalar load (one scalar load per k-row cost the weight gradients 1.5 % each: eight
    // per wave and slab 12 %; every lgkmcnt(0) of the loop waits for scalar loads too).
    template <int NW>
    struct Idx {
        int v[BLOCKS / NW][KPB];
    };
    template <int NW>
    static __device__ __forceinline__ void fetch(Idx<NW> &ix, const Lanes<NW> &ln, int k0, int k_last, int wave)
    {
        if (!MAY_GATHER || !ln.op.gather) return;
        const_i32_ptr g = (const_i32_ptr)(uintptr_t)ln.op.gather;
        constexpr int C = (BLOCKS / NW) * KPB;              // this wave's k-rows of the slab: consecutive
        const int first = k0 + block_of<NW>(wave, 0) * KPB;
        if (first + C - 1 <= k_last) {                      // all but a piece's last slab: no clamping
            const typename ScalarRun<C>::vec run = *(typename ScalarRun<C>::ptr)(g + first);
#pragma unroll
            for (int i = 0; i < BLOCKS / NW; ++i)
#pragma unroll
                for (int q = 0; q < KPB; ++q) ix.v[i][q] = run[i * KPB + q];
            return;
        }
#pragma unroll
        for (int i = 0; i < BLOCKS / NW; ++i)
#pragma unroll
            for (int q = 0; q < KPB; ++q) ix.v[i][q] = g[min(k0 + block_of<NW>(wave, i) * KPB + q, k_last)];
    }
    // The memory row of a k-row is the same for every lane that loads a piece of it, and a wave's
    // load block holds KPB k-rows: the rows (clamped, or looked up when the operand is gathered) and
    // their offsets are worked out with scalar instructions, one select per further k-row picks a
    // lane's own, and gathered and plain operands run the same branch-free sequence.
    // STEADY: the caller guarantees that every k-row of the slab exists (k0 + DEPTH - 1 <= k_last) and
    // that the operand has no row table; the address is then a uniform base plus the lane's constant.
    template <int NW, bool STEADY = false>
    static __device__ __forceinline__ void load_one(char *lds, const Lanes<NW> &ln, const Idx<NW> &ix, int k0, int k_last, int wave,
                                                    int lane, int i)
    {
        static_assert(BLOCKS % NW == 0, "k-rows must split evenly over the waves");
        const Operand &op = ln.op;
        const int j = block_of<NW>(wave, i);
        if (STEADY && steady_ok<NW>()) {
            load_lds16_sv(op.base + (long long)(k0 + j * KPB) * op.ld, ln.lane_off, lds + j * 1024);
            return;
        }
        const int kq = lane / SPR;                  // which of the block's k-rows this lane loads from
        const int s = (lane % SPR) ^ fk(j * KPB + kq);
        int grow = op.row0 + s * 8;
        if (grow > op.row_last) grow = op.row_last - 7;
        const bool gathered = MAY_GATHER && op.gather != nullptr;
        long long off = 0;
#pragma unroll
        for (int q = 0; q < KPB; ++q) {
            const int plain = min(k0 + j * KPB + q, k_last);
            const int looked = min(max(gathered ? ix.v[i][q] : 0, 0), op.gather_last);
            const long long row_off = (long long)(gathered ? looked : plain) * op.ld;       // scalar
            off = (q == 0 || kq == q) ? row_off : off;
        }
        load_lds16(op.base + off + grow, lds + j * 1024);
    }
    template <int NW>
    static __device__ __forceinline__ void load(char *lds, const Lanes<NW> &ln, const Idx<NW> &ix, int k0, int k_last, int wave,
                                                int lane)
    {
#pragma unroll
        for (int i = 0; i < BLOCKS / NW; ++i) load_one<NW>(lds, ln, ix, k0, k_last, wave, lane, i);
    }

    static __device__ __forceinline__ bf16x8_t frag(const char *lds, int r0, int kk, int lane)
    {
        const int b = lane >> 4, i = lane & 15;
        const int m = r0 + (b & 1) * 16 + (i & 3) * 4;
        const int kb = kk * 16 + (b >> 1) * 8 + (i >> 2);
        const int piece = (((m >> 3) ^ fk(kb)) * 16) + ((m >> 2) & 1) * 8;
        const s16x4_t lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
            (__attribute__((address_space(3))) s16x4_t *)RELIBRA_LDS(lds + kb * (ROWS * 2) + piece));
        const s16x4_t hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
            (__attribute__((address_space(3))) s16x4_t *)RELIBRA_LDS(lds + (kb + 4) * (ROWS * 2) + piece));
        const s16x8_t v = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
        return __builtin_bit_cast(bf16x8_t, v);
    }
};

// Zero the fragment elements whose k index is >= k_valid (ragged contraction, last slabs only).
__device__ __forceinline__ bf16x8_t mask_frag(bf16x8_t f, int k_first, int k_valid)
{
    s16x8_t v = __builtin_bit_cast(s16x8_t, f);
#pragma unroll
    for (int e = 0; e < 8; ++e)
        if (k_first + e >= k_valid) v[e] = 0;
    return __builtin_bit_cast(bf16x8_t, v);
}

// The k-loop.  "A side": operands whose row index lands in the accumulator registers (MFMA rows);
// "B side": operands whose row index lands on the lanes (MFMA columns).
//   acc[a*NB + b][ta][tb] += sum_k A_a[row_a][k] * B_b[row_b][k]
// Every operand tile has BA (A side) or BB (B side) rows; WA x WB wavefronts tile BA x BB.  NPH
// phases run back to back over the same accumulators with different operands (sum of products).
//
// Pipeline: a ring of STAGES LDS slabs of DEPTH k-values (DEPTH / 16 MFMA steps each).  Fragments
// of the next MFMA step are always requested one step ahead (interleaved with this step's MFMAs).  In the last step of slab t the wave
//   waits until its own loads of slab t+1 have landed (those of later slabs stay in flight) and
//   meets the other waves: slab t+1 is complete and nobody reads slab t any more,
//   so it issues the loads of slab t+STAGES into slab t's place, runs half of the step's MFMAs,
//   requests the first fragments of slab t+1 and runs the other half, which covers them.
template <class AT, class BT, int NA, int NB, int BA, int BB, int WA, int WB, int NPH, bool RAGGED_K, int STAGES = 4,
          bool SPREAD = false, bool B_FIRST = false>
struct KLoop {
    static constexpr int NW = WA * WB;
    static constexpr int DEPTH = AT::DEPTH;           // k-values per slab
    static constexpr int KSTEPS = DEPTH / 16;          // MFMA steps per slab
    // Deep B side (BD): the B tiles are twice as deep as a slab (a k-contiguous operand with 64
    // k-values per row is fetched in full 128-byte lines; with 32 every request is half a line and
    // costs the address unit a whole one).  B tile U serves slabs 2U and 2U+1 from a ring of its
    // own behind the A ring; it is loaded in two halves (KcTile::load_half_one), one per slab
    // period, so that a wave issues the same number of loads in every period: the period that
    // fills the A slab of slab w also fetches half (w+1) % 2 of B tile (w+1) / 2.  Row kernels only:
    // no ragged contraction, an even number of slabs per phase, spread loads.
    static constexpr bool BD = BT::DEPTH == 2 * AT::DEPTH;
    static_assert((AT::DEPTH == BT::DEPTH || BD) && KSTEPS >= 2 && KSTEPS % 2 == 0, "slab depth");
    static_assert(!BD || (!RAGGED_K && SPREAD && STAGES >= 3), "deep B side: row kernels");
    static constexpr int TA = BA / WA / 32, TB = BB / WB / 32;
    static constexpr int A_STAGE = NA * AT::BYTES, B_STAGE = NB * BT::BYTES;
    static constexpr int STAGE_BYTES = BD ? A_STAGE : A_STAGE + B_STAGE;      // stride of the (A) ring
    static constexpr int SB = (STAGES + 3) / 2;        // B ring depth (BD): tile U - SB is dead when tile U's first half is issued
    static constexpr int B_RING = STAGES * A_STAGE;    // offset of the B ring (BD)
    static constexpr int LDS_BYTES = BD ? STAGES * A_STAGE + SB * B_STAGE : STAGES * STAGE_BYTES;
    template <class T, bool DEEP> struct PerWaveB { static constexpr int N = T::template per_wave<NW>(); };
    template <class T> struct PerWaveB<T, true> { static constexpr int N = T::template per_wave_half<NW>(); };
    static constexpr int LA = AT::template per_wave<NW>(), LB = PerWaveB<BT, BD>::N;
    static constexpr int LOADS = NA * LA + NB * LB;   // per wave per slab
    typedef f32x16_t Acc[NA * NB][TA][TB];

    struct Frags {
        bf16x8_t a[NA][TA], b[NB][TB];
    };

    template <class T, bool DEEP> struct LanesOfB { typedef typename T::template Lanes<NW> type; };
    template <class T> struct LanesOfB<T, true> { typedef typename T::template LanesHalf<NW> type; };
    typedef typename AT::template Lanes<NW> LanesA;
    typedef typename LanesOfB<BT, BD>::type LanesB;
    typedef typename AT::template Idx<NW> IdxA;
    typedef typename BT::template Idx<NW> IdxB;

    // Where slab t's operands sit in LDS: the A tiles, the B tiles, and the MFMA step of the B
    // tile that is the slab's first (BD: the second slab of a B tile starts at step KSTEPS).
    struct Where {
        char *a, *b;
        int kb;
    };
    static __device__ __forceinline__ Where where(char *lds, int slot, int t)
    {
        if (BD) return Where{lds + slot * A_STAGE, lds + B_RING + ((t >> 1) % SB) * B_STAGE, (t & 1) * KSTEPS};
        return Where{lds + slot * STAGE_BYTES, lds + slot * STAGE_BYTES + A_STAGE, 0};
    }
    // BD: the B loads of the period that fills slab w's A tiles: half (w+1) % 2 of B tile (w+1) / 2; past the last
    // tile the last tile's first half again (same bytes to the same place), so that every period has LOADS loads.
    struct BWindow {
        char *tile;
        int k0, half, q;
    };
    static __device__ __forceinline__ BWindow b_window(char *lds, int w, int steps_per_phase, int n)
    {
        const int tiles = n >> 1;
        const int u = min((w + 1) >> 1, tiles - 1);
        const int ph = (NPH == 1) ? 0 : (2 * u >= steps_per_phase ? 1 : 0);
        return BWindow{lds + B_RING + (u % SB) * B_STAGE, (u - ph * (steps_per_phase >> 1)) * BT::DEPTH, (w + 1) & 1,
                       (NPH == 1 || ph == 0) ? 0 : NPH - 1};
    }
    struct Lookups {                                    // per-slab row lookups of gathered k-strided operands
        IdxA a[NA];
        IdxB b[NB];
    };

    static __device__ __forceinline__ void prepare(LanesA (&PA)[NPH][NA], LanesB (&PB)[NPH][NB], const Operand (&A)[NPH][NA],
                                                   const Operand (&B)[NPH][NB], int wave, int lane)
    {
#pragma unroll
        for (int ph = 0; ph < NPH; ++ph) {
#pragma unroll
            for (int a = 0; a < NA; ++a) PA[ph][a] = AT::template prepare<NW>(A[ph][a], wave, lane);
#pragma unroll
            for (int b = 0; b < NB; ++b) {
                if constexpr (BD) PB[ph][b] = BT::template prepare_half<NW>(B[ph][b], wave, lane);
                else PB[ph][b] = BT::template prepare<NW>(B[ph][b], wave, lane);
            }
        }
    }

    // Scalar row lookups of gathered k-strided operands for slab t (no-ops otherwise); to be called
    // before issue() of the same slab, early enough for the values to have arrived.
    static __device__ __forceinline__ void fetch(Lookups &lk, const LanesA (&PA)[NPH][NA], const LanesB (&PB)[NPH][NB], int t,
                                                 int steps_per_phase, int k_last, int wave)
    {
        const int ph = (NPH == 1) ? 0 : (t >= steps_per_phase ? 1 : 0);
        const int k0 = (t - ph * steps_per_phase) * DEPTH;
        if (NPH == 1 || ph == 0) {
#pragma unroll
            for (int a = 0; a < NA; ++a) AT::template fetch<NW>(lk.a[a], PA[0][a], k0, k_last, wave);
            if constexpr (!BD) {
#pragma unroll
                for (int b = 0; b < NB; ++b) BT::template fetch<NW>(lk.b[b], PB[0][b], k0, k_last, wave);
            }
        } else {
#pragma unroll
            for (int a = 0; a < NA; ++a) AT::template fetch<NW>(lk.a[a], PA[NPH - 1][a], k0, k_last, wave);
            if constexpr (!BD) {
#pragma unroll
                for (int b = 0; b < NB; ++b) BT::template fetch<NW>(lk.b[b], PB[NPH - 1][b], k0, k_last, wave);
            }
        }
    }

    // All loads of the period that fills slab t's A tiles (ring slot at `stage`), in one burst.
    static __device__ __forceinline__ void issue(char *stage, const LanesA (&PA)[NPH][NA], const LanesB (&PB)[NPH][NB],
                                                 const Lookups &lk, int t, int steps_per_phase, int k_last, int wave, int lane)
    {
        const int ph = (NPH == 1) ? 0 : (t >= steps_per_phase ? 1 : 0);
        const int k0 = (t - ph * steps_per_phase) * DEPTH;
        if constexpr (!BD) {
            if (NPH == 1 || ph == 0) {
#pragma unroll
                for (int a = 0; a < NA; ++a) AT::template load<NW>(stage + a * AT::BYTES, PA[0][a], lk.a[a], k0, k_last, wave, lane);
#pragma unroll
                for (int b = 0; b < NB; ++b)
                    BT::template load<NW>(stage + NA * AT::BYTES + b * BT::BYTES, PB[0][b], lk.b[b], k0, k_last, wave, lane);
            } else {
#pragma unroll
                for (int a = 0; a < NA; ++a)
                    AT::template load<NW>(stage + a * AT::BYTES, PA[NPH - 1][a], lk.a[a], k0, k_last, wave, lane);
#pragma unroll
                for (int b = 0; b < NB; ++b)
                    BT::template load<NW>(stage + NA * AT::BYTES + b * BT::BYTES, PB[NPH - 1][b], lk.b[b], k0, k_last, wave, lane);
            }
        }
    }

    static __device__ __forceinline__ void read_frags(Frags &f, const Where &at, int kk, int wa, int wb, int lane)
    {
#pragma unroll
        for (int a = 0; a < NA; ++a)
#pragma unroll
            for (int t = 0; t < TA; ++t) f.a[a][t] = AT::frag(at.a + a * AT::BYTES, wa * (BA / WA) + t * 32, kk, lane);
#pragma unroll
        for (int b = 0; b < NB; ++b)
#pragma unroll
            for (int t = 0; t < TB; ++t)
                f.b[b][t] = BT::frag(at.b + b * BT::BYTES, wb * (BB / WB) + t * 32, at.kb + kk, lane);
    }

    static __device__ __forceinline__ void mask_frags(Frags &f, int k_first, int k_valid)
    {
#pragma unroll
        for (int a = 0; a < NA; ++a)
#pragma unroll
            for (int t = 0; t < TA; ++t) f.a[a][t] = mask_frag(f.a[a][t], k_first, k_valid);
#pragma unroll
        for (int b = 0; b < NB; ++b)
#pragma unroll
            for (int t = 0; t < TB; ++t) f.b[b][t] = mask_frag(f.b[b][t], k_first, k_valid);
    }

    // Load number j (0 .. LOADS-1) of this wave's share of slab t: A-side operands first, or, with
    // B_FIRST, last (an operand gathered through per-slab row lookups belongs in the later part of
    // the window, where its lookups have had time to arrive).
    // stage: the ring slot of slab t's A tiles; lds: the ring's base; n: slabs of the whole loop (BD only).
    template <bool STEADY = false>
    static __device__ __forceinline__ void issue_one(char *stage, const LanesA (&PA)[NPH][NA], const LanesB (&PB)[NPH][NB],
                                                     const Lookups &lk, int t, int steps_per_phase, int k_last, int wave, int lane, int j,
                                                     char *lds = nullptr, int n = 0)
    {
        const int ph = (NPH == 1) ? 0 : (t >= steps_per_phase ? 1 : 0);
        const int k0 = (t - ph * steps_per_phase) * DEPTH;
        const int q = (NPH == 1 || ph == 0) ? 0 : NPH - 1;
        const bool a_side = B_FIRST ? j >= NB * LB : j < NA * LA;
        if (a_side) {
            const int ja = B_FIRST ? j - NB * LB : j, a = ja / LA;
            AT::template load_one<NW, STEADY>(stage + a * AT::BYTES, PA[q][a], lk.a[a], k0, k_last, wave, lane, ja % LA);
        } else {
            const int jb = B_FIRST ? j : j - NA * LA, b = jb / LB;
            if constexpr (BD) {
                const BWindow bw = b_window(lds, t, steps_per_phase, n);
                BT::template load_half_one<NW>(bw.tile + b * BT::BYTES, PB[bw.q][b], bw.k0, wave, bw.half, jb % LB);
            } else {
                BT::template load_one<NW, STEADY>(stage + NA * AT::BYTES + b * BT::BYTES, PB[q][b], lk.b[b], k0, k_last, wave, lane, jb % LB);
            }
        }
    }

    // Fragment number j (0 .. N_FRAGS-1) of MFMA step kk: A side first.
    static constexpr int N_FRAGS = NA * TA + NB * TB;
    static __device__ __forceinline__ void read_frag_one(Frags &f, const Where &at, int kk, int wa, int wb, int lane, int j)
    {
        if (j < NA * TA) {
            const int a = j / TA, t = j % TA;
            f.a[a][t] = AT::frag(at.a + a * AT::BYTES, wa * (BA / WA) + t * 32, kk, lane);
        } else {
            const int b = (j - NA * TA) / TB, t = (j - NA * TA) % TB;
            f.b[b][t] = BT::frag(at.b + b * BT::BYTES, wb * (BB / WB) + t * 32, at.kb + kk, lane);
        }
    }

    // MFMAs number lo .. hi-1 of the NA*NB*TA*TB of one k16 step (all of them: 0 .. N_MFMA)
    static constexpr int N_MFMA = NA * NB * TA * TB;
    template <int LO, int HI>
    static __device__ __forceinline__ void mfma_range(Acc &acc, const Frags &f)
    {
#pragma unroll
        for (int a = 0; a < NA; ++a)
#pragma unroll
            for (int b = 0; b < NB; ++b)
#pragma unroll
                for (int ta = 0; ta < TA; ++ta)
#pragma unroll
                    for (int tb = 0; tb < TB; ++tb) {
                        const int idx = ((a * NB + b) * TA + ta) * TB + tb;
                        if (idx >= LO && idx < HI)
                            acc[a * NB + b][ta][tb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(
                                f.a[a][ta], f.b[b][tb], acc[a * NB + b][ta][tb], 0, 0, 0);
                    }
    }
    static __device__ __forceinline__ void mfma_all(Acc &acc, const Frags &f) { mfma_range<0, N_MFMA>(acc, f); }

    static __device__ __forceinline__ void mfma_one(Acc &acc, const Frags &f, int idx)
    {
        const int tb = idx % TB, ta = (idx / TB) % TA, ab = idx / (TA * TB);
        acc[ab][ta][tb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f.a[ab / NB][ta], f.b[ab % NB][tb], acc[ab][ta][tb], 0, 0, 0);
    }

    // Spread loads (SPREAD): a slab's loads go out one by one between the MFMAs of a slab period
    // instead of in one burst.  The window of slab t+STAGES's loads runs from the last step of
    // slab t (its place in the ring is free after that step's barrier) through steps
    // 0 .. KSTEPS-2 of slab t+1; load j goes after MFMA number (2j+1) * WINDOW / (2 * LOADS).
    static constexpr int WINDOW = KSTEPS * N_MFMA;
    static constexpr int load_slot(int j) { return (2 * j + 1) * WINDOW / (2 * LOADS); }

    // One MFMA step in program order: MFMA, then a share of the next step's fragment reads
    // (all of them within the first three quarters of the step, so that the last have returned
    // when the step ends), then the loads whose window position falls behind this MFMA.
    // part = 0 for the last step of a slab, s + 1 for step s < KSTEPS - 1.
    // ALWAYS: the loads are issued unconditionally (steady state); otherwise if do_load.
    template <bool ALWAYS, class LoadFn>
    static __device__ __forceinline__ void step_spread(Acc &acc, const Frags &fc, Frags &fn, const Where &rd_stage, int rd_kk, int wa,
                                                       int wb, int lane, int part, bool do_load, const LoadFn &load_j)
    {
        constexpr int SPAN = N_MFMA >= 4 ? N_MFMA - N_MFMA / 4 : N_MFMA;
#pragma unroll
        for (int m = 0; m < N_MFMA; ++m) {
            mfma_one(acc, fc, m);
#pragma unroll
            for (int j = 0; j < N_FRAGS; ++j)
                if (j * SPAN / N_FRAGS == m) read_frag_one(fn, rd_stage, rd_kk, wa, wb, lane, j);
#pragma unroll
            for (int j = 0; j < LOADS; ++j)
                if (load_slot(j) == part * N_MFMA + m) {
                    if (ALWAYS || do_load) load_j(j);
                }
            __builtin_amdgcn_sched_barrier(0);
        }
    }

    // Scheduling pattern for a block of "all fragment reads of the next step, all MFMAs of this
    // step" placed in front of it in program order: one MFMA, then a share of the LDS reads, and
    // so on, so that the reads issue in the shadow of the MFMAs instead of ahead of them
    // (measured: 1.7 % on the row-tiled kernels).
    static __device__ __forceinline__ void interleave_reads_with_mfmas()
    {
        constexpr int N_READS = NA * TA * AT::READS + NB * TB * BT::READS;
        constexpr int PER = (N_READS + N_MFMA - 1) / N_MFMA;
#pragma unroll
        for (int i = 0; i < N_MFMA; ++i) {
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);     // one MFMA
            __builtin_amdgcn_sched_group_barrier(0x100, PER, 0);   // PER LDS reads
        }
    }

    // One trip of the steady state: slabs t .. t+STAGES-1 in ring slots 1, 2, .., 0 (t % STAGES == 1).
    template <class Slab, int U>
    static __device__ __forceinline__ void steady_trip(const Slab &slab, int t, std::integral_constant<int, U>)
    {
        if constexpr (U < STAGES) {
            slab(std::true_type{}, std::integral_constant<int, (1 + U) % STAGES>{}, t + U);
            steady_trip(slab, t, std::integral_constant<int, U + 1>{});
        }
    }

    // k extent per phase = steps_per_phase * DEPTH; k_valid (<= that) is the ragged contraction length.
    static __device__ __forceinline__ void run(Acc &acc, const Operand (&A)[NPH][NA], const Operand (&B)[NPH][NB],
                                               int steps_per_phase, int k_valid, char *lds, int tid)
    {
        const int lane = tid & 63;
        const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
        const int wa = wave / WB, wb = wave % WB;
        const int n = steps_per_phase * NPH;
        const int k_last = k_valid - 1;
        if (n <= 0) return;
        LanesA PA[NPH][NA];
        LanesB PB[NPH][NB];
        prepare(PA, PB, A, B, wave, lane);
        Lookups lk;
        Frags f[2];
        if constexpr (BD) {
            // the first half of B tile 0 belongs to no period of the loop: it goes first
#pragma unroll
            for (int j = 0; j < LOADS; ++j)
                if ((B_FIRST ? j < NB * LB : j >= NA * LA)) issue_one(lds, PA, PB, lk, -1, steps_per_phase, k_last, wave, lane, j, lds, n);
#pragma unroll
            for (int i = 0; i < STAGES; ++i)
                if (i < n) {
#pragma unroll
                    for (int j = 0; j < LOADS; ++j) issue_one(lds + i * STAGE_BYTES, PA, PB, lk, i, steps_per_phase, k_last, wave, lane, j, lds, n);
                }
        } else {
#pragma unroll
            for (int i = 0; i < STAGES; ++i)
                if (i < n) {
                    fetch(lk, PA, PB, i, steps_per_phase, k_last, wave);
                    issue(lds + i * STAGE_BYTES, PA, PB, lk, i, steps_per_phase, k_last, wave, lane);
                }
        }
        wait_younger(n - 1);
        __builtin_amdgcn_s_barrier();
        __builtin_amdgcn_sched_barrier(0);
        read_frags(f[0], where(lds, 0, 0), 0, wa, wb, lane);
        int slot = 0;
        if constexpr (SPREAD) {
            // Copies of the slab iteration: the steady state, where both load windows are live, the
            // loads carry no branch (measured: the branches alone cost 5 %), no k-row needs clamping
            // and the ring slot is a compile-time constant (LDS addresses become immediates, operand
            // addresses a uniform base plus a per-lane constant: the steady state spends no vector
            // instruction on addresses) - one copy per ring slot, run STAGES slabs per trip - and the
            // general one (ring slot in a register) for the first slab and the last few.
            char *prv = lds;
            auto slab = [&](auto steady, auto slot_c, int t) __attribute__((always_inline)) {
                constexpr bool SS = decltype(steady)::value;
                constexpr int SLOT = decltype(slot_c)::value;          // -1: the ring slot is the variable `slot`
                const bool ls = SS || (t >= 1 && t - 1 + STAGES < n), ll = SS || t + STAGES < n;
                char *cur, *before;
                Where cur_at, nxt_at;
                if (SLOT >= 0) {
                    cur = lds + SLOT * STAGE_BYTES;
                    cur_at = where(lds, SLOT, t);
                    nxt_at = where(lds, (SLOT + 1) % STAGES, t + 1);
                    before = lds + ((SLOT + STAGES - 1) % STAGES) * STAGE_BYTES;
                } else {
                    cur = lds + slot * STAGE_BYTES;
                    cur_at = where(lds, slot, t);
                    slot = (slot == STAGES - 1) ? 0 : slot + 1;
                    nxt_at = where(lds, slot, t + 1);
                    before = prv;
                }
                const bool tail = !SS && RAGGED_K && (t + 1) * DEPTH > k_valid;
                const int kf = t * DEPTH + (lane >> 5) * 8;
                // steps 0 .. KSTEPS-2: the rest of the loads of slab t-1+STAGES, into slab t-1's place
                auto load_prev = [&](int j) __attribute__((always_inline)) { issue_one<SS>(before, PA, PB, lk, t - 1 + STAGES, steps_per_phase, k_last, wave, lane, j, lds, n); };
#pragma unroll
                for (int s = 0; s < KSTEPS - 1; ++s) {
                    __builtin_amdgcn_s_waitcnt(0xC07F);          // lgkmcnt(0): f[s & 1] is there
                    __builtin_amdgcn_sched_barrier(0);
                    if (tail) mask_frags(f[s & 1], kf + s * 16, k_valid);
                    __builtin_amdgcn_sched_barrier(0);
                    step_spread<SS>(acc, f[s & 1], f[(s + 1) & 1], cur_at, s + 1, wa, wb, lane, s + 1, ls, load_prev);
                }
                if (SS) wait_younger(STAGES);  // slab t+1 has landed; later slabs may still be in flight
                else wait_younger(n - t - 2);
                __builtin_amdgcn_s_barrier();
                __builtin_amdgcn_sched_barrier(0);
                // Row lookups of the next window, requested behind the barrier (in front of it its
                // wait for the LDS reads would wait for them too).  A gathered operand on the B
                // side has its loads in the later part of the window, a step's MFMAs from here.
                if (ll) fetch(lk, PA, PB, t + STAGES, steps_per_phase, k_last, wave);
                // last step: the first loads of slab t+STAGES, into this slab's place
                auto load_cur = [&](int j) __attribute__((always_inline)) { issue_one<SS>(cur, PA, PB, lk, t + STAGES, steps_per_phase, k_last, wave, lane, j, lds, n); };
                constexpr int L = (KSTEPS - 1) & 1;
                if (tail) mask_frags(f[L], kf + (KSTEPS - 1) * 16, k_valid);
                step_spread<SS>(acc, f[L], f[0], nxt_at, 0, wa, wb, lane, 0, ll, load_cur);
                if (SLOT < 0) prv = cur;
            };
            constexpr auto dyn = std::integral_constant<int, -1>{};
            slab(std::false_type{}, dyn, 0);
            int t = 1;
            // Steady trips: slab t sits in ring slot t % STAGES (t = 1 in slot 1); a trip leaves `slot`
            // and `prv` as they are.  The loads a steady slab issues are those of slabs t-1+STAGES and
            // t+STAGES, which must be whole (no clamped k-rows): the last slab of a ragged contraction
            // is left to the general copy.
            const int steady_end = n - STAGES - (RAGGED_K ? 1 : 0);
            for (; t + STAGES <= steady_end; t += STAGES) steady_trip(slab, t, std::integral_constant<int, 0>{});
            for (; t < n; ++t) slab(std::false_type{}, dyn, t);
        } else {
        for (int t = 0; t < n; ++t) {
            char *cur = lds + slot * STAGE_BYTES;
            const Where cur_at = where(lds, slot, t);
            slot = (slot == STAGES - 1) ? 0 : slot + 1;
            const Where nxt = where(lds, slot, t + 1);
            const bool tail = RAGGED_K && (t + 1) * DEPTH > k_valid;
            const int kf = t * DEPTH + (lane >> 5) * 8;
#pragma unroll
            for (int s = 0; s < KSTEPS - 1; ++s) {
                // f[s & 1] was requested before the previous MFMA block: it is there by now.
                // Waiting for it here, before the next requests go out, lets the MFMAs below
                // start at once instead of waiting for the requests issued just above them.
                __builtin_amdgcn_s_waitcnt(0xC07F);          // lgkmcnt(0)
                __builtin_amdgcn_sched_barrier(0);
                if (tail) mask_frags(f[s & 1], kf + s * 16, k_valid);
                __builtin_amdgcn_sched_barrier(0);
                read_frags(f[(s + 1) & 1], cur_at, s + 1, wa, wb, lane);
                mfma_all(acc, f[s & 1]);
                interleave_reads_with_mfmas();
                __builtin_amdgcn_sched_barrier(0);
            }
            wait_younger(n - t - 2);       // slab t+1 has landed; later slabs may still be in flight
            __builtin_amdgcn_s_barrier();
            __builtin_amdgcn_sched_barrier(0);
            if (t + STAGES < n) {
                fetch(lk, PA, PB, t + STAGES, steps_per_phase, k_last, wave);
                issue(cur, PA, PB, lk, t + STAGES, steps_per_phase, k_last, wave, lane);
            }
            // First half of the last step's MFMAs, then the requests for the next slab's first
            // fragments (always issued: after the last slab they fetch stale LDS that nobody
            // uses, and a request that is not conditional lets the wait in front of these
            // MFMAs count only the older requests), then the second half, which covers them.
            constexpr int L = (KSTEPS - 1) & 1;
            if (tail) mask_frags(f[L], kf + (KSTEPS - 1) * 16, k_valid);
            mfma_range<0, N_MFMA / 2>(acc, f[L]);
            __builtin_amdgcn_sched_barrier(0);
            read_frags(f[0], nxt, 0, wa, wb, lane);
            __builtin_amdgcn_sched_barrier(0);
            mfma_range<N_MFMA / 2, N_MFMA>(acc, f[L]);
            __builtin_amdgcn_sched_barrier(0);
        }
        }
    }

    // The same loop over a list of pieces of the contraction (single phase, ragged pieces): piece i
    // has its own operands and length; a slab never spans two pieces (a piece's last slab is
    // masked), and the ring keeps running across piece boundaries, so that short pieces do not
    // pay a pipeline fill and drain each.  src.piece(i, A, B, k_valid) describes piece i
    // (k_valid >= 1); n_pieces and total_slabs = sum of ceil(k_valid / DEPTH) come from the caller.
    template <class Src>
    static __device__ __forceinline__ void run_pieces(Acc &acc, const Src &src, int n_pieces, int total_slabs, char *lds, int tid)
    {
        static_assert(NPH == 1 && RAGGED_K && !BD, "pieces: one phase, ragged contraction");
        const int lane = tid & 63;
        const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
        const int wa = wave / WB, wb = wave % WB;
        const int n = total_slabs;
        if (n <= 0 || n_pieces <= 0) return;
        // cursor of the loads (runs STAGES slabs ahead) and cursor of the MFMAs
        Operand Ai[1][NA], Bi[1][NB];
        LanesA PA[1][NA];
        LanesB PB[1][NB];
        int ip = 0, it = 0, i_valid = 0, i_slabs = 0;
        src.piece(0, Ai, Bi, i_valid);
        prepare(PA, PB, Ai, Bi, wave, lane);
        i_slabs = (i_valid + DEPTH - 1) / DEPTH;
        int ct = 0, c_valid = i_valid, c_slabs = i_slabs, cp = 0;
        Lookups lk;
        auto fetch_next = [&]() { fetch(lk, PA, PB, it, i_slabs, i_valid - 1, wave); };
        auto advance_loads = [&]() {                        // the load cursor moves on by one slab
            if (++it == i_slabs && ip + 1 < n_pieces) {
                ++ip;
                it = 0;
                src.piece(ip, Ai, Bi, i_valid);
                prepare(PA, PB, Ai, Bi, wave, lane);
                i_slabs = (i_valid + DEPTH - 1) / DEPTH;
            }
        };
        auto issue_next = [&](char *stage) {
            issue(stage, PA, PB, lk, it, i_slabs, i_valid - 1, wave, lane);
            advance_loads();
        };
        Frags f[2];
#pragma unroll
        for (int i = 0; i < STAGES; ++i)
            if (i < n) {
                fetch_next();
                issue_next(lds + i * STAGE_BYTES);
            }
        wait_younger(n - 1);
        __builtin_amdgcn_s_barrier();
        __builtin_amdgcn_sched_barrier(0);
        read_frags(f[0], where(lds, 0, 0), 0, wa, wb, lane);
        int slot = 0;
        if (SPREAD) {
            // as in run(): the load cursor stays on slab t+STAGES from the last step of slab t
            // through the steps of slab t+1 and moves on behind that window's last load
            char *prv = lds;
            auto slab = [&](auto steady, int t) __attribute__((always_inline)) {
                constexpr bool SS = decltype(steady)::value;
                const bool ls = SS || (t >= 1 && t - 1 + STAGES < n), ll = SS || t + STAGES < n;
                char *cur = lds + slot * STAGE_BYTES;
                const Where cur_at = where(lds, slot, 0);
                slot = (slot == STAGES - 1) ? 0 : slot + 1;
                const Where nxt = where(lds, slot, 0);
                const bool tail = (ct + 1) * DEPTH > c_valid;
                const int kf = ct * DEPTH + (lane >> 5) * 8;
                auto load_prev = [&](int j) __attribute__((always_inline)) { issue_one(prv, PA, PB, lk, it, i_slabs, i_valid - 1, wave, lane, j); };
#pragma unroll
                for (int s = 0; s < KSTEPS - 1; ++s) {
                    __builtin_amdgcn_s_waitcnt(0xC07F);          // lgkmcnt(0)
                    __builtin_amdgcn_sched_barrier(0);
                    if (tail) mask_frags(f[s & 1], kf + s * 16, c_valid);
                    __builtin_amdgcn_sched_barrier(0);
                    step_spread<SS>(acc, f[s & 1], f[(s + 1) & 1], cur_at, s + 1, wa, wb, lane, s + 1, ls, load_prev);
                }
                if (ls) advance_loads();
                wait_younger(n - t - 2);
                __builtin_amdgcn_s_barrier();
                __builtin_amdgcn_sched_barrier(0);
                if (ll) fetch_next();
                auto load_cur = [&](int j) __attribute__((always_inline)) { issue_one(cur, PA, PB, lk, it, i_slabs, i_valid - 1, wave, lane, j); };
                constexpr int L = (KSTEPS - 1) & 1;
                if (tail) mask_frags(f[L], kf + (KSTEPS - 1) * 16, c_valid);
                step_spread<SS>(acc, f[L], f[0], nxt, 0, wa, wb, lane, 0, ll, load_cur);
                prv = cur;
                if (++ct == c_slabs && cp + 1 < n_pieces) {      // the MFMAs move on to the next piece
                    ++cp;
                    ct = 0;
                    c_valid = src.valid(cp);
                    c_slabs = (c_valid + DEPTH - 1) / DEPTH;
                }
            };
            slab(std::false_type{}, 0);
            int t = 1;
            for (; t < n - STAGES; ++t) slab(std::true_type{}, t);
            for (; t < n; ++t) slab(std::false_type{}, t);
            return;
        }
        for (int t = 0; t < n; ++t) {
            char *cur = lds + slot * STAGE_BYTES;
            const Where cur_at = where(lds, slot, 0);
            slot = (slot == STAGES - 1) ? 0 : slot + 1;
            const Where nxt = where(lds, slot, 0);
            const bool tail = (ct + 1) * DEPTH > c_valid;
            const int kf = ct * DEPTH + (lane >> 5) * 8;
#pragma unroll
            for (int s = 0; s < KSTEPS - 1; ++s) {
                __builtin_amdgcn_s_waitcnt(0xC07F);          // lgkmcnt(0)
                __builtin_amdgcn_sched_barrier(0);
                // row lookups of the slab issued below: requested a whole MFMA block ahead
                if (s == 0 && t + STAGES < n) fetch_next();
                if (tail) mask_frags(f[s & 1], kf + s * 16, c_valid);
                __builtin_amdgcn_sched_barrier(0);
                read_frags(f[(s + 1) & 1], cur_at, s + 1, wa, wb, lane);
                mfma_all(acc, f[s & 1]);
                interleave_reads_with_mfmas();
                __builtin_amdgcn_sched_barrier(0);
            }
            wait_younger(n - t - 2);
            __builtin_amdgcn_s_barrier();
            __builtin_amdgcn_sched_barrier(0);
            if (t + STAGES < n) issue_next(cur);
            constexpr int L = (KSTEPS - 1) & 1;
            if (tail) mask_frags(f[L], kf + (KSTEPS - 1) * 16, c_valid);
            mfma_range<0, N_MFMA / 2>(acc, f[L]);
            __builtin_amdgcn_sched_barrier(0);
            read_frags(f[0], nxt, 0, wa, wb, lane);
            __builtin_amdgcn_sched_barrier(0);
            mfma_range<N_MFMA / 2, N_MFMA>(acc, f[L]);
            __builtin_amdgcn_sched_barrier(0);
            if (++ct == c_slabs && cp + 1 < n_pieces) {      // the MFMAs move on to the next piece
                ++cp;
                ct = 0;
                c_valid = src.valid(cp);
                c_slabs = (c_valid + DEPTH - 1) / DEPTH;
            }
        }
    }

    // Wait until at most min(younger, STAGES-2) slabs' worth of this wave's loads are outstanding,
    // and until its LDS reads have returned.
    static __device__ __forceinline__ void wait_younger(int younger)
    {
        static_assert(STAGES >= 2 && STAGES <= 5, "ring depth");
        static_assert(3 * LOADS < 64, "vmcnt has 6 bits");
        if (STAGES >= 5 && younger >= 3) wait_vm_lgkm0<3 * LOADS>();
        else if (STAGES >= 4 && younger >= 2) wait_vm_lgkm0<2 * LOADS>();
        else if (STAGES >= 3 && younger >= 1) wait_vm_lgkm0<1 * LOADS>();
        else wait_vm_lgkm0<0>();
    }

    static __device__ __forceinline__ void zero(Acc &acc)
    {
#pragma unroll
        for (int n = 0; n < NA * NB; ++n)
#pragma unroll
            for (int ta = 0; ta < TA; ++ta)
#pragma unroll
                for (int tb = 0; tb < TB; ++tb)
#pragma unroll
                    for (int v = 0; v < 16; ++v) acc[n][ta][tb][v] = 0.0f;
    }

    // Position of accumulator element v of MFMA tile (ta, tb) inside the BA x BB tile:
    // row on the A side, row on the B side.
    static __device__ __forceinline__ int a_row(int wave, int lane, int ta, int v)
    {
        return (wave / WB) * (BA / WA) + ta * 32 + 8 * (v >> 2) + 4 * (lane >> 5) + (v & 3);
    }
    static __device__ __forceinline__ int b_row(int wave, int lane, int tb) { return (wave % WB) * (BB / WB) + tb * 32 + (lane & 31); }
};

}  // namespace relibra
