// Fused base projection + grouped expand for small batches (row tiles of 64; which shapes take
// this kernel and which the tiled one, launch_fused_gemm decides; Eq. "pertok"):
//
//     h[perm[p]][:] = x[perm[p]] W  +  t_p B_{c(p)}
//
// With so few rows the step is bound by reading W (and the touched B_c) once from HBM,
// so the kernel is built around keeping many bytes in flight per compute unit and around
// spending few cache-line accesses per byte, with no workgroup barrier in the streaming loop:
//   * a workgroup owns 64 (or 32, where that is needed to occupy the chip) output columns and
//     up to 64 rows; its 8 wavefronts split the K range -- of the pieces of 64 rows of W every
//     8th one, then of the 16-row slabs of the B_c of the buckets that own rows every 8th
//     one -- and add their partial tiles in LDS at the end, in wavefront order, so the result
//     does not depend on timing and needs no scratch memory or atomics;
//   * every wavefront streams its 16 x 64 slabs of W straight from HBM into a private ring of
//     LDS slots (global_load_lds_dwordx4), 4 slabs ahead of the one it multiplies; the LDS
//     transpose read turns the K-major slab into the MFMA operand;
//   * the x operand of 64 k travels the same way, as whole 128-byte lines of 8 rows per
//     load instruction, into a private staging tile, one unit ahead; it is moved to registers
//     at the start of its unit, which frees the staging tile for the next one;
//   * chunks that must read as zero (k past d_in, padding of a wavefront's list) come from an
//     all-zero page, so every step issues the same number of loads and the explicit vmcnt
//     waits are compile-time constants;
//   * the grouped expand follows as a phase of its own: a few trips to memory, each for four
//     slabs of B and the matching columns of t per wavefront (as units of the streaming loop
//     they cost a full memory latency each: 46 us against 38 us at 64 tokens, 14 adapters of
//     rank 64).
#include <type_traits>

#include "common.h"
#include "lds_dma.h"

namespace molora {

namespace {

constexpr int kSbWaves = 8;                    // wavefronts per workgroup = K splits (4 in one form of the shrink)
constexpr int kSbRing = 5;                     // slab slots per wavefront
constexpr int kSbStage = 64 * 128;             // x / t staging tile: 64 rows x 64 k

// TN = 32-column blocks per workgroup: 2 (64 columns, 128-byte pieces of W rows) where the
// column groups alone fill the chip, 1 (32 columns) where they would leave it idle.
template <int TN, int NWV = kSbWaves>
struct SbGeom {
    static constexpr int COLS = 32 * TN;                // output columns per workgroup
    static constexpr int SLOT = 16 * COLS * 2;          // one 16-k slab of W
    static constexpr int NR = SLOT / 1024;              // load instructions per slab
    static constexpr int CPR = COLS / 8;                // 16-byte chunks per slab row
    static constexpr int RPD = 64 / CPR;                // slab rows per load instruction
    static constexpr int ROW_BYTES = COLS * 4 + 16;     // partial tile row in LDS (+16: bank shift)
    static constexpr int WAVE_LDS = kSbRing * SLOT + kSbStage;  // per wavefront; partial tile reuses it
    static constexpr size_t LDS_BYTES = (size_t)NWV * WAVE_LDS + (8 * 64 + 4) * sizeof(int32_t);
    static_assert(64 * ROW_BYTES <= WAVE_LDS, "partial tile fits the wavefront's region");
    // 32-byte chunk position inside a slab row that holds column chunk cc of k-row `row`
    // (keeps the transpose reads of the four 16-lane groups on different banks)
    __device__ static __forceinline__ int swz32(int cc, int row) {
        if constexpr (TN == 2) return cc ^ (row & 3);
        return cc ^ ((row >> 3) & 1);
    }
};

// four values of a row of the low-rank intermediate, scaled by the token's mixture weight, as
// t = hi + lo with hi = bf16(t), lo = bf16(t - hi); row of t = [hi | lo], R values each
__device__ __forceinline__ void store_t_hi_lo(uint16_t *row_dst, int R, int col, f32x4 sum, float wj) {
    u32x2 hi2 = {0, 0}, lo2 = {0, 0};
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const float tv = sum[i] * wj;
        const uint32_t hi = f32_to_bf16_bits(tv);
        const uint32_t lo = f32_to_bf16_bits(tv - bf16_bits_to_f32(hi));
        hi2[i >> 1] |= hi << (16 * (i & 1));
        lo2[i >> 1] |= lo << (16 * (i & 1));
    }
    *(u32x2 *)(row_dst + col) = hi2;
    *(u32x2 *)(row_dst + R + col) = lo2;
}

// one unit of a wavefront's work list: 64 k-rows of W, four steps of 16 k
struct Unit {
    bool real;  // false: past the end of the list, nothing (zeros)
    int k0;     // first k
    // fast: all 64 rows lie inside W and follow one another in memory from `base`; the loads
    // are a scalar base plus a fixed per-lane offset, nothing to decide
    bool fast;
    const unsigned char *base;
};

// SHRINK = false: the fused GEMM above (grid: column groups x row tiles of 64 sorted rows; a
//                 batch of more than 64 rows re-reads W once per row tile, from L2).
// SHRINK = true:  the shrink step t_p = x[perm[p]] A_c for the rows of bucket c = wg.y
//                 (workgroup = column group of the rank x 64-row tile of a bucket; which tile a
//                 workgroup is, small_batch_kernel finds from offsets); W is
//                 A, d_out is rank, there are no expand units and the result goes to t_out as
//                 [hi | lo] bf16 halves.  With ksplit > 1 the K range is cut into ksplit
//                 slices, one workgroup each (wg.z = tile * ksplit + slice): a batch of
//                 a few dozen tokens has too few (bucket, tile) pairs to draw the touched A_c
//                 from HBM at speed, a workgroup draws ~50 GB/s.  A slice's sums then go, in
//                 fp32, to plane `slice` of h [ksplit][N][R]; shrink_reduce_kernel adds the
//                 planes in ascending order (a fixed order: no atomics) and writes t_out.
//
// The body is a device function of the workgroup's place in its grid (wg) so that two grids
// can share one launch (shrink_base_small_kernel below).  GEMM modes (SHRINK = false, a batch
// of one row tile): kSbBaseOnly leaves the expand phase out and reads neither offsets nor perm
// (h = x W: nothing the dispatch step produces is needed); kSbExpandOnly leaves the W stream
// out and ADDS the expand to h (h += t B_c).  One after the other they give what mode 0 gives
// up to the order of the fp32 additions.  kSbBasePacked is kSbBaseOnly with W stored slab by
// slab (16 k-rows) and, inside a slab, column group by column group (see pack_w_kernel below):
// a wavefront's slab is then one contiguous piece instead of sixteen cache lines d_out elements
// apart, and the workgroups, which advance through W together, read one contiguous region at
// any time (27.0 against 31.4 us at 64 x 4096 -> 12288; column groups as whole [d_in][COLS]
// matrices, i.e. one contiguous stream per workgroup but 192 of them, gave 29.4 us).
struct SbBlock {
    int x, y, z;  // the workgroup's index in its grid
    int gy;       // the grid's extent in y
};
constexpr int kSbBaseOnly = 1, kSbExpandOnly = 2, kSbBasePacked = 3, kSbExpandPacked = 4;

template <int TM, int TN, bool SHRINK, int MODE = 0, int NWV = kSbWaves>  // TM: 32-row blocks, 1 (N <= 32) or 2
__device__ __forceinline__ void small_batch_body(
    const uint16_t *__restrict__ x, const uint16_t *__restrict__ W, const uint16_t *__restrict__ B,
    const uint16_t *__restrict__ t2, const int32_t *__restrict__ offsets,
    const int32_t *__restrict__ perm, float *__restrict__ h, uint16_t *__restrict__ t_out, int N,
    int d_in, int d_out, int C, int rank, Mix mix, int ksplit, SortArgs sort, SbBlock wg) {
    using Geo = SbGeom<TN, NWV>;
    constexpr int kSbCols = Geo::COLS, kSbSlot = Geo::SLOT, kSbRowBytes = Geo::ROW_BYTES,
                  kSbWaveLds = Geo::WAVE_LDS;
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    int32_t *tile_perm = (int32_t *)(smem + NWV * kSbWaveLds);  // [64] token per row, -1 = none
    int32_t *tile_pos = tile_perm + 64;                              // [64] sorted position per row
    int32_t *seg_lo = tile_pos + 64;                                 // buckets that own rows, ascending:
    int32_t *seg_hi = seg_lo + 64;                                   // their sorted-position ranges
    int32_t *nseg_p = seg_hi + 64;
    int32_t *seg_ad = nseg_p + 4;  // [64][4] pool positions of the adapters of a bucket's tuple

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int n0 = wg.x * kSbCols;
    unsigned char *ring = smem + wave * kSbWaveLds;
    unsigned char *stage = ring + kSbRing * kSbSlot;
    const uint16_t *zero = (const uint16_t *)g_zero_page;

    // ---- rows of this workgroup ----
    const int R = mix.k * rank;  // width of a bucket's intermediate (k adapters side by side)
    int row_base = 0, nrows = N, bucket = 0;
    // SHRINK with the dispatch step inside (sort.r given; N <= 64, so the targets of the whole
    // batch are one wavefront of keys): every wavefront derives the rows of its bucket from r
    // itself -- the tokens with that target in ascending order, which is the stable order of
    // the dispatch step -- instead of reading offsets and perm, and the workgroups of column
    // group 0 write offsets and perm for the step that follows (Alg. "Unified Dispatch Kernel").
    const bool sorting = SHRINK && sort.r != nullptr;
    int sort_tok = 0;  // sorting: token of row `lane` of the bucket (lanes past its rows: 0)
    if constexpr (SHRINK) {
        bucket = wg.y;
        if (sorting) {
            if (wg.z >= ksplit) return;  // a batch of one wavefront is one row tile
            int key = C + 1;  // lanes past the batch: no key at all
            if (lane < N) {
                const int c = sort.r[lane];
                key = (c >= 0 && c < C) ? c : C;  // C: no adapter
            }
            // lane j <- the j-th lane (ascending) of a ballot mask
            auto nth_lane = [&](uint64_t m) {
                int tok = 0, cnt = 0;
                while (m) {  // wave-uniform, at most 64 rounds
                    if (cnt == lane) tok = __builtin_ctzll(m);
                    ++cnt;
                    m &= m - 1;
                }
                return tok;
            };
            const uint64_t mine = __ballot(key == bucket);
            row_base = (int)__popcll(__ballot(key < bucket));  // sorted position of the bucket's first row
            nrows = (int)__popcll(mine);
            sort_tok = nth_lane(mine);
            if (wg.x == 0 && wg.z == 0 && wave == 0) {
                if (lane == 0) sort.offsets[bucket] = row_base;
                if (lane < nrows) sort.perm[row_base + lane] = sort_tok;
                if (bucket == C - 1) {  // ... and once: the end of the lists, the tokens without adapter
                    const uint64_t none = __ballot(key == C);
                    const int n_routed = (int)__popcll(__ballot(key < C));
                    const int tok = nth_lane(none);
                    if (lane == 0) sort.offsets[C] = n_routed;
                    if (lane < (int)__popcll(none)) sort.perm[n_routed + lane] = tok;
                    if (none != 0 && lane == 0 && sort.err_flag != nullptr) *sort.err_flag = 1;
                }
            }
            if (nrows <= 0) return;  // an empty bucket: its adapters are not touched
        } else {
            row_base = offsets[bucket] + 64 * (wg.z / ksplit);  // 64-row tile of the bucket
            nrows = min(64, offsets[bucket + 1] - row_base);
            if (nrows <= 0) return;  // nothing (left) in this bucket: its adapters are not touched
        }
    } else {
        row_base = wg.y * 64;  // row tile of 64 sorted positions
        nrows = min(64, N - row_base);
    }
    // A batch that fits one row tile keeps its rows in token order: x W then depends on nothing
    // the dispatch step produced, so the stream starts at once, and only the expand units (the
    // end of every wavefront's list) look up the sorted position of a row.
    const bool direct = !SHRINK && wg.gy == 1;
    // packed: the streamed matrix (W, or the stacked B of the expand alone) is stored slab by
    // slab, column group after column group; d_out % COLS == 0, and rank % 16 == 0 for B (host)
    constexpr bool packed = !SHRINK && (MODE == kSbBasePacked || MODE == kSbExpandPacked);
    constexpr bool base_only = !SHRINK && (MODE == kSbBaseOnly || MODE == kSbBasePacked);      // direct batches only (host)
    constexpr bool expand_only = !SHRINK && (MODE == kSbExpandOnly || MODE == kSbExpandPacked);  // direct batches only (host)

    // ---- this wavefront's share of W ----
    // Of the nub pieces of 64 k-rows of W (the last piece may be short) every 8th one, piece
    // 8 * u + wave.  Interleaved, so that the workgroups together sweep W from top to bottom
    // (measured 2% faster than giving every wavefront one contiguous eighth).
    const int two_r = 2 * R;
    const int nub_all = (d_in + 63) / 64;
    // K slice of this workgroup (SHRINK with ksplit > 1): pieces [u_lo, u_lo + nub)
    const int slice = SHRINK ? wg.z % ksplit : 0;
    const int per_slice = SHRINK ? (nub_all + ksplit - 1) / ksplit : nub_all;
    const int u_lo = slice * per_slice;
    const int nub = expand_only ? 0 : max(0, min(nub_all, u_lo + per_slice) - u_lo);
    const int nw = nub > wave ? (nub - wave + NWV - 1) / NWV : 0;

    // elements between consecutive k-rows of W (A); packed: inside a slab of 16 k-rows the
    // workgroup's column group is a [rows][COLS] matrix of its own
    const int pitch = SHRINK ? rank : (packed ? kSbCols : d_out);
    bool w_fast_ok = false, a_fast_ok = false;  // per-lane offsets fit 32 bits (set below)
    // wave-uniform by construction; says so to the compiler, which must keep them in scalar
    // registers for the load instruction
    auto uniform_ptr = [](const void *ptr) {
        const uint64_t v = (uint64_t)(uintptr_t)ptr;
        const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)v);
        const uint32_t hi = __builtin_amdgcn_readfirstlane((uint32_t)(v >> 32));
        return (const unsigned char *)(uintptr_t)(((uint64_t)hi << 32) | lo);
    };
    auto unit_of = [&](int u) {  // u-th unit of this wavefront
        Unit un;
        un.real = u < nw;
        un.k0 = un.real ? (u_lo + u * NWV + wave) * 64 : 0;
        un.fast = un.real && un.k0 + 64 <= d_in;
        if constexpr (packed)  // slab k / 16 starts at k * d_out; in it, group after group
            un.base = (const unsigned char *)(W + (int64_t)un.k0 * d_out + (int64_t)wg.x * 16 * kSbCols);
        else
            un.base = (const unsigned char *)(W + (int64_t)un.k0 * pitch);
        return un;
    };

    // ---- slab loads: 1 KB per instruction = RPD k-rows x (2 * COLS) bytes ----
    // lane -> row lane / CPR of the instruction's rows, 16-byte position lane % CPR of the slab
    // row, which holds the column chunk given by the swizzle.  A row past the end of its matrix
    // reads zeros instead.
    const int w_rr = lane / Geo::CPR, w_pos = lane % Geo::CPR;
    auto w_col_of = [&](int r) {  // columns of this lane in load r of a slab
        const int row = r * Geo::RPD + w_rr;
        const int u16 = (Geo::swz32(w_pos >> 1, row) << 1) | (w_pos & 1);
        if constexpr (packed) return u16 * 8;  // inside the group
        return min(n0 + u16 * 8, d_out - 8);  // columns past d_out: clamped, never stored
    };
    // SHRINK: the "matrix" is the tuple's A side by side, [d_in][R]; a group of 8 columns lies
    // inside one adapter, whose rows are rank elements apart
    const uint16_t *w_lane[Geo::NR];
    uint32_t w_off[Geo::NR];  // fast units: byte offset of this lane from the unit's base + row term
    int w_colv[Geo::NR];
    {
        bool ok = true;  // ... which must fit 32 bits in every lane for the fast form
#pragma unroll
        for (int r = 0; r < Geo::NR; ++r) {
            const int col = w_col_of(r);
            w_colv[r] = col;
            const int row = r * Geo::RPD + w_rr;
            w_lane[r] = SHRINK
                ? W + ((int64_t)mix_adapter(mix, bucket, col / rank) * d_in + row) * rank + col % rank
                : W + (int64_t)row * pitch + col;
            // the same lane offset serves W and B in the GEMM (both have d_out columns)
            const int64_t off = ((const unsigned char *)w_lane[r] - (const unsigned char *)W) -
                                (int64_t)r * Geo::RPD * pitch * 2;
            w_off[r] = (uint32_t)off;
            ok = ok && (off >> 32) == 0;
        }
        w_fast_ok = __all(ok) != 0;
    }
    auto issue_slab = [&](const Unit &un, int j, unsigned char *slot) {  // step j of the unit
#pragma unroll
        for (int r = 0; r < Geo::NR; ++r) {
            if (un.fast && w_fast_ok) {
                // packed: the unit's four slabs are full, 16 * d_out elements apart
                const int64_t step = packed ? (int64_t)j * 16 * (d_out * 2) + (int64_t)(r * Geo::RPD) * (pitch * 2)
                                            : (int64_t)(j * 16 + r * Geo::RPD) * (pitch * 2);
                load_to_lds16(un.base + step, w_off[r], slot + r * 1024);
                continue;
            }
            // d_in is a multiple of 8 and so is RPD: rows of a load leave the matrix together
            const int kk = un.k0 + j * 16 + r * Geo::RPD + w_rr;  // this lane's row
            const uint16_t *src = zero;
            if (un.real && kk < d_in) {
                if constexpr (packed) {  // the last slab of W may hold 8 rows only
                    const int ks = un.k0 + j * 16;
                    src = W + (int64_t)ks * d_out + (int64_t)wg.x * min(16, d_in - ks) * kSbCols +
                          (r * Geo::RPD + w_rr) * pitch + w_colv[r];
                } else
                    src = w_lane[r] + (int64_t)(un.k0 + j * 16) * pitch;
            }
            load_to_lds16_ptr(src, slot + r * 1024);
        }
    };

    // ---- x loads: 8 rows x 128 bytes (64 k) per instruction, 4 * TM instructions a unit ----
    // lane -> row i*8 + lane/8, 16-byte position lane%8 of the staged row, which holds the
    // 8-k chunk (position ^ swizzle(row)); the operand read below undoes the swizzle.
    const int a_sub = lane >> 3, a_pos = lane & 7;
    const uint16_t *a_xrow[4 * TM];
    int a_ch8[4 * TM];
    uint32_t a_off[4 * TM];  // byte offset of this lane's chunk from x + k0
    {
        bool ok = true;
#pragma unroll
        for (int i = 0; i < 4 * TM; ++i) {
            const int row = min(i * 8 + a_sub, nrows - 1);  // rows past the end repeat the last one; never stored
            const int tok = sorting ? __shfl(sort_tok, row, 64) : (direct ? row : perm[row_base + row]);
            a_ch8[i] = (a_pos ^ (((i * 8 + a_sub) ^ ((i * 8 + a_sub) >> 3)) & 7)) * 8;
            a_xrow[i] = x + (int64_t)tok * d_in + a_ch8[i];
            const int64_t off = (const unsigned char *)a_xrow[i] - (const unsigned char *)x;
            a_off[i] = (uint32_t)off;
            ok = ok && (off >> 32) == 0;
        }
        a_fast_ok = __all(ok) != 0;
    }
    auto issue_stage = [&](const Unit &un) {
        if (un.fast && a_fast_ok) {  // 64 k of x, all inside d_in
            const unsigned char *xb = (const unsigned char *)(x + un.k0);
#pragma unroll
            for (int i = 0; i < 4 * TM; ++i) load_to_lds16(xb, a_off[i], stage + i * 1024);
            return;
        }
#pragma unroll
        for (int i = 0; i < 4 * TM; ++i) {
            const uint16_t *src = (un.real && un.k0 + a_ch8[i] < d_in) ? a_xrow[i] + un.k0 : zero;
            load_to_lds16_ptr(src, stage + i * 1024);
        }
    };

    // expand alone: what h holds (the rows' x W) is fetched now and added at the end; in token
    // order the row of h is the tile row, so nothing has to be looked up first
    constexpr int kOutIters = (TM * 32 * (kSbCols / 4) + NWV * 64 - 1) / (NWV * 64);
    f32x4 h_old[kOutIters];
    if constexpr (expand_only) {
#pragma unroll
        for (int j = 0; j < kOutIters; ++j) {
            const int it = tid + j * NWV * 64;
            const int row = it / (kSbCols / 4), col = n0 + (it % (kSbCols / 4)) * 4;
            const bool ok = it < TM * 32 * (kSbCols / 4) && row < nrows && col < d_out;
            // (rows and columns past the end: read again from the first element, never used)
            h_old[j] = *(const f32x4 *)(h + (ok ? (int64_t)row * d_out + col : 0));
        }
    }

    f32x16 acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

    // operand reads.  x / t: lane -> row lane%32 (+32), k-group lane/32.  Slab: lane -> column
    // 16*(blk&1) + a16 of a 32-column block, k-rows (blk>>1)*8 + 0..7, through the transpose read.
    const int kg = lane >> 5, m_lo = lane & 31;
    const int blk = lane >> 4, a16 = lane & 15;
    const int b_kr0 = (blk >> 1) * 8 + (a16 >> 2);
    const int b_in = (a16 & 3) * 8;
    auto load_a_frag = [&](int j, int tm) -> bf16x8 {
        const int row = tm * 32 + m_lo;
        const int sw = (row ^ (row >> 3)) & 7;
        return *(const bf16x8 *)(stage + row * 128 + (((j * 2 + kg) ^ sw) << 4));
    };
    auto load_b_frag = [&](const unsigned char *slot, int tn) -> bf16x8 {
        const int cc = tn * 2 + (blk & 1);  // 32-byte chunk of the slab row
        const unsigned char *p = slot + b_kr0 * (kSbCols * 2) + (Geo::swz32(cc, b_kr0) << 5) + b_in;
        const i16x4 lo = lds_read_tr16((const MOLORA_LDS void *)p);
        const i16x4 hi = lds_read_tr16((const MOLORA_LDS void *)(p + 4 * kSbCols * 2));
        const i16x8 b8 = {lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
        return __builtin_bit_cast(bf16x8, b8);
    };

    // ---- streaming loop over W ----
    // Step s = 4 * unit + j.  Iteration s issues slab s + 4, and at j == 0 (after the staged
    // operand of its own unit has been moved to registers) the staged operand of the next
    // unit.  Loads return in order, so "at most n outstanding", n = the number of loads issued
    // after the needed one, is exactly "the needed one has landed":
    //   staged operand of the unit, at j == 0: the three slabs issued since         -> 3 NR
    //   slab s at j > 0: 4 slabs and one staged operand issued since                -> 4 NR + XD
    //   slab s at j == 0: older than the staged operand, already there.
    // Nothing here depends on the dispatch step's output (in token order not even the rows),
    // so the stream starts before the tables below are built.
    constexpr int XD = 4 * TM;
    constexpr int AHEAD = kSbRing - 1;
    static_assert(AHEAD == 4, "the wait counts above assume slabs are issued 4 steps ahead");
    int uw_i = 0, ux_i = 0;  // next unit of the slab stream, of the staged-operand stream
    Unit uw = unit_of(0);
    int qw = 0;  // step index of the next slab to issue; its unit is uw, its step qw % 4
    auto next_slab = [&]() {
        if ((qw & 3) == 0) uw = unit_of(uw_i++);
        issue_slab(uw, qw & 3, ring + (qw % kSbRing) * kSbSlot);
        ++qw;
    };
    // what iterations -4 .. -1 would have issued
    next_slab();
    issue_stage(unit_of(ux_i++));
    next_slab();
    next_slab();
    next_slab();

    // ---- tables: row -> token and sorted position; the buckets that own rows, ascending ----
    if (wave == 0) {
        tile_perm[lane] = lane < nrows ? (sorting ? sort_tok : (direct ? lane : perm[row_base + lane])) : -1;
        tile_pos[lane] = direct ? 0x7fffffff : row_base + lane;
        if (direct && !base_only && lane < nrows) {
            const int tok = perm[lane];
            if ((unsigned)tok < 64u) tile_pos[tok] = lane;  // same wavefront: after the line above
        }
    }
    if (wave == NWV - 1) {
        const uint64_t lower = (lane == 0) ? 0ull : (~0ull >> (64 - lane));
        int cnt = 0;
        for (int c0 = 0; !SHRINK && !base_only && c0 < C; c0 += 64) {
            const int c = min(c0 + lane, C - 1);
            // the bucket's sorted positions inside this row tile
            const int lo = max(offsets[c], row_base), hi = min(offsets[c + 1], row_base + nrows);
            const bool owns = (c0 + lane < C) && hi > lo;
            const uint64_t m = __ballot(owns);
            if (owns) {
                const int idx = cnt + __popcll(m & lower);
                seg_lo[idx] = lo;
                seg_hi[idx] = hi;
                // the tuple and the slot table are decoded here, once
                for (int j = 0; j < 4; ++j) seg_ad[idx * 4 + j] = j < mix.k ? mix_adapter(mix, c, j) : 0;
            }
            cnt += __popcll(m);
        }
        if (lane == 0) *nseg_p = cnt;
    }
    __syncthreads();

    for (int ui = 0; ui < nw; ++ui) {
        bf16x8 fa[4][TM];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int s = ui * 4 + j;
            if (j == 0) {
                wait_vmcnt<3 * Geo::NR>();
#pragma unroll
                for (int jj = 0; jj < 4; ++jj)
#pragma unroll
                    for (int tm = 0; tm < TM; ++tm) fa[jj][tm] = load_a_frag(jj, tm);
                wait_lds();  // the staging tile is in registers before it is refilled
            }
            next_slab();
            if (j == 0)
                issue_stage(unit_of(ux_i++));
            else
                wait_vmcnt<4 * Geo::NR + XD>();
            const unsigned char *slot = ring + (s % kSbRing) * kSbSlot;
            bf16x8 bfr[TN];
#pragma unroll
            for (int tn = 0; tn < TN; ++tn) bfr[tn] = load_b_frag(slot, tn);
#pragma unroll
            for (int tm = 0; tm < TM; ++tm)
#pragma unroll
                for (int tn = 0; tn < TN; ++tn)
                    acc[tm][tn] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[j][tm], bfr[tn],
                                                                          acc[tm][tn], 0, 0, 0);
            wait_lds();  // the slab has been read before its slot is refilled
        }
    }
    wait_vmcnt<0>();  // the trailing loads (zeros) have landed: the ring is free

    // ---- grouped expand: acc += t B for the buckets that own rows ----
    // The stacked B (R = k * rank rows) of every such bucket is cut into slabs of 16 rows;
    // wavefront w takes slabs w, w + 8, ... of that sequence, four at a time: their loads and
    // the loads of the matching columns of t (both halves, [hi | lo]; zero for rows outside
    // the bucket) are all issued before the first is waited for, so a round costs one trip to
    // memory.  One read of a slab serves both halves of t.
    if constexpr (!SHRINK && !base_only) {
        const int nseg = __builtin_amdgcn_readfirstlane(*nseg_p);
        const int nsl = (R + 15) / 16;  // slabs per bucket
        const int nq = nseg * nsl;
        // slabs per round: 4 behind the W stream (8 measured no faster: the phase is bound by
        // reading B there), 8 when the expand runs alone (bound by its trips to memory)
        constexpr int G = expand_only ? 8 : 4;
        static_assert(G * kSbSlot <= kSbWaveLds, "a round's slabs fit the wavefront's LDS");
        int p_row[TM];  // sorted position of this lane's rows
#pragma unroll
        for (int tm = 0; tm < TM; ++tm) p_row[tm] = tile_pos[tm * 32 + m_lo];
        for (int q0 = wave; q0 < nq; q0 += NWV * G) {
            bf16x8 ta[G][2][TM];
#pragma unroll
            for (int g = 0; g < G; ++g) {
                const int q = q0 + NWV * g;
                if (q >= nq) break;
                const int sg = nsl == 1 ? q : q / nsl;
                const int part = q - sg * nsl;
                unsigned char *slot = ring + g * kSbSlot;
                // rows part*16 .. +15 of the stacked B of the sg-th bucket
                const bool whole = (rank & 15) == 0 && w_fast_ok;  // 16 rows of one adapter, all there
                const unsigned char *bb = nullptr;
                if (whole) {
                    const int col = part * 16;
                    const int jj = (col >= rank) + (col >= 2 * rank) + (col >= 3 * rank);
                    const int ad = __builtin_amdgcn_readfirstlane(seg_ad[sg * 4 + jj]);
                    // (packed: the slab's rows of this column group follow one another)
                    const int64_t grp = packed ? (int64_t)wg.x * 16 * kSbCols : 0;
                    bb = uniform_ptr(B + ((int64_t)ad * rank + (col - jj * rank)) * d_out + grp);
                }
#pragma unroll
                for (int r = 0; r < Geo::NR; ++r) {
                    if (whole) {
                        load_to_lds16(bb + (int64_t)(r * Geo::RPD) * (pitch * 2), w_off[r], slot + r * 1024);
                        continue;
                    }
                    if constexpr (packed) {  // a packed B has whole slabs only (host): never here
                        load_to_lds16_ptr(zero, slot + r * 1024);
                        continue;
                    }
                    const int col = part * 16 + r * Geo::RPD + w_rr;  // this lane's row of the stacked B
                    const uint16_t *src = zero;
                    if (col < R) {
                        const int jj = mix.k > 1 ? (col >= rank) + (col >= 2 * rank) + (col >= 3 * rank) : 0;
                        const int ad = seg_ad[sg * 4 + jj];
                        src = B + ((int64_t)ad * rank + (col - jj * rank)) * d_out + w_colv[r];
                    }
                    load_to_lds16_ptr(src, slot + r * 1024);
                }
                const int lo = __builtin_amdgcn_readfirstlane(seg_lo[sg]);
                const int hi = __builtin_amdgcn_readfirstlane(seg_hi[sg]);
                const int col = part * 16 + kg * 8;  // this lane's 8 columns of t
#pragma unroll
                for (int hl = 0; hl < 2; ++hl)
#pragma unroll
                    for (int tm = 0; tm < TM; ++tm) {
                        const int p = p_row[tm];
                        const bool ok = col < R && p >= lo && p < hi;
                        const uint16_t *src = ok ? t2 + (int64_t)p * two_r + hl * R + col : zero;
                        ta[g][hl][tm] = *(const bf16x8 *)src;
                    }
            }
            wait_vmcnt<0>();
#pragma unroll
            for (int g = 0; g < G; ++g) {
                if (q0 + NWV * g >= nq) break;
                bf16x8 bfr[TN];
#pragma unroll
                for (int tn = 0; tn < TN; ++tn) bfr[tn] = load_b_frag(ring + g * kSbSlot, tn);
#pragma unroll
                for (int hl = 0; hl < 2; ++hl)
#pragma unroll
                    for (int tm = 0; tm < TM; ++tm)
#pragma unroll
                        for (int tn = 0; tn < TN; ++tn)
                            acc[tm][tn] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(
                                ta[g][hl][tm], bfr[tn], acc[tm][tn], 0, 0, 0);
            }
            wait_lds();  // the slabs have been read before the next round refills them
        }
    }

    // ---- add the wavefronts' partial tiles, every row to its original position ----
    // acc[tm][tn][v]: row tm*32 + (v/4)*8 + (lane/32)*4 + v%4, column tn*32 + lane%32
#pragma unroll
    for (int tm = 0; tm < TM; ++tm)
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const int row = tm * 32 + (v >> 2) * 8 + kg * 4 + (v & 3);
#pragma unroll
            for (int tn = 0; tn < TN; ++tn)
                *(float *)(ring + row * kSbRowBytes + (tn * 32 + m_lo) * 4) = acc[tm][tn][v];
        }
    __syncthreads();
#pragma unroll
    for (int j = 0; j < kOutIters; ++j) {
        const int it = tid + j * NWV * 64;
        if (it >= TM * 32 * (kSbCols / 4)) break;
        const int row = it / (kSbCols / 4), ch = it % (kSbCols / 4);
        const int tok = tile_perm[row];
        const int col = n0 + ch * 4;
        if (tok < 0 || col >= d_out) continue;
        f32x4 sum = *(const f32x4 *)(smem + row * kSbRowBytes + ch * 16);
#pragma unroll
        for (int w = 1; w < NWV; ++w)
            sum += *(const f32x4 *)(smem + w * kSbWaveLds + row * kSbRowBytes + ch * 16);
        if (SHRINK && ksplit > 1) {
            // partial sums of this K slice; weights and the bf16 split wait for the reduction
            *(f32x4 *)(h + ((int64_t)slice * N + row_base + row) * R + col) = sum;
        } else if constexpr (SHRINK) {
            // piece j of the row is scaled by the token's j-th mixture weight; then
            // t = hi + lo with hi = bf16(t), lo = bf16(t - hi); row of t_out = [hi | lo]
            const float wj = mix.w != nullptr ? mix.w[(int64_t)tok * mix.k + col / rank] : 1.f;
            store_t_hi_lo(t_out + (int64_t)(row_base + row) * 2 * R, R, col, sum, wj);
        } else {
            if constexpr (expand_only) sum += h_old[j];  // this row's x W, written by the launch before
            *(f32x4 *)(h + (int64_t)tok * d_out + col) = sum;
        }
    }
}

template <int TM, int TN, bool SHRINK, int MODE, int NWV>
__global__ __launch_bounds__(NWV * 64) void small_batch_kernel(
    const uint16_t *__restrict__ x, const uint16_t *__restrict__ W, const uint16_t *__restrict__ B,
    const uint16_t *__restrict__ t2, const int32_t *__restrict__ offsets,
    const int32_t *__restrict__ perm, float *__restrict__ h, uint16_t *__restrict__ t_out, int N,
    int d_in, int d_out, int C, int rank, Mix mix, int ksplit, SortArgs sort) {
    SbBlock wg = SbBlock{(int)blockIdx.x, (int)blockIdx.y, (int)blockIdx.z, (int)gridDim.y};
    if constexpr (SHRINK) {
        if (sort.r == nullptr) {
            // Grid (work items, column groups, K slices): the work items are the 64-row tiles of
            // the buckets, bucket after bucket, and every wavefront finds its own from `offsets`
            // (there are at most ceil(N / 64) + C of them; workgroups past the last leave).
            // Workgroups go to the XCDs round-robin and item = XCD-major, so an XCD takes a
            // contiguous range of tiles: a few whole buckets when the buckets are level (its L2
            // then holds their A_c, not everyone's), its share of the tiles when one bucket
            // holds most rows.  (The grid this replaces had a slot for every (bucket, tile a
            // bucket can have at most): 8192 workgroups for the 256-272 tiles of 16384 tokens in
            // 32 buckets.  While the buckets are level the tiles in use are the first workgroups
            // of such a grid and the empty ones cost little; under a skewed routing the tiles of
            // the long buckets lie far apart in it, one or two in every 32 workgroups, and the
            // launch took 87 us instead of 45 (zipf), 48 instead of 30-33 us (one bucket).)
            const int lane = threadIdx.x & 63;
            // tiles of the buckets of one group of 64: this lane's bucket, its inclusive prefix
            int lo = 0, hi = 0, tiles = 0, incl = 0;
            auto scan_group = [&](int c0) {
                const int c = c0 + lane;
                lo = hi = 0;
                if (c < C) {
                    lo = offsets[c];
                    hi = offsets[c + 1];
                }
                tiles = max(0, (hi - lo + 63) / 64);
                incl = tiles;
#pragma unroll
                for (int d = 1; d < 64; d <<= 1) {
                    const int up = __shfl_up(incl, d, 64);
                    if (lane >= d) incl += up;
                }
            };
            int total = 0;  // work items of the launch
            for (int c0 = 0; c0 < C; c0 += 64) {
                scan_group(c0);
                total += __shfl(incl, 63, 64);
            }
            // XCD j takes items [j * per_xcd, (j + 1) * per_xcd): an equal share of the items there
            // are, not of the slots of the grid (36 slots against 32 items per XCD made a second
            // round of workgroups on seven XCDs)
            const int per_xcd = (total + 7) / 8;
            const int in_xcd = (int)(blockIdx.x / 8);
            const int item = (int)(blockIdx.x % 8) * per_xcd + in_xcd;
            int bucket = -1, tile = 0;
            if (in_xcd < per_xcd && item < total) {
                int running = 0;  // tiles of the buckets before the current group
                for (int c0 = 0; c0 < C && bucket < 0; c0 += 64) {
                    if (C > 64) scan_group(c0);  // (one group: still in registers)
                    const int rel = item - (running + incl - tiles);
                    const uint64_t m = __ballot(rel >= 0 && rel < tiles);
                    if (m) {
                        const int src = __ffsll((long long)m) - 1;
                        bucket = __shfl(c0 + lane, src, 64);
                        tile = __shfl(rel, src, 64);
                    }
                    running += __shfl(incl, 63, 64);
                }
            }
            if (bucket < 0) return;  // (the same for every wavefront of the workgroup)
            // (every lane holds the same pair; said explicitly, so that what is derived from
            // it stays in scalar registers)
            bucket = __builtin_amdgcn_readfirstlane(bucket);
            tile = __builtin_amdgcn_readfirstlane(tile);
            wg = SbBlock{(int)blockIdx.y, bucket, tile * ksplit + (int)blockIdx.z, C};
        }
    }
    small_batch_body<TM, TN, SHRINK, MODE, NWV>(x, W, B, t2, offsets, perm, h, t_out, N, d_in, d_out, C, rank,
                                                mix, ksplit, sort, wg);
}

// A decode-sized batch (N <= 64): the shrink (with the dispatch step inside, see SortArgs) and
// the base projection h = x W in ONE launch.  Neither needs anything from the other -- the
// base projection of a batch of one row tile runs in token order -- so the latency-bound
// shrink (a dozen workgroups each draining one A_c) hides behind the stream of W instead of
// preceding it.  Workgroups [0, n_shrink) are the shrink's grid (column groups of the rank x
// buckets, K not split: there is no hurry now), the others the GEMM's column groups in
// kSbBaseOnly mode (PACKED: kSbBasePacked, W in the order of pack_w_kernel).  The expand follows
// as a launch of its own (kSbExpandOnly, or kSbExpandPacked for a B in that order).
template <int TM, int TN, bool PACKED>
__global__ __launch_bounds__(kSbWaves * 64) void shrink_base_small_kernel(
    const uint16_t *__restrict__ x, const uint16_t *__restrict__ W, const uint16_t *__restrict__ A,
    float *__restrict__ h, uint16_t *__restrict__ t_out, int N, int d_in, int d_out, int C, int rank,
    Mix mix, SortArgs sort, int shrink_groups, int n_shrink) {
    const int b = (int)blockIdx.x;
    if (b < n_shrink) {
        small_batch_body<TM, 1, true>(x, A, nullptr, nullptr, nullptr, nullptr, nullptr, t_out, N, d_in,
                                      mix.k * rank, C, rank, mix, 1, sort,
                                      SbBlock{b % shrink_groups, b / shrink_groups, 0, C});
    } else {
        small_batch_body<TM, TN, false, PACKED ? kSbBasePacked : kSbBaseOnly>(
            x, W, nullptr, nullptr, nullptr, nullptr, h, nullptr, N, d_in, d_out, C, rank, mix, 1, SortArgs{},
            SbBlock{b - n_shrink, 0, 0, 1});
    }
}

// Second pass of a K-split shrink: t_p = (sum over the slices, ascending, of plane[s][p]) * w,
// split into bf16 halves.  Four columns of one routed sorted position per thread.
__global__ __launch_bounds__(256) void shrink_reduce_kernel(const float *__restrict__ planes,
                                                            const int32_t *__restrict__ offsets,
                                                            const int32_t *__restrict__ perm,
                                                            uint16_t *__restrict__ t_out, int N, int C,
                                                            int R, int rank, int ksplit, Mix mix) {
    const int per_row = R / 4;
    const int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (e >= (int64_t)N * per_row) return;
    const int p = (int)(e / per_row), col = (int)(e % per_row) * 4;
    // all loads issued before any is used: one trip to memory (a row past the routed ones holds
    // whatever the scratch held: read, never stored)
    const int n_routed = offsets[C];
    const int tok = perm[p];
    f32x4 part[4];
#pragma unroll
    for (int s = 0; s < 4; ++s)
        part[s] = *(const f32x4 *)(planes + ((int64_t)(s < ksplit ? s : 0) * N + p) * R + col);
    f32x4 sum = part[0];
#pragma unroll
    for (int s = 1; s < 4; ++s)
        if (s < ksplit) sum += part[s];
    for (int s = 4; s < ksplit; ++s) sum += *(const f32x4 *)(planes + ((int64_t)s * N + p) * R + col);
    if (p >= n_routed) return;  // rows past the routed ones belong to no bucket
    const float wj = mix.w != nullptr ? mix.w[(int64_t)tok * mix.k + col / rank] : 1.f;
    store_t_hi_lo(t_out + (int64_t)p * 2 * R, R, col, sum, wj);
}

// more than 64 KB of dynamic LDS has to be asked for, once per device (see common.h)
template <int TM, int TN, bool SHRINK, int MODE, int NWV>
struct SmallBatchKernel {
    static inline LdsRegistrar lds{(const void *)small_batch_kernel<TM, TN, SHRINK, MODE, NWV>,
                                   SbGeom<TN, NWV>::LDS_BYTES};
};

template <int TM, int TN, bool SHRINK, int MODE = 0, int NWV = kSbWaves>
hipError_t launch_small(const uint16_t *x, const uint16_t *W, const uint16_t *B, const uint16_t *t2,
                        const int32_t *offsets, const int32_t *perm, float *h, uint16_t *t_out, int N,
                        int d_in, int d_out, int C, int rank, Mix mix, hipStream_t s, int ksplit,
                        SortArgs sort) {
    using Geo = SbGeom<TN, NWV>;
    auto kern = small_batch_kernel<TM, TN, SHRINK, MODE, NWV>;
    (void)&SmallBatchKernel<TM, TN, SHRINK, MODE, NWV>::lds;  // instantiates the registration
    const unsigned groups = (unsigned)((d_out + Geo::COLS - 1) / Geo::COLS);
    const unsigned row_tiles = (unsigned)((N + 63) / 64);
    // GEMM: column groups x row tiles of the batch.  SHRINK: the 64-row tiles of the buckets (at
    // most row_tiles + C, rounded up to the eight XCDs) x column groups x K slices; with the
    // dispatch step inside (one row tile) column groups x buckets x K slices.
    const unsigned items = (row_tiles + (unsigned)C + 7) / 8 * 8;
    const dim3 grid = !SHRINK ? dim3(groups, row_tiles)
                              : (sort.r != nullptr ? dim3(groups, (unsigned)C, (unsigned)ksplit)
                                                   : dim3(items, groups, (unsigned)ksplit));
    if constexpr (!SHRINK && MODE == 0)  // the small-batch GEMM: base projection and expand
        launch_base_kernel(kern, grid, dim3(NWV * 64), Geo::LDS_BYTES, s, x, W, B, t2, offsets, perm, h,
                           t_out, N, d_in, d_out, C, rank, mix, ksplit, sort);
    else
        hipLaunchKernelGGL(kern, grid, dim3(NWV * 64), Geo::LDS_BYTES, s, x, W, B, t2, offsets, perm,
                           h, t_out, N, d_in, d_out, C, rank, mix, ksplit, sort);
    return hipGetLastError();
}

template <bool SHRINK, int MODE = 0>
hipError_t launch_small_tn(const uint16_t *x, const uint16_t *W, const uint16_t *B, const uint16_t *t2,
                           const int32_t *offsets, const int32_t *perm, float *h, uint16_t *t_out,
                           int N, int d_in, int d_out, int C, int rank, Mix mix, hipStream_t s,
                           int ksplit = 1, SortArgs sort = SortArgs{}) {
    // 32-column groups when 64-column groups would occupy at most half of the compute units:
    // a workgroup draws ~40 GB/s from HBM whatever its width, so more, narrower ones win there.
    // The shrink has at most a few workgroups per bucket and always takes the narrow form.
    const int64_t wgs64 = (int64_t)((d_out + 63) / 64) * ((N + 63) / 64);
    const bool narrow = SHRINK || wgs64 <= 128;
#define MOLORA_SB_LAUNCH(TM, TN) \
    launch_small<TM, TN, SHRINK, MODE>(x, W, B, t2, offsets, perm, h, t_out, N, d_in, d_out, C, rank, mix, s, ksplit, sort)
    if constexpr (SHRINK) {
        // A shrink with more 64-row tiles than compute units (the buckets' ragged last tiles
        // included: about C / 2 of them) runs workgroups of four wavefronts, three of which fit a
        // compute unit's LDS, so that all tiles are resident at once.  With eight wavefronts a
        // compute unit holds one workgroup, and the 16 tiles that 16384 tokens in 32 buckets have
        // beyond 256 made a second round on an otherwise idle chip (40 us against 25 us for
        // the 256 tiles of 32 buckets of exactly 512 rows).
        if (sort.r == nullptr && N > 64 && (N + 63) / 64 + C / 2 > 256)
            return launch_small<2, 1, true, 0, 4>(x, W, B, t2, offsets, perm, h, t_out, N, d_in, d_out, C, rank,
                                                  mix, s, ksplit, sort);
    }
    if (N <= 32) return narrow ? MOLORA_SB_LAUNCH(1, 1) : MOLORA_SB_LAUNCH(1, 2);
    return narrow ? MOLORA_SB_LAUNCH(2, 1) : MOLORA_SB_LAUNCH(2, 2);
#undef MOLORA_SB_LAUNCH
}

}  // namespace

hipError_t launch_small_batch_gemm(const uint16_t *x, const uint16_t *W, const uint16_t *B,
                                   const uint16_t *t2, const int32_t *offsets, const int32_t *perm,
                                   float *h, int64_t N, int d_in, int d_out, int C, int rank, Mix mix,
                                   hipStream_t s) {
    return launch_small_tn<false>(x, W, B, t2, offsets, perm, h, nullptr, (int)N, d_in, d_out, C, rank,
                                  mix, s);
}

namespace {
// W [d_in][d_out] -> Wp: W cut into slabs of 16 k-rows (the last may hold 8), and inside a slab
// column group after column group, each a [rows][gc] matrix of its own (gc = the streaming
// kernel's columns per workgroup for this d_out).  Slab s starts at element 16 * s * d_out, as
// in W.  One 16-byte chunk (8 columns) per thread; writes in order.
__global__ __launch_bounds__(256) void pack_w_kernel(const uint16_t *__restrict__ W,
                                                     uint16_t *__restrict__ Wp, int d_in, int d_out,
                                                     int gc) {
    const int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;  // chunk of Wp
    if (e >= (int64_t)d_in * (d_out / 8)) return;
    const int64_t per_slab = (int64_t)16 * (d_out / 8);  // chunks in a full slab
    const int sl = (int)(e / per_slab);
    const int rem = (int)(e - (int64_t)sl * per_slab);   // < 16 * d_out / 8
    const int rows = min(16, d_in - 16 * sl);
    const int cpg = gc / 8;                               // chunks per row of a group
    const int g = rem / (rows * cpg);
    const int rem2 = rem - g * rows * cpg;
    const int kk = rem2 / cpg, cc = rem2 % cpg;
    *(u32x4 *)(Wp + e * 8) = *(const u32x4 *)(W + (int64_t)(16 * sl + kk) * d_out + (int64_t)g * gc + cc * 8);
}

// the column-group width of the one-row-tile streaming kernel: 32 where 64-column groups would
// occupy at most half of the compute units
inline bool sb_narrow_one_tile(int d_out) { return (int64_t)((d_out + 63) / 64) <= 128; }

template <int TM, int TN, bool PACKED>
struct ShrinkBaseKernel {
    static constexpr size_t LDS = (SbGeom<TN>::LDS_BYTES > SbGeom<1>::LDS_BYTES) ? SbGeom<TN>::LDS_BYTES
                                                                               : SbGeom<1>::LDS_BYTES;
    static inline LdsRegistrar lds{(const void *)shrink_base_small_kernel<TM, TN, PACKED>, LDS};
};
template <int TM, int TN, bool PACKED>
hipError_t launch_shrink_base(const uint16_t *x, const uint16_t *W, const uint16_t *A, float *h,
                              uint16_t *t_out, int N, int d_in, int d_out, int C, int rank, Mix mix,
                              SortArgs sort, hipStream_t s) {
    (void)&ShrinkBaseKernel<TM, TN, PACKED>::lds;  // instantiates the registration
    if (PACKED && d_out % SbGeom<TN>::COLS != 0) return hipErrorInvalidValue;  // whole groups only
    const int shrink_groups = (mix.k * rank + 31) / 32;
    const int n_shrink = shrink_groups * C;
    const int gemm_groups = (d_out + SbGeom<TN>::COLS - 1) / SbGeom<TN>::COLS;
    auto kern = shrink_base_small_kernel<TM, TN, PACKED>;
    constexpr size_t lds_bytes = ShrinkBaseKernel<TM, TN, PACKED>::LDS;
    launch_base_kernel(kern, dim3((unsigned)(n_shrink + gemm_groups)), dim3(kSbWaves * 64), lds_bytes, s, x, W,
                       A, h, t_out, N, d_in, d_out, C, rank, mix, sort, shrink_groups, n_shrink);
    return hipGetLastError();
}
}  // namespace

// N <= 64: dispatch + shrink + h = x W in one launch (sort.r, sort.offsets, sort.perm required)
hipError_t launch_small_shrink_base(const uint16_t *x, const uint16_t *W, const uint16_t *A, float *h,
                                    uint16_t *t_out, int64_t N, int d_in, int d_out, int C, int rank,
                                    Mix mix, SortArgs sort, hipStream_t s, bool w_packed) {
    if (N < 1 || N > 64 || mix.k != 1 || !sort.r || !sort.offsets || !sort.perm) return hipErrorInvalidValue;
    if (w_packed && small_pack_cols(d_out) == 0) return hipErrorInvalidValue;
    const bool narrow = sb_narrow_one_tile(d_out);
#define MOLORA_SBB(TM, TN)                                                                                   \
    (w_packed ? launch_shrink_base<TM, TN, true>(x, W, A, h, t_out, (int)N, d_in, d_out, C, rank, mix, sort, s) \
              : launch_shrink_base<TM, TN, false>(x, W, A, h, t_out, (int)N, d_in, d_out, C, rank, mix, sort, s))
    if (N <= 32) return narrow ? MOLORA_SBB(1, 1) : MOLORA_SBB(1, 2);
    return narrow ? MOLORA_SBB(2, 1) : MOLORA_SBB(2, 2);
#undef MOLORA_SBB
}

// columns per group of the packed form of a [d_in][d_out] matrix (0: d_out has no packed form)
int small_pack_cols(int d_out) {
    const int gc = sb_narrow_one_tile(d_out) ? 32 : 64;
    return (d_out >= gc && d_out % gc == 0) ? gc : 0;
}

hipError_t launch_pack_w(const uint16_t *W, uint16_t *Wp, int d_in, int d_out, hipStream_t s) {
    const int gc = small_pack_cols(d_out);
    if (gc == 0 || d_in < 1) return hipErrorInvalidValue;
    const int64_t items = (int64_t)d_in * (d_out / 8);
    hipLaunchKernelGGL(pack_w_kernel, dim3((unsigned)((items + 255) / 256)), dim3(256), 0, s, W, Wp, d_in,
                       d_out, gc);
    return hipGetLastError();
}

// N <= 64: h += t B_c (the expand alone, after launch_small_shrink_base).  b_packed: the
// stacked B, [C * rank][d_out], in the slab order of pack_w_kernel (rank a multiple of 16, so
// that a slab lies inside one adapter).
hipError_t launch_small_expand(const uint16_t *B, const uint16_t *t2, const int32_t *offsets,
                               const int32_t *perm, float *h, int64_t N, int d_in, int d_out, int C,
                               int rank, Mix mix, hipStream_t s, bool b_packed) {
    if (N < 1 || N > 64) return hipErrorInvalidValue;
    if (b_packed) {
        if (rank % 16 != 0 || mix.k != 1 || small_pack_cols(d_out) == 0) return hipErrorInvalidValue;
        return launch_small_tn<false, kSbExpandPacked>(nullptr, nullptr, B, t2, offsets, perm, h, nullptr, (int)N,
                                                       d_in, d_out, C, rank, mix, s);
    }
    return launch_small_tn<false, kSbExpandOnly>(nullptr, nullptr, B, t2, offsets, perm, h, nullptr, (int)N, d_in,
                                                 d_out, C, rank, mix, s);
}

int small_batch_shrink_ksplit(int64_t N, int d_in, int C, int R) {
    // an upper bound of the workgroups a plain launch would have (32-column groups x (bucket,
    // 64-row tile) pairs): K is split when they would occupy at most a quarter / half of the
    // compute units and K is long enough for every slice to keep its wavefronts busy
    const int64_t groups = (R + 31) / 32;
    const int64_t pairs = (N < C ? N : C) + N / 64;
    const int64_t wgs = groups * pairs;
    if (wgs <= 64 && d_in >= 2048) return 4;
    if (wgs <= 128 && d_in >= 1024) return 2;
    // A few more tiles than compute units (the buckets' ragged last tiles) and a long K: the
    // launch takes as long as the compute unit that got two tiles, and quarter tiles level the
    // shares.  It pays the second launch only when K is long: 16384 x 12288, 32 buckets of rank
    // 32: 119.5 -> 102.3 us; at d_in = 4096 45.0 -> 45.4 us (one bucket: 32.9 -> 37.6 us).
    const int64_t tiles = (N + 63) / 64 + C / 2;
    if (N > 64 && groups == 1 && tiles > 256 && tiles <= 512 && d_in >= 8192) return 4;
    return 1;
}

hipError_t launch_small_batch_shrink(const uint16_t *x, const uint16_t *A, const int32_t *offsets,
                                     const int32_t *perm, uint16_t *t_out, int64_t N, int d_in, int C,
                                     int rank, Mix mix, hipStream_t s, float *planes, int ksplit,
                                     SortArgs sort) {
    const int R = mix.k * rank;  // the kernel's "d_out" is the width of the intermediate
    if (planes == nullptr) ksplit = 1;
    if (sort.r != nullptr && N > 64) return hipErrorInvalidValue;  // one wavefront of targets
    hipError_t e = launch_small_tn<true>(x, A, nullptr, nullptr, offsets, perm, planes, t_out, (int)N, d_in,
                                         R, C, rank, mix, s, ksplit, sort);
    if (e != hipSuccess || ksplit <= 1) return e;
    const int64_t items = N * (R / 4);
    hipLaunchKernelGGL(shrink_reduce_kernel, dim3((unsigned)((items + 255) / 256)), dim3(256), 0, s, planes,
                       offsets, perm, t_out, (int)N, C, R, rank, ksplit, mix);
    return hipGetLastError();
}

}  // namespace molora
