// Fused base projection + grouped expand (Eq. "pertok"):
//
//     h[perm[p]][:] = x[perm[p]] W  +  t_p B_{c(p)}           for every sorted position p
//
// One bf16 MFMA GEMM over the rows in bucket order.  The grouped expand is not a second
// kernel: after the d_in-long K loop over (x, W) the same accumulators take a few extra
// K tiles whose A operand is the low-rank intermediate t (as [hi | lo] bf16 halves, K =
// 2*rank) and whose B operand is [B_c; B_c] for each bucket c that owns rows of the tile;
// rows of other buckets are zero in that operand.  h is then written once, in fp32, to the
// rows' original positions (the "scatter to original positions" of the paper's pipeline).
// Rows past offsets[C] (tokens without adapter) simply have no extra tiles.
//
// Tiling: BM x BN output tile per workgroup, WM x WN wavefronts, each owning a grid of
// 32x32 MFMA tiles (v_mfma_f32_32x32x16_bf16, fp32 accumulate).
//   x tile  [BM][BK]  16-byte chunks XOR-swizzled inside a row so that the operand read (one
//                     row per lane, ds_read_b128) is bank-conflict free;
//   W tile  [BK][BN]  exactly as it lies in HBM (K-major), 32-byte chunks swizzled by (k & 3);
//                     the LDS transpose read turns it into the k-contiguous operand, so W needs
//                     no packing pass and no transposed copy.
// Every K tile goes HBM -> LDS directly (global_load_lds_dwordx4: no staging registers; the
// gathered row address and the swizzle are applied on the global side, the LDS side is
// linear).  Whatever has to read as zero -- k past d_in, t rows of other buckets, padding of
// 2*rank up to the tile depth -- is fetched from a small all-zero page instead, so the K
// tail and the expand tiles travel the same path as the base tiles.
// One main loop for two to four LDS stages, with the operand fragments of the next k-step
// prefetched into registers behind the MFMAs.  (Small batches, which are bound by streaming W
// once, have a kernel of their own in small_batch.hip; launch_fused_gemm chooses.)
// Workgroups are numbered so that the 8 XCDs (blockIdx % 8) each walk a compact group of
// tiles and share x rows / W columns in their own L2.
#include <type_traits>

#include "common.h"
#include "lds_dma.h"

namespace molora {

namespace {

constexpr int kGroupM = 8;  // row tiles per scheduling group

// BM x BN output tile, WM x WN wavefronts, BK deep K tiles, STAGES LDS buffers.
template <int BM_, int BN_, int WM_, int WN_, int BK_, int STAGES_>
struct GemmCfg {
    static constexpr int BM = BM_, BN = BN_, WM = WM_, WN = WN_, BK = BK_, STAGES = STAGES_;
    static constexpr int NW = WM * WN, NT = 64 * NW;
    static constexpr int TM = BM / WM / 32, TN = BN / WN / 32;
    // A tile = x rows, B tile = W rows; a load instruction fills 1 KB = one "piece"
    static constexpr int A_RB = BK * 2, A_CPR = A_RB / 16, A_RPI = 64 / A_CPR;
    static constexpr int B_RB = BN * 2, B_CPR = B_RB / 16, B_RPI = 64 / B_CPR;
    static constexpr int A_PIECES = BM / A_RPI, B_PIECES = BK / B_RPI;
    static constexpr int LPW = (A_PIECES + B_PIECES) / NW;  // pieces (loads) per wavefront and tile
    static constexpr int A_BYTES = BM * A_RB, B_BYTES = BK * B_RB, STAGE = A_BYTES + B_BYTES;
    static constexpr size_t LDS_BYTES = (size_t)STAGES * STAGE + 8 * BM * sizeof(int32_t) + 16;
    static_assert(BK == 32 || BK == 64, "BK");
    static_assert(LPW * NW == A_PIECES + B_PIECES && LPW >= 1, "pieces split evenly over wavefronts");
    static_assert(STAGES >= 2 && STAGES <= 4, "stages");

    // Where the 32-byte chunk `chunk` (16 columns) of k-row `row` of the W tile lies in its LDS
    // row: XORed with row & 3, so that the four consecutive k-rows a group of 16 lanes takes in
    // a transpose read land in four different chunks of a 128-byte window.  (All rows start at
    // bank 0, and lanes 0-31 of a read, which the hardware serves together, take adjacent chunks
    // of the SAME window: SQ_LDS_BANK_CONFLICT counts 2 extra cycles on every such read and on
    // nothing else in the kernel.  Sending the two groups to different halves of the banks --
    // chunk bits 0 and 2 swapped -- brings the counter to zero and the LDS busy cycles down by
    // 24 %, and makes the kernel 1.5 % slower: the LDS-direct loads then fetch alternating
    // 32-byte pieces of two cache lines per 8 lanes, and the LDS, a third busy, is not what
    // the kernel waits for.  Measured, not kept.)
    __device__ static __forceinline__ int swz_b(int chunk, int row) { return chunk ^ (row & 3); }
    __device__ static __forceinline__ int swz_b_inv(int pos, int row) { return pos ^ (row & 3); }
    // XOR applied to the 16-byte chunk index of an x-tile row
    __device__ static __forceinline__ int swz_a(int row) {
        if constexpr (BK == 64) return (row ^ (row >> 3)) & 7;
        // 64-byte rows: distinct banks for 8 consecutive rows (32 banks) and 16 (64 banks)
        return (((row >> 2) & 1) << 1) | (((row >> 1) ^ (row >> 3)) & 1);
    }
};

// PACK: narrow adapters share an expand tile (launch_cfg picks it from the rank).  A template
// parameter, not a run-time branch: the kernel with 256 x 256 tiles has no register to spare,
// and with both forms of the expand tile in one kernel the ordinary form ran 2-3 % slower on
// expand-heavy shapes (top-2 / top-3 mixtures), with one form computing both 9-20 % slower.
template <class Cfg, bool PACK>
__global__ __launch_bounds__(Cfg::NT) void fused_gemm_kernel(
    const uint16_t *__restrict__ x, const uint16_t *__restrict__ W, const uint16_t *__restrict__ B,
    const uint16_t *__restrict__ t2, const int32_t *__restrict__ offsets,
    const int32_t *__restrict__ perm, float *__restrict__ h, int N, int d_in, int d_out, int C,
    int rank, int tiles_m, int tiles_n, Mix mix) {
    constexpr int BM = Cfg::BM, BN = Cfg::BN, BK = Cfg::BK, NT = Cfg::NT, TM = Cfg::TM,
                  TN = Cfg::TN, STAGES = Cfg::STAGES;
    // (1 KB alignment: the operand reads XOR k-step bits into addresses relative to this base)
    extern __shared__ __attribute__((aligned(1024))) unsigned char smem[];
    int32_t *tile_perm = (int32_t *)(smem + STAGES * Cfg::STAGE);  // [BM] token per row, -1 = none
    int32_t *seg_lo = tile_perm + BM;  // buckets intersecting the tile: their sorted-position ranges
    int32_t *seg_hi = seg_lo + BM;
    int32_t *nseg_p = seg_hi + BM;
    int32_t *seg_ad = nseg_p + 4;  // [BM][4] pool positions of the adapters of a bucket's tuple
    int32_t *seg_c = seg_ad + 4 * BM;  // [BM] the buckets' indices (the token-order intermediate is addressed by them)

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave / Cfg::WN, wn = wave % Cfg::WN;

    // ---- tile of this workgroup: XCD-major, then groups of kGroupM row tiles ----
    const int total = tiles_m * tiles_n;
    const int per_xcd = (total + 7) / 8;
    const int logical = (int)(blockIdx.x % 8) * per_xcd + (int)(blockIdx.x / 8);
    if (logical >= total) return;
    // Group g holds the row tiles g, g + ng, g + 2 ng, ... (at most kGroupM of them), not
    // kGroupM consecutive ones: the rows are gathered through perm, so consecutive row tiles
    // share nothing, but under a skewed routing the LAST row tiles are the ones crossed by many
    // small buckets (many expand tiles each), and consecutive grouping put them all on one XCD.
    const int ng = (tiles_m + kGroupM - 1) / kGroupM;
    const int q = tiles_m / ng, rem = tiles_m % ng;  // the first rem groups have q + 1 row tiles
    const int big = rem * (q + 1) * tiles_n;         // output tiles in those groups
    const int gm = logical < big ? q + 1 : q;
    const int rest = logical < big ? logical : logical - big;
    const int g = (logical < big ? 0 : rem) + rest / (gm * tiles_n);
    const int in_group = rest % (gm * tiles_n);
    const int tile_m = g + ng * (in_group % gm);
    const int tile_n = in_group / gm;
    const int p0 = tile_m * BM, n0 = tile_n * BN;

    const int R = mix.k * rank;  // width of a bucket's intermediate (k adapters side by side)
    const int two_r = 2 * R;
    const int tps = (two_r + BK - 1) / BK;  // extra K tiles per bucket
    // Narrow adapters share an expand tile (PACK; the host has checked that 2R is 16 or 32, a
    // power of two at most BK / 2, and that t is in bucket order): a K tile has room for
    // BK / 2R buckets side by side in k (bucket s of the tile at k = s * 2R: its rows read their
    // t there and zeros elsewhere, its [B; B] lies in those k-rows), so a row tile that many
    // small buckets cross pays one extra K tile per 2-4 of them, not one each.  Every row still
    // gets exactly its own products in the same order, plus exact zeros: same bits.
    const int two_r_shift = __builtin_ctz(two_r | BK);              // log2(2R) when PACK
    const int pk_shift = PACK ? __builtin_ctz(BK) - two_r_shift : 0;  // log2(buckets per tile)
    const int nkf = d_in / BK;              // full K tiles
    const int nkb = (d_in + BK - 1) / BK;   // K tiles of x.W, the last one possibly partial

    // ---- per-lane sources of this wavefront's load instructions ----
    // A stage is A_PIECES + B_PIECES pieces of 1 KB, x pieces (A_RPI rows each) first, then W
    // pieces (B_RPI k-rows each); load i of wavefront w is piece i*NW + w, so every wavefront
    // carries its share of the gathered x rows and of the W rows.
    // Rows past N and columns past d_out are clamped to valid memory: what they produce is
    // never stored.
    auto piece_of = [&](int i) { return i * Cfg::NW + wave; };
    auto slot_is_a = [&](int i) {  // wave-uniform; a compile-time fact when the pieces divide evenly
        if constexpr (Cfg::A_PIECES % Cfg::NW == 0) return i < Cfg::A_PIECES / Cfg::NW;
        return piece_of(i) < Cfg::A_PIECES;
    };
    // geometry of load i of this wavefront: x piece -> (tile row, 8-k chunk index after the
    // swizzle); W piece -> (k-row, global column).  Recomputed where needed instead of kept in
    // registers: only the special tiles and the set-up use it.
    auto slot_geom = [&](int i, int &row, int &col) {
        if (slot_is_a(i)) {
            row = piece_of(i) * Cfg::A_RPI + lane / Cfg::A_CPR;
            col = (lane % Cfg::A_CPR) ^ Cfg::swz_a(row);
        } else {
            row = (piece_of(i) - Cfg::A_PIECES) * Cfg::B_RPI + lane / Cfg::B_CPR;
            const int pos = lane % Cfg::B_CPR;
            // this lane fills 16-byte position pos of the LDS row, i.e. half pos & 1 of physical
            // 32-byte chunk pos >> 1, which holds the logical chunk given by swz_b's inverse
            const int u16 = (Cfg::swz_b_inv(pos >> 1, row) << 1) | (pos & 1);
            col = min(n0 + u16 * 8, d_out - 8);
        }
    };
    uint32_t off_g[Cfg::LPW];  // full tiles: byte offset from the scalar base
#pragma unroll
    for (int i = 0; i < Cfg::LPW; ++i) {  // W pieces (the x pieces need the row table, below)
        int row, col;
        slot_geom(i, row, col);
        off_g[i] = slot_is_a(i) ? 0u : (uint32_t)(((int64_t)row * d_out + col) * 2);
    }
    // scalar bases of the full tiles, advanced per tile (x and W are < 4 GiB each)
    const unsigned char *a_base = (const unsigned char *)x;
    const unsigned char *b_base = (const unsigned char *)W;
    const int64_t b_step = (int64_t)BK * d_out * 2;

    auto issue_one = [&](unsigned char *stage, int i) {  // i-th load of a full tile
        load_to_lds16(slot_is_a(i) ? a_base : b_base, off_g[i], stage + piece_of(i) * 1024);
    };
    // The x part (want_a) and / or the W part (want_b) of base tile T < nkb; a partial last
    // tile computes a source per lane, k past d_in reads from the zero page.  Each part must
    // be issued in ascending tile order (the fast form advances its base).
    auto issue_base_parts = [&](unsigned char *stage, int T, bool want_a, bool want_b) {
        if (T < nkf) {
#pragma unroll
            for (int i = 0; i < Cfg::LPW; ++i)
                if (slot_is_a(i) ? want_a : want_b) issue_one(stage, i);
            if (want_a) a_base += BK * 2;
            if (want_b) b_base += b_step;
            return;
        }
        const uint16_t *zero = (const uint16_t *)g_zero_page;
#pragma unroll
        for (int i = 0; i < Cfg::LPW; ++i) {
            if (!(slot_is_a(i) ? want_a : want_b)) continue;
            const uint16_t *src;
            int row, col;
            slot_geom(i, row, col);
            if (slot_is_a(i)) {
                const int k = T * BK + col * 8;
                const int tok = tile_perm[row];
                src = (k < d_in) ? x + (int64_t)(tok >= 0 ? tok : 0) * d_in + k : zero;
            } else {
                const int k = T * BK + row;
                src = (k < d_in) ? W + (int64_t)k * d_out + col : zero;
            }
            load_to_lds16_ptr(src, stage + piece_of(i) * 1024);
        }
    };
    // With two stages every wait of the main loop is for all outstanding loads, so the order in
    // which the first tiles' pieces are issued is free: their W pieces, which depend on nothing
    // the dispatch step produced, go out before the tables are even read.
    const bool early_w = STAGES == 2 && nkb >= STAGES;
    if (early_w) {
#pragma unroll
        for (int T = 0; T < STAGES; ++T) issue_base_parts(smem + T * Cfg::STAGE, T, false, true);
    }

    // ---- per-tile tables: the rows' tokens and the buckets that own rows, both global reads
    // in flight together ----
    if (tid == 0) *nseg_p = 0;
    int32_t my_tok = -1, o_lo = 0, o_hi = 0;
    if (tid < BM && p0 + tid < N) my_tok = perm[p0 + tid];
    if (tid < C) {
        o_lo = offsets[tid];
        o_hi = offsets[tid + 1];
    }
    __syncthreads();  // the segment counter is zero
    if (tid < BM) tile_perm[tid] = my_tok;
    for (int i = tid + NT; i < BM; i += NT) tile_perm[i] = (p0 + i < N) ? perm[p0 + i] : -1;
    for (int c = tid; c < C; c += NT) {
        if (c != tid) {
            o_lo = offsets[c];
            o_hi = offsets[c + 1];
        }
        const int lo = max(o_lo, p0), hi = min(o_hi, p0 + BM);
        if (lo < hi) {
            const int idx = atomicAdd(nseg_p, 1);
            seg_lo[idx] = lo;
            seg_hi[idx] = hi;
            seg_c[idx] = c;
            // slot table and tuple decoded once here, not inside the K loop
            for (int j = 0; j < mix.k; ++j) seg_ad[idx * 4 + j] = mix_adapter(mix, c, j);
        }
    }
    __syncthreads();
    const int nseg = *nseg_p;
    // all K tiles of this output tile
    const int nk = nkb + (PACK ? (nseg + (1 << pk_shift) - 1) >> pk_shift : nseg * tps);
#pragma unroll
    for (int i = 0; i < Cfg::LPW; ++i) {  // x pieces: the gathered row of every lane
        if (!slot_is_a(i)) continue;
        int row, col;
        slot_geom(i, row, col);
        const int tok = tile_perm[row];
        off_g[i] = (uint32_t)(((int64_t)(tok >= 0 ? tok : 0) * d_in + col * 8) * 2);
    }

    // Any K tile T.  The expand tiles compute a source per lane; chunks that must read as zero
    // come from the zero page.  Tiles must be issued in ascending order.
    auto issue_tile = [&](unsigned char *stage, int T) {
        if (T < nkb) return issue_base_parts(stage, T, true, true);
        const uint16_t *zero = (const uint16_t *)g_zero_page;
        // expand tile: A operand = t rows of one bucket (others zero), B operand = [B_c; B_c]
        const int e = T - nkb;
        if constexpr (PACK) {  // several narrow buckets side by side in k
#pragma unroll
            for (int i = 0; i < Cfg::LPW; ++i) {
                const uint16_t *src = zero;
                int row, col;
                slot_geom(i, row, col);
                const int kk = slot_is_a(i) ? col * 8 : row;            // k inside the tile
                const int sg = (e << pk_shift) + (kk >> two_r_shift);  // the bucket that owns this k
                const int vk = kk & (two_r - 1);                         // k inside the bucket's 2R
                if (sg < nseg) {
                    if (slot_is_a(i)) {
                        const int p = p0 + row;
                        if (p >= seg_lo[sg] && p < seg_hi[sg]) src = t2 + (int64_t)p * two_r + vk;
                    } else {
                        const int j = vk < R ? vk : vk - R;
                        const int jj = mix.k > 1 ? j / rank : 0;
                        const int64_t brow = (int64_t)seg_ad[sg * 4 + jj] * rank + (j - jj * rank);
                        src = B + brow * d_out + col;
                    }
                }
                load_to_lds16_ptr(src, stage + piece_of(i) * 1024);
            }
            return;
        }
        const int sg = e / tps, sub = e % tps;
        const int lo = seg_lo[sg], hi = seg_hi[sg];
#pragma unroll
        for (int i = 0; i < Cfg::LPW; ++i) {
            const uint16_t *src;
            int row, col;
            slot_geom(i, row, col);
            if (slot_is_a(i)) {
                const int p = p0 + row, vk = sub * BK + col * 8;
                const bool own = p >= lo && p < hi && vk < two_r;
                if (mix.t_dense) {
                    // token-order intermediate: the row of this token, the bucket's adapter;
                    // high parts in the first C * rank values, remainders in the second
                    const int64_t trow = (int64_t)max(tile_perm[row], 0) * (2 * mix.C * rank);
                    const int in_half = vk < rank ? vk : vk - rank;
                    src = own ? t2 + trow + (vk < rank ? 0 : mix.C * rank) + seg_c[sg] * rank + in_half : zero;
                } else {
                    src = own ? t2 + (int64_t)p * two_r + vk : zero;
                }
            } else {
                const int vk = sub * BK + row;
                const int j = vk < R ? vk : vk - R;        // row of the tuple's stacked B
                const int jj = mix.k > 1 ? j / rank : 0;   // which adapter of the tuple
                const int64_t brow = (int64_t)seg_ad[sg * 4 + jj] * rank + (j - jj * rank);
                src = (vk < two_r) ? B + brow * d_out + col : zero;
            }
            load_to_lds16_ptr(src, stage + piece_of(i) * 1024);
        }
    };

    f32x16 acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

    // operand read offsets that do not depend on the k-step
    const int a_row0 = wm * (BM / Cfg::WM) + (lane & 31);    // + tm*32
    const int a_kg = lane >> 5;                               // k-group inside a 16-wide step
    const int blk = lane >> 4, a16 = lane & 15;
    const int b_kr0 = (blk >> 1) * 8 + (a16 >> 2);            // + ks*16 (+4 for the upper half)
    const int b_col0 = wn * (BN / Cfg::WN) + 16 * (blk & 1);  // + tn*32 ; column of lane = +a16
    const int b_in = (a16 & 3) * 8;                           // byte inside the 32-byte chunk
    // Per-lane LDS addresses of the operand fragments in stage 0, k-step 0:
    //   x fragment tm: row a_row0 + tm*32, 16-byte chunk (2*ks + a_kg) ^ swizzle(row).  The
    //     chunk index is XORed, and 2*ks touches bits the rest of the address never carries into
    //     (rows are A_RB = 32*KS bytes long and so aligned), so k-step ks is the k-step-0
    //     address XOR ks*32: one operation per read;
    //   W fragment tn: k-row b_kr0 (+4), the swizzled position of 32-byte chunk
    //     (b_col0 + tn*32) / 16, which is the same for every k-step (the swizzle looks at bits
    //     0 and 1 of the row): k-step ks is a constant added, i.e. the read's immediate offset.
    // A tile's addresses are these plus its stage's offset, added once per tile.
    static_assert(Cfg::A_RB == 32 * (BK / 16), "the XOR form of the x fragment address");
    const uint32_t smem0 = (uint32_t)(uintptr_t)(MOLORA_LDS unsigned char *)smem;
    uint32_t pa[TM], pb[TN];
#pragma unroll
    for (int tm = 0; tm < TM; ++tm) {
        const int row = a_row0 + tm * 32;
        pa[tm] = smem0 + row * Cfg::A_RB + ((a_kg ^ Cfg::swz_a(row)) << 4);
    }
#pragma unroll
    for (int tn = 0; tn < TN; ++tn)
        pb[tn] = smem0 + Cfg::A_BYTES + b_kr0 * Cfg::B_RB + (Cfg::swz_b((b_col0 + tn * 32) >> 4, b_kr0) << 5) + b_in;

    // `opaque` keeps the compiler from precomputing one address register per (stage, k-step,
    // fragment) outside the loop, which costs far more registers than it saves.
    auto opaque = [](uint32_t v) {
        asm volatile("" : "+v"(v));
        return v;
    };
    // Addresses of the tile being multiplied (ca, cb) and of the next one (na, nb).  With two
    // stages the hot loop is unrolled by two, so each copy knows its stage: it reads through the
    // constant arrays p?0 / p?1 and spends nothing on addresses but the XOR; elsewhere the
    // stage offset is added once per tile.
    uint32_t ca_rt[TM], cb_rt[TN], na_rt[TM], nb_rt[TN];
    uint32_t pa1[TM], pb1[TN];  // stage 1
#pragma unroll
    for (int tm = 0; tm < TM; ++tm) pa1[tm] = pa[tm] + Cfg::STAGE;
#pragma unroll
    for (int tn = 0; tn < TN; ++tn) pb1[tn] = pb[tn] + Cfg::STAGE;
    auto stage_addresses = [&](uint32_t (&a)[TM], uint32_t (&b)[TN], int T) {
        const uint32_t so = (uint32_t)(T % STAGES) * Cfg::STAGE;
#pragma unroll
        for (int tm = 0; tm < TM; ++tm) a[tm] = opaque(pa[tm] + so);
#pragma unroll
        for (int tn = 0; tn < TN; ++tn) b[tn] = opaque(pb[tn] + so);
    };
    auto load_a_frag = [&](const uint32_t (&a)[TM], int ks, int tm) -> bf16x8 {
        return *(const MOLORA_LDS bf16x8 *)(uintptr_t)(a[tm] ^ (uint32_t)(ks * 32));
    };
    auto load_b_frag = [&](const uint32_t (&b)[TN], int ks, int tn) -> bf16x8 {
        const uint32_t p = b[tn] + (uint32_t)(ks * 16 * Cfg::B_RB);
        const i16x4 lo = lds_read_tr16((const MOLORA_LDS void *)(uintptr_t)p);
        const i16x4 hi = lds_read_tr16((const MOLORA_LDS void *)(uintptr_t)(p + 4 * Cfg::B_RB));
        const i16x8 b8 = {lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
        return __builtin_bit_cast(bf16x8, b8);
    };
    constexpr int KS = BK / 16;

    // ---- main loop ----
    // STAGES LDS stages (tile kt lives in stage kt % STAGES, tiles kt+1 .. kt+STAGES-1 are in
    // flight) and two register sets of operand fragments.  While the MFMAs of k-step ks run,
    // the fragments of step ks+1 are fetched from LDS, one read after each MFMA, so the matrix
    // pipe never waits for LDS.  The workgroup barrier sits in front of the LAST k-step of a
    // tile: at that point every wavefront holds the tile's last fragments in registers, so the
    // stage can be refilled (tile kt+STAGES) and the first fragments of tile kt+1 can be
    // fetched while the last MFMAs of tile kt still run.  Two stages are enough when a tile's
    // MFMAs outlast the load latency (256 x 256 tiles); smaller tiles need the next tiles
    // further ahead.
    static_assert(KS % 2 == 0, "two fragment register sets");
    bf16x8 fa[2][TM], fb[2][TN];
    auto fetch_one = [&](const uint32_t (&a)[TM], const uint32_t (&b)[TN], int ks, int set, int i) {  // i-th fragment
        if (i < TM)
            fa[set][i] = load_a_frag(a, ks, i);
        else if (i < TM + TN)
            fb[set][i - TM] = load_b_frag(b, ks, i - TM);
    };
    // loads return in order: tile T has landed once at most the loads of the `younger` tiles
    // issued after it are outstanding
    auto wait_tiles = [&](int younger) {
        if constexpr (STAGES >= 4)
            if (younger >= 2) return wait_vmcnt<2 * Cfg::LPW>();
        if constexpr (STAGES >= 3)
            if (younger >= 1) return wait_vmcnt<Cfg::LPW>();
        wait_vmcnt<0>();
    };
    auto stage_of = [&](int T) { return smem + (T % STAGES) * Cfg::STAGE; };
#pragma unroll
    for (int T = 0; T < STAGES; ++T) {
        if (early_w)
            issue_base_parts(smem + T * Cfg::STAGE, T, true, false);  // the W part is on its way
        else if (T < nk)
            issue_tile(smem + T * Cfg::STAGE, T);
    }
    wait_tiles(min(nk, STAGES) - 1);
    wg_barrier();
#pragma unroll
    for (int i = 0; i < TM + TN; ++i) fetch_one(pa, pb, 0, 0, i);

    // one K tile: KS-1 ordinary k-steps, then the last one.  MORE: another tile follows.
    // REFILL: 0 = nothing to load, 1 = tile kt+STAGES is a full tile and its loads are
    // interleaved with the MFMAs, 2 = tile kt+STAGES is of any kind, loaded in one go.
    // SP: the tile's stage when the caller knows it (two stages, hot loop), -1 otherwise.
    auto k_tile = [&](int kt, auto more_c, auto refill_c, auto sp_c) {
        constexpr bool MORE = decltype(more_c)::value;
        constexpr int REFILL = decltype(refill_c)::value;
        constexpr int SP = decltype(sp_c)::value;
        unsigned char *as = SP >= 0 ? smem + SP * Cfg::STAGE : stage_of(kt);
        const uint32_t (&ca)[TM] = SP < 0 ? ca_rt : (SP == 0 ? pa : pa1);
        const uint32_t (&cb)[TN] = SP < 0 ? cb_rt : (SP == 0 ? pb : pb1);
        const uint32_t (&na)[TM] = SP < 0 ? na_rt : (SP == 0 ? pa1 : pa);
        const uint32_t (&nb)[TN] = SP < 0 ? nb_rt : (SP == 0 ? pb1 : pb);
        if constexpr (MORE && SP < 0) stage_addresses(na_rt, nb_rt, kt + 1);
#pragma unroll
        for (int ks = 0; ks < KS - 1; ++ks) {
            const int cur = ks & 1, nxt = cur ^ 1;
#pragma unroll
            for (int i = 0; i < TM * TN; ++i) {
                acc[i / TN][i % TN] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(
                    fa[cur][i / TN], fb[cur][i % TN], acc[i / TN][i % TN], 0, 0, 0);
                fetch_one(ca, cb, ks + 1, nxt, i);
                __builtin_amdgcn_sched_barrier(0);
            }
#pragma unroll
            for (int i = TM * TN; i < TM + TN; ++i) fetch_one(ca, cb, ks + 1, nxt, i);
        }
        constexpr int cur = (KS - 1) & 1, nxt = cur ^ 1;
        if constexpr (MORE) {
            wait_lds();  // this wavefront's reads of stage kt are complete
            // its part of tile kt+1 has landed; tiles kt+2 .. may still be in flight
            if constexpr (REFILL != 0)
                wait_tiles(STAGES - 2);
            else
                wait_tiles(min(nk - 2 - kt, STAGES - 2));
            wg_barrier();  // ... and so has everyone else's; stage kt is free
        }
        if constexpr (REFILL == 2) issue_tile(as, kt + STAGES);
#pragma unroll
        for (int i = 0; i < TM * TN; ++i) {
            acc[i / TN][i % TN] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(
                fa[cur][i / TN], fb[cur][i % TN], acc[i / TN][i % TN], 0, 0, 0);
            if constexpr (MORE) fetch_one(na, nb, 0, nxt, i);
            if constexpr (REFILL == 1)
                if (i < Cfg::LPW) issue_one(as, i);
            __builtin_amdgcn_sched_barrier(0);
        }
        if constexpr (MORE) {
#pragma unroll
            for (int i = TM * TN; i < TM + TN; ++i) fetch_one(na, nb, 0, nxt, i);
        }
        if constexpr (REFILL == 1) {
#pragma unroll
            for (int i = TM * TN; i < Cfg::LPW; ++i) issue_one(as, i);
            a_base += BK * 2;
            b_base += b_step;
        }
        if constexpr (MORE && SP < 0) {  // the next tile becomes the current one
#pragma unroll
            for (int tm = 0; tm < TM; ++tm) ca_rt[tm] = na_rt[tm];
#pragma unroll
            for (int tn = 0; tn < TN; ++tn) cb_rt[tn] = nb_rt[tn];
        }
    };
    using I0 = std::integral_constant<int, 0>;
    using I1 = std::integral_constant<int, 1>;
    using I2 = std::integral_constant<int, 2>;
    using RT = std::integral_constant<int, -1>;
    int kt = 0;
    if constexpr (STAGES == 2) {  // the hot loop, two tiles per round: every copy knows its stage
        for (; kt + 1 + STAGES < nkf; kt += 2) {
            k_tile(kt, std::true_type{}, I1{}, I0{});
            k_tile(kt + 1, std::true_type{}, I1{}, I1{});
        }
    }
    stage_addresses(ca_rt, cb_rt, kt);
    for (; kt + STAGES < nkf; ++kt) k_tile(kt, std::true_type{}, I1{}, RT{});  // the hot loop
    for (; kt + STAGES < nk; ++kt) k_tile(kt, std::true_type{}, I2{}, RT{});   // last base + expand tiles
    for (; kt + 1 < nk; ++kt) k_tile(kt, std::true_type{}, I0{}, RT{});        // nothing left to load
    k_tile(kt, std::false_type{}, I0{}, RT{});

    // ---- epilogue: every row to its original position ----
    // acc[tm][tn][v]: row tm*32 + (v/4)*8 + (lane/32)*4 + v%4, column tn*32 + lane%32.
    // The accumulators go through LDS one 32-row band per wavefront row at a time, so that
    // the global stores are 16 bytes per lane and a whole BN-wide row segment (1 KB) per
    // instruction: the rows are scattered over all of h by the permutation, and narrow
    // stores to scattered rows are what the memory system handles worst.
    constexpr int EP_STRIDE = BN * 4 + 32;           // bytes per staged row (+32: bank shift)
    constexpr int EP_CPR = BN / 4;                   // 16-byte chunks per row
    {
        constexpr int EP_ROWS = Cfg::WM * 32;
        static_assert(EP_ROWS * EP_STRIDE <= STAGES * Cfg::STAGE, "epilogue staging fits the stages");
        static_assert(EP_ROWS * EP_CPR % NT == 0, "every thread stores the same number of chunks of a band");
        constexpr int EP_IT = EP_ROWS * EP_CPR / NT;
#pragma unroll
        for (int tm = 0; tm < TM; ++tm) {
            __syncthreads();  // operand stages (or the previous band) are no longer read
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int rr = wm * 32 + (v >> 2) * 8 + (lane >> 5) * 4 + (v & 3);
#pragma unroll
                for (int tn = 0; tn < TN; ++tn) {
                    const int col = wn * (BN / Cfg::WN) + tn * 32 + (lane & 31);
                    *(float *)(smem + rr * EP_STRIDE + col * 4) = acc[tm][tn][v];
                }
            }
            __syncthreads();
            // All of a thread's staged chunks and their rows' tokens are read before the first
            // store is issued: as a loop that reads one token, waits, reads one chunk, waits and
            // stores, the band took two LDS round trips per chunk, eight chunks in a row.
            int tok[EP_IT];
            f32x4 val[EP_IT];
#pragma unroll
            for (int j = 0; j < EP_IT; ++j) {
                const int it = tid + j * NT;
                const int r = it / EP_CPR, ch = it % EP_CPR;
                const int row = (r >> 5) * (BM / Cfg::WM) + tm * 32 + (r & 31);
                tok[j] = tile_perm[row];
                val[j] = *(const f32x4 *)(smem + r * EP_STRIDE + ch * 16);
            }
#pragma unroll
            for (int j = 0; j < EP_IT; ++j) {
                const int col = n0 + ((tid + j * NT) % EP_CPR) * 4;
                if (tok[j] >= 0 && col < d_out)
                    // h is written once and not read again here: a streaming store keeps it
                    // from displacing x and W tiles in L2 (measured: -11 % at config 1)
                    __builtin_nontemporal_store(val[j], (f32x4 *)(h + (int64_t)tok[j] * d_out + col));
            }
        }
    }
}

// more than 64 KB of dynamic LDS has to be asked for, once per device (see common.h)
template <class Cfg, bool PACK>
struct GemmKernel {
    static inline LdsRegistrar lds{(const void *)fused_gemm_kernel<Cfg, PACK>, Cfg::LDS_BYTES};
};

template <class Cfg, bool PACK>
hipError_t launch_cfg_pack(const uint16_t *x, const uint16_t *W, const uint16_t *B, const uint16_t *t2,
                           const int32_t *offsets, const int32_t *perm, float *h, int64_t N, int d_in,
                           int d_out, int C, int rank, Mix mix, hipStream_t s) {
    auto kern = fused_gemm_kernel<Cfg, PACK>;
    (void)&GemmKernel<Cfg, PACK>::lds;  // instantiates the registration
    const int tiles_m = (int)((N + Cfg::BM - 1) / Cfg::BM);
    const int tiles_n = (d_out + Cfg::BN - 1) / Cfg::BN;
    const int total = tiles_m * tiles_n;
    const unsigned blocks = (unsigned)(((total + 7) / 8) * 8);
    launch_base_kernel(kern, dim3(blocks), dim3(Cfg::NT), Cfg::LDS_BYTES, s, x, W, B, t2, offsets, perm, h,
                       (int)N, d_in, d_out, C, rank, tiles_m, tiles_n, mix);
    return hipGetLastError();
}

template <class Cfg>
hipError_t launch_cfg(const uint16_t *x, const uint16_t *W, const uint16_t *B, const uint16_t *t2,
                      const int32_t *offsets, const int32_t *perm, float *h, int64_t N, int d_in,
                      int d_out, int C, int rank, Mix mix, hipStream_t s) {
    // narrow adapters share an expand tile: 2R a power of two and at most half a K tile (16 or
    // 32 with 64-deep tiles), t in bucket order
    const int two_r = 2 * mix.k * rank;
    const bool pack = !mix.t_dense && 2 * two_r <= Cfg::BK && (two_r & (two_r - 1)) == 0;
    return pack ? launch_cfg_pack<Cfg, true>(x, W, B, t2, offsets, perm, h, N, d_in, d_out, C, rank, mix, s)
                : launch_cfg_pack<Cfg, false>(x, W, B, t2, offsets, perm, h, N, d_in, d_out, C, rank, mix, s);
}

}  // namespace

// Kernel and tile choice from static shapes only (no host read of the histogram); the
// thresholds are measured crossovers.
constexpr int kSmallBatchMax = 512;  // up to here W is streamed once per 64-row tile by the small-batch kernel
constexpr int kBigMinTiles = 256;    // 256 x 256 tiles as soon as they number one per compute unit
using GemmBig = GemmCfg<256, 256, 2, 4, 64, 2>;
using GemmSmall = GemmCfg<128, 128, 2, 2, 64, 2>;
// 128 x 128 tiles with at most one workgroup per compute unit: a third stage replaces the
// second resident workgroup as the way to cover the load latency
using GemmMid = GemmCfg<128, 128, 2, 2, 64, 3>;
// 128 x 256 tiles, eight wavefronts, three stages, one workgroup per compute unit: for shapes
// with too few 256 x 256 tiles to fill the chip whose 128 x 256 tiles number at most one per
// compute unit.  A K tile moves 48 KB for 128 x 256 x 64 products where two 128 x 128
// workgroups move 64 KB, and the loop runs at the rate at which lines arrive; its start and
// end cost more (one workgroup per unit: nothing overlaps them).  Measured against 128 x 128
// tiles at 4096 x K x 2048: level at K = 2048 (36.7 / 36.5 us), 67.3 / 76.0 us at K = 4096,
// 125.8 / 145.5 us at K = 8192.
using GemmWide = GemmCfg<128, 256, 2, 4, 64, 3>;

bool fused_gemm_sizes_ok(int64_t N, int d_in, int d_out, int force_tile) {
    const bool tiled = force_tile == 128 || force_tile == 256 || (force_tile == 0 && N > kSmallBatchMax);
    if (!tiled) return true;  // the small-batch kernel checks its own offsets
    const uint64_t lim = uint64_t(1) << 32;
    return (uint64_t)N * (uint64_t)d_in * 2 < lim && (uint64_t)d_in * (uint64_t)d_out * 2 < lim;
}

namespace {
// Streaming kernel (64-row tiles, W re-read per row tile) or 128 x 128 tiles, for batches of
// 129 .. 4096 rows?  Both run in rounds of 256 workgroups whose time grows with K; fitted to a
// sweep of 96 shapes (launch timer, rotating inputs; us, K in units of 1024):
//   streaming: ceil(workgroups / 256) * (5.0 + 3.3 K), workgroups = column groups of 64 (of 32
//              when that leaves at most 128) x row tiles of 64;
//   tiles:     8.0 + 6.6 K for up to 256 tiles (one per compute unit), 1.6 times that per 512
//              beyond (two per compute unit); K counts the expand tiles too, 64 k for each of the
//              ~(1 + 128 C / N, at most C) buckets that cross a 128-row tile and each 64 of its 2R
//              (narrow adapters share a tile), and a tie goes to the streaming kernel, whose
//              expand works on 16-row slabs (512 rows, 4096 -> 4096, 8 adapters of rank 64: 45.9
//              against 50.5 us).
// The fixed boundary at 512 rows that this replaces lost up to 1.9x on both sides of it: a
// narrow output (4096 -> 1024) streams faster up to ~1500 rows (19 against 34 us at 576), a wide
// one (1024 -> 8192, 4096 -> 12288) is faster in tiles from ~200 rows on (17 against 32 us at 512).
bool streaming_beats_tiles(int64_t N, int d_in, int d_out, int C, int two_r) {
    // one row of 128 x 128 tiles: level with or behind the streaming kernel on eight of ten shapes
    // (4096 -> 12288 at 97-128 rows: 46-47 against 43-45 us; 2048 -> 16384 the other way, 24 / 30)
    if (N <= 128) return true;
    if (N > 4096) return false;
    // operands beyond the tiled kernel's 32-bit offsets: up to kSmallBatchMax rows the streaming
    // kernel takes them (fused_gemm_sizes_ok refuses them above)
    const uint64_t lim = uint64_t(1) << 32;
    if (N <= kSmallBatchMax && ((uint64_t)N * (uint64_t)d_in * 2 >= lim || (uint64_t)d_in * (uint64_t)d_out * 2 >= lim))
        return true;
    int64_t wgs = (int64_t)((d_out + 63) / 64) * ((N + 63) / 64);
    if (wgs <= 128) wgs *= 2;     // the narrow form: groups of 32 columns
    const int64_t t128 = ((N + 127) / 128) * ((d_out + 127) / 128);
    const int64_t stream = ((wgs + 255) / 256) * (50 * 1024 + 33 * (int64_t)d_in);          // 10 * 1024 * us
    int64_t crossing = 1 + 128 * (int64_t)C / N;  // buckets that cross a 128-row tile
    if (crossing > C) crossing = C;
    const bool share = 2 * two_r <= 64 && (two_r & (two_r - 1)) == 0;  // as launch_cfg packs them
    const int64_t expand_k = share ? ((crossing * two_r + 63) / 64) * 64 : crossing * ((two_r + 63) / 64) * 64;
    const int64_t tile1 = 80 * 1024 + 66 * ((int64_t)d_in + expand_k);
    const int64_t tiles = t128 <= 256 ? tile1 : ((t128 + 511) / 512) * tile1 * 16 / 10;
    return stream * 100 <= tiles * 105;
}
}  // namespace

// force_tile: 0 = the choice below; 64 / 128 / 256 = that row-tile height whatever the shape
// (the tiling ablation compares the choice with fixed tiles).
hipError_t launch_fused_gemm(const uint16_t *x, const uint16_t *W, const uint16_t *B,
                             const uint16_t *t2, const int32_t *offsets, const int32_t *perm,
                             float *h, int64_t N, int d_in, int d_out, int C, int rank, Mix mix,
                             hipStream_t s, int force_tile) {
    if (N == 0) return hipSuccess;
    // the token-order intermediate is read by the tiled kernel only
    if (mix.t_dense && (force_tile == 64 || (force_tile == 0 && N <= kSmallBatchMax) || mix.k != 1))
        return hipErrorInvalidValue;
#define MOLORA_GEMM_ARGS x, W, B, t2, offsets, perm, h, N, d_in, d_out, C, rank, mix, s
    if (force_tile == 64) return launch_small_batch_gemm(MOLORA_GEMM_ARGS);
    if (force_tile == 128) return launch_cfg<GemmSmall>(MOLORA_GEMM_ARGS);
    if (force_tile == 256) return launch_cfg<GemmBig>(MOLORA_GEMM_ARGS);
    // (the token-order intermediate, N > 512, is read by the tiled kernel only)
    if (!mix.t_dense && streaming_beats_tiles(N, d_in, d_out, C, 2 * mix.k * rank))
        return launch_small_batch_gemm(MOLORA_GEMM_ARGS);
    const int64_t t256 = ((N + 255) / 256) * ((d_out + 255) / 256);
    const int64_t t128 = ((N + 127) / 128) * ((d_out + 127) / 128);
    // 256 x 256 tiles from one per compute unit on -- and already when the 128 x 128 tiles would
    // not fit one round of two per compute unit: 544 of them take 56.8 us where the 136 large
    // tiles of the same shape take 43.5 us (4352 x 2048 x 2048; 10-29 % over the whole range of
    // 136 .. 192 large tiles, K = 1024 .. 8192), while 512 take 36.6 us against 42.6 us
    if (t256 >= kBigMinTiles || t128 > 512) return launch_cfg<GemmBig>(MOLORA_GEMM_ARGS);
    // with fewer, 128 x 128 tiles keep more of the chip busy
    if (t128 <= 256) return launch_cfg<GemmMid>(MOLORA_GEMM_ARGS);
    const int64_t twide = ((N + 127) / 128) * ((d_out + 255) / 256);
    if (twide <= 256 && d_in >= 3072) return launch_cfg<GemmWide>(MOLORA_GEMM_ARGS);
    return launch_cfg<GemmSmall>(MOLORA_GEMM_ARGS);
#undef MOLORA_GEMM_ARGS
}

}  // namespace molora
