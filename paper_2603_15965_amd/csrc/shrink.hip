// Grouped shrink:  t_p = x_{perm[p]} A_{c(p)}  for every routed sorted position p (the
// "x A_{r(i)}" factor of Eq. "pertok", evaluated group by group as in the paper's grouped
// GEMM over buckets).
//
// The step is HBM bound (2*rank flops per 2 bytes of x), so the kernel is organised around
// streaming x: a work item is 64 consecutive sorted rows of one bucket; each of the 4
// wavefronts owns 16 rows and pulls them from HBM directly in the bf16 MFMA operand layout
// (4 lanes x 16 B = 64 contiguous bytes per row and instruction, prefetched one k-slab
// ahead).  The bucket's A_c is staged k-slab by k-slab in LDS, shared by the 4 wavefronts,
// and read back with the LDS transpose read so that the row-major [k][rank] slab becomes the
// "8 consecutive k per lane" operand.  Accumulation is fp32 (v_mfma_f32_16x16x32_bf16).
//
// The result is written as two bf16 halves, t = hi + lo with hi = bf16(t) and
// lo = bf16(t - hi), laid out [N][2*rank] = [hi | lo], so the expand step can feed it to a
// bf16 MFMA as a K = 2*rank contraction against [B_c; B_c] without losing t's fp32 precision.
#include "common.h"

namespace molora {

namespace {

constexpr int kShrinkThreads = 256;
constexpr int kShrinkRows = 64;   // sorted rows per work item (16 per wavefront)
constexpr int kSlabK = 128;       // k per A slab

template <int NJ>  // NJ = number of 16-column blocks covering rank
__global__ __launch_bounds__(kShrinkThreads) void shrink_kernel(
    const uint16_t *__restrict__ x, const uint16_t *__restrict__ A,
    const int32_t *__restrict__ offsets, const int32_t *__restrict__ perm,
    uint16_t *__restrict__ t2, int d_in, int C, int rank) {
    constexpr int RP = NJ * 16;                 // padded rank (LDS row length)
    constexpr int ROWB = RP * 2;                // bytes per LDS row
    constexpr int SLABB = kSlabK * ROWB;        // bytes per slab
    constexpr int CHUNKS = kSlabK * (RP / 8);   // 16-byte chunks per slab
    constexpr int CPT = (CHUNKS + kShrinkThreads - 1) / kShrinkThreads;
    __shared__ __attribute__((aligned(16))) unsigned char slab_mem[2 * SLABB];
    __shared__ int32_t item[3];  // bucket, first sorted row, end row

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;

    // ---- which (bucket, 64-row chunk) is this workgroup? ----
    if (wave == 0) {
        int found_c = -1, found_lo = 0, found_hi = 0;
        int running = 0;  // work items of the buckets before the current group of 64
        for (int c0 = 0; c0 < C && found_c < 0; c0 += 64) {
            const int c = c0 + lane;
            int lo = 0, hi = 0;
            if (c < C) {
                lo = offsets[c];
                hi = offsets[c + 1];
            }
            const int items = (hi - lo + kShrinkRows - 1) / kShrinkRows;
            int incl = items;
#pragma unroll
            for (int d = 1; d < 64; d <<= 1) {
                const int up = __shfl_up(incl, d, 64);
                if (lane >= d) incl += up;
            }
            const int first = running + incl - items;
            const int rel = (int)blockIdx.x - first;
            const bool hit = rel >= 0 && rel < items;
            const uint64_t m = __ballot(hit);
            if (m) {
                const int src = __ffsll((long long)m) - 1;
                found_c = __shfl(c, src, 64);
                found_lo = __shfl(lo + rel * kShrinkRows, src, 64);
                found_hi = __shfl(hi, src, 64);
            }
            running += __shfl(incl, 63, 64);
        }
        if (lane == 0) {
            item[0] = found_c;
            item[1] = found_lo;
            item[2] = found_hi;
        }
    }
    __syncthreads();
    const int c = item[0];
    if (c < 0) return;  // more workgroups than work items
    const int p_first = item[1];
    const int p_end = min(item[2], p_first + kShrinkRows);

    // ---- this lane's x row (A operand of the 16x16x32 MFMA: row lane%16, k-group lane/16) ----
    const int p_lane = p_first + wave * 16 + (lane & 15);
    const bool row_ok = p_lane < p_end;
    const uint16_t *xrow = x + (int64_t)(row_ok ? perm[p_lane] : 0) * d_in + (lane >> 4) * 8;
    const uint16_t *Ac = A + (int64_t)c * d_in * rank;

    constexpr int XL = kSlabK / 32;  // x loads (k-steps) per slab
    u32x4 xcur[XL], xnext[XL];
    auto x_load = [&](u32x4(&dst)[XL], int k0) {
#pragma unroll
        for (int j = 0; j < XL; ++j) {
            const int k = k0 + j * 32 + (lane >> 4) * 8;
            dst[j] = (row_ok && k < d_in) ? *(const u32x4 *)(xrow + k0 + j * 32)
                                          : u32x4{0u, 0u, 0u, 0u};
        }
    };
    u32x4 areg[CPT];
    auto a_load = [&](int k0) {
#pragma unroll
        for (int m = 0; m < CPT; ++m) {
            const int id = tid + m * kShrinkThreads;
            const int kr = id / (RP / 8), u = id % (RP / 8);
            const int k = k0 + kr;
            areg[m] = (id < CHUNKS && k < d_in && u * 8 < rank)
                          ? *(const u32x4 *)(Ac + (int64_t)k * rank + u * 8)
                          : u32x4{0u, 0u, 0u, 0u};
        }
    };
    auto a_store = [&](unsigned char *slab) {
#pragma unroll
        for (int m = 0; m < CPT; ++m) {
            const int id = tid + m * kShrinkThreads;
            if (id < CHUNKS) *(u32x4 *)(slab + id * 16) = areg[m];
        }
    };

    f32x4 acc[NJ];
#pragma unroll
    for (int j = 0; j < NJ; ++j) acc[j] = f32x4{0.f, 0.f, 0.f, 0.f};

    a_load(0);
    x_load(xcur, 0);
    a_store(slab_mem);
    __syncthreads();

    const int nslab = (d_in + kSlabK - 1) / kSlabK;
    const int a16 = lane & 15, kg = lane >> 4;
    for (int sl = 0; sl < nslab; ++sl) {
        const unsigned char *slab = slab_mem + (sl & 1) * SLABB;
        if (sl + 1 < nslab) a_load((sl + 1) * kSlabK);
        x_load(xnext, (sl + 1) * kSlabK);  // guarded by k < d_in
#pragma unroll
        for (int ks = 0; ks < XL; ++ks) {
            const bf16x8 afrag = __builtin_bit_cast(bf16x8, xcur[ks]);
#pragma unroll
            for (int jb = 0; jb < NJ; ++jb) {
                // rows ks*32 + kg*8 + {0..3 | 4..7}, columns jb*16 .. +15 of the slab
                const int krow = ks * 32 + kg * 8 + (a16 >> 2);
                const unsigned char *p0 = slab + krow * ROWB + jb * 32 + (a16 & 3) * 8;
                const i16x4 b_lo = lds_read_tr16((const MOLORA_LDS void *)p0);
                const i16x4 b_hi = lds_read_tr16((const MOLORA_LDS void *)(p0 + 4 * ROWB));
                const i16x8 b8 = {b_lo[0], b_lo[1], b_lo[2], b_lo[3], b_hi[0], b_hi[1], b_hi[2], b_hi[3]};
                acc[jb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(
                    afrag, __builtin_bit_cast(bf16x8, b8), acc[jb], 0, 0, 0);
            }
        }
#pragma unroll
        for (int j = 0; j < XL; ++j) xcur[j] = xnext[j];
        if (sl + 1 < nslab) a_store(slab_mem + ((sl + 1) & 1) * SLABB);
        __syncthreads();
    }

    // ---- epilogue: split t into bf16 hi + lo and store [hi | lo] ----
    // acc[jb][v] = t[row (lane/16)*4 + v][column jb*16 + lane%16] of this wavefront's 16 rows
#pragma unroll
    for (int jb = 0; jb < NJ; ++jb) {
        const int col = jb * 16 + (lane & 15);
#pragma unroll
        for (int v = 0; v < 4; ++v) {
            const int p = p_first + wave * 16 + (lane >> 4) * 4 + v;
            if (p < p_end && col < rank) {
                const float t = acc[jb][v];
                const uint32_t hi = f32_to_bf16_bits(t);
                const uint32_t lo = f32_to_bf16_bits(t - bf16_bits_to_f32(hi));
                uint16_t *dst = t2 + (int64_t)p * 2 * rank;
                dst[col] = (uint16_t)hi;
                dst[rank + col] = (uint16_t)lo;
            }
        }
    }
}

}  // namespace

hipError_t launch_shrink(const uint16_t *x, const uint16_t *A, const int32_t *offsets,
                         const int32_t *perm, uint16_t *t2, int64_t N, int d_in, int C, int rank,
                         hipStream_t s) {
    if (N == 0) return hipSuccess;
    const unsigned blocks = (unsigned)((N + kShrinkRows - 1) / kShrinkRows + C);
    const int nj = (rank + 15) / 16;
#define MOLORA_SHRINK_CASE(NJ)                                                                  \
    case NJ:                                                                                    \
        hipLaunchKernelGGL(shrink_kernel<NJ>, dim3(blocks), dim3(kShrinkThreads), 0, s, x, A,   \
                           offsets, perm, t2, d_in, C, rank);                                   \
        break;
    switch (nj) {
        MOLORA_SHRINK_CASE(1)
        MOLORA_SHRINK_CASE(2)
        MOLORA_SHRINK_CASE(3)
        MOLORA_SHRINK_CASE(4)
        MOLORA_SHRINK_CASE(5)
        MOLORA_SHRINK_CASE(6)
        MOLORA_SHRINK_CASE(7)
        MOLORA_SHRINK_CASE(8)
        default:
            return hipErrorInvalidValue;
    }
#undef MOLORA_SHRINK_CASE
    return hipGetLastError();
}

}  // namespace molora
