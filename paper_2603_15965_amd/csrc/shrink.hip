// Grouped shrink:  t_p = x_{perm[p]} A_{c(p)}  for every routed sorted position p (the
// "x A_{r(i)}" factor of Eq. "pertok", evaluated group by group as in the paper's grouped
// GEMM over buckets).
//
// The step is HBM bound (2*rank flops per 2 bytes of x), so the kernel is organised around
// keeping many bytes of x in flight.  A work item is 32 consecutive sorted rows of one
// bucket.  Its 4 wavefronts split the K range four ways (a workgroup per 32 rows gives N/32
// workgroups, enough to cover the chip even at 4096 tokens) and each wavefront streams on
// its own, with no workgroup barrier inside the loop:
//   x    straight from HBM into the bf16 MFMA operand layout (row lane%16, 8 consecutive k
//        per lane: 4 lanes = 64 contiguous bytes per row and instruction), two 16-row blocks;
//   A_c  its k-slice, 32 k at a time, into a wavefront-private LDS buffer and back through
//        the LDS transpose read, which turns the row-major [k][rank] slab into the
//        "8 consecutive k per lane" operand;
//   a ring of kDepth such steps is in flight per wavefront (v_mfma_f32_16x16x32_bf16, fp32
//   accumulate).  The four partial sums are added in a fixed order through LDS.
//
// The result is written as two bf16 halves, t = hi + lo with hi = bf16(t) and
// lo = bf16(t - hi), laid out [N][2*rank] = [hi | lo], so the expand step can feed it to a
// bf16 MFMA as a K = 2*rank contraction against [B_c; B_c] without losing t's fp32 precision.
#include "shrink_body.h"

namespace molora {

namespace {

template <int NJ, int RB, int KW, int kDepth>
__global__ __launch_bounds__(64 * KW) void shrink_kernel(
    const uint16_t *__restrict__ x, const uint16_t *__restrict__ A,
    const int32_t *__restrict__ offsets, const int32_t *__restrict__ perm,
    uint16_t *__restrict__ t2, int d_in, int C, int rank, Mix mix) {
    shrink_body<NJ, RB, KW, kDepth, false>(x, A, offsets, perm, t2, d_in, C, rank, mix, (int)blockIdx.x, 0);
}

}  // namespace

namespace {
// which of the two kernels: see launch_shrink
bool shrink_streams(int64_t N, int d_in, int C, int64_t R) {
    return N <= 64 || (N <= 2048 && d_in * R >= (1 << 17)) ||
           (N * (int64_t)d_in >= (1 << 24) && N >= 128 * (int64_t)C &&
            ((N + 63) / 64) * C <= 32768);  // (not too many buckets: every workgroup scans all offsets)
}
bool shrink_tiny(int64_t N, int64_t R) { return N <= kShrinkTinyMax && (R + 15) / 16 <= 2; }
}  // namespace

size_t shrink_scratch_bytes(int64_t N, int d_in, int C, int R) {
    if (N == 0 || shrink_tiny(N, R) || !shrink_streams(N, d_in, C, R)) return 0;
    const int ks = small_batch_shrink_ksplit(N, d_in, C, R);
    return ks > 1 ? (size_t)ks * (size_t)N * (size_t)R * sizeof(float) : 0;
}

bool sort_in_shrink_ok(int64_t N, int d_in, int C, int rank) {
    return N > 0 && N <= 64 && !shrink_tiny(N, rank) && shrink_streams(N, d_in, C, rank);
}

hipError_t launch_shrink(const uint16_t *x, const uint16_t *A, const int32_t *offsets,
                         const int32_t *perm, uint16_t *t2, int64_t N, int d_in, int C, int rank,
                         Mix mix, hipStream_t s, float *scratch, SortArgs sort) {
    if (N == 0) return hipSuccess;
    if (sort.r != nullptr) {
        if (mix.k != 1 || !sort_in_shrink_ok(N, d_in, C, rank) || !sort.offsets || !sort.perm)
            return hipErrorInvalidValue;
        offsets = sort.offsets;  // what the reduction pass of a K-split shrink reads afterwards
        perm = sort.perm;
    }
    // Two kernels (measured crossovers).  The streaming kernel (one workgroup per 64 rows of a
    // bucket, K split over its 8 wavefronts, x staged as whole 128-byte lines) wins for small
    // batches, which are bound by the latency of streaming the touched A_c, and for large ones
    // whose buckets fill its 64-row tiles (3.2-4.2 TB/s of x against 2.4-2.7 TB/s); the
    // row-item kernel below wins in between and when buckets are small.
    const int64_t R = (int64_t)mix.k * rank;
    const int nj = (mix.k * rank + 15) / 16;
    // a few work items only, narrow intermediate: 16 (8) wavefronts per 16-row item
    if (shrink_tiny(N, R)) {
        const unsigned blocks = (unsigned)((N + 15) / 16 + C);
        if (nj == 1)
            hipLaunchKernelGGL((shrink_kernel<1, 1, 16, 8>), dim3(blocks), dim3(1024), 0, s, x, A,
                               offsets, perm, t2, d_in, C, rank, mix);
        else
            hipLaunchKernelGGL((shrink_kernel<2, 1, 8, 8>), dim3(blocks), dim3(512), 0, s, x, A,
                               offsets, perm, t2, d_in, C, rank, mix);
        return hipGetLastError();
    }
    if (shrink_streams(N, d_in, C, R)) {
        // few (bucket, tile) pairs and a long K: K split over workgroups, when scratch is there
        const int ks = scratch != nullptr ? small_batch_shrink_ksplit(N, d_in, C, (int)R) : 1;
        return launch_small_batch_shrink(x, A, offsets, perm, t2, N, d_in, C, rank, mix, s, scratch, ks, sort);
    }
    // 32-row items when they still cover the chip twice, 16-row items otherwise
    const bool small_items = (N + 31) / 32 + C < 512;
    const int rows = small_items ? 16 : 32;
    const unsigned blocks = (unsigned)((N + rows - 1) / rows + C);
    // fewer items than compute units and a long K: 8 wavefronts split it (measured 11.3 us
    // against 14.9 us at 2048 tokens x 4096, 64 adapters; no gain once every unit has an item)
    const bool wide = blocks <= 256 && d_in >= 4096;
#define MOLORA_SHRINK_CASE(NJ)                                                                      \
    case NJ:                                                                                        \
        if (small_items && wide)                                                                    \
            hipLaunchKernelGGL((shrink_kernel<NJ, 1, (NJ <= 2 ? 8 : 4), 4>), dim3(blocks),          \
                               dim3(64 * (NJ <= 2 ? 8 : 4)), 0, s, x, A, offsets, perm, t2, d_in,   \
                               C, rank, mix);                                                       \
        else if (small_items)                                                                       \
            hipLaunchKernelGGL((shrink_kernel<NJ, 1, 4, 4>), dim3(blocks), dim3(256), 0, s, x, A,   \
                               offsets, perm, t2, d_in, C, rank, mix);                              \
        else                                                                                        \
            hipLaunchKernelGGL((shrink_kernel<NJ, 2, 4, 4>), dim3(blocks), dim3(256), 0, s, x, A,   \
                               offsets, perm, t2, d_in, C, rank, mix);                              \
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
