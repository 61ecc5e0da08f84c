// The grouped shrink t_p = x_{perm[p]} A_{c(p)} as a device function, shared by the shrink
// kernels (shrink.hip) and by the kernel that runs its token-order form beside the dispatch
// step in one launch (dispatch_shrink.hip).  See shrink.hip for the method.
#pragma once
#include "common.h"

namespace molora {
namespace {

constexpr int kStepK = 32;       // k per MFMA step
constexpr int kShrinkTinyMax = 64;  // batches up to this size take the many-wavefront form

// R = mix.k * rank is the width of a bucket's intermediate: piece j of it is x A of the j-th
// adapter of the bucket's tuple, scaled by the token's j-th mixture weight.
// NJ = number of 16-column blocks covering R; RB = 16-row blocks per work item (2 for large
// batches, 1 when 32-row items would leave compute units without work); KW = wavefronts of a
// workgroup = K splits, kDepth = steps in flight per wavefront.  A batch of a few dozen tokens
// has a handful of work items and is bound by the chain of load round trips of one wavefront:
// it takes 16 wavefronts x 8 steps, which puts a whole 4096-long row in flight at once.
// DENSE: the token-order form.  No bucketing is looked at: work item `block` is the 16 * RB
// consecutive TOKENS from block * 16 * RB on (n_dense tokens in all), and the intermediate is
// x times ALL C adapters side by side, R = C * rank wide, written per token as
// [hi of adapter 0 .. hi of adapter C-1 | lo of adapter 0 .. ]; the expand step then picks a
// row's adapter.  It costs C times the arithmetic of the grouped form, which the step, bound
// by reading x, does not notice for a few narrow adapters, and it can run beside the dispatch
// step instead of after it.
template <int NJ, int RB, int KW, int kDepth, bool DENSE>
__device__ __forceinline__ void shrink_body(
    const uint16_t *__restrict__ x, const uint16_t *__restrict__ A,
    const int32_t *__restrict__ offsets, const int32_t *__restrict__ perm,
    uint16_t *__restrict__ t2, int d_in, int C, int rank, Mix mix, int block, int n_dense) {
    const int R = DENSE ? C * rank : mix.k * rank;
    constexpr int kShrinkRows = 16 * RB;                 // sorted rows per work item
    constexpr int RP = NJ * 16;                          // padded rank
    constexpr int ROWB = RP * 2 + (RP >= 64 ? 32 : 0);   // LDS bytes per slab row (bank shift)
    constexpr int SLABB = kStepK * ROWB;                 // one step's slab of one wavefront
    constexpr int kShrinkThreads = 64 * KW;
    constexpr int RED_FLOATS = KW * kShrinkRows * RP;    // partial sums of the KW wavefronts
    constexpr int LDS_BYTES = (KW * 2 * SLABB > RED_FLOATS * 4) ? KW * 2 * SLABB : RED_FLOATS * 4;
    static_assert(LDS_BYTES <= 128 * 1024, "LDS");
    __shared__ __attribute__((aligned(16))) unsigned char lds[LDS_BYTES];
    __shared__ int32_t item[3];  // bucket, first sorted row, end row

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);

    // ---- which (bucket, 32-row chunk) is this workgroup? ----
    if (DENSE) {
        if (tid == 0) {
            item[0] = block * kShrinkRows < n_dense ? 0 : -1;
            item[1] = block * kShrinkRows;
            item[2] = n_dense;
        }
    } else if (wave == 0) {
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
            const int rel = block - first;
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

    // ---- this wavefront's k range (a multiple of 32 long) and operand addresses ----
    const int kq_len = ((d_in + KW * kStepK - 1) / (KW * kStepK)) * kStepK;
    const int k_begin = wave * kq_len;
    const int k_end = min(d_in, k_begin + kq_len);
    const int nsteps = k_begin < k_end ? (k_end - k_begin + kStepK - 1) / kStepK : 0;

    const int l16 = lane & 15, kg = lane >> 4;
    // x rows of this lane in the two 16-row blocks; a row past the chunk's end re-reads the
    // first row (its result is never stored), k past d_in is clamped and meets a zeroed A.
    const uint16_t *xrow[RB];
#pragma unroll
    for (int rb = 0; rb < RB; ++rb) {
        const int p = p_first + rb * 16 + l16;
        const int pp = p < p_end ? p : p_first;
        xrow[rb] = x + (int64_t)(DENSE ? pp : perm[pp]) * d_in;
    }
    // A slab staging: lane loads NJ pieces of 16 bytes of the step's [32][R] slab
    // piece id = lane + 64*m -> slab row id / (RP/8), 8-column group id % (RP/8); a group of
    // 8 columns lies inside one adapter of the tuple (rank is a multiple of 8)
    const uint16_t *acol[NJ];
#pragma unroll
    for (int m = 0; m < NJ; ++m) {
        const int u = (lane + 64 * m) % (RP / 8);
        const int uc = min(u * 8, R - 8);
        acol[m] = A + (int64_t)(DENSE ? uc / rank : mix_adapter(mix, c, uc / rank)) * d_in * rank + uc % rank;
    }
    unsigned char *slab0 = lds + wave * 2 * SLABB;

    u32x4 xg[kDepth][RB], ag[kDepth][NJ];
    // Loads are never predicated (addresses are clamped; what came from a clamped address is
    // zeroed when the slab is written, kDepth steps later) and nothing here touches the loaded
    // registers, so that a whole ring of steps really is in flight.
    auto load_step = [&](int slot, int s) {  // step s of this wavefront into ring slot
        const int k0 = k_begin + s * kStepK;
        const int kx = min(k0 + kg * 8, d_in - 8);
#pragma unroll
        for (int rb = 0; rb < RB; ++rb) xg[slot][rb] = *(const u32x4 *)(xrow[rb] + kx);
#pragma unroll
        for (int m = 0; m < NJ; ++m) {
            const int id = lane + 64 * m;
            const int kr = id / (RP / 8);
            ag[slot][m] = *(const u32x4 *)(acol[m] + (int64_t)min(k0 + kr, d_in - 1) * rank);
        }
    };

    f32x4 acc[RB][NJ];
#pragma unroll
    for (int rb = 0; rb < RB; ++rb)
#pragma unroll
        for (int j = 0; j < NJ; ++j) acc[rb][j] = f32x4{0.f, 0.f, 0.f, 0.f};

#pragma unroll
    for (int d = 0; d < kDepth; ++d) load_step(d, d);  // loads past the range are harmless

    for (int s0 = 0; s0 < nsteps; s0 += kDepth) {
#pragma unroll
        for (int d = 0; d < kDepth; ++d) {
            const int s = s0 + d;  // steps past nsteps meet an all-zero slab: harmless
            {
                unsigned char *slab = slab0 + (d & 1) * SLABB;
#pragma unroll
                for (int m = 0; m < NJ; ++m) {
                    const int id = lane + 64 * m;
                    const int kr = id / (RP / 8), u = id % (RP / 8);
                    // rows past this wavefront's k range and columns past R read as zero
                    const uint32_t ok = (k_begin + s * kStepK + kr < k_end && u * 8 < R) ? 0xFFFFFFFFu : 0u;
                    const u32x4 v = ag[d][m];
                    *(u32x4 *)(slab + kr * ROWB + u * 16) = u32x4{v[0] & ok, v[1] & ok, v[2] & ok, v[3] & ok};
                }
#pragma unroll
                for (int jb = 0; jb < NJ; ++jb) {
                    // rows kg*8 + {0..3 | 4..7}, columns jb*16 .. +15 of the slab
                    const unsigned char *p0 = slab + (kg * 8 + (l16 >> 2)) * ROWB + jb * 32 + (l16 & 3) * 8;
                    const i16x4 b_lo = lds_read_tr16((const MOLORA_LDS void *)p0);
                    const i16x4 b_hi = lds_read_tr16((const MOLORA_LDS void *)(p0 + 4 * ROWB));
                    const i16x8 b8 = {b_lo[0], b_lo[1], b_lo[2], b_lo[3],
                                      b_hi[0], b_hi[1], b_hi[2], b_hi[3]};
                    const bf16x8 bfrag = __builtin_bit_cast(bf16x8, b8);
#pragma unroll
                    for (int rb = 0; rb < RB; ++rb)
                        acc[rb][jb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(
                            __builtin_bit_cast(bf16x8, xg[d][rb]), bfrag, acc[rb][jb], 0, 0, 0);
                }
                load_step(d, s + kDepth);  // refill the ring slot
                // a step's loads stay where they are written: the scheduler must not gather the
                // refills of a round at its end
                __builtin_amdgcn_sched_barrier(0);
            }
        }
    }

    // ---- add the KW partial sums in a fixed order, split into bf16 hi + lo, store ----
    // acc[rb][jb][v] = t[row rb*16 + kg*4 + v][column jb*16 + l16]
    __syncthreads();  // all wavefronts are done with their slabs
    float *red = (float *)lds;  // [KW][rows][RP]
#pragma unroll
    for (int rb = 0; rb < RB; ++rb)
#pragma unroll
        for (int jb = 0; jb < NJ; ++jb)
#pragma unroll
            for (int v = 0; v < 4; ++v)
                red[(wave * kShrinkRows + rb * 16 + kg * 4 + v) * RP + jb * 16 + l16] = acc[rb][jb][v];
    __syncthreads();
    for (int e = tid; e < kShrinkRows * RP / 2; e += kShrinkThreads) {
        const int row = e / (RP / 2), col = (e % (RP / 2)) * 2;
        const int p = p_first + row;
        if (p >= p_end || col >= R) continue;
        const float wj = (!DENSE && mix.w != nullptr) ? mix.w[(int64_t)perm[p] * mix.k + col / rank] : 1.f;
        uint32_t hi2 = 0, lo2 = 0;
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            float t = 0.f;
#pragma unroll
            for (int w = 0; w < KW; ++w) t += red[(w * kShrinkRows + row) * RP + col + i];
            t *= wj;
            const uint32_t hi = f32_to_bf16_bits(t);
            const uint32_t lo = f32_to_bf16_bits(t - bf16_bits_to_f32(hi));
            hi2 |= hi << (16 * i);
            lo2 |= lo << (16 * i);
        }
        uint16_t *dst = t2 + (int64_t)p * 2 * R;
        *(uint32_t *)(dst + col) = hi2;
        *(uint32_t *)(dst + R + col) = lo2;
    }
}


}  // namespace
}  // namespace molora
