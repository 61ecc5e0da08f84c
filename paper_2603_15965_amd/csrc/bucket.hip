// Dispatch step (Sec. "Unified Dispatch Infrastructure", Alg. "Unified Dispatch Kernel") and
// vocabulary routing (Def. "Vocabulary Routing") for gfx950.
//
// The paper's dispatch hands out list positions with atomicAdd, which leaves the order
// inside a target's list to chance.  Here the lists are ordered by token index (a stable
// counting sort), so the output is unique, and it is unique BY CONSTRUCTION: nothing in the
// kernel depends on the order in which the hardware serves the lanes of an atomic
// instruction or on timing between wavefronts.
//
//   * The tokens are cut into contiguous ranges, one per wavefront (16 wavefronts per
//     workgroup, 1 to 16 workgroups).  Sweep 1 counts, per target, the tokens of every range of
//     the workgroup's own part (cnt[target][wavefront]) and the tokens before and after the
//     workgroup's part (pre[target], post[target]; every workgroup reads all of r for this,
//     <= 64 KB from L2, instead of waiting for the other workgroups' counts).  Counts are sums
//     of ones: LDS adds whose order does not matter.
//   * offsets[c] is the exclusive prefix of the totals; the first position of wavefront w's
//     tokens of target c is offsets[c] + pre[c] + sum_{w' < w} cnt[c][w'].
//   * Sweep 2: a wavefront walks its range in token order, 64 tokens per step.  Inside a step,
//     a token's place among the lanes with the same target is the number of LOWER lanes with
//     that target, read off a bit mask of those lanes: for up to three targets the mask comes
//     from wave ballots; for up to 255 from an LDS word per (wavefront, target) into which
//     every lane ORs its own bit (OR is commutative: the mask does not depend on the order of
//     service) and which every lane then reads and clears its bit from again; above that from
//     one ballot per bit of the target index.  LDS operations of one wavefront execute in the
//     order they are issued, so the running base of a (wavefront, target) pair, read by all
//     lanes and then advanced, needs no wait either.
//
// The whole problem (N <= a few 10^4 tokens, <= 131 KB of traffic) is latency bound, which
// is why it is one launch of a few workgroups that each recount rather than a multi-pass
// device-wide sort.
#include "../../include/molora.h"

#include "bucket_body.h"

namespace molora {

namespace {

constexpr int kBucketWaves = 16;
constexpr int kBucketThreads = kBucketWaves * 64;

__global__ __launch_bounds__(256) void route_vocab_kernel(const int32_t *__restrict__ v,
                                                          int32_t *__restrict__ r, int64_t N,
                                                          VocabBreaks br, int M) {
    int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= N) return;
    const int32_t id = v[i];
    int32_t m = 0;
    for (int j = 1; j < M; ++j)  // M - 1 integer comparisons
        if (id >= br.b[j]) m = j;
    if (id < br.b[0] || id >= br.b[M]) m = -1;
    r[i] = m;
}

template <bool GATE>
__global__ __launch_bounds__(kBucketThreads) void bucket_kernel(const int32_t *__restrict__ r,
                                                                int32_t *__restrict__ offsets,
                                                                int32_t *__restrict__ perm, int N,
                                                                int C, int32_t *err_flag,
                                                                GateArgs gate) {
    bucket_body<GATE, kBucketWaves>(r, offsets, perm, N, C, err_flag, gate, (int)gridDim.x, (int)blockIdx.x);
}

// more than 64 KB of dynamic LDS has to be asked for, once per device (see common.h)
LdsRegistrar g_bucket_lds{(const void *)bucket_kernel<false>, BucketLds(MOLORA_MAX_TARGETS, kBucketWaves).bytes()};
LdsRegistrar g_gate_bucket_lds{(const void *)bucket_kernel<true>, BucketLds(MOLORA_MAX_TARGETS, kBucketWaves).bytes()};

// Workgroups: every one recounts all tokens and scatters its own part, so more of them pay
// only when the scatter dominates.  Measured (kernel trace, 32 targets): 16384 tokens 19.8 /
// 12.4 / 9.4 / 8.2 / 7.6 us with 1 / 2 / 4 / 8 / 16 workgroups, 8192 tokens 12.7 / 9.1 / 7.1 /
// 6.8 us with 1 / 2 / 4 / 8, 65536 tokens 67 -> 16 us; at 4096 tokens no gain (5.7 us whatever
// the number), and with the gate evaluated in the kernel one workgroup is fastest there.
// Never more workgroups than 1024-token parts, so that every workgroup but the first has
// tokens before its part (and an empty batch gets one workgroup).
inline unsigned bucket_workgroups(int64_t N) {
    if (N <= 4096) return 1;
    const int64_t g = (N + 1023) / 1024;
    return (unsigned)(g > 16 ? 16 : g);
}

}  // namespace

hipError_t launch_route_vocab(const int32_t *v, const int32_t *breaks_host, int M, int32_t *r,
                              int64_t N, hipStream_t s) {
    if (N == 0) return hipSuccess;
    VocabBreaks br;
    for (int j = 0; j <= M; ++j) br.b[j] = breaks_host[j];
    for (int j = M + 1; j < 65; ++j) br.b[j] = 0;
    const unsigned blocks = (unsigned)((N + 255) / 256);
    hipLaunchKernelGGL(route_vocab_kernel, dim3(blocks), dim3(256), 0, s, v, r, N, br, M);
    return hipGetLastError();
}

hipError_t launch_bucket(const int32_t *r, int32_t *offsets, int32_t *perm, int64_t N, int C,
                         int32_t *err_flag, hipStream_t s) {
    hipLaunchKernelGGL(bucket_kernel<false>, dim3(bucket_workgroups(N)), dim3(kBucketThreads),
                       BucketLds(C, kBucketWaves).bytes(), s, r, offsets, perm, (int)N, C, err_flag, GateArgs{});
    return hipGetLastError();
}

hipError_t launch_gate_bucket(const int32_t *v, const int32_t *adapter, const int32_t *breaks_host,
                              int M, int n_adapters, int32_t *r, int32_t *offsets, int32_t *perm,
                              int64_t N, int32_t *err_flag, hipStream_t s) {
    const int C = n_adapters * M;
    GateArgs g;
    g.v = v;
    g.adapter = adapter;
    g.r_out = r;
    g.M = M;
    g.n_adapters = n_adapters;
    for (int j = 0; j <= M; ++j) g.br.b[j] = breaks_host[j];
    for (int j = M + 1; j < 65; ++j) g.br.b[j] = 0;
    hipLaunchKernelGGL(bucket_kernel<true>, dim3(bucket_workgroups(N)), dim3(kBucketThreads),
                       BucketLds(C, kBucketWaves).bytes(), s, nullptr, offsets, perm, (int)N, C, err_flag, g);
    return hipGetLastError();
}

}  // namespace molora
