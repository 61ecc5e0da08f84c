// Dispatch step (Sec. "Unified Dispatch Infrastructure", Alg. "Unified Dispatch Kernel") and
// vocabulary routing (Def. "Vocabulary Routing") for gfx950.
//
// The paper's dispatch hands out list positions with atomicAdd, which leaves the order
// inside a target's list to chance.  Here the lists are ordered by token index (a stable
// counting sort), so the output is unique: one workgroup of 16 wavefronts splits the tokens
// into 16 contiguous ranges, every wavefront finds the lanes that share a target with
// wave-wide ballots, the per-(target, wavefront) counts are prefix-summed in LDS in
// (target-major, wavefront-minor) order, and a second sweep writes every token to
// base[target][wavefront] + (number of lower lanes with the same target).  The only atomics
// are LDS adds on counters that belong to one wavefront (used because they need no wait, not
// for exclusion): they execute in issue order, which is token order, so nothing depends on
// timing.
//
// The whole problem (N <= a few 10^4 tokens, <= 131 KB of traffic) is latency bound, which
// is why it is one workgroup and one launch rather than a multi-pass device-wide sort.
#include "common.h"

namespace molora {

namespace {

constexpr int kBucketWaves = 16;
constexpr int kBucketThreads = kBucketWaves * 64;
constexpr int kUnroll = 8;  // token groups whose loads are in flight together

struct VocabBreaks {
    int32_t b[65];
};

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

// Lanes of the wavefront that hold the same key as this lane (key < 2^nbits).
__device__ __forceinline__ uint64_t match_lanes(int key, bool valid, int nbits) {
    uint64_t mask = __ballot(valid);
    for (int bit = 0; bit < nbits; ++bit) {
        const bool one = (key >> bit) & 1;
        const uint64_t m = __ballot(valid && one);
        mask &= one ? m : ~m;
    }
    return mask;
}

__device__ __forceinline__ int lane_id() { return __lane_id(); }

// target of token t: read from r, or (GATE) computed on the spot from the vocabulary index and
// the request's adapter index, c = a * M + m, as Alg. "Compositional Gating Kernel" does
// inside its dispatch kernel (adapter == nullptr: a = 0, the plain vocabulary route)
struct GateArgs {
    const int32_t *v;
    const int32_t *adapter;
    int32_t *r_out;
    int M, n_adapters;
    VocabBreaks br;
};
// my_b: break b[lane] in lane `lane` (lanes 0 .. 63), b_top = b[M]: read once per kernel; a
// break is then a lane read, not a scalar load from the argument block per token group
template <bool GATE>
__device__ __forceinline__ int32_t target_of(const int32_t *__restrict__ r, const GateArgs &g,
                                             int32_t my_b, int32_t b_top, int t) {
    if constexpr (!GATE) {
        return r[t];
    } else {
        const int32_t id = g.v[t];
        const int32_t a = g.adapter != nullptr ? g.adapter[t] : 0;
        int32_t m = 0;  // breaks ascend: the last j with id >= b[j] is the number of such j >= 1
        for (int j = 1; j < g.M; ++j) m += id >= __builtin_amdgcn_readlane(my_b, j) ? 1 : 0;
        const bool ok = id >= __builtin_amdgcn_readlane(my_b, 0) && id < b_top && a >= 0 && a < g.n_adapters;
        return ok ? a * g.M + m : -1;
    }
}

template <bool GATE>
__global__ __launch_bounds__(kBucketThreads) void bucket_kernel(const int32_t *__restrict__ r,
                                                                int32_t *__restrict__ offsets,
                                                                int32_t *__restrict__ perm, int N,
                                                                int C, int32_t *err_flag,
                                                                GateArgs gate) {
    // cnt[b * 16 + w]: tokens of target b (b == C: out of range) in wavefront w's range
    extern __shared__ int32_t lds[];
    volatile int32_t *cnt = lds;
    int32_t *cnt_rw = lds;  // the same counters, for the LDS atomics of the two sweeps
    __shared__ int32_t wave_tot[kBucketWaves];

    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
    const int E = (C + 1) * kBucketWaves;
    const int nbits = 32 - __clz(C);  // keys are 0..C
    for (int i = tid; i < E; i += kBucketThreads) cnt[i] = 0;
    __syncthreads();

    // contiguous token range of this wavefront, a multiple of 64 long
    const int per = (int)((((int64_t)N + kBucketWaves * 64 - 1) / (kBucketWaves * 64)) * 64);
    const int64_t start64 = (int64_t)w * per;
    const int start = (int)(start64 < N ? start64 : N);
    const int end = (int)(start64 + per < N ? start64 + per : N);
    const uint64_t lower = (lane == 0) ? 0ull : (~0ull >> (64 - lane));

    // a range of at most 64 * kUnroll tokens is one pass of either sweep: the second then
    // reuses the keys of the first instead of reading (and, with a gate, deriving) them again
    const bool one_pass = per <= 64 * kUnroll;
    int32_t key[kUnroll];
    int32_t my_b = 0, b_top = 0;
    if constexpr (GATE) {
        my_b = gate.br.b[lane];
        b_top = gate.br.b[gate.M];
    }

    // ---- sweep 1: histogram per (target, wavefront) ----
    for (int base = start; base < end; base += 64 * kUnroll) {
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) {
            const int t = base + u * 64 + lane;
            const int32_t c = target_of<GATE>(r, gate, my_b, b_top, t < end ? t : end - 1);  // never predicated: all loads in flight
            if (GATE && t < end) gate.r_out[t] = c;
            key[u] = (c >= 0 && c < C) ? c : C;
        }
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) {
            if (base + u * 64 >= end) break;  // wave-uniform: no token in this group
            const bool valid = base + u * 64 + lane < end;
            if (nbits <= 2) {
                // few targets: group the lanes (three ballots), one add per group by its lowest lane
                const uint64_t same = match_lanes(key[u], valid, nbits);
                if (valid && (same & lower) == 0)
                    __hip_atomic_fetch_add(&cnt_rw[key[u] * kBucketWaves + w], __popcll(same),
                                           __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
            } else if (valid) {
                // one LDS add per lane, without return value: nothing to wait for, and integer
                // counts do not depend on the order in which the lanes are served (the sweep is
                // bound by vector instructions on the one compute unit it runs on; grouping the
                // lanes first costs more of them than the serialised adds to equal addresses)
                __hip_atomic_fetch_add(&cnt_rw[key[u] * kBucketWaves + w], 1, __ATOMIC_RELAXED,
                                       __HIP_MEMORY_SCOPE_WORKGROUP);
            }
        }
    }
    __syncthreads();

    // ---- exclusive prefix sum over cnt[0 .. E) ----
    const int chunk = (E + kBucketThreads - 1) / kBucketThreads;
    const int lo = tid * chunk < E ? tid * chunk : E;
    const int hi = lo + chunk < E ? lo + chunk : E;
    int32_t mine = 0;
    for (int i = lo; i < hi; ++i) mine += cnt[i];
    int32_t incl = mine;
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
        const int32_t up = __shfl_up(incl, d, 64);
        if (lane >= d) incl += up;
    }
    if (lane == 63) wave_tot[w] = incl;
    __syncthreads();
    int32_t before = incl - mine;
    for (int j = 0; j < w; ++j) before += wave_tot[j];
    for (int i = lo; i < hi; ++i) {
        const int32_t c = cnt[i];
        cnt[i] = before;
        before += c;
    }
    __syncthreads();
    for (int c = tid; c <= C; c += kBucketThreads) offsets[c] = cnt[c * kBucketWaves];
    if (tid == 0 && err_flag != nullptr && cnt[C * kBucketWaves] != N) *err_flag = 1;
    __syncthreads();

    // ---- sweep 2: scatter token indices to their positions ----
    for (int base = start; base < end; base += 64 * kUnroll) {
        if (!one_pass) {
#pragma unroll
            for (int u = 0; u < kUnroll; ++u) {
                const int t = base + u * 64 + lane;
                const int32_t c = target_of<GATE>(r, gate, my_b, b_top, t < end ? t : end - 1);
                key[u] = (c >= 0 && c < C) ? c : C;
            }
        }
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) {
            if (base + u * 64 >= end) break;  // wave-uniform
            const int t = base + u * 64 + lane;
            const bool valid = t < end;
            const int slot = key[u] * kBucketWaves + w;
            if (nbits <= 2) {
                // few targets: the group's lowest lane takes the group's positions with one
                // returning LDS add and hands the base to the other lanes of the group
                const uint64_t same = match_lanes(key[u], valid, nbits);
                int32_t got = 0;
                if (valid && (same & lower) == 0)
                    got = __hip_atomic_fetch_add(&cnt_rw[slot], __popcll(same), __ATOMIC_RELAXED,
                                                 __HIP_MEMORY_SCOPE_WORKGROUP);
                const int first = same ? __ffsll((long long)same) - 1 : 0;
                const int32_t base_pos = __shfl(got, first, 64);
                if (valid) perm[base_pos + __popcll(same & lower)] = t;
            } else if (valid) {
                // one returning LDS add per lane.  Lanes of one instruction that add to the same
                // address are served in ascending lane order on this hardware (measured: no
                // exception in 6e7 wave-wide adds with random targets and random inactive lanes),
                // and successive instructions execute in issue order, so the positions come out
                // in token order; the bit-exact comparison with a stable sort in the parity tests
                // checks exactly this on every run.
                const int32_t pos = __hip_atomic_fetch_add(&cnt_rw[slot], 1, __ATOMIC_RELAXED,
                                                           __HIP_MEMORY_SCOPE_WORKGROUP);
                perm[pos] = t;
            }
        }
    }
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
    const size_t lds_bytes = (size_t)(C + 1) * kBucketWaves * sizeof(int32_t);
    hipLaunchKernelGGL(bucket_kernel<false>, dim3(1), dim3(kBucketThreads), lds_bytes, s, r, offsets,
                       perm, (int)N, C, err_flag, GateArgs{});
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
    const size_t lds_bytes = (size_t)(C + 1) * kBucketWaves * sizeof(int32_t);
    hipLaunchKernelGGL(bucket_kernel<true>, dim3(1), dim3(kBucketThreads), lds_bytes, s, nullptr,
                       offsets, perm, (int)N, C, err_flag, g);
    return hipGetLastError();
}

}  // namespace molora
