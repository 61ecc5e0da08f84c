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

constexpr int kMaskMaxKeys = 256;  // keys (targets + 1) up to which sweep 2 uses LDS lane masks

// LDS layout for `keys` = C + 1 keys (key C: target out of range)
struct BucketLds {
    int keys;
    bool masks;
    __host__ __device__ explicit BucketLds(int C) : keys(C + 1), masks(C + 1 > 4 && C + 1 <= kMaskMaxKeys) {}
    __host__ __device__ size_t cnt_off() const { return 0; }                                    // [keys][16]
    __host__ __device__ size_t pre_off() const { return (size_t)keys * kBucketWaves * 4; }     // [keys]
    __host__ __device__ size_t post_off() const { return pre_off() + (size_t)keys * 4; }       // [keys]
    __host__ __device__ size_t tot_off() const { return post_off() + (size_t)keys * 4; }       // [keys]
    __host__ __device__ size_t mask_off() const { return (tot_off() + (size_t)keys * 4 + 7) & ~size_t(7); }
    __host__ __device__ size_t bytes() const {
        return mask_off() + (masks ? (size_t)keys * kBucketWaves * 8 : 0);
    }
};

template <bool GATE>
__global__ __launch_bounds__(kBucketThreads) void bucket_kernel(const int32_t *__restrict__ r,
                                                                int32_t *__restrict__ offsets,
                                                                int32_t *__restrict__ perm, int N,
                                                                int C, int32_t *err_flag,
                                                                GateArgs gate) {
    extern __shared__ __attribute__((aligned(16))) unsigned char lds_raw[];
    const BucketLds L(C);
    int32_t *cnt = (int32_t *)(lds_raw + L.cnt_off());    // cnt[b * 16 + w]: own part, by wavefront
    int32_t *pre = (int32_t *)(lds_raw + L.pre_off());    // tokens of target b before the own part
    int32_t *post = (int32_t *)(lds_raw + L.post_off());  // ... after it
    int32_t *tot = (int32_t *)(lds_raw + L.tot_off());    // per-target totals, then their prefix
    uint64_t *mask = (uint64_t *)(lds_raw + L.mask_off());  // mask[w * keys + b]: lanes of the step with target b
    __shared__ int32_t wave_tot[kBucketWaves];

    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
    const int keys = C + 1;
    const int nbits = 32 - __clz(C);  // keys are 0..C
    {
        int32_t *z = (int32_t *)lds_raw;
        const int words = (int)(L.bytes() / 4);
        for (int i = tid; i < words; i += kBucketThreads) z[i] = 0;
    }
    __syncthreads();

    // contiguous token range of this wavefront, a multiple of 64 long; the workgroup's own part
    // is the 16 ranges of its wavefronts
    const int G = gridDim.x, g = blockIdx.x;
    const int per = (int)((((int64_t)N + (int64_t)G * kBucketWaves * 64 - 1) / ((int64_t)G * kBucketWaves * 64)) * 64);
    const int64_t own64 = (int64_t)g * kBucketWaves * per;
    const int own_lo = (int)(own64 < N ? own64 : N);
    const int own_hi = (int)(own64 + (int64_t)kBucketWaves * per < N ? own64 + (int64_t)kBucketWaves * per : N);
    const int64_t start64 = own64 + (int64_t)w * per;
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

    // ---- sweep 1a: histogram of the own part per (target, wavefront) ----
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
                    __hip_atomic_fetch_add(&cnt[key[u] * kBucketWaves + w], __popcll(same),
                                           __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
            } else if (valid) {
                // one LDS add per lane, without return value: nothing to wait for, and a count
                // does not depend on the order in which the lanes are served
                __hip_atomic_fetch_add(&cnt[key[u] * kBucketWaves + w], 1, __ATOMIC_RELAXED,
                                       __HIP_MEMORY_SCOPE_WORKGROUP);
            }
        }
    }
    // ---- sweep 1b: the tokens of the other workgroups' parts, before / after the own part ----
    const int n_other = N - (own_hi - own_lo);
    if (n_other > 0) {  // more than one workgroup
        for (int base = 0; base < n_other; base += kBucketThreads * kUnroll) {
            int32_t k2[kUnroll];
#pragma unroll
            for (int u = 0; u < kUnroll; ++u) {
                int i = base + u * kBucketThreads + tid;
                i = i < n_other ? i : n_other - 1;
                const int t = i < own_lo ? i : i + (own_hi - own_lo);
                const int32_t c = target_of<GATE>(r, gate, my_b, b_top, t);
                k2[u] = (c >= 0 && c < C) ? c : C;
            }
#pragma unroll
            for (int u = 0; u < kUnroll; ++u) {
                const int i = base + u * kBucketThreads + tid;
                if (i < n_other)
                    __hip_atomic_fetch_add(i < own_lo ? &pre[k2[u]] : &post[k2[u]], 1, __ATOMIC_RELAXED,
                                           __HIP_MEMORY_SCOPE_WORKGROUP);
            }
        }
    }
    __syncthreads();

    // ---- totals per target, their exclusive prefix (= offsets), first positions ----
    const int chunk = (keys + kBucketThreads - 1) / kBucketThreads;
    const int lo = tid * chunk < keys ? tid * chunk : keys;
    const int hi = lo + chunk < keys ? lo + chunk : keys;
    int32_t mine = 0;
    for (int b = lo; b < hi; ++b) {
        int32_t sum = pre[b] + post[b];
#pragma unroll
        for (int j = 0; j < kBucketWaves; ++j) sum += cnt[b * kBucketWaves + j];
        tot[b] = sum;
        mine += sum;
    }
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
    for (int b = lo; b < hi; ++b) {
        const int32_t total = tot[b];
        if (g == 0) offsets[b] = before;
        // cnt[b][j] becomes the first position of wavefront j's tokens of target b
        int32_t run = before + pre[b];
#pragma unroll
        for (int j = 0; j < kBucketWaves; ++j) {
            const int32_t c = cnt[b * kBucketWaves + j];
            cnt[b * kBucketWaves + j] = run;
            run += c;
        }
        // offsets[C] counts the routed tokens: fewer than N means some target was out of range
        if (b == C && g == 0 && err_flag != nullptr && before != N) *err_flag = 1;
        before += total;
    }
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
        if (L.masks) {
            // every step: OR the own bit into the (wavefront, target) word, read the word, clear
            // the bit again; read the running base, advance it by one per lane.  All of one
            // wavefront, executed in issue order, so the steps can be issued back to back.
            uint64_t m[kUnroll];
            int32_t first[kUnroll];
            uint64_t *my_mask = mask + w * keys;
            const uint64_t bit = 1ull << lane;
#pragma unroll
            for (int u = 0; u < kUnroll; ++u) {
                m[u] = 0;
                first[u] = 0;
                if (base + u * 64 + lane < end) {
                    uint64_t *mp = my_mask + key[u];
                    int32_t *cp = &cnt[key[u] * kBucketWaves + w];
                    __hip_atomic_fetch_or(mp, bit, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
                    m[u] = __hip_atomic_load(mp, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
                    __hip_atomic_fetch_and(mp, ~bit, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
                    first[u] = __hip_atomic_load(cp, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
                    __hip_atomic_fetch_add(cp, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
                }
            }
#pragma unroll
            for (int u = 0; u < kUnroll; ++u) {
                const int t = base + u * 64 + lane;
                if (t < end) perm[first[u] + __popcll(m[u] & lower)] = t;
            }
            continue;
        }
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) {
            if (base + u * 64 >= end) break;  // wave-uniform
            const int t = base + u * 64 + lane;
            const bool valid = t < end;
            // lanes with the same target from ballots; the group's lowest lane takes the group's
            // positions with one returning LDS add and hands the base to the other lanes
            const uint64_t same = match_lanes(key[u], valid, nbits);
            int32_t got = 0;
            if (valid && (same & lower) == 0)
                got = __hip_atomic_fetch_add(&cnt[key[u] * kBucketWaves + w], __popcll(same),
                                             __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
            const int first = same ? __ffsll((long long)same) - 1 : 0;
            const int32_t base_pos = __shfl(got, first, 64);
            if (valid) perm[base_pos + __popcll(same & lower)] = t;
        }
    }
}

// more than 64 KB of dynamic LDS has to be asked for, once per device (see common.h)
LdsRegistrar g_bucket_lds{(const void *)bucket_kernel<false>, BucketLds(MOLORA_MAX_TARGETS).bytes()};
LdsRegistrar g_gate_bucket_lds{(const void *)bucket_kernel<true>, BucketLds(MOLORA_MAX_TARGETS).bytes()};

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
                       BucketLds(C).bytes(), s, r, offsets, perm, (int)N, C, err_flag, GateArgs{});
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
                       BucketLds(C).bytes(), s, nullptr, offsets, perm, (int)N, C, err_flag, g);
    return hipGetLastError();
}

}  // namespace molora
