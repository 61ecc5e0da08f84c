// The dispatch step (Sec. "Unified Dispatch Infrastructure", Alg. "Unified Dispatch Kernel") as a
// device function, shared by the dispatch kernels (bucket.hip) and by the kernel that runs the
// dispatch beside the token-order shrink in one launch (dispatch_shrink.hip).  See bucket.hip
// for the method.
#pragma once
#include "common.h"

namespace molora {
namespace {


constexpr int kUnroll = 8;  // token groups whose loads are in flight together

struct VocabBreaks {
    int32_t b[65];
};

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

// Target of token t: read from r, or (GATE) computed on the spot from the vocabulary index and
// the request's adapter index, c = a * M + m, as Alg. "Compositional Gating Kernel" does
// inside its dispatch kernel (adapter == nullptr: a = 0, the plain vocabulary route).
// In two halves, so that a batch of tokens is FETCHED first and EVALUATED afterwards: the
// evaluation loops over the breaks, and a loop between two loads makes the compiler wait for
// the first load before it issues the second (one trip to memory per token instead of one per
// batch).
struct GateArgs {
    const int32_t *v;
    const int32_t *adapter;
    int32_t *r_out;
    int M, n_adapters;
    VocabBreaks br;
};
struct RawTarget {
    int32_t id;  // r[t], or the vocabulary index v[t]
    int32_t a;   // the request's adapter index (GATE with adapters), else 0
};
template <bool GATE>
__device__ __forceinline__ RawTarget fetch_target(const int32_t *__restrict__ r, const GateArgs &g, int t) {
    if constexpr (!GATE) {
        return RawTarget{r[t], 0};
    } else {
        return RawTarget{g.v[t], g.adapter != nullptr ? g.adapter[t] : 0};
    }
}
// my_b: break b[lane] in lane `lane` (lanes 0 .. 63), b_top = b[M]: read once per kernel; a
// break is then a lane read, not a scalar load from the argument block per token group
template <bool GATE>
__device__ __forceinline__ int32_t eval_target(const GateArgs &g, int32_t my_b, int32_t b_top, RawTarget raw) {
    if constexpr (!GATE) {
        return raw.id;
    } else {
        const int32_t id = raw.id, a = raw.a;
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
    int kBucketWaves;  // wavefronts per workgroup
    bool masks;
    __host__ __device__ BucketLds(int C, int waves) : keys(C + 1), kBucketWaves(waves), masks(C + 1 > 4 && C + 1 <= kMaskMaxKeys) {}
    // a row of cnt is one word longer than the wavefronts number: the lanes of a wavefront all
    // address column w, and with rows of 16 words they would share two banks
    __host__ __device__ size_t cnt_off() const { return 0; }                                      // [keys][waves + 1]
    __host__ __device__ size_t pre_off() const { return (size_t)keys * (kBucketWaves + 1) * 4; } // [keys]
    __host__ __device__ size_t post_off() const { return pre_off() + (size_t)keys * 4; }       // [keys]
    __host__ __device__ size_t tot_off() const { return post_off() + (size_t)keys * 4; }       // [keys]
    __host__ __device__ size_t mask_off() const { return (tot_off() + (size_t)keys * 4 + 7) & ~size_t(7); }
    __host__ __device__ size_t bytes() const {
        return mask_off() + (masks ? (size_t)keys * kBucketWaves * 8 : 0);
    }
};

// The dispatch step as run by workgroup g of G, each of BW wavefronts (BW * 64 threads).
// EARLY: the first 16 tokens per thread of the other workgroups' parts are read before the own
// part instead of after it, so that both reads are in flight together: one trip to memory
// less, which pays when the memory system is busy with something else (the shrink running
// beside the dispatch in one launch); run alone, the shorter code of the plain order is faster.
template <bool GATE, int BW, bool EARLY = false>
__device__ __forceinline__ void bucket_body(const int32_t *__restrict__ r, int32_t *__restrict__ offsets,
                                            int32_t *__restrict__ perm, int N, int C, int32_t *err_flag,
                                            const GateArgs &gate, int G, int g) {
    constexpr int kBucketWaves = BW, kBucketThreads = BW * 64;
    constexpr int kCntRow = BW + 1;  // words per row of cnt (see BucketLds)
    extern __shared__ __attribute__((aligned(16))) unsigned char lds_raw[];
    const BucketLds L(C, BW);
    int32_t *cnt = (int32_t *)(lds_raw + L.cnt_off());    // cnt[b * kCntRow + w]: own part, by wavefront
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

    // the tokens outside the own part, numbered 0 .. n_other - 1: key of the i-th (index clamped:
    // never predicated), and its count into pre / post
    const int n_other = N - (own_hi - own_lo);
    auto other_raw = [&](int i) {
        i = i < n_other ? i : n_other - 1;
        return fetch_target<GATE>(r, gate, i < own_lo ? i : i + (own_hi - own_lo));
    };
    auto key_of = [&](RawTarget raw) {
        const int32_t c = eval_target<GATE>(gate, my_b, b_top, raw);
        return (c >= 0 && c < C) ? c : C;
    };
    // (all lanes of the wavefront call it together)
    auto count_other = [&](int i, int32_t k) {
        const bool in = i < n_other;
        const int code = i < own_lo ? k : keys + k;  // pre[k] : post[k]
        // one target for the whole group of 64 (skewed or run-structured routing): one add of
        // the group's size by lane 0 instead of 64 adds that the LDS serves one after the other
        // (i grows with the lane: lane 0 is inside whenever any lane is).  No branch: the
        // callers issue a batch of loads before the first call and must stay straight-line.
        // (ballots and the lane-0 read are taken by all lanes, outside any condition; written
        // with masks, not with || and &&, which the compiler turns into branches around them)
        const uint64_t in_m = __ballot(in);
        const bool uni = (__ballot(code != __builtin_amdgcn_readfirstlane(code)) & in_m) == 0;
        const int32_t add = uni ? (lane == 0 ? (int32_t)__popcll(in_m) : 0) : (in ? 1 : 0);
        if (add != 0)
            __hip_atomic_fetch_add(i < own_lo ? &pre[k] : &post[k], add, __ATOMIC_RELAXED,
                                   __HIP_MEMORY_SCOPE_WORKGROUP);
    };
    constexpr int kEarly = 16;
    RawTarget raw_early[kEarly];
    if constexpr (EARLY) {
        if (n_other > 0) {
#pragma unroll
            for (int u = 0; u < kEarly; ++u) raw_early[u] = other_raw(u * kBucketThreads + tid);
        }
    }

    // ---- sweep 1a: histogram of the own part per (target, wavefront) ----
    for (int base = start; base < end; base += 64 * kUnroll) {
        RawTarget raw[kUnroll];
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) {
            const int t = base + u * 64 + lane;
            raw[u] = fetch_target<GATE>(r, gate, t < end ? t : end - 1);  // never predicated: all loads in flight
        }
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) {
            const int t = base + u * 64 + lane;
            const int32_t c = eval_target<GATE>(gate, my_b, b_top, raw[u]);
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
                    __hip_atomic_fetch_add(&cnt[key[u] * kCntRow + w], __popcll(same),
                                           __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
            } else {
                // one LDS add per lane, without return value: nothing to wait for, and a count
                // does not depend on the order in which the lanes are served.  One target for the
                // whole group (lane 0 holds a token whenever the group does): lane 0 adds the
                // group's size instead, as in count_other (same compact form: the kernel is short
                // enough for the size of its code to show in its time).
                const uint64_t vm = __ballot(valid);
                const bool uni = (__ballot(key[u] != __builtin_amdgcn_readfirstlane(key[u])) & vm) == 0;
                const int32_t add = uni ? (lane == 0 ? (int32_t)__popcll(vm) : 0) : (valid ? 1 : 0);
                if (add != 0)
                    __hip_atomic_fetch_add(&cnt[key[u] * kCntRow + w], add, __ATOMIC_RELAXED,
                                           __HIP_MEMORY_SCOPE_WORKGROUP);
            }
        }
    }
    // ---- sweep 1b: the tokens of the other workgroups' parts, before / after the own part ----
    if (n_other > 0) {  // more than one workgroup
        int first = 0;
        if constexpr (EARLY) {
#pragma unroll
            for (int u = 0; u < kEarly; ++u) count_other(u * kBucketThreads + tid, key_of(raw_early[u]));
            first = kEarly * kBucketThreads;
        }
        for (int base = first; base < n_other; base += kBucketThreads * kUnroll) {
            RawTarget raw2[kUnroll];
#pragma unroll
            for (int u = 0; u < kUnroll; ++u) raw2[u] = other_raw(base + u * kBucketThreads + tid);
#pragma unroll
            for (int u = 0; u < kUnroll; ++u) count_other(base + u * kBucketThreads + tid, key_of(raw2[u]));
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
        for (int j = 0; j < kBucketWaves; ++j) sum += cnt[b * kCntRow + j];
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
            const int32_t c = cnt[b * kCntRow + j];
            cnt[b * kCntRow + j] = run;
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
            RawTarget raw[kUnroll];
#pragma unroll
            for (int u = 0; u < kUnroll; ++u) {
                const int t = base + u * 64 + lane;
                raw[u] = fetch_target<GATE>(r, gate, t < end ? t : end - 1);
            }
#pragma unroll
            for (int u = 0; u < kUnroll; ++u) key[u] = key_of(raw[u]);
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
                const bool valid = base + u * 64 + lane < end;
                // one target for the whole group: the mask is the group itself (no mask words
                // touched, which would all be one word), and lane 0 advances the running base
                const uint64_t vm = __ballot(valid);
                const bool uni = (__ballot(key[u] != __builtin_amdgcn_readfirstlane(key[u])) & vm) == 0;
                uint64_t *mp = my_mask + key[u];
                int32_t *cp = &cnt[key[u] * kCntRow + w];
                uint64_t mine = 0;
                if (valid && !uni) {
                    __hip_atomic_fetch_or(mp, bit, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
                    mine = __hip_atomic_load(mp, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
                    __hip_atomic_fetch_and(mp, ~bit, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
                }
                m[u] = uni ? vm : mine;
                const int32_t add = uni ? (lane == 0 ? (int32_t)__popcll(vm) : 0) : 1;
                if (valid) {
                    first[u] = __hip_atomic_load(cp, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
                    if (add != 0)
                        __hip_atomic_fetch_add(cp, add, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
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
                got = __hip_atomic_fetch_add(&cnt[key[u] * kCntRow + w], __popcll(same),
                                             __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
            const int first = same ? __ffsll((long long)same) - 1 : 0;
            const int32_t base_pos = __shfl(got, first, 64);
            if (valid) perm[base_pos + __popcll(same & lower)] = t;
        }
    }
}


}  // namespace
}  // namespace molora
