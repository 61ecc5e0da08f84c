// Learned top-1 routing (Sec. "Router Architecture", k = 1; linear gate of Table
// "tab:moe_adapter"):  r[i] = argmax_c sum_k x[i][k] G[k][c], lowest index on ties.
//
// The result has to be a deterministic function of the input bits, so every logit is the
// strict fp32 chain  acc <- fl(acc + x_k * g_k),  k ascending (the bf16 x bf16 product is
// exact in fp32, so fused and unfused steps round identically).  That chain is exactly what
// the fp32 matrix instruction v_mfma_f32_16x16x4_f32 computes: it walks its 4 k in order
// with one fp32 rounding per step, so a sequence of them is the scalar chain for 16 tokens
// x 16 targets at the full fp32 MFMA rate.  A chain cannot be split over k, so parallelism
// comes only from (token, target) blocks: one wavefront owns 16 tokens and NB blocks of 16
// targets; the TB wavefronts that share a token group take different target blocks, so that
// a SIMD has two or more independent chains to interleave behind the ~44-cycle
// dependent-issue latency of the instruction, and merge their winners at the end.
//
// Operand layout of the instruction: lane l holds A[row l%16][k = l/16] and B[k = l/16][col
// l%16], so lane (t, kq) needs x[t][4s + kq] for consecutive steps s.  Both operands are
// therefore staged in LDS in [row][kq][s] order, which makes a lane's next 8 (x, bf16) or 4
// (G, fp32) steps one 16-byte read:
//   x: each lane loads 16 contiguous bytes of its token's row (4 lanes = 64 contiguous bytes
//      per token and instruction), a ring of kRing loads per wavefront is in flight, and the
//      loaded pieces are regrouped into a wavefront-private LDS buffer;
//   G: converted to fp32 once per workgroup and k-slab, shared by the workgroup's wavefronts.
#include "common.h"

namespace molora {

namespace {

constexpr int kRing = 8;        // x loads in flight per wavefront
constexpr int kXK = 32;         // k per x load instruction (chunk): 16 tokens x 64 bytes
constexpr int kSCK = kRing * kXK;  // k per unrolled super-chunk
constexpr int kXRow = 80;       // bytes per token in the x buffer: 4 kq x 16 B + 16 B bank shift
constexpr int kXBuf = 16 * kXRow;

// NB target blocks per wavefront, TB wavefronts per token group, TGW token groups per workgroup
template <int NB, int TB, int TGW>
struct RouteCfg {
    static constexpr int NWV = TB * TGW;
    static constexpr int NT = NWV * 64;
    static constexpr int TOK_WG = TGW * 16;
    static constexpr int CW = NB * TB * 16;  // targets per pass
    // k per G slab: about 4 staging items (32 elements) per thread, 128 or 256
    static constexpr int KS0 = 32 * NT / CW;
    static constexpr int KS = KS0 >= 256 ? 256 : 128;
    static constexpr int LDG = KS + 4;  // floats per target row: 4 kq x KS/4 steps + bank shift
    static constexpr int SLAB_FLOATS = CW * LDG;
    static constexpr size_t LDS_BYTES = 2ull * SLAB_FLOATS * sizeof(float) + (size_t)NWV * 2 * kXBuf;
    static_assert(kSCK % KS == 0, "slab boundaries fall on static positions of the super-chunk");
};

__device__ __forceinline__ void route_barrier() {
    // LDS-only workgroup barrier: the x ring stays in flight across it
    asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
}

template <int NB, int TB, int TGW, bool VEC8>
__global__ __launch_bounds__(TB * TGW * 64) void route_gate_kernel(
    const uint16_t *__restrict__ x, const uint16_t *__restrict__ G, int32_t *__restrict__ r,
    float *__restrict__ logits_out, int64_t N, int d_in, int C) {
    using K = RouteCfg<NB, TB, TGW>;
    extern __shared__ __attribute__((aligned(16))) unsigned char route_lds[];
    float *gs = (float *)route_lds;  // two fp32 slabs [CW][kq][KS/4] (+pad)
    unsigned char *xs_all = route_lds + 2 * K::SLAB_FLOATS * sizeof(float);

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int l16 = lane & 15, kq = lane >> 4;
    const int tb = wave % TB, tgw = wave / TB;  // target-block group, token group
    const int64_t tok_wave = (int64_t)blockIdx.x * K::TOK_WG + tgw * 16;
    unsigned char *xs = xs_all + wave * 2 * kXBuf;  // two chunk buffers of this wavefront

    // load side: lane (t = l16, cq = kq) fetches x[t][k0 + 8*cq .. +8)
    const int64_t tok = tok_wave + l16;
    const bool tok_ok = tok < N;
    const uint16_t *xrow = x + (tok_ok ? tok : 0) * (int64_t)d_in + kq * 8;  // + k0
    const int xs_wr = l16 * kXRow + kq * 4;   // + kq' * 16 : steps 2cq, 2cq+1 of group kq'
    const int xs_rd = l16 * kXRow + kq * 16;  // this lane's 8 steps of the chunk

    float best[4];
    int bidx[4];
#pragma unroll
    for (int v = 0; v < 4; ++v) {
        best[v] = -__builtin_huge_valf();
        bidx[v] = 0x7FFFFFFF;
    }

    for (int c0 = 0; c0 < C; c0 += K::CW) {  // passes of up to CW targets (one pass if C <= 128)
        f32x4 acc[NB];
#pragma unroll
        for (int b = 0; b < NB; ++b) acc[b] = f32x4{0.f, 0.f, 0.f, 0.f};

        // ---- G slab staging ----
        // element (k, c) of the slab goes to  c*LDG + (k%4)*(KS/4) + k/4  as fp32.
        // An item is 8 consecutive targets of one k: one 16-byte load when C is a multiple of 8,
        // eight 2-byte loads otherwise.  Loads are never predicated (addresses are clamped into
        // G, the value is zeroed afterwards) so that they all stay in flight.
        constexpr int IPT = K::KS * K::CW / 8 / K::NT;  // 8-element items per thread and slab
        static_assert(IPT * K::NT * 8 == K::KS * K::CW, "slab staging split");
        u32x4 greg[IPT];
        // geometry of staging item m of this thread: lanes of a wavefront cover 32 k (4 apart) x 2
        // groups of 8 targets, so that the 64 lanes of each LDS store below hit 64 different
        // banks (bank = 4c + k/4 mod 64)
        auto g_item = [&](int m, int &kk, int &c8) {
            const int item = tid + m * K::NT;
            const int lq = item % 64, gq = item / 64;
            kk = (gq / (4 * (K::CW / 16))) * 128 + 4 * (lq % 32) + gq % 4;
            c8 = 8 * (lq / 32) + 16 * ((gq / 4) % (K::CW / 16));
        };
        auto g_load = [&](int k0) {
#pragma unroll
            for (int m = 0; m < IPT; ++m) {
                int kk, c8;
                g_item(m, kk, c8);
                const int kc = min(k0 + kk, d_in - 1);
                if constexpr (VEC8) {
                    // raw: zeroing of what came from clamped addresses waits until the slab is
                    // stored, one slab later, so that nothing here waits for the load
                    greg[m] = *(const u32x4 *)(G + (int64_t)kc * C + min(c0 + c8, C - 8));
                } else {
                    const uint32_t km = (k0 + kk < d_in) ? 0xFFFFFFFFu : 0u;
                    uint32_t e[8];
#pragma unroll
                    for (int i = 0; i < 8; ++i) {
                        uint32_t raw = G[(int64_t)kc * C + min(c0 + c8 + i, C - 1)];
                        asm volatile("" : "+v"(raw));
                        e[i] = raw & ((c0 + c8 + i < C) ? km : 0u);
                    }
                    greg[m] = u32x4{e[0] | (e[1] << 16), e[2] | (e[3] << 16), e[4] | (e[5] << 16),
                                    e[6] | (e[7] << 16)};
                }
            }
        };
        // the slab that starts at k0 (loaded KS k ago) goes to LDS
        auto g_store = [&](float *slab, int k0) {
#pragma unroll
            for (int m = 0; m < IPT; ++m) {
                int kk, c8;
                g_item(m, kk, c8);
                u32x4 v = greg[m];
                if constexpr (VEC8) {
                    // rows past d_in and targets past C were fetched from clamped addresses: zero
                    const uint32_t m8 = (k0 + kk < d_in && c0 + c8 < C) ? 0xFFFFFFFFu : 0u;
                    v = u32x4{v[0] & m8, v[1] & m8, v[2] & m8, v[3] & m8};
                }
                float *dst = slab + c8 * K::LDG + (kk & 3) * (K::KS / 4) + (kk >> 2);
#pragma unroll
                for (int i = 0; i < 8; ++i) {
                    const uint32_t w = v[i >> 1];
                    dst[i * K::LDG] = __uint_as_float((i & 1) ? (w & 0xFFFF0000u) : (w << 16));
                }
            }
        };

        // ---- x ring: kRing chunks of 32 k in flight ----
        u32x4 xg[kRing];
        // Never predicated: a chunk past d_in re-reads the row's last 16 bytes (it meets an
        // all-zero G slab, so it adds +0), a token past N reads token 0 (never stored).
        auto x_load = [&](int j, int k0) {  // chunk starting at k0 into ring slot j
            xg[j] = *(const u32x4 *)(xrow + max(min(k0, d_in - 8 - kq * 8), -kq * 8));
        };

#pragma unroll
        for (int j = 0; j < kRing; ++j) x_load(j, j * kXK);
        if (c0 > 0) route_barrier();  // the previous pass has finished reading the slabs
        g_load(0);
        g_store(gs, 0);
        g_load(K::KS);
        route_barrier();

        // The loop is software-pipelined by one chunk: while the 8 MFMA steps of chunk j run,
        // chunk j+1 is regrouped into the other x buffer and its x and G fragments are read
        // from LDS into a second register set, so a chain never waits for an LDS round trip.
        int slab_idx = 0;  // slab of the chunk whose fragments are being read
        auto regroup = [&](int j) {  // ring slot j -> x buffer j & 1 (steps in MFMA order)
            unsigned char *xb = xs + (j & 1) * kXBuf;
            const u32x4 w = xg[j];
            *(uint32_t *)(xb + xs_wr + 0 * 16) = __builtin_amdgcn_perm(w[2], w[0], 0x05040100u);
            *(uint32_t *)(xb + xs_wr + 1 * 16) = __builtin_amdgcn_perm(w[2], w[0], 0x07060302u);
            *(uint32_t *)(xb + xs_wr + 2 * 16) = __builtin_amdgcn_perm(w[3], w[1], 0x05040100u);
            *(uint32_t *)(xb + xs_wr + 3 * 16) = __builtin_amdgcn_perm(w[3], w[1], 0x07060302u);
        };
        u32x4 xr[2];
        f32x4 g[2][NB][2];
        auto read_frags = [&](int j, int set) {  // fragments of the chunk in ring position j
            const float *slab = gs + (slab_idx & 1) * K::SLAB_FLOATS;
            xr[set] = *(const u32x4 *)(xs + (j & 1) * kXBuf + xs_rd);  // steps 0..7 of this lane
            const int st0 = ((j * kXK) % K::KS) / 4;  // first step of the chunk inside the slab
#pragma unroll
            for (int b = 0; b < NB; ++b) {
                const float *gp = slab + ((tb * NB + b) * 16 + l16) * K::LDG + kq * (K::KS / 4) + st0;
                g[set][b][0] = *(const f32x4 *)gp;
                g[set][b][1] = *(const f32x4 *)(gp + 4);
            }
        };
        regroup(0);
        x_load(0, kSCK);
        read_frags(0, 0);
        const int nsc = (d_in + kSCK - 1) / kSCK;
        for (int sc = 0; sc < nsc; ++sc) {
            const int k_sc = sc * kSCK;
#pragma unroll
            for (int j = 0; j < kRing; ++j) {
                const int jn = (j + 1) % kRing;            // ring position of the next chunk
                const int k_next = k_sc + (j + 1) * kXK;   // its first k (may be past d_in)
                const int cur = j & 1, nxt = cur ^ 1;
                regroup(jn);
                x_load(jn, k_next + kSCK);  // refill the ring slot
                if (((j + 1) * kXK) % K::KS == 0) {
                    // the next chunk starts a G slab: it was loaded into registers one slab ago
                    ++slab_idx;
                    g_store(gs + (slab_idx & 1) * K::SLAB_FLOATS, slab_idx * K::KS);
                    g_load((slab_idx + 1) * K::KS);
                    route_barrier();
                }
                read_frags(jn, nxt);
#pragma unroll
                for (int s = 0; s < 8; ++s) {
                    const uint32_t ww = xr[cur][s >> 1];
                    const float xa = __uint_as_float((s & 1) ? (ww & 0xFFFF0000u) : (ww << 16));
#pragma unroll
                    for (int b = 0; b < NB; ++b)
                        acc[b] = __builtin_amdgcn_mfma_f32_16x16x4f32(xa, g[cur][b][s >> 2][s & 3],
                                                                      acc[b], 0, 0, 0);
                }
                // nothing moves across a chunk boundary: left alone, the scheduler sinks all eight
                // x loads of a round to its end and the next round starts by waiting for them
                __builtin_amdgcn_sched_barrier(0);
            }
        }

        // acc[b][v] is the logit of token kq*4 + v and target c0 + (tb*NB + b)*16 + l16.
        if (logits_out != nullptr) {  // the chains themselves are wanted (first layer of a router MLP)
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                const int64_t t = tok_wave + kq * 4 + v;
#pragma unroll
                for (int b = 0; b < NB; ++b) {
                    const int tgt = c0 + (tb * NB + b) * 16 + l16;
                    if (t < N && tgt < C) logits_out[t * C + tgt] = acc[b][v];
                }
            }
        }
        // ---- running argmax: lexicographic (largest logit, then lowest index) ----
#pragma unroll
        for (int v = 0; v < 4; ++v) {
#pragma unroll
            for (int b = 0; b < NB; ++b) {
                const int tgt = c0 + (tb * NB + b) * 16 + l16;
                float val = acc[b][v];
                // a NaN logit never wins, except that target 0 is the scan's starting point
                if (val != val) val = (tgt == 0) ? __builtin_huge_valf() : -__builtin_huge_valf();
                if (tgt < C && (val > best[v] || (val == best[v] && tgt < bidx[v]))) {
                    best[v] = val;
                    bidx[v] = tgt;
                }
            }
        }
    }

    // winners of this wavefront's targets: reduce over the 16 lanes that hold a token's row
#pragma unroll
    for (int v = 0; v < 4; ++v) {
#pragma unroll
        for (int d = 1; d < 16; d <<= 1) {
            const float ov = __shfl_xor(best[v], d, 64);
            const int oi = __shfl_xor(bidx[v], d, 64);
            if (ov > best[v] || (ov == best[v] && oi < bidx[v])) {
                best[v] = ov;
                bidx[v] = oi;
            }
        }
    }
    if constexpr (TB > 1) {
        // merge the TB wavefronts of a token group through LDS (the slabs are done with)
        __syncthreads();
        float *red_v = (float *)route_lds;                 // [TB][TOK_WG]
        int32_t *red_i = (int32_t *)(red_v + TB * K::TOK_WG);
        if (l16 == 0) {
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                red_v[tb * K::TOK_WG + tgw * 16 + kq * 4 + v] = best[v];
                red_i[tb * K::TOK_WG + tgw * 16 + kq * 4 + v] = bidx[v];
            }
        }
        __syncthreads();
        if (tb == 0 && l16 == 0) {
#pragma unroll
            for (int v = 0; v < 4; ++v) {
#pragma unroll
                for (int o = 1; o < TB; ++o) {
                    const float ov = red_v[o * K::TOK_WG + tgw * 16 + kq * 4 + v];
                    const int oi = red_i[o * K::TOK_WG + tgw * 16 + kq * 4 + v];
                    if (ov > best[v] || (ov == best[v] && oi < bidx[v])) {
                        best[v] = ov;
                        bidx[v] = oi;
                    }
                }
            }
        }
    }
    if (tb == 0 && l16 == 0) {
#pragma unroll
        for (int v = 0; v < 4; ++v) {
            const int64_t t = tok_wave + kq * 4 + v;
            if (t < N && r != nullptr) r[t] = bidx[v];
        }
    }
}

// more than 64 KB of dynamic LDS has to be asked for, once per device (see common.h)
template <int NB, int TB, int TGW, bool VEC8>
struct RouteKernel {
    static inline LdsRegistrar lds{(const void *)route_gate_kernel<NB, TB, TGW, VEC8>,
                                   RouteCfg<NB, TB, TGW>::LDS_BYTES};
};

template <int NB, int TB, int TGW, bool VEC8>
hipError_t launch_cfg(const uint16_t *x, const uint16_t *G, int32_t *r, float *lo, int64_t N,
                      int d_in, int C, hipStream_t s) {
    using K = RouteCfg<NB, TB, TGW>;
    auto kern = route_gate_kernel<NB, TB, TGW, VEC8>;
    (void)&RouteKernel<NB, TB, TGW, VEC8>::lds;  // instantiates the registration
    const unsigned blocks = (unsigned)((N + K::TOK_WG - 1) / K::TOK_WG);
    hipLaunchKernelGGL(kern, dim3(blocks), dim3(K::NT), K::LDS_BYTES, s, x, G, r, lo, N, d_in, C);
    return hipGetLastError();
}

// Token groups per workgroup: a workgroup shares one fp32 copy of the G slab, so more groups
// per workgroup mean less staging work per token; the problem has only N/16 token groups, so
// fewer mean more workgroups to spread over the chip.
template <int NB, int TB>
hipError_t launch_tb(const uint16_t *x, const uint16_t *G, int32_t *r, float *lo, int64_t N,
                     int d_in, int C, hipStream_t s) {
    const int64_t groups = (N + 15) / 16;
    constexpr int kMaxTgw = 8 / TB;  // at most 8 wavefronts per workgroup
    if (C % 8 == 0) {                // rows of G can be fetched 16 bytes at a time
        if constexpr (kMaxTgw >= 4)
            // (measured: 63 against 70 us at 1024 groups x 32 targets, 20 against 23 us at 512
            // groups x 8 targets, but 51 against 41 us at 512 groups x 64 targets)
            if (groups >= 512 * TB * NB) return launch_cfg<NB, TB, 4, true>(x, G, r, lo, N, d_in, C, s);
        if constexpr (kMaxTgw >= 2)
            if (groups >= 2 * 512) return launch_cfg<NB, TB, 2, true>(x, G, r, lo, N, d_in, C, s);
        return launch_cfg<NB, TB, 1, true>(x, G, r, lo, N, d_in, C, s);
    }
    return launch_cfg<NB, TB, 1, false>(x, G, r, lo, N, d_in, C, s);
}

}  // namespace

hipError_t launch_route_gate(const uint16_t *x, const uint16_t *G, int32_t *r, float *logits_out,
                             int64_t N, int d_in, int C, hipStream_t s) {
    if (N == 0) return hipSuccess;
    if (C <= 16) return launch_tb<1, 1>(x, G, r, logits_out, N, d_in, C, s);
    if (C <= 32) return launch_tb<1, 2>(x, G, r, logits_out, N, d_in, C, s);
    if (C <= 64) return launch_tb<2, 2>(x, G, r, logits_out, N, d_in, C, s);
    return launch_tb<2, 4>(x, G, r, logits_out, N, d_in, C, s);  // 128 targets per pass
}

}  // namespace molora
