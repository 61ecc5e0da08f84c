// Learned top-1 routing (Sec. "Router Architecture", k = 1; linear gate of Table
// "tab:moe_adapter"):  r[i] = argmax_c sum_k x[i][k] G[k][c], lowest index on ties.
//
// The result has to be a deterministic function of the input bits, so every logit is the
// strict fp32 chain  acc <- fl(acc + x_k * g_k),  k ascending.  The chain is run on the
// matrix cores with the K = 1 fp32 MFMA (v_mfma_f32_4x4x1_16b_f32): one instruction is 16
// independent 4x4 outer-product updates, i.e. exactly one fused multiply-add per
// accumulator and therefore one chain step for 256 (token, target) pairs, at twice the
// rate of the vector ALU.  The bf16 x bf16 product is exact in fp32, so the fused and the
// unfused step round identically.
//
// Work split: a wavefront owns TOK tokens x (4*CG*P) targets; the 16 MFMA blocks are laid
// out as TG token groups x CG target groups.  x is read straight from HBM (each lane 16 B
// of its token's row, prefetched), G is converted to fp32 once per workgroup and k-slab
// into LDS, transposed to [target][k] so a lane fetches 4 consecutive k with one b128 read.
#include "common.h"

namespace molora {

namespace {

constexpr int kRouteWaves = 4;
constexpr int kRouteThreads = kRouteWaves * 64;

template <int CG, int P>
struct RouteCfg {
    static constexpr int TG = 16 / CG;             // token groups per MFMA
    static constexpr int S = 2;                    // independent token sets per wavefront
    static constexpr int TOK_SET = 4 * TG;         // tokens per set
    static constexpr int TOK_WAVE = S * TOK_SET;
    static constexpr int TOK_WG = kRouteWaves * TOK_WAVE;
    static constexpr int CPAD = 4 * CG * P;        // targets covered
    static constexpr int KS0 = 4096 / CPAD;
    static constexpr int KS = KS0 > 256 ? 256 : (KS0 < 8 ? 8 : KS0);  // k per G slab
    static constexpr int XS = KS < 64 ? KS : 64;   // k per x prefetch chunk
    static constexpr int XL = XS / 8;              // 16-byte x loads per chunk and set
    static constexpr int LDG = KS + 4;             // padded row of the fp32 slab
    static constexpr int SLAB_FLOATS = CPAD * LDG;
    static constexpr int QUADS = CPAD * KS / 4;    // (target, 4 k) items per slab
    static constexpr int QPT = (QUADS + kRouteThreads - 1) / kRouteThreads;
    static constexpr size_t LDS_BYTES = 2ull * SLAB_FLOATS * sizeof(float);
};

template <int CG, int P>
__global__ __launch_bounds__(kRouteThreads) void route_gate_kernel(
    const uint16_t *__restrict__ x, const uint16_t *__restrict__ G, int32_t *__restrict__ r,
    int64_t N, int d_in, int C) {
    using K = RouteCfg<CG, P>;
    extern __shared__ float gs[];  // two fp32 slabs [CPAD][LDG]

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int blk = lane >> 2, q = lane & 3;
    const int cg = blk % CG, tg = blk / CG;
    const int64_t tok_wave = (int64_t)blockIdx.x * K::TOK_WG + wave * K::TOK_WAVE;

    // x row of this lane for each set (A operand: row q of block (tg, cg))
    const uint16_t *xrow[K::S];
    bool xok[K::S];
#pragma unroll
    for (int s = 0; s < K::S; ++s) {
        const int64_t t = tok_wave + s * K::TOK_SET + tg * 4 + q;
        xok[s] = t < N;
        xrow[s] = x + (xok[s] ? t : 0) * (int64_t)d_in;
    }

    f32x4 acc[K::S][P];
#pragma unroll
    for (int s = 0; s < K::S; ++s)
#pragma unroll
        for (int p = 0; p < P; ++p) acc[s][p] = f32x4{0.f, 0.f, 0.f, 0.f};

    // ---- G slab staging: thread handles items (target, 4 consecutive k) ----
    uint32_t greg[K::QPT][2];
    auto g_load = [&](int k0) {
#pragma unroll
        for (int m = 0; m < K::QPT; ++m) {
            const int item = tid + m * kRouteThreads;
            const int c = item % K::CPAD, kq = item / K::CPAD;
            uint32_t v[4];
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const int k = k0 + kq * 4 + e;
                v[e] = (item < K::QUADS && c < C && k < d_in) ? G[(int64_t)k * C + c] : 0u;
            }
            greg[m][0] = v[0] | (v[1] << 16);
            greg[m][1] = v[2] | (v[3] << 16);
        }
    };
    auto g_store = [&](float *slab) {
#pragma unroll
        for (int m = 0; m < K::QPT; ++m) {
            const int item = tid + m * kRouteThreads;
            if (item < K::QUADS) {
                const int c = item % K::CPAD, kq = item / K::CPAD;
                f32x4 f;
                f[0] = __uint_as_float(greg[m][0] << 16);
                f[1] = __uint_as_float(greg[m][0] & 0xFFFF0000u);
                f[2] = __uint_as_float(greg[m][1] << 16);
                f[3] = __uint_as_float(greg[m][1] & 0xFFFF0000u);
                *(f32x4 *)(slab + c * K::LDG + kq * 4) = f;
            }
        }
    };

    // ---- x prefetch: XL loads of 8 bf16 per set ----
    u32x4 xcur[K::S][K::XL], xnext[K::S][K::XL];
    auto x_load = [&](u32x4(&dst)[K::S][K::XL], int k0) {
#pragma unroll
        for (int s = 0; s < K::S; ++s)
#pragma unroll
            for (int j = 0; j < K::XL; ++j) {
                const int k = k0 + j * 8;
                dst[s][j] = (xok[s] && k < d_in) ? *(const u32x4 *)(xrow[s] + k)
                                                 : u32x4{0u, 0u, 0u, 0u};
            }
    };

    g_load(0);
    x_load(xcur, 0);
    g_store(gs);
    __syncthreads();

    const int nslab = (d_in + K::KS - 1) / K::KS;
    for (int sl = 0; sl < nslab; ++sl) {
        const float *slab = gs + (sl & 1) * K::SLAB_FLOATS;
        const int k_slab = sl * K::KS;
        if (sl + 1 < nslab) g_load(k_slab + K::KS);
#pragma unroll 1
        for (int sub = 0; sub < K::KS / K::XS; ++sub) {
            const int k_sub = k_slab + sub * K::XS;
            x_load(xnext, k_sub + K::XS);  // guarded by k < d_in; harmless past the end
#pragma unroll
            for (int j = 0; j < K::XL; ++j) {
                // 8 k per group: fp32 G values of this lane's target(s)
                f32x4 g[P][2];
#pragma unroll
                for (int p = 0; p < P; ++p) {
                    const float *gp = slab + (p * 4 * CG + cg * 4 + q) * K::LDG + sub * K::XS + j * 8;
                    g[p][0] = *(const f32x4 *)gp;
                    g[p][1] = *(const f32x4 *)(gp + 4);
                }
#pragma unroll
                for (int e = 0; e < 8; ++e) {
#pragma unroll
                    for (int s = 0; s < K::S; ++s) {
                        const uint32_t w = xcur[s][j][e >> 1];
                        const float xa = __uint_as_float((e & 1) ? (w & 0xFFFF0000u) : (w << 16));
#pragma unroll
                        for (int p = 0; p < P; ++p)
                            acc[s][p] = __builtin_amdgcn_mfma_f32_4x4x1f32(xa, g[p][e >> 2][e & 3],
                                                                           acc[s][p], 0, 0, 0);
                    }
                }
            }
#pragma unroll
            for (int s = 0; s < K::S; ++s)
#pragma unroll
                for (int j = 0; j < K::XL; ++j) xcur[s][j] = xnext[s][j];
        }
        if (sl + 1 < nslab) g_store(gs + ((sl + 1) & 1) * K::SLAB_FLOATS);
        __syncthreads();
    }

    // ---- argmax: lexicographic (largest logit, then lowest index) ----
    // acc[s][p][i] is the logit of token (tg*4 + i) of set s and target p*4*CG + cg*4 + q.
    constexpr float kInf = __builtin_huge_valf();
#pragma unroll
    for (int s = 0; s < K::S; ++s) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            float best = -kInf;
            int bidx = 0x7FFFFFFF;
#pragma unroll
            for (int p = 0; p < P; ++p) {
                const int tgt = p * 4 * CG + cg * 4 + q;
                float v = acc[s][p][i];
                // a NaN logit never wins, except that target 0 is the scan's starting point
                if (v != v) v = (tgt == 0) ? kInf : -kInf;
                if (tgt < C && (v > best || (v == best && tgt < bidx))) {
                    best = v;
                    bidx = tgt;
                }
            }
#pragma unroll
            for (int d = 1; d < 4 * CG; d <<= 1) {
                const float ov = __shfl_xor(best, d, 64);
                const int oi = __shfl_xor(bidx, d, 64);
                if (ov > best || (ov == best && oi < bidx)) {
                    best = ov;
                    bidx = oi;
                }
            }
            const int64_t t = tok_wave + s * K::TOK_SET + tg * 4 + i;
            if (cg == 0 && q == 0 && t < N) r[t] = bidx;
        }
    }
}

template <int CG, int P>
hipError_t launch_cfg(const uint16_t *x, const uint16_t *G, int32_t *r, int64_t N, int d_in, int C,
                      hipStream_t s) {
    using K = RouteCfg<CG, P>;
    auto kern = route_gate_kernel<CG, P>;
    if (K::LDS_BYTES > 64 * 1024) {
        hipError_t e = hipFuncSetAttribute((const void *)kern,
                                           hipFuncAttributeMaxDynamicSharedMemorySize,
                                           (int)K::LDS_BYTES);
        if (e != hipSuccess) return e;
    }
    const unsigned blocks = (unsigned)((N + K::TOK_WG - 1) / K::TOK_WG);
    hipLaunchKernelGGL(kern, dim3(blocks), dim3(kRouteThreads), K::LDS_BYTES, s, x, G, r, N, d_in,
                       C);
    return hipGetLastError();
}

}  // namespace

hipError_t launch_route_gate(const uint16_t *x, const uint16_t *G, int32_t *r, int64_t N, int d_in,
                             int C, hipStream_t s) {
    if (N == 0) return hipSuccess;
    if (C <= 4) return launch_cfg<1, 1>(x, G, r, N, d_in, C, s);
    if (C <= 8) return launch_cfg<2, 1>(x, G, r, N, d_in, C, s);
    if (C <= 16) return launch_cfg<4, 1>(x, G, r, N, d_in, C, s);
    if (C <= 32) return launch_cfg<8, 1>(x, G, r, N, d_in, C, s);
    if (C <= 64) return launch_cfg<16, 1>(x, G, r, N, d_in, C, s);
    if (C <= 128) return launch_cfg<16, 2>(x, G, r, N, d_in, C, s);
    if (C <= 256) return launch_cfg<16, 4>(x, G, r, N, d_in, C, s);
    if (C <= 512) return launch_cfg<16, 8>(x, G, r, N, d_in, C, s);
    return launch_cfg<16, 16>(x, G, r, N, d_in, C, s);
}

}  // namespace molora
