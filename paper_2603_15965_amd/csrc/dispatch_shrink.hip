// Dispatch and shrink beside each other in ONE launch, for layers with a few narrow adapters.
//
// The grouped shrink t_p = x_{perm[p]} A_{c(p)} needs the dispatch step's permutation, so the
// two run one after the other, and for a batch of a few thousand tokens both are bound by
// latency (one small workgroup sorting, 17 MB of x streamed by 256 small workgroups): 7 + 9
// us plus a launch gap before a 40 us GEMM.  When C * rank <= 64 the shrink can do without the
// permutation: it computes x_i A_c for ALL c in token order (shrink_body<.., DENSE>; the step
// is bound by reading x, the extra arithmetic is free), and the expand step picks a row's
// adapter.  Then nothing links the two steps, and one launch holds both: workgroups [0, G) are
// the dispatch step (Alg. "Unified Dispatch Kernel", with the gate of Alg. "Compositional
// Gating Kernel" when token ids are given), the others are shrink work items.  No workgroup
// waits for another.
#include "../../include/molora.h"
#include "bucket_body.h"
#include "shrink_body.h"

namespace molora {

namespace {

constexpr int kDsWaves = 4;  // 256 threads: the shrink's work items (4-way K split) set the workgroup size

template <bool GATE, int NJ, int RB>
__global__ __launch_bounds__(64 * kDsWaves) void dispatch_shrink_kernel(
    const int32_t *__restrict__ r, int32_t *__restrict__ offsets, int32_t *__restrict__ perm, int N,
    int C, int32_t *err_flag, GateArgs gate, int G, const uint16_t *__restrict__ x,
    const uint16_t *__restrict__ A, uint16_t *__restrict__ t_dense, int d_in, int rank) {
    if ((int)blockIdx.x < G) {
        bucket_body<GATE, kDsWaves, true>(r, offsets, perm, N, C, err_flag, gate, G, (int)blockIdx.x);
    } else {
        shrink_body<NJ, RB, kDsWaves, 4, true>(x, A, nullptr, nullptr, t_dense, d_in, C, rank,
                                               Mix{1, C, nullptr, nullptr, 1}, (int)blockIdx.x - G, N);
    }
}

// dispatch workgroups of 4 wavefronts (every one recounts all tokens and scatters its own part):
// one per 1024 tokens when r is given, one per 512 when the gate is evaluated in the kernel
// (measured at 4096 tokens beside the shrink: 10.0 -> 9.6 us with the gate, 9.0 -> 9.7 us
// without), at most 16
inline int ds_dispatch_workgroups(int64_t N, bool gate) {
    const int64_t g = gate ? (N + 511) / 512 : (N + 1023) / 1024;
    return (int)(g < 1 ? 1 : (g > 16 ? 16 : g));
}

template <bool GATE, int NJ>
hipError_t launch_ds(const int32_t *r, int32_t *offsets, int32_t *perm, int64_t N, int C,
                     int32_t *err_flag, const GateArgs &g, const uint16_t *x, const uint16_t *A,
                     uint16_t *t_dense, int d_in, int rank, hipStream_t s, bool with_dispatch) {
    const int G = with_dispatch ? ds_dispatch_workgroups(N, GATE) : 0;  // 0: the shrink alone
    // 32-row items when they still cover the chip twice, 16-row items otherwise
    const bool small_items = (N + 31) / 32 < 512;
    const size_t lds = BucketLds(C, kDsWaves).bytes();
    if (small_items) {
        const unsigned blocks = (unsigned)(G + (N + 15) / 16);
        hipLaunchKernelGGL((dispatch_shrink_kernel<GATE, NJ, 1>), dim3(blocks), dim3(64 * kDsWaves), lds, s, r,
                           offsets, perm, (int)N, C, err_flag, g, G, x, A, t_dense, d_in, rank);
    } else {
        const unsigned blocks = (unsigned)(G + (N + 31) / 32);
        hipLaunchKernelGGL((dispatch_shrink_kernel<GATE, NJ, 2>), dim3(blocks), dim3(64 * kDsWaves), lds, s, r,
                           offsets, perm, (int)N, C, err_flag, g, G, x, A, t_dense, d_in, rank);
    }
    return hipGetLastError();
}

}  // namespace

bool dense_shrink_ok(int64_t N, int d_in, int C, int rank) {
    (void)d_in;
    return N > 512 && (int64_t)C * rank <= 64;
}

hipError_t launch_dispatch_shrink(const int32_t *v, const int32_t *adapter, const int32_t *breaks_host,
                                  int M, int n_adapters, int32_t *r, const uint16_t *x,
                                  const uint16_t *A, int32_t *offsets, int32_t *perm, uint16_t *t_dense,
                                  int64_t N, int d_in, int C, int rank, int32_t *err_flag, hipStream_t s,
                                  bool with_dispatch) {
    if (!dense_shrink_ok(N, d_in, C, rank)) return hipErrorInvalidValue;
    const int nj = (C * rank + 15) / 16;
    GateArgs g{};
    if (v != nullptr) {
        g.v = v;
        g.adapter = adapter;
        g.r_out = r;
        g.M = M;
        g.n_adapters = n_adapters;
        for (int j = 0; j <= M; ++j) g.br.b[j] = breaks_host[j];
        for (int j = M + 1; j < 65; ++j) g.br.b[j] = 0;
    }
#define MOLORA_DS_CASE(NJ)                                                                            \
    case NJ:                                                                                          \
        return v != nullptr                                                                           \
                   ? launch_ds<true, NJ>(nullptr, offsets, perm, N, C, err_flag, g, x, A, t_dense, d_in, rank, s, with_dispatch) \
                   : launch_ds<false, NJ>(r, offsets, perm, N, C, err_flag, g, x, A, t_dense, d_in, rank, s, with_dispatch);
    switch (nj) {
        MOLORA_DS_CASE(1)
        MOLORA_DS_CASE(2)
        MOLORA_DS_CASE(3)
        MOLORA_DS_CASE(4)
        default:
            return hipErrorInvalidValue;
    }
#undef MOLORA_DS_CASE
}

}  // namespace molora
