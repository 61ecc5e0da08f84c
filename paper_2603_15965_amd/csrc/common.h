// Internal declarations shared by the HIP translation units of libmolora (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <hip/hip_ext.h>
#include <stdint.h>

namespace molora {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) short i16x4;
typedef __attribute__((ext_vector_type(8))) short i16x8;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;
typedef __attribute__((ext_vector_type(2))) uint32_t u32x2;

#define MOLORA_LDS __attribute__((address_space(3)))

__device__ __forceinline__ float bf16_bits_to_f32(uint32_t b) { return __uint_as_float(b << 16); }

// Round-to-nearest-even fp32 -> bf16 bit pattern (finite inputs).
__device__ __forceinline__ uint32_t f32_to_bf16_bits(float f) {
    uint32_t u = __float_as_uint(f);
    return (u + 0x7FFFu + ((u >> 16) & 1u)) >> 16;
}

// LDS transpose read of gfx950: inside every group of 16 lanes, lane i receives the
// (i % 4)-th 16-bit element addressed by lanes i/4, i/4 + 4, i/4 + 8, i/4 + 12.  With lane a
// of the group pointing at row (a / 4), columns 4 * (a % 4) .. +3 of a row-major [4][16]
// block, lane i ends up with the 4 rows of column i: a K-major tile becomes the
// "consecutive k per lane" operand the bf16 MFMA wants.
__device__ __forceinline__ i16x4 lds_read_tr16(const MOLORA_LDS void *p) {
    return __builtin_amdgcn_ds_read_tr16_b64_v4i16((MOLORA_LDS i16x4 *)p);
}

// How a bucket maps to adapters (weighted top-k mixture of Sec. "Router Architecture", slot
// table of Def. "Hot-Set Layout").  Bucket b stands for the ordered tuple of k adapters
// c_j = (b / C^j) % C, j < k; adapter c lives in position slots[c] of the A / B pools
// (slots == nullptr: position c).  The low-rank intermediate of a bucket is k * rank wide,
// piece j scaled by w[token * k + j] (w == nullptr: 1).  {1, C, nullptr, nullptr} is the plain
// one-adapter-per-token case.
struct Mix {
    int k;
    int C;
    const int32_t *slots;
    const float *w;
    // 1: the low-rank intermediate is in the token-order form of the dense shrink, row of token
    // i = [x_i A_0 .. x_i A_{C-1} as bf16 high parts | the same as remainders], 2 * C * rank
    // values (k = 1, no slot table); 0: one row of 2 * k * rank values per sorted position
    int t_dense = 0;
};
__device__ __forceinline__ int mix_adapter(const Mix &m, int b, int j) {
    int c = b;
    if (m.k > 1) {
        for (int i = 0; i < j; ++i) c /= m.C;
        c %= m.C;
    }
    return m.slots != nullptr ? m.slots[c] : c;
}

// ---- once-per-device set-up ----
// A kernel that uses more than 64 KB of dynamic LDS has to be told so once (a function
// attribute).  Every such kernel registers itself in a list when the library is loaded (no HIP
// call happens then); ensure_device_ready() walks the list the first time any entry point runs
// on a device, and molora_init() / molora_graph_begin() call it eagerly, so that no attribute
// call ever falls inside a stream capture.
struct KernelLdsNeed {
    const void *fn;
    int bytes;
    KernelLdsNeed *next;
};
void register_kernel_lds(KernelLdsNeed *node);
struct LdsRegistrar {
    KernelLdsNeed node;
    LdsRegistrar(const void *fn, size_t bytes) : node{fn, (int)bytes, nullptr} { register_kernel_lds(&node); }
};
hipError_t ensure_device_ready();

// ---- benchmark aid: the device-side duration of a base-projection launch ----
// A pair of events armed by the calling thread is attached to the next launch of a kernel that
// holds the base projection (the tiled GEMM, the small-batch GEMM, the decode step's first
// launch): the launch records its own start and end on them (hipExtLaunchKernelGGL), which is
// the duration a kernel trace reports, with no marker packets beside the kernel.
struct LaunchEvents {
    hipEvent_t start = nullptr, stop = nullptr;
};
void arm_launch_events(hipEvent_t start, hipEvent_t stop);
LaunchEvents take_launch_events();  // the calling thread's pending pair, which is cleared
template <typename K, typename... Args>
inline void launch_base_kernel(K kern, dim3 grid, dim3 block, size_t lds, hipStream_t s, Args... args) {
    const LaunchEvents ev = take_launch_events();
    if (ev.start != nullptr && ev.stop != nullptr)
        hipExtLaunchKernelGGL(kern, grid, block, (uint32_t)lds, s, ev.start, ev.stop, 0, args...);
    else
        hipLaunchKernelGGL(kern, grid, block, lds, s, args...);
}

// the tiled GEMM keeps per-lane byte offsets into x and W in 32 bits: false when the kernel
// that launch_fused_gemm would pick for these sizes (force_tile as there) cannot address them
bool fused_gemm_sizes_ok(int64_t N, int d_in, int d_out, int force_tile = 0);

// Sizes for which the dispatch step and the shrink run beside each other in one launch
// (launch_dispatch_shrink) and the fused GEMM reads the token-order intermediate: a few narrow
// adapters (C * rank <= 64, so that computing x A_c for every c costs the memory-bound shrink
// nothing) and a batch that takes the tiled GEMM.
bool dense_shrink_ok(int64_t N, int d_in, int C, int rank);
// Gating (v != nullptr: vocabulary / composite target as launch_gate_bucket, r is then an
// output; else r is the input) + dispatch + token-order shrink in one launch.
hipError_t launch_dispatch_shrink(const int32_t *v, const int32_t *adapter, const int32_t *breaks_host,
                                  int M, int n_adapters, int32_t *r, const uint16_t *x,
                                  const uint16_t *A, int32_t *offsets, int32_t *perm, uint16_t *t_dense,
                                  int64_t N, int d_in, int C, int rank, int32_t *err_flag, hipStream_t s,
                                  bool with_dispatch = true);  // false: the token-order shrink alone

// ---- launchers implemented in the kernel translation units (all asynchronous) ----
// rank is the rank of one adapter; buckets number C (the tuples, when mix.k > 1)
// r and logits_out (fp32 [N][C], the chains themselves) are each optional
hipError_t launch_route_gate(const uint16_t *x, const uint16_t *G, int32_t *r, float *logits_out,
                             int64_t N, int d_in, int C, hipStream_t s);
// second half of the router MLP: u [N][H] = x W1 (fp32 chains) -> idx [N][k], w [N][k]
hipError_t launch_router_finish(const float *u, const float *b1, const uint16_t *W2, const float *b2,
                                int32_t *idx, float *w, int64_t N, int H, int K, int k, hipStream_t s);
// key[i] = sum_j idx[i][j] C^j and wq[i][j] = w[i][j] (1 if w == nullptr), with an index outside
// [0, C) replaced by adapter 0 at weight 0
hipError_t launch_mix_key(const int32_t *idx, const float *w, int32_t *key, float *wq, int64_t N,
                          int C, int k, hipStream_t s);
hipError_t launch_route_compose(const int32_t *v, const int32_t *adapter, const int32_t *breaks_host,
                                int M, int n_adapters, int32_t *r, int64_t N, hipStream_t s);
hipError_t launch_route_vocab(const int32_t *v, const int32_t *breaks_host, int M, int32_t *r,
                              int64_t N, hipStream_t s);
hipError_t launch_bucket(const int32_t *r, int32_t *offsets, int32_t *perm, int64_t N, int C,
                         int32_t *err_flag, hipStream_t s);
// route (vocabulary, or adapter x modality) and bucket in one kernel; C = n_adapters * M
hipError_t launch_gate_bucket(const int32_t *v, const int32_t *adapter, const int32_t *breaks_host,
                              int M, int n_adapters, int32_t *r, int32_t *offsets, int32_t *perm,
                              int64_t N, int32_t *err_flag, hipStream_t s);
// scratch: fp32 scratch of shrink_scratch_bytes(...) bytes or nullptr (then K is never split
// over workgroups); contents need no initialisation
size_t shrink_scratch_bytes(int64_t N, int d_in, int C, int R);
// The dispatch step inside the shrink launch, for a batch of at most 64 tokens (one wavefront
// of targets): r != nullptr makes every workgroup of the shrink derive its bucket's rows from r
// itself, and the workgroups of column group 0 write offsets and perm (molora_bucket's output:
// stable, tokens without adapter listed last, err_flag set if there are any) for the step
// that follows.  One launch and two dependent trips to memory less than bucket, then shrink.
struct SortArgs {
    const int32_t *r = nullptr;
    int32_t *offsets = nullptr;
    int32_t *perm = nullptr;
    int32_t *err_flag = nullptr;
};
// sizes for which launch_shrink takes SortArgs (its streaming kernel, N <= 64)
bool sort_in_shrink_ok(int64_t N, int d_in, int C, int rank);
// sort.r != nullptr: offsets and perm are ignored (sort.offsets / sort.perm are written)
hipError_t launch_shrink(const uint16_t *x, const uint16_t *A, const int32_t *offsets,
                         const int32_t *perm, uint16_t *t2, int64_t N, int d_in, int C, int rank,
                         Mix mix, hipStream_t s, float *scratch = nullptr, SortArgs sort = SortArgs{});
hipError_t launch_fused_gemm(const uint16_t *x, const uint16_t *W, const uint16_t *B,
                             const uint16_t *t2, const int32_t *offsets, const int32_t *perm,
                             float *h, int64_t N, int d_in, int d_out, int C, int rank, Mix mix,
                             hipStream_t s, int force_tile = 0);

// same contract, N <= 64 (the fused GEMM launcher routes such batches here)
hipError_t launch_small_batch_gemm(const uint16_t *x, const uint16_t *W, const uint16_t *B,
                                   const uint16_t *t2, const int32_t *offsets, const int32_t *perm,
                                   float *h, int64_t N, int d_in, int d_out, int C, int rank, Mix mix,
                                   hipStream_t s);
// A batch of at most 64 tokens in two launches instead of four: (1) the dispatch step, the shrink
// and the base projection h = x W side by side (the latency-bound shrink hides behind the
// stream of W), (2) the expand added to h.
hipError_t launch_small_shrink_base(const uint16_t *x, const uint16_t *W, const uint16_t *A, float *h,
                                    uint16_t *t_out, int64_t N, int d_in, int d_out, int C, int rank,
                                    Mix mix, SortArgs sort, hipStream_t s, bool w_packed = false);
// W for launch_small_shrink_base(..., w_packed = true): slabs of 16 rows, inside a slab groups of
// gc = small_pack_cols(d_out) columns one after the other (0: this d_out has no packed form)
int small_pack_cols(int d_out);
hipError_t launch_pack_w(const uint16_t *W, uint16_t *Wp, int d_in, int d_out, hipStream_t s);
hipError_t launch_small_expand(const uint16_t *B, const uint16_t *t2, const int32_t *offsets,
                               const int32_t *perm, float *h, int64_t N, int d_in, int d_out, int C,
                               int rank, Mix mix, hipStream_t s, bool b_packed = false);
// ksplit > 1 (with planes, fp32 [ksplit][N][R]): K cut into slices over workgroups, second pass adds them
int small_batch_shrink_ksplit(int64_t N, int d_in, int C, int R);
hipError_t launch_small_batch_shrink(const uint16_t *x, const uint16_t *A, const int32_t *offsets,
                                     const int32_t *perm, uint16_t *t2, int64_t N, int d_in, int C,
                                     int rank, Mix mix, hipStream_t s, float *planes = nullptr,
                                     int ksplit = 1, SortArgs sort = SortArgs{});

}  // namespace molora
