// C ABI of libmolora: argument checking and the order of launches.  No arithmetic here.
#include "../../include/molora.h"

#include "common.h"

#include <mutex>

// Scratch of molora_apply_static: one copy per GPU the library runs on, held until the process
// ends.  In host code this name is only a handle for hipGetSymbolAddress, never an address to
// pass on: the device address is resolved once per device in ensure_device_ready() and kept
// in g_scratch_ptr.
static __device__ __align__(256) unsigned char scratch[MOLORA_STATIC_WORKSPACE_BYTES];

namespace molora {

namespace {
constexpr int kMaxDevices = 64;
std::mutex g_init_mutex;
bool g_device_ready[kMaxDevices];
void *g_scratch_ptr[kMaxDevices];  // device address of `scratch` on each device
KernelLdsNeed *&lds_list() {
    static KernelLdsNeed *head = nullptr;
    return head;
}
}  // namespace

void register_kernel_lds(KernelLdsNeed *node) {  // from static initialisers: no HIP call here
    node->next = lds_list();
    lds_list() = node;
}

hipError_t ensure_device_ready() {
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
    std::lock_guard<std::mutex> lock(g_init_mutex);
    if (g_device_ready[dev]) return hipSuccess;
    for (KernelLdsNeed *n = lds_list(); n != nullptr; n = n->next) {
        if (n->bytes <= 64 * 1024) continue;
        e = hipFuncSetAttribute(n->fn, hipFuncAttributeMaxDynamicSharedMemorySize, n->bytes);
        if (e != hipSuccess) return e;
    }
    void *ptr = nullptr;
    e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
    if (e != hipSuccess) return e;
    if (ptr == nullptr) return hipErrorInvalidSymbol;
    g_scratch_ptr[dev] = ptr;
    g_device_ready[dev] = true;
    return hipSuccess;
}

namespace {
thread_local LaunchEvents t_launch_events;
}
void arm_launch_events(hipEvent_t start, hipEvent_t stop) { t_launch_events = LaunchEvents{start, stop}; }
LaunchEvents take_launch_events() {
    const LaunchEvents ev = t_launch_events;
    t_launch_events = LaunchEvents{};
    return ev;
}

namespace {
// the current device's copy of `scratch` (nullptr before ensure_device_ready() succeeded there)
void *static_scratch_of_current_device() {
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return nullptr;
    std::lock_guard<std::mutex> lock(g_init_mutex);
    return g_device_ready[dev] ? g_scratch_ptr[dev] : nullptr;
}
}  // namespace

}  // namespace molora

namespace {

inline bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }
inline bool aligned256(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 255u) == 0; }
inline size_t round256(size_t b) { return (b + 255u) & ~size_t(255); }

inline bool apply_sizes_ok(int64_t N, int32_t d_in, int32_t d_out, int32_t C, int32_t rank) {
    return N >= 0 && N < (int64_t(1) << 31) && d_in >= 8 && d_in % 8 == 0 && d_out >= 8 &&
           d_out % 8 == 0 && C >= 1 && C <= MOLORA_MAX_TARGETS && rank >= 8 && rank % 8 == 0 &&
           rank <= MOLORA_MAX_RANK;
}

struct Workspace {
    int32_t *offsets;
    int32_t *perm;
    uint16_t *t2;
    float *shrink_scratch;  // partial sums of a K-split shrink (nullptr: these sizes never split)
    size_t bytes;
};

inline Workspace carve(void *base, int64_t N, int32_t d_in, int32_t C, int32_t rank) {
    Workspace w;
    unsigned char *p = static_cast<unsigned char *>(base);
    size_t off = 0;
    w.offsets = reinterpret_cast<int32_t *>(p + off);
    off += round256(size_t(C + 1) * sizeof(int32_t));
    w.perm = reinterpret_cast<int32_t *>(p + off);
    off += round256(size_t(N) * sizeof(int32_t));
    w.t2 = reinterpret_cast<uint16_t *>(p + off);
    // token-order form (dispatch and shrink in one launch): a row holds x A_c for every c
    const size_t t_cols = molora::dense_shrink_ok(N, d_in, C, rank) ? size_t(C) * size_t(rank) : size_t(rank);
    off += round256(size_t(N) * 2 * t_cols * sizeof(uint16_t));
    const size_t sb = molora::shrink_scratch_bytes(N, d_in, C, rank);
    w.shrink_scratch = sb ? reinterpret_cast<float *>(p + off) : nullptr;
    off += round256(sb);
    w.bytes = off;
    return w;
}

inline molora_status from_hip(hipError_t e) { return e == hipSuccess ? MOLORA_OK : MOLORA_EHIP; }

molora_status apply_common(const void *x, const void *W, const void *A, const void *B,
                           const int32_t *r, const int32_t *offsets, const int32_t *perm, float *h,
                           int64_t N, int32_t d_in, int32_t d_out, int32_t C, int32_t rank,
                           void *workspace, size_t workspace_bytes, void *stream) {
    if (!apply_sizes_ok(N, d_in, d_out, C, rank) || !molora::fused_gemm_sizes_ok(N, d_in, d_out))
        return MOLORA_EINVAL;
    if (N == 0) return MOLORA_OK;
    if (!x || !W || !A || !B || !h || !workspace) return MOLORA_EINVAL;
    if (r == nullptr && (offsets == nullptr || perm == nullptr)) return MOLORA_EINVAL;
    if (!aligned16(x) || !aligned16(W) || !aligned16(A) || !aligned16(B) || !aligned16(h) ||
        (r && !aligned16(r)) || (offsets && !aligned16(offsets)) || (perm && !aligned16(perm)) ||
        !aligned256(workspace))
        return MOLORA_EALIGN;
    const Workspace ws = carve(workspace, N, d_in, C, rank);
    if (workspace_bytes < ws.bytes) return MOLORA_EWORKSPACE;
    if (molora::ensure_device_ready() != hipSuccess) return MOLORA_EHIP;

    hipStream_t s = static_cast<hipStream_t>(stream);
    const uint16_t *xb = static_cast<const uint16_t *>(x);
    const uint16_t *Ab = static_cast<const uint16_t *>(A);
    hipError_t e;
    if (molora::dense_shrink_ok(N, d_in, C, rank)) {
        // a few narrow adapters: dispatch and token-order shrink beside each other in one
        // launch (the shrink alone when the bucketing is given), then the fused GEMM
        const bool disp = r != nullptr;
        e = molora::launch_dispatch_shrink(nullptr, nullptr, nullptr, 0, 0, const_cast<int32_t *>(r), xb, Ab,
                                           disp ? ws.offsets : nullptr, disp ? ws.perm : nullptr, ws.t2, N,
                                           d_in, C, rank, nullptr, s, disp);
        if (e != hipSuccess) return MOLORA_EHIP;
        if (disp) {
            offsets = ws.offsets;
            perm = ws.perm;
        }
        e = molora::launch_fused_gemm(xb, static_cast<const uint16_t *>(W),
                                      static_cast<const uint16_t *>(B), ws.t2, offsets, perm, h, N,
                                      d_in, d_out, C, rank, molora::Mix{1, C, nullptr, nullptr, 1}, s);
        return from_hip(e);
    }
    // a batch of at most 64 tokens: dispatch, shrink and the base projection in one launch (the
    // latency-bound shrink hides behind the stream of W), then the expand added to h
    if (r != nullptr && molora::sort_in_shrink_ok(N, d_in, C, rank)) {
        const molora::Mix one{1, C, nullptr, nullptr};
        e = molora::launch_small_shrink_base(xb, static_cast<const uint16_t *>(W), Ab, h, ws.t2, N, d_in,
                                             d_out, C, rank, one,
                                             molora::SortArgs{r, ws.offsets, ws.perm, nullptr}, s);
        if (e != hipSuccess) return MOLORA_EHIP;
        return from_hip(molora::launch_small_expand(static_cast<const uint16_t *>(B), ws.t2, ws.offsets,
                                                    ws.perm, h, N, d_in, d_out, C, rank, one, s));
    }
    if (r != nullptr) {
        e = molora::launch_bucket(r, ws.offsets, ws.perm, N, C, nullptr, s);
        if (e != hipSuccess) return MOLORA_EHIP;
        offsets = ws.offsets;
        perm = ws.perm;
    }
    const molora::Mix plain{1, C, nullptr, nullptr};
    e = molora::launch_shrink(xb, Ab, offsets, perm, ws.t2, N, d_in,
                              C, rank, plain, s, ws.shrink_scratch);
    if (e != hipSuccess) return MOLORA_EHIP;
    e = molora::launch_fused_gemm(xb, static_cast<const uint16_t *>(W),
                                  static_cast<const uint16_t *>(B), ws.t2, offsets, perm, h, N,
                                  d_in, d_out, C, rank, plain, s);
    return from_hip(e);
}

}  // namespace

extern "C" {

molora_status molora_route(const void *x, const void *G, int32_t *r, int64_t N, int32_t d_in,
                           int32_t C, void *stream) {
    if (N < 0 || N >= (int64_t(1) << 31) || d_in < 8 || d_in % 8 != 0 || C < 1 ||
        C > MOLORA_MAX_TARGETS)
        return MOLORA_EINVAL;
    if (N == 0) return MOLORA_OK;
    if (!x || !G || !r) return MOLORA_EINVAL;
    if (!aligned16(x) || !aligned16(G) || !aligned16(r)) return MOLORA_EALIGN;
    if (molora::ensure_device_ready() != hipSuccess) return MOLORA_EHIP;
    return from_hip(molora::launch_route_gate(static_cast<const uint16_t *>(x),
                                              static_cast<const uint16_t *>(G), r, nullptr, N, d_in, C,
                                              static_cast<hipStream_t>(stream)));
}

molora_status molora_route_vocab(const int32_t *v, const int32_t *breaks, int32_t M, int32_t *r,
                                 int64_t N, void *stream) {
    if (N < 0 || N >= (int64_t(1) << 31) || M < 1 || M > MOLORA_MAX_BREAKS || !breaks)
        return MOLORA_EINVAL;
    for (int j = 0; j < M; ++j)
        if (breaks[j] >= breaks[j + 1]) return MOLORA_EINVAL;
    if (N == 0) return MOLORA_OK;
    if (!v || !r) return MOLORA_EINVAL;
    if (!aligned16(v) || !aligned16(r)) return MOLORA_EALIGN;
    return from_hip(molora::launch_route_vocab(v, breaks, M, r, N, static_cast<hipStream_t>(stream)));
}

molora_status molora_bucket(const int32_t *r, int32_t *offsets, int32_t *perm, int64_t N,
                            int32_t C, int32_t *err_flag, void *stream) {
    if (N < 0 || N >= (int64_t(1) << 31) || C < 1 || C > MOLORA_MAX_TARGETS) return MOLORA_EINVAL;
    if (!offsets || (N > 0 && (!r || !perm))) return MOLORA_EINVAL;
    if (!aligned16(offsets) || (N > 0 && (!aligned16(r) || !aligned16(perm)))) return MOLORA_EALIGN;
    if (molora::ensure_device_ready() != hipSuccess) return MOLORA_EHIP;
    return from_hip(molora::launch_bucket(r, offsets, perm, N, C, err_flag,
                                          static_cast<hipStream_t>(stream)));
}

molora_status molora_gate_dispatch(const int32_t *v, const int32_t *adapter, const int32_t *breaks,
                                   int32_t M, int32_t n_adapters, int32_t *r, int32_t *offsets,
                                   int32_t *perm, int64_t N, int32_t *err_flag, void *stream) {
    if (N < 0 || N >= (int64_t(1) << 31) || M < 1 || M > MOLORA_MAX_BREAKS || !breaks ||
        n_adapters < 1 || int64_t(n_adapters) * M > MOLORA_MAX_TARGETS)
        return MOLORA_EINVAL;
    for (int j = 0; j < M; ++j)
        if (breaks[j] >= breaks[j + 1]) return MOLORA_EINVAL;
    if (!offsets || (N > 0 && (!v || !r || !perm))) return MOLORA_EINVAL;
    if (!aligned16(offsets) ||
        (N > 0 && (!aligned16(v) || !aligned16(r) || !aligned16(perm) || (adapter && !aligned16(adapter)))))
        return MOLORA_EALIGN;
    if (molora::ensure_device_ready() != hipSuccess) return MOLORA_EHIP;
    return from_hip(molora::launch_gate_bucket(v, adapter, breaks, M, n_adapters, r, offsets, perm, N,
                                               err_flag, static_cast<hipStream_t>(stream)));
}

size_t molora_apply_workspace_bytes(int64_t N, int32_t d_in, int32_t d_out, int32_t C,
                                    int32_t rank) {
    if (!apply_sizes_ok(N, d_in, d_out, C, rank)) return 0;
    return carve(nullptr, N, d_in, C, rank).bytes;
}

molora_status molora_apply(const void *x, const void *W, const void *A, const void *B,
                           const int32_t *r, float *h, int64_t N, int32_t d_in, int32_t d_out,
                           int32_t C, int32_t rank, void *workspace, size_t workspace_bytes,
                           void *stream) {
    if (N > 0 && !r) return MOLORA_EINVAL;
    return apply_common(x, W, A, B, r, nullptr, nullptr, h, N, d_in, d_out, C, rank, workspace,
                        workspace_bytes, stream);
}

size_t molora_static_workspace_bytes(void) { return MOLORA_STATIC_WORKSPACE_BYTES; }

molora_status molora_apply_static(const void *x, const void *W, const void *A, const void *B,
                                  const int32_t *r, float *h, int64_t N, int32_t d_in,
                                  int32_t d_out, int32_t C, int32_t rank, void *stream) {
    if (N > 0 && !r) return MOLORA_EINVAL;
    const size_t need = molora_apply_workspace_bytes(N, d_in, d_out, C, rank);
    if (need == 0) return MOLORA_EINVAL;
    if (need > MOLORA_STATIC_WORKSPACE_BYTES) return MOLORA_EWORKSPACE;
    if (molora::ensure_device_ready() != hipSuccess) return MOLORA_EHIP;
    void *ws = molora::static_scratch_of_current_device();
    if (ws == nullptr) return MOLORA_EHIP;
    // nothing in the workspace has to start at zero: every word the kernels read (offsets,
    // perm, t) is written earlier in the same call
    return apply_common(x, W, A, B, r, nullptr, nullptr, h, N, d_in, d_out, C, rank, ws,
                        MOLORA_STATIC_WORKSPACE_BYTES, stream);
}

molora_status molora_apply_bucketed(const void *x, const void *W, const void *A, const void *B,
                                    const int32_t *offsets, const int32_t *perm, float *h,
                                    int64_t N, int32_t d_in, int32_t d_out, int32_t C, int32_t rank,
                                    void *workspace, size_t workspace_bytes, void *stream) {
    if (N > 0 && (!offsets || !perm)) return MOLORA_EINVAL;
    return apply_common(x, W, A, B, nullptr, offsets, perm, h, N, d_in, d_out, C, rank, workspace,
                        workspace_bytes, stream);
}

size_t molora_shrink_workspace_bytes(int64_t N, int32_t d_in, int32_t C, int32_t rank) {
    if (!apply_sizes_ok(N, d_in, 8, C, rank)) return 0;
    return round256(molora::shrink_scratch_bytes(N, d_in, C, rank));
}

molora_status molora_shrink(const void *x, const void *A, const int32_t *offsets,
                            const int32_t *perm, void *t, int64_t N, int32_t d_in, int32_t C,
                            int32_t rank, void *workspace, size_t workspace_bytes, void *stream) {
    if (!apply_sizes_ok(N, d_in, 8, C, rank)) return MOLORA_EINVAL;
    if (N == 0) return MOLORA_OK;
    if (!x || !A || !offsets || !perm || !t) return MOLORA_EINVAL;
    if (!aligned16(x) || !aligned16(A) || !aligned16(offsets) || !aligned16(perm) || !aligned16(t))
        return MOLORA_EALIGN;
    // the scratch is optional: without it (NULL, or too small) K is never split over workgroups
    float *scratch = nullptr;
    const size_t need = molora::shrink_scratch_bytes(N, d_in, C, rank);
    if (workspace != nullptr && need > 0 && workspace_bytes >= need) {
        if (!aligned256(workspace)) return MOLORA_EALIGN;
        scratch = static_cast<float *>(workspace);
    }
    if (molora::ensure_device_ready() != hipSuccess) return MOLORA_EHIP;
    return from_hip(molora::launch_shrink(static_cast<const uint16_t *>(x),
                                          static_cast<const uint16_t *>(A), offsets, perm,
                                          static_cast<uint16_t *>(t), N, d_in, C, rank,
                                          molora::Mix{1, C, nullptr, nullptr},
                                          static_cast<hipStream_t>(stream), scratch));
}

namespace {
molora_status base_expand_common(const void *x, const void *W, const void *B, const void *t,
                                 const int32_t *offsets, const int32_t *perm, float *h, int64_t N,
                                 int32_t d_in, int32_t d_out, int32_t C, int32_t rank, int tile,
                                 void *stream, bool t_dense = false) {
    if (!apply_sizes_ok(N, d_in, d_out, C, rank)) return MOLORA_EINVAL;
    if (t_dense && !molora::dense_shrink_ok(N, d_in, C, rank)) return MOLORA_EINVAL;
    if (!molora::fused_gemm_sizes_ok(N, d_in, d_out, tile)) return MOLORA_EINVAL;
    if (N == 0) return MOLORA_OK;
    if (!x || !W || !B || !t || !offsets || !perm || !h) return MOLORA_EINVAL;
    if (!aligned16(x) || !aligned16(W) || !aligned16(B) || !aligned16(t) || !aligned16(offsets) ||
        !aligned16(perm) || !aligned16(h))
        return MOLORA_EALIGN;
    if (molora::ensure_device_ready() != hipSuccess) return MOLORA_EHIP;
    return from_hip(molora::launch_fused_gemm(
        static_cast<const uint16_t *>(x), static_cast<const uint16_t *>(W),
        static_cast<const uint16_t *>(B), static_cast<const uint16_t *>(t), offsets, perm, h, N,
        d_in, d_out, C, rank, molora::Mix{1, C, nullptr, nullptr, t_dense ? 1 : 0},
        static_cast<hipStream_t>(stream), tile));
}
}  // namespace

molora_status molora_base_expand(const void *x, const void *W, const void *B, const void *t,
                                 const int32_t *offsets, const int32_t *perm, float *h,
                                 int64_t N, int32_t d_in, int32_t d_out, int32_t C, int32_t rank,
                                 void *stream) {
    return base_expand_common(x, W, B, t, offsets, perm, h, N, d_in, d_out, C, rank, 0, stream);
}

molora_status molora_base_expand_fixed(const void *x, const void *W, const void *B, const void *t,
                                       const int32_t *offsets, const int32_t *perm, float *h,
                                       int64_t N, int32_t d_in, int32_t d_out, int32_t C,
                                       int32_t rank, int32_t tile_rows, void *stream) {
    if (tile_rows != 64 && tile_rows != 128 && tile_rows != 256) return MOLORA_EINVAL;
    return base_expand_common(x, W, B, t, offsets, perm, h, N, d_in, d_out, C, rank, tile_rows,
                              stream);
}

int32_t molora_dense_shrink_supported(int64_t N, int32_t d_in, int32_t C, int32_t rank) {
    return apply_sizes_ok(N, d_in, 8, C, rank) && molora::dense_shrink_ok(N, d_in, C, rank) ? 1 : 0;
}

molora_status molora_bucket_shrink(const int32_t *r, const void *x, const void *A, int32_t *offsets,
                                   int32_t *perm, void *t, int64_t N, int32_t d_in, int32_t C,
                                   int32_t rank, int32_t *err_flag, void *stream) {
    if (!apply_sizes_ok(N, d_in, 8, C, rank) || !molora::dense_shrink_ok(N, d_in, C, rank))
        return MOLORA_EINVAL;
    if (!r || !x || !A || !offsets || !perm || !t) return MOLORA_EINVAL;
    if (!aligned16(r) || !aligned16(x) || !aligned16(A) || !aligned16(offsets) || !aligned16(perm) ||
        !aligned16(t))
        return MOLORA_EALIGN;
    if (molora::ensure_device_ready() != hipSuccess) return MOLORA_EHIP;
    return from_hip(molora::launch_dispatch_shrink(
        nullptr, nullptr, nullptr, 0, 0, const_cast<int32_t *>(r), static_cast<const uint16_t *>(x),
        static_cast<const uint16_t *>(A), offsets, perm, static_cast<uint16_t *>(t), N, d_in, C, rank,
        err_flag, static_cast<hipStream_t>(stream)));
}

int32_t molora_bucket_shrink_small_supported(int64_t N, int32_t d_in, int32_t C, int32_t rank) {
    return apply_sizes_ok(N, d_in, 8, C, rank) && molora::sort_in_shrink_ok(N, d_in, C, rank) ? 1 : 0;
}

molora_status molora_bucket_shrink_small(const int32_t *r, const void *x, const void *A,
                                         int32_t *offsets, int32_t *perm, void *t, int64_t N,
                                         int32_t d_in, int32_t C, int32_t rank, void *workspace,
                                         size_t workspace_bytes, int32_t *err_flag, void *stream) {
    if (!apply_sizes_ok(N, d_in, 8, C, rank) || !molora::sort_in_shrink_ok(N, d_in, C, rank))
        return MOLORA_EINVAL;
    if (!r || !x || !A || !offsets || !perm || !t) return MOLORA_EINVAL;
    if (!aligned16(r) || !aligned16(x) || !aligned16(A) || !aligned16(offsets) || !aligned16(perm) ||
        !aligned16(t))
        return MOLORA_EALIGN;
    float *scratch = nullptr;  // optional, as in molora_shrink
    const size_t need = molora::shrink_scratch_bytes(N, d_in, C, rank);
    if (workspace != nullptr && need > 0 && workspace_bytes >= need) {
        if (!aligned256(workspace)) return MOLORA_EALIGN;
        scratch = static_cast<float *>(workspace);
    }
    if (molora::ensure_device_ready() != hipSuccess) return MOLORA_EHIP;
    return from_hip(molora::launch_shrink(static_cast<const uint16_t *>(x),
                                          static_cast<const uint16_t *>(A), nullptr, nullptr,
                                          static_cast<uint16_t *>(t), N, d_in, C, rank,
                                          molora::Mix{1, C, nullptr, nullptr},
                                          static_cast<hipStream_t>(stream), scratch,
                                          molora::SortArgs{r, offsets, perm, err_flag}));
}

namespace {
molora_status shrink_base_small_common(const int32_t *r, const void *x, const void *W, const void *A,
                                       int32_t *offsets, int32_t *perm, void *t, float *h, int64_t N,
                                       int32_t d_in, int32_t d_out, int32_t C, int32_t rank,
                                       int32_t *err_flag, void *stream, bool w_packed) {
    if (!apply_sizes_ok(N, d_in, d_out, C, rank) || !molora::sort_in_shrink_ok(N, d_in, C, rank))
        return MOLORA_EINVAL;
    if (w_packed && molora::small_pack_cols(d_out) == 0) return MOLORA_EINVAL;
    if (!r || !x || !W || !A || !offsets || !perm || !t || !h) return MOLORA_EINVAL;
    if (!aligned16(r) || !aligned16(x) || !aligned16(W) || !aligned16(A) || !aligned16(offsets) ||
        !aligned16(perm) || !aligned16(t) || !aligned16(h))
        return MOLORA_EALIGN;
    if (molora::ensure_device_ready() != hipSuccess) return MOLORA_EHIP;
    return from_hip(molora::launch_small_shrink_base(
        static_cast<const uint16_t *>(x), static_cast<const uint16_t *>(W),
        static_cast<const uint16_t *>(A), h, static_cast<uint16_t *>(t), N, d_in, d_out, C, rank,
        molora::Mix{1, C, nullptr, nullptr}, molora::SortArgs{r, offsets, perm, err_flag},
        static_cast<hipStream_t>(stream), w_packed));
}
}  // namespace

molora_status molora_shrink_base_small(const int32_t *r, const void *x, const void *W, const void *A,
                                       int32_t *offsets, int32_t *perm, void *t, float *h, int64_t N,
                                       int32_t d_in, int32_t d_out, int32_t C, int32_t rank,
                                       int32_t *err_flag, void *stream) {
    return shrink_base_small_common(r, x, W, A, offsets, perm, t, h, N, d_in, d_out, C, rank, err_flag,
                                    stream, false);
}

molora_status molora_shrink_base_small_packed(const int32_t *r, const void *x, const void *Wp,
                                              const void *A, int32_t *offsets, int32_t *perm, void *t,
                                              float *h, int64_t N, int32_t d_in, int32_t d_out,
                                              int32_t C, int32_t rank, int32_t *err_flag,
                                              void *stream) {
    return shrink_base_small_common(r, x, Wp, A, offsets, perm, t, h, N, d_in, d_out, C, rank, err_flag,
                                    stream, true);
}

int32_t molora_pack_w_cols(int32_t d_out) { return d_out >= 8 ? molora::small_pack_cols(d_out) : 0; }

molora_status molora_pack_w(const void *W, void *Wp, int32_t d_in, int32_t d_out, void *stream) {
    if (d_in < 8 || d_in % 8 != 0 || d_out < 8 || molora::small_pack_cols(d_out) == 0) return MOLORA_EINVAL;
    if (!W || !Wp || W == Wp) return MOLORA_EINVAL;
    if (!aligned16(W) || !aligned16(Wp)) return MOLORA_EALIGN;
    if (molora::ensure_device_ready() != hipSuccess) return MOLORA_EHIP;
    return from_hip(molora::launch_pack_w(static_cast<const uint16_t *>(W), static_cast<uint16_t *>(Wp),
                                          d_in, d_out, static_cast<hipStream_t>(stream)));
}

namespace {
molora_status expand_small_common(const void *B, const void *t, const int32_t *offsets,
                                  const int32_t *perm, float *h, int64_t N, int32_t d_out, int32_t C,
                                  int32_t rank, void *stream, bool b_packed) {
    const int32_t d_in = 8;  // the step does not touch x or W
    if (!apply_sizes_ok(N, d_in, d_out, C, rank) || N > 64) return MOLORA_EINVAL;
    if (b_packed && (rank % 16 != 0 || molora::small_pack_cols(d_out) == 0)) return MOLORA_EINVAL;
    if (N == 0) return MOLORA_OK;
    if (!B || !t || !offsets || !perm || !h) return MOLORA_EINVAL;
    if (!aligned16(B) || !aligned16(t) || !aligned16(offsets) || !aligned16(perm) || !aligned16(h))
        return MOLORA_EALIGN;
    if (molora::ensure_device_ready() != hipSuccess) return MOLORA_EHIP;
    return from_hip(molora::launch_small_expand(static_cast<const uint16_t *>(B),
                                                static_cast<const uint16_t *>(t), offsets, perm, h, N, d_in,
                                                d_out, C, rank, molora::Mix{1, C, nullptr, nullptr},
                                                static_cast<hipStream_t>(stream), b_packed));
}
}  // namespace

molora_status molora_expand_small(const void *B, const void *t, const int32_t *offsets,
                                  const int32_t *perm, float *h, int64_t N, int32_t d_out, int32_t C,
                                  int32_t rank, void *stream) {
    return expand_small_common(B, t, offsets, perm, h, N, d_out, C, rank, stream, false);
}

molora_status molora_expand_small_packed(const void *Bp, const void *t, const int32_t *offsets,
                                         const int32_t *perm, float *h, int64_t N, int32_t d_out,
                                         int32_t C, int32_t rank, void *stream) {
    return expand_small_common(Bp, t, offsets, perm, h, N, d_out, C, rank, stream, true);
}

molora_status molora_gate_dispatch_shrink(const int32_t *v, const int32_t *adapter,
                                          const int32_t *breaks, int32_t M, int32_t n_adapters,
                                          const void *x, const void *A, int32_t *r, int32_t *offsets,
                                          int32_t *perm, void *t, int64_t N, int32_t d_in,
                                          int32_t rank, int32_t *err_flag, void *stream) {
    if (M < 1 || M > MOLORA_MAX_BREAKS || !breaks || n_adapters < 1 ||
        int64_t(n_adapters) * M > MOLORA_MAX_TARGETS)
        return MOLORA_EINVAL;
    const int32_t C = n_adapters * M;
    if (!apply_sizes_ok(N, d_in, 8, C, rank) || !molora::dense_shrink_ok(N, d_in, C, rank))
        return MOLORA_EINVAL;
    for (int j = 0; j < M; ++j)
        if (breaks[j] >= breaks[j + 1]) return MOLORA_EINVAL;
    if (!v || !x || !A || !r || !offsets || !perm || !t) return MOLORA_EINVAL;
    if (!aligned16(v) || (adapter && !aligned16(adapter)) || !aligned16(x) || !aligned16(A) ||
        !aligned16(r) || !aligned16(offsets) || !aligned16(perm) || !aligned16(t))
        return MOLORA_EALIGN;
    if (molora::ensure_device_ready() != hipSuccess) return MOLORA_EHIP;
    return from_hip(molora::launch_dispatch_shrink(
        v, adapter, breaks, M, n_adapters, r, static_cast<const uint16_t *>(x),
        static_cast<const uint16_t *>(A), offsets, perm, static_cast<uint16_t *>(t), N, d_in, C, rank,
        err_flag, static_cast<hipStream_t>(stream)));
}

molora_status molora_base_expand_dense(const void *x, const void *W, const void *B, const void *t,
                                       const int32_t *offsets, const int32_t *perm, float *h,
                                       int64_t N, int32_t d_in, int32_t d_out, int32_t C,
                                       int32_t rank, void *stream) {
    return base_expand_common(x, W, B, t, offsets, perm, h, N, d_in, d_out, C, rank, 0, stream, true);
}

size_t molora_route_mlp_workspace_bytes(int64_t N, int32_t H) {
    if (N < 0 || N >= (int64_t(1) << 31) || H < 8 || H % 8 != 0 || H > MOLORA_MAX_HIDDEN) return 0;
    return round256(size_t(N) * size_t(H) * sizeof(float));
}

molora_status molora_route_mlp(const void *x, const void *W1, const float *b1, const void *W2,
                               const float *b2, int32_t *idx, float *w, int64_t N, int32_t d_in,
                               int32_t H, int32_t K, int32_t k, void *workspace,
                               size_t workspace_bytes, void *stream) {
    if (N < 0 || N >= (int64_t(1) << 31) || d_in < 8 || d_in % 8 != 0 || H < 8 || H % 8 != 0 ||
        H > MOLORA_MAX_HIDDEN || K < 1 || K > MOLORA_MAX_TARGETS || k < 1 || k > MOLORA_MAX_TOPK ||
        k > K)
        return MOLORA_EINVAL;
    if (N == 0) return MOLORA_OK;
    if (!x || !W1 || !b1 || !W2 || !b2 || !idx || !w || !workspace) return MOLORA_EINVAL;
    if (!aligned16(x) || !aligned16(W1) || !aligned16(b1) || !aligned16(W2) || !aligned16(b2) ||
        !aligned16(idx) || !aligned16(w) || !aligned256(workspace))
        return MOLORA_EALIGN;
    if (workspace_bytes < molora_route_mlp_workspace_bytes(N, H)) return MOLORA_EWORKSPACE;
    if (molora::ensure_device_ready() != hipSuccess) return MOLORA_EHIP;
    hipStream_t s = static_cast<hipStream_t>(stream);
    float *u = static_cast<float *>(workspace);
    hipError_t e = molora::launch_route_gate(static_cast<const uint16_t *>(x),
                                             static_cast<const uint16_t *>(W1), nullptr, u, N, d_in,
                                             H, s);
    if (e != hipSuccess) return MOLORA_EHIP;
    return from_hip(molora::launch_router_finish(u, b1, static_cast<const uint16_t *>(W2), b2, idx, w,
                                                 N, H, K, k, s));
}

molora_status molora_route_compose(const int32_t *v, const int32_t *adapter, const int32_t *breaks,
                                   int32_t M, int32_t n_adapters, int32_t *r, int64_t N,
                                   void *stream) {
    if (N < 0 || N >= (int64_t(1) << 31) || M < 1 || M > MOLORA_MAX_BREAKS || !breaks ||
        n_adapters < 1 || int64_t(n_adapters) * M > MOLORA_MAX_TARGETS)
        return MOLORA_EINVAL;
    for (int j = 0; j < M; ++j)
        if (breaks[j] >= breaks[j + 1]) return MOLORA_EINVAL;
    if (N == 0) return MOLORA_OK;
    if (!v || !adapter || !r) return MOLORA_EINVAL;
    if (!aligned16(v) || !aligned16(adapter) || !aligned16(r)) return MOLORA_EALIGN;
    return from_hip(molora::launch_route_compose(v, adapter, breaks, M, n_adapters, r, N,
                                                 static_cast<hipStream_t>(stream)));
}

namespace {

// number of tuples C^k, or 0 when it exceeds the bucket limit
inline int64_t mix_buckets(int32_t C, int32_t k) {
    int64_t cb = 1;
    for (int j = 0; j < k; ++j) {
        cb *= C;
        if (cb > MOLORA_MAX_TARGETS) return 0;
    }
    return cb;
}

inline bool mix_sizes_ok(int64_t N, int32_t d_in, int32_t d_out, int32_t C, int32_t rank, int32_t k) {
    return k >= 1 && k <= MOLORA_MAX_TOPK && apply_sizes_ok(N, d_in, d_out, C, rank) &&
           int64_t(k) * rank <= MOLORA_MAX_RANK && mix_buckets(C, k) > 0;
}

struct MixWorkspace {
    int32_t *key;
    float *wq;
    int32_t *offsets;
    int32_t *perm;
    uint16_t *t2;
    float *shrink_scratch;
    size_t bytes;
};

inline MixWorkspace carve_mix(void *base, int64_t N, int32_t d_in, int32_t C, int32_t rank, int32_t k) {
    MixWorkspace w;
    unsigned char *p = static_cast<unsigned char *>(base);
    size_t off = 0;
    w.key = reinterpret_cast<int32_t *>(p + off);
    off += round256(size_t(N) * sizeof(int32_t));
    w.wq = reinterpret_cast<float *>(p + off);
    off += round256(size_t(N) * size_t(k) * sizeof(float));
    w.offsets = reinterpret_cast<int32_t *>(p + off);
    off += round256(size_t(mix_buckets(C, k) + 1) * sizeof(int32_t));
    w.perm = reinterpret_cast<int32_t *>(p + off);
    off += round256(size_t(N) * sizeof(int32_t));
    w.t2 = reinterpret_cast<uint16_t *>(p + off);
    off += round256(size_t(N) * 2 * size_t(k) * size_t(rank) * sizeof(uint16_t));
    const size_t sb = molora::shrink_scratch_bytes(N, d_in, (int)mix_buckets(C, k), k * rank);
    w.shrink_scratch = sb ? reinterpret_cast<float *>(p + off) : nullptr;
    off += round256(sb);
    w.bytes = off;
    return w;
}

}  // namespace

size_t molora_apply_mix_workspace_bytes(int64_t N, int32_t d_in, int32_t d_out, int32_t C,
                                        int32_t rank, int32_t k) {
    if (!mix_sizes_ok(N, d_in, d_out, C, rank, k)) return 0;
    return carve_mix(nullptr, N, d_in, C, rank, k).bytes;
}

molora_status molora_apply_mix(const void *x, const void *W, const void *A, const void *B,
                               const int32_t *idx, const float *w, const int32_t *slots, float *h,
                               int64_t N, int32_t d_in, int32_t d_out, int32_t C, int32_t rank,
                               int32_t k, void *workspace, size_t workspace_bytes, void *stream) {
    if (!mix_sizes_ok(N, d_in, d_out, C, rank, k) || !molora::fused_gemm_sizes_ok(N, d_in, d_out))
        return MOLORA_EINVAL;
    if (N == 0) return MOLORA_OK;
    if (!x || !W || !A || !B || !idx || !h || !workspace) return MOLORA_EINVAL;
    if (!aligned16(x) || !aligned16(W) || !aligned16(A) || !aligned16(B) || !aligned16(idx) ||
        (w && !aligned16(w)) || (slots && !aligned16(slots)) || !aligned16(h) ||
        !aligned256(workspace))
        return MOLORA_EALIGN;
    const MixWorkspace ws = carve_mix(workspace, N, d_in, C, rank, k);
    if (workspace_bytes < ws.bytes) return MOLORA_EWORKSPACE;
    if (molora::ensure_device_ready() != hipSuccess) return MOLORA_EHIP;
    const int Cb = (int)mix_buckets(C, k);
    hipStream_t s = static_cast<hipStream_t>(stream);
    const uint16_t *xb = static_cast<const uint16_t *>(x);
    if (molora::launch_mix_key(idx, w, ws.key, ws.wq, N, C, k, s) != hipSuccess) return MOLORA_EHIP;
    if (molora::launch_bucket(ws.key, ws.offsets, ws.perm, N, Cb, nullptr, s) != hipSuccess)
        return MOLORA_EHIP;
    const molora::Mix mix{k, C, slots, ws.wq};
    if (molora::launch_shrink(xb, static_cast<const uint16_t *>(A), ws.offsets, ws.perm, ws.t2, N,
                              d_in, Cb, rank, mix, s, ws.shrink_scratch) != hipSuccess)
        return MOLORA_EHIP;
    return from_hip(molora::launch_fused_gemm(xb, static_cast<const uint16_t *>(W),
                                              static_cast<const uint16_t *>(B), ws.t2, ws.offsets,
                                              ws.perm, h, N, d_in, d_out, Cb, rank, mix, s));
}

const char *molora_status_string(molora_status status) {
    switch (status) {
        case MOLORA_OK: return "ok";
        case MOLORA_EINVAL: return "invalid argument (null pointer or unsupported size)";
        case MOLORA_EALIGN: return "device pointer not sufficiently aligned";
        case MOLORA_EWORKSPACE: return "workspace too small";
        case MOLORA_EHIP: return "HIP runtime error at kernel launch";
        default: return "unknown status";
    }
}

const char *molora_version(void) { return "molora-gfx950 0.9"; }

molora_status molora_init(void) {
    return molora::ensure_device_ready() == hipSuccess ? MOLORA_OK : MOLORA_EHIP;
}

}  // extern "C"
