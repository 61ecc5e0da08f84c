// Small routing kernels around the learned router and compositional gating:
//   * the second half of the router MLP of Sec. "Router Architecture"
//       logits = W2^T GELU(u + b1) + b2,  idx = TopK(logits, k),  w = softmax(logits[idx])
//     (u = x W1 comes from the exact-chain gate kernel);
//   * the bucket key of a weighted top-k mixture (a tuple of k adapters per token);
//   * the composite target c = a |M| + m of Alg. "Compositional Gating Kernel".
//
// The top-k selection is an integer decision taken on fp32 values, so the logits are computed
// as a fixed sequence of individually rounded fp32 operations (no contraction into fused
// multiply-adds, no math library): sums are sequential in ascending index order from 0 with the
// bias added last; GELU is 0.5 u (1 + erf(u / sqrt 2)) with erf from the rational
// approximation 7.1.26 of Abramowitz and Stegun and exp(y) = 2^n exp(r), n = rint(y / ln 2),
// exp(r) a degree-7 Taylor polynomial.  Selection takes k times the largest remaining logit,
// the lowest index among equals.
#include "common.h"

// every fp32 operation below is rounded on its own: no fused multiply-add may be formed
#pragma clang fp contract(off)

namespace molora {

namespace {

struct Breaks {
    int32_t b[65];
};


__device__ float exp_fixed(float y) {
    const float LOG2E = 1.44269502162933349609375f;
    const float LN2_HI = 0.693145751953125f;   // 22713 / 32768: n * LN2_HI is exact for |n| <= 128
    const float LN2_LO = 1.428606820309417e-06f;
    if (!(y >= -87.0f)) return 0.0f;
    if (y > 88.0f) y = 88.0f;
    const float n = __builtin_rintf(y * LOG2E);
    float r = y - n * LN2_HI;
    r = r - n * LN2_LO;
    float p = 1.0f / 5040.0f;
    p = p * r + 1.0f / 720.0f;
    p = p * r + 1.0f / 120.0f;
    p = p * r + 1.0f / 24.0f;
    p = p * r + 1.0f / 6.0f;
    p = p * r + 0.5f;
    p = p * r + 1.0f;
    p = p * r + 1.0f;
    return ldexpf(p, (int)n);
}

__device__ float erf_rational(float z) {  // z >= 0
    const float t = 1.0f / (1.0f + 0.3275911f * z);
    float s = 1.061405429f;
    s = s * t + -1.453152027f;
    s = s * t + 1.421413741f;
    s = s * t + -0.284496736f;
    s = s * t + 0.254829592f;
    s = s * t;
    return 1.0f - s * exp_fixed(-(z * z));
}

__device__ float gelu_fixed(float u) {
    const float z = __builtin_fabsf(u) * 0.707106769084930419921875f;
    const float e = erf_rational(z);
    const float s = (u < 0.0f) ? -e : e;
    return (0.5f * u) * (1.0f + s);
}

constexpr int kFinTok = 8;        // tokens per workgroup
constexpr int kFinThreads = 256;

__global__ __launch_bounds__(kFinThreads) void router_finish_kernel(
    const float *__restrict__ u, const float *__restrict__ b1, const uint16_t *__restrict__ W2,
    const float *__restrict__ b2, int32_t *__restrict__ idx, float *__restrict__ w, int64_t N,
    int H, int K, int k) {
    extern __shared__ float fin_lds[];
    float *g = fin_lds;                // [kFinTok][H]
    float *logit = g + kFinTok * H;    // [kFinTok][K]
    const int tid = threadIdx.x;
    const int64_t t0 = (int64_t)blockIdx.x * kFinTok;
    const int nt = (int)min((int64_t)kFinTok, N - t0);

    for (int e = tid; e < nt * H; e += kFinThreads) {
        const int t = e / H, j = e % H;
        g[t * H + j] = gelu_fixed(u[(t0 + t) * H + j] + b1[j]);
    }
    __syncthreads();
    for (int e = tid; e < nt * K; e += kFinThreads) {
        const int t = e / K, c = e % K;
        float acc = 0.0f;
        for (int j = 0; j < H; ++j)
            acc = acc + g[t * H + j] * bf16_bits_to_f32(W2[(int64_t)j * K + c]);
        logit[t * K + c] = acc + b2[c];
    }
    __syncthreads();
    if (tid < nt) {
        const float *l = logit + tid * K;
        int32_t *id = idx + (t0 + tid) * k;
        float *wi = w + (t0 + tid) * k;
        int sel[4];
        for (int j = 0; j < k; ++j) {
            int best = -1;
            for (int c = 0; c < K; ++c) {
                bool taken = false;
                for (int q = 0; q < j; ++q) taken |= (sel[q] == c);
                if (taken) continue;
                if (best < 0 || l[c] > l[best]) best = c;
            }
            sel[j] = best;
            id[j] = best;
        }
        const float m = l[sel[0]];
        float e[4], sum = 0.0f;
        for (int j = 0; j < k; ++j) {
            e[j] = exp_fixed(l[sel[j]] - m);
            sum = sum + e[j];
        }
        for (int j = 0; j < k; ++j) wi[j] = e[j] / sum;
    }
}

__global__ __launch_bounds__(256) void mix_key_kernel(const int32_t *__restrict__ idx,
                                                      const float *__restrict__ w,
                                                      int32_t *__restrict__ key,
                                                      float *__restrict__ wq, int64_t N, int C, int k) {
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= N) return;
    int32_t kv = 0, mul = 1;
    for (int j = 0; j < k; ++j) {
        const int32_t c = idx[i * k + j];
        const bool ok = c >= 0 && c < C;
        kv += (ok ? c : 0) * mul;
        mul *= C;
        wq[i * k + j] = ok ? (w != nullptr ? w[i * k + j] : 1.0f) : 0.0f;
    }
    key[i] = kv;
}

__global__ __launch_bounds__(256) void route_compose_kernel(const int32_t *__restrict__ v,
                                                            const int32_t *__restrict__ adapter,
                                                            int32_t *__restrict__ r, int64_t N,
                                                            Breaks br, int M, int n_adapters) {
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= N) return;
    const int32_t id = v[i], a = adapter[i];
    int32_t m = 0;
    for (int j = 1; j < M; ++j)  // M - 1 integer comparisons
        if (id >= br.b[j]) m = j;
    const bool ok = id >= br.b[0] && id < br.b[M] && a >= 0 && a < n_adapters;
    r[i] = ok ? a * M + m : -1;
}

}  // namespace

hipError_t launch_router_finish(const float *u, const float *b1, const uint16_t *W2, const float *b2,
                                int32_t *idx, float *w, int64_t N, int H, int K, int k, hipStream_t s) {
    if (N == 0) return hipSuccess;
    const size_t lds = (size_t)kFinTok * (H + K) * sizeof(float);  // <= 40 KB at H = 256, K = 1024
    const unsigned blocks = (unsigned)((N + kFinTok - 1) / kFinTok);
    hipLaunchKernelGGL(router_finish_kernel, dim3(blocks), dim3(kFinThreads), lds, s, u, b1, W2, b2,
                       idx, w, N, H, K, k);
    return hipGetLastError();
}

hipError_t launch_mix_key(const int32_t *idx, const float *w, int32_t *key, float *wq, int64_t N,
                          int C, int k, hipStream_t s) {
    if (N == 0) return hipSuccess;
    hipLaunchKernelGGL(mix_key_kernel, dim3((unsigned)((N + 255) / 256)), dim3(256), 0, s, idx, w, key,
                       wq, N, C, k);
    return hipGetLastError();
}

hipError_t launch_route_compose(const int32_t *v, const int32_t *adapter, const int32_t *breaks_host,
                                int M, int n_adapters, int32_t *r, int64_t N, hipStream_t s) {
    if (N == 0) return hipSuccess;
    Breaks br;
    for (int j = 0; j <= M; ++j) br.b[j] = breaks_host[j];
    for (int j = M + 1; j < 65; ++j) br.b[j] = 0;
    hipLaunchKernelGGL(route_compose_kernel, dim3((unsigned)((N + 255) / 256)), dim3(256), 0, s, v,
                       adapter, r, N, br, M, n_adapters);
    return hipGetLastError();
}

}  // namespace molora
