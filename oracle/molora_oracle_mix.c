/*
 * CPU oracle, second part: the learned router of Sec. "Router Architecture", the weighted
 * top-k mixture it feeds, compositional gating (Alg. "Compositional Gating Kernel") and the
 * slot table of the hot-set layout (Def. "Hot-Set Layout").
 *
 * THIS IS TEST INFRASTRUCTURE, NOT THE PRODUCT (see molora_oracle.c).
 *
 *   g(x)  = W2^T GELU(W1^T x + b1) + b2            (2-layer MLP, hidden width H)
 *   w_i   = softmax(TopK(g(x_i), k))
 *   h_i   = x_i W + sum_{j in TopK} w_ij (x_i A_j) B_j
 *
 * Numerics.  x, W1, W2, W, A, B are bf16 bit patterns widened exactly; b1, b2 fp32.  Every
 * sum is a sequential fp32 accumulation in ascending index order starting from 0, one
 * rounded multiply and one rounded add per term (no fused multiply-add: compile with
 * -ffp-contract=off); a bias is added after the sum.  The top-k selection is an integer
 * decision taken on fp32 logits, so the logits must not depend on a math library: GELU is
 * the exact form 0.5 u (1 + erf(u / sqrt 2)) with erf from the rational approximation 7.1.26
 * of Abramowitz and Stegun (|error| <= 1.5e-7) and exp from the range reduction
 * exp(y) = 2^n exp(r), n = rint(y / ln 2), with a degree-7 Taylor polynomial in r; both are
 * written out below in plain fp32 operations whose order is part of the definition.  The
 * softmax weights use the same exp.  Selection: k times the largest remaining logit, the
 * lowest index among equals (strict '>' scan).  Inputs are expected to be finite: a NaN
 * logit is never selected over an earlier candidate, but the first remaining candidate of a
 * scan is its starting point and stays selected if it is NaN (nothing compares greater).
 *
 * Pins (tests/test_oracle_mix.py): float64 numpy MLP with math.erf, numpy argsort for the
 * selection, k = 1 reducing bit-exactly to the single-adapter oracle, equal logits giving
 * the plain average over brute-force single-adapter outputs, weights summing to 1,
 * numpy.searchsorted arithmetic for the composite target, identity / permuted slot tables.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

static inline float bf16_to_f32(uint16_t b)
{
    uint32_t u = (uint32_t)b << 16;
    float f;
    memcpy(&f, &u, sizeof f);
    return f;
}

/* exp(y) for y in [-87, 88]; 0 below.  n * LN2_HI is exact for |n| <= 128. */
float oracle_expf(float y)
{
    const float LOG2E = 1.44269502162933349609375f;
    const float LN2_HI = 0.693145751953125f;         /* 22713 / 32768 */
    const float LN2_LO = 1.428606820309417e-06f;       /* ln 2 - LN2_HI */
    if (!(y >= -87.0f)) return 0.0f;
    if (y > 88.0f) y = 88.0f;
    const float n = rintf(y * LOG2E);
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

/* erf(z), z >= 0: Abramowitz and Stegun 7.1.26 */
static float erf_as(float z)
{
    const float t = 1.0f / (1.0f + 0.3275911f * z);
    float s = 1.061405429f;
    s = s * t + -1.453152027f;
    s = s * t + 1.421413741f;
    s = s * t + -0.284496736f;
    s = s * t + 0.254829592f;
    s = s * t;
    return 1.0f - s * oracle_expf(-(z * z));
}

float oracle_gelu(float u)
{
    const float z = fabsf(u) * 0.707106769084930419921875f;
    const float e = erf_as(z);
    const float s = (u < 0.0f) ? -e : e;
    return (0.5f * u) * (1.0f + s);
}

/*
 * Router logits.  x [N][d] bf16, W1 [d][H] bf16, b1 [H] fp32, W2 [H][K] bf16, b2 [K] fp32
 * -> logits [N][K] fp32 (parameter count H d + H K, Sec. "Router Architecture").
 */
int oracle_mlp_logits(const uint16_t *x, const uint16_t *W1, const float *b1, const uint16_t *W2,
                      const float *b2, float *logits, int64_t N, int32_t d, int32_t H, int32_t K)
{
    float *u = (float *)malloc((size_t)(H > 0 ? H : 1) * sizeof(float));
    if (!u) return -1;
    for (int64_t i = 0; i < N; ++i) {
        for (int j = 0; j < H; ++j) {
            float acc = 0.0f;
            for (int k = 0; k < d; ++k) {
                const float p = bf16_to_f32(x[(size_t)i * d + k]) * bf16_to_f32(W1[(size_t)k * H + j]);
                acc = acc + p;
            }
            u[j] = oracle_gelu(acc + b1[j]);
        }
        for (int c = 0; c < K; ++c) {
            float acc = 0.0f;
            for (int j = 0; j < H; ++j) {
                const float p = u[j] * bf16_to_f32(W2[(size_t)j * K + c]);
                acc = acc + p;
            }
            logits[(size_t)i * K + c] = acc + b2[c];
        }
    }
    free(u);
    return 0;
}

/*
 * idx [N][k]: the k largest logits of each row in descending order (lowest index first
 * among equals); w [N][k] = softmax over the selected logits.
 */
void oracle_topk_softmax(const float *logits, int32_t *idx, float *w, int64_t N, int32_t K, int32_t k)
{
    for (int64_t i = 0; i < N; ++i) {
        const float *l = logits + (size_t)i * K;
        int32_t *id = idx + (size_t)i * k;
        float *wi = w + (size_t)i * k;
        for (int j = 0; j < k; ++j) {
            int best = -1;
            for (int c = 0; c < K; ++c) {
                int taken = 0;
                for (int q = 0; q < j; ++q) taken |= (id[q] == c);
                if (taken) continue;
                if (best < 0 || l[c] > l[best]) best = c;
            }
            id[j] = best;
        }
        const float m = l[id[0]];
        float sum = 0.0f;
        for (int j = 0; j < k; ++j) {
            wi[j] = oracle_expf(l[id[j]] - m);
            sum = sum + wi[j];
        }
        for (int j = 0; j < k; ++j) wi[j] = wi[j] / sum;
    }
}

/*
 * Weighted mixture, one token at a time:
 *   base[n] = sum_k x[k] W[k][n];  for j < k, c = slot(idx[j]):
 *   t[q] = sum_k x[k] A_c[k][q];  d_j[n] = sum_q t[q] B_c[q][n];  h[n] = base[n] + sum_j w[j] d_j[n]
 * (j ascending; an index outside [0, C) contributes nothing).  slots == NULL: slot(c) = c;
 * otherwise adapter c lives in position slots[c] of the pools A [S][d_in][rank],
 * B [S][rank][d_out] (Def. "Hot-Set Layout": a table maps what requests name to where it is
 * resident).  w == NULL: all weights 1.
 */
int oracle_apply_mix(const uint16_t *x, const uint16_t *W, const uint16_t *A, const uint16_t *B,
                     const int32_t *idx, const float *w, const int32_t *slots, float *h, int64_t N,
                     int32_t d_in, int32_t d_out, int32_t C, int32_t rank, int32_t k)
{
    float *base = (float *)malloc(((size_t)2 * d_out + rank) * sizeof(float));
    if (!base) return -1;
    float *dj = base + d_out, *t = dj + d_out;
    for (int64_t i = 0; i < N; ++i) {
        const uint16_t *xi = x + (size_t)i * d_in;
        for (int n = 0; n < d_out; ++n) base[n] = 0.0f;
        for (int kk = 0; kk < d_in; ++kk) {
            const float xv = bf16_to_f32(xi[kk]);
            for (int n = 0; n < d_out; ++n) {
                const float p = xv * bf16_to_f32(W[(size_t)kk * d_out + n]);
                base[n] = base[n] + p;
            }
        }
        float *hi = h + (size_t)i * d_out;
        for (int n = 0; n < d_out; ++n) hi[n] = base[n];
        for (int j = 0; j < k; ++j) {
            const int32_t c = idx[(size_t)i * k + j];
            if (c < 0 || c >= C) continue;
            const int32_t s = slots ? slots[c] : c;
            const uint16_t *Ac = A + (size_t)s * d_in * rank;
            const uint16_t *Bc = B + (size_t)s * rank * d_out;
            for (int q = 0; q < rank; ++q) t[q] = 0.0f;
            for (int kk = 0; kk < d_in; ++kk) {
                const float xv = bf16_to_f32(xi[kk]);
                for (int q = 0; q < rank; ++q) {
                    const float p = xv * bf16_to_f32(Ac[(size_t)kk * rank + q]);
                    t[q] = t[q] + p;
                }
            }
            for (int n = 0; n < d_out; ++n) dj[n] = 0.0f;
            for (int q = 0; q < rank; ++q)
                for (int n = 0; n < d_out; ++n) {
                    const float p = t[q] * bf16_to_f32(Bc[(size_t)q * d_out + n]);
                    dj[n] = dj[n] + p;
                }
            const float wj = w ? w[(size_t)i * k + j] : 1.0f;
            for (int n = 0; n < d_out; ++n) {
                const float p = wj * dj[n];
                hi[n] = hi[n] + p;
            }
        }
    }
    free(base);
    return 0;
}

/*
 * Compositional gating: c = a * M + m with a = adapter[i] (from request metadata) and m the
 * modality of vocabulary index v[i], breaks[m] <= v < breaks[m+1].  -1 when the vocabulary
 * index falls outside [breaks[0], breaks[M]) or the adapter index outside [0, n_adapters).
 */
void oracle_route_compose(const int32_t *v, const int32_t *adapter, const int32_t *breaks, int32_t M,
                          int32_t n_adapters, int32_t *r, int64_t N)
{
    for (int64_t i = 0; i < N; ++i) {
        int32_t m = -1;
        for (int j = 0; j < M; ++j)
            if (v[i] >= breaks[j] && v[i] < breaks[j + 1]) m = j;
        const int32_t a = adapter[i];
        r[i] = (m < 0 || a < 0 || a >= n_adapters) ? -1 : a * M + m;
    }
}
