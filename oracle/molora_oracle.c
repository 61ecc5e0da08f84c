/*
 * CPU oracle for the per-token routed LoRA projection (MoLoRA, Eq. "pertok"):
 *
 *     h_i = x_i W + x_i A_{r(i)} B_{r(i)},      r : [N] -> [C]
 *
 * THIS IS TEST INFRASTRUCTURE, NOT THE PRODUCT.  It is a slow, literal,
 * per-token transcription of the definitions in the paper and shares no code
 * with the HIP library.  Only the tests, the smoke check and the benchmark's
 * cpu_baseline leg may call it.
 *
 * Numerics (fixed by the build's problem statement, the paper being silent):
 * inputs are bf16 bit patterns widened exactly to fp32; every sum is an fp32
 * accumulation in ascending index order, one rounded add per term; the low-rank
 * intermediate t = x A_c stays in fp32; h is fp32.  Compile with
 * -ffp-contract=off and without fast-math so the order below is the order run.
 * OpenMP parallelises over tokens only, which changes no element's arithmetic.
 *
 * Pins (see tests/test_oracle_*.py): per-sequence formula when every r(i) is
 * equal (Eq. "perseq"), brute force over all adapters then selection (work
 * K*N vs N, Thm. "Computational Optimality"), zero-B adapters reduce to x W,
 * C = 1 reduces to the dense LoRA h = xW + xAB (Sec. 2.1), float64 numpy
 * cross-checks, exact integer-valued cases for the gate, numpy's stable
 * argsort / bincount / searchsorted for the dispatch and vocabulary routing.
 * The paper prints no numeric value of h, so absolute values of h are
 * pinned only by those invariants and cross-checks.
 */
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

static inline float bf16_to_f32(uint16_t b)
{
    uint32_t u = (uint32_t)b << 16;
    float f;
    memcpy(&f, &u, sizeof f);
    return f;
}

/* Widen a bf16 array to a freshly malloc'ed fp32 array (exact). */
static float *widen(const uint16_t *src, size_t n)
{
    float *dst = (float *)malloc((n ? n : 1) * sizeof(float));
    if (!dst) return NULL;
    for (size_t i = 0; i < n; ++i) dst[i] = bf16_to_f32(src[i]);
    return dst;
}

/*
 * Learned routing with k = 1 (Sec. "Router Architecture": top-1 of the gate
 * logits; the softmax over the single selected logit is 1, so the weighted
 * mixture collapses to Eq. "pertok").  The gate is the linear, bias-free MoE
 * form of Table "tab:moe_adapter": logits_i = x_i G, G is [d_in][C] row-major.
 * r[i] = argmax_c logits_i[c]; ties go to the lowest index (strict '>' scan).
 * A NaN logit above index 0 is never selected; logit 0 is the scan's starting point and
 * stays selected if it is NaN (nothing compares greater than a NaN).
 * Returns 0, or -1 on allocation failure.
 */
int oracle_route_gate(const uint16_t *x, const uint16_t *G, int32_t *r,
                      int64_t N, int32_t d_in, int32_t C)
{
    float *Gf = widen(G, (size_t)d_in * C);
    if (!Gf) return -1;
    int fail = 0;
#pragma omp parallel
    {
        float *logit = (float *)malloc((size_t)C * sizeof(float));
        if (!logit) {
#pragma omp atomic write
            fail = 1;
        }
#pragma omp for schedule(static)
        for (int64_t i = 0; i < N; ++i) {
            if (!logit) continue;
            for (int c = 0; c < C; ++c) logit[c] = 0.0f;
            const uint16_t *xi = x + (size_t)i * d_in;
            for (int k = 0; k < d_in; ++k) {          /* ascending k */
                const float xv = bf16_to_f32(xi[k]);
                const float *g = Gf + (size_t)k * C;
                for (int c = 0; c < C; ++c) {
                    const float p = xv * g[c];         /* exact: 8x8-bit significands */
                    logit[c] = logit[c] + p;
                }
            }
            int best = 0;
            for (int c = 1; c < C; ++c)
                if (logit[c] > logit[best]) best = c;
            r[i] = best;
        }
        free(logit);
    }
    free(Gf);
    return fail ? -1 : 0;
}

/* Same gate, but returns the fp32 logits [N][C] (used by tests that examine ties). */
int oracle_gate_logits(const uint16_t *x, const uint16_t *G, float *logits,
                       int64_t N, int32_t d_in, int32_t C)
{
    float *Gf = widen(G, (size_t)d_in * C);
    if (!Gf) return -1;
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < N; ++i) {
        float *logit = logits + (size_t)i * C;
        for (int c = 0; c < C; ++c) logit[c] = 0.0f;
        const uint16_t *xi = x + (size_t)i * d_in;
        for (int k = 0; k < d_in; ++k) {
            const float xv = bf16_to_f32(xi[k]);
            const float *g = Gf + (size_t)k * C;
            for (int c = 0; c < C; ++c) {
                const float p = xv * g[c];
                logit[c] = logit[c] + p;
            }
        }
    }
    free(Gf);
    return 0;
}

/*
 * Vocabulary routing (Def. "Vocabulary Routing"): with breaks b_0 < b_1 < ... < b_M,
 * token id v routes to the (0-based) range m with b_m <= v < b_{m+1}, found by
 * comparing v against the interior breaks.  Ids outside [b_0, b_M) get -1, which
 * the dispatch step treats as "no adapter".
 */
void oracle_route_vocab(const int32_t *v, const int32_t *breaks, int32_t M,
                        int32_t *r, int64_t N)
{
    for (int64_t i = 0; i < N; ++i) {
        const int32_t id = v[i];
        if (id < breaks[0] || id >= breaks[M]) { r[i] = -1; continue; }
        int32_t m = 0;
        for (int32_t j = 1; j < M; ++j)               /* M-1 integer comparisons */
            if (id >= breaks[j]) m = j;
        r[i] = m;
    }
}

/*
 * Dispatch (Sec. "Unified Dispatch Infrastructure", Alg. "Unified Dispatch Kernel"):
 * histogram cnt[c] = |{t : r(t) = c}|, then a position for every token inside its
 * target's list.  The paper allocates positions with an atomic counter, so any
 * order inside a list is valid there; this build fixes the order to ascending
 * token index (a stable counting sort) so that the result is unique:
 *   offsets[0] = 0, offsets[c+1] = offsets[c] + cnt[c]   (c = 0..C-1)
 *   perm[offsets[c] .. offsets[c+1]) = tokens with r = c, ascending
 *   perm[offsets[C] .. N)            = tokens with r outside [0, C), ascending
 * offsets has C+1 entries, perm has N.  Returns the number of out-of-range tokens.
 */
int64_t oracle_bucket(const int32_t *r, int32_t *offsets, int32_t *perm,
                      int64_t N, int32_t C)
{
    int64_t *cnt = (int64_t *)calloc((size_t)C + 1, sizeof(int64_t));
    if (!cnt) return -1;
    for (int64_t t = 0; t < N; ++t) {
        const int32_t c = r[t];
        cnt[(c >= 0 && c < C) ? c : C] += 1;
    }
    int64_t *next = (int64_t *)malloc(((size_t)C + 1) * sizeof(int64_t));
    if (!next) { free(cnt); return -1; }
    int64_t run = 0;
    for (int32_t c = 0; c <= C; ++c) {               /* exclusive prefix sum */
        next[c] = run;
        offsets[c] = (int32_t)run;
        run += cnt[c];
    }
    for (int64_t t = 0; t < N; ++t) {
        const int32_t c = r[t];
        const int32_t b = (c >= 0 && c < C) ? c : C;
        perm[next[b]++] = (int32_t)t;
    }
    const int64_t bad = cnt[C];
    free(cnt);
    free(next);
    return bad;
}

/*
 * One token of Eq. "pertok", literally:
 *   t[j]     = sum_k x[k] A_c[k][j]          (k ascending, fp32)
 *   base[n]  = sum_k x[k] W[k][n]            (k ascending, fp32)
 *   delta[n] = sum_j t[j] B_c[j][n]          (j ascending, fp32, t not re-rounded)
 *   h[n]     = base[n] + delta[n]
 * c outside [0, C) means "no adapter": h = base.
 * Wf, Af, Bf are the fp32-widened weights; scratch holds d_out + rank floats.
 */
static void apply_token(const uint16_t *xi, const float *Wf, const float *Af, const float *Bf,
                        int32_t c, float *hi, float *scratch,
                        int32_t d_in, int32_t d_out, int32_t C, int32_t rank)
{
    float *delta = scratch;
    float *t = scratch + d_out;
    for (int n = 0; n < d_out; ++n) hi[n] = 0.0f;
    for (int k = 0; k < d_in; ++k) {
        const float xv = bf16_to_f32(xi[k]);
        const float *w = Wf + (size_t)k * d_out;
        for (int n = 0; n < d_out; ++n) {
            const float p = xv * w[n];
            hi[n] = hi[n] + p;
        }
    }
    if (c < 0 || c >= C) return;
    const float *Ac = Af + (size_t)c * d_in * rank;
    const float *Bc = Bf + (size_t)c * rank * d_out;
    for (int j = 0; j < rank; ++j) t[j] = 0.0f;
    for (int k = 0; k < d_in; ++k) {
        const float xv = bf16_to_f32(xi[k]);
        const float *a = Ac + (size_t)k * rank;
        for (int j = 0; j < rank; ++j) {
            const float p = xv * a[j];
            t[j] = t[j] + p;
        }
    }
    for (int n = 0; n < d_out; ++n) delta[n] = 0.0f;
    for (int j = 0; j < rank; ++j) {
        const float tv = t[j];
        const float *b = Bc + (size_t)j * d_out;
        for (int n = 0; n < d_out; ++n) {
            const float p = tv * b[n];
            delta[n] = delta[n] + p;
        }
    }
    for (int n = 0; n < d_out; ++n) hi[n] = hi[n] + delta[n];
}

/*
 * h[q][:] for the tokens rows[0..n_rows) (rows == NULL: all N tokens, q = i).
 * x [N][d_in], W [d_in][d_out], A [C][d_in][rank], B [C][rank][d_out] are bf16
 * bit patterns, row-major (stacked weight shapes of Table "tab:moe_adapter");
 * r [N] int32; h [n_rows][d_out] fp32.  Returns 0, or -1 on allocation failure.
 */
int oracle_apply_rows(const uint16_t *x, const uint16_t *W, const uint16_t *A, const uint16_t *B,
                      const int32_t *r, const int64_t *rows, int64_t n_rows, float *h,
                      int64_t N, int32_t d_in, int32_t d_out, int32_t C, int32_t rank)
{
    float *Wf = widen(W, (size_t)d_in * d_out);
    float *Af = widen(A, (size_t)C * d_in * rank);
    float *Bf = widen(B, (size_t)C * rank * d_out);
    int fail = (!Wf || !Af || !Bf);
    if (rows == NULL) n_rows = N;
    if (!fail) {
#pragma omp parallel
        {
            float *scratch = (float *)malloc(((size_t)d_out + rank) * sizeof(float));
            if (!scratch) {
#pragma omp atomic write
                fail = 1;
            }
#pragma omp for schedule(dynamic, 4)
            for (int64_t q = 0; q < n_rows; ++q) {
                if (!scratch) continue;
                const int64_t i = rows ? rows[q] : q;
                apply_token(x + (size_t)i * d_in, Wf, Af, Bf, r[i], h + (size_t)q * d_out,
                            scratch, d_in, d_out, C, rank);
            }
            free(scratch);
        }
    }
    free(Wf);
    free(Af);
    free(Bf);
    return fail ? -1 : 0;
}

int oracle_apply(const uint16_t *x, const uint16_t *W, const uint16_t *A, const uint16_t *B,
                 const int32_t *r, float *h,
                 int64_t N, int32_t d_in, int32_t d_out, int32_t C, int32_t rank)
{
    return oracle_apply_rows(x, W, A, B, r, NULL, N, h, N, d_in, d_out, C, rank);
}

/* Threads the parallel regions above will use (for reporting). */
int oracle_num_threads(void)
{
    int n = 1;
#ifdef _OPENMP
#pragma omp parallel
    {
#pragma omp master
        n = omp_get_num_threads();
    }
#endif
    return n;
}
