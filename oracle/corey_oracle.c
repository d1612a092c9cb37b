/*
 * corey_oracle.c -- CPU oracle for the COREY hot path.  TEST INFRASTRUCTURE ONLY.
 *
 * A plain, slow, sequential, double-precision statement of what the path computes, written from the
 * paper so that it can be checked against the paper by eye.  It shares no code, header, table or
 * helper with the HIP library; only tests, the smoke check and the benchmark's cpu_baseline leg may
 * call it.  Nothing here is blocked, fused, vectorised or reordered beyond what the definitions say
 * (the optional OpenMP loop runs independent (batch, channel) rows on several cores and changes no
 * arithmetic).
 *
 * What follows which passage:
 *   oracle_entropy_hist   Method / Preliminaries, Eq. 1 (fixed-bin entropy, stability constant eps),
 *                         the normalisation r = H / log K that follows Eq. 1, and the two-pass
 *                         (min/max, then bin count) structure of "Entropy Estimation Protocol".
 *   oracle_select_chunk   Eq. 2 (entropy-guided chunk selection), the H_ref form of the same rule in
 *                         "H_ref Sensitivity Ablation" (r = min(H/H_ref, 1)), the sequence-length
 *                         rule of "Mixed-Regime Scheduler Comparison" (<= 50 tokens -> 128, else 512)
 *                         and the guarded fallback described there and in "Guarded and Learned
 *                         Variants" (fallback unless the prediction is >= 2 power-of-two buckets away).
 *   oracle_selective_scan Method / Preliminaries, the recurrence h_t = A_t h_{t-1} + B_t x_t,
 *                         y_t = C_t h_t + D_t x_t, in its Mamba-1 instantiation (the paper's cited
 *                         selective-SSM reference): A_t = exp(delta_t A), B_t x_t = delta_t B_t u_t,
 *                         delta_t = softplus(Delta_t + bias) ("delta_softplus=true" in the paper's
 *                         kernel call), SiLU(z) output gate.  The sequence is walked in tiles of
 *                         `chunk` steps with the state carried from tile to tile, which is the
 *                         recurrence-preserving run-time chunk of "End-to-End Routed Inference".
 *
 * Pins (tests/test_oracle_*.py): values the paper prints (tests/golden/), closed forms, brute force on
 * tiny inputs and special cases that reduce to numpy/scipy routines.  Scan parity against the original
 * Mamba implementation itself is unpinned: no such code, weights or outputs exist beside this file.
 *
 * Readings taken where the paper is silent:
 *   - bin index: t = x - lo and q = t * scale are each ONE IEEE binary32 operation (round to nearest
 *     even, no fused multiply-add), scale = (float)(K / ((double)hi - (double)lo)), k = trunc(q)
 *     clamped to K-1.  This is the precision the GPU kernel bins in, so both sides take the integer
 *     decision in the same arithmetic; everything that is not an integer decision is double.
 *   - bins are half open, the last one closed (x == hi lands in bin K-1).
 *   - hi == lo: all samples fall in bin 0.
 *   - non-finite min or max: status ORACLE_ENONFINITE, counts zero, H and r NaN.
 *   - natural logarithm (the paper reports nats); r is clamped to [0, 1].
 *   - an empty bin contributes nothing to Eq. 1 (the term p log(p + eps) is 0 at p = 0 for every eps > 0, and
 *     its limit is 0 for eps = 0, the usual 0 log 0 = 0 of Shannon entropy), so eps = 0 gives a finite H.
 *   - `round` in Eq. 2 is floor(v + 0.5) on v = log2(.) in double.
 *   - candidates above the next power of two >= L are never useful; Eq. 2's result is capped there
 *     (but never below c_min).  The sequence-length table and a static chunk are returned as given,
 *     because the paper prints 128 for prompts of about 25 tokens.
 *   - padded positions t >= seqlens[b] produce y = 0 and do not touch the state.
 *
 * Build: gcc -O2 -fPIC -shared -std=c11 -ffp-contract=off -fopenmp corey_oracle.c -lm
 */
#include <float.h>
#include <math.h>
#include <stddef.h>
#include <stdint.h>
#include <string.h>

#ifdef _OPENMP
#include <omp.h>
#endif

#if FLT_EVAL_METHOD != 0
#error "binary32 expressions must be evaluated in binary32 (the bin index depends on it)"
#endif

enum {
    ORACLE_OK = 0,
    ORACLE_EINVAL = 1,
    ORACLE_ENONFINITE = 4
};

/* ------------------------------------------------------------------------------------------------
 * Eq. 1 and the normalised signal r.
 *
 * x        float[B][D][L]; low-precision inputs are widened exactly by the caller.
 * seqlens  NULL: one histogram over every element.  Otherwise int32[B]: one histogram per sequence b
 *          over the valid positions t < seqlens[b] of all D channels (nh = B histograms).
 * stride, block  >= 1.  The valid elements of one histogram, taken in memory order (d major, t minor, and b
 *          outermost for the whole-tensor case), are numbered j = 0, 1, ... and cut into blocks of `block`
 *          consecutive elements; element j is used iff (j / block) % stride == 0, i.e. every stride-th block.
 *          stride 1 is the exact statistic; stride 8 with block 1 is the paper's sampled variant ("sampled
 *          histogram (stride 8)" of the routed ablation, which does not say along which axis it strides: memory
 *          order is the reading taken); block > 1 samples whole runs of memory instead of single elements.
 * range_all  0: lo and hi are the minimum and maximum of the sampled values.  1: of all valid values of the
 *          histogram, sampled or not (the paper does not say which values bound the bins of its sampled
 *          variant; this second reading is what a producer that tracks min / max while it writes the tensor
 *          hands over).  A NaN among the values the range is taken over makes the statistic non-finite.
 *          With stride 1 the two are the same.
 * counts   uint32[nh][K] out.   H, r: double[nh] out.   lo, hi: float[nh] out (may be NULL).
 * ---------------------------------------------------------------------------------------------- */
int oracle_entropy_hist(const float* x, int64_t B, int64_t D, int64_t L, const int32_t* seqlens,
                        int32_t K, double eps, int64_t stride, int64_t block, int32_t range_all,
                        uint32_t* counts, double* H, double* r, float* lo_out, float* hi_out)
{
    if (!x || !counts || !H || !r) return ORACLE_EINVAL;
    if (B < 1 || D < 1 || L < 1 || K < 2 || stride < 1 || block < 1 || !(eps >= 0.0)) return ORACLE_EINVAL;
    const int64_t nh = seqlens ? B : 1;
    int status = ORACLE_OK;

    for (int64_t hsel = 0; hsel < nh; ++hsel) {
        uint32_t* c = counts + hsel * (int64_t)K;
        memset(c, 0, sizeof(uint32_t) * (size_t)K);
        const int64_t b0 = seqlens ? hsel : 0;
        const int64_t b1 = seqlens ? hsel + 1 : B;

        /* pass 1: range of the sampled values (of all values with range_all) */
        float lo = INFINITY, hi = -INFINITY;
        int seen_nan = 0;
        int64_t j = 0, nsamp = 0;
        for (int64_t b = b0; b < b1; ++b) {
            int64_t len = seqlens ? seqlens[b] : L;
            if (len < 0 || len > L) return ORACLE_EINVAL;
            for (int64_t d = 0; d < D; ++d)
                for (int64_t t = 0; t < len; ++t, ++j) {
                    const int sampled = (j / block) % stride == 0;
                    if (!sampled && !range_all) continue;
                    float v = x[(b * D + d) * L + t];
                    if (v != v) seen_nan = 1;
                    if (v < lo) lo = v;
                    if (v > hi) hi = v;
                    if (sampled) ++nsamp;
                }
        }
        if (lo_out) lo_out[hsel] = lo;
        if (hi_out) hi_out[hsel] = hi;
        if (nsamp == 0 || seen_nan || !isfinite(lo) || !isfinite(hi)) {
            H[hsel] = NAN; r[hsel] = NAN;
            status = ORACLE_ENONFINITE;
            continue;
        }

        /* pass 2: K equal-width bins on [lo, hi] */
        if (hi == lo) {
            c[0] = (uint32_t)nsamp;
        } else {
            const float scale = (float)((double)K / ((double)hi - (double)lo));
            j = 0;
            for (int64_t b = b0; b < b1; ++b) {
                int64_t len = seqlens ? seqlens[b] : L;
                for (int64_t d = 0; d < D; ++d)
                    for (int64_t t = 0; t < len; ++t, ++j) {
                        if ((j / block) % stride) continue;
                        const float tt = x[(b * D + d) * L + t] - lo;   /* one binary32 subtract */
                        const float q = tt * scale;                     /* one binary32 multiply */
                        int64_t k = (int64_t)q;                            /* truncate, q >= 0 */
                        if (k > K - 1) k = K - 1;
                        if (k < 0) k = 0;
                        c[k] += 1u;
                    }
            }
        }

        /* Eq. 1: H = - sum_k p_k log(p_k + eps), then r = H / log K clamped to [0, 1] */
        double n = 0.0;
        for (int32_t k = 0; k < K; ++k) n += (double)c[k];
        double acc = 0.0;
        for (int32_t k = 0; k < K; ++k) {
            if (c[k] == 0) continue;       /* an empty bin adds nothing: p log(p + eps) is 0 at p = 0, also for eps = 0 */
            double p = (double)c[k] / n;
            acc += p * log(p + eps);
        }
        double h = -acc;
        double rr = h / log((double)K);
        if (rr < 0.0) rr = 0.0;
        if (rr > 1.0) rr = 1.0;
        H[hsel] = h;
        r[hsel] = rr;
    }
    return status;
}

/* ------------------------------------------------------------------------------------------------
 * Exponential moving average of the entropy estimate across calls ("Entropy Estimation Protocol"):
 *     H^_t = lambda * H^_{t-1} + (1 - lambda) * H_t,   0 <= lambda < 1   (the paper's prototype uses 0.85).
 * The paper does not say what H^_0 is (it only notes that short runs stay dominated by the initialisation): here a
 * NaN `prev` means "no estimate yet" and the first observation is taken as it is.  A NaN observation (non-finite
 * input) leaves the estimate unchanged.
 * ---------------------------------------------------------------------------------------------- */
double oracle_ema_update(double lambda, double prev, double H)
{
    if (H != H) return prev;
    if (prev != prev) return H;
    return lambda * prev + (1.0 - lambda) * H;
}

/* ------------------------------------------------------------------------------------------------
 * Eq. 2 and the scheduler family around it.
 *
 * mode 0  entropy rule (Eq. 2).
 * mode 1  sequence-length gate first (L <= short_len -> short_chunk), entropy rule otherwise.
 * mode 2  sequence-length table only (L <= short_len -> short_chunk, else long_chunk).
 * mode 3  static chunk.
 * mode 4  guarded entropy rule: the Eq. 2 prediction is kept only if it lies at least guard_buckets
 *         powers of two away from safe_chunk; otherwise safe_chunk is returned.
 * h_ref_scale multiplies r before Eq. 2 and the product is clamped to [0,1]: 1.0 is the calibrated
 * rule (H_ref = log K); log(K)/8 reproduces the legacy H_ref = 8 nats.
 * margin_out (may be NULL) receives |log2(v) - (k + 1/2)|, the distance of Eq. 2's argument from the
 * nearest rounding tie, or -1 when Eq. 2 was not evaluated.
 * ---------------------------------------------------------------------------------------------- */
typedef struct {
    int32_t mode;
    int32_t c_min, c_max;
    double  h_ref_scale;
    int32_t short_len, short_chunk, long_chunk;
    int32_t static_chunk;
    int32_t safe_chunk, guard_buckets;
} oracle_policy;

static int is_pow2(int64_t v) { return v > 0 && (v & (v - 1)) == 0; }

static int64_t pow2ceil(int64_t v) { int64_t p = 1; while (p < v) p <<= 1; return p; }

static int ilog2_exact(int64_t v) { int e = 0; while ((1LL << e) < v) ++e; return e; }

int oracle_select_chunk(double r, int64_t L, const oracle_policy* p, int32_t* chunk_out,
                        double* margin_out)
{
    if (!p || !chunk_out) return ORACLE_EINVAL;
    if (L < 1) return ORACLE_EINVAL;
    if (!is_pow2(p->c_min) || !is_pow2(p->c_max) || p->c_min > p->c_max) return ORACLE_EINVAL;
    if (margin_out) *margin_out = -1.0;
    int64_t cap = pow2ceil(L);
    if (cap < p->c_min) cap = p->c_min;
    int64_t c;

    if (p->mode == 3) {
        if (!is_pow2(p->static_chunk)) return ORACLE_EINVAL;
        c = p->static_chunk;
    } else if (p->mode == 2 || (p->mode == 1 && L <= p->short_len)) {
        if (!is_pow2(p->short_chunk)) return ORACLE_EINVAL;
        if (p->mode == 2 && !is_pow2(p->long_chunk)) return ORACLE_EINVAL;
        c = (L <= p->short_len) ? p->short_chunk : p->long_chunk;
    } else if (p->mode == 0 || p->mode == 1 || p->mode == 4) {
        if (!(r == r)) return ORACLE_ENONFINITE;
        double re = r * p->h_ref_scale;
        if (re < 0.0) re = 0.0;
        if (re > 1.0) re = 1.0;
        double v = (double)p->c_min + re * (double)(p->c_max - p->c_min);
        double lg = log2(v);
        double k = floor(lg + 0.5);
        if (margin_out) *margin_out = fabs(lg - (k - 0.5)) < fabs(lg - (k + 0.5))
                                          ? fabs(lg - (k - 0.5)) : fabs(lg - (k + 0.5));
        c = (int64_t)1 << (int)k;
        if (c < p->c_min) c = p->c_min;
        if (c > p->c_max) c = p->c_max;
        if (p->mode == 4) {
            if (!is_pow2(p->safe_chunk) || p->guard_buckets < 0) return ORACLE_EINVAL;
            int dist = ilog2_exact(c) - ilog2_exact(p->safe_chunk);
            if (dist < 0) dist = -dist;
            if (dist < p->guard_buckets) c = p->safe_chunk;
        }
        if (c > cap) c = cap;          /* only Eq. 2's own result is capped; table and static values are kept */
    } else {
        return ORACLE_EINVAL;
    }
    *chunk_out = (int32_t)c;
    return ORACLE_OK;
}

/* ------------------------------------------------------------------------------------------------
 * Selective-scan forward, one step at a time.
 *
 * u, delta, z   float[B][D][L]   (z may be NULL: no gate)
 * A             float[D][N]
 * Bm, Cm        float[B][N][L]   (input dependent, shared by all channels of a sequence)
 * Dv, dbias     float[D] or NULL
 * h0            float[B][D][N] or NULL (zero state)
 * seqlens       int32[B] or NULL
 * chunk         tile length along L (>= 1); the state is carried tile to tile, so the result does not
 *               depend on it.
 * y             double[B][D][L] out;  last_state double[B][D][N] out.
 * threads       OpenMP threads over the independent (b, d) rows (<= 1: sequential).
 * y_terms       double[B][D][L] out or NULL: the sum of the ABSOLUTE values of the terms y is made of,
 *               (sum_n |C h| + |D u|) |gate|.  Not part of the method: a checker that compares a single-precision y
 *               with this one needs the size of the terms to bound the rounding of a sum that cancels.
 * ---------------------------------------------------------------------------------------------- */
int oracle_selective_scan(const float* u, const float* delta, const float* A, const float* Bm,
                          const float* Cm, const float* Dv, const float* z, const float* dbias,
                          int delta_softplus, const float* h0, const int32_t* seqlens, int64_t chunk,
                          int64_t B, int64_t D, int64_t N, int64_t L,
                          double* y, double* last_state, int threads, double* y_terms)
{
    if (!u || !delta || !A || !Bm || !Cm || !y || !last_state) return ORACLE_EINVAL;
    if (B < 1 || D < 1 || N < 1 || N > 1024 || L < 1 || chunk < 1) return ORACLE_EINVAL;
    if (seqlens)
        for (int64_t b = 0; b < B; ++b)
            if (seqlens[b] < 0 || seqlens[b] > L) return ORACLE_EINVAL;
    (void)threads;

#ifdef _OPENMP
#pragma omp parallel for schedule(static) num_threads(threads > 1 ? threads : 1)
#endif
    for (int64_t row = 0; row < B * D; ++row) {
        const int64_t b = row / D, d = row % D;
        const int64_t len = seqlens ? seqlens[b] : L;
        double h[1024];
        for (int64_t n = 0; n < N; ++n) h[n] = h0 ? (double)h0[row * N + n] : 0.0;

        for (int64_t t0 = 0; t0 < len; t0 += chunk) {            /* tile loop: state h carried */
            const int64_t t1 = (t0 + chunk < len) ? t0 + chunk : len;
            for (int64_t t = t0; t < t1; ++t) {
                double dl = (double)delta[row * L + t] + (dbias ? (double)dbias[d] : 0.0);
                if (delta_softplus)
                    dl = (dl > 0.0 ? dl : 0.0) + log1p(exp(-fabs(dl)));   /* log(1 + e^dl) */
                const double uu = (double)u[row * L + t];
                double acc = 0.0, mag = 0.0;
                for (int64_t n = 0; n < N; ++n) {
                    const double abar = exp(dl * (double)A[d * N + n]);
                    const double bbar_u = dl * (double)Bm[(b * N + n) * L + t] * uu;
                    h[n] = abar * h[n] + bbar_u;
                    acc += (double)Cm[(b * N + n) * L + t] * h[n];
                    mag += fabs((double)Cm[(b * N + n) * L + t] * h[n]);
                }
                double yv = acc + (Dv ? (double)Dv[d] * uu : 0.0);
                if (z) {
                    const double zz = (double)z[row * L + t];
                    yv *= zz / (1.0 + exp(-zz));
                }
                y[row * L + t] = yv;
                if (y_terms) {
                    mag += Dv ? fabs((double)Dv[d] * uu) : 0.0;
                    if (z) mag *= fabs((double)z[row * L + t] / (1.0 + exp(-(double)z[row * L + t])));
                    y_terms[row * L + t] = mag;
                }
            }
        }
        for (int64_t t = len; t < L; ++t) y[row * L + t] = 0.0;
        if (y_terms)
            for (int64_t t = len; t < L; ++t) y_terms[row * L + t] = 0.0;
        for (int64_t n = 0; n < N; ++n) last_state[row * N + n] = h[n];
    }
    return ORACLE_OK;
}

int oracle_max_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* ------------------------------------------------------------------------------------------------
 * The step before the path: causal depthwise convolution and SiLU producing the scan input u (step (1) of the
 * paper's inline hook, "Active-Mode Overhead Budget"), in its Mamba-1 form:
 *     v[b,d,t] = bias[d] + sum_{k=0}^{W-1} weight[d,k] * x[b,d,t-(W-1)+k],   u = v / (1 + exp(-v)),
 * inputs before t = 0 taken from state_in[b,d,0..W-2] (oldest first) or zero.  Everything in double; u is returned
 * unrounded.  state_out (may be NULL) receives the last W-1 inputs of every row.
 * ---------------------------------------------------------------------------------------------- */
int oracle_causal_conv1d_silu(const float* x, const float* weight, const float* bias, const float* state_in,
                              int64_t B, int64_t D, int64_t L, int32_t W, double* u, float* state_out)
{
    if (!x || !weight || !u || B < 1 || D < 1 || L < 1 || W < 1) return ORACLE_EINVAL;
    for (int64_t r = 0; r < B * D; ++r) {
        const int64_t d = r % D;
        for (int64_t t = 0; t < L; ++t) {
            double v = bias ? (double)bias[d] : 0.0;
            for (int32_t k = 0; k < W; ++k) {
                const int64_t s = t - (W - 1) + k;
                double xv = 0.0;
                if (s >= 0) xv = (double)x[r * L + s];
                else if (state_in) xv = (double)state_in[r * (W - 1) + (s + (W - 1))];
                v += (double)weight[d * W + k] * xv;
            }
            u[r * L + t] = v / (1.0 + exp(-v));
        }
        if (state_out)
            for (int32_t k = 0; k < W - 1; ++k) {
                const int64_t s = L - (W - 1) + k;
                float xv = 0.f;
                if (s >= 0) xv = x[r * L + s];
                else if (state_in) xv = state_in[r * (W - 1) + (s + (W - 1))];
                state_out[r * (W - 1) + k] = xv;
            }
    }
    return ORACLE_OK;
}

/* ------------------------------------------------------------------------------------------------
 * One generated token: the recurrence of oracle_selective_scan taken for a single step from a carried state (what
 * runs after the prompt in the paper's greedy-generation checks, "Output Quality Preservation").
 *
 * state_in      float[B][D][N]  the state after the previous token
 * x, delta, z   float[B][D]     (z may be NULL)
 * A float[D][N];  Bt, Ct float[B][N];  Dv, dbias float[D] or NULL
 * state_out     double[B][D][N];  y double[B][D]
 *     dl = softplus(delta + dbias);  h'[n] = exp(dl A[d][n]) h[n] + dl Bt[b][n] x;  y = sum_n Ct[b][n] h'[n] + Dv[d] x;
 *     y *= z / (1 + exp(-z))
 * ---------------------------------------------------------------------------------------------- */
int oracle_selective_state_update(const float* state_in, const float* x, const float* delta, const float* A,
                                  const float* Bt, const float* Ct, const float* Dv, const float* z,
                                  const float* dbias, int delta_softplus, int64_t B, int64_t D, int64_t N,
                                  double* state_out, double* y)
{
    if (!state_in || !x || !delta || !A || !Bt || !Ct || !state_out || !y) return ORACLE_EINVAL;
    if (B < 1 || D < 1 || N < 1) return ORACLE_EINVAL;
    for (int64_t b = 0; b < B; ++b)
        for (int64_t d = 0; d < D; ++d) {
            const int64_t row = b * D + d;
            double dl = (double)delta[row] + (dbias ? (double)dbias[d] : 0.0);
            if (delta_softplus) dl = (dl > 0.0 ? dl : 0.0) + log1p(exp(-fabs(dl)));
            const double xx = (double)x[row];
            double acc = 0.0;
            for (int64_t n = 0; n < N; ++n) {
                const double hn = exp(dl * (double)A[d * N + n]) * (double)state_in[row * N + n]
                                  + dl * (double)Bt[b * N + n] * xx;
                state_out[row * N + n] = hn;
                acc += (double)Ct[b * N + n] * hn;
            }
            double yv = acc + (Dv ? (double)Dv[d] * xx : 0.0);
            if (z) {
                const double zz = (double)z[row];
                yv *= zz / (1.0 + exp(-zz));
            }
            y[row] = yv;
        }
    return ORACLE_OK;
}
