/*
 * spark_oracle.c -- CPU oracle for SparK channel pruning and recovered decode attention.
 *
 * THIS IS TEST INFRASTRUCTURE, NOT THE PRODUCT.  It is a plain, slow, double-precision
 * restatement of what the paper's method computes, written from the paper, and it shares
 * no code, header, table or helper with the HIP library.  Only the tests, the smoke check
 * and the CPU-baseline leg of the benchmark may call it.
 *
 * Notation follows the paper: head dimension D, T kept channels per (token, head),
 * observation window of W queries, saliency w, mask S, pruned keys K-hat, recovered
 * keys K-tilde, recovery function F.  Tensors are plain row-major arrays; K, V, Q
 * entries are bfloat16 bit patterns (uint16) exactly as the GPU sees them.
 *
 * Readings the paper leaves open (each stated again where it is used):
 *   - the query norm of a channel is |mean over the window| (the mean query is a vector
 *     of scalars, so its per-channel 2-norm is an absolute value);
 *   - with grouped-query attention one selection is made per KV head from the mean of
 *     the group's |mean query|, and the same vector is the denominator of F;
 *   - the compared saliency is the IEEE binary32 product a32 * |k| (a32 = the group
 *     weight rounded once to binary32), so the kept set is a pure function of bits;
 *   - equal saliencies: the lower channel index is kept;
 *   - a channel whose weight a is 0 recovers to 0.
 *
 * Parity pins (tests that hold this file to something other than itself): the hand
 * worked example under tests/golden, keep-all == dense attention == a library softmax
 * attention, brute-force subset optimality of Eq. (7), the exact-recovery construction,
 * window-scale invariance, and the invariants listed in tests/test_oracle_pins.py; the
 * value-cache functions by brute-force subset optimality, a second hand-worked case and
 * an independent masked-matrix product; the appended-token decode by a third hand-worked
 * case, dense attention on the concatenated cache (keep-all) and the empty-tail identity; the
 * sampled recovery by the invertibility and the statistics of its generator, the sigma = 0
 * reduction to the degenerate function, sample means, and a plain softmax attention over the
 * exported rebuilt keys; the top-p variant by exact rational arithmetic over every prefix of tiny
 * rows, the one-dominant-channel, equal-saliency and p = 100 % cases and the prefix property.  No
 * function in this file is "parity unpinned".
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

/* ---------------------------------------------------------------- helpers */

static float bf16_bits_to_f32(uint16_t b)
{
    uint32_t u = ((uint32_t)b) << 16;
    float f;
    memcpy(&f, &u, sizeof f);
    return f;
}

static double bf16_bits_to_f64(uint16_t b) { return (double)bf16_bits_to_f32(b); }

void oracle_set_threads(int n)
{
#ifdef _OPENMP
    if (n > 0) omp_set_num_threads(n);
#else
    (void)n;
#endif
}

int oracle_max_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* Sequence that owns global token n (cu has B+1 non-decreasing entries). */
static int seq_of_token(const int32_t *cu, int B, int64_t n)
{
    int b = 0;
    while (b + 1 < B && n >= cu[b + 1]) ++b;
    return b;
}

/* ------------------------------------------------- prefill: window statistic */

/*
 * Mean query over the observation window (Sec. "SparK", the mean-query formula):
 *     qbar[b,g,j] = (1/W) * sum_{t<W} Q_win[b,g,t,j]
 * and the per-KV-head channel weight used as the query norm in the saliency
 * (Sec. "Problem Formulation", w = ||q^j|| * ||k^j||):
 *     a[b,h,j] = (1/G) * sum_{g in group(h)} |qbar[b,g,j]|,   G = Hq / Hkv,
 * query head g belongs to KV head g / G.  a32 is a rounded once to binary32.
 *
 * qwin: [B, Hq, W, D] bf16 bits.  Outputs: qbar [B,Hq,D], a64 [B,Hkv,D], a32 [B,Hkv,D].
 */
void oracle_window_stat(const uint16_t *qwin, int B, int Hq, int Hkv, int W, int D,
                        double *qbar, double *a64, float *a32)
{
    const int G = Hq / Hkv;
    for (int b = 0; b < B; ++b)
        for (int g = 0; g < Hq; ++g)
            for (int j = 0; j < D; ++j) {
                double s = 0.0;
                for (int t = 0; t < W; ++t)
                    s += bf16_bits_to_f64(qwin[(((int64_t)b * Hq + g) * W + t) * D + j]);
                qbar[((int64_t)b * Hq + g) * D + j] = s / (double)W;
            }
    for (int b = 0; b < B; ++b)
        for (int h = 0; h < Hkv; ++h)
            for (int j = 0; j < D; ++j) {
                double s = 0.0;
                for (int gg = 0; gg < G; ++gg)
                    s += fabs(qbar[((int64_t)b * Hq + (h * G + gg)) * D + j]);
                const double a = s / (double)G;
                a64[((int64_t)b * Hkv + h) * D + j] = a;
                a32[((int64_t)b * Hkv + h) * D + j] = (float)a;
            }
}

/* ------------------------------------------------------ prefill: pruning */

/*
 * Saliency, top-T selection, mask, pruned keys and the cached statistic
 * (Sec. "Problem Formulation" Eq. (7) and its greedy solution; Sec. "SparK",
 * "Saliency Measurement and Unstructured Pruning"; App. "Caching Pruned Channel
 * Statistics", the mean over the pruned set).
 *
 * For every global token n (sequence b from cu) and KV head h:
 *   w[j]   = a32[b,h,j] * |K[n,h,j]|          as an IEEE binary32 product
 *   order  = channels sorted by w descending, equal w by ascending j (stable)
 *   kept   = first T of order;  mask bit j (word j/32, bit j%32) = 1 iff kept
 *   K-hat  = kept entries' original bf16 bits in ascending channel order
 *   mu     = mean of w over the D-T pruned channels, 0 when T == D
 *   gap    = (w_(T) - w_(T+1)) / w_(T), the relative margin of the selection
 *            (0 when w_(T) == 0; +inf when T == D)
 *
 * k: element (n,h,j) at k[n*k_tok_stride + h*k_head_stride + j].
 * mask [total,Hkv,MW] with MW = ceil(D/32); kept [total,Hkv,T]; mu64, mu32, gap
 * [total,Hkv]; w_out (may be NULL) [total,Hkv,D].
 * Returns 0, or -1 on bad arguments.
 */
int oracle_prune(const uint16_t *k, int64_t k_tok_stride, int64_t k_head_stride,
                 const float *a32, const int32_t *cu, int B, int Hkv, int D, int T,
                 uint32_t *mask, uint16_t *kept, double *mu64, float *mu32, double *gap,
                 float *w_out)
{
    if (D < 1 || D > 1024 || T < 1 || T > D || B < 1 || Hkv < 1) return -1;
    const int MW = (D + 31) / 32;
    const int64_t total = cu[B];
    int64_t n;
#pragma omp parallel for schedule(static)
    for (n = 0; n < total; ++n) {
        const int b = seq_of_token(cu, B, n);
        float w[1024];
        int order[1024];
        for (int h = 0; h < Hkv; ++h) {
            const uint16_t *krow = k + n * k_tok_stride + (int64_t)h * k_head_stride;
            const float *a = a32 + ((int64_t)b * Hkv + h) * D;
            const int64_t row = n * Hkv + h;
            for (int j = 0; j < D; ++j) {
                /* one binary32 multiply; volatile keeps it from being fused or widened */
                volatile float prod = a[j] * fabsf(bf16_bits_to_f32(krow[j]));
                w[j] = prod;
                if (w_out) w_out[row * D + j] = prod;
            }
            /* stable insertion sort of channel indices: w descending, ties by index */
            for (int j = 0; j < D; ++j) {
                int p = j;
                while (p > 0 && w[order[p - 1]] < w[j]) {
                    order[p] = order[p - 1];
                    --p;
                }
                order[p] = j;
            }
            for (int m = 0; m < MW; ++m) mask[row * MW + m] = 0u;
            for (int i = 0; i < T; ++i) {
                const int j = order[i];
                mask[row * MW + j / 32] |= (1u << (j % 32));
            }
            int c = 0;
            for (int j = 0; j < D; ++j)
                if (mask[row * MW + j / 32] >> (j % 32) & 1u) kept[row * T + c++] = krow[j];
            double s = 0.0;
            for (int i = T; i < D; ++i) s += (double)w[order[i]];
            const double mu = (T < D) ? s / (double)(D - T) : 0.0;
            mu64[row] = mu;
            mu32[row] = (float)mu;
            if (T == D)
                gap[row] = INFINITY;
            else {
                const double hi = (double)w[order[T - 1]], lo = (double)w[order[T]];
                gap[row] = (hi > 0.0) ? (hi - lo) / hi : 0.0;
            }
        }
    }
    return 0;
}

/*
 * Optional storage variant: symmetric int8 codes for the kept entries of one row,
 * one binary32 scale per (token, head).  The paper names quantisation only as a
 * compatible technique and gives no formula; this is the usual absmax rule:
 *     amax = max_i |khat_i|;  scale = amax / 127  (binary32 division)
 *     code_i = clamp(round-to-nearest-even(khat_i / scale), -127, 127), all 0 if scale == 0
 * Both divisions are single binary32 operations so the integer code is decided in the
 * same precision on the CPU and on the GPU.  (With an absmax scale |khat_i / scale| never
 * exceeds 127 by more than the rounding of the two divisions, which round-to-nearest
 * brings back to 127, so the clamp never changes a value; it is kept as a statement of
 * the code range.)
 */
void oracle_quant_int8(const uint16_t *kept, int64_t rows, int T, int8_t *codes, float *scale)
{
    for (int64_t r = 0; r < rows; ++r) {
        float amax = 0.0f;
        for (int i = 0; i < T; ++i) {
            const float v = fabsf(bf16_bits_to_f32(kept[r * T + i]));
            if (v > amax) amax = v;
        }
        volatile float sc = amax / 127.0f;
        scale[r] = sc;
        for (int i = 0; i < T; ++i) {
            if (sc == 0.0f) {
                codes[r * T + i] = 0;
                continue;
            }
            volatile float qf = bf16_bits_to_f32(kept[r * T + i]) / sc;
            float rq = nearbyintf(qf); /* default rounding mode: to nearest, ties to even */
            if (rq > 127.0f) rq = 127.0f;
            if (rq < -127.0f) rq = -127.0f;
            codes[r * T + i] = (int8_t)rq;
        }
    }
}

/*
 * The top-p variant, Sec. "Adaptive Variants of SparK" (and the "Ablation study on variants" table):
 * no fixed number of channels; per (token, KV head) the FEWEST most salient channels are kept
 * whose saliencies together reach a fraction p (99 % in the paper) of the row's total saliency.
 *
 *   w[j]   = a32[b,h,j] * |K[n,h,j]|                 the same binary32 product as in oracle_prune
 *   order  = channels by w descending, equal w by ascending j (stable), as in oracle_prune
 *   m      = the smallest m >= 1 with  sum_{i<m} w[order[i]]  >=  p * sum_j w[j]
 *   kept   = order[0..m);  mask, kept entries (ascending channel), count m
 *   mu     = mean of w over the D-m pruned channels (0 when m == D), as in oracle_prune
 *
 * Reading: the count m is an integer decided by sums, and a floating-point sum depends on the
 * order of its terms, which a parallel implementation cannot follow.  The decision is therefore
 * taken in exact integer arithmetic: every w of the row is expressed in units of the last place of
 * the row's LARGEST saliency, rounded down,
 *     ulp = 2^(E-150),  E = max(1, biased exponent of max_j w[j]);   q[j] = floor(w[j] / ulp) < 2^24,
 * p is a whole number of basis points (9900 for 99 %), and the rule is
 *     m = the smallest m >= 1 with  10000 * sum_{i<m} q[order[i]]  >=  p_bp * sum_j q[j].
 * The sums are below 2^31 and the products below 2^45: exact in 64-bit integers, in any order.  Rounding
 * down loses less than 128 units of 2^-23 of the largest element over a whole row, four orders of
 * magnitude below the 1 % the rule cuts at.  An all-zero row keeps one channel (m >= 1; channel 0).
 *
 * mask [total,Hkv,ceil(D/32)]; kept [total,Hkv,D] (first m entries of a row used, the rest 0);
 * count [total,Hkv]; mu64, mu32 [total,Hkv].  Returns 0, or -1 on bad arguments.
 */
int oracle_prune_topp(const uint16_t *k, int64_t k_tok_stride, int64_t k_head_stride,
                      const float *a32, const int32_t *cu, int B, int Hkv, int D, int p_bp,
                      uint32_t *mask, uint16_t *kept, int32_t *count, double *mu64, float *mu32)
{
    if (D < 1 || D > 128 || p_bp < 1 || p_bp > 10000 || B < 1 || Hkv < 1) return -1;
    const int MW = (D + 31) / 32;
    const int64_t total = cu[B];
    int64_t n;
#pragma omp parallel for schedule(static)
    for (n = 0; n < total; ++n) {
        const int b = seq_of_token(cu, B, n);
        float w[128];
        int order[128];
        int64_t q[128];
        for (int h = 0; h < Hkv; ++h) {
            const uint16_t *krow = k + n * k_tok_stride + (int64_t)h * k_head_stride;
            const float *a = a32 + ((int64_t)b * Hkv + h) * D;
            const int64_t row = n * Hkv + h;
            for (int j = 0; j < D; ++j) {
                volatile float prod = a[j] * fabsf(bf16_bits_to_f32(krow[j]));
                w[j] = prod;
            }
            for (int j = 0; j < D; ++j) {   /* stable: w descending, ties by index */
                int pos = j;
                while (pos > 0 && w[order[pos - 1]] < w[j]) {
                    order[pos] = order[pos - 1];
                    --pos;
                }
                order[pos] = j;
            }
            /* saliencies in units of the last place of the largest one, rounded down */
            int emax = 1;
            for (int j = 0; j < D; ++j) {
                uint32_t bits;
                memcpy(&bits, &w[j], sizeof bits);
                const int e = (int)((bits >> 23) & 0xFF);
                if (e > emax) emax = e;
            }
            int64_t S = 0;
            for (int j = 0; j < D; ++j) {
                uint32_t bits;
                memcpy(&bits, &w[j], sizeof bits);
                const int e = (int)((bits >> 23) & 0xFF);
                const int64_t mant = (int64_t)(bits & 0x7FFFFFu) | (e ? 0x800000 : 0);   /* w = mant * 2^(max(e,1)-150) */
                const int shift = emax - (e ? e : 1);
                q[j] = (shift < 24) ? (mant >> shift) : 0;
                S += q[j];
            }
            int m = 0;
            int64_t G = 0;
            do {
                G += q[order[m]];
                ++m;
            } while (m < D && 10000 * G < (int64_t)p_bp * S);
            for (int mw = 0; mw < MW; ++mw) mask[row * MW + mw] = 0u;
            for (int i = 0; i < m; ++i) mask[row * MW + order[i] / 32] |= (1u << (order[i] % 32));
            int c = 0;
            for (int j = 0; j < D; ++j)
                kept[row * D + j] = 0;
            for (int j = 0; j < D; ++j)
                if (mask[row * MW + j / 32] >> (j % 32) & 1u) kept[row * D + c++] = krow[j];
            count[row] = m;
            double s = 0.0;
            for (int i = m; i < D; ++i) s += (double)w[order[i]];
            const double mu = (m < D) ? s / (double)(D - m) : 0.0;
            mu64[row] = mu;
            mu32[row] = (float)mu;
        }
    }
    return 0;
}

/* ------------------------------------------------------------- value cache */

/*
 * Channel pruning of the value cache, App. "Pruning Value Cache Channels" (the extension
 * that prunes keys and values together, lambda_k + lambda_v).
 *
 * Values cannot be scored against a query, so the score of channel j of token t is the
 * magnitude of the entry itself ("norm-based": the 2-norm of a scalar is its absolute
 * value), and the T_v channels of largest |v| are retained per (token, KV head):
 *     order = channels sorted by |V[n,h,j]| descending, equal magnitudes by ascending j
 *     kept  = first Tv of order;  mask bit j = 1 iff kept
 *     V-hat = kept entries' original bf16 bits in ascending channel order
 *     gap   = (|v|_(Tv) - |v|_(Tv+1)) / |v|_(Tv)   (0 when |v|_(Tv) == 0; +inf when Tv == D)
 * |v| of a bf16 entry is exact in binary32, so the kept set is a pure function of bits.
 * Reading of the appendix (it is brief): the pruned entries are dropped and nothing is
 * cached in their place -- it says that values need no scaling or recombination because
 * they are consumed directly by the weighted sum -- so they contribute 0 at decode.
 *
 * v: element (n,h,j) at v[n*tok_stride + h*head_stride + j]; mask [total,Hkv,ceil(D/32)];
 * kept [total,Hkv,Tv]; gap [total,Hkv].  Returns 0, or -1 on bad arguments.
 */
int oracle_prune_values(const uint16_t *v, int64_t tok_stride, int64_t head_stride,
                        int64_t total, int Hkv, int D, int Tv, uint32_t *mask, uint16_t *kept,
                        double *gap)
{
    if (D < 1 || D > 1024 || Tv < 1 || Tv > D || Hkv < 1 || total < 0) return -1;
    const int MW = (D + 31) / 32;
    int64_t n;
#pragma omp parallel for schedule(static)
    for (n = 0; n < total; ++n) {
        float mag[1024];
        int order[1024];
        for (int h = 0; h < Hkv; ++h) {
            const uint16_t *vrow = v + n * tok_stride + (int64_t)h * head_stride;
            const int64_t row = n * Hkv + h;
            for (int j = 0; j < D; ++j) mag[j] = fabsf(bf16_bits_to_f32(vrow[j]));
            /* stable insertion sort of channel indices: magnitude descending, ties by index */
            for (int j = 0; j < D; ++j) {
                int p = j;
                while (p > 0 && mag[order[p - 1]] < mag[j]) {
                    order[p] = order[p - 1];
                    --p;
                }
                order[p] = j;
            }
            for (int m = 0; m < MW; ++m) mask[row * MW + m] = 0u;
            for (int i = 0; i < Tv; ++i) mask[row * MW + order[i] / 32] |= (1u << (order[i] % 32));
            int c = 0;
            for (int j = 0; j < D; ++j)
                if (mask[row * MW + j / 32] >> (j % 32) & 1u) kept[row * Tv + c++] = vrow[j];
            if (Tv == D)
                gap[row] = INFINITY;
            else {
                const double hi = (double)mag[order[Tv - 1]], lo = (double)mag[order[Tv]];
                gap[row] = (hi > 0.0) ? (hi - lo) / hi : 0.0;
            }
        }
    }
    return 0;
}

/*
 * The value rows as decode sees them: kept entries back at their channels, every pruned
 * entry 0 (see above).  vtilde [total,Hkv,D] bf16 bits; feeding it to the decode functions
 * below as V is decode attention over a cache with pruned keys AND pruned values.
 */
void oracle_expand_values(const uint32_t *mask, const uint16_t *kept, int64_t total, int Hkv,
                          int D, int Tv, uint16_t *vtilde)
{
    const int MW = (D + 31) / 32;
    for (int64_t row = 0; row < total * Hkv; ++row) {
        int c = 0;
        for (int j = 0; j < D; ++j)
            vtilde[row * D + j] =
                (mask[row * MW + j / 32] >> (j % 32) & 1u) ? kept[row * Tv + c++] : (uint16_t)0;
    }
}

/* ------------------------------------------------------------- decode */

/* value of the i-th kept entry of a packed row, from bf16 bits or from int8 code * scale */
static double kept_value(const uint16_t *kept_bf16, const int8_t *codes, const float *scale,
                         int64_t row, int T, int i)
{
    if (codes) return (double)codes[row * T + i] * (double)scale[row];
    return bf16_bits_to_f64(kept_bf16[row * T + i]);
}

/*
 * Softmax over scores s[0..S) and weighted sum of V rows: Eq. (4),
 *     p = softmax(s),  o = sum_t p_t * V[t,:]
 * (the maximum is subtracted before exponentiation; that is the same function).
 * S == 0 gives o = 0.  probs (may be NULL) receives p.
 */
static void softmax_weighted_sum(const double *s, int64_t S, const uint16_t *v,
                                 int64_t v_tok_stride, int D, double *o, double *probs)
{
    for (int j = 0; j < D; ++j) o[j] = 0.0;
    if (S <= 0) return;
    double m = s[0];
    for (int64_t t = 1; t < S; ++t)
        if (s[t] > m) m = s[t];
    double z = 0.0;
    for (int64_t t = 0; t < S; ++t) z += exp(s[t] - m);
    for (int64_t t = 0; t < S; ++t) {
        const double p = exp(s[t] - m) / z;
        if (probs) probs[t] = p;
        const uint16_t *vrow = v + t * v_tok_stride;
        for (int j = 0; j < D; ++j) o[j] += p * bf16_bits_to_f64(vrow[j]);
    }
}

/*
 * Decode attention over the pruned cache, LITERAL form (the oracle of record).
 * Sec. "SparK", "Channel Recovery": every pruned entry (t, j) is rebuilt with the
 * degenerate recovery function,  ktilde[t,j] = mu_pruned[t] / a[j]  (0 if a[j] == 0),
 * kept entries are copied back to their channels by the mask, which gives the full
 * K-tilde row; then standard attention, Eq. (4):
 *     s[g,t] = scale * <q[g,:], ktilde[t,:]>,  p = softmax_t(s),  o[g,:] = sum_t p[g,t] V[t,h,:]
 * with h = g / G and t running over the whole cached sequence of batch element b.
 *
 * q [B,Hq,D] bf16 bits; mask/kept/mu32/a32 as written by oracle_prune (kept_bf16 used
 * when codes == NULL, else codes [total,Hkv,T] int8 with scale [total,Hkv]);
 * v element (n,h,j) at v[n*v_tok_stride + h*v_head_stride + j];
 * out [B,Hq,D] double; probs (may be NULL) [Hq,total] double.
 */
void oracle_decode_literal(const uint16_t *q, const uint32_t *mask, const uint16_t *kept_bf16,
                           const int8_t *codes, const float *scale, const float *mu32,
                           const float *a32, const uint16_t *v, int64_t v_tok_stride,
                           int64_t v_head_stride, const int32_t *cu, int B, int Hq, int Hkv,
                           int D, int T, double softmax_scale, double *out, double *probs)
{
    const int G = Hq / Hkv;
    const int MW = (D + 31) / 32;
    const int64_t total = cu[B];
    int bg;
#pragma omp parallel for schedule(dynamic, 1)
    for (bg = 0; bg < B * Hq; ++bg) {
        const int b = bg / Hq, g = bg % Hq, h = g / G;
        const int64_t n0 = cu[b], S = cu[b + 1] - cu[b];
        const float *a = a32 + ((int64_t)b * Hkv + h) * D;
        double *s = (double *)malloc(sizeof(double) * (size_t)(S > 0 ? S : 1));
        double *ktilde = (double *)malloc(sizeof(double) * (size_t)D);
        for (int64_t t = 0; t < S; ++t) {
            const int64_t row = (n0 + t) * Hkv + h;
            int c = 0;
            for (int j = 0; j < D; ++j) {
                if (mask[row * MW + j / 32] >> (j % 32) & 1u)
                    ktilde[j] = kept_value(kept_bf16, codes, scale, row, T, c++);
                else
                    ktilde[j] = (a[j] != 0.0f) ? (double)mu32[row] / (double)a[j] : 0.0;
            }
            double dot = 0.0;
            for (int j = 0; j < D; ++j)
                dot += bf16_bits_to_f64(q[((int64_t)b * Hq + g) * D + j]) * ktilde[j];
            s[t] = softmax_scale * dot;
        }
        softmax_weighted_sum(s, S, v + n0 * v_tok_stride + (int64_t)h * v_head_stride,
                             v_tok_stride, D, out + ((int64_t)b * Hq + g) * D,
                             probs ? probs + (int64_t)g * total + n0 : NULL);
        free(s);
        free(ktilde);
    }
}

/*
 * The same decode with the recovery term taken out of the channel sum (an algebraic
 * identity of the literal form, used only to cross-check it):
 *     <q, ktilde_t> = sum_{j kept} q_j k_tj + mu_t * ( R - sum_{j kept} r_j ),
 *     r_j = q_j / a_j (0 if a_j == 0),  R = sum_j r_j.
 */
void oracle_decode_fused(const uint16_t *q, const uint32_t *mask, const uint16_t *kept_bf16,
                         const int8_t *codes, const float *scale, const float *mu32,
                         const float *a32, const uint16_t *v, int64_t v_tok_stride,
                         int64_t v_head_stride, const int32_t *cu, int B, int Hq, int Hkv, int D,
                         int T, double softmax_scale, double *out)
{
    const int G = Hq / Hkv;
    const int MW = (D + 31) / 32;
    int bg;
#pragma omp parallel for schedule(dynamic, 1)
    for (bg = 0; bg < B * Hq; ++bg) {
        const int b = bg / Hq, g = bg % Hq, h = g / G;
        const int64_t n0 = cu[b], S = cu[b + 1] - cu[b];
        const float *a = a32 + ((int64_t)b * Hkv + h) * D;
        double *s = (double *)malloc(sizeof(double) * (size_t)(S > 0 ? S : 1));
        double *r = (double *)malloc(sizeof(double) * (size_t)D);
        double R = 0.0;
        for (int j = 0; j < D; ++j) {
            const double qj = bf16_bits_to_f64(q[((int64_t)b * Hq + g) * D + j]);
            r[j] = (a[j] != 0.0f) ? qj / (double)a[j] : 0.0;
            R += r[j];
        }
        for (int64_t t = 0; t < S; ++t) {
            const int64_t row = (n0 + t) * Hkv + h;
            double qk = 0.0, rk = 0.0;
            int c = 0;
            for (int j = 0; j < D; ++j)
                if (mask[row * MW + j / 32] >> (j % 32) & 1u) {
                    qk += bf16_bits_to_f64(q[((int64_t)b * Hq + g) * D + j]) *
                          kept_value(kept_bf16, codes, scale, row, T, c++);
                    rk += r[j];
                }
            s[t] = softmax_scale * (qk + (double)mu32[row] * (R - rk));
        }
        softmax_weighted_sum(s, S, v + n0 * v_tok_stride + (int64_t)h * v_head_stride,
                             v_tok_stride, D, out + ((int64_t)b * Hq + g) * D, NULL);
        free(s);
        free(r);
    }
}

/* ------------------------------------------------------------- sampled recovery */

/*
 * Per-token statistics of the saliency over ALL channels, App. "Caching Pruned Channel
 * Statistics": for every (token n, KV head h), with w_j = a32[b,h,j] * |K[n,h,j]| (the same
 * binary32 product the selection compares),
 *     mu    = (1/D) sum_j w_j
 *     sigma = sqrt( (1/D) sum_j (w_j - mu)^2 )          (population standard deviation)
 * in double, each rounded once to binary32 for storage.  mu32, sigma32 [total,Hkv].
 */
void oracle_row_stats(const uint16_t *k, int64_t k_tok_stride, int64_t k_head_stride,
                      const float *a32, const int32_t *cu, int B, int Hkv, int D, float *mu32,
                      float *sigma32)
{
    const int64_t total = cu[B];
    int64_t n;
#pragma omp parallel for schedule(static)
    for (n = 0; n < total; ++n) {
        const int b = seq_of_token(cu, B, n);
        for (int h = 0; h < Hkv; ++h) {
            const uint16_t *krow = k + n * k_tok_stride + (int64_t)h * k_head_stride;
            const float *a = a32 + ((int64_t)b * Hkv + h) * D;
            double w[1024], s = 0.0;
            for (int j = 0; j < D; ++j) {
                volatile float prod = a[j] * fabsf(bf16_bits_to_f32(krow[j]));
                w[j] = (double)prod;
                s += w[j];
            }
            const double mu = s / (double)D;
            double ss = 0.0;
            for (int j = 0; j < D; ++j) ss += (w[j] - mu) * (w[j] - mu);
            mu32[n * Hkv + h] = (float)mu;
            sigma32[n * Hkv + h] = (float)sqrt(ss / (double)D);
        }
    }
}

/*
 * Random numbers of the sampled recovery functions.  The paper does not say how or when the
 * samples are drawn; here they are a pure function of (seed, token n, KV head h, counter c),
 * so a decode step can be repeated and both implementations can produce the same variates:
 *     mix(x):  x ^= x >> 16;  x *= 0x85EBCA6B;  x ^= x >> 13;  x *= 0xC2B2AE35;  x ^= x >> 16
 *              (the 32-bit finalizer of MurmurHash3, a bijection of the 32-bit words)
 *     base   = mix( mix( mix(n) + seed_lo ) + h * 0x9E3779B9 + seed_hi )
 *     x_c    = mix( base + c * 0x9E3779B9 )
 *     u_c    = ( (x_c >> 9) + 0.5 ) / 2^23            in (0, 1), 23 bits (exact in binary32 too)
 */
static uint32_t mix32(uint32_t x)
{
    x ^= x >> 16;
    x *= 0x85EBCA6Bu;
    x ^= x >> 13;
    x *= 0xC2B2AE35u;
    x ^= x >> 16;
    return x;
}

uint32_t oracle_mix32(uint32_t x) { return mix32(x); }

double oracle_uniform(uint32_t seed_lo, uint32_t seed_hi, uint32_t n, uint32_t h, uint32_t c)
{
    const uint32_t base = mix32(mix32(mix32(n) + seed_lo) + h * 0x9E3779B9u + seed_hi);
    const uint32_t x = mix32(base + c * 0x9E3779B9u);
    return ((double)(x >> 9) + 0.5) / 8388608.0;
}

/*
 * Sampled saliency of pruned channel j of row (n, h), Sec. "SparK", "Channel Recovery":
 *   kind 1, Gaussian:     w~ = mu + sigma * z_j,  z from the Box-Muller transform of the pair
 *                         (u_{2m}, u_{2m+1}) for channels j = 2m, 2m+1:
 *                         z_{2m} = sqrt(-2 ln u_{2m}) cos(2 pi u_{2m+1}),  z_{2m+1} = ... sin(...)
 *   kind 2, Exponential:  w~ = -mu * ln(u_j)        (rate 1/mu, i.e. mean mu)
 * mu, sigma are the all-channel statistics above.  A Gaussian sample may be negative; the
 * paper does not clamp it and neither does this.
 */
static double sampled_saliency(int kind, double mu, double sigma, uint32_t seed_lo,
                               uint32_t seed_hi, uint32_t n, uint32_t h, int j)
{
    const double two_pi = 6.283185307179586476925286766559;
    if (kind == 1) {
        const int m = j >> 1;
        const double u1 = oracle_uniform(seed_lo, seed_hi, n, h, (uint32_t)(2 * m));
        const double u2 = oracle_uniform(seed_lo, seed_hi, n, h, (uint32_t)(2 * m + 1));
        const double r = sqrt(-2.0 * log(u1));
        const double z = (j & 1) ? r * sin(two_pi * u2) : r * cos(two_pi * u2);
        return mu + sigma * z;
    }
    return -mu * log(oracle_uniform(seed_lo, seed_hi, n, h, (uint32_t)j));
}

/*
 * Decode attention with a sampled recovery function (literal form): pruned entry (n, j) is
 * rebuilt as  ktilde = w~ / a_j  (0 if a_j == 0) with w~ drawn as above, kept entries are
 * copied back, then Eq. (4).  kind: 1 Gaussian, 2 Exponential.  mu_all32, sigma32 from
 * oracle_row_stats.  ktilde_out (may be NULL) [total,Hkv,D] double receives the rebuilt keys.
 * Kept entries as in oracle_decode_literal: the original bf16 bits, or code * scale when the
 * int8 storage variant is in use (codes != NULL); the statistics are those of the saliencies
 * before quantisation either way.  Other arguments as oracle_decode_literal.
 */
void oracle_decode_sampled(int kind, uint32_t seed_lo, uint32_t seed_hi, const uint16_t *q,
                           const uint32_t *mask, const uint16_t *kept_bf16, const int8_t *codes,
                           const float *scale, const float *mu_all32,
                           const float *sigma32, const float *a32, const uint16_t *v,
                           int64_t v_tok_stride, int64_t v_head_stride, const int32_t *cu, int B,
                           int Hq, int Hkv, int D, int T, double softmax_scale, double *out,
                           double *ktilde_out)
{
    const int G = Hq / Hkv;
    const int MW = (D + 31) / 32;
    int bg;
#pragma omp parallel for schedule(dynamic, 1)
    for (bg = 0; bg < B * Hq; ++bg) {
        const int b = bg / Hq, g = bg % Hq, h = g / G;
        const int64_t n0 = cu[b], S = cu[b + 1] - cu[b];
        const float *a = a32 + ((int64_t)b * Hkv + h) * D;
        double *s = (double *)malloc(sizeof(double) * (size_t)(S > 0 ? S : 1));
        double *ktilde = (double *)malloc(sizeof(double) * (size_t)D);
        for (int64_t t = 0; t < S; ++t) {
            const int64_t row = (n0 + t) * Hkv + h;
            int c = 0;
            for (int j = 0; j < D; ++j) {
                if (mask[row * MW + j / 32] >> (j % 32) & 1u)
                    ktilde[j] = kept_value(kept_bf16, codes, scale, row, T, c++);
                else if (a[j] != 0.0f)
                    ktilde[j] = sampled_saliency(kind, (double)mu_all32[row], (double)sigma32[row], seed_lo,
                                                 seed_hi, (uint32_t)(n0 + t), (uint32_t)h, j) / (double)a[j];
                else
                    ktilde[j] = 0.0;
                if (ktilde_out && g % G == 0) ktilde_out[row * D + j] = ktilde[j];
            }
            double dot = 0.0;
            for (int j = 0; j < D; ++j)
                dot += bf16_bits_to_f64(q[((int64_t)b * Hq + g) * D + j]) * ktilde[j];
            s[t] = softmax_scale * dot;
        }
        softmax_weighted_sum(s, S, v + n0 * v_tok_stride + (int64_t)h * v_head_stride,
                             v_tok_stride, D, out + ((int64_t)b * Hq + g) * D, NULL);
        free(s);
        free(ktilde);
    }
}

/*
 * Decode attention when tokens have been appended after prefill.
 * Sec. "Preliminaries": at every decode step the new token's key and value are concatenated to
 * the cache; Sec. "SparK": pruning happens once, at prefill.  So the cache of sequence b is the
 * S_b pruned prefix rows followed by L_b appended rows that were never pruned (reading: appended
 * rows stay dense; the paper does not say that they are pruned later).  The literal form: rebuild
 * K-tilde for the prefix as in oracle_decode_literal, use the appended keys as they are, one
 * softmax over all S_b + L_b scores, weighted sum over the prefix values followed by the
 * appended values (Eq. (4) on the concatenated cache).
 *
 * tail_k, tail_v [B, cap, Hkv, D] bf16 bits; tail_len [B], 0 <= tail_len[b] <= cap.
 * Other arguments as oracle_decode_literal; out [B,Hq,D] double.
 */
void oracle_decode_literal_tail(const uint16_t *q, const uint32_t *mask, const uint16_t *kept_bf16,
                                const int8_t *codes, const float *scale, const float *mu32,
                                const float *a32, const uint16_t *v, int64_t v_tok_stride,
                                int64_t v_head_stride, const int32_t *cu, const uint16_t *tail_k,
                                const uint16_t *tail_v, const int32_t *tail_len, int cap, int B,
                                int Hq, int Hkv, int D, int T, double softmax_scale, double *out)
{
    const int G = Hq / Hkv;
    const int MW = (D + 31) / 32;
    int bg;
#pragma omp parallel for schedule(dynamic, 1)
    for (bg = 0; bg < B * Hq; ++bg) {
        const int b = bg / Hq, g = bg % Hq, h = g / G;
        const int64_t n0 = cu[b], S = cu[b + 1] - cu[b], Lb = tail_len[b], N = S + Lb;
        const float *a = a32 + ((int64_t)b * Hkv + h) * D;
        const uint16_t *qrow = q + ((int64_t)b * Hq + g) * D;
        double *s = (double *)malloc(sizeof(double) * (size_t)(N > 0 ? N : 1));
        double *ktilde = (double *)malloc(sizeof(double) * (size_t)D);
        double *o = out + ((int64_t)b * Hq + g) * D;
        for (int64_t t = 0; t < S; ++t) {
            const int64_t row = (n0 + t) * Hkv + h;
            int c = 0;
            for (int j = 0; j < D; ++j) {
                if (mask[row * MW + j / 32] >> (j % 32) & 1u)
                    ktilde[j] = kept_value(kept_bf16, codes, scale, row, T, c++);
                else
                    ktilde[j] = (a[j] != 0.0f) ? (double)mu32[row] / (double)a[j] : 0.0;
            }
            double dot = 0.0;
            for (int j = 0; j < D; ++j) dot += bf16_bits_to_f64(qrow[j]) * ktilde[j];
            s[t] = softmax_scale * dot;
        }
        for (int64_t t = 0; t < Lb; ++t) {
            const uint16_t *krow = tail_k + (((int64_t)b * cap + t) * Hkv + h) * D;
            double dot = 0.0;
            for (int j = 0; j < D; ++j) dot += bf16_bits_to_f64(qrow[j]) * bf16_bits_to_f64(krow[j]);
            s[S + t] = softmax_scale * dot;
        }
        for (int j = 0; j < D; ++j) o[j] = 0.0;
        if (N > 0) {
            double m = s[0];
            for (int64_t t = 1; t < N; ++t)
                if (s[t] > m) m = s[t];
            double z = 0.0;
            for (int64_t t = 0; t < N; ++t) z += exp(s[t] - m);
            for (int64_t t = 0; t < N; ++t) {
                const double p = exp(s[t] - m) / z;
                const uint16_t *vrow = (t < S) ? v + (n0 + t) * v_tok_stride + (int64_t)h * v_head_stride
                                               : tail_v + (((int64_t)b * cap + (t - S)) * Hkv + h) * D;
                for (int j = 0; j < D; ++j) o[j] += p * bf16_bits_to_f64(vrow[j]);
            }
        }
        free(s);
        free(ktilde);
    }
}

/*
 * Standard decode attention on the unpruned cache, Eq. (4) as printed:
 *     a = softmax(q K^T / sqrt(D)) (any scale may be passed),  o = a V.
 */
void oracle_dense_attn(const uint16_t *q, const uint16_t *k, int64_t k_tok_stride,
                       int64_t k_head_stride, const uint16_t *v, int64_t v_tok_stride,
                       int64_t v_head_stride, const int32_t *cu, int B, int Hq, int Hkv, int D,
                       double softmax_scale, double *out)
{
    const int G = Hq / Hkv;
    int bg;
#pragma omp parallel for schedule(dynamic, 1)
    for (bg = 0; bg < B * Hq; ++bg) {
        const int b = bg / Hq, g = bg % Hq, h = g / G;
        const int64_t n0 = cu[b], S = cu[b + 1] - cu[b];
        double *s = (double *)malloc(sizeof(double) * (size_t)(S > 0 ? S : 1));
        for (int64_t t = 0; t < S; ++t) {
            const uint16_t *krow = k + (n0 + t) * k_tok_stride + (int64_t)h * k_head_stride;
            double dot = 0.0;
            for (int j = 0; j < D; ++j)
                dot += bf16_bits_to_f64(q[((int64_t)b * Hq + g) * D + j]) * bf16_bits_to_f64(krow[j]);
            s[t] = softmax_scale * dot;
        }
        softmax_weighted_sum(s, S, v + n0 * v_tok_stride + (int64_t)h * v_head_stride,
                             v_tok_stride, D, out + ((int64_t)b * Hq + g) * D, NULL);
        free(s);
    }
}
