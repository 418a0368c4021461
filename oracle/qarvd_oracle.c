/*
 * CPU oracle for the dual-scale W8A8 linear layer of Q-ARVD.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain reference that the
 * GPU library is checked against.  It shares no code, header, table or helper
 * with the HIP implementation and must never be called from the product path.
 *
 * Everything is written as the definition it implements, one loop per
 * subscript, with no blocking, fusion or reordering.  Floating point follows
 * IEEE-754 round-to-nearest-even; build with -O2 -ffp-contract=off so that no
 * multiply-add is contracted.  The only parallelism is an OpenMP "parallel
 * for" over independent rows (token rows m, or weight rows j), which does not
 * change any result.
 *
 * Layouts (all row-major, unpadded, host memory):
 *   W  f32[N,K]   N = d_out rows, K = d_in input channels
 *   X  f32[M,K]   M tokens
 *   Wq i8[N,K], Xq i8[M,K]  packed channel order: position p holds channel perm[p];
 *                 positions [0,K_o) are the outlier block, [K_o,K) the normal block
 *
 * Paper passages followed:
 *   uniform symmetric quantizer          Sec. 2.2, Eq. (quantization)
 *   per-input-channel L2 norm vector v   Sec. 3.2, observations + "Given the L2 norm vector v"
 *   MAD, modified Z-score, threshold     Sec. 3.2, Eqs. (mad), (modified_zscore), (ori_threshold), (new_threshold)
 *   >=1 outlier gates dual-scale         Sec. 3.2, text after Eq. (new_threshold)
 *   align outlier count to 32            Fig. "outlier patterns" caption
 *   dual-scale concat [outlier|normal]   Sec. 3.2, Eq. (dual_scale)
 *   per-channel (per output row) weights Sec. 4.1 "Quantization Implementation"
 *   two kernels: act-quant, GEMM+dequant App. "Quantization Kernels and Extra Cost Analysis"
 *   4-bit weights (W4A8)                 Sec. 4.2 (result tables), Eq. (quantization) at b = 4
 *   static per-tensor activation scale   Sec. 4.1 "Quantization Implementation"
 *   percentile-clip scale initialisation Sec. 4.1 "Quantization Implementation"
 *
 * Readings taken where the paper is silent (each is listed in the design notes):
 *   median of an even-length vector = mean of the two middle values;
 *   alignment rounds the count UP and fills with the largest-norm unflagged channels;
 *   outlier block first, ascending channel index inside each block;
 *   weight scale = block absmax / 127 per output row, round-half-even, clip [-127,127];
 *   activation scale = per-token absmax / 127 over all K channels (dynamic);
 *   a zero scale quantizes to 0; absent bias is +0.0f;
 *   chained layers: GELU (tanh form) in fp32 with a fixed operation sequence, then the next layer's
 *   static scale; percentile clip: linear-interpolated quantile of |w| per row and block, squared
 *   error summed in double in packed order, the larger percentile on a tie.
 *
 * Parity status: every function below is pinned by tests/test_oracle_*.py
 * against brute force, library routines (numpy / scipy) and invariants.
 * Fidelity to the authors' unpublished code is unpinned (no numbers printed
 * by the paper for this path).
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#define ORACLE_OK 0
#define ORACLE_BAD_ARG -1

/* ------------------------------------------------------------------ helpers */

static int cmp_double(const void *a, const void *b)
{
    double x = *(const double *)a, y = *(const double *)b;
    return (x > y) - (x < y);
}

/* Textbook median: sort ascending; odd n -> middle, even n -> mean of the two middle. */
static double median_of(const double *x, int n)
{
    double *t = (double *)malloc((size_t)n * sizeof(double));
    double m;
    memcpy(t, x, (size_t)n * sizeof(double));
    qsort(t, (size_t)n, sizeof(double), cmp_double);
    if (n % 2 == 1)
        m = t[n / 2];
    else
        m = (t[n / 2 - 1] + t[n / 2]) / 2.0;
    free(t);
    return m;
}

/*
 * Eq. (quantization) with z = 0 and the symmetric range q in [-qmax, qmax],
 * qmax = 2^(b-1) - 1 (127 for b = 8, 7 for b = 4); s == 0 -> 0.
 */
static int8_t quantize_sym(float x, float s, float qmax)
{
    float r;
    if (s == 0.0f)
        return 0;
    r = rintf(x / s); /* round-half-to-even in the default rounding mode */
    if (r > qmax)
        r = qmax;
    if (r < -qmax)
        r = -qmax;
    return (int8_t)r;
}

static int8_t quantize_one(float x, float s) { return quantize_sym(x, s, 127.0f); }

/* float -> bfloat16 bits, round-to-nearest-even (finite inputs). */
static uint16_t bf16_rne(float f)
{
    uint32_t u;
    memcpy(&u, &f, 4);
    u += 0x7FFFu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}

/* ------------------------------------------------- detector (Sec. 3.2) ---- */

/*
 * Column norms: v[k] = (float) sqrt( sum_j (double)W[j,k]^2 ), rows summed in
 * ascending j.  Each square is exact in fp64.
 */
int oracle_column_norms(const float *W, int N, int K, float *v)
{
    if (!W || !v || N <= 0 || K <= 0)
        return ORACLE_BAD_ARG;
    for (int k = 0; k < K; ++k) {
        double S = 0.0;
        for (int j = 0; j < N; ++j) {
            double w = (double)W[(size_t)j * K + k];
            S = S + w * w;
        }
        v[k] = (float)sqrt(S);
    }
    return ORACLE_OK;
}

/*
 * Outlier detection on a norm vector.
 *   med  = median(v)                     Eq. (mad)
 *   MAD  = median(|v_k - med|)           Eq. (mad)
 *   T    = max(med + (tau/0.6745)*MAD, alpha*med)   Eq. (new_threshold)
 *   flag = v_k > T  (strict)
 * Outputs: flag[K] (0/1), stats[4] = {med, MAD, T, n_det}.
 */
int oracle_detect(const float *v, int K, double tau, double alpha, uint8_t *flag, double *stats)
{
    double *vd, *d, med, mad, c, T1, T2, T;
    int n_det = 0;
    if (!v || !flag || K <= 0)
        return ORACLE_BAD_ARG;
    vd = (double *)malloc((size_t)K * sizeof(double));
    d = (double *)malloc((size_t)K * sizeof(double));
    for (int k = 0; k < K; ++k)
        vd[k] = (double)v[k];
    med = median_of(vd, K);
    for (int k = 0; k < K; ++k)
        d[k] = fabs(vd[k] - med);
    mad = median_of(d, K);
    c = tau / 0.6745;
    T1 = c * mad;
    T1 = med + T1;
    T2 = alpha * med;
    T = (T1 > T2) ? T1 : T2;
    for (int k = 0; k < K; ++k) {
        flag[k] = (vd[k] > T) ? 1 : 0;
        n_det += flag[k];
    }
    if (stats) {
        stats[0] = med;
        stats[1] = mad;
        stats[2] = T;
        stats[3] = (double)n_det;
    }
    free(vd);
    free(d);
    return ORACLE_OK;
}

/*
 * Alignment (Fig. "outlier patterns" caption): if any channel is flagged, grow
 * the outlier set to the next multiple of `align` (capped at K) by adding, one
 * at a time, the not-yet-selected channel with the largest norm (ties: the
 * smaller index).  No flagged channel -> nothing is added.  `sel` is updated in
 * place; returns the final count through K_o.
 */
int oracle_align(const float *v, int K, int align, uint8_t *sel, int *K_o)
{
    int n = 0, target;
    if (!v || !sel || !K_o || K <= 0 || align <= 0)
        return ORACLE_BAD_ARG;
    for (int k = 0; k < K; ++k)
        n += sel[k] ? 1 : 0;
    if (n == 0) {
        *K_o = 0;
        return ORACLE_OK;
    }
    target = ((n + align - 1) / align) * align;
    if (target > K)
        target = K;
    while (n < target) {
        int best = -1;
        for (int k = 0; k < K; ++k) {
            if (sel[k])
                continue;
            if (best < 0 || v[k] > v[best])
                best = k;
        }
        sel[best] = 1;
        ++n;
    }
    *K_o = n;
    return ORACLE_OK;
}

/* Eq. (dual_scale): perm = [selected channels ascending | the rest ascending]. */
int oracle_build_perm(const uint8_t *sel, int K, int32_t *perm, int *K_o)
{
    int p = 0;
    if (!sel || !perm || K <= 0)
        return ORACLE_BAD_ARG;
    for (int k = 0; k < K; ++k)
        if (sel[k])
            perm[p++] = k;
    if (K_o)
        *K_o = p;
    for (int k = 0; k < K; ++k)
        if (!sel[k])
            perm[p++] = k;
    return ORACLE_OK;
}

/*
 * Dual-scale weight quantization for a given split (Eq. (dual_scale), Eq.
 * (quantization), one scale per output row per block).
 */
/*
 * `bits` = 8 or 4: the weight bit-width of the W8A8 and W4A8 settings (Sec. 4.2).  The codes are
 * returned one per int8 either way; only their range and the scale divisor (2^(bits-1) - 1) differ.
 */
int oracle_quantize_rows_bits(const float *W, int N, int K, const int32_t *perm, int K_o, int bits,
                              int8_t *Wq, float *s_normal, float *s_outlier)
{
    float qmax;
    if (!W || !perm || !Wq || !s_normal || !s_outlier || N <= 0 || K <= 0 || K_o < 0 || K_o > K ||
        (bits != 8 && bits != 4))
        return ORACLE_BAD_ARG;
    qmax = bits == 8 ? 127.0f : 7.0f;
#pragma omp parallel for schedule(static)
    for (int j = 0; j < N; ++j) {
        const float *w = W + (size_t)j * K;
        float a_o = 0.0f, a_n = 0.0f, so, sn;
        for (int p = 0; p < K_o; ++p) {
            float a = fabsf(w[perm[p]]);
            if (a > a_o)
                a_o = a;
        }
        for (int p = K_o; p < K; ++p) {
            float a = fabsf(w[perm[p]]);
            if (a > a_n)
                a_n = a;
        }
        so = a_o / qmax;
        sn = a_n / qmax;
        s_outlier[j] = so;
        s_normal[j] = sn;
        for (int p = 0; p < K_o; ++p)
            Wq[(size_t)j * K + p] = quantize_sym(w[perm[p]], so, qmax);
        for (int p = K_o; p < K; ++p)
            Wq[(size_t)j * K + p] = quantize_sym(w[perm[p]], sn, qmax);
    }
    return ORACLE_OK;
}

/* ---------------- percentile-clip initialisation of the weight scales (Sec. 4.1) */

static int cmp_float_asc(const void *a, const void *b)
{
    float x = *(const float *)a, y = *(const float *)b;
    return (x > y) - (x < y);
}

/*
 * Sec. 4.1 "Quantization Implementation": the scaling factors are initialised by searching the clipping
 * percentile over {0.999, 0.9999, 0.99999}.  The paper states neither the objective nor the percentile
 * convention; the reading taken (data-free, for one block of one output row, n values w[0..n-1]):
 *   a = |w| sorted ascending;  for p in the list:  h = (n-1) p,  lo = floor(h),
 *       clip_p = a[lo] + (h - lo) (a[min(lo+1, n-1)] - a[lo])      (linear interpolation, in double, rounded to float)
 *       s_p = clip_p / qmax,  q_i = clip(rint(w_i / s_p), -qmax, qmax),
 *       e_i = fmaf(-s_p, q_i, w_i) (float),  SSE_p = sum_i (double)e_i^2, i ascending, in double;
 *   the percentile with the smallest SSE wins, the LARGER percentile on a tie (least clipping).
 * Outputs: *s_out the chosen scale, *choice_out 0/1/2 = index into the list; clip_out[3], sse_out[3]
 * (nullable) the candidates.  n == 0: scale 0, choice 2.
 */
int oracle_clip_search(const float *w, int n, float qmax, float *s_out, int *choice_out,
                       float *clip_out, double *sse_out)
{
    static const double P[3] = {0.999, 0.9999, 0.99999};
    float *a, clip[3], s[3];
    double sse[3];
    int best;
    if (!w || n < 0 || !s_out || !choice_out || !(qmax >= 1.0f))
        return ORACLE_BAD_ARG;
    if (n == 0) {
        *s_out = 0.0f;
        *choice_out = 2;
        return ORACLE_OK;
    }
    a = (float *)malloc((size_t)n * sizeof(float));
    for (int i = 0; i < n; ++i)
        a[i] = fabsf(w[i]);
    qsort(a, (size_t)n, sizeof(float), cmp_float_asc);
    for (int c = 0; c < 3; ++c) {
        double h = (double)(n - 1) * P[c];
        int lo = (int)floor(h);
        int hi = lo + 1 < n ? lo + 1 : n - 1;
        double frac = h - (double)lo;
        clip[c] = (float)((double)a[lo] + frac * ((double)a[hi] - (double)a[lo]));
        s[c] = clip[c] / qmax;
        sse[c] = 0.0;
        for (int i = 0; i < n; ++i) {
            float q = (float)quantize_sym(w[i], s[c], qmax);
            float e = fmaf(-s[c], q, w[i]);
            sse[c] += (double)e * (double)e;
        }
    }
    free(a);
    best = 2;
    for (int c = 1; c >= 0; --c)
        if (sse[c] < sse[best])
            best = c;
    *s_out = s[best];
    *choice_out = best;
    for (int c = 0; c < 3; ++c) {
        if (clip_out)
            clip_out[c] = clip[c];
        if (sse_out)
            sse_out[c] = sse[c];
    }
    return ORACLE_OK;
}

/*
 * oracle_quantize_rows_bits with the two scales of every row chosen by oracle_clip_search over the
 * row's outlier block and normal block (values taken in packed order) instead of block absmax / qmax.
 * choice_n / choice_o (nullable, [N]): the winning percentile index of each block.
 */
int oracle_quantize_rows_clip(const float *W, int N, int K, const int32_t *perm, int K_o, int bits,
                              int8_t *Wq, float *s_normal, float *s_outlier, int8_t *choice_n,
                              int8_t *choice_o)
{
    float qmax;
    int bad = 0;
    if (!W || !perm || !Wq || !s_normal || !s_outlier || N <= 0 || K <= 0 || K_o < 0 || K_o > K ||
        (bits != 8 && bits != 4))
        return ORACLE_BAD_ARG;
    qmax = bits == 8 ? 127.0f : 7.0f;
#pragma omp parallel for schedule(static)
    for (int j = 0; j < N; ++j) {
        const float *w = W + (size_t)j * K;
        float *blk = (float *)malloc((size_t)K * sizeof(float));
        float so, sn;
        int co, cn;
        for (int p = 0; p < K; ++p)
            blk[p] = w[perm[p]];
        if (oracle_clip_search(blk, K_o, qmax, &so, &co, NULL, NULL) != ORACLE_OK ||
            oracle_clip_search(blk + K_o, K - K_o, qmax, &sn, &cn, NULL, NULL) != ORACLE_OK) {
#pragma omp atomic write
            bad = 1;
        } else {
            s_outlier[j] = so;
            s_normal[j] = sn;
            if (choice_o)
                choice_o[j] = (int8_t)co;
            if (choice_n)
                choice_n[j] = (int8_t)cn;
            for (int p = 0; p < K_o; ++p)
                Wq[(size_t)j * K + p] = quantize_sym(blk[p], so, qmax);
            for (int p = K_o; p < K; ++p)
                Wq[(size_t)j * K + p] = quantize_sym(blk[p], sn, qmax);
        }
        free(blk);
    }
    return bad ? ORACLE_BAD_ARG : ORACLE_OK;
}

int oracle_quantize_rows(const float *W, int N, int K, const int32_t *perm, int K_o,
                         int8_t *Wq, float *s_normal, float *s_outlier)
{
    return oracle_quantize_rows_bits(W, N, K, perm, K_o, 8, Wq, s_normal, s_outlier);
}

/*
 * Whole offline step: norms -> detect -> align -> perm -> dual scales + INT8.
 * forced_mask (nullable, [K] of 0/1): take this outlier set as given and skip
 * detection and alignment.  Optional outputs (nullable): v_out[K], flag_out[K]
 * (raw detector flags before alignment), stats[4].
 */
int oracle_quantize_weight_clip(const float *W, int N, int K, double tau, double alpha, int align,
                                const uint8_t *forced_mask, int bits, int clip_search, int8_t *Wq,
                                float *s_normal, float *s_outlier, int32_t *perm, int32_t *K_o_out,
                                float *v_out, uint8_t *flag_out, double *stats)
{
    float *v;
    uint8_t *sel;
    int K_o = 0, rc;
    if (!W || !Wq || !s_normal || !s_outlier || !perm || !K_o_out || N <= 0 || K <= 0)
        return ORACLE_BAD_ARG;
    v = (float *)malloc((size_t)K * sizeof(float));
    sel = (uint8_t *)malloc((size_t)K);
    rc = oracle_column_norms(W, N, K, v);
    if (rc == ORACLE_OK) {
        if (forced_mask) {
            for (int k = 0; k < K; ++k)
                sel[k] = forced_mask[k] ? 1 : 0;
            if (flag_out)
                memcpy(flag_out, sel, (size_t)K);
        } else {
            rc = oracle_detect(v, K, tau, alpha, sel, stats);
            if (rc == ORACLE_OK && flag_out)
                memcpy(flag_out, sel, (size_t)K);
            if (rc == ORACLE_OK)
                rc = oracle_align(v, K, align, sel, &K_o);
        }
    }
    if (rc == ORACLE_OK)
        rc = oracle_build_perm(sel, K, perm, &K_o);
    if (rc == ORACLE_OK)
        rc = clip_search ? oracle_quantize_rows_clip(W, N, K, perm, K_o, bits, Wq, s_normal, s_outlier, NULL, NULL)
                         : oracle_quantize_rows_bits(W, N, K, perm, K_o, bits, Wq, s_normal, s_outlier);
    if (rc == ORACLE_OK) {
        *K_o_out = K_o;
        if (v_out)
            memcpy(v_out, v, (size_t)K * sizeof(float));
    }
    free(v);
    free(sel);
    return rc;
}

int oracle_quantize_weight_bits(const float *W, int N, int K, double tau, double alpha, int align,
                                const uint8_t *forced_mask, int bits, int8_t *Wq, float *s_normal,
                                float *s_outlier, int32_t *perm, int32_t *K_o_out, float *v_out,
                                uint8_t *flag_out, double *stats)
{
    return oracle_quantize_weight_clip(W, N, K, tau, alpha, align, forced_mask, bits, 0, Wq, s_normal,
                                       s_outlier, perm, K_o_out, v_out, flag_out, stats);
}

int oracle_quantize_weight(const float *W, int N, int K, double tau, double alpha, int align,
                           const uint8_t *forced_mask, int8_t *Wq, float *s_normal,
                           float *s_outlier, int32_t *perm, int32_t *K_o_out, float *v_out,
                           uint8_t *flag_out, double *stats)
{
    return oracle_quantize_weight_bits(W, N, K, tau, alpha, align, forced_mask, 8, Wq, s_normal,
                                       s_outlier, perm, K_o_out, v_out, flag_out, stats);
}

/* --------------------------------- activation quantization (App., kernel i) */

/*
 * Per-token dynamic symmetric INT8: a_m = max_k |X[m,k]| over ALL channels,
 * s_x[m] = a_m / 127, Xq[m,p] = q(X[m,perm[p]], s_x[m]).  perm == NULL: identity.
 */
int oracle_quant_act(const float *X, int M, int K, const int32_t *perm, int8_t *Xq, float *s_x)
{
    if (!X || !Xq || !s_x || M <= 0 || K <= 0)
        return ORACLE_BAD_ARG;
#pragma omp parallel for schedule(static)
    for (int m = 0; m < M; ++m) {
        const float *x = X + (size_t)m * K;
        float a = 0.0f, s;
        for (int k = 0; k < K; ++k) {
            float t = fabsf(x[k]);
            if (t > a)
                a = t;
        }
        s = a / 127.0f;
        s_x[m] = s;
        for (int p = 0; p < K; ++p) {
            int k = perm ? perm[p] : p;
            Xq[(size_t)m * K + p] = quantize_one(x[k], s);
        }
    }
    return ORACLE_OK;
}

/* Static variant (Sec. 4.1: per-tensor static activations): the scale is given. */
int oracle_quant_act_static(const float *X, int M, int K, const int32_t *perm, float s,
                            int8_t *Xq)
{
    if (!X || !Xq || M <= 0 || K <= 0)
        return ORACLE_BAD_ARG;
#pragma omp parallel for schedule(static)
    for (int m = 0; m < M; ++m)
        for (int p = 0; p < K; ++p) {
            int k = perm ? perm[p] : p;
            Xq[(size_t)m * K + p] = quantize_one(X[(size_t)m * K + k], s);
        }
    return ORACLE_OK;
}

/* ------------------------------ dual GEMM + dequant (App., kernel ii) ----- */

/*
 * acc_o[m,j] = sum_{p<K_o}  Xq[m,p]*Wq[j,p]     (exact int32)
 * acc_n[m,j] = sum_{p>=K_o} Xq[m,p]*Wq[j,p]
 * r = (float)acc_o * s_o[j];  r = fmaf((float)acc_n, s_n[j], r);  r = fmaf(r, s_x[m], b[j])
 * Y = r (fp32) and/or bf16_rne(r).  Nullable outputs: Y_f32, Y_bf16, acc_n, acc_o.
 */
int oracle_dual_gemm(const int8_t *Xq, const float *s_x, const int8_t *Wq, const float *s_normal,
                     const float *s_outlier, const float *bias, int M, int N, int K, int K_o,
                     float *Y_f32, uint16_t *Y_bf16, int32_t *acc_n_out, int32_t *acc_o_out)
{
    if (!Xq || !s_x || !Wq || !s_normal || !s_outlier || M <= 0 || N <= 0 || K <= 0 || K_o < 0 ||
        K_o > K)
        return ORACLE_BAD_ARG;
#pragma omp parallel for schedule(static)
    for (int m = 0; m < M; ++m) {
        for (int j = 0; j < N; ++j) {
            const int8_t *x = Xq + (size_t)m * K;
            const int8_t *w = Wq + (size_t)j * K;
            int32_t acc_o = 0, acc_n = 0;
            float b = bias ? bias[j] : 0.0f;
            float r;
            for (int p = 0; p < K_o; ++p)
                acc_o += (int32_t)x[p] * (int32_t)w[p];
            for (int p = K_o; p < K; ++p)
                acc_n += (int32_t)x[p] * (int32_t)w[p];
            r = (float)acc_o * s_outlier[j];
            r = fmaf((float)acc_n, s_normal[j], r);
            r = fmaf(r, s_x[m], b);
            if (Y_f32)
                Y_f32[(size_t)m * N + j] = r;
            if (Y_bf16)
                Y_bf16[(size_t)m * N + j] = bf16_rne(r);
            if (acc_n_out)
                acc_n_out[(size_t)m * N + j] = acc_n;
            if (acc_o_out)
                acc_o_out[(size_t)m * N + j] = acc_o;
        }
    }
    return ORACLE_OK;
}

/* ----------- chained layers: the epilogue quantizes for the next layer (static scale) */

/*
 * GELU, tanh form, as it is defined:  gelu(x) = 0.5 x (1 + tanh(u)),  u = sqrt(2/pi) (x + 0.044715 x^3),
 * evaluated in double precision with the C library's tanh and rounded once to float.  The paper does
 * not name the FFN activation; this is the one the Wan-style DiT blocks of Sec. 4.1 use.  A GPU kernel
 * evaluates the same function in fp32 by its own sequence of operations, so codes derived from the
 * two may differ by one where a / s_out falls next to a rounding boundary; the parity tests state
 * that rule.
 */
float oracle_gelu_tanh(float x)
{
    double xd = (double)x;
    double u = sqrt(2.0 / 3.14159265358979323846) * (xd + 0.044715 * xd * xd * xd);
    return (float)(0.5 * xd * (1.0 + tanh(u)));
}

/*
 * The dual GEMM with the epilogue of a chained layer: the fp32 result r of oracle_dual_gemm
 * (same three operations), optionally through the activation (act = 1: GELU above), is quantized
 * with the NEXT layer's static per-tensor activation scale (Sec. 4.1 "per-tensor static
 * quantization for activations"; Eq. (quantization)):  Y8 = clip(rint(a / s_out), -127, 127).
 * A_f32 (optional) receives a, the value that is quantized.
 */
int oracle_dual_gemm_q8(const int8_t *Xq, const float *s_x, const int8_t *Wq, const float *s_normal,
                        const float *s_outlier, const float *bias, int M, int N, int K, int K_o,
                        int act, float s_out, int8_t *Y8, float *A_f32)
{
    if (!Xq || !s_x || !Wq || !s_normal || !s_outlier || !Y8 || M <= 0 || N <= 0 || K <= 0 || K_o < 0 ||
        K_o > K || (act != 0 && act != 1) || !(s_out > 0.0f))
        return ORACLE_BAD_ARG;
#pragma omp parallel for schedule(static)
    for (int m = 0; m < M; ++m) {
        for (int j = 0; j < N; ++j) {
            const int8_t *x = Xq + (size_t)m * K;
            const int8_t *w = Wq + (size_t)j * K;
            int32_t acc_o = 0, acc_n = 0;
            float b = bias ? bias[j] : 0.0f;
            float r;
            for (int p = 0; p < K_o; ++p)
                acc_o += (int32_t)x[p] * (int32_t)w[p];
            for (int p = K_o; p < K; ++p)
                acc_n += (int32_t)x[p] * (int32_t)w[p];
            r = (float)acc_o * s_outlier[j];
            r = fmaf((float)acc_n, s_normal[j], r);
            r = fmaf(r, s_x[m], b);
            if (act == 1)
                r = oracle_gelu_tanh(r);
            if (A_f32)
                A_f32[(size_t)m * N + j] = r;
            Y8[(size_t)m * N + j] = quantize_sym(r, s_out, 127.0f);
        }
    }
    return ORACLE_OK;
}

/* -------------------- independent single-scale W8A8 linear (invariant pin) */

/*
 * Ordinary per-row single-scale W8A8 linear written on its own (no perm, no
 * blocks): s_w[j] = max_k|W[j,k]|/127, Wq = q(W, s_w), per-token Xq/s_x,
 * acc = sum_k Xq*Wq, r = (float)acc * s_w[j]; r = fmaf(r, s_x[m], b[j]).
 * The dual path must reproduce it bit for bit when no channel is an outlier
 * and when every channel is one.
 */
int oracle_single_scale_linear(const float *X, const float *W, const float *bias, int M, int N,
                               int K, float *Y_f32, uint16_t *Y_bf16, int32_t *acc_out,
                               float *s_w_out, float *s_x_out)
{
    float *s_w, *s_x;
    int8_t *Wq, *Xq;
    if (!X || !W || M <= 0 || N <= 0 || K <= 0)
        return ORACLE_BAD_ARG;
    s_w = (float *)malloc((size_t)N * sizeof(float));
    s_x = (float *)malloc((size_t)M * sizeof(float));
    Wq = (int8_t *)malloc((size_t)N * K);
    Xq = (int8_t *)malloc((size_t)M * K);
    for (int j = 0; j < N; ++j) {
        float a = 0.0f;
        for (int k = 0; k < K; ++k)
            a = fmaxf(a, fabsf(W[(size_t)j * K + k]));
        s_w[j] = a / 127.0f;
        for (int k = 0; k < K; ++k)
            Wq[(size_t)j * K + k] = quantize_one(W[(size_t)j * K + k], s_w[j]);
    }
    for (int m = 0; m < M; ++m) {
        float a = 0.0f;
        for (int k = 0; k < K; ++k)
            a = fmaxf(a, fabsf(X[(size_t)m * K + k]));
        s_x[m] = a / 127.0f;
        for (int k = 0; k < K; ++k)
            Xq[(size_t)m * K + k] = quantize_one(X[(size_t)m * K + k], s_x[m]);
    }
#pragma omp parallel for schedule(static)
    for (int m = 0; m < M; ++m)
        for (int j = 0; j < N; ++j) {
            int32_t acc = 0;
            float r;
            for (int k = 0; k < K; ++k)
                acc += (int32_t)Xq[(size_t)m * K + k] * (int32_t)Wq[(size_t)j * K + k];
            r = (float)acc * s_w[j];
            r = fmaf(r, s_x[m], bias ? bias[j] : 0.0f);
            if (Y_f32)
                Y_f32[(size_t)m * N + j] = r;
            if (Y_bf16)
                Y_bf16[(size_t)m * N + j] = bf16_rne(r);
            if (acc_out)
                acc_out[(size_t)m * N + j] = acc;
        }
    if (s_w_out)
        memcpy(s_w_out, s_w, (size_t)N * sizeof(float));
    if (s_x_out)
        memcpy(s_x_out, s_x, (size_t)M * sizeof(float));
    free(s_w);
    free(s_x);
    free(Wq);
    free(Xq);
    return ORACLE_OK;
}
