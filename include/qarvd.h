/*
 * qarvd.h - C ABI of the MI355X (gfx950) dual-scale W8A8 linear layer of Q-ARVD.
 *
 * Three operations, split as the paper's deployment splits them (appendix
 * "Quantization Kernels and Extra Cost Analysis": the outlier/normal channel split is
 * done offline, an activation-quantization kernel and an INT8-GEMM-plus-dequantization
 * kernel run online):
 *
 *   qarvd_quantize_weight   offline: outlier detection, channel permutation, dual scales, INT8 weights
 *   qarvd_quant_act         online:  gather-permute + per-token dynamic symmetric INT8
 *   qarvd_w8a8_dual_gemm    online:  INT8xINT8->INT32 on MFMA, two accumulators, fp32 dequant + bias
 *
 * Conventions
 *   - Every pointer is DEVICE memory unless its comment says "host".  The caller owns every
 *     buffer; the library allocates nothing.  The only state it keeps between calls is what it
 *     has learnt about a device (its compute-unit count, which kernels already had their LDS
 *     limit raised) and, for qarvd_quantize_weight_static alone, one fixed device array.
 *   - `stream` is a hipStream_t passed as void* (NULL = the null stream).
 *   - W is fp32 [N,K] row-major: N = d_out rows, K = d_in input channels.  X is [M,K] row-major
 *     (tokens x channels).  Y is [M,N] row-major.  Leading dimensions are in ELEMENTS.
 *   - Functions return a qarvd_status and never abort or throw.  Arguments are validated on
 *     the host before anything is launched: with INVALID_ARG, UNSUPPORTED or WORKSPACE nothing
 *     has been written.  QARVD_ERR_HIP reports a failed HIP call or launch and can come after
 *     earlier kernels of the same call have run; the outputs are then unspecified.
 *
 * Packed K axis (the layout both INT8 operands share)
 *   Position p of a packed row holds input channel perm[p].  With K_o outlier channels:
 *
 *       [ outlier block: K_o bytes | zeros up to a multiple of 32 | normal block: K-K_o bytes | zeros ]
 *         ^0                                                       ^qarvd_packed_normal_offset(K_o)
 *
 *   and the whole row extent qarvd_packed_k(K, K_o) is a multiple of 128.  Both producers write
 *   the zero padding themselves; zeros add nothing to either INT32 sum.  A row stride (ldxq,
 *   ldwq) may be any multiple of 16 that is >= qarvd_packed_k(K, K_o); bytes past the packed
 *   extent are neither read nor written.  When K is a multiple of 128 and K_o a multiple of 32
 *   (every layer of the DiT workloads) there is no padding at all.
 */
#ifndef QARVD_H
#define QARVD_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    QARVD_OK = 0,
    QARVD_ERR_INVALID_ARG = -1, /* null pointer, non-positive size, K_o outside [0,K], ld too small ... */
    QARVD_ERR_UNSUPPORTED = -2, /* misaligned pointer / stride, unknown dtype, size beyond a kernel limit */
    QARVD_ERR_WORKSPACE = -3,   /* workspace missing or smaller than the query says */
    QARVD_ERR_HIP = -4          /* a HIP call or launch failed */
} qarvd_status;

typedef enum { QARVD_F32 = 0, QARVD_BF16 = 1 } qarvd_dtype;

/* K above this would let an INT32 accumulator overflow (K * 127^2 must stay below 2^31). */
#define QARVD_MAX_K 133143

/*
 * Detector parameters (Sec. 3.2, Eq. (new_threshold): tau = 3.5, alpha = 1.2; Fig. "outlier
 * patterns" caption: the outlier count is aligned to a multiple of 32).
 *   clip_search  0: each scale is the block's absmax / qmax (Eq. (quantization)).  1: percentile-clip
 *                initialisation (Sec. 4.1, quantization implementation: the scale is initialised at the
 *                best of the clipping percentiles 0.999, 0.9999 and 0.99999), data-free, per output row and block: the
 *                linear-interpolated p-quantile of |w| (h = (n-1) p, in double, rounded to float) over
 *                qmax is a candidate scale; the one with the smallest squared quantization error
 *                sum (fmaf(-s, q, w))^2 (summed in double in packed order) wins, the larger percentile
 *                on a tie.  Needs K <= 16384.
 *   forced_mask  HOST pointer to K bytes (0/1) or NULL.  Non-NULL: the outlier set is exactly
 *                the mask; detection and alignment are skipped (used for the all-outlier and
 *                arbitrary-split checks).
 */
typedef struct {
    double tau;
    double alpha;
    int32_t align;
    int32_t clip_search;
    const uint8_t *forced_mask;
} qarvd_detect_cfg;

/* Fills *cfg with the paper's defaults {3.5, 1.2, 32, 0, NULL}. */
void qarvd_default_detect_cfg(qarvd_detect_cfg *cfg);

/* Human-readable name of a status code (static storage). */
const char *qarvd_status_string(qarvd_status s);

/* Offset of the normal block inside a packed row: K_o rounded up to a multiple of 32. */
int32_t qarvd_packed_normal_offset(int32_t K_o);

/*
 * Extent in bytes of a packed row, a multiple of 128.  K_o < 0 returns the largest extent any
 * K_o in [0,K] can need, for allocating before the split is known.  Returns 0 on bad arguments.
 */
int32_t qarvd_packed_k(int32_t K, int32_t K_o);

/*
 * Recommended row stride in bytes for the packed INT8 operands (ldxq, ldwq) of a K-channel layer: the
 * packed extent qarvd_packed_k(K, K_o) plus 128 (plus 256 where that would be a multiple of 512).  Every
 * multiple of 16 that is >= the packed extent is
 * accepted; this one keeps all rows 128-byte aligned (a 64-byte stage segment never straddles a cache
 * line) and is never a multiple of 512, so the rows of an operand tile spread over the memory channels
 * (measured on MI355X: GEMMs run 4-16 % slower at row strides of 1536, 5120 or 13824 bytes).  The
 * bytes between the packed extent and the stride are neither read nor written.  Returns 0 on bad arguments.
 */
int32_t qarvd_packed_ld(int32_t K, int32_t K_o);

/* Bytes of device workspace qarvd_quantize_weight needs for an [N,K] layer. */
size_t qarvd_quantize_weight_workspace(int32_t N, int32_t K);

/*
 * OFFLINE weight step (Sec. 3.2; Sec. 2.2 Eq. (quantization); Sec. 4.1 per-channel weights).
 *   1. v[k] = (float) sqrt( sum_j (double)W[j,k]^2 ), rows added in ascending j      (L2 norm vector v)
 *   2. med = median(v), MAD = median(|v - med|)  (even K: mean of the two middle values) Eq. (mad)
 *   3. channel k is flagged iff v[k] > max(med + tau/0.6745*MAD, alpha*med), in fp64     Eq. (new_threshold)
 *   4. no flagged channel: K_o = 0 and the layer stays single-scale.  Otherwise K_o is the
 *      flagged count rounded UP to a multiple of `align` (capped at K); the added channels are
 *      the unflagged ones with the largest norm (ties: smaller index)                    Fig. caption
 *   5. perm = [outlier channels ascending | normal channels ascending]                   Eq. (dual_scale)
 *   6. per output row j and per block: s = max|W[j, block]| / 127 (fp32 division),
 *      Wq = clip(rint(W / s), -127, 127) (round-half-even), s == 0 -> 0                  Eq. (quantization)
 *
 *   W          in   f32 [N, ldw]
 *   cfg        in   host; NULL = defaults
 *   Wq         out  i8  [N, ldwq] packed (see above); ldwq a multiple of 16 and >= qarvd_packed_k(K, -1)
 *                   (K rounded up to 128 is enough when the outlier block cannot need padding: cfg->align a
 *                   multiple of 32 and no forced_mask)
 *   s_normal   out  f32 [N]     s_outlier  out f32 [N]  (0 for an empty block)
 *   perm       out  i32 [K]     gather index: packed position p reads channel perm[p]
 *   K_o_host   out  HOST int32
 *   v_out      out  f32 [K] or NULL (the norm vector)
 *   workspace       device, >= qarvd_quantize_weight_workspace(N, K) bytes, 256-byte aligned
 * Synchronises `stream` before returning (K_o is read back).
 */
qarvd_status qarvd_quantize_weight(const float *W, int32_t N, int32_t K, int64_t ldw,
                                   const qarvd_detect_cfg *cfg, int8_t *Wq, int64_t ldwq,
                                   float *s_normal, float *s_outlier, int32_t *perm,
                                   int32_t *K_o_host, float *v_out, void *workspace,
                                   size_t workspace_bytes, void *stream);

/*
 * qarvd_quantize_weight for callers that cannot allocate device memory or hand over a workspace:
 * code under HIP graph capture set-up, tight serving loops, harnesses that forbid hipMalloc.  Same
 * arguments minus the workspace, same results bit for bit.  The detector's workspace lives in a fixed
 * device array inside the library (528 KB on every GPU the library is used on, held until the
 * process ends), which limits K to qarvd_quantize_weight_static_max_k() = 16384: a larger K returns
 * QARVD_ERR_WORKSPACE before anything is launched.  The call allocates nothing (no hipMalloc/hipFree,
 * no allocating library routine).  All calls on one GPU share that array: two calls that overlap on
 * the same GPU (different streams or threads) race and give undefined results; calls on one stream,
 * or separated by a synchronisation, are safe, and nothing of an earlier call is ever read.
 * Synchronises `stream` before returning, like qarvd_quantize_weight.
 */
int32_t qarvd_quantize_weight_static_max_k(void);
qarvd_status qarvd_quantize_weight_static(const float *W, int32_t N, int32_t K, int64_t ldw,
                                          const qarvd_detect_cfg *cfg, int8_t *Wq, int64_t ldwq,
                                          float *s_normal, float *s_outlier, int32_t *perm,
                                          int32_t *K_o_host, float *v_out, void *stream);

/*
 * ONLINE activation quantization (appendix, kernel (i) plus the online permutation; Sec. 2.2
 * Eq. (quantization) with per-token dynamic symmetric scale):
 *     a_m = max_k |X[m,k]| over all K channels;  s_x[m] = a_m / 127 (fp32 division)
 *     Xq[m, pos(p)] = clip(rint(X[m, perm[p]] / s_x[m]), -127, 127);  s_x[m] == 0 -> 0
 *   X     in   [M, ldx] of `xdt` (QARVD_F32 or QARVD_BF16; bf16 is widened exactly first)
 *   perm  in   i32 [K] or NULL (identity; K_o must then be 0)
 *   Xq    out  i8 [M, ldxq] packed for (K, K_o);  s_x out f32 [M]
 * Fully asynchronous on `stream`.  The register-resident kernels need K % 4 == 0, ldx % 4 == 0, a
 * 16-byte (fp32) / 8-byte (bf16) aligned X and K <= 16384; anything else runs a slower general kernel.
 */
qarvd_status qarvd_quant_act(const void *X, qarvd_dtype xdt, int32_t M, int32_t K, int64_t ldx,
                             const int32_t *perm, int32_t K_o, int8_t *Xq, int64_t ldxq,
                             float *s_x, void *stream);

/*
 * Static-scale variant (Sec. 4.1 "per-tensor static quantization for activations"): the scale
 * is an input, there is no absmax pass, and the clip to [-127,127] can fire.
 */
qarvd_status qarvd_quant_act_static(const void *X, qarvd_dtype xdt, int32_t M, int32_t K,
                                    int64_t ldx, const int32_t *perm, int32_t K_o, float scale,
                                    int8_t *Xq, int64_t ldxq, void *stream);

/*
 * ONLINE GEMM + de-quantization (appendix, kernel (ii); Eq. (dual_scale)):
 *     acc_o[m,j] = sum over the outlier block of Xq[m,p]*Wq[j,p]     (INT32, exact)
 *     acc_n[m,j] = sum over the normal  block of Xq[m,p]*Wq[j,p]
 *     r = (float)acc_o * s_outlier[j];  r = fmaf((float)acc_n, s_normal[j], r);
 *     Y[m,j] = fmaf(r, s_x[m], bias[j])   stored as fp32, or rounded to bf16 (nearest-even)
 *   Xq, Wq  in  packed i8 for the same (K, K_o); 16-byte aligned, strides multiples of 16
 *   s_x     in  f32 [M];  s_normal, s_outlier in f32 [N];  bias in f32 [N] or NULL (+0.0f)
 *   Y       out [M, ldy] of `ydt`; 16-byte aligned, ldy*sizeof(elem) % 16 == 0
 *   dbg_acc_normal, dbg_acc_outlier   out i32 [M,N] (dense, ld = N) or NULL: raw accumulators
 *                                     for parity checks; pass NULL when timing.
 * Fully asynchronous on `stream`.
 */
qarvd_status qarvd_w8a8_dual_gemm(const int8_t *Xq, int64_t ldxq, const float *s_x,
                                  const int8_t *Wq, int64_t ldwq, const float *s_normal,
                                  const float *s_outlier, const float *bias, int32_t M, int32_t N,
                                  int32_t K, int32_t K_o, void *Y, qarvd_dtype ydt, int64_t ldy,
                                  int32_t *dbg_acc_normal, int32_t *dbg_acc_outlier, void *stream);

/*
 * W4A8 (Sec. 4.2, the W4A8 rows of the result tables; Sec. 4.3: the dual scale matters most at low
 * weight bit-width).  Same steps as qarvd_quantize_weight with Eq. (quantization) at b = 4:
 *     s = max|W[j, block]| / 7,  code = clip(rint(W / s), -7, 7)
 * and the codes stored two per byte.  Packed INT4 row: the packed K axis of the INT8 layout, each
 * aligned group of 16 positions 16g..16g+15 in 8 bytes at byte offset 8g: byte i (i < 4) holds
 * position 16g+i in its low nibble and 16g+4+i in its high nibble, byte 4+i positions 16g+8+i and
 * 16g+12+i (two's-complement nibbles).  Row extent qarvd_packed_k(K, K_o) / 2 bytes.
 *   Wq4   out  u8 [N, ldwq4]; ldwq4 in BYTES, >= qarvd_packed_k(K, -1) / 2, multiple of 16
 *   workspace  >= qarvd_quantize_weight_w4_workspace(N, K) bytes (it also holds one byte per code
 *              of the whole matrix until they are packed), 256-byte aligned
 * Everything else as qarvd_quantize_weight.  Synchronises `stream`.
 */
size_t qarvd_quantize_weight_w4_workspace(int32_t N, int32_t K);
qarvd_status qarvd_quantize_weight_w4(const float *W, int32_t N, int32_t K, int64_t ldw,
                                      const qarvd_detect_cfg *cfg, uint8_t *Wq4, int64_t ldwq4,
                                      float *s_normal, float *s_outlier, int32_t *perm,
                                      int32_t *K_o_host, float *v_out, void *workspace,
                                      size_t workspace_bytes, void *stream);

/*
 * ONLINE GEMM + de-quantization on packed INT4 weights: the operation of qarvd_w8a8_dual_gemm with
 * Wq given in the layout above.  The nibbles are widened to INT8 in registers (each code times 16,
 * which the scales undo exactly), so both INT32 sums and every output are those of the INT8 path on
 * the same codes.
 *   Wq4  in  packed u8 [N, ldwq4] for the same (K, K_o) as Xq; 16-byte aligned, ldwq4 % 16 == 0
 * Shapes outside the fast-path preconditions (N % 8 != 0, Y rows, scales or bias not 16-byte aligned,
 * an outlier block of more than 128 packed bytes) run on a slower register-staged kernel (the last
 * variant); asking for one of the fast variants by number on such a shape returns
 * QARVD_ERR_UNSUPPORTED.  variant: 0 = heuristic, 1..qarvd_w4_gemm_num_variants() pick a kernel.
 * Fully asynchronous on `stream`.
 */
qarvd_status qarvd_w4a8_dual_gemm(const int8_t *Xq, int64_t ldxq, const float *s_x,
                                  const uint8_t *Wq4, int64_t ldwq4, const float *s_normal,
                                  const float *s_outlier, const float *bias, int32_t M, int32_t N,
                                  int32_t K, int32_t K_o, void *Y, qarvd_dtype ydt, int64_t ldy,
                                  int32_t *dbg_acc_normal, int32_t *dbg_acc_outlier, int32_t variant,
                                  void *stream);
int32_t qarvd_w4_gemm_num_variants(void);

/*
 * ONLINE GEMM + de-quantization for CHAINED layers (Sec. 4.1: activations are quantized per tensor
 * with static, calibrated scales, so a layer can hand the next one INT8 codes directly; Eq.
 * (quantization) applied to this layer's output with the next layer's scale):
 *     y      = the fp32 result of qarvd_w8a8_dual_gemm (same epilogue arithmetic, bias included)
 *     a      = y                          act = QARVD_ACT_NONE
 *            = gelu_tanh(y)               act = QARVD_ACT_GELU_TANH:
 *              0.5 y (1 + tanh(sqrt(2/pi) (y + 0.044715 y^3)))
 *     Y8[m,n] = clip(rint(a / out_scale), -127, 127), round-half-even
 * Without an activation the quotient is the IEEE fp32 quotient and Y8 is exactly that code.  With GELU
 * the quotient is evaluated in fp32 as y / (s + s 2^t), t = -2 log2(e) sqrt(2/pi) (y + 0.044715 y^3)
 * (one hardware 2^t and one hardware reciprocal per value), which lies within
 * (4e-7 + 2e-6 |gelu(y)|) / out_scale of the real-valued quotient: Y8 is the code of the exact
 * activation except where that quotient is this close to a rounding boundary k + 1/2, where it may be
 * the neighbouring code.  Results are deterministic (the same inputs give the same bytes).
 * Column n of Y8 is output row n of Wq: to feed the next layer without a separate pass, give THIS
 * layer's weight rows (and bias) in the next layer's packed channel order, zero rows at its pad
 * positions, so that N = qarvd_packed_k(K_next, K_o_next) and Y8 is that layer's Xq with
 * s_x[m] = out_scale for every m.
 *   Y8     out  device i8 [M, ldy8]; ldy8 >= N; columns >= N are not written
 *   act, out_scale   out_scale in [1e-30, 1e30], else QARVD_ERR_INVALID_ARG
 * Needs N % 16 == 0, Y8 16-byte aligned, ldy8 % 16 == 0, 16-byte aligned scales and bias and an
 * outlier block of at most 128 packed bytes; otherwise QARVD_ERR_UNSUPPORTED.  Other arguments as
 * qarvd_w8a8_dual_gemm.  variant: 0 = heuristic, 1..qarvd_q8_gemm_num_variants() pick a kernel.
 * Fully asynchronous on `stream`.
 */
typedef enum { QARVD_ACT_NONE = 0, QARVD_ACT_GELU_TANH = 1 } qarvd_act;
qarvd_status qarvd_w8a8_dual_gemm_q8(const int8_t *Xq, int64_t ldxq, const float *s_x,
                                     const int8_t *Wq, int64_t ldwq, const float *s_normal,
                                     const float *s_outlier, const float *bias, int32_t M, int32_t N,
                                     int32_t K, int32_t K_o, qarvd_act act, float out_scale,
                                     int8_t *Y8, int64_t ldy8, int32_t variant, void *stream);
int32_t qarvd_q8_gemm_num_variants(void);

/*
 * Same operation with the kernel variant chosen by the caller instead of the built-in
 * heuristic (variant 0 = heuristic).  qarvd_gemm_num_variants() is the count of selectable
 * variants (1..count); qarvd_gemm_variant_name(i) describes one.  A variant that cannot run
 * the given shape returns QARVD_ERR_UNSUPPORTED.  Used by the parity tests and the tuner.
 */
qarvd_status qarvd_w8a8_dual_gemm_variant(int32_t variant, const int8_t *Xq, int64_t ldxq,
                                          const float *s_x, const int8_t *Wq, int64_t ldwq,
                                          const float *s_normal, const float *s_outlier,
                                          const float *bias, int32_t M, int32_t N, int32_t K,
                                          int32_t K_o, void *Y, qarvd_dtype ydt, int64_t ldy,
                                          int32_t *dbg_acc_normal, int32_t *dbg_acc_outlier,
                                          void *stream);
int32_t qarvd_gemm_num_variants(void);
const char *qarvd_gemm_variant_name(int32_t variant);

/*
 * Diagnostic for reports (not part of the layer): the measured issue-bound INT8 MFMA rate of the
 * current device, in TOPS.  Runs a register-resident loop of `iters` x 8 v_mfma_i32_32x32x32_i8
 * per wavefront on every CU (two wavefronts per SIMD) and times it with HIP events on `stream`.
 *   workspace  device, >= 4160 bytes, 4-byte aligned (operand seeds)
 *   tops_host  HOST out
 * Synchronises `stream`.  The result is below the datasheet figure when the MFMA clock is
 * power-limited; benchmark reports quote the GEMM against both.
 */
qarvd_status qarvd_probe_mfma_peak(int32_t iters, void *workspace, size_t workspace_bytes,
                                   double *tops_host, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* QARVD_H */
