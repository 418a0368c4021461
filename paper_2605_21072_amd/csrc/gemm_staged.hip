// Register-staged variant of the dual-scale W8A8 GEMM: global -> VGPR -> swizzled LDS, two LDS
// stages of 128 K-bytes, both accumulator sets live in registers.  Handles every shape and any
// outlier-block width; the general fallback behind the faster LDS-direct kernels.
// W4: the W operand is packed INT4 (two codes per byte, the nibble order of qarvd_quantize_weight_w4); a thread
// loads 8 bytes where the INT8 build loads 16 and widens them to sixteen INT8 lanes holding 16 * code on the
// way into LDS.  Both sums are then 16 times the INT8 ones and the weight scales are multiplied by 1/16 (exact
// in fp32: a power of two), so every product and fma of the epilogue rounds the same value as the INT8 path.
#include "gemm_common.h"

namespace qarvd_gemm {

template <int BM, int BN, int WM, int WN, bool DUAL, typename OutT, bool W4>
__global__ __launch_bounds__(TPB) void gemm_staged_kernel(GemmArgs g)
{
    static_assert(WM * WN == 4, "four wavefronts");
    constexpr int TM = BM / WM / 32, TN = BN / WN / 32;
    constexpr int ACH = BM * 8 / TPB, BCH = BN * 8 / TPB;   // 16-byte chunks per thread per stage
    constexpr int STAGE = (BM + BN) * BK;
    extern __shared__ __align__(16) unsigned char smem[];
    float *sx_lds = reinterpret_cast<float *>(smem + 2 * STAGE);

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave / WN, wn = wave % WN;
    int tm, tn;
    tile_coords(blockIdx.x, g.tiles_m, g.tiles_n, tm, tn);
    const int m0 = tm * BM, n0 = tn * BN;

    // ---- global -> register -> LDS staging ------------------------------------------------
    // chunk q = tid + 256*i covers row (q >> 3), 16-byte column (q & 7); rows past the matrix edge
    // re-read the last valid row (their results are never stored).
    const int lrow = tid >> 3, lcol = tid & 7;
    const int8_t *pa[ACH];
    const int8_t *pb[BCH];
#pragma unroll
    for (int i = 0; i < ACH; ++i) pa[i] = g.Xq + (size_t)min(m0 + lrow + 32 * i, g.M - 1) * g.ldxq + lcol * 16;
#pragma unroll
    for (int i = 0; i < BCH; ++i) pb[i] = g.Wq + (size_t)min(n0 + lrow + 32 * i, g.N - 1) * g.ldwq + lcol * (W4 ? 8 : 16);
    const int st_off = lrow * BK + ((lcol ^ swz(lrow)) << 4);   // + i*32*BK; swz(lrow + 32 i) == swz(lrow)

    v4i ra[ACH], rb[BCH];
    auto gload = [&](int kt) {
#pragma unroll
        for (int i = 0; i < ACH; ++i) ra[i] = *reinterpret_cast<const v4i *>(pa[i] + (size_t)kt * BK);
#pragma unroll
        for (int i = 0; i < BCH; ++i) {
            if constexpr (W4) {
                const v2i p = *reinterpret_cast<const v2i *>(pb[i] + (size_t)kt * (BK / 2));
                const int m = (int)0xF0F0F0F0u;
                rb[i] = v4i{(p.x << 4) & m, p.x & m, (p.y << 4) & m, p.y & m};
            } else {
                rb[i] = *reinterpret_cast<const v4i *>(pb[i] + (size_t)kt * BK);
            }
        }
    };
    auto sstore = [&](int s) {
        unsigned char *A = smem + s * STAGE, *B = A + BM * BK;
#pragma unroll
        for (int i = 0; i < ACH; ++i) *reinterpret_cast<v4i *>(A + st_off + i * 32 * BK) = ra[i];
#pragma unroll
        for (int i = 0; i < BCH; ++i) *reinterpret_cast<v4i *>(B + st_off + i * 32 * BK) = rb[i];
    };

    // ---- fragment addressing ----------------------------------------------------------------
    const int frow = lane & 31, fhalf = lane >> 5, fsw = swz(frow);
    const int a_base = (wm * (BM / WM) + frow) * BK;
    const int b_base = BM * BK + (wn * (BN / WN) + frow) * BK;

    v16i acc_n[TM][TN];
    v16i acc_o[DUAL ? TM : 1][DUAL ? TN : 1];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc_n[i][j][r] = 0;
    if constexpr (DUAL) {
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j)
#pragma unroll
                for (int r = 0; r < 16; ++r) acc_o[i][j][r] = 0;
    }

    // one 32-byte k-step: TM + TN fragment reads, TM*TN MFMAs into `acc`
    auto kstep = [&](const unsigned char *stage, int ks, v16i (*acc)[TN]) {
        const int coff = (((ks << 1) | fhalf) ^ fsw) << 4;
        v4i a[TM], b[TN];
#pragma unroll
        for (int i = 0; i < TM; ++i) a[i] = *reinterpret_cast<const v4i *>(stage + a_base + i * 32 * BK + coff);
#pragma unroll
        for (int j = 0; j < TN; ++j) b[j] = *reinterpret_cast<const v4i *>(stage + b_base + j * 32 * BK + coff);
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j) acc[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(a[i], b[j], acc[i][j], 0, 0, 0);
    };

    const int nk = g.kp / BK;
    const int o_steps = g.n_off / 32;   // k-steps that belong to the outlier range
    gload(0);
    // per-token scales of this tile's rows
    for (int i = tid; i < BM; i += TPB) sx_lds[i] = g.s_x[min(m0 + i, g.M - 1)];
    sstore(0);
    __syncthreads();
    for (int kt = 0; kt < nk; ++kt) {
        const unsigned char *stage = smem + (kt & 1) * STAGE;
        if (kt + 1 < nk) gload(kt + 1);
        bool done = false;
        if constexpr (DUAL) {
            if ((kt + 1) * 4 <= o_steps) {
#pragma unroll
                for (int ks = 0; ks < 4; ++ks) kstep(stage, ks, acc_o);
                done = true;
            } else if (kt * 4 < o_steps) {
                const int split = o_steps - kt * 4;   // 1..3 leading steps are outlier steps
#pragma unroll
                for (int ks = 0; ks < 4; ++ks) {
                    if (ks < split) kstep(stage, ks, acc_o);
                    else kstep(stage, ks, acc_n);
                }
                done = true;
            }
        }
        if (!done) {
#pragma unroll
            for (int ks = 0; ks < 4; ++ks) kstep(stage, ks, acc_n);
        }
        if (kt + 1 < nk) sstore((kt + 1) & 1);
        __syncthreads();
    }

    // ---- epilogue ---------------------------------------------------------------------------
    OutT *Y = reinterpret_cast<OutT *>(g.Y);
#pragma unroll
    for (int j = 0; j < TN; ++j) {
        const int n = n0 + wn * (BN / WN) + j * 32 + frow;
        const int nc = min(n, g.N - 1);
        const float wsc = W4 ? 0.0625f : 1.0f;
        const float sn = g.s_n[nc] * wsc, so = g.s_o[nc] * wsc;
        const float bs = g.bias ? g.bias[nc] : 0.0f;
#pragma unroll
        for (int i = 0; i < TM; ++i) {
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int ml = wm * (BM / WM) + i * 32 + 8 * (r >> 2) + 4 * fhalf + (r & 3);
                const int m = m0 + ml;
                const int an = acc_n[i][j][r];
                int ao = 0;
                if constexpr (DUAL) ao = acc_o[i][j][r];
                float v = (float)ao * so;
                v = fmaf((float)an, sn, v);
                v = fmaf(v, sx_lds[ml], bs);
                if (m < g.M && n < g.N) {
                    store_out<OutT>(Y + (size_t)m * g.ldy + n, v);
                    if (g.dbg_n) g.dbg_n[(size_t)m * g.N + n] = an >> (W4 ? 4 : 0);     // exact multiples of 16
                    if (g.dbg_o) g.dbg_o[(size_t)m * g.N + n] = ao >> (W4 ? 4 : 0);
                }
            }
        }
    }
}

template <int BM, int BN, int WM, int WN, bool DUAL, bool W4>
qarvd_status launch_staged(const GemmArgs &g0, qarvd_dtype ydt, hipStream_t st)
{
    GemmArgs g = g0;
    g.tiles_m = (g.M + BM - 1) / BM;
    g.tiles_n = (g.N + BN - 1) / BN;
    const size_t lds = 2 * (size_t)(BM + BN) * BK + BM * sizeof(float);
    const int grid = g.tiles_m * g.tiles_n;
    if (ydt == QARVD_BF16) {
        auto k = gemm_staged_kernel<BM, BN, WM, WN, DUAL, uint16_t, W4>;
        static unsigned long long raised = 0;
        if (qarvd_status s_a = qarvd_raise_lds_limit_once(k, (int)lds, raised); s_a != QARVD_OK) return s_a;
        hipLaunchKernelGGL(k, dim3(grid), dim3(TPB), lds, st, g);
    } else {
        auto k = gemm_staged_kernel<BM, BN, WM, WN, DUAL, float, W4>;
        static unsigned long long raised = 0;
        if (qarvd_status s_a = qarvd_raise_lds_limit_once(k, (int)lds, raised); s_a != QARVD_OK) return s_a;
        hipLaunchKernelGGL(k, dim3(grid), dim3(TPB), lds, st, g);
    }
    return qarvd_launch_status();
}


template qarvd_status launch_staged<256, 128, 2, 2, true, false>(const GemmArgs &, qarvd_dtype, hipStream_t);
template qarvd_status launch_staged<128, 128, 2, 2, true, false>(const GemmArgs &, qarvd_dtype, hipStream_t);
template qarvd_status launch_staged<256, 128, 2, 2, false, false>(const GemmArgs &, qarvd_dtype, hipStream_t);
template qarvd_status launch_staged<128, 128, 2, 2, false, false>(const GemmArgs &, qarvd_dtype, hipStream_t);
template qarvd_status launch_staged<128, 128, 2, 2, true, true>(const GemmArgs &, qarvd_dtype, hipStream_t);
template qarvd_status launch_staged<128, 128, 2, 2, false, true>(const GemmArgs &, qarvd_dtype, hipStream_t);

}  // namespace qarvd_gemm
