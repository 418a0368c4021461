// Dual-scale W8A8 GEMM + de-quantization for gfx950 (appendix "Quantization Kernels", kernel
// (ii); Eq. (dual_scale)): INT8 x INT8 -> INT32 on v_mfma_i32_32x32x32_i8, the outlier and the
// normal K range summed in separate INT32 accumulators and merged by the fp32 epilogue
//     r = (float)acc_o * s_o[n];  r = fmaf((float)acc_n, s_n[n], r);  y = fmaf(r, s_x[m], bias[n]).
//
// Operand geometry.  Both operands are K-contiguous ("NT"): Xq[M, ldxq], Wq[N, ldwq], packed K
// axis [outlier | pad to 32 | normal | pad to 128].  One MFMA consumes a 32-row x 32-byte slab
// of each operand: lane l supplies 16 consecutive K bytes of row (l & 31) starting at byte
// 16*(l >> 5).  A and B use the same lane -> K mapping, so the product is a plain dot product
// over those 32 bytes whatever order the hardware assigns to them.  The 32x32 INT32 result has
// lane l holding column (l & 31) and, in register r, row 8*(r >> 2) + 4*(l >> 5) + (r & 3).
// X rows feed the A operand (result rows = tokens), W rows the B operand (result columns =
// output features).
//
// Because K_o is a multiple of 32 after padding, every 32-byte k-step lies wholly in one of the
// two ranges: steps below the normal offset accumulate into acc_o, the rest into acc_n.
#include "qarvd_common.h"

namespace {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));

constexpr int TPB = 256;   // 4 wavefronts, one per SIMD
constexpr int BK = 128;    // K bytes per LDS stage (4 MFMA k-steps)

struct GemmArgs {
    const int8_t *Xq;
    const int8_t *Wq;
    const float *s_x, *s_n, *s_o, *bias;
    void *Y;
    int32_t *dbg_n, *dbg_o;
    int64_t ldxq, ldwq, ldy;
    int32_t M, N;
    int32_t n_off;     // first byte of the normal block (multiple of 32)
    int32_t kp;        // packed extent (multiple of 128)
    int32_t tiles_m, tiles_n;
};

// LDS image of an operand tile: row r at byte r*128, its eight 16-byte chunks XOR-swizzled by
// swz(r) so that both the row-contiguous stores and the 32-row column reads spread over banks.
__device__ __forceinline__ int swz(int r) { return (r & 7) ^ ((r >> 3) & 1); }

template <typename OutT> __device__ __forceinline__ void store_out(OutT *p, float y);
template <> __device__ __forceinline__ void store_out<float>(float *p, float y) { *p = y; }
template <> __device__ __forceinline__ void store_out<uint16_t>(uint16_t *p, float y) { *p = (uint16_t)f32_to_bf16_bits(y); }

// XCD-aware tile order: consecutive workgroup ids land on different XCDs (round robin over 8),
// so give each XCD a contiguous range of the tile sequence; within the sequence tiles walk down
// a panel of GROUP_M row-tiles before moving to the next column, which keeps an XCD's working set
// of X rows and W rows small enough for its own L2.
__device__ __forceinline__ void tile_coords(int bid, int tiles_m, int tiles_n, int &tm, int &tn)
{
    constexpr int XCD = 8, GROUP_M = 8;
    const int total = tiles_m * tiles_n;
    const int per = total / XCD, rem = total % XCD;
    const int x = bid % XCD, i = bid / XCD;
    // XCD x runs ids x, x+8, ...: per (+1 if x < rem) of them, mapped to one contiguous tile range
    const int t = x * per + min(x, rem) + i;
    const int panel = GROUP_M * tiles_n;
    const int pi = t / panel, within = t % panel;
    const int rows_here = min(GROUP_M, tiles_m - pi * GROUP_M);
    tm = pi * GROUP_M + within % rows_here;
    tn = within / rows_here;
}

template <int BM, int BN, int WM, int WN, bool DUAL, typename OutT>
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
    for (int i = 0; i < BCH; ++i) pb[i] = g.Wq + (size_t)min(n0 + lrow + 32 * i, g.N - 1) * g.ldwq + lcol * 16;
    const int st_off = lrow * BK + ((lcol ^ swz(lrow)) << 4);   // + i*32*BK; swz(lrow + 32 i) == swz(lrow)

    v4i ra[ACH], rb[BCH];
    auto gload = [&](int kt) {
#pragma unroll
        for (int i = 0; i < ACH; ++i) ra[i] = *reinterpret_cast<const v4i *>(pa[i] + (size_t)kt * BK);
#pragma unroll
        for (int i = 0; i < BCH; ++i) rb[i] = *reinterpret_cast<const v4i *>(pb[i] + (size_t)kt * BK);
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
        const float sn = g.s_n[nc], so = g.s_o[nc];
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
                    if (g.dbg_n) g.dbg_n[(size_t)m * g.N + n] = an;
                    if (g.dbg_o) g.dbg_o[(size_t)m * g.N + n] = ao;
                }
            }
        }
    }
}

// ------------------------------------------------------------------------------------------
struct Variant {
    const char *name;
    int BM, BN;
    bool dual;   // has the second accumulator set (can run K_o > 0)
    qarvd_status (*launch)(const GemmArgs &, qarvd_dtype, hipStream_t);
};

template <int BM, int BN, int WM, int WN, bool DUAL>
qarvd_status launch_staged(const GemmArgs &g0, qarvd_dtype ydt, hipStream_t st)
{
    GemmArgs g = g0;
    g.tiles_m = (g.M + BM - 1) / BM;
    g.tiles_n = (g.N + BN - 1) / BN;
    const size_t lds = 2 * (size_t)(BM + BN) * BK + BM * sizeof(float);
    const int grid = g.tiles_m * g.tiles_n;
    if (ydt == QARVD_BF16) {
        auto k = gemm_staged_kernel<BM, BN, WM, WN, DUAL, uint16_t>;
        QARVD_HIP_TRY(hipFuncSetAttribute(reinterpret_cast<const void *>(k), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
        hipLaunchKernelGGL(k, dim3(grid), dim3(TPB), lds, st, g);
    } else {
        auto k = gemm_staged_kernel<BM, BN, WM, WN, DUAL, float>;
        QARVD_HIP_TRY(hipFuncSetAttribute(reinterpret_cast<const void *>(k), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
        hipLaunchKernelGGL(k, dim3(grid), dim3(TPB), lds, st, g);
    }
    return qarvd_launch_status();
}

const Variant kVariants[] = {
    {"staged 256x128 dual", 256, 128, true, launch_staged<256, 128, 2, 2, true>},
    {"staged 128x128 dual", 128, 128, true, launch_staged<128, 128, 2, 2, true>},
    {"staged 256x128 single", 256, 128, false, launch_staged<256, 128, 2, 2, false>},
    {"staged 128x128 single", 128, 128, false, launch_staged<128, 128, 2, 2, false>},
};
constexpr int kNumVariants = sizeof(kVariants) / sizeof(kVariants[0]);

int pick_variant(int M, int N, int K_o)
{
    const long tiles_big = (long)((M + 255) / 256) * ((N + 127) / 128);
    if (K_o > 0) return tiles_big >= 256 ? 1 : 2;
    return tiles_big >= 256 ? 3 : 4;
}

}  // namespace

extern "C" int32_t qarvd_gemm_num_variants(void) { return kNumVariants; }

extern "C" const char *qarvd_gemm_variant_name(int32_t variant)
{
    if (variant < 1 || variant > kNumVariants) return "";
    return kVariants[variant - 1].name;
}

extern "C" qarvd_status qarvd_w8a8_dual_gemm_variant(int32_t variant, const int8_t *Xq, int64_t ldxq,
                                                     const float *s_x, const int8_t *Wq, int64_t ldwq,
                                                     const float *s_normal, const float *s_outlier,
                                                     const float *bias, int32_t M, int32_t N, int32_t K,
                                                     int32_t K_o, void *Y, qarvd_dtype ydt, int64_t ldy,
                                                     int32_t *dbg_acc_normal, int32_t *dbg_acc_outlier,
                                                     void *stream)
{
    if (!Xq || !Wq || !s_x || !s_normal || !s_outlier || !Y) return QARVD_ERR_INVALID_ARG;
    if (M <= 0 || N <= 0 || K <= 0 || K > QARVD_MAX_K || K_o < 0 || K_o > K) return QARVD_ERR_INVALID_ARG;
    if (variant < 0 || variant > kNumVariants) return QARVD_ERR_INVALID_ARG;
    const PackedK pk = qarvd_packed(K, K_o);
    if (ldxq < pk.kp || ldwq < pk.kp || ldy < N) return QARVD_ERR_INVALID_ARG;
    if (ydt != QARVD_F32 && ydt != QARVD_BF16) return QARVD_ERR_UNSUPPORTED;
    if (!qarvd_aligned16(Xq) || !qarvd_aligned16(Wq) || (ldxq % 16) || (ldwq % 16)) return QARVD_ERR_UNSUPPORTED;
    const size_t esz = ydt == QARVD_F32 ? 4 : 2;
    if (reinterpret_cast<uintptr_t>(Y) % esz) return QARVD_ERR_UNSUPPORTED;
    if ((reinterpret_cast<uintptr_t>(s_x) | reinterpret_cast<uintptr_t>(s_normal) | reinterpret_cast<uintptr_t>(s_outlier) |
         reinterpret_cast<uintptr_t>(bias) | reinterpret_cast<uintptr_t>(dbg_acc_normal) |
         reinterpret_cast<uintptr_t>(dbg_acc_outlier)) & 3u)
        return QARVD_ERR_UNSUPPORTED;
    if (variant == 0) variant = pick_variant(M, N, K_o);
    const Variant &v = kVariants[variant - 1];
    if (K_o > 0 && !v.dual) return QARVD_ERR_UNSUPPORTED;
    GemmArgs g;
    g.Xq = Xq; g.Wq = Wq; g.s_x = s_x; g.s_n = s_normal; g.s_o = s_outlier; g.bias = bias;
    g.Y = Y; g.dbg_n = dbg_acc_normal; g.dbg_o = dbg_acc_outlier;
    g.ldxq = ldxq; g.ldwq = ldwq; g.ldy = ldy; g.M = M; g.N = N; g.n_off = pk.n_off; g.kp = pk.kp;
    g.tiles_m = g.tiles_n = 0;
    return v.launch(g, ydt, reinterpret_cast<hipStream_t>(stream));
}

extern "C" qarvd_status qarvd_w8a8_dual_gemm(const int8_t *Xq, int64_t ldxq, const float *s_x,
                                             const int8_t *Wq, int64_t ldwq, const float *s_normal,
                                             const float *s_outlier, const float *bias, int32_t M, int32_t N,
                                             int32_t K, int32_t K_o, void *Y, qarvd_dtype ydt, int64_t ldy,
                                             int32_t *dbg_acc_normal, int32_t *dbg_acc_outlier, void *stream)
{
    return qarvd_w8a8_dual_gemm_variant(0, Xq, ldxq, s_x, Wq, ldwq, s_normal, s_outlier, bias, M, N, K, K_o, Y, ydt,
                                        ldy, dbg_acc_normal, dbg_acc_outlier, stream);
}
