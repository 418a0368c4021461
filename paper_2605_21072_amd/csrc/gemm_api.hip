// C entry points of the dual-scale W8A8 GEMM: argument validation, variant table and heuristic.
#include "gemm_common.h"

using namespace qarvd_gemm;

namespace {

const Variant kVariants[] = {
    // name, BM, BN, widest outlier block (packed bytes), needs vector output, launcher
    {"staged 256x128 dual", 256, 128, 1 << 30, false, launch_staged<256, 128, 2, 2, true>},
    {"staged 128x128 dual", 128, 128, 1 << 30, false, launch_staged<128, 128, 2, 2, true>},
    {"staged 256x128 single", 256, 128, 0, false, launch_staged<256, 128, 2, 2, false>},
    {"staged 128x128 single", 128, 128, 0, false, launch_staged<128, 128, 2, 2, false>},
    {"lds-direct 256x128 (4 waves, 3 stages) dual", 256, 128, 128, true, launch_dma<256, 128, 2, 2, 3, true>},
    {"lds-direct 256x128 (4 waves, 3 stages) single", 256, 128, 0, true, launch_dma<256, 128, 2, 2, 3, false>},
    {"lds-direct 192x128 (4 waves, 3 stages) dual", 192, 128, 128, true, launch_dma<192, 128, 2, 2, 3, true>},
    {"lds-direct 192x128 (4 waves, 3 stages) single", 192, 128, 0, true, launch_dma<192, 128, 2, 2, 3, false>},
    {"lds-direct 128x128 (4 waves, 4 stages) dual", 128, 128, 128, true, launch_dma<128, 128, 2, 2, 4, true>},
    {"lds-direct 128x128 (4 waves, 4 stages) single", 128, 128, 0, true, launch_dma<128, 128, 2, 2, 4, false>},
    {"lds-direct 256x256 (8 waves, 4 stages) dual", 256, 256, 128, true, launch_dma<256, 256, 2, 4, 4, true>},
    {"lds-direct 256x256 (8 waves, 4 stages) single", 256, 256, 0, true, launch_dma<256, 256, 2, 4, 4, false>},
    {"lds-direct 256x128 (8 waves, 4 stages) dual", 256, 128, 128, true, launch_dma<256, 128, 4, 2, 4, true>},
    {"lds-direct 256x128 (8 waves, 4 stages) single", 256, 128, 0, true, launch_dma<256, 128, 4, 2, 4, false>},
    {"lds-direct 128x256 (8 waves, 4 stages) dual", 128, 256, 128, true, launch_dma<128, 256, 2, 4, 4, true>},
    {"lds-direct 128x256 (8 waves, 4 stages) single", 128, 256, 0, true, launch_dma<128, 256, 2, 4, 4, false>},
    {"16x16x64 256x224 (8 waves, 4 stages) dual", 256, 224, 128, true, launch_mfma16<256, 224, 4, 2, 4, true>},
    {"16x16x64 256x224 (8 waves, 4 stages) single", 256, 224, 0, true, launch_mfma16<256, 224, 4, 2, 4, false>},
    {"lds-direct 64x128 (4 waves, 5 stages) dual", 64, 128, 128, true, launch_dma<64, 128, 2, 2, 5, true>},
    {"lds-direct 64x128 (4 waves, 5 stages) single", 64, 128, 0, true, launch_dma<64, 128, 2, 2, 5, false>},
    {"lds-direct 64x64 (4 waves, 6 stages) dual", 64, 64, 128, true, launch_dma<64, 64, 2, 2, 6, true>},
    {"lds-direct 64x64 (4 waves, 6 stages) single", 64, 64, 0, true, launch_dma<64, 64, 2, 2, 6, false>},
    {"lds-direct 256x128 (8 waves, 6 stages) dual", 256, 128, 128, true, launch_dma<256, 128, 4, 2, 6, true>},
    {"lds-direct 256x128 (8 waves, 6 stages) single", 256, 128, 0, true, launch_dma<256, 128, 4, 2, 6, false>},
    {"lds-direct 256x128 (8 waves, 5 stages) dual", 256, 128, 128, true, launch_dma<256, 128, 4, 2, 5, true>},
    {"lds-direct 256x128 (8 waves, 5 stages) single", 256, 128, 0, true, launch_dma<256, 128, 4, 2, 5, false>},
    {"128-byte stages 256x256 (8 waves, 2 stages) dual", 256, 256, 128, true, launch_dma128<256, 256, 2, 4, 2, true>},
    {"128-byte stages 256x256 (8 waves, 2 stages) single", 256, 256, 0, true, launch_dma128<256, 256, 2, 4, 2, false>},
    {"128-byte stages 256x128 (8 waves, 3 stages) dual", 256, 128, 128, true, launch_dma128<256, 128, 4, 2, 3, true>},
    {"128-byte stages 256x128 (8 waves, 3 stages) single", 256, 128, 0, true, launch_dma128<256, 128, 4, 2, 3, false>},
    {"128-byte stages 128x256 (8 waves, 3 stages) dual", 128, 256, 128, true, launch_dma128<128, 256, 2, 4, 3, true>},
    {"128-byte stages 128x256 (8 waves, 3 stages) single", 128, 256, 0, true, launch_dma128<128, 256, 2, 4, 3, false>},
};
constexpr int kNumVariants = sizeof(kVariants) / sizeof(kVariants[0]);

bool vector_out_ok(const GemmArgs &g, qarvd_dtype ydt)
{
    const size_t esz = ydt == QARVD_F32 ? 4 : 2;
    // the LDS-direct kernels also address a tile's rows with 32-bit byte offsets: 256 rows x stride x 4 < 2^31
    return (g.N % 8) == 0 && qarvd_aligned16(g.Y) && ((g.ldy * esz) % 16) == 0 && qarvd_aligned16(g.s_n) &&
           qarvd_aligned16(g.s_o) && qarvd_aligned16(g.bias) && g.ldxq <= (1 << 22) && g.ldwq <= (1 << 22) && g.ldy <= (1 << 20);
}

bool variant_fits(const Variant &v, const GemmArgs &g, qarvd_dtype ydt)
{
    if (g.n_off > v.max_n_off) return false;
    if (v.needs_vector_out && !vector_out_ok(g, ydt)) return false;
    return true;
}

// Heuristic: a three-constant cost model per candidate, fitted to back-to-back timings on MI355X over the
// DiT shapes (M = 256..4680, N and K in {1536, 4608, 5120, 8960, 13824}, operands at the padded strides of
// qarvd_packed_ld):
//     time ~ c + ceil(tiles / CUs) * (a + b * T),     T = packed K / 64          (constants in microseconds)
// c is launch plus the first tile's lead-in, a a tile's epilogue and hand-over, b one 64-byte K step of a tile
// that has its CU to itself (two four-wave workgroups sharing a CU each run at half speed, which the ceil over
// the CUs already accounts for).  The three eight-wave tiles run on 128-byte-deep stages (gemm_dma128.hip):
// 256x256 has the cheapest K step per MAC and wins when N is wide; the half tiles fill the chip when N = 1536
// (4680 x 8960 -> 1536: 61 us against 81 us for 256x256) and on M of a few hundred rows with N = 8960.  The
// four-wave tiles on 64-byte stages serve short M: 128x128 for M around 1500, 64x128 / 64x64 when even those
// would leave most CUs without a tile (M = 520, N = 1536, K = 8960: 24 us instead of 45 us).
int device_cus()
{
    int cus = 0;
    return (qarvd_current_device(nullptr, &cus) == QARVD_OK && cus > 0) ? cus : 256;
}

int pick_variant(const GemmArgs &g, qarvd_dtype ydt)
{
    const bool dual = g.n_off > 0;
    const int cus = device_cus();      // rounds are counted over the CUs of the device the call runs on
    if (g.n_off <= 128 && vector_out_ok(g, ydt)) {
        struct Cand { int variant, bm, bn; double c, a, b; };
        const Cand cand[6] = {{dual ? 27 : 28, 256, 256, 7.2, 9.2, 0.443},
                              {dual ? 29 : 30, 256, 128, 4.5, 3.6, 0.379},
                              {dual ? 31 : 32, 128, 256, 3.9, 3.9, 0.381},
                              {dual ? 9 : 10, 128, 128, 2.0, 1.5, 0.309},
                              {dual ? 19 : 20, 64, 128, 2.0, 0.8, 0.187},
                              {dual ? 21 : 22, 64, 64, 2.0, 0.77, 0.152}};
        const double T = g.kp / 64;
        int best = cand[0].variant;
        double best_cost = 1e300;
        const long tiles128 = (long)((g.M + 127) / 128) * ((g.N + 127) / 128);
        for (const Cand &c : cand) {
            if (c.bm == 64 && tiles128 > cus) continue;     // the small tiles only pay while 128x128 tiles leave CUs empty
            const long tiles = (long)((g.M + c.bm - 1) / c.bm) * ((g.N + c.bn - 1) / c.bn);
            const double cost = c.c + (double)((tiles + cus - 1) / cus) * (c.a + c.b * T);
            if (cost < best_cost) {
                best_cost = cost;
                best = c.variant;
            }
        }
        return best;
    }
    const long tiles_big = (long)((g.M + 255) / 256) * ((g.N + 127) / 128);
    if (dual) return tiles_big >= cus ? 1 : 2;
    return tiles_big >= cus ? 3 : 4;
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
    GemmArgs g;
    g.Xq = Xq; g.Wq = Wq; g.s_x = s_x; g.s_n = s_normal; g.s_o = s_outlier; g.bias = bias;
    g.Y = Y; g.dbg_n = dbg_acc_normal; g.dbg_o = dbg_acc_outlier;
    g.ldxq = ldxq; g.ldwq = ldwq; g.ldy = ldy; g.M = M; g.N = N; g.n_off = pk.n_off; g.kp = pk.kp;
    g.tiles_m = g.tiles_n = 0; g.act = 0; g.out_scale = 0.0f; g.store_wt = 0;
    if (variant == 0) variant = pick_variant(g, ydt);
    const Variant &v = kVariants[variant - 1];
    if (!variant_fits(v, g, ydt)) return QARVD_ERR_UNSUPPORTED;
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

// ---- W4A8: packed INT4 weights, the same kernels with the W operand widened in registers ----
namespace {
using namespace qarvd_gemm;
struct W4Variant {
    int BM, BN;
    qarvd_status (*dual)(const GemmArgs &, qarvd_dtype, hipStream_t);
    qarvd_status (*single)(const GemmArgs &, qarvd_dtype, hipStream_t);
};
const W4Variant kW4Variants[] = {
    {256, 256, launch_dma<256, 256, 2, 4, 4, true, true>, launch_dma<256, 256, 2, 4, 4, false, true>},
    {128, 128, launch_dma<128, 128, 2, 2, 4, true, true>, launch_dma<128, 128, 2, 2, 4, false, true>},
    // register-staged: any N, any outlier-block width, any output alignment
    {128, 128, launch_staged<128, 128, 2, 2, true, true>, launch_staged<128, 128, 2, 2, false, true>},
};
constexpr int kNumW4Variants = sizeof(kW4Variants) / sizeof(kW4Variants[0]);
}  // namespace

extern "C" int32_t qarvd_w4_gemm_num_variants(void) { return kNumW4Variants; }

extern "C" qarvd_status qarvd_w4a8_dual_gemm(const int8_t *Xq, int64_t ldxq, const float *s_x, const uint8_t *Wq4,
                                             int64_t ldwq4, const float *s_normal, const float *s_outlier,
                                             const float *bias, int32_t M, int32_t N, int32_t K, int32_t K_o, void *Y,
                                             qarvd_dtype ydt, int64_t ldy, int32_t *dbg_acc_normal,
                                             int32_t *dbg_acc_outlier, int32_t variant, void *stream)
{
    if (!Xq || !Wq4 || !s_x || !s_normal || !s_outlier || !Y) return QARVD_ERR_INVALID_ARG;
    if (M <= 0 || N <= 0 || K <= 0 || K > QARVD_MAX_K || K_o < 0 || K_o > K) return QARVD_ERR_INVALID_ARG;
    if (variant < 0 || variant > kNumW4Variants) return QARVD_ERR_INVALID_ARG;
    const PackedK pk = qarvd_packed(K, K_o);
    if (ldxq < pk.kp || ldwq4 < pk.kp / 2 || ldy < N) return QARVD_ERR_INVALID_ARG;
    if (ydt != QARVD_F32 && ydt != QARVD_BF16) return QARVD_ERR_UNSUPPORTED;
    if (!qarvd_aligned16(Xq) || !qarvd_aligned16(Wq4) || (ldxq % 16) || (ldwq4 % 16)) return QARVD_ERR_UNSUPPORTED;
    const size_t esz = ydt == QARVD_F32 ? 4 : 2;
    if (reinterpret_cast<uintptr_t>(Y) % esz) return QARVD_ERR_UNSUPPORTED;
    if ((reinterpret_cast<uintptr_t>(s_x) | reinterpret_cast<uintptr_t>(s_normal) | reinterpret_cast<uintptr_t>(s_outlier) |
         reinterpret_cast<uintptr_t>(bias) | reinterpret_cast<uintptr_t>(dbg_acc_normal) |
         reinterpret_cast<uintptr_t>(dbg_acc_outlier)) & 3u)
        return QARVD_ERR_UNSUPPORTED;
    GemmArgs g;
    g.Xq = Xq; g.Wq = reinterpret_cast<const int8_t *>(Wq4); g.s_x = s_x; g.s_n = s_normal; g.s_o = s_outlier; g.bias = bias;
    g.Y = Y; g.dbg_n = dbg_acc_normal; g.dbg_o = dbg_acc_outlier;
    g.ldxq = ldxq; g.ldwq = ldwq4; g.ldy = ldy; g.M = M; g.N = N; g.n_off = pk.n_off; g.kp = pk.kp;
    g.tiles_m = g.tiles_n = 0; g.act = 0; g.out_scale = 0.0f; g.store_wt = 0;
    const bool fast_ok = g.n_off <= 128 && vector_out_ok(g, ydt);
    if (!fast_ok) {
        if (variant == 1 || variant == 2) return QARVD_ERR_UNSUPPORTED;     // an LDS-direct tile asked for by name
        variant = kNumW4Variants;                                           // the register-staged kernel takes the rest
    }
    if (variant == 0) {     // same cost model as the INT8 path, restricted to the two tiles built for INT4
        const double T = g.kp / 64;
        const long t256 = (long)((M + 255) / 256) * ((N + 255) / 256), t128 = (long)((M + 127) / 128) * ((N + 127) / 128);
        const int cus = device_cus();
        const double c256 = 2.2 + (double)((t256 + cus - 1) / cus) * (8.9 + 0.688 * T);
        const double c128 = 2.0 + (double)((t128 + cus - 1) / cus) * (1.5 + 0.309 * T);
        variant = c256 <= c128 ? 1 : 2;
    }
    const W4Variant &v = kW4Variants[variant - 1];
    return (g.n_off > 0 ? v.dual : v.single)(g, ydt, reinterpret_cast<hipStream_t>(stream));
}

// ---- chained layers: INT8 output quantized in the epilogue ----------------------------------------------
namespace {
struct Q8Variant {
    int BM, BN;
    double c, a, b;     // cost model of pick_variant
    qarvd_status (*dual)(const GemmArgs &, hipStream_t);
    qarvd_status (*single)(const GemmArgs &, hipStream_t);
};
const Q8Variant kQ8Variants[] = {
    {256, 256, 2.2, 8.9, 0.688, launch_dma_q8<256, 256, 2, 4, 4, true>, launch_dma_q8<256, 256, 2, 4, 4, false>},
    {128, 256, 5.0, 2.75, 0.490, launch_dma_q8<128, 256, 2, 4, 4, true>, launch_dma_q8<128, 256, 2, 4, 4, false>},
    {128, 128, 2.0, 1.5, 0.309, launch_dma_q8<128, 128, 2, 2, 4, true>, launch_dma_q8<128, 128, 2, 2, 4, false>},
    {256, 256, 7.2, 9.2, 0.443, launch_dma128_q8<256, 256, 2, 4, 2, true>, launch_dma128_q8<256, 256, 2, 4, 2, false>},
    {256, 128, 4.5, 3.6, 0.379, launch_dma128_q8<256, 128, 4, 2, 3, true>, launch_dma128_q8<256, 128, 4, 2, 3, false>},
    {128, 256, 3.9, 3.9, 0.381, launch_dma128_q8<128, 256, 2, 4, 3, true>, launch_dma128_q8<128, 256, 2, 4, 3, false>},
};
constexpr int kNumQ8Variants = sizeof(kQ8Variants) / sizeof(kQ8Variants[0]);
}  // namespace

extern "C" int32_t qarvd_q8_gemm_num_variants(void) { return kNumQ8Variants; }

extern "C" qarvd_status qarvd_w8a8_dual_gemm_q8(const int8_t *Xq, int64_t ldxq, const float *s_x, const int8_t *Wq,
                                                int64_t ldwq, const float *s_normal, const float *s_outlier,
                                                const float *bias, int32_t M, int32_t N, int32_t K, int32_t K_o,
                                                qarvd_act act, float out_scale, int8_t *Y8, int64_t ldy8,
                                                int32_t variant, void *stream)
{
    if (!Xq || !Wq || !s_x || !s_normal || !s_outlier || !Y8) return QARVD_ERR_INVALID_ARG;
    if (M <= 0 || N <= 0 || K <= 0 || K > QARVD_MAX_K || K_o < 0 || K_o > K) return QARVD_ERR_INVALID_ARG;
    if (act != QARVD_ACT_NONE && act != QARVD_ACT_GELU_TANH) return QARVD_ERR_INVALID_ARG;
    if (!(out_scale >= 1.0e-30f) || out_scale > 1.0e30f) return QARVD_ERR_INVALID_ARG;     // NaN, zero, negative, inf; 1 / s must be normal
    if (variant < 0 || variant > kNumQ8Variants) return QARVD_ERR_INVALID_ARG;
    const PackedK pk = qarvd_packed(K, K_o);
    if (ldxq < pk.kp || ldwq < pk.kp || ldy8 < N) return QARVD_ERR_INVALID_ARG;
    if (!qarvd_aligned16(Xq) || !qarvd_aligned16(Wq) || (ldxq % 16) || (ldwq % 16)) return QARVD_ERR_UNSUPPORTED;
    if ((reinterpret_cast<uintptr_t>(s_x) & 3u) || !qarvd_aligned16(s_normal) || !qarvd_aligned16(s_outlier) ||
        !qarvd_aligned16(bias))
        return QARVD_ERR_UNSUPPORTED;
    // 16 codes per store; 32-bit byte offsets inside a tile
    if ((N % 16) || !qarvd_aligned16(Y8) || (ldy8 % 16) || ldxq > (1 << 22) || ldwq > (1 << 22) || ldy8 > (1 << 22))
        return QARVD_ERR_UNSUPPORTED;
    GemmArgs g;
    g.Xq = Xq; g.Wq = Wq; g.s_x = s_x; g.s_n = s_normal; g.s_o = s_outlier; g.bias = bias;
    g.Y = Y8; g.dbg_n = nullptr; g.dbg_o = nullptr;
    g.ldxq = ldxq; g.ldwq = ldwq; g.ldy = ldy8; g.M = M; g.N = N; g.n_off = pk.n_off; g.kp = pk.kp;
    g.tiles_m = g.tiles_n = 0; g.act = (int32_t)act; g.out_scale = out_scale; g.store_wt = 0;
    if (g.n_off > 128) return QARVD_ERR_UNSUPPORTED;
    if (variant == 0) {
        const double T = g.kp / 64;
        double best_cost = 1e300;
        const int cus = device_cus();
        for (int i = 0; i < kNumQ8Variants; ++i) {
            const Q8Variant &c = kQ8Variants[i];
            const long tiles = (long)((M + c.BM - 1) / c.BM) * ((N + c.BN - 1) / c.BN);
            const double cost = c.c + (double)((tiles + cus - 1) / cus) * (c.a + c.b * T);
            if (cost < best_cost) { best_cost = cost; variant = i + 1; }
        }
    }
    const Q8Variant &v = kQ8Variants[variant - 1];
    return (g.n_off > 0 ? v.dual : v.single)(g, reinterpret_cast<hipStream_t>(stream));
}
