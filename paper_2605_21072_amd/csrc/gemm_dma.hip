// LDS-direct variant of the dual-scale W8A8 GEMM for gfx950 (appendix "Quantization Kernels",
// kernel (ii); Eq. (dual_scale)).
//
// Design (two 256-thread workgroups per CU so that one workgroup's epilogue -- conversion,
// packing and the output store -- runs under the other's MFMA loop):
//   * Operand tiles of 64 K-bytes go from global memory straight into LDS with
//     global_load_lds_dwordx4 (no VGPR staging), three stages deep.  One such instruction fills
//     1 KB of LDS contiguously (16 rows x 64 B); the XOR swizzle that keeps the later 32-row
//     fragment reads off the same banks is applied on the GLOBAL side: the lane that fills slot s
//     of row r fetches 16-byte chunk s ^ swz64(r) of that row.
//   * Waits are explicit: s_waitcnt vmcnt(n) for the tile about to be consumed, then a bare
//     s_barrier (no fence, which would drain every outstanding load), then the loads of the
//     tile two steps ahead are issued into the stage everybody has just finished reading.
//   * The wave tile is (BM/2) x (BN/2) with the W fragment as the MFMA A operand and the X fragment
//     as the B operand, so a lane owns ONE token row and four consecutive output features per
//     register quad: the per-token scale is a per-lane scalar, the per-feature scales and bias are
//     float4 loads, and four results pack into one 8-byte LDS write.
//   * Only the normal-range sum lives in registers during the K loop.  The tiles that contain
//     the outlier range (at most two, since the outlier block is <= 128 bytes here) are visited
//     LAST, so they are still resident in LDS when the loop ends; the epilogue computes each
//     32x32 block's outlier sum into a 16-register temporary with 1-4 MFMAs and merges the two
//     INT32 accumulators through
//         r = (float)acc_o * s_o;  r = fmaf((float)acc_n, s_n, r);  y = fmaf(r, s_x, bias).
//   * Results are transposed through a wave-private LDS patch (row stride 144 B: conflict-free
//     8-byte writes and 16-byte reads) and leave as 16-byte stores covering whole 128-byte row
//     segments.
#include "gemm_common.h"

namespace qarvd_gemm {

namespace {

constexpr int BKD = 64;      // K bytes per stage
constexpr int NSTAGE = 3;
constexpr int PATCH_RS = 144;             // bytes per row of the output patch (128 + 16 pad)
constexpr int PATCH_BYTES = 32 * PATCH_RS;

#define QARVD_GPTR(p) ((const __attribute__((address_space(1))) void *)(p))
#define QARVD_LPTR(p) ((__attribute__((address_space(3))) void *)(p))

// Swizzle for 64-byte LDS rows (four 16-byte slots): any 8 consecutive rows spread over all
// (row parity, slot) pairs and any 16 consecutive rows over all (row mod 4, slot) pairs.
__device__ __forceinline__ int swz64(int r) { return (((r >> 1) ^ (r >> 3)) & 1) | (((r >> 2) & 1) << 1); }

// s_waitcnt with only vmcnt set (gfx9 encoding: vmcnt[3:0] | expcnt[6:4] | lgkmcnt[11:8] | vmcnt[15:14]).
template <int N> __device__ __forceinline__ void wait_vmcnt()
{
    __builtin_amdgcn_s_waitcnt((N & 15) | (7 << 4) | (15 << 8) | ((N >> 4) << 14));
}
__device__ __forceinline__ void wait_lgkmcnt0() { __builtin_amdgcn_s_waitcnt(63 | (7 << 4) | (0 << 8) | (3 << 14)); }

__device__ __forceinline__ uint32_t pack_bf16x2(float a, float b)
{
    return f32_to_bf16_bits(a) | (f32_to_bf16_bits(b) << 16);
}

template <int BM, int BN, bool DUAL, typename OutT>
__global__ __launch_bounds__(TPB, 2) void gemm_dma_kernel(GemmArgs g)
{
    constexpr int WTM = BM / 2, WTN = BN / 2;      // 2 x 2 wavefronts
    constexpr int TM = WTM / 32, TN = WTN / 32;    // 32x32 blocks per wave
    constexpr int NA = BM / 64, NB = BN / 64;      // LDS-direct loads per wave per stage
    constexpr int NLOAD = NA + NB;
    constexpr int STG = (BM + BN) * BKD;
    constexpr bool PATCH_IN_STAGE = 4 * PATCH_BYTES <= STG;   // else the patches follow the stages
    constexpr int SCALES_OFF = NSTAGE * STG + (PATCH_IN_STAGE ? 0 : 4 * PATCH_BYTES);
    extern __shared__ __align__(16) unsigned char smem[];
    float *sx_lds = reinterpret_cast<float *>(smem + SCALES_OFF);   // [BM]
    float *sn_lds = sx_lds + BM;                                      // [BN]
    float *so_lds = sn_lds + BN;                                      // [BN]
    float *bs_lds = so_lds + BN;                                      // [BN]

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave >> 1, wn = wave & 1;
    int tm, tn;
    tile_coords(blockIdx.x, g.tiles_m, g.tiles_n, tm, tn);
    const int m0 = tm * BM, n0 = tn * BN;

    // ---- scales and bias of this tile: global -> registers now, -> LDS after the first tile
    // loads have been issued (so their latency overlaps), read back by the epilogue ----------
    float r_sx = 0.f, r_sn = 0.f, r_so = 0.f, r_bs = 0.f;
    if (tid < BM) r_sx = g.s_x[min(m0 + tid, g.M - 1)];
    if (tid < BN) {
        const int nc = min(n0 + tid, g.N - 1);
        r_sn = g.s_n[nc];
        r_so = g.s_o[nc];
        if (g.bias) r_bs = g.bias[nc];
    }

    // ---- LDS-direct load addressing -------------------------------------------------------
    // Load i of this wave fills rows (4*i + wave)*16 .. +16 of the operand tile; lane l fills slot
    // (l & 3) of row (l >> 2) with global chunk (l & 3) ^ swz64(l >> 2).
    const int drow = lane >> 2;
    const int dchunk = ((lane & 3) ^ swz64(drow)) << 4;
    const int8_t *pa[NA];
    const int8_t *pb[NB];
#pragma unroll
    for (int i = 0; i < NA; ++i)
        pa[i] = g.Xq + (size_t)min(m0 + (4 * i + wave) * 16 + drow, g.M - 1) * g.ldxq + dchunk;
#pragma unroll
    for (int i = 0; i < NB; ++i)
        pb[i] = g.Wq + (size_t)min(n0 + (4 * i + wave) * 16 + drow, g.N - 1) * g.ldwq + dchunk;

    auto issue = [&](int tile, int stage) {
        unsigned char *sb = smem + stage * STG;
        const size_t koff = (size_t)tile * BKD;
#pragma unroll
        for (int i = 0; i < NA; ++i)
            __builtin_amdgcn_global_load_lds(QARVD_GPTR(pa[i] + koff), QARVD_LPTR(sb + (4 * i + wave) * 1024), 16, 0, 0);
#pragma unroll
        for (int i = 0; i < NB; ++i)
            __builtin_amdgcn_global_load_lds(QARVD_GPTR(pb[i] + koff), QARVD_LPTR(sb + BM * BKD + (4 * i + wave) * 1024), 16, 0, 0);
    };

    // ---- fragment addressing --------------------------------------------------------------
    const int frow = lane & 31, fhalf = lane >> 5, fsw = swz64(frow);
    const int x_base = (wm * WTM + frow) * BKD;               // X rows: MFMA B operand
    const int w_base = BM * BKD + (wn * WTN + frow) * BKD;    // W rows: MFMA A operand
    int coff[2];
    coff[0] = ((0 | fhalf) ^ fsw) << 4;
    coff[1] = ((2 | fhalf) ^ fsw) << 4;

    v16i acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0;

    v4i xf[2][TM], wf[2][TN];   // fragments of the two k-steps of a stage
    auto load_frags = [&](const unsigned char *sb, int ks) {
#pragma unroll
        for (int j = 0; j < TN; ++j) wf[ks][j] = *reinterpret_cast<const v4i *>(sb + w_base + j * 32 * BKD + coff[ks]);
#pragma unroll
        for (int i = 0; i < TM; ++i) xf[ks][i] = *reinterpret_cast<const v4i *>(sb + x_base + i * 32 * BKD + coff[ks]);
    };
    auto mma = [&](int ks) {
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j)
                acc[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(wf[ks][j], xf[ks][i], acc[i][j], 0, 0, 0);
    };

    // ---- K loop ---------------------------------------------------------------------------
    // T >= 2 tiles of 64 bytes.  The first H <= 2 of them hold the outlier range and are visited
    // last, so the visiting order is H, H+1, .., T-1, 0, .., H-1.  Iterations 0 .. T-3 are the
    // steady state (all of them normal tiles): wait for the tile, barrier, refill the stage read one
    // iteration ago, 12 fragment reads, 16 MFMAs, and no branch but the loop's own.
    const int T = g.kp / BKD;
    const int o_steps = DUAL ? g.n_off / 32 : 0;      // 32-byte k-steps of the outlier range (<= 4)
    const int H = (o_steps + 1) / 2;
    const int Tn = T - H;
    auto seq = [&](int it) { return it < Tn ? it + H : it - Tn; };

    issue(seq(0), 0);
    issue(seq(1), 1);
    // park the scales in LDS (the compiler waits for exactly those loads; the tile loads stay in flight)
    if (tid < BM) sx_lds[tid] = r_sx;
    if (tid < BN) {
        sn_lds[tid] = r_sn;
        so_lds[tid] = r_so;
        bs_lds[tid] = r_bs;
    }
    int stage = 0;
    for (int it = 0; it < T - 2; ++it) {
        wait_vmcnt<NLOAD>();
        __builtin_amdgcn_s_barrier();
        issue(seq(it + 2), stage >= 1 ? stage - 1 : NSTAGE - 1);   // stage (it + 2) % 3
        const unsigned char *sb = smem + stage * STG;
        load_frags(sb, 0);
        load_frags(sb, 1);
        // keep all twelve reads ahead of the first MFMA: the second k-step's fragments then arrive
        // under the first k-step's MFMAs instead of being re-serialised to save registers
        __builtin_amdgcn_sched_barrier(0);
        mma(0);
        mma(1);
        stage = stage + 1 == NSTAGE ? 0 : stage + 1;
    }
    // the last two tiles: nothing left to issue; either may be a head tile, of which only a
    // trailing normal k-step (when the range boundary falls inside the tile) is summed here
#pragma unroll 1
    for (int it = T - 2; it < T; ++it) {
        if (it + 1 < T) wait_vmcnt<NLOAD>();
        else wait_vmcnt<0>();
        __builtin_amdgcn_s_barrier();
        const unsigned char *sb = smem + stage * STG;
        const int hs = it - Tn;   // >= 0: head tile number
        if (hs < 0 || 2 * hs >= o_steps) {
            load_frags(sb, 0);
            mma(0);
        }
        if (hs < 0 || 2 * hs + 1 >= o_steps) {
            load_frags(sb, 1);
            mma(1);
        }
        stage = stage + 1 == NSTAGE ? 0 : stage + 1;
    }
    wait_lgkmcnt0();                // this wave's scale writes have landed ...
    __builtin_amdgcn_s_barrier();   // ... and everyone is done with the last normal tile's stage

    // ---- epilogue -------------------------------------------------------------------------
    // stage of iteration `it` is it % 3: head tile t sits in stage (Tn + t) % 3, the stage of the
    // last normal tile (free now) is (Tn + 2) % 3 when H > 0; with H == 0 every stage is free.
    const int free_stage = H > 0 ? (Tn + 2) % NSTAGE : 0;
    unsigned char *patch = smem + (PATCH_IN_STAGE ? free_stage : NSTAGE) * STG + wave * PATCH_BYTES;
    OutT *Y = reinterpret_cast<OutT *>(g.Y);
    constexpr int EPC = 16 / sizeof(OutT);          // output elements per 16-byte chunk
    constexpr int NBP = sizeof(OutT) == 2 ? TN : 1; // 32-column blocks per patch pass
    const bool dbg = g.dbg_n != nullptr || g.dbg_o != nullptr;

#pragma unroll
    for (int i = 0; i < TM; ++i) {
        const int ml = wm * WTM + i * 32 + frow;
        const int m_lane = m0 + ml;
        const float sx = sx_lds[ml];
#pragma unroll
        for (int jp = 0; jp < TN; jp += NBP) {
#pragma unroll
            for (int jj = 0; jj < NBP; ++jj) {
                const int j = jp + jj;
                v16i ao;
#pragma unroll
                for (int r = 0; r < 16; ++r) ao[r] = 0;
                if constexpr (DUAL) {
                    for (int s = 0; s < o_steps; ++s) {
                        const unsigned char *hb = smem + ((Tn + (s >> 1)) % NSTAGE) * STG;
                        const int c = coff[s & 1];
                        const v4i wo = *reinterpret_cast<const v4i *>(hb + w_base + j * 32 * BKD + c);
                        const v4i xo = *reinterpret_cast<const v4i *>(hb + x_base + i * 32 * BKD + c);
                        ao = __builtin_amdgcn_mfma_i32_32x32x32_i8(wo, xo, ao, 0, 0, 0);
                    }
                }
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const int nl = j * 32 + 8 * q + 4 * fhalf;            // column inside the wave tile
                    const int nt = wn * WTN + nl;                          // column inside the workgroup tile
                    const float4 sn = *reinterpret_cast<const float4 *>(sn_lds + nt);
                    const float4 so = *reinterpret_cast<const float4 *>(so_lds + nt);
                    const float4 bs = *reinterpret_cast<const float4 *>(bs_lds + nt);
                    float y[4];
                    const float snv[4] = {sn.x, sn.y, sn.z, sn.w}, sov[4] = {so.x, so.y, so.z, so.w};
                    const float bsv[4] = {bs.x, bs.y, bs.z, bs.w};
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        const int r = 4 * q + e;
                        float v = (float)ao[r] * sov[e];
                        v = fmaf((float)acc[i][j][r], snv[e], v);
                        y[e] = fmaf(v, sx, bsv[e]);
                    }
                    if (dbg) {
                        const int n = n0 + nt;
                        if (m_lane < g.M && n + 4 <= g.N) {
#pragma unroll
                            for (int e = 0; e < 4; ++e) {
                                if (g.dbg_n) g.dbg_n[(size_t)m_lane * g.N + n + e] = acc[i][j][4 * q + e];
                                if (g.dbg_o) g.dbg_o[(size_t)m_lane * g.N + n + e] = ao[4 * q + e];
                            }
                        }
                    }
                    if constexpr (sizeof(OutT) == 2) {
                        uint2 pk;
                        pk.x = pack_bf16x2(y[0], y[1]);
                        pk.y = pack_bf16x2(y[2], y[3]);
                        *reinterpret_cast<uint2 *>(patch + frow * PATCH_RS + nl * 2) = pk;
                    } else {
                        *reinterpret_cast<float4 *>(patch + frow * PATCH_RS + (nl - j * 32) * 4) = make_float4(y[0], y[1], y[2], y[3]);
                    }
                }
            }
            // wave-private patch: 32 rows x 128 bytes -> 16-byte stores, 8 rows per instruction
            const int n_patch0 = n0 + wn * WTN + (sizeof(OutT) == 2 ? 0 : jp * 32);
#pragma unroll
            for (int p = 0; p < 4; ++p) {
                const int row = p * 8 + (lane >> 3), ch = lane & 7;
                const uint4 v = *reinterpret_cast<const uint4 *>(patch + row * PATCH_RS + ch * 16);
                const int m = m0 + wm * WTM + i * 32 + row;
                const int n = n_patch0 + ch * EPC;
                const bool col_ok = sizeof(OutT) == 2 ? (ch * EPC < WTN) : true;
                if (m < g.M && n + EPC <= g.N && col_ok) *reinterpret_cast<uint4 *>(Y + (size_t)m * g.ldy + n) = v;
            }
        }
    }
}

}  // namespace

template <int BM, int BN, bool DUAL>
qarvd_status launch_dma(const GemmArgs &g0, qarvd_dtype ydt, hipStream_t st)
{
    GemmArgs g = g0;
    g.tiles_m = (g.M + BM - 1) / BM;
    g.tiles_n = (g.N + BN - 1) / BN;
    const size_t stg = (size_t)(BM + BN) * BKD;
    const size_t lds = NSTAGE * stg + (4 * PATCH_BYTES <= stg ? 0 : 4 * PATCH_BYTES) + (BM + 3 * BN) * sizeof(float);
    const int grid = g.tiles_m * g.tiles_n;
    if (ydt == QARVD_BF16) {
        auto k = gemm_dma_kernel<BM, BN, DUAL, uint16_t>;
        QARVD_HIP_TRY(hipFuncSetAttribute(reinterpret_cast<const void *>(k), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
        hipLaunchKernelGGL(k, dim3(grid), dim3(TPB), lds, st, g);
    } else {
        auto k = gemm_dma_kernel<BM, BN, DUAL, float>;
        QARVD_HIP_TRY(hipFuncSetAttribute(reinterpret_cast<const void *>(k), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
        hipLaunchKernelGGL(k, dim3(grid), dim3(TPB), lds, st, g);
    }
    return qarvd_launch_status();
}

template qarvd_status launch_dma<256, 128, true>(const GemmArgs &, qarvd_dtype, hipStream_t);
template qarvd_status launch_dma<256, 128, false>(const GemmArgs &, qarvd_dtype, hipStream_t);
template qarvd_status launch_dma<192, 128, true>(const GemmArgs &, qarvd_dtype, hipStream_t);
template qarvd_status launch_dma<192, 128, false>(const GemmArgs &, qarvd_dtype, hipStream_t);
template qarvd_status launch_dma<128, 128, true>(const GemmArgs &, qarvd_dtype, hipStream_t);
template qarvd_status launch_dma<128, 128, false>(const GemmArgs &, qarvd_dtype, hipStream_t);

}  // namespace qarvd_gemm
