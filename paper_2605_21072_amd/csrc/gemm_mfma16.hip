// LDS-direct dual-scale W8A8 GEMM for gfx950 on v_mfma_i32_16x16x64_i8 (appendix "Quantization
// Kernels", kernel (ii); Eq. (dual_scale)).
//
// Same data path as the 32x32x32 kernel (persistent workgroups, a ring of 64-byte-deep LDS stages
// filled by buffer_load ... lds, scales double-buffered in LDS, swizzled output patches), built on
// the 16x16x64 instruction instead:
//   * measured on MI355X with real (non-constant) INT8 operands a register-only MFMA loop sustains
//     about 20 % more 16x16x64 than 32x32x32 work before the clock is pulled down, at equal nominal
//     rate; in this kernel the higher clock is offset by more instructions per MAC, and on the DiT
//     shapes it runs level with the 256x256 32x32x32 kernel (which stays the default);
//   * blocks of 16 allow workgroup tiles such as 256 x 224, which cover M=4680 x N=8960 in 760 tiles
//     (2.97 rounds of 256 workgroups) where 256 x 256 needs three full rounds for 2.60 rounds of work.
//
// One MFMA consumes a whole 64-byte stage row: lane l supplies bytes [16*(l>>4), +16) of row (l&15)
// of each operand; the 16x16 INT32 result has lane l holding token (l&15) (X = B operand) and, in
// register r, feature 4*(l>>4)+r (W = A operand).  So a stage is ONE k-step: per iteration a wave
// reads MB + NBK fragments for the NEXT stage into the other register buffer while MB*NBK MFMAs run
// on the current one, and the stage just consumed is refilled NSTAGE tiles ahead.
//
// Outlier range.  The packed K axis puts the outlier block first, padded to a multiple of 32 bytes,
// so the first H <= 2 stage tiles hold it; they are loaded LAST and stay in LDS for the epilogue,
// which sums them block by block into a 4-register temporary.  When the block ends in the middle of
// a 64-byte tile (32 or 96 outlier bytes) that tile is multiplied twice with complementary halves of
// the W fragment zeroed: lanes 0-31 carry its first 32 bytes (outlier sum), lanes 32-63 the rest
// (added to the normal-range accumulator).  The two INT32 sums merge as
//     r = (float)acc_o * s_o;  r = fmaf((float)acc_n, s_n, r);  y = fmaf(r, s_x, bias).
#include <algorithm>
#include <type_traits>

#include "gemm_dma_common.h"

namespace qarvd_gemm {

namespace {

// Chunk swizzle of the 64-byte stage rows for 16-row fragment reads.  A ds_read_b128 is served in
// four passes of sixteen lanes, lanes 8p..8p+7 together with lanes 32+8p..32+8p+7 (measured: with
// that grouping a linear 1 KB read and the 32-row fragment read reach ~215 B/clk per CU, a 16-row
// read swizzled for sixteen CONSECUTIVE lanes only 129).  For the 16-row fragment (lane l: row l&15,
// chunk l>>4) a pass therefore covers eight consecutive rows and the chunk pair {c, c^2}; rows r and
// r+4 share their banks, so their pairs must differ in bit 0.
__device__ __forceinline__ int swz16(int r) { return (r >> 2) & 1; }

// Output patch of a wave: 16 rows x 64 bytes (two 16x16 blocks of bf16, one of fp32); the four
// 16-byte chunks of row r sit at chunk positions c ^ ((r >> 2) & 3).
constexpr int P16_RS = 64;
constexpr int P16_BYTES = 16 * P16_RS;

template <int BM, int BN, int WM, int WN, int NSTAGE>
struct Geo16 {
    static constexpr int NW = WM * WN;
    static constexpr int THREADS = 64 * NW;
    static constexpr int WTM = BM / WM, WTN = BN / WN;   // wave tile
    static constexpr int MB = WTM / 16, NBK = WTN / 16;  // 16x16 blocks per wave
    static constexpr int GA = BM / 16, GB = BN / 16;     // 16-row load groups per operand
    static constexpr int NA = GA / NW, NB = (GB + NW - 1) / NW;   // LDS-direct loads per wave per stage
    static constexpr int NLOAD = NA + NB;
    static constexpr int STG = (BM + BN) * BKD;
    static constexpr int SCALES_OFF = NSTAGE * STG;
    static constexpr int NSCALE = BM + 3 * BN;
    static constexpr int LDS_BYTES = SCALES_OFF + 2 * NSCALE * (int)sizeof(float);
    static constexpr int SPT = (NSCALE + THREADS - 1) / THREADS;
    static_assert(BM % (16 * NW) == 0, "X row groups divide evenly over the waves");
    static_assert(WTM % 16 == 0 && WTN % 16 == 0, "wave tile is made of 16x16 blocks");
    static_assert(MB * NBK * 4 <= 128, "accumulators fit beside two fragment buffers at two waves per SIMD");
    static_assert(NW * P16_BYTES <= STG, "the output patches share one free stage");
    static_assert(NSTAGE == 4, "the wait counts below are written for four stages");
    static_assert(LDS_BYTES <= 160 * 1024, "LDS per workgroup");
};

template <int BM, int BN, int WM, int WN, int NSTAGE, bool DUAL, bool DBG, typename OutT>
__global__ __launch_bounds__(64 * WM * WN, 2) void gemm16_kernel(GemmArgs g)
{
    extern __shared__ __align__(16) unsigned char smem[];
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    using G = Geo16<BM, BN, WM, WN, NSTAGE>;
    constexpr int MB = G::MB, NBK = G::NBK, NA = G::NA, NB = G::NB, NW = G::NW, STG = G::STG, NL = G::NLOAD;
    float *const sc_both = reinterpret_cast<float *>(smem + G::SCALES_OFF);   // 2 x { s_x[BM] | s_n[BN] | s_o[BN] | bias[BN] }

    const long long p_ts = QARVD_PROF ? clock64() : 0;
    const long long p_rs = QARVD_PROF ? wall_clock64() : 0;
    const int tid = threadIdx.x, lane = tid & 63;
    const int wm = wave / WN, wn = wave % WN;
    const int ntiles = g.tiles_m * g.tiles_n;
    int tile = blockIdx.x;
    int m0, n0;                                     // tile being computed

    // ---- LDS-direct load addressing (see gemm_dma.hip): 16 rows x 64 bytes per instruction ----
    const int drow = lane >> 2;
    const int dchunk = ((lane & 3) ^ swz16(drow)) << 4;
    const int8_t *base_a, *base_b;
    int va[NA], vb[NB];
    int lm0, ln0;                                   // tile the load addressing points at
    auto w_group = [&](int i) { return min(NW * i + wave, G::GB - 1); };   // past the last group: reload it (same bytes, same place)
    auto aim_loads = [&](int t) {
        int tm, tn;
        tile_coords(t, g.tiles_m, g.tiles_n, tm, tn);
        lm0 = tm * BM;
        ln0 = tn * BN;
        base_a = g.Xq + (size_t)lm0 * g.ldxq;
        base_b = g.Wq + (size_t)ln0 * g.ldwq;
#pragma unroll
        for (int i = 0; i < NA; ++i)
            va[i] = (min(lm0 + (NW * i + wave) * 16 + drow, g.M - 1) - lm0) * (int)g.ldxq + dchunk;
#pragma unroll
        for (int i = 0; i < NB; ++i)
            vb[i] = (min(ln0 + w_group(i) * 16 + drow, g.N - 1) - ln0) * (int)g.ldwq + dchunk;
    };
    auto issue = [&](int ktile, int stage) {
        unsigned char *sb = smem + stage * STG;
        const int koff = ktile * BKD;
#pragma unroll
        for (int i = 0; i < NA; ++i)
            buffer_load_lds16(base_a, va[i], koff, sb + (NW * i + wave) * 1024);
#pragma unroll
        for (int i = 0; i < NB; ++i)
            buffer_load_lds16(base_b, vb[i], koff, sb + BM * BKD + w_group(i) * 1024);
    };

    // ---- scales: registers during the previous tile's K loop, then the other LDS buffer ----
    float r_s[G::SPT];
    auto fetch_scales = [&](int sm0, int sn0) {
#pragma unroll
        for (int u = 0; u < G::SPT; ++u) {
            const int e = tid + u * G::THREADS;
            float v = 0.f;
            if (e < BM) v = g.s_x[min(sm0 + e, g.M - 1)];
            else if (e < BM + BN) v = g.s_n[min(sn0 + e - BM, g.N - 1)];
            else if (e < BM + 2 * BN) v = g.s_o[min(sn0 + e - BM - BN, g.N - 1)];
            else if (e < BM + 3 * BN && g.bias) v = g.bias[min(sn0 + e - BM - 2 * BN, g.N - 1)];
            r_s[u] = v;
        }
    };
    auto park_scales = [&](int buf) {
        float *dst = sc_both + buf * G::NSCALE;
#pragma unroll
        for (int u = 0; u < G::SPT; ++u) {
            const int e = tid + u * G::THREADS;
            if (e < G::NSCALE) dst[e] = r_s[u];
        }
    };
    // Fetched and parked on every pass, for the last tile too (it re-reads its own), so that each
    // fetch is followed by its use on every path and the compiler never drains the stage loads to
    // protect these registers.
    auto fetch_next_scales = [&](int t) {
        int tm, tn;
        tile_coords(min(t, ntiles - 1), g.tiles_m, g.tiles_n, tm, tn);
        fetch_scales(tm * BM, tn * BN);
    };

    // ---- fragment addressing: lane l reads row (l & 15), 16-byte chunk (l >> 4) of each block ----
    const int frow = lane & 15, fg = lane >> 4;
    const int coff = (fg ^ swz16(frow)) << 4;
    const int x_base = (wm * G::WTM + frow) * BKD + coff;              // X rows: MFMA B operand
    const int w_base = BM * BKD + (wn * G::WTN + frow) * BKD + coff;   // W rows: MFMA A operand

    v4i acc[MB][NBK];
    v4i xf[2][MB], wf[2][NBK];   // two fragment buffers: the MFMAs run on one while the other fills
    auto load_frags = [&](const unsigned char *sb, auto buf_tag) {
        constexpr int b = decltype(buf_tag)::value;
        wf[b][0] = *reinterpret_cast<const v4i *>(sb + w_base);
#pragma unroll
        for (int i = 0; i < MB; ++i) xf[b][i] = *reinterpret_cast<const v4i *>(sb + x_base + i * 16 * BKD);
#pragma unroll
        for (int j = 1; j < NBK; ++j) wf[b][j] = *reinterpret_cast<const v4i *>(sb + w_base + j * 16 * BKD);
    };
    auto mma = [&](auto buf_tag) {
        constexpr int b = decltype(buf_tag)::value;
#pragma unroll
        for (int j = 0; j < NBK; ++j)
#pragma unroll
            for (int i = 0; i < MB; ++i)
                acc[i][j] = __builtin_amdgcn_mfma_i32_16x16x64_i8(wf[b][j], xf[b][i], acc[i][j], 0, 0, 0);
    };
    // ---- K tiles: T >= 2 of 64 bytes; the first H hold the outlier range and are loaded last ----
    const int T = g.kp / BKD;
    const int o32 = DUAL ? g.n_off / 32 : 0;        // 32-byte units of the outlier range (<= 4)
    const int H = (o32 + 1) / 2;
    const int Tn = T - H;                           // tiles the K loop runs over
    const bool mixed_head = (o32 & 1) != 0;         // the last head tile is half outlier, half normal
    auto seq = [&](int it) { return it < Tn ? it + H : it - Tn; };
    const int NPRO = min(NSTAGE, T);                // stages filled before a tile's K loop starts
    const int PF = min(NSTAGE - H - 1, NPRO);       // of those, how many fit beside heads and patch stage (>= 1)

    int base = 0, sbuf = 0;
    bool first_stage_landed = false, rest_pending = false;
    aim_loads(tile);
    fetch_scales(lm0, ln0);
    issue(seq(0), 0);
    issue(seq(1), 1);   // T >= 2: a fixed number of loads, so the wait the compiler puts before the scale
    park_scales(0);     // writes covers exactly the scale fetch and leaves the stage loads in flight
#pragma unroll
    for (int p = 2; p < NSTAGE; ++p)
        if (p < T) issue(seq(p), p);
    long long p_first = 0, p_bar = 0, p_loop = 0, p_epi = 0, p_pro = 0, p_mark = p_ts;
    int p_tiles = 0;

    for (;;) {
        m0 = lm0;
        n0 = ln0;
        const int next_tile = tile + (int)gridDim.x;
        const bool more = next_tile < ntiles;
#pragma unroll
        for (int i = 0; i < MB; ++i)
#pragma unroll
            for (int j = 0; j < NBK; ++j) acc[i][j] = v4i{0, 0, 0, 0};

        // The wait counts assume only stage loads are outstanding; output stores of the previous tile
        // may still be, but they are older than every load issued after them, so the waits only get
        // stricter.  A tile whose first stages were prefetched under the previous epilogue waits for
        // nothing here: that epilogue waited for them before its first store.
        if (!first_stage_landed) {
            if (NPRO >= 4) wait_vmcnt<3 * NL>();
            else if (NPRO == 3) wait_vmcnt<2 * NL>();
            else wait_vmcnt<NL>();
        }
        __builtin_amdgcn_s_barrier();   // first stage visible; everyone has left the previous tile's epilogue
        fetch_next_scales(next_tile);   // before the stage loads: the waits count those from the youngest
        if (rest_pending) {
            for (int p = PF; p < NPRO; ++p) issue(seq(p), (base + p) % NSTAGE);
        }
        const int skip_waits = rest_pending ? PF - 1 : 0;   // iterations whose next stage is known to have landed
        if (Tn > 0) load_frags(smem + base * STG, std::integral_constant<int, 0>{});
        const long long p_t0 = QARVD_PROF ? clock64() : 0;

        // iteration it: F(it) is in registers.  Wait for stage it+1, barrier, refill stage it with K tile
        // it+NSTAGE, read F(it+1) into the other buffer, MFMAs on F(it).
        auto steady_iter = [&](auto buf_tag, int it) {
            constexpr int b = decltype(buf_tag)::value;
            const int st = (base + it) % NSTAGE, st1 = (st + 1) % NSTAGE;
            wait_lgkmcnt0();
#if QARVD_PROF
            const long long q1 = clock64();
#endif
            wait_vmcnt<(NSTAGE - 2) * NL>();
            __builtin_amdgcn_s_barrier();
#if QARVD_PROF
            p_bar += clock64() - q1;
#endif
            __builtin_amdgcn_sched_barrier(0);
            load_frags(smem + st1 * STG, std::integral_constant<int, b ^ 1>{});
            issue(seq(it + NSTAGE), st);
            mma(buf_tag);
            // Instruction order (masks: 0x008 MFMA, 0x100 LDS read, 0x020 VMEM read): the fragment reads and
            // then the refill loads, spread evenly over all but the last four MFMAs.  A wave cannot issue 1 KB LDS reads much
            // faster than about one per two MFMAs without stalling on the LDS queue, and the MFMAs left over at the end give
            // the last reads time to land before the next iteration waits for them.
            constexpr int S = MB * NBK, OPS = MB + NBK + NL, SPAN = S - 4 > OPS ? S - 4 : OPS;
#pragma unroll
            for (int m = 0; m < S; ++m) {
                __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
#pragma unroll
                for (int o = 0; o < OPS; ++o)
                    if (o * SPAN / OPS == m) {
                        if (o < MB + NBK) __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
                        else __builtin_amdgcn_sched_group_barrier(0x020, 1, 0);
                    }
            }
            __builtin_amdgcn_sched_barrier(0);
        };
        // The few iterations at either end of a tile (no wait needed yet, no refill due any more, no next
        // fragments): same steps with run-time conditions, always computing from buffer 0; the
        // fragments read into buffer 1 are copied over afterwards, so these iterations can start and
        // stop at any `it` without the two buffers' roles depending on its parity.
        auto general_iter = [&](int it) {
            const int st = (base + it) % NSTAGE, st1 = (st + 1) % NSTAGE;
            wait_lgkmcnt0();
            if (it + 1 < T && it >= skip_waits) {       // stage it+1: next fragments, or the first head tile
                const int later = min(T - 1, it + NSTAGE - 1) - (it + 1);   // stages issued after it
                if (later >= 2) wait_vmcnt<2 * NL>();
                else if (later == 1) wait_vmcnt<NL>();
                else wait_vmcnt<0>();
            }
            __builtin_amdgcn_s_barrier();
            const bool next_frags = it + 1 < Tn;
            if (next_frags) load_frags(smem + st1 * STG, std::integral_constant<int, 1>{});
            if (it + NSTAGE < T) issue(seq(it + NSTAGE), st);
            mma(std::integral_constant<int, 0>{});
            if (next_frags) {
#pragma unroll
                for (int i = 0; i < MB; ++i) xf[0][i] = xf[1][i];
#pragma unroll
                for (int j = 0; j < NBK; ++j) wf[0][j] = wf[1][j];
            }
        };
        int it = 0;
        for (; it < Tn && it < skip_waits; ++it) general_iter(it);
        // steady state, two iterations per pass (the fragment buffers alternate): next fragments exist
        // (it + 1 < Tn) and a refill is due (it + NSTAGE < T) in both
        const int steady_end = min(Tn - 1, T - NSTAGE);
        for (; it + 1 < steady_end; it += 2) {
            steady_iter(std::integral_constant<int, 0>{}, it);
            steady_iter(std::integral_constant<int, 1>{}, it + 1);
        }
#pragma unroll 1
        for (; it < Tn; ++it) general_iter(it);
        const long long p_t1 = QARVD_PROF ? clock64() : 0;
        wait_vmcnt<0>();                // the head tiles have landed (and nothing else is in flight) ...
        wait_lgkmcnt0();                // ... this wave's scale writes too ...
        __builtin_amdgcn_s_barrier();   // ... and everyone is done with every stage but the heads

        // ---- epilogue ---------------------------------------------------------------------
        // head tile t sits in stage (base + Tn + t) % NSTAGE, the patches go into the stage read just
        // before, the next tile's first PF stages into what is left of the ring.
        const int hstage0 = (base + Tn) % NSTAGE;
        const int pstage = (base + Tn - 1 + NSTAGE) % NSTAGE;
        const int nbase = (base + T) % NSTAGE;
        park_scales(sbuf ^ 1);          // free since the previous tile's epilogue; nothing else is in flight here
        if (more) {
            aim_loads(next_tile);
            for (int p = 0; p < PF; ++p) issue(seq(p), (nbase + p) % NSTAGE);
        }
        const float *sc_lds = sc_both + sbuf * G::NSCALE;
        const float *sx_lds = sc_lds, *sn_lds = sc_lds + BM, *so_lds = sc_lds + BM + BN, *bs_lds = sc_lds + BM + 2 * BN;
        unsigned char *const patch = smem + pstage * STG + wave * P16_BYTES;
        OutT *Y = reinterpret_cast<OutT *>(g.Y);
        constexpr int EPC = 16 / sizeof(OutT);          // output elements per 16-byte chunk
        constexpr int NBP = sizeof(OutT) == 2 ? 2 : 1;  // 16-column blocks per patch pass (64 bytes per row)
        const int pswz = (frow >> 2) & 3;
        const bool has_o = DUAL && o32 > 0;
        const bool wt = g.store_wt != 0;
        // patch -> global: 16 rows x (16 * chunks) bytes in one instruction through a buffer descriptor over
        // the rows of this tile that exist (rows below the matrix are dropped by its range check)
        constexpr int ESZ = (int)sizeof(OutT);
        unsigned char *const y_tile = reinterpret_cast<unsigned char *>(Y + (size_t)m0 * g.ldy);
        const int ldy_b = (int)g.ldy * ESZ;
        const int y_bytes = (min(BM, g.M - m0) - 1) * ldy_b + g.N * ESZ;
        const int y_lane = (wm * G::WTM + (lane >> 2)) * ldy_b + (n0 + wn * G::WTN + (lane & 3) * EPC) * ESZ;
        const int n_left = g.N - n0 - wn * G::WTN - (lane & 3) * EPC;   // columns from this lane's chunk to the matrix edge
        auto flush_patch = [&](int i, int col0, int chunks) {           // col0: first column of the pass inside the wave tile
            const int row = lane >> 2, ch = lane & 3;
            const v4i v = *reinterpret_cast<const v4i *>(patch + row * P16_RS + ((ch ^ ((row >> 2) & 3)) << 4));
            const int voff = (ch < chunks && col0 + EPC <= n_left) ? y_lane : 0x7ffffff0;
            buffer_store16(y_tile, y_bytes, voff, i * 16 * ldy_b + col0 * ESZ, v, wt);
        };

        auto epilogue = [&](auto haso_tag) {
            constexpr bool HASO = decltype(haso_tag)::value;
#pragma unroll
            for (int i = 0; i < MB; ++i) {
                const int ml = wm * G::WTM + i * 16 + frow;
                const int m_lane = m0 + ml;
                const float sx = sx_lds[ml];
                v4i xh[2];
                if constexpr (HASO) {
                    xh[0] = *reinterpret_cast<const v4i *>(smem + hstage0 * STG + x_base + i * 16 * BKD);
                    xh[1] = xh[0];
                    if (H > 1) xh[1] = *reinterpret_cast<const v4i *>(smem + ((hstage0 + 1) % NSTAGE) * STG + x_base + i * 16 * BKD);
                }
#pragma unroll
                for (int jp = 0; jp < NBK; jp += NBP) {
#pragma unroll
                    for (int jj = 0; jj < NBP; ++jj) {
                        const int j = jp + jj;
                        if (j >= NBK) break;
                        v4i ao = {0, 0, 0, 0};
                        if constexpr (HASO) {
                            for (int t = 0; t < H; ++t) {
                                const v4i wh = *reinterpret_cast<const v4i *>(smem + ((hstage0 + t) % NSTAGE) * STG + w_base + j * 16 * BKD);
                                const v4i xo = t == 0 ? xh[0] : xh[1];
                                if (t == H - 1 && mixed_head) {
                                    const v4i z = {0, 0, 0, 0};
                                    const v4i wlo = fg < 2 ? wh : z, whi = fg < 2 ? z : wh;
                                    ao = __builtin_amdgcn_mfma_i32_16x16x64_i8(wlo, xo, ao, 0, 0, 0);
                                    acc[i][j] = __builtin_amdgcn_mfma_i32_16x16x64_i8(whi, xo, acc[i][j], 0, 0, 0);
                                } else {
                                    ao = __builtin_amdgcn_mfma_i32_16x16x64_i8(wh, xo, ao, 0, 0, 0);
                                }
                            }
                        }
                        const int nt = wn * G::WTN + j * 16 + 4 * fg;   // first of this lane's four features, inside the workgroup tile
                        const v4f sn = *reinterpret_cast<const v4f *>(sn_lds + nt);
                        const v4f so = *reinterpret_cast<const v4f *>(so_lds + nt);
                        const v4f bs = *reinterpret_cast<const v4f *>(bs_lds + nt);
                        float y[4];
#pragma unroll
                        for (int e = 0; e < 4; ++e) {
                            float v;
                            if constexpr (HASO) {
                                v = (float)ao[e] * so[e];
                                v = fmaf((float)acc[i][j][e], sn[e], v);
                            } else {
                                // acc_o == 0: (float)0 * s_o is +0 and the first fma reduces to this one
                                v = fmaf((float)acc[i][j][e], sn[e], 0.0f);
                            }
                            y[e] = fmaf(v, sx, bs[e]);
                        }
                        if constexpr (DBG) {
                            const int n = n0 + nt;
                            if (m_lane < g.M && n + 4 <= g.N) {
#pragma unroll
                                for (int e = 0; e < 4; ++e) {
                                    if (g.dbg_n) g.dbg_n[(size_t)m_lane * g.N + n + e] = acc[i][j][e];
                                    if (g.dbg_o) g.dbg_o[(size_t)m_lane * g.N + n + e] = HASO ? ao[e] : 0;
                                }
                            }
                        }
                        if (i == 0 && j == 0) {
                            // The next tile's first stages were issued when this epilogue began and have had
                            // its first block's arithmetic to land.  Waiting for them here, before the first
                            // output store is issued, means no later wait for a stage load ever has an output
                            // store ahead of it in the (in-order) memory counter.
                            __builtin_amdgcn_sched_barrier(0);
                            wait_vmcnt<0>();
                            __builtin_amdgcn_sched_barrier(0);
                        }
                        if constexpr (sizeof(OutT) == 2) {
                            v2u pk;
                            pk.x = cvt_pk_bf16(y[0], y[1]);
                            pk.y = cvt_pk_bf16(y[2], y[3]);
                            const int c = 2 * jj + (fg >> 1);
                            *reinterpret_cast<v2u *>(patch + frow * P16_RS + ((c ^ pswz) << 4) + 8 * (fg & 1)) = pk;
                        } else {
                            *reinterpret_cast<v4f *>(patch + frow * P16_RS + ((fg ^ pswz) << 4)) = v4f{y[0], y[1], y[2], y[3]};
                        }
                    }
                    const int blocks = (jp + NBP <= NBK) ? NBP : NBK - jp;
                    flush_patch(i, jp * 16, sizeof(OutT) == 2 ? 2 * blocks : 4);
                }
            }
        };
        if constexpr (DUAL) {
            if (has_o) epilogue(std::true_type{});
            else epilogue(std::false_type{});
        } else {
            epilogue(std::false_type{});
        }
#if QARVD_PROF
        {
            const long long p_t2 = clock64();
            if (p_tiles == 0) p_first = p_t0 - p_mark; else p_pro += p_t0 - p_mark;
            p_loop += p_t1 - p_t0; p_epi += p_t2 - p_t1; p_mark = p_t2; ++p_tiles;
        }
#endif
        if (!more) break;
        first_stage_landed = true;      // PF >= 1
        rest_pending = true;
        base = nbase;
        sbuf ^= 1;
        tile = next_tile;
    }
#if QARVD_PROF
    if (lane == 0) {   // per wave: sums over its tiles of loop, barrier-wait, epilogue, transition ticks
        OutT *Yp = reinterpret_cast<OutT *>(g.Y);
        int *o = (DBG && g.dbg_o) ? g.dbg_o + ((size_t)blockIdx.x * NW + wave) * 8
                                  : reinterpret_cast<int *>(Yp + (size_t)g.M * g.ldy) + ((size_t)blockIdx.x * NW + wave) * 8;
        o[0] = (int)p_loop; o[1] = (int)p_first; o[2] = (int)p_bar; o[3] = (int)p_epi; o[4] = (int)(wall_clock64() - p_rs);
        o[5] = p_tiles; o[6] = (int)(clock64() - p_ts); o[7] = (int)p_pro;
    }
#else
    (void)p_first; (void)p_bar; (void)p_loop; (void)p_epi; (void)p_pro; (void)p_mark; (void)p_tiles; (void)p_rs;
#endif
}

template <int BM, int BN, int WM, int WN, int NSTAGE, bool DUAL, bool DBG, typename OutT>
qarvd_status launch16_one(const GemmArgs &g, hipStream_t st)
{
    using G = Geo16<BM, BN, WM, WN, NSTAGE>;
    auto k = gemm16_kernel<BM, BN, WM, WN, NSTAGE, DUAL, DBG, OutT>;
    static unsigned long long lds_limit_raised = 0;      // one mask per instantiation, i.e. per kernel symbol
    if (qarvd_status st_a = qarvd_raise_lds_limit_once(k, G::LDS_BYTES, lds_limit_raised); st_a != QARVD_OK) return st_a;
    constexpr int LDS_PER_CU = 160 * 1024;
    const int wg_per_cu = std::max(1, std::min(LDS_PER_CU / G::LDS_BYTES, 8 / G::NW));
    int grid = 0;
    if (qarvd_status st_g = persistent_grid(g.tiles_m * g.tiles_n, wg_per_cu, &grid); st_g != QARVD_OK) return st_g;
    hipLaunchKernelGGL(k, dim3(grid), dim3(G::THREADS), G::LDS_BYTES, st, g);
    return qarvd_launch_status();
}

}  // namespace

template <int BM, int BN, int WM, int WN, int NSTAGE, bool DUAL>
qarvd_status launch_mfma16(const GemmArgs &g0, qarvd_dtype ydt, hipStream_t st)
{
    GemmArgs g = g0;
    g.tiles_m = (g.M + BM - 1) / BM;
    g.tiles_n = (g.N + BN - 1) / BN;
    g.store_wt = store_write_through(g, ydt == QARVD_BF16 ? 2 : 4);
    const bool dbg = g.dbg_n != nullptr || g.dbg_o != nullptr;   // raw-accumulator dumps: separate, slower build
    if (ydt == QARVD_BF16)
        return !dbg ? launch16_one<BM, BN, WM, WN, NSTAGE, DUAL, false, uint16_t>(g, st)
                    : launch16_one<BM, BN, WM, WN, NSTAGE, DUAL, true, uint16_t>(g, st);
    return !dbg ? launch16_one<BM, BN, WM, WN, NSTAGE, DUAL, false, float>(g, st)
                : launch16_one<BM, BN, WM, WN, NSTAGE, DUAL, true, float>(g, st);
}

#define QARVD_INST16(BM, BN, WM, WN, NS)                                                                       \
    template qarvd_status launch_mfma16<BM, BN, WM, WN, NS, true>(const GemmArgs &, qarvd_dtype, hipStream_t); \
    template qarvd_status launch_mfma16<BM, BN, WM, WN, NS, false>(const GemmArgs &, qarvd_dtype, hipStream_t);
QARVD_INST16(256, 224, 4, 2, 4)

}  // namespace qarvd_gemm
