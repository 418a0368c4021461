// LDS-direct dual-scale W8A8 GEMM for gfx950 (appendix "Quantization Kernels", kernel (ii);
// Eq. (dual_scale)): INT8 x INT8 -> INT32 on v_mfma_i32_32x32x32_i8 with an fp32 dequant epilogue.
//
// One kernel template, instantiated for several workgroup shapes:
//   BM x BN  workgroup tile;  WM x WN wavefronts, each owning (BM/WM) x (BN/WN) = TM x TN MFMA
//            blocks of 32 x 32 (the accumulators are the only large register set);
//   NSTAGE   LDS stages of 64 K-bytes per operand row, filled NSTAGE-1 stages ahead.
// The big DiT shapes use 256 x 256 with eight waves (one workgroup per CU, 128 KB of stages):
// a 256 x 256 tile needs half the L1/L2 operand traffic per MAC of 256 x 128, and the MI355X
// retires 4096 INT8 MACs per clock per CU against 64 B/clk of vector L1.  Smaller shapes use
// four-wave tiles, two workgroups per CU.
//
// Data path
//   * persistent workgroups: the grid is as many workgroups as the chip holds at once and each walks
//     the tile list with that stride.  The LDS stages form one ring across tiles, so the first
//     stages of the next tile are issued before the epilogue of the current one starts and land
//     under it; its scales travel in registers during the K loop and sit in a second LDS buffer.
//   * global -> LDS with buffer_load_dwordx4 ... lds, no VGPR staging: tile base in SGPRs, one
//     constant byte offset per lane, the K position as scalar offset.  One instruction fills 1 KB
//     of LDS contiguously (16 rows x 64 B); the XOR swizzle that keeps the 32-row fragment reads
//     off the same banks is applied on the GLOBAL side: the lane that fills slot s of row r fetches
//     16-byte chunk s ^ swz64(r) of that row.  Measured load-to-use latency of these loads is
//     0.7 us from L2 and 1-1.4 us from memory, so NSTAGE-1 stages are kept in flight.
//   * explicit waits: s_waitcnt vmcnt(n) for the stage about to be read, then a bare s_barrier
//     (a fence would drain every outstanding load), then the refill of the stage everybody
//     finished reading one iteration ago.  The steady-state loop is a single basic block in which
//     fragment reads and refill loads alternate with the MFMAs (sched_group_barrier).
//   * W fragment = MFMA A operand, X fragment = B operand, so a lane owns ONE token row and four
//     consecutive output features per register quad: the per-token scale is a per-lane scalar, the
//     per-feature scales and bias are 16-byte LDS reads, four results pack into one 8-byte write.
//   * only the normal-range sum lives in registers through the K loop.  The (at most two)
//     64-byte tiles holding the outlier range are visited LAST and stay resident in LDS; the
//     epilogue sums each 32 x 32 block's outlier k-steps into a 16-register temporary (1-4
//     MFMAs) and merges the two INT32 accumulators as
//         r = (float)acc_o * s_o;  r = fmaf((float)acc_n, s_n, r);  y = fmaf(r, s_x, bias).
//   * bf16 results are packed with v_cvt_pk_bf16_f32 (round-to-nearest-even), transposed through a
//     wave-private swizzled LDS patch (32 rows x 64 B) and stored as 16-byte chunks, 16 rows x 64 B
//     per instruction.  The epilogue waits for the prefetched stages once, before its first store,
//     so that no stage wait of the next tile has output stores ahead of it in the memory counter.
//     The epilogue is software-pipelined: a patch is read back as soon as it is complete and stored
//     after the next block's arithmetic, and the next block's outlier MFMAs start before the current
//     block's arithmetic.
//   * INT8 output (chained layers): optional GELU and the next layer's static-scale quantization on
//     the fp32 result, four codes per dword, two 32-column blocks per 64-byte patch row.
#include <algorithm>

#include "gemm_dma_common.h"

#include <type_traits>

namespace qarvd_gemm {

namespace {

// Output patch of a wave: 32 rows x 64 bytes (one 32x32 block of bf16, half a block of fp32), the
// four 16-byte chunks of row r stored at chunk positions c ^ ((r >> 2) & 3) so that neither the
// accumulator-layout writes nor the row-layout reads pile up on LDS banks.
constexpr int PATCH_RS = 64;
constexpr int PATCH_BYTES = 32 * PATCH_RS;

// W4: the W operand is packed INT4 (32 bytes per row and stage instead of 64).
template <int BM, int BN, int WM, int WN, int NSTAGE, bool W4 = false>
struct Geo {
    static constexpr int NW = WM * WN;                 // wavefronts
    static constexpr int THREADS = 64 * NW;
    static constexpr int WTM = BM / WM, WTN = BN / WN; // wave tile
    static constexpr int TM = WTM / 32, TN = WTN / 32; // 32x32 blocks per wave
    static constexpr int WROW = W4 ? 32 : BKD;          // bytes of a W row in a stage
    static constexpr int WGRP = W4 ? 32 : 16;           // W rows one LDS-direct load covers (1 KB)
    static constexpr int NA = BM / 16 / NW, NB = BN / WGRP / NW;   // LDS-direct loads per wave per stage
    static constexpr int NLOAD = NA + NB;
    static constexpr int STG = BM * BKD + BN * WROW;
    static constexpr int PATCHES = NW * PATCH_BYTES;   // all of them fit into the one stage read last before the head tiles
    // where the output patches go: inside one free stage, split over two free stages, or behind the stages
    static_assert(PATCHES <= STG, "the output patches share one free stage");
    static constexpr int SCALES_OFF = NSTAGE * STG;
    static constexpr int NSCALE = BM + 3 * BN;
    static constexpr int LDS_BYTES = SCALES_OFF + 2 * NSCALE * (int)sizeof(float);   // two scale buffers: tile t uses buffer t & 1
    static constexpr int SPT = (NSCALE + THREADS - 1) / THREADS;   // scale values per thread
    static_assert(BM % (16 * NW) == 0 && BN % (WGRP * NW) == 0, "row groups must divide over the waves");
    static_assert(WTM % 32 == 0 && WTN % 32 == 0, "wave tile is TM x TN blocks of 32 x 32");
    // accumulators beyond 128 registers per lane need the whole register file: one wave per SIMD
    static constexpr int WAVES_PER_EU = (TM * TN * 16 > 128) ? 1 : 2;
    static_assert(NSTAGE >= 3, "two head tiles plus one free stage");
};

// widen eight packed INT4 codes (two dwords) to sixteen INT8 lanes, each code times 16: with the nibble
// order of the packed layout, (p << 4) & 0xF0F0F0F0 are four consecutive codes and p & 0xF0F0F0F0 the next four
__device__ __forceinline__ v4i unpack_w4(v2i p)
{
    const int m = (int)0xF0F0F0F0u;
    return v4i{(p.x << 4) & m, p.x & m, (p.y << 4) & m, p.y & m};
}

template <int BM, int BN, int WM, int WN, int NSTAGE, bool DUAL, bool DBG, typename OutT, bool W4>
__global__ __launch_bounds__(64 * WM * WN, (Geo<BM, BN, WM, WN, NSTAGE, W4>::WAVES_PER_EU)) void gemm_dma_kernel(GemmArgs g)
{
    using G = Geo<BM, BN, WM, WN, NSTAGE, W4>;
    constexpr int TM = G::TM, TN = G::TN, NA = G::NA, NB = G::NB, NW = G::NW, STG = G::STG;
    constexpr int AHEAD = NSTAGE - 1;                  // stages in flight
    extern __shared__ __align__(16) unsigned char smem[];
    float *const sc_both = reinterpret_cast<float *>(smem + G::SCALES_OFF);   // 2 x { s_x[BM] | s_n[BN] | s_o[BN] | bias[BN] }

    const long long p_ts = QARVD_PROF ? clock64() : 0;
    const long long p_rs = QARVD_PROF ? wall_clock64() : 0;
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave / WN, wn = wave % WN;
    // ---- persistent workgroup: tiles blockIdx.x, blockIdx.x + gridDim.x, ... ------------------
    // (m0, n0) is the tile being computed; the load addressing below may already point at the next one.
    const int ntiles = g.tiles_m * g.tiles_n;
    int tile = blockIdx.x;
    int m0, n0;

    // LDS-direct load addressing.  Load i of this wave fills rows (NW*i + wave)*16 .. +16 of the
    // operand tile; lane l fills slot (l & 3) of row (l >> 2) with global chunk (l & 3) ^ swz64(l >> 2).
    // Buffer addressing: a tile-relative base in SGPRs, a constant 32-bit byte offset per lane and the
    // K position as the scalar offset, so the K loop spends no vector ALU work on addresses.  Rows
    // past the matrix are clamped to its last row (their products land in rows/columns never stored).
    const int drow = lane >> 2;
    const int dchunk = ((lane & 3) ^ swz64(drow)) << 4;
    const int8_t *base_a, *base_b;
    int va[NA], vb[NB];
    int lm0, ln0;                                   // tile the load addressing points at
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
        for (int i = 0; i < NB; ++i) {
            if constexpr (W4) {   // 32 rows x 32 bytes per load: lane l fills half (l & 1) of row (l >> 1) with the
                const int wrow = lane >> 1;                    // global half (l & 1) ^ bit 3 of the row (read-side bank spread)
                vb[i] = (min(ln0 + (NW * i + wave) * 32 + wrow, g.N - 1) - ln0) * (int)g.ldwq + (((lane & 1) ^ ((wrow >> 3) & 1)) << 4);
            } else {
                vb[i] = (min(ln0 + (NW * i + wave) * 16 + drow, g.N - 1) - ln0) * (int)g.ldwq + dchunk;
            }
        }
    };
    auto issue = [&](int ktile, int stage) {
        unsigned char *sb = smem + stage * STG;
        const int koff = ktile * BKD;
#pragma unroll
        for (int i = 0; i < NA; ++i)
            buffer_load_lds16(base_a, va[i], koff, sb + (NW * i + wave) * 1024);
#pragma unroll
        for (int i = 0; i < NB; ++i)
            buffer_load_lds16(base_b, vb[i], W4 ? koff / 2 : koff, sb + BM * BKD + (NW * i + wave) * 1024);
    };

    // Scales and bias of a tile: global -> registers while the PREVIOUS tile's K loop runs, ->
    // the other LDS buffer when that loop is done; read back by the tile's own epilogue.
    float r_s[G::SPT];
    auto fetch_scales = [&](int sm0, int sn0) {
#pragma unroll
        for (int u = 0; u < G::SPT; ++u) {
            const int e = tid + u * G::THREADS;
            float v = 0.f;
            if (e < BM) v = g.s_x[min(sm0 + e, g.M - 1)];
            else if (e < BM + BN) v = g.s_n[min(sn0 + e - BM, g.N - 1)] * (W4 ? 0.0625f : 1.0f);   // INT4 codes enter the MFMA
            else if (e < BM + 2 * BN) v = g.s_o[min(sn0 + e - BM - BN, g.N - 1)] * (W4 ? 0.0625f : 1.0f);   // times 16 (exact)
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

    // ---- fragment addressing --------------------------------------------------------------
    const int frow = lane & 31, fhalf = lane >> 5, fsw = swz64(frow);
    const int x_base = (wm * G::WTM + frow) * BKD;               // X rows: MFMA B operand
    // W rows: MFMA A operand.  Packed INT4: 32-byte rows, k-step ks in 16-byte half ks ^ bit 3 of the row, this
    // lane's eight bytes at + 8 * fhalf.
    const int w_base = W4 ? BM * BKD + (wn * G::WTN + frow) * 32 + 8 * fhalf : BM * BKD + (wn * G::WTN + frow) * BKD;
    int coff[2];
    coff[0] = ((0 | fhalf) ^ fsw) << 4;
    coff[1] = ((2 | fhalf) ^ fsw) << 4;
    int wcoff[2];
    wcoff[0] = W4 ? ((0 ^ ((frow >> 3) & 1)) << 4) : coff[0];
    wcoff[1] = W4 ? ((1 ^ ((frow >> 3) & 1)) << 4) : coff[1];
    auto read_w = [&](const unsigned char *sb, int j, int c) -> v4i {   // W fragment of block j, k-step offset c
        if constexpr (W4) return unpack_w4(*reinterpret_cast<const v2i *>(sb + w_base + j * 32 * 32 + c));
        else return *reinterpret_cast<const v4i *>(sb + w_base + j * 32 * BKD + c);
    };

    v16i acc[TM][TN];
    v4i xf[2][TM], wf[2][TN];   // fragments of the two k-steps of a stage
    auto load_frags = [&](const unsigned char *sb, int ks) {
#pragma unroll
        for (int j = 0; j < TN; ++j) wf[ks][j] = read_w(sb, j, wcoff[ks]);
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

    // Last row of tiles: 32-row blocks that lie entirely below the matrix are skipped (their outputs are dropped
    // anyway); the power they would draw is what limits the clock of the whole chip.
    int i_lim = TM;
    auto mma_r = [&](int ks) {
#pragma unroll
        for (int i = 0; i < TM; ++i)
            if (i < i_lim) {
#pragma unroll
                for (int j = 0; j < TN; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(wf[ks][j], xf[ks][i], acc[i][j], 0, 0, 0);
            }
    };

    // Instruction-order hints for the scheduler (masks: 0x008 MFMA, 0x100 LDS read, 0x020 VMEM read):
    // one fragment read after each of the first TM+TN MFMAs, and in the second half-iteration the
    // LDS-direct loads spread over the following MFMAs.
    auto interleave_reads = [&]() {
#pragma unroll
        for (int i = 0; i < TM * TN; ++i) {
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
            if (i < TM + TN) __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
        }
    };
    // Second half of an iteration: the TM+TN fragment reads, then the NLOAD refill loads (the
    // loads write LDS, so they cannot move ahead of the reads), spread evenly over the MFMAs.
    auto interleave_reads_and_loads = [&]() {
        constexpr int S = TM * TN, R = TM + TN, OPS = R + G::NLOAD;
#pragma unroll
        for (int i = 0; i < S; ++i) {
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
#pragma unroll
            for (int j = 0; j < OPS; ++j)
                if (j * S / OPS == i) {
                    if (j < R) __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
                    else __builtin_amdgcn_sched_group_barrier(0x020, 1, 0);
                }
        }
    };

    // ---- K loop ---------------------------------------------------------------------------
    // T >= 2 tiles of 64 bytes.  The first H <= 2 of them hold the outlier range and are visited
    // last: order H, H+1, .., T-1, 0, .., H-1.  Iteration `it` reads stage it % NSTAGE.
    const int T = g.kp / BKD;
    const int o_steps = DUAL ? g.n_off / 32 : 0;      // 32-byte k-steps of the outlier range (<= 4)
    const int H = (o_steps + 1) / 2;
    const int Tn = T - H;
    auto seq = [&](int it) { return it < Tn ? it + H : it - Tn; };

    // Stages form a ring that runs on across tiles: K tile `it` of a tile whose first K tile sits in
    // stage `base` uses stage (base + it) % NSTAGE, and the next tile starts at (base + T) % NSTAGE.
    int base = 0, sbuf = 0;
    const int PF = min(min(NSTAGE - H - 1, AHEAD), T);   // next-tile stages that fit beside the heads and the patch stage
    bool first_stage_landed = false, rest_pending = false;
    aim_loads(tile);
    fetch_scales(lm0, ln0);
    issue(seq(0), 0);
    issue(seq(1), 1);   // T >= 2; a fixed number of loads, so the wait the compiler puts before the
    park_scales(0);     // scale writes covers exactly the scale fetch and leaves the stage loads in flight
#pragma unroll
    for (int p = 2; p < AHEAD; ++p)
        if (p < T) issue(seq(p), p);
    // The scales of the tile after the current one travel in registers while the current K loop runs.
    // They are fetched and parked on every pass, for the last tile too (it re-reads its own), so that
    // each fetch is followed by its use on every path and the compiler never has to drain the stage
    // loads to protect these registers.
    auto fetch_next_scales = [&](int t) {
        int tm, tn;
        tile_coords(min(t, ntiles - 1), g.tiles_m, g.tiles_n, tm, tn);
        fetch_scales(tm * BM, tn * BN);
    };
    long long p_vm = 0, p_vmw = 0, p_bar = 0, p_loop = 0, p_epi = 0, p_pro = 0, p_mark = p_ts;
    int p_tiles = 0;

    for (;;) {
    m0 = lm0;
    n0 = ln0;
    const int next_tile = tile + (int)gridDim.x;
    const bool more = next_tile < ntiles;
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0;

    // The fragments of a stage's FIRST k-step are read one half-iteration early, under the MFMAs of
    // the previous stage's second k-step; so the wait + barrier that makes stage it+1 visible sits in
    // the middle of iteration it, and the refill of the stage read in iteration it-1 follows it.
    //   iteration it:  read F1(it) | MFMA F0(it) | wait, barrier, refill | read F0(it+1) | MFMA F1(it)
    // The wait counts assume only stage loads are outstanding; the previous tile's output stores may
    // still be, but they are older than every load issued after them, so the waits only get stricter.
    // A tile whose first stage was prefetched during the previous epilogue needs no wait at all here:
    // that epilogue waited for the prefetch before its first store.
    if (!first_stage_landed) {
        if (AHEAD >= 3 && T >= 3) wait_vmcnt<2 * G::NLOAD>();
        else wait_vmcnt<G::NLOAD>();
    }
    __builtin_amdgcn_s_barrier();   // first stage visible; everyone has left the previous tile's epilogue
    fetch_next_scales(next_tile);   // so its patch and head stages and the other scale buffer can be reused
    if (rest_pending) {             // (fetch before the stage loads: the waits count those from the youngest)
        for (int p = PF; p < AHEAD; ++p)
            if (p < T) issue(seq(p), (base + p) % NSTAGE);
        if (PF == 0) {
            // No stage of this tile could be prefetched under the previous epilogue (three stages, two of them
            // head tiles, the third holding the patches): its first stage was issued just now and has to land,
            // for every wave, before the first fragment read.
            if (T >= AHEAD) wait_vmcnt<(AHEAD - 1) * G::NLOAD>();
            else wait_vmcnt<0>();
            __builtin_amdgcn_s_barrier();
        }
    }
    load_frags(smem + base * STG, 0);
    int stage = base;
    long long p_t0 = QARVD_PROF ? clock64() : 0;
    i_lim = min(TM, max(0, (min(BM, g.M - m0) - wm * G::WTM + 31) / 32));
    if (i_lim < TM) {                            // ragged tile: same steps, unneeded row blocks left out
#pragma unroll 1
        for (int it = 0; it < T - AHEAD; ++it) {
            const unsigned char *sb = smem + stage * STG;
            const int nstage = stage + 1 == NSTAGE ? 0 : stage + 1;
            load_frags(sb, 1);
            mma_r(0);
            wait_vmcnt<(AHEAD - 2) * G::NLOAD>();
            __builtin_amdgcn_s_barrier();
            load_frags(smem + nstage * STG, 0);
            issue(seq(it + AHEAD), stage >= 1 ? stage - 1 : NSTAGE - 1);
            mma_r(1);
            stage = nstage;
        }
    } else
    for (int it = 0; it < T - AHEAD; ++it) {     // steady state: every tile here is a normal tile
        const unsigned char *sb = smem + stage * STG;
        const int nstage = stage + 1 == NSTAGE ? 0 : stage + 1;
        // The fragments used here were read a half-iteration ago, one after each of the first MFMAs;
        // the compiler's counted waits (lgkmcnt(n) just before the first MFMA that needs a fragment)
        // give the last of them the longest time to land.
        load_frags(sb, 1);
        mma(0);
        interleave_reads();                      // MFMA, read, MFMA, read, ...: the MFMA pipe never drains
        __builtin_amdgcn_sched_barrier(0);       // the waits below must not float up into the MFMAs
#if QARVD_PROF
        long long q0 = clock64();
        wait_vmcnt<(AHEAD - 2) * G::NLOAD>();
        long long q1 = clock64();
        __builtin_amdgcn_s_barrier();
        long long q2 = clock64();
        p_bar += q2 - q1; p_vmw += q1 - q0;
#else
        wait_vmcnt<(AHEAD - 2) * G::NLOAD>();
        __builtin_amdgcn_s_barrier();
#endif
        load_frags(smem + nstage * STG, 0);
        issue(seq(it + AHEAD), stage >= 1 ? stage - 1 : NSTAGE - 1);   // stage (it + AHEAD) % NSTAGE
        mma(1);
        interleave_reads_and_loads();
        __builtin_amdgcn_sched_barrier(0);
        stage = nstage;
    }
    // drain: the last AHEAD tiles, nothing left to issue; the head tiles are among them and only
    // their trailing normal k-steps (when the range boundary falls inside a tile) are summed here
#pragma unroll 1
    for (int it = (T > AHEAD ? T - AHEAD : 0); it < T; ++it) {
        const unsigned char *sb = smem + stage * STG;
        const int nstage = stage + 1 == NSTAGE ? 0 : stage + 1;
        const int hs = it - Tn;                   // >= 0: head tile number
        const bool use0 = hs < 0 || 2 * hs >= o_steps, use1 = hs < 0 || 2 * hs + 1 >= o_steps;
        load_frags(sb, 1);
        if (use0) mma_r(0);
        if (it + 1 < T) {
            wait_stages_in_flight<(AHEAD >= 2 ? AHEAD - 2 : 0), G::NLOAD>(T - 2 - it);   // stage it + 1 has landed
            __builtin_amdgcn_s_barrier();
            load_frags(smem + nstage * STG, 0);
        }
        if (use1) mma_r(1);
        stage = nstage;
    }
    long long p_t1 = QARVD_PROF ? clock64() : 0;
    wait_lgkmcnt0();                // this wave's scale writes have landed ...
    __builtin_amdgcn_s_barrier();   // ... and everyone is done with every stage but the head tiles'

    // ---- epilogue -------------------------------------------------------------------------
    // head tile t sits in stage (base + Tn + t) % NSTAGE; the stage read just before the heads takes
    // the output patches; whatever is left of the ring is free for the next tile already.
    const int freeA = (base + Tn - 1 + 2 * NSTAGE) % NSTAGE;
    const int hstage0 = (base + Tn) % NSTAGE;
    const int nbase = (base + T) % NSTAGE;
    park_scales(sbuf ^ 1);          // free since the previous tile's epilogue; nothing else is in flight here
    if (more) {
        aim_loads(next_tile);
        for (int p = 0; p < PF; ++p) issue(seq(p), (nbase + p) % NSTAGE);
    }
    const float *sc_lds = sc_both + sbuf * G::NSCALE;
    const float *sx_lds = sc_lds, *sn_lds = sc_lds + BM, *so_lds = sc_lds + BM + BN, *bs_lds = sc_lds + BM + 2 * BN;
    unsigned char *const patch = smem + freeA * STG + wave * PATCH_BYTES;
    OutT *Y = reinterpret_cast<OutT *>(g.Y);
    constexpr int EPC = 16 / sizeof(OutT);          // output elements per 16-byte chunk
    const int pswz = (frow >> 2) & 3;               // chunk swizzle of this lane's patch row when writing
    // patch -> global: 16 rows x 64 bytes per instruction through a buffer descriptor over the rows of
    // this tile that exist (rows below the matrix are dropped by its range check); the lane part of the
    // address is one register per tile, the block part a scalar offset.
    constexpr int ESZ = (int)sizeof(OutT);
    unsigned char *const y_tile = reinterpret_cast<unsigned char *>(Y + (size_t)m0 * g.ldy);
    const int ldy_b = (int)g.ldy * ESZ;
    const int y_bytes = (min(BM, g.M - m0) - 1) * ldy_b + g.N * ESZ;
    const int y_lane = (wm * G::WTM + (lane >> 2)) * ldy_b + (n0 + wn * G::WTN + (lane & 3) * EPC) * ESZ;
    const int n_left = g.N - n0 - wn * G::WTN - (lane & 3) * EPC;     // columns from this lane's chunk to the matrix edge
    const bool has_o = DUAL && o_steps > 0;
    const bool wt = g.store_wt != 0;
    const StaticQuant sq = make_static_quant(sizeof(OutT) == 1 ? g.out_scale : 1.0f);

    // The epilogue is a chain of LDS round trips (scales in, patch out and back) around little arithmetic,
    // so it is written as a software pipeline over its units of work, in program order:
    //   * a patch is read back into registers as soon as it is complete, but stored to global memory only
    //     after the NEXT unit's arithmetic (LDS operations of a wave execute in order, so the next unit's
    //     patch writes cannot overtake that read);
    //   * the outlier sums of the next block are started (MFMA) before the current block's arithmetic;
    //   * each block loads its columns' scales and biases up front, in one batch.  The row block stays the
    //     outer loop: a wave's two column blocks complete a 128-byte line of a bf16 output row, and writing
    //     the halves four blocks apart (column block outermost, scales loaded once) made a third of the
    //     lines leave the L2 half-written: 30 % more bytes written to memory, measured with WRITE_SIZE.
    // The whole epilogue exists twice: with the outlier sum (HASO) and without it (a layer with no outlier
    // channels run through the dual kernel, or the single-accumulator build).
    auto epilogue = [&](auto haso_tag) {
        constexpr bool HASO = decltype(haso_tag)::value;
        constexpr int NBLK = TM * TN;
        auto blk_i = [&](int b) { return b / TN; };
        // column blocks run back and forth (0 .. TN-1, TN-1 .. 0, ...): consecutive row blocks then share a column
        // block at the turn, and its scales and biases -- twelve broadcast 16-byte LDS reads per lane, the
        // epilogue's largest LDS traffic -- are loaded once for both (5 loads instead of 8 per 4 x 2 wave tile)
        auto blk_j = [&](int b) { return ((b / TN) & 1) ? TN - 1 - b % TN : b % TN; };

        v4i pend[2];
        int pend_voff = 0, pend_soff = 0;
        bool pending = false, stored = false;       // compile-time after unrolling
        auto flush_commit = [&]() {                 // patch (already in registers) -> global
            if (!pending) return;
            if (!stored) {
                // The next tile's first stages were issued when this epilogue began and have had a unit's
                // arithmetic to land.  Waiting for them here, before the first output store is issued, means
                // no later wait for a stage load ever has an output store ahead of it in the (in-order)
                // memory counter.
                __builtin_amdgcn_sched_barrier(0);
                wait_vmcnt<0>();
                __builtin_amdgcn_sched_barrier(0);
                stored = true;
            }
#pragma unroll
            for (int p = 0; p < 2; ++p) buffer_store16(y_tile, y_bytes, pend_voff, pend_soff + p * 16 * ldy_b, pend[p], wt);
            pending = false;
        };
        auto flush_issue = [&](int i, int col0) {   // col0: first column of the pass inside the wave tile
#pragma unroll
            for (int p = 0; p < 2; ++p) {
                const int row = p * 16 + (lane >> 2), ch = lane & 3;
                pend[p] = *reinterpret_cast<const v4i *>(patch + row * PATCH_RS + ((ch ^ ((row >> 2) & 3)) << 4));
            }
            pend_voff = col0 + EPC <= n_left ? y_lane : 0x7ffffff0;
            pend_soff = i * 32 * ldy_b + col0 * ESZ;
            pending = true;
        };
        auto flush = [&](int i, int col0) {
            flush_commit();
            flush_issue(i, col0);
        };
        auto head_mma = [&](int i, int j) -> v16i {   // outlier sum of block (i, j): the first k-step starts from zero
            const v16i zero = {0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0};
            const unsigned char *hb0 = smem + hstage0 * STG;
            v16i ao = __builtin_amdgcn_mfma_i32_32x32x32_i8(
                read_w(hb0, j, wcoff[0]), *reinterpret_cast<const v4i *>(hb0 + x_base + i * 32 * BKD + coff[0]), zero, 0, 0, 0);
            for (int s = 1; s < o_steps; ++s) {
                const unsigned char *hb = smem + ((hstage0 + (s >> 1)) % NSTAGE) * STG;
                const v4i wo = read_w(hb, j, wcoff[s & 1]);
                const v4i xo = *reinterpret_cast<const v4i *>(hb + x_base + i * 32 * BKD + coff[s & 1]);
                ao = __builtin_amdgcn_mfma_i32_32x32x32_i8(wo, xo, ao, 0, 0, 0);
            }
            return ao;
        };

        float sxr[TM];
#pragma unroll
        for (int i = 0; i < TM; ++i) sxr[i] = sx_lds[wm * G::WTM + i * 32 + frow];
        v4f sn[4], so[4], bs[4];
        auto load_cols = [&](int j) {
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const int nt = wn * G::WTN + j * 32 + 8 * q + 4 * fhalf;      // column inside the workgroup tile
                sn[q] = *reinterpret_cast<const v4f *>(sn_lds + nt);
                if constexpr (HASO) so[q] = *reinterpret_cast<const v4f *>(so_lds + nt);
                bs[q] = *reinterpret_cast<const v4f *>(bs_lds + nt);
            }
        };
        // (the look-ahead costs 16 registers; only the bf16 build, the one that is timed, has them to spare)
        constexpr bool AO_AHEAD = HASO && sizeof(OutT) == 2 && !DBG && !W4;
        v16i ao_next;
        if constexpr (AO_AHEAD) ao_next = head_mma(blk_i(0), blk_j(0));
#pragma unroll
        for (int b = 0; b < NBLK; ++b) {
            const int i = blk_i(b), j = blk_j(b);
            if (b == 0 || blk_j(b - 1) != j) load_cols(j);
            v16i ao;
            if constexpr (AO_AHEAD) {
                ao = ao_next;
                if (b + 1 < NBLK) ao_next = head_mma(blk_i(b + 1), blk_j(b + 1));
            } else if constexpr (HASO) {
                ao = head_mma(i, j);
            }
            const int m_lane = m0 + wm * G::WTM + i * 32 + frow;
            const float sx = sxr[i];
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const int nt = wn * G::WTN + j * 32 + 8 * q + 4 * fhalf;
                float y[4];
                const float snv[4] = {sn[q].x, sn[q].y, sn[q].z, sn[q].w}, bsv[4] = {bs[q].x, bs[q].y, bs[q].z, bs[q].w};
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const int r = 4 * q + e;
                    float v;
                    if constexpr (HASO) {
                        const float sov[4] = {so[q].x, so[q].y, so[q].z, so[q].w};
                        v = (float)ao[r] * sov[e];
                        v = fmaf((float)acc[i][j][r], snv[e], v);
                    } else {
                        // acc_o == 0: (float)0 * s_o is +0 and the first fma reduces to this one
                        v = fmaf((float)acc[i][j][r], snv[e], 0.0f);
                    }
                    y[e] = fmaf(v, sx, bsv[e]);
                }
                if constexpr (DBG) {
                    const int n = n0 + nt;
                    if (m_lane < g.M && n + 4 <= g.N) {
#pragma unroll
                        for (int e = 0; e < 4; ++e) {
                            // (INT4 codes were multiplied by 16 on the way in: the sums are exact multiples)
                            if (g.dbg_n) g.dbg_n[(size_t)m_lane * g.N + n + e] = acc[i][j][4 * q + e] >> (W4 ? 4 : 0);
                            if (g.dbg_o) {
                                int aov = 0;
                                if constexpr (HASO) aov = ao[4 * q + e] >> (W4 ? 4 : 0);
                                g.dbg_o[(size_t)m_lane * g.N + n + e] = aov;
                            }
                        }
                    }
                }
                if constexpr (sizeof(OutT) == 1) {
                    // chained layer: activation, then the next layer's static scale (Eq. (quantization)); two
                    // blocks of 32 INT8 columns share a 64-byte patch row
                    static_assert(sizeof(OutT) != 1 || TN % 2 == 0, "INT8 output pairs the column blocks");
                    const unsigned pk = quantize4_static<out_is_gelu<OutT>::value>(y, sq);
                    const int c = 2 * (j & 1) + (q >> 1);
                    *reinterpret_cast<unsigned *>(patch + frow * PATCH_RS + ((c ^ pswz) << 4) + 8 * (q & 1) + 4 * fhalf) = pk;
                } else if constexpr (sizeof(OutT) == 2) {
                    v2u pk;
                    pk.x = cvt_pk_bf16(y[0], y[1]);
                    pk.y = cvt_pk_bf16(y[2], y[3]);
                    *reinterpret_cast<v2u *>(patch + frow * PATCH_RS + ((q ^ pswz) << 4) + 8 * fhalf) = pk;
                } else {
                    const int c = 2 * (q & 1) + fhalf;
                    *reinterpret_cast<v4f *>(patch + frow * PATCH_RS + ((c ^ pswz) << 4)) = v4f{y[0], y[1], y[2], y[3]};
                    if (q & 1) flush(i, j * 32 + (q >> 1) * 16);
                }
            }
            if constexpr (sizeof(OutT) == 2) flush(i, j * 32);
            if constexpr (sizeof(OutT) == 1) {
                if (b & 1) flush(i, (j & ~1) * 32);        // both blocks of a 64-column pair are in the patch
            }
        }
        flush_commit();
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
        if (p_tiles == 0) p_vm = p_t0 - p_mark; else p_pro += p_t0 - p_mark;
        p_loop += p_t1 - p_t0; p_epi += p_t2 - p_t1; p_mark = p_t2; ++p_tiles;
    }
#endif
    if (!more) break;
    first_stage_landed = PF >= 1;
    rest_pending = true;
    base = nbase;
    sbuf ^= 1;
    tile = next_tile;
    }
#if QARVD_PROF
    if (lane == 0) {   // per wave: sums over its tiles of loop, load-wait, barrier-wait, epilogue, lead-in ticks
        OutT *Yp = reinterpret_cast<OutT *>(g.Y);
        int *o = (DBG && g.dbg_o) ? g.dbg_o + ((size_t)blockIdx.x * NW + wave) * 8
                                  : reinterpret_cast<int *>(Yp + (size_t)g.M * g.ldy) + ((size_t)blockIdx.x * NW + wave) * 8;
        o[0] = (int)p_loop; o[1] = (int)(QARVD_PROF == 2 ? p_vmw : p_vm); o[2] = (int)p_bar; o[3] = (int)p_epi; o[4] = (int)(wall_clock64() - p_rs);
        o[5] = p_tiles; o[6] = (int)(clock64() - p_ts); o[7] = (int)p_pro;
    }
#endif
}

template <int BM, int BN, int WM, int WN, int NSTAGE, bool DUAL, bool DBG, typename OutT, bool W4>
qarvd_status launch_one(const GemmArgs &g, hipStream_t st)
{
    using G = Geo<BM, BN, WM, WN, NSTAGE, W4>;
    auto k = gemm_dma_kernel<BM, BN, WM, WN, NSTAGE, DUAL, DBG, OutT, W4>;
    static unsigned long long lds_limit_raised = 0;      // one mask per instantiation, i.e. per kernel symbol
    if (qarvd_status st_a = qarvd_raise_lds_limit_once(k, G::LDS_BYTES, lds_limit_raised); st_a != QARVD_OK) return st_a;
    constexpr int LDS_PER_CU = 160 * 1024;
    const int wg_per_cu = std::max(1, std::min(LDS_PER_CU / G::LDS_BYTES, (G::WAVES_PER_EU * 4) / G::NW));
    int grid = 0;
    if (qarvd_status st_g = persistent_grid(g.tiles_m * g.tiles_n, wg_per_cu, &grid); st_g != QARVD_OK) return st_g;
    hipLaunchKernelGGL(k, dim3(grid), dim3(G::THREADS), G::LDS_BYTES, st, g);
    return qarvd_launch_status();
}

}  // namespace

template <int BM, int BN, int WM, int WN, int NSTAGE, bool DUAL, bool W4>
qarvd_status launch_dma(const GemmArgs &g0, qarvd_dtype ydt, hipStream_t st)
{
    GemmArgs g = g0;
    g.tiles_m = (g.M + BM - 1) / BM;
    g.tiles_n = (g.N + BN - 1) / BN;
    g.store_wt = store_write_through(g, ydt == QARVD_BF16 ? 2 : 4);
    const bool dbg = g.dbg_n != nullptr || g.dbg_o != nullptr;   // raw-accumulator dumps: separate, slower build
    if (ydt == QARVD_BF16)
        return !dbg ? launch_one<BM, BN, WM, WN, NSTAGE, DUAL, false, uint16_t, W4>(g, st)
                    : launch_one<BM, BN, WM, WN, NSTAGE, DUAL, true, uint16_t, W4>(g, st);
    return !dbg ? launch_one<BM, BN, WM, WN, NSTAGE, DUAL, false, float, W4>(g, st)
                : launch_one<BM, BN, WM, WN, NSTAGE, DUAL, true, float, W4>(g, st);
}

template <int BM, int BN, int WM, int WN, int NSTAGE, bool DUAL>
qarvd_status launch_dma_q8(const GemmArgs &g0, hipStream_t st)
{
    GemmArgs g = g0;
    g.tiles_m = (g.M + BM - 1) / BM;
    g.tiles_n = (g.N + BN - 1) / BN;
    g.store_wt = store_write_through(g, 1);
    return g.act == 1 ? launch_one<BM, BN, WM, WN, NSTAGE, DUAL, false, Int8GeluOut, false>(g, st)
                      : launch_one<BM, BN, WM, WN, NSTAGE, DUAL, false, Int8Out, false>(g, st);
}

#define QARVD_INST_Q8(BM, BN, WM, WN, NS)                                                     \
    template qarvd_status launch_dma_q8<BM, BN, WM, WN, NS, true>(const GemmArgs &, hipStream_t); \
    template qarvd_status launch_dma_q8<BM, BN, WM, WN, NS, false>(const GemmArgs &, hipStream_t);
QARVD_INST_Q8(256, 256, 2, 4, 4)
QARVD_INST_Q8(128, 256, 2, 4, 4)
QARVD_INST_Q8(128, 128, 2, 2, 4)

#define QARVD_INST(BM, BN, WM, WN, NS)                                                                             \
    template qarvd_status launch_dma<BM, BN, WM, WN, NS, true, false>(const GemmArgs &, qarvd_dtype, hipStream_t); \
    template qarvd_status launch_dma<BM, BN, WM, WN, NS, false, false>(const GemmArgs &, qarvd_dtype, hipStream_t);
#define QARVD_INST_W4(BM, BN, WM, WN, NS)                                                                         \
    template qarvd_status launch_dma<BM, BN, WM, WN, NS, true, true>(const GemmArgs &, qarvd_dtype, hipStream_t); \
    template qarvd_status launch_dma<BM, BN, WM, WN, NS, false, true>(const GemmArgs &, qarvd_dtype, hipStream_t);
QARVD_INST(256, 256, 2, 4, 4)
QARVD_INST(256, 128, 4, 2, 4)
QARVD_INST(128, 256, 2, 4, 4)
QARVD_INST(256, 128, 4, 2, 6)
QARVD_INST(256, 128, 4, 2, 5)
QARVD_INST(256, 128, 2, 2, 3)
QARVD_INST(192, 128, 2, 2, 3)
QARVD_INST(128, 128, 2, 2, 4)
QARVD_INST(64, 128, 2, 2, 5)
QARVD_INST(64, 64, 2, 2, 6)
QARVD_INST_W4(256, 256, 2, 4, 4)
QARVD_INST_W4(128, 128, 2, 2, 4)

}  // namespace qarvd_gemm
