// LDS-direct dual-scale W8A8 GEMM for gfx950 with 128-byte-deep K stages (appendix "Quantization Kernels",
// kernel (ii); Eq. (dual_scale)): INT8 x INT8 -> INT32 on v_mfma_i32_32x32x32_i8, fp32 dequant epilogue.
//
// Same design as the 64-byte-stage kernel (persistent workgroups, a ring of LDS stages filled by
// buffer_load ... lds, the outlier head tile visited last and re-multiplied from LDS in the epilogue, scales
// double-buffered in LDS, swizzled output patches), with one difference that matters on MI355X: a stage row is
// a whole 128-byte cache line.  One LDS-direct load moves 8 rows x 128 bytes, so every line that leaves the L2
// is used completely by the instruction that asked for it; with 64-byte rows each line is requested twice, one
// iteration apart, and under load (all CUs streaming) the vector L1 fill path then delivers half as many useful
// bytes (measured with a K-loop skeleton on 256 CUs: 2500 against 1220 cycles per 256 x 256 x 64 step).
// Consequences:
//   * four MFMA k-steps of 32 bytes per stage and one barrier per 128 K-bytes (half as many as before);
//   * the outlier range (at most 128 packed bytes) is exactly the first K tile: one head tile, H <= 1;
//   * a stage is refilled by the iteration that consumed it (its last fragments are in registers before the
//     iteration's barrier, and each wave waits for its own LDS reads before arriving), so all NSTAGE stages are
//     in use and a load has NSTAGE - 1 iterations to land; 256 x 256 tiles run with two 64 KB stages;
//   * where the LDS has room (256 x 256) the output patches get their own 16 KB behind the stages, so a whole
//     stage is free for the next tile's first K tile during the epilogue; otherwise they sit in a free stage.
#include <algorithm>
#include <type_traits>

#include "gemm_dma_common.h"

namespace qarvd_gemm {

namespace {

constexpr int BK2 = 128;                  // K bytes per stage row
constexpr int KS2 = BK2 / 32;             // MFMA k-steps per stage
constexpr int PATCH2_RS = 64;
constexpr int PATCH2_BYTES = 32 * PATCH2_RS;

// Swizzle for 128-byte LDS rows (eight 16-byte slots).  A row covers half of the 64 banks, so rows of equal
// parity share their banks.  A fragment read (ds_read_b128, lane l -> row l & 31, half l >> 5 of a k-step)
// must spread over all banks both when the hardware groups lanes {8p..8p+7, 32+8p..32+8p+7} (eight consecutive
// rows times the two halves of a k-step) and when it groups sixteen consecutive lanes (sixteen consecutive
// rows, one half): rows r, r+2, r+4, r+6 take their chunk pair {2s, 2s+1} at four different slot pairs, and
// rows r and r+8 swap the two slots of a pair.  (With the first rule alone the bank-conflict counter of the
// target-shape kernel read ten times what the 64-byte-stage kernel's does.)
__device__ __forceinline__ int swz128(int r) { return (((r >> 1) & 3) << 1) | ((r >> 3) & 1); }

template <int BM, int BN, int WM, int WN, int NSTAGE>
struct Geo2 {
    static constexpr int NW = WM * WN;
    static constexpr int THREADS = 64 * NW;
    static constexpr int WTM = BM / WM, WTN = BN / WN;
    static constexpr int TM = WTM / 32, TN = WTN / 32;
    static constexpr int NA = BM / 8 / NW, NB = BN / 8 / NW;      // LDS-direct loads (8 rows x 128 B) per wave per stage
    static constexpr int NLOAD = NA + NB;
    static constexpr int STG = (BM + BN) * BK2;
    static constexpr int PATCHES = NW * PATCH2_BYTES;
    static constexpr int NSCALE = BM + 3 * BN;
    static constexpr int SCALE_BYTES = 2 * NSCALE * (int)sizeof(float);
    static constexpr bool PATCH_EXTRA = NSTAGE * STG + PATCHES + SCALE_BYTES <= 160 * 1024;   // patches behind the stages
    static constexpr int PATCH_OFF = NSTAGE * STG;
    static constexpr int SCALES_OFF = NSTAGE * STG + (PATCH_EXTRA ? PATCHES : 0);
    static constexpr int LDS_BYTES = SCALES_OFF + SCALE_BYTES;
    static constexpr int SPT = (NSCALE + THREADS - 1) / THREADS;
    static_assert(BM % (8 * NW) == 0 && BN % (8 * NW) == 0, "row groups of eight must divide over the waves");
    static_assert(NW % 2 == 0, "the load swizzle takes bit 3 of a row from the wave number");
    static_assert(WTM % 32 == 0 && WTN % 32 == 0, "wave tile is TM x TN blocks of 32 x 32");
    static_assert(TM * TN * 16 <= 128, "two waves per SIMD: at most 128 accumulator registers");
    static_assert(PATCHES <= STG, "the output patches fit into one stage");
    static_assert(PATCH_EXTRA ? NSTAGE >= 2 : NSTAGE >= 3, "a head tile, the patches and one stage for the next tile");
    static_assert(LDS_BYTES <= 160 * 1024, "LDS per workgroup");
    static_assert((NSTAGE - 1) * NLOAD < 64, "vmcnt is a 6-bit counter");
};

template <int BM, int BN, int WM, int WN, int NSTAGE, bool DUAL, bool DBG, typename OutT>
__global__ __launch_bounds__(64 * WM * WN, 2) void gemm_dma128_kernel(GemmArgs g)
{
    using G = Geo2<BM, BN, WM, WN, NSTAGE>;
    constexpr int TM = G::TM, TN = G::TN, NA = G::NA, NB = G::NB, NW = G::NW, STG = G::STG, NL = G::NLOAD;
    extern __shared__ __align__(16) unsigned char smem[];
    float *const sc_both = reinterpret_cast<float *>(smem + G::SCALES_OFF);   // 2 x { s_x[BM] | s_n[BN] | s_o[BN] | bias[BN] }

    const long long p_ts = QARVD_PROF ? clock64() : 0;
    const long long p_rs = QARVD_PROF ? wall_clock64() : 0;
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave / WN, wn = wave % WN;
    const int ntiles = g.tiles_m * g.tiles_n;
    int tile = blockIdx.x;
    int m0, n0;                                    // tile being computed

    // ---- LDS-direct load addressing: load i of this wave fills rows (NW*i + wave)*8 .. +8 of the operand tile;
    // lane l fills slot (l & 7) of row (l >> 3) of those with global chunk (l & 7) ^ swz128(row in the tile).  Tile base in SGPRs, one
    // byte offset per lane and load, the K position as scalar offset.  Rows past the matrix are clamped to its
    // last row (their products land in rows / columns that are never stored).
    const int drow = lane >> 3;
    const int dchunk = ((lane & 7) ^ swz128(8 * (wave & 1) + drow)) << 4;      // (NW is even: row bit 3 = wave bit 0)
    const int8_t *base_a, *base_b;
    int va[NA], vb[NB];
    int lm0, ln0;                                  // tile the load addressing points at
    auto aim_loads = [&](int t) {
        int tm, tn;
        tile_coords(t, g.tiles_m, g.tiles_n, tm, tn);
        lm0 = tm * BM;
        ln0 = tn * BN;
        base_a = g.Xq + (size_t)lm0 * g.ldxq;
        base_b = g.Wq + (size_t)ln0 * g.ldwq;
#pragma unroll
        for (int i = 0; i < NA; ++i)
            va[i] = (min(lm0 + (NW * i + wave) * 8 + drow, g.M - 1) - lm0) * (int)g.ldxq + dchunk;
#pragma unroll
        for (int i = 0; i < NB; ++i)
            vb[i] = (min(ln0 + (NW * i + wave) * 8 + drow, g.N - 1) - ln0) * (int)g.ldwq + dchunk;
    };
    auto issue = [&](int ktile, int stage) {
        unsigned char *sb = smem + stage * STG;
        const int koff = ktile * BK2;
#pragma unroll
        for (int i = 0; i < NA; ++i)
            buffer_load_lds16(base_a, va[i], koff, sb + (NW * i + wave) * 1024);
#pragma unroll
        for (int i = 0; i < NB; ++i)
            buffer_load_lds16(base_b, vb[i], koff, sb + BM * BK2 + (NW * i + wave) * 1024);
    };

    // ---- scales and bias: registers during the previous tile's K loop, then the other LDS buffer ----
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
    // fetched and parked on every pass, for the last tile too (it re-reads its own), so that each fetch is
    // followed by its use on every path and the compiler never drains the stage loads to protect these registers
    auto fetch_next_scales = [&](int t) {
        int tm, tn;
        tile_coords(min(t, ntiles - 1), g.tiles_m, g.tiles_n, tm, tn);
        fetch_scales(tm * BM, tn * BN);
    };

    // ---- fragment addressing: lane l reads row (l & 31), chunk 2*ks + (l >> 5) of a k-step ----
    const int frow = lane & 31, fhalf = lane >> 5, fsw = swz128(frow);
    const int x_base = (wm * G::WTM + frow) * BK2;               // X rows: MFMA B operand
    const int w_base = BM * BK2 + (wn * G::WTN + frow) * BK2;    // W rows: MFMA A operand
    int coff[KS2];
#pragma unroll
    for (int ks = 0; ks < KS2; ++ks) coff[ks] = (((2 * ks) | fhalf) ^ fsw) << 4;

    v16i acc[TM][TN];
    v4i xf[2][TM], wf[2][TN];   // fragments of k-steps of even / odd number
    auto load_frags = [&](const unsigned char *sb, int ks) {
#pragma unroll
        for (int j = 0; j < TN; ++j) wf[ks & 1][j] = *reinterpret_cast<const v4i *>(sb + w_base + j * 32 * BK2 + coff[ks]);
#pragma unroll
        for (int i = 0; i < TM; ++i) xf[ks & 1][i] = *reinterpret_cast<const v4i *>(sb + x_base + i * 32 * BK2 + coff[ks]);
    };
    auto mma = [&](int ks) {
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j)
                acc[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(wf[ks & 1][j], xf[ks & 1][i], acc[i][j], 0, 0, 0);
    };
    auto mma_z = [&](int ks) {      // the same from zero accumulators (first k-step of a tile)
        const v16i zero = {0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0};
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j)
                acc[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(wf[ks & 1][j], xf[ks & 1][i], zero, 0, 0, 0);
    };
    auto clear_acc = [&]() {
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j)
#pragma unroll
                for (int r = 0; r < 16; ++r) acc[i][j][r] = 0;
    };
    // last row of tiles: 32-row blocks that lie entirely below the matrix are left out
    int i_lim = TM;
    auto mma_r = [&](int ks) {
#pragma unroll
        for (int i = 0; i < TM; ++i)
            if (i < i_lim) {
#pragma unroll
                for (int j = 0; j < TN; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(wf[ks & 1][j], xf[ks & 1][i], acc[i][j], 0, 0, 0);
            }
    };
    // instruction-order hints (masks: 0x008 MFMA, 0x100 LDS read, 0x020 VMEM read)
    auto interleave_reads = [&]() {
#pragma unroll
        for (int i = 0; i < TM * TN; ++i) {
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
            if (i < TM + TN) __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
        }
    };
    auto interleave_reads_and_loads = [&]() {
        constexpr int S = TM * TN, R = TM + TN, OPS = R + NL;
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

    // ---- K tiles: T >= 1 of 128 bytes.  Tile 0 holds the outlier range (when there is one) and is visited last:
    // order H, .., T-1, 0.  Iteration `it` reads stage (base + it) % NSTAGE and, once read, refills it.
    const int T = g.kp / BK2;
    const int o_steps = DUAL ? g.n_off / 32 : 0;      // 32-byte k-steps of the outlier range (<= 4)
    const int H = o_steps > 0 ? 1 : 0;
    const int Tn = T - H;
    auto seq = [&](int it) { return it < Tn ? it + H : it - Tn; };
    const int NPRO = min(NSTAGE, T);                  // stages filled before a tile's K loop starts
    const int PF = min(NSTAGE - H - (G::PATCH_EXTRA ? 0 : 1), NPRO);   // of those, under the previous epilogue (>= 1)

    int base = 0, sbuf = 0;
    bool first_stage_landed = false, rest_pending = false;
    aim_loads(tile);
    fetch_scales(lm0, ln0);
    issue(seq(0), 0);   // a fixed number of loads, so the wait the compiler puts before the scale writes covers
    park_scales(0);     // exactly the scale fetch and leaves the stage loads in flight
#pragma unroll
    for (int p = 1; p < NSTAGE; ++p)
        if (p < T) issue(seq(p), p);
    long long p_vm = 0, p_bar = 0, p_loop = 0, p_epi = 0, p_pro = 0, p_mark = p_ts;
    int p_tiles = 0;

    for (;;) {
    m0 = lm0;
    n0 = ln0;
    const int next_tile = tile + (int)gridDim.x;
    const bool more = next_tile < ntiles;
    // The wait counts assume only stage loads are outstanding; the previous tile's output stores may still be,
    // but they are older than every load issued after them, so the waits only get stricter.  A tile whose first
    // stage was prefetched under the previous epilogue waits for nothing here: that epilogue waited for the
    // prefetch before its first store.
    if (!first_stage_landed) wait_stages_in_flight<NSTAGE - 1, NL>(NPRO - 1);
    __builtin_amdgcn_s_barrier();   // first stage visible; everyone has left the previous tile's epilogue
    fetch_next_scales(next_tile);   // (before the stage loads: the waits count those from the youngest)
    if (rest_pending) {
        for (int p = PF; p < NPRO; ++p) issue(seq(p), (base + p) % NSTAGE);
    }
    load_frags(smem + base * STG, 0);
    int stage = base;
    const long long p_t0 = QARVD_PROF ? clock64() : 0;
    i_lim = min(TM, max(0, (min(BM, g.M - m0) - wm * G::WTM + 31) / 32));

    // iteration it:  read F1 | MFMA F0 | read F2 | MFMA F1 | read F3 | MFMA F2 | wait, barrier |
    //                read F0(it+1), refill this stage with K tile it+NSTAGE | MFMA F3
    // Before the barrier a wave waits for its own loads of stage it+1 and for its own LDS reads (the last
    // fragments of this stage), so after the barrier stage it+1 is complete and stage `it` is dead.
    if (i_lim < TM) {                            // ragged tile: same steps, unneeded row blocks left out
        clear_acc();
#pragma unroll 1
        for (int it = 0; it < T - NSTAGE; ++it) {
            const unsigned char *sb = smem + stage * STG;
            const int nstage = stage + 1 == NSTAGE ? 0 : stage + 1;
            load_frags(sb, 1);
            mma_r(0);
            load_frags(sb, 2);
            mma_r(1);
            load_frags(sb, 3);
            mma_r(2);
            wait_vmcnt<(NSTAGE - 2) * NL>();
            wait_lgkmcnt0();
            __builtin_amdgcn_s_barrier();
            load_frags(smem + nstage * STG, 0);
            issue(seq(it + NSTAGE), stage);
            mma_r(3);
            stage = nstage;
        }
    } else {
    // The accumulators start from the MFMA's inline zero in a first iteration of its own (128 register moves less
    // per tile and wave than clearing them, in a phase that is bound by vector-ALU issue).
    int it0 = 0;
    if (T > NSTAGE) {
        const unsigned char *sb = smem + stage * STG;
        const int nstage = stage + 1 == NSTAGE ? 0 : stage + 1;
        load_frags(sb, 1);
        mma_z(0);
        interleave_reads();
        __builtin_amdgcn_sched_barrier(0);
        load_frags(sb, 2);
        mma(1);
        interleave_reads();
        __builtin_amdgcn_sched_barrier(0);
        load_frags(sb, 3);
        mma(2);
        interleave_reads();
        __builtin_amdgcn_sched_barrier(0);
        wait_vmcnt<(NSTAGE - 2) * NL>();
        wait_lgkmcnt0();
        __builtin_amdgcn_s_barrier();
        load_frags(smem + nstage * STG, 0);
        issue(seq(NSTAGE), stage);
        mma(3);
        interleave_reads_and_loads();
        __builtin_amdgcn_sched_barrier(0);
        stage = nstage;
        it0 = 1;
    } else {
        clear_acc();
    }
    for (int it = it0; it < T - NSTAGE; ++it) {    // steady state: every tile here is a normal tile
        const unsigned char *sb = smem + stage * STG;
        const int nstage = stage + 1 == NSTAGE ? 0 : stage + 1;
        load_frags(sb, 1);
        mma(0);
        interleave_reads();
        __builtin_amdgcn_sched_barrier(0);
        load_frags(sb, 2);
        mma(1);
        interleave_reads();
        __builtin_amdgcn_sched_barrier(0);
        load_frags(sb, 3);
        mma(2);
        interleave_reads();
        __builtin_amdgcn_sched_barrier(0);       // the waits below must not float up into the MFMAs
#if QARVD_PROF
        const long long q1 = clock64();
#endif
        wait_vmcnt<(NSTAGE - 2) * NL>();
        wait_lgkmcnt0();
        __builtin_amdgcn_s_barrier();
#if QARVD_PROF
        p_bar += clock64() - q1;
#endif
        load_frags(smem + nstage * STG, 0);
        issue(seq(it + NSTAGE), stage);
        mma(3);
        interleave_reads_and_loads();
        __builtin_amdgcn_sched_barrier(0);
        stage = nstage;
    }
    }
    // Two stages: the second-to-last K tile is always a normal one; it runs through a copy of the scheduled
    // iteration that has nothing to refill, which leaves only the last tile (the head tile, if any) to the
    // unscheduled drain loop below.
    int drain_from = T > NSTAGE ? T - NSTAGE : 0;
    if (NSTAGE == 2 && i_lim == TM && T >= 2) {
        const unsigned char *sb = smem + stage * STG;
        const int nstage = stage + 1 == NSTAGE ? 0 : stage + 1;
        load_frags(sb, 1);
        mma(0);
        interleave_reads();
        __builtin_amdgcn_sched_barrier(0);
        load_frags(sb, 2);
        mma(1);
        interleave_reads();
        __builtin_amdgcn_sched_barrier(0);
        load_frags(sb, 3);
        mma(2);
        interleave_reads();
        __builtin_amdgcn_sched_barrier(0);
        wait_vmcnt<0>();
        wait_lgkmcnt0();
        __builtin_amdgcn_s_barrier();
        load_frags(smem + nstage * STG, 0);
        mma(3);
        interleave_reads();
        __builtin_amdgcn_sched_barrier(0);
        stage = nstage;
        drain_from = T - 1;
    }
    // drain: the last tiles, nothing left to issue; the head tile is the last of them and only its
    // normal k-steps (those past the outlier range) are summed here
#pragma unroll 1
    for (int it = drain_from; it < T; ++it) {
        const unsigned char *sb = smem + stage * STG;
        const int nstage = stage + 1 == NSTAGE ? 0 : stage + 1;
        const int first = it < Tn ? 0 : o_steps;    // first k-step of this tile that belongs to the normal range
        load_frags(sb, 1);
        if (0 >= first) mma_r(0);
        load_frags(sb, 2);
        if (1 >= first) mma_r(1);
        load_frags(sb, 3);
        if (2 >= first) mma_r(2);
        if (it + 1 < T) {
            wait_stages_in_flight<(NSTAGE >= 2 ? NSTAGE - 2 : 0), NL>(T - 2 - it);   // stage it + 1 has landed
            wait_lgkmcnt0();
            __builtin_amdgcn_s_barrier();
            load_frags(smem + nstage * STG, 0);
        }
        if (3 >= first) mma_r(3);
        stage = nstage;
    }
    const long long p_t1 = QARVD_PROF ? clock64() : 0;
    wait_lgkmcnt0();                // this wave's scale writes and fragment reads have landed ...
    __builtin_amdgcn_s_barrier();   // ... and everyone is done with every stage but the head tile's

    // ---- epilogue -------------------------------------------------------------------------
    // the head tile sits in stage (base + Tn) % NSTAGE; the patches behind the stages, or in the stage read just
    // before the head; the rest of the ring takes the next tile's first PF stages
    const int hstage0 = (base + Tn) % NSTAGE;
    const int pstage = (base + Tn - 1 + 2 * NSTAGE) % NSTAGE;
    const int nbase = (base + T) % NSTAGE;
    park_scales(sbuf ^ 1);          // free since the previous tile's epilogue; nothing else is in flight here
    if (more) {
        aim_loads(next_tile);
        for (int p = 0; p < PF; ++p) issue(seq(p), (nbase + p) % NSTAGE);
    }
    const float *sc_lds = sc_both + sbuf * G::NSCALE;
    const float *sx_lds = sc_lds, *sn_lds = sc_lds + BM, *so_lds = sc_lds + BM + BN, *bs_lds = sc_lds + BM + 2 * BN;
    unsigned char *const patch = (G::PATCH_EXTRA ? smem + G::PATCH_OFF : smem + pstage * STG) + wave * PATCH2_BYTES;
    OutT *Y = reinterpret_cast<OutT *>(g.Y);
    constexpr int EPC = 16 / sizeof(OutT);          // output elements per 16-byte chunk
    const int pswz = (frow >> 2) & 3;               // chunk swizzle of this lane's patch row when writing
    constexpr int ESZ = (int)sizeof(OutT);
    unsigned char *const y_tile = reinterpret_cast<unsigned char *>(Y + (size_t)m0 * g.ldy);
    const int ldy_b = (int)g.ldy * ESZ;
    const int y_bytes = (min(BM, g.M - m0) - 1) * ldy_b + g.N * ESZ;
    const int y_lane = (wm * G::WTM + (lane >> 2)) * ldy_b + (n0 + wn * G::WTN + (lane & 3) * EPC) * ESZ;
    const int n_left = g.N - n0 - wn * G::WTN - (lane & 3) * EPC;     // columns from this lane's chunk to the matrix edge
    const bool has_o = DUAL && o_steps > 0;
    const bool wt = g.store_wt != 0;
    const StaticQuant sq = make_static_quant(sizeof(OutT) == 1 ? g.out_scale : 1.0f);

    // Software pipeline over 32 x 32 blocks, as in the 64-byte-stage kernel: a patch is read back as soon as it
    // is complete and stored after the next block's arithmetic; the outlier MFMAs of the next block start before
    // the current block's arithmetic; the row block is the outer loop so that the two halves of a 128-byte
    // output line are written back to back.
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
                // the next tile's first stages were issued when this epilogue began; waiting for them before the
                // first output store means no later stage wait has an output store ahead of it in the counter
                __builtin_amdgcn_sched_barrier(0);
#if QARVD_PROF == 2
                const long long q0 = clock64();
#endif
                wait_vmcnt<0>();
#if QARVD_PROF == 2
                p_vm += clock64() - q0;      // (diagnostic build 2: o[1] = ticks spent in this wait, summed over the tiles)
#endif
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
                pend[p] = *reinterpret_cast<const v4i *>(patch + row * PATCH2_RS + ((ch ^ ((row >> 2) & 3)) << 4));
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
            const unsigned char *hb = smem + hstage0 * STG;
            v16i ao = __builtin_amdgcn_mfma_i32_32x32x32_i8(
                *reinterpret_cast<const v4i *>(hb + w_base + j * 32 * BK2 + coff[0]),
                *reinterpret_cast<const v4i *>(hb + x_base + i * 32 * BK2 + coff[0]), zero, 0, 0, 0);
            for (int s = 1; s < o_steps; ++s) {
                const int c = s == 1 ? coff[1] : s == 2 ? coff[2] : coff[3];
                const v4i wo = *reinterpret_cast<const v4i *>(hb + w_base + j * 32 * BK2 + c);
                const v4i xo = *reinterpret_cast<const v4i *>(hb + x_base + i * 32 * BK2 + c);
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
        constexpr bool AO_AHEAD = HASO && sizeof(OutT) <= 2 && !DBG && TM * TN < 8;   // 16 registers: only where they are to spare
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
                            if (g.dbg_n) g.dbg_n[(size_t)m_lane * g.N + n + e] = acc[i][j][4 * q + e];
                            if (g.dbg_o) {
                                int aov = 0;
                                if constexpr (HASO) aov = ao[4 * q + e];
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
                    *reinterpret_cast<unsigned *>(patch + frow * PATCH2_RS + ((c ^ pswz) << 4) + 8 * (q & 1) + 4 * fhalf) = pk;
                } else if constexpr (sizeof(OutT) == 2) {
                    v2u pk;
                    pk.x = cvt_pk_bf16(y[0], y[1]);
                    pk.y = cvt_pk_bf16(y[2], y[3]);
                    *reinterpret_cast<v2u *>(patch + frow * PATCH2_RS + ((q ^ pswz) << 4) + 8 * fhalf) = pk;
                } else {
                    const int c = 2 * (q & 1) + fhalf;
                    *reinterpret_cast<v4f *>(patch + frow * PATCH2_RS + ((c ^ pswz) << 4)) = v4f{y[0], y[1], y[2], y[3]};
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
        if (p_tiles == 0) { if (QARVD_PROF != 2) p_vm = p_t0 - p_mark; } else p_pro += p_t0 - p_mark;
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
    if (lane == 0) {   // per wave: sums over its tiles of loop, lead-in, barrier-wait, epilogue, hand-over ticks
        OutT *Yp = reinterpret_cast<OutT *>(g.Y);
        int *o = (DBG && g.dbg_o) ? g.dbg_o + ((size_t)blockIdx.x * NW + wave) * 8
                                  : reinterpret_cast<int *>(Yp + (size_t)g.M * g.ldy) + ((size_t)blockIdx.x * NW + wave) * 8;
        o[0] = (int)p_loop; o[1] = (int)p_vm; o[2] = (int)p_bar; o[3] = (int)p_epi; o[4] = (int)(wall_clock64() - p_rs);
        o[5] = p_tiles; o[6] = (int)(clock64() - p_ts); o[7] = (int)p_pro;
    }
#else
    (void)p_vm; (void)p_bar; (void)p_loop; (void)p_epi; (void)p_pro; (void)p_mark; (void)p_tiles; (void)p_rs;
#endif
}

template <int BM, int BN, int WM, int WN, int NSTAGE, bool DUAL, bool DBG, typename OutT>
qarvd_status launch128_one(const GemmArgs &g, hipStream_t st)
{
    using G = Geo2<BM, BN, WM, WN, NSTAGE>;
    auto k = gemm_dma128_kernel<BM, BN, WM, WN, NSTAGE, DUAL, DBG, OutT>;
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
qarvd_status launch_dma128(const GemmArgs &g0, qarvd_dtype ydt, hipStream_t st)
{
    GemmArgs g = g0;
    g.tiles_m = (g.M + BM - 1) / BM;
    g.tiles_n = (g.N + BN - 1) / BN;
    g.store_wt = store_write_through(g, ydt == QARVD_BF16 ? 2 : 4);
    const bool dbg = g.dbg_n != nullptr || g.dbg_o != nullptr;   // raw-accumulator dumps: separate, slower build
    if (ydt == QARVD_BF16)
        return !dbg ? launch128_one<BM, BN, WM, WN, NSTAGE, DUAL, false, uint16_t>(g, st)
                    : launch128_one<BM, BN, WM, WN, NSTAGE, DUAL, true, uint16_t>(g, st);
    return !dbg ? launch128_one<BM, BN, WM, WN, NSTAGE, DUAL, false, float>(g, st)
                : launch128_one<BM, BN, WM, WN, NSTAGE, DUAL, true, float>(g, st);
}

template <int BM, int BN, int WM, int WN, int NSTAGE, bool DUAL>
qarvd_status launch_dma128_q8(const GemmArgs &g0, hipStream_t st)
{
    GemmArgs g = g0;
    g.tiles_m = (g.M + BM - 1) / BM;
    g.tiles_n = (g.N + BN - 1) / BN;
    g.store_wt = store_write_through(g, 1);
    return g.act == 1 ? launch128_one<BM, BN, WM, WN, NSTAGE, DUAL, false, Int8GeluOut>(g, st)
                      : launch128_one<BM, BN, WM, WN, NSTAGE, DUAL, false, Int8Out>(g, st);
}

#define QARVD_INST128_Q8(BM, BN, WM, WN, NS)                                                         \
    template qarvd_status launch_dma128_q8<BM, BN, WM, WN, NS, true>(const GemmArgs &, hipStream_t); \
    template qarvd_status launch_dma128_q8<BM, BN, WM, WN, NS, false>(const GemmArgs &, hipStream_t);
QARVD_INST128_Q8(256, 256, 2, 4, 2)
QARVD_INST128_Q8(256, 128, 4, 2, 3)
QARVD_INST128_Q8(128, 256, 2, 4, 3)

#define QARVD_INST128(BM, BN, WM, WN, NS)                                                                        \
    template qarvd_status launch_dma128<BM, BN, WM, WN, NS, true>(const GemmArgs &, qarvd_dtype, hipStream_t);   \
    template qarvd_status launch_dma128<BM, BN, WM, WN, NS, false>(const GemmArgs &, qarvd_dtype, hipStream_t);
QARVD_INST128(256, 256, 2, 4, 2)
QARVD_INST128(256, 128, 4, 2, 3)
QARVD_INST128(128, 256, 2, 4, 3)

}  // namespace qarvd_gemm
