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
#pragma once
#include "qarvd_common.h"

namespace qarvd_gemm {

typedef int v2i __attribute__((ext_vector_type(2)));
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
    // chained layers (INT8 output for the next layer): activation applied to the fp32 result and the
    // next layer's static activation scale; unused for fp32 / bf16 outputs
    int32_t act;
    float out_scale;
    int32_t store_wt;  // output stores write through the L2 (small outputs); set by the launchers
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
// of X rows and W rows small enough for its own L2.  GROUP_M = 4: the 28 workgroups an XCD runs at a
// time then cover 4 row-tiles x 7 column-tiles; measured inside a sequence of layers (weights coming
// from memory) the target shape takes 79 us with 4, 83-87 us with 2, 6, 7, 8 or 14.
__device__ __forceinline__ void tile_coords(int bid, int tiles_m, int tiles_n, int &tm, int &tn)
{
    constexpr int XCD = 8, GROUP_M = 4;
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


// A selectable kernel configuration.  `max_n_off` is the widest outlier block (in packed bytes)
// the variant can run; 0 means it has no outlier path at all.
struct Variant {
    const char *name;
    int BM, BN;
    int max_n_off;
    bool needs_vector_out;   // needs N % 8 == 0 and 16-byte aligned Y rows, scales and bias
    qarvd_status (*launch)(const GemmArgs &, qarvd_dtype, hipStream_t);
};

// launchers defined in gemm_staged.hip / gemm_dma.hip
template <int BM, int BN, int WM, int WN, bool DUAL, bool W4 = false>
qarvd_status launch_staged(const GemmArgs &g, qarvd_dtype ydt, hipStream_t st);
template <int BM, int BN, int WM, int WN, int NSTAGE, bool DUAL, bool W4 = false>   // W4: Wq is packed INT4, ldwq in bytes
qarvd_status launch_dma(const GemmArgs &g, qarvd_dtype ydt, hipStream_t st);
template <int BM, int BN, int WM, int WN, int NSTAGE, bool DUAL>   // INT8 output quantized in the epilogue
qarvd_status launch_dma_q8(const GemmArgs &g, hipStream_t st);
template <int BM, int BN, int WM, int WN, int NSTAGE, bool DUAL>
qarvd_status launch_dma128_q8(const GemmArgs &g, hipStream_t st);
template <int BM, int BN, int WM, int WN, int NSTAGE, bool DUAL>   // 128-byte-deep K stages (gemm_dma128.hip)
qarvd_status launch_dma128(const GemmArgs &g, qarvd_dtype ydt, hipStream_t st);
template <int BM, int BN, int WM, int WN, int NSTAGE, bool DUAL>
qarvd_status launch_mfma16(const GemmArgs &g, qarvd_dtype ydt, hipStream_t st);

}  // namespace qarvd_gemm
