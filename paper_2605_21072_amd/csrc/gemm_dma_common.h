// Device helpers shared by the LDS-direct GEMM kernels (gfx950).
#pragma once
#include "gemm_common.h"

namespace qarvd_gemm {

#ifndef QARVD_PROF
#define QARVD_PROF 0
#endif
#ifndef QARVD_NO_STORE
#define QARVD_NO_STORE 0                   // diagnostic builds: 1 = output stores dropped by the range check, 2 = not issued
#endif
#ifndef QARVD_STORE_AUX
#define QARVD_STORE_AUX 0                  // cache policy bits of the output stores
#endif
constexpr int BKD = 64;                   // K bytes per stage row
#define QARVD_GPTR(p) ((const __attribute__((address_space(1))) void *)(p))
#define QARVD_LPTR(p) ((__attribute__((address_space(3))) void *)(p))

typedef float v2f __attribute__((ext_vector_type(2)));
// LDS is read and written through these native vector types only: accesses typed with the HIP
// float4 / uint4 structs make the compiler drain every LDS-direct load in flight (s_waitcnt vmcnt(0))
// before them, which would serialise the next tile's prefetch with the epilogue.
typedef float v4f __attribute__((ext_vector_type(4)));
typedef unsigned int v2u __attribute__((ext_vector_type(2)));
typedef __bf16 v2bf __attribute__((ext_vector_type(2)));

// Swizzle for 64-byte LDS rows (four 16-byte slots): any 8 consecutive rows spread over all
// (row parity, slot) pairs and any 16 consecutive rows over all (row mod 4, slot) pairs.
__device__ __forceinline__ int swz64(int r) { return (((r >> 1) ^ (r >> 3)) & 1) | (((r >> 2) & 1) << 1); }

// s_waitcnt with only vmcnt set (gfx9 encoding: vmcnt[3:0] | expcnt[6:4] | lgkmcnt[11:8] | vmcnt[15:14]).
template <int N> __device__ __forceinline__ void wait_vmcnt()
{
    static_assert(N >= 0 && N < 64, "vmcnt is a 6-bit counter");
    __builtin_amdgcn_s_waitcnt((N & 15) | (7 << 4) | (15 << 8) | ((N >> 4) << 14));
}
// Waits until at most min(stages, MAXS) stages of NLOAD loads each are still in flight (`stages` is wave-uniform).
template <int MAXS, int NLOAD> __device__ __forceinline__ void wait_stages_in_flight(int stages)
{
    if constexpr (MAXS > 0) {
        if (stages >= MAXS) wait_vmcnt<MAXS * NLOAD>();
        else wait_stages_in_flight<MAXS - 1, NLOAD>(stages);
    } else {
        wait_vmcnt<0>();
    }
}
__device__ __forceinline__ void wait_lgkmcnt0() { __builtin_amdgcn_s_waitcnt(15 | (7 << 4) | (0 << 8) | (3 << 14)); }

// One LDS-direct load: lane l moves the 16 bytes at base + voffset(l) + soffset to lds + 16*l (lds and
// soffset wave-uniform).  The buffer descriptor (raw, no stride, no bounds) is rebuilt from `base` at
// each call; it is wave-uniform, so the compiler keeps it in four SGPRs across the K loop.  The body
// exists in the device pass only: the host pass has neither the descriptor type nor the builtin.
__device__ __forceinline__ void buffer_load_lds16(const void *base, int voffset, int soffset, unsigned char *lds)
{
#if defined(__HIP_DEVICE_COMPILE__)
    const __amdgpu_buffer_rsrc_t r = __builtin_amdgcn_make_buffer_rsrc(const_cast<void *>(base), 0, 0x7fffffff, 0x00020000);
    __builtin_amdgcn_raw_ptr_buffer_load_lds(r, QARVD_LPTR(lds), 16, voffset, soffset, 0, 0);
#else
    (void)base; (void)voffset; (void)soffset; (void)lds;
#endif
}

// One 16-byte store per lane through a raw buffer descriptor over [base, base + bytes): lanes whose
// byte offset voffset + soffset falls at or past `bytes` are dropped by the hardware, which is how the
// output rows below a ragged last tile are masked (checked on MI355X).  base, bytes, soffset wave-uniform.
// `write_through` (wave-uniform) sends the data on to memory at once instead of leaving dirty lines in the
// L2: a kernel ends with a write-back of what its XCDs' L2s still hold, which for an output of a few MB is
// most of it -- 1-2 us at the end of a 17 us GEMM; for outputs much larger than the L2s it only adds traffic
// while the kernel computes (measured: 4680 x 1536 bf16 18.0 -> 16.2 us, 4680 x 8960 72 -> 75 us).
__device__ __forceinline__ void buffer_store16(void *base, int bytes, int voffset, int soffset, v4i data, bool write_through = false)
{
#if defined(__HIP_DEVICE_COMPILE__) && QARVD_NO_STORE != 2
    typedef unsigned int v4u_t __attribute__((ext_vector_type(4)));
    // (diagnostic build QARVD_NO_STORE = 1: an empty range, so every store is issued and then dropped)
    const __amdgpu_buffer_rsrc_t r = __builtin_amdgcn_make_buffer_rsrc(base, 0, QARVD_NO_STORE == 1 ? 0 : bytes, 0x00020000);
    if (write_through)
        __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(v4u_t, data), r, voffset, soffset, 17);   // sc0 sc1
    else
        __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(v4u_t, data), r, voffset, soffset, QARVD_STORE_AUX);
    // A 16-byte buffer store still reads its data registers in the cycle after it issues.  The compiler
    // keeps that slot free of VALU writes to them only when the scalar offset is an immediate; with a
    // register offset it let one through, and the first dword of some lanes went out overwritten
    // (seen on MI355X as sporadic wrong outputs).  Hold the registers for two more wait states.
    asm volatile("s_nop 1" : : "v"(data));
#else
    (void)base; (void)bytes; (void)voffset; (void)soffset; (void)data; (void)write_through;
#endif
}

// ---- chained-layer epilogue: activation, then the next layer's static-scale INT8 code ---------------------
// Output types of the chained kernels: one byte per element either way; the type only selects the activation
// at compile time (the epilogue is straight-line code, unrolled over the whole wave tile, and a run-time
// choice doubled it past what the instruction cache holds).
struct Int8Out { int8_t v; };          // no activation
struct Int8GeluOut { int8_t v; };      // GELU (tanh form) before the quantization
template <typename T> struct out_is_gelu { static constexpr bool value = false; };
template <> struct out_is_gelu<Int8GeluOut> { static constexpr bool value = true; };

// Per-wave constants of the static-scale quantizer below.
struct StaticQuant {
    float s, rs, bound;      // the scale, RN(1 / s) by IEEE division, RN(127 s)
};
__device__ __forceinline__ StaticQuant make_static_quant(float s)
{
    return StaticQuant{s, 1.0f / s, 127.0f * s};
}

// Four fp32 results -> four INT8 codes in one dword (byte e = code of y[e]):
//     code = clip(rint(a / s), -127, 127),  a = y (the IEEE fp32 quotient, exactly) or gelu(y) (see below).
// The epilogue is bound by vector-ALU issue (a wave64 instruction occupies its SIMD for four cycles and the
// code is unrolled over 128 values per lane), so the quotient is not taken with the ~13-instruction division
// sequence but as a product with RN(1 / s) corrected twice with fused multiply-adds,
//     q0 = a rs;  q1 = q0 + (a - q0 s) rs;  q2 = q1 + (a - q1 s) rs,
// which IS the correctly rounded quotient RN(a / s): rs has a relative error below 2^-24, so q0 is within
// 1.5 ulp of a / s; the first step leaves q1 a faithful rounding (the residual, rounded or not, puts
// q0 + r rs within 2^-21 ulp of a / s before the rounding), and for a faithful q1 the residual a - q1 s is
// exact and the second step rounds correctly (Markstein's theorem on FMA division).  No intermediate can
// overflow because a is first clamped to +-RN(127 s): beyond that bound the code is +-127 on both sides, and
// at the bound the quotient is within 2^-23 of 127, so no clip of the result is needed either.  Residuals
// stay exact down to s = 1e-30 (their last bit is above 2^-149).  Adding 1.5 * 2^23 rounds half-to-even and
// leaves the two's-complement code in the low byte of the sum.
//
// With GELU (tanh form) the activation and the quotient share one reciprocal:
//   gelu(x) = x * sigma(2u),  u = sqrt(2/pi) (x + 0.044715 x^3),  sigma(z) = 1 / (1 + exp(-z)),
//   exp(-z) = 2^t,  t = x (C0 + C1 x^2)  (C0 = -2 log2(e) sqrt(2/pi), C1 = 0.044715 C0),
//   gelu(x) / s = x / (s + s 2^t)
// with the hardware 2^t and reciprocal (1 ulp each; 2^t overflows to inf and underflows to 0 where sigma is 0
// and 1 to working precision).  Against the real-valued gelu(x) / s: t carries at most four roundings
// (2.4e-7 |t|), which 2^t turns into a relative error of 1.7e-7 |t| on exp(-z); sigma damps that by
// exp(-z) / (1 + exp(-z)), and where |t| is large either that factor or the result itself is tiny; 2^t, the
// fma, the reciprocal and the product add under 4e-7.  The quotient is within (4e-7 + 2e-6 |gelu(x)|) / s of
// the definition's, so the code can differ from the one rounded from the exact activation, by one, only
// where that quotient is this close to a rounding boundary (the rule the parity tests apply).
template <bool GELU>
__device__ __forceinline__ unsigned quantize4_static(const float (&y)[4], const StaticQuant &sq)
{
    constexpr float MAGIC = 12582912.0f;      // 1.5 * 2^23
    float m[4];
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        if constexpr (GELU) {
            const float x = y[e];
            const float inner = fmaf(-0.102943240f, x * x, -2.30220820f);
            const float d = fmaf(sq.s, __builtin_amdgcn_exp2f(x * inner), sq.s);
            const float q = x * __builtin_amdgcn_rcpf(d);
            m[e] = __builtin_amdgcn_fmed3f(q, -127.0f, 127.0f) + MAGIC;
        } else {
            const float a = __builtin_amdgcn_fmed3f(y[e], -sq.bound, sq.bound);
            const float q0 = a * sq.rs;
            const float q1 = fmaf(fmaf(-q0, sq.s, a), sq.rs, q0);
            const float q2 = fmaf(fmaf(-q1, sq.s, a), sq.rs, q1);
            m[e] = q2 + MAGIC;
        }
    }
    // byte 0 of each sum, gathered: v_perm_b32 picks bytes 0..3 from its second operand, 4..7 from its first
    const unsigned lo = __builtin_amdgcn_perm(__float_as_uint(m[1]), __float_as_uint(m[0]), 0x0c0c0400u);
    const unsigned hi = __builtin_amdgcn_perm(__float_as_uint(m[3]), __float_as_uint(m[2]), 0x0c0c0400u);
    return __builtin_amdgcn_perm(hi, lo, 0x05040100u);
}

// two fp32 -> packed bf16, round-to-nearest-even (one v_cvt_pk_bf16_f32)
__device__ __forceinline__ uint32_t cvt_pk_bf16(float a, float b)
{
    v2f f = {a, b};
    v2bf h = __builtin_convertvector(f, v2bf);
    return __builtin_bit_cast(uint32_t, h);
}

// Outputs up to 40 MB are stored write-through (see buffer_store16): 4680 x 1536 and 1560 x 8960 bf16 gain
// 1-2 us, 4680 x 8960 (84 MB) loses 3.
inline int32_t store_write_through(const GemmArgs &g, int elem_bytes)
{
    return (size_t)g.M * (size_t)g.N * (size_t)elem_bytes <= ((size_t)40 << 20) ? 1 : 0;
}

// persistent grid size: as many workgroups as the chip holds at once (a multiple of the XCD count,
// so that the tiles one workgroup walks through stay on its XCD), at most one per tile
inline qarvd_status persistent_grid(int tiles, int wg_per_cu, int *grid)
{
    int cus = 0;
    if (qarvd_status st = qarvd_current_device(nullptr, &cus); st != QARVD_OK) return st;
    const int slots = cus * wg_per_cu / 8 * 8;
    *grid = tiles < slots || slots < 8 ? tiles : slots;
    // More tiles than slots: the number of rounds is fixed by the slot count, so use only as many workgroups as
    // spread the tiles evenly over those rounds (665 tiles: 224 workgroups x 3 instead of 256 with 103 of them
    // idle in the last round).  The chip is power-limited on real data and the CUs left empty raise the clock of
    // the others: 380 tiles of 256x256 at K = 5120 take 122 us on 192 workgroups against 128 us on 256.
    if (tiles > slots && slots >= 8) {
        const int rounds = (tiles + slots - 1) / slots;
        const int even = ((tiles + rounds - 1) / rounds + 7) / 8 * 8;
        if (even < *grid) *grid = even;
    }
    return QARVD_OK;
}

}  // namespace qarvd_gemm
