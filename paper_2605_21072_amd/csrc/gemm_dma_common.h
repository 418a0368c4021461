// Device helpers shared by the LDS-direct GEMM kernels (gfx950).
#pragma once
#include "gemm_common.h"

namespace qarvd_gemm {

#ifndef QARVD_PROF
#define QARVD_PROF 0
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
__device__ __forceinline__ void buffer_store16(void *base, int bytes, int voffset, int soffset, v4i data)
{
#if defined(__HIP_DEVICE_COMPILE__)
    typedef unsigned int v4u_t __attribute__((ext_vector_type(4)));
    const __amdgpu_buffer_rsrc_t r = __builtin_amdgcn_make_buffer_rsrc(base, 0, bytes, 0x00020000);
    __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(v4u_t, data), r, voffset, soffset, 0);
    // A 16-byte buffer store still reads its data registers in the cycle after it issues.  The compiler
    // keeps that slot free of VALU writes to them only when the scalar offset is an immediate; with a
    // register offset it let one through, and the first dword of some lanes went out overwritten
    // (seen on MI355X as sporadic wrong outputs).  Hold the registers for two more wait states.
    asm volatile("s_nop 1" : : "v"(data));
#else
    (void)base; (void)bytes; (void)voffset; (void)soffset; (void)data;
#endif
}

// two fp32 -> packed bf16, round-to-nearest-even (one v_cvt_pk_bf16_f32)
__device__ __forceinline__ uint32_t cvt_pk_bf16(float a, float b)
{
    v2f f = {a, b};
    v2bf h = __builtin_convertvector(f, v2bf);
    return __builtin_bit_cast(uint32_t, h);
}

// persistent grid size: as many workgroups as the chip holds at once (a multiple of the XCD count,
// so that the tiles one workgroup walks through stay on its XCD), at most one per tile
inline qarvd_status persistent_grid(int tiles, int wg_per_cu, int *grid)
{
    int dev = 0;
    QARVD_HIP_TRY(hipGetDevice(&dev));
    static int cu_count[64] = {0};              // per device, filled on first use (same value from any thread)
    int cus = (dev >= 0 && dev < 64) ? cu_count[dev] : 0;
    if (cus <= 0) {
        QARVD_HIP_TRY(hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev));
        if (dev >= 0 && dev < 64) cu_count[dev] = cus;
    }
    const int slots = cus * wg_per_cu / 8 * 8;
    *grid = tiles < slots || slots < 8 ? tiles : slots;
    return QARVD_OK;
}

}  // namespace qarvd_gemm
