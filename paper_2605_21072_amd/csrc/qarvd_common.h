// Shared host/device helpers of the gfx950 library (not used by the CPU oracle).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/qarvd.h"

#define QARVD_HIP_TRY(expr)                      \
    do {                                         \
        hipError_t e__ = (expr);                 \
        if (e__ != hipSuccess) {                 \
            (void)hipGetLastError();             \
            return QARVD_ERR_HIP;                \
        }                                        \
    } while (0)

static inline qarvd_status qarvd_launch_status()
{
    hipError_t e = hipGetLastError();
    return e == hipSuccess ? QARVD_OK : QARVD_ERR_HIP;
}

// Compute-unit count of the current device.  Device attributes are read once per device and kept for the life
// of the process (the only state the library holds besides which kernels already had their LDS limit raised).
static inline qarvd_status qarvd_current_device(int *dev_out, int *cus_out)
{
    static int cu_count[64] = {0};              // filled on first use; the same value from any thread
    int dev = 0;
    QARVD_HIP_TRY(hipGetDevice(&dev));
    int cus = (dev >= 0 && dev < 64) ? cu_count[dev] : 0;
    if (cus <= 0) {
        QARVD_HIP_TRY(hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev));
        if (dev >= 0 && dev < 64) cu_count[dev] = cus;
    }
    if (dev_out) *dev_out = dev;
    if (cus_out) *cus_out = cus;
    return QARVD_OK;
}

// Raises a kernel's dynamic-LDS limit the first time it is launched on a device instead of on every launch
// (the call costs microseconds of host time, as much as a short kernel).  `done` is one bit per device,
// a static of the calling launcher, so there is one mask per kernel symbol; the attribute only ever grows.
template <typename Kernel>
static inline qarvd_status qarvd_raise_lds_limit_once(Kernel kernel, int bytes, unsigned long long &done)
{
    int dev = 0;
    QARVD_HIP_TRY(hipGetDevice(&dev));
    const unsigned long long bit = (dev >= 0 && dev < 64) ? (1ull << dev) : 0ull;
    if (bit && (__atomic_load_n(&done, __ATOMIC_ACQUIRE) & bit)) return QARVD_OK;
    QARVD_HIP_TRY(hipFuncSetAttribute(reinterpret_cast<const void *>(kernel), hipFuncAttributeMaxDynamicSharedMemorySize, bytes));
    if (bit) __atomic_fetch_or(&done, bit, __ATOMIC_RELEASE);
    return QARVD_OK;
}

static inline bool qarvd_aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

static inline int32_t qarvd_round_up(int32_t x, int32_t m) { return (x + m - 1) / m * m; }

// Packed-row geometry (see the layout comment in qarvd.h).
struct PackedK {
    int32_t K, K_o;
    int32_t n_off;   // start of the normal block
    int32_t kp;      // packed extent, multiple of 128
};
static inline PackedK qarvd_packed(int32_t K, int32_t K_o)
{
    PackedK g;
    g.K = K;
    g.K_o = K_o;
    g.n_off = qarvd_round_up(K_o, 32);
    g.kp = qarvd_round_up(g.n_off + (K - K_o), 128);
    return g;
}

// Eq. (quantization), symmetric, z = 0, clip to [-127,127], round-half-even; s == 0 -> 0.
// The division is the IEEE-correct fp32 division hipcc emits by default.
__device__ __forceinline__ int quantize_i8(float x, float s)
{
    if (s == 0.0f) return 0;
    float r = rintf(x / s);
    r = fminf(fmaxf(r, -127.0f), 127.0f);
    return (int)r;
}

// The same quantizer with the symmetric range of another bit-width: q in [-qmax, qmax], qmax = 2^(b-1) - 1.
__device__ __forceinline__ int quantize_sym(float x, float s, float qmax)
{
    if (s == 0.0f) return 0;
    float r = rintf(x / s);
    r = fminf(fmaxf(r, -qmax), qmax);
    return (int)r;
}

// Same result as quantize_i8, without the ~10-instruction IEEE division on the common path.
//   y' = x * rcp(s) is within |x/s| * 2^-22 <= 127 * 2^-22 < 4e-5 of the true quotient (|x/s| <= 127
//   under an absmax scale; larger quotients only occur with a static scale and are far from any
//   boundary that matters or land in the slow path), and the oracle's RN(x/s) is within 8e-6 of it,
//   so rint(y') == rint(RN(x/s)) whenever y' is at least 1e-4 away from a half-integer.  The few
//   lanes closer than that (about 2 in 10^4) redo the exact division.  `r` must be rcp(s), s > 0.
__device__ __forceinline__ int quantize_i8_fast(float x, float s, float r)
{
    const float y = x * r;
    float q = rintf(y);
    if (!(fabsf(y - q) < 0.4999f)) q = rintf(x / s);   // also taken for NaN / inf intermediates
    q = fminf(fmaxf(q, -127.0f), 127.0f);
    return (int)q;
}

__device__ __forceinline__ float bf16_bits_to_f32(uint16_t h) { return __uint_as_float((uint32_t)h << 16); }

// fp32 -> bf16 bits, round-to-nearest-even (finite inputs).
__device__ __forceinline__ uint32_t f32_to_bf16_bits(float f)
{
    uint32_t u = __float_as_uint(f);
    u += 0x7FFFu + ((u >> 16) & 1u);
    return u >> 16;
}

__device__ __forceinline__ float wave_max(float v)
{
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v = fmaxf(v, __shfl_xor(v, off, 64));
    return v;
}
