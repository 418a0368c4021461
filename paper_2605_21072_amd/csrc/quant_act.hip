// Activation quantization for gfx950: fused gather-permute + per-token dynamic (or static)
// symmetric INT8 (appendix "Quantization Kernels", kernel (i) and the online permutation;
// Sec. 2.2 Eq. (quantization)).
//
// HBM-bound: every X element is read from memory exactly once and one byte is written.
//
// One 256-thread workgroup owns whole token rows.  A row is read with coalesced 16-byte
// loads in natural channel order and stays in registers; the per-token absmax is a wavefront
// shuffle reduction plus a 4-entry LDS exchange; each value is quantized and its byte is
// scattered into an LDS image of the packed row at the position its channel takes in the
// [outlier | normal] order; the image is then written out with coalesced 16-byte stores.
// The channel -> packed-position table is built once per workgroup in LDS from `perm`.
#include "qarvd_common.h"

namespace {

constexpr int TPB = 256;

template <typename T> struct Vec4Loader;
template <> struct Vec4Loader<float> {
    static __device__ __forceinline__ float4 load(const float *p) { return *reinterpret_cast<const float4 *>(p); }
    static __device__ __forceinline__ float load1(const float *p) { return *p; }
};
template <> struct Vec4Loader<uint16_t> {   // bf16 bit patterns, widened exactly
    static __device__ __forceinline__ float4 load(const uint16_t *p)
    {
        uint2 u = *reinterpret_cast<const uint2 *>(p);
        float4 f;
        f.x = __uint_as_float(u.x << 16);
        f.y = __uint_as_float(u.x & 0xFFFF0000u);
        f.z = __uint_as_float(u.y << 16);
        f.w = __uint_as_float(u.y & 0xFFFF0000u);
        return f;
    }
    static __device__ __forceinline__ float load1(const uint16_t *p) { return bf16_bits_to_f32(*p); }
};

struct ActArgs {
    const void *X;
    int64_t ldx;
    const int32_t *perm;
    int8_t *Xq;
    int64_t ldxq;
    float *s_x;
    float static_scale;
    int32_t M, K, K_o, n_off, kp;
};

// Workgroup-wide max of a non-negative value; `red` holds one float per wave.
__device__ __forceinline__ float block_max(float v, float *red)
{
    v = wave_max(v);
    const int wave = threadIdx.x >> 6;
    if ((threadIdx.x & 63) == 0) red[wave] = v;
    __syncthreads();
    float r = fmaxf(fmaxf(red[0], red[1]), fmaxf(red[2], red[3]));
    return r;
}

// Register-resident rows: CH chunks of 4 channels per thread (K <= CH*1024, K % 4 == 0).
// PosT is uint16_t when the packed extent fits, else uint32_t.
template <typename T, typename PosT, int CH, bool STATIC>
__global__ __launch_bounds__(TPB) void quant_act_rows_kernel(ActArgs a)
{
    extern __shared__ __align__(16) unsigned char smem[];
    // layout: qbuf[2][kp] | pos[K] | red[2][4]
    int8_t *qbuf = reinterpret_cast<int8_t *>(smem);
    PosT *pos = reinterpret_cast<PosT *>(smem + 2 * (size_t)a.kp);
    float *red = reinterpret_cast<float *>(smem + 2 * (size_t)a.kp + (((size_t)a.K * sizeof(PosT) + 15) & ~(size_t)15));
    const int tid = threadIdx.x;
    const int K = a.K, kp = a.kp;

    // channel -> packed position (a perm that is not a bijection gives undefined bytes, never an
    // out-of-range LDS access: every entry starts at a valid position and bad indices are skipped)
    if (a.perm) {
        for (int k = tid; k < K; k += TPB) pos[k] = (PosT)a.n_off;
        __syncthreads();
        for (int p = tid; p < K; p += TPB) {
            const int k = a.perm[p];
            if ((unsigned)k < (unsigned)K) pos[k] = (PosT)(p < a.K_o ? p : a.n_off + (p - a.K_o));
        }
    } else {
        for (int k = tid; k < K; k += TPB) pos[k] = (PosT)k;
    }
    // zero both row images once: padding bytes are never overwritten afterwards
    for (int i = tid; i < (2 * kp) / 16; i += TPB) reinterpret_cast<uint4 *>(qbuf)[i] = make_uint4(0, 0, 0, 0);
    __syncthreads();

    const T *X = reinterpret_cast<const T *>(a.X);
    int buf = 0;
    for (int m = blockIdx.x; m < a.M; m += gridDim.x, buf ^= 1) {
        const T *x = X + (size_t)m * a.ldx;
        float4 v[CH];
        float amax = 0.0f;
#pragma unroll
        for (int c = 0; c < CH; ++c) {
            const int k = 4 * (tid + c * TPB);
            if (k < K) {
                v[c] = Vec4Loader<T>::load(x + k);
                amax = fmaxf(amax, fmaxf(fmaxf(fabsf(v[c].x), fabsf(v[c].y)), fmaxf(fabsf(v[c].z), fabsf(v[c].w))));
            }
        }
        float s;
        if (STATIC) {
            s = a.static_scale;
        } else {
            amax = block_max(amax, red + 4 * buf);
            s = amax / 127.0f;
            if (tid == 0) a.s_x[m] = s;
        }
        int8_t *q = qbuf + (size_t)buf * kp;
#pragma unroll
        for (int c = 0; c < CH; ++c) {
            const int k = 4 * (tid + c * TPB);
            if (k < K) {
                q[pos[k + 0]] = (int8_t)quantize_i8(v[c].x, s);
                q[pos[k + 1]] = (int8_t)quantize_i8(v[c].y, s);
                q[pos[k + 2]] = (int8_t)quantize_i8(v[c].z, s);
                q[pos[k + 3]] = (int8_t)quantize_i8(v[c].w, s);
            }
        }
        __syncthreads();
        int8_t *out = a.Xq + (size_t)m * a.ldxq;
        for (int i = tid; i < kp / 16; i += TPB)
            reinterpret_cast<uint4 *>(out)[i] = reinterpret_cast<const uint4 *>(q)[i];
    }
}

// General fallback (any K, any alignment): one workgroup per row, two passes over the row
// (the second is served by the cache), gather through perm from global memory.
template <typename T, bool STATIC>
__global__ __launch_bounds__(TPB) void quant_act_generic_kernel(ActArgs a)
{
    __shared__ float red[4];
    const int tid = threadIdx.x;
    const T *X = reinterpret_cast<const T *>(a.X);
    for (int m = blockIdx.x; m < a.M; m += gridDim.x) {
        const T *x = X + (size_t)m * a.ldx;
        float s;
        if (STATIC) {
            s = a.static_scale;
        } else {
            float amax = 0.0f;
            for (int k = tid; k < a.K; k += TPB) amax = fmaxf(amax, fabsf(Vec4Loader<T>::load1(x + k)));
            amax = block_max(amax, red);
            s = amax / 127.0f;
            if (tid == 0) a.s_x[m] = s;
            __syncthreads();   // red is reused by the next row
        }
        int8_t *out = a.Xq + (size_t)m * a.ldxq;
        for (int pp = tid; pp < a.kp; pp += TPB) {
            int p = -1;                                   // logical packed index, -1 = padding
            if (pp < a.K_o) p = pp;
            else if (pp >= a.n_off && pp - a.n_off < a.K - a.K_o) p = a.K_o + (pp - a.n_off);
            int8_t q = 0;
            if (p >= 0) {
                const int k = a.perm ? a.perm[p] : p;
                if ((unsigned)k < (unsigned)a.K) q = (int8_t)quantize_i8(Vec4Loader<T>::load1(x + k), s);
            }
            out[pp] = q;
        }
    }
}

int g_num_cu = 0;
int num_cu()
{
    if (g_num_cu == 0) {
        int dev = 0;
        hipDeviceProp_t prop;
        if (hipGetDevice(&dev) == hipSuccess && hipGetDeviceProperties(&prop, dev) == hipSuccess)
            g_num_cu = prop.multiProcessorCount;
        else
            g_num_cu = 256;
    }
    return g_num_cu;
}

constexpr size_t LDS_LIMIT = 160 * 1024;

template <typename T, typename PosT, int CH, bool STATIC>
qarvd_status launch_rows(const ActArgs &a, hipStream_t st)
{
    const size_t lds = 2 * (size_t)a.kp + (((size_t)a.K * sizeof(PosT) + 15) & ~(size_t)15) + 8 * sizeof(float);
    auto kern = quant_act_rows_kernel<T, PosT, CH, STATIC>;
    if (lds > 64 * 1024)
        QARVD_HIP_TRY(hipFuncSetAttribute(reinterpret_cast<const void *>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
    int occ = (int)(LDS_LIMIT / lds);
    occ = occ < 1 ? 1 : (occ > 8 ? 8 : occ);
    int grid = num_cu() * occ;
    if (grid > a.M) grid = a.M;
    hipLaunchKernelGGL(kern, dim3(grid), dim3(TPB), lds, st, a);
    return qarvd_launch_status();
}

template <typename T, bool STATIC>
qarvd_status dispatch(const ActArgs &a, hipStream_t st)
{
    const bool vec_ok = (a.K % 4 == 0) && (a.ldx % 4 == 0) && ((reinterpret_cast<uintptr_t>(a.X) % (4 * sizeof(T))) == 0);
    const size_t lds16 = 2 * (size_t)a.kp + (size_t)a.K * 2 + 64;
    if (vec_ok && a.kp <= 65535 && a.K <= 14 * 1024 && lds16 <= LDS_LIMIT) {
        if (a.K <= 2 * 1024) return launch_rows<T, uint16_t, 2, STATIC>(a, st);
        if (a.K <= 5 * 1024) return launch_rows<T, uint16_t, 5, STATIC>(a, st);
        if (a.K <= 9 * 1024) return launch_rows<T, uint16_t, 9, STATIC>(a, st);
        return launch_rows<T, uint16_t, 14, STATIC>(a, st);
    }
    int grid = a.M < num_cu() * 8 ? a.M : num_cu() * 8;
    hipLaunchKernelGGL((quant_act_generic_kernel<T, STATIC>), dim3(grid), dim3(TPB), 0, st, a);
    return qarvd_launch_status();
}

qarvd_status quant_act_common(const void *X, qarvd_dtype xdt, int32_t M, int32_t K, int64_t ldx,
                              const int32_t *perm, int32_t K_o, int8_t *Xq, int64_t ldxq, float *s_x,
                              bool is_static, float scale, void *stream)
{
    if (!X || !Xq || (!is_static && !s_x)) return QARVD_ERR_INVALID_ARG;
    if (M <= 0 || K <= 0 || K > QARVD_MAX_K || K_o < 0 || K_o > K || ldx < K) return QARVD_ERR_INVALID_ARG;
    if (!perm && K_o != 0) return QARVD_ERR_INVALID_ARG;
    if (is_static && !(scale >= 0.0f)) return QARVD_ERR_INVALID_ARG;
    const PackedK g = qarvd_packed(K, K_o);
    if (ldxq < g.kp) return QARVD_ERR_INVALID_ARG;
    if (xdt != QARVD_F32 && xdt != QARVD_BF16) return QARVD_ERR_UNSUPPORTED;
    if (!qarvd_aligned16(Xq) || (ldxq % 16) != 0) return QARVD_ERR_UNSUPPORTED;
    const size_t esz = xdt == QARVD_F32 ? 4 : 2;
    if (reinterpret_cast<uintptr_t>(X) % esz) return QARVD_ERR_UNSUPPORTED;
    ActArgs a;
    a.X = X; a.ldx = ldx; a.perm = perm; a.Xq = Xq; a.ldxq = ldxq; a.s_x = s_x; a.static_scale = scale;
    a.M = M; a.K = K; a.K_o = K_o; a.n_off = g.n_off; a.kp = g.kp;
    hipStream_t st = reinterpret_cast<hipStream_t>(stream);
    if (xdt == QARVD_F32)
        return is_static ? dispatch<float, true>(a, st) : dispatch<float, false>(a, st);
    return is_static ? dispatch<uint16_t, true>(a, st) : dispatch<uint16_t, false>(a, st);
}

}  // namespace

extern "C" qarvd_status qarvd_quant_act(const void *X, qarvd_dtype xdt, int32_t M, int32_t K, int64_t ldx,
                                        const int32_t *perm, int32_t K_o, int8_t *Xq, int64_t ldxq,
                                        float *s_x, void *stream)
{
    return quant_act_common(X, xdt, M, K, ldx, perm, K_o, Xq, ldxq, s_x, false, 0.0f, stream);
}

extern "C" qarvd_status qarvd_quant_act_static(const void *X, qarvd_dtype xdt, int32_t M, int32_t K,
                                               int64_t ldx, const int32_t *perm, int32_t K_o, float scale,
                                               int8_t *Xq, int64_t ldxq, void *stream)
{
    return quant_act_common(X, xdt, M, K, ldx, perm, K_o, Xq, ldxq, nullptr, true, scale, stream);
}
