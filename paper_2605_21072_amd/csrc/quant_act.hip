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
    int32_t store_wt;      // 1: Xq leaves through write-through stores (see store_q)
};

// Stores of the quantized rows.  A kernel ends with a write-back of what its XCDs' L2s still hold, and the
// consumer (the GEMM, on any XCD) reads Xq from memory either way; for an Xq of a few MB that write-back is
// 1-2 us at the end of a 9 us kernel.  Write-through stores (sc0 sc1) send the bytes on while the kernel still
// computes.  Used when the whole Xq is at most 40 MB (beyond that the extra traffic during the kernel costs
// more than the tail); `off` is the byte offset from a.Xq (the host checked that it fits 31 bits).
template <typename V>
__device__ __forceinline__ void store_q(const ActArgs &a, size_t off, V v)
{
    static_assert(sizeof(V) == 16 || sizeof(V) == 4, "16-byte image chunks or 4-byte words");
#if defined(__HIP_DEVICE_COMPILE__)
    if (a.store_wt) {
        const __amdgpu_buffer_rsrc_t r = __builtin_amdgcn_make_buffer_rsrc(a.Xq, 0, 0x7fffffff, 0x00020000);
        if constexpr (sizeof(V) == 16) {
            typedef unsigned int v4u_t __attribute__((ext_vector_type(4)));
            const v4u_t d = __builtin_bit_cast(v4u_t, v);
            __builtin_amdgcn_raw_buffer_store_b128(d, r, (int)off, 0, 17);
            asm volatile("s_nop 1" : : "v"(d));      // a 16-byte store reads its data registers a cycle late
        } else {
            __builtin_amdgcn_raw_buffer_store_b32(__builtin_bit_cast(unsigned int, v), r, (int)off, 0, 17);
        }
        return;
    }
#endif
    *reinterpret_cast<V *>(a.Xq + off) = v;
}

// Workgroup-wide max of a non-negative value; `red` holds one float per wave.
template <int NWAVE = 4>
__device__ __forceinline__ float block_max(float v, float *red)
{
    v = wave_max(v);
    const int wave = threadIdx.x >> 6;
    if ((threadIdx.x & 63) == 0) red[wave] = v;
    __syncthreads();
    float r = red[0];
#pragma unroll
    for (int w = 1; w < NWAVE; ++w) r = fmaxf(r, red[w]);
    return r;
}

// Register-resident rows: a workgroup of NT threads owns a token row at a time, CH chunks of 4
// channels per thread (K <= CH*NT*4, K % 4 == 0).  IDENT: no permutation -- the quantized bytes
// go straight from registers to memory (4 bytes per lane, contiguous over the wave) and no LDS
// image or position table exists.  PosT is uint16_t when the packed extent fits, else uint32_t.
template <typename T, typename PosT, int CH, int NT, bool STATIC, bool IDENT>
__global__ __launch_bounds__(NT) void quant_act_rows_kernel(ActArgs a)
{
    constexpr int NWAVE = NT / 64;
    extern __shared__ __align__(16) unsigned char smem[];
    // layout (permuted): qbuf[2][kp] | pos[K] | red[2][NWAVE];  (identity): red[2][NWAVE]
    const size_t img_bytes = IDENT ? 0 : 2 * (size_t)a.kp;
    const size_t pos_bytes = IDENT ? 0 : (((size_t)a.K * sizeof(PosT) + 15) & ~(size_t)15);
    int8_t *qbuf = reinterpret_cast<int8_t *>(smem);
    PosT *pos = reinterpret_cast<PosT *>(smem + img_bytes);
    float *red = reinterpret_cast<float *>(smem + img_bytes + pos_bytes);
    const int tid = threadIdx.x;
    const int K = a.K, kp = a.kp;

    const T *X = reinterpret_cast<const T *>(a.X);
    auto load_row = [&](int m, float4 (&v)[CH]) {
        const T *x = X + (size_t)m * a.ldx;
#pragma unroll
        for (int c = 0; c < CH; ++c) {
            const int k = 4 * (tid + c * NT);
            if (k < K) v[c] = Vec4Loader<T>::load(x + k);
        }
    };
    float4 v[CH], vn[CH];
    int m = blockIdx.x;

    if constexpr (!IDENT) {
        // channel -> packed position (a perm that is not a bijection gives undefined bytes, never an
        // out-of-range LDS access: every entry starts at a valid position and bad indices are skipped).
        // perm is fetched first, four entries per lane, then the first row: both are in flight while the
        // table and the row images are initialised, and the table is complete before the row lands.
        const bool pvec = a.perm && (reinterpret_cast<uintptr_t>(a.perm) & 15) == 0;
        int4 pv[CH];
        if (pvec) {
#pragma unroll
            for (int c = 0; c < CH; ++c) {
                const int i4 = tid + c * NT;
                if (4 * i4 < K) pv[c] = reinterpret_cast<const int4 *>(a.perm)[i4];
            }
        }
        if (m < a.M) load_row(m, v);
        for (int k = tid; k < K; k += NT) pos[k] = (PosT)(a.perm ? a.n_off : k);
        // zero both row images once: padding bytes are never overwritten afterwards
        for (int i = tid; i < (2 * kp) / 16; i += NT) reinterpret_cast<uint4 *>(qbuf)[i] = make_uint4(0, 0, 0, 0);
        __syncthreads();
        if (a.perm) {
            auto place = [&](int p, int k) {
                if ((unsigned)k < (unsigned)K) pos[k] = (PosT)(p < a.K_o ? p : a.n_off + (p - a.K_o));
            };
            if (pvec) {
#pragma unroll
                for (int c = 0; c < CH; ++c) {
                    const int p = 4 * (tid + c * NT);
                    if (p < K) {
                        place(p, pv[c].x);
                        place(p + 1, pv[c].y);
                        place(p + 2, pv[c].z);
                        place(p + 3, pv[c].w);
                    }
                }
            } else {
                for (int p = tid; p < K; p += NT) place(p, a.perm[p]);
            }
            __syncthreads();
        }
    } else {
        if (m < a.M) load_row(m, v);
    }

    int buf = 0;
    for (; m < a.M; m += gridDim.x, buf ^= 1) {
        float amax = 0.0f;
#pragma unroll
        for (int c = 0; c < CH; ++c) {
            const int k = 4 * (tid + c * NT);
            if (k < K) amax = fmaxf(amax, fmaxf(fmaxf(fabsf(v[c].x), fabsf(v[c].y)), fmaxf(fabsf(v[c].z), fabsf(v[c].w))));
        }
        // the next row's loads fly under this row's reduction, quantization and copy-out
        const bool more = m + (int)gridDim.x < a.M;
        if (more) load_row(m + gridDim.x, vn);
        float s;
        if (STATIC) {
            s = a.static_scale;
        } else {
            amax = block_max<NWAVE>(amax, red + NWAVE * buf);
            s = amax / 127.0f;
            if (tid == 0) a.s_x[m] = s;
        }
        const bool zero = s == 0.0f;                       // all-zero token (or zero static scale): q = 0
        const float r = __builtin_amdgcn_rcpf(s);
        const size_t out = (size_t)m * a.ldxq;             // byte offset of the row in Xq
        if constexpr (IDENT) {
#pragma unroll
            for (int c = 0; c < CH; ++c) {
                const int k = 4 * (tid + c * NT);
                if (k < kp) {                                // k >= K: zero padding up to the packed extent
                    uint32_t w = 0;
                    if (k < K && !zero) {
                        w = (uint32_t)(quantize_i8_fast(v[c].x, s, r) & 255) | ((uint32_t)(quantize_i8_fast(v[c].y, s, r) & 255) << 8) |
                            ((uint32_t)(quantize_i8_fast(v[c].z, s, r) & 255) << 16) | ((uint32_t)(quantize_i8_fast(v[c].w, s, r) & 255) << 24);
                    }
                    store_q(a, out + k, w);
                }
            }
        } else {
            int8_t *q = qbuf + (size_t)buf * kp;
#pragma unroll
            for (int c = 0; c < CH; ++c) {
                const int k = 4 * (tid + c * NT);
                if (k < K) {
                    q[pos[k + 0]] = zero ? (int8_t)0 : (int8_t)quantize_i8_fast(v[c].x, s, r);
                    q[pos[k + 1]] = zero ? (int8_t)0 : (int8_t)quantize_i8_fast(v[c].y, s, r);
                    q[pos[k + 2]] = zero ? (int8_t)0 : (int8_t)quantize_i8_fast(v[c].z, s, r);
                    q[pos[k + 3]] = zero ? (int8_t)0 : (int8_t)quantize_i8_fast(v[c].w, s, r);
                }
            }
            __syncthreads();
            for (int i = tid; i < kp / 16; i += NT) store_q(a, out + 16 * (size_t)i, reinterpret_cast<const uint4 *>(q)[i]);
        }
        if (more) {
#pragma unroll
            for (int c = 0; c < CH; ++c) v[c] = vn[c];
        }
    }
}

// Wave-per-row variant for short rows (K <= CH*256, K % 4 == 0): each of the four wavefronts of a
// workgroup owns a token row at a time, so the absmax is a pure shuffle reduction, the packed row
// image is wave-private and no workgroup barrier is needed after the position table is built.
template <typename T, int CH, bool STATIC>
__global__ __launch_bounds__(TPB) void quant_act_wave_kernel(ActArgs a)
{
    extern __shared__ __align__(16) unsigned char smem[];
    // layout: image[4][kp] | pos[K] (uint16)
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int K = a.K, kp = a.kp;
    int8_t *img = reinterpret_cast<int8_t *>(smem) + (size_t)wave * kp;
    uint16_t *pos = reinterpret_cast<uint16_t *>(smem + 4 * (size_t)kp);
    const T *X = reinterpret_cast<const T *>(a.X);
    const int wave_id = blockIdx.x * 4 + wave, n_waves = gridDim.x * 4;

    // perm is fetched first (four entries per lane), then the first row: both are in flight while the table
    // and the images are initialised, and the table is complete before the row lands
    constexpr int PCH = (CH + 3) / 4;
    const bool pvec = a.perm && (reinterpret_cast<uintptr_t>(a.perm) & 15) == 0;
    int4 pv[PCH];
    if (pvec) {
#pragma unroll
        for (int c = 0; c < PCH; ++c) {
            const int i4 = tid + c * TPB;
            if (4 * i4 < K) pv[c] = reinterpret_cast<const int4 *>(a.perm)[i4];
        }
    }
    float4 v[CH];
    auto load_row = [&](int m) {
        const T *x = X + (size_t)m * a.ldx;
#pragma unroll
        for (int c = 0; c < CH; ++c) {
            const int k = 4 * (lane + c * 64);
            if (k < K) v[c] = Vec4Loader<T>::load(x + k);
        }
    };
    int m = wave_id;
    if (m < a.M) load_row(m);

    for (int k = tid; k < K; k += TPB) pos[k] = (uint16_t)(a.perm ? a.n_off : k);
    for (int i = tid; i < (4 * kp) / 16; i += TPB) reinterpret_cast<uint4 *>(smem)[i] = make_uint4(0, 0, 0, 0);
    __syncthreads();
    if (a.perm) {
        auto place = [&](int p, int k) {
            if ((unsigned)k < (unsigned)K) pos[k] = (uint16_t)(p < a.K_o ? p : a.n_off + (p - a.K_o));
        };
        if (pvec) {
#pragma unroll
            for (int c = 0; c < PCH; ++c) {
                const int p = 4 * (tid + c * TPB);
                if (p < K) {
                    place(p, pv[c].x);
                    place(p + 1, pv[c].y);
                    place(p + 2, pv[c].z);
                    place(p + 3, pv[c].w);
                }
            }
        } else {
            for (int p = tid; p < K; p += TPB) place(p, a.perm[p]);
        }
        __syncthreads();
    }

    for (; m < a.M; m += n_waves) {
        float amax = 0.0f;
#pragma unroll
        for (int c = 0; c < CH; ++c) {
            const int k = 4 * (lane + c * 64);
            if (k < K) amax = fmaxf(amax, fmaxf(fmaxf(fabsf(v[c].x), fabsf(v[c].y)), fmaxf(fabsf(v[c].z), fabsf(v[c].w))));
        }
        float s;
        if (STATIC) {
            s = a.static_scale;
        } else {
            amax = wave_max(amax);
            s = amax / 127.0f;
            if (lane == 0) a.s_x[m] = s;
        }
        const bool zero = s == 0.0f;
        const float r = __builtin_amdgcn_rcpf(s);
#pragma unroll
        for (int c = 0; c < CH; ++c) {
            const int k = 4 * (lane + c * 64);
            if (k < K) {
                img[pos[k + 0]] = zero ? (int8_t)0 : (int8_t)quantize_i8_fast(v[c].x, s, r);
                img[pos[k + 1]] = zero ? (int8_t)0 : (int8_t)quantize_i8_fast(v[c].y, s, r);
                img[pos[k + 2]] = zero ? (int8_t)0 : (int8_t)quantize_i8_fast(v[c].z, s, r);
                img[pos[k + 3]] = zero ? (int8_t)0 : (int8_t)quantize_i8_fast(v[c].w, s, r);
            }
        }
        if (m + n_waves < a.M) load_row(m + n_waves);     // next row in flight during the copy-out
        // the image is private to this wave and LDS operations of one wave complete in order
        const size_t out = (size_t)m * a.ldxq;
        for (int i = lane; i < kp / 16; i += 64) store_q(a, out + 16 * (size_t)i, reinterpret_cast<const uint4 *>(img)[i]);
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

int num_cu()
{
    int cus = 0;
    return (qarvd_current_device(nullptr, &cus) == QARVD_OK && cus > 0) ? cus : 256;
}

constexpr size_t LDS_LIMIT = 160 * 1024;

template <typename T, typename PosT, int CH, int NT, bool STATIC, bool IDENT>
qarvd_status launch_rows_one(const ActArgs &a, hipStream_t st)
{
    const size_t lds = (IDENT ? 0 : 2 * (size_t)a.kp + (((size_t)a.K * sizeof(PosT) + 15) & ~(size_t)15)) + 2 * (NT / 64) * sizeof(float);
    auto kern = quant_act_rows_kernel<T, PosT, CH, NT, STATIC, IDENT>;
    if (lds > 64 * 1024) {      // the limit goes to the hardware's whole LDS, once per kernel and device
        static unsigned long long raised = 0;
        if (qarvd_status s_a = qarvd_raise_lds_limit_once(kern, (int)LDS_LIMIT, raised); s_a != QARVD_OK) return s_a;
    }
    int occ = (int)(LDS_LIMIT / (lds < 1024 ? 1024 : lds));
    const int occ_threads = 2048 / NT;
    occ = occ < 1 ? 1 : (occ > occ_threads ? occ_threads : occ);
    // as many workgroups as the chip holds, trimmed so that all of them walk the same number of rows
    // (4680 rows on 1024 slots: 936 workgroups of exactly 5 rows instead of 1024 of 4 or 5)
    const int slots = num_cu() * occ;
    const int rounds = (a.M + slots - 1) / slots;
    const int grid = (a.M + rounds - 1) / rounds;
    hipLaunchKernelGGL(kern, dim3(grid), dim3(NT), lds, st, a);
    return qarvd_launch_status();
}

template <typename T, typename PosT, int CH, int NT, bool STATIC>
qarvd_status launch_rows(const ActArgs &a, hipStream_t st)
{
    // no permutation and a packed extent that whole 4-byte words cover: straight register -> memory path
    if (!a.perm && a.kp <= CH * NT * 4) return launch_rows_one<T, PosT, CH, NT, STATIC, true>(a, st);
    return launch_rows_one<T, PosT, CH, NT, STATIC, false>(a, st);
}

template <typename T, int CH, bool STATIC>
qarvd_status launch_wave(const ActArgs &a, hipStream_t st)
{
    const size_t lds = 4 * (size_t)a.kp + (((size_t)a.K * 2 + 15) & ~(size_t)15);
    auto kern = quant_act_wave_kernel<T, CH, STATIC>;
    int occ = (int)(LDS_LIMIT / lds);
    occ = occ < 1 ? 1 : (occ > 8 ? 8 : occ);
    int grid = num_cu() * occ;
    const int need = (a.M + 3) / 4;
    if (grid > need) grid = need;
    hipLaunchKernelGGL(kern, dim3(grid), dim3(TPB), lds, st, a);
    return qarvd_launch_status();
}

template <typename T, bool STATIC>
qarvd_status dispatch(const ActArgs &a, hipStream_t st)
{
    const bool vec_ok = (a.K % 4 == 0) && (a.ldx % 4 == 0) && ((reinterpret_cast<uintptr_t>(a.X) % (4 * sizeof(T))) == 0);
    const size_t lds16 = 2 * (size_t)a.kp + (size_t)a.K * 2 + 64;
    if (vec_ok && a.kp <= 65535 && a.K <= 16 * 1024 && lds16 <= LDS_LIMIT) {
        if (a.perm && a.K <= 6 * 256) return launch_wave<T, 6, STATIC>(a, st);
        if (a.perm && a.K <= 12 * 256) return launch_wave<T, 12, STATIC>(a, st);
        if (!a.perm && a.K <= 5 * 1024) return launch_rows<T, uint16_t, 5, 256, STATIC>(a, st);
        if (a.K <= 6 * 1024) return launch_rows<T, uint16_t, 3, 512, STATIC>(a, st);
        if (a.K <= 10 * 1024) return launch_rows<T, uint16_t, 5, 512, STATIC>(a, st);
        return launch_rows<T, uint16_t, 4, 1024, STATIC>(a, st);
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
    a.store_wt = ((size_t)M * (size_t)g.kp <= ((size_t)40 << 20) && (size_t)M * (size_t)ldxq < ((size_t)1 << 31)) ? 1 : 0;
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
