// Offline weight step for gfx950 (Sec. 3.2): input-channel L2 norms, Modified-Z-score +
// minimum-magnitude outlier detection (Eqs. (mad), (new_threshold)), alignment of the outlier
// count (Fig. "outlier patterns" caption), [outlier | normal] permutation and dual per-row scales
// with INT8 rounding (Eq. (dual_scale), Eq. (quantization)).
//
// Runs once per layer and is not on the timed path; the kernels favour exact, order-defined
// arithmetic over speed:
//   - a column norm is accumulated by ONE thread in ascending row order in fp64, so the sum has
//     the same rounding sequence as a sequential loop (loads are coalesced across columns);
//   - medians come from exact ranks: rank_i = #{j : x_j > x_i or (x_j == x_i and j < i)} is a
//     bijection onto 0..K-1, scattering by rank sorts the vector, and the detector's flagged set
//     plus its largest-norm fillers is simply {i : rank_i < K_o};
//   - every floating-point expression of the detector is evaluated in fp64 with separate
//     multiply and add (the library is built with -ffp-contract=off).
#include "qarvd_common.h"

namespace {

struct DetectScalars {   // lives in the workspace
    double med, mad, T;
    int32_t n_det, K_o;
};

// ---- norms -------------------------------------------------------------------------------
__global__ __launch_bounds__(64) void column_norm_kernel(const float *__restrict__ W, int N, int K, int64_t ldw,
                                                         float *__restrict__ v)
{
    const int k = blockIdx.x * 64 + threadIdx.x;
    if (k >= K) return;
    const float *w = W + k;
    double S = 0.0;
    int j = 0;
    for (; j + 8 <= N; j += 8) {
        float t[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) t[u] = w[(size_t)(j + u) * ldw];
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            const double d = (double)t[u];
            S = S + d * d;
        }
    }
    for (; j < N; ++j) {
        const double d = (double)w[(size_t)j * ldw];
        S = S + d * d;
    }
    v[k] = (float)sqrt(S);
}

// ---- ranks (descending, ties by smaller index first) and sort-by-rank --------------------
template <typename T>
__global__ __launch_bounds__(256) void rank_desc_kernel(const T *__restrict__ x, int K, int32_t *__restrict__ rank,
                                                        T *__restrict__ sorted_desc)
{
    __shared__ T tile[256];
    const int i = blockIdx.x * 256 + threadIdx.x;
    const T xi = i < K ? x[i] : (T)0;
    int r = 0;
    for (int j0 = 0; j0 < K; j0 += 256) {
        const int j = j0 + threadIdx.x;
        tile[threadIdx.x] = j < K ? x[j] : (T)0;
        __syncthreads();
        const int lim = min(256, K - j0);
        for (int t = 0; t < lim; ++t) {
            const T xj = tile[t];
            r += (xj > xi || (xj == xi && (j0 + t) < i)) ? 1 : 0;
        }
        __syncthreads();
    }
    if (i < K) {
        if (rank) rank[i] = r;
        sorted_desc[r] = xi;
    }
}

// med = median(v) (even K: mean of the two middle values), d = |v - med| in fp64.
__global__ void median_dev_kernel(const float *__restrict__ v, const float *__restrict__ sorted_desc, int K,
                                  DetectScalars *sc, double *__restrict__ d)
{
    // the two middle order statistics are the same pair counted from either end
    const double med = (K & 1) ? (double)sorted_desc[K / 2]
                               : ((double)sorted_desc[K / 2] + (double)sorted_desc[K / 2 - 1]) / 2.0;
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < K) d[i] = fabs((double)v[i] - med);
    if (i == 0) sc->med = med;
}

// MAD, threshold, flagged count, aligned K_o.  One workgroup.
__global__ __launch_bounds__(256) void threshold_kernel(const float *__restrict__ v, const double *__restrict__ sorted_d,
                                                        int K, double c, double alpha, int align, DetectScalars *sc)
{
    __shared__ int cnt[256];
    const double mad = (K & 1) ? sorted_d[K / 2] : (sorted_d[K / 2] + sorted_d[K / 2 - 1]) / 2.0;
    const double med = sc->med;
    double T1 = c * mad;
    T1 = med + T1;
    const double T2 = alpha * med;
    const double T = T1 > T2 ? T1 : T2;
    int n = 0;
    for (int i = threadIdx.x; i < K; i += 256) n += ((double)v[i] > T) ? 1 : 0;
    cnt[threadIdx.x] = n;
    __syncthreads();
    for (int s = 128; s > 0; s >>= 1) {
        if (threadIdx.x < s) cnt[threadIdx.x] += cnt[threadIdx.x + s];
        __syncthreads();
    }
    if (threadIdx.x == 0) {
        const int n_det = cnt[0];
        int K_o = 0;
        if (n_det > 0) {
            K_o = (n_det + align - 1) / align * align;
            if (K_o > K) K_o = K;
        }
        sc->mad = mad;
        sc->T = T;
        sc->n_det = n_det;
        sc->K_o = K_o;
    }
}

__global__ void select_by_rank_kernel(const int32_t *__restrict__ rank, int K, const DetectScalars *sc,
                                      uint8_t *__restrict__ sel)
{
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < K) sel[i] = rank[i] < sc->K_o ? 1 : 0;
}

// Stable partition: perm = [selected ascending | rest ascending]; pos = packed position of each
// channel.  One workgroup of 1024 threads, each owning a contiguous run of channels.
__global__ __launch_bounds__(1024) void build_perm_kernel(const uint8_t *__restrict__ sel, int K, DetectScalars *sc,
                                                          int forced, int32_t *__restrict__ perm,
                                                          int32_t *__restrict__ pos)
{
    __shared__ int part[1024];
    __shared__ int total;
    const int t = threadIdx.x;
    const int per = (K + 1023) / 1024;
    const int b = min(K, t * per), e = min(K, b + per);
    int n = 0;
    for (int k = b; k < e; ++k) n += sel[k] ? 1 : 0;
    part[t] = n;
    __syncthreads();
    if (t == 0) {
        int run = 0;
        for (int i = 0; i < 1024; ++i) {
            const int c = part[i];
            part[i] = run;
            run += c;
        }
        total = run;
        if (forced) sc->K_o = run;
    }
    __syncthreads();
    const int K_o = total;
    const int n_off = (K_o + 31) / 32 * 32;
    int so = part[t];          // selected channels before k
    for (int k = b; k < e; ++k) {
        if (sel[k]) {
            perm[so] = k;
            pos[k] = so;
            ++so;
        } else {
            const int p = K_o + (k - so);
            perm[p] = k;
            pos[k] = n_off + (k - so);
        }
    }
}

// ---- dual scales + INT8 rows -------------------------------------------------------------
// Percentile-clip initialisation of the two scales of every output row (Sec. 4.1 "Quantization
// Implementation": the clipping percentile is searched over {0.999, 0.9999, 0.99999}).  Per row and block,
// with the block's n values taken in packed order:
//     clip_p = linear-interpolated p-quantile of |w|  (h = (n-1) p, a[floor h] + frac (a[floor h + 1] - a[floor h]),
//              in double, rounded to float),  s_p = clip_p / qmax,
//     SSE_p  = sum (double) e^2,  e = fmaf(-s_p, q(w, s_p), w),  summed in packed order in double;
//     the smallest SSE wins, the larger percentile on a tie.
// The sums are order-dependent in their last bits and decide an integer, so one thread owns one block of one
// row and walks it serially (this is the offline step).  Only the CLIP_TOP largest magnitudes are ever needed:
// n - 1 - floor(0.999 (n-1)) < CLIP_TOP for n <= 16384.
constexpr int CLIP_TOP = 20;
__global__ __launch_bounds__(64) void clip_search_kernel(const float *__restrict__ W, int N, int K, int64_t ldw,
                                                         const int32_t *__restrict__ perm, const DetectScalars *sc,
                                                         float qmax, float *__restrict__ s_normal,
                                                         float *__restrict__ s_outlier)
{
    const int t = blockIdx.x * 64 + threadIdx.x;
    if (t >= 2 * N) return;
    const int blk = t / N, j = t - blk * N;            // the first N threads take the outlier blocks
    const int K_o = sc->K_o;
    const int p0 = blk ? K_o : 0, n = blk ? K - K_o : K_o;
    float *dst = blk ? s_normal : s_outlier;
    if (n == 0) {
        dst[j] = 0.0f;
        return;
    }
    const float *w = W + (size_t)j * ldw;
    float top[CLIP_TOP];                               // ascending; -1 marks an empty slot (magnitudes are >= 0)
#pragma unroll
    for (int i = 0; i < CLIP_TOP; ++i) top[i] = -1.0f;
    for (int p = p0; p < p0 + n; ++p) {
        const float a = fabsf(w[perm[p]]);
        if (a > top[0]) {
            top[0] = a;
#pragma unroll
            for (int i = 0; i + 1 < CLIP_TOP; ++i) {
                const float lo = fminf(top[i], top[i + 1]), hi = fmaxf(top[i], top[i + 1]);
                top[i] = lo;
                top[i + 1] = hi;
            }
        }
    }
    auto order_stat = [&](int i) {                     // a_(i) of the ascending order, i >= n - CLIP_TOP
        const int slot = CLIP_TOP - n + i;
        float r = top[0];
#pragma unroll
        for (int u = 1; u < CLIP_TOP; ++u) r = u == slot ? top[u] : r;
        return r;
    };
    const double P[3] = {0.999, 0.9999, 0.99999};
    float s[3];
#pragma unroll
    for (int c = 0; c < 3; ++c) {
        const double h = (double)(n - 1) * P[c];
        const int lo = (int)floor(h);
        const int hi = lo + 1 < n ? lo + 1 : n - 1;
        const double frac = h - (double)lo;
        const double alo = (double)order_stat(lo), ahi = (double)order_stat(hi);
        const float clip = (float)(alo + frac * (ahi - alo));
        s[c] = clip / qmax;
    }
    double sse[3] = {0.0, 0.0, 0.0};
    for (int p = p0; p < p0 + n; ++p) {
        const float x = w[perm[p]];
#pragma unroll
        for (int c = 0; c < 3; ++c) {
            const float q = (float)quantize_sym(x, s[c], qmax);
            const float e = fmaf(-s[c], q, x);
            sse[c] += (double)e * (double)e;
        }
    }
    int best = 2;
    if (sse[1] < sse[best]) best = 1;
    if (sse[0] < sse[best]) best = 0;
    dst[j] = best == 2 ? s[2] : best == 1 ? s[1] : s[0];
}

// One workgroup per output row.  Pass 1: absmax of each block; pass 2: quantize and store each
// byte at its packed position (the row is re-read from cache).  K_o is read from the workspace
// scalars so that no host round trip sits between detection and quantization.
__global__ __launch_bounds__(256) void quantize_rows_kernel(const float *__restrict__ W, int N, int K, int64_t ldw,
                                                            const int32_t *__restrict__ pos, const DetectScalars *sc,
                                                            int8_t *__restrict__ Wq, int64_t ldwq,
                                                            float *__restrict__ s_normal, float *__restrict__ s_outlier,
                                                            float qmax, bool scales_given)
{
    __shared__ float red[8];
    const int j = blockIdx.x;
    const int tid = threadIdx.x;
    const int K_o = sc->K_o;
    const int n_off = (K_o + 31) / 32 * 32;
    const int kp = (n_off + (K - K_o) + 127) / 128 * 128;
    const float *w = W + (size_t)j * ldw;
    float so, sn;
    if (scales_given) {              // (uniform) the clip search has written this row's scales
        so = s_outlier[j];
        sn = s_normal[j];
    } else {
        float a_o = 0.0f, a_n = 0.0f;
        for (int k = tid; k < K; k += 256) {
            const float a = fabsf(w[k]);
            if (pos[k] < K_o) a_o = fmaxf(a_o, a);
            else a_n = fmaxf(a_n, a);
        }
        a_o = wave_max(a_o);
        a_n = wave_max(a_n);
        if ((tid & 63) == 0) {
            red[tid >> 6] = a_o;
            red[4 + (tid >> 6)] = a_n;
        }
        __syncthreads();
        a_o = fmaxf(fmaxf(red[0], red[1]), fmaxf(red[2], red[3]));
        a_n = fmaxf(fmaxf(red[4], red[5]), fmaxf(red[6], red[7]));
        so = a_o / qmax;     // qmax = 127 (INT8 codes) or 7 (INT4 codes)
        sn = a_n / qmax;
        if (tid == 0) {
            s_outlier[j] = so;
            s_normal[j] = sn;
        }
    }
    int8_t *out = Wq + (size_t)j * ldwq;
    for (int k = tid; k < K; k += 256) {
        const int p = pos[k];
        out[p] = (int8_t)quantize_sym(w[k], p < K_o ? so : sn, qmax);
    }
    // zero padding: [K_o, n_off) and [n_off + K_n, kp)
    for (int p = K_o + tid; p < n_off; p += 256) out[p] = 0;
    for (int p = n_off + (K - K_o) + tid; p < kp; p += 256) out[p] = 0;
}

// INT4 packing: the codes of each aligned group of 16 packed positions g go into 8 bytes; byte i < 4
// holds positions 16g+i (low nibble) and 16g+4+i (high nibble), byte 4+i positions 16g+8+i and
// 16g+12+i.  (Shifting a packed dword left by 4 and masking 0xF0F0F0F0 then yields four consecutive
// codes, each times 16, in byte order; masking the dword itself the next four.)
__global__ __launch_bounds__(256) void pack_w4_kernel(const int8_t *__restrict__ codes, int64_t ldc, int N, int kp,
                                                      uint8_t *__restrict__ Wq4, int64_t ldwq4)
{
    const int j = blockIdx.x;
    const int b = blockIdx.y * 256 + threadIdx.x;      // output byte of the row
    if (b >= kp / 2) return;
    const int g = b >> 3, i = b & 7;
    const int lo = 16 * g + (i < 4 ? i : 8 + (i - 4));
    const int8_t *c = codes + (size_t)j * ldc;
    Wq4[(size_t)j * ldwq4 + b] = (uint8_t)((c[lo] & 0xF) | ((c[lo + 4] & 0xF) << 4));
}

struct Workspace {
    float *v, *sorted_v;
    int32_t *rank, *pos;
    double *d, *sorted_d;
    uint8_t *sel;
    DetectScalars *sc;
};

size_t align256(size_t x) { return (x + 255) & ~(size_t)255; }

size_t carve(void *base, int32_t K, Workspace *ws)
{
    unsigned char *p = reinterpret_cast<unsigned char *>(base);
    size_t off = 0;
    auto take = [&](size_t bytes) {
        void *r = p ? p + off : nullptr;
        off += align256(bytes);
        return r;
    };
    void *sc = take(sizeof(DetectScalars));
    void *v = take((size_t)K * 4), *sv = take((size_t)K * 4), *rk = take((size_t)K * 4), *ps = take((size_t)K * 4);
    void *d = take((size_t)K * 8), *sd = take((size_t)K * 8), *sel = take((size_t)K);
    if (ws) {
        ws->sc = reinterpret_cast<DetectScalars *>(sc);
        ws->v = reinterpret_cast<float *>(v);
        ws->sorted_v = reinterpret_cast<float *>(sv);
        ws->rank = reinterpret_cast<int32_t *>(rk);
        ws->pos = reinterpret_cast<int32_t *>(ps);
        ws->d = reinterpret_cast<double *>(d);
        ws->sorted_d = reinterpret_cast<double *>(sd);
        ws->sel = reinterpret_cast<uint8_t *>(sel);
    }
    return off;
}

}  // namespace

extern "C" void qarvd_default_detect_cfg(qarvd_detect_cfg *cfg)
{
    if (!cfg) return;
    cfg->tau = 3.5;
    cfg->alpha = 1.2;
    cfg->align = 32;
    cfg->clip_search = 0;
    cfg->forced_mask = nullptr;
}

extern "C" const char *qarvd_status_string(qarvd_status s)
{
    switch (s) {
        case QARVD_OK: return "QARVD_OK";
        case QARVD_ERR_INVALID_ARG: return "QARVD_ERR_INVALID_ARG";
        case QARVD_ERR_UNSUPPORTED: return "QARVD_ERR_UNSUPPORTED";
        case QARVD_ERR_WORKSPACE: return "QARVD_ERR_WORKSPACE";
        case QARVD_ERR_HIP: return "QARVD_ERR_HIP";
    }
    return "QARVD_ERR_UNKNOWN";
}

extern "C" int32_t qarvd_packed_normal_offset(int32_t K_o) { return K_o < 0 ? 0 : qarvd_round_up(K_o, 32); }

extern "C" int32_t qarvd_packed_k(int32_t K, int32_t K_o)
{
    if (K <= 0 || K > QARVD_MAX_K || K_o > K) return 0;
    if (K_o >= 0) return qarvd_packed(K, K_o).kp;
    // worst case over K_o: the outlier padding adds at most 31 bytes
    return qarvd_round_up(K + 31, 128);
}

extern "C" int32_t qarvd_packed_ld(int32_t K, int32_t K_o)
{
    const int32_t kp = qarvd_packed_k(K, K_o);
    if (kp <= 0) return 0;
    const int32_t ld = kp + 128;                  // multiples of 128, skipping the multiples of 512
    return (ld % 512) == 0 ? ld + 128 : ld;
}

extern "C" size_t qarvd_quantize_weight_workspace(int32_t N, int32_t K)
{
    if (N <= 0 || K <= 0 || K > QARVD_MAX_K) return 0;
    return carve(nullptr, K, nullptr);
}

namespace {

// bits = 8: Wq is the INT8 output [N, ldwq].  bits = 4: Wq is the packed INT4 output [N, ldwq bytes]; the
// one-byte codes go to a temporary behind the detector's workspace and are packed by a second kernel.
qarvd_status quantize_weight_impl(int bits, const float *W, int32_t N, int32_t K, int64_t ldw,
                                  const qarvd_detect_cfg *cfg, void *Wq, int64_t ldwq, float *s_normal,
                                  float *s_outlier, int32_t *perm, int32_t *K_o_host, float *v_out,
                                  void *workspace, size_t workspace_bytes, void *stream)
{
    if (!W || !Wq || !s_normal || !s_outlier || !perm || !K_o_host) return QARVD_ERR_INVALID_ARG;
    if (N <= 0 || K <= 0 || K > QARVD_MAX_K || ldw < K) return QARVD_ERR_INVALID_ARG;
    qarvd_detect_cfg c;
    qarvd_default_detect_cfg(&c);
    if (cfg) c = *cfg;
    if (!c.forced_mask && (!(c.tau >= 0.0) || !(c.alpha >= 0.0) || c.align <= 0)) return QARVD_ERR_INVALID_ARG;
    if (c.clip_search != 0 && c.clip_search != 1) return QARVD_ERR_INVALID_ARG;
    if (c.clip_search && K > 16384) return QARVD_ERR_UNSUPPORTED;     // the search keeps the 20 largest magnitudes
    // The split is not known yet, so the row stride must hold the widest packed row the call can
    // produce: K rounded up to 128 when the aligned count is a multiple of 32 (no inner padding),
    // else the general worst case.
    const bool no_inner_pad = !c.forced_mask && (c.align % 32) == 0;
    const int64_t kp_max = no_inner_pad ? qarvd_round_up(K, 128) : qarvd_packed_k(K, -1);
    if (ldwq < (bits == 8 ? kp_max : kp_max / 2)) return QARVD_ERR_INVALID_ARG;
    if (!qarvd_aligned16(Wq) || (ldwq % 16) != 0 || (reinterpret_cast<uintptr_t>(W) & 3u)) return QARVD_ERR_UNSUPPORTED;
    if (!workspace || (reinterpret_cast<uintptr_t>(workspace) & 255u)) return QARVD_ERR_WORKSPACE;
    const size_t ws_detect = carve(nullptr, K, nullptr);
    const int64_t ld_codes = qarvd_packed_k(K, -1);
    if (workspace_bytes < ws_detect + (bits == 4 ? (size_t)N * ld_codes : 0)) return QARVD_ERR_WORKSPACE;

    hipStream_t st = reinterpret_cast<hipStream_t>(stream);
    Workspace ws;
    carve(workspace, K, &ws);
    int8_t *codes = bits == 8 ? reinterpret_cast<int8_t *>(Wq) : reinterpret_cast<int8_t *>(workspace) + ws_detect;
    const int64_t ldc = bits == 8 ? ldwq : ld_codes;
    const int gK256 = (K + 255) / 256;

    hipLaunchKernelGGL(column_norm_kernel, dim3((K + 63) / 64), dim3(64), 0, st, W, N, K, ldw, ws.v);
    if (c.forced_mask) {
        QARVD_HIP_TRY(hipMemcpyAsync(ws.sel, c.forced_mask, (size_t)K, hipMemcpyHostToDevice, st));
        // normalise to 0/1 is unnecessary: the kernels test for non-zero
    } else {
        hipLaunchKernelGGL((rank_desc_kernel<float>), dim3(gK256), dim3(256), 0, st, ws.v, K, ws.rank, ws.sorted_v);
        hipLaunchKernelGGL(median_dev_kernel, dim3(gK256), dim3(256), 0, st, ws.v, ws.sorted_v, K, ws.sc, ws.d);
        hipLaunchKernelGGL((rank_desc_kernel<double>), dim3(gK256), dim3(256), 0, st, ws.d, K, (int32_t *)nullptr, ws.sorted_d);
        hipLaunchKernelGGL(threshold_kernel, dim3(1), dim3(256), 0, st, ws.v, ws.sorted_d, K, c.tau / 0.6745, c.alpha,
                           c.align, ws.sc);
        hipLaunchKernelGGL(select_by_rank_kernel, dim3(gK256), dim3(256), 0, st, ws.rank, K, ws.sc, ws.sel);
    }
    hipLaunchKernelGGL(build_perm_kernel, dim3(1), dim3(1024), 0, st, ws.sel, K, ws.sc, c.forced_mask ? 1 : 0, perm, ws.pos);
    const float qmax = bits == 8 ? 127.0f : 7.0f;
    if (c.clip_search)
        hipLaunchKernelGGL(clip_search_kernel, dim3((2 * N + 63) / 64), dim3(64), 0, st, W, N, K, ldw, perm, ws.sc, qmax,
                           s_normal, s_outlier);
    hipLaunchKernelGGL(quantize_rows_kernel, dim3(N), dim3(256), 0, st, W, N, K, ldw, ws.pos, ws.sc, codes, ldc, s_normal,
                       s_outlier, qmax, c.clip_search != 0);
    if (v_out) QARVD_HIP_TRY(hipMemcpyAsync(v_out, ws.v, (size_t)K * 4, hipMemcpyDeviceToDevice, st));
    qarvd_status ls = qarvd_launch_status();
    if (ls != QARVD_OK) return ls;
    DetectScalars host_sc;
    QARVD_HIP_TRY(hipMemcpyAsync(&host_sc, ws.sc, sizeof(host_sc), hipMemcpyDeviceToHost, st));
    QARVD_HIP_TRY(hipStreamSynchronize(st));
    *K_o_host = host_sc.K_o;
    if (bits == 4) {    // the packed extent depends on K_o, which is known on the host only now
        const int kp = qarvd_packed(K, host_sc.K_o).kp;
        hipLaunchKernelGGL(pack_w4_kernel, dim3(N, (kp / 2 + 255) / 256), dim3(256), 0, st, codes, ldc, N, kp,
                           reinterpret_cast<uint8_t *>(Wq), ldwq);
        ls = qarvd_launch_status();
        if (ls != QARVD_OK) return ls;
        QARVD_HIP_TRY(hipStreamSynchronize(st));   // the temporary lives in the caller's workspace
    }
    return QARVD_OK;
}

}  // namespace

extern "C" qarvd_status qarvd_quantize_weight(const float *W, int32_t N, int32_t K, int64_t ldw,
                                              const qarvd_detect_cfg *cfg, int8_t *Wq, int64_t ldwq,
                                              float *s_normal, float *s_outlier, int32_t *perm,
                                              int32_t *K_o_host, float *v_out, void *workspace,
                                              size_t workspace_bytes, void *stream)
{
    return quantize_weight_impl(8, W, N, K, ldw, cfg, Wq, ldwq, s_normal, s_outlier, perm, K_o_host, v_out, workspace,
                                workspace_bytes, stream);
}

// ---- the same offline step for callers that cannot allocate ----------------------------------------------
// The detector's workspace (norms, ranks, sorted copies, deviations, selection flags, the scalars) lives in a
// file-scope device array instead of a caller buffer: 528 KB per GPU the library runs on, held until the
// process ends.  In host code the array's name is only a stand-in; its device address is looked up once per
// device with hipGetSymbolAddress and that pointer is what the kernels get.
namespace {
constexpr int32_t STATIC_SCRATCH_MAX_K = 16384;
// carve() for K = 16384: 256 (scalars) + 4 x 65536 (v, sorted v, rank, pos) + 2 x 131072 (d, sorted d) + 16384 (flags)
constexpr size_t STATIC_SCRATCH_BYTES = 256 + 4 * 65536 + 2 * 131072 + 16384;
static __device__ __align__(256) unsigned char scratch[STATIC_SCRATCH_BYTES];

// device address of `scratch` on the current device (each GPU holds its own copy at its own address)
qarvd_status static_scratch_ptr(void **out)
{
    static void *ptr[64] = {nullptr};
    int dev = 0;
    QARVD_HIP_TRY(hipGetDevice(&dev));
    if (dev < 0 || dev >= 64) return QARVD_ERR_UNSUPPORTED;
    void *p = __atomic_load_n(&ptr[dev], __ATOMIC_ACQUIRE);
    if (!p) {
        QARVD_HIP_TRY(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
        if (!p) return QARVD_ERR_HIP;
        __atomic_store_n(&ptr[dev], p, __ATOMIC_RELEASE);
    }
    *out = p;
    return QARVD_OK;
}
}  // namespace

extern "C" int32_t qarvd_quantize_weight_static_max_k(void) { return STATIC_SCRATCH_MAX_K; }

extern "C" qarvd_status qarvd_quantize_weight_static(const float *W, int32_t N, int32_t K, int64_t ldw,
                                                     const qarvd_detect_cfg *cfg, int8_t *Wq, int64_t ldwq,
                                                     float *s_normal, float *s_outlier, int32_t *perm,
                                                     int32_t *K_o_host, float *v_out, void *stream)
{
    if (K > STATIC_SCRATCH_MAX_K) return QARVD_ERR_WORKSPACE;      // the fixed array holds the workspace of K <= 16384
    if (K > 0 && carve(nullptr, K, nullptr) > STATIC_SCRATCH_BYTES) return QARVD_ERR_WORKSPACE;
    void *ws = nullptr;
    if (qarvd_status st = static_scratch_ptr(&ws); st != QARVD_OK) return st;
    // Every kernel of the step writes the part of the workspace it owns before anything reads it (the existing
    // entry point is given uninitialised memory too), so what an earlier call left behind is never read.
    return quantize_weight_impl(8, W, N, K, ldw, cfg, Wq, ldwq, s_normal, s_outlier, perm, K_o_host, v_out, ws,
                                STATIC_SCRATCH_BYTES, stream);
}

extern "C" size_t qarvd_quantize_weight_w4_workspace(int32_t N, int32_t K)
{
    if (N <= 0 || K <= 0 || K > QARVD_MAX_K) return 0;
    return carve(nullptr, K, nullptr) + (size_t)N * qarvd_packed_k(K, -1);
}

extern "C" qarvd_status qarvd_quantize_weight_w4(const float *W, int32_t N, int32_t K, int64_t ldw,
                                                 const qarvd_detect_cfg *cfg, uint8_t *Wq4, int64_t ldwq4,
                                                 float *s_normal, float *s_outlier, int32_t *perm,
                                                 int32_t *K_o_host, float *v_out, void *workspace,
                                                 size_t workspace_bytes, void *stream)
{
    return quantize_weight_impl(4, W, N, K, ldw, cfg, Wq4, ldwq4, s_normal, s_outlier, perm, K_o_host, v_out, workspace,
                                workspace_bytes, stream);
}
