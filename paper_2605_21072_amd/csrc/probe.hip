// Diagnostic: measured issue-bound INT8 MFMA rate of the device this process runs on.
// Every wavefront issues back-to-back independent v_mfma_i32_32x32x32_i8 on register-resident
// operands (no memory traffic), two wavefronts per SIMD on every CU, and the whole-chip rate is
// 2 * 32*32*32 operations per instruction over the elapsed event time.  On MI355X this sits
// below the datasheet peak because the MFMA clock is power-limited; reports quote both.
#include "qarvd_common.h"

namespace {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));

__global__ __launch_bounds__(512, 2) void mfma_probe_kernel(int iters, const int *seed, int *sink)
{
    v16i acc[8];
#pragma unroll
    for (int i = 0; i < 8; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[i][r] = seed[(i * 16 + r + threadIdx.x) & 1023];
    const int t = threadIdx.x;
    v4i a = {seed[t & 1023], seed[(t + 1) & 1023], seed[(t + 2) & 1023], seed[(t + 3) & 1023]};
    v4i b = {seed[(t + 4) & 1023], seed[(t + 5) & 1023], seed[(t + 6) & 1023], seed[(t + 7) & 1023]};
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int i = 0; i < 8; ++i) acc[i] = __builtin_amdgcn_mfma_i32_32x32x32_i8(a, b, acc[i], 0, 0, 0);
    }
    int s = 0;
#pragma unroll
    for (int i = 0; i < 8; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) s ^= acc[i][r];
    if (s == 0x7fffffff) sink[0] = s;   // keeps the accumulators alive
}

}  // namespace

extern "C" qarvd_status qarvd_probe_mfma_peak(int32_t iters, void *workspace, size_t workspace_bytes, double *tops_host,
                                              void *stream)
{
    if (!tops_host || iters <= 0) return QARVD_ERR_INVALID_ARG;
    if (!workspace || workspace_bytes < 4096 + 64 || (reinterpret_cast<uintptr_t>(workspace) & 3u)) return QARVD_ERR_WORKSPACE;
    hipStream_t st = reinterpret_cast<hipStream_t>(stream);
    int dev = 0, ncu = 256;
    hipDeviceProp_t prop;
    if (hipGetDevice(&dev) == hipSuccess && hipGetDeviceProperties(&prop, dev) == hipSuccess) ncu = prop.multiProcessorCount;
    int *seed = reinterpret_cast<int *>(workspace);
    int *sink = seed + 1024;
    int host_seed[1024];
    for (int i = 0; i < 1024; ++i) host_seed[i] = (int)((unsigned)i * 2654435761u >> 3);
    QARVD_HIP_TRY(hipMemcpyAsync(seed, host_seed, sizeof(host_seed), hipMemcpyHostToDevice, st));
    QARVD_HIP_TRY(hipStreamSynchronize(st));
    hipEvent_t e0, e1;
    QARVD_HIP_TRY(hipEventCreate(&e0));
    QARVD_HIP_TRY(hipEventCreate(&e1));
    hipLaunchKernelGGL(mfma_probe_kernel, dim3(ncu), dim3(512), 0, st, iters, seed, sink);   // warm-up
    hipEventRecord(e0, st);
    hipLaunchKernelGGL(mfma_probe_kernel, dim3(ncu), dim3(512), 0, st, iters, seed, sink);
    hipEventRecord(e1, st);
    hipError_t err = hipEventSynchronize(e1);
    float ms = 0.f;
    if (err == hipSuccess) err = hipEventElapsedTime(&ms, e0, e1);
    hipEventDestroy(e0);
    hipEventDestroy(e1);
    if (err != hipSuccess || hipGetLastError() != hipSuccess || ms <= 0.f) return QARVD_ERR_HIP;
    const double mfma = (double)iters * 8.0 * 8.0 * ncu;   // per wave x waves per CU x CUs
    *tops_host = mfma * 65536.0 / (ms * 1e-3) / 1e12;
    return QARVD_OK;
}
