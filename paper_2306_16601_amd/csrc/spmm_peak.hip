// Measured ceilings of the two candidate multiply instructions (the choice between a 4-wide int8 dot
// product per 4-element block -- the direct analogue of Algorithm 1's multiply -- and the int8 matrix
// instruction over gathered tiles is to be made on measured rates, not on data-sheet ones): registers
// only, no memory traffic, enough independent accumulators to keep the pipe full.
#include <hip/hip_runtime.h>

#include <cstdint>

#include "spmm.h"

namespace {

typedef int v4i __attribute__((ext_vector_type(4)));

__global__ void __launch_bounds__(256) peak_mfma_16x16x64_i8(int* sink, const int iters)
{
    v4i a = {(int)threadIdx.x, 1, 2, 3}, b = {4, 5, 6, (int)blockIdx.x};
    v4i acc[8];
    for (int i = 0; i < 8; ++i) acc[i] = (v4i){i, i, i, i};
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int i = 0; i < 8; ++i) acc[i] = __builtin_amdgcn_mfma_i32_16x16x64_i8(a, b, acc[i], 0, 0, 0);
    }
    int s = 0;
    for (int i = 0; i < 8; ++i) s += acc[i][0] + acc[i][1] + acc[i][2] + acc[i][3];
    if (s == 0x7fffffff) sink[0] = s;   // keeps the loop alive; practically never true
}

__global__ void __launch_bounds__(256) peak_dot4_i8(int* sink, const int iters)
{
    const int a = (int)threadIdx.x * 0x01010101, b = (int)blockIdx.x | 0x01020304;
    int acc[16];
    for (int i = 0; i < 16; ++i) acc[i] = i;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int i = 0; i < 16; ++i) acc[i] = __builtin_amdgcn_sdot4(a, b, acc[i], false);
    }
    int s = 0;
    for (int i = 0; i < 16; ++i) s += acc[i];
    if (s == 0x7fffffff) sink[0] = s;
}

}  // namespace

extern "C" spmm_status_t spmm_measure_peak(int32_t which, double* tera_ops_per_s)
{
    if (!tera_ops_per_s || (which != 0 && which != 1)) return SPMM_E_ARG;
    int dev = 0, cus = 0;
    if (hipGetDevice(&dev) != hipSuccess) return SPMM_E_DEVICE;
    if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus <= 0) return SPMM_E_DEVICE;
    int* sink = nullptr;
    if (hipMalloc((void**)&sink, 256) != hipSuccess) return SPMM_E_ALLOC;
    hipEvent_t e0, e1;
    if (hipEventCreate(&e0) != hipSuccess || hipEventCreate(&e1) != hipSuccess) {
        (void)hipFree(sink);
        return SPMM_E_DEVICE;
    }
    const int iters = 20000, blocks = cus * 2;   // 8 waves per CU: two per SIMD
    double best_ms = 0.0;
    hipError_t err = hipSuccess;
    for (int rep = 0; rep < 3 && err == hipSuccess; ++rep) {   // first repetition warms up
        (void)hipEventRecord(e0, nullptr);
        if (which == 0) hipLaunchKernelGGL(peak_mfma_16x16x64_i8, dim3(blocks), dim3(256), 0, nullptr, sink, iters);
        else hipLaunchKernelGGL(peak_dot4_i8, dim3(blocks), dim3(256), 0, nullptr, sink, iters);
        (void)hipEventRecord(e1, nullptr);
        err = hipEventSynchronize(e1);
        float ms = 0.0f;
        if (err == hipSuccess) err = hipEventElapsedTime(&ms, e0, e1);
        if (rep > 0 && (best_ms == 0.0 || ms < best_ms)) best_ms = ms;
    }
    (void)hipEventDestroy(e0);
    (void)hipEventDestroy(e1);
    (void)hipFree(sink);
    if (err != hipSuccess || best_ms <= 0.0) return SPMM_E_DEVICE;
    // operations = 2 x multiply-accumulates: a 16x16x64 matrix instruction does 16384 of them per wave,
    // a 4-wide dot product 4 per lane
    const double waves = (double)blocks * 4.0;
    const double ops = (which == 0) ? waves * iters * 8.0 * 2.0 * 16384.0 : waves * iters * 16.0 * 2.0 * 4.0 * 64.0;
    *tera_ops_per_s = ops / (best_ms * 1e-3) / 1e12;
    return SPMM_OK;
}
