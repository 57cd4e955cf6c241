// Stand-in for <hip/hip_runtime.h> that lets the library's HIP sources compile for the HOST, so that
// the kernels can run on the CPU under memory checks (test infrastructure; never part of the product).
// Every GPU thread is a fiber, a workgroup runs on one OS thread, workgroups run on a few OS threads;
// the cross-lane instructions the kernels use (transposing LDS read, matrix instruction, lane reads,
// lane-row swaps) are emulated by exchanging operands between the 64 fibers of a wave.  Device memory
// is host memory fenced by protected pages: an access outside an allocation is a segmentation fault
// at the faulting kernel line.  A barrier that not every wave of a workgroup reaches is reported as a
// deadlock instead of hanging.
#pragma once
#include <cmath>
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <algorithm>
#include <functional>

#define __global__
#define __device__
#define __host__
#define __forceinline__ inline __attribute__((always_inline))
#define __launch_bounds__(...)
#define __shared__ static thread_local

struct dim3 {
    unsigned x, y, z;
    dim3(unsigned x_ = 1, unsigned y_ = 1, unsigned z_ = 1) : x(x_), y(y_), z(z_) {}
};
struct float2 { float x, y; };
static inline float2 make_float2(float x, float y) { return float2{x, y}; }

typedef int hipError_t;
typedef void* hipStream_t;
enum { hipSuccess = 0, hipErrorInvalidValue = 1, hipErrorOutOfMemory = 2 };
enum { hipMemcpyHostToDevice = 1, hipMemcpyDeviceToHost = 2 };
enum { hipDeviceAttributeMultiprocessorCount = 1 };

namespace emu {
typedef int v4i_t __attribute__((ext_vector_type(4)));
typedef int v2i_t __attribute__((ext_vector_type(2)));
struct Fiber;
Fiber* cur();
dim3& thread_idx();
dim3& block_idx();
dim3& grid_dim();
dim3& block_dim();
void syncthreads();
v2i_t tr8(const void* p);
v4i_t mfma_i8_16x16x64(v4i_t a, v4i_t b, v4i_t c);
int readfirstlane(int v);
void wave_barrier();
typedef unsigned v2u_t __attribute__((ext_vector_type(2)));
v2u_t permlane_swap(unsigned a, unsigned b, int rows);
int readlane(int v, int lane);
void launch(dim3 grid, dim3 block, const std::function<void()>& fn);
void* dev_alloc(size_t bytes);
void dev_free(void* p);
}  // namespace emu

#define threadIdx (emu::thread_idx())
#define blockIdx (emu::block_idx())
#define gridDim (emu::grid_dim())
#define blockDim (emu::block_dim())
#define __syncthreads() emu::syncthreads()

#define __builtin_amdgcn_readfirstlane(v) emu::readfirstlane((int)(v))
#define __builtin_amdgcn_readlane(v, l) emu::readlane((int)(v), (int)(l))
#define __builtin_amdgcn_ds_read_tr8_b64_v2i32(p) emu::tr8((const void*)(uintptr_t)(p))
#define __builtin_amdgcn_mfma_i32_16x16x64_i8(a, b, c, x, y, z) emu::mfma_i8_16x16x64((a), (b), (c))
#define __builtin_amdgcn_sched_barrier(m) ((void)0)
#define __builtin_amdgcn_permlane16_swap(a, b, fi, bc) emu::permlane_swap((a), (b), 16)
#define __builtin_amdgcn_permlane32_swap(a, b, fi, bc) emu::permlane_swap((a), (b), 32)
#define __builtin_amdgcn_sched_group_barrier(a, b, c) ((void)0)
#define __builtin_amdgcn_s_waitcnt(m) ((void)0)
#define __builtin_amdgcn_s_setprio(m) ((void)0)
#define __builtin_amdgcn_rcpf(x) (1.0f / (x))
#define __builtin_amdgcn_exp2f(x) exp2f(x)
#define __fmaf_rn(a, b, c) fmaf((a), (b), (c))
static inline float emu_fmed3f(float a, float b, float c)
{
    if (a != a || b != b || c != c) return fminf(fminf(a, b), c);
    return fmaxf(fminf(a, b), fminf(fmaxf(a, b), c));
}
#define __builtin_amdgcn_fmed3f(a, b, c) emu_fmed3f((a), (b), (c))
static inline uint32_t emu_cvt_pk_u8_f32(float f, uint32_t sel, uint32_t old)
{
    int v = 0;
    if (f == f) { float r = nearbyintf(f); v = r < 0.0f ? 0 : (r > 255.0f ? 255 : (int)r); }
    const uint32_t sh = 8 * (sel & 3);
    return (old & ~(0xffu << sh)) | ((uint32_t)v << sh);
}
#define __builtin_amdgcn_cvt_pk_u8_f32(f, sel, old) emu_cvt_pk_u8_f32((f), (sel), (old))
static inline uint32_t emu_alignbyte(uint32_t hi, uint32_t lo, uint32_t sh)
{
    const uint64_t v = ((uint64_t)hi << 32) | lo;
    return (uint32_t)(v >> (8 * (sh & 3)));
}
#define __builtin_amdgcn_alignbyte(hi, lo, sh) emu_alignbyte((hi), (lo), (sh))
// buffer resource + raw buffer store: base pointer and size.  The hardware drops a store that would leave the
// buffer; the kernels never rely on that, so here it ends the run with a message
struct emu_buffer_rsrc { uint8_t* base; uint32_t bytes; };
typedef emu_buffer_rsrc __amdgpu_buffer_rsrc_t;
#define __builtin_amdgcn_make_buffer_rsrc(p, stride, num, flags) (emu_buffer_rsrc{(uint8_t*)(p), (uint32_t)(num)})
template <typename V>
static inline void emu_buffer_store(const V v, const emu_buffer_rsrc r, const int voff, const int soff)
{
    const uint64_t off = (uint64_t)(uint32_t)voff + (uint32_t)soff;
    if (off + sizeof(V) > r.bytes) {
        fprintf(stderr, "emu: buffer store of %zu bytes at offset %llu leaves the buffer of %u bytes\n", sizeof(V),
                (unsigned long long)off, r.bytes);
        abort();
    }
    memcpy(r.base + off, &v, sizeof(V));
}
#define __builtin_amdgcn_raw_buffer_store_b128(v, r, vo, so, aux) emu_buffer_store((v), (r), (vo), (so))
using std::min;
using std::max;

static inline hipError_t hipMalloc(void** p, size_t n) { *p = emu::dev_alloc(n); return *p ? hipSuccess : hipErrorOutOfMemory; }
static inline hipError_t hipFree(void* p) { emu::dev_free(p); return hipSuccess; }
static inline hipError_t hipMemset(void* p, int v, size_t n) { memset(p, v, n); return hipSuccess; }
static inline hipError_t hipMemcpy(void* d, const void* s, size_t n, int) { memcpy(d, s, n); return hipSuccess; }
static inline hipError_t hipGetDevice(int* d) { *d = 0; return hipSuccess; }
static inline hipError_t hipDeviceGetAttribute(int* v, int, int)
{
    const char* e = getenv("EMU_CUS");
    *v = e ? atoi(e) : 256;
    return hipSuccess;
}
static inline hipError_t hipGetLastError() { return hipSuccess; }
#define hipLaunchKernelGGL(kernel, grid, block, shmem, stream, ...) \
    emu::launch((grid), (block), [=]() { kernel(__VA_ARGS__); })
