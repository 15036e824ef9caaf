// TEST INFRASTRUCTURE ONLY.  A CPU stand-in for <hip/hip_runtime.h> so that the library's kernel
// sources can be compiled by the host compiler and run under AddressSanitizer and UBSan on tiny
// inputs: a launch runs block after block, one OS thread per lane, with __syncthreads and the
// wave64 cross-lane builtins (DPP permutations, readlane, shuffles) emulated through barriers.
// It checks indexing and logic and is hopeless for speed.  By default blocks run one after the other in
// index order; with EMU_CONCURRENT_BLOCKS=K they run K at a time in a shuffled order, each in a process of
// its own (emu_rt.cpp), so that ticket hand-overs between blocks happen in any order.  Nothing in the product includes or links it: the library
// itself has no CPU path.
#pragma once
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include <atomic>
#include <barrier>
#include <functional>
#include <memory>
#include <thread>
#include <vector>

#define __global__
#define __device__
#define __host__
#define __forceinline__ inline __attribute__((always_inline))
#define __shared__ static
#define __launch_bounds__(...)
#define __align__(n) __attribute__((aligned(n)))

struct dim3 {
    unsigned x, y, z;
    dim3(unsigned a = 1, unsigned b = 1, unsigned c = 1) : x(a), y(b), z(c) {}
};
struct float4 { float x, y, z, w; };
struct uint4 { uint32_t x, y, z, w; };
struct uint2 { uint32_t x, y; };
static inline float4 make_float4(float a, float b, float c, float d) { return float4{a, b, c, d}; }
static inline uint4 make_uint4(uint32_t a, uint32_t b, uint32_t c, uint32_t d) { return uint4{a, b, c, d}; }
static inline uint2 make_uint2(uint32_t a, uint32_t b) { return uint2{a, b}; }

typedef void *hipStream_t;
enum hipError_t { hipSuccess = 0, hipErrorInvalidValue = 1 };
enum { hipMemcpyDeviceToHost = 2, hipMemcpyDeviceToDevice = 3, hipDeviceAttributeMultiprocessorCount = 63 };
#ifndef __HIP_MEMORY_SCOPE_AGENT
#define __HIP_MEMORY_SCOPE_AGENT 4
#endif

namespace emu {
extern thread_local dim3 t_threadIdx, t_blockIdx;
extern dim3 g_blockDim, g_gridDim;
extern int g_occupancy, g_cus;
struct BlockCtx {
    std::unique_ptr<std::barrier<>> block_bar;
    std::vector<std::unique_ptr<std::barrier<>>> wave_bar;
    std::vector<uint32_t> xbuf;   // [wave][2][64]
    std::atomic<int> and_flag{1};
};
extern BlockCtx *g_ctx;
extern thread_local unsigned t_opcount;
void launch(dim3 grid, dim3 block, const std::function<void()> &fn);
void *shared_alloc(size_t bytes);   // "device memory" that the per-block processes of the concurrent mode share
uint32_t exchange(uint32_t v, int src_lane_or_minus1, int ctrl, int xor_mask);
}  // namespace emu

#define threadIdx emu::t_threadIdx
#define blockIdx emu::t_blockIdx
#define blockDim emu::g_blockDim
#define gridDim emu::g_gridDim

#define hipLaunchKernelGGL(kernel, grid, block, shmem, stream, ...) \
    emu::launch((grid), (block), [&]() { kernel(__VA_ARGS__); })

static inline hipError_t hipGetLastError() { return hipSuccess; }
static inline hipError_t hipStreamSynchronize(hipStream_t) { return hipSuccess; }
static inline hipError_t hipMemcpyAsync(void *d, const void *s, size_t n, int, hipStream_t) { memcpy(d, s, n); return hipSuccess; }
#define HIP_SYMBOL(x) x
template <typename T> static inline hipError_t hipGetSymbolAddress(void **p, const T &sym) { *p = (void *)&sym; return hipSuccess; }
static inline hipError_t hipGetDevice(int *d) { *d = 0; return hipSuccess; }
static inline hipError_t hipDeviceGetAttribute(int *v, int, int) { *v = emu::g_cus; return hipSuccess; }
template <typename K> static inline hipError_t hipOccupancyMaxActiveBlocksPerMultiprocessor(int *n, K, int, size_t) { *n = emu::g_occupancy; return hipSuccess; }

static inline void __syncthreads() { emu::g_ctx->block_bar->arrive_and_wait(); }
static inline int __syncthreads_and(int p)
{
    __syncthreads();
    if (threadIdx.x == 0) emu::g_ctx->and_flag.store(1);
    __syncthreads();
    if (!p) emu::g_ctx->and_flag.store(0);
    __syncthreads();
    const int r = emu::g_ctx->and_flag.load();
    __syncthreads();
    return r;
}

static inline uint32_t atomicAdd(uint32_t *p, uint32_t v) { return __atomic_fetch_add(p, v, __ATOMIC_SEQ_CST); }
#define __builtin_amdgcn_fence(order, scope) ((void)0)

static inline float __uint_as_float(uint32_t u) { float f; memcpy(&f, &u, 4); return f; }
static inline uint32_t __float_as_uint(float f) { uint32_t u; memcpy(&u, &f, 4); return u; }
static inline int __float_as_int(float f) { int u; memcpy(&u, &f, 4); return u; }
static inline float __int_as_float(int u) { float f; memcpy(&f, &u, 4); return f; }
static inline long long __double_as_longlong(double d) { long long u; memcpy(&u, &d, 8); return u; }
static inline double __longlong_as_double(long long u) { double d; memcpy(&d, &u, 8); return d; }
static inline int __double2hiint(double d) { return (int)((uint64_t)__double_as_longlong(d) >> 32); }
static inline int __double2loint(double d) { return (int)(uint32_t)__double_as_longlong(d); }
static inline double __hiloint2double(int hi, int lo) { return __longlong_as_double((long long)(((uint64_t)(uint32_t)hi << 32) | (uint32_t)lo)); }

static inline float emu_med3(float a, float b, float c)
{
    if (a != a || b != b || c != c) return fminf(fminf(a, b), c);
    return fmaxf(fminf(a, b), fminf(fmaxf(a, b), c));
}
#define __builtin_amdgcn_fmed3f(a, b, c) emu_med3((a), (b), (c))
#define __builtin_amdgcn_alignbit(hi, lo, sh) ((uint32_t)(((((uint64_t)(hi)) << 32) | (uint32_t)(lo)) >> ((sh) & 31)))
#define __builtin_amdgcn_readlane(v, l) ((int)emu::exchange((uint32_t)(v), (l), -1, 0))
#define __builtin_amdgcn_readfirstlane(v) ((int)emu::exchange((uint32_t)(v), 0, -1, 0))   /* every lane of the wave is active where the kernels use it */
#define __builtin_amdgcn_update_dpp(old, v, ctrl, rm, bm, bc) ((int)emu::exchange((uint32_t)(v), -1, (ctrl), 0))
static inline double __shfl_xor(double v, int m, int)
{
    const uint32_t lo = emu::exchange((uint32_t)__double2loint(v), -1, -1, m), hi = emu::exchange((uint32_t)__double2hiint(v), -1, -1, m);
    return __hiloint2double((int)hi, (int)lo);
}
static inline uint32_t __shfl_xor(uint32_t v, int m, int) { return emu::exchange(v, -1, -1, m); }

template <typename T> static inline T min(T a, T b) { return b < a ? b : a; }
template <typename T> static inline T max(T a, T b) { return a < b ? b : a; }
