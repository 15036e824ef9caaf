// Shared device-side helpers and the workspace layout of the gfx950 kernels.
// Wave size is 64 throughout (CDNA4); nothing here is written for 32-wide warps.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "quantpipe.h"

namespace qp {

constexpr int kWave = 64;
constexpr uint32_t kMaxBins = 4096;
constexpr uint32_t kMaxT = 1023;           // candidates j = 0..t, t <= kMaxT
constexpr uint32_t kMaxCandsPerRound = 32;
constexpr uint32_t kMaxStat1Blocks = 512;  // most blocks of statistics pass 1 (256 lanes each)
constexpr uint32_t kMaxStat2Blocks = 256;  // most blocks of pass 2 (512 lanes each): one per CU measured best
constexpr uint32_t kMaxSearchBlocks = 1024;
constexpr uint32_t kNumValues16 = 65536;   // bit patterns of a bfloat16
// bf16 tensors at least this large go through their value table (counting the values and working on
// 65536 of them costs about 30 us; the per-element kernels pass that at about a million elements)
#ifndef QP_VALUE_TABLE_MIN_N
#define QP_VALUE_TABLE_MIN_N (1ull << 20)
#endif
constexpr uint64_t kValueTableMinN = QP_VALUE_TABLE_MIN_N;
// Tensors at least this large take the forms of quantize+pack (3 and 6 bit) and unpack+dequantize that pay on
// large tensors only (measured break-even between 9.7 M and 77 M elements).
#ifndef QP_LARGE_FORMS_MIN_N
#define QP_LARGE_FORMS_MIN_N (1ull << 24)
#endif
constexpr uint64_t kLargeFormsMinN = QP_LARGE_FORMS_MIN_N;

// Per-block partial of the first statistics pass.
struct Part1 {
    double sum;
    double sum_abs;
    float mn;
    float mx;
    uint32_t bad;   // NaN/Inf elements seen by this block
    uint32_t pad;
};
static_assert(sizeof(Part1) == 32, "Part1 layout");

// Per-block partial of the second pass.
struct Part2 {
    double dev;     // sum |x - mu|
    double sq;      // sum (x - mu)^2
};

// One search candidate: the quantization grid it induces.
struct Cand {
    float lo, hi, scale, inv_scale;
};
static_assert(sizeof(Cand) == 16, "Cand layout");

// How a search kernel's candidate list maps to grid indices j (Eq. 1's b_j = b_E + j step).
enum ListMode : uint32_t {
    kListFull = 0,     // i -> j = i, i = 0..t: the paper's sweep
    kListCoarse = 1,   // i -> j = min(i * stride, t)
    kListFine = 2      // i -> j = clamp(j1 - (stride - 1) + i, 0, t), i = 0..2 stride - 2, j1 the coarse winner
};
__device__ __host__ inline uint32_t list_index(uint32_t mode, uint32_t stride, uint32_t j1, uint32_t t_steps, uint32_t i)
{
    if (mode == kListFull) return i;
    if (mode == kListCoarse) {
        const uint64_t j = (uint64_t)i * stride;
        return j > t_steps ? t_steps : (uint32_t)j;
    }
    const int64_t j = (int64_t)j1 - (int64_t)(stride - 1u) + (int64_t)i;
    return j < 0 ? 0u : (j > (int64_t)t_steps ? t_steps : (uint32_t)j);
}

// Device-resident control block.
struct Ctl {
    uint32_t ticket_stats;    // blocks of statistics pass 2 that have finished
    uint32_t ticket_search;   // rounds (or candidates) of the search that have finished
    uint32_t short_seq;       // 1: the search may drop the clamp of the rounded level
    uint32_t clip;            // 1: candidate ranges are intersected with [clip_lo, clip_hi]
    double b_e, b_r, step, F; // search grid: b_j = b_e + j*step, alpha_j = F*b_j
    double mean;
    uint32_t bits, t_steps;
    uint64_t n;
    uint32_t list_mode, list_stride, list_j1, pad2;
    float clip_lo, clip_hi;   // the data's range
    double score0;            // score of j = 0 (plain ACIQ), kept from the coarse sweep for the fine one
};

// Workspace layout (byte offsets).  Fixed-size regions first, the search partials last.
constexpr size_t kOffStats = 0;                                   // qp_stats_t (88 B)
constexpr size_t kOffResult = 128;                                // qp_search_result_t (56 B)
constexpr size_t kOffQParams = 192;                               // qp_qparams_t (32 B)
constexpr size_t kOffModel = 224;                                 // qp_model_fit_t (24 B)
constexpr size_t kOffCtl = 256;                                   // Ctl
constexpr size_t kOffHist = 512;                                  // uint32_t[kMaxBins]
constexpr size_t kOffCands = kOffHist + kMaxBins * 4;             // Cand[kMaxT + 1]
constexpr size_t kOffScores = kOffCands + (kMaxT + 1) * sizeof(Cand);   // double[kMaxT + 1]
constexpr size_t kOffRoundTickets = kOffScores + (kMaxT + 1) * 8; // uint32_t[kMaxT + 1]: per-round block counters
constexpr size_t kOffPart1 = kOffRoundTickets + (kMaxT + 1) * 4;  // Part1[kMaxStat1Blocks]
constexpr size_t kOffPart2 = kOffPart1 + kMaxStat1Blocks * sizeof(Part1);  // Part2[kMaxStat2Blocks]
constexpr size_t kOffValueCounts = kOffPart2 + kMaxStat2Blocks * sizeof(Part2);  // uint32_t[65536]: bf16 value table
constexpr size_t kOffListScores = kOffValueCounts + 65536 * 4;   // double[kMaxT + 1]: scores in list order (coarse-to-fine)
constexpr size_t kOffSearchPart = kOffListScores + (kMaxT + 1) * 8;  // double[t + 1][blocks]
static_assert(sizeof(qp_stats_t) <= 128 && sizeof(qp_search_result_t) <= 64 && sizeof(qp_qparams_t) == 32 &&
              sizeof(qp_model_fit_t) <= 32 && sizeof(Ctl) <= 256, "fixed workspace regions");
static_assert(kOffSearchPart % 16 == 0, "alignment");

// native vector types (the nontemporal builtins want them)
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

// ---- element loads: four consecutive elements, widened to fp32 ----------------------
// fp32: one 16-byte load; bf16: one 8-byte load, the 16 bits become the top half.
template <int DT> struct Vec4;
template <> struct Vec4<QP_F32> {
    static __device__ __forceinline__ void load(const void *base, uint64_t vec, float (&f)[4])
    {
        const float4 v = reinterpret_cast<const float4 *>(base)[vec];
        f[0] = v.x; f[1] = v.y; f[2] = v.z; f[3] = v.w;
    }
    static __device__ __forceinline__ float load1(const void *base, uint64_t i)
    {
        return reinterpret_cast<const float *>(base)[i];
    }
};
template <> struct Vec4<QP_BF16> {
    static __device__ __forceinline__ void load(const void *base, uint64_t vec, float (&f)[4])
    {
        const uint2 v = reinterpret_cast<const uint2 *>(base)[vec];
        f[0] = __uint_as_float(v.x << 16);
        f[1] = __uint_as_float(v.x & 0xffff0000u);
        f[2] = __uint_as_float(v.y << 16);
        f[3] = __uint_as_float(v.y & 0xffff0000u);
    }
    static __device__ __forceinline__ float load1(const void *base, uint64_t i)
    {
        return __uint_as_float(static_cast<uint32_t>(reinterpret_cast<const uint16_t *>(base)[i]) << 16);
    }
};

// ---- 16-byte loads for the streaming reductions: 4 fp32 or 8 bf16 elements per lane -------
template <int DT> struct Vec16;
template <> struct Vec16<QP_F32> {
    static constexpr int kElems = 4;
    static __device__ __forceinline__ void load(const void *base, uint64_t vec, float (&f)[4])
    {
        const float4 v = reinterpret_cast<const float4 *>(base)[vec];
        f[0] = v.x; f[1] = v.y; f[2] = v.z; f[3] = v.w;
    }
};
template <> struct Vec16<QP_BF16> {
    static constexpr int kElems = 8;
    static __device__ __forceinline__ void load(const void *base, uint64_t vec, float (&f)[8])
    {
        const uint4 v = reinterpret_cast<const uint4 *>(base)[vec];
        const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            f[2 * i] = __uint_as_float(w[i] << 16);
            f[2 * i + 1] = __uint_as_float(w[i] & 0xffff0000u);
        }
    }
};

// the same 16-byte load, nontemporal: for data a kernel touches exactly once
template <int DT> __device__ __forceinline__ void load16_stream(const void *base, uint64_t vec, float (&f)[Vec16<DT>::kElems])
{
    if constexpr (DT == QP_F32) {
        const f32x4 v = __builtin_nontemporal_load(reinterpret_cast<const f32x4 *>(base) + vec);
        f[0] = v.x; f[1] = v.y; f[2] = v.z; f[3] = v.w;
    } else {
        const u32x4 v = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(base) + vec);
        const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            f[2 * i] = __uint_as_float(w[i] << 16);
            f[2 * i + 1] = __uint_as_float(w[i] & 0xffff0000u);
        }
    }
}

// ---- device-coherent accesses ---------------------------------------------------------------
// For data that blocks of one kernel hand to each other ("the block that draws the last ticket finishes
// the job").  The L2 of an XCD is not coherent with
// the other XCDs' for ordinary loads and stores; a device-scope release / acquire pair repairs
// that by writing the whole L2 back and invalidating it, which costs microseconds per block.
// Device-scope atomic accesses go to the point of coherence themselves, so a producer that
// writes with st_dev, waits for its stores (wait_stores) and only then signals, and a consumer
// that reads with ld_dev after seeing the signal, need no cache maintenance at all.
__device__ __forceinline__ uint32_t ld_dev(const uint32_t *p)
{
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ uint64_t ld_dev(const uint64_t *p)
{
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ double ld_dev(const double *p)
{
    return __longlong_as_double((long long)ld_dev(reinterpret_cast<const uint64_t *>(p)));
}
__device__ __forceinline__ void st_dev(uint32_t *p, uint32_t v)
{
    __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void st_dev(uint64_t *p, uint64_t v)
{
    __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void st_dev(double *p, double v)
{
    st_dev(reinterpret_cast<uint64_t *>(p), (uint64_t)__double_as_longlong(v));
}
// all of this lane's outstanding memory operations (stores included) have been acknowledged
__device__ __forceinline__ void wait_stores()
{
#if defined(__AMDGCN__)   // (the host pass of the compiler only parses this function)
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
#endif
}

__device__ __forceinline__ void st_dev(Part1 *dst, const Part1 &p)
{
    uint64_t *d = reinterpret_cast<uint64_t *>(dst);
    st_dev(d, (uint64_t)__double_as_longlong(p.sum));
    st_dev(d + 1, (uint64_t)__double_as_longlong(p.sum_abs));
    st_dev(d + 2, (uint64_t)__float_as_uint(p.mn) | ((uint64_t)__float_as_uint(p.mx) << 32));
    st_dev(d + 3, (uint64_t)p.bad);
}
__device__ __forceinline__ Part1 ld_dev(const Part1 *src)
{
    const uint64_t *s = reinterpret_cast<const uint64_t *>(src);
    const uint64_t a = ld_dev(s), b = ld_dev(s + 1), c = ld_dev(s + 2), d = ld_dev(s + 3);
    Part1 p;
    p.sum = __longlong_as_double((long long)a);
    p.sum_abs = __longlong_as_double((long long)b);
    p.mn = __uint_as_float((uint32_t)c);
    p.mx = __uint_as_float((uint32_t)(c >> 32));
    p.bad = (uint32_t)d;
    p.pad = 0u;
    return p;
}

// ---- wave64 reductions -------------------------------------------------------------------
// Four DPP steps (lane permutations inside a row of 16 lanes, executed in the vector ALU, no
// LDS traffic) leave each row's result in all of its lanes; the four rows are then read with
// v_readlane and combined in a fixed order.  All 64 lanes must be active.  The result is
// wave-uniform and the order of operations is fixed, so results are bit-reproducible.
constexpr int kDppQuadSwap1 = 0xB1;      // quad_perm [1,0,3,2]
constexpr int kDppQuadSwap2 = 0x4E;      // quad_perm [2,3,0,1]
constexpr int kDppHalfMirror = 0x141;    // lane i <-> 7-i inside each group of 8
constexpr int kDppRowMirror = 0x140;     // lane i <-> 15-i inside each row of 16

template <int CTRL> __device__ __forceinline__ int dpp_i32(int v)
{
    return __builtin_amdgcn_update_dpp(0, v, CTRL, 0xf, 0xf, true);
}
template <int CTRL> __device__ __forceinline__ float dpp_f32(float v)
{
    return __int_as_float(dpp_i32<CTRL>(__float_as_int(v)));
}
template <int CTRL> __device__ __forceinline__ double dpp_f64(double v)
{
    return __hiloint2double(dpp_i32<CTRL>(__double2hiint(v)), dpp_i32<CTRL>(__double2loint(v)));
}
__device__ __forceinline__ double readlane_f64(double v, int lane)
{
    return __hiloint2double(__builtin_amdgcn_readlane(__double2hiint(v), lane),
                            __builtin_amdgcn_readlane(__double2loint(v), lane));
}
__device__ __forceinline__ double wave_sum(double v)
{
    v += dpp_f64<kDppQuadSwap1>(v);
    v += dpp_f64<kDppQuadSwap2>(v);
    v += dpp_f64<kDppHalfMirror>(v);
    v += dpp_f64<kDppRowMirror>(v);
    return (readlane_f64(v, 0) + readlane_f64(v, 16)) + (readlane_f64(v, 32) + readlane_f64(v, 48));
}
__device__ __forceinline__ float wave_min(float v)
{
    v = fminf(v, dpp_f32<kDppQuadSwap1>(v));
    v = fminf(v, dpp_f32<kDppQuadSwap2>(v));
    v = fminf(v, dpp_f32<kDppHalfMirror>(v));
    v = fminf(v, dpp_f32<kDppRowMirror>(v));
    const int b = __float_as_int(v);
    return fminf(fminf(__int_as_float(__builtin_amdgcn_readlane(b, 0)), __int_as_float(__builtin_amdgcn_readlane(b, 16))),
                 fminf(__int_as_float(__builtin_amdgcn_readlane(b, 32)), __int_as_float(__builtin_amdgcn_readlane(b, 48))));
}
__device__ __forceinline__ float wave_max(float v)
{
    v = fmaxf(v, dpp_f32<kDppQuadSwap1>(v));
    v = fmaxf(v, dpp_f32<kDppQuadSwap2>(v));
    v = fmaxf(v, dpp_f32<kDppHalfMirror>(v));
    v = fmaxf(v, dpp_f32<kDppRowMirror>(v));
    const int b = __float_as_int(v);
    return fmaxf(fmaxf(__int_as_float(__builtin_amdgcn_readlane(b, 0)), __int_as_float(__builtin_amdgcn_readlane(b, 16))),
                 fmaxf(__int_as_float(__builtin_amdgcn_readlane(b, 32)), __int_as_float(__builtin_amdgcn_readlane(b, 48))));
}
__device__ __forceinline__ uint32_t wave_sum_u32(uint32_t v)
{
    int x = (int)v;
    x += dpp_i32<kDppQuadSwap1>(x);
    x += dpp_i32<kDppQuadSwap2>(x);
    x += dpp_i32<kDppHalfMirror>(x);
    x += dpp_i32<kDppRowMirror>(x);
    return (uint32_t)(__builtin_amdgcn_readlane(x, 0) + __builtin_amdgcn_readlane(x, 16) +
                      __builtin_amdgcn_readlane(x, 32) + __builtin_amdgcn_readlane(x, 48));
}
__device__ __forceinline__ uint32_t wave_max_u32(uint32_t v)
{
    v = max(v, (uint32_t)dpp_i32<kDppQuadSwap1>((int)v));
    v = max(v, (uint32_t)dpp_i32<kDppQuadSwap2>((int)v));
    v = max(v, (uint32_t)dpp_i32<kDppHalfMirror>((int)v));
    v = max(v, (uint32_t)dpp_i32<kDppRowMirror>((int)v));
    const int b = (int)v;
    return max(max((uint32_t)__builtin_amdgcn_readlane(b, 0), (uint32_t)__builtin_amdgcn_readlane(b, 16)),
               max((uint32_t)__builtin_amdgcn_readlane(b, 32), (uint32_t)__builtin_amdgcn_readlane(b, 48)));
}

// ---- the per-element arithmetic of quantize / dequantize ------------------------------
// fp32, fixed order: clamp, subtract, multiply (not fused), round half to even, clamp.
// Returns the code as a float in [0, L].
__device__ __forceinline__ float quant_level(float x, float lo, float hi, float inv_scale, float L)
{
    const float xc = fminf(fmaxf(x, lo), hi);   // NaN -> lo
    const float d = xc - lo;
    const float t = d * inv_scale;
    const float r = rintf(t);
    return fminf(fmaxf(r, 0.0f), L);            // NaN -> 0
}
// A value that every lane of the wave holds: moves it to a scalar register.
__device__ __forceinline__ float wave_uniform(float v)
{
    return __builtin_bit_cast(float, __builtin_amdgcn_readfirstlane(__builtin_bit_cast(int, v)));
}
// lo + c*scale rounded once.
__device__ __forceinline__ float dequant_level(float c, float scale, float lo)
{
    return __builtin_fmaf(c, scale, lo);
}

// ---- statistics: partials -> record ------------------------------------------------------
// Run by one whole block of kFinThreads lanes after both streaming passes have completed (a
// kernel boundary, so no fences are needed).  Everything is added in a fixed order.
constexpr int kFinThreads = 512;   // same block size as pass 2, so that both reduce the pass-1 partials identically

// Sum of the pass-1 partials over one block of T lanes, in an order that depends only on T:
// pass 2 (for mu, min, max) and the finalizer (for the record) get bit-identical values.
// DEV: the partials were written by other blocks of the same kernel (read them coherently).
template <int T, bool DEV = false>
__device__ __forceinline__ Part1 reduce_part1_block(const Part1 *__restrict__ part1, uint32_t nb1, Part1 *sh /*[T / 64]*/)
{
    const uint32_t tid = threadIdx.x, wave = tid / kWave, lane = tid % kWave;
    Part1 t{0.0, 0.0, INFINITY, -INFINITY, 0u, 0u};
    for (uint32_t i = tid; i < nb1; i += T) {
        Part1 p;
        if constexpr (DEV) p = ld_dev(part1 + i);
        else p = part1[i];
        t.sum += p.sum;
        t.sum_abs += p.sum_abs;
        t.mn = fminf(t.mn, p.mn);
        t.mx = fmaxf(t.mx, p.mx);
        t.bad += p.bad;
    }
    t.sum = wave_sum(t.sum);
    t.sum_abs = wave_sum(t.sum_abs);
    t.mn = wave_min(t.mn);
    t.mx = wave_max(t.mx);
    t.bad = wave_sum_u32(t.bad);
    if (lane == 0) sh[wave] = t;
    __syncthreads();
    Part1 tot = sh[0];
#pragma unroll
    for (int w = 1; w < T / kWave; ++w) {
        tot.sum += sh[w].sum;
        tot.sum_abs += sh[w].sum_abs;
        tot.mn = fminf(tot.mn, sh[w].mn);
        tot.mx = fmaxf(tot.mx, sh[w].mx);
        tot.bad += sh[w].bad;
    }
    return tot;
}

// The statistics record from the tensor-wide sums (Sec. 3: mu and b_E of the Laplace model, the
// histogram's peak density and the bound b_R = 1 / (2 peak density) it gives).
__device__ inline qp_stats_t stats_record(const Part1 &a, const Part2 &b, uint32_t pk, uint32_t nbins, uint64_t n)
{
    qp_stats_t st;
    st.n = n;
    st.n_nonfinite = a.bad;
    st.mean = a.sum / (double)n;
    st.mad = b.dev / (double)n;
    st.abs_mean = a.sum_abs / (double)n;
    st.var = b.sq / (double)n;
    st.min = (double)a.mn;
    st.max = (double)a.mx;
    st.nbins = nbins;
    st.peak_count = pk;
    if (a.mx == a.mn) {   // one distinct value: the density peak is unbounded, the bound is 0
        st.peak_density = 0.0;
        st.b_r = 0.0;
    } else {
        const double binw = ((double)a.mx - (double)a.mn) / (double)nbins;
        st.peak_density = (double)pk / ((double)n * binw);
        st.b_r = 1.0 / (2.0 * st.peak_density);
    }
    return st;
}

// DEV: the pass-2 partials and the histogram come from other blocks of the SAME kernel (the block
// that draws pass 2's last ticket finalizes): they are read with device-coherent loads.
template <bool DEV = false>
__device__ inline void finalize_stats_block(const Part1 *__restrict__ part1, uint32_t nb1,
                                            const Part2 *__restrict__ part2, uint32_t nb2,
                                            const uint32_t *__restrict__ hist, uint32_t nbins, uint64_t n,
                                            qp_stats_t *__restrict__ out)
{
    __shared__ Part1 f1[kFinThreads / kWave];
    __shared__ Part2 f2[kFinThreads / kWave];
    __shared__ uint32_t fpk[kFinThreads / kWave];
    const uint32_t tid = threadIdx.x, wave = tid / kWave, lane = tid % kWave;
    // The pass-2 partials and the histogram are requested before the pass-1 partials are reduced (that
    // reduction holds a barrier, which loads do not cross by themselves): one trip to memory, not three.
    static_assert(kMaxStat2Blocks <= kFinThreads && kMaxBins <= 8 * kFinThreads, "one partial and eight bins per lane");
    Part2 q{0.0, 0.0};
    if (tid < nb2) {
        if constexpr (DEV) q = Part2{ld_dev(&part2[tid].dev), ld_dev(&part2[tid].sq)};
        else q = part2[tid];
    }
    uint32_t h[8];
#pragma unroll
    for (uint32_t k = 0; k < 8; ++k) {
        const uint32_t b = tid + k * kFinThreads;
        h[k] = 0u;
        if (b < nbins) h[k] = DEV ? ld_dev(&hist[b]) : hist[b];
    }
    const Part1 a = reduce_part1_block<kFinThreads>(part1, nb1, f1);
    uint32_t peak = 0u;
#pragma unroll
    for (uint32_t k = 0; k < 8; ++k) peak = max(peak, h[k]);
    q.dev = wave_sum(q.dev);
    q.sq = wave_sum(q.sq);
    peak = wave_max_u32(peak);
    if (lane == 0) {
        f2[wave] = q;
        fpk[wave] = peak;
    }
    __syncthreads();
    if (tid == 0) {
        Part2 b = f2[0];
        uint32_t pk = fpk[0];
        for (int w = 1; w < kFinThreads / kWave; ++w) {
            b.dev += f2[w].dev;
            b.sq += f2[w].sq;
            pk = max(pk, fpk[w]);
        }
        const qp_stats_t st = stats_record(a, b, pk, nbins, n);
        *out = st;
    }
    __syncthreads();   // the record is visible to the whole block from here on
}

// The grid a clipping threshold induces; same statement as qp_make_qparams on the host.  With
// `clip` the range is first intersected with [mn, mx] (the data's range) and an empty range gives
// scale 0, as in qp_make_qparams_clipped.
__device__ __host__ inline void make_grid(double center, double alpha, uint32_t bits, float &lo, float &hi,
                                          float &scale, float &inv_scale, bool clip = false, float mn = 0.0f,
                                          float mx = 0.0f)
{
    const float a32 = (float)alpha;
    const float c32 = (float)center;
    const double L = (double)((1u << bits) - 1u);
    lo = (float)((double)c32 - (double)a32);
    hi = (float)((double)c32 + (double)a32);
    bool empty = (hi == lo);
    if (clip) {
        if (lo < mn) lo = mn;
        if (hi > mx) hi = mx;
        empty = !(hi > lo);
    }
    if (empty) {
        scale = 0.0f;
        inv_scale = 0.0f;
    } else {
        const double range = (double)hi - (double)lo;
        scale = (float)(range / L);
        inv_scale = (float)(L / range);
    }
}

// What the host decides about one search: the model, the constant of its threshold, the sweep.
struct SearchPlan {
    uint32_t bits, t_steps, cpr;
    double C;            // F(q) (Laplace) or G(q) (Gaussian): alpha = C * scale
    double C_alt;        // dist == QP_DIST_AUTO: C is F(q) and this is G(q); the device picks
    uint32_t dist;       // QP_LAPLACE / QP_GAUSS / QP_DIST_AUTO
    uint32_t clip;       // intersect candidate ranges with the data's range
    uint32_t stride;     // 1: all t + 1 candidates; > 1: coarse sweep with this stride, then a fine one
    uint32_t aciq_only;  // 1: score nothing, the result is plain ACIQ (j = 0)
};

// The two ends of the scale grid under a model: the moment estimate and the bound given by the
// histogram's peak.  Laplace (Sec. 3): b_E = MAD, b_R = 1 / (2 max D_R).  Gaussian: sigma_E =
// sqrt(var), sigma_R = 1 / (sqrt(2 pi) max D_R); 0 when the data has one distinct value.
__device__ __host__ inline void scale_ends(const qp_stats_t &st, uint32_t dist, double &s_e, double &s_r)
{
    if (dist == QP_GAUSS) {
        s_e = sqrt(st.var);
        s_r = (st.peak_density == 0.0) ? 0.0 : 1.0 / (2.5066282746310002 /* sqrt(2 pi) */ * st.peak_density);
    } else {
        s_e = st.mad;
        s_r = st.b_r;
    }
}

// First minimum of scores[0 .. ncand) taken by one full wave: a candidate replaces the incumbent
// only if its score is strictly lower, so ties keep the smaller index (b_E is kept unless
// something is strictly better) and a NaN score never wins.  Lanes scan j = lane, lane + 64, ...
// in ascending order, then a shuffle tree.  Every lane returns the winner's index.  (The caller
// applies the rule that a NaN score of plain ACIQ, j = 0, is never beaten.)
__device__ __forceinline__ uint32_t first_min_wave(const double *scores, uint32_t ncand, uint32_t lane)
{
    double bs = INFINITY;
    uint32_t bj = 0xffffffffu;
    for (uint32_t j = lane; j < ncand; j += kWave) {
        const double s = scores[j];
        if (bj == 0xffffffffu || s < bs) {
            bs = (s == s) ? s : INFINITY;
            bj = j;
        }
    }
#pragma unroll
    for (int o = kWave / 2; o > 0; o >>= 1) {
        const double os = __shfl_xor(bs, o, kWave);
        const uint32_t oj = __shfl_xor(bj, o, kWave);
        if (os < bs || (os == bs && oj < bj)) {
            bs = os;
            bj = oj;
        }
    }
    return bj;
}

// What the winner of a candidate list means for the search, written by one lane: the result
// record, the winner's grid and (for the fine sweep that may follow) the score of j = 0.
// `scores` holds the list's scores; in a coarse-to-fine search they are also scattered to
// scores_by_j (which the set-up filled with NaN).
__device__ inline void write_search_result(Ctl *ctl, const double *scores, uint32_t ncand, uint32_t bi, uint64_t n_total,
                                           double *scores_by_j, qp_search_result_t *res, qp_qparams_t *best)
{
    const uint32_t mode = ctl->list_mode, stride = ctl->list_stride, j1 = ctl->list_j1, t = ctl->t_steps;
    // plain ACIQ's score: entry 0 of the full and of the coarse list; the fine list may not hold j = 0
    const double s0 = (mode == kListFine) ? ctl->score0 : scores[0];
    uint32_t j = list_index(mode, stride, j1, t, bi);
    double sbest = scores[bi];
    if (!(s0 == s0)) {   // a NaN incumbent is never beaten
        j = 0u;
        sbest = s0;
    }
    if (mode != kListFull)
        for (uint32_t i = 0; i < ncand; ++i) scores_by_j[list_index(mode, stride, j1, t, i)] = scores[i];
    qp_search_result_t r;
    r.b_e = ctl->b_e;
    r.b_r = ctl->b_r;
    r.b_star = ctl->b_e + (double)j * ctl->step;
    r.alpha_star = ctl->F * r.b_star;
    r.mse_aciq = s0 / (double)n_total;
    r.mse_star = sbest / (double)n_total;
    r.j_star = j;
    r.t_steps = t;
    *res = r;
    qp_qparams_t q;
    q.bits = ctl->bits;
    q.reserved = 0u;
    q.n = n_total;
    make_grid(ctl->mean, r.alpha_star, ctl->bits, q.lo, q.hi, q.scale, q.inv_scale, ctl->clip != 0u, ctl->clip_lo,
              ctl->clip_hi);
    *best = q;
    ctl->score0 = s0;
    ctl->ticket_search = 0u;
}

// What a kernel needs to build one sweep's candidate table.
struct ModelArgs {
    double mean_h, s_e_h, s_r_h;    // statistics from the host (from_ws == 0): mean and the two scale ends
    float clip_lo_h, clip_hi_h;     // ... and the data's range
    int from_ws;                    // 1: take them from the statistics record in the workspace
    uint32_t dist, clip;
    uint32_t list_mode, list_stride, count;   // the sweep: count candidates, list entry i -> grid index j
    uint32_t bits, t_steps;
    double C;
    double C_alt;                   // dist == QP_DIST_AUTO: the Gaussian constant (C holds the Laplace one)
    const qp_model_fit_t *model;    // ... and the record that says which model the tensor's histogram fits
};

// A search with dist = QP_DIST_AUTO: the model that the fit (k_model_fit, an earlier kernel on the stream) chose.
__device__ inline ModelArgs resolve_model(ModelArgs m)
{
    if (m.dist == QP_DIST_AUTO) {
        const bool gauss = m.model->dist == QP_GAUSS;
        m.dist = gauss ? QP_GAUSS : QP_LAPLACE;
        if (gauss) m.C = m.C_alt;
    }
    return m;
}

// The scalars every candidate of a search shares: the centre, the two ends of the scale grid and its step
// (Eq. 1), and the data's range.  A bound or estimate that is zero, negative or not finite collapses the
// grid onto s_E (step 0).
struct GridModel {
    double mean, s_e, s_r, step;
    float clo, chi;
};
__device__ inline GridModel grid_model(const ModelArgs &m, const qp_stats_t *st)
{
    GridModel g{m.mean_h, m.s_e_h, m.s_r_h, 0.0, m.clip_lo_h, m.clip_hi_h};
    if (st) {
        g.mean = st->mean;
        scale_ends(*st, m.dist, g.s_e, g.s_r);
        g.clo = (float)st->min;
        g.chi = (float)st->max;
    }
    g.step = (g.s_r - g.s_e) / (double)m.t_steps;
    const bool ok = (g.s_e > 0.0) && (g.s_r > 0.0) && isfinite(g.s_r) && isfinite(g.s_e) && isfinite(g.step);
    if (!ok) g.step = 0.0;
    return g;
}

// The grid of candidate j: scale s_j = s_E + j step, alpha_j = C s_j, centred on the mean (Eq. 1).
// `safe` tells whether the search may use its short per-element sequence for it.  The full sequence
// clamps twice: x to [lo, hi] before the subtraction and the rounded level to [0, L] after it.  With x
// already clamped, d = x - lo lies in [0, fl(hi - lo)], t = d*inv is monotone in d (inv >= 0) and rounding
// is monotone, so the level lies in [0, rint(fl(fl(hi - lo)*inv))]: if that upper end, evaluated here in
// the kernels' own fp32 arithmetic, is at most L (it is whenever the range is a normal number), the second
// clamp can never act.
__device__ inline Cand candidate_grid(const ModelArgs &m, const GridModel &g, uint32_t j, int &safe)
{
    const double s_j = g.s_e + (double)j * g.step;
    Cand c;
    make_grid(g.mean, m.C * s_j, m.bits, c.lo, c.hi, c.scale, c.inv_scale, m.clip != 0u, g.clo, g.chi);
    const float Lf = (float)((1u << m.bits) - 1u);
    const float top = rintf((c.hi - c.lo) * c.inv_scale);
    safe = (isfinite(c.lo) && isfinite(c.hi) && top >= 0.0f && top <= Lf) ? 1 : 0;
    return c;
}

// The control record of a search, written by one lane.
__device__ inline void write_ctl(Ctl *ctl, const ModelArgs &m, const GridModel &g, int safe, uint32_t j1, uint64_t n)
{
    ctl->ticket_search = 0u;
    ctl->short_seq = (uint32_t)safe;
    ctl->clip = m.clip;
    ctl->b_e = g.s_e;
    ctl->b_r = g.s_r;
    ctl->step = g.step;
    ctl->F = m.C;
    ctl->mean = g.mean;
    ctl->bits = m.bits;
    ctl->t_steps = m.t_steps;
    ctl->n = n;
    ctl->list_mode = m.list_mode;
    ctl->list_stride = m.list_stride;
    ctl->list_j1 = j1;
    ctl->clip_lo = g.clo;
    ctl->clip_hi = g.chi;
}

// Run by a whole block: candidate i of the list gets the grid of its index j (list_index).  Writes the
// table to cands_a (and cands_b if given), the control record if given, and before a coarse sweep fills
// scores_by_j with NaN ("not evaluated").  Returns (to every lane) whether the search may use its short
// per-element sequence for every candidate of the list.
__device__ inline int setup_candidates(const ModelArgs &m, const qp_stats_t *st, uint32_t j1, uint64_t n, Cand *cands_a,
                                       Cand *cands_b, Ctl *ctl, double *scores_by_j)
{
    const GridModel g = grid_model(m, st);
    int safe = 1;
    for (uint32_t i = threadIdx.x; i < m.count; i += blockDim.x) {
        const uint32_t j = list_index(m.list_mode, m.list_stride, j1, m.t_steps, i);
        int ok;
        const Cand c = candidate_grid(m, g, j, ok);
        cands_a[i] = c;
        if (cands_b) cands_b[i] = c;
        if (!ok) safe = 0;
    }
    if (scores_by_j && m.list_mode == kListCoarse)
        for (uint32_t j = threadIdx.x; j <= m.t_steps; j += blockDim.x) scores_by_j[j] = __longlong_as_double(0x7ff8000000000000ll);
    safe = __syncthreads_and(safe);
    if (ctl && threadIdx.x == 0) write_ctl(ctl, m, g, safe, j1, n);
    return safe;
}

// What a search kernel needs to turn the partials of the statistics passes into the record itself
// (the sender path launches no separate finalizer).
struct FinalizeArgs {
    const Part1 *part1;
    const Part2 *part2;
    const uint32_t *hist;
    uint32_t nb1, nb2, nbins;   // nbins == 0: nothing to finalize
};

// Tensors of at most this many elements are searched with one candidate per lane.
#ifndef QP_TILE_SEARCH_MAX_N
#define QP_TILE_SEARCH_MAX_N (1ull << 21)
#endif
constexpr uint64_t kTileSearchMaxN = QP_TILE_SEARCH_MAX_N;

inline uint32_t ceil_div_u64(uint64_t a, uint64_t b) { return (uint32_t)((a + b - 1) / b); }

// Kernel launchers (one per translation unit); all return hipError_t from hipGetLastError().
// The two streaming passes of the statistics; `finalize` adds the one-block kernel that turns the
// partials into the qp_stats_t record (left out when the search set-up kernel will do it).
hipError_t launch_stats(const void *x, uint64_t n, int dtype, uint32_t nbins, void *ws, hipStream_t s, bool finalize);
void stats_grid(uint64_t n, int dtype, uint32_t &nb1, uint32_t &nb2);
// Set-up + search.  stats_host_or_null: statistics from the host, else they are taken from the
// workspace; finalize_nbins != 0: the search first finalizes the statistics that
// launch_stats(..., finalize = false) left as partials (histogram of finalize_nbins bins).
hipError_t launch_search(const void *x, uint64_t n, int dtype, const SearchPlan &plan, const qp_stats_t *stats_host_or_null,
                         uint32_t finalize_nbins, bool value_table_ready, void *ws, hipStream_t s);
// Large bf16 tensors: the table of value counts (zeroed and built in one pass over the tensor) and the
// statistics record and histogram computed from it.
bool uses_value_table(uint64_t n, int dtype);
hipError_t launch_value_table(const void *x, uint64_t n, void *ws, hipStream_t s);
hipError_t launch_stats_from_table(uint64_t n, uint32_t nbins, void *ws, hipStream_t s);
// The directed search over the value table (which must be built): one launch, no set-up kernel.
hipError_t launch_table_search(uint64_t n, const SearchPlan &plan, const qp_stats_t *stats_host_or_null, void *ws, hipStream_t s);
bool coarse_to_fine_supported(uint64_t n, int dtype, const SearchPlan &plan);
// The host's part of ModelArgs for one sweep of a plan.
ModelArgs model_args(const SearchPlan &plan, const qp_stats_t *stats_host_or_null, uint32_t list_mode, uint32_t count,
                     const void *ws);
// Which model the histogram in the workspace fits (one block; writes the qp_model_fit_t record).
hipError_t launch_model_fit(void *ws, hipStream_t s);
uint32_t search_blocks(uint64_t n);
hipError_t launch_hist_search(uint32_t bits, uint32_t t_steps, double F, void *ws, hipStream_t s);
hipError_t launch_quant_pack(const void *x, uint64_t n, int dtype, uint32_t bits, const qp_qparams_t *host_qp,
                             const qp_qparams_t *dev_qp, void *packed, hipStream_t s);
// The search with one candidate per lane over LDS-staged tiles, for tensors of at most
// kTileSearchMaxN elements and at most 256 candidates (same arguments as launch_search).
bool tile_search_eligible(uint64_t n, const SearchPlan &plan);
bool tile_search_can_run(const SearchPlan &plan);
uint32_t tile_search_blocks(uint64_t n);
hipError_t launch_tile_search(const void *x, uint64_t n, int dtype, const SearchPlan &plan,
                              const qp_stats_t *stats_host_or_null, uint32_t finalize_nbins, void *ws, hipStream_t s);
hipError_t launch_unpack_dequant(const void *packed, uint32_t bits, const qp_qparams_t *host_qp,
                                 const qp_qparams_t *dev_qp, float *y, uint64_t n, hipStream_t s);

}  // namespace qp
