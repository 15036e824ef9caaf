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
constexpr uint32_t kMaxStat1Blocks = 1024; // capacity of the pass-1 partial array
constexpr uint32_t kMaxStat2Blocks = 512;
constexpr uint32_t kMaxSearchBlocks = 1024;

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

// Device-resident control block.
struct Ctl {
    uint32_t ticket_stats2;   // blocks of the second statistics pass that have finished
    uint32_t ticket_search;   // blocks of the search kernel that have finished
    uint32_t pad0, pad1;
    double b_e, b_r, step, F; // search grid: b_j = b_e + j*step, alpha_j = F*b_j
    double mean;
    uint32_t bits, t_steps;
    uint64_t n;
};

// Workspace layout (byte offsets).  Fixed-size regions first, the search partials last.
constexpr size_t kOffStats = 0;                                   // qp_stats_t (88 B)
constexpr size_t kOffResult = 128;                                // qp_search_result_t (56 B)
constexpr size_t kOffQParams = 192;                               // qp_qparams_t (32 B)
constexpr size_t kOffCtl = 256;                                   // Ctl
constexpr size_t kOffHist = 512;                                  // uint32_t[kMaxBins]
constexpr size_t kOffCands = kOffHist + kMaxBins * 4;             // Cand[kMaxT + 1]
constexpr size_t kOffScores = kOffCands + (kMaxT + 1) * sizeof(Cand);   // double[kMaxT + 1]
constexpr size_t kOffPart1 = kOffScores + (kMaxT + 1) * 8;        // Part1[kMaxStat1Blocks]
constexpr size_t kOffPart2 = kOffPart1 + kMaxStat1Blocks * sizeof(Part1);  // Part2[kMaxStat2Blocks]
constexpr size_t kOffSearchPart = kOffPart2 + kMaxStat2Blocks * sizeof(Part2);  // double[blocks][t + 1]
static_assert(sizeof(qp_stats_t) <= 128 && sizeof(qp_search_result_t) <= 64 && sizeof(qp_qparams_t) == 32 &&
              sizeof(Ctl) <= 256, "fixed workspace regions");
static_assert(kOffSearchPart % 16 == 0, "alignment");

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

// ---- wave64 reductions (shuffles), then one LDS slot per wave -------------------------
__device__ __forceinline__ double wave_sum(double v)
{
#pragma unroll
    for (int o = kWave / 2; o > 0; o >>= 1) v += __shfl_xor(v, o, kWave);
    return v;
}
__device__ __forceinline__ float wave_min(float v)
{
#pragma unroll
    for (int o = kWave / 2; o > 0; o >>= 1) v = fminf(v, __shfl_xor(v, o, kWave));
    return v;
}
__device__ __forceinline__ float wave_max(float v)
{
#pragma unroll
    for (int o = kWave / 2; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, kWave));
    return v;
}
__device__ __forceinline__ uint32_t wave_sum_u32(uint32_t v)
{
#pragma unroll
    for (int o = kWave / 2; o > 0; o >>= 1) v += __shfl_xor(v, o, kWave);
    return v;
}
__device__ __forceinline__ uint32_t wave_max_u32(uint32_t v)
{
#pragma unroll
    for (int o = kWave / 2; o > 0; o >>= 1) v = max(v, (uint32_t)__shfl_xor(v, o, kWave));
    return v;
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
// lo + c*scale rounded once.
__device__ __forceinline__ float dequant_level(float c, float scale, float lo)
{
    return __builtin_fmaf(c, scale, lo);
}

// The grid a clipping threshold induces; same statement as qp_make_qparams on the host.
__device__ __host__ inline void make_grid(double center, double alpha, uint32_t bits, float &lo, float &hi,
                                          float &scale, float &inv_scale)
{
    const float a32 = (float)alpha;
    const float c32 = (float)center;
    const double L = (double)((1u << bits) - 1u);
    lo = (float)((double)c32 - (double)a32);
    hi = (float)((double)c32 + (double)a32);
    if (hi == lo) {
        scale = 0.0f;
        inv_scale = 0.0f;
    } else {
        const double range = (double)hi - (double)lo;
        scale = (float)(range / L);
        inv_scale = (float)(L / range);
    }
}

inline uint32_t ceil_div_u64(uint64_t a, uint64_t b) { return (uint32_t)((a + b - 1) / b); }

// Kernel launchers (one per translation unit); all return hipError_t from hipGetLastError().
hipError_t launch_stats(const void *x, uint64_t n, int dtype, uint32_t nbins, void *ws, hipStream_t s);
hipError_t launch_search(const void *x, uint64_t n, int dtype, uint32_t bits, uint32_t t_steps, uint32_t cpr,
                         double F, const qp_stats_t *stats_host_or_null, void *ws, hipStream_t s);
uint32_t search_blocks(uint64_t n);
hipError_t launch_quant_pack(const void *x, uint64_t n, int dtype, uint32_t bits, const qp_qparams_t *host_qp,
                             const qp_qparams_t *dev_qp, void *packed, hipStream_t s);
hipError_t launch_unpack_dequant(const void *packed, uint32_t bits, const qp_qparams_t *host_qp,
                                 const qp_qparams_t *dev_qp, float *y, uint64_t n, hipStream_t s);

}  // namespace qp
