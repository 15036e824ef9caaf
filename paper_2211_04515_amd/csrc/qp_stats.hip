// Step 1: per-tensor statistics and histogram (Sec. 3: mu and b of L(mu, b); the
// estimate b_E; the histogram D_R of the real data; the bound b_R from its peak).
//
// Two streaming passes, both HBM-bound (4 B per fp32 element each):
//   pass 1  sum, sum|x|, min, max, NaN/Inf count        -> one partial per block
//   pass 2  sum|x - mu|, sum (x - mu)^2, histogram      -> partial per block + LDS histogram
// Accumulation is fp64 per lane, reduced inside each wave64 with DPP lane permutations, one
// LDS slot per wave, then across blocks in a fixed order: no floating-point atomics, so
// results are bit-reproducible from run to run.  Pass 2 needs mu, min and max; every block of
// pass 2 re-reduces the (at most 1024) pass-1 partials itself, with its first loads of the
// tensor already in flight, which saves a launch and a grid-wide dependency.  A one-block
// kernel after pass 2 (or the search's set-up kernel, when the search follows) turns the
// partials and the histogram into the qp_stats_t record: kernel boundaries order the memory,
// so neither pass needs a fence.
#include "qp_common.hpp"

namespace qp {

constexpr int kS1Threads = 256;
constexpr int kS1Unroll = 4;     // 16-byte loads in flight per lane
constexpr int kS2Threads = 512;
constexpr int kS2Unroll = 4;

struct Acc1 {
    double s, sa;
    float mn, mx;
    uint32_t bad;
};

__device__ __forceinline__ void acc1_add(Acc1 &a, float v)
{
    const double d = (double)v;
    a.s += d;
    a.sa += fabs(d);
    a.mn = fminf(a.mn, v);
    a.mx = fmaxf(a.mx, v);
    a.bad += (__builtin_isfinite(v) ? 0u : 1u);
}

template <int DT>
__global__ __launch_bounds__(kS1Threads) void k_stats_pass1(const void *__restrict__ x, uint64_t n,
                                                            Part1 *__restrict__ part, uint32_t *__restrict__ hist,
                                                            uint32_t nbins, Ctl *__restrict__ ctl)
{
    const uint32_t tid = threadIdx.x;
    // Clear what pass 2 and the search accumulate into (they run after this kernel on the stream).
    if (blockIdx.x == 0) {
        for (uint32_t b = tid; b < nbins; b += kS1Threads) hist[b] = 0u;
        if (tid == 0) ctl->ticket_search = 0u;
    }

    Acc1 a0{0.0, 0.0, INFINITY, -INFINITY, 0u};
    Acc1 a1 = a0;
    const uint64_t nvec = n / 4;
    const uint64_t tile = (uint64_t)kS1Threads * kS1Unroll;
    uint64_t base = (uint64_t)blockIdx.x * tile;
    const uint64_t stride = (uint64_t)gridDim.x * tile;
    for (; base + tile <= nvec; base += stride) {
        float f[kS1Unroll][4];
#pragma unroll
        for (int u = 0; u < kS1Unroll; ++u) Vec4<DT>::load(x, base + (uint64_t)u * kS1Threads + tid, f[u]);
#pragma unroll
        for (int u = 0; u < kS1Unroll; ++u) {
            acc1_add(a0, f[u][0]);
            acc1_add(a1, f[u][1]);
            acc1_add(a0, f[u][2]);
            acc1_add(a1, f[u][3]);
        }
    }
    // the block whose turn it is takes the ragged remainder of whole vectors
    if (base < nvec) {
        for (uint64_t v = base + tid; v < nvec; v += kS1Threads) {
            float f[4];
            Vec4<DT>::load(x, v, f);
            acc1_add(a0, f[0]);
            acc1_add(a1, f[1]);
            acc1_add(a0, f[2]);
            acc1_add(a1, f[3]);
        }
    }
    // last n mod 4 elements
    if (blockIdx.x == 0 && tid < (uint32_t)(n - nvec * 4)) acc1_add(a0, Vec4<DT>::load1(x, nvec * 4 + tid));

    double s = wave_sum(a0.s + a1.s);
    double sa = wave_sum(a0.sa + a1.sa);
    float mn = wave_min(fminf(a0.mn, a1.mn));
    float mx = wave_max(fmaxf(a0.mx, a1.mx));
    uint32_t bad = wave_sum_u32(a0.bad + a1.bad);

    __shared__ Part1 sh[kS1Threads / kWave];
    const uint32_t wave = tid / kWave, lane = tid % kWave;
    if (lane == 0) sh[wave] = Part1{s, sa, mn, mx, bad, 0u};
    __syncthreads();
    if (tid == 0) {
        Part1 p = sh[0];
        for (int w = 1; w < kS1Threads / kWave; ++w) {
            p.sum += sh[w].sum;
            p.sum_abs += sh[w].sum_abs;
            p.mn = fminf(p.mn, sh[w].mn);
            p.mx = fmaxf(p.mx, sh[w].mx);
            p.bad += sh[w].bad;
        }
        part[blockIdx.x] = p;
    }
}

template <int DT>
__global__ __launch_bounds__(kS2Threads) void k_stats_pass2(const void *__restrict__ x, uint64_t n,
                                                            const Part1 *__restrict__ part1, uint32_t nb1,
                                                            Part2 *__restrict__ part2, uint32_t *__restrict__ hist,
                                                            uint32_t nbins)
{
    __shared__ uint32_t sh_hist[kMaxBins];
    __shared__ Part1 sh1[kS2Threads / kWave];
    __shared__ Part2 sh2[kS2Threads / kWave];
    const uint32_t tid = threadIdx.x;
    const uint32_t wave = tid / kWave, lane = tid % kWave;

    for (uint32_t b = tid; b < nbins; b += kS2Threads) sh_hist[b] = 0u;

    // the block's first tile is requested before anything else, so that the tensor is already
    // streaming while the pass-1 partials are being reduced
    const uint64_t nvec = n / 4;
    const uint64_t tile = (uint64_t)kS2Threads * kS2Unroll;
    uint64_t base = (uint64_t)blockIdx.x * tile;
    const uint64_t stride = (uint64_t)gridDim.x * tile;
    float pre[kS2Unroll][4];
    const bool have_pre = base + tile <= nvec;
    if (have_pre) {
#pragma unroll
        for (int u = 0; u < kS2Unroll; ++u) Vec4<DT>::load(x, base + (uint64_t)u * kS2Threads + tid, pre[u]);
    }

    // ---- every block reduces the pass-1 partials in the same fixed order ----
    static_assert(kS2Threads == kFinThreads, "pass 2 and the finalizer must reduce the partials identically");
    const Part1 tot = reduce_part1_block<kS2Threads>(part1, nb1, sh1);
    const double mean = tot.sum / (double)n;
    const float mn = tot.mn, mx = tot.mx;
    // bin index arithmetic in fp32: one subtraction and one division here (the fp64 quotient of
    // two fp32 values rounded to fp32 equals the correctly rounded fp32 quotient), then one
    // subtraction and one product per element
    const float range = mx - mn;
    const float w_inv = (float)((double)(float)nbins / (double)range);
    const float top = (float)(nbins - 1u);

    double dev0 = 0.0, dev1 = 0.0, sq0 = 0.0, sq1 = 0.0;
    auto add = [&](float v, double &dev, double &sq) {
        const double d = (double)v - mean;
        dev += fabs(d);
        sq = fma(d, d, sq);
        const float tt = (v - mn) * w_inv;
        const uint32_t idx = (uint32_t)fminf(fmaxf(tt, 0.0f), top);   // NaN (0*inf) -> 0
        atomicAdd(&sh_hist[idx], 1u);
    };
    if (have_pre) {
#pragma unroll
        for (int u = 0; u < kS2Unroll; ++u) {
            add(pre[u][0], dev0, sq0);
            add(pre[u][1], dev1, sq1);
            add(pre[u][2], dev0, sq0);
            add(pre[u][3], dev1, sq1);
        }
        base += stride;
    }
    for (; base + tile <= nvec; base += stride) {
        float f[kS2Unroll][4];
#pragma unroll
        for (int u = 0; u < kS2Unroll; ++u) Vec4<DT>::load(x, base + (uint64_t)u * kS2Threads + tid, f[u]);
#pragma unroll
        for (int u = 0; u < kS2Unroll; ++u) {
            add(f[u][0], dev0, sq0);
            add(f[u][1], dev1, sq1);
            add(f[u][2], dev0, sq0);
            add(f[u][3], dev1, sq1);
        }
    }
    if (base < nvec) {
        for (uint64_t v = base + tid; v < nvec; v += kS2Threads) {
            float f[4];
            Vec4<DT>::load(x, v, f);
            add(f[0], dev0, sq0);
            add(f[1], dev1, sq1);
            add(f[2], dev0, sq0);
            add(f[3], dev1, sq1);
        }
    }
    if (blockIdx.x == 0 && tid < (uint32_t)(n - nvec * 4)) add(Vec4<DT>::load1(x, nvec * 4 + tid), dev0, sq0);

    const double dev = wave_sum(dev0 + dev1);
    const double sq = wave_sum(sq0 + sq1);
    if (lane == 0) sh2[wave] = Part2{dev, sq};
    __syncthreads();   // also orders the LDS histogram updates before the merge below
    for (uint32_t b = tid; b < nbins; b += kS2Threads) {
        const uint32_t c = sh_hist[b];
        if (c) atomicAdd(&hist[b], c);
    }
    if (tid == 0) {
        Part2 p = sh2[0];
        for (int w = 1; w < kS2Threads / kWave; ++w) {
            p.dev += sh2[w].dev;
            p.sq += sh2[w].sq;
        }
        part2[blockIdx.x] = p;
    }
}

__global__ __launch_bounds__(kFinThreads) void k_stats_finalize(const Part1 *__restrict__ part1, uint32_t nb1,
                                                                const Part2 *__restrict__ part2, uint32_t nb2,
                                                                const uint32_t *__restrict__ hist, uint32_t nbins,
                                                                uint64_t n, qp_stats_t *__restrict__ out)
{
    finalize_stats_block(part1, nb1, part2, nb2, hist, nbins, n, out);
}

// Whole tiles per block: with T tiles and at most B blocks, every block takes ceil(T/B) tiles and
// the grid shrinks to the number of blocks that this needs.
void stats_grid(uint64_t n, uint32_t &nb1, uint32_t &nb2)
{
    const uint64_t nvec = n / 4;
    auto even_grid = [](uint64_t tiles, uint32_t max_blocks) -> uint32_t {
        if (tiles < 1) return 1u;
        const uint64_t per = (tiles + max_blocks - 1) / max_blocks;
        return (uint32_t)((tiles + per - 1) / per);
    };
    nb1 = even_grid((nvec + kS1Threads * kS1Unroll - 1) / (kS1Threads * kS1Unroll), kMaxStat1Blocks);
    nb2 = even_grid((nvec + kS2Threads * kS2Unroll - 1) / (kS2Threads * kS2Unroll), kMaxStat2Blocks);
}

hipError_t launch_stats_finalize(uint64_t n, uint32_t nbins, void *ws, hipStream_t s)
{
    char *w = static_cast<char *>(ws);
    uint32_t nb1, nb2;
    stats_grid(n, nb1, nb2);
    hipLaunchKernelGGL(k_stats_finalize, dim3(1), dim3(kFinThreads), 0, s, reinterpret_cast<const Part1 *>(w + kOffPart1),
                       nb1, reinterpret_cast<const Part2 *>(w + kOffPart2), nb2,
                       reinterpret_cast<const uint32_t *>(w + kOffHist), nbins, n,
                       reinterpret_cast<qp_stats_t *>(w + kOffStats));
    return hipGetLastError();
}

hipError_t launch_stats(const void *x, uint64_t n, int dtype, uint32_t nbins, void *ws, hipStream_t s, bool finalize)
{
    char *w = static_cast<char *>(ws);
    Part1 *p1 = reinterpret_cast<Part1 *>(w + kOffPart1);
    Part2 *p2 = reinterpret_cast<Part2 *>(w + kOffPart2);
    uint32_t *hist = reinterpret_cast<uint32_t *>(w + kOffHist);
    Ctl *ctl = reinterpret_cast<Ctl *>(w + kOffCtl);
    uint32_t nb1, nb2;
    stats_grid(n, nb1, nb2);
    if (dtype == QP_F32) {
        hipLaunchKernelGGL(k_stats_pass1<QP_F32>, dim3(nb1), dim3(kS1Threads), 0, s, x, n, p1, hist, nbins, ctl);
        hipLaunchKernelGGL(k_stats_pass2<QP_F32>, dim3(nb2), dim3(kS2Threads), 0, s, x, n, p1, nb1, p2, hist, nbins);
    } else {
        hipLaunchKernelGGL(k_stats_pass1<QP_BF16>, dim3(nb1), dim3(kS1Threads), 0, s, x, n, p1, hist, nbins, ctl);
        hipLaunchKernelGGL(k_stats_pass2<QP_BF16>, dim3(nb2), dim3(kS2Threads), 0, s, x, n, p1, nb1, p2, hist, nbins);
    }
    hipError_t e = hipGetLastError();
    if (e != hipSuccess || !finalize) return e;
    return launch_stats_finalize(n, nbins, ws, s);
}

}  // namespace qp
