// Step 1: per-tensor statistics and histogram (Sec. 3: mu and b of L(mu, b); the
// estimate b_E; the histogram D_R of the real data; the bound b_R from its peak).
//
// Two streaming passes, both HBM-bound (4 B per fp32 element each), 16-byte loads (4 fp32 or 8
// bf16 elements per lane):
//   pass 1  sum, sum|x|, min, max, NaN/Inf count        -> one partial per block
//   pass 2  sum|x - mu|, sum (x - mu)^2, histogram      -> partial per block + LDS histogram
// Accumulation is fp64 per lane, reduced inside each wave64 with DPP lane permutations, one
// LDS slot per wave, then across blocks in a fixed order: no floating-point atomics, so
// results are bit-reproducible from run to run.  Pass 2 needs mu, min and max; every block of
// pass 2 re-reduces the (at most 512) pass-1 partials itself, with its first loads of the
// tensor already in flight, which saves a launch and a grid-wide dependency.  The partials and
// the histogram become the qp_stats_t record either in the search that follows (the sender
// path) or in the block of pass 2 that draws the last ticket.  That hand-over uses
// device-coherent stores and loads plus a relaxed ticket, so it costs no cache write-back or
// invalidation (with a release/acquire pair per block it cost more than a separate one-block
// kernel; that kernel, 4 us and a launch gap, is what the ticket now saves).
#include "qp_common.hpp"

namespace qp {

constexpr int kS1Threads = 256;
constexpr int kS1Unroll = 4;     // 16-byte loads in flight per lane
constexpr int kS2Threads = 512;
constexpr int kS2Unroll = 4;
constexpr uint32_t kHistWords = 16384;   // 64 KB of LDS: two blocks of pass 2 per CU
// copies of the LDS histogram: as many as fit, at most 8 (2048 bins -> 8, 4096 -> 4)
inline uint32_t hist_rep_shift(uint32_t nbins)
{
    uint32_t s = 0;
    while (s < 3 && (nbins << (s + 1)) <= kHistWords) ++s;
    return s;
}

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
        if (tid == 0) {
            ctl->ticket_search = 0u;
            ctl->ticket_stats = 0u;
        }
    }

    Acc1 a0{0.0, 0.0, INFINITY, -INFINITY, 0u};
    Acc1 a1 = a0;
    constexpr int E = Vec16<DT>::kElems;   // elements per 16-byte load
    const uint64_t nvec = n / E;
    const uint64_t tile = (uint64_t)kS1Threads * kS1Unroll;
    uint64_t base = (uint64_t)blockIdx.x * tile;
    const uint64_t stride = (uint64_t)gridDim.x * tile;
    for (; base + tile <= nvec; base += stride) {
        float f[kS1Unroll][E];
#pragma unroll
        for (int u = 0; u < kS1Unroll; ++u) Vec16<DT>::load(x, base + (uint64_t)u * kS1Threads + tid, f[u]);
#pragma unroll
        for (int u = 0; u < kS1Unroll; ++u) {
#pragma unroll
            for (int e = 0; e < E; e += 2) {
                acc1_add(a0, f[u][e]);
                acc1_add(a1, f[u][e + 1]);
            }
        }
    }
    // the block whose turn it is takes the ragged remainder of whole vectors
    if (base < nvec) {
        for (uint64_t v = base + tid; v < nvec; v += kS1Threads) {
            float f[E];
            Vec16<DT>::load(x, v, f);
#pragma unroll
            for (int e = 0; e < E; e += 2) {
                acc1_add(a0, f[e]);
                acc1_add(a1, f[e + 1]);
            }
        }
    }
    // last n mod E elements
    if (blockIdx.x == 0 && tid < (uint32_t)(n - nvec * E)) acc1_add(a0, Vec4<DT>::load1(x, nvec * E + tid));

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

// REP_SHIFT: log2 of the number of LDS histogram copies (compile-time so that the address is one
// shift-add).
template <int DT, int REP_SHIFT>
__global__ __launch_bounds__(kS2Threads) void k_stats_pass2(const void *__restrict__ x, uint64_t n,
                                                            const Part1 *__restrict__ part1, uint32_t nb1,
                                                            Part2 *__restrict__ part2, uint32_t *__restrict__ hist,
                                                            uint32_t nbins, Ctl *__restrict__ ctl,
                                                            qp_stats_t *__restrict__ out /* null: leave the partials */)
{
    // The LDS histogram is kept in `rep` interleaved copies (copy = lane mod rep): lanes that hit the
    // same bin then update different addresses in different banks, which divides the serialisation
    // of LDS atomics on peaked data (most of the mass in a few bins) by rep.
    __shared__ uint32_t sh_hist[kHistWords];
    __shared__ Part1 sh1[kS2Threads / kWave];
    __shared__ Part2 sh2[kS2Threads / kWave];
    const uint32_t tid = threadIdx.x;
    const uint32_t wave = tid / kWave, lane = tid % kWave;

    constexpr uint32_t rep_shift = REP_SHIFT;
    const uint32_t copy = tid & ((1u << rep_shift) - 1u);
    for (uint32_t b = tid; b < (nbins << rep_shift); b += kS2Threads) sh_hist[b] = 0u;

    // the block's first tile is requested before anything else, so that the tensor is already
    // streaming while the pass-1 partials are being reduced
    constexpr int E = Vec16<DT>::kElems;   // elements per 16-byte load
    const uint64_t nvec = n / E;
    const uint64_t tile = (uint64_t)kS2Threads * kS2Unroll;
    uint64_t base = (uint64_t)blockIdx.x * tile;
    const uint64_t stride = (uint64_t)gridDim.x * tile;
    float pre[kS2Unroll][E];
    const bool have_pre = base + tile <= nvec;
    if (have_pre) {
#pragma unroll
        for (int u = 0; u < kS2Unroll; ++u) Vec16<DT>::load(x, base + (uint64_t)u * kS2Threads + tid, pre[u]);
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
        // clamp to [0, nbins-1] in one operation; a NaN (0*inf when min == max) gives 0
        const uint32_t idx = (uint32_t)__builtin_amdgcn_fmed3f(tt, 0.0f, top);
        atomicAdd(&sh_hist[(idx << rep_shift) + copy], 1u);
    };
    if (have_pre) {
#pragma unroll
        for (int u = 0; u < kS2Unroll; ++u) {
#pragma unroll
            for (int e = 0; e < E; e += 2) {
                add(pre[u][e], dev0, sq0);
                add(pre[u][e + 1], dev1, sq1);
            }
        }
        base += stride;
    }
    for (; base + tile <= nvec; base += stride) {
        float f[kS2Unroll][E];
#pragma unroll
        for (int u = 0; u < kS2Unroll; ++u) Vec16<DT>::load(x, base + (uint64_t)u * kS2Threads + tid, f[u]);
#pragma unroll
        for (int u = 0; u < kS2Unroll; ++u) {
#pragma unroll
            for (int e = 0; e < E; e += 2) {
                add(f[u][e], dev0, sq0);
                add(f[u][e + 1], dev1, sq1);
            }
        }
    }
    if (base < nvec) {
        for (uint64_t v = base + tid; v < nvec; v += kS2Threads) {
            float f[E];
            Vec16<DT>::load(x, v, f);
#pragma unroll
            for (int e = 0; e < E; e += 2) {
                add(f[e], dev0, sq0);
                add(f[e + 1], dev1, sq1);
            }
        }
    }
    if (blockIdx.x == 0 && tid < (uint32_t)(n - nvec * E)) add(Vec4<DT>::load1(x, nvec * E + tid), dev0, sq0);

    const double dev = wave_sum(dev0 + dev1);
    const double sq = wave_sum(sq0 + sq1);
    if (lane == 0) sh2[wave] = Part2{dev, sq};
    __syncthreads();   // also orders the LDS histogram updates before the merge below
    for (uint32_t b = tid; b < nbins; b += kS2Threads) {
        uint32_t c = 0u;
        for (uint32_t r = 0; r < (1u << rep_shift); ++r) c += sh_hist[(b << rep_shift) + r];
        if (c) atomicAdd(&hist[b], c);
    }
    if (tid == 0) {
        Part2 p = sh2[0];
        for (int w = 1; w < kS2Threads / kWave; ++w) {
            p.dev += sh2[w].dev;
            p.sq += sh2[w].sq;
        }
        if (out) {
            st_dev(&part2[blockIdx.x].dev, p.dev);
            st_dev(&part2[blockIdx.x].sq, p.sq);
        } else {
            part2[blockIdx.x] = p;
        }
    }
    if (!out) return;

    // ---- the last block to get here turns the partials into the record ----
    __shared__ uint32_t sh_last;
    wait_stores();     // this lane's histogram atomics and partial have arrived ...
    __syncthreads();   // ... and so have those of every lane of the block
    if (tid == 0) {
        const uint32_t prev = __hip_atomic_fetch_add(&ctl->ticket_stats, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        sh_last = (prev == gridDim.x - 1u) ? 1u : 0u;
    }
    __syncthreads();
    if (!sh_last) return;
    finalize_stats_block<true>(part1, nb1, part2, gridDim.x, hist, nbins, n, out);
    if (tid == 0) ctl->ticket_stats = 0u;
}

// Whole tiles per block: with T tiles and at most B blocks, every block takes ceil(T/B) tiles and
// the grid shrinks to the number of blocks that this needs.
void stats_grid(uint64_t n, int dtype, uint32_t &nb1, uint32_t &nb2)
{
    const uint64_t nvec = n / (dtype == QP_BF16 ? 8 : 4);   // 16-byte vectors
    auto even_grid = [](uint64_t tiles, uint32_t max_blocks) -> uint32_t {
        if (tiles < 1) return 1u;
        const uint64_t per = (tiles + max_blocks - 1) / max_blocks;
        return (uint32_t)((tiles + per - 1) / per);
    };
    nb1 = even_grid((nvec + kS1Threads * kS1Unroll - 1) / (kS1Threads * kS1Unroll), kMaxStat1Blocks);
    nb2 = even_grid((nvec + kS2Threads * kS2Unroll - 1) / (kS2Threads * kS2Unroll), kMaxStat2Blocks);
}

hipError_t launch_stats(const void *x, uint64_t n, int dtype, uint32_t nbins, void *ws, hipStream_t s, bool finalize)
{
    if (uses_value_table(n, dtype)) {   // one pass over the tensor; the record is always finalized here
        const hipError_t e = launch_value_table(x, n, ws, s);
        return e != hipSuccess ? e : launch_stats_from_table(n, nbins, ws, s);
    }
    char *w = static_cast<char *>(ws);
    Part1 *p1 = reinterpret_cast<Part1 *>(w + kOffPart1);
    Part2 *p2 = reinterpret_cast<Part2 *>(w + kOffPart2);
    uint32_t *hist = reinterpret_cast<uint32_t *>(w + kOffHist);
    Ctl *ctl = reinterpret_cast<Ctl *>(w + kOffCtl);
    qp_stats_t *out = finalize ? reinterpret_cast<qp_stats_t *>(w + kOffStats) : nullptr;
    uint32_t nb1, nb2;
    stats_grid(n, dtype, nb1, nb2);
    if (dtype == QP_F32)
        hipLaunchKernelGGL(k_stats_pass1<QP_F32>, dim3(nb1), dim3(kS1Threads), 0, s, x, n, p1, hist, nbins, ctl);
    else
        hipLaunchKernelGGL(k_stats_pass1<QP_BF16>, dim3(nb1), dim3(kS1Threads), 0, s, x, n, p1, hist, nbins, ctl);
#define QP_PASS2(DT, R) \
    hipLaunchKernelGGL((k_stats_pass2<DT, R>), dim3(nb2), dim3(kS2Threads), 0, s, x, n, p1, nb1, p2, hist, nbins, ctl, out)
    const uint32_t rs = hist_rep_shift(nbins);
    if (dtype == QP_F32) {
        if (rs == 3) QP_PASS2(QP_F32, 3); else if (rs == 2) QP_PASS2(QP_F32, 2); else QP_PASS2(QP_F32, 1);
    } else {
        if (rs == 3) QP_PASS2(QP_BF16, 3); else if (rs == 2) QP_PASS2(QP_BF16, 2); else QP_PASS2(QP_BF16, 1);
    }
#undef QP_PASS2
    return hipGetLastError();
}

}  // namespace qp
