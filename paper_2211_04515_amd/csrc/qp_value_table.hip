// The value table of a large bfloat16 tensor, and what can be read off it.
//
// A bf16 tensor has at most 65536 distinct values.  counts[p] = number of elements with bit
// pattern p is built in one streaming pass (k_value_hist_bf16), and both the per-tensor
// statistics (Sec. 3: mu, b_E, the histogram D_R and its peak) and the scores of the directed
// search (Eq. 1) are sums over elements of functions of the value alone, so they can be taken
// over the 65536 table entries, each weighted by its count, instead of over the tensor: the same
// sums with equal terms grouped.  For a tensor of 151 M elements that replaces two reads of the
// tensor for the statistics and one per search round by a single read.
#include <type_traits>

#include "qp_common.hpp"

namespace qp {

bool uses_value_table(uint64_t n, int dtype) { return dtype == QP_BF16 && n >= kValueTableMinN; }

// Also clears the search's ticket: the search over the table has no set-up launch that could.
__global__ __launch_bounds__(1024) void k_value_table_zero(uint32_t *__restrict__ counts, Ctl *__restrict__ ctl)
{
    reinterpret_cast<uint4 *>(counts)[blockIdx.x * 1024u + threadIdx.x] = make_uint4(0u, 0u, 0u, 0u);
    if (blockIdx.x == 0 && threadIdx.x == 0) ctl->ticket_search = 0u;
}

// A block counts one sign (32768 patterns, 128 KB of LDS, plain u32 counters) of one chunk of the
// tensor; blocks b and b+8 sit on the same XCD (blocks are dealt round-robin to the 8 XCDs) and
// take the two signs of the same chunk, so the second reader of a chunk hits in that XCD's L2.
constexpr int kVhThreads = 1024;
constexpr int kVhUnroll = 4;

// The streaming loop for one sign (compile-time, so that the test of an element's sign is a single
// signed compare of the dword or of its low half).  On 151 M elements the kernel takes 65 us: 9 LDS
// increments per nanosecond and compute unit, about 4.2 per clock, i.e. 15 clocks per wave64 ds_add_u32 (64
// lanes into 32 banks at random addresses conflict about 3.5-fold, and an atomic is a read and a write).
// That rate is the bound: HBM delivers the tensor once (302 MB) at 4.6 TB/s and is not the limit, and every
// arrangement puts the same number of increments on each compute unit's LDS.  Prefetching the next tile,
// counting the other sign into dummy slots instead of branching, and one block per compute unit over all
// 65536 patterns in packed 16-bit counters (each element examined once) all measured the same or worse.
template <int SIGN>
__device__ __forceinline__ void value_hist_loop(const uint16_t *__restrict__ x, uint64_t n, uint32_t chunk,
                                                uint32_t nchunks, uint32_t *sh)
{
    const uint32_t tid = threadIdx.x;
    // both halves of a dword: the high half's sign is the dword's, the low half's that of its 16-bit value
    auto count2 = [&](uint32_t w) {
        const bool hi_neg = (int32_t)w < 0, lo_neg = (int16_t)(uint16_t)w < 0;
        if (hi_neg == (SIGN != 0)) atomicAdd(&sh[(w >> 16) & 0x7fffu], 1u);
        if (lo_neg == (SIGN != 0)) atomicAdd(&sh[w & 0x7fffu], 1u);
    };
    const uint64_t nvec = n / 8;   // 16-byte vectors of 8 elements
    const uint4 *__restrict__ x16 = reinterpret_cast<const uint4 *>(x);
    const uint64_t tile = (uint64_t)kVhThreads * kVhUnroll;
    uint64_t base = (uint64_t)chunk * tile;
    const uint64_t stride = (uint64_t)nchunks * tile;
    for (; base < nvec; base += stride) {
        uint4 v[kVhUnroll];
#pragma unroll
        for (int u = 0; u < kVhUnroll; ++u) {
            const uint64_t i = base + (uint64_t)u * kVhThreads + tid;
            v[u] = (i < nvec) ? x16[i] : make_uint4(0, 0, 0, 0);
        }
#pragma unroll
        for (int u = 0; u < kVhUnroll; ++u) {
            if (base + (uint64_t)u * kVhThreads + tid < nvec) {
                count2(v[u].x);
                count2(v[u].y);
                count2(v[u].z);
                count2(v[u].w);
            }
        }
    }
    if (chunk == 0 && tid < (uint32_t)(n - nvec * 8)) {
        const uint32_t h = x[nvec * 8 + tid];
        if ((h >> 15) == (uint32_t)SIGN) atomicAdd(&sh[h & 0x7fffu], 1u);
    }
}

__global__ __launch_bounds__(kVhThreads) void k_value_hist_bf16(const uint16_t *__restrict__ x, uint64_t n,
                                                                uint32_t *__restrict__ counts)
{
    __shared__ uint32_t sh[32768];
    const uint32_t tid = threadIdx.x;
    const uint32_t sign = (blockIdx.x >> 3) & 1u;
    const uint32_t chunk = ((blockIdx.x >> 4) << 3) | (blockIdx.x & 7u);
    const uint32_t nchunks = gridDim.x / 2;
    for (uint32_t i = tid; i < 32768u; i += kVhThreads) sh[i] = 0u;
    __syncthreads();
    // (counting the other sign's elements into dummy slots to avoid the branch was measured slower:
    // the LDS atomics are a scarce resource too)
    if (sign) value_hist_loop<1>(x, n, chunk, nchunks, sh);
    else value_hist_loop<0>(x, n, chunk, nchunks, sh);
    __syncthreads();
    for (uint32_t i = tid; i < 32768u; i += kVhThreads) {
        const uint32_t c = sh[i];
        if (c) atomicAdd(&counts[(sign << 15) | i], c);
    }
}

hipError_t launch_value_table(const void *x, uint64_t n, void *ws, hipStream_t s)
{
    uint32_t *counts = reinterpret_cast<uint32_t *>(static_cast<char *>(ws) + kOffValueCounts);
    hipLaunchKernelGGL(k_value_table_zero, dim3(kNumValues16 / 4096u), dim3(1024), 0, s, counts,
                       reinterpret_cast<Ctl *>(static_cast<char *>(ws) + kOffCtl));
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    const uint64_t tile = (uint64_t)kVhThreads * kVhUnroll;               // 16-byte vectors per block step
    uint64_t chunks = ((n / 8) + tile - 1) / tile;
    chunks = (chunks + 7) / 8 * 8;                                        // whole groups of 8 (one per XCD)
    if (chunks > 128) chunks = 128;                                       // two blocks (signs) per chunk: one block per compute unit
    hipLaunchKernelGGL(k_value_hist_bf16, dim3((uint32_t)(2 * chunks)), dim3(kVhThreads), 0, s,
                       static_cast<const uint16_t *>(x), n, counts);
    return hipGetLastError();
}

// ---- statistics from the table ---------------------------------------------------------------
// One block.  Pass A over the table: sum c v, sum c |v|, min, max, count of NaN/Inf patterns;
// pass B: sum c |v - mu|, sum c (v - mu)^2 and the histogram (bin of the value, weight c), with
// exactly the per-value arithmetic of the streaming kernels (fp32 bin index, fp64 moments).
// c v is exact in fp64 (c < 2^32, v has 8 significant bits); sums are taken in a fixed order.
constexpr int kTsThreads = 1024;
__global__ __launch_bounds__(kTsThreads) void k_stats_from_table(const uint32_t *__restrict__ counts, uint64_t n,
                                                                 uint32_t nbins, uint32_t *__restrict__ hist,
                                                                 qp_stats_t *__restrict__ out)
{
    // the histogram in 8 (more than 2048 bins: 4) interleaved copies, copy = lane mod 8: neighbouring
    // lanes hold neighbouring values, which mostly fall into the same bin
    __shared__ uint32_t sh_hist[4 * kMaxBins];
    __shared__ Part1 sh1[kTsThreads / kWave];
    __shared__ Part2 sh2[kTsThreads / kWave];
    __shared__ uint32_t sh_pk[kTsThreads / kWave];
    __shared__ Part1 tot1;
    const uint32_t tid = threadIdx.x, wave = tid / kWave, lane = tid % kWave;
    constexpr uint32_t per = kNumValues16 / kTsThreads;   // 64 table entries per lane
    const uint32_t rep_shift = nbins <= kMaxBins / 2 ? 3u : 2u;
    const uint32_t copy = tid & ((1u << rep_shift) - 1u);
    for (uint32_t b = tid; b < (nbins << rep_shift); b += kTsThreads) sh_hist[b] = 0u;

    // ---- pass A ----
    // a lane's 64 entries are four consecutive ones in each of 16 strides: 16 independent 16-byte loads,
    // all in flight at once (one block reads the whole 256 KB table, so latency is what counts)
    uint32_t cnt[per];
#pragma unroll
    for (uint32_t k = 0; k < per / 4; ++k) {
        const uint4 c4 = reinterpret_cast<const uint4 *>(counts)[k * kTsThreads + tid];
        cnt[4 * k] = c4.x;
        cnt[4 * k + 1] = c4.y;
        cnt[4 * k + 2] = c4.z;
        cnt[4 * k + 3] = c4.w;
    }
    double s = 0.0, sa = 0.0;
    float mn = INFINITY, mx = -INFINITY;
    uint32_t bad = 0u;
#pragma unroll
    for (uint32_t k = 0; k < per; ++k) {
        const uint32_t p = ((k / 4) * kTsThreads + tid) * 4 + (k % 4);
        const uint32_t c = cnt[k];
        if (c) {
            const float v = __uint_as_float(p << 16);
            const double d = (double)v, w = (double)c;
            s = fma(w, d, s);
            sa = fma(w, fabs(d), sa);
            mn = fminf(mn, v);
            mx = fmaxf(mx, v);
            bad += __builtin_isfinite(v) ? 0u : c;
        }
    }
    s = wave_sum(s);
    sa = wave_sum(sa);
    mn = wave_min(mn);
    mx = wave_max(mx);
    bad = wave_sum_u32(bad);
    if (lane == 0) sh1[wave] = Part1{s, sa, mn, mx, bad, 0u};
    __syncthreads();
    if (tid == 0) {
        Part1 t = sh1[0];
        for (int k = 1; k < kTsThreads / kWave; ++k) {
            t.sum += sh1[k].sum;
            t.sum_abs += sh1[k].sum_abs;
            t.mn = fminf(t.mn, sh1[k].mn);
            t.mx = fmaxf(t.mx, sh1[k].mx);
            t.bad += sh1[k].bad;
        }
        tot1 = t;
    }
    __syncthreads();

    // ---- pass B ----
    const double mean = tot1.sum / (double)n;
    const float lo = tot1.mn;
    const float range = tot1.mx - lo;
    const float w_inv = (float)((double)(float)nbins / (double)range);
    const float top = (float)(nbins - 1u);
    double dev = 0.0, sq = 0.0;
    // a lane's four consecutive values usually share a bin: their counts are added up first
    uint32_t run_idx = 0u, run_cnt = 0u;
#pragma unroll
    for (uint32_t k = 0; k < per; ++k) {
        const uint32_t c = cnt[k];
        if (c) {
            const float v = __uint_as_float((((k / 4) * kTsThreads + tid) * 4 + (k % 4)) << 16);
            const double d = (double)v - mean, w = (double)c;
            dev = fma(w, fabs(d), dev);
            sq = fma(w * d, d, sq);
            const float tt = (v - lo) * w_inv;
            const uint32_t idx = (uint32_t)__builtin_amdgcn_fmed3f(tt, 0.0f, top);   // NaN -> 0
            if (idx != run_idx && run_cnt) {
                atomicAdd(&sh_hist[(run_idx << rep_shift) + copy], run_cnt);
                run_cnt = 0u;
            }
            run_idx = idx;
            run_cnt += c;
        }
    }
    if (run_cnt) atomicAdd(&sh_hist[(run_idx << rep_shift) + copy], run_cnt);
    dev = wave_sum(dev);
    sq = wave_sum(sq);
    if (lane == 0) sh2[wave] = Part2{dev, sq};
    __syncthreads();   // also: the histogram is complete
    uint32_t peak = 0u;
    for (uint32_t b = tid; b < nbins; b += kTsThreads) {
        uint32_t c = 0u;
        for (uint32_t r = 0; r < (1u << rep_shift); ++r) c += sh_hist[(b << rep_shift) + r];
        hist[b] = c;
        peak = max(peak, c);
    }
    peak = wave_max_u32(peak);
    if (lane == 0) sh_pk[wave] = peak;
    __syncthreads();
    if (tid == 0) {
        Part2 t2 = sh2[0];
        uint32_t pk = sh_pk[0];
        for (int k = 1; k < kTsThreads / kWave; ++k) {
            t2.dev += sh2[k].dev;
            t2.sq += sh2[k].sq;
            pk = max(pk, sh_pk[k]);
        }
        *out = stats_record(tot1, t2, pk, nbins, n);
    }
}

hipError_t launch_stats_from_table(uint64_t n, uint32_t nbins, void *ws, hipStream_t s)
{
    char *w = static_cast<char *>(ws);
    hipLaunchKernelGGL(k_stats_from_table, dim3(1), dim3(kTsThreads), 0, s,
                       reinterpret_cast<const uint32_t *>(w + kOffValueCounts), n, nbins,
                       reinterpret_cast<uint32_t *>(w + kOffHist), reinterpret_cast<qp_stats_t *>(w + kOffStats));
    return hipGetLastError();
}

// ---- the directed search over the table ------------------------------------------------------
// Eq. 1's score of a candidate is a sum over elements of a function of the value alone, so it is taken over
// the 65536 table entries, each squared error weighted by its count: the same sum with equal terms grouped.
// One block per candidate (t + 1 blocks of 1024 lanes, 64 entries per lane, all requested before anything
// else).  A block builds its own candidate's grid (the arithmetic of setup_candidates), so there is no
// set-up launch, and hands its score to the block that draws the last ticket through device-coherent
// accesses; that block takes the first minimum and writes the control record, the result and the winner's
// grid.  Sums in a fixed order: bit-reproducible.
constexpr int kTbThreads = 1024;
__global__ __launch_bounds__(kTbThreads) void k_search_table(const uint32_t *__restrict__ counts, ModelArgs m_in,
                                                             const qp_stats_t *__restrict__ stats_dev, uint64_t n_total,
                                                             Cand *__restrict__ cands, double *__restrict__ scores,
                                                             Ctl *__restrict__ ctl, qp_search_result_t *__restrict__ res,
                                                             qp_qparams_t *__restrict__ best)
{
    __shared__ double sh[kTbThreads / kWave];
    __shared__ double sh_scores[kMaxT + 1];
    __shared__ uint32_t sh_flag;
    const uint32_t tid = threadIdx.x, wave = tid / kWave, lane = tid % kWave;
    const uint32_t j = blockIdx.x, ncand = gridDim.x;
    constexpr uint32_t per = kNumValues16 / kTbThreads;   // 64 table entries per lane, four consecutive ones per load
    uint32_t cnt[per];
#pragma unroll
    for (uint32_t k = 0; k < per / 4; ++k) {
        const uint4 c4 = reinterpret_cast<const uint4 *>(counts)[k * kTbThreads + tid];
        cnt[4 * k] = c4.x;
        cnt[4 * k + 1] = c4.y;
        cnt[4 * k + 2] = c4.z;
        cnt[4 * k + 3] = c4.w;
    }
    const ModelArgs m = resolve_model(m_in);
    const GridModel g = grid_model(m, m.from_ws ? stats_dev : nullptr);
    int safe;
    const Cand p = candidate_grid(m, g, j, safe);
    if (tid == 0) cands[j] = p;
    const float Lf = (float)((1u << m.bits) - 1u);
    double acc = 0.0;
    auto run = [&](auto short_tag) {
        constexpr bool SHORT = decltype(short_tag)::value;
#pragma unroll
        for (uint32_t k = 0; k < per; ++k) {
            const uint32_t c = cnt[k];
            if (c) {   // patterns that do not occur contribute nothing (NaN/Inf patterns among them, for finite tensors)
                const float v = __uint_as_float((((k / 4) * kTbThreads + tid) * 4 + (k % 4)) << 16);
                float r;
                if constexpr (SHORT) {
                    const float xc = __builtin_amdgcn_fmed3f(v, p.lo, p.hi);
                    const float d = xc - p.lo;
                    const float t = d * p.inv_scale;
                    r = rintf(t);
                } else {
                    r = quant_level(v, p.lo, p.hi, p.inv_scale, Lf);
                }
                const float err = v - dequant_level(r, p.scale, p.lo);
                // count * err^2: count < 2^32 and err has 24 significant bits, so count * err is exact in fp64
                // and the term is rounded once, like an unweighted one
                const double de = (double)err;
                acc = fma((double)c * de, de, acc);
            }
        }
    };
    if (safe) run(std::true_type{});
    else run(std::false_type{});
    acc = wave_sum(acc);
    if (lane == 0) sh[wave] = acc;
    __syncthreads();
    if (tid == 0) {
        double tot = sh[0];
        for (int w = 1; w < kTbThreads / kWave; ++w) tot += sh[w];
        st_dev(&scores[j], tot);
        wait_stores();   // the score has arrived before the ticket is drawn
        const uint32_t prev = __hip_atomic_fetch_add(&ctl->ticket_search, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        sh_flag = (prev == ncand - 1u) ? 1u : 0u;
    }
    __syncthreads();
    if (!sh_flag) return;
    // the last block: every score has arrived; read them coherently
    for (uint32_t i = tid; i < ncand; i += kTbThreads) sh_scores[i] = ld_dev(&scores[i]);
    __syncthreads();
    if (wave != 0) return;
    const uint32_t bi = first_min_wave(sh_scores, ncand, lane);
    if (lane == 0) {
        write_ctl(ctl, m, g, 1, 0u, n_total);
        write_search_result(ctl, sh_scores, ncand, bi, n_total, scores, res, best);
    }
}

hipError_t launch_table_search(uint64_t n, const SearchPlan &plan, const qp_stats_t *st, void *ws, hipStream_t s)
{
    char *w = static_cast<char *>(ws);
    const uint32_t ncand = plan.t_steps + 1u;
    hipLaunchKernelGGL(k_search_table, dim3(ncand), dim3(kTbThreads), 0, s,
                       reinterpret_cast<const uint32_t *>(w + kOffValueCounts), model_args(plan, st, kListFull, ncand, ws),
                       reinterpret_cast<const qp_stats_t *>(w + kOffStats), n, reinterpret_cast<Cand *>(w + kOffCands),
                       reinterpret_cast<double *>(w + kOffScores), reinterpret_cast<Ctl *>(w + kOffCtl),
                       reinterpret_cast<qp_search_result_t *>(w + kOffResult),
                       reinterpret_cast<qp_qparams_t *>(w + kOffQParams));
    return hipGetLastError();
}

}  // namespace qp
