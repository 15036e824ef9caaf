// Step 2b: DS-ACIQ directed search (Sec. 3, Eq. 1): the streaming kernel for large tensors (above
// 2^21 elements; smaller ones, and every coarse-to-fine sweep, take the tile search in
// qp_search_tile.hip; large bf16 tensors are searched through their value table, qp_value_table.hip).
//
// t+1 candidate scales b_j = b_E + j (b_R - b_E)/t walk from the ACIQ estimate towards the
// bound given by the real histogram's peak.  Each candidate is scored by the squared
// quantization error it causes on the real tensor.  This is plain vector-ALU work (eight
// lane operations per element and candidate, no contraction), so the kernel is organised
// around registers, not bandwidth:
//   - the candidates are cut into rounds of exactly 13 or 12 (101 = 5 x 13 + 3 x 12; other round sizes
//     for other lists); blockIdx.y selects the round, so the whole search is one launch and the
//     tensor is read once per round (mostly from L2 / Infinity Cache after the first);
//   - a lane keeps 8 elements in VGPRs and runs the round's candidates over them; a candidate's
//     grid is read from LDS once: lo lives in a VGPR, hi, scale and 1/scale in SGPRs, the running
//     sums are fp64 accumulators in VGPRs: the inner loop touches no memory and holds no
//     per-candidate test; the register budget is held to five waves per SIMD (the sequence is a
//     dependent chain per element and its issue rate depends on how many waves interleave: three
//     waves cost a fifth more cycles, four to seven measure the same);
//   - the grid is sized to the number of blocks the device keeps resident (one wave of
//     blocks, no tail);
//   - per-block partial sums go to the workspace, candidate-major; the last block of a round
//     (integer ticket) adds that round's partials, one wave per candidate, and the last round
//     to finish takes the first minimum and writes the result record and the winner's grid.
//     No floating-point atomics: bit-reproducible.
// The per-element arithmetic is that of quantize+pack and unpack+dequantize, so a candidate's
// score is exactly the error of the tensor that would come out of the receiver.
#include <atomic>

#include "qp_common.hpp"

namespace qp {

constexpr int kSrThreads = 256;
constexpr int kSrElems = 8;   // elements per lane per batch (two 4-element vectors)

// One block: fills the candidate table and the control record for one sweep (setup_candidates).
// When the statistics passes have only left their partials (the fused sender path), this block
// first turns them into the qp_stats_t record, which saves a launch.  Before the fine sweep of a
// coarse-to-fine search it reads the coarse winner from the result record (prev).
__global__ __launch_bounds__(kFinThreads) void k_search_setup(ModelArgs m, qp_stats_t *__restrict__ stats_dev, uint64_t n,
                                                              Cand *__restrict__ cands, Ctl *__restrict__ ctl,
                                                              uint32_t *__restrict__ round_tickets, FinalizeArgs fin,
                                                              const qp_search_result_t *__restrict__ prev,
                                                              double *__restrict__ scores_by_j)
{
    for (uint32_t j = threadIdx.x; j <= kMaxT; j += blockDim.x) round_tickets[j] = 0u;
    if (fin.nbins) finalize_stats_block(fin.part1, fin.nb1, fin.part2, fin.nb2, fin.hist, fin.nbins, n, stats_dev);
    m = resolve_model(m);
    const uint32_t j1 = (m.list_mode == kListFine) ? prev->j_star : 0u;
    setup_candidates(m, m.from_ws ? stats_dev : nullptr, j1, n, cands, nullptr, ctl, scores_by_j);
}

// No search: the result is plain ACIQ, candidate j = 0 (the paper's deployment switches the directed search
// off above 4 bit).  One block; finalizes the statistics first when the sender path left partials.
__global__ __launch_bounds__(kFinThreads) void k_aciq_only(ModelArgs m, qp_stats_t *__restrict__ stats_dev, uint64_t n,
                                                           Cand *__restrict__ cands, Ctl *__restrict__ ctl, FinalizeArgs fin,
                                                           double *__restrict__ scores_by_j,
                                                           qp_search_result_t *__restrict__ res,
                                                           qp_qparams_t *__restrict__ best)
{
    if (fin.nbins) finalize_stats_block(fin.part1, fin.nb1, fin.part2, fin.nb2, fin.hist, fin.nbins, n, stats_dev);
    m = resolve_model(m);
    m.list_mode = kListFull;
    m.count = 1u;
    setup_candidates(m, m.from_ws ? stats_dev : nullptr, 0u, n, cands, nullptr, ctl, nullptr);
    const double nan = __longlong_as_double(0x7ff8000000000000ll);
    for (uint32_t j = threadIdx.x; j <= m.t_steps; j += blockDim.x) scores_by_j[j] = nan;
    __syncthreads();   // the control record written by lane 0 above
    if (threadIdx.x == 0) {
        qp_search_result_t r;
        r.b_e = ctl->b_e;
        r.b_r = ctl->b_r;
        r.b_star = ctl->b_e;
        r.alpha_star = ctl->F * ctl->b_e;
        r.mse_aciq = nan;
        r.mse_star = nan;
        r.j_star = 0u;
        r.t_steps = m.t_steps;
        *res = r;
        qp_qparams_t q;
        q.bits = m.bits;
        q.reserved = 0u;
        q.n = n;
        make_grid(ctl->mean, r.alpha_star, m.bits, q.lo, q.hi, q.scale, q.inv_scale, ctl->clip != 0u, ctl->clip_lo, ctl->clip_hi);
        *best = q;
    }
}

// The scoring pass of one block: lanes stride over batches of kSrElems elements; for each
// batch the round's candidates (at most 16, wave-uniform) are applied to the elements held in
// registers.  SHORT selects the sequence without the second clamp (see setup_candidates).
template <int DT, int NC, bool SHORT, int CMAX>
__device__ __forceinline__ void score_pass(const void *__restrict__ x, uint64_t n, const Cand *sh_cands, float Lf,
                                           double (&acc)[CMAX])
{
    const uint32_t tid = threadIdx.x;
    // The round's grids, read once (LDS broadcast reads).  hi, scale and 1/scale go to scalar registers
    // (every lane holds the same values); lo stays in a vector register because an instruction takes one
    // scalar operand at most.  That leaves the vector registers to the running sums and the elements, so
    // that more waves fit a SIMD.
    Cand grid[NC];
#pragma unroll
    for (int c = 0; c < NC; ++c) {
        const Cand p = sh_cands[c];
        grid[c].lo = p.lo;
        grid[c].hi = wave_uniform(p.hi);
        grid[c].scale = wave_uniform(p.scale);
        grid[c].inv_scale = wave_uniform(p.inv_scale);
    }
    auto score = [&](const float (&v)[kSrElems], int ne) {
#pragma unroll
        for (int c = 0; c < NC; ++c) {
            const Cand p = grid[c];
#pragma unroll
            for (int e = 0; e < kSrElems; ++e) {
                if (e < ne) {
                    float r;
                    if constexpr (SHORT) {
                        // med3(x, lo, hi) == min(max(x, lo), hi) for lo <= hi, NaN -> lo as well
                        const float xc = __builtin_amdgcn_fmed3f(v[e], p.lo, p.hi);
                        const float d = xc - p.lo;
                        const float t = d * p.inv_scale;
                        r = rintf(t);
                    } else {
                        r = quant_level(v[e], p.lo, p.hi, p.inv_scale, Lf);
                    }
                    const float err = v[e] - dequant_level(r, p.scale, p.lo);
                    const double de = (double)err;
                    acc[c] = fma(de, de, acc[c]);   // de*de is exact in fp64
                }
            }
        }
    };

    const uint64_t nbatch = n / kSrElems;
    const uint64_t bstride = (uint64_t)gridDim.x * kSrThreads;
    for (uint64_t b = (uint64_t)blockIdx.x * kSrThreads + tid; b < nbatch; b += bstride) {
        float v[kSrElems];
#pragma unroll
        for (int q = 0; q < kSrElems / 4; ++q) {
            float f[4];
            Vec4<DT>::load(x, (kSrElems / 4) * b + q, f);
#pragma unroll
            for (int e = 0; e < 4; ++e) v[4 * q + e] = f[e];
        }
        score(v, kSrElems);
    }
    // ragged tail: fewer than kSrElems elements, taken by one lane of block column 0
    const uint32_t rem = (uint32_t)(n - nbatch * kSrElems);
    if (rem && blockIdx.x == 0 && tid == 0) {
        float v[kSrElems];
#pragma unroll
        for (int e = 0; e < kSrElems; ++e) v[e] = ((uint32_t)e < rem) ? Vec4<DT>::load1(x, nbatch * kSrElems + e) : 0.0f;
        score(v, (int)rem);
    }
}

// CMAX: the candidates of a round (sizes the register file: 2*CMAX running-sum, CMAX + 8 other vector
// registers and 3*CMAX scalar registers per wave).  The loop has no per-candidate tests (they would cost a
// second register pair per running sum, and with it two of the waves that fit a SIMD), so a round scores
// either exactly CMAX candidates (the first `full` rounds) or exactly CMAX - 1 (the others): 101 candidates
// are 5 rounds of 13 and 3 of 12.  Where a list does not split that way every round takes CMAX and the slots
// past the end of the list repeat the last candidate and are not stored.
// Waves per SIMD that the register allocation is held to.  The search alone takes the same time with four to
// seven (it is bound by instruction issue); with five, work that other streams launch beside it (the HBM-bound
// steps of other tensors) gets through 2 % sooner than with seven.
template <int DT, int CMAX> constexpr int search_waves()
{
    return 5;
}

template <int DT, int CMAX>
__global__ __launch_bounds__(kSrThreads, (search_waves<DT, CMAX>())) void k_search_mse(const void *__restrict__ x, uint64_t n,
                                                           const Cand *__restrict__ cands, uint32_t ncand, uint32_t full,
                                                           float Lf, double *__restrict__ partials,
                                                           double *__restrict__ scores, Ctl *__restrict__ ctl,
                                                           uint32_t *__restrict__ round_tickets,
                                                           qp_search_result_t *__restrict__ res,
                                                           qp_qparams_t *__restrict__ best,
                                                           double *__restrict__ scores_by_j)
{
    const uint32_t tid = threadIdx.x;
    const bool is_full = blockIdx.y < full;
    const uint32_t slots = is_full ? (uint32_t)CMAX : (uint32_t)CMAX - 1u;
    const uint32_t c0 = is_full ? blockIdx.y * (uint32_t)CMAX : full * (uint32_t)CMAX + (blockIdx.y - full) * ((uint32_t)CMAX - 1u);
    const uint32_t nc = min(slots, ncand - c0);   // slots of this round that are candidates of the list

    double acc[CMAX];
#pragma unroll
    for (int c = 0; c < CMAX; ++c) acc[c] = 0.0;

    // the round's candidate grids: one coalesced load into LDS, read back per candidate as a broadcast
    __shared__ Cand sh_cands[CMAX];
    if (tid < (uint32_t)CMAX) sh_cands[tid] = cands[min(c0 + tid, ncand - 1u)];
    const uint32_t short_seq = ctl->short_seq;
    __syncthreads();

    if (is_full) {
        if (short_seq) score_pass<DT, CMAX, true>(x, n, sh_cands, Lf, acc);
        else score_pass<DT, CMAX, false>(x, n, sh_cands, Lf, acc);
    } else if constexpr (CMAX > 1) {
        if (short_seq) score_pass<DT, CMAX - 1, true>(x, n, sh_cands, Lf, acc);
        else score_pass<DT, CMAX - 1, false>(x, n, sh_cands, Lf, acc);
    }

    // ---- block reduction: DPP inside each wave64, one LDS row per wave ----
    __shared__ double sh[kSrThreads / kWave][CMAX];
    __shared__ uint32_t sh_flag;
    const uint32_t wave = tid / kWave, lane = tid % kWave;
    const uint32_t gx = gridDim.x;
#pragma unroll
    for (int c = 0; c < CMAX; ++c) {
        const double s = wave_sum(acc[c]);
        if (lane == 0) sh[wave][c] = s;
    }
    __syncthreads();
    if (tid < nc) {
        double s = sh[0][tid];
        for (int w = 1; w < kSrThreads / kWave; ++w) s += sh[w][tid];
        // candidate-major: a candidate's partials are contiguous.  Device-coherent store, waited for before
        // the ticket below: other blocks read it without any cache write-back or invalidation.
        st_dev(&partials[(uint64_t)(c0 + tid) * gx + blockIdx.x], s);
        wait_stores();
    }

    // ---- first ticket: the last block of this round adds the round's partials ----
    __syncthreads();
    if (tid == 0) {
        const uint32_t prev = __hip_atomic_fetch_add(&round_tickets[blockIdx.y], 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        sh_flag = (prev == gx - 1u) ? 1u : 0u;
    }
    __syncthreads();
    if (!sh_flag) return;

    // One wave per candidate (a wave takes candidates wave, wave + 4, ...): lanes stride over the blocks'
    // partials (coalesced), each lane adds its own in ascending order, then the wave's lanes are added.
    // A coherent load is a round trip to the point of coherence, so a candidate's loads are issued four at
    // a time before the first is used (one group when the grid has at most 256 columns, the usual case), and
    // the scores are waited for once.
    constexpr uint32_t kWaves = kSrThreads / kWave;
    for (uint32_t c = wave; c < nc; c += kWaves) {
        const double *col = partials + (uint64_t)(c0 + c) * gx;
        double s = 0.0;
        for (uint32_t b0 = lane; b0 < gx; b0 += 4u * kWave) {
            double v[4];
#pragma unroll
            for (uint32_t k = 0; k < 4; ++k) v[k] = (b0 + kWave * k < gx) ? ld_dev(&col[b0 + kWave * k]) : 0.0;
#pragma unroll
            for (uint32_t k = 0; k < 4; ++k)
                if (b0 + kWave * k < gx) s += v[k];
        }
        s = wave_sum(s);
        if (lane == 0) st_dev(&scores[c0 + c], s);
    }
    if (lane == 0) wait_stores();

    // ---- second ticket: the last round to finish picks the winner ----
    __syncthreads();
    if (tid == 0) {
        round_tickets[blockIdx.y] = 0u;
        const uint32_t prev = __hip_atomic_fetch_add(&ctl->ticket_search, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        sh_flag = (prev == gridDim.y - 1u) ? 1u : 0u;
    }
    __syncthreads();
    if (!sh_flag) return;
    __shared__ double sh_scores[kMaxT + 1];
    for (uint32_t j = tid; j < ncand; j += kSrThreads) sh_scores[j] = ld_dev(&scores[j]);
    __syncthreads();
    if (wave != 0) return;
    const uint32_t bi = first_min_wave(sh_scores, ncand, lane);
    if (lane == 0) write_search_result(ctl, sh_scores, ncand, bi, n, scores_by_j, res, best);
}

// ---- which model fits: Laplace or Gaussian ---------------------------------------------------
// One block over the histogram: the squared distance between the histogram density and each model's pdf at its
// moment estimates (b_E = MAD, sigma = sqrt(var)), fp64, fixed order.  Gaussian only if strictly closer; NaN
// (one distinct value, a record the statistics never wrote) keeps the paper's Laplace model.
constexpr int kMfThreads = 512;
__global__ __launch_bounds__(kMfThreads) void k_model_fit(const qp_stats_t *__restrict__ st, const uint32_t *__restrict__ hist,
                                                          qp_model_fit_t *__restrict__ out)
{
    __shared__ double sh_l[kMfThreads / kWave], sh_g[kMfThreads / kWave];
    const uint32_t tid = threadIdx.x, wave = tid / kWave, lane = tid % kWave;
    const uint32_t nb_rec = st->nbins;
    const uint64_t n = st->n;
    const bool rec_ok = nb_rec >= 16u && nb_rec <= kMaxBins && n != 0u;
    const uint32_t B = rec_ok ? nb_rec : 0u;
    const double mean = st->mean, mn = st->min, mx = st->max;
    const double b = st->mad, sg = sqrt(st->var);
    const double binw = (mx - mn) / (double)B;
    const double g_norm = sg * 2.5066282746310002 /* sqrt(2 pi) */, g_den = 2.0 * sg * sg;
    double fl = 0.0, fg = 0.0;
    for (uint32_t i = tid; i < B; i += kMfThreads) {
        const double c = mn + ((double)i + 0.5) * binw;
        const double d_r = (double)hist[i] / ((double)n * binw);
        const double z = c - mean;
        const double d_l = exp(-fabs(z) / b) / (2.0 * b);
        const double d_g = exp(-(z * z) / g_den) / g_norm;
        fl = fma(d_r - d_l, d_r - d_l, fl);
        fg = fma(d_r - d_g, d_r - d_g, fg);
    }
    fl = wave_sum(fl);
    fg = wave_sum(fg);
    if (lane == 0) {
        sh_l[wave] = fl;
        sh_g[wave] = fg;
    }
    __syncthreads();
    if (tid == 0) {
        double tl = sh_l[0], tg = sh_g[0];
        for (int w = 1; w < kMfThreads / kWave; ++w) {
            tl += sh_l[w];
            tg += sh_g[w];
        }
        if (!rec_ok) tl = tg = __longlong_as_double(0x7ff8000000000000ll);
        qp_model_fit_t r;
        r.fit_laplace = tl;
        r.fit_gauss = tg;
        r.dist = (tg < tl) ? (uint32_t)QP_GAUSS : (uint32_t)QP_LAPLACE;   // false whenever either is NaN
        r.reserved = 0u;
        *out = r;
    }
}

hipError_t launch_model_fit(void *ws, hipStream_t s)
{
    char *w = static_cast<char *>(ws);
    hipLaunchKernelGGL(k_model_fit, dim3(1), dim3(kMfThreads), 0, s, reinterpret_cast<const qp_stats_t *>(w + kOffStats),
                       reinterpret_cast<const uint32_t *>(w + kOffHist), reinterpret_cast<qp_model_fit_t *>(w + kOffModel));
    return hipGetLastError();
}

// ---- the other reading of Eq. 1: fit the Laplace pdf to the histogram -----------------
// One block per candidate: lanes stride over the bins, score_j = sum_i (D_R,i - pdf(c_i; mu, b_j))^2
// in fp64 (D_R,i = count_i / (N binwidth), c_i the bin centre).  The block that draws the last
// ticket takes the first minimum, as in the tensor-error search.  Reads the statistics record
// and the histogram that the statistics step left in the workspace; no pass over the tensor.
constexpr int kHsThreads = 256;
__global__ __launch_bounds__(kHsThreads) void k_hist_search(const qp_stats_t *__restrict__ st,
                                                            const uint32_t *__restrict__ hist, uint32_t bits,
                                                            uint32_t t_steps, double F, double *__restrict__ scores,
                                                            Ctl *__restrict__ ctl, qp_search_result_t *__restrict__ res,
                                                            qp_qparams_t *__restrict__ best)
{
    __shared__ double sh[kHsThreads / kWave];
    __shared__ uint32_t sh_flag;
    const uint32_t tid = threadIdx.x, wave = tid / kWave, lane = tid % kWave;
    const uint32_t j = blockIdx.x, ncand = t_steps + 1u;
    // The record is whatever the workspace holds: a bin count outside the histogram region, or no elements,
    // means the statistics never ran on it.  Then nothing is read (B = 0) and every score is NaN.
    const uint32_t nb_rec = st->nbins;
    const uint64_t n = st->n;
    const bool rec_ok = nb_rec >= 16u && nb_rec <= kMaxBins && n != 0u;
    const uint32_t B = rec_ok ? nb_rec : 0u;
    const double mean = st->mean, mn = st->min, mx = st->max;
    const double b_e = st->mad, b_r = st->b_r;
    double step = (b_r - b_e) / (double)t_steps;
    const bool ok = (b_e > 0.0) && (b_r > 0.0) && isfinite(b_r) && isfinite(b_e) && isfinite(step);
    if (!ok) step = 0.0;
    const double b_j = b_e + (double)j * step;
    const double binw = (mx - mn) / (double)B;
    double s = 0.0;
    for (uint32_t i = tid; i < B; i += kHsThreads) {
        const double c = mn + ((double)i + 0.5) * binw;
        const double d_r = (double)hist[i] / ((double)n * binw);
        const double d_e = exp(-fabs(c - mean) / b_j) / (2.0 * b_j);
        const double diff = d_r - d_e;
        s = fma(diff, diff, s);
    }
    s = wave_sum(s);
    if (lane == 0) sh[wave] = s;
    __syncthreads();
    if (tid == 0) {
        double tot = sh[0];
        for (int w = 1; w < kHsThreads / kWave; ++w) tot += sh[w];
        if (!rec_ok) tot = __longlong_as_double(0x7ff8000000000000ll);
        st_dev(&scores[j], tot);
        wait_stores();   // the score has arrived before the ticket is drawn
        const uint32_t prev = __hip_atomic_fetch_add(&ctl->ticket_search, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        sh_flag = (prev == gridDim.x - 1u) ? 1u : 0u;
    }
    __syncthreads();
    if (!sh_flag) return;
    // the last block: every score has arrived; read them coherently
    __shared__ double sh_scores[kMaxT + 1];
    for (uint32_t i = tid; i < ncand; i += kHsThreads) sh_scores[i] = ld_dev(&scores[i]);
    __syncthreads();
    if (wave != 0) return;

    uint32_t bj = first_min_wave(sh_scores, ncand, lane);
    if (lane == 0) {
        const double s0 = sh_scores[0];
        if (!(s0 == s0)) bj = 0u;   // a NaN incumbent is never beaten
        qp_search_result_t r;
        r.b_e = b_e;
        r.b_r = b_r;
        r.b_star = b_e + (double)bj * step;
        r.alpha_star = F * r.b_star;
        r.mse_aciq = s0 / (double)B;
        r.mse_star = sh_scores[bj] / (double)B;
        r.j_star = bj;
        r.t_steps = t_steps;
        *res = r;
        qp_qparams_t q;
        q.bits = bits;
        q.reserved = 0u;
        q.n = n;
        make_grid(mean, r.alpha_star, bits, q.lo, q.hi, q.scale, q.inv_scale);
        *best = q;
        ctl->ticket_search = 0u;
    }
}

hipError_t launch_hist_search(uint32_t bits, uint32_t t_steps, double F, void *ws, hipStream_t s)
{
    char *w = static_cast<char *>(ws);
    hipLaunchKernelGGL(k_hist_search, dim3(t_steps + 1u), dim3(kHsThreads), 0, s,
                       reinterpret_cast<const qp_stats_t *>(w + kOffStats),
                       reinterpret_cast<const uint32_t *>(w + kOffHist), bits, t_steps, F,
                       reinterpret_cast<double *>(w + kOffScores), reinterpret_cast<Ctl *>(w + kOffCtl),
                       reinterpret_cast<qp_search_result_t *>(w + kOffResult),
                       reinterpret_cast<qp_qparams_t *>(w + kOffQParams));
    return hipGetLastError();
}

// Upper bound on the number of block columns (sizes the partial-sum region of the workspace).
uint32_t search_blocks(uint64_t n)
{
    const uint64_t nbatch = n / kSrElems;
    uint32_t nb = ceil_div_u64(nbatch, kSrThreads);
    if (nb < 1) nb = 1;
    if (nb > kMaxSearchBlocks) nb = kMaxSearchBlocks;
    return nb;
}

// Blocks of the search kernel that the device keeps resident at once (all CUs, at the kernel's
// own occupancy); the grid is sized to this so that there is one wave of blocks and no tail.
template <int DT, int CMAX> static uint32_t resident_blocks()
{
    static std::atomic<uint32_t> cached[16];   // zero-initialised; a race only repeats the same query
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 16) dev = 0;
    uint32_t v = cached[dev].load(std::memory_order_relaxed);
    if (v == 0) {
        int per_cu = 0, cus = 0;
        if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, k_search_mse<DT, CMAX>, kSrThreads, 0) != hipSuccess ||
            per_cu < 1)
            per_cu = 2;
        if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus < 1) cus = 256;
        v = (uint32_t)per_cu * (uint32_t)cus;
        cached[dev].store(v, std::memory_order_relaxed);
    }
    return v;
}

struct SearchArgs {
    const void *x;
    uint64_t n;
    const Cand *cands;
    uint32_t ncand;
    float Lf;
    double *partials, *scores;
    Ctl *ctl;
    uint32_t *round_tickets;
    qp_search_result_t *res;
    qp_qparams_t *best;
    double *scores_by_j;   // where a coarse-to-fine sweep scatters its scores
};

// One kernel variant: the grid is one wave of resident blocks, split over the rounds.
template <int DT, int CMAX> static hipError_t launch_variant(const SearchArgs &a, hipStream_t s)
{
    const uint32_t resident = resident_blocks<DT, CMAX>();
    const uint32_t cols = search_blocks(a.n);
    const uint32_t rounds = (a.ncand + (uint32_t)CMAX - 1u) / (uint32_t)CMAX;
    // `full` rounds of CMAX candidates and rounds - full of CMAX - 1, if the list splits that way
    // (ncand = full CMAX + (rounds - full)(CMAX - 1)); else every round takes CMAX and the last one is padded
    uint32_t full = rounds;
    if (CMAX > 1 && a.ncand >= rounds * ((uint32_t)CMAX - 1u)) full = a.ncand - rounds * ((uint32_t)CMAX - 1u);
    // a list that fits one round is the tile search's job (launch_search sends it there); this kernel has
    // only ever run with two rounds or more
#ifndef QP_EMULATE_STREAMING_C2F
    if (rounds < 2u) return hipErrorInvalidValue;
#endif
    uint32_t gx = resident / rounds;
    if (gx > cols) gx = cols;
    if (gx < 1) gx = 1;
    hipLaunchKernelGGL((k_search_mse<DT, CMAX>), dim3(gx, rounds), dim3(kSrThreads), 0, s, a.x, a.n, a.cands, a.ncand, full,
                       a.Lf, a.partials, a.scores, a.ctl, a.round_tickets, a.res, a.best, a.scores_by_j);
    return hipGetLastError();
}

// The kernel exists for these round sizes (more candidates per round leave too few waves on a SIMD).  The
// caller's cands_per_round is an upper bound.  Among the sizes within it: one that gives the device at least
// two blocks per compute unit (a short tensor, such as a value table, needs many short rounds for that), then
// the fewest candidate slots (101 candidates: 13 -> 101 slots, 16 -> 112), then the largest.  The grouping
// never changes a candidate's score beyond the order of its fp64 partial sums.
constexpr uint32_t kRoundSizes[] = {16u, 13u, 8u, 4u, 2u, 1u};
#ifndef QP_SEARCH_FILL_BLOCKS
#define QP_SEARCH_FILL_BLOCKS 512   // two blocks per compute unit
#endif

static uint32_t round_slots(uint32_t ncand, uint32_t size)
{
    const uint32_t rounds = (ncand + size - 1u) / size;
    return (size > 1u && ncand >= rounds * (size - 1u)) ? ncand : rounds * size;
}

template <int DT> static hipError_t launch_rounds(const SearchArgs &a, uint32_t cpr_limit, hipStream_t s)
{
    const uint32_t cols = search_blocks(a.n);
    uint32_t pick = 1u, pick_slots = 0u;
    bool pick_fills = false;
    for (uint32_t size : kRoundSizes) {   // descending
        if (size > cpr_limit) continue;
        const uint32_t rounds = (a.ncand + size - 1u) / size;
        const bool fills = (uint64_t)cols * rounds >= (uint64_t)QP_SEARCH_FILL_BLOCKS;
        const uint32_t slots = round_slots(a.ncand, size);
        const bool better = pick_slots == 0u || (fills && !pick_fills) || (fills == pick_fills && fills && slots < pick_slots) ||
                            (!fills && !pick_fills);   // nothing fills the device: the most rounds
        if (better) {
            pick = size;
            pick_slots = slots;
            pick_fills = fills;
        }
    }
    switch (pick) {
    case 16u: return launch_variant<DT, 16>(a, s);
    case 13u: return launch_variant<DT, 13>(a, s);
    case 8u: return launch_variant<DT, 8>(a, s);
    case 4u: return launch_variant<DT, 4>(a, s);
    case 2u: return launch_variant<DT, 2>(a, s);
    default: return launch_variant<DT, 1>(a, s);
    }
}

ModelArgs model_args(const SearchPlan &plan, const qp_stats_t *st, uint32_t list_mode, uint32_t count, const void *ws)
{
    ModelArgs m{};
    // the model chosen on the device: the grid is built there too, from the record the choice was made on
    if (plan.dist == QP_DIST_AUTO) st = nullptr;
    m.C_alt = plan.C_alt;
    m.model = reinterpret_cast<const qp_model_fit_t *>(static_cast<const char *>(ws) + kOffModel);
    m.from_ws = st ? 0 : 1;
    if (st) {
        m.mean_h = st->mean;
        scale_ends(*st, plan.dist, m.s_e_h, m.s_r_h);
        m.clip_lo_h = (float)st->min;
        m.clip_hi_h = (float)st->max;
    }
    m.dist = plan.dist;
    m.clip = plan.clip;
    m.list_mode = list_mode;
    m.list_stride = plan.stride;
    m.count = count;
    m.bits = plan.bits;
    m.t_steps = plan.t_steps;
    m.C = plan.C;
    return m;
}

// One sweep of the streaming search: set-up kernel, then the search kernel.
static hipError_t launch_sweep(const void *x, uint64_t n, int dtype, const SearchPlan &plan, const qp_stats_t *st,
                               uint32_t finalize_nbins, uint32_t list_mode, uint32_t count, void *ws, hipStream_t s)
{
    // Only the full sweep: this kernel has never completed a run with a coarse or fine candidate list on the GPU
    // (its one attempt ended in a fault whose cause was not found), so such a list is an error here whatever
    // the caller above does; those sweeps run on the tile search.
    // (QP_EMULATE_STREAMING_C2F is defined by one build of the CPU emulation under tests/ only, which runs that
    // very sequence on the host in search of the cause; no build of the library defines it.)
#ifndef QP_EMULATE_STREAMING_C2F
    if (list_mode != kListFull) return hipErrorInvalidValue;
#endif
    char *w = static_cast<char *>(ws);
    Cand *cands = reinterpret_cast<Cand *>(w + kOffCands);
    Ctl *ctl = reinterpret_cast<Ctl *>(w + kOffCtl);
    qp_stats_t *stats_dev = reinterpret_cast<qp_stats_t *>(w + kOffStats);
    uint32_t *round_tickets = reinterpret_cast<uint32_t *>(w + kOffRoundTickets);
    double *scores_by_j = reinterpret_cast<double *>(w + kOffScores);
    double *scores_list = list_mode == kListFull ? scores_by_j : reinterpret_cast<double *>(w + kOffListScores);
    qp_search_result_t *res = reinterpret_cast<qp_search_result_t *>(w + kOffResult);

    FinalizeArgs fin{reinterpret_cast<const Part1 *>(w + kOffPart1), reinterpret_cast<const Part2 *>(w + kOffPart2),
                     reinterpret_cast<const uint32_t *>(w + kOffHist), 0u, 0u, finalize_nbins};
    if (finalize_nbins) stats_grid(n, dtype, fin.nb1, fin.nb2);
    const ModelArgs m = model_args(plan, st, list_mode, count, ws);
    hipLaunchKernelGGL(k_search_setup, dim3(1), dim3(kFinThreads), 0, s, m, stats_dev, n, cands, ctl, round_tickets, fin,
                       res, scores_by_j);
    const hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;

    const SearchArgs a{x, n, cands, count, (float)((1u << plan.bits) - 1u),
                       reinterpret_cast<double *>(w + kOffSearchPart), scores_list, ctl, round_tickets, res,
                       reinterpret_cast<qp_qparams_t *>(w + kOffQParams), scores_by_j};
    return dtype == QP_F32 ? launch_rounds<QP_F32>(a, plan.cpr, s) : launch_rounds<QP_BF16>(a, plan.cpr, s);
}

hipError_t launch_search(const void *x, uint64_t n, int dtype, const SearchPlan &plan, const qp_stats_t *st,
                         uint32_t finalize_nbins, bool value_table_ready, void *ws, hipStream_t s)
{
    if (plan.aciq_only) {
        char *w = static_cast<char *>(ws);
        FinalizeArgs fin{reinterpret_cast<const Part1 *>(w + kOffPart1), reinterpret_cast<const Part2 *>(w + kOffPart2),
                         reinterpret_cast<const uint32_t *>(w + kOffHist), 0u, 0u, finalize_nbins};
        if (finalize_nbins) stats_grid(n, dtype, fin.nb1, fin.nb2);
        hipLaunchKernelGGL(k_aciq_only, dim3(1), dim3(kFinThreads), 0, s, model_args(plan, st, kListFull, 1u, ws),
                           reinterpret_cast<qp_stats_t *>(w + kOffStats), n, reinterpret_cast<Cand *>(w + kOffCands),
                           reinterpret_cast<Ctl *>(w + kOffCtl), fin, reinterpret_cast<double *>(w + kOffScores),
                           reinterpret_cast<qp_search_result_t *>(w + kOffResult),
                           reinterpret_cast<qp_qparams_t *>(w + kOffQParams));
        return hipGetLastError();
    }
    // A bf16 tensor has at most 65536 distinct values: above a modest size it is cheaper to count them once
    // (one pass over the tensor) and run the candidates over the value table.
    if (uses_value_table(n, dtype)) {
        if (plan.stride > 1u || finalize_nbins) return hipErrorInvalidValue;   // refused / the table path finalizes itself
        if (!value_table_ready) {
            const hipError_t e = launch_value_table(x, n, ws, s);
            if (e != hipSuccess) return e;
        }
        return launch_table_search(n, plan, st, ws, s);
    }
    // other small and medium tensors: one candidate per lane over LDS tiles
    if (tile_search_eligible(n, plan)) return launch_tile_search(x, n, dtype, plan, st, finalize_nbins, ws, s);
    // A coarse-to-fine sweep always runs on the tile search, whatever the size (its short candidate lists
    // suit the one-candidate-per-lane layout; on this file's streaming kernel the sweep faulted the GPU once,
    // cause not found, so it is not launched from here).
    if (plan.stride > 1u) {
        if (!coarse_to_fine_supported(n, dtype, plan)) return hipErrorInvalidValue;
#ifdef QP_EMULATE_STREAMING_C2F
        {   // CPU emulation only: the two sweeps on the streaming kernel, as the run that faulted launched them
            const uint32_t coarse = (plan.t_steps + plan.stride - 1u) / plan.stride + 1u;
            const hipError_t e = launch_sweep(x, n, dtype, plan, st, finalize_nbins, kListCoarse, coarse, ws, s);
            if (e != hipSuccess) return e;
            return launch_sweep(x, n, dtype, plan, st, 0u, kListFine, 2u * plan.stride - 1u, ws, s);
        }
#endif
        return launch_tile_search(x, n, dtype, plan, st, finalize_nbins, ws, s);
    }
    // So does a full sweep short enough for one round (t + 1 <= cands_per_round): the streaming kernel's
    // strength is many candidates held in registers, and its one-round grid is the one that faulted.
    if (plan.t_steps + 1u <= plan.cpr && tile_search_can_run(plan))
        return launch_tile_search(x, n, dtype, plan, st, finalize_nbins, ws, s);
    return launch_sweep(x, n, dtype, plan, st, finalize_nbins, kListFull, plan.t_steps + 1u, ws, s);
}

// Whether a coarse-to-fine search of such a tensor is available: wherever the tile search can take it.  Large
// bf16 tensors are searched through their value table (a full sweep over 65536 entries costs a few microseconds,
// so there is nothing to gain) and are refused.
bool coarse_to_fine_supported(uint64_t n, int dtype, const SearchPlan &plan)
{
    return !uses_value_table(n, dtype) && tile_search_can_run(plan);
}

}  // namespace qp
