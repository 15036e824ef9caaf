// Step 2b for small and medium tensors: the DS-ACIQ directed search (Sec. 3, Eq. 1) with
// the roles of lanes and elements exchanged.
//
// The streaming search kernel gives a lane its own elements and runs the candidates over them;
// every candidate then needs a reduction across lanes, blocks and rounds, and for a tensor of a
// few hundred thousand elements (one image's activations) those hand-overs cost several times
// the arithmetic.  Here a block stages a tile of the tensor in LDS and a lane owns ONE
// CANDIDATE: it walks a slice of the tile (LDS broadcast reads: the lanes of a wave read the
// same address), applies its candidate's grid, which it keeps in registers, and accumulates in
// one fp64 register.  A candidate's score on the tile is then the sum of a handful of lanes'
// registers: no cross-lane reduction trees, no rounds, all t+1 candidates in one pass over the
// tensor.
//   k_search_tile   one block per share of the tensor: (optionally) turns the statistics partials
//                   into the record, builds the candidate table (every block the same values in
//                   the same order), scores, writes one partial per candidate and block;
//   k_search_pick   one block per candidate adds that candidate's partials in a fixed order; the
//                   block that draws the last ticket takes the first minimum and writes the
//                   result record and the winner's grid.
// The per-element arithmetic is that of quantize+pack and unpack+dequantize; sums are fp64 in a
// fixed order (bit-reproducible).  Scores handed from block to block inside k_search_pick use
// device-coherent accesses, so the ticket needs no cache write-back or invalidation.
#include <type_traits>

#include "qp_common.hpp"

namespace qp {

constexpr int kStThreads = kFinThreads;          // 512: finalize_stats_block fixes it
constexpr uint32_t kStVecs = 2;                  // 4-element vectors a lane stages per sub-tile
constexpr uint32_t kStSub = kStThreads * kStVecs * 4;   // 4096 elements per sub-tile (16 KB of LDS)
constexpr uint32_t kStMaxCands = 256;            // every candidate gets a lane (or several)
constexpr uint32_t kStMaxBlocks = 256;              // one block per compute unit: no unit gets two while others idle

struct TileSearchArgs {
    const void *x;
    uint64_t n;
    uint64_t share;          // elements per block, a multiple of 4
    uint32_t bits, t_steps;
    double F;
    double mean_h, b_e_h, b_r_h;   // statistics from the host (from_ws == 0)
    int from_ws;
    FinalizeArgs fin;        // fin.nbins != 0: the statistics passes left partials only
    qp_stats_t *stats_dev;
    Cand *cands;
    Ctl *ctl;
    double *partials;        // [t_steps + 1][gridDim.x]
};

template <int DT> __global__ __launch_bounds__(kStThreads) void k_search_tile(TileSearchArgs a)
{
    __shared__ __align__(16) float sh_x[kStSub];
    __shared__ Cand sh_cands[kStMaxCands];
    __shared__ double sh_acc[kStThreads];
    __shared__ qp_stats_t sh_st;

    const uint32_t tid = threadIdx.x;
    const uint32_t G = gridDim.x, blk = blockIdx.x;
    const uint32_t ncand = a.t_steps + 1u;
    const uint64_t e_begin = (uint64_t)blk * a.share;
    const uint64_t e_end = min(a.n, e_begin + a.share);

    // a sub-tile's load: lane -> two 4-element vectors; elements past the end read as 0 (never scored)
    float f[kStVecs][4];
    auto load_sub = [&](uint64_t e0) {
#pragma unroll
        for (uint32_t v = 0; v < kStVecs; ++v) {
            const uint64_t e = e0 + 4ull * (v * kStThreads + tid);
            if (e + 4 <= e_end) {
                Vec4<DT>::load(a.x, e / 4, f[v]);
            } else {
#pragma unroll
                for (uint32_t i = 0; i < 4; ++i) f[v][i] = (e + i < e_end) ? Vec4<DT>::load1(a.x, e + i) : 0.0f;
            }
        }
    };
    // the first sub-tile is requested before the statistics are touched
    load_sub(e_begin);

    // ---- statistics record and candidate table ----
    if (a.fin.nbins) {
        finalize_stats_block(a.fin.part1, a.fin.nb1, a.fin.part2, a.fin.nb2, a.fin.hist, a.fin.nbins, a.n, &sh_st);
        if (blk == 0 && tid == 0) *a.stats_dev = sh_st;
    }
    double mean = a.mean_h, b_e = a.b_e_h, b_r = a.b_r_h;
    if (a.fin.nbins) {
        mean = sh_st.mean;
        b_e = sh_st.mad;
        b_r = sh_st.b_r;
    } else if (a.from_ws) {
        mean = a.stats_dev->mean;
        b_e = a.stats_dev->mad;
        b_r = a.stats_dev->b_r;
    }
    double step = (b_r - b_e) / (double)a.t_steps;
    {
        const bool ok = (b_e > 0.0) && (b_r > 0.0) && isfinite(b_r) && isfinite(b_e) && isfinite(step);
        if (!ok) step = 0.0;   // the grid collapses onto b_E
    }
    const float Lf = (float)((1u << a.bits) - 1u);
    int safe = 1;
    if (tid < ncand) {
        const double b_j = b_e + (double)tid * step;
        Cand c;
        make_grid(mean, a.F * b_j, a.bits, c.lo, c.hi, c.scale, c.inv_scale);
        sh_cands[tid] = c;
        if (blk == 0) a.cands[tid] = c;
        // With x clamped to [lo, hi], the level is at most rint(fl(fl(hi - lo) * inv_scale)); if that is
        // at most L for every candidate, the clamp of the rounded level can never act and is dropped.
        const float topl = rintf((c.hi - c.lo) * c.inv_scale);
        if (!(isfinite(c.lo) && isfinite(c.hi) && topl >= 0.0f && topl <= Lf)) safe = 0;
    }
    safe = __syncthreads_and(safe);
    if (blk == 0 && tid == 0) {
        a.ctl->ticket_search = 0u;
        a.ctl->short_seq = (uint32_t)safe;
        a.ctl->b_e = b_e;
        a.ctl->b_r = b_r;
        a.ctl->step = step;
        a.ctl->F = a.F;
        a.ctl->mean = mean;
        a.ctl->bits = a.bits;
        a.ctl->t_steps = a.t_steps;
        a.ctl->n = a.n;
    }

    // ---- scoring: lane -> (slice of the sub-tile, candidate) ----
    const uint32_t S = kStThreads / ncand;            // slices, >= 2
    const uint32_t slice = tid / ncand, c = tid - slice * ncand;
    const bool active = slice < S;
    const Cand p = sh_cands[active ? c : 0u];
    double acc = 0.0;
    for (uint64_t e0 = e_begin; e0 < e_end; e0 += kStSub) {
        __syncthreads();   // the previous sub-tile has been read
#pragma unroll
        for (uint32_t v = 0; v < kStVecs; ++v)
            reinterpret_cast<float4 *>(sh_x)[v * kStThreads + tid] = make_float4(f[v][0], f[v][1], f[v][2], f[v][3]);
        __syncthreads();
        if (e0 + kStSub < e_end) load_sub(e0 + kStSub);   // next sub-tile in flight while this one is scored
        const uint32_t nv = (uint32_t)min((uint64_t)kStSub, e_end - e0);
        const uint32_t nv4 = nv / 4u;
        const uint32_t per = (nv4 + S - 1u) / S;
        if (active) {
            const uint32_t g0 = min(slice * per, nv4), g1 = min(g0 + per, nv4);
            auto run = [&](auto short_tag) {
                constexpr bool SHORT = decltype(short_tag)::value;
                auto one = [&](float xv) {
                    float r;
                    if constexpr (SHORT) {
                        // med3(x, lo, hi) == min(max(x, lo), hi) for lo <= hi, NaN -> lo as well
                        const float xc = __builtin_amdgcn_fmed3f(xv, p.lo, p.hi);
                        const float d = xc - p.lo;
                        const float t = d * p.inv_scale;
                        r = rintf(t);
                    } else {
                        r = quant_level(xv, p.lo, p.hi, p.inv_scale, Lf);
                    }
                    const float err = xv - dequant_level(r, p.scale, p.lo);
                    const double de = (double)err;
                    acc = fma(de, de, acc);   // de*de is exact in fp64
                };
                for (uint32_t g = g0; g < g1; ++g) {
                    const float4 xv = reinterpret_cast<const float4 *>(sh_x)[g];
                    one(xv.x);
                    one(xv.y);
                    one(xv.z);
                    one(xv.w);
                }
                if (slice == 0)   // the tensor's ragged end (fewer than 4 elements)
                    for (uint32_t e = 4u * nv4; e < nv; ++e) one(sh_x[e]);
            };
            if (safe) run(std::true_type{});
            else run(std::false_type{});
        }
    }
    if (active) sh_acc[tid] = acc;
    __syncthreads();
    if (tid < ncand) {
        double s = sh_acc[tid];
        for (uint32_t k = 1; k < S; ++k) s += sh_acc[k * ncand + tid];
        a.partials[(uint64_t)tid * G + blk] = s;   // candidate-major: a candidate's partials are contiguous
    }
}

constexpr int kPkThreadsPick = 256;
__global__ __launch_bounds__(kPkThreadsPick) void k_search_pick(const double *__restrict__ partials, uint32_t nblocks,
                                                                double *__restrict__ scores, Ctl *__restrict__ ctl,
                                                                qp_search_result_t *__restrict__ res,
                                                                qp_qparams_t *__restrict__ best, uint64_t n)
{
    __shared__ double sh[kStMaxCands];
    __shared__ uint32_t sh_flag;
    const uint32_t tid = threadIdx.x, wave = tid / kWave, lane = tid % kWave;
    const uint32_t c = blockIdx.x, ncand = gridDim.x;
    double s = 0.0;
    for (uint32_t b = tid; b < nblocks; b += kPkThreadsPick) s += partials[(uint64_t)c * nblocks + b];
    s = wave_sum(s);
    if (lane == 0) sh[wave] = s;
    __syncthreads();
    if (tid == 0) {
        double tot = sh[0];
        for (int k = 1; k < kPkThreadsPick / kWave; ++k) tot += sh[k];
        st_dev(&scores[c], tot);
        wait_stores();   // the score has arrived before the ticket is drawn
        const uint32_t prev = __hip_atomic_fetch_add(&ctl->ticket_search, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        sh_flag = (prev == ncand - 1u) ? 1u : 0u;
    }
    __syncthreads();
    if (!sh_flag) return;
    // the last block: every score has arrived; read them coherently
    for (uint32_t j = tid; j < ncand; j += kPkThreadsPick) sh[j] = ld_dev(&scores[j]);
    __syncthreads();
    if (wave != 0) return;
    const uint32_t bj = first_min_wave(sh, ncand, lane);
    if (lane == 0) {
        qp_search_result_t r;
        r.b_e = ctl->b_e;
        r.b_r = ctl->b_r;
        r.b_star = ctl->b_e + (double)bj * ctl->step;
        r.alpha_star = ctl->F * r.b_star;
        r.mse_aciq = sh[0] / (double)n;
        r.mse_star = sh[bj] / (double)n;
        r.j_star = bj;
        r.t_steps = ncand - 1u;
        *res = r;
        qp_qparams_t q;
        q.bits = ctl->bits;
        q.reserved = 0u;
        q.n = n;
        make_grid(ctl->mean, r.alpha_star, ctl->bits, q.lo, q.hi, q.scale, q.inv_scale);
        *best = q;
        ctl->ticket_search = 0u;
    }
}

bool tile_search_eligible(uint64_t n, uint32_t t_steps)
{
    return t_steps + 1u <= kStMaxCands && n <= kTileSearchMaxN;
}

uint32_t tile_search_blocks(uint64_t n)
{
    // shares of whole 128-element groups; as many blocks as shares of at least 512 elements allow
    uint64_t share = (n + kStMaxBlocks - 1) / kStMaxBlocks;
    share = (share + 127) / 128 * 128;
    if (share < 512) share = 512;
    return ceil_div_u64(n, share);
}

hipError_t launch_tile_search(const void *x, uint64_t n, int dtype, uint32_t bits, uint32_t t_steps, double F,
                              const qp_stats_t *st, uint32_t finalize_nbins, void *ws, hipStream_t s)
{
    if (!tile_search_eligible(n, t_steps)) return hipErrorInvalidValue;
    char *w = static_cast<char *>(ws);
    TileSearchArgs a;
    a.x = x;
    a.n = n;
    uint64_t share = (n + kStMaxBlocks - 1) / kStMaxBlocks;
    share = (share + 127) / 128 * 128;
    if (share < 512) share = 512;
    a.share = share;
    a.bits = bits;
    a.t_steps = t_steps;
    a.F = F;
    a.mean_h = st ? st->mean : 0.0;
    a.b_e_h = st ? st->mad : 0.0;
    a.b_r_h = st ? st->b_r : 0.0;
    a.from_ws = st ? 0 : 1;
    a.fin = FinalizeArgs{reinterpret_cast<const Part1 *>(w + kOffPart1), reinterpret_cast<const Part2 *>(w + kOffPart2),
                         reinterpret_cast<const uint32_t *>(w + kOffHist), 0u, 0u, finalize_nbins};
    if (finalize_nbins) stats_grid(n, dtype, a.fin.nb1, a.fin.nb2);
    a.stats_dev = reinterpret_cast<qp_stats_t *>(w + kOffStats);
    a.cands = reinterpret_cast<Cand *>(w + kOffCands);
    a.ctl = reinterpret_cast<Ctl *>(w + kOffCtl);
    a.partials = reinterpret_cast<double *>(w + kOffSearchPart);
    const uint32_t blocks = ceil_div_u64(n, share);
    if (dtype == QP_F32) hipLaunchKernelGGL(k_search_tile<QP_F32>, dim3(blocks), dim3(kStThreads), 0, s, a);
    else hipLaunchKernelGGL(k_search_tile<QP_BF16>, dim3(blocks), dim3(kStThreads), 0, s, a);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(k_search_pick, dim3(t_steps + 1u), dim3(kPkThreadsPick), 0, s, a.partials, blocks,
                       reinterpret_cast<double *>(w + kOffScores), a.ctl,
                       reinterpret_cast<qp_search_result_t *>(w + kOffResult),
                       reinterpret_cast<qp_qparams_t *>(w + kOffQParams), n);
    return hipGetLastError();
}

}  // namespace qp
