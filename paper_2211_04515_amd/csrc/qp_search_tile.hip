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
    ModelArgs m;             // the model and this sweep's candidate list
    FinalizeArgs fin;        // fin.nbins != 0: the statistics passes left partials only
    qp_stats_t *stats_dev;
    Cand *cands;
    Ctl *ctl;
    const qp_search_result_t *prev;   // the coarse winner, read before a fine sweep
    double *scores_by_j;
    double *partials;        // [m.count][gridDim.x]
};

template <int DT> __global__ __launch_bounds__(kStThreads) void k_search_tile(TileSearchArgs a)
{
    __shared__ __align__(16) float sh_x[kStSub];
    __shared__ Cand sh_cands[kStMaxCands];
    __shared__ double sh_acc[kStThreads];
    __shared__ qp_stats_t sh_st;

    const uint32_t tid = threadIdx.x;
    const uint32_t G = gridDim.x, blk = blockIdx.x;
    const uint32_t ncand = a.m.count;
    const ModelArgs m = resolve_model(a.m);
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

    // ---- statistics record and candidate table (every block the same values in the same order) ----
    const qp_stats_t *st = nullptr;
    if (a.fin.nbins) {
        finalize_stats_block(a.fin.part1, a.fin.nb1, a.fin.part2, a.fin.nb2, a.fin.hist, a.fin.nbins, a.n, &sh_st);
        if (blk == 0 && tid == 0) *a.stats_dev = sh_st;
        st = &sh_st;
    } else if (m.from_ws) {
        st = a.stats_dev;
    }
    const uint32_t j1 = (m.list_mode == kListFine) ? a.prev->j_star : 0u;
    const int safe = setup_candidates(m, st, j1, a.n, sh_cands, blk == 0 ? a.cands : nullptr, blk == 0 ? a.ctl : nullptr,
                                      blk == 0 ? a.scores_by_j : nullptr);
    const float Lf = (float)((1u << m.bits) - 1u);

    // ---- scoring: lane -> (slice of the sub-tile, candidate) ----
    const uint32_t S = kStThreads / ncand;            // slices, >= 2
    const uint32_t slice = tid / ncand, c = tid - slice * ncand;
    const bool active = slice < S;
    const Cand p = sh_cands[active ? c : 0u];
    double acc0 = 0.0, acc1 = 0.0;
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
                auto one = [&](float xv, double &acc) {
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
                // two groups of four per step, each with its own running sum: both LDS reads are issued
                // before the arithmetic, and the two fp64 accumulation chains interleave
                uint32_t g = g0;
                for (; g + 2 <= g1; g += 2) {
                    const float4 xa = reinterpret_cast<const float4 *>(sh_x)[g];
                    const float4 xb = reinterpret_cast<const float4 *>(sh_x)[g + 1];
                    one(xa.x, acc0);
                    one(xb.x, acc1);
                    one(xa.y, acc0);
                    one(xb.y, acc1);
                    one(xa.z, acc0);
                    one(xb.z, acc1);
                    one(xa.w, acc0);
                    one(xb.w, acc1);
                }
                if (g < g1) {
                    const float4 xa = reinterpret_cast<const float4 *>(sh_x)[g];
                    one(xa.x, acc0);
                    one(xa.y, acc0);
                    one(xa.z, acc0);
                    one(xa.w, acc0);
                }
                if (slice == 0)   // the tensor's ragged end (fewer than 4 elements)
                    for (uint32_t e = 4u * nv4; e < nv; ++e) one(sh_x[e], acc0);
            };
            if (safe) run(std::true_type{});
            else run(std::false_type{});
        }
    }
    if (active) sh_acc[tid] = acc0 + acc1;
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
                                                                qp_qparams_t *__restrict__ best, uint64_t n,
                                                                double *__restrict__ scores_by_j)
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
    const uint32_t bi = first_min_wave(sh, ncand, lane);
    if (lane == 0) write_search_result(ctl, sh, ncand, bi, n, scores_by_j, res, best);
}

static uint32_t plan_max_count(const SearchPlan &plan)
{
    if (plan.stride <= 1u) return plan.t_steps + 1u;
    const uint32_t coarse = (plan.t_steps + plan.stride - 1u) / plan.stride + 1u, fine = 2u * plan.stride - 1u;
    return coarse > fine ? coarse : fine;
}

// the kernel takes a tensor of any size; above kTileSearchMaxN the streaming search is the faster one
bool tile_search_can_run(const SearchPlan &plan) { return plan_max_count(plan) <= kStMaxCands; }

bool tile_search_eligible(uint64_t n, const SearchPlan &plan)
{
    return n <= kTileSearchMaxN && tile_search_can_run(plan);
}

static uint64_t tile_share(uint64_t n)
{
    // Shares of whole 128-element groups, at least 512 elements.  The grid is a whole number of blocks per
    // compute unit (no unit gets one more than another): one, or two from about two sub-tiles per unit on,
    // whose staging and scoring then overlap (2 M elements: 62 -> 57 us; coarse-to-fine on 9.7 M: 103 -> 90 us).
    const uint64_t per_cu = (n + (uint64_t)kStMaxBlocks * kStSub / 2) / ((uint64_t)kStMaxBlocks * kStSub);   // rounded
    const uint64_t blocks = (uint64_t)kStMaxBlocks * (per_cu >= 2 ? 2 : 1);
    uint64_t share = (n + blocks - 1) / blocks;
    share = (share + 127) / 128 * 128;
    return share < 512 ? 512 : share;
}

uint32_t tile_search_blocks(uint64_t n) { return ceil_div_u64(n, tile_share(n)); }

static hipError_t launch_tile_sweep(const void *x, uint64_t n, int dtype, const SearchPlan &plan, const qp_stats_t *st,
                                    uint32_t finalize_nbins, uint32_t list_mode, uint32_t count, void *ws, hipStream_t s)
{
    char *w = static_cast<char *>(ws);
    TileSearchArgs a;
    a.x = x;
    a.n = n;
    a.share = tile_share(n);
    a.m = model_args(plan, st, list_mode, count, ws);
    a.fin = FinalizeArgs{reinterpret_cast<const Part1 *>(w + kOffPart1), reinterpret_cast<const Part2 *>(w + kOffPart2),
                         reinterpret_cast<const uint32_t *>(w + kOffHist), 0u, 0u, finalize_nbins};
    if (finalize_nbins) stats_grid(n, dtype, a.fin.nb1, a.fin.nb2);
    a.stats_dev = reinterpret_cast<qp_stats_t *>(w + kOffStats);
    a.cands = reinterpret_cast<Cand *>(w + kOffCands);
    a.ctl = reinterpret_cast<Ctl *>(w + kOffCtl);
    a.prev = reinterpret_cast<const qp_search_result_t *>(w + kOffResult);
    a.scores_by_j = reinterpret_cast<double *>(w + kOffScores);
    a.partials = reinterpret_cast<double *>(w + kOffSearchPart);
    double *scores_list = list_mode == kListFull ? a.scores_by_j : reinterpret_cast<double *>(w + kOffListScores);
    const uint32_t blocks = ceil_div_u64(n, a.share);
    if (dtype == QP_F32) hipLaunchKernelGGL(k_search_tile<QP_F32>, dim3(blocks), dim3(kStThreads), 0, s, a);
    else hipLaunchKernelGGL(k_search_tile<QP_BF16>, dim3(blocks), dim3(kStThreads), 0, s, a);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(k_search_pick, dim3(count), dim3(kPkThreadsPick), 0, s, a.partials, blocks, scores_list, a.ctl,
                       reinterpret_cast<qp_search_result_t *>(w + kOffResult),
                       reinterpret_cast<qp_qparams_t *>(w + kOffQParams), n, a.scores_by_j);
    return hipGetLastError();
}

hipError_t launch_tile_search(const void *x, uint64_t n, int dtype, const SearchPlan &plan, const qp_stats_t *st,
                              uint32_t finalize_nbins, void *ws, hipStream_t s)
{
    if (!tile_search_can_run(plan)) return hipErrorInvalidValue;
    if (plan.stride <= 1u)
        return launch_tile_sweep(x, n, dtype, plan, st, finalize_nbins, kListFull, plan.t_steps + 1u, ws, s);
    const uint32_t coarse = (plan.t_steps + plan.stride - 1u) / plan.stride + 1u;
    hipError_t e = launch_tile_sweep(x, n, dtype, plan, st, finalize_nbins, kListCoarse, coarse, ws, s);
    if (e != hipSuccess) return e;
    return launch_tile_sweep(x, n, dtype, plan, st, 0u, kListFine, 2u * plan.stride - 1u, ws, s);
}

}  // namespace qp
