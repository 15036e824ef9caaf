// Step 2b: DS-ACIQ directed search (Sec. 3, Eq. 1).
//
// t+1 candidate scales b_j = b_E + j (b_R - b_E)/t walk from the ACIQ estimate towards the
// bound given by the real histogram's peak.  Each candidate is scored by the squared
// quantization error it causes on the real tensor.  This is plain vector-ALU work
// (about ten lane operations per element and candidate, no contraction), so the kernel is
// organised around registers, not bandwidth:
//   - a lane keeps 8 elements in VGPRs and runs up to 32 candidates over them; the
//     candidates' grids are wave-uniform (scalar loads), the 32 running sums are fp64
//     accumulators in VGPRs;
//   - blockIdx.y selects the round (a group of cands_per_round candidates), so the whole
//     search is one launch and the tensor is read once per round (mostly from the
//     Infinity Cache after the first round);
//   - per-block partial sums go to the workspace; the last block to finish (integer ticket)
//     adds them in block order, takes the first minimum and writes the result record and
//     the winner's quantization grid.  No floating-point atomics: bit-reproducible.
// The per-element arithmetic is the same inline code that quantize+pack and
// unpack+dequantize use, so a candidate's score is exactly the error of the tensor that
// would come out of the receiver.
#include "qp_common.hpp"

namespace qp {

constexpr int kSrThreads = 256;
constexpr int kSrElems = 8;   // elements per lane per batch (two 4-element vectors)

// One block of 256 lanes: fills the candidate table and the control record.
__global__ __launch_bounds__(256) void k_search_setup(const qp_stats_t *__restrict__ stats_dev, double mean_h,
                                                      double b_e_h, double b_r_h, int from_ws, uint32_t bits,
                                                      uint32_t t_steps, double F, uint64_t n,
                                                      Cand *__restrict__ cands, Ctl *__restrict__ ctl)
{
    double mean = mean_h, b_e = b_e_h, b_r = b_r_h;
    if (from_ws) {
        mean = stats_dev->mean;
        b_e = stats_dev->mad;
        b_r = stats_dev->b_r;
    }
    double step = (b_r - b_e) / (double)t_steps;
    const bool ok = (b_e > 0.0) && (b_r > 0.0) && isfinite(b_r) && isfinite(b_e) && isfinite(step);
    if (!ok) step = 0.0;   // the grid collapses onto b_E
    for (uint32_t j = threadIdx.x; j <= t_steps; j += blockDim.x) {
        const double b_j = b_e + (double)j * step;
        const double alpha = F * b_j;
        Cand c;
        make_grid(mean, alpha, bits, c.lo, c.hi, c.scale, c.inv_scale);
        cands[j] = c;
    }
    if (threadIdx.x == 0) {
        ctl->ticket_search = 0u;
        ctl->b_e = b_e;
        ctl->b_r = b_r;
        ctl->step = step;
        ctl->F = F;
        ctl->mean = mean;
        ctl->bits = bits;
        ctl->t_steps = t_steps;
        ctl->n = n;
    }
}

template <int DT>
__global__ __launch_bounds__(kSrThreads) void k_search_mse(const void *__restrict__ x, uint64_t n,
                                                           const Cand *__restrict__ cands, uint32_t ncand,
                                                           uint32_t cpr, float Lf, double *__restrict__ partials,
                                                           double *__restrict__ scores, Ctl *__restrict__ ctl,
                                                           qp_search_result_t *__restrict__ res,
                                                           qp_qparams_t *__restrict__ best)
{
    const uint32_t tid = threadIdx.x;
    const uint32_t c0 = blockIdx.y * cpr;
    const uint32_t nc = min(cpr, ncand - c0);

    double acc[kMaxCandsPerRound];
#pragma unroll
    for (int c = 0; c < (int)kMaxCandsPerRound; ++c) acc[c] = 0.0;

    auto score = [&](const float (&v)[kSrElems], int ne) {
#pragma unroll
        for (int c = 0; c < (int)kMaxCandsPerRound; ++c) {
            if ((uint32_t)c < nc) {   // wave-uniform
                const Cand p = cands[c0 + c];
#pragma unroll
                for (int e = 0; e < kSrElems; ++e) {
                    if (e < ne) {
                        const float r = quant_level(v[e], p.lo, p.hi, p.inv_scale, Lf);
                        const float err = v[e] - dequant_level(r, p.scale, p.lo);
                        const double de = (double)err;
                        acc[c] = fma(de, de, acc[c]);   // de*de is exact in fp64
                    }
                }
            }
        }
    };

    const uint64_t nbatch = n / kSrElems;
    for (uint64_t b = (uint64_t)blockIdx.x * kSrThreads + tid; b < nbatch; b += (uint64_t)gridDim.x * kSrThreads) {
        float v[kSrElems];
        float lo4[4], hi4[4];
        Vec4<DT>::load(x, 2 * b, lo4);
        Vec4<DT>::load(x, 2 * b + 1, hi4);
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            v[e] = lo4[e];
            v[4 + e] = hi4[e];
        }
        score(v, kSrElems);
    }
    // ragged tail: fewer than 8 elements, taken by one lane of block column 0
    const uint32_t rem = (uint32_t)(n - nbatch * kSrElems);
    if (rem && blockIdx.x == 0 && tid == 0) {
        float v[kSrElems];
#pragma unroll
        for (int e = 0; e < kSrElems; ++e) v[e] = ((uint32_t)e < rem) ? Vec4<DT>::load1(x, nbatch * kSrElems + e) : 0.0f;
        score(v, (int)rem);
    }

    // ---- block reduction: shuffles inside each wave64, one LDS row per wave ----
    __shared__ double sh[kSrThreads / kWave][kMaxCandsPerRound];
    __shared__ uint32_t sh_flag;
    const uint32_t wave = tid / kWave, lane = tid % kWave;
#pragma unroll
    for (int c = 0; c < (int)kMaxCandsPerRound; ++c) {
        const double s = wave_sum(acc[c]);
        if (lane == 0) sh[wave][c] = s;
    }
    __syncthreads();
    if (tid < nc) {
        double s = sh[0][tid];
        for (int w = 1; w < kSrThreads / kWave; ++w) s += sh[w][tid];
        partials[(uint64_t)blockIdx.x * ncand + c0 + tid] = s;
    }

    // ---- ticket: the last block of the whole grid finishes ----
    // (the barrier orders all lanes' writes before lane 0's device-scope release and lane 0's
    // acquire before all lanes' reads: one fencing lane per block, not one per wave)
    __syncthreads();
    if (tid == 0) {
        const uint32_t total = gridDim.x * gridDim.y;
        const uint32_t prev = __hip_atomic_fetch_add(&ctl->ticket_search, 1u, __ATOMIC_ACQ_REL, __HIP_MEMORY_SCOPE_AGENT);
        sh_flag = (prev == total - 1u) ? 1u : 0u;
    }
    __syncthreads();
    if (!sh_flag) return;

    for (uint32_t j = tid; j < ncand; j += kSrThreads) {
        double s = 0.0;
        for (uint32_t b = 0; b < gridDim.x; ++b) s += partials[(uint64_t)b * ncand + j];
        scores[j] = s;
    }
    __syncthreads();
    if (tid == 0) {
        uint32_t bj = 0;
        double bs = scores[0];
        for (uint32_t j = 1; j < ncand; ++j) {
            const double s = scores[j];
            if (s < bs) {   // strict: ties keep the smaller j
                bs = s;
                bj = j;
            }
        }
        qp_search_result_t r;
        r.b_e = ctl->b_e;
        r.b_r = ctl->b_r;
        r.b_star = ctl->b_e + (double)bj * ctl->step;
        r.alpha_star = ctl->F * r.b_star;
        r.mse_aciq = scores[0] / (double)n;
        r.mse_star = bs / (double)n;
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

uint32_t search_blocks(uint64_t n)
{
    const uint64_t nbatch = n / kSrElems;
    uint32_t nb = ceil_div_u64(nbatch, kSrThreads);
    if (nb < 1) nb = 1;
    if (nb > 512) nb = 512;
    return nb;
}

hipError_t launch_search(const void *x, uint64_t n, int dtype, uint32_t bits, uint32_t t_steps, uint32_t cpr,
                         double F, const qp_stats_t *st, void *ws, hipStream_t s)
{
    char *w = static_cast<char *>(ws);
    Cand *cands = reinterpret_cast<Cand *>(w + kOffCands);
    Ctl *ctl = reinterpret_cast<Ctl *>(w + kOffCtl);
    double *scores = reinterpret_cast<double *>(w + kOffScores);
    double *partials = reinterpret_cast<double *>(w + kOffSearchPart);
    qp_stats_t *stats_dev = reinterpret_cast<qp_stats_t *>(w + kOffStats);
    qp_search_result_t *res = reinterpret_cast<qp_search_result_t *>(w + kOffResult);
    qp_qparams_t *best = reinterpret_cast<qp_qparams_t *>(w + kOffQParams);

    hipLaunchKernelGGL(k_search_setup, dim3(1), dim3(256), 0, s, stats_dev, st ? st->mean : 0.0, st ? st->mad : 0.0,
                       st ? st->b_r : 0.0, st ? 0 : 1, bits, t_steps, F, n, cands, ctl);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;

    const uint32_t ncand = t_steps + 1u;
    const uint32_t rounds = (ncand + cpr - 1u) / cpr;
    const dim3 grid(search_blocks(n), rounds);
    const float Lf = (float)((1u << bits) - 1u);
    if (dtype == QP_F32)
        hipLaunchKernelGGL(k_search_mse<QP_F32>, grid, dim3(kSrThreads), 0, s, x, n, cands, ncand, cpr, Lf, partials,
                           scores, ctl, res, best);
    else
        hipLaunchKernelGGL(k_search_mse<QP_BF16>, grid, dim3(kSrThreads), 0, s, x, n, cands, ncand, cpr, Lf, partials,
                           scores, ctl, res, best);
    return hipGetLastError();
}

}  // namespace qp
