// The C ABI: argument checks, host-side scalar work (ACIQ constants, quantization grid),
// kernel launches, result copies.  Every per-element step runs in the HIP kernels; there
// is no CPU fallback.
#include <atomic>
#include <cmath>
#include <cstring>

#include "qp_common.hpp"

using namespace qp;

namespace {

bool bits_ok(uint32_t b) { return b == 2 || b == 3 || b == 4 || b == 6 || b == 8 || b == 16; }
bool dtype_ok(int d) { return d == QP_F32 || d == QP_BF16; }
bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }
constexpr uint64_t kMaxN = 0xffffffffull;   // histogram counts and block partial counters are 32-bit

// Principal Lambert W for z >= e: Newton on g(w) = w + ln w - ln z (well conditioned for large z).
double lambert_w0_large(double z)
{
    const double lz = std::log(z);
    double w = lz - std::log(lz);
    for (int i = 0; i < 64; ++i) {
        const double g = w + std::log(w) - lz;
        const double wn = w - g / (1.0 + 1.0 / w);
        if (std::fabs(wn - w) <= 4e-16 * std::fabs(wn)) return wn;
        w = wn;
    }
    return w;
}

// Laplace: the minimiser of 2 e^{-a} + a^2/(3 4^q) satisfies a e^a = 3 4^q.
double laplace_constant(uint32_t bits) { return lambert_w0_large(3.0 * std::ldexp(1.0, 2 * (int)bits)); }

// Gaussian: the minimiser of 2[(1+a^2)Q(a) - a phi(a)] + a^2/(3 4^q) satisfies
// phi(a) - a Q(a) = a / (6 4^q).  Safeguarded Newton: the left side minus the right is convex
// and decreasing, its derivative is -Q(a) - 1/(6 4^q).
double gauss_constant(uint32_t bits)
{
    const double k = 1.0 / (6.0 * std::ldexp(1.0, 2 * (int)bits));
    const double c = 0.3989422804014326779399461;   // 1/sqrt(2 pi)
    double a = 1.0;
    for (int i = 0; i < 200; ++i) {
        const double phi = c * std::exp(-0.5 * a * a);
        const double Q = 0.5 * std::erfc(a * 0.7071067811865475244008444);
        const double h = phi - a * Q - a * k;
        const double an = a + h / (Q + k);
        if (std::fabs(an - a) <= 2e-16 * std::fabs(an)) return an;
        a = an;
    }
    return a;
}

qp_status check_ws(uint64_t n, const qp_search_cfg_t *cfg, const void *ws, size_t ws_bytes)
{
    if (!ws || !aligned16(ws)) return QP_EINVAL;
    const size_t need = qp_workspace_bytes(n, cfg);
    if (need == 0) return QP_EINVAL;
    if (ws_bytes < need) return QP_ENOSPC;
    return QP_OK;
}

qp_status check_cfg(const qp_search_cfg_t *cfg)
{
    if (!cfg) return QP_OK;
    if (cfg->t_steps < 1 || cfg->t_steps > kMaxT) return QP_EINVAL;
    if (cfg->cands_per_round < 1 || cfg->cands_per_round > kMaxCandsPerRound) return QP_EINVAL;
    if (cfg->dist != QP_LAPLACE && cfg->dist != QP_GAUSS && cfg->dist != QP_DIST_AUTO) return QP_EINVAL;
    if (cfg->flags & ~(QP_SEARCH_CLIP_TO_DATA | QP_SEARCH_COARSE_TO_FINE | QP_SEARCH_LOW_BITS_ONLY)) return QP_EINVAL;
    if (cfg->coarse_stride > 64u) return QP_EINVAL;
    return QP_OK;
}

// The host's decisions about one search (cfg already checked).
SearchPlan make_plan(uint32_t bits, const qp_search_cfg_t *cfg)
{
    SearchPlan p;
    p.bits = bits;
    p.t_steps = cfg ? cfg->t_steps : 100u;
    p.cpr = cfg ? cfg->cands_per_round : 13u;
    p.dist = cfg ? cfg->dist : (uint32_t)QP_LAPLACE;
    p.C = p.dist == QP_GAUSS ? gauss_constant(bits) : laplace_constant(bits);
    p.C_alt = p.dist == QP_DIST_AUTO ? gauss_constant(bits) : 0.0;
    p.clip = (cfg && (cfg->flags & QP_SEARCH_CLIP_TO_DATA)) ? 1u : 0u;
    p.stride = 1u;
    if (cfg && (cfg->flags & QP_SEARCH_COARSE_TO_FINE)) p.stride = cfg->coarse_stride ? cfg->coarse_stride : 10u;
    p.aciq_only = (cfg && (cfg->flags & QP_SEARCH_LOW_BITS_ONLY) && bits > 4u) ? 1u : 0u;
    return p;
}

qp_status hip_status(hipError_t e) { return e == hipSuccess ? QP_OK : QP_EHIP; }

// ---- the sender path for callers that cannot allocate ----------------------------------------
// The workspace of qp_compress_async, kept in the library's own image: a file-scope device array
// (each GPU that loads the library holds its own copy until the process ends).  In host code the
// array's name only stands for the symbol; its device address comes from hipGetSymbolAddress, once
// per device, and that address is what is handed to the kernels.
constexpr uint32_t kScratchMaxT = 127u;   // most search steps the static workspace is sized for
constexpr size_t kScratchBytes = kOffSearchPart + (size_t)kMaxSearchBlocks * (kScratchMaxT + 1u) * sizeof(double);
static __device__ __align__(256) unsigned char scratch[kScratchBytes];
constexpr int kScratchMaxDevices = 64;
std::atomic<void *> scratch_ptr[kScratchMaxDevices];   // zero-initialised; a race only repeats the same query

qp_status scratch_on_current_device(void **out)
{
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess) return QP_EHIP;
    if (dev < 0 || dev >= kScratchMaxDevices) return QP_EINVAL;
    void *p = scratch_ptr[dev].load(std::memory_order_acquire);
    if (!p) {
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return QP_EHIP;
        scratch_ptr[dev].store(p, std::memory_order_release);
    }
    *out = p;
    return QP_OK;
}

}  // namespace

extern "C" {

size_t qp_packed_bytes(uint64_t n, uint32_t bits)
{
    if (!bits_ok(bits)) return 0;
    return (size_t)(4u * ((n * (uint64_t)bits + 31u) / 32u));
}

void qp_default_search_cfg(qp_search_cfg_t *cfg)
{
    if (!cfg) return;
    cfg->t_steps = 100;
    cfg->cands_per_round = 13;
    cfg->nbins = 2048;
    cfg->dist = QP_LAPLACE;
    cfg->flags = 0;
    cfg->coarse_stride = 0;
}

size_t qp_workspace_bytes(uint64_t n, const qp_search_cfg_t *cfg)
{
    if (n == 0 || n > kMaxN) return 0;
    if (check_cfg(cfg) != QP_OK) return 0;
    const uint32_t t = cfg ? cfg->t_steps : 100u;
    // partial sums: one column per block of whichever search kernel the size selects, one row per
    // candidate of the longest sweep (the fine sweep of a coarse-to-fine search has up to 127)
    uint32_t cols = search_blocks(n);
    if (tile_search_blocks(n) > cols) cols = tile_search_blocks(n);
    const uint32_t rows = t + 1u > 128u ? t + 1u : 128u;
    return kOffSearchPart + (size_t)cols * rows * sizeof(double);
}

size_t qp_ws_offset(qp_ws_region region)
{
    switch (region) {
        case QP_WS_STATS: return kOffStats;
        case QP_WS_RESULT: return kOffResult;
        case QP_WS_QPARAMS: return kOffQParams;
        case QP_WS_HIST: return kOffHist;
        case QP_WS_CANDS: return kOffCands;
        case QP_WS_SCORES: return kOffScores;
        case QP_WS_MODEL: return kOffModel;
        default: return (size_t)-1;
    }
}

qp_status qp_stats_async(const void *x_dev, uint64_t n, qp_dtype dtype, uint32_t nbins, void *ws_dev, size_t ws_bytes,
                         void *stream)
{
    if (!x_dev || n == 0 || n > kMaxN || !dtype_ok(dtype) || nbins < 16 || nbins > kMaxBins || !aligned16(x_dev))
        return QP_EINVAL;
    if (!ws_dev || !aligned16(ws_dev)) return QP_EINVAL;
    if (ws_bytes < kOffSearchPart) return QP_ENOSPC;   // the statistics use only the fixed-size head
    return hip_status(launch_stats(x_dev, n, dtype, nbins, ws_dev, static_cast<hipStream_t>(stream), true));
}

qp_status qp_stats(const void *x_dev, uint64_t n, qp_dtype dtype, uint32_t nbins, void *ws_dev, size_t ws_bytes,
                   void *stream, qp_stats_t *out_host)
{
    if (!out_host) return QP_EINVAL;
    const qp_status st = qp_stats_async(x_dev, n, dtype, nbins, ws_dev, ws_bytes, stream);
    if (st != QP_OK) return st;
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (hipMemcpyAsync(out_host, static_cast<char *>(ws_dev) + kOffStats, sizeof(qp_stats_t), hipMemcpyDeviceToHost,
                       s) != hipSuccess)
        return QP_EHIP;
    if (hipStreamSynchronize(s) != hipSuccess) return QP_EHIP;
    return out_host->n_nonfinite ? QP_ENONFINITE : QP_OK;
}

double qp_aciq_constant(uint32_t bits, qp_dist dist)
{
    if (!bits_ok(bits)) return NAN;
    if (dist == QP_LAPLACE) return laplace_constant(bits);
    if (dist == QP_GAUSS) return gauss_constant(bits);
    return NAN;
}

qp_status qp_aciq_alpha(const qp_stats_t *stats, uint32_t bits, qp_dist dist, double *alpha_out)
{
    if (!stats || !alpha_out || !bits_ok(bits)) return QP_EINVAL;
    if (dist == QP_LAPLACE) *alpha_out = laplace_constant(bits) * stats->mad;
    else if (dist == QP_GAUSS) *alpha_out = gauss_constant(bits) * std::sqrt(stats->var);
    else return QP_EINVAL;
    return QP_OK;
}

qp_status qp_make_qparams(double center, double alpha, uint32_t bits, uint64_t n, qp_qparams_t *out)
{
    if (!out || !bits_ok(bits)) return QP_EINVAL;
    out->bits = bits;
    out->reserved = 0;
    out->n = n;
    make_grid(center, alpha, bits, out->lo, out->hi, out->scale, out->inv_scale);
    return QP_OK;
}

qp_status qp_make_qparams_clipped(double center, double alpha, double data_min, double data_max, uint32_t bits,
                                  uint64_t n, qp_qparams_t *out)
{
    if (!out || !bits_ok(bits)) return QP_EINVAL;
    out->bits = bits;
    out->reserved = 0;
    out->n = n;
    make_grid(center, alpha, bits, out->lo, out->hi, out->scale, out->inv_scale, true, (float)data_min, (float)data_max);
    return QP_OK;
}

static qp_status search_common(const void *x_dev, uint64_t n, qp_dtype dtype, const qp_stats_t *stats, uint32_t bits,
                               const qp_search_cfg_t *cfg, void *ws_dev, size_t ws_bytes, void *stream,
                               uint32_t finalize_nbins = 0, bool value_table_ready = false)
{
    if (!x_dev || n == 0 || n > kMaxN || !dtype_ok(dtype) || !bits_ok(bits) || !aligned16(x_dev)) return QP_EINVAL;
    if (check_cfg(cfg) != QP_OK) return QP_EINVAL;
    const qp_status w = check_ws(n, cfg, ws_dev, ws_bytes);
    if (w != QP_OK) return w;
    const SearchPlan plan = make_plan(bits, cfg);
    if (!plan.aciq_only && plan.stride > 1u && !coarse_to_fine_supported(n, dtype, plan)) return QP_EINVAL;   // see quantpipe.h
    if (plan.dist == QP_DIST_AUTO) {   // the choice of the model, on the record and histogram in the workspace
        if (finalize_nbins) return QP_EINVAL;   // (internal: the record must already be final)
        const qp_status m = hip_status(launch_model_fit(ws_dev, static_cast<hipStream_t>(stream)));
        if (m != QP_OK) return m;
    }
    return hip_status(launch_search(x_dev, n, dtype, plan, stats, finalize_nbins, value_table_ready, ws_dev,
                                    static_cast<hipStream_t>(stream)));
}

qp_status qp_dsaciq_search_async(const void *x_dev, uint64_t n, qp_dtype dtype, uint32_t bits,
                                 const qp_search_cfg_t *cfg, void *ws_dev, size_t ws_bytes, void *stream)
{
    return search_common(x_dev, n, dtype, nullptr, bits, cfg, ws_dev, ws_bytes, stream);
}

qp_status qp_dsaciq_search(const void *x_dev, uint64_t n, qp_dtype dtype, const qp_stats_t *stats, uint32_t bits,
                           const qp_search_cfg_t *cfg, void *ws_dev, size_t ws_bytes, void *stream,
                           qp_search_result_t *res_host, qp_qparams_t *qparams_out_host)
{
    if (!stats) return QP_EINVAL;
    const qp_status st = search_common(x_dev, n, dtype, stats, bits, cfg, ws_dev, ws_bytes, stream);
    if (st != QP_OK) return st;
    hipStream_t s = static_cast<hipStream_t>(stream);
    char *w = static_cast<char *>(ws_dev);
    if (res_host &&
        hipMemcpyAsync(res_host, w + kOffResult, sizeof(qp_search_result_t), hipMemcpyDeviceToHost, s) != hipSuccess)
        return QP_EHIP;
    if (qparams_out_host &&
        hipMemcpyAsync(qparams_out_host, w + kOffQParams, sizeof(qp_qparams_t), hipMemcpyDeviceToHost, s) != hipSuccess)
        return QP_EHIP;
    if (hipStreamSynchronize(s) != hipSuccess) return QP_EHIP;
    return QP_OK;
}

qp_status qp_model_fit_async(void *ws_dev, size_t ws_bytes, void *stream)
{
    if (!ws_dev || !aligned16(ws_dev)) return QP_EINVAL;
    if (ws_bytes < kOffSearchPart) return QP_ENOSPC;   // only the fixed-size head of the workspace is used
    return hip_status(launch_model_fit(ws_dev, static_cast<hipStream_t>(stream)));
}

qp_status qp_model_fit(void *ws_dev, size_t ws_bytes, void *stream, qp_model_fit_t *out_host)
{
    if (!out_host) return QP_EINVAL;
    const qp_status st = qp_model_fit_async(ws_dev, ws_bytes, stream);
    if (st != QP_OK) return st;
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (hipMemcpyAsync(out_host, static_cast<char *>(ws_dev) + kOffModel, sizeof(qp_model_fit_t), hipMemcpyDeviceToHost,
                       s) != hipSuccess)
        return QP_EHIP;
    if (hipStreamSynchronize(s) != hipSuccess) return QP_EHIP;
    return QP_OK;
}

qp_status qp_dsaciq_hist_search_async(uint32_t bits, const qp_search_cfg_t *cfg, void *ws_dev, size_t ws_bytes,
                                      void *stream)
{
    if (!bits_ok(bits) || check_cfg(cfg) != QP_OK) return QP_EINVAL;
    if (cfg && (cfg->dist != QP_LAPLACE || cfg->flags != 0u)) return QP_EINVAL;   // only the paper's form
    if (!ws_dev || !aligned16(ws_dev)) return QP_EINVAL;
    if (ws_bytes < kOffSearchPart) return QP_ENOSPC;   // only the fixed-size head of the workspace is used
    const uint32_t t = cfg ? cfg->t_steps : 100u;
    return hip_status(launch_hist_search(bits, t, laplace_constant(bits), ws_dev, static_cast<hipStream_t>(stream)));
}

qp_status qp_dsaciq_hist_search(uint32_t bits, const qp_search_cfg_t *cfg, void *ws_dev, size_t ws_bytes, void *stream,
                                qp_search_result_t *res_host, qp_qparams_t *qparams_out_host)
{
    const qp_status st = qp_dsaciq_hist_search_async(bits, cfg, ws_dev, ws_bytes, stream);
    if (st != QP_OK) return st;
    hipStream_t s = static_cast<hipStream_t>(stream);
    char *w = static_cast<char *>(ws_dev);
    if (res_host &&
        hipMemcpyAsync(res_host, w + kOffResult, sizeof(qp_search_result_t), hipMemcpyDeviceToHost, s) != hipSuccess)
        return QP_EHIP;
    if (qparams_out_host &&
        hipMemcpyAsync(qparams_out_host, w + kOffQParams, sizeof(qp_qparams_t), hipMemcpyDeviceToHost, s) != hipSuccess)
        return QP_EHIP;
    if (hipStreamSynchronize(s) != hipSuccess) return QP_EHIP;
    return QP_OK;
}

static qp_status pack_common(const void *x_dev, uint64_t n, qp_dtype dtype, uint32_t bits, const qp_qparams_t *hq,
                             const qp_qparams_t *dq, void *packed_dev, size_t packed_bytes, void *stream)
{
    if (!x_dev || !packed_dev || n == 0 || n > kMaxN || !dtype_ok(dtype) || !bits_ok(bits) || !aligned16(x_dev) ||
        !aligned16(packed_dev))
        return QP_EINVAL;
    if (packed_bytes < qp_packed_bytes(n, bits)) return QP_ENOSPC;
    return hip_status(launch_quant_pack(x_dev, n, dtype, bits, hq, dq, packed_dev, static_cast<hipStream_t>(stream)));
}

qp_status qp_quant_pack(const void *x_dev, uint64_t n, qp_dtype dtype, const qp_qparams_t *qparams, void *packed_dev,
                        size_t packed_bytes, void *stream)
{
    if (!qparams || qparams->n != n) return QP_EINVAL;
    return pack_common(x_dev, n, dtype, qparams->bits, qparams, nullptr, packed_dev, packed_bytes, stream);
}

qp_status qp_quant_pack_dev(const void *x_dev, uint64_t n, qp_dtype dtype, uint32_t bits,
                            const qp_qparams_t *qparams_dev, void *packed_dev, size_t packed_bytes, void *stream)
{
    if (!qparams_dev) return QP_EINVAL;
    return pack_common(x_dev, n, dtype, bits, nullptr, qparams_dev, packed_dev, packed_bytes, stream);
}

static qp_status unpack_common(const void *packed_dev, size_t packed_bytes, uint32_t bits, const qp_qparams_t *hq,
                               const qp_qparams_t *dq, float *y_dev, uint64_t n, void *stream)
{
    if (!packed_dev || !y_dev || n == 0 || n > kMaxN || !bits_ok(bits) || !aligned16(packed_dev) || !aligned16(y_dev))
        return QP_EINVAL;
    if (packed_bytes < qp_packed_bytes(n, bits)) return QP_ENOSPC;
    return hip_status(launch_unpack_dequant(packed_dev, bits, hq, dq, y_dev, n, static_cast<hipStream_t>(stream)));
}

qp_status qp_unpack_dequant(const void *packed_dev, size_t packed_bytes, const qp_qparams_t *qparams, float *y_dev,
                            uint64_t n, void *stream)
{
    if (!qparams || qparams->n != n) return QP_EINVAL;
    return unpack_common(packed_dev, packed_bytes, qparams->bits, qparams, nullptr, y_dev, n, stream);
}

qp_status qp_unpack_dequant_dev(const void *packed_dev, size_t packed_bytes, uint32_t bits,
                                const qp_qparams_t *qparams_dev, float *y_dev, uint64_t n, void *stream)
{
    if (!qparams_dev) return QP_EINVAL;
    return unpack_common(packed_dev, packed_bytes, bits, nullptr, qparams_dev, y_dev, n, stream);
}

// Everything qp_compress_async refuses, before anything is launched.
static qp_status check_compress(const void *x_dev, uint64_t n, qp_dtype dtype, uint32_t bits, const qp_search_cfg_t *cfg,
                                void *ws_dev, size_t ws_bytes, void *packed_dev, size_t packed_bytes)
{
    if (!packed_dev || !bits_ok(bits) || !aligned16(packed_dev)) return QP_EINVAL;
    if (packed_bytes < qp_packed_bytes(n, bits)) return QP_ENOSPC;
    const uint32_t nbins = (cfg && cfg->nbins) ? cfg->nbins : 2048u;
    if (!x_dev || n == 0 || n > kMaxN || !dtype_ok(dtype) || nbins < 16 || nbins > kMaxBins || !aligned16(x_dev))
        return QP_EINVAL;
    if (check_cfg(cfg) != QP_OK) return QP_EINVAL;
    const qp_status st = check_ws(n, cfg, ws_dev, ws_bytes);
    if (st != QP_OK) return st;
    // what the search would refuse
    const SearchPlan plan = make_plan(bits, cfg);
    if (!plan.aciq_only && plan.stride > 1u && !coarse_to_fine_supported(n, dtype, plan)) return QP_EINVAL;
    return QP_OK;
}

qp_status qp_compress_async(const void *x_dev, uint64_t n, qp_dtype dtype, uint32_t bits, const qp_search_cfg_t *cfg,
                            void *ws_dev, size_t ws_bytes, void *packed_dev, size_t packed_bytes,
                            qp_qparams_t *qparams_out_dev, void *stream)
{
    qp_status st = check_compress(x_dev, n, dtype, bits, cfg, ws_dev, ws_bytes, packed_dev, packed_bytes);
    if (st != QP_OK) return st;
    const uint32_t nbins = (cfg && cfg->nbins) ? cfg->nbins : 2048u;
    // The two statistics passes leave partials and the search finalizes them itself; a large bf16 tensor goes
    // through its value table instead, which the statistics build and finalize and the search then reuses.
    // (With the model chosen on the device the record is needed before the search starts: the statistics finalize it.)
    const bool table = uses_value_table(n, dtype);
    const bool final_record = table || (cfg && cfg->dist == QP_DIST_AUTO);
    st = hip_status(launch_stats(x_dev, n, dtype, nbins, ws_dev, static_cast<hipStream_t>(stream), final_record));
    if (st != QP_OK) return st;
    st = search_common(x_dev, n, dtype, nullptr, bits, cfg, ws_dev, ws_bytes, stream, final_record ? 0u : nbins, table);
    if (st != QP_OK) return st;
    const qp_qparams_t *qdev = reinterpret_cast<const qp_qparams_t *>(static_cast<char *>(ws_dev) + kOffQParams);
    st = qp_quant_pack_dev(x_dev, n, dtype, bits, qdev, packed_dev, packed_bytes, stream);
    if (st != QP_OK) return st;
    if (qparams_out_dev &&
        hipMemcpyAsync(qparams_out_dev, qdev, sizeof(qp_qparams_t), hipMemcpyDeviceToDevice,
                       static_cast<hipStream_t>(stream)) != hipSuccess)
        return QP_EHIP;
    return QP_OK;
}

qp_status qp_compress_many_async(const qp_job_t *jobs, uint32_t count, const qp_search_cfg_t *cfg, const qp_lane_t *lanes,
                                 uint32_t n_lanes)
{
    if (!jobs || !lanes || count == 0 || n_lanes == 0 || n_lanes > 64u) return QP_EINVAL;
    // lanes must not share workspace memory (their calls overlap in time)
    for (uint32_t a = 0; a < n_lanes; ++a) {
        if (!lanes[a].ws_dev) return QP_EINVAL;
        const char *a0 = static_cast<const char *>(lanes[a].ws_dev), *a1 = a0 + lanes[a].ws_bytes;
        for (uint32_t b = a + 1; b < n_lanes; ++b) {
            const char *b0 = static_cast<const char *>(lanes[b].ws_dev), *b1 = b0 + lanes[b].ws_bytes;
            if (b0 && a0 < b1 && b0 < a1) return QP_EINVAL;
        }
    }
    // every job is checked before the first is launched
    for (uint32_t i = 0; i < count; ++i) {
        const qp_job_t &j = jobs[i];
        const qp_lane_t &l = lanes[i % n_lanes];
        if (j.dtype != (uint32_t)QP_F32 && j.dtype != (uint32_t)QP_BF16) return QP_EINVAL;
        const qp_status st = check_compress(j.x_dev, j.n, (qp_dtype)j.dtype, j.bits, cfg, l.ws_dev, l.ws_bytes, j.packed_dev,
                                            (size_t)j.packed_bytes);
        if (st != QP_OK) return st;
        // a later job of this call overwrites the lane's records: this one's grid must leave the workspace
        if ((uint64_t)i + n_lanes < count && !j.qparams_out_dev) return QP_EINVAL;
    }
    for (uint32_t i = 0; i < count; ++i) {
        const qp_job_t &j = jobs[i];
        const qp_lane_t &l = lanes[i % n_lanes];
        const qp_status st = qp_compress_async(j.x_dev, j.n, (qp_dtype)j.dtype, j.bits, cfg, l.ws_dev, l.ws_bytes, j.packed_dev,
                                               (size_t)j.packed_bytes, j.qparams_out_dev, l.stream);
        if (st != QP_OK) return st;
    }
    return QP_OK;
}

qp_status qp_compress_noalloc(const void *x_dev, uint64_t n, qp_dtype dtype, uint32_t bits, const qp_search_cfg_t *cfg,
                              void *packed_dev, size_t packed_bytes, qp_qparams_t *qparams_out_dev, void *stream)
{
    if (!qparams_out_dev) return QP_EINVAL;   // the caller has no other way to the winner's grid
    if (n == 0 || n > kMaxN || check_cfg(cfg) != QP_OK) return QP_EINVAL;
    // sizes beyond what the static workspace holds
    if (cfg && cfg->t_steps > kScratchMaxT) return QP_ENOSPC;
    const size_t need = qp_workspace_bytes(n, cfg);
    if (need == 0) return QP_EINVAL;
    if (need > kScratchBytes) return QP_ENOSPC;
    void *ws = nullptr;
    const qp_status st = scratch_on_current_device(&ws);
    if (st != QP_OK) return st;
    return qp_compress_async(x_dev, n, dtype, bits, cfg, ws, kScratchBytes, packed_dev, packed_bytes, qparams_out_dev,
                             stream);
}

qp_status qp_next_bits(double v_bits, uint32_t q_cur, double s_images, double r_images_per_s,
                       double bandwidth_bits_per_s, uint32_t *q_next)
{
    if (!q_next || !(bits_ok(q_cur) || q_cur == 32)) return QP_EINVAL;
    if (!(v_bits > 0.0) || !(s_images > 0.0) || !(r_images_per_s > 0.0) || !(bandwidth_bits_per_s > 0.0))
        return QP_EINVAL;   // also rejects NaN
    if (std::isinf(v_bits) || std::isinf(s_images) || std::isinf(r_images_per_s)) return QP_EINVAL;
    const double uncompressed = v_bits * 32.0 / (double)q_cur;
    const double budget = s_images / r_images_per_s * bandwidth_bits_per_s;   // bits per microbatch period
    // smallest m >= 0 with uncompressed <= 2^m * budget, i.e. ceil(log2(ratio)) clamped at 0
    uint32_t q = 32;
    double fits = budget;
    while (q > 2 && uncompressed > fits) {
        q >>= 1;
        fits *= 2.0;
    }
    *q_next = q;
    return QP_OK;
}

qp_status qp_controller_init(qp_controller_t *c, uint32_t window, double s_images, double r_images_per_s,
                             uint32_t q_start)
{
    if (!c || window == 0 || !(s_images > 0.0) || !(r_images_per_s > 0.0) || std::isinf(s_images) ||
        std::isinf(r_images_per_s) || !(bits_ok(q_start) || q_start == 32))
        return QP_EINVAL;
    c->window = window;
    c->count = 0;
    c->bits_sum = 0.0;
    c->seconds_sum = 0.0;
    c->s_images = s_images;
    c->r_images_per_s = r_images_per_s;
    c->q_cur = q_start;
    c->decisions = 0;
    return QP_OK;
}

qp_status qp_controller_update(qp_controller_t *c, double payload_bits, double seconds, uint32_t *q_next)
{
    if (!c || !q_next || !(payload_bits > 0.0) || !(seconds > 0.0) || std::isinf(payload_bits) || std::isinf(seconds))
        return QP_EINVAL;
    if (c->count + 1 == c->window) {   // this report closes the window: decide on its averages
        const double bits = c->bits_sum + payload_bits, secs = c->seconds_sum + seconds;
        uint32_t q = c->q_cur;
        const qp_status st = qp_next_bits(bits / (double)c->window, c->q_cur, c->s_images, c->r_images_per_s, bits / secs, &q);
        if (st != QP_OK) return st;
        c->q_cur = q;
        c->count = 0;
        c->bits_sum = 0.0;
        c->seconds_sum = 0.0;
        c->decisions += 1;
    } else {
        c->bits_sum += payload_bits;
        c->seconds_sum += seconds;
        c->count += 1;
    }
    *q_next = c->q_cur;
    return QP_OK;
}

const char *qp_strerror(qp_status status)
{
    switch (status) {
        case QP_OK: return "ok";
        case QP_EINVAL: return "invalid argument";
        case QP_ENOSPC: return "buffer or workspace too small";
        case QP_EHIP: return "HIP runtime error";
        case QP_ENONFINITE: return "tensor contains NaN or Inf";
        default: return "unknown status";
    }
}

}  // extern "C"
