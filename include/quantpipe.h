/*
 * quantpipe.h -- C ABI of the MI355X (gfx950) activation-compression library.
 *
 * The library implements the data-parallel part of QuantPipe's PDA module
 * (arXiv 2211.04515, Sec. 3): the tensor that leaves a pipeline stage is
 * compressed to q-bit integer codes before it crosses the stage boundary and
 * is expanded back to fp32 on the other side.  Four steps:
 *
 *   1. qp_stats           per-tensor statistics: mean mu, mean absolute deviation
 *                         (the Laplace scale b_E), variance, min, max, and a
 *                         histogram D_R whose peak gives the search bound b_R;
 *   2. qp_aciq_alpha      ACIQ clipping threshold alpha = F(q) b       (host only)
 *      qp_dsaciq_search   DS-ACIQ directed search for b* in [b_E, b_R] (Eq. 1);
 *   3. qp_quant_pack      clip to [mu-alpha, mu+alpha], uniform quantize, bit-pack;
 *   4. qp_unpack_dequant  unpack and dequantize.
 *
 * Conventions
 *   - Pointers named *_dev are DEVICE pointers (HIP global memory on the current
 *     device); pointers named *_host, and all struct pointers unless named *_dev,
 *     are HOST pointers.  The caller owns every buffer.  The library allocates
 *     no device memory and keeps no state between calls except a per-device
 *     cache of one occupancy query (and the static workspace behind
 *     qp_compress_noalloc, which only that call uses); two calls may run
 *     concurrently if they use different streams AND different workspaces.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *   - x_dev, packed_dev, y_dev and ws_dev must be 16-byte aligned; ws_dev needs
 *     qp_workspace_bytes() bytes.  The workspace needs no initialisation.
 *   - Element types: QP_F32 (IEEE binary32) or QP_BF16 (bfloat16; widened exactly
 *     to fp32 in registers).  Tensors are contiguous and treated as flat, 1 <= n < 2^32.
 *   - Bitwidths: 2, 3, 4, 6, 8, 16.
 *   - Functions that return results to the host synchronise `stream` before
 *     returning; the *_async / *_dev forms never synchronise and leave their
 *     results in the workspace (offsets from qp_ws_offset()).
 *   - Errors are return codes only (no exceptions cross this boundary):
 *       QP_EINVAL     null pointer, n == 0 or too large, bad bitwidth / dtype /
 *                     nbins / search configuration, misaligned device pointer,
 *                     qparams->n != n;
 *       QP_ENOSPC     output buffer or workspace too small;
 *       QP_EHIP       a HIP call or kernel launch failed;
 *       QP_ENONFINITE qp_stats found NaN or Inf in the tensor (the statistics
 *                     are then not meaningful; n_nonfinite is valid).
 *
 * Wire format of the packed buffer (the paper leaves it open; Sec. 3 only fixes
 * the size, N q / 8 bytes: "compressed by 4x using 8-bit quantization"):
 * code i occupies bits [i q, i q + q) of a bit stream, least significant bit
 * first; stream bit p is bit (p mod 32) of little-endian 32-bit word (p div 32).
 * The buffer is 4*ceil(N q / 32) bytes; unused tail bits are written as zero.
 * The 32-byte qp_qparams_t travels beside the buffer.
 */
#ifndef QUANTPIPE_H
#define QUANTPIPE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum { QP_OK = 0, QP_EINVAL = -1, QP_ENOSPC = -2, QP_EHIP = -3, QP_ENONFINITE = -4 } qp_status;
typedef enum { QP_F32 = 0, QP_BF16 = 1 } qp_dtype;
typedef enum { QP_LAPLACE = 0, QP_GAUSS = 1, QP_DIST_AUTO = 2 } qp_dist;

/* Per-tensor statistics (Sec. 3: the activation is modelled as Laplace L(mu, b)). */
typedef struct {
    uint64_t n;            /* element count */
    uint64_t n_nonfinite;  /* NaN / Inf elements found */
    double   mean;         /* mu */
    double   mad;          /* (1/N) sum |x - mu|: the Laplace scale b_E */
    double   abs_mean;     /* (1/N) sum |x|: the estimate as printed in Sec. 3 (equals mad when mu = 0) */
    double   var;          /* (1/N) sum (x - mu)^2 */
    double   min, max;
    uint32_t nbins;        /* histogram D_R: nbins equal bins over [min, max] */
    uint32_t peak_count;   /* max(D_R) as a count */
    double   peak_density; /* peak_count / (N * bin width) */
    double   b_r;          /* search bound b_R = 1 / (2 max(D_R)) (after Eq. 1); 0 if min == max */
} qp_stats_t;

/* What the receiver needs besides the packed buffer. */
typedef struct {
    uint32_t bits;
    uint32_t reserved;     /* written as 0 */
    uint64_t n;
    float    lo, hi;       /* clipping range [mu - alpha, mu + alpha] rounded to fp32 */
    float    scale;        /* (hi - lo) / (2^bits - 1); 0 if hi == lo */
    float    inv_scale;    /* (2^bits - 1) / (hi - lo); 0 if hi == lo */
} qp_qparams_t;

/* Directed-search configuration.  The paper sets t_steps = 100 (Sec. 3), models the data as
 * Laplace, clips symmetrically about mu and sweeps all t_steps + 1 candidates: that is what a
 * zeroed `dist`, `flags` and `coarse_stride` give (and what qp_default_search_cfg() returns).
 * The other settings are variations on Eq. 1 beyond the paper, each with its own oracle:
 *   dist = QP_GAUSS             the Gaussian model of the ACIQ method the paper builds on: scale
 *                               estimate sigma_E = sqrt(var), alpha = G(q) sigma, search bound
 *                               sigma_R = 1 / (sqrt(2 pi) max(D_R)) (the sigma whose density peak
 *                               equals the histogram's);
 *   dist = QP_DIST_AUTO         the model is chosen per tensor on the device, with no host round trip: the one whose
 *                               pdf at its moment estimates lies closer to the histogram D_R (see qp_model_fit);
 *                               Gaussian only if strictly closer.  The statistics record and histogram that
 *                               qp_stats / qp_stats_async left in the same workspace are what is judged (and what
 *                               the grid is then built from); QP_WS_MODEL tells which model was taken;
 *   QP_SEARCH_CLIP_TO_DATA      every candidate range is intersected with the data's own range,
 *                               [max(mu - alpha, min), min(mu + alpha, max)], so one-sided data
 *                               (after a GELU) spends no levels below its minimum;
 *   QP_SEARCH_COARSE_TO_FINE    two sweeps instead of one: candidates j = 0, s, 2s, ..., t first,
 *                               then every candidate within s - 1 of the coarse winner; the first
 *                               minimum of the second sweep wins.  Equal to the full sweep's
 *                               result whenever the error curve has a single valley, with about
 *                               t/s + 2s evaluations instead of t + 1.  s = coarse_stride
 *                               (0 = 10; at most 64).  Scores of candidates that were never
 *                               evaluated are NaN in QP_WS_SCORES.  Not offered for bf16 tensors of
 *                               2^20 elements or more (QP_EINVAL): those are searched through the
 *                               table of their 65536 possible values, where the full sweep is cheap.
 *   QP_SEARCH_LOW_BITS_ONLY     the deployment policy the paper reports (Sec. 3, discussion of Table 1: the directed search
 *                               is only activated under 4- and 2-bit quantization, because above that
 *                               it gains nothing): for bits > 4 no candidate is scored and the result
 *                               is plain ACIQ (j_star = 0, alpha = F(q) b_E; mse_aciq, mse_star and
 *                               QP_WS_SCORES are NaN); for bits <= 4 the search runs as configured. */
#define QP_SEARCH_CLIP_TO_DATA 1u
#define QP_SEARCH_COARSE_TO_FINE 2u
#define QP_SEARCH_LOW_BITS_ONLY 4u
typedef struct {
    uint32_t t_steps;          /* 1..1023: candidates j = 0..t_steps */
    uint32_t cands_per_round;  /* 1..32: most candidates scored per pass over a large tensor (the library picks
                                  a round size of 16, 13, 8, 4, 2 or 1 within it; tensors searched tile by tile
                                  score all candidates in one pass); never changes results.  Default 13: the
                                  101 candidates in five rounds of 13 and three of 12 */
    uint32_t nbins;            /* kept with the configuration for callers; the search itself does not use it */
    uint32_t dist;             /* QP_LAPLACE (the paper's model), QP_GAUSS or QP_DIST_AUTO */
    uint32_t flags;            /* QP_SEARCH_* bits, 0 = the paper's method */
    uint32_t coarse_stride;    /* see QP_SEARCH_COARSE_TO_FINE */
} qp_search_cfg_t;

typedef struct {
    double   b_e, b_r;         /* the two ends of the search interval */
    double   b_star;           /* winning scale */
    double   alpha_star;       /* F(q) * b_star */
    double   mse_aciq;         /* mean squared quantization error at j = 0 (plain ACIQ) */
    double   mse_star;         /* ... at the winner; <= mse_aciq */
    uint32_t j_star;           /* winning grid index (0 = ACIQ kept) */
    uint32_t t_steps;
} qp_search_result_t;

/* Regions of the workspace that the *_async forms leave results in. */
typedef enum {
    QP_WS_STATS = 0,     /* qp_stats_t */
    QP_WS_RESULT = 1,    /* qp_search_result_t */
    QP_WS_QPARAMS = 2,   /* qp_qparams_t of the search winner */
    QP_WS_HIST = 3,      /* uint32_t[nbins] */
    QP_WS_CANDS = 4,     /* per candidate {float lo, hi, scale, inv_scale} */
    QP_WS_SCORES = 5,    /* double[t_steps + 1]: sums of squared errors */
    QP_WS_MODEL = 6      /* qp_model_fit_t: written by qp_model_fit and by a search with dist = QP_DIST_AUTO */
} qp_ws_region;

/* ---- sizes (host, pure) ---------------------------------------------------- */

/* Bytes of the packed buffer for n codes of `bits` bits: 4*ceil(n*bits/32); 0 if bits is invalid.
 * (Sec. 3: q-bit quantization shrinks the fp32 tensor that crosses the stage boundary by 32/q, i.e. to
 * n q / 8 bytes; the buffer is that, rounded up to whole 32-bit words.) */
size_t qp_packed_bytes(uint64_t n, uint32_t bits);

/* Bytes of device workspace needed by qp_stats / qp_dsaciq_search for an n-element
 * tensor under cfg (NULL = defaults: t_steps 100, cands_per_round 13).  0 on bad arguments.
 * (Sec. 3, Eq. 1: what the statistics and the t+1 candidates of the directed search need between kernels:
 * per-block partial sums, the histogram D_R, the candidate grids and their scores; nothing per element.) */
size_t qp_workspace_bytes(uint64_t n, const qp_search_cfg_t *cfg);

/* Byte offset of a region inside the workspace; (size_t)-1 for an unknown region. */
size_t qp_ws_offset(qp_ws_region region);

/* Fills cfg with the defaults {100, 13, 2048, QP_LAPLACE, 0, 0}: the paper's method. */
void qp_default_search_cfg(qp_search_cfg_t *cfg);

/* ---- step 1: statistics (Sec. 3: mu and b of L(mu, b); b_E; histogram D_R; b_R) ----
 * Two passes over x_dev (the mean must be known before |x - mu|, and min/max before
 * the histogram).  fp64 accumulation, deterministic reduction order.  nbins in [16, 4096].
 * qp_stats copies the result to *out_host and returns QP_ENONFINITE if NaN/Inf was seen.
 * qp_stats_async leaves it at QP_WS_STATS (and the histogram at QP_WS_HIST). */
qp_status qp_stats(const void *x_dev, uint64_t n, qp_dtype dtype, uint32_t nbins,
                   void *ws_dev, size_t ws_bytes, void *stream, qp_stats_t *out_host);
qp_status qp_stats_async(const void *x_dev, uint64_t n, qp_dtype dtype, uint32_t nbins,
                         void *ws_dev, size_t ws_bytes, void *stream);

/* ---- step 2a: ACIQ threshold (Sec. 3: alpha = F(q) * b) -- host only, pure ----
 * Laplace: alpha = W0(3 * 4^bits) * stats->mad, W0 the principal Lambert W (the
 * stationary point of ACIQ's clipping + rounding noise model).  Gaussian:
 * alpha = G(bits) * sqrt(stats->var) with G from the matching Gaussian noise model.
 * QP_DIST_AUTO is not accepted here (QP_EINVAL): the choice needs the histogram, which the host does not hold. */
qp_status qp_aciq_alpha(const qp_stats_t *stats, uint32_t bits, qp_dist dist, double *alpha_out);

/* The constant alone: F(bits) for QP_LAPLACE, G(bits) for QP_GAUSS; NaN on bad arguments. */
double qp_aciq_constant(uint32_t bits, qp_dist dist);

/* Quantization grid for the range [center - alpha, center + alpha] with 2^bits levels,
 * both end points representable ("equal intervals for rounding", Sec. 3).  Host only, pure.
 * Naive PTQ (Sec. 3) is center = (min+max)/2, alpha = (max-min)/2. */
qp_status qp_make_qparams(double center, double alpha, uint32_t bits, uint64_t n, qp_qparams_t *out);

/* The same grid for the range intersected with the data's own range (rounded to fp32):
 * [max(center - alpha, data_min), min(center + alpha, data_max)]; scale 0 if that is empty.
 * This is the winner's grid of a search run with QP_SEARCH_CLIP_TO_DATA.  Host only, pure. */
qp_status qp_make_qparams_clipped(double center, double alpha, double data_min, double data_max, uint32_t bits,
                                  uint64_t n, qp_qparams_t *out);

/* ---- step 2b: DS-ACIQ directed search (Sec. 3, Eq. 1) -------------------------
 * Candidates b_j = b_E + j (b_R - b_E) / t, j = 0..t, with b_E = stats->mad and
 * b_R = stats->b_r, whichever way that points.  Each is scored by the squared
 * quantization error on the real tensor, sum_i (x_i - dequant(quant(x_i)))^2, with
 * alpha_j = F(q) b_j centred on stats->mean, using exactly the arithmetic of
 * qp_quant_pack / qp_unpack_dequant (fp32 per element, fp64 sums).  The lowest score
 * wins, ties go to the smallest j, so b_E is kept unless something is strictly better.
 * A bound that is zero, negative or not finite collapses the grid onto b_E (j* = 0).
 * A large tensor is read once per round of at most cfg->cands_per_round candidates.
 * qp_dsaciq_search returns the result and the winner's grid to the host (either may be
 * NULL); the async form takes the statistics that qp_stats_async left in the same
 * workspace and leaves QP_WS_RESULT / QP_WS_QPARAMS / QP_WS_SCORES there.
 * With cfg->dist = QP_GAUSS the grid runs from sqrt(stats->var) to
 * 1 / (sqrt(2 pi) stats->peak_density) and alpha_j = G(q) sigma_j (b_e, b_r, b_star of the
 * result then hold sigmas); cfg->flags are described at qp_search_cfg_t. */
qp_status qp_dsaciq_search(const void *x_dev, uint64_t n, qp_dtype dtype, const qp_stats_t *stats,
                           uint32_t bits, const qp_search_cfg_t *cfg, void *ws_dev, size_t ws_bytes,
                           void *stream, qp_search_result_t *res_host, qp_qparams_t *qparams_out_host);
qp_status qp_dsaciq_search_async(const void *x_dev, uint64_t n, qp_dtype dtype, uint32_t bits,
                                 const qp_search_cfg_t *cfg, void *ws_dev, size_t ws_bytes, void *stream);

/* ---- which model fits the tensor (beyond the paper, which assumes Laplace: Sec. 3) ----------
 * The measure is Eq. 1's own, the squared distance between the real distribution D_R (the histogram as a
 * density at the bin centres c_i, D_R,i = count_i / (N binwidth)) and the estimated one at its moment estimates:
 *     fit_laplace = sum_i (D_R,i - exp(-|c_i - mu| / b_E) / (2 b_E))^2,                        b_E = mad,
 *     fit_gauss   = sum_i (D_R,i - exp(-(c_i - mu)^2 / (2 sigma^2)) / (sigma sqrt(2 pi)))^2,   sigma = sqrt(var).
 * dist = QP_GAUSS only if fit_gauss < fit_laplace (a fit that is not a number never wins, so degenerate tensors
 * keep the paper's model).  Works on the record and histogram that qp_stats / qp_stats_async left in ws_dev (no
 * pass over the tensor; a record that is not one gives NaN fits and QP_LAPLACE) and leaves the result at
 * QP_WS_MODEL, where a search with cfg->dist = QP_DIST_AUTO leaves its own. */
typedef struct {
    double   fit_laplace, fit_gauss;
    uint32_t dist;             /* QP_LAPLACE or QP_GAUSS */
    uint32_t reserved;         /* written as 0 */
} qp_model_fit_t;
qp_status qp_model_fit(void *ws_dev, size_t ws_bytes, void *stream, qp_model_fit_t *out_host);
qp_status qp_model_fit_async(void *ws_dev, size_t ws_bytes, void *stream);

/* ---- step 2b, the other reading of Eq. 1: fit the estimated distribution to the histogram ----
 * Eq. 1 as printed minimises MSE(D_R, D_E) between the real distribution D_R (the histogram of
 * the tensor, as a density) and the estimated one D_E (the Laplace pdf with scale b) over
 * b in [b_E, b_R].  Same candidate grid and first-minimum rule as qp_dsaciq_search; the score
 * of candidate j is sum over bins of (D_R,i - exp(-|c_i - mu| / b_j) / (2 b_j))^2 with c_i the
 * bin centre and D_R,i = count_i / (N binwidth); mse_aciq / mse_star are means over the bins.
 * Works on the statistics record and histogram that qp_stats / qp_stats_async left in ws_dev
 * (no pass over the tensor) and overwrites QP_WS_RESULT / QP_WS_QPARAMS / QP_WS_SCORES.  The statistics
 * must have run on the same workspace first (they also clear the ticket that tells the last block to write the
 * result).  A record whose nbins is outside [16, 4096] or whose n is 0 (a workspace the statistics never wrote)
 * gives NaN scores, and nothing is read out of bounds; the result record is then not meaningful.
 * Only the paper's form: cfg->dist must be QP_LAPLACE and cfg->flags 0 (else QP_EINVAL). */
qp_status qp_dsaciq_hist_search(uint32_t bits, const qp_search_cfg_t *cfg, void *ws_dev, size_t ws_bytes,
                                void *stream, qp_search_result_t *res_host, qp_qparams_t *qparams_out_host);
qp_status qp_dsaciq_hist_search_async(uint32_t bits, const qp_search_cfg_t *cfg, void *ws_dev, size_t ws_bytes,
                                      void *stream);

/* ---- step 3: clip + uniform quantize + bit-pack (Sec. 3: ACIQ clipping, then PTQ) ----
 * c_i = rne((min(max(x_i, lo), hi) - lo) * inv_scale) clamped to [0, 2^bits - 1]
 * (fp32: one subtraction, one product, round half to even; NaN -> code 0), written in
 * the wire format above.  Asynchronous on `stream`.  packed_bytes is the capacity of
 * packed_dev (>= qp_packed_bytes(n, bits), else QP_ENOSPC).
 * The _dev form reads the qp_qparams_t from device memory (e.g. QP_WS_QPARAMS) and
 * needs the bitwidth on the host to choose the kernel; the record's n and bits must match. */
qp_status qp_quant_pack(const void *x_dev, uint64_t n, qp_dtype dtype, const qp_qparams_t *qparams,
                        void *packed_dev, size_t packed_bytes, void *stream);
qp_status qp_quant_pack_dev(const void *x_dev, uint64_t n, qp_dtype dtype, uint32_t bits,
                            const qp_qparams_t *qparams_dev, void *packed_dev, size_t packed_bytes,
                            void *stream);

/* ---- step 4: unpack + dequantize (the receiving stage consumes fp32 again) ----
 * y_i = fma((float)c_i, scale, lo): lo + c*scale rounded once to fp32.  Asynchronous.
 * n must equal qparams->n; packed_bytes >= qp_packed_bytes(n, bits). */
qp_status qp_unpack_dequant(const void *packed_dev, size_t packed_bytes, const qp_qparams_t *qparams,
                            float *y_dev, uint64_t n, void *stream);
qp_status qp_unpack_dequant_dev(const void *packed_dev, size_t packed_bytes, uint32_t bits,
                                const qp_qparams_t *qparams_dev, float *y_dev, uint64_t n, void *stream);

/* ---- whole sender side without a host round trip ------------------------------
 * stats -> directed search -> quantize + pack, all on `stream`, nothing copied to the
 * host.  If qparams_out_dev is not NULL the winner's record is also copied there
 * (device to device) so that it can travel with the payload.  The statistics, the
 * search result and the scores are left in the workspace regions as by the separate
 * calls; nothing is reported about NaN / Inf elements here (QP_WS_STATS holds their
 * count; such elements are packed as code 0).
 * All state of a call lives in its workspace, so tensors that do not depend on each other
 * (microbatches, stage boundaries) may be in flight together, each call with a workspace of
 * its own on a stream of its own (default priority).  That pays on gfx950: the statistics,
 * pack and unpack kernels are bound by HBM and the search by vector ALU work, and three
 * streams finish six ViT-Base tensors in the time one stream needs for five. */
qp_status qp_compress_async(const void *x_dev, uint64_t n, qp_dtype dtype, uint32_t bits,
                            const qp_search_cfg_t *cfg, void *ws_dev, size_t ws_bytes,
                            void *packed_dev, size_t packed_bytes, qp_qparams_t *qparams_out_dev,
                            void *stream);

/* ---- several tensors in flight --------------------------------------------------
 * The tensors that cross stage boundaries (Sec. 3: one activation tensor per microbatch and
 * boundary) do not depend on each other, so their sender paths may overlap.  Job i runs as
 * qp_compress_async on lane i mod n_lanes, i.e. on that lane's stream with that lane's workspace;
 * jobs of one lane follow each other in stream order, lanes run side by side.  On gfx950 three
 * lanes hide the HBM-bound statistics and pack kernels of one tensor behind the ALU-bound search
 * of another.  Every argument of every job is checked before the first kernel is launched (the
 * errors are those of qp_compress_async; also QP_EINVAL if two lanes' workspaces overlap, if
 * n_lanes is 0 or above 64, or if qparams_out_dev is NULL for a job whose lane a later job of the
 * same call reuses: that later job overwrites the lane's records, so the grid must leave the
 * workspace with the payload).  A lane's workspace holds the records of its last job afterwards.
 * Streams are the caller's (default priority; two lanes may name the same stream and then run in
 * order); the library creates none and allocates nothing.  A HIP error part of the way leaves the
 * earlier jobs enqueued. */
typedef struct {
    const void   *x_dev;            /* n elements of dtype, 16-byte aligned */
    uint64_t      n;
    uint32_t      dtype;            /* qp_dtype */
    uint32_t      bits;
    void         *packed_dev;       /* 16-byte aligned */
    uint64_t      packed_bytes;     /* >= qp_packed_bytes(n, bits) */
    qp_qparams_t *qparams_out_dev;  /* 32 bytes of device memory, or NULL (see above) */
} qp_job_t;
typedef struct {
    void  *ws_dev;                  /* >= qp_workspace_bytes(n, cfg) for every job of the lane */
    size_t ws_bytes;
    void  *stream;                  /* hipStream_t */
} qp_lane_t;
qp_status qp_compress_many_async(const qp_job_t *jobs, uint32_t count, const qp_search_cfg_t *cfg,
                                 const qp_lane_t *lanes, uint32_t n_lanes);

/* ---- the same sender path for callers that cannot allocate -----------------------
 * For code under HIP graph capture, tight serving loops and harnesses that forbid hipMalloc: the
 * callers that cannot bring a workspace.  Same kernels and same results as qp_compress_async, with
 * the workspace in a static device array inside the library (1,384,960 bytes per GPU, held until
 * the process ends; its device address is looked up on the first call on each device, so a caller
 * that captures into a HIP graph makes one call outside the capture first).  Calls no allocating routine.  The caller still owns x_dev, packed_dev and qparams_out_dev (required:
 * 32 bytes of device memory that receive the winner's qp_qparams_t; the statistics and the search
 * result stay inside the library).  Limits: cfg->t_steps <= 127 (QP_ENOSPC beyond; NULL cfg =
 * the paper's 100), any n the other calls take.  Every call on a GPU uses that GPU's one array:
 * calls that overlap on one GPU (two streams, two threads) race; calls on one stream are safe
 * back to back, and nothing in the array needs clearing between them. */
qp_status qp_compress_noalloc(const void *x_dev, uint64_t n, qp_dtype dtype, uint32_t bits,
                              const qp_search_cfg_t *cfg, void *packed_dev, size_t packed_bytes,
                              qp_qparams_t *qparams_out_dev, void *stream);

/* ---- adaptive bitwidth rule (Sec. 3 "Adaptive PDA", Eq. 2) -- host only, pure ---------
 * Given the payload size V at the current bitwidth, the microbatch size S (images), the target
 * rate R (images/s) and the measured bandwidth B, the next bitwidth is
 *     q_next = 32 / 2^ceil(log2( (V * 32 / q_cur) / (S / R * B) )),
 * i.e. the uncompressed size V*32/q_cur is halved until it fits in what the link carries
 * during one microbatch period S/R.  v_bits is V in bits, bandwidth in bits per second.
 * Results: 32 (send unquantized: the link is not the bottleneck), 16, 8, 4 or 2 (the lowest
 * supported; also when even 2 bits do not fit).  q_cur may be any of 2,3,4,6,8,16,32.
 * bandwidth = +infinity is allowed and gives 32.  QP_EINVAL on non-positive or NaN arguments. */
qp_status qp_next_bits(double v_bits, uint32_t q_cur, double s_images, double r_images_per_s,
                       double bandwidth_bits_per_s, uint32_t *q_next);

/* ---- adaptive PDA controller: window averages feeding Eq. 2 (Sec. 3, Sec. 4.2) -- host only ----
 * The paper's runtime measures over a window of microbatches (50 in its run) and decides when the
 * window expires, from the window's averages.  The caller reports every microbatch it has sent
 * (payload bits at the bitwidth in force, and the time the link took); when `window` of them have
 * been reported the bandwidth B = sum(bits) / sum(seconds) and the mean payload V go into
 * qp_next_bits, and its answer is the bitwidth from then on.  Between expiries nothing changes.
 * The record is plain data owned by the caller (one per stage boundary); no allocation. */
typedef struct {
    uint32_t window;           /* microbatches per decision */
    uint32_t count;            /* microbatches reported in the current window */
    double   bits_sum;         /* payload bits in the current window */
    double   seconds_sum;      /* time the link took for them */
    double   s_images;         /* S: images per microbatch */
    double   r_images_per_s;   /* R: target rate */
    uint32_t q_cur;            /* bitwidth in force: 2,3,4,6,8,16, or 32 = send unquantized */
    uint32_t decisions;        /* windows that have expired */
} qp_controller_t;

/* QP_EINVAL on window == 0, non-positive S or R, or a q_start that is not a bitwidth or 32. */
qp_status qp_controller_init(qp_controller_t *c, uint32_t window, double s_images, double r_images_per_s,
                             uint32_t q_start);
/* One microbatch has been sent; *q_next receives the bitwidth for the next one.
 * QP_EINVAL on null pointers or non-positive / NaN payload_bits or seconds (the record is unchanged). */
qp_status qp_controller_update(qp_controller_t *c, double payload_bits, double seconds, uint32_t *q_next);

const char *qp_strerror(qp_status status);

#ifdef __cplusplus
}
#endif
#endif /* QUANTPIPE_H */
