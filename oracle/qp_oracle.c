/*
 * CPU oracle for the activation-compression path of QuantPipe
 * (statistics -> ACIQ clipping -> DS-ACIQ directed search -> clip + uniform
 * quantize + bit-pack -> unpack + dequantize).
 *
 * THIS IS TEST INFRASTRUCTURE, NOT THE PRODUCT.  It is a plain, slow, sequential
 * statement of what the path computes, written from the paper so that the HIP
 * library can be compared with it element by element.  It shares no code,
 * header, table or constant with the HIP library, and only the tests, the smoke
 * check and the benchmark's CPU-baseline leg may call it.
 *
 * Arithmetic: every reduction is a sequential fp64 sum in index order.  The
 * per-element quantization arithmetic is fp32 in a fixed operation order (so
 * that integer codes are well defined); build with -ffp-contract=off so that
 * no multiply-add is fused except where fmaf() is written.
 *
 * Pins (see the CPU tests): statistics against closed forms and numpy; the
 * histogram against numpy.histogram on dyadic data; the Laplace constant
 * against scipy's Lambert W, a brute-force minimum of the noise model and the
 * 2/3/4-bit constants printed in the ACIQ paper the method cites; the Gaussian
 * constant against a brute-force minimum of numerically integrated noise; the
 * search against an independent numpy sweep on tiny tensors; quantize against
 * invariants and the 8-bit identity; pack/unpack against numpy.packbits and
 * uint8/uint16 views; dequantize against the fp64 definition; the search variants
 * (Gaussian model, range intersected with the data's, coarse-to-fine sweep) against
 * the paper's search at their defaults, an independent numpy sweep, a hand-worked
 * grid, an exact normal histogram, and (the sweep's index logic) the plain argmin of
 * unimodal curves.
 */
#include <math.h>
#include <stddef.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

/* ---- plain-data records (the oracle's own; the Python side mirrors them) ---- */

typedef struct {
    uint64_t n;            /* element count */
    uint64_t n_nonfinite;  /* NaN or +-Inf elements */
    double mean;           /* mu = (1/N) sum x */
    double mad;            /* (1/N) sum |x - mu|   : the Laplace scale b_E */
    double abs_mean;       /* (1/N) sum |x|        : the paper's literal b_E formula */
    double var;            /* (1/N) sum (x - mu)^2 : population variance */
    double min;
    double max;
    uint32_t nbins;
    uint32_t peak_count;   /* largest histogram count */
    double peak_density;   /* peak_count / (N * bin width) */
    double b_r;            /* 1 / (2 * peak_density) */
} orc_stats_t;

typedef struct {
    uint32_t bits;
    uint32_t levels;       /* L = 2^bits - 1 */
    uint64_t n;
    float lo, hi, scale, inv_scale;
} orc_qparams_t;

typedef struct {
    double b_e, b_r, b_star, alpha_star, mse_aciq, mse_star;
    uint32_t j_star;
    uint32_t t_steps;
} orc_search_result_t;

enum { ORC_LAPLACE = 0, ORC_GAUSS = 1 };

static int orc_bits_ok(uint32_t bits)
{
    return bits == 2 || bits == 3 || bits == 4 || bits == 6 || bits == 8 || bits == 16;
}

/* ---- bf16 -> fp32: exact widening (the 16 bits become the top half) ---- */

void orc_widen_bf16(const uint16_t *h, uint64_t n, float *out)
{
    for (uint64_t i = 0; i < n; ++i) {
        uint32_t u = (uint32_t)h[i] << 16;
        memcpy(&out[i], &u, 4);
    }
}

/* ---- Step 1: statistics and histogram (Sec. 3: L(mu, b); b_E; D_R; b_R) ----
 *
 * mu and b_E: the activation is modelled as Laplace L(mu, b) (Sec. 3, ACIQ
 * paragraph); b is its mean absolute deviation about mu.  The paper's printed
 * estimate sum|X|/N (Sec. 3, Directed Search) is abs_mean; they agree at mu=0.
 * D_R: nbins equal-width bins over [min, max]; bin index in fp32.
 * b_R = 1 / (2 max(D_R)) with D_R as a density (Sec. 3, after Eq. 1): the
 * Laplace pdf peaks at 1/(2b).
 * Returns 0, or 1 if any element is NaN/Inf (then the other fields are not
 * meaningful).  hist may be NULL.
 */
int orc_stats(const float *x, uint64_t n, uint32_t nbins, orc_stats_t *out, uint32_t *hist)
{
    memset(out, 0, sizeof *out);
    out->n = n;
    out->nbins = nbins;
    if (n == 0 || nbins == 0) return 2;

    double sum = 0.0, sum_abs = 0.0;
    float mn = INFINITY, mx = -INFINITY;
    uint64_t bad = 0;
    for (uint64_t i = 0; i < n; ++i) {
        float v = x[i];
        if (!isfinite(v)) { ++bad; continue; }
        sum += (double)v;
        sum_abs += fabs((double)v);
        if (v < mn) mn = v;
        if (v > mx) mx = v;
    }
    out->n_nonfinite = bad;
    if (bad) return 1;

    double mean = sum / (double)n;
    double dev = 0.0, sq = 0.0;
    for (uint64_t i = 0; i < n; ++i) {
        double d = (double)x[i] - mean;
        dev += fabs(d);
        sq += d * d;
    }
    out->mean = mean;
    out->abs_mean = sum_abs / (double)n;
    out->mad = dev / (double)n;
    out->var = sq / (double)n;
    out->min = (double)mn;
    out->max = (double)mx;

    uint32_t peak = 0;
    if (mx == mn) {
        /* one distinct value: everything sits in bin 0 and the density peak is unbounded */
        if (hist) { memset(hist, 0, (size_t)nbins * 4); hist[0] = (uint32_t)n; }
        out->peak_count = (uint32_t)n;
        out->peak_density = 0.0;
        out->b_r = 0.0;
        return 0;
    }
    /* fp32: one subtraction, one division, then per element one subtraction and one product */
    float range = mx - mn;
    float w_inv = (float)nbins / range;
    uint32_t *h = hist;
    uint32_t local[4096];
    if (!h) { if (nbins > 4096) return 2; h = local; }
    memset(h, 0, (size_t)nbins * 4);
    for (uint64_t i = 0; i < n; ++i) {
        float t = (x[i] - mn) * w_inv;
        uint32_t idx;
        if (!(t >= 0.0f)) idx = 0;                       /* also NaN (0 * inf) */
        else if (t >= (float)nbins) idx = nbins - 1;     /* x == max, or overflow */
        else idx = (uint32_t)t;                          /* truncation == floor for t >= 0 */
        ++h[idx];
    }
    for (uint32_t b = 0; b < nbins; ++b)
        if (h[b] > peak) peak = h[b];
    out->peak_count = peak;
    double binw = ((double)mx - (double)mn) / (double)nbins;
    out->peak_density = (double)peak / ((double)n * binw);
    out->b_r = 1.0 / (2.0 * out->peak_density);
    return 0;
}

/* ---- Step 2a: the ACIQ constants -------------------------------------------
 *
 * Laplace (the paper's model, Sec. 3: alpha = F(q) b).  The ACIQ noise model for
 * unit scale is clipping noise 2 e^{-a} plus rounding noise a^2 / (3 4^q); its
 * stationary point satisfies a e^a = 3 4^q, so F(q) = W0(3 4^q), W0 the
 * principal Lambert W.
 */
double orc_lambert_w0(double z)
{
    if (!(z >= 0.0)) return NAN;
    if (z == 0.0) return 0.0;
    double w = (z < 3.0) ? z / (1.0 + z) * 1.2 : log(z) - log(log(z));
    for (int it = 0; it < 100; ++it) {
        double ew = exp(w);
        double f = w * ew - z;
        /* Halley step for f(w) = w e^w - z */
        double denom = ew * (w + 1.0) - (w + 2.0) * f / (2.0 * w + 2.0);
        double wn = w - f / denom;
        if (fabs(wn - w) <= 1e-16 * fabs(wn)) { w = wn; break; }
        w = wn;
    }
    return w;
}

double orc_laplace_F(uint32_t bits)
{
    return orc_lambert_w0(3.0 * pow(4.0, (double)bits));
}

/* Gaussian variant: for unit sigma the clipping noise is
 * 2[(1+a^2) Q(a) - a phi(a)] and the rounding noise a^2/(3 4^q); the stationary
 * point satisfies phi(a) - a Q(a) = a / (6 4^q).  Solved by bisection. */
double orc_gauss_G(uint32_t bits)
{
    const double inv_sqrt_2pi = 0.39894228040143267794;
    double rhs_coef = 1.0 / (6.0 * pow(4.0, (double)bits));
    double lo = 0.0, hi = 40.0;
    for (int it = 0; it < 200; ++it) {
        double a = 0.5 * (lo + hi);
        double phi = inv_sqrt_2pi * exp(-0.5 * a * a);
        double q = 0.5 * erfc(a / sqrt(2.0));
        double f = phi - a * q - a * rhs_coef;   /* decreasing in a */
        if (f > 0.0) lo = a; else hi = a;
    }
    return 0.5 * (lo + hi);
}

/* alpha = F(q) * b_E (Laplace) or G(q) * sigma (Gaussian). */
int orc_aciq_alpha(const orc_stats_t *st, uint32_t bits, int dist, double *alpha)
{
    if (!orc_bits_ok(bits)) return 2;
    if (dist == ORC_LAPLACE) *alpha = orc_laplace_F(bits) * st->mad;
    else if (dist == ORC_GAUSS) *alpha = orc_gauss_G(bits) * sqrt(st->var);
    else return 2;
    return 0;
}

/* ---- quantization grid: [center - alpha, center + alpha], 2^k levels with the
 * two end points representable ("equal intervals", Sec. 3) ---- */
int orc_make_qparams(double center, double alpha, uint32_t bits, uint64_t n, orc_qparams_t *q)
{
    if (!orc_bits_ok(bits)) return 2;
    float a32 = (float)alpha;
    float c32 = (float)center;
    q->bits = bits;
    q->levels = (1u << bits) - 1u;
    q->n = n;
    q->lo = (float)((double)c32 - (double)a32);
    q->hi = (float)((double)c32 + (double)a32);
    double range = (double)q->hi - (double)q->lo;
    if (q->hi == q->lo) {
        q->scale = 0.0f;
        q->inv_scale = 0.0f;
    } else {
        q->scale = (float)(range / (double)q->levels);
        q->inv_scale = (float)((double)q->levels / range);
    }
    return 0;
}

/* ---- Step 3: clip + uniform quantize (Sec. 3: clamp outliers, equal intervals) ---- */
uint32_t orc_quant_one(float x, const orc_qparams_t *q)
{
    float xc = fminf(fmaxf(x, q->lo), q->hi);     /* NaN -> lo */
    float d = xc - q->lo;                         /* fp32 subtraction */
    float t = d * q->inv_scale;                   /* fp32 product, not fused */
    float r = rintf(t);                           /* round half to even */
    float L = (float)q->levels;
    if (!(r >= 0.0f)) r = 0.0f;
    if (r > L) r = L;
    return (uint32_t)r;
}

/* ---- Step 4: dequantize: lo + c*scale rounded once to fp32 ---- */
float orc_dequant_one(uint32_t c, const orc_qparams_t *q)
{
    return fmaf((float)c, q->scale, q->lo);
}

void orc_quantize(const float *x, uint64_t n, const orc_qparams_t *q, uint32_t *codes)
{
    for (uint64_t i = 0; i < n; ++i) codes[i] = orc_quant_one(x[i], q);
}

void orc_dequantize(const uint32_t *codes, uint64_t n, const orc_qparams_t *q, float *y)
{
    for (uint64_t i = 0; i < n; ++i) y[i] = orc_dequant_one(codes[i], q);
}

/* ---- wire format: code i occupies stream bits [i k, i k + k), least significant
 * bit first; stream bit p is bit (p mod 8) of byte (p div 8); the length is a
 * whole number of 32-bit words and unused tail bits are zero. ---- */
uint64_t orc_packed_bytes(uint64_t n, uint32_t bits)
{
    if (!orc_bits_ok(bits)) return 0;
    return 4u * ((n * (uint64_t)bits + 31u) / 32u);
}

int orc_pack(const uint32_t *codes, uint64_t n, uint32_t bits, uint8_t *out, uint64_t out_bytes)
{
    uint64_t need = orc_packed_bytes(n, bits);
    if (need == 0 || out_bytes < need) return 2;
    memset(out, 0, need);
    for (uint64_t i = 0; i < n; ++i)
        for (uint32_t b = 0; b < bits; ++b)
            if ((codes[i] >> b) & 1u) {
                uint64_t p = i * bits + b;
                out[p >> 3] |= (uint8_t)(1u << (p & 7u));
            }
    return 0;
}

int orc_unpack(const uint8_t *in, uint64_t n, uint32_t bits, uint32_t *codes)
{
    if (!orc_bits_ok(bits)) return 2;
    for (uint64_t i = 0; i < n; ++i) {
        uint32_t c = 0;
        for (uint32_t b = 0; b < bits; ++b) {
            uint64_t p = i * bits + b;
            c |= (uint32_t)((in[p >> 3] >> (p & 7u)) & 1u) << b;
        }
        codes[i] = c;
    }
    return 0;
}

/* sum over the tensor of (x - dequant(quant(x)))^2: fp32 error, fp64 square and sum */
double orc_sq_error(const float *x, uint64_t n, const orc_qparams_t *q)
{
    double s = 0.0;
    for (uint64_t i = 0; i < n; ++i) {
        float xh = orc_dequant_one(orc_quant_one(x[i], q), q);
        float e = x[i] - xh;
        s += (double)e * (double)e;
    }
    return s;
}

/* ---- Step 2b: DS-ACIQ directed search (Sec. 3, Eq. 1) -----------------------
 *
 * Candidates b_j = b_E + j (b_R - b_E)/t, j = 0..t, walk from the ACIQ estimate
 * towards the bound given by the real peak, in whichever direction that is.
 * Each is scored by the quantization error on the real tensor with
 * alpha_j = F(q) b_j and the grid centred on mu.  The lowest score wins and ties
 * go to the smallest j, so b_E is kept unless something is strictly better.
 * A bound that is zero, negative or not finite (or b_E <= 0) collapses the grid
 * onto b_E.  scores (t+1 doubles) receives the sums of squared errors.
 */
/* The scale grid of Eq. 1: b_j = b_e + j step (the loop below and orc_search_candidate use it). */
static void orc_search_grid(const orc_stats_t *st, uint32_t t_steps, double *b_e, double *b_r, double *step)
{
    *b_e = st->mad;
    *b_r = st->b_r;
    *step = (*b_r - *b_e) / (double)t_steps;
    if (!(*b_e > 0.0) || !(*b_r > 0.0) || !isfinite(*b_r) || !isfinite(*b_e) || !isfinite(*step))
        *step = 0.0;
}

/* The quantization grid of candidate j alone (alpha_j = F(q) b_j, centred on mu): lets a test harness
 * score the candidates of one search separately (orc_sq_error on each), e.g. on several host threads. */
int orc_search_candidate(const orc_stats_t *st, uint32_t bits, uint32_t t_steps, uint64_t n, uint32_t j,
                         orc_qparams_t *q)
{
    if (!orc_bits_ok(bits) || t_steps == 0 || n == 0 || j > t_steps) return 2;
    double b_e, b_r, step;
    orc_search_grid(st, t_steps, &b_e, &b_r, &step);
    double b_j = b_e + (double)j * step;
    double alpha = orc_laplace_F(bits) * b_j;
    return orc_make_qparams(st->mean, alpha, bits, n, q);
}

/* The search's decision from the t+1 scores: the lowest wins, ties go to the smallest j. */
int orc_search_pick(const orc_stats_t *st, uint32_t bits, uint32_t t_steps, uint64_t n, const double *scores,
                    orc_search_result_t *res, orc_qparams_t *best_q)
{
    if (!orc_bits_ok(bits) || t_steps == 0 || n == 0) return 2;
    double F = orc_laplace_F(bits);
    double b_e, b_r, step;
    orc_search_grid(st, t_steps, &b_e, &b_r, &step);
    uint32_t best_j = 0;
    double best = 0.0, first = 0.0;
    for (uint32_t j = 0; j <= t_steps; ++j) {
        double s = scores[j];
        if (j == 0) first = s;
        if (j == 0 || s < best) { best = s; best_j = j; }
    }
    double b_star = b_e + (double)best_j * step;
    res->b_e = b_e;
    res->b_r = b_r;
    res->b_star = b_star;
    res->alpha_star = F * b_star;
    res->j_star = best_j;
    res->t_steps = t_steps;
    res->mse_aciq = first / (double)n;   /* j = 0 is plain ACIQ */
    res->mse_star = best / (double)n;
    if (best_q) orc_make_qparams(st->mean, res->alpha_star, bits, n, best_q);
    return 0;
}

int orc_dsaciq_search(const float *x, uint64_t n, const orc_stats_t *st, uint32_t bits,
                      uint32_t t_steps, orc_search_result_t *res, orc_qparams_t *best_q,
                      double *scores)
{
    if (!orc_bits_ok(bits) || t_steps == 0 || n == 0) return 2;
    double *sc = scores ? scores : (double *)malloc(((size_t)t_steps + 1) * sizeof(double));
    if (!sc) return 2;
    for (uint32_t j = 0; j <= t_steps; ++j) {
        orc_qparams_t q;
        orc_search_candidate(st, bits, t_steps, n, j, &q);
        sc[j] = orc_sq_error(x, n, &q);
    }
    int rc = orc_search_pick(st, bits, t_steps, n, sc, res, best_q);
    if (!scores) free(sc);
    return rc;
}

/* ---- Adaptive PDA bitwidth rule (Sec. 3, Eq. 2) -----------------------------
 * q_next = 32 / 2^ceil(log2((V 32/q_cur) / (S/R B))), written as printed, with the two
 * clamps the text implies: no quantization (32) when the link is not the bottleneck, and
 * 2 bits as the lowest bitwidth the system has.  V and B in bits and bits per second.
 * Pinned by the paper's own run (Sec. 4.2): ViT-Base boundary tensor, microbatch 64,
 * about 100 images/s: 400 Mbps -> 16 bit, 50 Mbps -> 2 bit, 200 Mbps -> 8 bit, unlimited -> 32. */
int orc_next_bits(double v_bits, uint32_t q_cur, double s_images, double r_rate, double bandwidth, uint32_t *q_next)
{
    if (!(v_bits > 0.0) || !(s_images > 0.0) || !(r_rate > 0.0) || !(bandwidth > 0.0) || q_cur == 0) return 2;
    double ratio = (v_bits * 32.0 / (double)q_cur) / (s_images / r_rate * bandwidth);
    double e = ceil(log2(ratio));
    if (e < 0.0) e = 0.0;
    if (e > 4.0) e = 4.0;
    *q_next = 32u >> (uint32_t)e;
    return 0;
}

/* ---- DS-ACIQ, the other reading of Eq. 1: fit the Laplace pdf to the histogram -------
 *
 * Eq. 1 literally minimises MSE(D_R, D_E) between the real distribution D_R (the histogram,
 * as a density) and the estimated one D_E (the Laplace pdf with scale b) over b in
 * [b_E, b_R].  Same candidate grid and first-minimum rule as the tensor-error search;
 * the score of candidate j is the sum over bins of (D_R,i - pdf(c_i; mu, b_j))^2 with
 * c_i the bin centre, D_R,i = count_i / (N binwidth), pdf = exp(-|c - mu| / b) / (2 b).
 * mse_* are the means over the bins.  No pass over the tensor.
 */
int orc_hist_search(const orc_stats_t *st, const uint32_t *hist, uint32_t bits, uint32_t t_steps,
                    orc_search_result_t *res, orc_qparams_t *best_q, double *scores)
{
    if (!orc_bits_ok(bits) || t_steps == 0 || st->n == 0 || st->nbins == 0) return 2;
    const uint32_t B = st->nbins;
    double F = orc_laplace_F(bits);
    double b_e = st->mad, b_r = st->b_r;
    double step = (b_r - b_e) / (double)t_steps;
    if (!(b_e > 0.0) || !(b_r > 0.0) || !isfinite(b_r) || !isfinite(b_e) || !isfinite(step))
        step = 0.0;
    double binw = (st->max - st->min) / (double)B;
    uint32_t best_j = 0;
    double best = 0.0, first = 0.0;
    for (uint32_t j = 0; j <= t_steps; ++j) {
        double b_j = b_e + (double)j * step;
        double s = 0.0;
        for (uint32_t i = 0; i < B; ++i) {
            double c = st->min + ((double)i + 0.5) * binw;
            double d_r = (double)hist[i] / ((double)st->n * binw);
            double d_e = exp(-fabs(c - st->mean) / b_j) / (2.0 * b_j);
            double diff = d_r - d_e;
            s += diff * diff;
        }
        if (scores) scores[j] = s;
        if (j == 0) first = s;
        if (j == 0 || s < best) { best = s; best_j = j; }
    }
    double b_star = b_e + (double)best_j * step;
    res->b_e = b_e;
    res->b_r = b_r;
    res->b_star = b_star;
    res->alpha_star = F * b_star;
    res->j_star = best_j;
    res->t_steps = t_steps;
    res->mse_aciq = first / (double)B;
    res->mse_star = best / (double)B;
    if (best_q) orc_make_qparams(st->mean, res->alpha_star, bits, st->n, best_q);
    return 0;
}

/* ---- Variants of the directed search (beyond the paper's method) ----------------
 *
 * The paper models activations as Laplace and clips symmetrically about mu (Sec. 3).
 * Three variations on Eq. 1 that keep its structure (candidates on a straight grid of scale
 * values from the moment estimate to the bound given by the histogram peak, scored by the
 * quantization error on the real tensor, first minimum wins):
 *
 *   dist = ORC_GAUSS   the Gaussian model of the cited ACIQ method: scale estimate
 *                      sigma_E = sqrt(var), threshold alpha = G(q) sigma, and the bound is the
 *                      sigma whose density peak 1/(sigma sqrt(2 pi)) equals the histogram's:
 *                      sigma_R = 1 / (sqrt(2 pi) max D_R).
 *   clip_to_data       the clipping range is intersected with the data's own range,
 *                      [max(mu - alpha, min), min(mu + alpha, max)]: one-sided data (after a
 *                      GELU, say) then spends no levels below its minimum.
 *   stride > 1         coarse-to-fine sweep: first the candidates j = 0, s, 2s, ... and t; then all
 *                      candidates within s - 1 of the coarse winner j1.  The result is the first
 *                      minimum of the second sweep (which contains j1; no other coarse candidate
 *                      can beat or tie it at a smaller index).  On a curve that falls to its
 *                      minimum and rises after it this is the full sweep's answer with about
 *                      t/s + 2s evaluations instead of t + 1.  scores[] entries that were never
 *                      evaluated are NaN.
 * With dist = ORC_LAPLACE, clip_to_data = 0 and stride = 1 this is orc_dsaciq_search.
 */
int orc_make_qparams_clipped(double center, double alpha, double data_min, double data_max, uint32_t bits,
                             uint64_t n, orc_qparams_t *q)
{
    int rc = orc_make_qparams(center, alpha, bits, n, q);
    if (rc) return rc;
    float mn = (float)data_min, mx = (float)data_max;
    if (q->lo < mn) q->lo = mn;
    if (q->hi > mx) q->hi = mx;
    double range = (double)q->hi - (double)q->lo;
    if (!(q->hi > q->lo)) {
        q->scale = 0.0f;
        q->inv_scale = 0.0f;
    } else {
        q->scale = (float)(range / (double)q->levels);
        q->inv_scale = (float)((double)q->levels / range);
    }
    return 0;
}

/* a NaN score never wins a comparison: it counts as +infinity */
static double orc_key(double s) { return s == s ? s : INFINITY; }

/* which candidate a coarse-to-fine sweep picks if the full score table were `scores` (only the
 * entries the sweep would evaluate are read); evaluated[j] is set for those, if given */
uint32_t orc_c2f_pick(const double *scores, uint32_t t_steps, uint32_t stride, uint8_t *evaluated)
{
    if (evaluated) memset(evaluated, 0, (size_t)t_steps + 1);
    uint32_t j1 = 0;
    double best = 0.0;
    for (uint32_t i = 0;; ++i) {                      /* coarse sweep: 0, s, 2s, ..., t */
        uint64_t jj = (uint64_t)i * stride;
        uint32_t j = jj > t_steps ? t_steps : (uint32_t)jj;
        if (evaluated) evaluated[j] = 1;
        if (i == 0 || scores[j] < best) { best = orc_key(scores[j]); j1 = j; }
        if (j == t_steps) break;
    }
    uint32_t from = j1 >= stride - 1 ? j1 - (stride - 1) : 0;
    uint32_t to = (uint64_t)j1 + stride - 1 > t_steps ? t_steps : j1 + stride - 1;
    uint32_t j2 = from;
    for (uint32_t j = from; j <= to; ++j) {           /* fine sweep around the coarse winner */
        if (evaluated) evaluated[j] = 1;
        if (j == from || scores[j] < best) { best = orc_key(scores[j]); j2 = j; }
    }
    if (!(scores[0] == scores[0])) j2 = 0;             /* a NaN incumbent is never beaten */
    return j2;
}

int orc_dsaciq_search_variant(const float *x, uint64_t n, const orc_stats_t *st, uint32_t bits, uint32_t t_steps,
                              int dist, int clip_to_data, uint32_t stride, orc_search_result_t *res,
                              orc_qparams_t *best_q, double *scores /* t_steps + 1 */)
{
    if (!orc_bits_ok(bits) || t_steps == 0 || n == 0 || stride == 0 || !scores) return 2;
    double C, s_e, s_r;
    if (dist == ORC_LAPLACE) {
        C = orc_laplace_F(bits);
        s_e = st->mad;
        s_r = st->b_r;
    } else if (dist == ORC_GAUSS) {
        C = orc_gauss_G(bits);
        s_e = sqrt(st->var);
        s_r = 1.0 / (sqrt(2.0 * 3.14159265358979323846) * st->peak_density);
        if (st->peak_density == 0.0) s_r = 0.0;        /* one distinct value: same convention as b_R */
    } else {
        return 2;
    }
    double step = (s_r - s_e) / (double)t_steps;
    if (!(s_e > 0.0) || !(s_r > 0.0) || !isfinite(s_r) || !isfinite(s_e) || !isfinite(step)) step = 0.0;
    /* evaluate lazily: exactly the candidates the sweep asks for (NaN marks "not evaluated"; a score
     * that is really NaN is merely computed again) */
    for (uint32_t j = 0; j <= t_steps; ++j) scores[j] = NAN;
#define ORC_EVAL(j)                                                                                         \
    do {                                                                                                    \
        if (!(scores[(j)] == scores[(j)])) {                                                                \
            orc_qparams_t q_;                                                                               \
            double a_ = C * (s_e + (double)(j) * step);                                                     \
            if (clip_to_data) orc_make_qparams_clipped(st->mean, a_, st->min, st->max, bits, n, &q_);       \
            else orc_make_qparams(st->mean, a_, bits, n, &q_);                                              \
            scores[(j)] = orc_sq_error(x, n, &q_);                                                          \
        }                                                                                                   \
    } while (0)
    uint32_t j1 = 0, j_star;
    double best = 0.0;
    for (uint32_t i = 0;; ++i) {
        uint64_t jj = (uint64_t)i * stride;
        uint32_t j = jj > t_steps ? t_steps : (uint32_t)jj;
        ORC_EVAL(j);
        if (i == 0 || scores[j] < best) { best = orc_key(scores[j]); j1 = j; }
        if (j == t_steps) break;
    }
    j_star = j1;
    if (stride > 1) {
        uint32_t from = j1 >= stride - 1 ? j1 - (stride - 1) : 0;
        uint32_t to = (uint64_t)j1 + stride - 1 > t_steps ? t_steps : j1 + stride - 1;
        j_star = from;
        for (uint32_t j = from; j <= to; ++j) {
            ORC_EVAL(j);
            if (j == from || scores[j] < best) { best = orc_key(scores[j]); j_star = j; }
        }
    }
#undef ORC_EVAL
    if (!(scores[0] == scores[0])) j_star = 0;
    double s_star = s_e + (double)j_star * step;
    res->b_e = s_e;
    res->b_r = s_r;
    res->b_star = s_star;
    res->alpha_star = C * s_star;
    res->j_star = j_star;
    res->t_steps = t_steps;
    res->mse_aciq = scores[0] / (double)n;
    res->mse_star = scores[j_star] / (double)n;
    if (best_q) {
        if (clip_to_data) orc_make_qparams_clipped(st->mean, res->alpha_star, st->min, st->max, bits, n, best_q);
        else orc_make_qparams(st->mean, res->alpha_star, bits, n, best_q);
    }
    return 0;
}

/* ---- Which model fits the tensor: Laplace or Gaussian (beyond the paper's method) -------------
 *
 * The paper takes the Laplace model for granted ("ACIQ assumes the activation follows a Laplace
 * distribution", Sec. 3); the ACIQ method it builds on also has a Gaussian form.  This picks one per
 * tensor with the measure Eq. 1 itself uses, the squared distance between the real distribution D_R
 * (the histogram as a density at the bin centres c_i, D_R,i = count_i / (N binwidth)) and the estimated
 * one D_E at its moment estimates:
 *     fit_L = sum_i (D_R,i - exp(-|c_i - mu| / b_E) / (2 b_E))^2,                b_E = MAD,
 *     fit_G = sum_i (D_R,i - exp(-(c_i - mu)^2 / (2 s^2)) / (s sqrt(2 pi)))^2,   s = sqrt(var).
 * Gaussian is chosen only if fit_G is strictly below fit_L; a fit that is not a number (one distinct
 * value, zero scale) never wins, so the paper's model is the default.  Returns ORC_LAPLACE or ORC_GAUSS.
 */
int orc_model_fit(const orc_stats_t *st, const uint32_t *hist, double *fit_laplace, double *fit_gauss)
{
    const uint32_t B = st->nbins;
    double binw = (st->max - st->min) / (double)B;
    double b = st->mad, sg = sqrt(st->var);
    double fl = 0.0, fg = 0.0;
    for (uint32_t i = 0; i < B; ++i) {
        double c = st->min + ((double)i + 0.5) * binw;
        double d_r = (double)hist[i] / ((double)st->n * binw);
        double z = c - st->mean;
        double d_l = exp(-fabs(z) / b) / (2.0 * b);
        double d_g = exp(-(z * z) / (2.0 * sg * sg)) / (sg * sqrt(2.0 * 3.14159265358979323846));
        fl += (d_r - d_l) * (d_r - d_l);
        fg += (d_r - d_g) * (d_r - d_g);
    }
    if (B == 0 || st->n == 0) fl = fg = NAN;
    if (fit_laplace) *fit_laplace = fl;
    if (fit_gauss) *fit_gauss = fg;
    return (fg < fl) ? ORC_GAUSS : ORC_LAPLACE;    /* false whenever either is NaN */
}

/* ---- Adaptive PDA controller: window averages feeding Eq. 2 (Sec. 3 "Adaptive PDA", Sec. 4.2) ----
 * The runtime measures over a window of microbatches (50 in the paper's run) and decides when the
 * window expires, from the window's averages: the bandwidth is what the link carried in the window,
 * B = (sum of payload bits) / (sum of sending times), and V is the window's mean payload per
 * microbatch at the current bitwidth.  Between expiries the bitwidth stays as it is. */
typedef struct {
    uint32_t window;       /* microbatches per decision */
    uint32_t count;        /* microbatches seen in the current window */
    double bits_sum;       /* payload bits sent in the current window */
    double seconds_sum;    /* time the link took for them */
    double s_images;       /* S: images per microbatch */
    double r_rate;         /* R: target images per second */
    uint32_t q_cur;        /* bitwidth in force (32 = unquantized) */
    uint32_t decisions;    /* windows that have expired */
} orc_controller_t;

int orc_controller_init(orc_controller_t *c, uint32_t window, double s_images, double r_rate, uint32_t q_start)
{
    if (!c || window == 0 || !(s_images > 0.0) || !(r_rate > 0.0) || q_start == 0) return 2;
    c->window = window;
    c->count = 0;
    c->bits_sum = 0.0;
    c->seconds_sum = 0.0;
    c->s_images = s_images;
    c->r_rate = r_rate;
    c->q_cur = q_start;
    c->decisions = 0;
    return 0;
}

/* one microbatch has been sent; *q_next is the bitwidth for the next one */
int orc_controller_update(orc_controller_t *c, double payload_bits, double seconds, uint32_t *q_next)
{
    if (!c || !q_next || !(payload_bits > 0.0) || !(seconds > 0.0)) return 2;
    c->bits_sum += payload_bits;
    c->seconds_sum += seconds;
    c->count += 1;
    if (c->count == c->window) {
        double bandwidth = c->bits_sum / c->seconds_sum;
        double v_mean = c->bits_sum / (double)c->window;
        uint32_t q;
        int rc = orc_next_bits(v_mean, c->q_cur, c->s_images, c->r_rate, bandwidth, &q);
        if (rc) return rc;
        c->q_cur = q;
        c->count = 0;
        c->bits_sum = 0.0;
        c->seconds_sum = 0.0;
        c->decisions += 1;
    }
    *q_next = c->q_cur;
    return 0;
}
