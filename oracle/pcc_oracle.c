/*
 * pcc_oracle.c -- TEST INFRASTRUCTURE, not the product.
 *
 * A plain, slow, single-threaded CPU statement of what the per-pixel coding
 * path computes, written from the paper (arXiv 2212.01185) so that the HIP
 * library can be checked against it.  It shares no code, tables, headers or
 * helpers with the HIP library.  Only tests, the smoke check and the
 * benchmark's cpu-baseline leg may build, load or call it.
 *
 * Floating point is fp64 throughout (the paper fixes no precision); the normal
 * CDF comes from libm's erfc.  No blocking, fusion or reordering: one pixel at
 * a time, one full 257-entry table per sub-pixel when decoding.
 *
 * What follows the paper and where:
 *   - causal neighbourhood C_ij and "network on C_ij" as a fully connected
 *     net: Sec. III-A (Fig. 1) and Sec. III-C, second paragraph;
 *   - discretised Gaussian mixture pmf: Eq. (1);
 *   - R -> G -> B factorisation with mean-only coupling: Eq. (2), (3), (4);
 *   - encoder sees the whole image, decoder is sequential: Sec. III-C, first
 *     paragraph; the wavefront order and its pass count: Sec. III-C, Eq. (6);
 *     the diagonal order, its pass count and its copied neighbours: Sec. III-C, Eq. (7).
 * What the paper leaves open and this file fixes (each stated at its place):
 *   input scaling x/256, open tails, softmax / exp(clamp) parameterisation,
 *   per-component coupling coefficients, 16-bit integer CDF rule, the rANS
 *   coder (the paper used an arithmetic coder on the CPU, Sec. IV-A) and the
 *   container format.
 *
 * Pins (tests/test_oracle_*.py): closed-form parameter counts, schedule
 * invariants by brute force, raster == wavefront decode, table sums and
 * minimum frequency, single-component reduction to scipy's normal CDF and the
 * direct Eq. (1) pmf, MLP against a float64 numpy matrix product, rANS
 * round-trip and code-length bound, encode -> decode identity on edge shapes.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#define ORC_OK 0
#define ORC_E_ARG (-1)
#define ORC_E_BLOB (-2)
#define ORC_E_CAP (-3)
#define ORC_E_STREAM (-4)
#define ORC_E_INTERNAL (-6)

#define ORC_MAX_LAYERS 7
#define ORC_MAX_WIDTH 512
#define ORC_MAX_K 8

enum { ORC_MODE_EXACT = 0, ORC_MODE_SPLIT_BF16 = 1 };
enum { ORC_ORDER_RASTER = 0, ORC_ORDER_WAVEFRONT = 1 };

typedef struct {
    int n_layers;
    int dims[ORC_MAX_LAYERS + 1];
    int K;      /* mixture components */
    int nbhd;   /* neighbourhood size in pixels */
    int delay;  /* wavefront step = delay*r + c */
    int dist;   /* component distribution: 0 Gaussian (Eq. (1)), 1 logistic (Eq. (8)) */
    int act;    /* 0 ReLU, 1 LeakyReLU with slope 0.01 */
    double *W[ORC_MAX_LAYERS]; /* [out][in] */
    double *b[ORC_MAX_LAYERS];
} orc_model;

/* Causal neighbourhood (Sec. III-A, Fig. 1), raster order, (row offset, column
 * offset).  Ten pixels: rows r-2 and r-1 at columns c-2..c+1, row r at c-2,c-1
 * (the measured workloads).  Twelve pixels: the unmasked taps of the paper's
 * 5x5 first layer (Sec. III-B), rows r-2 and r-1 at columns c-2..c+2, row r at
 * c-2,c-1; the figure is lost, the count follows from the printed parameter
 * numbers (37 C = (12 taps x 3 channels + 1 bias) C) and from the three
 * upper-right pixels the diagonal variant cannot use (Sec. III-C). */
static const int NBHD10[10][2] = {
    {-2, -2}, {-2, -1}, {-2, 0}, {-2, 1},
    {-1, -2}, {-1, -1}, {-1, 0}, {-1, 1},
    {0, -2}, {0, -1}};
static const int NBHD12[12][2] = {
    {-2, -2}, {-2, -1}, {-2, 0}, {-2, 1}, {-2, 2},
    {-1, -2}, {-1, -1}, {-1, 0}, {-1, 1}, {-1, 2},
    {0, -2}, {0, -1}};

static uint32_t rd32(const uint8_t *p) {
    return (uint32_t)p[0] | ((uint32_t)p[1] << 8) | ((uint32_t)p[2] << 16) | ((uint32_t)p[3] << 24);
}
static uint64_t rd64(const uint8_t *p) { return (uint64_t)rd32(p) | ((uint64_t)rd32(p + 4) << 32); }
static void wr32(uint8_t *p, uint32_t v) {
    p[0] = (uint8_t)v; p[1] = (uint8_t)(v >> 8); p[2] = (uint8_t)(v >> 16); p[3] = (uint8_t)(v >> 24);
}
static void wr64(uint8_t *p, uint64_t v) { wr32(p, (uint32_t)v); wr32(p + 4, (uint32_t)(v >> 32)); }

/* ------------------------------------------------------------------ model */

void orc_model_destroy(orc_model *m) {
    if (!m) return;
    for (int l = 0; l < ORC_MAX_LAYERS; ++l) { free(m->W[l]); free(m->b[l]); }
    free(m);
}

/* Weight blob: 16 little-endian uint32 header words (magic "PCCW", version,
 * n_layers, dims[8], K, neighbourhood size, delay, activation id, distribution
 * id), then per layer W[out][in] and b[out] as fp32. */
int orc_model_create(const void *blob, size_t nbytes, orc_model **out) {
    if (!blob || !out) return ORC_E_ARG;
    const uint8_t *p = (const uint8_t *)blob;
    if (nbytes < 64 || rd32(p) != 0x57434350u || rd32(p + 4) != 1u) return ORC_E_BLOB;
    orc_model *m = (orc_model *)calloc(1, sizeof(orc_model));
    if (!m) return ORC_E_INTERNAL;
    m->n_layers = (int)rd32(p + 8);
    if (m->n_layers < 1 || m->n_layers > ORC_MAX_LAYERS) { free(m); return ORC_E_BLOB; }
    for (int i = 0; i <= m->n_layers; ++i) {
        m->dims[i] = (int)rd32(p + 12 + 4 * i);
        if (m->dims[i] < 1 || m->dims[i] > ORC_MAX_WIDTH) { free(m); return ORC_E_BLOB; }
    }
    m->K = (int)rd32(p + 44);
    m->nbhd = (int)rd32(p + 48);
    m->delay = (int)rd32(p + 52);
    uint32_t act = rd32(p + 56), dist = rd32(p + 60);
    m->dist = (int)dist;
    m->act = (int)act;
    /* the wavefront delay per row is the neighbourhood's right reach + 1: Eq. (6) with h = reach;
     * delay 1 with the 12-pixel neighbourhood is the diagonal variant (Eq. (7)), whose three
     * not yet decoded neighbours are replaced by a copy (see orc_tap_source) */
    if (m->K < 1 || m->K > ORC_MAX_K ||
        !((m->nbhd == 10 && m->delay == 2) || (m->nbhd == 12 && (m->delay == 3 || m->delay == 1))) ||
        act > 1 || dist > 1 ||
        m->dims[0] != 3 * m->nbhd || m->dims[m->n_layers] != 12 * m->K) { free(m); return ORC_E_BLOB; }
    size_t need = 64;
    for (int l = 0; l < m->n_layers; ++l) need += 4 * ((size_t)m->dims[l] * m->dims[l + 1] + m->dims[l + 1]);
    if (nbytes != need) { free(m); return ORC_E_BLOB; }
    const uint8_t *q = p + 64;
    for (int l = 0; l < m->n_layers; ++l) {
        size_t nw = (size_t)m->dims[l] * m->dims[l + 1], nb = (size_t)m->dims[l + 1];
        m->W[l] = (double *)malloc(nw * sizeof(double));
        m->b[l] = (double *)malloc(nb * sizeof(double));
        if (!m->W[l] || !m->b[l]) { orc_model_destroy(m); return ORC_E_INTERNAL; }
        for (size_t i = 0; i < nw; ++i, q += 4) { uint32_t u = rd32(q); float f; memcpy(&f, &u, 4); m->W[l][i] = f; }
        for (size_t i = 0; i < nb; ++i, q += 4) { uint32_t u = rd32(q); float f; memcpy(&f, &u, 4); m->b[l][i] = f; }
    }
    *out = m;
    return ORC_OK;
}

/* ------------------------------------------------------------------ network */

/* Position the network input for neighbour j of pixel (r, c) is read from.
 * Wavefront models: the neighbour itself.  Diagonal model (Sec. III-C, text
 * after Eq. (7)): a pass decodes all pixels of one anti-diagonal r + c = t, so
 * the three neighbours on or beyond the pixel's own anti-diagonal -- (r-2,c+2),
 * (r-1,c+1), (r-1,c+2) -- are not yet decoded and carry a copy of an available
 * pixel instead.  Which pixel the paper copies is shown only in a figure that
 * is lost; this build takes (r-1, c), the nearest decoded pixel to all three.
 * The copy is made on the zero-padded patch: it applies wherever the three
 * positions fall, and copies zero when (r-1, c) itself is outside the image. */
void orc_tap_source(const orc_model *m, int r, int c, int j, int *rr, int *cc) {
    const int (*nb)[2] = m->nbhd == 10 ? NBHD10 : NBHD12;
    int dr = nb[j][0], dc = nb[j][1];
    if (m->delay == 1 && dr + dc >= 0) { dr = -1; dc = 0; }
    *rr = r + dr;
    *cc = c + dc;
}

/* C_ij as the network input vector (Sec. III-A; Sec. III-C, second paragraph):
 * u[3*j + ch] = img[source of neighbour j][ch] / 256, and 0 where that position
 * lies outside the image (the zero padding of the first convolution).  The
 * scaling by 1/256 is this build's choice; the paper does not state one. */
void orc_gather(const orc_model *m, const uint8_t *img, int H, int W, int r, int c, double *u) {
    (void)H;
    for (int j = 0; j < m->nbhd; ++j) {
        int rr, cc;
        orc_tap_source(m, r, c, j, &rr, &cc);
        for (int ch = 0; ch < 3; ++ch) {
            double v = 0.0;
            if (rr >= 0 && cc >= 0 && cc < W) v = img[((size_t)rr * W + cc) * 3 + ch] / 256.0;
            u[3 * j + ch] = v;
        }
    }
}

/* Nearest bf16 (8 significant bits), ties to even. */
static double round_bf16(double x) {
    if (x == 0.0 || !isfinite(x)) return x;
    int e;
    double f = frexp(x, &e);            /* x = f * 2^e, 0.5 <= |f| < 1 */
    double s = ldexp(f, 8);             /* 128 <= |s| < 256 */
    double r = nearbyint(s);            /* default rounding mode: to nearest, ties to even */
    return ldexp(r, e - 8);
}

/* The probability network as a fully connected stack on C_ij (Sec. III-B with
 * the equivalence of Sec. III-C, second paragraph): ReLU (or the paper's
 * LeakyReLU, slope 0.01 -- the paper gives none) between layers, none after the last.  Mode EXACT is the definition.  Mode SPLIT_BF16 rounds every
 * hidden activation a to hi + lo with hi = bf16(a), lo = bf16(a - hi), i.e. to
 * about 16 significant bits -- the representation the matrix-core path feeds
 * to its bf16 multipliers; it exists to show how little that rounding moves
 * the outputs, not as a second definition. */
void orc_mlp(const orc_model *m, const double *u, int mode, double *o) {
    double a[ORC_MAX_WIDTH], z[ORC_MAX_WIDTH];
    for (int i = 0; i < m->dims[0]; ++i) a[i] = u[i];
    for (int l = 0; l < m->n_layers; ++l) {
        int nin = m->dims[l], nout = m->dims[l + 1];
        for (int j = 0; j < nout; ++j) {
            double s = 0.0;
            for (int i = 0; i < nin; ++i) s += m->W[l][(size_t)j * nin + i] * a[i];
            z[j] = s + m->b[l][j];
        }
        if (l + 1 < m->n_layers) {
            for (int j = 0; j < nout; ++j) {
                double h = z[j] > 0.0 ? z[j] : (m->act == 1 ? 0.01 * z[j] : 0.0);
                if (mode == ORC_MODE_SPLIT_BF16) { double hi = round_bf16(h); h = hi + round_bf16(h - hi); }
                a[j] = h;
            }
        } else {
            for (int j = 0; j < nout; ++j) o[j] = z[j];
        }
    }
}

/* Raw head outputs of one pixel: gather + network. */
void orc_params_at(const orc_model *m, const uint8_t *img, int H, int W, int r, int c, int mode, double *o) {
    double u[ORC_MAX_WIDTH];
    orc_gather(m, img, H, W, r, c, u);
    orc_mlp(m, u, mode, o);
}

/* ------------------------------------------------------------------ mixture */

/* Head layout o[12K]: channel ch in R,G,B occupies o[3K*ch ..]: K mixture
 * logits, K means, K log-sigmas; then K alphas, K betas, K gammas.
 *
 * Mixture parameters of channel ch (Eq. (1)-(4)), in units of 1/256 of the
 * grey-level range (mu = 256*mu_hat, s = 256*sigma_hat turns Eq. (1) into the
 * form used below):
 *   pi    = softmax(logits)
 *   sigma = exp(clamp(log-sigma, -8, 4))
 *   mu_R  = mean_R
 *   mu_G  = mean_G + alpha * r/256                    (Eq. (3))
 *   mu_B  = mean_B + beta * r/256 + gamma * g/256     (Eq. (4))
 * The coupling coefficients are per mixture component (the head has 12
 * outputs per component: 3 x (pi, mu, s) + alpha, beta, gamma). */
void orc_mixture(const orc_model *m, const double *o, int ch, int r, int g,
                 double *pi, double *mu, double *sigma) {
    int K = m->K;
    const double *lg = o + 3 * K * ch, *mn = lg + K, *ls = lg + 2 * K;
    const double *alpha = o + 9 * K, *beta = alpha + K, *gamma = alpha + 2 * K;
    double mx = lg[0], sum = 0.0;
    for (int k = 1; k < K; ++k) if (lg[k] > mx) mx = lg[k];
    for (int k = 0; k < K; ++k) { pi[k] = exp(lg[k] - mx); sum += pi[k]; }
    for (int k = 0; k < K; ++k) pi[k] /= sum;
    for (int k = 0; k < K; ++k) {
        double t = ls[k] < -8.0 ? -8.0 : (ls[k] > 4.0 ? 4.0 : ls[k]);
        sigma[k] = exp(t);
        mu[k] = mn[k];
        if (ch == 1) mu[k] += alpha[k] * (r / 256.0);
        if (ch == 2) mu[k] += beta[k] * (r / 256.0) + gamma[k] * (g / 256.0);
    }
}

/* Mixture CDF at the lower edge of bin e, i.e. at grey level e - 0.5 (Eq. (1)
 * sums pi_i [F(x+0.5) - F(x-0.5)], so the pmf of x is mixcdf(x+1) - mixcdf(x)). */
static double mixcdf(int dist, int K, const double *pi, const double *mu, const double *sigma, int e) {
    double F = 0.0;
    for (int k = 0; k < K; ++k) {
        double z = ((e - 0.5) / 256.0 - mu[k]) / sigma[k];
        /* standard normal CDF, or the logistic CDF of Eq. (8) with scale s = sigma */
        F += pi[k] * (dist == 0 ? 0.5 * erfc(-z / sqrt(2.0)) : 1.0 / (1.0 + exp(-z)));
    }
    return F;
}

/* Integer CDF with 16-bit total (this build's rule; the paper hands real CDF
 * values to its coder and does not say how they are quantised):
 *   Cq(0) = 0, Cq(256) = 65536                      (open tails: bins 0 and 255
 *                                                    take the mass beyond the range)
 *   Cq(e) = e + min(floor(F(e) * 65280), 65280)      for 1 <= e <= 255
 * so every symbol has frequency >= 1 whenever F is non-decreasing in e. */
static uint32_t cq_at(int dist, int K, const double *pi, const double *mu, const double *sigma, int e) {
    if (e <= 0) return 0;
    if (e >= 256) return 65536;
    double v = floor(mixcdf(dist, K, pi, mu, sigma, e) * 65280.0);
    if (v > 65280.0) v = 65280.0;
    if (v < 0.0) v = 0.0;
    return (uint32_t)e + (uint32_t)v;
}

/* Full table of one sub-pixel: cq[0..256].  Returns ORC_E_INTERNAL if it is
 * not strictly increasing (would mean a zero frequency). */
int orc_cdf_table(const orc_model *m, const double *o, int ch, int r, int g, uint32_t *cq) {
    double pi[ORC_MAX_K], mu[ORC_MAX_K], sigma[ORC_MAX_K];
    orc_mixture(m, o, ch, r, g, pi, mu, sigma);
    for (int e = 0; e <= 256; ++e) cq[e] = cq_at(m->dist, m->K, pi, mu, sigma, e);
    for (int e = 0; e < 256; ++e) if (cq[e + 1] <= cq[e]) return ORC_E_INTERNAL;
    return ORC_OK;
}

/* (start, freq) of symbol x in channel ch. */
static void sym_interval(const orc_model *m, const double *o, int ch, int r, int g, int x,
                         uint32_t *start, uint32_t *freq) {
    double pi[ORC_MAX_K], mu[ORC_MAX_K], sigma[ORC_MAX_K];
    orc_mixture(m, o, ch, r, g, pi, mu, sigma);
    uint32_t lo = cq_at(m->dist, m->K, pi, mu, sigma, x), hi = cq_at(m->dist, m->K, pi, mu, sigma, x + 1);
    *start = lo;
    *freq = hi - lo;
}

/* Continuous (unquantised) pmf of Eq. (1) with open tails, for tests. */
void orc_pmf(const orc_model *m, const double *o, int ch, int r, int g, double *p256) {
    double pi[ORC_MAX_K], mu[ORC_MAX_K], sigma[ORC_MAX_K];
    orc_mixture(m, o, ch, r, g, pi, mu, sigma);
    for (int x = 0; x < 256; ++x) {
        double lo = x == 0 ? 0.0 : mixcdf(m->dist, m->K, pi, mu, sigma, x);
        double hi = x == 255 ? 1.0 : mixcdf(m->dist, m->K, pi, mu, sigma, x + 1);
        p256[x] = hi - lo;
    }
}

/* ------------------------------------------------------------------ rANS */

/* Range asymmetric numeral system, one independent stream per image row, coded
 * with two interleaved states: symbol i of the row (i = 3 c + channel) is coded
 * on state i mod 2.  Both states share the row's one sequence of words, so the
 * row stays one stream; two states halve the chain of dependent operations that
 * a coder has to go through per row (this build's choice, like the coder itself:
 * the paper used an arithmetic coder on the CPU).
 * 64-bit states x in [2^31, 2^63), 16-bit frequencies (total 2^16), 32-bit
 * renormalisation words.  A row payload is: the final encoder states 0 and 1
 * (8 bytes each, little-endian), then the words in the order the decoder
 * consumes them.  Symbols are pushed last-to-first so the decoder pops them
 * first-to-last; a word written before symbol i is pushed is the word read
 * after symbol i is popped, whichever state it belongs to. */
#define RANS_L ((uint64_t)1 << 31)

size_t orc_rans_bound(size_t nsym) { return 16 + 4 * (nsym / 2 + 2); }

/* start[i], freq[i] for i in decode order.  Returns payload bytes or 0 on error. */
size_t orc_rans_encode(const uint32_t *start, const uint32_t *freq, size_t nsym, uint8_t *out, size_t cap) {
    uint32_t *words = (uint32_t *)malloc(sizeof(uint32_t) * (nsym / 2 + 2));
    if (!words) return 0;
    size_t nw = 0;
    uint64_t x[2] = {RANS_L, RANS_L};
    for (size_t i = nsym; i-- > 0;) {
        uint64_t f = freq[i], s = start[i];
        uint64_t *xs = &x[i & 1];
        if (f == 0 || s + f > 65536) { free(words); return 0; }
        if (*xs >= (f << 47)) { words[nw++] = (uint32_t)*xs; *xs >>= 32; }
        *xs = ((*xs / f) << 16) + (*xs % f) + s;
    }
    size_t nbytes = 16 + 4 * nw;
    if (nbytes > cap) { free(words); return 0; }
    wr64(out, x[0]);
    wr64(out + 8, x[1]);
    for (size_t j = 0; j < nw; ++j) wr32(out + 16 + 4 * j, words[nw - 1 - j]);
    free(words);
    return nbytes;
}

typedef struct { uint64_t x[2]; size_t n; const uint8_t *p, *end; int bad; } rans_dec;   /* n: symbols popped so far */

static void rans_dec_init(rans_dec *d, const uint8_t *payload, size_t nbytes) {
    d->bad = nbytes < 16;
    d->n = 0;
    for (int k = 0; k < 2; ++k) {
        d->x[k] = d->bad ? RANS_L : rd64(payload + 8 * k);
        if (!d->bad && (d->x[k] < RANS_L || (d->x[k] >> 63))) d->bad = 1;
    }
    d->p = payload + 16;
    d->end = payload + nbytes;
}
static uint32_t rans_dec_peek(const rans_dec *d) { return (uint32_t)(d->x[d->n & 1] & 0xFFFF); }
static void rans_dec_advance(rans_dec *d, uint32_t start, uint32_t freq) {
    uint64_t *xs = &d->x[d->n & 1];
    d->n += 1;
    *xs = (uint64_t)freq * (*xs >> 16) + (*xs & 0xFFFF) - start;
    if (*xs < RANS_L) {
        if (d->p + 4 > d->end) { d->bad = 1; *xs |= RANS_L; return; }
        *xs = (*xs << 32) | rd32(d->p);
        d->p += 4;
    }
}
/* A well-formed payload ends exactly where the encoder began. */
static int rans_dec_finished(const rans_dec *d) { return !d->bad && d->x[0] == RANS_L && d->x[1] == RANS_L && d->p == d->end; }

/* Decode nsym symbols against explicit tables cq[i][0..256] (test hook for the coder alone). */
int orc_rans_decode_tables(const uint8_t *payload, size_t nbytes, const uint32_t *cq_tables, size_t nsym, uint8_t *sym_out) {
    rans_dec d;
    rans_dec_init(&d, payload, nbytes);
    for (size_t i = 0; i < nsym; ++i) {
        const uint32_t *cq = cq_tables + 257 * i;
        uint32_t slot = rans_dec_peek(&d);
        int x = 0;
        for (int e = 0; e < 256; ++e) if (cq[e] <= slot) x = e;
        sym_out[i] = (uint8_t)x;
        rans_dec_advance(&d, cq[x], cq[x + 1] - cq[x]);
        if (d.bad) return ORC_E_STREAM;
    }
    return rans_dec_finished(&d) ? ORC_OK : ORC_E_STREAM;
}

/* ------------------------------------------------------------------ container */

/* Stream: 8 little-endian uint32 header words (magic "PCC1", version 2, n, H,
 * W, K | nbhd<<8 | delay<<16 | 16<<24 (CDF bits), distribution id, 0), then uint64
 * offsets[n*H + 1] of the row payloads relative to the end of the offset
 * table, then the payloads back to back (each a multiple of 4 bytes). */
#define STREAM_MAGIC 0x31434350u
#define STREAM_HEADER 32
#define STREAM_VERSION 2   /* 1: one coder state per row */

size_t orc_stream_bound(int n, int H, int W) {
    size_t rows = (size_t)n * H;
    return STREAM_HEADER + 8 * (rows + 1) + rows * orc_rans_bound(3 * (size_t)W);
}

static uint32_t model_tag(const orc_model *m) {
    return (uint32_t)m->K | ((uint32_t)m->nbhd << 8) | ((uint32_t)m->delay << 16) | (16u << 24);
}

/* Encoder (Sec. III-C first paragraph; Sec. IV-C first paragraph): every
 * pixel's parameters come from the true image, CDF values follow, and the
 * entropy coder receives them with the pixel values.  Rows are independent
 * streams, so any decoding order that respects causality reads them the same
 * way.  bits_out (optional, [n*H*W]) receives -log2 of the quantised joint
 * probability of each pixel, the per-pixel term of the loss of Eq. (5). */
int orc_encode(const orc_model *m, const uint8_t *img, int n, int H, int W, int mode,
               uint8_t *stream, size_t cap, size_t *nbytes_out, double *bits_out) {
    if (!m || !img || !stream || !nbytes_out || n < 1 || H < 1 || W < 1) return ORC_E_ARG;
    size_t rows = (size_t)n * H, nsym = 3 * (size_t)W;
    size_t table = STREAM_HEADER + 8 * (rows + 1);
    if (cap < table) return ORC_E_CAP;
    uint32_t *start = (uint32_t *)malloc(nsym * sizeof(uint32_t));
    uint32_t *freq = (uint32_t *)malloc(nsym * sizeof(uint32_t));
    if (!start || !freq) { free(start); free(freq); return ORC_E_INTERNAL; }
    wr32(stream, STREAM_MAGIC); wr32(stream + 4, STREAM_VERSION); wr32(stream + 8, (uint32_t)n);
    wr32(stream + 12, (uint32_t)H); wr32(stream + 16, (uint32_t)W); wr32(stream + 20, model_tag(m));
    wr32(stream + 24, (uint32_t)m->dist); wr32(stream + 28, 0);
    size_t off = 0;
    int rc = ORC_OK;
    double o[ORC_MAX_WIDTH];
    for (int i = 0; i < n && rc == ORC_OK; ++i) {
        const uint8_t *im = img + (size_t)i * H * W * 3;
        for (int r = 0; r < H && rc == ORC_OK; ++r) {
            for (int c = 0; c < W; ++c) {
                const uint8_t *px = im + ((size_t)r * W + c) * 3;
                orc_params_at(m, im, H, W, r, c, mode, o);
                double bits = 0.0;
                for (int ch = 0; ch < 3; ++ch) {
                    sym_interval(m, o, ch, px[0], px[1], px[ch], &start[3 * c + ch], &freq[3 * c + ch]);
                    if (freq[3 * c + ch] == 0 || freq[3 * c + ch] > 65536) rc = ORC_E_INTERNAL;
                    else bits -= log2(freq[3 * c + ch] / 65536.0);
                }
                if (bits_out) bits_out[((size_t)i * H + r) * W + c] = bits;
            }
            if (rc != ORC_OK) break;
            wr64(stream + STREAM_HEADER + 8 * ((size_t)i * H + r), off);
            size_t room = cap - table - off;
            size_t nb = orc_rans_encode(start, freq, nsym, stream + table + off, room);
            if (nb == 0) { rc = ORC_E_CAP; break; }
            off += nb;
        }
    }
    if (rc == ORC_OK) { wr64(stream + STREAM_HEADER + 8 * rows, off); *nbytes_out = table + off; }
    free(start); free(freq);
    return rc;
}

/* Pass count for an H x W image when each row trails the one above by `delay`
 * columns: Eq. (6) generalised to W != H, T = W + (H-1)*delay (the paper's
 * D + (D-1)(h+1) has delay = h+1 and W = H = D); delay = 1 is the diagonal
 * order, T = W + H - 1, Eq. (7)'s 2D - 1. */
long orc_wavefront_steps(int H, int W, int delay) { return (long)W + (long)(H - 1) * delay; }

/* Decoder (Sec. III-C): a pixel is decoded by evaluating the network on its
 * already decoded neighbourhood, then R, then G given R, then B given R and G.
 * order = RASTER is the fully sequential decoder (one pass per pixel);
 * order = WAVEFRONT visits passes t = 0,1,..., and in pass t every row r whose
 * column c = t - delay*r lies in the image (delay = 1: the anti-diagonal
 * r + c = t).  A pass is parallel: the networks of all its pixels are
 * evaluated on the image as it stood before the pass, and only then are its
 * pixels decoded.  Both orders must give the same image. */
int orc_decode(const orc_model *m, const uint8_t *stream, size_t nbytes, int n, int H, int W,
               int mode, int order, uint8_t *img_out) {
    if (!m || !stream || !img_out || n < 1 || H < 1 || W < 1) return ORC_E_ARG;
    size_t rows = (size_t)n * H;
    size_t table = STREAM_HEADER + 8 * (rows + 1);
    if (nbytes < table) return ORC_E_STREAM;
    if (rd32(stream) != STREAM_MAGIC || rd32(stream + 4) != STREAM_VERSION || rd32(stream + 8) != (uint32_t)n ||
        rd32(stream + 12) != (uint32_t)H || rd32(stream + 16) != (uint32_t)W || rd32(stream + 20) != model_tag(m) ||
        rd32(stream + 24) != (uint32_t)m->dist)
        return ORC_E_STREAM;
    rans_dec *dec = (rans_dec *)malloc(rows * sizeof(rans_dec));
    if (!dec) return ORC_E_INTERNAL;
    for (size_t k = 0; k < rows; ++k) {
        uint64_t a = rd64(stream + STREAM_HEADER + 8 * k), b = rd64(stream + STREAM_HEADER + 8 * (k + 1));
        if (a > b || b > nbytes - table || (k == 0 && a != 0)) { free(dec); return ORC_E_STREAM; }
        rans_dec_init(&dec[k], stream + table + a, (size_t)(b - a));
    }
    if (rd64(stream + STREAM_HEADER + 8 * rows) != nbytes - table) { free(dec); return ORC_E_STREAM; }
    memset(img_out, 0, (size_t)n * H * W * 3);
    int rc = ORC_OK;
    uint32_t cq[257];
    double *o_pass = (double *)malloc((size_t)H * ORC_MAX_WIDTH * sizeof(double));   /* head outputs of one pass, per row */
    if (!o_pass) { free(dec); return ORC_E_INTERNAL; }
    long T = order == ORC_ORDER_WAVEFRONT ? orc_wavefront_steps(H, W, m->delay) : (long)H * W;
    for (int i = 0; i < n && rc == ORC_OK; ++i) {
        uint8_t *im = img_out + (size_t)i * H * W * 3;
        for (long t = 0; t < T && rc == ORC_OK; ++t) {
            int r_lo, r_hi;
            if (order == ORC_ORDER_WAVEFRONT) { r_lo = 0; r_hi = H - 1; }
            else { r_lo = r_hi = (int)(t / W); }
            /* first every network of the pass, on the image before the pass ... */
            for (int r = r_lo; r <= r_hi; ++r) {
                long c = order == ORC_ORDER_WAVEFRONT ? t - (long)m->delay * r : t % W;
                if (c < 0 || c >= W) continue;
                orc_params_at(m, im, H, W, r, (int)c, mode, o_pass + (size_t)r * ORC_MAX_WIDTH);
            }
            /* ... then its symbols */
            for (int r = r_lo; r <= r_hi && rc == ORC_OK; ++r) {
                long c = order == ORC_ORDER_WAVEFRONT ? t - (long)m->delay * r : t % W;
                if (c < 0 || c >= W) continue;
                rans_dec *d = &dec[(size_t)i * H + r];
                uint8_t *px = im + ((size_t)r * W + c) * 3;
                const double *o = o_pass + (size_t)r * ORC_MAX_WIDTH;
                for (int ch = 0; ch < 3; ++ch) {
                    if (orc_cdf_table(m, o, ch, px[0], px[1], cq) != ORC_OK) { rc = ORC_E_INTERNAL; break; }
                    uint32_t slot = rans_dec_peek(d);
                    int x = 0;
                    for (int e = 0; e < 256; ++e) if (cq[e] <= slot) x = e;   /* largest e with Cq(e) <= slot */
                    px[ch] = (uint8_t)x;
                    rans_dec_advance(d, cq[x], cq[x + 1] - cq[x]);
                    if (d->bad) { rc = ORC_E_STREAM; break; }
                }
            }
        }
    }
    free(o_pass);
    for (size_t k = 0; k < rows && rc == ORC_OK; ++k) if (!rans_dec_finished(&dec[k])) rc = ORC_E_STREAM;
    free(dec);
    return rc;
}
