/*
 * e4q_oracle.c -- plain, slow, single-threaded CPU oracle for row-wise 4-bit
 * uniform quantization of embedding tables with greedy clip search, as in
 * "Post-Training 4-bit Quantization on Embedding Tables" (arXiv 1911.02079).
 *
 * THIS IS TEST INFRASTRUCTURE, NOT THE PRODUCT.  Only the test-suite, the smoke
 * check and the benchmark's CPU-baseline leg may call it.  It shares no code,
 * header, table or helper with the HIP library, and neither includes the other.
 *
 * What it follows:
 *   - the uniform quantizer Q and its dequantizer  (Eq. 1 and the sentence
 *     after it: scale = (xmax - xmin)/(2^n - 1), bias = xmin,
 *     x_float = scale * x_int + bias),
 *   - the loss f(xmin, xmax) = || X - Q(X, xmin, xmax) ||_2^2      (Eq. 2),
 *   - the greedy search over clipping ranges                  (Algorithm 1),
 *   - FP16 storage of the per-row scale and bias   (Section 5, "(FP16)" rows
 *     of Tables 2 and 3).
 *
 * The paper leaves the floating-point realisation open.  The readings taken
 * here (every one is a reading, not a quotation):
 *   - all arithmetic is IEEE binary32, round-to-nearest-even, each operation
 *     rounded on its own; the one fused operation is the dequantizer
 *     scale*q+bias, written fmaf below;
 *   - scale and bias are rounded to binary16 BEFORE a candidate range is
 *     scored, so the search minimises the error of what is actually stored;
 *   - Eq. 1 is evaluated as (x - bias) * (1/scale) with a correctly rounded
 *     reciprocal; round() is round-half-to-even; the result is clamped to
 *     [0, 15] (that is the clipping of x to [xmin, xmax]);
 *   - the squared errors of a row are summed by a fixed balanced tree over
 *     index-adjacent pairs (zero padded to a power of two);
 *   - the while-test of Algorithm 1 is replaced by its exact-arithmetic trip
 *     count n_iter = ceil(b*r), clamped to [0, b-1] (the float test sits exactly
 *     on the boundary for the default b = 200, r = 0.16);
 *   - the best (xmin, xmax) is tracked as a PAIR together with its loss
 *     ("joint" tracking).  Algorithm 1 as printed updates only one of the two
 *     on an improvement; `literal_alg1 != 0` reproduces that bookkeeping;
 *   - codes are packed 8/n per byte, the first element in the lowest bits (n = 4: low nibble =
 *     even element, high nibble = odd element);
 *   - n = 4 is the paper's subject; n = 8 (its ASYM-8BITS baseline) and n = 2 run through the
 *     same code with 2^n - 1 levels.
 *
 * Pins (see tests): exact 16-point grids, never worse than min/max,
 * brute force over the (i, j) grid, exact rational re-execution of
 * Algorithm 1 on integer lattices, power-of-two equivariance, r = 0 against
 * the textbook affine quantizer, binary16 conversion against an independent
 * library, Table 3's size column.
 *
 * Build: gcc -O2 -ffp-contract=off -mfma -msse4.1 -shared -fPIC (no fast-math).
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

/* Largest code, 2^n - 1 (Eq. 1); n = 4 is the paper's subject, n = 8 its ASYM-8BITS baseline. */
static float qmax_of(int nbits) { return (float)((1 << nbits) - 1); }
static int nbits_ok(int nbits) { return nbits == 2 || nbits == 4 || nbits == 8; }
/* Codes are packed 8/n per byte, element k in bits [(k mod 8/n) * n, +n) of byte k / (8/n). */
static int64_t packed_bytes(int dim, int nbits) { int per = 8 / nbits; return (dim + per - 1) / per; }

/* ------------------------------------------------------------------ */
/* binary16 <-> binary32, written out so that it can be audited.       */
/* ------------------------------------------------------------------ */

static uint32_t f32_bits(float f) { uint32_t u; memcpy(&u, &f, 4); return u; }
static float bits_f32(uint32_t u) { float f; memcpy(&f, &u, 4); return f; }

/* binary32 -> binary16, round-to-nearest-even, subnormals kept, overflow to inf. */
uint16_t e4q_oracle_f32_to_f16(float f)
{
    uint32_t u = f32_bits(f);
    uint32_t sign = (u >> 16) & 0x8000u;
    int32_t exp = (int32_t)((u >> 23) & 0xffu);
    uint32_t man = u & 0x7fffffu;

    if (exp == 0xff) /* inf or NaN */
        return (uint16_t)(sign | 0x7c00u | (man ? 0x200u : 0u));

    int32_t e = exp - 127 + 15; /* biased binary16 exponent */
    if (e >= 31)
        return (uint16_t)(sign | 0x7c00u);

    if (e <= 0) {
        /* result is subnormal (or zero): value = man24 * 2^(exp-150),
           one binary16 subnormal unit is 2^-24, so shift right by 14 - e. */
        if (e < -10)
            return (uint16_t)sign; /* below half of the smallest subnormal */
        uint32_t man24 = man | 0x800000u;
        int shift = 14 - e; /* 14 .. 24 */
        uint32_t q = man24 >> shift;
        uint32_t rem = man24 & ((1u << shift) - 1u);
        uint32_t half = 1u << (shift - 1);
        if (rem > half || (rem == half && (q & 1u)))
            q++;
        return (uint16_t)(sign | q); /* a carry lands in the exponent field, which is right */
    }

    uint32_t h = ((uint32_t)e << 10) | (man >> 13);
    uint32_t rem = man & 0x1fffu;
    if (rem > 0x1000u || (rem == 0x1000u && (h & 1u)))
        h++; /* may carry up to 0x7c00 = inf, which is the correct rounding */
    return (uint16_t)(sign | h);
}

/* binary16 -> binary32 (always exact). */
float e4q_oracle_f16_to_f32(uint16_t h)
{
    uint32_t sign = ((uint32_t)h & 0x8000u) << 16;
    uint32_t exp = (h >> 10) & 0x1fu;
    uint32_t man = h & 0x3ffu;
    if (exp == 0x1f)
        return bits_f32(sign | 0x7f800000u | (man << 13));
    if (exp == 0) {
        /* subnormal: man * 2^-24 */
        float v = (float)man * 0x1p-24f;
        return sign ? -v : v;
    }
    return bits_f32(sign | ((exp - 15 + 127) << 23) | (man << 13));
}

static float round_through_f16(float f) { return e4q_oracle_f16_to_f32(e4q_oracle_f32_to_f16(f)); }

/* ------------------------------------------------------------------ */
/* Eq. 1 on one element, for stored parameters (scale, bias).          */
/* ------------------------------------------------------------------ */

/* x_int of Eq. 1, as a float in {0, ..., qmax}.  `inv` is 1/scale, or unused when scale == 0. */
static float quantize_elem(float x, float scale, float bias, float inv, float qmax)
{
    if (scale == 0.0f)
        return 0.0f; /* degenerate range: one grid point, code 0 */
    float t = (x - bias) * inv; /* subtract, then multiply: two roundings */
    float q = rintf(t);         /* round-half-to-even (default rounding mode) */
    if (q < 0.0f) q = 0.0f;     /* x below xmin is clipped to xmin */
    if (q > qmax) q = qmax;     /* x above xmax is clipped to xmax */
    return q;
}

/* The parameters that would be stored for the range [lo, hi] (Eq. 1, FP16 storage). */
static void stored_params(float lo, float hi, float qmax, float *scale, float *bias)
{
    float scale32 = (hi - lo) / qmax;
    *scale = round_through_f16(scale32);
    *bias = round_through_f16(lo);
}

static int next_pow2(int d)
{
    int p = 1;
    while (p < d) p *= 2;
    return p;
}

/* Balanced pairwise sum of s[0..d), zero-padded to `p` (a power of two >= d).
   Overwrites s (which must hold p floats). */
static float tree_sum(float *s, int d, int p)
{
    for (int k = d; k < p; ++k) s[k] = 0.0f;
    for (int m = p; m > 1; m /= 2)
        for (int i = 0; i < m / 2; ++i)
            s[i] = s[2 * i] + s[2 * i + 1];
    return s[0];
}

/* Eq. 2 for the range [lo, hi]: || X - Q(X, lo, hi) ||_2^2.  `work` holds next_pow2(d) floats. */
static float range_loss(const float *x, int d, float lo, float hi, float qmax, float *work)
{
    float scale, bias;
    stored_params(lo, hi, qmax, &scale, &bias);
    float inv = (scale == 0.0f) ? 0.0f : 1.0f / scale;
    for (int k = 0; k < d; ++k) {
        float q = quantize_elem(x[k], scale, bias, inv, qmax);
        float xh = fmaf(q, scale, bias); /* dequantizer of Eq. 1 */
        float e = x[k] - xh;
        work[k] = e * e;
    }
    return tree_sum(work, d, next_pow2(d));
}

/* Trip count of Algorithm 1's loop in exact arithmetic: the range shrinks by one
   stepsize = range/b per trip and the loop runs while it exceeds (1 - r) * range, i.e. for
   ceil(b*r) trips.  r arrives as a binary32 number, which may sit a relative 2^-24 above the
   decimal the caller wrote (0.4f * 20 = 8.0000001); the product is therefore shrunk by a
   relative 2^-22 before the ceiling so that b*r "= 8" gives 8 trips, not 9. */
int32_t e4q_oracle_n_iter(int32_t n_bins, float ratio)
{
    double br = (double)n_bins * (double)ratio;
    double t = ceil(br - br * 0x1p-22);
    if (t < 0.0) t = 0.0;
    if (t > (double)(n_bins - 1)) t = (double)(n_bins - 1);
    return (int32_t)t;
}

/* ------------------------------------------------------------------ */
/* Algorithm 1 on one row.                                             */
/* ------------------------------------------------------------------ */

typedef struct {
    float xmin, xmax; /* the returned clipping range */
    float loss;       /* the loss the search associates with it */
    int32_t i, j;     /* how many steps each bound was moved for (xmin, xmax) */
} greedy_result;

static greedy_result greedy_row(const float *x, int d, int32_t n_bins, int32_t n_iter,
                                int literal_alg1, float qmax, float *work)
{
    float lo0 = x[0], hi0 = x[0];
    for (int k = 1; k < d; ++k) {
        if (x[k] < lo0) lo0 = x[k];
        if (x[k] > hi0) hi0 = x[k];
    }
    /* -0 and +0 are the same number, so "min X" and "max X" (Algorithm 1, lines 1-2) do not say which
       one a zero bound is when a row holds both: a zero bound is taken as +0 (adding +0 does that and
       changes nothing else). */
    lo0 = lo0 + 0.0f;
    hi0 = hi0 + 0.0f;
    greedy_result best = {lo0, hi0, 0.0f, 0, 0};
    if (hi0 == lo0) /* constant row: stepsize is 0 and the loop of Algorithm 1 never runs */
        return best;

    best.loss = range_loss(x, d, lo0, hi0, qmax, work);
    float stepsize = (hi0 - lo0) / (float)n_bins;
    float cur_min = lo0, cur_max = hi0;
    int32_t i = 0, j = 0;

    for (int32_t it = 0; it < n_iter; ++it) {
        float next_min = cur_min + stepsize;
        float next_max = cur_max - stepsize;
        float loss_l = range_loss(x, d, next_min, cur_max, qmax, work);
        float loss_r = range_loss(x, d, cur_min, next_max, qmax, work);
        if (loss_l < loss_r) {
            cur_min = next_min;
            ++i;
            if (loss_l < best.loss) {
                best.loss = loss_l;
                best.xmin = cur_min;
                best.i = i;
                if (!literal_alg1) { best.xmax = cur_max; best.j = j; }
            }
        } else {
            cur_max = next_max;
            ++j;
            if (loss_r < best.loss) {
                best.loss = loss_r;
                best.xmax = cur_max;
                best.j = j;
                if (!literal_alg1) { best.xmin = cur_min; best.i = i; }
            }
        }
    }
    return best;
}

/* Codes of Eq. 1 for the range [lo, hi], packed 8/nbits per byte, plus the stored parameters. */
static void encode_row(const float *x, int d, float lo, float hi, int nbits, uint8_t *codes,
                       uint16_t *scale_f16, uint16_t *bias_f16)
{
    float qmax = qmax_of(nbits);
    float scale32 = (hi - lo) / qmax;
    *scale_f16 = e4q_oracle_f32_to_f16(scale32);
    *bias_f16 = e4q_oracle_f32_to_f16(lo);
    float scale = e4q_oracle_f16_to_f32(*scale_f16);
    float bias = e4q_oracle_f16_to_f32(*bias_f16);
    float inv = (scale == 0.0f) ? 0.0f : 1.0f / scale;
    int per = 8 / nbits;
    int64_t nbytes = packed_bytes(d, nbits);
    for (int64_t b = 0; b < nbytes; ++b) {
        unsigned byte = 0;
        for (int s = 0; s < per; ++s) {
            int64_t k = b * per + s;
            unsigned q = (k < d) ? (unsigned)quantize_elem(x[k], scale, bias, inv, qmax) : 0u;
            byte |= q << (s * nbits); /* lowest bits = first element */
        }
        codes[b] = (uint8_t)byte;
    }
}

static void widen_row(const void *table, int dtype, int64_t row, int64_t row_stride, int d, float *dst)
{
    if (dtype == 0) {
        memcpy(dst, (const float *)table + row * row_stride, (size_t)d * sizeof(float));
    } else {
        const uint16_t *src = (const uint16_t *)table + row * row_stride;
        for (int k = 0; k < d; ++k) dst[k] = e4q_oracle_f16_to_f32(src[k]);
    }
}

/*
 * Row-wise greedy n-bit quantization of a table (Algorithm 1 per row, then Eq. 1); n = 2, 4 or 8.
 *   table       rows x dim, row-major with `row_stride` elements between rows,
 *               dtype 0 = binary32, 1 = binary16
 *   codes       rows x ceil(dim * nbits / 8) bytes out
 *   scale_f16, bias_f16   rows binary16 bit patterns out
 *   loss_out    optional (may be NULL): rows floats, the search's loss of the result
 *               (for constant rows: 0)
 *   ij_out      optional (may be NULL): rows x 2 int32, steps taken by xmin and by xmax
 * Returns 0, or -1 on bad arguments.
 */
int e4q_oracle_quantize_rowwise_greedy(const void *table, int dtype, int64_t rows, int32_t dim,
                                       int64_t row_stride, int32_t n_bins, float ratio,
                                       int literal_alg1, uint8_t *codes, uint16_t *scale_f16,
                                       uint16_t *bias_f16, float *loss_out, int32_t *ij_out, int32_t nbits)
{
    if (!nbits_ok(nbits)) return -1;
    float qmax = qmax_of(nbits);
    if (!table || !codes || !scale_f16 || !bias_f16 || rows < 0 || dim <= 0 || n_bins < 1 ||
        !(ratio >= 0.0f && ratio < 1.0f) || row_stride < dim || (dtype != 0 && dtype != 1))
        return -1;
    int32_t n_iter = e4q_oracle_n_iter(n_bins, ratio);
    int p = next_pow2(dim);
    float *x = (float *)malloc((size_t)dim * sizeof(float));
    float *work = (float *)malloc((size_t)p * sizeof(float));
    if (!x || !work) { free(x); free(work); return -1; }
    int64_t nbytes = packed_bytes(dim, nbits);
    for (int64_t r = 0; r < rows; ++r) {
        widen_row(table, dtype, r, row_stride, dim, x);
        greedy_result g = greedy_row(x, dim, n_bins, n_iter, literal_alg1, qmax, work);
        encode_row(x, dim, g.xmin, g.xmax, nbits, codes + r * nbytes, scale_f16 + r, bias_f16 + r);
        if (loss_out) loss_out[r] = g.loss;
        if (ij_out) { ij_out[2 * r] = g.i; ij_out[2 * r + 1] = g.j; }
    }
    free(x);
    free(work);
    return 0;
}

/* Eq. 2 of one row for an explicit range, in the oracle's arithmetic (for tests). */
float e4q_oracle_range_loss(const float *x, int32_t dim, float lo, float hi, int32_t nbits)
{
    float *work = (float *)malloc((size_t)next_pow2(dim) * sizeof(float));
    float l = range_loss(x, dim, lo, hi, qmax_of(nbits), work);
    free(work);
    return l;
}

/*
 * Exhaustive search over the grid Algorithm 1 walks on: every (i, j) with i + j <= n_iter,
 * range [min + i*stepsize, max - j*stepsize] (bounds formed by repeated addition, as the
 * algorithm forms them).  Writes the smallest loss and one (i, j) that attains it.
 */
int e4q_oracle_brute_force_row(const float *x, int32_t dim, int32_t n_bins, int32_t n_iter,
                               float *best_loss, int32_t *best_i, int32_t *best_j, int32_t nbits)
{
    if (!x || dim <= 0 || n_bins < 1 || n_iter < 0 || !nbits_ok(nbits)) return -1;
    float qmax = qmax_of(nbits);
    float *work = (float *)malloc((size_t)next_pow2(dim) * sizeof(float));
    float lo0 = x[0], hi0 = x[0];
    for (int k = 1; k < dim; ++k) {
        if (x[k] < lo0) lo0 = x[k];
        if (x[k] > hi0) hi0 = x[k];
    }
    lo0 = lo0 + 0.0f; /* a zero bound is +0, as in greedy_row */
    hi0 = hi0 + 0.0f;
    float stepsize = (hi0 - lo0) / (float)n_bins;
    float bl = INFINITY;
    int32_t bi = 0, bj = 0;
    float lo = lo0;
    for (int32_t i = 0; i <= n_iter; ++i) {
        float hi = hi0;
        for (int32_t j = 0; i + j <= n_iter; ++j) {
            float l = range_loss(x, dim, lo, hi, qmax, work);
            if (l < bl) { bl = l; bi = i; bj = j; }
            hi = hi - stepsize;
        }
        lo = lo + stepsize;
    }
    free(work);
    *best_loss = bl; *best_i = bi; *best_j = bj;
    return 0;
}

/* x_float = scale * x_int + bias (sentence after Eq. 1), one fused multiply-add per element. */
int e4q_oracle_dequantize(const uint8_t *codes, const uint16_t *scale_f16, const uint16_t *bias_f16,
                          int64_t rows, int32_t dim, float *out, int32_t nbits)
{
    if (!codes || !scale_f16 || !bias_f16 || !out || rows < 0 || dim <= 0 || !nbits_ok(nbits)) return -1;
    int per = 8 / nbits;
    unsigned mask = (1u << nbits) - 1u;
    int64_t nbytes = packed_bytes(dim, nbits);
    for (int64_t r = 0; r < rows; ++r) {
        float scale = e4q_oracle_f16_to_f32(scale_f16[r]);
        float bias = e4q_oracle_f16_to_f32(bias_f16[r]);
        for (int k = 0; k < dim; ++k) {
            uint8_t byte = codes[r * nbytes + k / per];
            unsigned q = (byte >> ((k % per) * nbits)) & mask;
            out[r * dim + k] = fmaf((float)q, scale, bias);
        }
    }
    return 0;
}
