/*
 * e4q_oracle_kmeans.c -- CPU oracle for the row-wise 16-value codebook ("KMEANS") of
 * "Post-Training 4-bit Quantization on Embedding Tables" (arXiv 1911.02079).
 *
 * TEST INFRASTRUCTURE, NOT THE PRODUCT (see e4q_oracle.c): plain, slow, single-threaded; shares
 * nothing with the HIP library.
 *
 * What it follows: Section 3, "Codebook-based Quantization" -- k-means clustering of each row
 * vector into a 16-value codebook, each value replaced by the index of its cluster; Section 5 --
 * cluster centres initialised from the uniform quantization grid of ASYM, codebooks stored in
 * binary16 ("(FP16)").  Bytes per row: d/2 of indices + 16 * 2 of codebook (Table 3, KMEANS row).
 *
 * The paper names the method and its initialisation but not the iteration details.  Readings:
 *   - Lloyd's algorithm with a FIXED number of rounds (`lloyd_iters`, no convergence test);
 *   - initial centres c_k = min + k * (max - min)/15, k = 0..15, in binary32 (one division, then
 *     a fused multiply-add per centre);
 *   - assignment: nearest centre by |x - c_k| computed in binary32, the first (lowest) index
 *     among equal distances;
 *   - update: mean of the assigned values, summed in binary64 in index order, one binary64
 *     division by the count, rounded to binary32; a cluster with no member keeps its centre;
 *   - after the last round the centres are rounded to binary16, and the emitted indices are the
 *     nearest ROUNDED centre (same distance rule), so indices and stored codebook are consistent;
 *   - rows with dim <= 16 need no clustering: codebook entry k is the binary16 rounding of
 *     element k (unused entries are +0) and index k is k (Table 2 prints a loss of 0 for KMEANS
 *     at d = 8 and 16, which grid-initialised Lloyd rounds alone would not guarantee);
 *   - index packing as for the uniform codes: low nibble = even element.
 *
 * Pins (tests/test_oracle_kmeans_pins.py): rows already on a populated 16-point grid are
 * reproduced exactly; dim <= 16 is lossless up to binary16; the Lloyd objective never increases
 * from round to round and is never above the min/max grid's; exact rational Lloyd rounds on
 * integer lattices; scikit-learn's Lloyd with the same initial centres on rows where no cluster
 * runs empty; the optimal 1-D clustering (dynamic programme) as a lower bound; Table 3's size
 * column.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

uint16_t e4q_oracle_f32_to_f16(float f);
float e4q_oracle_f16_to_f32(uint16_t h);

#define K 16

static int nearest_centre(float x, const float *c)
{
    int best = 0;
    float bd = fabsf(x - c[0]);
    for (int k = 1; k < K; ++k) {
        float dk = fabsf(x - c[k]);
        if (dk < bd) { bd = dk; best = k; }
    }
    return best;
}

static void load_row(const void *table, int dtype, int64_t row, int64_t row_stride, int d, float *dst)
{
    if (dtype == 0) {
        memcpy(dst, (const float *)table + row * row_stride, (size_t)d * sizeof(float));
    } else {
        const uint16_t *src = (const uint16_t *)table + row * row_stride;
        for (int k = 0; k < d; ++k) dst[k] = e4q_oracle_f16_to_f32(src[k]);
    }
}

/* `lloyd_iters` rounds of (assign, update) from the min/max grid; c receives the 16 centres. */
static void lloyd_row(const float *x, int d, int lloyd_iters, float *c)
{
    float lo = x[0], hi = x[0];
    for (int k = 1; k < d; ++k) {
        if (x[k] < lo) lo = x[k];
        if (x[k] > hi) hi = x[k];
    }
    float step = (hi - lo) / 15.0f;
    for (int k = 0; k < K; ++k) c[k] = fmaf((float)k, step, lo);
    for (int it = 0; it < lloyd_iters; ++it) {
        double sum[K] = {0};
        int cnt[K] = {0};
        for (int e = 0; e < d; ++e) {
            int a = nearest_centre(x[e], c);
            sum[a] += (double)x[e];
            cnt[a]++;
        }
        for (int k = 0; k < K; ++k)
            if (cnt[k] > 0) c[k] = (float)(sum[k] / (double)cnt[k]);
    }
}

/*
 *   table          rows x dim, row-major, `row_stride` elements between rows, dtype 0 = binary32,
 *                  1 = binary16
 *   idx            rows x ceil(dim/2) bytes out (two 4-bit indices per byte)
 *   centroids_f16  rows x 16 binary16 bit patterns out
 *   centres_f32    optional (may be NULL): rows x 16 floats, the centres before binary16 rounding
 */
int e4q_oracle_quantize_rowwise_kmeans16(const void *table, int dtype, int64_t rows, int32_t dim,
                                         int64_t row_stride, int32_t lloyd_iters, uint8_t *idx,
                                         uint16_t *centroids_f16, float *centres_f32)
{
    if (!table || !idx || !centroids_f16 || rows < 0 || dim <= 0 || lloyd_iters < 0 ||
        row_stride < dim || (dtype != 0 && dtype != 1))
        return -1;
    float *x = (float *)malloc((size_t)dim * sizeof(float));
    if (!x) return -1;
    int64_t nbytes = (dim + 1) / 2;
    for (int64_t r = 0; r < rows; ++r) {
        load_row(table, dtype, r, row_stride, dim, x);
        uint16_t *cb = centroids_f16 + r * K;
        uint8_t *out = idx + r * nbytes;
        float c[K];
        if (dim <= K) {
            for (int k = 0; k < K; ++k) c[k] = (k < dim) ? x[k] : 0.0f;
            for (int k = 0; k < K; ++k) cb[k] = e4q_oracle_f32_to_f16(c[k]);
            for (int b = 0; b < nbytes; ++b) {
                unsigned q0 = (unsigned)(2 * b);
                unsigned q1 = (2 * b + 1 < dim) ? (unsigned)(2 * b + 1) : 0u;
                out[b] = (uint8_t)(q0 | (q1 << 4));
            }
        } else {
            lloyd_row(x, dim, lloyd_iters, c);
            float ch[K];
            for (int k = 0; k < K; ++k) {
                cb[k] = e4q_oracle_f32_to_f16(c[k]);
                ch[k] = e4q_oracle_f16_to_f32(cb[k]);
            }
            for (int b = 0; b < nbytes; ++b) {
                unsigned q0 = (unsigned)nearest_centre(x[2 * b], ch);
                unsigned q1 = (2 * b + 1 < dim) ? (unsigned)nearest_centre(x[2 * b + 1], ch) : 0u;
                out[b] = (uint8_t)(q0 | (q1 << 4));
            }
        }
        if (centres_f32) memcpy(centres_f32 + r * K, c, sizeof(c));
    }
    free(x);
    return 0;
}

/* Codebook dequantizer: out[r][k] = codebook[r][index[r][k]]. */
int e4q_oracle_dequantize_codebook(const uint8_t *idx, const uint16_t *centroids_f16, int64_t rows,
                                   int32_t dim, float *out)
{
    if (!idx || !centroids_f16 || !out || rows < 0 || dim <= 0) return -1;
    int64_t nbytes = (dim + 1) / 2;
    for (int64_t r = 0; r < rows; ++r)
        for (int k = 0; k < dim; ++k) {
            uint8_t byte = idx[r * nbytes + k / 2];
            unsigned q = (k & 1) ? (byte >> 4) : (byte & 0xfu);
            out[r * dim + k] = e4q_oracle_f16_to_f32(centroids_f16[r * K + q]);
        }
    return 0;
}
