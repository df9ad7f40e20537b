/*
 * e4q_oracle_sls.c -- CPU oracle for the 4-bit SparseLengthsSum operator of "Post-Training 4-bit
 * Quantization on Embedding Tables" (arXiv 1911.02079), Section 4 ("Efficient 4-bit Embedding
 * Operation Implementation", Table 1): the lookup operator that reads a row-wise 4-bit quantized
 * table -- for every bag, the rows named by the bag's indices are de-quantized
 * (x_float = scale * x_int + bias, sentence after Eq. 1) and summed.
 *
 * TEST INFRASTRUCTURE, NOT THE PRODUCT (see e4q_oracle.c): plain, slow, single-threaded; shares
 * nothing with the HIP library.
 *
 * Readings (the paper describes the operator, not its arithmetic):
 *   - bag b owns indices[offsets[b] .. offsets[b+1]); offsets has n_bags + 1 entries and is the
 *     exclusive prefix sum of the operator's LENGTHS input;
 *   - out[b][k] starts at +0 and adds the de-quantized values in index order, in binary32:
 *     acc = acc + fmaf(q, scale, bias) (one rounding for the de-quantizer, one for the add);
 *   - an index outside [0, rows) contributes nothing; an empty bag gives zeros;
 *   - table layout as the quantizer writes it: packed codes (low nibble = even element), binary16
 *     scale and bias arrays.
 *
 * Pins (tests/test_oracle_sls_pins.py): integer-valued tables against an exact sparse
 * incidence-matrix product; float tables against the float64 product; bags of one index reproduce
 * the de-quantizer; left-to-right accumulation order; empty bags and out-of-range indices.
 */
#include <math.h>
#include <stdint.h>

float e4q_oracle_f16_to_f32(uint16_t h);

int e4q_oracle_sparse_lengths_sum(const uint8_t *codes, const uint16_t *scale_f16, const uint16_t *bias_f16,
                                  int64_t rows, int32_t dim, const int64_t *indices,
                                  const int64_t *offsets, int64_t n_bags, float *out)
{
    if (!codes || !scale_f16 || !bias_f16 || !offsets || !out || rows < 0 || dim <= 0 || n_bags < 0)
        return -1;
    int64_t nbytes = (dim + 1) / 2;
    for (int64_t b = 0; b < n_bags; ++b) {
        for (int k = 0; k < dim; ++k) {
            float acc = 0.0f;
            for (int64_t i = offsets[b]; i < offsets[b + 1]; ++i) {
                int64_t r = indices[i];
                if (r < 0 || r >= rows) continue;
                uint8_t byte = codes[r * nbytes + k / 2];
                unsigned q = (k & 1) ? (byte >> 4) : (byte & 0xfu);
                float x = fmaf((float)q, e4q_oracle_f16_to_f32(scale_f16[r]), e4q_oracle_f16_to_f32(bias_f16[r]));
                acc = acc + x;
            }
            out[b * dim + k] = acc;
        }
    }
    return 0;
}

/*
 * Fused row layout for lookups: one record per row, `row_pitch` bytes apart, holding the row's
 * packed codes followed (at the next even offset) by its binary16 scale and bias -- everything a
 * lookup of that row needs sits in one place.  The layout is this build's own choice: Section 4 and
 * Table 1 define what the lookup operator computes and time it, and describe no record layout.
 *   record = [ codes: ceil(dim/2) bytes ][ pad to even ][ scale: 2 bytes ][ bias: 2 bytes ][ pad ]
 * Padding bytes are written as 0.  Returns -1 if row_pitch is odd or too small.
 */
int e4q_oracle_fuse_rows(const uint8_t *codes, const uint16_t *scale_f16, const uint16_t *bias_f16,
                         int64_t rows, int32_t dim, int64_t row_pitch, uint8_t *fused)
{
    int64_t nbytes = (dim + 1) / 2;
    int64_t params_at = (nbytes + 1) & ~(int64_t)1;
    if (!codes || !scale_f16 || !bias_f16 || !fused || rows < 0 || dim <= 0 || (row_pitch & 1) ||
        row_pitch < params_at + 4)
        return -1;
    for (int64_t r = 0; r < rows; ++r) {
        uint8_t *rec = fused + r * row_pitch;
        for (int64_t k = 0; k < row_pitch; ++k) rec[k] = 0;
        for (int64_t k = 0; k < nbytes; ++k) rec[k] = codes[r * nbytes + k];
        rec[params_at + 0] = (uint8_t)(scale_f16[r] & 0xff);
        rec[params_at + 1] = (uint8_t)(scale_f16[r] >> 8);
        rec[params_at + 2] = (uint8_t)(bias_f16[r] & 0xff);
        rec[params_at + 3] = (uint8_t)(bias_f16[r] >> 8);
    }
    return 0;
}
