/*
 * e4q.h -- C ABI of libe4q: row-wise 4-bit quantization of embedding tables on one
 * AMD MI355X (gfx950), after "Post-Training 4-bit Quantization on Embedding Tables"
 * (arXiv 1911.02079).
 *
 * Conventions that hold for every call
 * ------------------------------------
 *  - Every data pointer is a DEVICE pointer into memory the caller owns (for example a
 *    PyTorch tensor's storage).  The library never frees or reallocates caller memory, keeps
 *    no pointer after the call returns, and allocates nothing that outlives a call.
 *  - `hip_stream` is a hipStream_t passed as an opaque pointer (NULL = the null stream).
 *    Calls are asynchronous: kernels are enqueued on that stream and the call returns; the
 *    library never synchronises the device.  Inputs must stay valid and outputs must not be
 *    read until the stream has reached the end of the enqueued work.
 *  - The current HIP device must be the one that owns the buffers.
 *  - Return value: E4Q_OK (0) on success, a negative E4Q_ERR_* code otherwise; no exception
 *    or signal crosses the boundary.  Arguments are validated before anything is launched, so
 *    a failed call has written nothing.  rows == 0 is a successful no-op.
 *  - Tables are row-major.  `row_stride` is the distance between consecutive rows in ELEMENTS
 *    (>= dim).  Packed codes are dense: 8/nbits codes per byte, ceil(dim * nbits / 8) bytes per
 *    row, no padding between rows; the first element of a byte sits in its lowest bits (nbits = 4:
 *    element 2k in the low nibble and element 2k+1 in the high nibble of byte k); unused bits of a
 *    row's last byte are 0.  scale, bias and codebook entries are IEEE binary16 bit
 *    patterns stored as uint16_t.
 *  - Inputs containing NaN or infinities, and rows whose minimum or range exceeds the
 *    binary16 range (65504), give unspecified codes and parameters (never a fault).
 */
#ifndef E4Q_H
#define E4Q_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* Error codes. */
#define E4Q_OK 0
#define E4Q_ERR_NULL_POINTER (-1)   /* a required pointer is NULL */
#define E4Q_ERR_BAD_SHAPE (-2)      /* rows < 0 or > E4Q_MAX_ROWS, dim <= 0 or > E4Q_MAX_DIM, row_stride < dim, bad row_pitch */
#define E4Q_ERR_BAD_NBITS (-3)      /* nbits not in {2, 4, 8} (quantizer, dequantizer) or != 4 (lookup operator) */
#define E4Q_ERR_BAD_SEARCH (-4)     /* n_bins < 1, ratio outside [0, 1), ratio NaN, lloyd_iters < 0 */
#define E4Q_ERR_BAD_DTYPE (-5)      /* dtype is neither E4Q_F32 nor E4Q_F16; index_bytes is neither 4 nor 8 */
#define E4Q_ERR_LAUNCH (-6)         /* HIP reported an error when the kernel was enqueued */
#define E4Q_ERR_BAD_ALIGNMENT (-7)  /* table pointer not aligned to its element size */
#define E4Q_ERR_BAD_OPTION (-8)     /* unknown diagnostic option or value; a forced layout that cannot hold the call's dim */

/* Element type of an input table. */
#define E4Q_F32 0
#define E4Q_F16 1

/* Largest supported embedding dimension, row count and bag count.  (A grid dimension holds fewer
 * than 2^32 work-items; launches that need more are folded into two dimensions inside the library.) */
#define E4Q_MAX_DIM 4096
#define E4Q_MAX_ROWS 2147483648LL

/*
 * Row-wise uniform n-bit quantization (n = 4 in the paper) with greedy search of the clipping range
 * (Algorithm 1; quantizer and stored parameters of Eq. 1; loss of Eq. 2; binary16 scale and
 * bias as in the "(FP16)" variants of Section 5).
 *
 * For each row X independently: start from [min X, max X], stepsize = (max - min)/n_bins;
 * n_iter = ceil(n_bins * ratio) times (at most n_bins - 1) score "lower bound up one step"
 * against "upper bound down one step" by the squared quantize->dequantize error of the row,
 * move the bound with the smaller error (ties move the upper bound) and remember the range
 * with the smallest error seen (strictly smaller replaces; the pair of bounds is remembered
 * together).  The row is then encoded with that range: scale = (xmax - xmin)/(2^nbits - 1) and bias =
 * xmin rounded to binary16, code = clamp(round_half_even((x - bias) * (1/scale)), 0, 2^nbits - 1),
 * all in binary32.  Candidates are scored with the binary16-rounded parameters, i.e. with
 * what is stored.  ratio == 0 gives plain min/max ("ASYM") quantization.  A row with
 * max == min, or whose scale rounds to 0 in binary16, gets scale 0 and all codes 0.  A row's minimum
 * or maximum that is zero is taken as +0 whichever zeros the row holds (-0 = +0, and Algorithm 1 does
 * not say which one "min X" is): such a minimum is stored as the bias 0x0000, never 0x8000.
 *
 *   table       [in]  rows x dim elements of `dtype`, `row_stride` elements between rows
 *   dtype             E4Q_F32 or E4Q_F16 (binary16 inputs are widened exactly)
 *   nbits             4 (the paper's subject); 8 (its ASYM-8BITS baseline, Section 5) and 2 are
 *                     accepted too and differ only in the number of levels and the packing
 *   n_bins            b of Algorithm 1 (default in the paper: 200)
 *   ratio             r of Algorithm 1 (default in the paper: 0.16), 0 <= ratio < 1
 *   codes       [out] rows x ceil(dim * nbits / 8) bytes
 *   scale_f16   [out] rows binary16 values
 *   bias_f16    [out] rows binary16 values
 */
int e4q_quantize_rowwise_greedy(const void* table, int dtype, int64_t rows, int32_t dim,
                                int64_t row_stride, int32_t nbits, int32_t n_bins, float ratio,
                                uint8_t* codes, uint16_t* scale_f16, uint16_t* bias_f16,
                                void* hip_stream);

/*
 * De-quantization x_float = scale * x_int + bias (the sentence after Eq. 1), one fused
 * multiply-add per element in binary32.
 *
 *   codes, scale_f16, bias_f16  [in]  as written by e4q_quantize_rowwise_greedy
 *   out                         [out] rows x dim binary32, dense (row stride = dim)
 */
int e4q_dequantize(const uint8_t* codes, const uint16_t* scale_f16, const uint16_t* bias_f16,
                   int64_t rows, int32_t dim, int32_t nbits, float* out, void* hip_stream);

/*
 * One table of a batch.  The array of descriptors itself lives in HOST memory and is only
 * read during the call; the pointers inside are device pointers with the meaning they have in
 * e4q_quantize_rowwise_greedy.
 */
typedef struct e4q_table_desc {
    const void* table;
    int32_t dtype;
    int32_t dim;
    int64_t rows;
    int64_t row_stride;
    uint8_t* codes;
    uint16_t* scale_f16;
    uint16_t* bias_f16;
} e4q_table_desc;

/*
 * Greedy quantization (as above) of `n_tables` tables in one launch sequence on one stream:
 * all descriptors are validated first, then every table's work is enqueued back to back with
 * no host synchronisation in between (tables that share a dimension and an input type may share a
 * launch).  On a validation error nothing is enqueued; E4Q_ERR_LAUNCH can leave earlier tables of
 * the batch enqueued.
 */
int e4q_quantize_rowwise_greedy_batch(const e4q_table_desc* descs, int32_t n_tables,
                                      int32_t nbits, int32_t n_bins, float ratio,
                                      void* hip_stream);

/*
 * Row-wise codebook quantization ("KMEANS": Section 3, "Codebook-based Quantization"; initial
 * centres and binary16 codebooks as in Section 5).  For each row independently, 1-D k-means with
 * 16 centres: centres start on the uniform grid min + k*(max-min)/15; `lloyd_iters` rounds of
 * (assign every value to its nearest centre -- |x - c| in binary32, the lowest index among equal
 * distances --, move every non-empty cluster's centre to the mean of its members -- summed in
 * binary64 in element order, one division, rounded to binary32); no convergence test.  The
 * centres are then rounded to binary16 and each value is stored as the 4-bit index of its nearest
 * ROUNDED centre.  Rows with dim <= 16 are not clustered: codebook entry k is element k rounded
 * to binary16 (unused entries +0) and index k is k.
 *
 *   table, dtype, rows, dim, row_stride   as for e4q_quantize_rowwise_greedy
 *   lloyd_iters          >= 0 (the benchmark configuration uses 20)
 *   idx            [out] rows x ceil(dim/2) bytes, two indices per byte, low nibble first
 *   centroids_f16  [out] rows x 16 binary16 values (32 bytes per row, dense)
 * Bytes per row: dim/2 + 32 (the KMEANS (FP16) sizes of Table 3).
 *
 * (Diagnostic option "kmeans_force_scan", see e4q_set_option: the kernels then find the nearest
 * centre by scanning all 16 instead of bisecting the ordered centres; same outputs bit for bit.)
 */
int e4q_quantize_rowwise_kmeans16(const void* table, int dtype, int64_t rows, int32_t dim,
                                  int64_t row_stride, int32_t lloyd_iters, uint8_t* idx,
                                  uint16_t* centroids_f16, void* hip_stream);

/*
 * Codebook de-quantization: out[r][k] = codebook[r][index[r][k]] widened to binary32
 * (Section 3: each value is represented by the codebook entry its index names).
 *   out  [out] rows x dim binary32, dense
 */
int e4q_dequantize_codebook(const uint8_t* idx, const uint16_t* centroids_f16, int64_t rows, int32_t dim,
                            float* out, void* hip_stream);

/*
 * 4-bit SparseLengthsSum: the pooled embedding lookup that reads the quantized table (Section 4,
 * "Efficient 4-bit Embedding Operation Implementation", Table 1).  Bag b owns
 * indices[offsets[b] .. offsets[b+1]); out[b][k] = sum over the bag of scale[r] * code[r][k] + bias[r],
 * accumulated from +0 in index order in binary32 (the de-quantizer is one fused multiply-add, the
 * accumulation a separate add).  An empty bag gives zeros; an index outside [0, rows) adds
 * nothing; offsets are clamped to [0, n_indices], so malformed offsets cannot cause a fault.
 *
 *   codes, scale_f16, bias_f16  [in]  the table, as written by e4q_quantize_rowwise_greedy
 *   indices      [in]  n_indices row numbers, int32 (index_bytes = 4) or int64 (index_bytes = 8)
 *   offsets      [in]  n_bags + 1 int64 values, non-decreasing: the exclusive prefix sum of the
 *                      operator's LENGTHS input
 *   out          [out] n_bags x dim binary32, dense
 */
int e4q_sparse_lengths_sum(const uint8_t* codes, const uint16_t* scale_f16, const uint16_t* bias_f16,
                           int64_t rows, int32_t dim, int32_t nbits, const void* indices, int32_t index_bytes,
                           int64_t n_indices, const int64_t* offsets, int64_t n_bags, float* out,
                           void* hip_stream);

/*
 * Fused lookup records.  A lookup of one row needs its codes, its scale and its bias; kept in
 * three arrays they sit in three different places of HBM.  e4q_fuse_rows copies a quantized table
 * into one record per row, `row_pitch` bytes apart:
 *     [ codes: ceil(dim/2) bytes ][ pad to an even offset ][ scale f16 ][ bias f16 ][ pad: zeros ]
 * This record layout is a choice of this library, not the paper's: Section 4 and Table 1 say what
 * the lookup operator computes (4-bit rows are read and de-quantized while they are summed) and time
 * it in sums per second, and describe no memory layout.
 * e4q_fused_row_bytes(dim) is the smallest record (dim/2 + 4 for even dim/2: the d/2 + 4 bytes per
 * row behind Table 3's sizes); row_pitch must be even and at least that (for example 128 to give
 * every record of a dim-128 table its own 128-byte line).  Host-only helper; negative on bad dim.
 *
 *   fused  [out] rows * row_pitch bytes
 */
int64_t e4q_fused_row_bytes(int32_t dim);
int e4q_fuse_rows(const uint8_t* codes, const uint16_t* scale_f16, const uint16_t* bias_f16, int64_t rows,
                  int32_t dim, int32_t nbits, int64_t row_pitch, uint8_t* fused, void* hip_stream);

/*
 * e4q_sparse_lengths_sum over fused records (same arithmetic, same result bit for bit; about one
 * half to one third of the HBM traffic per lookup).
 */
int e4q_sparse_lengths_sum_fused(const uint8_t* fused, int64_t rows, int32_t dim, int32_t nbits, int64_t row_pitch,
                                 const void* indices, int32_t index_bytes, int64_t n_indices,
                                 const int64_t* offsets, int64_t n_bags, float* out, void* hip_stream);

/*
 * n_iter = ceil(n_bins * ratio) clamped to [0, n_bins - 1]: the number of trips of the loop of
 * Algorithm 1 in exact arithmetic (each trip scores two candidate ranges).  `ratio` is a
 * binary32 number and may sit a relative 2^-24 off the decimal the caller wrote, so the product
 * is shrunk by a relative 2^-22 before the ceiling.  Host-only helper; returns a negative
 * error code for invalid arguments.
 */
int32_t e4q_greedy_iterations(int32_t n_bins, float ratio);

/*
 * Diagnostic options, for tests, benchmarks and profiling (no passage of the paper: they change how
 * a result is computed, never the result).  Process-wide, initially 0, read once per call by the
 * entry points they concern; setting one while another thread is inside such a call affects that
 * call or the next.  Host-only.
 *
 *   "greedy_layout"      0: the library picks the thread layout of the greedy search (default).
 *                        1: one table row per lane (dim <= 224 only).
 *                        (E << 8) | L: L lanes per row with E contiguous elements each,
 *                        E in {8, 16, 32, 64, 128}, 1 <= L <= 64 (not 64 for E = 128); an L that is not a
 *                        power of two leaves 64 % L lanes of every wave idle.
 *                        (1 << 16) | (E << 8) | L: two such groups of L lanes per row, each holding the whole
 *                        row; the two candidate ranges of every trip of Algorithm 1's loop are scored at the
 *                        same time, one by each group (for small tables, where the duration of the launch is
 *                        the duration of one wave).  E in {8, 16}, L a power of two up to 32.
 *                        A forced layout needs E * L >= dim; the quantize calls return
 *                        E4Q_ERR_BAD_OPTION otherwise.  The batch call then launches table by table.
 *   "kmeans_force_scan"  1: e4q_quantize_rowwise_kmeans16 scans all 16 centres for every value
 *                        instead of bisecting (the path otherwise taken only by rows whose centres
 *                        fall out of order).
 *   "sls_nontemporal"    1: e4q_sparse_lengths_sum_fused gathers records with non-temporal loads.
 *   "workgroup_waves"    1 or 4: waves per workgroup of the kernels that give every table row a lane of its own (the
 *                        greedy search in the one-row-per-lane layout, single tables and grouped batch launches, and
 *                        the register-resident 16-means kernels); 0: the library chooses by the number of rows (four
 *                        for small launches, whose waves then land one on each SIMD of a compute unit).  Kernels
 *                        that stage rows in LDS per workgroup keep their own size.
 *   "greedy_layout_chosen"  read-only (e4q_get_option): the layout the last table handed to a
 *                        single-table greedy launch ran with, in the encoding of "greedy_layout"
 *                        (0 before the first such launch); grouped batch launches, which are
 *                        always one row per lane, do not change it.
 *
 * e4q_set_option returns E4Q_OK, or E4Q_ERR_BAD_OPTION for an unknown name or a value the option
 * does not take (nothing changes then).  e4q_get_option returns the value, or E4Q_ERR_BAD_OPTION.
 */
int e4q_set_option(const char* name, int64_t value);
int64_t e4q_get_option(const char* name);

/*
 * The estimate behind the automatic choice of "greedy_layout": SIMD cycles the greedy search of a
 * rows x dim table with n_iter trips would take in the given layout (encoding of "greedy_layout",
 * not 0), from the instruction count of the layout and the issue rates measured on gfx950.  The
 * library runs the layout with the smallest estimate.  Diagnostic, host-only; negative if the layout
 * cannot hold a row of `dim` elements or an argument is out of range.
 */
double e4q_greedy_layout_cost(int64_t rows, int32_t dim, int32_t n_iter, int64_t layout);

/* Static, human-readable text for a return code (never NULL). */
const char* e4q_strerror(int code);

/* Text of the last HIP error seen by this thread inside the library ("" if none). */
const char* e4q_last_hip_error(void);

/* Library version: major * 10000 + minor * 100 + patch. */
int e4q_version(void);

#ifdef __cplusplus
}
#endif
#endif /* E4Q_H */
