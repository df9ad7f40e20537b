// 4-bit SparseLengthsSum (Section 4, "Efficient 4-bit Embedding Operation Implementation", Table 1):
// for every bag, gather the rows its indices name from a row-wise 4-bit table, de-quantize them
// (x_float = scale * x_int + bias) and add them up.
//
// Bound by HBM gathers: d/2 bytes of codes plus two binary16 parameters per looked-up row, at
// random rows.  One thread owns 8 consecutive elements of one bag (one 32-bit word of every row it
// gathers) and accumulates them left to right in binary32, so the result does not depend on the
// launch shape.  The index stream of a bag is read four at a time so that four row gathers are in
// flight per thread; the accumulation order stays the index order.  Indices outside [0, rows) add
// nothing; offsets are clamped to [0, n_indices], so no input can cause an out-of-range read.
#include "e4q_device.h"
#include "e4q_index.h"
#include "e4q_launch.h"

namespace e4q {

constexpr int kSlsBlock = 256;
typedef float floatx4 __attribute__((ext_vector_type(4)));

// Adds the eight de-quantized codes of one 32-bit word.  The even and the odd nibbles are first spread over the
// bytes of two words, so that each code is one byte-to-float conversion away (two masks and a shift per word
// instead of a bit-field extract per code).
__device__ __forceinline__ void sls_add_word(float (&acc)[8], uint32_t c, float s, float b)
{
    uint32_t even = c & 0x0f0f0f0fu, odd = (c >> 4) & 0x0f0f0f0fu;
    asm("" : "+v"(even));  // or the optimizer folds the masks back into one extract per code
    asm("" : "+v"(odd));
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        acc[2 * k] = acc[2 * k] + __builtin_fmaf((float)((even >> (8 * k)) & 0xffu), s, b);
        acc[2 * k + 1] = acc[2 * k + 1] + __builtin_fmaf((float)((odd >> (8 * k)) & 0xffu), s, b);
    }
}

// A gathered row as it was read: one word of codes, the binary16 scale and bias, and whether the index was inside
// the table.  Nothing is converted or dropped before all the rows in flight have been requested (no branch and
// no wait between the loads of different rows); an index outside the table reads row 0 and is dropped when
// it is added (scale = bias = 0 make every term fma(q, 0, 0) = +0).  Needs rows > 0.
struct SlsRow {
    uint32_t c;
    uint16_t s, b;
    bool ok;
};

template <typename Tidx>
__device__ __forceinline__ SlsRow sls_gather(const uint32_t* __restrict__ codes, const uint16_t* __restrict__ sc,
                                             const uint16_t* __restrict__ bi, int64_t rows, uint32_t wpr,
                                             uint32_t word, Tidx idx)
{
    const int64_t r = (int64_t)idx;
    SlsRow g;
    g.ok = r >= 0 && r < rows;
    const int64_t rr = g.ok ? r : 0;
    g.c = codes[rr * wpr + word];
    g.s = sc[rr];
    g.b = bi[rr];
    return g;
}

__device__ __forceinline__ void sls_add_row(float (&acc)[8], const SlsRow& g)
{
    sls_add_word(acc, g.c, f16_bits_to_float(g.ok ? g.s : (uint16_t)0), f16_bits_to_float(g.ok ? g.b : (uint16_t)0));
}

// dim % 8 == 0, codes 4-byte aligned, out 16-byte aligned.
template <typename Tidx>
__global__ void __launch_bounds__(kSlsBlock) sls_w8_kernel(const uint32_t* __restrict__ codes,
                                                           const uint16_t* __restrict__ sc,
                                                           const uint16_t* __restrict__ bi, int64_t rows,
                                                           uint32_t wpr, const Tidx* __restrict__ indices,
                                                           int64_t n_indices, const int64_t* __restrict__ offsets,
                                                           int64_t n_bags, floatx4* __restrict__ out)
{
    const int64_t t = linear_block() * kSlsBlock + threadIdx.x;
    const int64_t n_threads = n_bags * wpr;
    if (t >= n_threads) return;  // tested in 64 bits: the padded grid may run past 2^32
    const int64_t bag = group_of(t, n_threads, wpr);
    const uint32_t word = offset_in_group(t, bag, wpr);
    const int64_t lo = offsets[bag], hi = offsets[bag + 1];
    const int64_t begin = lo < 0 ? 0 : (lo > n_indices ? n_indices : lo);
    const int64_t end = (hi < begin || rows == 0) ? begin : (hi > n_indices ? n_indices : hi);  // empty table: no row 0

    float acc[8] = {0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f};
    int64_t i = begin;
    for (; i + 4 <= end; i += 4) {
        const Tidx i0 = indices[i], i1 = indices[i + 1], i2 = indices[i + 2], i3 = indices[i + 3];
        const SlsRow g0 = sls_gather(codes, sc, bi, rows, wpr, word, i0);
        const SlsRow g1 = sls_gather(codes, sc, bi, rows, wpr, word, i1);
        const SlsRow g2 = sls_gather(codes, sc, bi, rows, wpr, word, i2);
        const SlsRow g3 = sls_gather(codes, sc, bi, rows, wpr, word, i3);
        __builtin_amdgcn_sched_barrier(0);  // all twelve loads are on their way before the first row is unpacked
        sls_add_row(acc, g0);
        sls_add_row(acc, g1);
        sls_add_row(acc, g2);
        sls_add_row(acc, g3);
    }
    for (; i < end; ++i) sls_add_row(acc, sls_gather(codes, sc, bi, rows, wpr, word, indices[i]));
    floatx4 v0 = {acc[0], acc[1], acc[2], acc[3]}, v1 = {acc[4], acc[5], acc[6], acc[7]};
    out[2 * t] = v0;
    out[2 * t + 1] = v1;
}

// The same row with its parameters already widened (the generic kernels below fill it piece by piece).
struct SlsRowF {
    uint32_t c;
    float s, b;
};

// Any dim, pitch and alignment, 8 elements per thread: the loop shared by the two kernels below.
// `gather(r)` returns code word `word` of row r (bytes beyond the row's codes read as 0) and its
// parameters, all zero for an index outside the table.  Only the elements that exist are stored.
template <typename Tidx, class Gather>
__device__ __forceinline__ void sls_bytes_body(Gather&& gather, uint32_t dim, uint32_t word,
                                               const Tidx* __restrict__ indices, int64_t n_indices,
                                               const int64_t* __restrict__ offsets, int64_t bag,
                                               float* __restrict__ out)
{
    const int64_t lo = offsets[bag], hi = offsets[bag + 1];
    const int64_t begin = lo < 0 ? 0 : (lo > n_indices ? n_indices : lo);
    const int64_t end = hi < begin ? begin : (hi > n_indices ? n_indices : hi);
    float acc[8] = {0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f};
    int64_t i = begin;
    for (; i + 4 <= end; i += 4) {
        const Tidx i0 = indices[i], i1 = indices[i + 1], i2 = indices[i + 2], i3 = indices[i + 3];
        const SlsRowF g0 = gather((int64_t)i0), g1 = gather((int64_t)i1), g2 = gather((int64_t)i2), g3 = gather((int64_t)i3);
        sls_add_word(acc, g0.c, g0.s, g0.b);
        sls_add_word(acc, g1.c, g1.s, g1.b);
        sls_add_word(acc, g2.c, g2.s, g2.b);
        sls_add_word(acc, g3.c, g3.s, g3.b);
    }
    for (; i < end; ++i) {
        const SlsRowF g = gather((int64_t)indices[i]);
        sls_add_word(acc, g.c, g.s, g.b);
    }
    float* o = out + bag * dim + 8 * word;
#pragma unroll
    for (int e = 0; e < 8; ++e)
        if (8 * word + e < dim) o[e] = acc[e];
}

// Reads up to four code bytes at p (those below `limit` bytes from the row start at offset `at`).
__device__ __forceinline__ uint32_t sls_code_bytes(const uint8_t* __restrict__ p, uint32_t at, uint32_t limit)
{
    uint32_t c = 0;
#pragma unroll
    for (uint32_t j = 0; j < 4; ++j)
        if (at + j < limit) c |= (uint32_t)p[at + j] << (8 * j);
    return c;
}

// Separate arrays, any dim and alignment: one thread per 8 output elements, byte reads.
template <typename Tidx>
__global__ void __launch_bounds__(kSlsBlock) sls_bytes_kernel(const uint8_t* __restrict__ codes,
                                                              const uint16_t* __restrict__ sc,
                                                              const uint16_t* __restrict__ bi, int64_t rows,
                                                              uint32_t dim, const Tidx* __restrict__ indices,
                                                              int64_t n_indices, const int64_t* __restrict__ offsets,
                                                              int64_t n_bags, float* __restrict__ out)
{
    const uint32_t wpr = (dim + 7) / 8, nbytes = (dim + 1) / 2;
    const int64_t t = linear_block() * kSlsBlock + threadIdx.x;
    const int64_t n_threads = n_bags * wpr;
    if (t >= n_threads) return;
    const int64_t bag = group_of(t, n_threads, wpr);
    const uint32_t word = offset_in_group(t, bag, wpr);
    sls_bytes_body<Tidx>([&](int64_t r) {
        SlsRowF g = {0u, 0.0f, 0.0f};
        if (r >= 0 && r < rows) {
            g.c = sls_code_bytes(codes + r * nbytes, 4 * word, nbytes);
            g.s = f16_bits_to_float(sc[r]);
            g.b = f16_bits_to_float(bi[r]);
        }
        return g;
    }, dim, word, indices, n_indices, offsets, bag, out);
}

// Fused records, any dim and pitch: one thread per 8 output elements, 2-byte reads (records are 2-byte
// aligned: the buffer is, and the pitch is even; so are a record's code words and its parameters).
template <typename Tidx>
__global__ void __launch_bounds__(kSlsBlock) sls_fused_h8_kernel(const uint8_t* __restrict__ fused, int64_t rows,
                                                                 uint32_t dim, int64_t pitch,
                                                                 const Tidx* __restrict__ indices, int64_t n_indices,
                                                                 const int64_t* __restrict__ offsets, int64_t n_bags,
                                                                 float* __restrict__ out)
{
    const uint32_t wpr = (dim + 7) / 8, nbytes = (dim + 1) / 2;
    const uint32_t params_at = (nbytes + 1u) & ~1u;
    const int64_t t = linear_block() * kSlsBlock + threadIdx.x;
    const int64_t n_threads = n_bags * wpr;
    if (t >= n_threads) return;
    const int64_t bag = group_of(t, n_threads, wpr);
    const uint32_t word = offset_in_group(t, bag, wpr);
    sls_bytes_body<Tidx>([&](int64_t r) {
        SlsRowF g = {0u, 0.0f, 0.0f};
        if (r >= 0 && r < rows) {
            // both halves of the word lie inside the record (its parameters follow the codes)
            const uint16_t* h = reinterpret_cast<const uint16_t*>(fused + r * pitch);
            const uint32_t c = (uint32_t)h[2 * word] | ((uint32_t)h[2 * word + 1] << 16);
            const uint32_t valid = nbytes - 4 * word;  // code bytes in this word, if fewer than 4
            g.c = valid >= 4 ? c : (c & ((1u << (8 * valid)) - 1u));
            g.s = f16_bits_to_float(h[params_at / 2]);
            g.b = f16_bits_to_float(h[params_at / 2 + 1]);
        }
        return g;
    }, dim, word, indices, n_indices, offsets, bag, out);
}

// ---------------------------------------------------------------------------------------------
// Fused records: [codes | pad to even | scale f16 | bias f16 | pad] every `row_pitch` bytes, so
// that one lookup touches one place in memory instead of three (the separate scale and bias
// arrays cost a 128-byte line each per lookup).
// ---------------------------------------------------------------------------------------------

// Any shape: one thread per byte of the records.
__global__ void __launch_bounds__(kSlsBlock) fuse_rows_any_kernel(const uint8_t* __restrict__ codes,
                                                                  const uint16_t* __restrict__ sc,
                                                                  const uint16_t* __restrict__ bi, int64_t rows,
                                                                  uint32_t nbytes, uint32_t pitch,
                                                                  uint8_t* __restrict__ fused)
{
    const int64_t t = linear_block() * kSlsBlock + threadIdx.x;
    const int64_t r = t / pitch;
    if (r >= rows) return;
    const uint32_t k = (uint32_t)(t - r * pitch);
    const uint32_t params_at = (nbytes + 1u) & ~1u;
    uint8_t v = 0;
    if (k < nbytes) v = codes[r * nbytes + k];
    else if (k >= params_at && k < params_at + 2) v = (uint8_t)(sc[r] >> (8 * (k - params_at)));
    else if (k >= params_at + 2 && k < params_at + 4) v = (uint8_t)(bi[r] >> (8 * (k - params_at - 2)));
    fused[t] = v;
}

// nbytes % 4 == 0, pitch % 4 == 0, 4-byte aligned buffers: one thread per 32-bit word.
__global__ void __launch_bounds__(kSlsBlock) fuse_rows_w_kernel(const uint32_t* __restrict__ codes,
                                                                const uint16_t* __restrict__ sc,
                                                                const uint16_t* __restrict__ bi, int64_t rows,
                                                                uint32_t wpr, uint32_t pitch_words,
                                                                uint32_t* __restrict__ fused)
{
    const int64_t t = linear_block() * kSlsBlock + threadIdx.x;
    const int64_t r = t / pitch_words;
    if (r >= rows) return;
    const uint32_t k = (uint32_t)(t - r * pitch_words);
    uint32_t v = 0;
    if (k < wpr) v = codes[r * wpr + k];
    else if (k == wpr) v = (uint32_t)sc[r] | ((uint32_t)bi[r] << 16);
    fused[t] = v;
}

hipError_t launch_fuse_rows(const uint8_t* codes, const uint16_t* sc, const uint16_t* bi, int64_t rows,
                            int32_t dim, int64_t row_pitch, uint8_t* fused, hipStream_t stream)
{
    const uint32_t nbytes = (uint32_t)((dim + 1) / 2);
    const bool words = nbytes % 4 == 0 && row_pitch % 4 == 0 && reinterpret_cast<uintptr_t>(codes) % 4 == 0 &&
                       reinterpret_cast<uintptr_t>(fused) % 4 == 0;
    const int64_t threads = words ? rows * (row_pitch / 4) : rows * row_pitch;
    const int64_t blocks = blocks_for(threads, kSlsBlock);
    if (blocks < 0) return hipErrorInvalidValue;
    if (words)
        hipLaunchKernelGGL(fuse_rows_w_kernel, grid_for(blocks), dim3(kSlsBlock), 0, stream,
                           reinterpret_cast<const uint32_t*>(codes), sc, bi, rows, nbytes / 4,
                           (uint32_t)(row_pitch / 4), reinterpret_cast<uint32_t*>(fused));
    else
        hipLaunchKernelGGL(fuse_rows_any_kernel, grid_for(blocks), dim3(kSlsBlock), 0, stream, codes, sc, bi,
                           rows, nbytes, (uint32_t)row_pitch, fused);
    return hipGetLastError();
}

// Lookup over fused records; dim % 8 == 0, pitch % 4 == 0, 4-byte aligned records, 16-byte aligned out.
// One thread owns WPT consecutive code words (8 * WPT elements) of one bag.
template <typename Tidx, int WPT, bool NT, int G = 4>
__global__ void __launch_bounds__(kSlsBlock) sls_fused_w8_kernel(const uint32_t* __restrict__ fused, int64_t rows,
                                                                 uint32_t wpr, uint32_t pitch_words,
                                                                 const Tidx* __restrict__ indices, int64_t n_indices,
                                                                 const int64_t* __restrict__ offsets, int64_t n_bags,
                                                                 floatx4* __restrict__ out)
{
    typedef uint32_t words_t __attribute__((ext_vector_type(WPT), aligned(4)));
    const uint32_t tpb = wpr / WPT;  // threads per bag
    const int64_t t = linear_block() * kSlsBlock + threadIdx.x;
    const int64_t n_threads = n_bags * tpb;
    if (t >= n_threads) return;  // tested in 64 bits: the padded grid may run past 2^32
    const int64_t bag = group_of(t, n_threads, tpb);
    const uint32_t word = offset_in_group(t, bag, tpb) * WPT;
    const int64_t lo = offsets[bag], hi = offsets[bag + 1];
    const int64_t begin = lo < 0 ? 0 : (lo > n_indices ? n_indices : lo);
    const int64_t end = (hi < begin || rows == 0) ? begin : (hi > n_indices ? n_indices : hi);

    // A gathered record as it was read.  Scale and bias are converted, and a record of an index outside the table
    // is dropped, only when the record is added: the loads of all records in flight are issued first, and
    // nothing that waits for one of them stands between them.
    struct Rec {
        uint32_t c[WPT];
        uint32_t sb;  // scale in the low half, bias in the high half
        bool ok;      // the index was inside the table
    };
    // No branch: an index outside the table reads record 0, which is dropped later (scale = bias = 0 make every
    // term fma(q, 0, 0) = +0, whatever the codes).  With a branch per record the gathers of a round sit in
    // separate basic blocks and each waits for the one before it.  An empty table is kept away from here (no
    // record 0 to read: the bag loops then run over nothing).
    auto gather = [&](Tidx idx) {
        const int64_t r = (int64_t)idx;
        Rec g;
        g.ok = r >= 0 && r < rows;
        const uint32_t* rec = fused + (g.ok ? r : 0) * pitch_words;
        g.sb = NT ? __builtin_nontemporal_load(rec + wpr) : rec[wpr];
        if constexpr (WPT == 1) {
            g.c[0] = NT ? __builtin_nontemporal_load(rec + word) : rec[word];
        } else {
            const words_t* pv = reinterpret_cast<const words_t*>(rec + word);
            const words_t v = NT ? __builtin_nontemporal_load(pv) : *pv;
#pragma unroll
            for (int w = 0; w < WPT; ++w) g.c[w] = v[w];
        }
        return g;
    };
    float acc[WPT][8];
#pragma unroll
    for (int w = 0; w < WPT; ++w)
#pragma unroll
        for (int e = 0; e < 8; ++e) acc[w][e] = 0.0f;
    auto add = [&](const Rec& g) {
        const uint32_t sb = g.ok ? g.sb : 0u;
        const float sc = f16_bits_to_float((uint16_t)(sb & 0xffffu)), bi = f16_bits_to_float((uint16_t)(sb >> 16));
#pragma unroll
        for (int w = 0; w < WPT; ++w) sls_add_word(acc[w], g.c[w], sc, bi);
    };

    // Four gathers in flight per thread.  (Requesting the next four indices before the current records are added,
    // to take their latency out of the index -> record -> add chain, measured 4 - 12 % slower.)
    int64_t i = begin;
    for (; i + G <= end; i += G) {
        Tidx ix[G];
#pragma unroll
        for (int k = 0; k < G; ++k) ix[k] = indices[i + k];
        Rec g[G];
#pragma unroll
        for (int k = 0; k < G; ++k) g[k] = gather(ix[k]);
        __builtin_amdgcn_sched_barrier(0);  // all the loads are on their way before the first record is unpacked
#pragma unroll
        for (int k = 0; k < G; ++k) add(g[k]);
    }
    for (; i < end; ++i) add(gather(indices[i]));
    floatx4* o = out + 2 * (bag * wpr + word);
#pragma unroll
    for (int w = 0; w < WPT; ++w) {
        floatx4 v0 = {acc[w][0], acc[w][1], acc[w][2], acc[w][3]}, v1 = {acc[w][4], acc[w][5], acc[w][6], acc[w][7]};
        o[2 * w] = v0;
        o[2 * w + 1] = v1;
    }
}

template <typename Tidx>
static hipError_t launch_sls_fused_t(const uint8_t* fused, int64_t rows, int32_t dim, int64_t pitch,
                                     const void* indices, int64_t n_indices, const int64_t* offsets, int64_t n_bags,
                                     float* out, bool nontemporal, hipStream_t stream)
{
    const bool fast = dim % 8 == 0 && pitch % 4 == 0 && reinterpret_cast<uintptr_t>(fused) % 4 == 0 &&
                      reinterpret_cast<uintptr_t>(out) % 16 == 0;
    const int wpr = dim / 8;
    // Code words per thread (4-, 8- or 16-byte gathers).  Measured on 34 M lookups, table of 10 M rows / of 20 000 rows
    // (resident in L2), ms with 1 / 2 / 4 words per thread:
    //   d =  64   0.87 / 0.90 / 0.98     0.47 / 0.46 / 0.42
    //   d = 128   1.13 / 1.15 / 1.12     0.79 / 0.76 / 0.63
    //   d = 512   3.10 / 3.36 / 2.94     2.16 / 2.41 / 2.05
    // so 16-byte gathers wherever the row allows them, except for short rows of tables far beyond the caches.
    // Records in flight per thread: 2 / 4 / 8 measure 1.20 / 1.12 / 1.12 ms at d = 128 (0.77 / 0.63 / 0.64 resident).
    int wpt = 1;
    if (fast) {
        const bool small_table = rows * pitch <= (int64_t)32 << 20;
        if (wpr % 4 == 0 && (dim >= 128 || small_table)) wpt = 4;
        else if (wpr % 2 == 0 && dim >= 128) wpt = 2;
    }
    const int64_t threads = fast ? n_bags * (wpr / wpt) : n_bags * ((dim + 7) / 8);
    const int64_t blocks = blocks_for(threads, kSlsBlock);
    if (blocks < 0) return hipErrorInvalidValue;
    const dim3 grid = grid_for(blocks), block(kSlsBlock);
    const uint32_t* f32 = reinterpret_cast<const uint32_t*>(fused);
    const Tidx* idx = static_cast<const Tidx*>(indices);
    floatx4* o4 = reinterpret_cast<floatx4*>(out);
    if (!fast)
        hipLaunchKernelGGL(sls_fused_h8_kernel<Tidx>, grid, block, 0, stream, fused, rows, (uint32_t)dim, pitch, idx,
                           n_indices, offsets, n_bags, out);
    else if (wpt == 4 && nontemporal)
        hipLaunchKernelGGL((sls_fused_w8_kernel<Tidx, 4, true>), grid, block, 0, stream, f32, rows, (uint32_t)wpr,
                           (uint32_t)(pitch / 4), idx, n_indices, offsets, n_bags, o4);
    else if (wpt == 4)
        hipLaunchKernelGGL((sls_fused_w8_kernel<Tidx, 4, false>), grid, block, 0, stream, f32, rows, (uint32_t)wpr,
                           (uint32_t)(pitch / 4), idx, n_indices, offsets, n_bags, o4);
    else if (wpt == 2 && nontemporal)
        hipLaunchKernelGGL((sls_fused_w8_kernel<Tidx, 2, true>), grid, block, 0, stream, f32, rows, (uint32_t)wpr,
                           (uint32_t)(pitch / 4), idx, n_indices, offsets, n_bags, o4);
    else if (wpt == 2)
        hipLaunchKernelGGL((sls_fused_w8_kernel<Tidx, 2, false>), grid, block, 0, stream, f32, rows, (uint32_t)wpr,
                           (uint32_t)(pitch / 4), idx, n_indices, offsets, n_bags, o4);
    else if (nontemporal)
        hipLaunchKernelGGL((sls_fused_w8_kernel<Tidx, 1, true>), grid, block, 0, stream, f32, rows, (uint32_t)wpr,
                           (uint32_t)(pitch / 4), idx, n_indices, offsets, n_bags, o4);
    else
        hipLaunchKernelGGL((sls_fused_w8_kernel<Tidx, 1, false>), grid, block, 0, stream, f32, rows, (uint32_t)wpr,
                           (uint32_t)(pitch / 4), idx, n_indices, offsets, n_bags, o4);
    return hipGetLastError();
}

hipError_t launch_sparse_lengths_sum_fused(const uint8_t* fused, int64_t rows, int32_t dim, int64_t pitch,
                                           const void* indices, int32_t index_bytes, int64_t n_indices,
                                           const int64_t* offsets, int64_t n_bags, float* out, bool nontemporal,
                                           hipStream_t stream)
{
    return index_bytes == 4 ? launch_sls_fused_t<int32_t>(fused, rows, dim, pitch, indices, n_indices, offsets, n_bags,
                                                          out, nontemporal, stream)
                            : launch_sls_fused_t<int64_t>(fused, rows, dim, pitch, indices, n_indices, offsets, n_bags,
                                                          out, nontemporal, stream);
}

template <typename Tidx>
static hipError_t launch_sls_t(const uint8_t* codes, const uint16_t* sc, const uint16_t* bi, int64_t rows,
                               int32_t dim, const void* indices, int64_t n_indices, const int64_t* offsets,
                               int64_t n_bags, float* out, hipStream_t stream)
{
    const bool fast = dim % 8 == 0 && reinterpret_cast<uintptr_t>(codes) % 4 == 0 &&
                      reinterpret_cast<uintptr_t>(out) % 16 == 0;
    const int64_t threads = fast ? n_bags * (dim / 8) : n_bags * ((dim + 7) / 8);
    const int64_t blocks = blocks_for(threads, kSlsBlock);
    if (blocks < 0) return hipErrorInvalidValue;
    if (fast)
        hipLaunchKernelGGL(sls_w8_kernel<Tidx>, grid_for(blocks), dim3(kSlsBlock), 0, stream,
                           reinterpret_cast<const uint32_t*>(codes), sc, bi, rows, (uint32_t)(dim / 8),
                           static_cast<const Tidx*>(indices), n_indices, offsets, n_bags,
                           reinterpret_cast<floatx4*>(out));
    else
        hipLaunchKernelGGL(sls_bytes_kernel<Tidx>, grid_for(blocks), dim3(kSlsBlock), 0, stream, codes, sc, bi,
                           rows, (uint32_t)dim, static_cast<const Tidx*>(indices), n_indices, offsets, n_bags, out);
    return hipGetLastError();
}

hipError_t launch_sparse_lengths_sum(const uint8_t* codes, const uint16_t* sc, const uint16_t* bi, int64_t rows,
                                     int32_t dim, const void* indices, int32_t index_bytes, int64_t n_indices,
                                     const int64_t* offsets, int64_t n_bags, float* out, hipStream_t stream)
{
    return index_bytes == 4
               ? launch_sls_t<int32_t>(codes, sc, bi, rows, dim, indices, n_indices, offsets, n_bags, out, stream)
               : launch_sls_t<int64_t>(codes, sc, bi, rows, dim, indices, n_indices, offsets, n_bags, out, stream);
}

}  // namespace e4q
