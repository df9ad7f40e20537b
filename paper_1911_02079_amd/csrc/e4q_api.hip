// C ABI of libe4q (see include/e4q.h for the contract of every entry point).
// Host code only: argument validation, choice of kernel, launch on the caller's stream.
#include "../../include/e4q.h"

#include <algorithm>
#include <atomic>
#include <cmath>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <vector>

#include "e4q_launch.h"

namespace {

thread_local char g_hip_error[256] = "";

int fail_launch(hipError_t err)
{
    std::snprintf(g_hip_error, sizeof(g_hip_error), "%s: %s", hipGetErrorName(err), hipGetErrorString(err));
    return E4Q_ERR_LAUNCH;
}

// Diagnostic options (e4q_set_option): process-wide, read once per call.
// 0 automatic, 1 one row per lane, (E << 8) | L sub-wave layout, kTwin | (E << 8) | L the same with two groups of
// L lanes per row (one per candidate range of a trip)
std::atomic<int64_t> g_greedy_layout{0};
constexpr int64_t kTwin = (int64_t)1 << 16;
std::atomic<int64_t> g_kmeans_force_scan{0};  // 1: scan all 16 centres instead of bisecting
std::atomic<int64_t> g_workgroup_waves{0};    // 1 or 4: waves per workgroup of the row-per-lane kernels; 0: by row count
std::atomic<int64_t> g_sls_nontemporal{0};    // 1: gather records with non-temporal loads
std::atomic<int64_t> g_greedy_layout_chosen{0};  // read-only: layout of the last single-table greedy launch

std::atomic<int64_t>* find_option(const char* name)
{
    if (!name) return nullptr;
    if (std::strcmp(name, "greedy_layout") == 0) return &g_greedy_layout;
    if (std::strcmp(name, "kmeans_force_scan") == 0) return &g_kmeans_force_scan;
    if (std::strcmp(name, "workgroup_waves") == 0) return &g_workgroup_waves;
    if (std::strcmp(name, "sls_nontemporal") == 0) return &g_sls_nontemporal;
    if (std::strcmp(name, "greedy_layout_chosen") == 0) return &g_greedy_layout_chosen;
    return nullptr;
}

bool layout_value_ok(int64_t v)
{
    if (v == 0 || v == 1) return true;
    if (v < 0 || v >= 2 * kTwin) return false;
    if (v & kTwin) {  // instantiated for 8 and 16 elements per lane, two groups of at most 32 lanes
        const int64_t e = (v & ~kTwin) >> 8, l = v & 0xff;
        return (e == 8 || e == 16) && l >= 1 && l <= 32 && (l & (l - 1)) == 0;
    }
    const int64_t e = v >> 8, l = v & 0xff;
    if (e != 8 && e != 16 && e != 32 && e != 64 && e != 128) return false;
    if (l < 1 || l > 64) return false;
    if ((l & (l - 1)) == 0 && e == 128 && l > 32) return false;  // not instantiated: dim <= 4096
    return true;
}

inline bool aligned(const void* p, size_t a) { return reinterpret_cast<uintptr_t>(p) % a == 0; }

bool nbits_ok(int32_t nbits) { return nbits == 2 || nbits == 4 || nbits == 8; }

int validate_search(int32_t nbits, int32_t n_bins, float ratio)
{
    if (!nbits_ok(nbits)) return E4Q_ERR_BAD_NBITS;
    if (n_bins < 1 || !(ratio >= 0.0f && ratio < 1.0f)) return E4Q_ERR_BAD_SEARCH;
    return E4Q_OK;
}

int validate_table(const void* table, int dtype, int64_t rows, int32_t dim, int64_t row_stride,
                   const uint8_t* codes, const uint16_t* scale_f16, const uint16_t* bias_f16)
{
    if (dtype != E4Q_F32 && dtype != E4Q_F16) return E4Q_ERR_BAD_DTYPE;
    if (rows < 0 || rows > E4Q_MAX_ROWS || dim <= 0 || dim > E4Q_MAX_DIM || row_stride < dim) return E4Q_ERR_BAD_SHAPE;
    if (rows == 0) return E4Q_OK;
    if (!table || !codes || !scale_f16 || !bias_f16) return E4Q_ERR_NULL_POINTER;
    if (!aligned(table, dtype == E4Q_F32 ? 4 : 2) || !aligned(scale_f16, 2) || !aligned(bias_f16, 2))
        return E4Q_ERR_BAD_ALIGNMENT;
    return E4Q_OK;
}

// A layout forced through the "greedy_layout" option must be able to hold a row of `dim` elements.
int validate_forced_layout(int32_t dim)
{
    const int64_t forced = g_greedy_layout.load(std::memory_order_relaxed);
    if (forced == 0) return E4Q_OK;
    if (forced == 1) return (e4q::rpl_supports_dim(dim) || e4q::rpl_tail_supports_dim(dim)) ? E4Q_OK : E4Q_ERR_BAD_OPTION;
    return ((forced & ~kTwin) >> 8) * (forced & 0xff) >= dim ? E4Q_OK : E4Q_ERR_BAD_OPTION;
}

// Estimated duration of the greedy search, in SIMD cycles, for `rows` rows with `elems` elements per
// lane and `lanes` lanes per row.  Instructions per wave and scored range: 8 per element, about 30 of
// per-range scalar work (two short divisions, two binary16 round trips, the decisions) and 6 per butterfly
// step.  Cycles per instruction as measured on gfx950: a SIMD with one or two waves issues one
// instruction per wave every 5.2 cycles (so two waves cost what one costs), three waves 8.3 in total,
// four or more 2.45 each.  Every kernel runs in four-wave workgroups, whose waves land one on each SIMD of a compute
// unit, so a SIMD holds the average number of waves rounded up.  Fitted on 1 k - 1 M rows at dim 32 / 64 / 128; within
// 10 % of the measured times (plus some 10 us of launch and first load that every layout pays) except where the next
// smaller layout is equally fast.
// `twin`: two groups of `lanes` lanes per row score the two ranges of a trip at the same time: a wave holds half as many
// rows and its chain is 1 + n_iter ranges long instead of 1 + 2 * n_iter (and three instructions per trip to swap sums).
double layout_cost(int64_t rows, int32_t elems, int32_t lanes, int32_t n_iter, bool row_per_lane, bool twin = false)
{
    int steps = 0;
    while ((1 << steps) < lanes) ++steps;
    // a lane count that is not a power of two sums across lanes by ds_bpermute (one per step and one to hand
    // the result round, each worth some 14 instructions with its select and addition) instead of DPP moves
    const bool pow2 = (lanes & (lanes - 1)) == 0;
    const double per_range = 8.0 * elems + 30.0 + (pow2 ? 6.0 * steps : 14.0 * (steps + 1));
    const double instructions = twin ? (1.0 + n_iter) * per_range + 3.0 * n_iter + 10.0 * elems
                                     : (1.0 + 2.0 * n_iter) * per_range + 10.0 * elems;
    const int64_t rows_per_wave = row_per_lane ? 64 : 64 / (twin ? 2 * lanes : lanes);
    const int64_t waves = (rows + rows_per_wave - 1) / rows_per_wave;
    const int64_t per_simd = (waves + 1023) / 1024;
    const double cycles_per_instruction = per_simd <= 2 ? 5.2 : per_simd == 3 ? 8.3 : 2.45 * (double)per_simd;
    // measured, two groups per row gain less than their instruction count says (every row is loaded twice, and a
    // launch has some 10 us that no layout shortens): a tenth is added so that a near tie goes to the plain layout
    return instructions * cycles_per_instruction * (twin ? 1.1 : 1.0);
}

int enqueue_greedy(const void* table, int dtype, int64_t rows, int32_t dim, int64_t row_stride, int32_t nbits,
                   int32_t n_bins, int32_t n_iter, uint8_t* codes, uint16_t* scale_f16,
                   uint16_t* bias_f16, hipStream_t stream)
{
    if (rows == 0) return E4Q_OK;
    const size_t esz = dtype == E4Q_F32 ? 4 : 2;
    e4q::GreedyArgs a;
    a.table = table;
    a.rows = rows;
    a.row_stride = row_stride;
    a.n_iter = n_iter;
    a.n_bins = (float)n_bins;
    a.codes = codes;
    a.scale_f16 = scale_f16;
    a.bias_f16 = bias_f16;
    a.vec_loads = (aligned(table, 16) && (row_stride * esz) % 16 == 0) ? 1u : 0u;
    a.vec_stores = aligned(codes, 16) ? 2u : (aligned(codes, 4) ? 1u : 0u);
    a.nbits = nbits;
    a.qmax = (float)((1 << nbits) - 1);
    a.rpl_waves = (uint32_t)g_workgroup_waves.load(std::memory_order_relaxed);

    // Kernel choice.  One row per lane (rows/64 waves, the row in registers, ~3 % overhead over the
    // algorithmic operation count) does the arithmetic with the fewest instructions; a row spread over
    // L lanes with E contiguous elements each (E * L >= dim) repeats the per-range scalar work in every
    // lane but makes L times as many waves.  Which is faster depends on how many waves a SIMD gets:
    // see layout_cost.  ratio == 0 is bound by HBM and always takes E = 8 (a wave then reads and
    // writes contiguous memory).
    int E = 0, L = 1;  // E == 0: one row per lane
    bool twin = false;
    const int64_t forced = g_greedy_layout.load(std::memory_order_relaxed);
    if (forced == 1) {
        if (!(e4q::rpl_supports_dim(dim) || e4q::rpl_tail_supports_dim(dim))) return E4Q_ERR_BAD_OPTION;
    } else if (forced != 0) {
        twin = (forced & kTwin) != 0;
        E = (int)((forced & ~kTwin) >> 8);
        L = (int)(forced & 0xff);
        if ((int64_t)E * L < dim) return E4Q_ERR_BAD_OPTION;
    } else if (n_iter == 0) {
        E = dim <= 512 ? 8 : dim <= 1024 ? 16 : dim <= 2048 ? 32 : 64;
        while (E * L < dim) L *= 2;
    } else {
        const bool rpl = e4q::rpl_supports_dim(dim) || e4q::rpl_tail_supports_dim(dim);
        double best = rpl ? layout_cost(rows, (dim + 7) / 8 * 8, 1, n_iter, true) : -1.0;
        // A dimension that is not a multiple of 8 carries mask factors in registers of their own, one per
        // element that some lane of the row's group may lack.  On the fewest lanes that hold the row only the
        // last lane lacks any, and if it is at least half full the factors are few (greedy_swl.h).  64 elements
        // per lane then measure best (128 M elements at dim 999: E = 32 1.40 ms, E = 64 1.21 ms, E = 128
        // 1.31 ms; 2.76 ms for E = 128 with a factor per element, which leaves one wave per SIMD); 128 per lane
        // only pay where 64 would leave most of a wave's lanes idle (dim 2500: 20 lanes of 128 1.73 ms, 40 or
        // 64 lanes of 64 2.15 / 1.96 ms).
        for (int e = 8; e <= 128; e *= 2) {
            if (e > 8 && e / 2 >= dim) break;  // more than half of every lane would be padding
            // the fewest lanes that hold the row, and the next power of two (sums by DPP moves)
            const int l_min = (dim + e - 1) / e;
            int l_pow2 = 1;
            while (l_pow2 < l_min) l_pow2 *= 2;
            const bool few_factors = dim - (l_min - 1) * e >= e / 2;
            for (int l : {l_min, l_pow2}) {
                if (l > 64) continue;
                if (dim % 8 != 0 && e == 128 && !(l == l_min && few_factors && dim > 2048)) continue;
                const double c = layout_cost(rows, e, l, n_iter, false);
                if (best < 0.0 || c < best) {
                    best = c;
                    E = e;
                    L = l;
                    twin = false;
                }
                // few rows: the same lanes twice, one group per candidate range of a trip
                if (e <= 16 && l == l_pow2 && l <= 32) {
                    const double ct = layout_cost(rows, e, l, n_iter, false, true);
                    if (ct < best) {
                        best = ct;
                        E = e;
                        L = l;
                        twin = true;
                    }
                }
            }
        }
    }
    g_greedy_layout_chosen.store(E == 0 ? 1 : (twin ? kTwin : 0) | ((int64_t)E << 8) | L, std::memory_order_relaxed);
    hipError_t err;
    if (twin) {
        err = dtype == E4Q_F32 ? e4q::launch_greedy_swl_twin_f32(a, dim, E, L, stream)
                               : e4q::launch_greedy_swl_twin_f16(a, dim, E, L, stream);
    } else if (E == 0 && dim % 8 == 0 && dim > 128) {
        err = dtype == E4Q_F32 ? e4q::launch_greedy_rpl_wide_f32(a, dim, stream)
                               : e4q::launch_greedy_rpl_wide_f16(a, dim, stream);
    } else if (E == 0 && dim % 8 == 0) {
        err = dtype == E4Q_F32 ? e4q::launch_greedy_rpl_f32(a, dim, stream)
                               : e4q::launch_greedy_rpl_f16(a, dim, stream);
    } else if (E == 0 && dim > 128) {
        err = dtype == E4Q_F32 ? e4q::launch_greedy_rpl_wide_tail_f32(a, dim, stream)
                               : e4q::launch_greedy_rpl_wide_tail_f16(a, dim, stream);
    } else if (E == 0) {
        err = dtype == E4Q_F32 ? e4q::launch_greedy_rpl_tail_f32(a, dim, stream)
                               : e4q::launch_greedy_rpl_tail_f16(a, dim, stream);
    } else if ((L & (L - 1)) != 0 || (dim % 8 != 0 && E >= 32 && L >= 2 && L == (dim + E - 1) / E)) {
        // a lane count that is not a power of two, or the fewest lanes for a dimension that is not a multiple
        // of 8: the run-time lane-count kernels have the variants with few mask factors
        err = dtype == E4Q_F32 ? e4q::launch_greedy_swl_any_f32(a, dim, E, L, stream)
                               : e4q::launch_greedy_swl_any_f16(a, dim, E, L, stream);
    } else {
        if (E == 128)
            err = dtype == E4Q_F32 ? e4q::launch_greedy_swl_f32_big(a, dim, E, L, stream)
                                   : e4q::launch_greedy_swl_f16_big(a, dim, E, L, stream);
        else if (E >= 32)
            err = dtype == E4Q_F32 ? e4q::launch_greedy_swl_f32_mid(a, dim, E, L, stream)
                                   : e4q::launch_greedy_swl_f16_mid(a, dim, E, L, stream);
        else
            err = dtype == E4Q_F32 ? e4q::launch_greedy_swl_f32_small(a, dim, E, L, stream)
                                   : e4q::launch_greedy_swl_f16_small(a, dim, E, L, stream);
    }
    return err == hipSuccess ? E4Q_OK : fail_launch(err);
}

}  // namespace

extern "C" {

int32_t e4q_greedy_iterations(int32_t n_bins, float ratio)
{
    if (n_bins < 1 || !(ratio >= 0.0f && ratio < 1.0f)) return E4Q_ERR_BAD_SEARCH;
    const double br = (double)n_bins * (double)ratio;
    double t = std::ceil(br - br * 0x1p-22);
    if (t < 0.0) t = 0.0;
    if (t > (double)(n_bins - 1)) t = (double)(n_bins - 1);
    return (int32_t)t;
}

int e4q_quantize_rowwise_greedy(const void* table, int dtype, int64_t rows, int32_t dim,
                                int64_t row_stride, int32_t nbits, int32_t n_bins, float ratio,
                                uint8_t* codes, uint16_t* scale_f16, uint16_t* bias_f16,
                                void* hip_stream)
{
    int rc = validate_search(nbits, n_bins, ratio);
    if (rc != E4Q_OK) return rc;
    rc = validate_table(table, dtype, rows, dim, row_stride, codes, scale_f16, bias_f16);
    if (rc != E4Q_OK) return rc;
    rc = validate_forced_layout(dim);
    if (rc != E4Q_OK) return rc;
    return enqueue_greedy(table, dtype, rows, dim, row_stride, nbits, n_bins, e4q_greedy_iterations(n_bins, ratio),
                          codes, scale_f16, bias_f16, static_cast<hipStream_t>(hip_stream));
}

int e4q_quantize_rowwise_greedy_batch(const e4q_table_desc* descs, int32_t n_tables, int32_t nbits,
                                      int32_t n_bins, float ratio, void* hip_stream)
{
    int rc = validate_search(nbits, n_bins, ratio);
    if (rc != E4Q_OK) return rc;
    if (n_tables < 0) return E4Q_ERR_BAD_SHAPE;
    if (n_tables == 0) return E4Q_OK;
    if (!descs) return E4Q_ERR_NULL_POINTER;
    for (int32_t t = 0; t < n_tables; ++t) {
        const e4q_table_desc& d = descs[t];
        rc = validate_table(d.table, d.dtype, d.rows, d.dim, d.row_stride, d.codes, d.scale_f16, d.bias_f16);
        if (rc != E4Q_OK) return rc;
        rc = validate_forced_layout(d.dim);
        if (rc != E4Q_OK) return rc;
    }
    const int32_t n_iter = e4q_greedy_iterations(n_bins, ratio);
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    try {  // the bookkeeping below allocates host memory; nothing may be thrown across the C boundary
    std::vector<char> done((size_t)n_tables, 0);
    // Tables that share a dimension (one with a row-per-lane kernel) and an input type go out in grouped
    // launches of up to kMaxGroupTables tables.
    if (n_iter > 0 && g_greedy_layout.load(std::memory_order_relaxed) == 0) {
        for (int32_t t = 0; t < n_tables; ++t) {
            if (done[t] || descs[t].rows == 0 || !e4q::rpl_group_supports_dim(descs[t].dim)) continue;
            std::vector<int32_t> members;
            int64_t waves = 0;
            for (int32_t u = t; u < n_tables; ++u)
                if (!done[u] && descs[u].rows > 0 && descs[u].dim == descs[t].dim && descs[u].dtype == descs[t].dtype) {
                    members.push_back(u);
                    waves += (descs[u].rows + 63) / 64;
                }
            // Two tables or more always share launches: small tables then run side by side instead of one after the
            // other (26 tables of 1 000 x 64: 171 us one by one), and one row per lane is the fastest layout from
            // some 100 000 rows in the launch on.
            if (members.size() < 2 || waves > 0x3ffffffLL) continue;  // below 2^32 work-items per launch
            for (size_t first = 0; first < members.size(); first += e4q::kMaxGroupTables) {
                e4q::GreedyGroup g;
                g.n_tables = (int32_t)std::min<size_t>(e4q::kMaxGroupTables, members.size() - first);
                int64_t rows_in_launch = 0;
                for (int32_t k = 0; k < g.n_tables; ++k) rows_in_launch += descs[members[first + k]].rows;
                g.rows_per_block = e4q::rpl_rows_per_block(rows_in_launch, (uint32_t)g_workgroup_waves.load(std::memory_order_relaxed));
                g.n_iter = n_iter;
                g.n_bins = (float)n_bins;
                g.nbits = nbits;
                g.qmax = (float)((1 << nbits) - 1);
                uint32_t blocks = 0;
                for (int32_t k = 0; k < e4q::kMaxGroupTables; ++k) {
                    if (k < g.n_tables) {
                        const e4q_table_desc& d = descs[members[first + k]];
                        const size_t esz = d.dtype == E4Q_F32 ? 4 : 2;
                        e4q::GreedyTable& e = g.tables[k];
                        e.table = d.table;
                        e.rows = d.rows;
                        e.row_stride = d.row_stride;
                        e.codes = d.codes;
                        e.scale_f16 = d.scale_f16;
                        e.bias_f16 = d.bias_f16;
                        e.vec_loads = (aligned(d.table, 16) && (d.row_stride * esz) % 16 == 0) ? 1u : 0u;
                        e.vec_stores = aligned(d.codes, 16) ? 2u : (aligned(d.codes, 4) ? 1u : 0u);
                        blocks += (uint32_t)((d.rows + g.rows_per_block - 1) / g.rows_per_block);
                        done[members[first + k]] = 1;
                    } else {
                        g.tables[k] = e4q::GreedyTable{};
                    }
                    g.block_end[k] = blocks;
                }
                const hipError_t err = descs[t].dtype == E4Q_F32 ? e4q::launch_greedy_rpl_group_f32(g, descs[t].dim, stream)
                                                                 : e4q::launch_greedy_rpl_group_f16(g, descs[t].dim, stream);
                if (err != hipSuccess) return fail_launch(err);
            }
        }
    }
    for (int32_t t = 0; t < n_tables; ++t) {
        if (done[t]) continue;
        const e4q_table_desc& d = descs[t];
        rc = enqueue_greedy(d.table, d.dtype, d.rows, d.dim, d.row_stride, nbits, n_bins, n_iter, d.codes,
                            d.scale_f16, d.bias_f16, stream);
        if (rc != E4Q_OK) return rc;
    }
    } catch (...) {
        std::snprintf(g_hip_error, sizeof(g_hip_error), "host memory allocation failed");
        return E4Q_ERR_LAUNCH;
    }
    return E4Q_OK;
}

int e4q_dequantize(const uint8_t* codes, const uint16_t* scale_f16, const uint16_t* bias_f16,
                   int64_t rows, int32_t dim, int32_t nbits, float* out, void* hip_stream)
{
    if (!nbits_ok(nbits)) return E4Q_ERR_BAD_NBITS;
    if (rows < 0 || rows > E4Q_MAX_ROWS || dim <= 0 || dim > E4Q_MAX_DIM) return E4Q_ERR_BAD_SHAPE;
    if (rows == 0) return E4Q_OK;
    if (!codes || !scale_f16 || !bias_f16 || !out) return E4Q_ERR_NULL_POINTER;
    if (!aligned(scale_f16, 2) || !aligned(bias_f16, 2) || !aligned(out, 4)) return E4Q_ERR_BAD_ALIGNMENT;
    const hipError_t err = e4q::launch_dequantize(codes, scale_f16, bias_f16, rows, dim, nbits, out,
                                                  static_cast<hipStream_t>(hip_stream));
    return err == hipSuccess ? E4Q_OK : fail_launch(err);
}

int e4q_quantize_rowwise_kmeans16(const void* table, int dtype, int64_t rows, int32_t dim,
                                  int64_t row_stride, int32_t lloyd_iters, uint8_t* idx,
                                  uint16_t* centroids_f16, void* hip_stream)
{
    if (lloyd_iters < 0) return E4Q_ERR_BAD_SEARCH;
    if (dtype != E4Q_F32 && dtype != E4Q_F16) return E4Q_ERR_BAD_DTYPE;
    if (rows < 0 || rows > E4Q_MAX_ROWS || dim <= 0 || dim > E4Q_MAX_DIM || row_stride < dim) return E4Q_ERR_BAD_SHAPE;
    if (rows == 0) return E4Q_OK;
    if (!table || !idx || !centroids_f16) return E4Q_ERR_NULL_POINTER;
    const size_t esz = dtype == E4Q_F32 ? 4 : 2;
    if (!aligned(table, esz) || !aligned(centroids_f16, 2)) return E4Q_ERR_BAD_ALIGNMENT;
    e4q::KMeansArgs a;
    a.table = table;
    a.rows = rows;
    a.row_stride = row_stride;
    a.lloyd_iters = lloyd_iters;
    a.idx = idx;
    a.centroids_f16 = centroids_f16;
    a.vec_loads = (aligned(table, 16) && (row_stride * esz) % 16 == 0) ? 1u : 0u;
    a.vec_stores = aligned(idx, 16) ? 2u : (aligned(idx, 4) ? 1u : 0u);
    a.force_scan = g_kmeans_force_scan.load(std::memory_order_relaxed) != 0 ? 1u : 0u;
    a.waves = (uint32_t)g_workgroup_waves.load(std::memory_order_relaxed);
    const hipError_t err = e4q::launch_kmeans16(a, dtype, dim, static_cast<hipStream_t>(hip_stream));
    return err == hipSuccess ? E4Q_OK : fail_launch(err);
}

int e4q_dequantize_codebook(const uint8_t* idx, const uint16_t* centroids_f16, int64_t rows, int32_t dim,
                            float* out, void* hip_stream)
{
    if (rows < 0 || rows > E4Q_MAX_ROWS || dim <= 0 || dim > E4Q_MAX_DIM) return E4Q_ERR_BAD_SHAPE;
    if (rows == 0) return E4Q_OK;
    if (!idx || !centroids_f16 || !out) return E4Q_ERR_NULL_POINTER;
    if (!aligned(centroids_f16, 2) || !aligned(out, 4)) return E4Q_ERR_BAD_ALIGNMENT;
    const hipError_t err = e4q::launch_dequantize_codebook(idx, centroids_f16, rows, dim, out,
                                                           static_cast<hipStream_t>(hip_stream));
    return err == hipSuccess ? E4Q_OK : fail_launch(err);
}

int e4q_sparse_lengths_sum(const uint8_t* codes, const uint16_t* scale_f16, const uint16_t* bias_f16,
                           int64_t rows, int32_t dim, int32_t nbits, const void* indices, int32_t index_bytes,
                           int64_t n_indices, const int64_t* offsets, int64_t n_bags, float* out,
                           void* hip_stream)
{
    if (nbits != 4) return E4Q_ERR_BAD_NBITS;
    if (index_bytes != 4 && index_bytes != 8) return E4Q_ERR_BAD_DTYPE;
    if (rows < 0 || rows > E4Q_MAX_ROWS || dim <= 0 || dim > E4Q_MAX_DIM || n_indices < 0 || n_bags < 0 ||
        n_bags > E4Q_MAX_ROWS)
        return E4Q_ERR_BAD_SHAPE;
    if (n_bags == 0) return E4Q_OK;
    if (!offsets || !out || (n_indices > 0 && !indices)) return E4Q_ERR_NULL_POINTER;
    if (rows > 0 && (!codes || !scale_f16 || !bias_f16)) return E4Q_ERR_NULL_POINTER;
    if (!aligned(scale_f16, 2) || !aligned(bias_f16, 2) || !aligned(out, 4) || !aligned(offsets, 8) ||
        !aligned(indices, (size_t)index_bytes))
        return E4Q_ERR_BAD_ALIGNMENT;
    const hipError_t err = e4q::launch_sparse_lengths_sum(codes, scale_f16, bias_f16, rows, dim, indices, index_bytes,
                                                          n_indices, offsets, n_bags, out,
                                                          static_cast<hipStream_t>(hip_stream));
    return err == hipSuccess ? E4Q_OK : fail_launch(err);
}

static int64_t fused_min_pitch(int32_t dim) { return ((((int64_t)dim + 1) / 2 + 1) & ~(int64_t)1) + 4; }

int64_t e4q_fused_row_bytes(int32_t dim)
{
    if (dim <= 0 || dim > E4Q_MAX_DIM) return E4Q_ERR_BAD_SHAPE;
    return fused_min_pitch(dim);
}

int e4q_fuse_rows(const uint8_t* codes, const uint16_t* scale_f16, const uint16_t* bias_f16, int64_t rows,
                  int32_t dim, int32_t nbits, int64_t row_pitch, uint8_t* fused, void* hip_stream)
{
    if (nbits != 4) return E4Q_ERR_BAD_NBITS;
    if (rows < 0 || rows > E4Q_MAX_ROWS || dim <= 0 || dim > E4Q_MAX_DIM || (row_pitch & 1) ||
        row_pitch < fused_min_pitch(dim) || row_pitch > 0x7ffffffeLL)
        return E4Q_ERR_BAD_SHAPE;
    if (rows == 0) return E4Q_OK;
    if (!codes || !scale_f16 || !bias_f16 || !fused) return E4Q_ERR_NULL_POINTER;
    if (!aligned(scale_f16, 2) || !aligned(bias_f16, 2) || !aligned(fused, 2)) return E4Q_ERR_BAD_ALIGNMENT;
    const hipError_t err = e4q::launch_fuse_rows(codes, scale_f16, bias_f16, rows, dim, row_pitch, fused,
                                                 static_cast<hipStream_t>(hip_stream));
    return err == hipSuccess ? E4Q_OK : fail_launch(err);
}

int e4q_sparse_lengths_sum_fused(const uint8_t* fused, int64_t rows, int32_t dim, int32_t nbits, int64_t row_pitch,
                                 const void* indices, int32_t index_bytes, int64_t n_indices,
                                 const int64_t* offsets, int64_t n_bags, float* out, void* hip_stream)
{
    if (nbits != 4) return E4Q_ERR_BAD_NBITS;
    if (index_bytes != 4 && index_bytes != 8) return E4Q_ERR_BAD_DTYPE;
    if (rows < 0 || rows > E4Q_MAX_ROWS || dim <= 0 || dim > E4Q_MAX_DIM || n_indices < 0 || n_bags < 0 ||
        n_bags > E4Q_MAX_ROWS || (row_pitch & 1) ||
        row_pitch < fused_min_pitch(dim))
        return E4Q_ERR_BAD_SHAPE;
    if (n_bags == 0) return E4Q_OK;
    if (!offsets || !out || (n_indices > 0 && !indices) || (rows > 0 && !fused)) return E4Q_ERR_NULL_POINTER;
    if (!aligned(fused, 2) || !aligned(out, 4) || !aligned(offsets, 8) || !aligned(indices, (size_t)index_bytes))
        return E4Q_ERR_BAD_ALIGNMENT;
    const hipError_t err = e4q::launch_sparse_lengths_sum_fused(fused, rows, dim, row_pitch, indices, index_bytes,
                                                                n_indices, offsets, n_bags, out,
                                                                g_sls_nontemporal.load(std::memory_order_relaxed) != 0,
                                                                static_cast<hipStream_t>(hip_stream));
    return err == hipSuccess ? E4Q_OK : fail_launch(err);
}

double e4q_greedy_layout_cost(int64_t rows, int32_t dim, int32_t n_iter, int64_t layout)
{
    if (rows < 0 || dim <= 0 || dim > E4Q_MAX_DIM || n_iter < 0 || layout == 0 || !layout_value_ok(layout)) return -1.0;
    if (layout == 1) {
        if (!(e4q::rpl_supports_dim(dim) || e4q::rpl_tail_supports_dim(dim))) return -1.0;
        return layout_cost(rows, (dim + 7) / 8 * 8, 1, n_iter, true);
    }
    const int32_t e = (int32_t)((layout & ~kTwin) >> 8), l = (int32_t)(layout & 0xff);
    if ((int64_t)e * l < dim) return -1.0;
    return layout_cost(rows, e, l, n_iter, false, (layout & kTwin) != 0);
}

int e4q_set_option(const char* name, int64_t value)
{
    std::atomic<int64_t>* opt = find_option(name);
    if (!opt || opt == &g_greedy_layout_chosen) return E4Q_ERR_BAD_OPTION;
    const bool ok = opt == &g_greedy_layout ? layout_value_ok(value)
                    : opt == &g_workgroup_waves ? (value == 0 || value == 1 || value == 4)
                                                : (value == 0 || value == 1);
    if (!ok) return E4Q_ERR_BAD_OPTION;
    opt->store(value, std::memory_order_relaxed);
    return E4Q_OK;
}

int64_t e4q_get_option(const char* name)
{
    std::atomic<int64_t>* opt = find_option(name);
    return opt ? opt->load(std::memory_order_relaxed) : (int64_t)E4Q_ERR_BAD_OPTION;
}

const char* e4q_strerror(int code)
{
    switch (code) {
        case E4Q_OK: return "success";
        case E4Q_ERR_NULL_POINTER: return "a required pointer is NULL";
        case E4Q_ERR_BAD_SHAPE: return "bad shape: need 0 <= rows <= 2^31, 0 < dim <= 4096, row_stride >= dim, an even row_pitch >= e4q_fused_row_bytes(dim)";
        case E4Q_ERR_BAD_NBITS: return "nbits must be 2, 4 or 8 for the uniform quantizer and its dequantizer, 4 for the lookup operator";
        case E4Q_ERR_BAD_SEARCH: return "bad search parameters: need n_bins >= 1, 0 <= ratio < 1, lloyd_iters >= 0";
        case E4Q_ERR_BAD_DTYPE: return "dtype must be E4Q_F32 (0) or E4Q_F16 (1); index_bytes must be 4 or 8";
        case E4Q_ERR_LAUNCH: return "HIP reported an error at kernel launch (see e4q_last_hip_error)";
        case E4Q_ERR_BAD_ALIGNMENT: return "a pointer is not aligned to its element size";
        case E4Q_ERR_BAD_OPTION: return "unknown diagnostic option, a value it does not take, or a forced layout that does not fit the call's dimension";
        default: return "unknown e4q error code";
    }
}

const char* e4q_last_hip_error(void) { return g_hip_error; }

int e4q_version(void) { return 400; }  // 0.4.0

}  // extern "C"
