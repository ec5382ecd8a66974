/*
 * Host side of libzipccl.so: the code-table builder (paper section 4.1), size / offset
 * arithmetic for the chunked layout (section 4.2.1) and argument checking + launch logic
 * of compress / decompress.  No device memory is allocated here.
 */
#include <cmath>
#include <cstdint>
#include <algorithm>
#include <cstring>
#include <vector>

#include "zipccl_internal.h"

using namespace zipccl;

namespace {

bool dtype_ok(int dt) { return dt == ZIPCCL_BF16 || dt == ZIPCCL_FP32; }

/* Eq.2 of section 4.1: P(|w| in [2^x, 2^(x+7))) for w ~ N(0, sigma^2). */
double window_coverage(double sigma, int x)
{
    const double s = sigma * std::sqrt(2.0);
    return std::erf(std::ldexp(1.0, x + 7) / s) - std::erf(std::ldexp(1.0, x) / s);
}

/* Resolve the chunk split into explicit element counts; false if it is not a valid split. */
bool resolve_split(size_t n_elems, uint32_t n_chunks, const uint64_t* chunk_elems, std::vector<uint64_t>& ce)
{
    if (n_chunks == 0) return false;
    ce.resize(n_chunks);
    if (!chunk_elems) {
        if (n_elems % n_chunks) return false;
        for (uint32_t c = 0; c < n_chunks; ++c) ce[c] = n_elems / n_chunks;
    } else {
        uint64_t total = 0;
        for (uint32_t c = 0; c < n_chunks; ++c) {
            ce[c] = chunk_elems[c];
            if (total + ce[c] < total) return false;
            total += ce[c];
        }
        if (total != n_elems) return false;
    }
    for (uint32_t c = 0; c < n_chunks; ++c)
        if (ce[c] > ZIPCCL_MAX_CHUNK_ELEMS) return false;
    return true;
}

bool table_ok(const zipccl_table_t* t)
{
    if (!t) return false;
    if (t->dec[1] < 1 || t->dec[1] > 249) return false;
    for (int k = 2; k <= 7; ++k)
        if (t->dec[k] != t->dec[1] + k - 1) return false;
    return true;
}

/* Fill the by-value chunk table of one launch covering chunks [c0, c0 + nb). */
uint32_t fill_tab(ChunkTab& tab, const std::vector<uint64_t>& ce, const std::vector<uint64_t>& slot_off,
                  uint32_t c0, uint32_t nb)
{
    tab.n_chunks = nb;
    uint64_t eoff = 0;
    uint32_t tiles = 0;
    for (uint32_t i = 0; i < nb; ++i) {
        tab.tile_start[i] = tiles;
        tab.elem_off[i] = eoff;
        tab.slot_off[i] = slot_off[c0 + i] - slot_off[c0];
        tiles += (uint32_t)tiles_of(ce[c0 + i]);
        eoff += ce[c0 + i];
    }
    for (uint32_t i = nb; i <= kMaxBatch; ++i) {
        tab.tile_start[i] = tiles;
        tab.elem_off[i] = eoff;
        tab.slot_off[i] = slot_off[c0 + nb] - slot_off[c0];
    }
    return tiles;
}

uint64_t total_tiles(const std::vector<uint64_t>& ce)
{
    uint64_t t = 0;
    for (uint64_t n : ce) t += tiles_of(n);
    return t;
}

/* Workspace layout: header | u32 count per tile | u32 prefix per tile | [stash (one byte per element)]. */
struct WorkspacePlan {
    uint64_t tiles, total_off, prefix_off, stash_off, min_bytes, full_bytes;
};

WorkspacePlan plan_workspace(const std::vector<uint64_t>& ce, uint64_t n_elems)
{
    WorkspacePlan w{};
    for (uint64_t n : ce) w.tiles += tiles_of(n);
    const uint64_t arr = (4 * w.tiles + 15) & ~15ull;
    w.total_off = kWorkspaceHeader;
    w.prefix_off = w.total_off + arr;
    w.stash_off = w.prefix_off + arr;
    w.min_bytes = w.stash_off;
    w.full_bytes = w.stash_off + ((n_elems + kStashSlack + 15) & ~15ull);
    return w;
}

} // namespace

extern "C" {

zipccl_status_t zipccl_build_table(double sigma, zipccl_dtype_t dt, zipccl_table_t* out)
{
    if (!dtype_ok(dt)) return ZIPCCL_ERR_UNSUPPORTED_DTYPE;
    if (!out || !(sigma > 0.0) || std::isinf(sigma)) return ZIPCCL_ERR_INVALID_ARG;
    /* Eq.5: continuous optimum of the window base */
    const double x_opt = std::log2(sigma) + 0.5 * std::log2(14.0 * std::log(2.0) / 16383.0);
    const int lo = (int)std::floor(x_opt), hi = (int)std::ceil(x_opt);
    const int x = window_coverage(sigma, hi) > window_coverage(sigma, lo) ? hi : lo;
    int e0 = x + 127;
    e0 = e0 < 1 ? 1 : (e0 > 248 ? 248 : e0);
    out->dec[0] = 0;
    for (int k = 1; k <= 7; ++k) out->dec[k] = (uint8_t)(e0 + k - 1);
    return ZIPCCL_OK;
}

zipccl_status_t zipccl_chunk_slot_offsets(size_t n_elems, zipccl_dtype_t dt, uint32_t n_chunks,
                                          const uint64_t* chunk_elems, uint64_t* slot_off)
{
    if (!dtype_ok(dt)) return ZIPCCL_ERR_UNSUPPORTED_DTYPE;
    std::vector<uint64_t> ce;
    if (!slot_off || !resolve_split(n_elems, n_chunks, chunk_elems, ce)) return ZIPCCL_ERR_INVALID_ARG;
    uint64_t off = 0;
    for (uint32_t c = 0; c < n_chunks; ++c) {
        slot_off[c] = off;
        off += slot_layout(ce[c], dt).cap;
    }
    slot_off[n_chunks] = off;
    return ZIPCCL_OK;
}

zipccl_status_t zipccl_chunk_static_bytes(size_t n_elems, zipccl_dtype_t dt, uint32_t n_chunks,
                                          const uint64_t* chunk_elems, uint64_t* static_bytes)
{
    if (!dtype_ok(dt)) return ZIPCCL_ERR_UNSUPPORTED_DTYPE;
    std::vector<uint64_t> ce;
    if (!static_bytes || !resolve_split(n_elems, n_chunks, chunk_elems, ce)) return ZIPCCL_ERR_INVALID_ARG;
    for (uint32_t c = 0; c < n_chunks; ++c) static_bytes[c] = slot_layout(ce[c], dt).esc;
    return ZIPCCL_OK;
}

size_t zipccl_max_compressed_size(size_t n_elems, zipccl_dtype_t dt, uint32_t n_chunks,
                                  const uint64_t* chunk_elems)
{
    if (!dtype_ok(dt)) return 0;
    std::vector<uint64_t> ce;
    if (!resolve_split(n_elems, n_chunks, chunk_elems, ce)) return 0;
    uint64_t off = 0;
    for (uint64_t n : ce) off += slot_layout(n, dt).cap;
    return (size_t)off;
}

size_t zipccl_compress_workspace_size(size_t n_elems, zipccl_dtype_t dt, uint32_t n_chunks,
                                      const uint64_t* chunk_elems)
{
    if (!dtype_ok(dt)) return 0;
    std::vector<uint64_t> ce;
    if (!resolve_split(n_elems, n_chunks, chunk_elems, ce)) return 0;
    return (size_t)plan_workspace(ce, n_elems).full_bytes;
}

size_t zipccl_compress_min_workspace_size(size_t n_elems, zipccl_dtype_t dt, uint32_t n_chunks,
                                          const uint64_t* chunk_elems)
{
    if (!dtype_ok(dt)) return 0;
    std::vector<uint64_t> ce;
    if (!resolve_split(n_elems, n_chunks, chunk_elems, ce)) return 0;
    return (size_t)plan_workspace(ce, n_elems).min_bytes;
}

} // extern "C"

namespace {

/* compress with the table either on the host (checked here) or in device memory (d_table) */
zipccl_status_t compress_impl(const void* d_in, size_t n_elems, zipccl_dtype_t dt,
                              uint32_t n_chunks, const uint64_t* chunk_elems,
                              const zipccl_table_t* table, const zipccl_table_t* d_table, bool table_per_chunk,
                              void* d_out, size_t out_capacity, uint64_t* d_chunk_bytes,
                              void* d_workspace, size_t workspace_bytes, void* stream)
{
    if (!dtype_ok(dt)) return ZIPCCL_ERR_UNSUPPORTED_DTYPE;
    std::vector<uint64_t> ce;
    if (!resolve_split(n_elems, n_chunks, chunk_elems, ce)) return ZIPCCL_ERR_INVALID_ARG;
    if (d_table ? (reinterpret_cast<uintptr_t>(d_table) % 8) != 0 : !table_ok(table)) return ZIPCCL_ERR_INVALID_ARG;
    if (!d_out || !d_workspace || (!d_in && n_elems)) return ZIPCCL_ERR_INVALID_ARG;
    const uint32_t es = elem_size(dt);
    if ((reinterpret_cast<uintptr_t>(d_in) % es) || (reinterpret_cast<uintptr_t>(d_out) % ZIPCCL_ALIGN) ||
        (reinterpret_cast<uintptr_t>(d_workspace) % 16) || (reinterpret_cast<uintptr_t>(d_chunk_bytes) % 8))
        return ZIPCCL_ERR_INVALID_ARG;

    std::vector<uint64_t> slot_off(n_chunks + 1);
    uint64_t off = 0;
    for (uint32_t c = 0; c < n_chunks; ++c) {
        slot_off[c] = off;
        off += slot_layout(ce[c], dt).cap;
    }
    slot_off[n_chunks] = off;
    if (off > out_capacity) return ZIPCCL_ERR_BUFFER_TOO_SMALL;
    const WorkspacePlan wp = plan_workspace(ce, n_elems);
    if (wp.tiles > 0x7FFFFFFFull) return ZIPCCL_ERR_INVALID_ARG;
    if (wp.min_bytes > workspace_bytes) return ZIPCCL_ERR_BUFFER_TOO_SMALL;
    /* without room for the stash the input is read twice instead */
    const bool stash = wp.full_bytes <= workspace_bytes;

    CompressArgs a;
    std::memset(&a, 0, sizeof a);
    if (d_table) {
        a.d_table = reinterpret_cast<const uint32_t*>(d_table);
        a.table_stride = table_per_chunk ? 2u : 0u;
    } else {
        a.e0 = table->dec[1];
        std::memcpy(&a.dec_lo, table->dec, 4);
        std::memcpy(&a.dec_hi, table->dec + 4, 4);
    }
    uint64_t elem_base = 0, tile_base = 0;
    uint8_t* const ws = static_cast<uint8_t*>(d_workspace);
    for (uint32_t c0 = 0; c0 < n_chunks; c0 += kMaxBatch) {
        const uint32_t nb = (n_chunks - c0) < kMaxBatch ? (n_chunks - c0) : kMaxBatch;
        const uint32_t nt = fill_tab(a.tab, ce, slot_off, c0, nb);
        a.in = static_cast<const uint8_t*>(d_in) + elem_base * es;
        a.out = static_cast<uint8_t*>(d_out) + slot_off[c0];
        a.chunk_bytes = d_chunk_bytes ? d_chunk_bytes + c0 : nullptr;
        if (d_table && table_per_chunk) a.d_table = reinterpret_cast<const uint32_t*>(d_table) + 2 * (uint64_t)c0;
        a.tile_total = reinterpret_cast<uint32_t*>(ws + wp.total_off) + tile_base;
        a.tile_prefix = reinterpret_cast<uint32_t*>(ws + wp.prefix_off) + tile_base;
        a.stash = stash ? ws + wp.stash_off + elem_base : nullptr;
        if (stash) {
            uint32_t max_tiles = 0;
            for (uint32_t c = 0; c < nb; ++c) max_tiles = std::max(max_tiles, a.tab.tile_start[c + 1] - a.tab.tile_start[c]);
            const bool fused_scan = max_tiles <= kPlaceScanTiles;
            if (launch_compress(dt, kModeStash, a, stream) != 0) return ZIPCCL_ERR_DEVICE;
            if (!fused_scan && launch_tile_scan(a, stream) != 0) return ZIPCCL_ERR_DEVICE;
            if (launch_place(dt, fused_scan, a, stream) != 0) return ZIPCCL_ERR_DEVICE;
        } else {
            if (launch_compress(dt, kModeCount, a, stream) != 0) return ZIPCCL_ERR_DEVICE;
            if (launch_tile_scan(a, stream) != 0) return ZIPCCL_ERR_DEVICE;
            if (launch_compress(dt, kModeEmit, a, stream) != 0) return ZIPCCL_ERR_DEVICE;
        }
        elem_base += a.tab.elem_off[nb];
        tile_base += nt;
    }
    return ZIPCCL_OK;
}

} // namespace

extern "C" {

zipccl_status_t zipccl_compress(const void* d_in, size_t n_elems, zipccl_dtype_t dt,
                                uint32_t n_chunks, const uint64_t* chunk_elems,
                                const zipccl_table_t* table,
                                void* d_out, size_t out_capacity, uint64_t* d_chunk_bytes,
                                void* d_workspace, size_t workspace_bytes, void* stream)
{
    return compress_impl(d_in, n_elems, dt, n_chunks, chunk_elems, table, nullptr, false, d_out, out_capacity,
                         d_chunk_bytes, d_workspace, workspace_bytes, stream);
}

zipccl_status_t zipccl_compress_device_table(const void* d_in, size_t n_elems, zipccl_dtype_t dt,
                                             uint32_t n_chunks, const uint64_t* chunk_elems,
                                             const zipccl_table_t* d_table,
                                             void* d_out, size_t out_capacity, uint64_t* d_chunk_bytes,
                                             void* d_workspace, size_t workspace_bytes, void* stream)
{
    if (!d_table) return ZIPCCL_ERR_INVALID_ARG;
    return compress_impl(d_in, n_elems, dt, n_chunks, chunk_elems, nullptr, d_table, false, d_out, out_capacity,
                         d_chunk_bytes, d_workspace, workspace_bytes, stream);
}

zipccl_status_t zipccl_compress_chunk_tables(const void* d_in, size_t n_elems, zipccl_dtype_t dt,
                                             uint32_t n_chunks, const uint64_t* chunk_elems,
                                             const zipccl_table_t* d_tables,
                                             void* d_out, size_t out_capacity, uint64_t* d_chunk_bytes,
                                             void* d_workspace, size_t workspace_bytes, void* stream)
{
    if (!d_tables) return ZIPCCL_ERR_INVALID_ARG;
    return compress_impl(d_in, n_elems, dt, n_chunks, chunk_elems, nullptr, d_tables, true, d_out, out_capacity,
                         d_chunk_bytes, d_workspace, workspace_bytes, stream);
}

zipccl_status_t zipccl_compress_static(const void* d_in, size_t n_elems, zipccl_dtype_t dt,
                                       uint32_t n_chunks, const uint64_t* chunk_elems,
                                       const zipccl_table_t* table,
                                       void* d_out, size_t out_capacity, uint64_t* d_chunk_bytes, void* stream)
{
    if (!dtype_ok(dt)) return ZIPCCL_ERR_UNSUPPORTED_DTYPE;
    /* the size limit first, so that it is reported whatever else is wrong with a call that large */
    const size_t need = zipccl_compress_min_workspace_size(n_elems, dt, n_chunks, chunk_elems);
    if (need == 0) return ZIPCCL_ERR_INVALID_ARG;
    if (need > ZIPCCL_STATIC_SCRATCH_BYTES) return ZIPCCL_ERR_BUFFER_TOO_SMALL;
    void* ws = nullptr;
    size_t ws_bytes = 0;
    if (static_scratch(&ws, &ws_bytes) != 0) return ZIPCCL_ERR_DEVICE;
    return compress_impl(d_in, n_elems, dt, n_chunks, chunk_elems, table, nullptr, false, d_out, out_capacity,
                         d_chunk_bytes, ws, ws_bytes, stream);
}

size_t zipccl_estimate_workspace_size(void) { return 16 * (size_t)kMomentBlocks; }

zipccl_status_t zipccl_estimate_table(const void* d_in, size_t n_elems, zipccl_dtype_t dt,
                                      zipccl_table_t* d_table, double* d_sigma,
                                      void* d_workspace, size_t workspace_bytes, void* stream)
{
    if (!dtype_ok(dt)) return ZIPCCL_ERR_UNSUPPORTED_DTYPE;
    if (!d_table || !d_workspace || (!d_in && n_elems)) return ZIPCCL_ERR_INVALID_ARG;
    if ((reinterpret_cast<uintptr_t>(d_in) % elem_size(dt)) || (reinterpret_cast<uintptr_t>(d_table) % 8) ||
        (reinterpret_cast<uintptr_t>(d_sigma) % 8) || (reinterpret_cast<uintptr_t>(d_workspace) % 8))
        return ZIPCCL_ERR_INVALID_ARG;
    if (workspace_bytes < zipccl_estimate_workspace_size()) return ZIPCCL_ERR_BUFFER_TOO_SMALL;
    MomentArgs a;
    a.in = static_cast<const uint8_t*>(d_in);
    a.n = n_elems;
    a.partial = static_cast<double*>(d_workspace);
    const uint64_t want = (n_elems + 16383) / 16384;             /* about 64 values per thread at least */
    a.n_blocks = (uint32_t)(want < 1 ? 1 : (want > kMomentBlocks ? kMomentBlocks : want));
    a.table = reinterpret_cast<uint8_t*>(d_table);
    a.sigma = d_sigma;
    return launch_estimate(dt, a, stream) == 0 ? ZIPCCL_OK : ZIPCCL_ERR_DEVICE;
}

size_t zipccl_estimate_robust_workspace_size(void) { return kHistBytes; }

size_t zipccl_estimate_chunk_tables_workspace_size(uint32_t n_chunks) { return (size_t)kHistBytes * n_chunks; }

static zipccl_status_t estimate_chunk_tables_impl(const void* d_in, size_t n_elems, zipccl_dtype_t dt,
                                                  uint32_t n_chunks, const uint64_t* chunk_elems, uint32_t sample_stride,
                                                  zipccl_table_t* d_tables, double* d_sigmas,
                                                  void* d_workspace, size_t workspace_bytes, void* stream)
{
    if (!dtype_ok(dt)) return ZIPCCL_ERR_UNSUPPORTED_DTYPE;
    if (sample_stride == 0 || sample_stride > ZIPCCL_MAX_SAMPLE_STRIDE || (sample_stride & (sample_stride - 1u)))
        return ZIPCCL_ERR_INVALID_ARG;
    std::vector<uint64_t> ce;
    if (!resolve_split(n_elems, n_chunks, chunk_elems, ce)) return ZIPCCL_ERR_INVALID_ARG;
    if (!d_tables || !d_workspace || (!d_in && n_elems)) return ZIPCCL_ERR_INVALID_ARG;
    if ((reinterpret_cast<uintptr_t>(d_in) % elem_size(dt)) || (reinterpret_cast<uintptr_t>(d_tables) % 8) ||
        (reinterpret_cast<uintptr_t>(d_sigmas) % 8) || (reinterpret_cast<uintptr_t>(d_workspace) % 8))
        return ZIPCCL_ERR_INVALID_ARG;
    if (workspace_bytes < zipccl_estimate_chunk_tables_workspace_size(n_chunks)) return ZIPCCL_ERR_BUFFER_TOO_SMALL;
    if ((uint64_t)n_chunks * (32768 / 1024) > 0x7FFFFFFFull) return ZIPCCL_ERR_INVALID_ARG;
    unsigned long long* const hist = static_cast<unsigned long long*>(d_workspace);
    /* when every chunk's sample is small enough for one workgroup, one kernel does it all inside LDS: no histogram
       in the workspace, nothing to clear */
    uint64_t largest_of_all = 0;
    for (uint32_t c = 0; c < n_chunks; ++c) largest_of_all = std::max(largest_of_all, ce[c]);
    const bool fused = ((largest_of_all + kGroup - 1) / kGroup + sample_stride - 1) / sample_stride <= kFusedGroups;
    if (!fused && launch_clear_hist(hist, n_chunks, stream) != 0) return ZIPCCL_ERR_DEVICE;
    const std::vector<uint64_t> no_slots(n_chunks + 1, 0);            /* slot offsets play no part here */
    HistArgs a;
    uint64_t elem_base = 0;
    for (uint32_t c0 = 0; c0 < n_chunks; c0 += kMaxBatch) {
        const uint32_t nb = (n_chunks - c0) < kMaxBatch ? (n_chunks - c0) : kMaxBatch;
        fill_tab(a.tab, ce, no_slots, c0, nb);
        uint64_t largest = 0;
        for (uint32_t c = 0; c < nb; ++c) largest = std::max(largest, ce[c0 + c]);
        if (fused) {
            a.n_blocks = 1;
            a.sample_stride = sample_stride;
            a.in = static_cast<const uint8_t*>(d_in) + elem_base * elem_size(dt);
            a.hist = hist;
            a.table = reinterpret_cast<uint8_t*>(d_tables + c0);
            a.sigma = d_sigmas ? d_sigmas + c0 : nullptr;
            if (launch_estimate_robust_fused(dt, a, stream) != 0) return ZIPCCL_ERR_DEVICE;
            elem_base += a.tab.elem_off[nb];
            continue;
        }
        /* a workgroup counts in 32 bits, and wants about 64 values per thread at least (of a sample: four groups
           per wave); about one workgroup per compute unit in all */
        const uint64_t sampled = (largest + sample_stride - 1) / sample_stride;
        const uint64_t want = sample_stride > 1 ? (sampled + 32767) / 32768 : (largest + 65535) / 65536;
        const uint64_t cap = std::max<uint64_t>(1, kHistBlocks / nb);
        a.n_blocks = (uint32_t)std::min(std::max<uint64_t>(want, 1), cap);
        a.sample_stride = sample_stride;
        if (largest / a.n_blocks >= 0xFFFFFFFFull) return ZIPCCL_ERR_INVALID_ARG;
        a.in = static_cast<const uint8_t*>(d_in) + elem_base * elem_size(dt);
        a.hist = hist + (uint64_t)c0 * 32768;
        a.table = reinterpret_cast<uint8_t*>(d_tables + c0);
        a.sigma = d_sigmas ? d_sigmas + c0 : nullptr;
        if (launch_estimate_robust(dt, a, stream) != 0) return ZIPCCL_ERR_DEVICE;
        elem_base += a.tab.elem_off[nb];
    }
    return ZIPCCL_OK;
}

zipccl_status_t zipccl_estimate_chunk_tables(const void* d_in, size_t n_elems, zipccl_dtype_t dt,
                                             uint32_t n_chunks, const uint64_t* chunk_elems,
                                             zipccl_table_t* d_tables, double* d_sigmas,
                                             void* d_workspace, size_t workspace_bytes, void* stream)
{
    return estimate_chunk_tables_impl(d_in, n_elems, dt, n_chunks, chunk_elems, 1, d_tables, d_sigmas, d_workspace,
                                      workspace_bytes, stream);
}

zipccl_status_t zipccl_estimate_chunk_tables_sampled(const void* d_in, size_t n_elems, zipccl_dtype_t dt,
                                                     uint32_t n_chunks, const uint64_t* chunk_elems,
                                                     uint32_t sample_stride,
                                                     zipccl_table_t* d_tables, double* d_sigmas,
                                                     void* d_workspace, size_t workspace_bytes, void* stream)
{
    return estimate_chunk_tables_impl(d_in, n_elems, dt, n_chunks, chunk_elems, sample_stride, d_tables, d_sigmas,
                                      d_workspace, workspace_bytes, stream);
}

zipccl_status_t zipccl_estimate_table_robust(const void* d_in, size_t n_elems, zipccl_dtype_t dt,
                                             zipccl_table_t* d_table, double* d_sigma,
                                             void* d_workspace, size_t workspace_bytes, void* stream)
{
    if (n_elems >= ((size_t)1 << 40)) return ZIPCCL_ERR_INVALID_ARG;      /* a workgroup counts in 32 bits */
    const uint64_t whole = n_elems;                                   /* the tensor as one chunk of any length */
    if (!dtype_ok(dt)) return ZIPCCL_ERR_UNSUPPORTED_DTYPE;
    if (!d_table || !d_workspace || (!d_in && n_elems)) return ZIPCCL_ERR_INVALID_ARG;
    if ((reinterpret_cast<uintptr_t>(d_in) % elem_size(dt)) || (reinterpret_cast<uintptr_t>(d_table) % 8) ||
        (reinterpret_cast<uintptr_t>(d_sigma) % 8) || (reinterpret_cast<uintptr_t>(d_workspace) % 8))
        return ZIPCCL_ERR_INVALID_ARG;
    if (workspace_bytes < zipccl_estimate_robust_workspace_size()) return ZIPCCL_ERR_BUFFER_TOO_SMALL;
    unsigned long long* const hist = static_cast<unsigned long long*>(d_workspace);
    HistArgs a;
    std::memset(&a.tab, 0, sizeof a.tab);
    a.tab.n_chunks = 1;
    for (uint32_t i = 1; i <= kMaxBatch; ++i) a.tab.elem_off[i] = whole;
    const uint64_t want = (whole + 65535) / 65536;                    /* about 64 values per thread at least */
    a.n_blocks = (uint32_t)(want < 1 ? 1 : (want > kHistBlocks ? kHistBlocks : want));
    a.sample_stride = 1;
    a.in = static_cast<const uint8_t*>(d_in);
    a.hist = hist;
    a.table = reinterpret_cast<uint8_t*>(d_table);
    a.sigma = d_sigma;
    /* a tensor one workgroup can take on its own: one kernel, nothing to clear */
    if ((whole + kGroup - 1) / kGroup <= kFusedGroups)
        return launch_estimate_robust_fused(dt, a, stream) == 0 ? ZIPCCL_OK : ZIPCCL_ERR_DEVICE;
    if (launch_clear_hist(hist, 1, stream) != 0) return ZIPCCL_ERR_DEVICE;
    return launch_estimate_robust(dt, a, stream) == 0 ? ZIPCCL_OK : ZIPCCL_ERR_DEVICE;
}

zipccl_status_t zipccl_decompress(const void* d_comp, size_t comp_capacity,
                                  void* d_out, size_t n_elems, zipccl_dtype_t dt,
                                  uint32_t n_chunks, const uint64_t* chunk_elems,
                                  uint32_t* d_status, void* stream)
{
    if (!dtype_ok(dt)) return ZIPCCL_ERR_UNSUPPORTED_DTYPE;
    std::vector<uint64_t> ce;
    if (!resolve_split(n_elems, n_chunks, chunk_elems, ce)) return ZIPCCL_ERR_INVALID_ARG;
    if (!d_comp || (!d_out && n_elems)) return ZIPCCL_ERR_INVALID_ARG;
    const uint32_t es = elem_size(dt);
    if ((reinterpret_cast<uintptr_t>(d_comp) % ZIPCCL_ALIGN) || (reinterpret_cast<uintptr_t>(d_out) % es) ||
        (reinterpret_cast<uintptr_t>(d_status) % 4))
        return ZIPCCL_ERR_INVALID_ARG;

    std::vector<uint64_t> slot_off(n_chunks + 1);
    uint64_t off = 0;
    for (uint32_t c = 0; c < n_chunks; ++c) {
        slot_off[c] = off;
        const SlotLayout L = slot_layout(ce[c], dt);
        if (off + L.esc > comp_capacity) return ZIPCCL_ERR_BUFFER_TOO_SMALL; /* static part must be readable */
        off += L.cap;
    }
    slot_off[n_chunks] = off;
    if (total_tiles(ce) > 0x7FFFFFFFull) return ZIPCCL_ERR_INVALID_ARG;

    DecompressArgs a;
    std::memset(&a, 0, sizeof a);
    a.status = d_status;
    uint64_t elem_base = 0;
    for (uint32_t c0 = 0; c0 < n_chunks; c0 += kMaxBatch) {
        const uint32_t nb = (n_chunks - c0) < kMaxBatch ? (n_chunks - c0) : kMaxBatch;
        fill_tab(a.tab, ce, slot_off, c0, nb);
        a.comp = static_cast<const uint8_t*>(d_comp) + slot_off[c0];
        a.comp_capacity = comp_capacity - slot_off[c0];
        a.out = static_cast<uint8_t*>(d_out) + elem_base * es;
        if (launch_decompress(dt, a, stream) != 0) return ZIPCCL_ERR_DEVICE;
        elem_base += a.tab.elem_off[nb];
    }
    return ZIPCCL_OK;
}

zipccl_status_t zipccl_decompress_reduce(const void* d_comp, size_t comp_capacity, void* d_out, size_t n_elems,
                                         zipccl_dtype_t dt, uint32_t n_peers, zipccl_dtype_t out_dt,
                                         uint32_t* d_status, void* stream)
{
    if (!dtype_ok(dt) || !dtype_ok(out_dt)) return ZIPCCL_ERR_UNSUPPORTED_DTYPE;
    if (n_peers == 0 || n_peers > kMaxPeers || n_elems > ZIPCCL_MAX_CHUNK_ELEMS || !d_comp || (!d_out && n_elems))
        return ZIPCCL_ERR_INVALID_ARG;
    if ((reinterpret_cast<uintptr_t>(d_comp) % ZIPCCL_ALIGN) || (reinterpret_cast<uintptr_t>(d_out) % elem_size(out_dt)) ||
        (reinterpret_cast<uintptr_t>(d_status) % 4))
        return ZIPCCL_ERR_INVALID_ARG;
    const SlotLayout L = slot_layout(n_elems, dt);
    if ((uint64_t)(n_peers - 1) * L.cap + L.esc > comp_capacity) return ZIPCCL_ERR_BUFFER_TOO_SMALL;
    ReduceArgs a;
    a.comp = static_cast<const uint8_t*>(d_comp);
    a.comp_capacity = comp_capacity;
    a.slot_cap = L.cap;
    a.out = static_cast<uint8_t*>(d_out);
    a.status = d_status;
    a.n = n_elems;
    a.n_peers = n_peers;
    return launch_decompress_reduce(dt, out_dt, a, stream) == 0 ? ZIPCCL_OK : ZIPCCL_ERR_DEVICE;
}

int zipccl_switch_prefers_zipped(const zipccl_link_model_t* m, double d_bytes, double e, double s,
                                 double* t_rs, double* t_a2a)
{
    auto ok = [](double v) { return std::isfinite(v) && v >= 0.0; };
    if (!m || !ok(m->alpha_rs) || !ok(m->beta_rs) || !ok(m->alpha_a2a) || !ok(m->beta_a2a) || !ok(d_bytes) ||
        !ok(e) || !ok(s))
        return -1;
    const double rs = m->alpha_rs + m->beta_rs * d_bytes;                  /* Eq.6 */
    const double a2a = m->alpha_a2a + m->beta_a2a * e * s * d_bytes;       /* Eq.7 */
    if (t_rs) *t_rs = rs;
    if (t_a2a) *t_a2a = a2a;
    return a2a < rs ? 1 : 0;
}

zipccl_status_t zipccl_fit_link_model(const double* d_bytes, const double* t_seconds, size_t k,
                                      double* alpha, double* beta)
{
    if (!d_bytes || !t_seconds || !alpha || !beta || k < 2) return ZIPCCL_ERR_INVALID_ARG;
    double md = 0.0, mt = 0.0;
    for (size_t i = 0; i < k; ++i) {
        if (!std::isfinite(d_bytes[i]) || !std::isfinite(t_seconds[i])) return ZIPCCL_ERR_INVALID_ARG;
        md += d_bytes[i];
        mt += t_seconds[i];
    }
    md /= (double)k;
    mt /= (double)k;
    double sxx = 0.0, sxy = 0.0;
    for (size_t i = 0; i < k; ++i) {
        sxx += (d_bytes[i] - md) * (d_bytes[i] - md);
        sxy += (d_bytes[i] - md) * (t_seconds[i] - mt);
    }
    if (!(sxx > 0.0)) return ZIPCCL_ERR_INVALID_ARG;
    *beta = sxy / sxx;
    *alpha = mt - *beta * md;
    return ZIPCCL_OK;
}

const char* zipccl_status_string(zipccl_status_t s)
{
    switch (s) {
        case ZIPCCL_OK: return "ok";
        case ZIPCCL_ERR_INVALID_ARG: return "invalid argument";
        case ZIPCCL_ERR_UNSUPPORTED_DTYPE: return "unsupported dtype";
        case ZIPCCL_ERR_BUFFER_TOO_SMALL: return "buffer too small";
        case ZIPCCL_ERR_CORRUPT: return "corrupt compressed data";
        case ZIPCCL_ERR_DEVICE: return "device error";
    }
    return "unknown status";
}

} // extern "C"
