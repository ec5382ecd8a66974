/*
 * Sanitizer driver for the host side of libzipccl.so (csrc/zipccl_host.cpp): built with g++ under
 * -fsanitize=address,undefined together with stand-ins for the kernel launchers (no HIP, no GPU), and run by
 * tests/test_sanitizers.py.  It calls the pure-host entry points (table, sizes, offsets, switcher) on exact-size
 * host arrays, and the device entry points with arguments that must be rejected before anything is launched;
 * calls that pass the checks reach the stand-in launchers, which verify the geometry they are handed.
 */
#include <cmath>
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <vector>

#include "zipccl_internal.h"

#define CHECK(c) do { if (!(c)) { std::fprintf(stderr, "check failed at line %d: %s\n", __LINE__, #c); std::exit(1); } } while (0)

namespace zipccl {

static int g_launches = 0;

/* the geometry every launch is handed must be consistent: tiles ascending, offsets ascending */
static void check_tab(const ChunkTab& t)
{
    CHECK(t.n_chunks >= 1 && t.n_chunks <= kMaxBatch);
    for (uint32_t c = 0; c < kMaxBatch; ++c) {
        CHECK(t.tile_start[c] <= t.tile_start[c + 1]);
        CHECK(t.elem_off[c] <= t.elem_off[c + 1]);
        CHECK(t.slot_off[c] <= t.slot_off[c + 1]);
        CHECK(t.slot_off[c] % ZIPCCL_ALIGN == 0);
    }
}

int launch_estimate(int, const MomentArgs& a, void*) { CHECK(a.n_blocks >= 1 && a.n_blocks <= kMomentBlocks); ++g_launches; return 0; }
int launch_clear_hist(unsigned long long* hist, uint32_t n_chunks, void*) { CHECK(hist != nullptr && n_chunks >= 1); ++g_launches; return 0; }
int launch_estimate_robust(int, const HistArgs& a, void*)
{
    CHECK(a.n_blocks >= 1 && a.n_blocks <= kHistBlocks && a.tab.n_chunks >= 1 && a.tab.n_chunks <= kMaxBatch);
    CHECK(a.sample_stride >= 1 && a.sample_stride <= ZIPCCL_MAX_SAMPLE_STRIDE && (a.sample_stride & (a.sample_stride - 1)) == 0);
    for (uint32_t c = 0; c < kMaxBatch; ++c) CHECK(a.tab.elem_off[c] <= a.tab.elem_off[c + 1]);
    ++g_launches;
    return 0;
}
int launch_estimate_robust_fused(int dt, const HistArgs& a, void* s)
{
    for (uint32_t c = 0; c < a.tab.n_chunks; ++c)           /* one workgroup per chunk: its sample must be small */
        CHECK(((a.tab.elem_off[c + 1] - a.tab.elem_off[c] + kGroup - 1) / kGroup + a.sample_stride - 1) / a.sample_stride <= kFusedGroups);
    return launch_estimate_robust(dt, a, s);
}
int launch_compress(int, int, const CompressArgs& a, void*) { check_tab(a.tab); ++g_launches; return 0; }
int launch_tile_scan(const CompressArgs& a, void*) { check_tab(a.tab); ++g_launches; return 0; }
int launch_place(int, bool, const CompressArgs& a, void*) { check_tab(a.tab); ++g_launches; return 0; }
int launch_decompress(int, const DecompressArgs& a, void*) { check_tab(a.tab); ++g_launches; return 0; }
int launch_decompress_reduce(int, int, const ReduceArgs& a, void*) { CHECK(a.n_peers >= 1 && a.n_peers <= kMaxPeers); ++g_launches; return 0; }
int static_scratch(void** ptr, size_t* bytes)
{
    static uint64_t fake[4];                        /* never dereferenced: the stand-in launchers touch no buffer */
    *ptr = fake;
    *bytes = ZIPCCL_STATIC_SCRATCH_BYTES;
    return 0;
}

} // namespace zipccl

int main()
{
    using namespace zipccl;
    /* table builder over a wide sigma range, clamps and rejections */
    zipccl_table_t t;
    for (int k = -1100; k <= 1100; ++k) {
        const double s = std::ldexp(1.37, k);
        if (!(s > 0.0) || std::isinf(s)) continue;
        CHECK(zipccl_build_table(s, ZIPCCL_BF16, &t) == ZIPCCL_OK);
        CHECK(t.dec[1] >= 1 && t.dec[1] <= 248 && t.dec[7] == t.dec[1] + 6);
    }
    CHECK(zipccl_build_table(0.0, ZIPCCL_BF16, &t) == ZIPCCL_ERR_INVALID_ARG);
    CHECK(zipccl_build_table(NAN, ZIPCCL_BF16, &t) == ZIPCCL_ERR_INVALID_ARG);
    CHECK(zipccl_build_table(INFINITY, ZIPCCL_FP32, &t) == ZIPCCL_ERR_INVALID_ARG);
    CHECK(zipccl_build_table(1.0, ZIPCCL_BF16, nullptr) == ZIPCCL_ERR_INVALID_ARG);
    CHECK(zipccl_build_table(1.0, (zipccl_dtype_t)9, &t) == ZIPCCL_ERR_UNSUPPORTED_DTYPE);
    CHECK(zipccl_build_table(1.0, ZIPCCL_BF16, &t) == ZIPCCL_OK && t.dec[1] == 122);

    /* sizes and offsets: exact-size arrays, more chunks than one launch holds, empty chunks, bad splits */
    const uint32_t C = 300;
    std::vector<uint64_t> ce(C), off(C + 1), st(C);
    uint64_t n = 0;
    for (uint32_t c = 0; c < C; ++c) { ce[c] = (c * 7919u) % 20000u * (c % 5 != 0); n += ce[c]; }
    CHECK(zipccl_chunk_slot_offsets(n, ZIPCCL_FP32, C, ce.data(), off.data()) == ZIPCCL_OK);
    CHECK(zipccl_chunk_static_bytes(n, ZIPCCL_FP32, C, ce.data(), st.data()) == ZIPCCL_OK);
    CHECK(zipccl_max_compressed_size(n, ZIPCCL_FP32, C, ce.data()) == off[C]);
    for (uint32_t c = 0; c < C; ++c) CHECK(off[c] % 128 == 0 && st[c] <= off[c + 1] - off[c]);
    CHECK(zipccl_max_compressed_size(n + 1, ZIPCCL_FP32, C, ce.data()) == 0);
    CHECK(zipccl_max_compressed_size(10, ZIPCCL_BF16, 3, nullptr) == 0);
    CHECK(zipccl_max_compressed_size(10, ZIPCCL_BF16, 0, nullptr) == 0);
    ce[0] = ZIPCCL_MAX_CHUNK_ELEMS + 1;
    CHECK(zipccl_chunk_slot_offsets(n, ZIPCCL_FP32, C, ce.data(), off.data()) == ZIPCCL_ERR_INVALID_ARG);
    ce[0] = ~0ull; ce[1] = 2;                                         /* a sum that wraps */
    CHECK(zipccl_max_compressed_size(1, ZIPCCL_BF16, C, ce.data()) == 0);
    ce[0] = 0; ce[1] = (1 * 7919u) % 20000u;
    CHECK(zipccl_compress_workspace_size(n, ZIPCCL_FP32, C, ce.data()) > zipccl_compress_min_workspace_size(n, ZIPCCL_FP32, C, ce.data()));

    /* device entry points: rejected arguments never reach a launcher; accepted ones hand over consistent geometry.
       The pointers are only compared and aligned, never dereferenced by the stand-ins. */
    alignas(256) static uint8_t in[64], out[256], ws[256];
    const size_t big = (size_t)1 << 40;
    CHECK(zipccl_build_table(1.0, ZIPCCL_BF16, &t) == ZIPCCL_OK);
    g_launches = 0;
    CHECK(zipccl_compress(nullptr, 8, ZIPCCL_BF16, 1, nullptr, &t, out, big, nullptr, ws, big, nullptr) == ZIPCCL_ERR_INVALID_ARG);
    CHECK(zipccl_compress(in + 1, 8, ZIPCCL_BF16, 1, nullptr, &t, out, big, nullptr, ws, big, nullptr) == ZIPCCL_ERR_INVALID_ARG);
    CHECK(zipccl_compress(in, 8, ZIPCCL_BF16, 1, nullptr, &t, out + 64, big, nullptr, ws, big, nullptr) == ZIPCCL_ERR_INVALID_ARG);
    CHECK(zipccl_compress(in, 8, ZIPCCL_BF16, 1, nullptr, &t, out, 100, nullptr, ws, big, nullptr) == ZIPCCL_ERR_BUFFER_TOO_SMALL);
    CHECK(zipccl_compress(in, 8, ZIPCCL_BF16, 1, nullptr, &t, out, big, nullptr, ws, 16, nullptr) == ZIPCCL_ERR_BUFFER_TOO_SMALL);
    zipccl_table_t bad = t; bad.dec[3] = 7;
    CHECK(zipccl_compress(in, 8, ZIPCCL_BF16, 1, nullptr, &bad, out, big, nullptr, ws, big, nullptr) == ZIPCCL_ERR_INVALID_ARG);
    CHECK(zipccl_compress(in, 8, ZIPCCL_BF16, 1, nullptr, nullptr, out, big, nullptr, ws, big, nullptr) == ZIPCCL_ERR_INVALID_ARG);
    CHECK(zipccl_decompress(out, 100, in, 8, ZIPCCL_BF16, 1, nullptr, nullptr, nullptr) == ZIPCCL_ERR_BUFFER_TOO_SMALL);
    CHECK(zipccl_decompress(out + 1, big, in, 8, ZIPCCL_BF16, 1, nullptr, nullptr, nullptr) == ZIPCCL_ERR_INVALID_ARG);
    CHECK(zipccl_decompress_reduce(out, big, in, 8, ZIPCCL_BF16, 0, ZIPCCL_FP32, nullptr, nullptr) == ZIPCCL_ERR_INVALID_ARG);
    CHECK(zipccl_decompress_reduce(out, big, in, 8, ZIPCCL_BF16, 1025, ZIPCCL_FP32, nullptr, nullptr) == ZIPCCL_ERR_INVALID_ARG);
    CHECK(zipccl_decompress_reduce(out, 100, in, 8, ZIPCCL_BF16, 2, ZIPCCL_FP32, nullptr, nullptr) == ZIPCCL_ERR_BUFFER_TOO_SMALL);
    CHECK(zipccl_estimate_table(in, 8, ZIPCCL_BF16, (zipccl_table_t*)out, nullptr, ws, 8, nullptr) == ZIPCCL_ERR_BUFFER_TOO_SMALL);
    CHECK(zipccl_estimate_table_robust(in, 8, ZIPCCL_BF16, (zipccl_table_t*)out, nullptr, ws, 8, nullptr) == ZIPCCL_ERR_BUFFER_TOO_SMALL);
    CHECK(zipccl_compress_static(in, (size_t)16 << 31, ZIPCCL_BF16, 16, nullptr, &t, out, big * 1024, nullptr, nullptr) == ZIPCCL_ERR_BUFFER_TOO_SMALL);
    CHECK(g_launches == 0);
    /* accepted calls, with the 300-chunk split (three launches' worth of chunk tables) */
    CHECK(zipccl_compress(in, n, ZIPCCL_FP32, C, ce.data(), &t, out, big, nullptr, ws, big, nullptr) == ZIPCCL_OK);
    CHECK(zipccl_compress(in, n, ZIPCCL_FP32, C, ce.data(), &t, out, big, nullptr, ws,
                          zipccl_compress_min_workspace_size(n, ZIPCCL_FP32, C, ce.data()), nullptr) == ZIPCCL_OK);
    CHECK(zipccl_compress_static(in, n, ZIPCCL_FP32, C, ce.data(), &t, out, big, nullptr, nullptr) == ZIPCCL_OK);
    CHECK(zipccl_decompress(out, big, in, n, ZIPCCL_FP32, C, ce.data(), nullptr, nullptr) == ZIPCCL_OK);
    CHECK(zipccl_decompress_reduce(out, big, in, 5000, ZIPCCL_BF16, 1024, ZIPCCL_BF16, nullptr, nullptr) == ZIPCCL_OK);
    CHECK(zipccl_estimate_table(in, 100000, ZIPCCL_BF16, (zipccl_table_t*)out, nullptr, ws, big, nullptr) == ZIPCCL_OK);
    CHECK(zipccl_estimate_table_robust(in, 100000, ZIPCCL_BF16, (zipccl_table_t*)out, nullptr, ws, big, nullptr) == ZIPCCL_OK);
    CHECK(zipccl_estimate_chunk_tables(in, n, ZIPCCL_FP32, C, ce.data(), (zipccl_table_t*)out, nullptr, ws, big, nullptr) == ZIPCCL_OK);
    CHECK(zipccl_estimate_chunk_tables(in, n, ZIPCCL_FP32, C, ce.data(), (zipccl_table_t*)out, nullptr, ws, 1000, nullptr) == ZIPCCL_ERR_BUFFER_TOO_SMALL);
    CHECK(zipccl_estimate_chunk_tables(in, n + 1, ZIPCCL_FP32, C, ce.data(), (zipccl_table_t*)out, nullptr, ws, big, nullptr) == ZIPCCL_ERR_INVALID_ARG);
    for (uint32_t stride : {1u, 2u, 16u, 4096u})
        CHECK(zipccl_estimate_chunk_tables_sampled(in, n, ZIPCCL_FP32, C, ce.data(), stride, (zipccl_table_t*)out, nullptr, ws, big, nullptr) == ZIPCCL_OK);
    for (uint32_t stride : {0u, 3u, 48u, 8192u, 0x80000000u})
        CHECK(zipccl_estimate_chunk_tables_sampled(in, n, ZIPCCL_FP32, C, ce.data(), stride, (zipccl_table_t*)out, nullptr, ws, big, nullptr) == ZIPCCL_ERR_INVALID_ARG);
    CHECK(zipccl_compress_chunk_tables(in, n, ZIPCCL_FP32, C, ce.data(), (const zipccl_table_t*)out, out, big, nullptr, ws, big, nullptr) == ZIPCCL_OK);
    CHECK(zipccl_compress_chunk_tables(in, n, ZIPCCL_FP32, C, ce.data(), nullptr, out, big, nullptr, ws, big, nullptr) == ZIPCCL_ERR_INVALID_ARG);
    CHECK(g_launches > 0);

    /* switcher */
    zipccl_link_model_t m{1e-5, 1e-10, 2e-5, 1e-10};
    double a = 0, b = 0;
    CHECK(zipccl_switch_prefers_zipped(&m, 1e9, 0.7, 1.0, &a, &b) == 1 && b < a);
    CHECK(zipccl_switch_prefers_zipped(&m, 1e3, 0.7, 1.0, nullptr, nullptr) == 0);
    CHECK(zipccl_switch_prefers_zipped(nullptr, 1e3, 0.7, 1.0, nullptr, nullptr) == -1);
    CHECK(zipccl_switch_prefers_zipped(&m, NAN, 0.7, 1.0, nullptr, nullptr) == -1);
    const double ds[4] = {1e6, 2e6, 4e6, 8e6}, ts[4] = {1.1e-3, 2.1e-3, 4.1e-3, 8.1e-3};
    CHECK(zipccl_fit_link_model(ds, ts, 4, &a, &b) == ZIPCCL_OK && std::fabs(a - 1e-4) < 1e-9 && std::fabs(b - 1e-9) < 1e-15);
    CHECK(zipccl_fit_link_model(ds, ts, 1, &a, &b) == ZIPCCL_ERR_INVALID_ARG);
    const double same[2] = {5.0, 5.0};
    CHECK(zipccl_fit_link_model(same, ts, 2, &a, &b) == ZIPCCL_ERR_INVALID_ARG);
    for (int s = 0; s <= 6; ++s) CHECK(zipccl_status_string((zipccl_status_t)s) != nullptr);
    std::puts("host sanitizer driver: ok");
    return 0;
}
