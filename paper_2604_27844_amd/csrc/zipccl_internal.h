/* Internal declarations shared by the host logic and the HIP kernels of libzipccl.so. */
#ifndef ZIPCCL_INTERNAL_H
#define ZIPCCL_INTERNAL_H

#include <stddef.h>
#include <stdint.h>
#include "zipccl.h"

#if defined(__HIPCC__)
#define ZIPCCL_HD __host__ __device__ inline
#else
#define ZIPCCL_HD inline
#endif

namespace zipccl {

/* Work decomposition: a workgroup of 4 wave64 handles one TILE of 16 groups; a wave handles
 * a group of 512 elements at a time, 8 consecutive elements per lane (one 16-byte bf16 load). */
constexpr uint32_t kLaneElems = 8;
constexpr uint32_t kGroup = ZIPCCL_GROUP;
constexpr uint32_t kWavesPerBlock = 4;
constexpr uint32_t kThreads = 64 * kWavesPerBlock;
constexpr uint32_t kGroupsPerWave = 4;
constexpr uint32_t kGroupsPerTile = kWavesPerBlock * kGroupsPerWave;
constexpr uint32_t kTile = kGroup * kGroupsPerTile; /* 8192 elements */
constexpr uint32_t kMaxBatch = 128;                 /* chunks per kernel launch */
constexpr uint32_t kVersion = 1;
constexpr uint32_t kMagic = 0x4C43505Au;            /* "ZPCL" little-endian */
constexpr uint32_t kWorkspaceHeader = 256;          /* reserved bytes before the per-tile arrays */
constexpr uint32_t kMaxPeers = 1024;                /* slots one zipccl_decompress_reduce call can sum */
constexpr uint32_t kFusedGroups = 512;              /* sampled groups of a chunk that one workgroup takes on its own */
constexpr uint32_t kStashSlack = 64;                /* readable bytes past the last stash byte */

/* header words (u32 index): 0 magic, 1 version, 2 dtype, 3 G, 4-5 n, 6-7 n_esc, 8-9 chunk_bytes, 10-11 dec[8] */

ZIPCCL_HD uint64_t pad128(uint64_t x) { return (x + 127u) & ~(uint64_t)127u; }
ZIPCCL_HD uint32_t elem_size(int dt) { return dt == ZIPCCL_BF16 ? 2u : 4u; }

/* Byte offsets of the sections inside a slot of n elements (all multiples of 128). */
struct SlotLayout {
    uint64_t sm, lo, p0, plane_bytes, idx, esc, cap;
};

ZIPCCL_HD SlotLayout slot_layout(uint64_t n, int dt)
{
    SlotLayout L;
    L.sm = 128;
    L.lo = L.sm + pad128(n);
    L.p0 = L.lo + (dt == ZIPCCL_FP32 ? pad128(2 * n) : 0);
    L.plane_bytes = pad128((n + 7) / 8);
    L.idx = L.p0 + 3 * L.plane_bytes;
    L.esc = L.idx + pad128(4 * ((n + kGroup - 1) / kGroup));
    L.cap = L.esc + pad128(n);
    return L;
}

ZIPCCL_HD uint64_t tiles_of(uint64_t n) { return n == 0 ? 1 : (n + kTile - 1) / kTile; }

/* Per-launch chunk table, passed by value in the kernel argument segment. */
struct ChunkTab {
    uint32_t n_chunks;
    uint32_t tile_start[kMaxBatch + 1]; /* first tile of chunk c in this launch */
    uint64_t elem_off[kMaxBatch + 1];   /* first element of chunk c, relative to the launch's input */
    uint64_t slot_off[kMaxBatch + 1];   /* byte offset of slot c, relative to the launch's output */
};

struct CompressArgs {
    const uint8_t* in;       /* first element of the launch's first chunk */
    uint8_t* out;            /* compressed buffer base for this launch */
    uint64_t* chunk_bytes;   /* entry of the launch's first chunk, or null */
    uint32_t* tile_total;    /* one u32 per tile of this launch: its zero-point count */
    uint32_t* tile_prefix;   /* one u32 per tile: zero-points of its chunk before it */
    uint8_t* stash;          /* stash mode: one byte per input element of this launch (+ slack) */
    uint32_t e0;             /* dec[1] */
    uint32_t dec_lo, dec_hi; /* dec[0..3], dec[4..7] packed little-endian */
    const uint32_t* d_table; /* when not null: the table lives in device memory (two words), e0/dec_* unused */
    uint32_t table_stride;   /* words from one chunk's table to the next: 0 = one table for all chunks, 2 = one each */
    ChunkTab tab;
};

constexpr uint32_t kPlaceScanTiles = 4096;            /* largest chunk (in tiles) for which k_place does the tile scan itself */
constexpr uint32_t kMomentBlocks = 2048;             /* workgroups (and partial sums) of the sigma estimate */

struct MomentArgs {
    const uint8_t* in;
    uint64_t n;
    double* partial;         /* 2 doubles per workgroup: sum d, sum d^2 with d = x - first value */
    uint32_t n_blocks;
    uint8_t* table;          /* device zipccl_table_t (8 bytes) */
    double* sigma;           /* may be null */
};

constexpr uint32_t kHistBlocks = 256;                /* workgroups of the magnitude histogram: one per compute unit */
constexpr uint32_t kHistBytes = 32768 * 8;           /* its workspace: one 64-bit count per 15-bit magnitude */

struct HistArgs {
    const uint8_t* in;       /* first element of the launch's first chunk */
    unsigned long long* hist;   /* 32768 counts per chunk of the launch, zeroed by the first kernel of the call */
    uint32_t n_blocks;       /* workgroups per chunk */
    uint32_t sample_stride;  /* 1: every value counts; a power of two S: one group of 512 values per S groups */
    uint8_t* table;          /* device zipccl_table_t (8 bytes) per chunk of the launch */
    double* sigma;           /* one per chunk of the launch; may be null */
    ChunkTab tab;            /* the launch's chunks (elem_off; the other fields are not used) */
};

struct DecompressArgs {
    const uint8_t* comp;
    uint64_t comp_capacity;  /* readable bytes from comp */
    uint8_t* out;
    uint32_t* status;        /* may be null */
    ChunkTab tab;
};

/* kModeStash: single pass over the input; zero-point exponents go to a stash at a position that
 * does not depend on other tiles, and k_place moves them once the tile prefixes are known.
 * kModeCount + kModeEmit: the same without a stash, reading the input twice. */
struct ReduceArgs {
    const uint8_t* comp;     /* n_peers slots of n values each, back to back */
    uint64_t comp_capacity;  /* readable bytes from comp */
    uint64_t slot_cap;       /* bytes from one slot to the next */
    uint8_t* out;            /* n sums */
    uint32_t* status;        /* may be null */
    uint64_t n;
    uint32_t n_peers;
    /* set by the launcher: */
    uint32_t gpw;            /* groups per wave in the workgroups that take whole tiles */
    uint32_t n_full;         /* how many those are: workgroups 0 .. n_full - 1 */
    uint32_t gpw_rest;       /* groups per wave in the workgroups after them, which take the rest of the shard */
};

enum CompressMode { kModeCount = 0, kModeEmit = 1, kModeStash = 2 };

/* launchers implemented next to their kernels (zipccl_compress.hip, zipccl_decompress.hip, zipccl_aux.hip);
 * they return a hipError_t as int */
int launch_estimate(int dt, const MomentArgs& a, void* stream);
int launch_clear_hist(unsigned long long* hist, uint32_t n_chunks, void* stream);
int launch_estimate_robust(int dt, const HistArgs& a, void* stream);
int launch_estimate_robust_fused(int dt, const HistArgs& a, void* stream);   /* chunks of at most kFusedGroups sampled groups */
int launch_compress(int dt, int mode, const CompressArgs& a, void* stream);
/* device address and size of the library's own workspace on the current GPU (zipccl_compress_static) */
int static_scratch(void** ptr, size_t* bytes);
int launch_tile_scan(const CompressArgs& a, void* stream);
int launch_place(int dt, bool scan, const CompressArgs& a, void* stream);
int launch_decompress(int dt, const DecompressArgs& a, void* stream);
int launch_decompress_reduce(int dt, int out_dt, const ReduceArgs& a, void* stream);

} // namespace zipccl
#endif
