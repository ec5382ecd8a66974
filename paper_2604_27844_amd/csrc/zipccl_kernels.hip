/*
 * HIP kernels of libzipccl.so for gfx950 (CDNA4, wave64).
 *
 * compress   : paper section 4 (split, 3-bit code, zero-points) with the kernel steps of
 *              section 4.2 re-designed for wave64: one wave handles a group of 512 values,
 *              8 consecutive values per lane (one 16-byte load for bf16), a workgroup of
 *              4 waves handles a tile of 16 groups.  Per lane the work is SWAR on packed
 *              words: v_perm_b32 gathers the sign/mantissa and exponent bytes, packed 16-bit
 *              sub/min produce the codes, v_dot4_u32_u8 transposes code bits into plane bytes.
 *              Plane bytes and zero-point exponents are staged in LDS and leave as wide
 *              stores.  The zero-point offsets of section 4.2.3 are an exclusive prefix in
 *              element order (lane -> wave -> tile -> chunk), so the output is deterministic.
 *              No workgroup ever waits for another: the chunk-wide level, which the paper does
 *              with a block-level atomic add inside the kernel, is a kernel boundary here.
 *              k_compress<kModeStash> writes everything whose place is known (SM, LO, planes,
 *              tile-local index) and parks the zero-point exponents of its tile in a stash;
 *              k_tile_scan turns the per-tile counts into per-chunk prefixes; k_place moves
 *              each tile's exponents to their final place and finishes index and header.
 *              (Waiting in-kernel for the predecessors' counts costs a tile ~10 us of lateness
 *              of the slowest of them, measured; the stash costs ~2 % extra traffic.)
 * decompress : section 4, third paragraph.  No dependency between workgroups.
 *
 * Everything is integer work; sigma / erf live on the host.
 */
#include <hip/hip_runtime.h>

#include "zipccl_internal.h"

namespace zipccl {
namespace {

typedef unsigned short us2 __attribute__((ext_vector_type(2)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

/* streaming accesses: every tensor byte is touched once, so keep it out of the way of the caches */
template <typename T>
__device__ __forceinline__ T ld_stream(const void* p) { return __builtin_nontemporal_load(static_cast<const T*>(p)); }
template <typename T>
__device__ __forceinline__ void st_stream(void* p, T v) { __builtin_nontemporal_store(v, static_cast<T*>(p)); }

__device__ __forceinline__ uint32_t pk_sub_u16(uint32_t a, uint32_t b)
{
    return __builtin_bit_cast(uint32_t, (us2)(__builtin_bit_cast(us2, a) - __builtin_bit_cast(us2, b)));
}
__device__ __forceinline__ uint32_t pk_min_u16(uint32_t a, uint32_t b)
{
    return __builtin_bit_cast(uint32_t, __builtin_elementwise_min(__builtin_bit_cast(us2, a), __builtin_bit_cast(us2, b)));
}
/* byte k of the result = byte sel.k of the 8-byte pool {hi:lo} (indices 0-3 = lo, 4-7 = hi, 0x0c = 0) */
__device__ __forceinline__ uint32_t perm(uint32_t hi, uint32_t lo, uint32_t sel)
{
    return __builtin_amdgcn_perm(hi, lo, sel);
}
__device__ __forceinline__ uint32_t bfi(uint32_t mask, uint32_t a, uint32_t b) { return (a & mask) | (b & ~mask); }

__device__ __forceinline__ uint32_t lane_id()
{
    return __builtin_amdgcn_mbcnt_hi(~0u, __builtin_amdgcn_mbcnt_lo(~0u, 0u));
}

/* inclusive prefix sum over the 64 lanes of a wave (DPP row shifts, then row broadcasts) */
__device__ __forceinline__ uint32_t wave_incl_scan(uint32_t x)
{
    x += __builtin_amdgcn_update_dpp(0u, x, 0x111, 0xF, 0xF, true);  /* row_shr:1 */
    x += __builtin_amdgcn_update_dpp(0u, x, 0x112, 0xF, 0xF, true);  /* row_shr:2 */
    x += __builtin_amdgcn_update_dpp(0u, x, 0x114, 0xF, 0xF, true);  /* row_shr:4 */
    x += __builtin_amdgcn_update_dpp(0u, x, 0x118, 0xF, 0xF, true);  /* row_shr:8 */
    x += __builtin_amdgcn_update_dpp(0u, x, 0x142, 0xA, 0xF, false); /* row_bcast:15 into rows 1,3 */
    x += __builtin_amdgcn_update_dpp(0u, x, 0x143, 0xC, 0xF, false); /* row_bcast:31 into rows 2,3 */
    return x;
}

/* inclusive prefix sum inside each row of 16 lanes */
__device__ __forceinline__ uint32_t row_incl_scan(uint32_t x)
{
    x += __builtin_amdgcn_update_dpp(0u, x, 0x111, 0xF, 0xF, true);
    x += __builtin_amdgcn_update_dpp(0u, x, 0x112, 0xF, 0xF, true);
    x += __builtin_amdgcn_update_dpp(0u, x, 0x114, 0xF, 0xF, true);
    x += __builtin_amdgcn_update_dpp(0u, x, 0x118, 0xF, 0xF, true);
    return x;
}

/*
 * Load the lane's 8 consecutive values starting at chunk-relative element e.
 * hp[k] packs the high 16-bit words of values 2k (low half) and 2k+1 (high half);
 * lp[k] the low words (fp32 only).  vmask bit j = value j exists (e + j < n).
 * Values that do not exist read as 0.
 */
template <int DT, bool FAST>
__device__ __forceinline__ void load_lane(const uint8_t* __restrict__ cin, uint64_t gbase, uint32_t lane, uint64_t n,
                                          uint32_t hp[4], uint32_t lp[4], uint32_t& vmask)
{
    /* gbase (first value of the group) is wave-uniform: uniform 64-bit base + 32-bit lane offset */
    const uint64_t e = gbase + lane * kLaneElems;
    if (FAST) {
        vmask = 0xFFu;
        if (DT == ZIPCCL_BF16) {
            const u32x4 v = ld_stream<u32x4>((cin + gbase * 2) + lane * 16u);
            hp[0] = v.x; hp[1] = v.y; hp[2] = v.z; hp[3] = v.w;
            lp[0] = lp[1] = lp[2] = lp[3] = 0;
        } else {
            const u32x4 a = ld_stream<u32x4>((cin + gbase * 4) + lane * 32u);
            const u32x4 b = ld_stream<u32x4>((cin + gbase * 4 + 16) + lane * 32u);
            const uint32_t x[8] = {a.x, a.y, a.z, a.w, b.x, b.y, b.z, b.w};
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                hp[k] = perm(x[2 * k + 1], x[2 * k], 0x07060302u);
                lp[k] = perm(x[2 * k + 1], x[2 * k], 0x05040100u);
            }
        }
    } else {
        vmask = 0;
#pragma unroll
        for (int k = 0; k < 4; ++k) { hp[k] = 0; lp[k] = 0; }
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const uint64_t i = e + j;
            if (i < n) {
                uint32_t hi16, lo16 = 0;
                if (DT == ZIPCCL_BF16) {
                    hi16 = *reinterpret_cast<const uint16_t*>(cin + i * 2);
                } else {
                    const uint32_t x = *reinterpret_cast<const uint32_t*>(cin + i * 4);
                    hi16 = x >> 16;
                    lo16 = x & 0xFFFFu;
                }
                hp[j >> 1] |= hi16 << (16 * (j & 1));
                lp[j >> 1] |= lo16 << (16 * (j & 1));
                vmask |= 1u << j;
            }
        }
    }
}

/* What a lane derives from its 8 values (section 4: split, code, zero-point detection). */
struct LaneEnc {
    uint32_t sm0, sm1;      /* 8 sign+mantissa bytes */
    uint32_t ex0, ex1;      /* 8 raw exponent bytes */
    uint32_t b0, b1, b2;    /* plane bytes: bit j = bit k of the code of value j */
    uint32_t m;             /* bit j = value j is a zero-point (before masking non-existent values) */
};

/*
 * SWAR encode of 8 values held as four packed pairs of 16-bit words.
 * k7 = (dec[1] - 1) << 7 in both halves; a value of exponent E has
 * t = E - (dec[1] - 1): code = t for t in 1..7, zero-point otherwise.
 */
__device__ __forceinline__ LaneEnc encode8(const uint32_t w[4], uint32_t k7)
{
    LaneEnc r;
    uint32_t c4[2];
#pragma unroll
    for (int h = 0; h < 2; ++h) {
        const uint32_t wa = w[2 * h], wb = w[2 * h + 1];
        const uint32_t lo = perm(wb, wa, 0x06040200u);   /* low bytes: mantissa | E bit 0 << 7 */
        const uint32_t hi = perm(wb, wa, 0x07050301u);   /* high bytes: sign << 7 | E >> 1 */
        const uint32_t sm = bfi(0x7F7F7F7Fu, lo, hi);
        const uint32_t ex = bfi(0xFEFEFEFEu, hi << 1, lo >> 7);
        /* (E << 7) - k7 per half, clamped to 8 << 7: 1..7 << 7 inside the window */
        const uint32_t qa = pk_min_u16(pk_sub_u16(wa & 0x7F807F80u, k7), 0x04000400u) >> 7;
        const uint32_t qb = pk_min_u16(pk_sub_u16(wb & 0x7F807F80u, k7), 0x04000400u) >> 7;
        c4[h] = perm(qb, qa, 0x06040200u);               /* 4 code bytes, 8 = outside the window */
        if (h == 0) { r.sm0 = sm; r.ex0 = ex; } else { r.sm1 = sm; r.ex1 = ex; }
    }
    /* bit-matrix transpose with dot products: sum of bit * 2^j over the 8 code bytes */
    const uint32_t p0 = __builtin_amdgcn_udot4(c4[1] & 0x01010101u, 0x80402010u,
                        __builtin_amdgcn_udot4(c4[0] & 0x01010101u, 0x08040201u, 0u, false), false);
    const uint32_t p1 = __builtin_amdgcn_udot4(c4[1] & 0x02020202u, 0x80402010u,
                        __builtin_amdgcn_udot4(c4[0] & 0x02020202u, 0x08040201u, 0u, false), false);
    const uint32_t p2 = __builtin_amdgcn_udot4(c4[1] & 0x04040404u, 0x80402010u,
                        __builtin_amdgcn_udot4(c4[0] & 0x04040404u, 0x08040201u, 0u, false), false);
    r.b0 = p0;
    r.b1 = p1 >> 1;
    r.b2 = p2 >> 2;
    r.m = ~(r.b0 | r.b1 | r.b2) & 0xFFu;
    return r;
}

struct CompressShared {
    uint8_t planes[3][kTile / 8];          /* plane bytes of the tile, natural order */
    uint8_t esc[kGroupsPerTile][kGroup];   /* zero-point exponents, one region per group */
    uint32_t gcnt[kGroupsPerTile];         /* zero-points per group */
};

/* One group of one wave: load, encode, store SM/LO, stage planes and zero-points in LDS. */
template <int DT, bool FAST, bool STORE>
__device__ __forceinline__ void compress_group(const uint8_t* __restrict__ cin, uint8_t* __restrict__ slot,
                                               const SlotLayout& L, uint64_t n, uint64_t ts, uint32_t gi,
                                               uint32_t k7, uint32_t lane, CompressShared& sh)
{
    const uint64_t gbase = ts + (uint64_t)gi * kGroup;      /* wave-uniform */
    const uint64_t e = gbase + lane * kLaneElems;
    uint32_t hp[4], lp[4], vmask;
    load_lane<DT, FAST>(cin, gbase, lane, n, hp, lp, vmask);
    const LaneEnc r = encode8(hp, k7);
    const uint32_t m = r.m & vmask;
    if (STORE) {
        if (FAST || e < pad128(n)) st_stream<u32x2>((slot + L.sm + gbase) + lane * 8u, u32x2{r.sm0, r.sm1});
        if (DT == ZIPCCL_FP32) {
            if (FAST || 2 * e < pad128(2 * n))
                st_stream<u32x4>((slot + L.lo + 2 * gbase) + lane * 16u, u32x4{lp[0], lp[1], lp[2], lp[3]});
        }
        const uint32_t pi = gi * 64u + lane;
        sh.planes[0][pi] = (uint8_t)r.b0;
        sh.planes[1][pi] = (uint8_t)r.b1;
        sh.planes[2][pi] = (uint8_t)r.b2;
    }
    const uint32_t cnt = __popc(m);
    const uint32_t inc = wave_incl_scan(cnt);
    if (lane == 63) sh.gcnt[gi] = inc;
    if (STORE) {
        /* the lane's zero-point exponents, in element order, at its offset inside the group */
        uint8_t* dst = &sh.esc[gi][inc - cnt];
        uint32_t mm = m;
        while (mm) {
            const uint32_t j = __builtin_ctz(mm);
            mm &= mm - 1u;
            *dst++ = (uint8_t)perm(r.ex1, r.ex0, j | 0x0C0C0C00u);
        }
    }
}

/*
 * Chunk header, zeroed IDX / ESC padding and chunk_bytes, once the chunk's zero-point count is
 * known.  Called by NT cooperating threads numbered tid = 0..NT-1.
 */
template <int DT, uint32_t NT>
__device__ __forceinline__ void finish_chunk(uint8_t* __restrict__ slot, const SlotLayout& L, uint64_t n,
                                             uint64_t n_esc, uint32_t dec_lo, uint32_t dec_hi,
                                             uint64_t* chunk_bytes, uint32_t tid)
{
    const uint64_t ng = (n + kGroup - 1) / kGroup;
    const uint64_t cbytes = L.esc + pad128(n_esc);
    uint32_t* __restrict__ idx = reinterpret_cast<uint32_t*>(slot + L.idx);
    uint8_t* __restrict__ esc = slot + L.esc;
    for (uint32_t i = tid; i < 32u; i += NT) {
        uint32_t w = 0;
        switch (i) {
            case 0: w = kMagic; break;
            case 1: w = kVersion; break;
            case 2: w = (uint32_t)DT; break;
            case 3: w = kGroup; break;
            case 4: w = (uint32_t)n; break;
            case 5: w = (uint32_t)(n >> 32); break;
            case 6: w = n_esc; break;
            case 7: w = (uint32_t)(n_esc >> 32); break;
            case 8: w = (uint32_t)cbytes; break;
            case 9: w = (uint32_t)(cbytes >> 32); break;
            case 10: w = dec_lo; break;
            case 11: w = dec_hi; break;
            default: break;
        }
        reinterpret_cast<uint32_t*>(slot)[i] = w;
        const uint64_t ie = ng + i;                         /* zero the IDX padding */
        if (4 * ie < pad128(4 * ng)) idx[ie] = 0;
    }
    for (uint32_t i = tid; i < 128u; i += NT) {             /* zero the ESC padding */
        const uint64_t je = n_esc + i;
        if (je < pad128(n_esc)) esc[je] = 0;
    }
    if (tid == 0 && chunk_bytes) *chunk_bytes = cbytes;
}

template <int DT, int MODE>
__global__ __launch_bounds__(kThreads) void k_compress(const CompressArgs a)
{
    constexpr uint32_t ES = DT == ZIPCCL_BF16 ? 2u : 4u;
    constexpr bool STORE = MODE != kModeCount;
    __shared__ CompressShared sh;

    /* grid = (tiles of the largest chunk, chunks): no search, the chunk's geometry is three scalar loads */
    const uint32_t c = blockIdx.y;
    const uint32_t first = a.tab.tile_start[c];
    const uint32_t ntc = a.tab.tile_start[c + 1] - first;
    if (blockIdx.x >= ntc) return;
    const uint32_t t = first + blockIdx.x;
    const bool last_tile = blockIdx.x + 1u == ntc;
    const uint64_t n = a.tab.elem_off[c + 1] - a.tab.elem_off[c];
    const uint64_t ts = (uint64_t)blockIdx.x * kTile;
    const uint8_t* __restrict__ cin = a.in + a.tab.elem_off[c] * ES;
    uint8_t* __restrict__ slot = a.out + a.tab.slot_off[c];
    const SlotLayout L = slot_layout(n, DT);
    const bool fast = (ts + kTile <= n) && ((reinterpret_cast<uintptr_t>(cin) & 15u) == 0);
    const uint32_t lane = lane_id();
    const uint32_t wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);   /* keep wave-derived math scalar */
    /* the table is a kernel argument, or (estimated on the device) two words in device memory */
    const uint32_t dec_lo = a.d_table ? a.d_table[0] : a.dec_lo;
    const uint32_t dec_hi = a.d_table ? a.d_table[1] : a.dec_hi;
    const uint32_t e0 = a.d_table ? (dec_lo >> 8) & 0xFFu : a.e0;
    const uint32_t k7 = ((e0 - 1u) << 7) * 0x00010001u;

    if (fast) {
#pragma unroll
        for (uint32_t u = 0; u < kGroupsPerWave; ++u)
            compress_group<DT, true, STORE>(cin, slot, L, n, ts, u * kWavesPerBlock + wave, k7, lane, sh);
    } else {
#pragma unroll
        for (uint32_t u = 0; u < kGroupsPerWave; ++u)
            compress_group<DT, false, STORE>(cin, slot, L, n, ts, u * kWavesPerBlock + wave, k7, lane, sh);
    }
    __syncthreads();

    /* every wave: tile-level exclusive prefix of the 16 group counts (lanes 0..15 hold them) */
    const uint32_t gc = lane < kGroupsPerTile ? sh.gcnt[lane] : 0u;
    const uint32_t ginc = row_incl_scan(gc);
    const uint32_t gex = ginc - gc;
    const uint32_t tile_total = __builtin_amdgcn_readlane(ginc, kGroupsPerTile - 1);
    if (MODE == kModeCount) {
        if (threadIdx.x == 0) a.tile_total[t] = tile_total;
        return;
    }
    if (MODE == kModeStash && threadIdx.x == 0) a.tile_total[t] = tile_total;

    /* kModeEmit knows the zero-points of the chunk before this tile; kModeStash works tile-local */
    const uint32_t P = MODE == kModeEmit ? a.tile_prefix[t] : 0u;
    const uint64_t ng = (n + kGroup - 1) / kGroup;
    uint32_t* __restrict__ idx = reinterpret_cast<uint32_t*>(slot + L.idx);
    uint8_t* __restrict__ esc = MODE == kModeEmit ? slot + L.esc + P : a.stash + a.tab.elem_off[c] + ts;

    if (wave == 0) {
        /* group index (section 4.2.3); k_place adds the tile's prefix in stash mode */
        const uint64_t g = ts / kGroup + lane;
        if (lane < kGroupsPerTile && g < ng) idx[g] = P + gex;
    } else {
        /* waves 1..3: one plane each, 16 bytes per lane */
        const uint32_t k = wave - 1u;
        const uint64_t pb = ts / 8 + lane * 16u;
        if (fast || pb < L.plane_bytes)
            st_stream<u32x4>((slot + L.p0 + k * L.plane_bytes + ts / 8) + lane * 16u,
                             *reinterpret_cast<const u32x4*>(&sh.planes[k][lane * 16u]));
    }
    /* zero-point exponents: every wave copies the segments of its own groups, in element order */
#pragma unroll
    for (uint32_t u = 0; u < kGroupsPerWave; ++u) {
        const uint32_t gi = u * kWavesPerBlock + wave;
        const uint32_t cnt = __builtin_amdgcn_readlane(gc, gi);
        uint8_t* dst = esc + __builtin_amdgcn_readlane(gex, gi);
#pragma unroll 1
        for (uint32_t i = lane; i < cnt; i += 64u) dst[i] = sh.esc[gi][i];
    }

    if (MODE == kModeEmit && last_tile)
        finish_chunk<DT, kThreads>(slot, L, n, (uint64_t)P + tile_total, dec_lo, dec_hi,
                                   a.chunk_bytes ? a.chunk_bytes + c : nullptr, threadIdx.x);
}

/* Move nw aligned words: word i of dst = bytes [4i + sh8, 4i + sh8 + 4) of the aligned word array s32.
 * `width` lanes (this one is number `lane`) share the job, four words per lane and step, with all
 * loads of a step issued before its stores.  Reads reach at most 7 bytes past the last source byte. */
__device__ __forceinline__ void move_words(uint32_t* __restrict__ d32, const uint32_t* __restrict__ s32,
                                           uint32_t nw, uint32_t sh8, uint32_t lane, uint32_t width)
{
    for (uint32_t i0 = 0; i0 < nw; i0 += 4u * width) {
        uint32_t lo[4], hi[4];
#pragma unroll
        for (uint32_t k = 0; k < 4; ++k) {
            const uint32_t i = i0 + k * width + lane;
            lo[k] = hi[k] = 0;
            if (i < nw) { lo[k] = s32[i]; hi[k] = s32[i + 1]; }
        }
#pragma unroll
        for (uint32_t k = 0; k < 4; ++k) {
            const uint32_t i = i0 + k * width + lane;
            if (i < nw) d32[i] = __builtin_amdgcn_alignbyte(hi[k], lo[k], sh8);
        }
    }
}

/*
 * Stash mode, after k_tile_scan: 16 lanes per tile (16 tiles per workgroup, so that many tiles'
 * dependent loads are in flight per wave) move the tile's zero-point exponents from the stash
 * to ESC[P, P + count), add P to the tile's 16 index entries, and the last tile of a chunk
 * writes header, padding and chunk_bytes.  Tiles dense in zero-points (more than kPlaceBig
 * bytes) are moved by the whole workgroup afterwards.
 */
template <int DT>
__global__ __launch_bounds__(kThreads) void k_place(const CompressArgs a)
{
    constexpr uint32_t kSub = 16;                       /* lanes per tile */
    constexpr uint32_t kPlaceBig = 1024;                /* bytes a 16-lane group moves on its own */
    __shared__ uint32_t s_nbig;
    __shared__ uint32_t s_big[kThreads / kSub];
    __shared__ uint64_t s_src[kThreads / kSub], s_dst[kThreads / kSub];
    __shared__ uint32_t s_nw[kThreads / kSub], s_sh[kThreads / kSub];
    if (threadIdx.x == 0) s_nbig = 0;
    __syncthreads();

    /* grid = (16-tile groups of the largest chunk, chunks): the chunk's geometry is wave-uniform */
    const uint32_t c = blockIdx.y;
    const uint32_t first = a.tab.tile_start[c];
    const uint32_t ntc = a.tab.tile_start[c + 1] - first;
    const uint64_t n = a.tab.elem_off[c + 1] - a.tab.elem_off[c];
    uint8_t* __restrict__ slot = a.out + a.tab.slot_off[c];
    const SlotLayout L = slot_layout(n, DT);
    const uint32_t dec_lo = a.d_table ? a.d_table[0] : a.dec_lo;
    const uint32_t dec_hi = a.d_table ? a.d_table[1] : a.dec_hi;

    const uint32_t sub = threadIdx.x % kSub;
    const uint32_t tw = threadIdx.x / kSub;             /* tile inside the workgroup */
    const uint32_t ti = blockIdx.x * (kThreads / kSub) + tw;
    if (ti < ntc) {
        const uint32_t t = first + ti;
        const uint8_t* __restrict__ src = a.stash + a.tab.elem_off[c] + (uint64_t)ti * kTile;
        /* everything that does not depend on the counts is loaded together with them:
           the tile's 16 index entries and the first 64 bytes of its stash */
        const uint64_t ng = (n + kGroup - 1) / kGroup;
        uint32_t* __restrict__ idx = reinterpret_cast<uint32_t*>(slot + L.idx);
        const uint64_t g = (uint64_t)ti * kGroupsPerTile + sub;
        uint32_t idx_local = 0;
        if (g < ng) idx_local = idx[g];
        const uint32_t P = a.tile_prefix[t];
        const uint32_t cnt = a.tile_total[t];
        if (P != 0u && g < ng) idx[g] = idx_local + P;

        /* byte-exact move to an arbitrarily aligned destination: head bytes, aligned words, tail bytes */
        uint8_t* __restrict__ dst = slot + L.esc + P;
        const uint32_t head = min((uint32_t)(-(int64_t)reinterpret_cast<uintptr_t>(dst)) & 3u, cnt);
        const uint32_t nw = (cnt - head) >> 2;
        const uint32_t done = head + 4u * nw;
        const uint32_t sh8 = reinterpret_cast<uintptr_t>(src + head) & 3u;
        const uint32_t* __restrict__ s32 = reinterpret_cast<const uint32_t*>(
            reinterpret_cast<uintptr_t>(src + head) & ~(uintptr_t)3);
        uint32_t* __restrict__ d32 = reinterpret_cast<uint32_t*>(dst + head);
        uint8_t hb = 0, tb = 0;
        if (sub < head) hb = src[sub];
        if (sub < cnt - done) tb = src[done + sub];
        if (cnt <= kPlaceBig) {
            move_words(d32, s32, nw, sh8, sub, kSub);
        } else if (sub == 0) {
            const uint32_t k = atomicAdd(&s_nbig, 1u);
            s_big[k] = tw;
            s_src[tw] = reinterpret_cast<uint64_t>(s32);
            s_dst[tw] = reinterpret_cast<uint64_t>(d32);
            s_nw[tw] = nw;
            s_sh[tw] = sh8;
        }
        if (sub < head) dst[sub] = hb;
        if (sub < cnt - done) dst[done + sub] = tb;
        if (ti + 1u == ntc)
            finish_chunk<DT, kSub>(slot, L, n, (uint64_t)P + cnt, dec_lo, dec_hi,
                                   a.chunk_bytes ? a.chunk_bytes + c : nullptr, sub);
    }
    __syncthreads();
    const uint32_t nbig = s_nbig;
    for (uint32_t b = 0; b < nbig; ++b) {
        const uint32_t k = s_big[b];
        move_words(reinterpret_cast<uint32_t*>(s_dst[k]), reinterpret_cast<const uint32_t*>(s_src[k]), s_nw[k],
                   s_sh[k], threadIdx.x, kThreads);
    }
}

/*
 * Exclusive prefix of every chunk's per-tile zero-point counts.  Workgroup (x, y) owns segment x
 * (kScanSeg tiles) of chunk y: it sums the chunk's counts before its segment itself (the count
 * array is small and cache-resident, and this keeps workgroups independent of each other), then
 * scans its segment.
 */
constexpr uint32_t kScanSeg = 4 * kThreads;

__global__ __launch_bounds__(kThreads) void k_tile_scan(const CompressArgs a)
{
    __shared__ uint32_t s_wave[kWavesPerBlock];
    const uint32_t c = blockIdx.y;
    const uint32_t first = a.tab.tile_start[c], end = a.tab.tile_start[c + 1];
    const uint32_t seg0 = first + blockIdx.x * kScanSeg;
    if (seg0 >= end) return;
    const uint32_t lane = lane_id(), wave = threadIdx.x >> 6;

    /* counts of the chunk before this segment */
    uint32_t part[8] = {0, 0, 0, 0, 0, 0, 0, 0};
    uint32_t i = first + threadIdx.x;
    for (; i + 7u * kThreads < seg0; i += 8u * kThreads) {     /* eight independent loads in flight per thread */
#pragma unroll
        for (uint32_t k = 0; k < 8; ++k) part[k] += a.tile_total[i + k * kThreads];
    }
    for (; i < seg0; i += kThreads) part[0] += a.tile_total[i];
    uint32_t before = ((part[0] + part[1]) + (part[2] + part[3])) + ((part[4] + part[5]) + (part[6] + part[7]));
    before = wave_incl_scan(before);
    if (lane == 63) s_wave[wave] = before;
    __syncthreads();
    uint32_t base = 0;
#pragma unroll
    for (uint32_t w = 0; w < kWavesPerBlock; ++w) base += s_wave[w];
    __syncthreads();

    /* scan of the segment: four consecutive tiles per thread */
    const uint32_t i0 = seg0 + 4u * threadIdx.x;
    uint32_t v[4], mine = 0;
#pragma unroll
    for (uint32_t k = 0; k < 4; ++k) {
        v[k] = i0 + k < end ? a.tile_total[i0 + k] : 0u;
        mine += v[k];
    }
    const uint32_t inc = wave_incl_scan(mine);
    if (lane == 63) s_wave[wave] = inc;
    __syncthreads();
    uint32_t run = base + inc - mine;
    for (uint32_t w = 0; w < wave; ++w) run += s_wave[w];
#pragma unroll
    for (uint32_t k = 0; k < 4; ++k) {
        if (i0 + k < end) a.tile_prefix[i0 + k] = run;
        run += v[k];
    }
}

/*
 * Decoder tables in LDS, indexed by a 4-bit zero-point mask q of four values:
 * .x = v_perm selector putting the r-th byte of a compacted list at the position of the r-th
 * set bit of q (0x0c = constant 0 elsewhere), .y = 0xff in the bytes of set bits.
 */
__device__ __forceinline__ uint2 expand_entry(uint32_t q)
{
    uint32_t sel = 0, msk = 0, r = 0;
#pragma unroll
    for (uint32_t i = 0; i < 4; ++i) {
        if ((q >> i) & 1u) { sel |= r << (8 * i); msk |= 0xFFu << (8 * i); ++r; }
        else sel |= 0x0Cu << (8 * i);
    }
    return make_uint2(sel, msk);
}

/* bits 0..3 of x -> bit 0 of bytes 0..3 */
__device__ __forceinline__ uint32_t spread4(uint32_t x)
{
    return __umul24(x, 0x204081u) & 0x01010101u;
}

/* Decoder tables in LDS, built once per workgroup (one entry per thread). */
struct DecTables {
    uint2 spread[256];   /* plane byte -> its 8 bits in bit 0 of 8 bytes (.x = values 0..3, .y = values 4..7) */
    uint2 expand[16];    /* 4-bit zero-point mask -> v_perm selector and byte mask, see expand_entry */
};

__device__ __forceinline__ void build_tables(DecTables& t)
{
    t.spread[threadIdx.x] = make_uint2(spread4(threadIdx.x & 15u), spread4(threadIdx.x >> 4));   /* kThreads == 256 */
    if (threadIdx.x < 16) t.expand[threadIdx.x] = expand_entry(threadIdx.x);
}

/* Bytes of LDS per group for its zero-point exponents: 512 + up to 7 of misalignment, rounded up,
 * + 8 so that a lane's three aligned words never leave the region. */
constexpr uint32_t kEscRegion = 544;

/* What a lane reads for its 8 values of one group. */
struct DecIn {
    uint32_t sm0, sm1;       /* 8 sign+mantissa bytes */
    uint32_t b0, b1, b2;     /* plane bytes */
    uint32_t lo[4];          /* fp32: 8 low 16-bit words */
    uint32_t base;           /* IDX entry of the group = list position of its first zero-point */
    uint32_t count;          /* zero-points of the group according to IDX (next entry - this one) */
    uint32_t vmask;          /* bit j = value j exists */
    bool idx_ok;             /* base <= next <= n_esc and count <= 512 */
};

/* The lane's zero-point bytes (up to 8, in element order) and where its mask says they go. */
struct DecEsc {
    uint32_t m;              /* bit j = value j is a zero-point */
    uint32_t sh;             /* byte offset of the lane's first zero-point inside d0 */
    uint32_t d0, d1, d2;     /* three aligned words covering the lane's 8 list bytes */
    bool bad;                /* planes and IDX disagree about the group */
};

/* Phase 0: the group's slice of the zero-point list by IDX alone (scalar loads). */
__device__ __forceinline__ void decode_index(const uint8_t* __restrict__ slot, const SlotLayout& L, uint64_t n,
                                             uint32_t n_esc, uint64_t gstart, DecIn& r, uint32_t& next)
{
    const uint64_t g = gstart / kGroup, ng = (n + kGroup - 1) / kGroup;
    const uint32_t* __restrict__ idx = reinterpret_cast<const uint32_t*>(slot + L.idx);
    r.base = idx[g];
    next = g + 1 < ng ? idx[g + 1] : n_esc;
    r.idx_ok = r.base <= next && next <= n_esc && next - r.base <= kGroup;
    r.count = r.idx_ok ? next - r.base : 0u;
}

/* Phase 1a: fetch the slice [base, base + count), 8 aligned bytes per lane (+ 8 more by lane 0 when a
 * full group starts off alignment).  Aligned reads stay inside pad128(n_esc); lanes past the slice read
 * the 8 bytes in front of the list instead (the end of the static part), so the load needs no predicate. */
__device__ __forceinline__ void decode_fetch_list(const uint8_t* __restrict__ slot, const SlotLayout& L,
                                                  const DecIn& r, uint32_t next, uint32_t lane, u32x2& v, u32x2& tail)
{
    const uint32_t end = r.count != 0u ? next : 0u;              /* nothing to fetch for an empty slice */
    const uint32_t a8 = r.base & ~7u;
    const uint32_t a = a8 + 8u * lane;
    const uint8_t* __restrict__ esc = slot + L.esc;
    v = *reinterpret_cast<const u32x2*>(esc + (a < end ? (int64_t)a : (int64_t)-8));
    tail = u32x2{0u, 0u};
    if (a8 + kGroup < end) {                                      /* wave-uniform and rare */
        if (lane == 0) tail = *reinterpret_cast<const u32x2*>(esc + a8 + kGroup);
    }
}

/* Phase 1b: the lane's SM bytes, plane bytes and (fp32) low words. */
template <int DT, bool FAST>
__device__ __forceinline__ void decode_load(const uint8_t* __restrict__ slot, const SlotLayout& L, uint64_t n,
                                            uint64_t gstart, uint32_t lane, DecIn& r)
{
    /* gstart is wave-uniform: uniform 64-bit base + 32-bit lane offset */
    const uint64_t e = gstart + lane * kLaneElems;
    r.sm0 = r.sm1 = r.b0 = r.b1 = r.b2 = 0;
    r.lo[0] = r.lo[1] = r.lo[2] = r.lo[3] = 0;
    if (FAST || e < pad128(n)) {
        const u32x2 v = ld_stream<u32x2>((slot + L.sm + gstart) + lane * 8u);
        r.sm0 = v.x; r.sm1 = v.y;
    }
    const uint64_t pb = e >> 3;
    if (FAST || pb < L.plane_bytes) {
        const uint8_t* pl = slot + L.p0 + (gstart >> 3);
        r.b0 = ld_stream<uint8_t>(pl + lane);
        r.b1 = ld_stream<uint8_t>((pl + L.plane_bytes) + lane);
        r.b2 = ld_stream<uint8_t>((pl + 2 * L.plane_bytes) + lane);
    }
    if (DT == ZIPCCL_FP32) {
        if (FAST || 2 * e < pad128(2 * n)) {
            const u32x4 v = ld_stream<u32x4>((slot + L.lo + 2 * gstart) + lane * 16u);
            r.lo[0] = v.x; r.lo[1] = v.y; r.lo[2] = v.z; r.lo[3] = v.w;
        }
    }
    r.vmask = 0xFFu;
    if (!FAST) r.vmask = e >= n ? 0u : (n - e >= 8 ? 0xFFu : ((1u << (uint32_t)(n - e)) - 1u));
}

/* Phase 1c: park the slice in the wave's LDS region so that lanes can pick their bytes by position. */
__device__ __forceinline__ void decode_park_list(uint8_t* lds, uint32_t lane, const u32x2& v, const u32x2& tail)
{
    *reinterpret_cast<u32x2*>(lds + 8u * lane) = v;
    if (lane == 0) *reinterpret_cast<u32x2*>(lds + kGroup) = tail;
}

/* Phase 2: wave scan of the per-lane zero-point counts, then the lane's bytes from the LDS region.
 * Straight-line code (no branch on whether the group has zero-points) so that the four groups a
 * wave works on can be interleaved by the scheduler. */
__device__ __forceinline__ DecEsc decode_locate(const DecIn& in, const uint8_t* lds)
{
    DecEsc r;
    r.m = ~(in.b0 | in.b1 | in.b2) & in.vmask;     /* code 0 = zero-point; tail bits are not */
    const uint32_t cnt = __popc(r.m);
    const uint32_t inc = wave_incl_scan(cnt);
    const uint32_t gtot = __builtin_amdgcn_readlane(inc, 63);
    r.bad = !in.idx_ok || gtot != in.count;        /* planes and IDX must agree */
    /* the lane's zero-point exponents are the bytes [p, p + cnt) of the region, p <= 7 + 512 - cnt
       (clamped, so that a corrupt stream still reads inside the region) */
    const uint32_t p = min((in.base & 7u) + (inc - cnt), kGroup + 7u);
    const uint32_t* w = reinterpret_cast<const uint32_t*>(lds + (p & ~3u));
    r.d0 = w[0]; r.d1 = w[1]; r.d2 = w[2];
    r.sh = p & 3u;
    return r;
}

/* Rebuild the high 16-bit words of the lane's 8 values (section 4, third paragraph), packed in pairs. */
__device__ __forceinline__ void decode_values(const DecIn& in, const DecEsc& es, uint32_t e0,
                                              const DecTables& tab, uint32_t hp[4])
{
    /* code bytes of values 0..3 and 4..7 (plane bits spread by table), then exponent = dec[1] - 1 + code */
    const uint32_t k4 = (e0 - 1u) * 0x01010101u;
    const uint2 t0 = tab.spread[in.b0], t1 = tab.spread[in.b1], t2 = tab.spread[in.b2];
    uint32_t eA = (t0.x | (t1.x << 1) | (t2.x << 2)) + k4;
    uint32_t eB = (t0.y | (t1.y << 1) | (t2.y << 2)) + k4;
    const uint2* __restrict__ lut = tab.expand;
    {   /* zero-point exponents dropped in place; a lane without zero-points selects nothing */
        const uint32_t l8 = __builtin_amdgcn_alignbyte(es.d1, es.d0, es.sh);
        const uint32_t h8 = __builtin_amdgcn_alignbyte(es.d2, es.d1, es.sh);
        const uint32_t mA = es.m & 15u, mB = es.m >> 4;
        const uint32_t nA = __popc(mA);
        const uint2 tA = lut[mA], tB = lut[mB];
        const uint32_t xB = nA == 4u ? h8 : __builtin_amdgcn_alignbyte(h8, l8, nA);
        eA = bfi(tA.y, perm(0u, l8, tA.x), eA);
        eB = bfi(tB.y, perm(0u, xB, tB.x), eB);
    }
    /* recombine with sign and mantissa: low byte = mantissa | E bit 0 << 7, high = sign | E >> 1 */
    const uint32_t lA = bfi(0x7F7F7F7Fu, in.sm0, eA << 7), hA = bfi(0x80808080u, in.sm0, eA >> 1);
    const uint32_t lB = bfi(0x7F7F7F7Fu, in.sm1, eB << 7), hB = bfi(0x80808080u, in.sm1, eB >> 1);
    hp[0] = perm(hA, lA, 0x05010400u);
    hp[1] = perm(hA, lA, 0x07030602u);
    hp[2] = perm(hB, lB, 0x05010400u);
    hp[3] = perm(hB, lB, 0x07030602u);
}

/* Rebuild the 8 values and store them. */
template <int DT, bool FAST>
__device__ __forceinline__ void decode_store(uint8_t* __restrict__ cout, const DecIn& in, const DecEsc& es,
                                             uint64_t gstart, uint32_t e0, uint32_t lane, const DecTables& tab)
{
    const uint64_t e = gstart + lane * kLaneElems;
    uint32_t hp[4];
    decode_values(in, es, e0, tab, hp);
    if (FAST) {
        if (DT == ZIPCCL_BF16) {
            st_stream<u32x4>((cout + gstart * 2) + lane * 16u, u32x4{hp[0], hp[1], hp[2], hp[3]});
        } else {
            uint32_t x[8];
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                x[2 * k] = perm(hp[k], in.lo[k], 0x05040100u);
                x[2 * k + 1] = perm(hp[k], in.lo[k], 0x07060302u);
            }
            st_stream<u32x4>((cout + gstart * 4) + lane * 32u, u32x4{x[0], x[1], x[2], x[3]});
            st_stream<u32x4>((cout + gstart * 4 + 16) + lane * 32u, u32x4{x[4], x[5], x[6], x[7]});
        }
    } else {
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            if ((in.vmask >> j) & 1u) {
                const uint32_t h = (hp[j >> 1] >> (16 * (j & 1))) & 0xFFFFu;
                if (DT == ZIPCCL_BF16) {
                    *reinterpret_cast<uint16_t*>(cout + (e + j) * 2) = (uint16_t)h;
                } else {
                    const uint32_t l = (in.lo[j >> 1] >> (16 * (j & 1))) & 0xFFFFu;
                    *reinterpret_cast<uint32_t*>(cout + (e + j) * 4) = (h << 16) | l;
                }
            }
        }
    }
}

/*
 * Chunk header check (all wave-uniform): the static part is readable (the host checked it), magic,
 * version, dtype, G and n must match the call, the table must be a window, and the zero-point
 * list the header promises must fit into the readable bytes.
 */
template <int DT>
__device__ __forceinline__ bool check_header(const uint8_t* __restrict__ slot, const SlotLayout& L, uint64_t n,
                                             uint64_t slot_off, uint64_t comp_capacity, uint32_t& e0, uint32_t& n_esc)
{
    const uint32_t* hw = reinterpret_cast<const uint32_t*>(slot);
    const uint64_t n_hdr = (uint64_t)hw[4] | ((uint64_t)hw[5] << 32);
    const uint64_t ne = (uint64_t)hw[6] | ((uint64_t)hw[7] << 32);
    const uint64_t cbytes = (uint64_t)hw[8] | ((uint64_t)hw[9] << 32);
    const uint32_t dec_lo = hw[10], dec_hi = hw[11];
    e0 = (dec_lo >> 8) & 0xFFu;
    n_esc = (uint32_t)ne;
    bool ok = hw[0] == kMagic && hw[1] == kVersion && hw[2] == (uint32_t)DT && hw[3] == kGroup;
    ok = ok && n_hdr == n && ne <= n && cbytes == L.esc + pad128(ne);
    ok = ok && slot_off + cbytes <= comp_capacity;
    ok = ok && e0 >= 1u && e0 <= 249u && (dec_lo >> 8) == (e0 | ((e0 + 1u) << 8) | ((e0 + 2u) << 16)) &&
         dec_hi == ((e0 + 3u) | ((e0 + 4u) << 8) | ((e0 + 5u) << 16) | ((e0 + 6u) << 24));
    return ok;
}

template <int DT>
__global__ __launch_bounds__(kThreads, DT == ZIPCCL_BF16 ? 8 : 6)   /* waves per SIMD: <= 64 VGPRs for bf16, <= 80 for fp32 */
void k_decompress(const DecompressArgs a)
{
    constexpr uint32_t ES = DT == ZIPCCL_BF16 ? 2u : 4u;
    __shared__ DecTables s_tab;
    __shared__ __attribute__((aligned(16))) uint8_t s_esc[kWavesPerBlock][kGroupsPerWave][kEscRegion];
    build_tables(s_tab);

    /* grid = (tiles of the largest chunk, chunks) */
    const uint32_t c = blockIdx.y;
    if (blockIdx.x >= a.tab.tile_start[c + 1] - a.tab.tile_start[c]) return;
    const uint64_t n = a.tab.elem_off[c + 1] - a.tab.elem_off[c];
    const uint64_t ts = (uint64_t)blockIdx.x * kTile;
    const uint8_t* __restrict__ slot = a.comp + a.tab.slot_off[c];
    uint8_t* __restrict__ cout = a.out + a.tab.elem_off[c] * ES;
    const SlotLayout L = slot_layout(n, DT);

    uint32_t e0, n_esc;
    const bool ok = check_header<DT>(slot, L, n, a.tab.slot_off[c], a.comp_capacity, e0, n_esc);
    __syncthreads();
    if (!ok) {
        if (threadIdx.x == 0 && a.status) atomicOr(a.status, (uint32_t)ZIPCCL_ERR_CORRUPT);
        return;
    }

    const bool fast = (ts + kTile <= n) && ((reinterpret_cast<uintptr_t>(cout) & 15u) == 0);
    const uint32_t lane = lane_id();
    const uint32_t wave = threadIdx.x >> 6;   /* left in a vector register: measured faster here than scalar addressing */
    bool bad = false;
    if (fast) {
        /* phases over the wave's four groups, so that each phase's loads are all in flight together
           and no vector load depends on another vector load */
        DecIn in[kGroupsPerWave];
        DecEsc es[kGroupsPerWave];
        uint32_t next[kGroupsPerWave];
        u32x2 lv[kGroupsPerWave], lt[kGroupsPerWave];
#pragma unroll
        for (uint32_t u = 0; u < kGroupsPerWave; ++u)
            decode_index(slot, L, n, n_esc, ts + (uint64_t)(u * kWavesPerBlock + wave) * kGroup, in[u], next[u]);
#pragma unroll
        for (uint32_t u = 0; u < kGroupsPerWave; ++u) decode_fetch_list(slot, L, in[u], next[u], lane, lv[u], lt[u]);
#pragma unroll
        for (uint32_t u = 0; u < kGroupsPerWave; ++u)
            decode_load<DT, true>(slot, L, n, ts + (uint64_t)(u * kWavesPerBlock + wave) * kGroup, lane, in[u]);
#pragma unroll
        for (uint32_t u = 0; u < kGroupsPerWave; ++u) decode_park_list(s_esc[wave][u], lane, lv[u], lt[u]);
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
#pragma unroll
        for (uint32_t u = 0; u < kGroupsPerWave; ++u) es[u] = decode_locate(in[u], s_esc[wave][u]);
#pragma unroll
        for (uint32_t u = 0; u < kGroupsPerWave; ++u) {
            decode_store<DT, true>(cout, in[u], es[u], ts + (uint64_t)(u * kWavesPerBlock + wave) * kGroup, e0, lane, s_tab);
            bad |= es[u].bad;
        }
    } else {
        for (uint32_t u = 0; u < kGroupsPerWave; ++u) {
            const uint64_t gstart = ts + (uint64_t)(u * kWavesPerBlock + wave) * kGroup;
            if (gstart < n) {
                DecIn in;
                uint32_t next;
                u32x2 lv, lt;
                decode_index(slot, L, n, n_esc, gstart, in, next);
                decode_fetch_list(slot, L, in, next, lane, lv, lt);
                decode_load<DT, false>(slot, L, n, gstart, lane, in);
                decode_park_list(s_esc[wave][u], lane, lv, lt);
                __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
                __builtin_amdgcn_wave_barrier();
                __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
                const DecEsc es = decode_locate(in, s_esc[wave][u]);
                decode_store<DT, false>(cout, in, es, gstart, e0, lane, s_tab);
                bad |= es.bad;
            }
        }
    }
    if (bad && a.status) atomicOr(a.status, (uint32_t)ZIPCCL_ERR_CORRUPT);
}

/* fp32 bits -> bf16 bits, round to nearest even; NaN keeps sign and top payload bits and is made quiet */
__device__ __forceinline__ uint32_t f32_to_bf16_bits(float f)
{
    const uint32_t u = __float_as_uint(f);
    const bool nan = (u & 0x7F800000u) == 0x7F800000u && (u & 0x007FFFFFu) != 0u;
    return nan ? ((u >> 16) | 0x0040u) : ((u + 0x7FFFu + ((u >> 16) & 1u)) >> 16);
}

/*
 * Local reduction of the zipped Reduce-Scatter (paper sections 3.3 and 5.2): decode the slices
 * received from n_peers peers (slots back to back, n values each) and sum them in FP32, peers in
 * slot order starting from peer 0's value.  One pass: every compressed byte is read once and
 * only the sum is written.  Work decomposition as in k_decompress; the peer loop is innermost.
 */
/* GPW = groups per wave: 4 for large shards, 1 for small ones (four times as many workgroups, each with a
 * quarter of the sequential peer loop). */
template <int DT, int ODT, uint32_t GPW>
__global__ __launch_bounds__(kThreads) void k_decompress_reduce(const ReduceArgs a)
{
    constexpr uint32_t kRTile = kGroup * kWavesPerBlock * GPW;
    constexpr uint32_t OES = ODT == ZIPCCL_BF16 ? 2u : 4u;
    __shared__ DecTables s_tab;
    __shared__ __attribute__((aligned(16))) uint8_t s_esc[kWavesPerBlock][kEscRegion];
    __shared__ uint32_t s_e0[kMaxPeers];      /* dec[1] of peer p's slot, 0 = header rejected */
    __shared__ uint32_t s_nesc[kMaxPeers];    /* zero-points of peer p's slot */
    build_tables(s_tab);

    const uint64_t n = a.n;
    const uint64_t ts = (uint64_t)blockIdx.x * kRTile;
    const SlotLayout L = slot_layout(n, DT);
    bool bad = false;
    /* every slot's header is checked once per workgroup, one peer per thread */
    for (uint32_t p = threadIdx.x; p < a.n_peers; p += kThreads) {
        const uint64_t slot_off = (uint64_t)p * a.slot_cap;
        uint32_t e0, n_esc;
        const bool ok = check_header<DT>(a.comp + slot_off, L, n, slot_off, a.comp_capacity, e0, n_esc);
        s_e0[p] = ok ? e0 : 0u;
        s_nesc[p] = n_esc;
        bad |= !ok;
    }
    __syncthreads();

    const bool fast = (ts + kRTile <= n) && ((reinterpret_cast<uintptr_t>(a.out) & 15u) == 0);
    const uint32_t lane = lane_id();
    const uint32_t wave = threadIdx.x >> 6;
    const uint64_t ng = (n + kGroup - 1) / kGroup;
    for (uint32_t u = 0; u < GPW; ++u) {
        const uint64_t gstart = ts + (uint64_t)(u * kWavesPerBlock + wave) * kGroup;
        if (gstart >= n) continue;
        const uint64_t g = gstart / kGroup;
        float acc[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) acc[j] = 0.0f;
        bool have = false;
        const uint64_t e = gstart + lane * kLaneElems;
        const uint32_t vmask = fast ? 0xFFu : (e >= n ? 0u : (n - e >= 8 ? 0xFFu : ((1u << (uint32_t)(n - e)) - 1u)));
        /* the IDX entries of the next peer are fetched one iteration ahead (scalar loads) */
        const uint32_t* idx0 = reinterpret_cast<const uint32_t*>(a.comp + L.idx);
        uint32_t nb = idx0[g], nn = g + 1 < ng ? idx0[g + 1] : 0u;
        for (uint32_t p = 0; p < a.n_peers; ++p) {
            const uint8_t* __restrict__ slot = a.comp + (uint64_t)p * a.slot_cap;
            const uint32_t e0 = s_e0[p], n_esc = s_nesc[p];
            const uint32_t base = nb, next = g + 1 < ng ? nn : n_esc;
            if (p + 1 < a.n_peers) {
                const uint32_t* idxn = reinterpret_cast<const uint32_t*>(slot + a.slot_cap + L.idx);
                nb = idxn[g];
                if (g + 1 < ng) nn = idxn[g + 1];
            }
            if (e0 == 0u) continue;                      /* rejected slot: left out of the sum */
            DecIn in;
            u32x2 lv, lt;
            in.base = base;
            in.idx_ok = base <= next && next <= n_esc && next - base <= kGroup;
            in.count = in.idx_ok ? next - base : 0u;
            decode_fetch_list(slot, L, in, next, lane, lv, lt);
            if (fast) decode_load<DT, true>(slot, L, n, gstart, lane, in);
            else decode_load<DT, false>(slot, L, n, gstart, lane, in);
            decode_park_list(s_esc[wave], lane, lv, lt);
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
            const DecEsc es = decode_locate(in, s_esc[wave]);
            __builtin_amdgcn_wave_barrier();
            bad |= es.bad;
            uint32_t hp[4];
            decode_values(in, es, e0, s_tab, hp);
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                uint32_t w0, w1;
                if (DT == ZIPCCL_BF16) { w0 = hp[k] << 16; w1 = hp[k] & 0xFFFF0000u; }
                else { w0 = perm(hp[k], in.lo[k], 0x05040100u); w1 = perm(hp[k], in.lo[k], 0x07060302u); }
                const float x0 = __uint_as_float(w0), x1 = __uint_as_float(w1);
                acc[2 * k] = have ? acc[2 * k] + x0 : x0;
                acc[2 * k + 1] = have ? acc[2 * k + 1] + x1 : x1;
            }
            have = true;
        }
        uint8_t* __restrict__ og = a.out + gstart * OES;
        if (fast) {
            if (ODT == ZIPCCL_FP32) {
                st_stream<u32x4>(og + lane * 32u, u32x4{__float_as_uint(acc[0]), __float_as_uint(acc[1]),
                                                        __float_as_uint(acc[2]), __float_as_uint(acc[3])});
                st_stream<u32x4>((og + 16) + lane * 32u, u32x4{__float_as_uint(acc[4]), __float_as_uint(acc[5]),
                                                               __float_as_uint(acc[6]), __float_as_uint(acc[7])});
            } else {
                uint32_t o[4];
#pragma unroll
                for (int k = 0; k < 4; ++k) o[k] = f32_to_bf16_bits(acc[2 * k]) | (f32_to_bf16_bits(acc[2 * k + 1]) << 16);
                st_stream<u32x4>(og + lane * 16u, u32x4{o[0], o[1], o[2], o[3]});
            }
        } else {
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                if ((vmask >> j) & 1u) {
                    const uint64_t i = lane * kLaneElems + j;
                    if (ODT == ZIPCCL_FP32) *reinterpret_cast<float*>(og + i * 4) = acc[j];
                    else *reinterpret_cast<uint16_t*>(og + i * 2) = (uint16_t)f32_to_bf16_bits(acc[j]);
                }
            }
        }
    }
    if (bad && a.status) atomicOr(a.status, (uint32_t)ZIPCCL_ERR_CORRUPT);
}

/*
 * sigma of a tensor as the paper takes it (section 4.1: torch.std = unbiased sample standard
 * deviation), in FP64: every workgroup writes its partial sum x and sum x^2; k_estimate_finish adds the
 * partials in a fixed order, forms sigma, and picks the window with Eq.5 / Eq.2 (erf in FP64),
 * exactly as the host builder does.  A sigma that is not positive and finite selects the lowest window.
 */
template <int DT>
__global__ __launch_bounds__(kThreads) void k_moments(const MomentArgs a)
{
    constexpr uint32_t ES = DT == ZIPCCL_BF16 ? 2u : 4u;
    constexpr uint32_t PER16 = 16u / ES;               /* values per 16-byte load */
    __shared__ double s_sum[kWavesPerBlock], s_sq[kWavesPerBlock];
    double sum = 0.0, sq = 0.0;
    const bool aligned = (reinterpret_cast<uintptr_t>(a.in) & 15u) == 0;
    const uint64_t n16 = aligned ? a.n / PER16 : 0;    /* 16-byte pieces handled with vector loads */
    for (uint64_t i = (uint64_t)blockIdx.x * kThreads + threadIdx.x; i < n16; i += (uint64_t)gridDim.x * kThreads) {
        const u32x4 v = ld_stream<u32x4>(a.in + i * 16);
        const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            if (DT == ZIPCCL_BF16) {
                const double x0 = (double)__uint_as_float(w[k] << 16), x1 = (double)__uint_as_float(w[k] & 0xFFFF0000u);
                sum += x0; sq += x0 * x0;
                sum += x1; sq += x1 * x1;
            } else {
                const double x = (double)__uint_as_float(w[k]);
                sum += x; sq += x * x;
            }
        }
    }
    /* the tail (and everything, for a misaligned tensor) element by element */
    for (uint64_t i = n16 * PER16 + (uint64_t)blockIdx.x * kThreads + threadIdx.x; i < a.n; i += (uint64_t)gridDim.x * kThreads) {
        uint32_t bits;
        if (DT == ZIPCCL_BF16) bits = (uint32_t)(*reinterpret_cast<const uint16_t*>(a.in + i * 2)) << 16;
        else bits = *reinterpret_cast<const uint32_t*>(a.in + i * 4);
        const double x = (double)__uint_as_float(bits);
        sum += x; sq += x * x;
    }
    /* fixed-order reduction: lanes by butterfly, waves in order */
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) {
        sum += __shfl_xor(sum, d, 64);
        sq += __shfl_xor(sq, d, 64);
    }
    const uint32_t wave = threadIdx.x >> 6;
    if ((threadIdx.x & 63u) == 0) { s_sum[wave] = sum; s_sq[wave] = sq; }
    __syncthreads();
    if (threadIdx.x == 0) {
        double ts = 0.0, tq = 0.0;
        for (uint32_t w = 0; w < kWavesPerBlock; ++w) { ts += s_sum[w]; tq += s_sq[w]; }
        a.partial[2 * blockIdx.x] = ts;
        a.partial[2 * blockIdx.x + 1] = tq;
    }
}

__global__ __launch_bounds__(kThreads) void k_estimate_finish(const MomentArgs a)
{
    __shared__ double s_sum[kThreads], s_sq[kThreads];
    double sum = 0.0, sq = 0.0;
    for (uint32_t i = threadIdx.x; i < a.n_blocks; i += kThreads) { sum += a.partial[2 * i]; sq += a.partial[2 * i + 1]; }
    s_sum[threadIdx.x] = sum;
    s_sq[threadIdx.x] = sq;
    __syncthreads();
    for (uint32_t d = kThreads / 2; d >= 1; d >>= 1) {
        if (threadIdx.x < d) { s_sum[threadIdx.x] += s_sum[threadIdx.x + d]; s_sq[threadIdx.x] += s_sq[threadIdx.x + d]; }
        __syncthreads();
    }
    if (threadIdx.x != 0) return;
    const double N = (double)a.n;
    double sigma = __longlong_as_double(0x7FF8000000000000ll);          /* NaN for fewer than two values */
    if (a.n >= 2) {
        const double mean = s_sum[0] / N;
        const double var = (s_sq[0] - N * mean * mean) / (N - 1.0);
        sigma = sqrt(var > 0.0 ? var : (var == var ? 0.0 : var));
    }
    uint32_t e0 = 1;
    if (sigma > 0.0 && sigma < __longlong_as_double(0x7FF0000000000000ll)) {
        const double x_opt = log2(sigma) + 0.5 * log2(14.0 * log(2.0) / 16383.0);     /* Eq.5 */
        const int lo = (int)floor(x_opt), hi = (int)ceil(x_opt);
        const double s2 = sigma * sqrt(2.0);
        const double p_lo = erf(ldexp(1.0, lo + 7) / s2) - erf(ldexp(1.0, lo) / s2);    /* Eq.2 */
        const double p_hi = erf(ldexp(1.0, hi + 7) / s2) - erf(ldexp(1.0, hi) / s2);
        int e = (p_hi > p_lo ? hi : lo) + 127;
        e = e < 1 ? 1 : (e > 248 ? 248 : e);
        e0 = (uint32_t)e;
    }
    a.table[0] = 0;
    for (uint32_t k = 1; k <= 7; ++k) a.table[k] = (uint8_t)(e0 + k - 1);
    if (a.sigma) *a.sigma = sigma;
}

/* Yardstick: plain copy, 16 bytes per lane, one load and one store per thread. */
__global__ __launch_bounds__(kThreads) void k_copy(const u32x4* __restrict__ src, u32x4* __restrict__ dst, uint64_t n16)
{
    const uint64_t i = (uint64_t)blockIdx.x * kThreads + threadIdx.x;
    if (i < n16) dst[i] = src[i];
}

} // namespace

int launch_decompress_reduce(int dt, int out_dt, const ReduceArgs& a, void* stream)
{
    hipStream_t s = (hipStream_t)stream;
    const dim3 block(kThreads);
    /* at least ~8 workgroups per CU before a workgroup takes four groups per wave */
    const bool big = a.n >= (uint64_t)kTile * 2048u;
    const uint64_t per = big ? kTile : kTile / kGroupsPerWave;
    const dim3 grid((uint32_t)(a.n == 0 ? 1 : (a.n + per - 1) / per));
#define ZIPCCL_REDUCE(DT, ODT)                                                                          \
    do {                                                                                                \
        if (big) hipLaunchKernelGGL((k_decompress_reduce<DT, ODT, kGroupsPerWave>), grid, block, 0, s, a); \
        else hipLaunchKernelGGL((k_decompress_reduce<DT, ODT, 1u>), grid, block, 0, s, a);              \
    } while (0)
    if (dt == ZIPCCL_BF16 && out_dt == ZIPCCL_FP32) ZIPCCL_REDUCE(ZIPCCL_BF16, ZIPCCL_FP32);
    else if (dt == ZIPCCL_BF16) ZIPCCL_REDUCE(ZIPCCL_BF16, ZIPCCL_BF16);
    else if (out_dt == ZIPCCL_FP32) ZIPCCL_REDUCE(ZIPCCL_FP32, ZIPCCL_FP32);
    else ZIPCCL_REDUCE(ZIPCCL_FP32, ZIPCCL_BF16);
#undef ZIPCCL_REDUCE
    return (int)hipGetLastError();
}

int launch_estimate(int dt, const MomentArgs& a, void* stream)
{
    hipStream_t s = (hipStream_t)stream;
    if (dt == ZIPCCL_BF16) hipLaunchKernelGGL((k_moments<ZIPCCL_BF16>), dim3(a.n_blocks), dim3(kThreads), 0, s, a);
    else hipLaunchKernelGGL((k_moments<ZIPCCL_FP32>), dim3(a.n_blocks), dim3(kThreads), 0, s, a);
    if (hipGetLastError() != hipSuccess) return 1;
    hipLaunchKernelGGL(k_estimate_finish, dim3(1), dim3(kThreads), 0, s, a);
    return (int)hipGetLastError();
}

int launch_copy(void* d_dst, const void* d_src, uint64_t bytes, void* stream)
{
    const uint64_t n16 = bytes / 16;
    if (n16 == 0) return (int)hipSuccess;
    const uint64_t blocks = (n16 + kThreads - 1) / kThreads;
    hipLaunchKernelGGL(k_copy, dim3((uint32_t)blocks), dim3(kThreads), 0, (hipStream_t)stream,
                       static_cast<const u32x4*>(d_src), static_cast<u32x4*>(d_dst), n16);
    return (int)hipGetLastError();
}

/* tiles of the largest chunk of the launch */
static uint32_t max_chunk_tiles(const ChunkTab& tab)
{
    uint32_t m = 1;
    for (uint32_t c = 0; c < tab.n_chunks; ++c) {
        const uint32_t nt = tab.tile_start[c + 1] - tab.tile_start[c];
        m = nt > m ? nt : m;
    }
    return m;
}

int launch_compress(int dt, int mode, const CompressArgs& a, void* stream)
{
    const dim3 grid(max_chunk_tiles(a.tab), a.tab.n_chunks), block(kThreads);
    hipStream_t s = (hipStream_t)stream;
#define ZIPCCL_LAUNCH(DT, MODE) hipLaunchKernelGGL((k_compress<DT, MODE>), grid, block, 0, s, a)
    if (dt == ZIPCCL_BF16) {
        if (mode == kModeCount) ZIPCCL_LAUNCH(ZIPCCL_BF16, kModeCount);
        else if (mode == kModeEmit) ZIPCCL_LAUNCH(ZIPCCL_BF16, kModeEmit);
        else ZIPCCL_LAUNCH(ZIPCCL_BF16, kModeStash);
    } else {
        if (mode == kModeCount) ZIPCCL_LAUNCH(ZIPCCL_FP32, kModeCount);
        else if (mode == kModeEmit) ZIPCCL_LAUNCH(ZIPCCL_FP32, kModeEmit);
        else ZIPCCL_LAUNCH(ZIPCCL_FP32, kModeStash);
    }
#undef ZIPCCL_LAUNCH
    return (int)hipGetLastError();
}

int launch_tile_scan(const CompressArgs& a, void* stream)
{
    const dim3 grid((max_chunk_tiles(a.tab) + kScanSeg - 1) / kScanSeg, a.tab.n_chunks);
    hipLaunchKernelGGL(k_tile_scan, grid, dim3(kThreads), 0, (hipStream_t)stream, a);
    return (int)hipGetLastError();
}

int launch_place(int dt, const CompressArgs& a, void* stream)
{
    const dim3 grid((max_chunk_tiles(a.tab) + 15) / 16, a.tab.n_chunks), block(kThreads);   /* 16 tiles per workgroup */
    if (dt == ZIPCCL_BF16)
        hipLaunchKernelGGL((k_place<ZIPCCL_BF16>), grid, block, 0, (hipStream_t)stream, a);
    else
        hipLaunchKernelGGL((k_place<ZIPCCL_FP32>), grid, block, 0, (hipStream_t)stream, a);
    return (int)hipGetLastError();
}

int launch_decompress(int dt, const DecompressArgs& a, void* stream)
{
    const dim3 grid(max_chunk_tiles(a.tab), a.tab.n_chunks), block(kThreads);
    if (dt == ZIPCCL_BF16)
        hipLaunchKernelGGL((k_decompress<ZIPCCL_BF16>), grid, block, 0, (hipStream_t)stream, a);
    else
        hipLaunchKernelGGL((k_decompress<ZIPCCL_FP32>), grid, block, 0, (hipStream_t)stream, a);
    return (int)hipGetLastError();
}

} // namespace zipccl
