/*
 * Compress side of libzipccl.so for gfx950 (CDNA4, wave64): k_compress, k_tile_scan, k_place.
 *
 * compress   : paper section 4 (split, 3-bit code, zero-points) with the kernel steps of
 *              section 4.2 re-designed for wave64: one wave handles a group of 512 values,
 *              8 values per lane (consecutive: one 16-byte load for bf16; whole fp32 groups: two
 *              quads, one from each half of the group, one 16-byte load each), a workgroup of
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
 *              the per-tile counts become per-chunk prefixes inside k_place (chunks of up to
 *              kPlaceScanTiles tiles) or in k_tile_scan; k_place moves each tile's exponents
 *              to their final place and finishes index and header.
 *              (Waiting in-kernel for the predecessors' counts costs a tile ~10 us of lateness
 *              of the slowest of them, measured; the stash costs ~5 % extra traffic.)
 * Everything here is integer work.
 */
#include <mutex>

#include "zipccl_device.h"

namespace zipccl {
namespace {

/*
 * Workspace of zipccl_compress_static: device memory that belongs to the library, one copy per GPU, held until
 * the process ends.  Host code never uses this name as an address: static_scratch() asks the runtime for the
 * array's device address, once per device, and hands that out.
 */
static __device__ __align__(256) uint8_t scratch[ZIPCCL_STATIC_SCRATCH_BYTES];

/*
 * Load the lane's 8 consecutive values starting at chunk-relative element e.
 * hp[k] packs the high 16-bit words of values 2k (low half) and 2k+1 (high half);
 * lp[k] the low words (fp32 only).  vmask bit j = value j exists (e + j < n).
 * Values that do not exist read as 0.
 */
/* FAST, bf16: `skew` says that the chunk starts at an odd element of the tensor, i.e. its bytes are 2 but
 * not 4-byte aligned; the lane's 16 bytes then come as halfword + three dwords + halfword. */
template <int DT, bool FAST>
__device__ __forceinline__ void load_lane(const uint8_t* __restrict__ cin, uint64_t gbase, uint32_t lane, uint64_t n,
                                          uint32_t hp[4], uint32_t lp[4], uint32_t& vmask, bool skew = false)
{
    /* gbase (first value of the group) is wave-uniform: uniform 64-bit base + 32-bit lane offset */
    const uint64_t e = gbase + lane * kLaneElems;
    if (FAST) {
        vmask = 0xFFu;
        if (DT == ZIPCCL_BF16) {
            const uint8_t* __restrict__ p = (cin + gbase * 2) + lane * 16u;
            if (!skew) {
                const u32x4 v = ld_stream_a4(p);
                hp[0] = v.x; hp[1] = v.y; hp[2] = v.z; hp[3] = v.w;
            } else {
                const uint32_t h0 = ld_stream<uint16_t>(p);
                const u32x3 d = __builtin_nontemporal_load(reinterpret_cast<const u32x3_a4*>(p + 2));
                const uint32_t h7 = ld_stream<uint16_t>(p + 14);
                hp[0] = h0 | (d.x << 16);
                hp[1] = __builtin_amdgcn_alignbyte(d.y, d.x, 2u);
                hp[2] = __builtin_amdgcn_alignbyte(d.z, d.y, 2u);
                hp[3] = (d.z >> 16) | (h7 << 16);
            }
            lp[0] = lp[1] = lp[2] = lp[3] = 0;
        } else {
            /* fp32, whole groups: the lane's 8 values are two quads, [4 lane, 4 lane + 4) of the group's first
               half and of its second half, so that each load is 16 contiguous bytes per lane (32 contiguous
               bytes per lane cost ~7 % of the bandwidth, measured).  Values 0..3 = first quad, 4..7 = second. */
            const u32x4 a = ld_stream_a4((cin + gbase * 4) + lane * 16u);
            const u32x4 b = ld_stream_a4((cin + gbase * 4 + 2 * kGroup) + lane * 16u);
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

/* One group of one wave, its values already loaded (load_lane): encode, store SM/LO, stage planes and
 * zero-points in LDS. */
template <int DT, bool FAST, bool STORE>
__device__ __forceinline__ void compress_group(uint8_t* __restrict__ slot, const SlotLayout& L, uint64_t n,
                                               uint64_t ts, uint32_t gi, uint32_t k7, uint32_t lane,
                                               CompressShared& sh, const uint32_t hp[4], const uint32_t lp[4],
                                               uint32_t vmask)
{
    const uint64_t gbase = ts + (uint64_t)gi * kGroup;      /* wave-uniform */
    const uint64_t e = gbase + lane * kLaneElems;
    const LaneEnc r = encode8(hp, k7);
    const uint32_t m = r.m & vmask;
    if (DT == ZIPCCL_FP32 && FAST) {
        /* two quads per lane (see load_lane): bits 0..3 of the plane bytes and of m belong to values
           [4 lane, 4 lane + 4) of the group, bits 4..7 to the same values of its second half */
        if (STORE) {
            uint8_t* __restrict__ sm = slot + L.sm + gbase;
            st_stream<uint32_t>(sm + lane * 4u, r.sm0);
            st_stream<uint32_t>((sm + kGroup / 2) + lane * 4u, r.sm1);
            uint8_t* __restrict__ lo = slot + L.lo + 2 * gbase;
            st_stream<u32x2>(lo + lane * 8u, u32x2{lp[0], lp[1]});
            st_stream<u32x2>((lo + kGroup) + lane * 8u, u32x2{lp[2], lp[3]});
            /* a plane byte = the nibbles of two neighbouring lanes: even lanes assemble the byte of the
               first half, odd lanes that of the second (three planes at once, one byte each) */
            const uint32_t p3 = r.b0 | (r.b1 << 8) | (r.b2 << 16);
            const uint32_t q3 = __builtin_amdgcn_update_dpp(0u, p3, 0xB1, 0xF, 0xF, false);   /* quad_perm [1,0,3,2] */
            const uint32_t b3 = (lane & 1u) ? (((q3 >> 4) & 0x0F0F0Fu) | (p3 & 0xF0F0F0u))
                                            : ((p3 & 0x0F0F0Fu) | ((q3 & 0x0F0F0Fu) << 4));
            const uint32_t pi = gi * 64u + (lane >> 1) + 32u * (lane & 1u);
            sh.planes[0][pi] = (uint8_t)b3;
            sh.planes[1][pi] = (uint8_t)(b3 >> 8);
            sh.planes[2][pi] = (uint8_t)(b3 >> 16);
        }
        /* element order = all first quads by lane, then all second quads: one scan of both counts */
        const uint32_t mA = m & 15u, mB = m >> 4;
        const uint32_t cA = __popc(mA), cB = __popc(mB);
        const uint32_t inc = wave_incl_scan(cA | (cB << 16));
        const uint32_t totA = __builtin_amdgcn_readlane(inc, 63) & 0xFFFFu;
        if (lane == 63) sh.gcnt[gi] = (inc & 0xFFFFu) + (inc >> 16);
        if (STORE) {
            uint8_t* dst = &sh.esc[gi][(inc & 0xFFFFu) - cA];
            uint32_t mm = mA;
            while (mm) {
                const uint32_t j = __builtin_ctz(mm);
                mm &= mm - 1u;
                *dst++ = (uint8_t)perm(r.ex1, r.ex0, j | 0x0C0C0C00u);
            }
            dst = &sh.esc[gi][totA + (inc >> 16) - cB];
            mm = mB << 4;
            while (mm) {
                const uint32_t j = __builtin_ctz(mm);
                mm &= mm - 1u;
                *dst++ = (uint8_t)perm(r.ex1, r.ex0, j | 0x0C0C0C00u);
            }
        }
        return;
    }
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
    /* whole tiles take the vector path; a chunk of the tensor starts at some element of it, so its bytes are
       dword-aligned or (bf16, odd element) skewed by one halfword */
    const bool fast = ts + kTile <= n;
    const bool skew = (reinterpret_cast<uintptr_t>(cin) & 2u) != 0;
    const uint32_t lane = lane_id();
    const uint32_t wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);   /* keep wave-derived math scalar */
    /* the table is a kernel argument, or (estimated on the device) two words in device memory */
    const uint32_t* __restrict__ tab_c = a.d_table + c * a.table_stride;      /* one table for all chunks, or one each */
    const uint32_t dec_lo = a.d_table ? tab_c[0] : a.dec_lo;
    const uint32_t dec_hi = a.d_table ? tab_c[1] : a.dec_hi;
    const uint32_t e0 = a.d_table ? (dec_lo >> 8) & 0xFFu : a.e0;
    const uint32_t k7 = ((e0 - 1u) << 7) * 0x00010001u;

    if (fast) {
        /* all four groups' loads go out before the first is encoded: four times the bytes in flight per
           wave, and no wait for a load ever includes the stores of the group before */
        uint32_t hp[kGroupsPerWave][4], lp[kGroupsPerWave][4], vm[kGroupsPerWave];
#pragma unroll
        for (uint32_t u = 0; u < kGroupsPerWave; ++u)
            load_lane<DT, true>(cin, ts + (uint64_t)(u * kWavesPerBlock + wave) * kGroup, lane, n, hp[u], lp[u], vm[u], skew);
#pragma unroll
        for (uint32_t u = 0; u < kGroupsPerWave; ++u)
            compress_group<DT, true, STORE>(slot, L, n, ts, u * kWavesPerBlock + wave, k7, lane, sh, hp[u], lp[u], vm[u]);
    } else {
#pragma unroll
        for (uint32_t u = 0; u < kGroupsPerWave; ++u) {
            const uint32_t gi = u * kWavesPerBlock + wave;
            uint32_t hp[4], lp[4], vm;
            load_lane<DT, false>(cin, ts + (uint64_t)gi * kGroup, lane, n, hp, lp, vm);
            compress_group<DT, false, STORE>(slot, L, n, ts, gi, k7, lane, sh, hp, lp, vm);
        }
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
 * `width` lanes (this one is number `lane`) share the job, W words per lane and step, with all
 * loads of a step issued before its stores.  Reads reach at most 7 bytes past the last source byte. */
template <uint32_t W>
__device__ __forceinline__ void move_words(uint32_t* __restrict__ d32, const uint32_t* __restrict__ s32,
                                           uint32_t nw, uint32_t sh8, uint32_t lane, uint32_t width)
{
    for (uint32_t i0 = 0; i0 < nw; i0 += W * width) {
        uint32_t lo[W], hi[W];
#pragma unroll
        for (uint32_t k = 0; k < W; ++k) {
            const uint32_t i = i0 + k * width + lane;
            lo[k] = hi[k] = 0;
            if (i < nw) { lo[k] = s32[i]; hi[k] = s32[i + 1]; }
        }
#pragma unroll
        for (uint32_t k = 0; k < W; ++k) {
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
/* SCAN: there was no k_tile_scan; the workgroup sums the chunk's tile counts before its own tiles itself
 * (chunks of at most kPlaceScanTiles tiles: the counts are few and cache-resident). */
template <int DT, bool SCAN>
__global__ __launch_bounds__(kThreads) void k_place(const CompressArgs a)
{
    constexpr uint32_t kSub = 16;                       /* lanes per tile */
    constexpr uint32_t kPlaceBig = 1024;                /* bytes a 16-lane group moves on its own */
    __shared__ uint32_t s_wave[kWavesPerBlock];
    __shared__ uint32_t s_ex[kThreads / kSub];
    __shared__ uint32_t s_nbig;
    __shared__ uint32_t s_big[kThreads / kSub];
    __shared__ uint64_t s_src[kThreads / kSub], s_dst[kThreads / kSub];
    __shared__ uint32_t s_nw[kThreads / kSub], s_sh[kThreads / kSub];
    if (threadIdx.x == 0) s_nbig = 0;

    /* grid = (16-tile groups of the largest chunk, chunks): the chunk's geometry is wave-uniform */
    const uint32_t c = blockIdx.y;
    const uint32_t first = a.tab.tile_start[c];
    const uint32_t ntc = a.tab.tile_start[c + 1] - first;
    if (blockIdx.x * (kThreads / kSub) >= ntc) return;  /* a shorter chunk than the largest of the launch */
    if (SCAN) {
        /* counts of the chunk's tiles before this workgroup's, and the exclusive prefix inside it */
        const uint32_t t0 = blockIdx.x * (kThreads / kSub);
        uint32_t part[4] = {0, 0, 0, 0};
        uint32_t i = threadIdx.x;
        for (; i + 3u * kThreads < t0; i += 4u * kThreads) {
#pragma unroll
            for (uint32_t k = 0; k < 4; ++k) part[k] += a.tile_total[first + i + k * kThreads];
        }
        for (; i < t0; i += kThreads) part[0] += a.tile_total[first + i];
        const uint32_t inc = wave_incl_scan((part[0] + part[1]) + (part[2] + part[3]));
        if ((threadIdx.x & 63u) == 63u) s_wave[threadIdx.x >> 6] = inc;
        if (threadIdx.x < kThreads / kSub) {            /* one row of 16 lanes */
            const uint32_t mine = t0 + threadIdx.x < ntc ? a.tile_total[first + t0 + threadIdx.x] : 0u;
            s_ex[threadIdx.x] = row_incl_scan(mine) - mine;
        }
    }
    __syncthreads();
    const uint64_t n = a.tab.elem_off[c + 1] - a.tab.elem_off[c];
    uint8_t* __restrict__ slot = a.out + a.tab.slot_off[c];
    const SlotLayout L = slot_layout(n, DT);
    const uint32_t* __restrict__ tab_c = a.d_table + c * a.table_stride;
    const uint32_t dec_lo = a.d_table ? tab_c[0] : a.dec_lo;
    const uint32_t dec_hi = a.d_table ? tab_c[1] : a.dec_hi;

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
        uint32_t P;
        if (SCAN) P = ((s_wave[0] + s_wave[1]) + (s_wave[2] + s_wave[3])) + s_ex[tw];
        else P = a.tile_prefix[t];
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
            move_words<4>(d32, s32, nw, sh8, sub, kSub);
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
        /* 8 words per lane: a whole tile (at most 2048 words) in one step */
        move_words<8>(reinterpret_cast<uint32_t*>(s_dst[k]), reinterpret_cast<const uint32_t*>(s_src[k]), s_nw[k],
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

} // namespace

int static_scratch(void** ptr, size_t* bytes)
{
    constexpr int kMaxDevices = 64;
    static std::mutex mu;
    static void* addr[kMaxDevices];            /* device address of `scratch` on each GPU, once resolved */
    int dev = -1;
    const hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return (int)e;
    if (dev < 0 || dev >= kMaxDevices) return (int)hipErrorInvalidDevice;
    std::lock_guard<std::mutex> lock(mu);
    if (!addr[dev]) {
        void* p = nullptr;
        const hipError_t es = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));   /* for the current device */
        if (es != hipSuccess) return (int)es;
        if (!p) return (int)hipErrorInvalidSymbol;
        addr[dev] = p;
    }
    *ptr = addr[dev];
    *bytes = sizeof scratch;
    return 0;
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

int launch_place(int dt, bool scan, const CompressArgs& a, void* stream)
{
    const dim3 grid((max_chunk_tiles(a.tab) + 15) / 16, a.tab.n_chunks), block(kThreads);   /* 16 tiles per workgroup */
    hipStream_t s = (hipStream_t)stream;
    if (dt == ZIPCCL_BF16) {
        if (scan) hipLaunchKernelGGL((k_place<ZIPCCL_BF16, true>), grid, block, 0, s, a);
        else hipLaunchKernelGGL((k_place<ZIPCCL_BF16, false>), grid, block, 0, s, a);
    } else {
        if (scan) hipLaunchKernelGGL((k_place<ZIPCCL_FP32, true>), grid, block, 0, s, a);
        else hipLaunchKernelGGL((k_place<ZIPCCL_FP32, false>), grid, block, 0, s, a);
    }
    return (int)hipGetLastError();
}

} // namespace zipccl
