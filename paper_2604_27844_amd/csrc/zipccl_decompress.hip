/*
 * Decompress side of libzipccl.so for gfx950 (CDNA4, wave64): k_decompress (paper section 4, third
 * paragraph) and k_decompress_reduce (decode + local FP32 reduction of the zipped Reduce-Scatter,
 * sections 3.3 and 5.2).  No workgroup depends on another.  Work decomposition as on the compress side:
 * a wave owns a group of 512 values at a time, 8 values per lane (consecutive ones; for whole fp32 groups
 * two quads, one from each half of the group, so that every tensor access is 16 contiguous bytes per
 * lane); decoding is SWAR on packed bytes (table-driven bit spread, v_perm_b32 / v_bfi_b32
 * recombination) with a DPP wave scan to locate each lane's zero-point exponents.
 */
#include "zipccl_device.h"

namespace zipccl {
namespace {

/*
 * Entry of the 4-bit stage of the expand table, for a zero-point mask q of four values:
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

/*
 * Decoder tables in LDS, built once per workgroup (one entry of each per thread):
 * spread[k][b]  = the 8 bits of plane byte b at bit k of 8 bytes (.x = values 0..3, .y = values 4..7),
 *                 so that the three planes of a lane combine with one OR;
 * expand[m]     = for the lane's 8-bit zero-point mask m: v_perm selectors (.x for values 0..3, .y for
 *                 values 4..7) that put the r-th byte of the lane's 8-byte list window at the position
 *                 of the r-th set bit of m, and the byte masks of the set bits (.z, .w).
 */
struct DecTables {
    uint2 spread[3][256];
    u32x4 expand[256];
    uint2 expand4[16];   /* building block of expand[] */
};

/* Contains a workgroup barrier; the caller's next barrier makes the tables visible. */
__device__ __forceinline__ void build_tables(DecTables& t)
{
    const uint32_t b = threadIdx.x;                                   /* kThreads == 256 */
    if (b < 16) t.expand4[b] = expand_entry(b);
    const uint32_t lo = spread4(b & 15u), hi = spread4(b >> 4);
    t.spread[0][b] = make_uint2(lo, hi);
    t.spread[1][b] = make_uint2(lo << 1, hi << 1);
    t.spread[2][b] = make_uint2(lo << 2, hi << 2);
    __syncthreads();
    /* values 4..7 continue in the window where values 0..3 stopped */
    const uint2 a = t.expand4[b & 15u], c = t.expand4[b >> 4];
    const uint32_t skip = __popc(b & 15u) * 0x01010101u;
    t.expand[b] = u32x4{a.x, c.x + (skip & c.y), a.y, c.y};
}

/* Bytes of LDS per group for its zero-point exponents: 512 + up to 15 of misalignment, rounded up to
 * whole 16-byte words (33 of them) + 16 so that a lane's three aligned words never leave the region. */
constexpr uint32_t kEscRegion = 544;
constexpr uint32_t kListLanes = 33;     /* lanes that fetch 16 bytes of the list each */

/* What a lane reads for its 8 values of one group. */
struct DecIn {
    uint32_t sm0, sm1;       /* 8 sign+mantissa bytes */
    uint32_t b0, b1, b2;     /* plane bytes */
    uint32_t lo[4];          /* fp32: 8 low 16-bit words */
    uint32_t base;           /* IDX entry of the group = list position of its first zero-point */
    uint32_t count;          /* zero-points of the group according to IDX (next entry - this one) */
    uint32_t vmask;          /* bit j = value j exists */
    uint32_t idx_bad;        /* nonzero unless base <= next <= n_esc and next - base <= 512 */
};

/* The lane's zero-point bytes (up to 8, in element order) and where its mask says they go. */
struct DecEsc {
    uint32_t m;              /* bit j = value j is a zero-point */
    uint32_t l8, h8;         /* the 8 list bytes from the lane's first zero-point on */
    uint32_t wA, wB;         /* two-quad lanes (fp32): the list bytes of the first and of the second quad */
    uint32_t bad;            /* nonzero: planes and IDX disagree about the group */
};

/* r.base and next bound the group's slice of the zero-point list: check them, set r.count.
 * (next - base wraps to a large number when next < base) */
__device__ __forceinline__ void check_index(DecIn& r, uint32_t next, uint32_t n_esc)
{
    const uint32_t d = next - r.base;
    r.idx_bad = (uint32_t)(d > kGroup) | (uint32_t)(next > n_esc);
    r.count = r.idx_bad ? 0u : d;
}

/* Phase 0: the group's slice of the zero-point list by IDX alone (scalar loads). */
__device__ __forceinline__ void decode_index(const uint8_t* __restrict__ slot, const SlotLayout& L, uint64_t n,
                                             uint32_t n_esc, uint64_t gstart, DecIn& r, uint32_t& next)
{
    const uint64_t g = gstart / kGroup, ng = (n + kGroup - 1) / kGroup;
    const uint32_t* __restrict__ idx = reinterpret_cast<const uint32_t*>(slot + L.idx);
    r.base = idx[g];
    next = g + 1 < ng ? idx[g + 1] : n_esc;
    check_index(r, next, n_esc);
}

/* Phase 1a: fetch the slice [base, base + count): 16 aligned bytes per lane by the first 33 lanes, which
 * covers 512 bytes at any alignment.  Aligned reads stay inside pad128(n_esc); lanes past the slice read
 * the 16 bytes in front of the list instead (the end of the static part), so the load needs no predicate
 * and every group issues the same number of loads. */
__device__ __forceinline__ void decode_fetch_list(const uint8_t* __restrict__ slot, const SlotLayout& L,
                                                  const DecIn& r, uint32_t next, uint32_t lane, u32x4& v)
{
    const uint32_t end = r.count != 0u ? next : 0u;              /* nothing to fetch for an empty slice */
    const uint32_t a = (r.base & ~15u) + 16u * lane;
    const uint8_t* __restrict__ esc = slot + L.esc;
    v = *reinterpret_cast<const u32x4*>(esc + (a < end ? (int64_t)a : (int64_t)-16));
}

/* Phase 1b: the lane's SM bytes, plane bytes and (fp32) low words. */
/* WORDS: b0..b2 receive the aligned 32-bit word holding the lane's plane byte (see plane_bytes_of_words)
 * instead of the byte itself. */
template <int DT, bool FAST, bool WORDS = false, bool QUAD = false>
__device__ __forceinline__ void decode_load(const uint8_t* __restrict__ slot, const SlotLayout& L, uint64_t n,
                                            uint64_t gstart, uint32_t lane, DecIn& r)
{
    if (QUAD) {
        /* fp32, whole groups: the lane's 8 values are two quads, [4 lane, 4 lane + 4) of the group's first
           and of its second half, so that its 32 output bytes are two contiguous 16-byte stores per wave row.
           The lane fetches one plane byte per plane, the one it shares with its neighbour: even lanes that
           of the first half, odd lanes that of the second (quad_plane_bytes sorts the nibbles out). */
        const uint8_t* __restrict__ sm = slot + L.sm + gstart;
        r.sm0 = ld_stream<uint32_t>(sm + lane * 4u);
        r.sm1 = ld_stream<uint32_t>((sm + kGroup / 2) + lane * 4u);
        const uint8_t* pl = slot + L.p0 + (gstart >> 3);
        const uint32_t pi = (lane >> 1) + 32u * (lane & 1u);
        r.b0 = ld_stream<uint8_t>(pl + pi);
        r.b1 = ld_stream<uint8_t>((pl + L.plane_bytes) + pi);
        r.b2 = ld_stream<uint8_t>((pl + 2 * L.plane_bytes) + pi);
        const uint8_t* __restrict__ lo = slot + L.lo + 2 * gstart;
        const u32x2 la = ld_stream<u32x2>(lo + lane * 8u);
        const u32x2 lb = ld_stream<u32x2>((lo + kGroup) + lane * 8u);
        r.lo[0] = la.x; r.lo[1] = la.y; r.lo[2] = lb.x; r.lo[3] = lb.y;
        r.vmask = 0xFFu;
        return;
    }
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
        const uint8_t* pl = slot + L.p0 + (gstart >> 3);     /* 64-byte aligned: a group's 64 plane bytes */
        if (WORDS) {
            r.b0 = ld_stream<uint32_t>(pl + (lane & ~3u));
            r.b1 = ld_stream<uint32_t>((pl + L.plane_bytes) + (lane & ~3u));
            r.b2 = ld_stream<uint32_t>((pl + 2 * L.plane_bytes) + (lane & ~3u));
        } else {
            r.b0 = ld_stream<uint8_t>(pl + lane);
            r.b1 = ld_stream<uint8_t>((pl + L.plane_bytes) + lane);
            r.b2 = ld_stream<uint8_t>((pl + 2 * L.plane_bytes) + lane);
        }
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

/* After decode_load<.., WORDS = true>: the lane's plane bytes out of the words that hold them. */
__device__ __forceinline__ void plane_bytes_of_words(DecIn& r, uint32_t lane)
{
    const uint32_t sh = 8u * (lane & 3u);
    r.b0 = __builtin_amdgcn_ubfe(r.b0, sh, 8u);
    r.b1 = __builtin_amdgcn_ubfe(r.b1, sh, 8u);
    r.b2 = __builtin_amdgcn_ubfe(r.b2, sh, 8u);
}

/* After decode_load<.., QUAD = true>: from the plane bytes shared by a pair of lanes to each lane's own
 * byte (bits 0..3 = its first quad, bits 4..7 = its second), the three planes at once. */
__device__ __forceinline__ void quad_plane_bytes(DecIn& r, uint32_t lane)
{
    const uint32_t p3 = (r.b0 & 0xFFu) | ((r.b1 & 0xFFu) << 8) | ((r.b2 & 0xFFu) << 16);
    const uint32_t q3 = __builtin_amdgcn_update_dpp(0u, p3, 0xB1, 0xF, 0xF, false);   /* quad_perm [1,0,3,2] */
    const uint32_t b3 = (lane & 1u) ? (((q3 >> 4) & 0x0F0F0Fu) | (p3 & 0xF0F0F0u))
                                    : ((p3 & 0x0F0F0Fu) | ((q3 & 0x0F0F0Fu) << 4));
    r.b0 = b3 & 0xFFu;
    r.b1 = (b3 >> 8) & 0xFFu;
    r.b2 = b3 >> 16;
}

/* Phase 1c: park the slice in the wave's LDS region so that lanes can pick their bytes by position. */
__device__ __forceinline__ void decode_park_list(uint8_t* lds, uint32_t lane, const u32x4& v)
{
    if (lane < kListLanes) *reinterpret_cast<u32x4*>(lds + 16u * lane) = v;
}

/* Phase 2: wave scan of the per-lane zero-point counts, then the lane's bytes from the LDS region.
 * Straight-line code (no branch on whether the group has zero-points) so that the four groups a
 * wave works on can be interleaved by the scheduler. */
__device__ __forceinline__ DecEsc decode_locate(const DecIn& in, const uint8_t* lds)
{
    DecEsc r;
    r.m = ((in.b0 | in.b1 | in.b2) ^ 0xFFu) & in.vmask;     /* code 0 = zero-point; tail bits are not */
    const uint32_t cnt = __popc(r.m);
    const uint32_t inc = wave_incl_scan(cnt);
    const uint32_t gtot = __builtin_amdgcn_readlane(inc, 63);
    r.bad = in.idx_bad | (gtot ^ in.count);   /* planes and IDX must agree */
    /* the lane's zero-point exponents are the bytes [p, p + cnt) of the region, p <= 15 + 512 - cnt
       (clamped, so that a corrupt stream still reads inside the region) */
    const uint32_t p = min((in.base & 15u) + (inc - cnt), kGroup + 15u);
    /* three aligned words and two byte alignments: a single 8-byte read at the byte address p is accepted by the
       hardware but made the fused reduce, whose LDS pipe is two thirds busy, 35 % slower (measured) */
    const uint32_t* w = reinterpret_cast<const uint32_t*>(lds + (p & ~3u));
    r.l8 = __builtin_amdgcn_alignbyte(w[1], w[0], p & 3u);
    r.h8 = __builtin_amdgcn_alignbyte(w[2], w[1], p & 3u);
    return r;
}

/* Phase 2 for two-quad lanes: element order is all first quads by lane, then all second quads, so the
 * lane's zero-points sit in two places of the slice; one scan carries both counts. */
__device__ __forceinline__ DecEsc decode_locate_quad(const DecIn& in, const uint8_t* lds)
{
    DecEsc r;
    r.m = (in.b0 | in.b1 | in.b2) ^ 0xFFu;
    const uint32_t cA = __popc(r.m & 15u), cB = __popc(r.m >> 4);
    const uint32_t inc = wave_incl_scan(cA | (cB << 16));
    const uint32_t tot = __builtin_amdgcn_readlane(inc, 63);
    const uint32_t totA = tot & 0xFFFFu;
    r.bad = in.idx_bad | ((totA + (tot >> 16)) ^ in.count);
    const uint32_t pA = min((in.base & 15u) + (inc & 0xFFFFu) - cA, kGroup + 15u);
    const uint32_t pB = min((in.base & 15u) + totA + (inc >> 16) - cB, kGroup + 15u);
    const uint32_t* wa = reinterpret_cast<const uint32_t*>(lds + (pA & ~3u));
    const uint32_t* wb = reinterpret_cast<const uint32_t*>(lds + (pB & ~3u));
    r.wA = __builtin_amdgcn_alignbyte(wa[1], wa[0], pA & 3u);
    r.wB = __builtin_amdgcn_alignbyte(wb[1], wb[0], pB & 3u);
    r.l8 = r.h8 = 0;
    return r;
}

/* Rebuild the bytes of the high 16-bit words of the lane's 8 values (section 4, third paragraph):
 * lA / hA = low / high bytes of values 0..3, lB / hB of values 4..7. */
template <bool QUAD = false>
__device__ __forceinline__ void decode_bytes(const DecIn& in, const DecEsc& es, uint32_t e0, const DecTables& tab,
                                             uint32_t& lA, uint32_t& hA, uint32_t& lB, uint32_t& hB)
{
    /* code bytes of values 0..3 and 4..7 (plane bits spread by table), then exponent = dec[1] - 1 + code */
    const uint32_t k4 = (e0 - 1u) * 0x01010101u;
    const uint2 t0 = tab.spread[0][in.b0], t1 = tab.spread[1][in.b1], t2 = tab.spread[2][in.b2];
    uint32_t eA = (t0.x | t1.x | t2.x) + k4;
    uint32_t eB = (t0.y | t1.y | t2.y) + k4;
    if (QUAD) {   /* each quad's zero-point exponents from its own window */
        const uint2 xa = tab.expand4[es.m & 15u], xb = tab.expand4[es.m >> 4];
        eA = bfi(xa.y, perm(0u, es.wA, xa.x), eA);
        eB = bfi(xb.y, perm(0u, es.wB, xb.x), eB);
    } else {   /* zero-point exponents dropped in place: the lane's list bytes are the 8-byte window l8:h8 */
        const u32x4 x = tab.expand[es.m];
        eA = bfi(x.z, perm(es.h8, es.l8, x.x), eA);
        eB = bfi(x.w, perm(es.h8, es.l8, x.y), eB);
    }
    /* recombine with sign and mantissa: low byte = mantissa | E bit 0 << 7, high = sign | E >> 1 */
    lA = bfi(0x7F7F7F7Fu, in.sm0, eA << 7); hA = bfi(0x80808080u, in.sm0, eA >> 1);
    lB = bfi(0x7F7F7F7Fu, in.sm1, eB << 7); hB = bfi(0x80808080u, in.sm1, eB >> 1);
}

/* The same as four words holding the 8 high 16-bit words in element order. */
template <bool QUAD = false>
__device__ __forceinline__ void decode_values(const DecIn& in, const DecEsc& es, uint32_t e0,
                                              const DecTables& tab, uint32_t hp[4])
{
    uint32_t lA, hA, lB, hB;
    decode_bytes<QUAD>(in, es, e0, tab, lA, hA, lB, hB);
    hp[0] = perm(hA, lA, 0x05010400u);
    hp[1] = perm(hA, lA, 0x07030602u);
    hp[2] = perm(hB, lB, 0x05010400u);
    hp[3] = perm(hB, lB, 0x07030602u);
}

/* Rebuild the 8 values and store them. */
template <int DT, bool FAST>
__device__ __forceinline__ void decode_store(uint8_t* __restrict__ cout, const DecIn& in, const DecEsc& es,
                                             uint64_t gstart, uint32_t e0, uint32_t lane, const DecTables& tab,
                                             bool skew = false)
{
    const uint64_t e = gstart + lane * kLaneElems;
    uint32_t hp[4];
    decode_values<DT == ZIPCCL_FP32 && FAST>(in, es, e0, tab, hp);
    if (FAST) {
        if (DT == ZIPCCL_BF16) {
            uint8_t* __restrict__ p = (cout + gstart * 2) + lane * 16u;
            if (!skew) {
                st_stream_a4(p, u32x4{hp[0], hp[1], hp[2], hp[3]});
            } else {
                /* the chunk starts at an odd element of the tensor (bytes 2 but not 4-byte aligned):
                   halfword + three dwords + halfword */
                st_stream<uint16_t>(p, (uint16_t)hp[0]);
                __builtin_nontemporal_store(u32x3{__builtin_amdgcn_alignbyte(hp[1], hp[0], 2u),
                                                  __builtin_amdgcn_alignbyte(hp[2], hp[1], 2u),
                                                  __builtin_amdgcn_alignbyte(hp[3], hp[2], 2u)},
                                            reinterpret_cast<u32x3_a4*>(p + 2));
                st_stream<uint16_t>(p + 14, (uint16_t)(hp[3] >> 16));
            }
        } else {
            /* two quads per lane (decode_load<.., QUAD>): values 0..3 belong to the group's first half,
               4..7 to its second; each store is 16 contiguous bytes per lane */
            uint32_t x[8];
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                x[2 * k] = perm(hp[k], in.lo[k], 0x05040100u);
                x[2 * k + 1] = perm(hp[k], in.lo[k], 0x07060302u);
            }
            st_stream_a4((cout + gstart * 4) + lane * 16u, u32x4{x[0], x[1], x[2], x[3]});
            st_stream_a4((cout + gstart * 4 + 2 * kGroup) + lane * 16u, u32x4{x[4], x[5], x[6], x[7]});
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
 * version, dtype, G and n must match the call, the table must be a window (dec[0] = 0, dec[1..7]
 * consecutive), and the zero-point list the header promises must fit into the readable bytes.  The
 * reserved bytes 48..127 are not looked at.
 */
struct HeaderWords { uint32_t h[12]; };

/* All twelve words are fetched before any is looked at (one round of scalar loads, no chain of
 * dependent ones); a kernel can request them early and look at them later. */
__device__ __forceinline__ HeaderWords load_header(const uint8_t* __restrict__ slot)
{
    const uint32_t* hw = reinterpret_cast<const uint32_t*>(slot);
    HeaderWords r;
#pragma unroll
    for (int i = 0; i < 12; ++i) r.h[i] = hw[i];
    return r;
}

template <int DT>
__device__ __forceinline__ bool check_header(const HeaderWords& hdr, const SlotLayout& L, uint64_t n,
                                             uint64_t slot_off, uint64_t comp_capacity, uint32_t& e0, uint32_t& n_esc)
{
    const uint32_t* h = hdr.h;
    const uint64_t n_hdr = (uint64_t)h[4] | ((uint64_t)h[5] << 32);
    const uint64_t ne = (uint64_t)h[6] | ((uint64_t)h[7] << 32);
    const uint64_t cbytes = (uint64_t)h[8] | ((uint64_t)h[9] << 32);
    const uint32_t dec_lo = h[10], dec_hi = h[11];
    e0 = (dec_lo >> 8) & 0xFFu;
    n_esc = (uint32_t)ne;
    uint32_t wrong = (h[0] ^ kMagic) | (h[1] ^ kVersion) | (h[2] ^ (uint32_t)DT) | (h[3] ^ kGroup);
    wrong |= (uint32_t)(n_hdr != n) | (uint32_t)(ne > n) | (uint32_t)(cbytes != L.esc + pad128(ne));
    wrong |= (uint32_t)(slot_off + cbytes > comp_capacity);
    wrong |= (uint32_t)(e0 < 1u) | (uint32_t)(e0 > 249u);
    wrong |= dec_lo & 0xFFu;                                   /* dec[0] is written as 0 */
    wrong |= (dec_lo >> 8) ^ (e0 | ((e0 + 1u) << 8) | ((e0 + 2u) << 16));
    wrong |= dec_hi ^ ((e0 + 3u) | ((e0 + 4u) << 8) | ((e0 + 5u) << 16) | ((e0 + 6u) << 24));
    const bool ok = wrong == 0u;
    return ok;
}

/* GPW groups per wave: a workgroup decodes a tile of 4 * GPW groups.  The compressed format does not know
 * tiles (groups are located through IDX alone), so this is free to differ from the compress side's tile. */
template <int DT, uint32_t GPW>
__global__ __launch_bounds__(kThreads, DT == ZIPCCL_BF16 ? 8 : 6)   /* waves per SIMD: <= 64 VGPRs for bf16, <= 80 for fp32 */
void k_decompress(const DecompressArgs a)
{
    constexpr uint32_t ES = DT == ZIPCCL_BF16 ? 2u : 4u;
    constexpr uint32_t TILE = kGroup * kWavesPerBlock * GPW;
    __shared__ DecTables s_tab;
    __shared__ __attribute__((aligned(16))) uint8_t s_esc[kWavesPerBlock][GPW][kEscRegion];

    /* grid = (tiles of the largest chunk, chunks) */
    const uint32_t c = blockIdx.y;
    const uint64_t n = a.tab.elem_off[c + 1] - a.tab.elem_off[c];
    if (blockIdx.x >= (n == 0 ? 1u : (n + TILE - 1) / TILE)) return;   /* an empty chunk still has its header checked */
    const uint64_t ts = (uint64_t)blockIdx.x * TILE;
    const uint8_t* __restrict__ slot = a.comp + a.tab.slot_off[c];
    uint8_t* __restrict__ cout = a.out + a.tab.elem_off[c] * ES;
    const SlotLayout L = slot_layout(n, DT);
    /* whole tiles take the vector path; a chunk of the tensor starts at some element of it, so its bytes are
       dword-aligned or (bf16, odd element) skewed by one halfword */
    const bool fast = ts + TILE <= n;
    const bool skew = (reinterpret_cast<uintptr_t>(cout) & 2u) != 0;
    const uint32_t lane = lane_id();
    const uint32_t wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);   /* scalar: group addresses and index entries stay out of the vector registers */
    const uint64_t ng = (n + kGroup - 1) / kGroup;

    /* What does not depend on the header or on IDX goes out first (the static part is readable: the host
       checked it): SM, planes and low words of the wave's groups, and the groups' index entries.
       The table build and the header check run while these loads are in flight. */
    const HeaderWords hdr = load_header(slot);
    DecIn in[GPW];
    uint32_t next[GPW];
    if (fast) {
#pragma unroll
        for (uint32_t u = 0; u < GPW; ++u) {
            const uint64_t gstart = ts + (uint64_t)(u * kWavesPerBlock + wave) * kGroup;
            decode_load<DT, true, false, DT == ZIPCCL_FP32>(slot, L, n, gstart, lane, in[u]);
            const uint64_t g = gstart / kGroup;
            const uint32_t* __restrict__ idx = reinterpret_cast<const uint32_t*>(slot + L.idx);
            in[u].base = idx[g];
            next[u] = idx[g + 1 < ng ? g + 1 : g];
        }
    }
    build_tables(s_tab);

    uint32_t e0, n_esc;
    const bool ok = check_header<DT>(hdr, L, n, a.tab.slot_off[c], a.comp_capacity, e0, n_esc);
    __syncthreads();
    if (!ok) {
        if (threadIdx.x == 0 && a.status) atomicOr(a.status, (uint32_t)ZIPCCL_ERR_CORRUPT);
        return;
    }

    uint32_t bad = 0;
    if (fast) {
        /* phases over the wave's groups, so that each phase's loads are all in flight together */
        DecEsc es[GPW];
        u32x4 lv[GPW];
#pragma unroll
        for (uint32_t u = 0; u < GPW; ++u) {
            const uint64_t g = (ts + (uint64_t)(u * kWavesPerBlock + wave) * kGroup) / kGroup;
            if (g + 1 >= ng) next[u] = n_esc;
            check_index(in[u], next[u], n_esc);
        }
#pragma unroll
        for (uint32_t u = 0; u < GPW; ++u) decode_fetch_list(slot, L, in[u], next[u], lane, lv[u]);
#pragma unroll
        for (uint32_t u = 0; u < GPW; ++u) decode_park_list(s_esc[wave][u], lane, lv[u]);
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
#pragma unroll
        for (uint32_t u = 0; u < GPW; ++u) {
            if (DT == ZIPCCL_FP32) {
                quad_plane_bytes(in[u], lane);
                es[u] = decode_locate_quad(in[u], s_esc[wave][u]);
            } else {
                es[u] = decode_locate(in[u], s_esc[wave][u]);
            }
        }
#pragma unroll
        for (uint32_t u = 0; u < GPW; ++u) {
            decode_store<DT, true>(cout, in[u], es[u], ts + (uint64_t)(u * kWavesPerBlock + wave) * kGroup, e0, lane, s_tab,
                                   DT == ZIPCCL_BF16 && skew);
            bad |= es[u].bad;
        }
    } else {
        for (uint32_t u = 0; u < GPW; ++u) {
            const uint64_t gstart = ts + (uint64_t)(u * kWavesPerBlock + wave) * kGroup;
            if (gstart < n) {
                DecIn r;
                uint32_t nx;
                u32x4 lv;
                decode_index(slot, L, n, n_esc, gstart, r, nx);
                decode_fetch_list(slot, L, r, nx, lane, lv);
                decode_load<DT, false>(slot, L, n, gstart, lane, r);
                decode_park_list(s_esc[wave][u], lane, lv);
                __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
                __builtin_amdgcn_wave_barrier();
                __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
                const DecEsc es = decode_locate(r, s_esc[wave][u]);
                decode_store<DT, false>(cout, r, es, gstart, e0, lane, s_tab);
                bad |= es.bad;
            }
        }
    }
    if (bad && a.status) atomicOr(a.status, (uint32_t)ZIPCCL_ERR_CORRUPT);
}

/* The bits a sum is stored as: a NaN sum becomes the one quiet NaN 0x7FC00000 (which payload and sign a NaN
 * result carries is left to the implementation by IEEE 754; this makes the output the same bits everywhere). */
__device__ __forceinline__ uint32_t sum_bits(float f)
{
    return f != f ? 0x7FC00000u : __float_as_uint(f);
}

/* fp32 bits (from sum_bits: no NaN other than 0x7FC00000, which this maps to 0x7FC0) -> bf16 bits, round to nearest even */
__device__ __forceinline__ uint32_t f32_bits_to_bf16_bits(uint32_t u)
{
    return (u + 0x7FFFu + ((u >> 16) & 1u)) >> 16;
}

/* A 32-bit load through the constant address space: for a wave-uniform address the compiler issues it
 * as a scalar load whatever stores the kernel contains.  Only for memory no kernel writes while this one
 * runs (the compressed input). */
__device__ __forceinline__ uint32_t load_const_u32(const uint8_t* p)
{
    typedef const uint32_t __attribute__((address_space(4))) * cptr;
    return *reinterpret_cast<cptr>(reinterpret_cast<uintptr_t>(p));
}

/*
 * A stage of the reduce pipeline = one peer's copy of one group.  The buffer holds the stage's loads in
 * flight and what describes it (cur_*), and, fetched ahead with scalar loads, the description and index
 * entries of the stage that uses the buffer next (pre_*).  Everything but the loaded words is wave-uniform.
 */
struct StageBuf {
    DecIn in;
    u32x4 lv;
    uint64_t pre_off;                 /* next stage: slot offset, */
    uint32_t pre_g;                   /* group, */
    uint32_t pre_base, pre_next;      /* the group's index entry and the following one, */
    uint32_t pre_nesc, pre_dec;       /* the slot's zero-point count and header word holding dec[0..3] */
    bool pre_last;                    /* and whether it is the last peer of its group */
    uint32_t cur_g, cur_e0;
    bool cur_last;
};

/*
 * Local reduction of the zipped Reduce-Scatter (paper sections 3.3 and 5.2): decode the slices
 * received from the peers (slots back to back, n values each) and sum them in FP32, peers in slot
 * order.  One pass: every compressed byte is read once and only the sum is written.
 *
 * A wave owns n_groups groups (gs0, gs0 + 2048, ...) and walks the stages (group, peer), peers
 * innermost, as one software pipeline that does not drain between groups: while stage k is decoded,
 * the loads of stage k + 1 are in flight and the index entries of stage k + 2 have been requested.
 * Every stage issues the same number of loads, so that a wait for the older ones never has to drain
 * the younger ones; past the last stage the look-ahead repeats the last stage's requests.
 * The sum starts at -0.0f, the identity of FP32 addition for everything that is not a NaN, and one
 * addition per accepted slot follows; a NaN sum is stored as 0x7FC00000 (sum_bits).
 */
template <int DT, int ODT, bool FAST>
__device__ __forceinline__ void reduce_stages(const ReduceArgs& a, const SlotLayout& L, uint64_t gs0, uint32_t n_groups,
                                              uint32_t n_acc, uint32_t lane, uint8_t* lds, const DecTables& tab,
                                              const uint32_t* s_peer, bool all_ok, uint32_t& bad)
{
    constexpr uint32_t OES = ODT == ZIPCCL_BF16 ? 2u : 4u;
    const uint64_t n = a.n;
    const uint32_t ng = (uint32_t)((n + kGroup - 1) / kGroup);     /* n < 2^32: group numbers fit 32 bits */
    const uint32_t T = n_acc * n_groups;
    float acc[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) acc[j] = -0.0f;

    /* the look-ahead front: describe its stage into r.pre_* (the slot's header was checked by the
       workgroup; zero-point count, table and index entries come by scalar loads), then advance.
       The index position moves along with the stage instead of being recomputed. */
    uint32_t jf = 0, adv_left = T - 1u;
    uint32_t gf = (uint32_t)(gs0 / kGroup);
    uint64_t idx_f = L.idx + 4u * (uint64_t)gf;                /* of IDX[gf] in a slot */
    uint32_t next_f = gf + 1u < ng ? 4u : 0u;                  /* from there to the following entry, if any */
    uint64_t off_f = 0;                                        /* all slots accepted: offset of slot jf */
    auto front = [&](StageBuf& r) {
        /* some slot rejected: the j-th accepted one is not slot j */
        r.pre_off = all_ok ? off_f : (uint64_t)__builtin_amdgcn_readfirstlane(s_peer[jf]) * a.slot_cap;
        const uint8_t* __restrict__ slot = a.comp + r.pre_off;
        r.pre_nesc = load_const_u32(slot + 24);
        r.pre_dec = load_const_u32(slot + 40);
        r.pre_g = gf;
        r.pre_last = jf + 1u == n_acc;
        r.pre_base = load_const_u32(slot + idx_f);
        r.pre_next = load_const_u32(slot + idx_f + next_f);
        if (adv_left != 0u) {
            --adv_left;
            ++jf;
            off_f += a.slot_cap;
            if (jf == n_acc) {
                jf = 0;
                off_f = 0;
                gf += kWavesPerBlock;
                idx_f += 4u * kWavesPerBlock;
                next_f = gf + 1u < ng ? 4u : 0u;
            }
        }
    };
    /* issue every vector load of the stage r.pre_* describes.  FAST: the lanes' offsets inside a slot
       (section + group + lane) are kept in vector registers and renewed when the group changes, so that
       a stage adds nothing but the slot's address. */
    uint32_t g_iss = 0xFFFFFFFFu;
    uint64_t v_sm = 0, v_pl = 0, v_lo = 0;
    auto issue = [&](StageBuf& r) {
        r.cur_g = r.pre_g; r.cur_e0 = (r.pre_dec >> 8) & 0xFFu; r.cur_last = r.pre_last;
        const uint8_t* __restrict__ slot = a.comp + r.pre_off;
        const uint32_t next = r.pre_g + 1u < ng ? r.pre_next : r.pre_nesc;
        r.in.base = r.pre_base;
        check_index(r.in, next, r.pre_nesc);
        if (FAST) {
            if (r.pre_g != g_iss) {
                g_iss = r.pre_g;
                const uint64_t gs = (uint64_t)g_iss * kGroup;
                v_sm = L.sm + gs + lane * 8u;
                /* the group's 3 x 64 plane bytes in one load: lanes 0..15 fetch the words of plane 0,
                   16..31 those of plane 1, 32..47 (and again 48..63) those of plane 2 */
                v_pl = L.p0 + (gs >> 3) + (lane & 15u) * 4u + (uint64_t)min(lane >> 4, 2u) * L.plane_bytes;
                v_lo = L.lo + 2 * gs + lane * 16u;
            }
            /* the list as in decode_fetch_list, relative to 16 bytes before it */
            const uint32_t end = r.in.count != 0u ? next : 0u;
            const uint32_t a16 = (r.in.base & ~15u) + 16u * lane;
            r.lv = *reinterpret_cast<const u32x4*>((slot + (L.esc - 16)) + (a16 < end ? a16 + 16u : 0u));
            const u32x2 sm = ld_stream<u32x2>(slot + v_sm);
            r.in.sm0 = sm.x; r.in.sm1 = sm.y;
            /* a plain load, not a streaming one: a group's 64 bytes of a plane are half a cache line, and the
               other half is the neighbouring group's, which another wave decodes at another time (streamed,
               such lines came from memory twice: 13 % more bytes fetched and 204 instead of 179 us for
               8 x 2^26 values) */
            r.in.b0 = *reinterpret_cast<const uint32_t*>(slot + v_pl);
            if (DT == ZIPCCL_FP32) {
                const u32x4 lo = ld_stream<u32x4>(slot + v_lo);
                r.in.lo[0] = lo.x; r.in.lo[1] = lo.y; r.in.lo[2] = lo.z; r.in.lo[3] = lo.w;
            }
            r.in.vmask = 0xFFu;
        } else {
            decode_fetch_list(slot, L, r.in, next, lane, r.lv);
            decode_load<DT, false, true>(slot, L, n, (uint64_t)r.pre_g * kGroup, lane, r.in);
        }
    };
    /* decode the stage in r and add it; after a group's last peer the sums are stored */
    auto consume = [&](StageBuf& r) {
        /* nothing that uses the stage's loaded words may be scheduled before this point (among the loads
           of the next stage, where it would wait for them to land as well) */
        __builtin_amdgcn_sched_barrier(0);
        if (FAST) {
            /* the word holding the lane's byte of plane k sits in lane 16 k + lane / 4 */
            const uint32_t w = r.in.b0, from = (lane >> 2) * 4u;
            r.in.b0 = __builtin_amdgcn_ds_bpermute(from, w);
            r.in.b1 = __builtin_amdgcn_ds_bpermute(from + 64u, w);
            r.in.b2 = __builtin_amdgcn_ds_bpermute(from + 128u, w);
        }
        plane_bytes_of_words(r.in, lane);
        /* park the slice; the wave's region holds 64 x 16 bytes, so every lane writes what it fetched and the
           store needs no predicate (lanes past the slice hold bytes that no lane picks) */
        *reinterpret_cast<u32x4*>(lds + 16u * lane) = r.lv;
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
        const DecEsc es = decode_locate(r.in, lds);
        __builtin_amdgcn_wave_barrier();
        bad |= es.bad;
        float x[8];
        if (DT == ZIPCCL_BF16) {
            uint32_t lA, hA, lB, hB;
            decode_bytes(r.in, es, r.cur_e0, tab, lA, hA, lB, hB);
#pragma unroll
            for (uint32_t j = 0; j < 4; ++j) {    /* value j as FP32 bits: high byte, low byte, 16 zero bits */
                const uint32_t sel = ((4u + j) << 24) | (j << 16) | 0x0C0Cu;
                x[j] = __uint_as_float(perm(hA, lA, sel));
                x[4 + j] = __uint_as_float(perm(hB, lB, sel));
            }
        } else {
            uint32_t hp[4];
            decode_values(r.in, es, r.cur_e0, tab, hp);
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                x[2 * k] = __uint_as_float(perm(hp[k], r.in.lo[k], 0x05040100u));
                x[2 * k + 1] = __uint_as_float(perm(hp[k], r.in.lo[k], 0x07060302u));
            }
        }
#pragma unroll
        for (int j = 0; j < 8; ++j) acc[j] += x[j];
        if (r.cur_last) {
            uint8_t* __restrict__ og = a.out + (uint64_t)r.cur_g * kGroup * OES;
            if (FAST) {
                /* a NaN among the lane's sums is rare: one unordered compare per pair of sums finds out, and
                   only then are the eight looked at one by one (sum_bits) */
                const bool any_nan = (acc[0] != acc[0] || acc[1] != acc[1]) | (acc[2] != acc[2] || acc[3] != acc[3]) |
                                     (acc[4] != acc[4] || acc[5] != acc[5]) | (acc[6] != acc[6] || acc[7] != acc[7]);
                if (__builtin_expect(__ballot(any_nan) != 0ull, 0)) {
#pragma unroll
                    for (int j = 0; j < 8; ++j) acc[j] = __uint_as_float(sum_bits(acc[j]));
                }
                if (ODT == ZIPCCL_FP32) {
                    /* The lane's 8 sums are 32 contiguous bytes, a pattern that stores slowly.  Once per
                       group they go through the wave's LDS region (free between decodes), half a group at
                       a time, and come back as 16 contiguous bytes per lane: two streaming stores of 1 KiB. */
                    const u32x4 lo4 = u32x4{__float_as_uint(acc[0]), __float_as_uint(acc[1]),
                                            __float_as_uint(acc[2]), __float_as_uint(acc[3])};
                    const u32x4 hi4 = u32x4{__float_as_uint(acc[4]), __float_as_uint(acc[5]),
                                            __float_as_uint(acc[6]), __float_as_uint(acc[7])};
                    u32x4 row[2];
#pragma unroll
                    for (uint32_t h = 0; h < 2; ++h) {
                        if ((lane >> 5) == h) {
                            *reinterpret_cast<u32x4*>(lds + (lane & 31u) * 32u) = lo4;
                            *reinterpret_cast<u32x4*>(lds + (lane & 31u) * 32u + 16u) = hi4;
                        }
                        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
                        __builtin_amdgcn_wave_barrier();
                        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
                        row[h] = *reinterpret_cast<const u32x4*>(lds + lane * 16u);
                        __builtin_amdgcn_wave_barrier();
                    }
                    st_stream_a4(og + lane * 16u, row[0]);
                    st_stream_a4((og + 2 * kGroup) + lane * 16u, row[1]);
                } else {
                    uint32_t o[4];
#pragma unroll
                    for (int k = 0; k < 4; ++k)
                        o[k] = f32_bits_to_bf16_bits(__float_as_uint(acc[2 * k])) | (f32_bits_to_bf16_bits(__float_as_uint(acc[2 * k + 1])) << 16);
                    st_stream_a4(og + lane * 16u, u32x4{o[0], o[1], o[2], o[3]});
                }
            } else {
#pragma unroll
                for (int j = 0; j < 8; ++j) {
                    if ((r.in.vmask >> j) & 1u) {
                        const uint64_t i = lane * kLaneElems + j;
                        if (ODT == ZIPCCL_FP32) *reinterpret_cast<uint32_t*>(og + i * 4) = sum_bits(acc[j]);
                        else *reinterpret_cast<uint16_t*>(og + i * 2) = (uint16_t)f32_bits_to_bf16_bits(sum_bits(acc[j]));
                    }
                }
            }
#pragma unroll
            for (int j = 0; j < 8; ++j) acc[j] = -0.0f;
        }
    };

    /* two buffers used in turn (a copy from one to the other would have to wait for the loads).
       front()'s scalar loads return out of order, so any wait for one of them (or for an LDS access)
       waits for all: a stage requests them first, then issues its vector loads with what the previous
       stage's requests brought (long complete: the LDS waits of its decode saw to that), then decodes. */
    StageBuf bufA, bufB;
    front(bufA);
    front(bufB);
    __builtin_amdgcn_s_waitcnt(0xC07F);  /* lgkmcnt(0): nothing pending when the loop is entered */
    issue(bufA);
    uint32_t k = 0;                      /* stage whose loads bufA holds */
    while (k + 2u < T) {                 /* two stages, each with a real stage to look ahead to */
        front(bufA);
        asm volatile("" ::: "memory");
        issue(bufB);
        consume(bufA);
        front(bufB);
        asm volatile("" ::: "memory");
        issue(bufA);
        consume(bufB);
        k += 2u;
    }
    if (k + 2u == T) {                   /* two stages left */
        issue(bufB);
        consume(bufA);
        consume(bufB);
    } else {
        consume(bufA);
    }
}

/*
 * One launch covers a call: workgroups 0 .. a.n_full - 1 take whole tiles of a.gpw groups per wave (every group
 * complete, the output dword-aligned: the form without bounds checks), the workgroups after them the rest of the
 * shard in tiles of a.gpw_rest groups per wave through the general form.  Groups per wave: the larger, the fewer
 * workgroups pay for the header checks and the table build; 1 for small shards, and for the rest behind whole
 * tiles, so that there are enough workgroups to fill the chip.  REST = false: the launch holds whole tiles only
 * (the general form is compiled out: it costs the whole-tile workgroups a few per cent of vector instructions
 * to share a kernel with it).  Dynamic LDS: one 32-bit word per peer.
 */
template <int DT, int ODT, bool REST>
__global__ __launch_bounds__(kThreads, DT == ZIPCCL_BF16 ? 8 : 6) void k_decompress_reduce(const ReduceArgs a)
{
    extern __shared__ __attribute__((aligned(16))) uint8_t s_dyn[];
    uint32_t* s_peer = reinterpret_cast<uint32_t*>(s_dyn);     /* the accepted slots, in slot order */
    __shared__ DecTables s_tab;
    /* per wave: the zero-point slice of the group being decoded, or half a group of FP32 sums on their way out */
    constexpr uint32_t kRegion = kEscRegion > 1024u ? kEscRegion : 1024u;
    __shared__ __attribute__((aligned(16))) uint8_t s_esc[kWavesPerBlock][kRegion];
    __shared__ uint32_t s_wcnt[kWavesPerBlock];
    build_tables(s_tab);

    const uint64_t n = a.n;
    const bool whole = !REST || blockIdx.x < a.n_full;        /* workgroup-uniform */
    const uint32_t gpw = whole ? a.gpw : a.gpw_rest;
    constexpr uint64_t kGroupStride = (uint64_t)kGroup * kWavesPerBlock;
    const uint64_t ts = whole ? (uint64_t)blockIdx.x * (kGroupStride * a.gpw)
                              : (uint64_t)a.n_full * (kGroupStride * a.gpw) + (uint64_t)(blockIdx.x - a.n_full) * (kGroupStride * a.gpw_rest);
    const SlotLayout L = slot_layout(n, DT);
    const uint32_t lane = lane_id();
    const uint32_t wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);   /* scalar: group addresses are wave-uniform */

    /* every slot's header is checked once per workgroup, one peer per thread; the accepted ones are
       listed in slot order (ballot + per-wave counts), the others are left out of the sum */
    uint32_t n_acc = 0;
    for (uint32_t r = 0; r < a.n_peers; r += kThreads) {
        const uint32_t p = r + threadIdx.x;
        const uint64_t slot_off = (uint64_t)p * a.slot_cap;
        uint32_t e0 = 0, n_esc = 0;
        const bool ok = p < a.n_peers && check_header<DT>(load_header(a.comp + slot_off), L, n, slot_off, a.comp_capacity, e0, n_esc);
        const uint64_t votes = __ballot(ok);
        if (lane == 0) s_wcnt[wave] = (uint32_t)__popcll(votes);
        __syncthreads();
        uint32_t before = 0, total = 0;
#pragma unroll
        for (uint32_t w = 0; w < kWavesPerBlock; ++w) {
            const uint32_t c = s_wcnt[w];
            before += w < wave ? c : 0u;
            total += c;
        }
        if (ok) {
            const uint32_t pos = n_acc + before + (uint32_t)__popcll(votes & ((1ull << lane) - 1ull));
            s_peer[pos] = p;
        }
        n_acc += total;
        __syncthreads();
    }
    n_acc = __builtin_amdgcn_readfirstlane(n_acc);
    uint32_t bad = n_acc != a.n_peers;

    /* this wave's groups start at gs0, gs0 + 2048, ...; those that begin inside n count */
    const uint64_t gs0 = ts + (uint64_t)wave * kGroup;
    uint32_t n_groups = gpw;
    if (!whole) n_groups = gs0 >= n ? 0u : (uint32_t)min((uint64_t)gpw, (n - gs0 + kGroupStride - 1) / kGroupStride);
    if (n_groups != 0u) {
        if (n_acc != 0u) {
            if (whole) reduce_stages<DT, ODT, true>(a, L, gs0, n_groups, n_acc, lane, s_esc[wave], s_tab, s_peer, n_acc == a.n_peers, bad);
            else if (REST) reduce_stages<DT, ODT, false>(a, L, gs0, n_groups, n_acc, lane, s_esc[wave], s_tab, s_peer, n_acc == a.n_peers, bad);
        } else {
            /* no slot accepted: the sum of nothing */
            constexpr uint32_t OES = ODT == ZIPCCL_BF16 ? 2u : 4u;
            for (uint32_t u = 0; u < n_groups; ++u) {
                const uint64_t e = gs0 + u * kGroupStride + lane * kLaneElems;
                for (uint32_t j = 0; j < kLaneElems; ++j) {
                    if (e + j < n) {
                        if (ODT == ZIPCCL_FP32) *reinterpret_cast<uint32_t*>(a.out + (e + j) * OES) = 0u;
                        else *reinterpret_cast<uint16_t*>(a.out + (e + j) * OES) = 0u;
                    }
                }
            }
        }
    }
    if (bad && a.status) atomicOr(a.status, (uint32_t)ZIPCCL_ERR_CORRUPT);
}

} // namespace

/* launches that write at least this many bytes decode in tiles of 8 groups, smaller ones in tiles of 16 */
constexpr uint64_t kDecSmallTileFrom = 64ull << 20;

template <uint32_t GPW>
static int launch_decompress_gpw(int dt, const DecompressArgs& a, void* stream)
{
    constexpr uint64_t TILE = (uint64_t)kGroup * kWavesPerBlock * GPW;
    uint64_t tiles = 1;
    for (uint32_t c = 0; c < a.tab.n_chunks; ++c) {
        const uint64_t t = (a.tab.elem_off[c + 1] - a.tab.elem_off[c] + TILE - 1) / TILE;
        tiles = t > tiles ? t : tiles;
    }
    const dim3 grid((uint32_t)tiles, a.tab.n_chunks), block(kThreads);
    if (dt == ZIPCCL_BF16)
        hipLaunchKernelGGL((k_decompress<ZIPCCL_BF16, GPW>), grid, block, 0, (hipStream_t)stream, a);
    else
        hipLaunchKernelGGL((k_decompress<ZIPCCL_FP32, GPW>), grid, block, 0, (hipStream_t)stream, a);
    return (int)hipGetLastError();
}

int launch_decompress(int dt, const DecompressArgs& a, void* stream)
{
    /* Measured on MI355X: tiles of 8 groups (4096 values) decode 2-3 % faster than tiles of 16 once the launch
       holds many workgroups per compute unit; a launch of about one round of workgroups is faster with 16. */
    const uint64_t total = (a.tab.elem_off[a.tab.n_chunks] - a.tab.elem_off[0]) * (dt == ZIPCCL_BF16 ? 2u : 4u);
    return total >= kDecSmallTileFrom ? launch_decompress_gpw<2>(dt, a, stream) : launch_decompress_gpw<kGroupsPerWave>(dt, a, stream);
}


/*
 * Groups per wave of the fused reduce, from timings on MI355X over shards of 2^22 to 2^27 values.  One group per
 * wave while the shard gives the chip's resident workgroups (256 CUs x 8, or x 6 for fp32) too little to do
 * for a second group to pay; two from there on; four only for bf16 shards that fill the chip a whole number of
 * times with four (2048 workgroups at once), where the last round leaves no compute unit idle: 3 % faster than two
 * at 2^26 values, while between such sizes two groups per wave are 1-6 % faster than four.
 */
static uint32_t reduce_groups_per_wave(uint64_t n, int dt)
{
    const uint64_t tiles = n / kTile;
    if (dt == ZIPCCL_FP32) return tiles < 2560u ? 1u : 2u;
    if (tiles < 640u) return 1u;
    return tiles % 2048u == 0 ? 4u : 2u;
}

int launch_decompress_reduce(int dt, int out_dt, const ReduceArgs& a, void* stream)
{
    hipStream_t s = (hipStream_t)stream;
    const dim3 block(kThreads);
    ReduceArgs b = a;
    b.gpw = reduce_groups_per_wave(a.n, dt);
    const uint64_t per = (uint64_t)kGroup * kWavesPerBlock * b.gpw;
    /* whole tiles with a dword-aligned output go through the form without bounds checks, the rest (under one
       tile, or everything when the output is only 2-byte aligned) through the general one, in the same launch */
    const size_t lds_bytes = sizeof(uint32_t) * a.n_peers;
    const bool aligned = (reinterpret_cast<uintptr_t>(a.out) & 3u) == 0;
    const uint64_t full = aligned ? a.n / per : 0;
    const uint64_t rest = a.n - full * per;
    b.n_full = (uint32_t)full;
    b.gpw_rest = full ? 1u : b.gpw;     /* under a tile is left: one group per wave, so that it is not one workgroup's crawl */
    const uint64_t per_rest = (uint64_t)kGroup * kWavesPerBlock * b.gpw_rest;
    uint64_t n_rest = (rest + per_rest - 1) / per_rest;
    if (a.n == 0) n_rest = 1;           /* one workgroup that only checks the headers */
    const dim3 grid((uint32_t)(full + n_rest));
#define ZIPCCL_REDUCE(REST)                                                                                            \
    do {                                                                                                               \
        if (dt == ZIPCCL_BF16 && out_dt == ZIPCCL_FP32)                                                                \
            hipLaunchKernelGGL((k_decompress_reduce<ZIPCCL_BF16, ZIPCCL_FP32, REST>), grid, block, lds_bytes, s, b);   \
        else if (dt == ZIPCCL_BF16)                                                                                    \
            hipLaunchKernelGGL((k_decompress_reduce<ZIPCCL_BF16, ZIPCCL_BF16, REST>), grid, block, lds_bytes, s, b);   \
        else if (out_dt == ZIPCCL_FP32)                                                                                \
            hipLaunchKernelGGL((k_decompress_reduce<ZIPCCL_FP32, ZIPCCL_FP32, REST>), grid, block, lds_bytes, s, b);   \
        else                                                                                                           \
            hipLaunchKernelGGL((k_decompress_reduce<ZIPCCL_FP32, ZIPCCL_BF16, REST>), grid, block, lds_bytes, s, b);   \
    } while (0)
    if (n_rest) ZIPCCL_REDUCE(true);
    else ZIPCCL_REDUCE(false);
#undef ZIPCCL_REDUCE
    return (int)hipGetLastError();
}


} // namespace zipccl
