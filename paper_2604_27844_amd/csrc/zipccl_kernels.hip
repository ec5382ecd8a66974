/*
 * HIP kernels of libzipccl.so for gfx950 (CDNA4, wave64).
 *
 * compress   : paper section 4 (split, 3-bit code, zero-points) with the kernel steps of
 *              section 4.2 re-designed for wave64: one wave handles a group of 512 values,
 *              8 consecutive values per lane (one 16-byte load for bf16), a workgroup of
 *              4 waves handles a tile of 16 groups.  The zero-point offsets of section 4.2.3
 *              are an exclusive prefix in element order (lane -> wave -> tile -> chunk), so the
 *              output is deterministic; the chunk-wide part is a decoupled look-back over
 *              per-tile state words instead of the paper's block-level atomic add.
 * decompress : section 4, third paragraph.  No dependency between workgroups.
 *
 * Everything is integer work; sigma / erf live on the host.
 */
#include <hip/hip_runtime.h>

#include "zipccl_internal.h"

namespace zipccl {
namespace {

constexpr uint64_t kFlagAgg = 1ull << 32;  /* tile state: low 32 bits = this tile's zero-point count */
constexpr uint64_t kFlagInc = 2ull << 32;  /* tile state: low 32 bits = count of this and all earlier tiles of the chunk */
constexpr uint32_t kSpinLimit = 1u << 22;  /* polls before the look-back gives up and flags an error */

__device__ __forceinline__ uint32_t lane_id()
{
    return __builtin_amdgcn_mbcnt_hi(~0u, __builtin_amdgcn_mbcnt_lo(~0u, 0u));
}

/* inclusive prefix sum over the 64 lanes of a wave */
__device__ __forceinline__ uint32_t wave_incl_scan(uint32_t x, uint32_t lane)
{
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
        const uint32_t y = __shfl_up(x, d, 64);
        if (lane >= (uint32_t)d) x += y;
    }
    return x;
}

__device__ __forceinline__ uint32_t wave_sum(uint32_t x)
{
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) x += __shfl_xor(x, d, 64);
    return x;
}

/* largest c with tile_start[c] <= t (every chunk owns at least one tile) */
__device__ __forceinline__ uint32_t find_chunk(const ChunkTab& tab, uint32_t t)
{
    uint32_t lo = 0, hi = tab.n_chunks;
    while (hi - lo > 1) {
        const uint32_t mid = (lo + hi) >> 1;
        if (tab.tile_start[mid] <= t) lo = mid; else hi = mid;
    }
    return lo;
}

__device__ __forceinline__ void store_state(uint64_t* p, uint64_t v)
{
    __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ uint64_t load_state(const uint64_t* p)
{
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

/*
 * Load the lane's 8 consecutive values starting at chunk-relative element e.
 * hp[k] packs the high 16-bit words of values 2k (low half) and 2k+1 (high half);
 * lp[k] the low words (fp32 only).  vmask bit j = value j exists (e + j < n).
 */
template <int DT, bool FAST>
__device__ __forceinline__ void load_lane(const uint8_t* __restrict__ cin, uint64_t e, uint64_t n,
                                          uint32_t hp[4], uint32_t lp[4], uint32_t& vmask)
{
    if (FAST) {
        vmask = 0xFFu;
        if (DT == ZIPCCL_BF16) {
            const uint4 v = *reinterpret_cast<const uint4*>(cin + e * 2);
            hp[0] = v.x; hp[1] = v.y; hp[2] = v.z; hp[3] = v.w;
            lp[0] = lp[1] = lp[2] = lp[3] = 0;
        } else {
            const uint4 a = *reinterpret_cast<const uint4*>(cin + e * 4);
            const uint4 b = *reinterpret_cast<const uint4*>(cin + e * 4 + 16);
            const uint32_t x[8] = {a.x, a.y, a.z, a.w, b.x, b.y, b.z, b.w};
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                hp[k] = (x[2 * k] >> 16) | (x[2 * k + 1] & 0xFFFF0000u);
                lp[k] = (x[2 * k] & 0xFFFFu) | (x[2 * k + 1] << 16);
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

/*
 * Encode one group (section 4: split / code / zero-point detection).  Writes the SM, LO and
 * plane bytes of the lane when STORE; returns the lane's 8 raw exponents (ex_lo, ex_hi), its
 * zero-point mask m, its exclusive offset inside the group and the group's zero-point count.
 */
template <int DT, bool FAST, bool STORE>
__device__ __forceinline__ void encode_group(const uint8_t* __restrict__ cin, uint8_t* __restrict__ slot,
                                             const SlotLayout& L, uint64_t n, uint64_t e, uint32_t e0m1,
                                             uint32_t lane, uint32_t& ex_lo, uint32_t& ex_hi, uint32_t& m,
                                             uint32_t& loff, uint32_t& gtot)
{
    uint32_t hp[4], lp[4], vmask;
    load_lane<DT, FAST>(cin, e, n, hp, lp, vmask);
    uint32_t sm[2] = {0, 0}, ex[2] = {0, 0}, b0 = 0, b1 = 0, b2 = 0;
    m = 0;
#pragma unroll
    for (int j = 0; j < 8; ++j) {
        const uint32_t h = (j & 1) ? (hp[j >> 1] >> 16) : (hp[j >> 1] & 0xFFFFu);
        const uint32_t E = (h >> 7) & 0xFFu;
        const uint32_t t = E - e0m1;               /* 1..7 inside the window (mod 2^32) */
        uint32_t code = t < 8u ? t : 0u;
        if (!FAST) code = ((vmask >> j) & 1u) ? code : 0u;
        const uint32_t smb = ((h >> 8) & 0x80u) | (h & 0x7Fu);
        sm[j >> 2] |= smb << (8 * (j & 3));
        ex[j >> 2] |= E << (8 * (j & 3));
        b0 |= (code & 1u) << j;
        b1 |= ((code >> 1) & 1u) << j;
        b2 |= (code >> 2) << j;
        m |= (code == 0u ? 1u : 0u) << j;
    }
    m &= vmask;
    if (STORE) {
        if (FAST || e < pad128(n))
            *reinterpret_cast<uint2*>(slot + L.sm + e) = make_uint2(sm[0], sm[1]);
        if (DT == ZIPCCL_FP32) {
            if (FAST || 2 * e < pad128(2 * n))
                *reinterpret_cast<uint4*>(slot + L.lo + 2 * e) = make_uint4(lp[0], lp[1], lp[2], lp[3]);
        }
        const uint64_t pb = e >> 3;
        if (FAST || pb < L.plane_bytes) {
            slot[L.p0 + pb] = (uint8_t)b0;
            slot[L.p0 + L.plane_bytes + pb] = (uint8_t)b1;
            slot[L.p0 + 2 * L.plane_bytes + pb] = (uint8_t)b2;
        }
    }
    const uint32_t cnt = __popc(m);
    const uint32_t inc = wave_incl_scan(cnt, lane);
    loff = inc - cnt;
    gtot = __shfl(inc, 63, 64);
    ex_lo = ex[0];
    ex_hi = ex[1];
}

/*
 * Decoupled look-back (run by one wave): sum of the zero-point counts of tiles [first, t).
 * Lane i inspects tile t-1-i; a tile state is 0 (not yet published), an aggregate, or an
 * inclusive prefix.  Tiles before `first` count as an inclusive prefix of 0.  The wait is
 * bounded: past kSpinLimit polls the error word is set and the result is unspecified.
 */
__device__ __forceinline__ uint32_t look_back(const uint64_t* state, uint32_t t, uint32_t first,
                                              uint32_t lane, uint32_t* err)
{
    uint32_t prefix = 0, spins = 0;
    int64_t look = (int64_t)t - 1;
    for (;;) {
        const int64_t i = look - (int64_t)lane;
        uint64_t s = kFlagInc; /* before the chunk's first tile: nothing */
        if (i >= (int64_t)first) s = load_state(state + i);
        const uint32_t flag = (uint32_t)(s >> 32);
        const uint64_t invalid = __ballot(flag == 0u);
        const uint64_t incl = __ballot(flag == 2u);
        const uint32_t j = incl ? (uint32_t)__builtin_ctzll(incl) : 64u; /* nearest inclusive */
        const uint64_t need = j >= 63u ? ~0ull : ((2ull << j) - 1ull);   /* lanes 0..j */
        if (invalid & need) {
            if (++spins > kSpinLimit) {
                if (lane == 0) atomicOr(err, (uint32_t)ZIPCCL_ERR_DEVICE);
                return prefix;
            }
            __builtin_amdgcn_s_sleep(1);
            continue;
        }
        prefix += wave_sum(lane <= j ? (uint32_t)s : 0u);
        if (j < 64u) return prefix;
        look -= 64;
    }
}

template <int DT, int MODE>
__global__ __launch_bounds__(kThreads) void k_compress(const CompressArgs a)
{
    constexpr uint32_t ES = DT == ZIPCCL_BF16 ? 2u : 4u;
    constexpr bool STORE = MODE != kModeCount;
    __shared__ uint32_t s_gcnt[kGroupsPerTile];
    __shared__ uint32_t s_prefix;

    const uint32_t t = blockIdx.x;
    const uint32_t c = find_chunk(a.tab, t);
    const uint32_t first = a.tab.tile_start[c];
    const bool last_tile = (t + 1u == a.tab.tile_start[c + 1]);
    const uint64_t n = a.tab.elem_off[c + 1] - a.tab.elem_off[c];
    const uint64_t ts = (uint64_t)(t - first) * kTile;
    const uint8_t* __restrict__ cin = a.in + a.tab.elem_off[c] * ES;
    uint8_t* __restrict__ slot = a.out + a.tab.slot_off[c];
    const SlotLayout L = slot_layout(n, DT);
    const bool fast = (ts + kTile <= n) && ((reinterpret_cast<uintptr_t>(cin) & 15u) == 0);
    const uint32_t lane = lane_id();
    const uint32_t wave = threadIdx.x >> 6;
    const uint32_t e0m1 = a.e0 - 1u;

    uint32_t ex_lo[kGroupsPerWave], ex_hi[kGroupsPerWave], em[kGroupsPerWave], loff[kGroupsPerWave],
        gtot[kGroupsPerWave];
    if (fast) {
#pragma unroll
        for (uint32_t u = 0; u < kGroupsPerWave; ++u) {
            const uint64_t e = ts + (uint64_t)(u * kWavesPerBlock + wave) * kGroup + lane * kLaneElems;
            encode_group<DT, true, STORE>(cin, slot, L, n, e, e0m1, lane, ex_lo[u], ex_hi[u], em[u], loff[u], gtot[u]);
        }
    } else {
#pragma unroll
        for (uint32_t u = 0; u < kGroupsPerWave; ++u) {
            const uint64_t e = ts + (uint64_t)(u * kWavesPerBlock + wave) * kGroup + lane * kLaneElems;
            encode_group<DT, false, STORE>(cin, slot, L, n, e, e0m1, lane, ex_lo[u], ex_hi[u], em[u], loff[u], gtot[u]);
        }
    }

    /* tile-level exclusive prefix of the 16 group counts, in element order */
    if (lane == 0) {
#pragma unroll
        for (uint32_t u = 0; u < kGroupsPerWave; ++u) s_gcnt[u * kWavesPerBlock + wave] = gtot[u];
    }
    __syncthreads();
    uint32_t goff[kGroupsPerWave], tile_total = 0;
#pragma unroll
    for (uint32_t g = 0; g < kGroupsPerTile; ++g) {
        if ((g % kWavesPerBlock) == wave) goff[g / kWavesPerBlock] = tile_total;
        tile_total += s_gcnt[g];
    }

    if (MODE == kModeCount) {
        if (threadIdx.x == 0) a.tile_state[t] = tile_total;
        return;
    }

    /* chunk-level exclusive prefix P = zero-points of this chunk before this tile */
    uint32_t P;
    if (MODE == kModeEmit) {
        P = (uint32_t)a.tile_state[t];
    } else {
        if (wave == 0) {
            uint32_t p = 0;
            if (t != first) {
                if (lane == 0) store_state(a.tile_state + t, kFlagAgg | tile_total);
                p = look_back(a.tile_state, t, first, lane, a.err);
            }
            if (lane == 0) {
                store_state(a.tile_state + t, kFlagInc | (uint64_t)(p + tile_total));
                s_prefix = p;
            }
        }
        __syncthreads();
        P = s_prefix;
    }

    /* group index (section 4.2.3) and zero-point exponents in element order */
    const uint64_t ng = (n + kGroup - 1) / kGroup;
    uint32_t* __restrict__ idx = reinterpret_cast<uint32_t*>(slot + L.idx);
    uint8_t* __restrict__ esc = slot + L.esc;
#pragma unroll
    for (uint32_t u = 0; u < kGroupsPerWave; ++u) {
        const uint64_t g = ts / kGroup + (u * kWavesPerBlock + wave);
        if (lane == 0 && g < ng) idx[g] = P + goff[u];
        uint8_t* dst = esc + (uint64_t)P + goff[u] + loff[u];
        uint32_t mm = em[u];
        const uint64_t ex = (uint64_t)ex_lo[u] | ((uint64_t)ex_hi[u] << 32);
        while (mm) {
            const uint32_t j = __builtin_ctz(mm);
            mm &= mm - 1u;
            *dst++ = (uint8_t)(ex >> (8 * j));
        }
    }

    if (last_tile) {
        const uint64_t n_esc = (uint64_t)P + tile_total;
        const uint64_t cbytes = L.esc + pad128(n_esc);
        if (threadIdx.x < 32) {
            uint32_t w = 0;
            switch (threadIdx.x) {
                case 0: w = kMagic; break;
                case 1: w = kVersion; break;
                case 2: w = (uint32_t)DT; break;
                case 3: w = kGroup; break;
                case 4: w = (uint32_t)n; break;
                case 5: w = (uint32_t)(n >> 32); break;
                case 6: w = (uint32_t)n_esc; break;
                case 7: w = (uint32_t)(n_esc >> 32); break;
                case 8: w = (uint32_t)cbytes; break;
                case 9: w = (uint32_t)(cbytes >> 32); break;
                case 10: w = a.dec_lo; break;
                case 11: w = a.dec_hi; break;
                default: break;
            }
            reinterpret_cast<uint32_t*>(slot)[threadIdx.x] = w;
            const uint64_t ie = ng + threadIdx.x;           /* zero the IDX padding */
            if (4 * ie < pad128(4 * ng)) idx[ie] = 0;
        }
        if (threadIdx.x < 128) {                            /* zero the ESC padding */
            const uint64_t je = n_esc + threadIdx.x;
            if (je < pad128(n_esc)) esc[je] = 0;
        }
        if (threadIdx.x == 0 && a.chunk_bytes) a.chunk_bytes[c] = cbytes;
    }
}

/* Three-kernel path only: turn the per-tile counts of every chunk into exclusive prefixes. */
__global__ __launch_bounds__(kThreads) void k_tile_scan(const CompressArgs a)
{
    __shared__ uint32_t s_part[kThreads];
    const uint32_t c = blockIdx.x;
    const uint32_t first = a.tab.tile_start[c], end = a.tab.tile_start[c + 1];
    const uint32_t nt = end - first;
    const uint32_t per = (nt + kThreads - 1) / kThreads;
    const uint32_t b = first + threadIdx.x * per;
    uint32_t sum = 0;
    for (uint32_t i = 0; i < per; ++i)
        if (b + i < end) sum += (uint32_t)a.tile_state[b + i];
    s_part[threadIdx.x] = sum;
    __syncthreads();
    uint32_t run = 0;
    for (uint32_t i = 0; i < threadIdx.x; ++i) run += s_part[i];
    for (uint32_t i = 0; i < per; ++i)
        if (b + i < end) {
            const uint32_t v = (uint32_t)a.tile_state[b + i];
            a.tile_state[b + i] = run;
            run += v;
        }
}

template <int DT, bool FAST>
__device__ __forceinline__ bool decode_group(const uint8_t* __restrict__ slot, uint8_t* __restrict__ cout,
                                             const SlotLayout& L, uint64_t n, uint64_t n_esc, uint64_t gstart,
                                             uint32_t e0, uint32_t lane)
{
    const uint64_t e = gstart + lane * kLaneElems;
    uint2 sm = make_uint2(0, 0);
    if (FAST || e < pad128(n)) sm = *reinterpret_cast<const uint2*>(slot + L.sm + e);
    const uint64_t pb = e >> 3;
    uint32_t b0 = 0, b1 = 0, b2 = 0;
    if (FAST || pb < L.plane_bytes) {
        b0 = slot[L.p0 + pb];
        b1 = slot[L.p0 + L.plane_bytes + pb];
        b2 = slot[L.p0 + 2 * L.plane_bytes + pb];
    }
    uint4 lo = make_uint4(0, 0, 0, 0);
    if (DT == ZIPCCL_FP32) {
        if (FAST || 2 * e < pad128(2 * n)) lo = *reinterpret_cast<const uint4*>(slot + L.lo + 2 * e);
    }
    const uint32_t base = reinterpret_cast<const uint32_t*>(slot + L.idx)[gstart / kGroup];
    uint32_t vmask = 0xFFu;
    if (!FAST) vmask = e >= n ? 0u : (n - e >= 8 ? 0xFFu : ((1u << (uint32_t)(n - e)) - 1u));
    const uint32_t m = ~(b0 | b1 | b2) & vmask;    /* code 0 = zero-point; tail bits are not */
    const uint32_t cnt = __popc(m);
    const uint32_t inc = wave_incl_scan(cnt, lane);
    uint64_t pos = (uint64_t)base + (inc - cnt);
    const uint8_t* __restrict__ esc = slot + L.esc;
    bool bad = false;
    uint32_t hp[4] = {0, 0, 0, 0};
    const uint32_t smw[2] = {sm.x, sm.y};
#pragma unroll
    for (int j = 0; j < 8; ++j) {
        const uint32_t code = ((b0 >> j) & 1u) | (((b1 >> j) & 1u) << 1) | (((b2 >> j) & 1u) << 2);
        uint32_t E = e0 + code - 1u;
        if ((m >> j) & 1u) {
            if (pos < n_esc) E = esc[pos]; else { bad = true; E = 0; }
            ++pos;
        }
        const uint32_t s = (smw[j >> 2] >> (8 * (j & 3))) & 0xFFu;
        const uint32_t h = ((s & 0x80u) << 8) | ((E & 0xFFu) << 7) | (s & 0x7Fu);
        hp[j >> 1] |= h << (16 * (j & 1));
    }
    const uint32_t low[4] = {lo.x, lo.y, lo.z, lo.w};
    if (FAST) {
        if (DT == ZIPCCL_BF16) {
            *reinterpret_cast<uint4*>(cout + e * 2) = make_uint4(hp[0], hp[1], hp[2], hp[3]);
        } else {
            uint32_t x[8];
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                x[2 * k] = (hp[k] << 16) | (low[k] & 0xFFFFu);
                x[2 * k + 1] = (hp[k] & 0xFFFF0000u) | (low[k] >> 16);
            }
            *reinterpret_cast<uint4*>(cout + e * 4) = make_uint4(x[0], x[1], x[2], x[3]);
            *reinterpret_cast<uint4*>(cout + e * 4 + 16) = make_uint4(x[4], x[5], x[6], x[7]);
        }
    } else {
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            if ((vmask >> j) & 1u) {
                const uint32_t h = (hp[j >> 1] >> (16 * (j & 1))) & 0xFFFFu;
                if (DT == ZIPCCL_BF16) {
                    *reinterpret_cast<uint16_t*>(cout + (e + j) * 2) = (uint16_t)h;
                } else {
                    const uint32_t l = (low[j >> 1] >> (16 * (j & 1))) & 0xFFFFu;
                    *reinterpret_cast<uint32_t*>(cout + (e + j) * 4) = (h << 16) | l;
                }
            }
        }
    }
    return bad;
}

template <int DT>
__global__ __launch_bounds__(kThreads) void k_decompress(const DecompressArgs a)
{
    constexpr uint32_t ES = DT == ZIPCCL_BF16 ? 2u : 4u;
    const uint32_t t = blockIdx.x;
    const uint32_t c = find_chunk(a.tab, t);
    const uint64_t n = a.tab.elem_off[c + 1] - a.tab.elem_off[c];
    const uint64_t ts = (uint64_t)(t - a.tab.tile_start[c]) * kTile;
    const uint8_t* __restrict__ slot = a.comp + a.tab.slot_off[c];
    uint8_t* __restrict__ cout = a.out + a.tab.elem_off[c] * ES;
    const SlotLayout L = slot_layout(n, DT);

    /* header check: the static part is readable (the host checked it), the rest must match */
    const uint32_t* hw = reinterpret_cast<const uint32_t*>(slot);
    const uint64_t n_hdr = (uint64_t)hw[4] | ((uint64_t)hw[5] << 32);
    const uint64_t n_esc = (uint64_t)hw[6] | ((uint64_t)hw[7] << 32);
    const uint64_t cbytes = (uint64_t)hw[8] | ((uint64_t)hw[9] << 32);
    const uint32_t dec_lo = hw[10], dec_hi = hw[11];
    const uint32_t e0 = (dec_lo >> 8) & 0xFFu;
    bool ok = hw[0] == kMagic && hw[1] == kVersion && hw[2] == (uint32_t)DT && hw[3] == kGroup;
    ok = ok && n_hdr == n && n_esc <= n && cbytes == L.esc + pad128(n_esc);
    ok = ok && a.tab.slot_off[c] + cbytes <= a.comp_capacity;
    ok = ok && e0 <= 249u && (dec_lo >> 8) == (e0 | ((e0 + 1u) << 8) | ((e0 + 2u) << 16)) &&
         dec_hi == ((e0 + 3u) | ((e0 + 4u) << 8) | ((e0 + 5u) << 16) | ((e0 + 6u) << 24));
    if (!ok) {
        if (threadIdx.x == 0 && a.status) atomicOr(a.status, (uint32_t)ZIPCCL_ERR_CORRUPT);
        return;
    }

    const bool fast = (ts + kTile <= n) && ((reinterpret_cast<uintptr_t>(cout) & 15u) == 0);
    const uint32_t lane = lane_id();
    const uint32_t wave = threadIdx.x >> 6;
    bool bad = false;
    if (fast) {
#pragma unroll
        for (uint32_t u = 0; u < kGroupsPerWave; ++u) {
            const uint64_t gstart = ts + (uint64_t)(u * kWavesPerBlock + wave) * kGroup;
            bad |= decode_group<DT, true>(slot, cout, L, n, n_esc, gstart, e0, lane);
        }
    } else {
        for (uint32_t u = 0; u < kGroupsPerWave; ++u) {
            const uint64_t gstart = ts + (uint64_t)(u * kWavesPerBlock + wave) * kGroup;
            if (gstart < n) bad |= decode_group<DT, false>(slot, cout, L, n, n_esc, gstart, e0, lane);
        }
    }
    if (bad && a.status) atomicOr(a.status, (uint32_t)ZIPCCL_ERR_CORRUPT);
}

__global__ __launch_bounds__(kThreads) void k_fill_zero(uint64_t* p, uint64_t n_words)
{
    const uint64_t i = (uint64_t)blockIdx.x * kThreads + threadIdx.x;
    if (i < n_words) p[i] = 0;
}

} // namespace

int launch_fill_zero(void* d_ptr, uint64_t bytes, void* stream)
{
    const uint64_t words = (bytes + 7) / 8;
    if (words == 0) return (int)hipSuccess;
    const uint32_t blocks = (uint32_t)((words + kThreads - 1) / kThreads);
    hipLaunchKernelGGL(k_fill_zero, dim3(blocks), dim3(kThreads), 0, (hipStream_t)stream,
                       reinterpret_cast<uint64_t*>(d_ptr), words);
    return (int)hipGetLastError();
}

int launch_compress(int dt, int mode, const CompressArgs& a, uint32_t n_tiles, void* stream)
{
    const dim3 grid(n_tiles), block(kThreads);
    hipStream_t s = (hipStream_t)stream;
#define ZIPCCL_LAUNCH(DT, MODE) hipLaunchKernelGGL((k_compress<DT, MODE>), grid, block, 0, s, a)
    if (dt == ZIPCCL_BF16) {
        if (mode == kModeCount) ZIPCCL_LAUNCH(ZIPCCL_BF16, kModeCount);
        else if (mode == kModeEmit) ZIPCCL_LAUNCH(ZIPCCL_BF16, kModeEmit);
        else ZIPCCL_LAUNCH(ZIPCCL_BF16, kModeFused);
    } else {
        if (mode == kModeCount) ZIPCCL_LAUNCH(ZIPCCL_FP32, kModeCount);
        else if (mode == kModeEmit) ZIPCCL_LAUNCH(ZIPCCL_FP32, kModeEmit);
        else ZIPCCL_LAUNCH(ZIPCCL_FP32, kModeFused);
    }
#undef ZIPCCL_LAUNCH
    return (int)hipGetLastError();
}

int launch_tile_scan(const CompressArgs& a, void* stream)
{
    hipLaunchKernelGGL(k_tile_scan, dim3(a.tab.n_chunks), dim3(kThreads), 0, (hipStream_t)stream, a);
    return (int)hipGetLastError();
}

int launch_decompress(int dt, const DecompressArgs& a, uint32_t n_tiles, void* stream)
{
    const dim3 grid(n_tiles), block(kThreads);
    if (dt == ZIPCCL_BF16)
        hipLaunchKernelGGL((k_decompress<ZIPCCL_BF16>), grid, block, 0, (hipStream_t)stream, a);
    else
        hipLaunchKernelGGL((k_decompress<ZIPCCL_FP32>), grid, block, 0, (hipStream_t)stream, a);
    return (int)hipGetLastError();
}

} // namespace zipccl
