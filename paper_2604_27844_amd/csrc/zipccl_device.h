/*
 * Device helpers shared by the HIP kernels of libzipccl.so (gfx950, wave64): vector types, streaming
 * accesses, the byte-permute / bit-field primitives the SWAR code is written in, and DPP scans.
 */
#ifndef ZIPCCL_DEVICE_H
#define ZIPCCL_DEVICE_H

#include <hip/hip_runtime.h>

#include "zipccl_internal.h"

namespace zipccl {

typedef unsigned short us2 __attribute__((ext_vector_type(2)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

/* 16 bytes at an address that is only known to be 4-byte aligned: a chunk of the caller's tensor may start
 * at any element (the hardware takes multi-dword accesses at dword alignment; the type tells the compiler) */
typedef u32x4 u32x4_a4 __attribute__((aligned(4)));
typedef uint32_t u32x3 __attribute__((ext_vector_type(3)));
typedef u32x3 u32x3_a4 __attribute__((aligned(4)));

/* streaming accesses: every tensor byte is touched once, so keep it out of the way of the caches */
template <typename T>
__device__ __forceinline__ T ld_stream(const void* p) { return __builtin_nontemporal_load(static_cast<const T*>(p)); }
template <typename T>
__device__ __forceinline__ void st_stream(void* p, T v) { __builtin_nontemporal_store(v, static_cast<T*>(p)); }
__device__ __forceinline__ u32x4 ld_stream_a4(const void* p) { return __builtin_nontemporal_load(static_cast<const u32x4_a4*>(p)); }
__device__ __forceinline__ void st_stream_a4(void* p, u32x4 v) { __builtin_nontemporal_store(v, static_cast<u32x4_a4*>(p)); }

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


/* tiles of the largest chunk of a launch: the x extent of the (tile, chunk) grids */
inline uint32_t max_chunk_tiles(const ChunkTab& tab)
{
    uint32_t m = 1;
    for (uint32_t c = 0; c < tab.n_chunks; ++c) {
        const uint32_t nt = tab.tile_start[c + 1] - tab.tile_start[c];
        m = nt > m ? nt : m;
    }
    return m;
}

} // namespace zipccl
#endif
