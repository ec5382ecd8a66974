/*
 * Auxiliary kernels of libzipccl.so: the sigma estimates / table choice on the device (paper section 4.1).
 */
#include "zipccl_device.h"

namespace zipccl {
namespace {

/* The table for a given sigma by Eq.5 / Eq.2 (erf in FP64), exactly as the host builder does; a sigma that is
 * not positive and finite selects the lowest window.  One thread. */
__device__ void table_from_sigma(double sigma, uint8_t* table, double* sigma_out)
{
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
    table[0] = 0;
    for (uint32_t k = 1; k <= 7; ++k) table[k] = (uint8_t)(e0 + k - 1);
    if (sigma_out) *sigma_out = sigma;
}

/* Value of element i as a double (bf16 widened exactly). */
template <int DT>
__device__ __forceinline__ double value_at(const uint8_t* in, uint64_t i)
{
    uint32_t bits;
    if (DT == ZIPCCL_BF16) bits = (uint32_t)(*reinterpret_cast<const uint16_t*>(in + i * 2)) << 16;
    else bits = *reinterpret_cast<const uint32_t*>(in + i * 4);
    return (double)__uint_as_float(bits);
}

/*
 * sigma of a tensor as the paper takes it (section 4.1: torch.std = unbiased sample standard
 * deviation), in FP64.  Sums are taken of d = x - pivot, the pivot being the tensor's first value (0 if that
 * is not finite): sum d^2 - (sum d)^2 / N then cancels only as far as the pivot is from the mean, not as far
 * as the mean is from zero.  Every workgroup writes its partial sums; k_estimate_finish adds the partials in a
 * fixed order, forms sigma, and picks the window (table_from_sigma).
 */
template <int DT>
__global__ __launch_bounds__(kThreads) void k_moments(const MomentArgs a)
{
    constexpr uint32_t ES = DT == ZIPCCL_BF16 ? 2u : 4u;
    constexpr uint32_t PER16 = 16u / ES;               /* values per 16-byte load */
    __shared__ double s_sum[kWavesPerBlock], s_sq[kWavesPerBlock];
    double sum = 0.0, sq = 0.0;
    double pivot = a.n ? value_at<DT>(a.in, 0) : 0.0;
    if (!(fabs(pivot) < __longlong_as_double(0x7FF0000000000000ll))) pivot = 0.0;
    const bool aligned = (reinterpret_cast<uintptr_t>(a.in) & 15u) == 0;
    const uint64_t n16 = aligned ? a.n / PER16 : 0;    /* 16-byte pieces handled with vector loads */
    for (uint64_t i = (uint64_t)blockIdx.x * kThreads + threadIdx.x; i < n16; i += (uint64_t)gridDim.x * kThreads) {
        const u32x4 v = ld_stream<u32x4>(a.in + i * 16);
        const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            if (DT == ZIPCCL_BF16) {
                const double x0 = (double)__uint_as_float(w[k] << 16) - pivot, x1 = (double)__uint_as_float(w[k] & 0xFFFF0000u) - pivot;
                sum += x0; sq += x0 * x0;
                sum += x1; sq += x1 * x1;
            } else {
                const double x = (double)__uint_as_float(w[k]) - pivot;
                sum += x; sq += x * x;
            }
        }
    }
    /* the tail (and everything, for a misaligned tensor) element by element */
    for (uint64_t i = n16 * PER16 + (uint64_t)blockIdx.x * kThreads + threadIdx.x; i < a.n; i += (uint64_t)gridDim.x * kThreads) {
        const double x = value_at<DT>(a.in, i) - pivot;
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
        const double var = (s_sq[0] - s_sum[0] * s_sum[0] / N) / (N - 1.0);      /* sums of x - pivot */
        sigma = sqrt(var > 0.0 ? var : (var == var ? 0.0 : var));
    }
    table_from_sigma(sigma, a.table, a.sigma);
}

/*
 * Robust sigma (for Eq.5 / Eq.2 when the tensor is not the zero-mean Gaussian of section 4.1: outlier
 * channels, LayerNorm gains among matrix weights): the median of |w| over Phi^-1(3/4).  The median is taken
 * over the 15-bit magnitudes of the values' high 16-bit words, so it is a count: k_magnitude_hist builds the
 * histogram of all 32768 magnitudes (about one workgroup per compute unit, the whole histogram in its LDS, one
 * LDS atomic per value; nonzero bins are added to the chunk's 64-bit histogram in the workspace, which
 * k_clear_hist zeroed), k_robust_finish finds the bin of rank (K - 1) / 2 among the K magnitudes that are neither
 * zero nor Inf/NaN.  Integer work until the final division: the result does not depend on any order.
 * Both take several chunks at once (one histogram and one table per chunk); the whole tensor is one chunk.
 */
constexpr uint32_t kMagBins = 32768;
constexpr uint32_t kHistThreads = 1024;

/* One workgroup per chunk's histogram, 64 stores per thread: with the same bytes spread over 16 or 32 times as many
 * workgroups the kernel took 5 us longer for 64 histograms (the launch, not the memory, was its limit). */
constexpr uint32_t kClearThreads = 256, kClearPer = 64;  /* 16-byte stores per thread */

__global__ __launch_bounds__(kClearThreads) void k_clear_hist(unsigned long long* hist)
{
    /* grid = chunks (the workspace is 8-byte aligned: the 16-byte stores are issued at that alignment) */
    u32x4_a4* const p = reinterpret_cast<u32x4_a4*>(hist) + (uint64_t)blockIdx.x * (kClearPer * kClearThreads) + threadIdx.x;
    const u32x4 zero = {0u, 0u, 0u, 0u};
#pragma unroll
    for (uint32_t k = 0; k < kClearPer; ++k) p[k * kClearThreads] = zero;
}

template <int DT>
__global__ __launch_bounds__(kHistThreads) void k_magnitude_hist(const HistArgs a)
{
    constexpr uint32_t ES = DT == ZIPCCL_BF16 ? 2u : 4u;
    constexpr uint32_t PER16 = 16u / ES;
    __shared__ uint32_t s_hist[kMagBins];                  /* 128 KiB */
    for (uint32_t i = threadIdx.x; i < kMagBins; i += kHistThreads) s_hist[i] = 0u;
    __syncthreads();
    /* grid = (workgroups per chunk, chunks); a chunk starts at some element of the tensor: the values in front of
       its first 16-byte boundary and behind its last one are taken one by one, the rest in 16-byte pieces */
    const uint32_t c = blockIdx.y;
    const uint8_t* __restrict__ in = a.in + a.tab.elem_off[c] * ES;
    const uint64_t n = a.tab.elem_off[c + 1] - a.tab.elem_off[c];
    const uint64_t head = min(n, (uint64_t)(((16u - (uint32_t)(reinterpret_cast<uintptr_t>(in) & 15u)) & 15u) / ES));
    const uint64_t n16 = (n - head) / PER16;
    const uint8_t* __restrict__ mid = in + head * ES;
    const uint64_t stride = (uint64_t)gridDim.x * kHistThreads;
    auto count = [&](const u32x4& v) {
        const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            if (DT == ZIPCCL_BF16) atomicAdd(&s_hist[w[k] & 0x7FFFu], 1u);
            atomicAdd(&s_hist[(w[k] >> 16) & 0x7FFFu], 1u);
        }
    };
    auto count_one = [&](uint64_t e) {
        const uint32_t hi = DT == ZIPCCL_BF16 ? *reinterpret_cast<const uint16_t*>(in + e * 2)
                                              : *reinterpret_cast<const uint32_t*>(in + e * 4) >> 16;
        atomicAdd(&s_hist[hi & 0x7FFFu], 1u);
    };
    uint64_t i = (uint64_t)blockIdx.x * kHistThreads + threadIdx.x;
    for (; i + 3 * stride < n16; i += 4 * stride) {           /* four loads in flight per thread */
        u32x4 v[4];
#pragma unroll
        for (uint32_t k = 0; k < 4; ++k) v[k] = ld_stream<u32x4>(mid + (i + k * stride) * 16);
#pragma unroll
        for (uint32_t k = 0; k < 4; ++k) count(v[k]);
    }
    for (; i < n16; i += stride) count(ld_stream<u32x4>(mid + i * 16));
    if (blockIdx.x == 0) {                                    /* head and tail: fewer than 16 bytes each */
        if (threadIdx.x < head) count_one(threadIdx.x);
        const uint64_t done = head + n16 * PER16;
        if (done + threadIdx.x < n) count_one(done + threadIdx.x);
    }
    __syncthreads();
    unsigned long long* __restrict__ hist = a.hist + (uint64_t)c * kMagBins;
    for (uint32_t b = threadIdx.x; b < kMagBins; b += kHistThreads) {
        const uint32_t cnt = s_hist[b];
        if (cnt) atomicAdd(&hist[b], (unsigned long long)cnt);
    }
}

/*
 * The same histogram over a sample of the chunk: its groups of 512 values are cut into blocks of S consecutive
 * groups (S = a.sample_stride, a power of two) and one group is taken from every block, at position
 * ((k * 2654435761 mod 2^32) >> 16) mod S inside block k (Knuth's multiplicative hash: the position varies from
 * block to block, so the sample does not alias with the periods of the tensor itself, rows of 8 or 16 groups
 * say).  A wave takes a group at a time, 8 values per lane, several groups in flight; a group that is cut short by
 * the chunk's end, and every group of a chunk that does not start on a 16-byte boundary, is read value by value.
 */
template <int DT, uint32_t NF>   /* NF groups in flight per wave */
__device__ __forceinline__ void sample_into_lds(uint32_t* s_hist, const uint8_t* __restrict__ in, uint64_t n, uint32_t S,
                                                uint32_t first_wave, uint32_t n_waves)
{
    constexpr uint32_t ES = DT == ZIPCCL_BF16 ? 2u : 4u;
    constexpr uint32_t NV = DT == ZIPCCL_BF16 ? 1u : 2u;    /* 16-byte pieces per lane and group */
    const uint64_t ng = (n + kGroup - 1) / kGroup;           /* at most 2^23 */
    const uint32_t n_blk = (uint32_t)((ng + S - 1) / S);
    /* vector loads need a chunk that starts on a 16-byte boundary; then group 0, if whole, is an address that is
       always safe to load from */
    const bool vec = (reinterpret_cast<uintptr_t>(in) & 15u) == 0 && n >= kGroup;
    const uint32_t lane = threadIdx.x & 63u;
    auto one_by_one = [&](uint64_t first) {
        for (uint32_t j = 0; j < kLaneElems; ++j) {
            const uint64_t e = first + lane * kLaneElems + j;
            if (e < n) {
                const uint32_t hi = DT == ZIPCCL_BF16 ? *reinterpret_cast<const uint16_t*>(in + e * 2)
                                                      : *reinterpret_cast<const uint32_t*>(in + e * 4) >> 16;
                atomicAdd(&s_hist[hi & 0x7FFFu], 1u);
            }
        }
    };
    for (uint32_t k0 = first_wave; k0 < n_blk; k0 += NF * n_waves) {
        u32x4 v[NF][NV];
        uint64_t first[NF];
        bool some[NF], whole[NF];
        /* the loads of all NF groups go out back to back: no branch between them (a group that is not there, or
           not whole, loads group 0 instead and is not counted from it) */
#pragma unroll
        for (uint32_t u = 0; u < NF; ++u) {
            const uint32_t k = k0 + u * n_waves;
            const uint64_t g = (uint64_t)k * S + (((k * 2654435761u) >> 16) & (S - 1u));
            first[u] = g * kGroup;
            some[u] = k < n_blk && g < ng;
            whole[u] = some[u] && vec && first[u] + kGroup <= n;
        }
        if (vec) {
#pragma unroll
            for (uint32_t u = 0; u < NF; ++u) {
                const uint64_t from = whole[u] ? first[u] : 0ull;
#pragma unroll
                for (uint32_t q = 0; q < NV; ++q)
                    v[u][q] = ld_stream<u32x4>(in + (from + lane * kLaneElems) * ES + 16u * q);
            }
        }
#pragma unroll
        for (uint32_t u = 0; u < NF; ++u) {
            if (whole[u]) {
#pragma unroll
                for (uint32_t q = 0; q < NV; ++q) {
                    const uint32_t w[4] = {v[u][q].x, v[u][q].y, v[u][q].z, v[u][q].w};
#pragma unroll
                    for (int j = 0; j < 4; ++j) {
                        if (DT == ZIPCCL_BF16) atomicAdd(&s_hist[w[j] & 0x7FFFu], 1u);
                        atomicAdd(&s_hist[(w[j] >> 16) & 0x7FFFu], 1u);
                    }
                }
            }
        }
        /* a group cut short by the chunk's end, or any group of a chunk that is only element-aligned */
#pragma unroll
        for (uint32_t u = 0; u < NF; ++u)
            if (some[u] && !whole[u]) one_by_one(first[u]);
    }
}

template <int DT>
__global__ __launch_bounds__(kHistThreads) void k_magnitude_hist_sampled(const HistArgs a)
{
    constexpr uint32_t ES = DT == ZIPCCL_BF16 ? 2u : 4u;
    __shared__ uint32_t s_hist[kMagBins];                  /* 128 KiB */
    for (uint32_t i = threadIdx.x; i < kMagBins; i += kHistThreads) s_hist[i] = 0u;
    __syncthreads();
    /* grid = (workgroups per chunk, chunks) */
    const uint32_t c = blockIdx.y;
    const uint32_t wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    sample_into_lds<DT, 4>(s_hist, a.in + a.tab.elem_off[c] * ES, a.tab.elem_off[c + 1] - a.tab.elem_off[c], a.sample_stride,
                           blockIdx.x * (kHistThreads / 64u) + wave, gridDim.x * (kHistThreads / 64u));
    __syncthreads();
    unsigned long long* __restrict__ hist = a.hist + (uint64_t)c * kMagBins;
    for (uint32_t b = threadIdx.x; b < kMagBins; b += kHistThreads) {
        const uint32_t cnt = s_hist[b];
        if (cnt) atomicAdd(&hist[b], (unsigned long long)cnt);
    }
}

/*
 * A chunk whose sample is small enough for one workgroup (at most kFusedGroups groups): histogram, rank and table
 * in one kernel, nothing outside LDS, no histogram in the workspace to clear and no second or third launch.
 * grid = chunks.  Thread t answers for bins [32 t, 32 t + 32) as in k_robust_finish; a chunk holds fewer than 2^32
 * values, so 32-bit counts do.
 */
template <int DT>
__global__ __launch_bounds__(kHistThreads) void k_robust_chunk_fused(const HistArgs a)
{
    constexpr uint32_t ES = DT == ZIPCCL_BF16 ? 2u : 4u;
    constexpr uint32_t kPer = kMagBins / kHistThreads;       /* 32 */
    constexpr uint32_t kWaves = kHistThreads / 64;
    constexpr uint32_t kFirstNonFinite = 0x7F80u;
    __shared__ uint32_t s_hist[kMagBins];                  /* 128 KiB */
    __shared__ uint32_t s_wave[kWaves];
    for (uint32_t i = threadIdx.x; i < kMagBins; i += kHistThreads) s_hist[i] = 0u;
    __syncthreads();
    const uint32_t c = blockIdx.x;
    const uint32_t t = threadIdx.x, lane = t & 63u;
    const uint32_t wave = __builtin_amdgcn_readfirstlane(t >> 6);
    /* one workgroup per chunk has the chunk's whole latency to hide: eight groups in flight per wave */
    sample_into_lds<DT, 8>(s_hist, a.in + a.tab.elem_off[c] * ES, a.tab.elem_off[c + 1] - a.tab.elem_off[c], a.sample_stride,
                           wave, kWaves);
    __syncthreads();
    uint8_t* const table = a.table + 8u * c;
    double* const sigma = a.sigma ? a.sigma + c : nullptr;
    auto counted = [&](uint32_t b) { return (b != 0u && b < kFirstNonFinite) ? s_hist[b] : 0u; };
    uint32_t mine = 0;
#pragma unroll
    for (uint32_t k = 0; k < kPer; ++k) mine += counted(t * kPer + ((k + t) & (kPer - 1u)));   /* rotated: no bank conflicts */
    const uint32_t inc = wave_incl_scan(mine);
    if (lane == 63u) s_wave[wave] = inc;
    __syncthreads();
    uint32_t before = 0, total = 0;
    for (uint32_t w = 0; w < kWaves; ++w) {
        const uint32_t cw = s_wave[w];
        before += w < wave ? cw : 0u;
        total += cw;
    }
    if (total == 0u) {
        if (t == 0) table_from_sigma(__longlong_as_double(0x7FF8000000000000ll), table, sigma);
        return;
    }
    const uint32_t rank = (total - 1u) / 2u, excl = before + inc - mine;
    if (rank < excl || rank - excl >= mine) return;          /* exactly one thread holds the rank */
    uint32_t run = excl, bin = 0;
    bool found = false;
    for (uint32_t k = 0; k < kPer; ++k) {
        run += counted(t * kPer + k);
        if (!found && rank < run) { found = true; bin = t * kPer + k; }
    }
    const double med = (double)__uint_as_float(bin << 16);
    table_from_sigma(med / 0.6744897501960817, table, sigma);     /* Phi^-1(3/4) */
}

/* Inclusive prefix sum of 64-bit values over the 64 lanes of a wave, exact, without going through LDS: the four
 * 16-bit limbs are scanned separately with DPP (each limb sum stays below 2^22) and put together again.
 * (64-bit shuffles are two LDS permutes each, and a chain of several hundred of them took 20 us here.) */
__device__ __forceinline__ unsigned long long wave_incl_scan_u64(unsigned long long x)
{
    unsigned long long r = 0;
#pragma unroll
    for (uint32_t k = 0; k < 4; ++k)
        r += (unsigned long long)wave_incl_scan((uint32_t)(x >> (16 * k)) & 0xFFFFu) << (16 * k);
    return r;
}

/*
 * One workgroup per chunk.  Thread t answers for the 32 consecutive bins [32 t, 32 t + 32).  The 32768 counts are read
 * with coalesced loads (thread t holds bin 1024 r + t of every row r, all loads in flight together) and handed to their
 * owners through LDS, 4096 bins at a time; every thread sums its 32 bins, one scan over the 1024 sums finds the
 * thread that holds the rank, and that thread walks its bins.  Bins 0 (zero) and 0x7F80.. (Inf / NaN) do not count.
 */
__global__ __launch_bounds__(kHistThreads) void k_robust_finish(const HistArgs a)
{
    /* grid = chunks */
    const unsigned long long* __restrict__ hist = a.hist + (uint64_t)blockIdx.x * kMagBins;
    uint8_t* const table = a.table + 8u * blockIdx.x;
    double* const sigma = a.sigma ? a.sigma + blockIdx.x : nullptr;
    constexpr uint32_t kPer = kMagBins / kHistThreads;       /* 32 bins per thread, and rows of the coalesced read */
    constexpr uint32_t kWaves = kHistThreads / 64;           /* 16 */
    constexpr uint32_t kRound = 4096;                        /* bins handed over per round: 128 owners */
    constexpr uint32_t kFirstNonFinite = 0x7F80u;            /* magnitudes from here on are Inf / NaN */
    __shared__ unsigned long long s_buf[kRound + kRound / kPer];     /* one pad word per owner: bank-conflict relief */
    __shared__ unsigned long long s_wave[kWaves];
    const uint32_t t = threadIdx.x, lane = t & 63u, wave = t >> 6;
    unsigned long long v[kPer];
#pragma unroll
    for (uint32_t r = 0; r < kPer; ++r) {
        const uint32_t b = r * kHistThreads + t;
        v[r] = (b != 0u && b < kFirstNonFinite) ? hist[b] : 0ull;
    }
    unsigned long long mine = 0;
#pragma unroll
    for (uint32_t q = 0; q < kMagBins / kRound; ++q) {       /* 8 rounds; round q = bins [4096 q, 4096 q + 4096) */
#pragma unroll
        for (uint32_t j = 0; j < kRound / kHistThreads; ++j) {
            const uint32_t e = j * kHistThreads + t;         /* bin inside the round */
            s_buf[e + e / kPer] = v[q * (kRound / kHistThreads) + j];
        }
        __syncthreads();
        if (t / (kRound / kPer) == q) {
            const uint32_t o = (t % (kRound / kPer)) * (kPer + 1);
#pragma unroll
            for (uint32_t k = 0; k < kPer; ++k) mine += s_buf[o + k];
        }
        __syncthreads();
    }
    const unsigned long long inc = wave_incl_scan_u64(mine);
    if (lane == 63u) s_wave[wave] = inc;
    __syncthreads();
    unsigned long long before = 0, total = 0;
    for (uint32_t w = 0; w < kWaves; ++w) {
        const unsigned long long c = s_wave[w];
        before += w < wave ? c : 0ull;
        total += c;
    }
    if (total == 0ull) {
        if (t == 0) table_from_sigma(__longlong_as_double(0x7FF8000000000000ll), table, sigma);
        return;
    }
    const unsigned long long rank = (total - 1ull) / 2ull, excl = before + inc - mine;
    if (rank < excl || rank >= excl + mine) return;          /* exactly one thread holds the rank */
    unsigned long long c[kPer];
#pragma unroll
    for (uint32_t k = 0; k < kPer; ++k) {
        const uint32_t b = t * kPer + k;
        c[k] = (b != 0u && b < kFirstNonFinite) ? hist[b] : 0ull;
    }
    unsigned long long run = excl;
    uint32_t bin = 0;
    bool found = false;
#pragma unroll
    for (uint32_t k = 0; k < kPer; ++k) {
        run += c[k];
        if (!found && rank < run) { found = true; bin = t * kPer + k; }
    }
    const double med = (double)__uint_as_float(bin << 16);
    table_from_sigma(med / 0.6744897501960817, table, sigma);     /* Phi^-1(3/4) */
}

} // namespace

int launch_estimate(int dt, const MomentArgs& a, void* stream)
{
    hipStream_t s = (hipStream_t)stream;
    if (dt == ZIPCCL_BF16) hipLaunchKernelGGL((k_moments<ZIPCCL_BF16>), dim3(a.n_blocks), dim3(kThreads), 0, s, a);
    else hipLaunchKernelGGL((k_moments<ZIPCCL_FP32>), dim3(a.n_blocks), dim3(kThreads), 0, s, a);
    if (hipGetLastError() != hipSuccess) return 1;
    hipLaunchKernelGGL(k_estimate_finish, dim3(1), dim3(kThreads), 0, s, a);
    return (int)hipGetLastError();
}


int launch_clear_hist(unsigned long long* hist, uint32_t n_chunks, void* stream)
{
    hipLaunchKernelGGL(k_clear_hist, dim3(n_chunks * (kMagBins * 8u / (16u * kClearPer * kClearThreads))), dim3(kClearThreads), 0, (hipStream_t)stream, hist);
    return (int)hipGetLastError();
}

int launch_estimate_robust_fused(int dt, const HistArgs& a, void* stream)
{
    const dim3 grid(a.tab.n_chunks);
    if (dt == ZIPCCL_BF16) hipLaunchKernelGGL((k_robust_chunk_fused<ZIPCCL_BF16>), grid, dim3(kHistThreads), 0, (hipStream_t)stream, a);
    else hipLaunchKernelGGL((k_robust_chunk_fused<ZIPCCL_FP32>), grid, dim3(kHistThreads), 0, (hipStream_t)stream, a);
    return (int)hipGetLastError();
}

int launch_estimate_robust(int dt, const HistArgs& a, void* stream)
{
    hipStream_t s = (hipStream_t)stream;
    const dim3 grid(a.n_blocks, a.tab.n_chunks);
    if (a.sample_stride > 1u) {
        if (dt == ZIPCCL_BF16) hipLaunchKernelGGL((k_magnitude_hist_sampled<ZIPCCL_BF16>), grid, dim3(kHistThreads), 0, s, a);
        else hipLaunchKernelGGL((k_magnitude_hist_sampled<ZIPCCL_FP32>), grid, dim3(kHistThreads), 0, s, a);
    } else if (dt == ZIPCCL_BF16) hipLaunchKernelGGL((k_magnitude_hist<ZIPCCL_BF16>), grid, dim3(kHistThreads), 0, s, a);
    else hipLaunchKernelGGL((k_magnitude_hist<ZIPCCL_FP32>), grid, dim3(kHistThreads), 0, s, a);
    if (hipGetLastError() != hipSuccess) return 1;
    hipLaunchKernelGGL(k_robust_finish, dim3(a.tab.n_chunks), dim3(kHistThreads), 0, s, a);
    return (int)hipGetLastError();
}

} // namespace zipccl
