/*
 * Auxiliary kernels of libzipccl.so: the sigma estimate / table choice on the device (paper section 4.1)
 * and the plain-copy yardstick used by the benchmark.
 */
#include "zipccl_device.h"

namespace zipccl {
namespace {

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


} // namespace zipccl
