// tq_stats: the reductions the parameter design of arXiv 2402.01798 consumes -- a
// log-spaced histogram of |g| per bucket (the empirical density behind Q_U(alpha) of
// Sec. IV-A and the integral of p^(1/3) of Sec. IV-B), max|g|, the NaN/Inf count and, for a
// caller-fixed g_min, the two terms of the tail-index estimator of Sec. V,
//   gamma = 1 + n_tail / sum_j ln(|g_j| / g_min).
//
// One read pass.  Each workgroup histograms a chunk of one bucket into replicated LDS
// histograms (heavy-tailed data puts most lanes into a handful of bins; replicas spread the
// same-address atomics) and merges the non-empty bins into the caller's record with integer
// atomics, so the counts do not depend on scheduling.
#include "tq_device.h"

namespace tq {

constexpr int kStatsReplicas = 8;
constexpr int kStatsStride = 929;            // >= TQ_NBINS and = 1 mod 32: replicas fall in different banks
constexpr int kStatsChunk = 8 * kTile;       // elements per workgroup (16384)
constexpr int kBinBias = 1391;               // 16 * (biased exponent of 2^-40) - 1

__global__ __launch_bounds__(kBlock) void tq_stats_init_kernel(tq_stats_t* stats, uint64_t d,
                                                               uint64_t bucket_elems, float g_min)
{
    tq_stats_t* S = stats + blockIdx.x;
    uint32_t* w = reinterpret_cast<uint32_t*>(S);
    for (uint32_t i = threadIdx.x; i < sizeof(tq_stats_t) / 4; i += kBlock) w[i] = 0u;
    __syncthreads();
    if (threadIdx.x == 0) {
        const uint64_t lo = (uint64_t)blockIdx.x * bucket_elems;
        const uint64_t hi = lo + bucket_elems < d ? lo + bucket_elems : d;
        S->n = hi - lo;
        S->g_min = g_min > 0.0f ? g_min : 0.0f;
    }
}

template <typename T>
__device__ __forceinline__ T wave_reduce_add(T v)
{
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, 64);
    return v;
}

__device__ __forceinline__ uint32_t wave_reduce_max(uint32_t v)
{
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) {
        const uint32_t o = __shfl_xor(v, off, 64);
        v = o > v ? o : v;
    }
    return v;
}

template <int DTYPE>
__global__ __launch_bounds__(kBlock) void tq_stats_kernel(const void* __restrict__ g, uint64_t d,
                                                          uint64_t bucket_elems, uint32_t chunks_per_bucket,
                                                          float g_min, tq_stats_t* __restrict__ stats)
{
    __shared__ uint32_t hist[kStatsReplicas * kStatsStride];
    for (int i = threadIdx.x; i < kStatsReplicas * kStatsStride; i += kBlock) hist[i] = 0u;
    __syncthreads();

    const uint32_t bucket = blockIdx.x / chunks_per_bucket;
    const uint32_t chunk = blockIdx.x - bucket * chunks_per_bucket;
    const uint64_t bstart = (uint64_t)bucket * bucket_elems;
    const uint64_t bend = bstart + bucket_elems < d ? bstart + bucket_elems : d;
    const uint64_t cstart = bstart + (uint64_t)chunk * kStatsChunk;
    const uint64_t cend = cstart + kStatsChunk < bend ? cstart + kStatsChunk : bend;

    uint32_t* my_hist = hist + (threadIdx.x & (kStatsReplicas - 1)) * kStatsStride;
    const bool want_tail = g_min > 0.0f;
    const uint32_t gmin_bits = __float_as_uint(g_min);
    uint32_t amax_bits = 0u, nonfinite = 0u, n_tail = 0u;
    int32_t exp_sum = 0;          // sum of unbiased exponents of the tail elements
    double log2m_sum = 0.0;       // sum of log2(mantissa in [1,2)) of the tail elements

    // One finite-or-not magnitude into the lane's running statistics.
    auto take = [&](uint32_t raw) {
        const uint32_t a = raw & 0x7FFFFFFFu;                          // |g| as an ordered integer
        if (a >= 0x7F800000u) { ++nonfinite; return; }                 // Inf or NaN
        int32_t idx = (int32_t)(a >> 19) - kBinBias;
        idx = idx < 0 ? 0 : (idx > TQ_NBINS - 1 ? TQ_NBINS - 1 : idx);
        atomicAdd(&my_hist[idx], 1u);
        amax_bits = a > amax_bits ? a : amax_bits;
        if (want_tail && a > gmin_bits) {                              // g_min >= 2^-40: a is normal
            ++n_tail;
            exp_sum += (int32_t)(a >> 23) - 127;
            log2m_sum += (double)__log2f(__uint_as_float((a & 0x007FFFFFu) | 0x3F800000u));
        }
    };

    for (uint64_t e0 = cstart + (uint64_t)threadIdx.x * kGroup; e0 < cend; e0 += kTile) {
        if (e0 + kGroup <= cend) {
            uint32_t bits[8];
            if constexpr (DTYPE == TQ_F32) {
                const uint4* p = reinterpret_cast<const uint4*>(static_cast<const float*>(g) + e0);
                const uint4 a = p[0], b = p[1];
                bits[0] = a.x; bits[1] = a.y; bits[2] = a.z; bits[3] = a.w;
                bits[4] = b.x; bits[5] = b.y; bits[6] = b.z; bits[7] = b.w;
            } else {
                const uint4 v = *reinterpret_cast<const uint4*>(static_cast<const uint16_t*>(g) + e0);
                const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
                for (int i = 0; i < 4; ++i) { bits[2 * i] = w[i] << 16; bits[2 * i + 1] = w[i] & 0xFFFF0000u; }
            }
#pragma unroll
            for (int j = 0; j < 8; ++j) take(bits[j]);
        } else {                                                       // ragged end of the tensor
            for (uint64_t e = e0; e < cend; ++e) {
                if constexpr (DTYPE == TQ_F32) take(static_cast<const uint32_t*>(g)[e]);
                else take((uint32_t) static_cast<const uint16_t*>(g)[e] << 16);
            }
        }
    }
    __syncthreads();

    tq_stats_t* S = stats + bucket;
    for (int b = threadIdx.x; b < TQ_NBINS; b += kBlock) {
        uint32_t total = 0u;
#pragma unroll
        for (int r = 0; r < kStatsReplicas; ++r) total += hist[r * kStatsStride + b];
        if (total) atomicAdd(&S->hist[b], total);
    }

    amax_bits = wave_reduce_max(amax_bits);
    nonfinite = wave_reduce_add(nonfinite);
    if ((threadIdx.x & 63) == 0) {
        if (amax_bits) atomicMax(reinterpret_cast<uint32_t*>(&S->absmax), amax_bits);  // non-negative floats order as integers
        if (nonfinite) atomicAdd(&S->n_nonfinite, nonfinite);
    }
    if (want_tail) {
        n_tail = wave_reduce_add(n_tail);
        // ln(a / g_min) = ln2 * (exponent + log2 mantissa) - ln g_min, summed per wavefront
        double part = (double)exp_sum + log2m_sum;
        part = wave_reduce_add(part);
        if ((threadIdx.x & 63) == 0 && n_tail) {
            const double sum_log = 0.6931471805599453 * part - (double)n_tail * log((double)g_min);
            atomicAdd(reinterpret_cast<unsigned long long*>(&S->n_tail), (unsigned long long)n_tail);
            atomicAdd(&S->sum_log_tail, sum_log);
        }
    }
}

}  // namespace tq

// Host side of tq_stats after the argument checks of the C entry point.
hipError_t tq_launch_stats(const void* g, int dtype, uint64_t d, uint64_t bucket_elems, float g_min,
                           tq_stats_t* stats, hipStream_t st)
{
    const uint64_t be = bucket_elems ? bucket_elems : d;
    const uint64_t nb = (d + be - 1) / be;
    const uint64_t cpb = (be + tq::kStatsChunk - 1) / tq::kStatsChunk;
    const uint64_t nblocks = nb * cpb;
    if (nblocks == 0 || nblocks > 0x7FFFFFFFull) return hipErrorInvalidValue;
    hipLaunchKernelGGL(tq::tq_stats_init_kernel, dim3((unsigned)nb), dim3(tq::kBlock), 0, st, stats, d, be, g_min);
    hipError_t err = hipGetLastError();
    if (err != hipSuccess) return err;
    if (dtype == TQ_F32)
        hipLaunchKernelGGL((tq::tq_stats_kernel<TQ_F32>), dim3((unsigned)nblocks), dim3(tq::kBlock), 0, st, g, d, be,
                           (uint32_t)cpb, g_min, stats);
    else
        hipLaunchKernelGGL((tq::tq_stats_kernel<TQ_BF16>), dim3((unsigned)nblocks), dim3(tq::kBlock), 0, st, g, d,
                           be, (uint32_t)cpb, g_min, stats);
    return hipGetLastError();
}
