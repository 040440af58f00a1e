// tq_stats: the reductions the parameter design of arXiv 2402.01798 consumes -- a
// log-spaced histogram of |g| per bucket (the empirical density behind Q_U(alpha) of
// Sec. IV-A and the integral of p^(1/3) of Sec. IV-B), max|g|, the NaN/Inf count and, for a
// caller-fixed g_min, the two terms of the tail-index estimator of Sec. V,
//   gamma = 1 + n_tail / sum_j ln(|g_j| / g_min).
//
// Two launches (one when the first kernel can write every record itself), no atomics on
// global memory (same-address atomics from many workgroups serialise at about 0.14 us each on
// this part):
//   1. each workgroup reads contiguous pieces of buckets once, histograms a piece into
//      replicated LDS histograms (heavy-tailed data puts most lanes into a handful of bins;
//      replicas spread the same-address LDS atomics) and writes the piece's counts either as
//      the bucket's finished record or to the caller's workspace as one contiguous row
//      (scattering them bin-major cost ten times their size in partial-line HBM writes).
//      Buckets of 32768 elements or more: tq_stats_balanced_kernel, the batch cut into equal
//      shares whatever the buckets are.  Smaller buckets: tq_stats_partial_kernel, a
//      workgroup per bucket or per slice of one.
//   2. a second kernel adds the rows of the buckets that were cut, with coalesced loads, and
//      combines max, counts and the log-sum.
// Counts are integers and the tail's log-sum travels as exact integer sums, so the result
// depends neither on scheduling nor on how the tensor was sliced or batched.
#include <atomic>
#include <type_traits>

#include "tq_device.h"

// Scratch of tq_stats_static: the partial histograms of the workgroups, held by the library in
// place of the caller's workspace, for callers that cannot allocate.  Every device the library
// runs on holds its own copy of the array until the process ends.  Host code never passes
// this name to a kernel or a copy: it is a host-side stand-in, and the device address comes
// from hipGetSymbolAddress (tq_stats_static_scratch below).
static __device__ __align__(256) unsigned char scratch[TQ_STATS_STATIC_SCRATCH_BYTES];

namespace tq {

constexpr int kStatsBlock = 512;                       // threads per workgroup of the partial kernel
constexpr int kStatsTile = kStatsBlock * kGroup;       // elements per workgroup pass (4096)
constexpr int kStatsReplicas = 8;
constexpr int kStatsStride = 929;                      // >= TQ_NBINS and = 1 mod 32: replicas in different banks
constexpr int kStatsMinSlice = 4 * kStatsTile;         // smallest slice worth a workgroup (16384 elements)
constexpr int kStatsMaxSlices = 256;                   // slices per bucket at most
constexpr int kStatsTargetGroups = 256;                // workgroups per tensor the workspace is sized for (one per CU)
constexpr int kStatsResidentGroups = 1024;             // workgroups that can run at the same time (4 per CU)
constexpr int kReduceBlock = 1024;                     // threads of the reduce kernel: 64 bins x 16 slice lanes
constexpr int kReduceBins = 64;
constexpr int kBinBias = 1391;                         // 16 * (biased exponent of 2^-40) - 1

// Per (bucket, slice).  The log-sum of the tail travels as two exact integer sums (ln(a/g_min)
// = ln2 (exponent + log2 mantissa) - ln g_min; the log2 of the mantissas is taken once per
// aligned group of 8 elements, of their product, and kept in 2^-28 fixed point), so the final
// value does not depend on how the tensor was cut into slices or batched.
struct StatsExtra {            // 32 bytes
    uint32_t absmax_bits;
    uint32_t n_nonfinite;
    unsigned long long n_tail;
    long long exp_sum;             // sum of unbiased exponents of the tail elements
    unsigned long long log2m_fix;  // sum over groups of log2(product of the tail mantissas) * 2^28
};

__host__ __device__ inline uint64_t stats_ws_hist_words(uint64_t nb, uint32_t slices)
{
    return nb * TQ_NBINS * (uint64_t)slices;
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

// One lane's group of 8 consecutive elements as it is loaded (32 bytes of fp32, 16 of bf16), and
// as fp32 bit patterns.  The two are separate so that nothing that needs the loaded value stands
// between a request and the work it is meant to overlap.
template <int DTYPE> struct RawGroup { uint4 q[DTYPE == TQ_F32 ? 2 : 1]; };

template <int DTYPE>
__device__ __forceinline__ void load_raw(const void* g, uint64_t e0, RawGroup<DTYPE>& r)
{
    if constexpr (DTYPE == TQ_F32) {
        const uint4* p = reinterpret_cast<const uint4*>(static_cast<const float*>(g) + e0);
        r.q[0] = p[0];
        r.q[1] = p[1];
    } else {
        r.q[0] = *reinterpret_cast<const uint4*>(static_cast<const uint16_t*>(g) + e0);
    }
}

template <int DTYPE>
__device__ __forceinline__ void raw_bits(const RawGroup<DTYPE>& r, uint32_t (&bits)[8])
{
    if constexpr (DTYPE == TQ_F32) {
        bits[0] = r.q[0].x; bits[1] = r.q[0].y; bits[2] = r.q[0].z; bits[3] = r.q[0].w;
        bits[4] = r.q[1].x; bits[5] = r.q[1].y; bits[6] = r.q[1].z; bits[7] = r.q[1].w;
    } else {
        const uint32_t w[4] = {r.q[0].x, r.q[0].y, r.q[0].z, r.q[0].w};
#pragma unroll
        for (int i = 0; i < 4; ++i) { bits[2 * i] = w[i] << 16; bits[2 * i + 1] = w[i] & 0xFFFF0000u; }
    }
}

// The scalar fields of a bucket's record from its combined integer sums:
// ln(a / g_min) = ln2 * (exponent + log2 mantissa) - ln g_min.
__device__ __forceinline__ void write_scalars(tq_stats_t* S, const StatsExtra& x, uint64_t n, float g_min)
{
    double sum_log = 0.0;
    if (x.n_tail)
        sum_log = 0.6931471805599453 * ((double)x.exp_sum + (double)x.log2m_fix * 3.725290298461914e-09) -
                  (double)x.n_tail * log((double)g_min);
    S->n_nonfinite = x.n_nonfinite;
    S->absmax = __uint_as_float(x.absmax_bits);            // non-negative floats order as integers
    S->n = n;
    S->g_min = g_min > 0.0f ? g_min : 0.0f;
    S->reserved = 0u;
    S->n_tail = x.n_tail;
    S->sum_log_tail = sum_log;
}

// LDS of one workgroup of the statistics kernels.
struct StatsLds {
    uint32_t hist[kStatsReplicas * kStatsStride];
    uint32_t red_u32[2][kStatsBlock / 64];
    unsigned long long red_u64[4][kStatsBlock / 64];
};

// One workgroup (kStatsBlock threads) takes the elements [cstart, cend) of one tensor: their
// histogram goes to `row` (TQ_NBINS counts, every bin written), and thread 0 returns the other
// sums (meaningless in the other threads).  cstart is a multiple of 8 elements.
template <int DTYPE, bool TAIL>
__device__ __forceinline__ StatsExtra stats_slice(const void* __restrict__ g, uint64_t cstart, uint64_t cend,
                                                  float g_min, StatsLds& L, uint32_t* __restrict__ row)
{
    // Full trips of kTrip tiles each, two register buffers: the next trip's 16-byte loads are
    // requested before the current trip's values are histogrammed.  The trip count is the same
    // for every lane of the workgroup; what is left after the full trips is less than a trip.
    //  - bf16 is bound by instruction issue: trips of two tiles, and the wavefront works on one
    //    buffer while the other one's loads are in flight.
    //  - fp32 is bound by memory and runs with two wavefronts per SIMD: trips of four tiles
    //    (eight 16-byte loads per lane), and the wavefront waits for ALL its loads, the ones
    //    just requested included, before it works on the older buffer -- so it has nothing in
    //    flight while it computes, and the other wavefront of the SIMD fills the gap.  Measured
    //    on 8 x 124 M fp32: 705 us when a wavefront keeps loads in flight under its own work,
    //    677-682 us this way (698 with trips of two tiles, 697 with six, 709 with eight); the
    //    memory system gives more with fewer requests outstanding per compute unit, as it
    //    does for a plain read loop once arithmetic is added to it.
    constexpr int kTrip = DTYPE == TQ_F32 ? 4 : 2;
    constexpr bool kWaitAll = DTYPE == TQ_F32;
    const uint64_t lane_e = cstart + (uint64_t)threadIdx.x * kGroup;
    const uint32_t n_trips = (uint32_t)((cend - cstart) / ((uint64_t)kTrip * kStatsTile));
    // Two register buffers that swap roles (no copies: a copy would wait for the loads in
    // flight); sched_barrier keeps each request ahead of the work it overlaps.  The requests
    // of the loop are unconditional: a branch between a request and the work after it would
    // make the compiler wait for every load in flight where the paths join.  What is left
    // after the full trips is at most kTrip tiles; there a lane requests the whole groups it has.
    RawGroup<DTYPE> bufA[kTrip], bufB[kTrip];
    const uint64_t rest = lane_e + (uint64_t)n_trips * kTrip * kStatsTile;
    auto request = [&](RawGroup<DTYPE> (&buf)[kTrip], uint32_t trip) {
#pragma unroll
        for (int t = 0; t < kTrip; ++t)
            load_raw<DTYPE>(g, lane_e + ((uint64_t)trip * kTrip + t) * kStatsTile, buf[t]);
    };
    auto request_rest = [&](RawGroup<DTYPE> (&buf)[kTrip]) {
#pragma unroll
        for (int t = 0; t < kTrip; ++t) {
            const uint64_t e0 = rest + (uint64_t)t * kStatsTile;
            if (e0 + kGroup <= cend) load_raw<DTYPE>(g, e0, buf[t]);
        }
    };
    // on its way while the histograms are cleared
    if (n_trips > 0) request(bufA, 0); else request_rest(bufA);
    __builtin_amdgcn_sched_barrier(0);

    uint32_t* hist = L.hist;
    for (int i = threadIdx.x; i < kStatsReplicas * kStatsStride; i += kStatsBlock) hist[i] = 0u;
    __syncthreads();

    uint32_t* my_hist = hist + (threadIdx.x & (kStatsReplicas - 1)) * kStatsStride;
    // LDS byte address of the lane's replica, less the bias of the bin index, as one opaque
    // register: the address of a bin is then one shift-and-add on the clamped magnitude bits
    using lds_u32 = __attribute__((address_space(3))) uint32_t;
    uint32_t biased_base = (uint32_t)(uintptr_t)(lds_u32*)my_hist - 4u * (uint32_t)kBinBias;
    asm volatile("" : "+v"(biased_base));
    const uint32_t gmin_bits = __float_as_uint(g_min);
    uint32_t amax_bits = 0u, nonfinite = 0u;
    uint32_t n_tail_wave = 0u;           // tail elements the whole wavefront has seen in the full trips (same in every lane)
    uint32_t n_tail_lane = 0u;           // tail elements this lane has seen where only part of the wavefront runs
    uint32_t not_counted = 0u;           // values this lane put into bin 0 that do not belong there
    // The tail's sum of exponents is not accumulated per element: a bin of the histogram lies inside
    // one octave, so the counts give it -- every element of a bin above g_min's bin is a tail element
    // with that bin's exponent, and the tail elements of g_min's own bin are the rest of the tail
    // count.  Only the last bin (65536 and up) spans octaves; its rare elements are taken one by one.
    constexpr uint32_t kTopBits = (uint32_t)(kBinBias + TQ_NBINS - 1) << 19;   // 65536.0f
    uint32_t exp_top = 0u, cnt_top = 0u; // BIASED exponents and number of the tail elements in the last bin
    unsigned long long log2m_fix = 0ull; // sum of log2(product of 8 mantissas in [1,2)) in 2^-28 fixed point

    // Eight magnitudes (one lane's group of consecutive elements) into the lane's running
    // statistics.  NaN and Inf are rare, so the common path does not test for them per value:
    // the largest of the eight tells whether the wavefront saw one at all, and only then are
    // they counted and replaced by 0 -- which lands in bin 0 and is taken out of it again
    // before the counts are written.  The tail's log-sum costs one logarithm per group: the
    // eight mantissas (1.0 for a value outside the tail) are multiplied in a fixed tree order.
    // ALL_LANES: called with the whole wavefront active; the tail count is then taken by the scalar
    // unit from the compare masks, which saves a vector instruction per element.
    auto take_group = [&](const uint32_t (&raw)[8], auto all_lanes) {
        constexpr bool ALL_LANES = decltype(all_lanes)::value;
        uint32_t a[8];                                                 // |g| as ordered integers
#pragma unroll
        for (int j = 0; j < 8; ++j) a[j] = raw[j] & 0x7FFFFFFFu;
        auto max8 = [&]() {
            const uint32_t m01 = a[0] > a[1] ? a[0] : a[1], m23 = a[2] > a[3] ? a[2] : a[3];
            const uint32_t m45 = a[4] > a[5] ? a[4] : a[5], m67 = a[6] > a[7] ? a[6] : a[7];
            const uint32_t m03 = m01 > m23 ? m01 : m23, m47 = m45 > m67 ? m45 : m67;
            return m03 > m47 ? m03 : m47;
        };
        uint32_t m = max8();
        if (__builtin_amdgcn_ballot_w64(m >= kTopBits) != 0ull) {      // wavefront-uniform, rare
            if (__builtin_amdgcn_ballot_w64(m >= 0x7F800000u) != 0ull) {
#pragma unroll
                for (int j = 0; j < 8; ++j) {
                    const bool finite = a[j] < 0x7F800000u;
                    nonfinite += finite ? 0u : 1u;
                    a[j] = finite ? a[j] : 0u;
                }
                m = max8();
            }
            if constexpr (TAIL) {
#pragma unroll
                for (int j = 0; j < 8; ++j) {
                    const bool top = a[j] >= kTopBits && a[j] > gmin_bits;
                    exp_top += top ? a[j] >> 23 : 0u;
                    cnt_top += top ? 1u : 0u;
                }
            }
        }
        amax_bits = m > amax_bits ? m : amax_bits;
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            uint32_t c = a[j] >> 19;                                   // bin = 16 per octave, counted from 2^-40
            c = c < (uint32_t)kBinBias ? (uint32_t)kBinBias : (c > (uint32_t)(kBinBias + TQ_NBINS - 1) ? (uint32_t)(kBinBias + TQ_NBINS - 1) : c);
            __hip_atomic_fetch_add((lds_u32*)(uintptr_t)(biased_base + (c << 2)), 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
        }
        if constexpr (TAIL) {                                          // g_min >= 2^-40: a tail value is normal
            float mant[8];
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                const bool in_tail = a[j] > gmin_bits;
                if constexpr (ALL_LANES) n_tail_wave += (uint32_t)__builtin_popcountll(__builtin_amdgcn_ballot_w64(in_tail));
                else n_tail_lane += in_tail ? 1u : 0u;
                const uint32_t am = in_tail ? a[j] : 0u;              // mantissa 1.0 outside the tail
                mant[j] = __uint_as_float((am & 0x007FFFFFu) | 0x3F800000u);
            }
            const float prod = ((mant[0] * mant[1]) * (mant[2] * mant[3])) * ((mant[4] * mant[5]) * (mant[6] * mant[7]));
            log2m_fix += (uint32_t)(__log2f(prod) * 268435456.0f);     // prod in [1, 256]: at most 2^31
        }
    };

    auto consume = [&](const RawGroup<DTYPE> (&buf)[kTrip]) {
#pragma unroll
        for (int t = 0; t < kTrip; ++t) {
            uint32_t bits[8];
            raw_bits<DTYPE>(buf[t], bits);
            take_group(bits, std::true_type{});
        }
    };
    // what is left after the full trips: whole groups from the buffer, the one group that the
    // end of the range cuts value by value
    auto consume_rest = [&](const RawGroup<DTYPE> (&buf)[kTrip]) {
#pragma unroll
        for (int t = 0; t < kTrip; ++t) {
            const uint64_t e0 = rest + (uint64_t)t * kStatsTile;
            if (e0 + kGroup <= cend) {
                uint32_t bits[8];
                raw_bits<DTYPE>(buf[t], bits);
                take_group(bits, std::false_type{});
            } else if (e0 < cend) {                                    // ragged end of the range
                const int n_valid = (int)(cend - e0);                  // the absent values enter as 0
                uint32_t b0[8];
#pragma unroll
                for (int j = 0; j < 8; ++j) {
                    b0[j] = 0u;
                    if (j < n_valid) {
                        if constexpr (DTYPE == TQ_F32) b0[j] = static_cast<const uint32_t*>(g)[e0 + j];
                        else b0[j] = (uint32_t) static_cast<const uint16_t*>(g)[e0 + j] << 16;
                    }
                }
                take_group(b0, std::false_type{});
                not_counted += (uint32_t)(8 - n_valid);
            }
        }
    };
    // bufA holds trip 2p; the loop ends with the last or the last but one full trip in bufA
    const uint32_t loops = n_trips > 0 ? (n_trips - 1) >> 1 : 0;
    for (uint32_t p = 0; p < loops; ++p) {
        request(bufB, 2 * p + 1);
        if constexpr (kWaitAll) asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        __builtin_amdgcn_sched_barrier(0);
        consume(bufA);
        __builtin_amdgcn_sched_barrier(0);
        request(bufA, 2 * p + 2);
        if constexpr (kWaitAll) asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        __builtin_amdgcn_sched_barrier(0);
        consume(bufB);
        __builtin_amdgcn_sched_barrier(0);
    }
    if (n_trips == 0) {                                                // bufA holds the rest
        consume_rest(bufA);
    } else if (n_trips & 1u) {                                         // bufA holds the last full trip
        request_rest(bufB);
        __builtin_amdgcn_sched_barrier(0);
        consume(bufA);
        __builtin_amdgcn_sched_barrier(0);
        consume_rest(bufB);
    } else {                                                           // bufA holds the last but one
        request(bufB, n_trips - 1);
        __builtin_amdgcn_sched_barrier(0);
        consume(bufA);
        __builtin_amdgcn_sched_barrier(0);
        request_rest(bufA);
        __builtin_amdgcn_sched_barrier(0);
        consume(bufB);
        __builtin_amdgcn_sched_barrier(0);
        consume_rest(bufA);
    }
    // NaN, Inf and the absent values of a ragged group were counted as zeros: take them out again
    not_counted += nonfinite;
    if (not_counted) atomicSub(&my_hist[0], not_counted);
    __syncthreads();

    // the slice's counts, every bin (the destination is not pre-cleared)
    // ... and, from the same counts, the exponents of the tail elements in the bins above g_min's
    uint32_t gbin = gmin_bits >> 19;                                   // g_min's bin (g_min >= 2^-40: at least 1)
    gbin = (gbin > (uint32_t)kBinBias ? gbin - (uint32_t)kBinBias : 0u);
    gbin = gbin < (uint32_t)(TQ_NBINS - 1) ? gbin : (uint32_t)(TQ_NBINS - 1);
    unsigned long long exp_bins = 0ull, cnt_bins = 0ull;
    for (int b = threadIdx.x; b < TQ_NBINS; b += kStatsBlock) {
        uint32_t total = 0u;
#pragma unroll
        for (int r = 0; r < kStatsReplicas; ++r) total += hist[r * kStatsStride + b];
        row[b] = total;
        if (TAIL && (uint32_t)b > gbin && b < TQ_NBINS - 1) {
            exp_bins += (unsigned long long)((uint32_t)(kBinBias + b) >> 4) * total;
            cnt_bins += total;
        }
    }

    // max, counts and log-sum of the slice: wavefront reduction, then thread 0 adds the 8 waves
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    amax_bits = wave_reduce_max(amax_bits);
    nonfinite = wave_reduce_add(nonfinite);
    const unsigned long long nt = wave_reduce_add((unsigned long long)n_tail_lane) + n_tail_wave;
    const unsigned long long es = wave_reduce_add(exp_bins + exp_top);     // exponents counted so far
    const unsigned long long cs = wave_reduce_add(cnt_bins + cnt_top);     // ... of this many tail elements
    const unsigned long long lf = wave_reduce_add(log2m_fix);
    if (lane == 0) {
        L.red_u32[0][wave] = amax_bits; L.red_u32[1][wave] = nonfinite;
        L.red_u64[0][wave] = nt; L.red_u64[1][wave] = es; L.red_u64[2][wave] = lf; L.red_u64[3][wave] = cs;
    }
    __syncthreads();
    StatsExtra x{0u, 0u, 0ull, 0ll, 0ull};
    if (threadIdx.x == 0) {
        unsigned long long counted = 0ull;
        for (int w = 0; w < kStatsBlock / 64; ++w) {
            x.absmax_bits = L.red_u32[0][w] > x.absmax_bits ? L.red_u32[0][w] : x.absmax_bits;
            x.n_nonfinite += L.red_u32[1][w];
            x.n_tail += L.red_u64[0][w];
            x.exp_sum += (long long)L.red_u64[1][w];
            x.log2m_fix += L.red_u64[2][w];
            counted += L.red_u64[3][w];
        }
        // the tail elements not counted yet are those of g_min's own bin
        x.exp_sum += (long long)((uint32_t)(kBinBias + gbin) >> 4) * (long long)(x.n_tail - counted);
        x.exp_sum -= 127ll * (long long)x.n_tail;                      // biased -> unbiased exponents
    }
    return x;
}

template <int DTYPE, bool TAIL>
__global__ __launch_bounds__(kStatsBlock) void tq_stats_partial_kernel(
    const PtrTable g_tab, uint64_t d, uint64_t bucket_elems, uint32_t slices, uint64_t slice_elems,
    float g_min, char* __restrict__ ws, uint64_t ws_tensor_bytes, uint64_t ws_hist_bytes,
    const MutPtrTable stats_tab)
{
    // blockIdx.y = tensor of the batch; each tensor has its own region of the workspace
    const void* __restrict__ g = g_tab.p[blockIdx.y];
    char* my_ws = ws + (uint64_t)blockIdx.y * ws_tensor_bytes;
    uint32_t* __restrict__ ws_hist = reinterpret_cast<uint32_t*>(my_ws);
    StatsExtra* __restrict__ ws_extra = reinterpret_cast<StatsExtra*>(my_ws + ws_hist_bytes);
    const uint32_t blk = linear_block();
    if ((uint64_t)(blk / slices) * bucket_elems >= d) return;          // padding of a folded grid
    __shared__ StatsLds L;

    const uint32_t bucket = blk / slices;
    const uint32_t slice = blk - bucket * slices;
    const uint64_t bstart = (uint64_t)bucket * bucket_elems;
    const uint64_t bend = bstart + bucket_elems < d ? bstart + bucket_elems : d;
    uint64_t cstart = bstart + (uint64_t)slice * slice_elems;
    cstart = cstart < bend ? cstart : bend;
    const uint64_t cend = cstart + slice_elems < bend ? cstart + slice_elems : bend;

    // partial counts of this slice as one contiguous row of the workspace; a bucket that is one
    // slice writes its record directly and no second kernel follows
    const bool final_record = slices == 1u;
    tq_stats_t* S = static_cast<tq_stats_t*>(stats_tab.p[blockIdx.y]) + bucket;
    uint32_t* row = final_record ? S->hist : ws_hist + ((uint64_t)bucket * slices + slice) * TQ_NBINS;
    const StatsExtra x = stats_slice<DTYPE, TAIL>(g, cstart, cend, g_min, L, row);
    if (threadIdx.x == 0) {
        if (final_record) write_scalars(S, x, bend - bstart, g_min);
        else ws_extra[(uint64_t)bucket * slices + slice] = x;
    }
}

// Adds `rows` consecutive partial rows (row0 onwards) of one bucket into its record S.  The
// bucket's workgroups are numbered grp = 0 .. groups_per_bucket - 1: all but the last take 64
// bins each, the last one the scalar fields.  n = elements of the bucket.
__device__ __forceinline__ void reduce_rows(const uint32_t* __restrict__ ws_hist, const StatsExtra* __restrict__ ws_extra,
                                            uint64_t row0, uint32_t rows, uint32_t grp, uint32_t groups_per_bucket,
                                            tq_stats_t* __restrict__ S, uint64_t n, float g_min, uint32_t* part)
{
    if (grp + 1 < groups_per_bucket) {
        // 64 consecutive bins x 16 interleaved row lanes; a wavefront reads 256 contiguous bytes
        const uint32_t bin = grp * kReduceBins + (threadIdx.x & (kReduceBins - 1));
        const uint32_t sl = threadIdx.x / kReduceBins;
        uint32_t total = 0u;
        if (bin < TQ_NBINS) {
            const uint32_t* col = ws_hist + row0 * TQ_NBINS + bin;
            for (uint32_t p = sl; p < rows; p += kReduceBlock / kReduceBins) total += col[(uint64_t)p * TQ_NBINS];
        }
        part[threadIdx.x] = total;
        __syncthreads();
        if (threadIdx.x < kReduceBins && bin < TQ_NBINS) {
#pragma unroll
            for (int k = 1; k < kReduceBlock / kReduceBins; ++k) total += part[threadIdx.x + k * kReduceBins];
            S->hist[bin] = total;
        }
    } else if (threadIdx.x < 64) {
        // last workgroup of the bucket: max, counts and the log-sum of the rows (integer sums)
        const int lane = threadIdx.x;
        const StatsExtra* row = ws_extra + row0;
        uint32_t amax = 0u, nonfinite = 0u;
        unsigned long long n_tail = 0ull, log2m_fix = 0ull;
        long long exp_sum = 0ll;
        for (uint32_t p = lane; p < rows; p += 64) {
            const StatsExtra x = row[p];
            amax = x.absmax_bits > amax ? x.absmax_bits : amax;
            nonfinite += x.n_nonfinite;
            n_tail += x.n_tail;
            exp_sum += x.exp_sum;
            log2m_fix += x.log2m_fix;
        }
        amax = wave_reduce_max(amax);
        nonfinite = wave_reduce_add(nonfinite);
        n_tail = wave_reduce_add(n_tail);
        exp_sum = wave_reduce_add(exp_sum);
        log2m_fix = wave_reduce_add(log2m_fix);
        if (lane == 0) {
            const StatsExtra x{amax, nonfinite, n_tail, exp_sum, log2m_fix};
            write_scalars(S, x, n, g_min);
        }
    }
}

__global__ __launch_bounds__(kReduceBlock) void tq_stats_reduce_kernel(
    const char* __restrict__ ws, uint64_t ws_tensor_bytes, uint64_t ws_hist_bytes, uint32_t slices,
    uint32_t groups_per_bucket, uint64_t d, uint64_t bucket_elems, float g_min, const MutPtrTable stats_tab)
{
    __shared__ uint32_t part[kReduceBlock];
    const char* my_ws = ws + (uint64_t)blockIdx.y * ws_tensor_bytes;
    const uint32_t* __restrict__ ws_hist = reinterpret_cast<const uint32_t*>(my_ws);
    const StatsExtra* __restrict__ ws_extra = reinterpret_cast<const StatsExtra*>(my_ws + ws_hist_bytes);
    tq_stats_t* __restrict__ stats = static_cast<tq_stats_t*>(stats_tab.p[blockIdx.y]);
    const uint32_t blk = linear_block();
    const uint32_t bucket = blk / groups_per_bucket;
    const uint32_t grp = blk - bucket * groups_per_bucket;
    if ((uint64_t)bucket * bucket_elems >= d) return;                  // padding of a folded grid
    const uint64_t lo = (uint64_t)bucket * bucket_elems;
    const uint64_t hi = lo + bucket_elems < d ? lo + bucket_elems : d;
    reduce_rows(ws_hist, ws_extra, (uint64_t)bucket * slices, slices, grp, groups_per_bucket, stats + bucket,
                hi - lo, g_min, part);
}


// ---- large buckets: the whole batch cut into equal shares ---------------------------------
//
// With buckets of 32768 elements or more the launch is `groups` workgroups (one per compute
// unit for fp32, four for bf16) and the batch -- the tensors laid end to end, counted in tiles of
// 4096 elements -- is cut into that many equal shares, whatever the buckets are: share w is the
// tiles [w TT / groups, (w+1) TT / groups).  A workgroup takes the pieces of the buckets that
// overlap its share one after the other.  A bucket that lies inside one share is written as a
// finished record; the pieces of the others go to partial rows, numbered share + global bucket
// index (from one piece to the next one of the two advances, so the number is unique and a
// bucket's rows are consecutive), and a second kernel adds them.  Every workgroup reads the
// same number of bytes, so no compute unit is left idle at the end: with one bucket per
// workgroup 8 x 119 buckets of 2^20 on 256 compute units took four passes for 3.7 passes of work.

constexpr uint64_t kBalancedMinBucket = 32768;

template <int DTYPE, bool TAIL>
__global__ __launch_bounds__(kStatsBlock) void tq_stats_balanced_kernel(
    const PtrTable g_tab, uint64_t d, uint64_t be, uint64_t nb, uint64_t tiles_per_tensor, uint64_t total_tiles,
    float g_min, uint32_t* __restrict__ ws_hist, StatsExtra* __restrict__ ws_extra, const MutPtrTable stats_tab)
{
    const uint32_t w = blockIdx.x;
    uint64_t tile = share_start(w, total_tiles, gridDim.x);
    const uint64_t tile_end = share_start((uint64_t)w + 1, total_tiles, gridDim.x);
    __shared__ StatsLds L;
    bool first = true;
    while (tile < tile_end) {                                          // one pass per tensor the share touches
        const uint64_t t = tile / tiles_per_tensor, i = tile - t * tiles_per_tensor;
        const uint64_t i_end = i + (tile_end - tile) < tiles_per_tensor ? i + (tile_end - tile) : tiles_per_tensor;
        const uint64_t e0 = i * kStatsTile;
        const uint64_t e1 = i_end * kStatsTile < d ? i_end * kStatsTile : d;
        const void* __restrict__ g = g_tab.p[t];
        tq_stats_t* __restrict__ stats = static_cast<tq_stats_t*>(stats_tab.p[t]);
        for (uint64_t b = e0 / be; b * be < e1; ++b) {
            const uint64_t lo = b * be, hi = lo + be < d ? lo + be : d;
            const uint64_t cs = e0 > lo ? e0 : lo, ce = e1 < hi ? e1 : hi;
            const bool whole = cs == lo && ce == hi;                   // no other share has a piece of this bucket
            const uint64_t r = (uint64_t)w + t * nb + b;
            if (!first) __syncthreads();                               // the histograms are cleared again
            first = false;
            const StatsExtra x = stats_slice<DTYPE, TAIL>(g, cs, ce, g_min, L, whole ? stats[b].hist : ws_hist + r * TQ_NBINS);
            if (threadIdx.x == 0) {
                if (whole) write_scalars(stats + b, x, hi - lo, g_min);
                else ws_extra[r] = x;
            }
        }
        tile += i_end - i;
    }
}

// Adds the rows of the buckets that more than one share has a piece of.  One unit of
// groups_per_bucket workgroups per bucket (by_boundary = 0), or -- when there are more buckets
// than shares -- per boundary between two shares: the unit of boundary k takes the bucket the
// boundary cuts, if it cuts one and if it is the first boundary inside that bucket.
// The bucket a unit of the second kernel adds up, if any: tensor t, bucket b, its first row and
// the number of rows.
struct SplitBucket { uint64_t t, b, row0, n; uint32_t rows; bool any; };

__device__ __forceinline__ SplitBucket split_bucket(uint64_t unit, uint32_t by_boundary, uint64_t d, uint64_t be, uint64_t nb,
                                                    uint64_t tiles_per_tensor, uint64_t total_tiles, uint32_t groups)
{
    SplitBucket k{0, 0, 0, 0, 0, false};
    if (by_boundary) {
        const uint64_t tile = share_start(unit + 1, total_tiles, groups);
        k.t = tile / tiles_per_tensor;
        const uint64_t e = (tile - k.t * tiles_per_tensor) * kStatsTile;
        k.b = e / be;
        if (e == k.b * be) return k;                                   // the shares meet where a bucket (or tensor) begins
    } else {
        k.t = unit / nb;
        k.b = unit - k.t * nb;
    }
    const uint64_t lo = k.b * be, hi = lo + be < d ? lo + be : d;
    const uint32_t w0 = share_of_tile(k.t * tiles_per_tensor + lo / kStatsTile, total_tiles, groups);
    const uint32_t w1 = share_of_tile(k.t * tiles_per_tensor + (hi - 1) / kStatsTile, total_tiles, groups);
    if (w0 == w1) return k;                                            // written as a finished record already
    if (by_boundary && w0 != unit) return k;                           // added at the first boundary inside it
    k.row0 = (uint64_t)w0 + k.t * nb + k.b;
    k.rows = w1 - w0 + 1;
    k.n = hi - lo;
    k.any = true;
    return k;
}

// The same for buckets of a few rows each (at most kNarrowRows): one small workgroup per unit.
constexpr int kNarrowBlock = 256;
constexpr uint32_t kNarrowRows = 8;
__global__ __launch_bounds__(kNarrowBlock) void tq_stats_balanced_reduce_narrow_kernel(
    uint64_t d, uint64_t be, uint64_t nb, uint64_t tiles_per_tensor, uint64_t total_tiles, uint32_t groups,
    uint32_t by_boundary, uint64_t n_units, float g_min,
    const uint32_t* __restrict__ ws_hist, const StatsExtra* __restrict__ ws_extra, const MutPtrTable stats_tab)
{
    const uint64_t unit = linear_block();
    if (unit >= n_units) return;                                       // padding of a folded grid
    const SplitBucket k = split_bucket(unit, by_boundary, d, be, nb, tiles_per_tensor, total_tiles, groups);
    if (!k.any) return;
    tq_stats_t* __restrict__ S = static_cast<tq_stats_t*>(stats_tab.p[k.t]) + k.b;
    for (int bin = threadIdx.x; bin < TQ_NBINS; bin += kNarrowBlock) {
        uint32_t total = 0u;
        for (uint32_t r = 0; r < k.rows; ++r) total += ws_hist[(k.row0 + r) * TQ_NBINS + bin];
        S->hist[bin] = total;
    }
    if (threadIdx.x == 0) {
        StatsExtra x{0u, 0u, 0ull, 0ll, 0ull};
        for (uint32_t r = 0; r < k.rows; ++r) {
            const StatsExtra y = ws_extra[k.row0 + r];
            x.absmax_bits = y.absmax_bits > x.absmax_bits ? y.absmax_bits : x.absmax_bits;
            x.n_nonfinite += y.n_nonfinite;
            x.n_tail += y.n_tail;
            x.exp_sum += y.exp_sum;
            x.log2m_fix += y.log2m_fix;
        }
        write_scalars(S, x, k.n, g_min);
    }
}

__global__ __launch_bounds__(kReduceBlock) void tq_stats_balanced_reduce_kernel(
    uint64_t d, uint64_t be, uint64_t nb, uint64_t tiles_per_tensor, uint64_t total_tiles, uint32_t groups,
    uint32_t by_boundary, uint64_t n_units, uint32_t groups_per_bucket, float g_min,
    const uint32_t* __restrict__ ws_hist, const StatsExtra* __restrict__ ws_extra, const MutPtrTable stats_tab)
{
    __shared__ uint32_t part[kReduceBlock];
    const uint32_t blk = linear_block();
    const uint64_t unit = blk / groups_per_bucket;
    const uint32_t grp = blk - (uint32_t)unit * groups_per_bucket;
    if (unit >= n_units) return;                                       // padding of a folded grid
    const SplitBucket k = split_bucket(unit, by_boundary, d, be, nb, tiles_per_tensor, total_tiles, groups);
    if (!k.any) return;
    reduce_rows(ws_hist, ws_extra, k.row0, k.rows, grp, groups_per_bucket,
                static_cast<tq_stats_t*>(stats_tab.p[k.t]) + k.b, k.n, g_min, part);
}


// ---- variable-size segments (Sec. V: the layers of a network are quantized independently) ----
//
// Every tensor of the batch is cut at seg_off[0] = 0 < ... < seg_off[nseg] = d (interior offsets
// multiples of 128) and there is one record per tensor and segment.  Work is cut as for large
// buckets: the batch in equal shares of tiles, one workgroup each, whatever the segments are.
// A workgroup takes the pieces of the segments that overlap its share one after the other and
// writes one partial row per piece, numbered share + global segment index (from one piece to
// the next one of the two advances: the number is unique and a segment's rows are
// consecutive); a second kernel adds each segment's rows.  Every access is bounded by d, nseg
// and the number of rows, whatever the table holds.

template <int DTYPE, bool TAIL>
__global__ __launch_bounds__(kStatsBlock) void tq_stats_segments_partial_kernel(
    const PtrTable g_tab, uint64_t d, uint64_t tiles_per_tensor, uint64_t total_tiles,
    const uint64_t* __restrict__ seg_off, uint32_t nseg, float g_min,
    uint32_t* __restrict__ ws_hist, StatsExtra* __restrict__ ws_extra)
{
    const uint32_t w = blockIdx.x;
    uint64_t tile = share_start(w, total_tiles, gridDim.x);
    const uint64_t tile_end = share_start((uint64_t)w + 1, total_tiles, gridDim.x);
    __shared__ StatsLds L;
    bool first = true;
    while (tile < tile_end) {                                          // one pass per tensor the share touches
        const uint64_t t = tile / tiles_per_tensor, i = tile - t * tiles_per_tensor;
        const uint64_t i_end = i + (tile_end - tile) < tiles_per_tensor ? i + (tile_end - tile) : tiles_per_tensor;
        const uint64_t cstart = i * kStatsTile;
        const uint64_t cend = i_end * kStatsTile < d ? i_end * kStatsTile : d;
        const void* __restrict__ g = g_tab.p[t];
        uint32_t s = find_segment(seg_off, nseg, cstart);
        for (;;) {
            // the last segment ends at d whatever the table says: the loop ends with the share
            uint64_t seg_lo = seg_off[s], seg_hi = s + 1 < nseg ? seg_off[s + 1] : d;
            seg_lo = seg_lo > cstart ? (seg_lo < cend ? seg_lo : cend) : cstart;
            seg_hi = seg_hi < cend ? (seg_hi > seg_lo ? seg_hi : seg_lo) : cend;
            seg_lo &= ~7ull;                                           // groups of 8 never straddle a segment
            const uint64_t r = (uint64_t)w + t * nseg + s;
            if (!first) __syncthreads();                               // the histograms are cleared again
            first = false;
            const StatsExtra x = stats_slice<DTYPE, TAIL>(g, seg_lo, seg_hi, g_min, L, ws_hist + r * TQ_NBINS);
            if (threadIdx.x == 0) ws_extra[r] = x;
            if (seg_hi >= cend || s + 1 >= nseg) break;
            ++s;
        }
        tile += i_end - i;
    }
}

// One workgroup per tensor and segment adds the rows of the shares the segment reaches into.
__global__ __launch_bounds__(kStatsBlock) void tq_stats_segments_reduce_kernel(
    uint64_t d, uint64_t tiles_per_tensor, uint64_t total_tiles, uint32_t groups, uint32_t count,
    const uint64_t* __restrict__ seg_off, uint32_t nseg, float g_min,
    const uint32_t* __restrict__ ws_hist, const StatsExtra* __restrict__ ws_extra, uint64_t n_rows,
    const MutPtrTable stats_tab)
{
    const uint32_t unit = linear_block();
    const uint32_t t = unit / nseg, s = unit - t * nseg;
    if (t >= count) return;                                            // padding of a folded grid
    const uint64_t lo = seg_off[s] < d ? seg_off[s] : d;
    uint64_t hi = s + 1 < nseg ? seg_off[s + 1] : d;
    hi = hi < d ? hi : d;
    tq_stats_t* S = static_cast<tq_stats_t*>(stats_tab.p[t]) + s;
    const bool empty = hi <= lo;                                       // only with a malformed table
    uint64_t r0 = 0, r1 = 0;                                           // first and last row
    if (!empty) {
        const uint64_t base = (uint64_t)t * nseg + s;
        r0 = share_of_tile((uint64_t)t * tiles_per_tensor + lo / kStatsTile, total_tiles, groups) + base;
        r1 = share_of_tile((uint64_t)t * tiles_per_tensor + (hi - 1) / kStatsTile, total_tiles, groups) + base;
        r1 = r1 < n_rows ? r1 : n_rows - 1;
        r0 = r0 < r1 ? r0 : r1;
    }
    for (int b = threadIdx.x; b < TQ_NBINS; b += kStatsBlock) {
        uint32_t total = 0u;
        if (!empty) {
#pragma unroll 8
            for (uint64_t r = r0; r <= r1; ++r) total += ws_hist[r * TQ_NBINS + b];
        }
        S->hist[b] = total;
    }
    if (threadIdx.x == 0) {
        StatsExtra x{0u, 0u, 0ull, 0ll, 0ull};
        if (!empty)
            for (uint64_t r = r0; r <= r1; ++r) {
                const StatsExtra y = ws_extra[r];
                x.absmax_bits = y.absmax_bits > x.absmax_bits ? y.absmax_bits : x.absmax_bits;
                x.n_nonfinite += y.n_nonfinite;
                x.n_tail += y.n_tail;
                x.exp_sum += y.exp_sum;
                x.log2m_fix += y.log2m_fix;
            }
        write_scalars(S, x, empty ? 0 : hi - lo, g_min);
    }
}

}  // namespace tq

namespace {

struct StatsPlan {
    uint64_t be, nb, slice_elems;
    uint32_t slices;
};

// Most slices a bucket is ever cut into: slices of at least 16384 elements, and no more than
// about one workgroup per compute unit when a single tensor is processed.  The workspace is
// sized for this many.
uint32_t max_slices(uint64_t be, uint64_t nb)
{
    const uint64_t want = (be + tq::kStatsMinSlice - 1) / tq::kStatsMinSlice;
    uint64_t cap = (tq::kStatsTargetGroups + nb - 1) / nb;
    cap = cap > tq::kStatsMaxSlices ? tq::kStatsMaxSlices : cap;
    const uint64_t m = want < cap ? want : cap;
    return (uint32_t)(m < 1 ? 1 : m);
}

// Slices per bucket for a batch of `count` tensors with buckets of fewer than 32768 elements.
// Each workgroup pays for clearing and flushing its LDS histograms -- about what reading
// 16384 elements costs -- so fewer, longer-lived workgroups win as long as the machine is full,
// and a launch of W workgroups takes ceil(W / resident) times one workgroup's time, `resident`
// being the workgroups the launch should keep running at the same time.  The slice count
// minimises that product.
StatsPlan plan_stats(uint64_t d, uint64_t bucket_elems, int count, uint64_t resident)
{
    StatsPlan p;
    p.be = bucket_elems ? bucket_elems : d;
    p.nb = (d + p.be - 1) / p.be;
    const uint64_t units = p.nb * (uint64_t)(count < 1 ? 1 : count);
    const uint32_t smax = max_slices(p.be, p.nb);
    uint32_t best = 1;
    uint64_t best_cost = ~0ull;
    for (uint32_t sl = 1; sl <= smax; ++sl) {
        const uint64_t rounds = (units * sl + resident - 1) / resident;
        const uint64_t cost = rounds * ((p.be + sl - 1) / sl + (uint64_t)tq::kStatsMinSlice);
        if (cost < best_cost) { best_cost = cost; best = sl; }
    }
    p.slices = best;
    const uint64_t per = (p.be + p.slices - 1) / p.slices;
    p.slice_elems = (per + tq::kStatsTile - 1) / tq::kStatsTile * tq::kStatsTile;
    return p;
}

// Whether the launch is cut into equal shares (large buckets) or into buckets and their slices.
bool uses_shares(uint64_t d, uint64_t bucket_elems)
{
    const uint64_t be = bucket_elems && bucket_elems < d ? bucket_elems : d;
    return be >= tq::kBalancedMinBucket;
}

}  // namespace

uint64_t tq_stats_workspace_bytes_impl(uint64_t d, uint64_t bucket_elems)
{
    if (d == 0) return 0;
    const uint64_t be = bucket_elems ? bucket_elems : d;
    const uint64_t nb = (d + be - 1) / be;
    const uint32_t slices = max_slices(be, nb);                        // no plan uses more
    const uint64_t hist_bytes = tq::stats_ws_hist_words(nb, slices) * 4;
    uint64_t bytes = (hist_bytes + 15) / 16 * 16 + nb * slices * sizeof(tq::StatsExtra);
    if (uses_shares(d, bucket_elems)) {
        // one row per share and per bucket; a batch of `count` tensors has count times this much
        const uint64_t shared = (tq::kStatsResidentGroups + nb) * (TQ_NBINS * 4 + sizeof(tq::StatsExtra));
        bytes = bytes > shared ? bytes : shared;
    }
    return (bytes + 255) / 256 * 256;                                  // regions of a batch stay aligned
}

// Device address of this device's copy of `scratch`, looked up once per device with that
// device current and kept for the life of the process.  Devices beyond the table are refused.
hipError_t tq_stats_static_scratch(void** out)
{
    constexpr int kMaxDevices = 64;
    static std::atomic<void*> known[kMaxDevices];
    int dev = -1;
    hipError_t err = hipGetDevice(&dev);
    if (err != hipSuccess) return err;
    if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
    void* ptr = known[dev].load(std::memory_order_acquire);
    if (!ptr) {
        err = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
        if (err != hipSuccess) return err;
        if (!ptr) return hipErrorInvalidSymbol;
        known[dev].store(ptr, std::memory_order_release);          // every thread finds the same address
    }
    *out = ptr;
    return hipSuccess;
}

// Host side of tq_stats / tq_stats_multi after the argument checks of the C entry points:
// `count` same-shaped tensors in one pair of launches (grid.y), each with its own region of
// tq_stats_workspace_bytes(d, bucket_elems) bytes of the workspace.
hipError_t tq_launch_stats(const void* const* g, int count, int dtype, uint64_t d, uint64_t bucket_elems,
                           float g_min, tq_stats_t* const* stats, void* workspace, hipStream_t st)
{
    if (count < 1 || count > tq::kMaxBatch) return hipErrorInvalidValue;
    // bf16 elements cost half the bytes but all the instructions: that kernel is bound by issue and
    // wants every wavefront slot (4 x 10^9 bf16 with tail terms: 1650 us with 256 workgroups, 1440
    // with 512, 1410 with 1024; waiting for all loads as the fp32 kernel does: 1550-2050); the fp32 ones are bound by memory and read fastest with one
    // workgroup per compute unit (8 x 124 M fp32: 740 us with four per compute unit, 691 with one)
    const uint64_t resident = dtype == TQ_BF16 ? tq::kStatsResidentGroups : tq::kStatsTargetGroups;
    if (uses_shares(d, bucket_elems)) {
        tq::PtrTable gt{};
        tq::MutPtrTable stt{};
        for (int i = 0; i < count; ++i) { gt.p[i] = g[i]; stt.p[i] = stats[i]; }
        const uint64_t be = bucket_elems ? bucket_elems : d;
        const uint64_t nb = (d + be - 1) / be;
        const uint64_t tiles_per_tensor = (d + tq::kStatsTile - 1) / tq::kStatsTile;
        const uint64_t total_tiles = tiles_per_tensor * (uint64_t)count;
        const uint64_t fit = total_tiles * tq::kStatsTile / tq::kStatsMinSlice;   // shares of at least 16384 elements
        const uint32_t groups = (uint32_t)(fit < 1 ? 1 : (fit < resident ? fit : resident));
        const uint64_t rows = groups + nb * (uint64_t)count;
        uint32_t* ws_hist = static_cast<uint32_t*>(workspace);
        tq::StatsExtra* ws_extra = reinterpret_cast<tq::StatsExtra*>(static_cast<char*>(workspace) + rows * TQ_NBINS * 4);
#define TQ_LAUNCH_SHARES(DT, TL)                                                                                  \
    hipLaunchKernelGGL((tq::tq_stats_balanced_kernel<DT, TL>), dim3(groups), dim3(tq::kStatsBlock), 0, st, gt, d, be, \
                       nb, tiles_per_tensor, total_tiles, g_min, ws_hist, ws_extra, stt)
        if (dtype == TQ_F32) {
            if (g_min > 0.0f) { TQ_LAUNCH_SHARES(TQ_F32, true); } else { TQ_LAUNCH_SHARES(TQ_F32, false); }
        } else {
            if (g_min > 0.0f) { TQ_LAUNCH_SHARES(TQ_BF16, true); } else { TQ_LAUNCH_SHARES(TQ_BF16, false); }
        }
#undef TQ_LAUNCH_SHARES
        hipError_t err = hipGetLastError();
        if (err != hipSuccess || groups == 1) return err;
        const uint32_t gpb = (TQ_NBINS + tq::kReduceBins - 1) / tq::kReduceBins + 1;
        const uint64_t n_buckets = nb * (uint64_t)count;
        const uint32_t by_boundary = n_buckets > groups - 1 ? 1u : 0u;
        const uint64_t n_units = by_boundary ? groups - 1 : n_buckets;
        dim3 rgrid;
        // rows of a bucket: one per share it reaches into
        const uint64_t share_tiles = total_tiles / groups, bucket_tiles = (be < d ? be : d) / tq::kStatsTile + 2;
        if (bucket_tiles / share_tiles + 2 <= tq::kNarrowRows) {
            if (!tq::fold_grid(n_units, tq::kNarrowBlock, 1, rgrid)) return hipErrorInvalidValue;
            hipLaunchKernelGGL(tq::tq_stats_balanced_reduce_narrow_kernel, rgrid, dim3(tq::kNarrowBlock), 0, st, d, be, nb,
                               tiles_per_tensor, total_tiles, groups, by_boundary, n_units, g_min, ws_hist, ws_extra, stt);
            return hipGetLastError();
        }
        if (!tq::fold_grid(n_units * gpb, tq::kReduceBlock, 1, rgrid)) return hipErrorInvalidValue;
        hipLaunchKernelGGL(tq::tq_stats_balanced_reduce_kernel, rgrid, dim3(tq::kReduceBlock), 0, st, d, be, nb,
                           tiles_per_tensor, total_tiles, groups, by_boundary, n_units, gpb, g_min, ws_hist, ws_extra, stt);
        return hipGetLastError();
    }
    const StatsPlan p = plan_stats(d, bucket_elems, count, resident);
    const uint64_t nblocks = p.nb * p.slices;
    dim3 pgrid;
    if (!tq::fold_grid(nblocks, tq::kStatsBlock, (unsigned)count, pgrid))
        return hipErrorInvalidValue;
    const uint64_t hist_bytes = (tq::stats_ws_hist_words(p.nb, p.slices) * 4 + 15) / 16 * 16;
    const uint64_t tensor_bytes = tq_stats_workspace_bytes_impl(d, bucket_elems);
    tq::PtrTable gt{};
    tq::MutPtrTable stt{};
    for (int i = 0; i < count; ++i) { gt.p[i] = g[i]; stt.p[i] = stats[i]; }
    char* ws = static_cast<char*>(workspace);
#define TQ_LAUNCH_PARTIAL(DT, TL)                                                                             \
    hipLaunchKernelGGL((tq::tq_stats_partial_kernel<DT, TL>), pgrid, dim3(tq::kStatsBlock), 0, st, gt, d, p.be,   \
                       p.slices, p.slice_elems, g_min, ws, tensor_bytes, hist_bytes, stt)
    if (dtype == TQ_F32) {
        if (g_min > 0.0f) TQ_LAUNCH_PARTIAL(TQ_F32, true); else TQ_LAUNCH_PARTIAL(TQ_F32, false);
    } else {
        if (g_min > 0.0f) TQ_LAUNCH_PARTIAL(TQ_BF16, true); else TQ_LAUNCH_PARTIAL(TQ_BF16, false);
    }
#undef TQ_LAUNCH_PARTIAL
    hipError_t err = hipGetLastError();
    if (err != hipSuccess || p.slices == 1) return err;           // one slice per bucket: records are written
    // one workgroup per 64 bins, plus one per bucket for the scalar fields
    const uint32_t gpb = (TQ_NBINS + tq::kReduceBins - 1) / tq::kReduceBins + 1;
    const uint64_t rblocks = p.nb * gpb;
    dim3 rgrid;
    if (!tq::fold_grid(rblocks, tq::kReduceBlock, (unsigned)count, rgrid)) return hipErrorInvalidValue;
    hipLaunchKernelGGL(tq::tq_stats_reduce_kernel, rgrid, dim3(tq::kReduceBlock), 0,
                       st, ws, tensor_bytes, hist_bytes, p.slices, gpb, d, p.be, g_min, stt);
    return hipGetLastError();
}


uint64_t tq_stats_segments_workspace_bytes_impl(uint64_t d, uint64_t nseg)
{
    if (d == 0 || nseg == 0) return 0;
    // one row per share and per segment; a batch of `count` tensors has count times this much
    const uint64_t rows = tq::kStatsResidentGroups + nseg;
    return (rows * (TQ_NBINS * 4 + sizeof(tq::StatsExtra)) + 255) / 256 * 256;
}

// Host side of tq_stats_segments / tq_stats_segments_multi after the argument checks of the C
// entry points: `count` same-shaped tensors with one segment table in one pair of launches.
hipError_t tq_launch_stats_segments(const void* const* g, int count, int dtype, uint64_t d, const uint64_t* seg_off,
                                    uint64_t nseg, float g_min, tq_stats_t* const* stats, void* workspace,
                                    hipStream_t st)
{
    if (count < 1 || count > tq::kMaxBatch || nseg > 0xFFFFFFFFull) return hipErrorInvalidValue;
    tq::PtrTable gt{};
    tq::MutPtrTable stt{};
    for (int i = 0; i < count; ++i) { gt.p[i] = g[i]; stt.p[i] = stats[i]; }
    const uint64_t resident = dtype == TQ_BF16 ? tq::kStatsResidentGroups : tq::kStatsTargetGroups;
    const uint64_t tiles_per_tensor = (d + tq::kStatsTile - 1) / tq::kStatsTile;
    const uint64_t total_tiles = tiles_per_tensor * (uint64_t)count;
    const uint64_t fit = total_tiles * tq::kStatsTile / tq::kStatsMinSlice;       // shares of at least 16384 elements
    const uint32_t groups = (uint32_t)(fit < 1 ? 1 : (fit < resident ? fit : resident));
    const uint64_t rows = groups + nseg * (uint64_t)count;
    uint32_t* ws_hist = static_cast<uint32_t*>(workspace);
    tq::StatsExtra* ws_extra = reinterpret_cast<tq::StatsExtra*>(static_cast<char*>(workspace) + rows * TQ_NBINS * 4);
    dim3 rgrid;
    if (!tq::fold_grid(nseg * (uint64_t)count, tq::kStatsBlock, 1, rgrid)) return hipErrorInvalidValue;
#define TQ_LAUNCH_SEG_PARTIAL(DT, TL)                                                                              \
    hipLaunchKernelGGL((tq::tq_stats_segments_partial_kernel<DT, TL>), dim3(groups), dim3(tq::kStatsBlock), 0, st, gt, \
                       d, tiles_per_tensor, total_tiles, seg_off, (uint32_t)nseg, g_min, ws_hist, ws_extra)
    if (dtype == TQ_F32) {
        if (g_min > 0.0f) TQ_LAUNCH_SEG_PARTIAL(TQ_F32, true); else TQ_LAUNCH_SEG_PARTIAL(TQ_F32, false);
    } else {
        if (g_min > 0.0f) TQ_LAUNCH_SEG_PARTIAL(TQ_BF16, true); else TQ_LAUNCH_SEG_PARTIAL(TQ_BF16, false);
    }
#undef TQ_LAUNCH_SEG_PARTIAL
    hipError_t err = hipGetLastError();
    if (err != hipSuccess) return err;
    hipLaunchKernelGGL(tq::tq_stats_segments_reduce_kernel, rgrid, dim3(tq::kStatsBlock), 0, st, d, tiles_per_tensor,
                       total_tiles, groups, (uint32_t)count, seg_off, (uint32_t)nseg, g_min, ws_hist, ws_extra, rows, stt);
    return hipGetLastError();
}
