// C entry points of libtq: argument checks, then the launch helpers of the kernel files.
// Nothing here touches the data; every step of the path runs in the kernels.
#include <hip/hip_runtime.h>

#include "tq.h"

hipError_t tq_launch_stats(const void* const* g, int count, int dtype, uint64_t d, uint64_t bucket_elems,
                           float g_min, tq_stats_t* const* stats, void* workspace, hipStream_t st);
uint64_t tq_stats_workspace_bytes_impl(uint64_t d, uint64_t bucket_elems);
hipError_t tq_stats_static_scratch(void** out);
hipError_t tq_launch_params(const tq_stats_t* const* stats, int count, uint64_t nb, int bits, int grid,
                            float alpha_override, tq_params_t* const* params, hipStream_t st);
hipError_t tq_launch_compress(const void* const* g, int count, int dtype, uint64_t d, uint64_t bucket_elems,
                              const tq_params_t* const* params, int bits, int grid, uint64_t seed,
                              uint32_t first_worker, uint32_t step, void* const* payload, hipStream_t st);
hipError_t tq_launch_decode(const void* const* payload, const tq_params_t* const* params,
                            const float* weights, int N, uint64_t d, uint64_t bucket_elems, int bits,
                            int mode, float eta, float momentum, float weight_decay, float* velocity,
                            float* out, hipStream_t st);

hipError_t tq_launch_simulate(const void* g, int dtype, uint64_t d, uint64_t bucket_elems, const tq_params_t* params,
                              int bits, uint64_t seed, uint32_t worker, uint32_t step, int accumulate, float* out,
                              hipStream_t st);

uint64_t tq_stats_segments_workspace_bytes_impl(uint64_t d, uint64_t nseg);
hipError_t tq_launch_stats_segments(const void* const* g, int count, int dtype, uint64_t d, const uint64_t* seg_off,
                                    uint64_t nseg, float g_min, tq_stats_t* const* stats, void* workspace,
                                    hipStream_t st);
hipError_t tq_launch_compress_segments(const void* const* g, int count, int dtype, uint64_t d, const uint64_t* seg_off,
                                       const uint64_t* seg_host, uint64_t nseg, const tq_params_t* const* params, int bits, uint64_t seed,
                                       uint32_t first_worker, uint32_t step, void* const* payload, hipStream_t st);
hipError_t tq_launch_decode_segments(const void* const* payload, const tq_params_t* const* params,
                                     const float* weights, int N, uint64_t d, const uint64_t* seg_off,
                                     const uint64_t* seg_host, uint64_t nseg, int bits, int accumulate, float* out,
                                     hipStream_t st);

static_assert(sizeof(tq_stats_t) == 3632, "tq_stats_t layout is part of the interface");
static_assert(sizeof(tq_params_t) == 160, "tq_params_t layout is part of the interface");

namespace {

bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

int check_layout(uint64_t d, uint64_t bucket_elems)
{
    if (d == 0) return TQ_EINVAL;
    if (bucket_elems != 0 && bucket_elems % 128 != 0) return TQ_EINVAL;
    if (d > (1ull << 40)) return TQ_EUNSUPPORTED;
    return TQ_OK;
}

int check_dtype(int dtype) { return (dtype == TQ_F32 || dtype == TQ_BF16) ? TQ_OK : TQ_EINVAL; }
int check_bits(int bits) { return (bits >= 2 && bits <= 4) ? TQ_OK : TQ_EINVAL; }
int check_grid(int grid)
{
    return (grid == TQ_GRID_UNIFORM || grid == TQ_GRID_NONUNIFORM || grid == TQ_GRID_BISCALED) ? TQ_OK : TQ_EINVAL;
}
int from_hip(hipError_t e) { return e == hipSuccess ? TQ_OK : (e == hipErrorInvalidValue ? TQ_EUNSUPPORTED : TQ_EHIP); }

}  // namespace

extern "C" {

uint64_t tq_num_buckets(uint64_t d, uint64_t bucket_elems)
{
    if (d == 0) return 0;
    if (bucket_elems == 0) return 1;
    return (d + bucket_elems - 1) / bucket_elems;
}

uint64_t tq_payload_bytes(uint64_t d, int bits)
{
    const uint64_t nbytes = (d * (uint64_t)bits + 7) / 8;
    return (nbytes + 15) / 16 * 16;
}

uint64_t tq_stats_workspace_bytes(uint64_t d, uint64_t bucket_elems)
{
    if (check_layout(d, bucket_elems) != TQ_OK) return 0;
    return tq_stats_workspace_bytes_impl(d, bucket_elems);
}

int tq_stats_multi(const void* const* g_host, int count, int dtype, uint64_t d, uint64_t bucket_elems,
                   float g_min, tq_stats_t* const* stats_host, void* workspace_dev, uint64_t workspace_bytes,
                   void* stream)
{
    int rc;
    if ((rc = check_layout(d, bucket_elems)) || (rc = check_dtype(dtype))) return rc;
    if (count < 1 || !g_host || !stats_host || !workspace_dev) return TQ_EINVAL;
    if (count > TQ_MAX_WORKERS) return TQ_EUNSUPPORTED;
    // the counts of tq_stats_t are 32-bit: one bucket holds fewer than 2^32 elements
    if ((bucket_elems ? (bucket_elems < d ? bucket_elems : d) : d) > 0xFFFFFFFFull) return TQ_EUNSUPPORTED;
    if (workspace_bytes < (uint64_t)count * tq_stats_workspace_bytes_impl(d, bucket_elems)) return TQ_EINVAL;
    if (g_min != g_min || (g_min > 0.0f && g_min < 9.094947017729282e-13f) || g_min > 3.0e38f) return TQ_EINVAL;
    if (!aligned16(workspace_dev)) return TQ_EALIGN;
    for (int i = 0; i < count; ++i) {
        if (!g_host[i] || !stats_host[i]) return TQ_EINVAL;
        if (!aligned16(g_host[i]) || !aligned16(stats_host[i])) return TQ_EALIGN;
    }
    return from_hip(tq_launch_stats(g_host, count, dtype, d, bucket_elems, g_min, stats_host, workspace_dev,
                                    static_cast<hipStream_t>(stream)));
}

int tq_stats(const void* g_dev, int dtype, uint64_t d, uint64_t bucket_elems, float g_min,
             tq_stats_t* stats_dev, void* workspace_dev, uint64_t workspace_bytes, void* stream)
{
    return tq_stats_multi(&g_dev, 1, dtype, d, bucket_elems, g_min, &stats_dev, workspace_dev, workspace_bytes,
                          stream);
}

int tq_stats_static(const void* g_dev, int dtype, uint64_t d, uint64_t bucket_elems, float g_min,
                    tq_stats_t* stats_dev, void* stream)
{
    int rc;
    if ((rc = check_layout(d, bucket_elems)) || (rc = check_dtype(dtype))) return rc;
    if (tq_stats_workspace_bytes_impl(d, bucket_elems) > TQ_STATS_STATIC_SCRATCH_BYTES) return TQ_EUNSUPPORTED;
    void* ws = nullptr;
    if (tq_stats_static_scratch(&ws) != hipSuccess) return TQ_EHIP;
    // the remaining checks, and the launch, are tq_stats's own
    return tq_stats_multi(&g_dev, 1, dtype, d, bucket_elems, g_min, &stats_dev, ws,
                          TQ_STATS_STATIC_SCRATCH_BYTES, stream);
}

int tq_params_multi(const tq_stats_t* const* stats_host, int count, uint64_t nb, int bits, int grid,
                    float alpha_override, tq_params_t* const* params_host, void* stream)
{
    int rc;
    if ((rc = check_bits(bits))) return rc;
    if ((rc = check_grid(grid))) return rc;
    if (nb == 0 || count < 1 || !stats_host || !params_host) return TQ_EINVAL;
    if (count > TQ_MAX_WORKERS) return TQ_EUNSUPPORTED;
    if (alpha_override != alpha_override || alpha_override > 3.0e38f) return TQ_EINVAL;
    for (int i = 0; i < count; ++i) {
        if (!stats_host[i] || !params_host[i]) return TQ_EINVAL;
        if (!aligned16(stats_host[i]) || !aligned16(params_host[i])) return TQ_EALIGN;
    }
    return from_hip(tq_launch_params(stats_host, count, nb, bits, grid, alpha_override, params_host,
                                     static_cast<hipStream_t>(stream)));
}

int tq_params(const tq_stats_t* stats_dev, uint64_t nb, int bits, int grid, float alpha_override,
              tq_params_t* params_dev, void* stream)
{
    return tq_params_multi(&stats_dev, 1, nb, bits, grid, alpha_override, &params_dev, stream);
}

int tq_compress_multi(const void* const* g_host, int count, int dtype, uint64_t d, uint64_t bucket_elems,
                      const tq_params_t* const* params_host, int bits, int grid, uint64_t seed,
                      uint32_t first_worker, uint32_t step, void* const* payload_host, void* stream)
{
    int rc;
    if ((rc = check_layout(d, bucket_elems)) || (rc = check_dtype(dtype)) || (rc = check_bits(bits))) return rc;
    if ((rc = check_grid(grid))) return rc;
    if (count < 1 || !g_host || !params_host || !payload_host) return TQ_EINVAL;
    if (count > TQ_MAX_WORKERS) return TQ_EUNSUPPORTED;
    for (int i = 0; i < count; ++i) {
        if (!g_host[i] || !params_host[i] || !payload_host[i]) return TQ_EINVAL;
        if (!aligned16(g_host[i]) || !aligned16(params_host[i]) || !aligned16(payload_host[i])) return TQ_EALIGN;
    }
    return from_hip(tq_launch_compress(g_host, count, dtype, d, bucket_elems, params_host, bits, grid, seed,
                                       first_worker, step, payload_host, static_cast<hipStream_t>(stream)));
}

int tq_compress(const void* g_dev, int dtype, uint64_t d, uint64_t bucket_elems,
                const tq_params_t* params_dev, int bits, int grid, uint64_t seed, uint32_t worker, uint32_t step,
                void* payload_dev, void* stream)
{
    return tq_compress_multi(&g_dev, 1, dtype, d, bucket_elems, &params_dev, bits, grid, seed, worker, step,
                             &payload_dev, stream);
}

int tq_quantize_dequantize(const void* g_dev, int dtype, uint64_t d, uint64_t bucket_elems,
                           const tq_params_t* params_dev, int bits, uint64_t seed, uint32_t worker, uint32_t step,
                           int accumulate, float* out_dev, void* stream)
{
    int rc;
    if ((rc = check_layout(d, bucket_elems)) || (rc = check_dtype(dtype)) || (rc = check_bits(bits))) return rc;
    if (!g_dev || !params_dev || !out_dev) return TQ_EINVAL;
    if (!aligned16(g_dev) || !aligned16(params_dev) || !aligned16(out_dev)) return TQ_EALIGN;
    return from_hip(tq_launch_simulate(g_dev, dtype, d, bucket_elems, params_dev, bits, seed, worker, step,
                                       accumulate ? 1 : 0, out_dev, static_cast<hipStream_t>(stream)));
}

// Checks shared by the two server-side calls.
static int check_decode(const void* const* payload_host, const tq_params_t* const* params_host,
                        const float* weights_host, int N, uint64_t d, uint64_t bucket_elems, int bits,
                        const float* out_dev)
{
    int rc;
    if ((rc = check_layout(d, bucket_elems)) || (rc = check_bits(bits))) return rc;
    if (N < 1 || !payload_host || !params_host || !out_dev) return TQ_EINVAL;
    if (N > TQ_MAX_WORKERS) return TQ_EUNSUPPORTED;
    if (!aligned16(out_dev)) return TQ_EALIGN;
    for (int i = 0; i < N; ++i) {
        if (!payload_host[i] || !params_host[i]) return TQ_EINVAL;
        if (!aligned16(payload_host[i]) || !aligned16(params_host[i])) return TQ_EALIGN;
        if (weights_host && weights_host[i] != weights_host[i]) return TQ_EINVAL;
    }
    return TQ_OK;
}

int tq_decompress_aggregate(const void* const* payload_host, const tq_params_t* const* params_host,
                            const float* weights_host, int N, uint64_t d, uint64_t bucket_elems, int bits,
                            int accumulate, float* out_dev, void* stream)
{
    const int rc = check_decode(payload_host, params_host, weights_host, N, d, bucket_elems, bits, out_dev);
    if (rc) return rc;
    return from_hip(tq_launch_decode(payload_host, params_host, weights_host, N, d, bucket_elems, bits,
                                     accumulate ? 1 : 0, 0.0f, 0.0f, 0.0f, nullptr, out_dev,
                                     static_cast<hipStream_t>(stream)));
}

int tq_decompress_aggregate_update(const void* const* payload_host, const tq_params_t* const* params_host,
                                   const float* weights_host, int N, uint64_t d, uint64_t bucket_elems,
                                   int bits, float eta, float momentum, float weight_decay, float* theta_dev,
                                   float* velocity_dev, void* stream)
{
    const int rc = check_decode(payload_host, params_host, weights_host, N, d, bucket_elems, bits, theta_dev);
    if (rc) return rc;
    if (eta != eta || momentum != momentum || weight_decay != weight_decay) return TQ_EINVAL;
    if (velocity_dev && !aligned16(velocity_dev)) return TQ_EALIGN;
    if (velocity_dev == theta_dev) return TQ_EINVAL;
    return from_hip(tq_launch_decode(payload_host, params_host, weights_host, N, d, bucket_elems, bits,
                                     velocity_dev ? 3 : 2, eta, momentum, weight_decay, velocity_dev, theta_dev,
                                     static_cast<hipStream_t>(stream)));
}

// Checks shared by the three segment calls: sizes, the device table's alignment and, when the
// caller also passes the table in host memory, the table itself.
static int check_segments(uint64_t d, const uint64_t* seg_dev, const uint64_t* seg_host, uint64_t nseg)
{
    if (d == 0 || nseg == 0 || !seg_dev) return TQ_EINVAL;
    if (d > (1ull << 40) || nseg > 0xFFFFFFFFull) return TQ_EUNSUPPORTED;
    if (reinterpret_cast<uintptr_t>(seg_dev) & 7u) return TQ_EALIGN;
    if (seg_host) {
        if (seg_host[0] != 0 || seg_host[nseg] != d) return TQ_EINVAL;
        for (uint64_t s = 0; s < nseg; ++s) {
            if (seg_host[s + 1] <= seg_host[s]) return TQ_EINVAL;
            if (s + 1 < nseg && seg_host[s + 1] % 128 != 0) return TQ_EINVAL;
        }
    }
    return TQ_OK;
}

uint64_t tq_stats_segments_workspace_bytes(uint64_t d, uint64_t nseg)
{
    if (d == 0 || nseg == 0 || d > (1ull << 40) || nseg > 0xFFFFFFFFull) return 0;
    return tq_stats_segments_workspace_bytes_impl(d, nseg);
}

int tq_stats_segments_multi(const void* const* g_host, int count, int dtype, uint64_t d,
                            const uint64_t* seg_offsets_dev, const uint64_t* seg_offsets_host, uint64_t nseg,
                            float g_min, tq_stats_t* const* stats_host, void* workspace_dev, uint64_t workspace_bytes,
                            void* stream)
{
    int rc;
    if ((rc = check_segments(d, seg_offsets_dev, seg_offsets_host, nseg)) || (rc = check_dtype(dtype))) return rc;
    if (count < 1 || !g_host || !stats_host || !workspace_dev) return TQ_EINVAL;
    if (count > TQ_MAX_WORKERS || nseg * (uint64_t)count > 0xFFFFFFFFull) return TQ_EUNSUPPORTED;
    if (d > 0xFFFFFFFFull) return TQ_EUNSUPPORTED;          // the counts of tq_stats_t are 32-bit
    if (workspace_bytes < (uint64_t)count * tq_stats_segments_workspace_bytes_impl(d, nseg)) return TQ_EINVAL;
    if (g_min != g_min || (g_min > 0.0f && g_min < 9.094947017729282e-13f) || g_min > 3.0e38f) return TQ_EINVAL;
    if (!aligned16(workspace_dev)) return TQ_EALIGN;
    for (int i = 0; i < count; ++i) {
        if (!g_host[i] || !stats_host[i]) return TQ_EINVAL;
        if (!aligned16(g_host[i]) || !aligned16(stats_host[i])) return TQ_EALIGN;
    }
    return from_hip(tq_launch_stats_segments(g_host, count, dtype, d, seg_offsets_dev, nseg, g_min, stats_host,
                                             workspace_dev, static_cast<hipStream_t>(stream)));
}

int tq_stats_segments(const void* g_dev, int dtype, uint64_t d, const uint64_t* seg_offsets_dev,
                      const uint64_t* seg_offsets_host, uint64_t nseg, float g_min, tq_stats_t* stats_dev,
                      void* workspace_dev, uint64_t workspace_bytes, void* stream)
{
    return tq_stats_segments_multi(&g_dev, 1, dtype, d, seg_offsets_dev, seg_offsets_host, nseg, g_min, &stats_dev,
                                   workspace_dev, workspace_bytes, stream);
}

int tq_compress_segments_multi(const void* const* g_host, int count, int dtype, uint64_t d,
                               const uint64_t* seg_offsets_dev, const uint64_t* seg_offsets_host, uint64_t nseg,
                               const tq_params_t* const* params_host, int bits, uint64_t seed, uint32_t first_worker,
                               uint32_t step, void* const* payload_host, void* stream)
{
    int rc;
    if ((rc = check_segments(d, seg_offsets_dev, seg_offsets_host, nseg)) || (rc = check_dtype(dtype)) ||
        (rc = check_bits(bits)))
        return rc;
    if (count < 1 || !g_host || !params_host || !payload_host) return TQ_EINVAL;
    if (count > TQ_MAX_WORKERS) return TQ_EUNSUPPORTED;
    for (int i = 0; i < count; ++i) {
        if (!g_host[i] || !params_host[i] || !payload_host[i]) return TQ_EINVAL;
        if (!aligned16(g_host[i]) || !aligned16(params_host[i]) || !aligned16(payload_host[i])) return TQ_EALIGN;
    }
    return from_hip(tq_launch_compress_segments(g_host, count, dtype, d, seg_offsets_dev, seg_offsets_host, nseg, params_host, bits, seed,
                                                first_worker, step, payload_host, static_cast<hipStream_t>(stream)));
}

int tq_compress_segments(const void* g_dev, int dtype, uint64_t d, const uint64_t* seg_offsets_dev,
                         const uint64_t* seg_offsets_host, uint64_t nseg, const tq_params_t* params_dev, int bits,
                         uint64_t seed, uint32_t worker, uint32_t step, void* payload_dev, void* stream)
{
    return tq_compress_segments_multi(&g_dev, 1, dtype, d, seg_offsets_dev, seg_offsets_host, nseg, &params_dev, bits,
                                      seed, worker, step, &payload_dev, stream);
}

int tq_decompress_aggregate_segments(const void* const* payload_host, const tq_params_t* const* params_host,
                                     const float* weights_host, int N, uint64_t d, const uint64_t* seg_offsets_dev,
                                     const uint64_t* seg_offsets_host, uint64_t nseg, int bits, int accumulate,
                                     float* out_dev, void* stream)
{
    int rc;
    if ((rc = check_segments(d, seg_offsets_dev, seg_offsets_host, nseg))) return rc;
    if ((rc = check_decode(payload_host, params_host, weights_host, N, d, 0, bits, out_dev))) return rc;
    return from_hip(tq_launch_decode_segments(payload_host, params_host, weights_host, N, d, seg_offsets_dev,
                                              seg_offsets_host, nseg,
                                              bits, accumulate ? 1 : 0, out_dev, static_cast<hipStream_t>(stream)));
}

const char* tq_strerror(int code)
{
    switch (code) {
        case TQ_OK: return "ok";
        case TQ_EINVAL: return "invalid argument";
        case TQ_EALIGN: return "device pointer not 16-byte aligned";
        case TQ_EUNSUPPORTED: return "size not supported";
        case TQ_EHIP: return "HIP launch failed";
        default: return "unknown error";
    }
}

}  // extern "C"
