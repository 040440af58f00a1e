// C entry points of libtq: argument checks, then the launch helpers of the kernel files.
// Nothing here touches the data; every step of the path runs in the kernels.
#include <hip/hip_runtime.h>

#include "tq.h"

hipError_t tq_launch_stats(const void* g, int dtype, uint64_t d, uint64_t bucket_elems, float g_min,
                           tq_stats_t* stats, hipStream_t st);
hipError_t tq_launch_params(const tq_stats_t* stats, uint64_t nb, int bits, int grid, float alpha_override,
                            tq_params_t* params, hipStream_t st);
hipError_t tq_launch_compress(const void* g, int dtype, uint64_t d, uint64_t bucket_elems,
                              const tq_params_t* params, int bits, uint64_t seed, uint32_t worker,
                              uint32_t step, void* payload, hipStream_t st);
hipError_t tq_launch_decode(const void* const* payload, const tq_params_t* const* params,
                            const float* weights, int N, uint64_t d, uint64_t bucket_elems, int bits,
                            int accumulate, float* out, hipStream_t st);

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

int tq_stats(const void* g_dev, int dtype, uint64_t d, uint64_t bucket_elems, float g_min,
             tq_stats_t* stats_dev, void* stream)
{
    int rc;
    if ((rc = check_layout(d, bucket_elems)) || (rc = check_dtype(dtype))) return rc;
    if (!g_dev || !stats_dev) return TQ_EINVAL;
    if (g_min != g_min || (g_min > 0.0f && g_min < 9.094947017729282e-13f) || g_min > 3.0e38f) return TQ_EINVAL;
    if (!aligned16(g_dev) || !aligned16(stats_dev)) return TQ_EALIGN;
    return from_hip(tq_launch_stats(g_dev, dtype, d, bucket_elems, g_min, stats_dev,
                                    static_cast<hipStream_t>(stream)));
}

int tq_params(const tq_stats_t* stats_dev, uint64_t nb, int bits, int grid, float alpha_override,
              tq_params_t* params_dev, void* stream)
{
    int rc;
    if ((rc = check_bits(bits))) return rc;
    if (grid != TQ_GRID_UNIFORM && grid != TQ_GRID_NONUNIFORM) return TQ_EINVAL;
    if (nb == 0 || !stats_dev || !params_dev) return TQ_EINVAL;
    if (alpha_override != alpha_override || alpha_override > 3.0e38f) return TQ_EINVAL;
    if (!aligned16(stats_dev) || !aligned16(params_dev)) return TQ_EALIGN;
    return from_hip(tq_launch_params(stats_dev, nb, bits, grid, alpha_override, params_dev,
                                     static_cast<hipStream_t>(stream)));
}

int tq_compress(const void* g_dev, int dtype, uint64_t d, uint64_t bucket_elems,
                const tq_params_t* params_dev, int bits, uint64_t seed, uint32_t worker, uint32_t step,
                void* payload_dev, void* stream)
{
    int rc;
    if ((rc = check_layout(d, bucket_elems)) || (rc = check_dtype(dtype)) || (rc = check_bits(bits))) return rc;
    if (!g_dev || !params_dev || !payload_dev) return TQ_EINVAL;
    if (!aligned16(g_dev) || !aligned16(params_dev) || !aligned16(payload_dev)) return TQ_EALIGN;
    return from_hip(tq_launch_compress(g_dev, dtype, d, bucket_elems, params_dev, bits, seed, worker, step,
                                       payload_dev, static_cast<hipStream_t>(stream)));
}

int tq_decompress_aggregate(const void* const* payload_host, const tq_params_t* const* params_host,
                            const float* weights_host, int N, uint64_t d, uint64_t bucket_elems, int bits,
                            int accumulate, float* out_dev, void* stream)
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
    return from_hip(tq_launch_decode(payload_host, params_host, weights_host, N, d, bucket_elems, bits,
                                     accumulate ? 1 : 0, out_dev, static_cast<hipStream_t>(stream)));
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
