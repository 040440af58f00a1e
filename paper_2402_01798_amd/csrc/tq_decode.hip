// tq_decompress_aggregate: Alg. 1 server step of arXiv 2402.01798,
//   out[e] = sum_i w_i * L_i[code_i(e)],
// for all N workers in one pass: each lane owns 8 consecutive output elements, reads the b
// bytes that hold their codes from every worker's stream, looks the levels up in LDS and
// writes 32 bytes of fp32 once.
#include "tq_device.h"

namespace tq {

struct DecodeArgs {
    const uint8_t* payload[TQ_MAX_WORKERS];
    const tq_params_t* params[TQ_MAX_WORKERS];
    float weight[TQ_MAX_WORKERS];
};

template <int BITS>
__device__ __forceinline__ uint32_t load_codes(const uint8_t* p)
{
    if constexpr (BITS == 4) return *reinterpret_cast<const uint32_t*>(p);
    if constexpr (BITS == 2) return *reinterpret_cast<const uint16_t*>(p);
    return (uint32_t)p[0] | ((uint32_t)p[1] << 8) | ((uint32_t)p[2] << 16);
}

template <int BITS>
__global__ __launch_bounds__(kBlock) void tq_decode_kernel(
    const DecodeArgs args, int N, int weighted, float scale, uint64_t d, uint64_t d_pad,
    uint64_t bucket_elems, uint32_t tiles_per_bucket, int accumulate, float* __restrict__ out)
{
    constexpr uint32_t MASK = (1u << BITS) - 1u;
    const TileGeom t = tile_geom(blockIdx.x, d_pad, bucket_elems, tiles_per_bucket);
    if (t.ebase >= t.eend) return;

    // Level tables of this bucket, one row of 16 per worker, pre-multiplied by w_i when
    // explicit weights are given (one rounding per level, as the sum is defined).
    __shared__ float table[TQ_MAX_WORKERS * 16];
    for (int idx = threadIdx.x; idx < N * 16; idx += kBlock) {
        const int i = idx >> 4;
        float l = args.params[i][t.bucket].level[idx & 15];
        if (weighted) l = args.weight[i] * l;
        table[idx] = l;
    }
    __syncthreads();

    const uint64_t e0 = t.ebase + (uint64_t)threadIdx.x * kGroup;
    if (e0 >= t.eend || e0 >= d) return;
    const uint64_t byte_off = (e0 >> 3) * (uint64_t)BITS;

    float acc[8];
    {
        const uint32_t w = load_codes<BITS>(args.payload[0] + byte_off);
#pragma unroll
        for (int j = 0; j < 8; ++j) acc[j] = table[(w >> (j * BITS)) & MASK];
    }
    for (int i = 1; i < N; ++i) {
        const uint32_t w = load_codes<BITS>(args.payload[i] + byte_off);
        const float* row = table + i * 16;
#pragma unroll
        for (int j = 0; j < 8; ++j) acc[j] = acc[j] + row[(w >> (j * BITS)) & MASK];
    }
    if (!weighted) {
#pragma unroll
        for (int j = 0; j < 8; ++j) acc[j] = acc[j] * scale;
    }

    float* o = out + e0;
    if (e0 + kGroup <= d) {
        float4* o4 = reinterpret_cast<float4*>(o);
        float4 a = make_float4(acc[0], acc[1], acc[2], acc[3]);
        float4 b = make_float4(acc[4], acc[5], acc[6], acc[7]);
        if (accumulate) {
            const float4 pa = o4[0], pb = o4[1];
            a.x = pa.x + a.x; a.y = pa.y + a.y; a.z = pa.z + a.z; a.w = pa.w + a.w;
            b.x = pb.x + b.x; b.y = pb.y + b.y; b.z = pb.z + b.z; b.w = pb.w + b.w;
        }
        o4[0] = a;
        o4[1] = b;
    } else {
        const int n_valid = (int)(d - e0);
#pragma unroll
        for (int j = 0; j < 8; ++j)
            if (j < n_valid) o[j] = accumulate ? o[j] + acc[j] : acc[j];
    }
}

}  // namespace tq

// Host side of tq_decompress_aggregate after the argument checks of the C entry point.
hipError_t tq_launch_decode(const void* const* payload, const tq_params_t* const* params,
                            const float* weights, int N, uint64_t d, uint64_t bucket_elems, int bits,
                            int accumulate, float* out, hipStream_t st)
{
    tq::DecodeArgs args;
    for (int i = 0; i < TQ_MAX_WORKERS; ++i) {
        args.payload[i] = i < N ? static_cast<const uint8_t*>(payload[i]) : nullptr;
        args.params[i] = i < N ? params[i] : nullptr;
        args.weight[i] = (i < N && weights) ? weights[i] : 0.0f;
    }
    const float scale = 1.0f / (float)N;
    const uint64_t d_pad = (d + 127) / 128 * 128;
    const uint64_t be = bucket_elems ? bucket_elems : d_pad;
    const uint64_t nb = (d_pad + be - 1) / be;
    const uint64_t tpb = (be + tq::kTile - 1) / tq::kTile;
    const uint64_t nblocks = nb * tpb;
    if (nblocks == 0 || nblocks > 0x7FFFFFFFull) return hipErrorInvalidValue;
    const dim3 blocks((unsigned)nblocks), threads(tq::kBlock);
    const int weighted = weights ? 1 : 0;
    switch (bits) {
        case 2:
            hipLaunchKernelGGL((tq::tq_decode_kernel<2>), blocks, threads, 0, st, args, N, weighted, scale, d,
                               d_pad, be, (uint32_t)tpb, accumulate, out);
            break;
        case 3:
            hipLaunchKernelGGL((tq::tq_decode_kernel<3>), blocks, threads, 0, st, args, N, weighted, scale, d,
                               d_pad, be, (uint32_t)tpb, accumulate, out);
            break;
        default:
            hipLaunchKernelGGL((tq::tq_decode_kernel<4>), blocks, threads, 0, st, args, N, weighted, scale, d,
                               d_pad, be, (uint32_t)tpb, accumulate, out);
            break;
    }
    return hipGetLastError();
}
