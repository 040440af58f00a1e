// tq_decompress_aggregate: Alg. 1 server step of arXiv 2402.01798,
//   out[e] = sum_i w_i * L_i[code_i(e)],
// for all N workers in one pass.  Each lane owns 8 consecutive output elements: it reads the
// b bytes that hold their codes from every worker's stream, looks the levels up in LDS, adds
// them in worker order and writes 32 contiguous bytes of fp32 once.
//
// Two kernels share that shape:
//   tq_decode_pair_kernel  the fast path: per worker a table indexed by TWO adjacent codes
//                          (2^(2b) entries of float2), so one 8-byte LDS read serves two
//                          elements; a workgroup owns four tiles and requests all their code
//                          words before anything else.
//   tq_decode_kernel       the general path (any N up to 64 at any b): one 4-byte LDS read
//                          per code from the plain 16-entry tables.
#include <type_traits>

#include "tq_device.h"

namespace tq {

struct DecodeArgs {
    const uint8_t* payload[TQ_MAX_WORKERS];
    const tq_params_t* params[TQ_MAX_WORKERS];
    float weight[TQ_MAX_WORKERS];
};

// The 8 codes of group q (b bytes at byte q*b), little-endian in the low 8b bits.
template <int BITS>
__device__ __forceinline__ uint32_t load_codes(const uint8_t* p, bool room_for_dword)
{
    if constexpr (BITS == 4) return *reinterpret_cast<const uint32_t*>(p);
    if constexpr (BITS == 2) return *reinterpret_cast<const uint16_t*>(p);
    // 3 bytes at an odd offset: one unaligned dword load.  The very last group of a payload
    // may have no fourth byte after it; it reads the dword that ends with its third byte.
    const uint8_t* q = room_for_dword ? p : p - 1;
    uint32_t w;
    __builtin_memcpy(&w, q, 4);
    w = room_for_dword ? w : w >> 8;
    return w & 0x00FFFFFFu;
}

__device__ __forceinline__ void store_group(float* o, const float (&acc)[8], uint64_t e0, uint64_t d, int accumulate)
{
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
    } else {                                  // ragged end of the tensor
        const int n_valid = (int)(d - e0);
#pragma unroll
        for (int j = 0; j < 8; ++j)
            if (j < n_valid) o[j] = accumulate ? o[j] + acc[j] : acc[j];
    }
}

// Plain level tables of one bucket: row i = worker i's 16 levels, pre-multiplied by w_i
// when explicit weights are given (one rounding per level, as the weighted sum is defined).
__device__ __forceinline__ void fill_level_rows(float* table, const DecodeArgs& args, int N, int weighted,
                                                uint64_t bucket)
{
    for (int idx = threadIdx.x; idx < N * 16; idx += kBlock) {
        const int i = idx >> 4;
        float l = args.params[i][bucket].level[idx & 15];
        if (weighted) l = args.weight[i] * l;
        table[idx] = l;
    }
}

// The kernel is bound by how many bytes a wavefront keeps in flight per memory round trip,
// not by arithmetic: a workgroup therefore owns T consecutive tiles and requests the code
// words of all of them (U workers at a time, U a divisor of N so that no branch sits between
// the loads) before it builds its tables; the round trip that fetches the levels overlaps
// with the one that fetches the codes.  Nothing is stored before the last load has been
// consumed: on this ISA loads and stores retire through one in-order counter, so a wave that
// stored a tile and then waited for further loads would wait for its own stores to land.
template <int BITS, int T, int U>
__global__ __launch_bounds__(kBlock) void tq_decode_pair_kernel(
    const DecodeArgs args, int N, int weighted, float scale, uint64_t d, uint64_t d_pad, uint64_t bucket_elems,
    uint32_t groups_per_bucket, int accumulate, uint64_t payload_bytes, float* __restrict__ out)
{
    constexpr int PAIRS = 1 << (2 * BITS);
    constexpr uint32_t PMASK = PAIRS - 1;
    extern __shared__ float2 pair_tab[];                       // [N][PAIRS]
    __shared__ float rows[TQ_MAX_WORKERS * 16];

    const uint32_t bucket = blockIdx.x / groups_per_bucket;
    const uint32_t grp = blockIdx.x - bucket * groups_per_bucket;
    const uint64_t bstart = (uint64_t)bucket * bucket_elems;
    uint64_t bend = bstart + bucket_elems < d_pad ? bstart + bucket_elems : d_pad;
    bend = bend < d ? bend : d;
    const uint64_t gstart = bstart + (uint64_t)grp * T * kTile;
    if (gstart >= bend) return;

    // This lane's group in each of the T tiles.  Lanes past the end of the bucket read group 0
    // of the payload (always present) and store nothing.
    uint64_t e0[T], off[T];
    bool room[T];
#pragma unroll
    for (int t = 0; t < T; ++t) {
        e0[t] = gstart + (uint64_t)t * kTile + (uint64_t)threadIdx.x * kGroup;
        off[t] = e0[t] < bend ? (e0[t] >> 3) * (uint64_t)BITS : 0;
        room[t] = off[t] + 4 <= payload_bytes;
    }
    auto request = [&](uint32_t (&w)[T][U], int c) {
#pragma unroll
        for (int u = 0; u < U; ++u)
#pragma unroll
            for (int t = 0; t < T; ++t) w[t][u] = load_codes<BITS>(args.payload[U * c + u] + off[t], room[t]);
    };

    uint32_t w[T][U];
    request(w, 0);                                             // in flight while the tables are built

    fill_level_rows(rows, args, N, weighted, bucket);
    __syncthreads();
    for (int idx = threadIdx.x; idx < N * PAIRS; idx += kBlock) {
        const float* r = rows + (idx / PAIRS) * 16;
        const int e = idx & PMASK;
        pair_tab[idx] = make_float2(r[e & ((1 << BITS) - 1)], r[e >> BITS]);
    }
    __syncthreads();

    float acc[T][8];
#pragma unroll
    for (int t = 0; t < T; ++t)
#pragma unroll
        for (int j = 0; j < 8; ++j) acc[t][j] = 0.0f;

    const int n_chunks = N / U;
    for (int c = 0; c < n_chunks; ++c) {
        if (c > 0) request(w, c);
        const float2* row0 = pair_tab + U * c * PAIRS;
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const float2* row = row0 + u * PAIRS;
#pragma unroll
            for (int t = 0; t < T; ++t)
#pragma unroll
                for (int m = 0; m < 4; ++m) {
                    const float2 v = row[(w[t][u] >> (2 * BITS * m)) & PMASK];
                    acc[t][2 * m] = acc[t][2 * m] + v.x;
                    acc[t][2 * m + 1] = acc[t][2 * m + 1] + v.y;
                }
        }
    }

#pragma unroll
    for (int t = 0; t < T; ++t) {
        if (!weighted) {
#pragma unroll
            for (int j = 0; j < 8; ++j) acc[t][j] = acc[t][j] * scale;
        }
        if (e0[t] < bend) store_group(out + e0[t], acc[t], e0[t], d, accumulate);
    }
}

template <int BITS>
__global__ __launch_bounds__(kBlock) void tq_decode_kernel(
    const DecodeArgs args, int N, int weighted, float scale, uint64_t d, uint64_t d_pad,
    uint64_t bucket_elems, uint32_t tiles_per_bucket, int accumulate, uint64_t payload_bytes,
    float* __restrict__ out)
{
    constexpr uint32_t MASK = (1u << BITS) - 1u;
    const TileGeom t = tile_geom(blockIdx.x, d_pad, bucket_elems, tiles_per_bucket);
    if (t.ebase >= t.eend) return;

    __shared__ float table[TQ_MAX_WORKERS * 16];
    fill_level_rows(table, args, N, weighted, t.bucket);
    __syncthreads();

    const uint64_t e0 = t.ebase + (uint64_t)threadIdx.x * kGroup;
    if (e0 >= t.eend || e0 >= d) return;
    const uint64_t byte_off = (e0 >> 3) * (uint64_t)BITS;
    const bool room = byte_off + 4 <= payload_bytes;

    float acc[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) acc[j] = 0.0f;
    for (int i = 0; i < N; ++i) {
        const uint32_t w = load_codes<BITS>(args.payload[i] + byte_off, room);
        const float* row = table + i * 16;
#pragma unroll
        for (int j = 0; j < 8; ++j) acc[j] = acc[j] + row[(w >> (j * BITS)) & MASK];
    }
    if (!weighted) {
#pragma unroll
        for (int j = 0; j < 8; ++j) acc[j] = acc[j] * scale;
    }
    store_group(out + e0, acc, e0, d, accumulate);
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
    const uint64_t tpb = (be + tq::kTile - 1) / tq::kTile;             // tiles per bucket
    const uint64_t pbytes = tq_payload_bytes(d, bits);
    const int weighted = weights ? 1 : 0;
    const dim3 threads(tq::kBlock);

    const size_t pair_lds = (size_t)N * (1u << (2 * bits)) * sizeof(float2);
    if (pair_lds <= 48 * 1024) {
        constexpr int T = 4;                                           // tiles per workgroup
        const uint64_t gpb = (tpb + T - 1) / T;
        const uint64_t nblocks = nb * gpb;
        if (nblocks == 0 || nblocks > 0x7FFFFFFFull) return hipErrorInvalidValue;
        const dim3 blocks((unsigned)nblocks);
        const int U = N % 8 == 0 ? 8 : (N % 4 == 0 ? 4 : (N % 2 == 0 ? 2 : 1));
#define TQ_LAUNCH_PAIR(B, UU)                                                                             \
    hipLaunchKernelGGL((tq::tq_decode_pair_kernel<B, T, UU>), blocks, threads, pair_lds, st, args, N, weighted, \
                       scale, d, d_pad, be, (uint32_t)gpb, accumulate, pbytes, out)
#define TQ_LAUNCH_PAIR_U(B)                  \
    switch (U) {                             \
        case 8: TQ_LAUNCH_PAIR(B, 8); break; \
        case 4: TQ_LAUNCH_PAIR(B, 4); break; \
        case 2: TQ_LAUNCH_PAIR(B, 2); break; \
        default: TQ_LAUNCH_PAIR(B, 1); break; \
    }
        switch (bits) {
            case 2: TQ_LAUNCH_PAIR_U(2) break;
            case 3: TQ_LAUNCH_PAIR_U(3) break;
            default: TQ_LAUNCH_PAIR_U(4) break;
        }
#undef TQ_LAUNCH_PAIR_U
#undef TQ_LAUNCH_PAIR
        return hipGetLastError();
    }

    const uint64_t nblocks = nb * tpb;
    if (nblocks == 0 || nblocks > 0x7FFFFFFFull) return hipErrorInvalidValue;
    const dim3 blocks((unsigned)nblocks);
    switch (bits) {
        case 2:
            hipLaunchKernelGGL((tq::tq_decode_kernel<2>), blocks, threads, 0, st, args, N, weighted, scale, d,
                               d_pad, be, (uint32_t)tpb, accumulate, pbytes, out);
            break;
        case 3:
            hipLaunchKernelGGL((tq::tq_decode_kernel<3>), blocks, threads, 0, st, args, N, weighted, scale, d,
                               d_pad, be, (uint32_t)tpb, accumulate, pbytes, out);
            break;
        default:
            hipLaunchKernelGGL((tq::tq_decode_kernel<4>), blocks, threads, 0, st, args, N, weighted, scale, d,
                               d_pad, be, (uint32_t)tpb, accumulate, pbytes, out);
            break;
    }
    return hipGetLastError();
}
