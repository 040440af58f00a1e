// tq_decompress_aggregate: Alg. 1 server step of arXiv 2402.01798,
//   out[e] = sum_i w_i * L_i[code_i(e)],
// for all N workers in one pass.  Each lane owns 8 consecutive output elements: it reads the
// b bytes that hold their codes from every worker's stream, looks the levels up in LDS, adds
// them in worker order and writes 32 contiguous bytes of fp32 once.
//
// Two kernels share that shape:
//   tq_decode_fast_kernel    the fast path (N <= 16; N <= 8 at b = 4): per worker a table
//                            indexed by TWO adjacent codes (2^(2b) entries of float2), so one
//                            8-byte LDS read serves two elements; a single memory round trip
//                            per workgroup.
//   tq_decode_kernel         the general path (any N up to 64 at any b): one 4-byte LDS read
//                            per code from the plain 16-entry tables.
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

// ACC is a template parameter on purpose: with a run-time flag the read-modify-write branch
// leaves "a load may be pending" on every path, and the compiler then waits for ALL
// outstanding memory operations -- the tile's own stores included -- before the next tile.
template <bool ACC>
__device__ __forceinline__ void store_group(float* o, const float (&acc)[8], uint64_t e0, uint64_t d)
{
    if (e0 + kGroup <= d) {
        float4* o4 = reinterpret_cast<float4*>(o);
        float4 a = make_float4(acc[0], acc[1], acc[2], acc[3]);
        float4 b = make_float4(acc[4], acc[5], acc[6], acc[7]);
        if constexpr (ACC) {
            const float4 pa = o4[0], pb = o4[1];
            a.x = pa.x + a.x; a.y = pa.y + a.y; a.z = pa.z + a.z; a.w = pa.w + a.w;
            b.x = pb.x + b.x; b.y = pb.y + b.y; b.z = pb.z + b.z; b.w = pb.w + b.w;
        }
        o4[0] = a;
        o4[1] = b;
    } else {                                  // ragged end of the tensor
        // A rolled loop on purpose: unrolled, its last store was merged into the vector path
        // above, which then wrote 16 + 12 + 4 bytes per lane and lost a third of the bandwidth.
        const int n_valid = (int)(d - e0);
#pragma clang loop unroll(disable)
        for (int j = 0; j < n_valid; ++j) {
            float v = acc[0];
#pragma unroll
            for (int k = 1; k < 8; ++k) v = (j == k) ? acc[k] : v;
            if constexpr (ACC) v = o[j] + v;
            o[j] = v;
        }
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

// tq_decode_fast_kernel<BITS, U, T, ACC>: U = workers handled (N rounded up to 1, 2, 4, 8 or 16;
// the rows of the missing workers are zero and their stream is worker 0's, so they add 0),
// T = tiles per workgroup, ACC = add to `out` instead of overwriting it.
//
// One shot per workgroup, no loop over tiles: on this ISA loads and stores retire through ONE
// in-order counter, so a wave that stores a tile and then waits for further loads also waits
// for its stores to reach memory; a wave that ends after its stores waits for nothing.  What
// is left on the critical path is one memory round trip, so the kernel is arranged to make it
// exactly one: the code words of all T tiles are requested first; meanwhile each wavefront
// fetches the level rows of "its" workers through a scalar (wave-uniform) pointer, expands
// them to pair entries with two cross-lane reads and writes them to LDS; one barrier.
template <int BITS, int U, int T, bool ACC>
__global__ __launch_bounds__(kBlock) void tq_decode_fast_kernel(
    const DecodeArgs args, int N, int weighted, float scale, uint64_t d, uint64_t d_pad, uint64_t bucket_elems,
    uint32_t groups_per_bucket, uint64_t payload_bytes, float* __restrict__ out)
{
    constexpr int PAIRS = 1 << (2 * BITS);
    constexpr uint32_t PMASK = PAIRS - 1;
    constexpr uint32_t CMASK = (1u << BITS) - 1u;
    __shared__ float2 pair_tab[U * PAIRS];

    const uint32_t bucket = blockIdx.x / groups_per_bucket;
    const uint32_t grp = blockIdx.x - bucket * groups_per_bucket;
    const uint64_t bstart = (uint64_t)bucket * bucket_elems;
    uint64_t bend = bstart + bucket_elems < d_pad ? bstart + bucket_elems : d_pad;
    bend = bend < d ? bend : d;
    const uint64_t gstart = bstart + (uint64_t)grp * T * kTile;
    if (gstart >= bend) return;

    // this lane's group in each tile; lanes past the end read group 0 (always present)
    uint64_t e0[T], off[T];
    bool room[T];
#pragma unroll
    for (int t = 0; t < T; ++t) {
        e0[t] = gstart + (uint64_t)t * kTile + (uint64_t)threadIdx.x * kGroup;
        off[t] = e0[t] < bend ? (e0[t] >> 3) * (uint64_t)BITS : 0;
        room[t] = off[t] + 4 <= payload_bytes;
    }
    uint32_t w[T][U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
        const uint8_t* stream = args.payload[u < N ? u : 0];
#pragma unroll
        for (int t = 0; t < T; ++t) w[t][u] = load_codes<BITS>(stream + off[t], room[t]);
    }

    // pair tables: wavefront `wave` expands workers wave, wave + 4, ...  The wave index is
    // read into a scalar register so that the worker's pointer and weight are scalar loads.
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    float lrow[(U + 3) / 4];
#pragma unroll
    for (int k = 0; k < (U + 3) / 4; ++k) {
        const int i = wave + 4 * k;
        lrow[k] = 0.0f;
        if (i < N) {
            const tq_params_t* P = args.params[i] + bucket;
            const float wsel = weighted ? args.weight[i] : 1.0f;   // x * 1.0f is exact
            lrow[k] = wsel * P->level[lane & 15];
        }
    }
#pragma unroll
    for (int k = 0; k < (U + 3) / 4; ++k) {
        const int i = wave + 4 * k;
        if (i < U) {
#pragma unroll
            for (int e = lane; e < PAIRS; e += 64) {
                const float lo = __shfl(lrow[k], (int)(e & CMASK), 64);
                const float hi = __shfl(lrow[k], (int)(e >> BITS), 64);
                pair_tab[i * PAIRS + e] = make_float2(lo, hi);
            }
        }
    }
    __syncthreads();
    const float post = weighted ? 1.0f : scale;                // x * 1.0f is exact

    auto lookup = [&](int t, float (&acc)[8]) {
#pragma unroll
        for (int j = 0; j < 8; ++j) acc[j] = 0.0f;
#pragma unroll
        for (int u = 0; u < U; ++u)
#pragma unroll
            for (int m = 0; m < 4; ++m) {
                const float2 v = pair_tab[u * PAIRS + ((w[t][u] >> (2 * BITS * m)) & PMASK)];
                acc[2 * m] = acc[2 * m] + v.x;
                acc[2 * m + 1] = acc[2 * m + 1] + v.y;
            }
#pragma unroll
        for (int j = 0; j < 8; ++j) acc[j] = acc[j] * post;
    };

    if (gstart + (uint64_t)T * kTile <= bend) {
        // Every lane of the workgroup owns a whole group (all but the last workgroup of a
        // bucket): straight-line code, each tile stored as soon as it is looked up.
#pragma unroll
        for (int t = 0; t < T; ++t) {
            float acc[8];
            lookup(t, acc);
            store_group<ACC>(out + e0[t], acc, 0, kGroup);
        }
    } else {
        float acc[T][8];
#pragma unroll
        for (int t = 0; t < T; ++t) lookup(t, acc[t]);
#pragma unroll
        for (int t = 0; t < T; ++t)
            if (e0[t] < bend) store_group<ACC>(out + e0[t], acc[t], e0[t], d);
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
    if (accumulate) store_group<true>(out + e0, acc, e0, d); else store_group<false>(out + e0, acc, e0, d);
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

    if (N <= 16 && !(bits == 4 && N > 8)) {
        constexpr int T = 2;                                           // tiles per workgroup
        const uint64_t gpb = (tpb + T - 1) / T;
        const uint64_t nblocks = nb * gpb;
        if (nblocks == 0 || nblocks > 0x7FFFFFFFull) return hipErrorInvalidValue;
        const dim3 blocks((unsigned)nblocks);
        const int U = N <= 1 ? 1 : (N <= 2 ? 2 : (N <= 4 ? 4 : (N <= 8 ? 8 : 16)));
#define TQ_LAUNCH_FAST(B, UU)                                                                               \
    do {                                                                                                    \
        if (accumulate)                                                                                     \
            hipLaunchKernelGGL((tq::tq_decode_fast_kernel<B, UU, T, true>), blocks, threads, 0, st, args, N, \
                               weighted, scale, d, d_pad, be, (uint32_t)gpb, pbytes, out);                  \
        else                                                                                                \
            hipLaunchKernelGGL((tq::tq_decode_fast_kernel<B, UU, T, false>), blocks, threads, 0, st, args, N, \
                               weighted, scale, d, d_pad, be, (uint32_t)gpb, pbytes, out);                  \
    } while (0)
#define TQ_LAUNCH_FAST_U(B)                     \
    switch (U) {                                \
        case 1: TQ_LAUNCH_FAST(B, 1); break;    \
        case 2: TQ_LAUNCH_FAST(B, 2); break;    \
        case 4: TQ_LAUNCH_FAST(B, 4); break;    \
        case 8: TQ_LAUNCH_FAST(B, 8); break;    \
        default: TQ_LAUNCH_FAST(B, 16); break;  \
    }
        switch (bits) {
            case 2: TQ_LAUNCH_FAST_U(2) break;
            case 3: TQ_LAUNCH_FAST_U(3) break;
            default:
                switch (U) {                    // 16 workers at b = 4 would need 32 KiB of tables
                    case 1: TQ_LAUNCH_FAST(4, 1); break;
                    case 2: TQ_LAUNCH_FAST(4, 2); break;
                    case 4: TQ_LAUNCH_FAST(4, 4); break;
                    default: TQ_LAUNCH_FAST(4, 8); break;
                }
                break;
        }
#undef TQ_LAUNCH_FAST_U
#undef TQ_LAUNCH_FAST
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
