// tq_decompress_aggregate and tq_decompress_aggregate_update: Alg. 1 server steps of
// arXiv 2402.01798,
//   g_bar[e] = sum_i w_i * L_i[code_i(e)],   then out = g_bar or theta <- theta - eta * g_bar,
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
#include "tq_layout.h"

namespace tq {

struct DecodeArgs {
    const uint8_t* payload[TQ_MAX_WORKERS];
    const tq_params_t* params[TQ_MAX_WORKERS];
    float weight[TQ_MAX_WORKERS];
};

// The word that holds the 8 codes of a group, as code_load (tq_layout.h) places it.  Nothing
// here depends on the loaded value, so the load stays in flight until the codes are used; the
// caller shifts by CodeLoad::first_bit (non-zero only for the last groups of a 3-bit payload).
template <int BITS>
__device__ __forceinline__ uint32_t load_code_word(const uint8_t* stream, const CodeLoad& c)
{
    if constexpr (BITS == 2) return *reinterpret_cast<const uint16_t*>(stream + c.load_off);
    uint32_t w;
    __builtin_memcpy(&w, stream + c.load_off, 4);          // b = 3: byte-aligned only
    return w;
}

// What happens to the aggregate g_bar of an element (the MODE of the kernels below):
//   kStore        out = g_bar                           Alg. 1, server step "aggregate"
//   kStoreStream  the same, stored with the non-temporal hint (small outputs, see store8)
//   kAccumulate   out = out + g_bar
//   kSgd          theta = theta - eta * u,  u = g_bar + weight_decay * theta
//                                                       Alg. 1, server step "update", fused
//   kSgdMomentum  v = momentum * v + u;  theta = theta - eta * v
//                                                       the momentum SGD of the Sec. V experiments
// every product and sum rounded once to binary32, in that order.  MODE is a template parameter
// on purpose: with a run-time flag the read-modify-write branch leaves "a load may be pending"
// on every path, and the compiler then waits for ALL outstanding memory operations -- the
// tile's own stores included -- before the next tile.
enum { kStore = 0, kAccumulate = 1, kSgd = 2, kSgdMomentum = 3, kStoreStream = 4 };

struct Update {
    float eta, momentum, weight_decay;
    float* velocity;
};

template <int MODE>
__device__ __forceinline__ float finish(float g_bar, float prev, float& vel, const Update& up)
{
    if constexpr (MODE == kStore || MODE == kStoreStream) {
        return g_bar;
    } else if constexpr (MODE == kAccumulate) {
        return prev + g_bar;
    } else {
        float u = g_bar;
        if (up.weight_decay != 0.0f) {
            const float decay = up.weight_decay * prev;
            u = g_bar + decay;
        }
        if constexpr (MODE == kSgdMomentum) {
            const float carried = up.momentum * vel;
            u = carried + u;
            vel = u;
        }
        const float delta = up.eta * u;
        return prev - delta;
    }
}

__device__ __forceinline__ void load8(const float* p, float (&x)[8])
{
    const float4 a = reinterpret_cast<const float4*>(p)[0], b = reinterpret_cast<const float4*>(p)[1];
    x[0] = a.x; x[1] = a.y; x[2] = a.z; x[3] = a.w;
    x[4] = b.x; x[5] = b.y; x[6] = b.z; x[7] = b.w;
}

typedef float float4_native __attribute__((ext_vector_type(4)));

// STREAM: stored with the non-temporal hint.  Used for a plain aggregate small enough to stay
// in the memory-side cache: written normally it stays behind as dirty lines, and their
// write-back then competes with the next kernel's reads (12 us on the statistics launch that
// follows a 45 MB output).  The hint has a price -- the two 16-byte halves of a lane's 32 bytes
// leave L2 as separate partial writes, and a write-bound launch with a large output runs up to
// 1.8x slower with it -- so large outputs, which are evicted while the kernel runs anyway, and
// the buffers of the fused update, which the next step reads again, are stored normally.
template <bool STREAM>
__device__ __forceinline__ void store8(float* p, const float (&x)[8])
{
    if constexpr (STREAM) {
        float4_native a = {x[0], x[1], x[2], x[3]}, b = {x[4], x[5], x[6], x[7]};
        __builtin_nontemporal_store(a, reinterpret_cast<float4_native*>(p));
        __builtin_nontemporal_store(b, reinterpret_cast<float4_native*>(p) + 1);
    } else {
        reinterpret_cast<float4*>(p)[0] = make_float4(x[0], x[1], x[2], x[3]);
        reinterpret_cast<float4*>(p)[1] = make_float4(x[4], x[5], x[6], x[7]);
    }
}

// A lane's whole group: prev (and vel) were loaded by the caller, early, when MODE needs them.
template <int MODE>
__device__ __forceinline__ void finish_group(float* o, uint64_t e0, float (&acc)[8], const float (&prev)[8],
                                             float (&vel)[8], const Update& up)
{
#pragma unroll
    for (int j = 0; j < 8; ++j) acc[j] = finish<MODE>(acc[j], prev[j], vel[j], up);
    store8<MODE == kStoreStream>(o, acc);
    if constexpr (MODE == kSgdMomentum) store8<false>(up.velocity + e0, vel);
}

// The same 32 bytes per lane, stored by a WHOLE wavefront (every lane owns a group; `o` is lane
// 0's address).  Stored directly, each of the wavefront's two 16-byte store instructions would
// touch every line of its 2 KiB half-way; exchanged through LDS, lane l stores the l-th and the
// (64 + l)-th 16 bytes, so that each store instruction writes 1 KiB in one piece (measured: the
// aggregate of 8 x 124 M elements 139 us -> 118 us, of 8 x 11.2 M 20.8 -> 15.6 us).  `wb` is the
// wavefront's own 2 KiB of LDS; a wavefront's LDS operations complete in order, so no barrier.
template <bool STREAM>
__device__ __forceinline__ void store8_wave(float* o, int lane, const float (&x)[8], float4* wb)
{
    wb[2 * lane] = make_float4(x[0], x[1], x[2], x[3]);
    wb[2 * lane + 1] = make_float4(x[4], x[5], x[6], x[7]);
    const float4 a = wb[lane], b = wb[64 + lane];
    if constexpr (STREAM) {
        float4_native an = {a.x, a.y, a.z, a.w}, bn = {b.x, b.y, b.z, b.w};
        __builtin_nontemporal_store(an, reinterpret_cast<float4_native*>(o) + lane);
        __builtin_nontemporal_store(bn, reinterpret_cast<float4_native*>(o) + 64 + lane);
    } else {
        reinterpret_cast<float4*>(o)[lane] = a;
        reinterpret_cast<float4*>(o)[64 + lane] = b;
    }
}

template <int MODE>
__device__ __forceinline__ void finish_group_wave(float* out, uint64_t e0, int lane, float (&acc)[8],
                                                  const float (&prev)[8], float (&vel)[8], const Update& up,
                                                  float4* wb)
{
#pragma unroll
    for (int j = 0; j < 8; ++j) acc[j] = finish<MODE>(acc[j], prev[j], vel[j], up);
    const uint64_t wave_e0 = e0 - (uint64_t)lane * kGroup;
    store8_wave<MODE == kStoreStream>(out + wave_e0, lane, acc, wb);
    if constexpr (MODE == kSgdMomentum) store8_wave<false>(up.velocity + wave_e0, lane, vel, wb);
}

// The ragged end of the tensor, element by element (only in the last workgroup of the tensor;
// the workgroups whose lanes all own whole groups take a separate, straight-line path, so
// that whatever the compiler makes of these predicated stores does not touch theirs).
template <int MODE>
__device__ __forceinline__ void finish_ragged(float* o, uint64_t e0, const float (&acc)[8], int n_valid,
                                              const Update& up)
{
#pragma unroll
    for (int j = 0; j < 7; ++j) {                          // a ragged group has at most 7 elements
        if (j < n_valid) {
            float prev = 0.0f, vel = 0.0f;
            if constexpr (MODE != kStore && MODE != kStoreStream) prev = o[j];
            if constexpr (MODE == kSgdMomentum) vel = up.velocity[e0 + j];
            o[j] = finish<MODE>(acc[j], prev, vel, up);
            if constexpr (MODE == kSgdMomentum) up.velocity[e0 + j] = vel;
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

// tq_decode_fast_kernel<BITS, U, T, MODE>: U = workers handled (N rounded up to 1, 2, 4, 8 or 16;
// the rows of the missing workers are zero and their stream is worker 0's, so they add 0),
// T = tiles per workgroup, MODE = what is done with the aggregate (see above).
//
// One shot per workgroup, no loop over tiles: on this ISA loads and stores retire through ONE
// in-order counter, so a wave that stores a tile and then waits for further loads also waits
// for its stores to reach memory; a wave that ends after its stores waits for nothing.  What
// is left on the critical path is one memory round trip, so the kernel is arranged to make it
// exactly one: the code words of all T tiles are requested first; meanwhile each wavefront
// fetches the level rows of "its" workers through a scalar (wave-uniform) pointer, expands
// them to pair entries with two cross-lane reads and writes them to LDS; one barrier.
//
// SEG: the records are those of variable-size segments instead of buckets.  A workgroup takes
// T tiles wherever they fall; its reads are requested before the segment is looked up, and
// when its whole range lies inside one segment (nearly always) the rest is the bucketed code
// with that segment's record.  Otherwise it takes its tiles one by one, the segments that
// overlap a tile one after the other, with plain level rows -- the same sums in the same order.
template <int BITS, int U, int T, int MODE, bool SEG>
__global__ __launch_bounds__(kBlock) void tq_decode_fast_kernel(
    const DecodeArgs args, int N, int weighted, float scale, uint64_t d, uint64_t d_pad, uint64_t bucket_elems,
    uint32_t groups_per_bucket, uint64_t payload_bytes, float* __restrict__ out, const Update up,
    const uint64_t* __restrict__ seg_off, uint32_t nseg, const SegHints hints)
{
    constexpr int PAIRS = 1 << (2 * BITS);
    constexpr uint32_t PMASK = PAIRS - 1;
    constexpr uint32_t CMASK = (1u << BITS) - 1u;
    __shared__ float2 pair_tab[U * PAIRS];
    __shared__ float4 xbuf[kBlock / 64][128];                  // store8_wave's exchange buffers

    const uint32_t blk = linear_block();
    uint32_t bucket = 0;                                       // the record of the workgroup's range
    uint64_t gstart, bend;                                     // its first element, the end of what it may take
    if constexpr (!SEG) {
        bucket = blk / groups_per_bucket;
        const uint32_t grp = blk - bucket * groups_per_bucket;
        const uint64_t bstart = (uint64_t)bucket * bucket_elems;
        bend = bstart + bucket_elems < d_pad ? bstart + bucket_elems : d_pad;
        bend = bend < d ? bend : d;
        gstart = bstart + (uint64_t)grp * T * kTile;
    } else {
        gstart = (uint64_t)blk * T * kTile;
        bend = d;                                              // for the reads; the segment's end comes later
    }
    if (gstart >= bend) return;

    // this lane's group in each tile; lanes past the end read group 0 (always present)
    uint64_t e0[T];
    CodeLoad cl[T];
#pragma unroll
    for (int t = 0; t < T; ++t) {
        e0[t] = gstart + (uint64_t)t * kTile + (uint64_t)threadIdx.x * kGroup;
        cl[t] = code_load(e0[t] < bend ? e0[t] >> 3 : 0, BITS, payload_bytes);
    }
    uint32_t w[T][U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
        const uint8_t* stream = args.payload[u < N ? u : 0];
#pragma unroll
        for (int t = 0; t < T; ++t) w[t][u] = load_code_word<BITS>(stream, cl[t]);
    }
    // what the epilogue reads back (the old output, the parameters, the velocity) is requested
    // now as well, for the lanes that own a whole group
    float prev[T][8], vel[T][8];
#pragma unroll
    for (int t = 0; t < T; ++t) {
#pragma unroll
        for (int j = 0; j < 8; ++j) { prev[t][j] = 0.0f; vel[t][j] = 0.0f; }
        if (e0[t] + kGroup <= bend) {
            if constexpr (MODE != kStore && MODE != kStoreStream) load8(out + e0[t], prev[t]);
            if constexpr (MODE == kSgdMomentum) load8(up.velocity + e0[t], vel[t]);
        }
    }

    if constexpr (SEG) {
        __shared__ float rows[16 * 16];                        // plain level rows: U <= 16 workers
        constexpr uint32_t MASK = (1u << BITS) - 1u;
        const uint32_t s0 = find_segment(seg_off, nseg, gstart, hints);
        const uint64_t lo0 = seg_off[s0];
        const uint64_t hi0 = s0 + 1 < nseg ? seg_off[s0 + 1] : d_pad;
        if (lo0 <= gstart && gstart + (uint64_t)T * kTile <= (hi0 < d ? hi0 : d)) {
            bucket = s0;                                       // one record for the whole range: as for a bucket
        } else {
            for (int t = 0; t < T; ++t) {                      // the same for the whole workgroup
                const uint64_t tbase = gstart + (uint64_t)t * kTile;
                if (tbase >= d) break;
                const uint64_t tile_end = tbase + kTile < d_pad ? tbase + kTile : d_pad;
                uint32_t s = t == 0 ? s0 : find_segment(seg_off, nseg, tbase, hints);
                for (;;) {
                    const uint64_t seg_lo = seg_off[s];
                    const uint64_t seg_hi = s + 1 < nseg ? seg_off[s + 1] : d_pad;
                    __syncthreads();                           // the rows of the segment before are done with
                    fill_level_rows(rows, args, N, weighted, s);
                    __syncthreads();
                    if (e0[t] >= seg_lo && e0[t] < seg_hi && e0[t] < d) {
                        float acc[8];
#pragma unroll
                        for (int j = 0; j < 8; ++j) acc[j] = 0.0f;
#pragma unroll
                        for (int u = 0; u < U; ++u) {
                            if (u < N) {
                                const uint32_t codes = w[t][u] >> cl[t].first_bit;
#pragma unroll
                                for (int j = 0; j < 8; ++j) acc[j] = acc[j] + rows[u * 16 + ((codes >> (j * BITS)) & MASK)];
                            }
                        }
                        if (!weighted) {
#pragma unroll
                            for (int j = 0; j < 8; ++j) acc[j] = acc[j] * scale;
                        }
                        if (e0[t] + kGroup <= d) finish_group<MODE>(out + e0[t], e0[t], acc, prev[t], vel[t], up);
                        else finish_ragged<MODE>(out + e0[t], e0[t], acc, (int)(d - e0[t]), up);
                    }
                    if (seg_hi >= tile_end || s + 1 >= nseg) break;
                    ++s;
                }
            }
            return;
        }
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
                const uint32_t codes = BITS == 3 ? w[t][u] >> cl[t].first_bit : w[t][u];
                const float2 v = pair_tab[u * PAIRS + ((codes >> (2 * BITS * m)) & PMASK)];
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
            finish_group_wave<MODE>(out, e0[t], lane, acc, prev[t], vel[t], up, xbuf[wave]);
        }
    } else {
        // the last workgroup of a bucket: tile by tile (one tile's values live at a time)
#pragma unroll
        for (int t = 0; t < T; ++t) {
            float acc[8];
            lookup(t, acc);
            if (e0[t] + kGroup <= bend) finish_group<MODE>(out + e0[t], e0[t], acc, prev[t], vel[t], up);
            else if (e0[t] < bend) finish_ragged<MODE>(out + e0[t], e0[t], acc, (int)(bend - e0[t]), up);
        }
    }
}

template <int BITS, int MODE>
__global__ __launch_bounds__(kBlock) void tq_decode_kernel(
    const DecodeArgs args, int N, int weighted, float scale, uint64_t d, uint64_t d_pad,
    uint64_t bucket_elems, uint32_t tiles_per_bucket, uint64_t payload_bytes, float* __restrict__ out,
    const Update up)
{
    constexpr uint32_t MASK = (1u << BITS) - 1u;
    const TileGeom t = tile_geom(linear_block(), d_pad, bucket_elems, tiles_per_bucket);
    if (t.ebase >= t.eend) return;

    __shared__ float table[TQ_MAX_WORKERS * 16];
    fill_level_rows(table, args, N, weighted, t.bucket);
    __syncthreads();

    const uint64_t e0 = t.ebase + (uint64_t)threadIdx.x * kGroup;
    if (e0 >= t.eend || e0 >= d) return;
    const CodeLoad cl = code_load(e0 >> 3, BITS, payload_bytes);

    const bool whole = e0 + kGroup <= d;
    float acc[8], prev[8], vel[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) { acc[j] = 0.0f; prev[j] = 0.0f; vel[j] = 0.0f; }
    if (whole) {
        if constexpr (MODE != kStore && MODE != kStoreStream) load8(out + e0, prev);
        if constexpr (MODE == kSgdMomentum) load8(up.velocity + e0, vel);
    }
    for (int i = 0; i < N; ++i) {
        const uint32_t w = load_code_word<BITS>(args.payload[i], cl) >> cl.first_bit;
        const float* row = table + i * 16;
#pragma unroll
        for (int j = 0; j < 8; ++j) acc[j] = acc[j] + row[(w >> (j * BITS)) & MASK];
    }
    if (!weighted) {
#pragma unroll
        for (int j = 0; j < 8; ++j) acc[j] = acc[j] * scale;
    }
    if (whole) finish_group<MODE>(out + e0, e0, acc, prev, vel, up);
    else finish_ragged<MODE>(out + e0, e0, acc, (int)(d - e0), up);
}

// tq_decompress_aggregate_segments: the server step with one codebook per variable-size
// segment (and worker).  Shape of tq_compress_segments_kernel: one tile per workgroup, the
// segments that overlap it taken one after the other, each with the N workers' level rows of
// that segment in LDS.
template <int BITS, int MODE>
__global__ __launch_bounds__(kBlock) void tq_decode_segments_kernel(
    const DecodeArgs args, int N, int weighted, float scale, uint64_t d, uint64_t d_pad,
    const uint64_t* __restrict__ seg_off, uint32_t nseg, const SegHints hints, uint64_t payload_bytes,
    float* __restrict__ out, const Update up)
{
    constexpr uint32_t MASK = (1u << BITS) - 1u;
    const uint64_t ebase = (uint64_t)linear_block() * kTile;
    if (ebase >= d) return;
    const uint64_t tile_end = ebase + kTile < d_pad ? ebase + kTile : d_pad;
    const uint64_t e0 = ebase + (uint64_t)threadIdx.x * kGroup;
    __shared__ float table[TQ_MAX_WORKERS * 16];

    uint32_t s = find_segment(seg_off, nseg, ebase, hints);
    for (;;) {
        const uint64_t seg_lo = seg_off[s];
        const uint64_t seg_hi = s + 1 < nseg ? seg_off[s + 1] : d_pad;
        fill_level_rows(table, args, N, weighted, s);
        __syncthreads();
        if (e0 >= seg_lo && e0 < seg_hi && e0 < d) {
            const CodeLoad cl = code_load(e0 >> 3, BITS, payload_bytes);
            const bool whole = e0 + kGroup <= d;
            float acc[8], prev[8], vel[8];
#pragma unroll
            for (int j = 0; j < 8; ++j) { acc[j] = 0.0f; prev[j] = 0.0f; vel[j] = 0.0f; }
            if (whole) {
                if constexpr (MODE != kStore && MODE != kStoreStream) load8(out + e0, prev);
            }
            for (int i = 0; i < N; ++i) {
                const uint32_t w = load_code_word<BITS>(args.payload[i], cl) >> cl.first_bit;
                const float* row = table + i * 16;
#pragma unroll
                for (int j = 0; j < 8; ++j) acc[j] = acc[j] + row[(w >> (j * BITS)) & MASK];
            }
            if (!weighted) {
#pragma unroll
                for (int j = 0; j < 8; ++j) acc[j] = acc[j] * scale;
            }
            if (whole) finish_group<MODE>(out + e0, e0, acc, prev, vel, up);
            else finish_ragged<MODE>(out + e0, e0, acc, (int)(d - e0), up);
        }
        if (seg_hi >= tile_end || s + 1 >= nseg) break;
        ++s;
        __syncthreads();                                       // before the next segment's rows replace these
    }
}

}  // namespace tq

namespace {

struct DecodeGeom {
    tq::DecodeArgs args;
    int N, weighted, bits;
    float scale;
    uint64_t d, d_pad, be, nb, tpb, pbytes;
};

// One launch with the epilogue MODE fixed at compile time.
template <int MODE>
hipError_t launch_mode(const DecodeGeom& g, float* out, const tq::Update& up, hipStream_t st)
{
    const dim3 threads(tq::kBlock);
    const int N = g.N;
    if (N <= 16 && !(g.bits == 4 && N > 8)) {
        const int U = N <= 1 ? 1 : (N <= 2 ? 2 : (N <= 4 ? 4 : (N <= 8 ? 8 : 16)));
        // tiles per workgroup: two, so that the tables are built once per 4096 elements (measured
        // with 1 / 2 / 4 tiles: 8 x 124 M at b = 2 131 / 119 / 122 us; 16 x 25.6 M at b = 3, where two
        // tiles' code words take 122 registers and halve the resident wavefronts, 74 / 66 / - us)
        constexpr int T = 2;
        const uint64_t gpb = (g.tpb + T - 1) / T;
        const uint64_t nblocks = g.nb * gpb;
        dim3 blocks;
        if (!tq::fold_grid(nblocks, tq::kBlock, 1, blocks)) return hipErrorInvalidValue;
        const tq::SegHints no_hints{};
#define TQ_LAUNCH_FAST(B, UU, TT)                                                                            \
    hipLaunchKernelGGL((tq::tq_decode_fast_kernel<B, UU, TT, MODE, false>), blocks, threads, 0, st, g.args, N, \
                       g.weighted, g.scale, g.d, g.d_pad, g.be, (uint32_t)gpb, g.pbytes, out, up,               \
                       static_cast<const uint64_t*>(nullptr), 0u, no_hints)
#define TQ_LAUNCH_FAST_U(B)                                          \
    switch (U) {                                                     \
        case 1: TQ_LAUNCH_FAST(B, 1, T); break;                      \
        case 2: TQ_LAUNCH_FAST(B, 2, T); break;                      \
        case 4: TQ_LAUNCH_FAST(B, 4, T); break;                      \
        case 8: TQ_LAUNCH_FAST(B, 8, T); break;                      \
        default: TQ_LAUNCH_FAST(B, 16, T); break;  \
    }
        switch (g.bits) {
            case 2: TQ_LAUNCH_FAST_U(2) break;
            case 3: TQ_LAUNCH_FAST_U(3) break;
            default:
                switch (U) {                    // 16 workers at b = 4 would need 32 KiB of tables
                    case 1: TQ_LAUNCH_FAST(4, 1, T); break;
                    case 2: TQ_LAUNCH_FAST(4, 2, T); break;
                    case 4: TQ_LAUNCH_FAST(4, 4, T); break;
                    default: TQ_LAUNCH_FAST(4, 8, T); break;
                }
                break;
        }
#undef TQ_LAUNCH_FAST_U
#undef TQ_LAUNCH_FAST
        return hipGetLastError();
    }

    const uint64_t nblocks = g.nb * g.tpb;
    dim3 blocks;
    if (!tq::fold_grid(nblocks, tq::kBlock, 1, blocks)) return hipErrorInvalidValue;
#define TQ_LAUNCH_GENERAL(B)                                                                                 \
    hipLaunchKernelGGL((tq::tq_decode_kernel<B, MODE>), blocks, threads, 0, st, g.args, N, g.weighted,       \
                       g.scale, g.d, g.d_pad, g.be, (uint32_t)g.tpb, g.pbytes, out, up)
    switch (g.bits) {
        case 2: TQ_LAUNCH_GENERAL(2); break;
        case 3: TQ_LAUNCH_GENERAL(3); break;
        default: TQ_LAUNCH_GENERAL(4); break;
    }
#undef TQ_LAUNCH_GENERAL
    return hipGetLastError();
}

}  // namespace

// Host side of tq_decompress_aggregate and tq_decompress_aggregate_update after the argument
// checks of the C entry points.  mode: 0 store, 1 accumulate, 2 SGD step on `out` (= theta),
// 3 the same with the velocity buffer.
hipError_t tq_launch_decode(const void* const* payload, const tq_params_t* const* params,
                            const float* weights, int N, uint64_t d, uint64_t bucket_elems, int bits,
                            int mode, float eta, float momentum, float weight_decay, float* velocity,
                            float* out, hipStream_t st)
{
    DecodeGeom g;
    for (int i = 0; i < TQ_MAX_WORKERS; ++i) {
        g.args.payload[i] = i < N ? static_cast<const uint8_t*>(payload[i]) : nullptr;
        g.args.params[i] = i < N ? params[i] : nullptr;
        g.args.weight[i] = (i < N && weights) ? weights[i] : 0.0f;
    }
    g.N = N;
    g.bits = bits;
    g.weighted = weights ? 1 : 0;
    g.scale = 1.0f / (float)N;
    g.d = d;
    g.d_pad = (d + 127) / 128 * 128;
    g.be = bucket_elems ? bucket_elems : g.d_pad;
    g.nb = (g.d_pad + g.be - 1) / g.be;
    g.tpb = (g.be + tq::kTile - 1) / tq::kTile;                        // tiles per bucket
    g.pbytes = tq_payload_bytes(d, bits);
    const tq::Update up{eta, momentum, weight_decay, velocity};
    // outputs up to 64 MiB are streamed past the caches (see store8)
    if (mode == tq::kStore && d * sizeof(float) <= (64ull << 20)) mode = tq::kStoreStream;
    switch (mode) {
        case tq::kStore: return launch_mode<tq::kStore>(g, out, up, st);
        case tq::kStoreStream: return launch_mode<tq::kStoreStream>(g, out, up, st);
        case tq::kAccumulate: return launch_mode<tq::kAccumulate>(g, out, up, st);
        case tq::kSgd: return launch_mode<tq::kSgd>(g, out, up, st);
        case tq::kSgdMomentum: return launch_mode<tq::kSgdMomentum>(g, out, up, st);
        default: return hipErrorInvalidValue;
    }
}


// Host side of tq_decompress_aggregate_segments after the argument checks of the C entry point.
hipError_t tq_launch_decode_segments(const void* const* payload, const tq_params_t* const* params,
                                     const float* weights, int N, uint64_t d, const uint64_t* seg_off,
                                     const uint64_t* seg_host, uint64_t nseg, int bits, int accumulate, float* out,
                                     hipStream_t st)
{
    const tq::SegHints hints = tq::make_seg_hints(seg_host, nseg, d);
    tq::DecodeArgs args;
    for (int i = 0; i < TQ_MAX_WORKERS; ++i) {
        args.payload[i] = i < N ? static_cast<const uint8_t*>(payload[i]) : nullptr;
        args.params[i] = i < N ? params[i] : nullptr;
        args.weight[i] = (i < N && weights) ? weights[i] : 0.0f;
    }
    const uint64_t d_pad = (d + 127) / 128 * 128;
    const uint64_t nblocks = (d + tq::kTile - 1) / tq::kTile;
    dim3 blocks;
    if (nseg > 0xFFFFFFFFull || !tq::fold_grid(nblocks, tq::kBlock, 1, blocks)) return hipErrorInvalidValue;
    const uint64_t pbytes = tq_payload_bytes(d, bits);
    const tq::Update up{0.0f, 0.0f, 0.0f, nullptr};
    const float scale = 1.0f / (float)N;
    const int weighted = weights ? 1 : 0;
    const dim3 threads(tq::kBlock);
    if (N <= 16 && !(bits == 4 && N > 8)) {
        // the bucketed kernel's code with the segments' records: two tiles per workgroup wherever they fall
        constexpr int T = 2;
        const int U = N <= 1 ? 1 : (N <= 2 ? 2 : (N <= 4 ? 4 : (N <= 8 ? 8 : 16)));
        dim3 fblocks;
        if (!tq::fold_grid((d + (uint64_t)T * tq::kTile - 1) / ((uint64_t)T * tq::kTile), tq::kBlock, 1, fblocks))
            return hipErrorInvalidValue;
#define TQ_LAUNCH_FSEG(B, UU, M)                                                                                  \
    hipLaunchKernelGGL((tq::tq_decode_fast_kernel<B, UU, T, M, true>), fblocks, threads, 0, st, args, N, weighted, \
                       scale, d, d_pad, (uint64_t)0, 0u, pbytes, out, up, seg_off, (uint32_t)nseg, hints)
#define TQ_LAUNCH_FSEG_M(B, UU) \
    if (accumulate) TQ_LAUNCH_FSEG(B, UU, tq::kAccumulate); else TQ_LAUNCH_FSEG(B, UU, tq::kStore)
#define TQ_LAUNCH_FSEG_U(B)                          \
    switch (U) {                                     \
        case 1: TQ_LAUNCH_FSEG_M(B, 1); break;       \
        case 2: TQ_LAUNCH_FSEG_M(B, 2); break;       \
        case 4: TQ_LAUNCH_FSEG_M(B, 4); break;       \
        case 8: TQ_LAUNCH_FSEG_M(B, 8); break;       \
        default: TQ_LAUNCH_FSEG_M(B, 16); break;     \
    }
        switch (bits) {
            case 2: TQ_LAUNCH_FSEG_U(2) break;
            case 3: TQ_LAUNCH_FSEG_U(3) break;
            default:
                switch (U) {
                    case 1: TQ_LAUNCH_FSEG_M(4, 1); break;
                    case 2: TQ_LAUNCH_FSEG_M(4, 2); break;
                    case 4: TQ_LAUNCH_FSEG_M(4, 4); break;
                    default: TQ_LAUNCH_FSEG_M(4, 8); break;
                }
                break;
        }
#undef TQ_LAUNCH_FSEG_U
#undef TQ_LAUNCH_FSEG_M
#undef TQ_LAUNCH_FSEG
        return hipGetLastError();
    }
#define TQ_LAUNCH_DSEG(B, M)                                                                                   \
    hipLaunchKernelGGL((tq::tq_decode_segments_kernel<B, M>), blocks, threads, 0, st, args, N, weighted, scale, \
                       d, d_pad, seg_off, (uint32_t)nseg, hints, pbytes, out, up)
#define TQ_LAUNCH_DSEG_M(B) \
    if (accumulate) TQ_LAUNCH_DSEG(B, tq::kAccumulate); else TQ_LAUNCH_DSEG(B, tq::kStore)
    switch (bits) {
        case 2: TQ_LAUNCH_DSEG_M(2); break;
        case 3: TQ_LAUNCH_DSEG_M(3); break;
        default: TQ_LAUNCH_DSEG_M(4); break;
    }
#undef TQ_LAUNCH_DSEG_M
#undef TQ_LAUNCH_DSEG
    return hipGetLastError();
}
