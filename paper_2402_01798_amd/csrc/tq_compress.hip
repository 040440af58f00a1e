// tq_compress: Alg. 1 client step of arXiv 2402.01798 -- truncate (Eq. 1), locate the cell
// and its rounding probability, round stochastically (Eq. 2), pack b-bit codes.
//
// One lane owns 8 consecutive elements: they share one Philox4x32-10 call (8 x 16 random
// bits) and their codes are exactly b bytes of the payload, so a wavefront reads 2 KiB
// (fp32) or 1 KiB (bf16) of gradient and writes 64*b contiguous bytes.
#include <type_traits>

#include "tq_device.h"


namespace tq {

// STREAM: non-temporal loads.  This is the last read of the gradient; when the whole batch is
// small enough that the memory-side cache still holds much of what the statistics pass read,
// the hint keeps this kernel's misses from displacing the lines it is about to hit (-6 % on
// 8 x 45 MB).  On data that cannot be cached anyway the same hint costs 12 % (misses are
// slower with it), so the host turns it on by size.
template <int DTYPE, bool STREAM>
__device__ __forceinline__ void load_group(const void* g, uint64_t e0, float (&x)[8])
{
    typedef float f4 __attribute__((ext_vector_type(4)));
    typedef uint32_t u4 __attribute__((ext_vector_type(4)));
    if constexpr (DTYPE == TQ_F32) {
        const f4* p = reinterpret_cast<const f4*>(static_cast<const float*>(g) + e0);
        f4 a, b;
        if constexpr (STREAM) { a = __builtin_nontemporal_load(p); b = __builtin_nontemporal_load(p + 1); }
        else { a = p[0]; b = p[1]; }
        x[0] = a.x; x[1] = a.y; x[2] = a.z; x[3] = a.w;
        x[4] = b.x; x[5] = b.y; x[6] = b.z; x[7] = b.w;
    } else {
        const u4* p = reinterpret_cast<const u4*>(static_cast<const uint16_t*>(g) + e0);
        u4 v;
        if constexpr (STREAM) v = __builtin_nontemporal_load(p);
        else v = p[0];
        const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            x[2 * i] = __uint_as_float(w[i] << 16);
            x[2 * i + 1] = __uint_as_float(w[i] & 0xFFFF0000u);
        }
    }
}

template <int DTYPE>
__device__ __forceinline__ float load_one(const void* g, uint64_t e)
{
    if constexpr (DTYPE == TQ_F32) return static_cast<const float*>(g)[e];
    return __uint_as_float((uint32_t) static_cast<const uint16_t*>(g)[e] << 16);
}

// Levels and inverse widths of one bucket, kept in LDS for the per-lane look-ups of the
// level-table path: entry j = (l_j, inv_w[j], pivot_j, -), 16 bytes, where pivot_j = l_j for
// j < s and +inf from j = s on: the table the cell search walks.  The search carries the
// BYTE offset of its current entry, so no look-up needs an index-to-address shift.
struct LevelLds {
    float4 e[16];
};

__device__ __forceinline__ void fill_level_lds(LevelLds& tab, const tq_params_t* P, uint32_t s)
{
    if (threadIdx.x < 16) {
        const float l = P->level[threadIdx.x];
        tab.e[threadIdx.x] = make_float4(l, P->inv_w[threadIdx.x], threadIdx.x < s ? l : __builtin_inff(), 0.0f);
    }
}

// NaN -> +0 for a lane's 8 values.  NaN is rare, so the test is made as cheap as it can be:
// one unordered compare per PAIR of values, and the replacement itself only in wavefronts
// in which some lane saw one.
__device__ __forceinline__ void replace_nan(float (&x)[8])
{
    unsigned long long any = 0ull;                             // lane masks, combined on the scalar unit
#pragma unroll
    for (int i = 0; i < 4; ++i) any |= __builtin_amdgcn_ballot_w64(__builtin_isunordered(x[2 * i], x[2 * i + 1]));
    if (any != 0ull) {
#pragma unroll
        for (int j = 0; j < 8; ++j) x[j] = (x[j] != x[j]) ? 0.0f : x[j];
    }
}

// Eq. (1) then Eq. (2) for one element; `rf` is the element's 16-bit draw as a float.
// Any codebook: cell k by comparison with the levels, p_r = (x - l_k) * inv_w[k] (two
// roundings), the upper end iff u = 1 - (rf + 1/2) / 2^16 <= p_r.  The uniform codebook: the
// same rounding stated through the position in units of cells, floor(t + U), U = (rf + 1/2) / 2^16.
// Uniform codebook: the code of one element.
template <int BITS>
__device__ __forceinline__ uint32_t quantize_uniform(float x, float rf, float alpha, float inv_step)
{
    constexpr uint32_t S = (1u << BITS) - 1u;
    const float xc = __builtin_amdgcn_fmed3f(x, -alpha, alpha);  // Eq. (1); the caller has replaced NaN
    // position in units of cells from -alpha, plus the dither's half grain; then the draw
    const float u = fmaf(xc, inv_step, 0.5f * (float)S + 1.0f / 131072.0f);
    const float v = fmaf(rf, 1.0f / 65536.0f, u);              // floor(v) = k + [rnd >= 1 - frac]
    const uint32_t code = (uint32_t)v;
    return code > S ? S : code;
}

// Level-table path: 16 * k for the cell k that holds x (l_k <= x < l_{k+1}; levels ascending),
// i.e. the byte offset of the cell's entry in LevelLds.
template <int BITS>
__device__ __forceinline__ uint32_t cell_offset(float x, const float (&lv)[16], const LevelLds& tab)
{
    uint32_t a;
    if constexpr (BITS == 2) {
        a = (x >= lv[1]) ? 16u : 0u;                           // two selects, no adds
        a = (x >= lv[2]) ? 32u : a;
    } else {
        // binary search over the pivots (padded with +inf to 2^b entries): the first pivot is a
        // scalar, the second a select between two scalars, the others are read from LDS at
        // (current entry + step), the step folded into the instruction's offset field
        constexpr uint32_t HALF = 1u << (BITS - 1), QUARTER = HALF >> 1;
        const bool top = x >= lv[HALF];
        const float pivot = top ? lv[HALF + QUARTER] : lv[QUARTER];
        a = top ? 16u * HALF : 0u;
        a |= (x >= pivot) ? 16u * QUARTER : 0u;
        const char* base = reinterpret_cast<const char*>(tab.e);
#pragma unroll
        for (uint32_t h = QUARTER >> 1; h >= 1; h >>= 1) {
            const float pv = *reinterpret_cast<const float*>(base + a + (16u * h + 8u));
            a |= (x >= pv) ? 16u * h : 0u;
        }
    }
    return a;
}

// Level-table path: does the element take the upper end of its cell?  p_r and the draw.
__device__ __forceinline__ bool rounds_up(float x, float rf, uint32_t a, const LevelLds& tab)
{
    const float2 cell = *reinterpret_cast<const float2*>(reinterpret_cast<const char*>(tab.e) + a);
    const float p_r = (x - cell.x) * cell.y;                   // (g - l_k) / |Delta_k| of Eq. (2)
    const float u = fmaf(rf, -1.0f / 65536.0f, 1.0f - 1.0f / 131072.0f);   // 1 - (r + 1/2) / 2^16, exact
    return u <= p_r;
}

template <int BITS, int GRID>
__device__ __forceinline__ uint32_t quantize(float x, float rf, float alpha, float inv_step,
                                             const float (&lv)[16], const LevelLds& tab)
{
    if constexpr (GRID == TQ_GRID_UNIFORM) {
        return quantize_uniform<BITS>(x, rf, alpha, inv_step);
    } else {
        const float xc = __builtin_amdgcn_fmed3f(x, -alpha, alpha);  // Eq. (1)
        const uint32_t a = cell_offset<BITS>(xc, lv, tab);
        return (a >> 4) + (rounds_up(xc, rf, a, tab) ? 1u : 0u);
    }
}

// Codes of one lane's 8 elements, packed little-endian into the low 8*BITS bits.
// PARTIAL: only the first n_valid elements exist; the others encode as 0 (pad bits).
// CLAMP (level-table path): whether the truncation of Eq. (1) is written out.  It changes the
// code only when the FIRST cell of the codebook is empty (l_1 = l_0 = -alpha, a degenerate
// bucket): a value below -alpha is truncated onto that repeated level and then belongs to the
// cell above it.  Otherwise it changes nothing -- below -alpha the cell is the first one and
// p_r < 0, beyond +alpha it is the last one and p_r >= 1 (or 0 for an empty last cell), +-Inf
// go the same ways (Inf times a zero reciprocal is NaN, and u <= NaN is false: the lower end,
// as for the truncated value) -- so the caller leaves it out unless l_1 = l_0: one
// instruction per element of a kernel that is bound by instruction issue.
template <int BITS, int GRID, bool PARTIAL, bool CLAMP = true>
__device__ __forceinline__ uint32_t encode_group(const float (&x)[8], const uint32_t (&rw)[4], int n_valid,
                                                 float alpha, float inv_step, const float (&lv)[16],
                                                 const LevelLds& tab)
{
    if constexpr (GRID == TQ_GRID_UNIFORM) {
        uint32_t word = 0;
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const uint32_t r = (j & 1) ? (rw[j >> 1] >> 16) : (rw[j >> 1] & 0xFFFFu);
            uint32_t code = quantize_uniform<BITS>(x[j], (float)r, alpha, inv_step);
            if (PARTIAL && j >= n_valid) code = 0;
            word |= code << (j * BITS);
        }
        return word;
    } else {
        // code = k + up: the cells' offsets 16 k are merged into one word (shifted into place,
        // four bits too high), the upward roundings into another; their sum is the packed group
        uint32_t cells = 0, ups = 0;
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const uint32_t r = (j & 1) ? (rw[j >> 1] >> 16) : (rw[j >> 1] & 0xFFFFu);
            const float xc = CLAMP ? __builtin_amdgcn_fmed3f(x[j], -alpha, alpha) : x[j];   // Eq. (1); NaN is gone
            uint32_t a = cell_offset<BITS>(xc, lv, tab);
            bool up = rounds_up(xc, (float)r, a, tab);
            if (PARTIAL && j >= n_valid) { a = 0; up = false; }
            cells |= (j * BITS >= 4) ? a << (j * BITS - 4) : a >> (4 - j * BITS);
            ups |= up ? 1u << (j * BITS) : 0u;
        }
        return cells + ups;
    }
}

// `room` = bytes of the payload from `out` on.  A payload is a multiple of 16 bytes, so a
// group's 2 or 4 bytes are either wholly inside or wholly outside; its 3 bytes at b = 3 can
// straddle the end (the last, ragged group of a short tensor), hence the per-byte test.
template <int BITS>
__device__ __forceinline__ void store_codes(uint8_t* out, uint32_t word, uint64_t room = 4)
{
    if constexpr (BITS == 4) {
        *reinterpret_cast<uint32_t*>(out) = word;
    } else if constexpr (BITS == 2) {
        *reinterpret_cast<uint16_t*>(out) = (uint16_t)word;
    } else {
        out[0] = (uint8_t)word;
        if (room > 1) out[1] = (uint8_t)(word >> 8);
        if (room > 2) out[2] = (uint8_t)(word >> 16);
    }
}

// Tiles per workgroup (256 threads, every thread one group in every tile, all reads requested
// first).  The two codebook families want different numbers, measured on MI355X:
//   * the uniform path costs few instructions per element and runs at the speed of its memory
//     traffic when the running wavefronts together cover a small window of the gradient: on
//     8 x 124 M fp32, 670 us with one tile per workgroup against 745 us with two, whether the
//     two are requested together, one after the other, adjacent or far apart;
//   * the level-table path costs twice the instructions, and a wavefront that holds only one
//     group has nothing in flight while it computes: with two tiles 8 x 124 M fp32 at b = 2 take
//     718 us instead of 785, 16 x 25.6 M at b = 3 307 instead of 346, and 4 x 10^9 bf16 with four
//     tiles (a bf16 tile is half the bytes) 1790 instead of 2440.
// The family is a property of the parameter records, which live on the device, so the host
// chooses by the family the caller names (tq_compress's `grid`); the kernel itself reads every
// bucket's record and computes what the record says, whatever shape it was launched in.
constexpr int compress_tiles(int dtype, bool table_path)
{
    return dtype == TQ_F32 ? (table_path ? 2 : 1) : (table_path ? 4 : 2);
}

template <int DTYPE, int BITS, bool STREAM, int T>
__global__ __launch_bounds__(kBlock) void tq_compress_kernel(
    const PtrTable g_tab, uint64_t d, uint64_t d_pad, uint64_t bucket_elems,
    uint32_t groups_per_bucket, const PtrTable params_tab, uint32_t seed_lo,
    uint32_t seed_hi, uint32_t first_worker, uint32_t step, const MutPtrTable payload_tab,
    uint64_t payload_bytes)
{
    const uint32_t blk = linear_block();
    const uint32_t bucket = blk / groups_per_bucket;
    const uint32_t grp = blk - bucket * groups_per_bucket;
    const uint64_t bstart = (uint64_t)bucket * bucket_elems;
    const uint64_t bend = bstart + bucket_elems < d_pad ? bstart + bucket_elems : d_pad;
    const uint64_t gbase = bstart + (uint64_t)grp * T * kTile;            // first element of the workgroup
    if (gbase >= bend) return;                                 // idle workgroup of a short last bucket
    // blockIdx.y = tensor of the batch; its worker id keys the random draws
    const void* __restrict__ g = g_tab.p[blockIdx.y];
    uint8_t* __restrict__ payload = static_cast<uint8_t*>(payload_tab.p[blockIdx.y]);
    const uint32_t worker = first_worker + blockIdx.y;
    const tq_params_t* P = static_cast<const tq_params_t*>(params_tab.p[blockIdx.y]) + bucket;

    __shared__ LevelLds tab;
    float lv[16];
    const float alpha = P->alpha;
    const float inv_step = P->inv_w[0];
    const bool nonuniform = P->grid != TQ_GRID_UNIFORM;        // uniform over the workgroup
    const uint32_t lane = threadIdx.x;                         // this thread's group within a tile
    bool first_cell_empty = false;                             // see encode_group's CLAMP
    if (nonuniform) {
        fill_level_lds(tab, P, (1u << BITS) - 1u);
#pragma unroll
        for (int j = 0; j < 16; ++j) lv[j] = P->level[j];       // wave-uniform: scalar loads
        first_cell_empty = !(lv[1] > lv[0]);
        __syncthreads();
    }

    // One Philox call per lane and tile; the high counter word stays scalar unless the low
    // word wraps inside the tile.
    auto draw = [&](uint64_t ebase, uint32_t (&rw)[4]) {
        const uint64_t qb = ebase >> 3;                        // first group of the tile (uniform)
        const uint32_t qb_lo = (uint32_t)qb, qb_hi = (uint32_t)(qb >> 32);
        const uint32_t q_lo = qb_lo + lane;
        if (qb_lo <= 0xFFFFFFFFu - kBlock) philox4x32_10(q_lo, qb_hi, worker, step, seed_lo, seed_hi, rw);
        else philox4x32_10(q_lo, qb_hi + (q_lo < qb_lo ? 1u : 0u), worker, step, seed_lo, seed_hi, rw);
    };

    const uint64_t lim = bend < d ? bend : d;
    if (gbase + (uint64_t)T * kTile <= lim) {
        // every lane owns a whole group in every tile: all reads first, the draws under them
        // (requesting the reads even earlier, before the codebook is set up, was slower: 708 us
        // against 668 on 8 x 124 M fp32)
        float x[T][8];
        uint32_t rw[T][4];
#pragma unroll
        for (int t = 0; t < T; ++t) load_group<DTYPE, STREAM>(g, gbase + (uint64_t)t * kTile + (uint64_t)lane * kGroup, x[t]);
#pragma unroll
        for (int t = 0; t < T; ++t) {
            draw(gbase + (uint64_t)t * kTile, rw[t]);
            asm volatile("" : "+v"(rw[t][0]));                 // computed here, under the loads
        }
#pragma unroll
        for (int t = 0; t < T; ++t) {
            replace_nan(x[t]);
            uint32_t word;
            if (!nonuniform) word = encode_group<BITS, TQ_GRID_UNIFORM, false>(x[t], rw[t], 8, alpha, inv_step, lv, tab);
            else if (first_cell_empty) word = encode_group<BITS, TQ_GRID_NONUNIFORM, false, true>(x[t], rw[t], 8, alpha, inv_step, lv, tab);
            else word = encode_group<BITS, TQ_GRID_NONUNIFORM, false, false>(x[t], rw[t], 8, alpha, inv_step, lv, tab);
            store_codes<BITS>(payload + (((gbase + (uint64_t)t * kTile) >> 3) + lane) * (uint64_t)BITS, word);
        }
        return;
    }

    // the last workgroup of a bucket: tile by tile, lanes past the end idle, the tensor's
    // ragged last group element by element
    for (int t = 0; t < T; ++t) {
        const uint64_t ebase = gbase + (uint64_t)t * kTile;
        const uint64_t e0 = ebase + (uint64_t)lane * kGroup;
        const uint64_t byte_off = ((ebase >> 3) + lane) * (uint64_t)BITS;
        if (e0 >= bend || byte_off >= payload_bytes) continue;
        uint32_t word = 0;                                     // groups wholly in the padding encode as 0
        if (e0 + kGroup <= d) {
            float x[8];
            load_group<DTYPE, false>(g, e0, x);
            uint32_t rw[4];
            draw(ebase, rw);
            replace_nan(x);
            word = nonuniform ? encode_group<BITS, TQ_GRID_NONUNIFORM, false>(x, rw, 8, alpha, inv_step, lv, tab)
                              : encode_group<BITS, TQ_GRID_UNIFORM, false>(x, rw, 8, alpha, inv_step, lv, tab);
        } else if (e0 < d) {
            const int n_valid = (int)(d - e0);
            float x[8];
#pragma unroll
            for (int j = 0; j < 8; ++j) x[j] = (j < n_valid) ? load_one<DTYPE>(g, e0 + j) : 0.0f;
            uint32_t rw[4];
            draw(ebase, rw);
            replace_nan(x);
            word = nonuniform ? encode_group<BITS, TQ_GRID_NONUNIFORM, true>(x, rw, n_valid, alpha, inv_step, lv, tab)
                              : encode_group<BITS, TQ_GRID_UNIFORM, true>(x, rw, n_valid, alpha, inv_step, lv, tab);
        }
        store_codes<BITS>(payload + byte_off, word, payload_bytes - byte_off);
    }
}

// tq_compress_segments: the same client step with one (alpha, codebook) per variable-size
// segment of the flat gradient (Sec. V: the layers of a network are quantized independently).
// One tile of 2048 elements per workgroup, wherever the segments fall: the workgroup finds the
// segment its tile starts in and takes the segments that overlap the tile one after the other
// (a lane's group of 8 lies in exactly one, the offsets being multiples of 128); large layers
// are the rule, so almost every workgroup makes one pass.  The last segment also owns the
// padding up to a multiple of 128 elements.  No access depends on the table being well-formed:
// the segment index stays inside [0, nseg) and every element access is bounded by d.
template <int DTYPE, int BITS>
__global__ __launch_bounds__(kBlock) void tq_compress_segments_kernel(
    const PtrTable g_tab, uint64_t d, uint64_t d_pad, const uint64_t* __restrict__ seg_off, uint32_t nseg,
    const SegHints hints, const PtrTable params_tab, uint32_t seed_lo, uint32_t seed_hi, uint32_t first_worker, uint32_t step,
    const MutPtrTable payload_tab, uint64_t payload_bytes)
{
    const uint64_t ebase = (uint64_t)linear_block() * kTile;
    if (ebase >= d_pad) return;                                // padding of a folded grid
    // blockIdx.y = tensor of the batch; its worker id keys the random draws
    const void* __restrict__ g = g_tab.p[blockIdx.y];
    const tq_params_t* __restrict__ params = static_cast<const tq_params_t*>(params_tab.p[blockIdx.y]);
    uint8_t* __restrict__ payload = static_cast<uint8_t*>(payload_tab.p[blockIdx.y]);
    const uint32_t worker = first_worker + blockIdx.y;
    // positions inside the tile are 32-bit offsets from its first element (which is the same for
    // the whole workgroup): the tensor's end, the payload's end and the segments' ends as such
    const uint32_t lane = threadIdx.x;
    const uint32_t rel = lane * kGroup;                                              // this lane's group
    const uint32_t tile_len = (uint32_t)(ebase + kTile < d_pad ? kTile : d_pad - ebase);   // multiple of 128
    const uint32_t d_rel = ebase < d ? (uint32_t)(d - ebase < (uint64_t)kTile ? d - ebase : kTile) : 0u;
    const uint64_t tile_byte = (ebase >> 3) * (uint64_t)BITS;                         // payload offset of the tile
    const uint32_t pay_rel =                                                          // payload bytes from there on, capped
        tile_byte < payload_bytes ? (uint32_t)(payload_bytes - tile_byte < (uint64_t)kTile ? payload_bytes - tile_byte : kTile) : 0u;
    const uint32_t byte_rel = lane * (uint32_t)BITS;
    __shared__ LevelLds tab;

    // The lane's group and its draws depend on its position alone: the values are requested and
    // the draws computed before the segment is looked up (a chain of dependent scalar loads).
    const int n_valid = rel >= d_rel ? 0 : (d_rel - rel >= (uint32_t)kGroup ? kGroup : (int)(d_rel - rel));
    float x[8];
    if (n_valid == kGroup) {
        load_group<DTYPE, false>(g, ebase + rel, x);
    } else {
#pragma unroll
        for (int j = 0; j < 8; ++j) x[j] = (j < n_valid) ? load_one<DTYPE>(g, ebase + rel + j) : 0.0f;
    }
    uint32_t rw[4];
    {
        // one Philox call per lane; the high counter word stays scalar unless the low word wraps inside the tile
        const uint64_t qb = ebase >> 3;
        const uint32_t qb_lo = (uint32_t)qb, qb_hi = (uint32_t)(qb >> 32);
        const uint32_t q_lo = qb_lo + lane;
        if (qb_lo <= 0xFFFFFFFFu - kBlock) philox4x32_10(q_lo, qb_hi, worker, step, seed_lo, seed_hi, rw);
        else philox4x32_10(q_lo, qb_hi + (q_lo < qb_lo ? 1u : 0u), worker, step, seed_lo, seed_hi, rw);
        asm volatile("" : "+v"(rw[0]));                        // computed here, under the loads
    }

    uint32_t s = find_segment(seg_off, nseg, ebase < d ? ebase : d - 1, hints);
    replace_nan(x);
    {
        // Nearly every tile lies inside one segment, with all its groups whole and its codes inside
        // the payload: straight-line code, as for a bucket.  The test uses the very segment ends
        // the loop below would use, so both ways write the same bytes.
        const uint64_t seg_lo = seg_off[s];
        const uint64_t seg_hi = s + 1 < nseg ? seg_off[s + 1] : d_pad;
        if (seg_lo <= ebase && seg_hi >= ebase + kTile && d_rel == (uint32_t)kTile &&
            pay_rel >= (uint32_t)kBlock * (uint32_t)BITS) {
            const tq_params_t* P = params + s;
            const float alpha = P->alpha;
            const float inv_step = P->inv_w[0];
            float lv[16];
            uint32_t word;
            if (P->grid != TQ_GRID_UNIFORM) {                  // uniform over the workgroup
                fill_level_lds(tab, P, (1u << BITS) - 1u);
#pragma unroll
                for (int j = 0; j < 16; ++j) lv[j] = P->level[j];
                __syncthreads();
                word = encode_group<BITS, TQ_GRID_NONUNIFORM, false>(x, rw, 8, alpha, inv_step, lv, tab);
            } else {
                word = encode_group<BITS, TQ_GRID_UNIFORM, false>(x, rw, 8, alpha, inv_step, lv, tab);
            }
            store_codes<BITS>(payload + tile_byte + byte_rel, word);
            return;
        }
    }
    for (;;) {
        const uint64_t seg_lo = seg_off[s];
        const uint64_t seg_hi = s + 1 < nseg ? seg_off[s + 1] : d_pad;
        // the part of the tile that belongs to this segment, as offsets from the tile's start
        const uint32_t lo_rel = (uint32_t)(seg_lo > ebase ? (seg_lo - ebase < (uint64_t)tile_len ? seg_lo - ebase : tile_len) : 0);
        const uint32_t hi_rel = (uint32_t)(seg_hi > ebase ? (seg_hi - ebase < (uint64_t)tile_len ? seg_hi - ebase : tile_len) : 0);
        const tq_params_t* P = params + s;
        float lv[16];
        const float alpha = P->alpha;
        const float inv_step = P->inv_w[0];
        const bool nonuniform = P->grid != TQ_GRID_UNIFORM;    // uniform over the workgroup
        if (nonuniform) {
            fill_level_lds(tab, P, (1u << BITS) - 1u);
#pragma unroll
            for (int j = 0; j < 16; ++j) lv[j] = P->level[j];   // wave-uniform: scalar loads
            __syncthreads();
        }
        if (rel >= lo_rel && rel < hi_rel && byte_rel < pay_rel) {
            uint32_t word = 0;                                 // a group wholly in the padding encodes as 0
            if (n_valid == kGroup)
                word = nonuniform ? encode_group<BITS, TQ_GRID_NONUNIFORM, false>(x, rw, 8, alpha, inv_step, lv, tab)
                                  : encode_group<BITS, TQ_GRID_UNIFORM, false>(x, rw, 8, alpha, inv_step, lv, tab);
            else if (n_valid > 0)
                word = nonuniform ? encode_group<BITS, TQ_GRID_NONUNIFORM, true>(x, rw, n_valid, alpha, inv_step, lv, tab)
                                  : encode_group<BITS, TQ_GRID_UNIFORM, true>(x, rw, n_valid, alpha, inv_step, lv, tab);
            store_codes<BITS>(payload + tile_byte + byte_rel, word, (uint64_t)(pay_rel - byte_rel));
        }
        if (hi_rel >= tile_len || s + 1 >= nseg) break;
        ++s;
        __syncthreads();                                       // before the next segment's table replaces this one
    }
}

// tq_quantize_dequantize: out[e] = Q[T_alpha(g[e])] as the server would reconstruct it from
// this worker's message (the level of the code tq_compress_kernel would have written: same
// draws, same arithmetic), without the round trip through a payload.  One tile per workgroup.
template <int DTYPE, int BITS, bool ACC>
__global__ __launch_bounds__(kBlock) void tq_simulate_kernel(
    const void* __restrict__ g, uint64_t d, uint64_t d_pad, uint64_t bucket_elems, uint32_t tiles_per_bucket,
    const tq_params_t* __restrict__ params, uint32_t seed_lo, uint32_t seed_hi, uint32_t worker, uint32_t step,
    float* __restrict__ out)
{
    constexpr uint32_t S = (1u << BITS) - 1u;
    const TileGeom t = tile_geom(linear_block(), d_pad, bucket_elems, tiles_per_bucket);
    const uint64_t bend = t.eend < d ? t.eend : d;
    if (t.ebase >= bend) return;
    const tq_params_t* P = params + t.bucket;

    __shared__ LevelLds tab;                                   // levels for the look-up of both families
    float lv[16];
    const float alpha = P->alpha;
    const float inv_step = P->inv_w[0];
    const bool nonuniform = P->grid != TQ_GRID_UNIFORM;        // uniform over the workgroup
    fill_level_lds(tab, P, S);
#pragma unroll
    for (int j = 0; j < 16; ++j) lv[j] = P->level[j];           // wave-uniform: scalar loads
    __syncthreads();

    const uint64_t e0 = t.ebase + (uint64_t)threadIdx.x * kGroup;
    if (e0 >= bend) return;
    const int n_valid = bend - e0 >= (uint64_t)kGroup ? kGroup : (int)(bend - e0);
    float x[8];
    if (n_valid == kGroup) {
        load_group<DTYPE, false>(g, e0, x);
    } else {
#pragma unroll
        for (int j = 0; j < 8; ++j) x[j] = (j < n_valid) ? load_one<DTYPE>(g, e0 + j) : 0.0f;
    }
    const uint64_t q = e0 >> 3;
    uint32_t rw[4];
    philox4x32_10((uint32_t)q, (uint32_t)(q >> 32), worker, step, seed_lo, seed_hi, rw);
    replace_nan(x);
    float y[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) {
        const uint32_t r = (j & 1) ? (rw[j >> 1] >> 16) : (rw[j >> 1] & 0xFFFFu);
        const uint32_t code = nonuniform ? quantize<BITS, TQ_GRID_NONUNIFORM>(x[j], (float)r, alpha, inv_step, lv, tab)
                                         : quantize<BITS, TQ_GRID_UNIFORM>(x[j], (float)r, alpha, inv_step, lv, tab);
        y[j] = tab.e[code & S].x;
    }
    float* o = out + e0;
    if (n_valid == kGroup) {
        float4* o4 = reinterpret_cast<float4*>(o);
        float4 a = make_float4(y[0], y[1], y[2], y[3]), b = make_float4(y[4], y[5], y[6], y[7]);
        if constexpr (ACC) {
            const float4 pa = o4[0], pb = o4[1];
            a.x = pa.x + a.x; a.y = pa.y + a.y; a.z = pa.z + a.z; a.w = pa.w + a.w;
            b.x = pb.x + b.x; b.y = pb.y + b.y; b.z = pb.z + b.z; b.w = pb.w + b.w;
        }
        o4[0] = a;
        o4[1] = b;
    } else {
#pragma clang loop unroll(disable)
        for (int j = 0; j < n_valid; ++j) {
            float v = y[0];
#pragma unroll
            for (int k = 1; k < 8; ++k) v = (j == k) ? y[k] : v;
            o[j] = ACC ? o[j] + v : v;
        }
    }
}

}  // namespace tq

namespace {

template <int DTYPE, bool STREAM, int T>
hipError_t launch(int bits, dim3 blocks, hipStream_t st, const tq::PtrTable& g, uint64_t d, uint64_t d_pad,
                  uint64_t be, uint32_t tpb, const tq::PtrTable& params, uint64_t seed, uint32_t first_worker,
                  uint32_t step, const tq::MutPtrTable& payload, uint64_t pbytes)
{
    const uint32_t slo = (uint32_t)seed, shi = (uint32_t)(seed >> 32);
    const dim3 threads(tq::kBlock);
    switch (bits) {
        case 2:
            hipLaunchKernelGGL((tq::tq_compress_kernel<DTYPE, 2, STREAM, T>), blocks, threads, 0, st, g, d, d_pad, be,
                               tpb, params, slo, shi, first_worker, step, payload, pbytes);
            break;
        case 3:
            hipLaunchKernelGGL((tq::tq_compress_kernel<DTYPE, 3, STREAM, T>), blocks, threads, 0, st, g, d, d_pad, be,
                               tpb, params, slo, shi, first_worker, step, payload, pbytes);
            break;
        default:
            hipLaunchKernelGGL((tq::tq_compress_kernel<DTYPE, 4, STREAM, T>), blocks, threads, 0, st, g, d, d_pad, be,
                               tpb, params, slo, shi, first_worker, step, payload, pbytes);
            break;
    }
    return hipGetLastError();
}

}  // namespace

// Host side of tq_compress / tq_compress_multi after the argument checks of the C entry
// points: `count` same-shaped tensors in one launch (grid.y), workers first_worker + 0..count-1.
// `grid` (the family the caller names) only chooses the number of tiles per workgroup.
hipError_t tq_launch_compress(const void* const* g, int count, int dtype, uint64_t d, uint64_t bucket_elems,
                              const tq_params_t* const* params, int bits, int grid, uint64_t seed,
                              uint32_t first_worker, uint32_t step, void* const* payload, hipStream_t st)
{
    const uint64_t d_pad = (d + 127) / 128 * 128;
    const uint64_t be = bucket_elems ? bucket_elems : d_pad;
    const uint64_t nb = (d_pad + be - 1) / be;
    const bool table_path = grid != TQ_GRID_UNIFORM;
    const uint64_t tt = (uint64_t)tq::compress_tiles(dtype, table_path);
    const uint64_t tpb = ((be + tq::kTile - 1) / tq::kTile + tt - 1) / tt;    // workgroups per bucket
    const uint64_t nblocks = nb * tpb;
    dim3 blocks;
    if (count < 1 || count > tq::kMaxBatch || !tq::fold_grid(nblocks, tq::kBlock, (unsigned)count, blocks))
        return hipErrorInvalidValue;
    const uint64_t pbytes = tq_payload_bytes(d, bits);
    tq::PtrTable gt{}, pt{};
    tq::MutPtrTable yt{};
    for (int i = 0; i < count; ++i) { gt.p[i] = g[i]; pt.p[i] = params[i]; yt.p[i] = payload[i]; }
    // non-temporal loads while the batch can still be (partly) cached from the statistics pass:
    // up to twice the 256 MiB of the memory-side cache
    const bool stream = (uint64_t)count * d * (dtype == TQ_F32 ? 4u : 2u) <= (512ull << 20);
#define TQ_LAUNCH_COMPRESS(DT, ST, TP) \
    launch<DT, ST, tq::compress_tiles(DT, TP)>(bits, blocks, st, gt, d, d_pad, be, (uint32_t)tpb, pt, seed, \
                                               first_worker, step, yt, pbytes)
#define TQ_LAUNCH_COMPRESS_ST(DT, TP) (stream ? TQ_LAUNCH_COMPRESS(DT, true, TP) : TQ_LAUNCH_COMPRESS(DT, false, TP))
    if (dtype == TQ_F32) return table_path ? TQ_LAUNCH_COMPRESS_ST(TQ_F32, true) : TQ_LAUNCH_COMPRESS_ST(TQ_F32, false);
    return table_path ? TQ_LAUNCH_COMPRESS_ST(TQ_BF16, true) : TQ_LAUNCH_COMPRESS_ST(TQ_BF16, false);
#undef TQ_LAUNCH_COMPRESS_ST
#undef TQ_LAUNCH_COMPRESS
}

// Host side of tq_quantize_dequantize after the argument checks of the C entry point.
hipError_t tq_launch_simulate(const void* g, int dtype, uint64_t d, uint64_t bucket_elems, const tq_params_t* params,
                              int bits, uint64_t seed, uint32_t worker, uint32_t step, int accumulate, float* out,
                              hipStream_t st)
{
    const uint64_t d_pad = (d + 127) / 128 * 128;
    const uint64_t be = bucket_elems ? bucket_elems : d_pad;
    const uint64_t nb = (d_pad + be - 1) / be;
    const uint64_t tpb = (be + tq::kTile - 1) / tq::kTile;
    const uint64_t nblocks = nb * tpb;
    dim3 blocks;
    if (!tq::fold_grid(nblocks, tq::kBlock, 1, blocks)) return hipErrorInvalidValue;
    const uint32_t slo = (uint32_t)seed, shi = (uint32_t)(seed >> 32);
    const dim3 threads(tq::kBlock);
#define TQ_LAUNCH_SIM(DT, B)                                                                                      \
    do {                                                                                                          \
        if (accumulate)                                                                                           \
            hipLaunchKernelGGL((tq::tq_simulate_kernel<DT, B, true>), blocks, threads, 0, st, g, d, d_pad, be,    \
                               (uint32_t)tpb, params, slo, shi, worker, step, out);                               \
        else                                                                                                      \
            hipLaunchKernelGGL((tq::tq_simulate_kernel<DT, B, false>), blocks, threads, 0, st, g, d, d_pad, be,   \
                               (uint32_t)tpb, params, slo, shi, worker, step, out);                               \
    } while (0)
#define TQ_LAUNCH_SIM_B(DT)                      \
    switch (bits) {                              \
        case 2: TQ_LAUNCH_SIM(DT, 2); break;     \
        case 3: TQ_LAUNCH_SIM(DT, 3); break;     \
        default: TQ_LAUNCH_SIM(DT, 4); break;    \
    }
    if (dtype == TQ_F32) { TQ_LAUNCH_SIM_B(TQ_F32) } else { TQ_LAUNCH_SIM_B(TQ_BF16) }
#undef TQ_LAUNCH_SIM_B
#undef TQ_LAUNCH_SIM
    return hipGetLastError();
}


// Host side of tq_compress_segments after the argument checks of the C entry point.
hipError_t tq_launch_compress_segments(const void* const* g, int count, int dtype, uint64_t d, const uint64_t* seg_off,
                                       const uint64_t* seg_host, uint64_t nseg, const tq_params_t* const* params, int bits, uint64_t seed,
                                       uint32_t first_worker, uint32_t step, void* const* payload, hipStream_t st)
{
    const uint64_t d_pad = (d + 127) / 128 * 128;
    const uint64_t nblocks = (d_pad + tq::kTile - 1) / tq::kTile;
    dim3 blocks;
    if (count < 1 || count > tq::kMaxBatch || nseg > 0xFFFFFFFFull ||
        !tq::fold_grid(nblocks, tq::kBlock, (unsigned)count, blocks))
        return hipErrorInvalidValue;
    tq::PtrTable gt{}, pt{};
    tq::MutPtrTable yt{};
    for (int i = 0; i < count; ++i) { gt.p[i] = g[i]; pt.p[i] = params[i]; yt.p[i] = payload[i]; }
    const uint32_t slo = (uint32_t)seed, shi = (uint32_t)(seed >> 32);
    const uint64_t pbytes = tq_payload_bytes(d, bits);
    const dim3 threads(tq::kBlock);
    const tq::SegHints hints = tq::make_seg_hints(seg_host, nseg, d);
#define TQ_LAUNCH_CSEG(DT, B)                                                                                   \
    hipLaunchKernelGGL((tq::tq_compress_segments_kernel<DT, B>), blocks, threads, 0, st, gt, d, d_pad, seg_off, \
                       (uint32_t)nseg, hints, pt, slo, shi, first_worker, step, yt, pbytes)
#define TQ_LAUNCH_CSEG_B(DT)                      \
    switch (bits) {                               \
        case 2: TQ_LAUNCH_CSEG(DT, 2); break;     \
        case 3: TQ_LAUNCH_CSEG(DT, 3); break;     \
        default: TQ_LAUNCH_CSEG(DT, 4); break;    \
    }
    if (dtype == TQ_F32) { TQ_LAUNCH_CSEG_B(TQ_F32) } else { TQ_LAUNCH_CSEG_B(TQ_BF16) }
#undef TQ_LAUNCH_CSEG_B
#undef TQ_LAUNCH_CSEG
    return hipGetLastError();
}
