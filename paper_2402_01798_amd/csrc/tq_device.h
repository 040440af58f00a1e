// Device-side helpers shared by the gfx950 kernels of libtq.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stdlib.h>

#include "tq.h"
#include "tq_layout.h"

namespace tq {

constexpr int kGroup = 8;            // elements served by one Philox4x32 call = one lane's work item
constexpr int kBlock = 256;          // threads per workgroup (4 wavefronts of 64)
constexpr int kTile = kBlock * kGroup;  // elements per workgroup tile (2048)

// a ^ b ^ c in one instruction (the three-input bitwise operation of this ISA, truth table 0x96).
__device__ __forceinline__ uint32_t xor3(uint32_t a, uint32_t b, uint32_t c)
{
    return __builtin_amdgcn_bitop3_b32(a, b, c, 0x96);
}

// Philox4x32-10 (Salmon et al., SC'11): ten rounds of two 32x32->64 multiplies whose
// halves are crossed over and xored with a Weyl-sequence round key.  Operands that are
// uniform over the wavefront (key, worker, step, high counter word) stay in SGPRs and
// their multiplies run on the scalar unit; only the lane's counter word c0 is per-lane.
// The xors of the first three rounds are grouped so that the uniform pair is combined on
// the scalar unit (first round: c1, c2, c3 uniform; second: c0, c1; third: c3); from then
// on every word differs per lane and each output word is one three-input xor.
__device__ __forceinline__ void philox4x32_10(uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3,
                                              uint32_t k0, uint32_t k1, uint32_t (&out)[4])
{
#pragma unroll
    for (int r = 0; r < 10; ++r) {
        const uint64_t p0 = (uint64_t)0xD2511F53u * c0;
        const uint64_t p1 = (uint64_t)0xCD9E8D57u * c2;
        const uint32_t h0 = (uint32_t)(p0 >> 32), h1 = (uint32_t)(p1 >> 32);
        uint32_t n0, n2;
        if (r == 0) { n0 = h1 ^ c1 ^ k0; n2 = h0 ^ (c3 ^ k1); }
        else if (r == 1) { n0 = h1 ^ (c1 ^ k0); n2 = c3 ^ (h0 ^ k1); }
        else if (r == 2) { n0 = xor3(h1, c1, k0); n2 = h0 ^ (c3 ^ k1); }
        else { n0 = xor3(h1, c1, k0); n2 = xor3(h0, c3, k1); }
        c1 = (uint32_t)p1;
        c3 = (uint32_t)p0;
        c0 = n0;
        c2 = n2;
        k0 += 0x9E3779B9u;
        k1 += 0xBB67AE85u;
    }
    out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

// Pointer table of a batched launch: blockIdx.y selects the tensor (one simulated worker, or
// one of several same-shaped tensors of one worker).  Passed by value in the kernel arguments.
constexpr int kMaxBatch = TQ_MAX_WORKERS;
struct PtrTable {
    const void* p[kMaxBatch];
};
struct MutPtrTable {
    void* p[kMaxBatch];
};

// A launch of `nblocks` workgroups.  The dispatch packet counts work-items per dimension in 32
// bits, so blocks * threads of one dimension must stay below 2^32: long grids are folded into
// (x, z), grid.y being the tensor of a batch.  Workgroups past `nblocks` (the last z-row is
// padded) find nothing to do and exit; every kernel tests for that before touching memory.
__device__ __forceinline__ uint32_t linear_block() { return blockIdx.x + blockIdx.z * gridDim.x; }

// Builds with -DTQ_TEST_GRID_FOLD (the test build only) read TQ_TEST_MAX_GRID_X from the
// environment, once, to lower the fold point, so that tests can drive the folded path of every
// kernel with small inputs; the product build has no such hook.
inline bool fold_grid(uint64_t nblocks, unsigned threads, unsigned count, dim3& grid)
{
#ifdef TQ_TEST_GRID_FOLD
    static const uint64_t forced = [] {
        const char* e = getenv("TQ_TEST_MAX_GRID_X");
        return e ? strtoull(e, nullptr, 10) : 0ull;
    }();
#else
    constexpr uint64_t forced = 0;
#endif
    uint64_t max_x = (1ull << 31) / threads;                       // x * threads <= 2^31
    if (forced > 0 && forced < max_x) max_x = forced;
    if (nblocks == 0 || nblocks > 0xFFFFFFFFull) return false;
    const uint64_t gx = nblocks < max_x ? nblocks : max_x;
    const uint64_t gz = (nblocks + gx - 1) / gx;
    if (gz > 65535 || gx * gz > 0xFFFFFFFFull) return false;
    grid = dim3((unsigned)gx, count, (unsigned)gz);
    return true;
}

// Tile geometry shared by compress and decode.  Workgroup `blk` owns elements
// [ebase, ebase + kTile) of bucket `bucket`, cut at `eend` (the bucket's end, the last
// bucket's end being d rounded up to a multiple of 128 so the payload padding is covered).
struct TileGeom {
    uint64_t bucket;
    uint64_t ebase;
    uint64_t eend;
};

__device__ __forceinline__ TileGeom tile_geom(uint32_t blk, uint64_t d_pad, uint64_t bucket_elems,
                                              uint32_t tiles_per_bucket)
{
    TileGeom t;
    const uint32_t b = blk / tiles_per_bucket;
    const uint32_t tile = blk - b * tiles_per_bucket;
    t.bucket = b;
    const uint64_t bstart = (uint64_t)b * bucket_elems;
    t.ebase = bstart + (uint64_t)tile * kTile;
    const uint64_t bend = bstart + bucket_elems;
    t.eend = bend < d_pad ? bend : d_pad;
    return t;
}

}  // namespace tq
