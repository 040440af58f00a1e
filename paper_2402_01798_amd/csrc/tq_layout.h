// Address arithmetic of the packed payload and the segment look-up, free of any HIP type so that
// the very functions the kernels use can also be compiled for the host and checked there.
#pragma once

#include <stdint.h>

#if defined(__HIPCC__)
#define TQ_HD __host__ __device__ __forceinline__
#else
#define TQ_HD inline
#endif

namespace tq {

// Where the decode kernels read the 8 codes of group q (b bytes at byte q*b of a payload of
// `payload_bytes` bytes, a multiple of 16): one load of `width` bytes at byte `load_off`,
// the codes starting at bit `first_bit` of the loaded word.
//   b = 2: the group's own 2 bytes;  b = 4: its own 4 bytes;
//   b = 3: the 4 bytes starting at the group (an unaligned dword; the fourth byte belongs to
//          the next group) -- unless those 4 bytes would reach past the end of the payload,
//          which happens for the last group(s): then the payload's LAST dword, in which the
//          group starts at byte 1, 2 or 3.  A ragged last group needs only its first 1 or 2
//          bytes; the bytes "missing" after the end would hold codes of elements that do
//          not exist, and the kernels never use those.
// No byte outside [0, payload_bytes) is ever touched.
struct CodeLoad {
    uint64_t load_off;
    uint32_t first_bit;
    uint32_t width;
};

TQ_HD CodeLoad code_load(uint64_t q, int bits, uint64_t payload_bytes)
{
    CodeLoad c;
    const uint64_t off = q * (uint64_t)bits;
    c.load_off = off;
    c.first_bit = 0;
    c.width = bits == 2 ? 2u : 4u;
    if (bits == 3 && off + 4 > payload_bytes) {
        c.load_off = payload_bytes - 4;
        c.first_bit = (uint32_t)(off - c.load_off) * 8u;
    }
    return c;
}


// Variable-size segments: the largest s in [0, nseg) with seg_off[s] <= pos.  Every step reads
// inside [0, nseg], whatever the table holds.
TQ_HD uint32_t find_segment(const uint64_t* __restrict__ seg_off, uint32_t nseg, uint64_t pos)
{
    uint32_t lo = 0, hi = nseg;
    while (hi - lo > 1) {
        const uint32_t mid = lo + ((hi - lo) >> 1);
        if (seg_off[mid] <= pos) lo = mid; else hi = mid;
    }
    return lo;
}

// Hints that shorten the search: the tensor in kSegHintBlocks blocks of 2^shift elements (a
// power of two of at least one tile, so a tile lies in one block) and, per block, the segment
// that holds its first element.  Built on the host from the caller's host copy of the table;
// without one, a single block that spans the tensor (the search is then the full one).  The
// hints only narrow the range: every read stays inside [0, nseg) whatever they hold.
constexpr int kSegHintBlocks = 256;
struct SegHints {
    uint32_t shift;
    uint32_t first[kSegHintBlocks + 1];
};

inline SegHints make_seg_hints(const uint64_t* seg_host, uint64_t nseg, uint64_t d)
{
    SegHints h;
    h.shift = 63;
    for (int j = 0; j <= kSegHintBlocks; ++j) h.first[j] = j == 0 ? 0u : (uint32_t)(nseg - 1);
    if (!seg_host || nseg < 2) return h;
    uint32_t shift = 11;                                            // 2048 elements: one tile
    while (((uint64_t)kSegHintBlocks << shift) < d) ++shift;
    h.shift = shift;
    uint64_t s = 0;                                                 // the table ascends: one sweep
    for (int j = 0; j <= kSegHintBlocks; ++j) {
        const uint64_t pos = (uint64_t)j << shift;
        while (s + 1 < nseg && seg_host[s + 1] <= pos) ++s;
        h.first[j] = (uint32_t)s;
    }
    return h;
}

TQ_HD uint32_t find_segment(const uint64_t* __restrict__ seg_off, uint32_t nseg, uint64_t pos,
                                                 const SegHints& hints)
{
    uint64_t j = pos >> hints.shift;
    j = j < (uint64_t)(kSegHintBlocks - 1) ? j : (uint64_t)(kSegHintBlocks - 1);
    uint32_t lo = hints.first[j], hi = hints.first[j + 1] + 1u;
    lo = lo < nseg ? lo : nseg - 1;
    hi = hi < nseg ? hi : nseg;
    hi = hi > lo ? hi : lo + 1;
    while (hi - lo > 1) {
        const uint32_t mid = lo + ((hi - lo) >> 1);
        if (seg_off[mid] <= pos) lo = mid; else hi = mid;
    }
    return lo;
}

// Equal shares of a batch counted in tiles (the statistics kernels): share w of `groups` is the
// tiles [share_start(w), share_start(w + 1)) of `total_tiles`.
TQ_HD uint64_t share_start(uint64_t w, uint64_t total_tiles, uint32_t groups)
{
    return w * total_tiles / groups;
}

// The share that holds a tile: the largest w with share_start(w) <= tile.
TQ_HD uint32_t share_of_tile(uint64_t tile, uint64_t total_tiles, uint32_t groups)
{
    return (uint32_t)(((tile + 1) * groups - 1) / total_tiles);
}

}  // namespace tq
