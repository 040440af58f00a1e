// Address arithmetic of the packed payload, free of any HIP type so that the very functions
// the kernels use can also be compiled for the host and checked there over every size.
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

}  // namespace tq
