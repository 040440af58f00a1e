// Host check of the payload address arithmetic the decode kernels use (tq_layout.h, compiled
// here for the CPU): for every tensor length d and code width b, every group's load must lie
// inside the payload, and the bits it selects must be the group's own.
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <vector>

#include "tq_layout.h"

static uint64_t payload_bytes(uint64_t d, int bits) { return ((d * bits + 7) / 8 + 15) / 16 * 16; }

int main(int argc, char** argv)
{
    const uint64_t d_max = argc > 1 ? strtoull(argv[1], nullptr, 10) : 4096;
    unsigned long long checked = 0;
    for (int bits = 2; bits <= 4; ++bits) {
        for (uint64_t d = 1; d <= d_max; ++d) {
            const uint64_t pb = payload_bytes(d, bits);
            std::vector<unsigned char> pay(pb, 0);
            // reference stream: element e holds code (e * 7 + 3) mod 2^b at bits [e b, e b + b)
            for (uint64_t e = 0; e < d; ++e) {
                const unsigned code = (unsigned)((e * 7 + 3) & ((1u << bits) - 1u));
                for (int t = 0; t < bits; ++t)
                    if ((code >> t) & 1u) pay[(e * bits + t) >> 3] |= (unsigned char)(1u << ((e * bits + t) & 7));
            }
            const uint64_t groups = (d + 7) / 8;
            for (uint64_t q = 0; q < groups; ++q) {
                const tq::CodeLoad c = tq::code_load(q, bits, pb);
                if (c.load_off + c.width > pb || c.first_bit > 24 || (bits != 3 && c.first_bit != 0)) {
                    printf("out of bounds: bits %d d %llu group %llu load [%llu, +%u) payload %llu\n", bits,
                           (unsigned long long)d, (unsigned long long)q, (unsigned long long)c.load_off, c.width,
                           (unsigned long long)pb);
                    return 1;
                }
                uint32_t w = 0;
                memcpy(&w, pay.data() + c.load_off, c.width);
                w >>= c.first_bit;
                const uint64_t n_valid = d - q * 8 < 8 ? d - q * 8 : 8;
                for (uint64_t j = 0; j < n_valid; ++j) {
                    const uint64_t e = q * 8 + j;
                    const unsigned want = (unsigned)((e * 7 + 3) & ((1u << bits) - 1u));
                    const unsigned got = (w >> (j * bits)) & ((1u << bits) - 1u);
                    if (got != want) {
                        printf("wrong code: bits %d d %llu element %llu got %u want %u\n", bits,
                               (unsigned long long)d, (unsigned long long)e, got, want);
                        return 1;
                    }
                    ++checked;
                }
            }
        }
    }
    printf("ok %llu codes\n", checked);
    return 0;
}
