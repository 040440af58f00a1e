// Host check of the payload address arithmetic the decode kernels use (tq_layout.h, compiled
// here for the CPU): for every tensor length d and code width b, every group's load must lie
// inside the payload, and the bits it selects must be the group's own.  Also the segment look-up
// (plain, hinted, and with arbitrary hints) and the arithmetic of the statistics kernels' shares.
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
    // Segment look-up: with hints built from the table, with no hints, and with hints that hold
    // anything at all, the answer is the plain search's and every read stays inside the table.
    unsigned long long looked = 0;
    uint64_t rng = 0x9E3779B97F4A7C15ull;
    auto next = [&]() { rng ^= rng << 13; rng ^= rng >> 7; rng ^= rng << 17; return rng; };
    for (int rep = 0; rep < 150; ++rep) {
        const uint64_t nseg = 1 + next() % (rep < 50 ? 5 : (rep < 100 ? 300 : 3000));
        std::vector<uint64_t> off(nseg + 1, 0);
        for (uint64_t s = 1; s <= nseg; ++s) off[s] = off[s - 1] + 128 * (1 + next() % (next() % 16 == 0 ? 4000 : 40));
        const uint64_t d = off[nseg] - next() % 128;                  // a ragged last segment
        off[nseg] = d;
        const tq::SegHints good = tq::make_seg_hints(off.data(), nseg, d);
        const tq::SegHints none = tq::make_seg_hints(nullptr, nseg, d);
        tq::SegHints junk = good;
        for (int j = 0; j <= tq::kSegHintBlocks; ++j) junk.first[j] = (uint32_t)next();
        uint64_t want = 0;
        for (uint64_t pos = 0; pos < d; pos += 2048) {                // the tile starts the kernels ask for
            while (want + 1 < nseg && off[want + 1] <= pos) ++want;
            const uint32_t a = tq::find_segment(off.data(), (uint32_t)nseg, pos);
            const uint32_t b = tq::find_segment(off.data(), (uint32_t)nseg, pos, good);
            const uint32_t c = tq::find_segment(off.data(), (uint32_t)nseg, pos, none);
            const uint32_t e = tq::find_segment(off.data(), (uint32_t)nseg, pos, junk);
            if (a != want || b != want || c != want || e >= nseg) {
                printf("segment look-up: nseg %llu pos %llu want %llu got %u %u %u %u\n", (unsigned long long)nseg,
                       (unsigned long long)pos, (unsigned long long)want, a, b, c, e);
                return 1;
            }
            ++looked;
        }
    }
    // Equal shares: share_of_tile inverts share_start, no share is empty when there are at least as
    // many tiles as shares.
    for (int rep = 0; rep < 2000; ++rep) {
        const uint32_t groups = 1 + (uint32_t)(next() % 1024);
        const uint64_t total = groups + next() % (rep % 2 ? 5000 : 3000000);
        for (int k = 0; k < 200; ++k) {
            const uint64_t tile = k < 2 ? (k ? total - 1 : 0) : next() % total;
            const uint32_t w = tq::share_of_tile(tile, total, groups);
            if (w >= groups || tq::share_start(w, total, groups) > tile || tq::share_start((uint64_t)w + 1, total, groups) <= tile) {
                printf("shares: total %llu groups %u tile %llu -> %u\n", (unsigned long long)total, groups,
                       (unsigned long long)tile, w);
                return 1;
            }
        }
        for (uint32_t w = 0; w < groups; w += 1 + groups / 50)
            if (tq::share_start((uint64_t)w + 1, total, groups) <= tq::share_start(w, total, groups)) { printf("empty share\n"); return 1; }
    }
    printf("ok %llu codes %llu look-ups\n", checked, looked);
    return 0;
}
