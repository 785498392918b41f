// Host-side check of pq_layout.h against tiles written by the numpy layout reference: reads tiles from stdin
// (kind, number of tiles, then per tile 2944 code bytes and 512 radii), prints for every slot and block the fields
// that pql_read_block finds.  Compiled with g++ by tests/test_layout_cpu.py; the header has no HIP dependency.
#include <cstdio>
#include <cstdlib>
#include <vector>

#include "../paper_2502_02617_amd/csrc/pq_layout.h"

int main()
{
    int kind = 0, tiles = 0;
    if (std::fread(&kind, 4, 1, stdin) != 1 || std::fread(&tiles, 4, 1, stdin) != 1) return 1;
    std::vector<uint8_t> codes(PQL_CODE_BYTES);
    std::vector<uint16_t> radii(PQL_RADII);
    for (int t = 0; t < tiles; ++t) {
        if (std::fread(codes.data(), 1, PQL_CODE_BYTES, stdin) != PQL_CODE_BYTES) return 1;
        if (std::fread(radii.data(), 2, PQL_RADII, stdin) != PQL_RADII) return 1;
        for (int tau = 0; tau < 64; ++tau)
            for (int b = 0; b < 8; ++b) {
                const PqBlockFields f = pql_read_block(kind, codes.data(), radii.data(), tau, b);
                std::printf("%u %u %u %u %u\n", f.l1, f.g6[0], f.g6[1], f.c4, (unsigned)f.radius);
            }
    }
    return 0;
}
