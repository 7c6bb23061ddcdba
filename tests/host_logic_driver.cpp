// CPU test driver: C entry points over the launcher's host-side planning helpers
// (paper_2502_20566_amd/csrc/sr_host.h), compiled with g++ by tests/test_host_logic.py.
#include "../paper_2502_20566_amd/csrc/sr_host.h"

extern "C" {

// Writes up to `cap` pieces as triples (local, numel, elem_offset); returns the number of pieces
// the walk produced (also beyond cap), or -1 - k when the callback's failure at piece k stopped it.
long long plan_pieces(unsigned long long numel, unsigned long long elem_offset, unsigned long long blocks_per_piece,
                      unsigned long long* out, long long cap, long long fail_at)
{
    long long n = 0;
    const int rc = sr_host::split_tensor(numel, elem_offset, blocks_per_piece,
                                         [&](uint64_t local, uint64_t piece, uint64_t goff) -> int {
        if (n == fail_at) return 7;
        if (n < cap) { out[3 * n] = local; out[3 * n + 1] = piece; out[3 * n + 2] = goff; }
        ++n;
        return 0;
    });
    return rc == 0 ? n : -1 - n;
}

int range_wraps(unsigned long long elem_offset, unsigned long long numel) { return sr_host::range_wraps(elem_offset, numel) ? 1 : 0; }

unsigned long long blocks_spanned(unsigned long long numel, unsigned long long elem_offset) { return sr_host::blocks_spanned(numel, elem_offset); }

long long chunks_of(unsigned long long numel, unsigned long long chunk_elems)
{
    uint64_t out = 0;
    return sr_host::chunks_of(numel, chunk_elems, &out) ? (long long)out : -1;
}

unsigned occupancy_lds(unsigned waves) { return sr_host::occupancy_lds(waves); }

}
