// Host-side planning of the launcher, free of HIP types so that a CPU build can compile and test it
// alone: index-range checks, the cut of a tensor slice into launch-sized pieces at counter-block
// boundaries, and the LDS reservation that caps the waves resident per CU.
#pragma once
#include <stdint.h>

namespace sr_host {

// True when the counter indices elem_offset .. elem_offset + numel (rounded up to a block) leave 64 bits.
inline bool range_wraps(uint64_t elem_offset, uint64_t numel)
{
    return numel > UINT64_MAX - 8 || elem_offset > UINT64_MAX - 8 - numel;
}

// Counter blocks (8 elements, aligned to multiples of 8 of the counter index) that the slice touches.
inline uint64_t blocks_spanned(uint64_t numel, uint64_t elem_offset)
{
    return ((elem_offset + numel - 1) >> 3) - (elem_offset >> 3) + 1;
}

// Chunks of chunk_elems elements that numel elements need; false when the rounding would wrap.
inline bool chunks_of(uint64_t numel, uint64_t chunk_elems, uint64_t* out)
{
    if (numel > UINT64_MAX - (chunk_elems - 1)) return false;
    *out = (numel + chunk_elems - 1) / chunk_elems;
    return true;
}

// Calls f(local, numel, elem_offset) for consecutive pieces of a tensor slice of `numel` >= 1
// elements whose element 0 has counter index `elem_offset`; every piece spans at most
// blocks_per_piece counter blocks and all but the first start on a block boundary.  local = index
// of the piece's first element in the slice.  f returns a status whose zero value means success;
// the first other value stops the walk and is returned.
template <class F>
auto split_tensor(uint64_t numel, uint64_t elem_offset, uint64_t blocks_per_piece, F f) -> decltype(f(0, 0, 0))
{
    using R = decltype(f(0, 0, 0));
    const uint64_t G0 = elem_offset, gblk0 = G0 >> 3;
    const uint64_t nblk = blocks_spanned(numel, elem_offset);
    for (uint64_t b = 0; b < nblk; b += blocks_per_piece) {
        const uint64_t bend = nblk - b < blocks_per_piece ? nblk : b + blocks_per_piece;
        const uint64_t gfirst = b == 0 ? G0 : (gblk0 + b) << 3;
        const uint64_t gend = bend == nblk ? G0 + numel : (gblk0 + bend) << 3;
        const R e = f(gfirst - G0, gend - gfirst, gfirst);
        if (e != R{}) return e;
    }
    return R{};
}

// Bytes of LDS a single-wave workgroup reserves so that about `waves` of them reside on a CU
// (0: no reservation, for waves = 0 or >= 32, the hardware's own limit).  The CU's 160 KiB are
// granted in units of 1280 bytes (128 units per CU): a workgroup gets floor(128 / waves) units,
// the largest reservation that still lets `waves` workgroups fit.  Measured on MI355X with
// workgroups that only sleep: 5 / 6 / 7 / 8 / 9 / 10 / 11 / 12 / 16 units per workgroup let
// 23-24 / 20 / 17-18 / 16 / 14 / 12 / 11 / 10 / 8 reside (the count steps exactly at multiples
// of 1280 bytes), 4 units or fewer all 32.  A launch may ask for at most 64 KiB, so fewer than 3
// waves cannot be forced.
constexpr uint32_t kLdsUnitBytes = 1280u;
constexpr uint32_t kLdsUnitsPerCu = 160u * 1024u / kLdsUnitBytes;
inline uint32_t occupancy_lds(uint32_t waves)
{
    if (waves == 0 || waves >= 32) return 0;
    return (kLdsUnitsPerCu / (waves < 3 ? 3 : waves)) * kLdsUnitBytes;
}

}  // namespace sr_host
