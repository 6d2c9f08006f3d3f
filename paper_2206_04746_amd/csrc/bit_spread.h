// Bit gathering and spreading used to leave level-invariant dimensions out of the encoder: plain
// host functions (no GPU types), also compiled on their own by the CPU tests.
#pragma once

#include <stdint.h>

namespace hdc {

// The set bits of `keep`, lowest first, picked out of `word` and packed to the low end.
inline uint32_t gather_bits(uint32_t word, uint32_t keep) {
    uint32_t out = 0;
    for (int k = 0; keep; keep &= keep - 1, ++k) out |= ((word >> __builtin_ctz(keep)) & 1u) << k;
    return out;
}

// Appends the kept bits of a W-word row to a densely packed row of Wc words (zeroed by the caller).
inline void compact_row(const uint32_t *row, const uint32_t *keep, int W, uint32_t *dst) {
    uint64_t acc = 0;
    int have = 0, at = 0;
    for (int w = 0; w < W; ++w) {
        const int cnt = __builtin_popcount(keep[w]);
        if (!cnt) continue;
        acc |= (uint64_t)gather_bits(row[w], keep[w]) << have;
        have += cnt;
        if (have >= 32) {
            dst[at++] = (uint32_t)acc;
            acc >>= 32;
            have -= 32;
        }
    }
    if (have) dst[at] = (uint32_t)acc;
}

// The inverse of gather_bits in five stages, as expand_kernel applies them: bit j of the packed
// word belongs at the j-th set bit of `keep`, a distance z to the left; stage i (4 down to 0)
// moves the bits whose z has bit i set by 2^i, and stage[i] marks where they land (the place a
// bit has when only the lower i bits of its distance are still to go).
inline void spread_stages(uint32_t keep, uint32_t stage[5]) {
    for (int i = 0; i < 5; ++i) stage[i] = 0;
    int j = 0;
    for (uint32_t m = keep; m; m &= m - 1, ++j) {
        const int pos = __builtin_ctz(m), z = pos - j;
        for (int i = 0; i < 5; ++i)
            if ((z >> i) & 1) stage[i] |= 1u << (pos - (z & ((1 << i) - 1)));
    }
}

inline uint32_t spread_bits(uint32_t x, uint32_t keep, const uint32_t stage[5]) {
    for (int i = 4; i >= 0; --i) x = (x & ~stage[i]) | ((x << (1 << i)) & stage[i]);
    return x & keep;
}

}  // namespace hdc
