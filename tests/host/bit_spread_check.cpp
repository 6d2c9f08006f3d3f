// CPU check of the bit gather / spread helpers behind the encoder's level-invariant-dimension path:
// against bit-by-bit definitions, over structured and random masks, and a round trip through whole rows.
#include <stdio.h>
#include <stdlib.h>

#include <vector>

#include "bit_spread.h"

static uint64_t rng_state = 0x243F6A8885A308D3ull;
static uint32_t rnd() {
    rng_state ^= rng_state << 13;
    rng_state ^= rng_state >> 7;
    rng_state ^= rng_state << 17;
    return (uint32_t)(rng_state >> 16);
}

static uint32_t deposit_naive(uint32_t x, uint32_t keep) {   // bit j of x -> j-th set bit of keep
    uint32_t out = 0;
    int j = 0;
    for (int p = 0; p < 32; ++p)
        if ((keep >> p) & 1u) out |= ((x >> j++) & 1u) << p;
    return out;
}
static uint32_t extract_naive(uint32_t w, uint32_t keep) {   // set bits of keep, packed low
    uint32_t out = 0;
    int j = 0;
    for (int p = 0; p < 32; ++p)
        if ((keep >> p) & 1u) out |= ((w >> p) & 1u) << j++;
    return out;
}

int main() {
    long checked = 0;
    std::vector<uint32_t> masks = {0u, 1u, 0x80000000u, 0xffffffffu, 0x55555555u, 0xaaaaaaaau, 0xffff0000u,
                                   0x0000ffffu, 0xf0f0f0f0u, 0x80000001u, 0x7fffffffu, 0xfffffffeu};
    for (int i = 0; i < 32; ++i) masks.push_back(1u << i);
    for (int i = 0; i < 200000; ++i) masks.push_back((rnd() & (i % 3 ? rnd() : 0xffffffffu)) | (i % 5 ? 0u : rnd()));
    for (uint32_t keep : masks) {
        uint32_t stage[5];
        hdc::spread_stages(keep, stage);
        for (int t = 0; t < 6; ++t) {
            const uint32_t x = t == 0 ? 0xffffffffu : t == 1 ? 0u : rnd();
            if (hdc::spread_bits(x, keep, stage) != deposit_naive(x, keep)) {
                printf("spread mismatch keep=%08x x=%08x\n", keep, x);
                return 1;
            }
            if (hdc::gather_bits(x, keep) != extract_naive(x, keep)) {
                printf("gather mismatch keep=%08x x=%08x\n", keep, x);
                return 1;
            }
            // a spread after a gather restores the kept bits
            if (hdc::spread_bits(hdc::gather_bits(x, keep), keep, stage) != (x & keep)) {
                printf("round trip mismatch keep=%08x x=%08x\n", keep, x);
                return 1;
            }
            ++checked;
        }
    }
    // whole rows: compact_row concatenates the gathered bits of the words, lowest word first
    for (int trial = 0; trial < 2000; ++trial) {
        const int W = 1 + (int)(rnd() % 40);
        std::vector<uint32_t> row(W), keep(W);
        long bits = 0;
        for (int w = 0; w < W; ++w) {
            row[w] = rnd();
            keep[w] = trial % 4 == 0 ? 0xffffffffu : trial % 4 == 1 ? (rnd() & rnd() & rnd()) : rnd();
            if (trial % 7 == 0 && w % 2) keep[w] = 0;
            bits += __builtin_popcount(keep[w]);
        }
        const int Wc = (int)((bits + 31) / 32);
        std::vector<uint32_t> got(Wc + 1, 0u), want(Wc + 1, 0u);
        hdc::compact_row(row.data(), keep.data(), W, got.data());
        long at = 0;
        for (int w = 0; w < W; ++w)
            for (int p = 0; p < 32; ++p)
                if ((keep[w] >> p) & 1u) {
                    want[at >> 5] |= ((row[w] >> p) & 1u) << (at & 31);
                    ++at;
                }
        if (got != want) {
            printf("compact_row mismatch trial=%d W=%d\n", trial, W);
            return 1;
        }
        ++checked;
    }
    printf("OK %ld\n", checked);
    return 0;
}
