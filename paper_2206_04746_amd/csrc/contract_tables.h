// Host-side construction of the model tables of the two contraction encoders (encode_contract.hip,
// encode_wide.hip; arXiv 2206.04746, Sec. III Eq. 1): thresholds of the dimensions, tiles and
// columns, model-side operands, the table that names the column of every bit of a row, and the
// feature slots that carry the vote threshold.  Plain C++ without any GPU call, so that a host
// program can build the tables under the sanitizers and check them against the definition.
#pragma once

#include <stdint.h>

#include <algorithm>
#include <cstdlib>
#include <map>
#include <vector>

namespace hdc {

// The model as hdc_create receives it: item [F][W], level [L][W], tie [W] packed words (bit d & 31
// of word d >> 5), `votes` = F, or F + 1 when the tie vector casts the extra vote of an even F.
struct ModelView {
    int D, W, F, L, votes;
    const uint32_t *item, *level, *tie;
};

// by_tau[t] = the dimensions whose level bit differs from level 0's from level t on (t >= 1).
// False if some dimension flips back: such a model is not of the contraction's shape.
inline bool flip_thresholds(const ModelView &m, std::vector<std::vector<int>> *by_tau) {
    by_tau->assign((size_t)m.L, std::vector<int>());
    for (int d = 0; d < m.D; ++d) {
        const int w = d >> 5, b = d & 31;
        const uint32_t first = (m.level[w] >> b) & 1u;
        int tau = 0;
        for (int l = 1; l < m.L; ++l) {
            const uint32_t bit = (m.level[(size_t)l * m.W + w] >> b) & 1u;
            if (!tau && bit != first) tau = l;
            else if (tau && bit == first) return false;
        }
        if (tau) (*by_tau)[(size_t)tau].push_back(d);
    }
    return true;
}

// Dimensions that flip more than once along the levels, kept together where they flip at the
// same levels: with t_1 < t_2 < ... the levels at which the bit changes, the level bit is
// level0 ^ [q >= t_1] ^ [q >= t_2] ^ ..., and as [q >= t_2] implies [q >= t_1] the vote of a
// feature is B ^ ([q >= t_1] - [q >= t_2] + ...): the sums of the single-flip form, one per t_i,
// with alternating sign.
constexpr int kCtMaxChain = 8;   // most flips of a dimension that the contraction follows
struct FlipChain {
    std::vector<int> taus;   // ascending, two at least
    std::vector<int> dims;   // ascending
};

// by_tau as flip_thresholds leaves it for the dimensions that flip once; the others in chains,
// ordered by their levels.  False if some dimension flips more than kCtMaxChain times.
inline bool flip_chains(const ModelView &m, std::vector<std::vector<int>> *by_tau, std::vector<FlipChain> *chains) {
    by_tau->assign((size_t)m.L, std::vector<int>());
    chains->clear();
    std::map<std::vector<int>, std::vector<int>> sets;
    std::vector<int> taus;
    for (int d = 0; d < m.D; ++d) {
        const int w = d >> 5, b = d & 31;
        taus.clear();
        uint32_t before = (m.level[w] >> b) & 1u;
        for (int l = 1; l < m.L; ++l) {
            const uint32_t bit = (m.level[(size_t)l * m.W + w] >> b) & 1u;
            if (bit != before) taus.push_back(l);
            before = bit;
        }
        if ((int)taus.size() > kCtMaxChain) return false;
        if (taus.size() == 1) (*by_tau)[(size_t)taus[0]].push_back(d);
        else if (taus.size() > 1) sets[taus].push_back(d);
    }
    for (auto &kv : sets) chains->push_back(FlipChain{kv.first, kv.second});
    return true;
}

// Where feature f sits in its word of 32 features, on both sides of the contraction: the kernels
// turn 32 bin numbers (bytes, four to a word) into bit planes with three rounds of masked swaps
// among eight words, which leaves feature 4 m + i of a lane's 32 at bit 8 i + m.
inline int feature_bit(int f) { return 8 * (f & 3) + ((f & 31) >> 2); }

// ---- encode_contract.hip --------------------------------------------------------------------
// bits 0..2 of every nibble reversed, bit 3 in place
inline uint32_t reverse3_host(uint32_t x) {
    return (x & 0xaaaaaaaau) | ((x & 0x11111111u) << 2) | ((x >> 2) & 0x11111111u);
}

constexpr int kCtCols = 32;       // dimensions per tile
constexpr float kCtNever = -1.0e30f;
// Flags beside the threshold in tau_of, set only in the tables of a model with chains: a chain's
// 32 dimensions take one tile per threshold, one after the other, whose sums the kernel carries
// from tile to tile with a change of sign each time; the bit comes out of the last one, inverted
// where the chain has an even number of tiles.  A tile of dimensions that flip once is first and last.
constexpr int32_t kCtTauMask = 0xffff, kCtFirst = 1 << 16, kCtLast = 1 << 17, kCtInvert = 1 << 18;

// One table set: the row's words in 1 << v ranges, the tiles of a range together.
struct CtTables {
    std::vector<int32_t> tau_of;       // [tiles] the level at which the tile's dimensions flip (and the flags above)
    std::vector<int32_t> range_tile;   // [(1 << v) + 1] first tile of every range, then the end
    std::vector<uint32_t> src_of;      // [32][W]: (tile in its range) * 32 + column holding that bit, ~0 for a constant bit
    std::vector<float> kc;             // [tiles][32]: the bit is set iff 2 <U,B> - |U| <= this
    std::vector<uint32_t> bt;          // [tile][step][lane]: the column's bits of item ^ level 0 (every nibble reversed)
    int range_max = 0;                 // most tiles of one range
    bool chained = false;              // tau_of carries flags
};

inline void build_contract_tables(const ModelView &m, const std::vector<std::vector<int>> &by_tau,
                                  const std::vector<FlipChain> &chains, int steps, int v, CtTables *t_out) {
    CtTables &T = *t_out;
    const int W = m.W, F = m.F, L = m.L, S = 1 << v;
    const int thr = (m.votes + 1) / 2;
    const bool tie_votes = m.votes != F;
    T = CtTables();
    T.chained = !chains.empty();
    T.src_of.assign((size_t)32 * W, 0xffffffffu);
    std::vector<uint32_t> vec((size_t)2 * steps);
    for (int r = 0; r < S; ++r) {
        const int w_lo = (int)((int64_t)r * W >> v), w_hi = (int)((int64_t)(r + 1) * W >> v);
        const size_t t_first = T.tau_of.size();
        T.range_tile.push_back((int32_t)t_first);
        // one tile: columns dims[at ...] (32 at most) against threshold tau; the row's bits point at tile `owner`
        auto add_tile = [&](const std::vector<int> &dims, size_t at, int32_t tau_entry, size_t owner, bool negated_start) {
            const size_t t = T.tau_of.size();
            T.tau_of.push_back(tau_entry);
            T.kc.resize((t + 1) * 32, kCtNever);
            T.bt.resize((t + 1) * steps * 64, 0u);
            for (int j = 0; j < 32; ++j) {
                std::fill(vec.begin(), vec.end(), 0u);
                if (j < kCtCols && at + j < dims.size()) {
                    const int d = dims[at + j], w = d >> 5, b = d & 31;
                    const uint32_t l0 = (m.level[w] >> b) & 1u;
                    int ones = 0;
                    for (int f = 0; f < F; ++f) {
                        const uint32_t bit = ((m.item[(size_t)f * W + w] >> b) & 1u) ^ l0;
                        ones += (int)bit;
                        vec[(size_t)f >> 5] |= bit << feature_bit(f);
                    }
                    const int tie_vote = tie_votes ? (int)((m.tie[w] >> b) & 1u) : 0;
                    T.src_of[(size_t)b * W + w] = (uint32_t)((owner - t_first) * 32 + j);
                    // (the kernel starts a column at -kc / 2 - 1 / 4; a chain that wants the opposite start says -kc - 1)
                    const int kc = ones + tie_vote - thr;
                    T.kc[t * 32 + j] = (float)(negated_start ? -kc - 1 : kc);
                }
                for (int k = 0; k < steps; ++k)
                    for (int h = 0; h < 2; ++h)
                        T.bt[(t * steps + k) * 64 + h * 32 + j] = reverse3_host(vec[(size_t)2 * k + h]);
            }
        };
        std::vector<int> dims;
        for (int tau = 1; tau < L; ++tau) {
            dims.clear();
            for (int d : by_tau[(size_t)tau])
                if ((d >> 5) >= w_lo && (d >> 5) < w_hi) dims.push_back(d);
            for (size_t at = 0; at < dims.size(); at += kCtCols)
                add_tile(dims, at, T.chained ? tau | kCtFirst | kCtLast : tau, T.tau_of.size(), false);
        }
        for (const FlipChain &ch : chains) {
            dims.clear();
            for (int d : ch.dims)
                if ((d >> 5) >= w_lo && (d >> 5) < w_hi) dims.push_back(d);
            // The kernel negates the running value at every further tile, so the i-th of n tiles
            // enters with the sign (-1)^(n - i).  Thresholds in ascending order: the wanted sums
            // times (-1)^(n - 1), hence the inverted bits for even n.  In descending order the signs
            // are the wanted ones and only the start value needs the factor (-1)^(n - 1).  The
            // groups of 32 dimensions of a chain take the two orders in turn, so that a group's
            // first threshold is its predecessor's last and the kernel forms its masks once for both.
            const size_t n = ch.taus.size();
            bool descending = false;
            for (size_t at = 0; at < dims.size(); at += kCtCols, descending = !descending) {
                const size_t owner = T.tau_of.size() + n - 1;   // the chain's last tile holds the bits
                for (size_t i = 0; i < n; ++i) {
                    const int tau = ch.taus[descending ? n - 1 - i : i];
                    const int32_t last = kCtLast | (!descending && n % 2 == 0 ? kCtInvert : 0);
                    add_tile(dims, at, tau | (i == 0 ? kCtFirst : 0) | (i + 1 == n ? last : 0), owner,
                             descending && n % 2 == 0);
                }
            }
        }
        T.range_max = std::max(T.range_max, (int)(T.tau_of.size() - t_first));
    }
    T.range_tile.push_back((int32_t)T.tau_of.size());
}

// ---- encode_wide.hip ------------------------------------------------------------------------
// 4-bit float (1 sign, 2 exponent, 1 mantissa bit) of a value it can hold exactly
inline uint32_t fp4_of(float v) {
    const uint32_t s = v < 0.0f ? 8u : 0u;
    const float a = v < 0.0f ? -v : v;
    const float mags[8] = {0.0f, 0.5f, 1.0f, 1.5f, 2.0f, 3.0f, 4.0f, 6.0f};
    for (uint32_t i = 0; i < 8; ++i)
        if (mags[i] == a) return s | i;
    return 0u;   // never asked for
}
inline float fp4_value(uint32_t nib) {
    const float mags[8] = {0.0f, 0.5f, 1.0f, 1.5f, 2.0f, 3.0f, 4.0f, 6.0f};
    return (nib & 8u) ? -mags[nib & 7u] : mags[nib & 7u];
}

// the value the sample side has at feature f's place when U = 1: operand word (bit & 3) holds a
// nibble with that one bit set (bit 3 moved to bit 2)
inline float wd_sample_value(int f) {
    const float v[4] = {0.5f, 1.0f, 2.0f, 2.0f};
    return v[feature_bit(f) & 3];
}

// Model-side values of the feature slots past F that add up to a target (a multiple of 1/2) when
// every such slot has U = 1.  Which sums the slots can reach is worked out once per model, slot
// after slot (in halves; a slot's sample-side value times each 4-bit float that gives a multiple
// of 1/2); a dimension's values are then read off backwards from its target.
struct WdBias {
    int F = 0, slots = 0, bound = 0;
    std::vector<std::vector<uint8_t>> reach;   // [slot count][sum + bound]: reachable with the first slots
    static constexpr float kMags[8] = {0.0f, 0.5f, 1.0f, 1.5f, 2.0f, 3.0f, 4.0f, 6.0f};
    void prepare(int F_, int slots_end, int max_halves) {
        F = F_, slots = slots_end - F_, bound = max_halves;
        reach.assign((size_t)slots + 1, std::vector<uint8_t>((size_t)2 * bound + 1, 0));
        reach[0][(size_t)bound] = 1;
        for (int i = 0; i < slots; ++i) {
            const float a = wd_sample_value(F + i);
            for (int sum = -bound; sum <= bound; ++sum) {
                if (!reach[(size_t)i][(size_t)(sum + bound)]) continue;
                for (float m : kMags)
                    for (int sg = -1; sg <= 1; sg += 2) {
                        const float c2 = 2.0f * a * m * (float)sg;   // the slot's contribution in halves
                        if (c2 != (float)(int)c2) continue;
                        const int to = sum + (int)c2;
                        if (to >= -bound && to <= bound) reach[(size_t)i + 1][(size_t)(to + bound)] = 1;
                    }
            }
        }
    }
    // false if the slots cannot make the target
    bool solve(int target_halves, std::vector<float> &val) const {
        val.assign((size_t)slots, 0.0f);
        if (target_halves < -bound || target_halves > bound || !reach[(size_t)slots][(size_t)(target_halves + bound)]) return false;
        int sum = target_halves;
        for (int i = slots - 1; i >= 0; --i) {
            const float a = wd_sample_value(F + i);
            bool found = false;
            for (int mi = 0; mi < 8 && !found; ++mi)
                for (int sg = -1; sg <= 1 && !found; sg += 2) {
                    const float c2 = 2.0f * a * kMags[mi] * (float)sg;
                    if (c2 != (float)(int)c2) continue;
                    const int from = sum - (int)c2;
                    if (from >= -bound && from <= bound && reach[(size_t)i][(size_t)(from + bound)]) {
                        val[(size_t)i] = kMags[mi] * (float)sg;
                        sum = from;
                        found = true;
                    }
                }
            if (!found) return false;   // (never: reach says otherwise)
        }
        return sum == 0;
    }
};

constexpr int kWdTileCols = 16;   // dimensions of a tile: the N of the 16 x 16 x 128 matrix instruction

struct WdTables {
    int steps = 0;                  // 64-feature steps per tile (two to a matrix instruction); 0: the model does not fit
    int tiles = 0, cols = 0;        // tiles of 16 dimensions, columns = varying dimensions
    std::vector<int32_t> items;     // [n][4]: threshold, first tile, dimensions, first column
    std::vector<uint32_t> bx;       // [tile][step / 2][lane][4]: 4-bit floats +-1 / (sample-side value), bias in the slots past F
    std::vector<uint32_t> src;      // [32][W]: the column of every varying bit of a row (constant bits: left at 0 here)
    std::vector<uint8_t> is_var;    // [D]
};

// tiles_per_item tiles of one threshold at most per work item; steps even, at most max_steps.
// Operand layout: lane 16 b + j of (tile, matrix instruction s) holds column j of the tile
// against the 32 feature slots 128 s + 32 b ..., a slot's nibble where feature_bit puts the
// feature's bit in the sample side's plane word.
inline void build_wide_tables(const ModelView &m, const std::vector<std::vector<int>> &by_tau, int max_steps,
                              int tiles_per_item, WdTables *t_out) {
    WdTables &T = *t_out;
    T = WdTables();
    const int W = m.W, F = m.F, L = m.L, D = m.D;
    const int thr = (m.votes + 1) / 2;
    const bool tie_votes = m.votes != F;
    // K_d of every dimension and the most slots any of the varying ones needs
    std::vector<int> ones((size_t)D, 0);
    for (int f = 0; f < F; ++f)
        for (int d = 0; d < D; ++d)
            ones[(size_t)d] += (int)(((m.item[(size_t)f * W + (d >> 5)] ^ m.level[d >> 5]) >> (d & 31)) & 1u);
    auto target_of = [&](int d) {   // in halves: -(2 K_d + 1); the bit is set iff sum_f U (2B - 1) <= K_d
        const int tie_vote = tie_votes ? (int)((m.tie[d >> 5] >> (d & 31)) & 1u) : 0;
        return -(2 * (ones[(size_t)d] + tie_vote - thr) + 1);
    };
    int max_halves = 0;
    bool any = false;
    for (int tau = 1; tau < L; ++tau)
        for (int d : by_tau[(size_t)tau]) max_halves = std::max(max_halves, std::abs(target_of(d))), any = true;
    if (!any) return;
    int steps = 0;
    std::vector<float> val;
    WdBias bias;
    for (int ks = ((F + 63) / 64 + 1) / 2 * 2; ks <= max_steps && !steps; ks += 2) {   // two steps to a matrix instruction
        if (ks * 64 == F) continue;
        bias.prepare(F, ks * 64, max_halves);
        bool ok = true;
        for (int tau = 1; tau < L && ok; ++tau)
            for (int d : by_tau[(size_t)tau])
                if (!bias.solve(target_of(d), val)) {
                    ok = false;
                    break;
                }
        if (ok) steps = ks;
    }
    if (!steps) return;

    // work items: a threshold and up to tiles_per_item tiles of its dimensions; columns in item order
    T.src.assign((size_t)32 * W, 0u);
    T.is_var.assign((size_t)D, 0);
    const int per_item = kWdTileCols * tiles_per_item, mis = steps / 2;
    int tiles = 0, cols = 0;
    for (int tau = 1; tau < L; ++tau) {
        const std::vector<int> &dims = by_tau[(size_t)tau];
        for (size_t at = 0; at < dims.size(); at += (size_t)per_item) {
            const int nd = (int)std::min<size_t>(dims.size() - at, (size_t)per_item);
            const int nt = (nd + kWdTileCols - 1) / kWdTileCols;
            T.items.insert(T.items.end(), {tau, tiles, nd, cols});
            T.bx.resize((size_t)(tiles + nt) * mis * 64 * 4, 0u);
            for (int i = 0; i < nd; ++i) {
                const int d = dims[at + i], w = d >> 5, b = d & 31, t = tiles + i / kWdTileCols, j = i % kWdTileCols;
                const uint32_t l0 = (m.level[w] >> b) & 1u;
                T.src[(size_t)b * W + w] = (uint32_t)(cols + i);
                T.is_var[(size_t)d] = 1;
                if (!bias.solve(target_of(d), val)) return;   // (checked above; leaves steps at 0)
                for (int f = 0; f < steps * 64; ++f) {
                    uint32_t nib;
                    if (f < F) {
                        const uint32_t bit = ((m.item[(size_t)f * W + w] >> b) & 1u) ^ l0;
                        nib = fp4_of((bit ? 1.0f : -1.0f) / wd_sample_value(f));
                    } else {
                        nib = fp4_of(val[(size_t)(f - F)]);
                    }
                    const int s = f >> 7, blk = (f >> 5) & 3, at_bit = feature_bit(f);
                    T.bx[(((size_t)t * mis + s) * 64 + blk * kWdTileCols + j) * 4 + (at_bit & 3)] |= nib << (4 * (at_bit >> 2));
                }
            }
            tiles += nt;
            cols += nd;
        }
    }
    T.steps = steps, T.tiles = tiles, T.cols = cols;
}

// The table the placement reads: per pair of bits of every word of a row the two columns that
// hold them, 16 bits each, [16][W].  Constant bits of the model (const_row: the row every sample
// gets at the level-invariant dimensions; pad bits are zero) point at column `cols`, an all-zero
// word, or `cols + 1`, an all-one word.  False if a column number does not fit 16 bits.
inline bool wide_place_table(const WdTables &T, const uint32_t *const_row, int D, int W, std::vector<uint32_t> *src2) {
    if (T.cols + 1 > 65535) return false;
    std::vector<uint32_t> src = T.src;
    for (int w = 0; w < W; ++w)
        for (int b = 0; b < 32; ++b) {
            const int d = 32 * w + b;
            if (d < D && T.is_var[(size_t)d]) continue;
            src[(size_t)b * W + w] = (uint32_t)(T.cols + (int)((const_row[w] >> b) & 1u));
        }
    src2->assign((size_t)16 * W, 0u);
    for (int i = 0; i < 16; ++i)
        for (int w = 0; w < W; ++w)
            (*src2)[(size_t)i * W + w] = src[(size_t)(2 * i) * W + w] | (src[(size_t)(2 * i + 1) * W + w] << 16);
    return true;
}

}  // namespace hdc
