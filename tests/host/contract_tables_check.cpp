// CPU check of the model tables of the two contraction encoders (csrc/contract_tables.h), meant to
// be built with -fsanitize=address,undefined: for a handful of model shapes it builds the tables as
// hdc_create does and then encodes random samples FROM THE TABLES ALONE, the way the kernels use
// them (thresholds, columns, operands, the placement table, the feature slots that carry the vote
// threshold), and compares every bit with the definition of Sec. III Eq. (1) written out bit by
// bit: hv[d] = majority over f of item[f][d] ^ level[q_f][d], the tie vector casting the extra
// vote of an even F.
#include <stdio.h>
#include <stdlib.h>

#include <vector>

#include "contract_tables.h"

static uint64_t rng_state = 0x9E3779B97F4A7C15ull;
static uint32_t rnd() {
    rng_state ^= rng_state << 13;
    rng_state ^= rng_state >> 7;
    rng_state ^= rng_state << 17;
    return (uint32_t)(rng_state >> 16);
}

struct Model {
    int D, W, F, L, votes;
    std::vector<uint32_t> item, level, tie;
    hdc::ModelView view() const { return {D, W, F, L, votes, item.data(), level.data(), tie.data()}; }
};

// flips_per_level fresh positions flip at every level (never the same twice), pad bits zero.
// twice: dimension 3 flips at level 2 and back at level 3 (needs L >= 4).
static Model make_model(int D, int F, int L, int flips_per_level, bool twice) {
    Model m;
    m.D = D, m.W = (D + 31) / 32, m.F = F, m.L = L, m.votes = F % 2 ? F : F + 1;
    const uint32_t last = D % 32 ? (1u << (D % 32)) - 1u : 0xffffffffu;
    auto row = [&](std::vector<uint32_t> &t, size_t r) {
        for (int w = 0; w < m.W; ++w) t[r * m.W + w] = rnd() ^ (rnd() << 16);
        t[r * m.W + m.W - 1] &= last;
    };
    m.item.assign((size_t)F * m.W, 0u);
    m.level.assign((size_t)L * m.W, 0u);
    m.tie.assign((size_t)m.W, 0u);
    for (int f = 0; f < F; ++f) row(m.item, (size_t)f);
    row(m.level, 0);
    row(m.tie, 0);
    std::vector<int> order((size_t)D);
    for (int d = 0; d < D; ++d) order[(size_t)d] = d;
    for (int d = D - 1; d > 0; --d) std::swap(order[(size_t)d], order[rnd() % (uint32_t)(d + 1)]);
    int next = 0;
    for (int l = 1; l < L; ++l) {
        for (int w = 0; w < m.W; ++w) m.level[(size_t)l * m.W + w] = m.level[(size_t)(l - 1) * m.W + w];
        for (int i = 0; i < flips_per_level && next < D; ++i, ++next) {
            const int d = order[(size_t)next];
            m.level[(size_t)l * m.W + (d >> 5)] ^= 1u << (d & 31);
        }
    }
    if (twice)
        for (int l = 0; l < L; ++l) {   // level 2 alone differs from level 0 at dimension 3, whatever the flips above did there
            const uint32_t want = (m.level[0] & 8u) ^ (l == 2 ? 8u : 0u);
            m.level[(size_t)l * m.W] = (m.level[(size_t)l * m.W] & ~8u) | want;
        }
    return m;
}

// On top of make_model: `sets` sets of 2 to `most` levels each, and some 40 dimensions per set
// (more than a tile's 32) that flip at exactly those levels, whatever the flips above did there.
static Model make_chain_model(int D, int F, int L, int flips_per_level, int sets, int most) {
    Model m = make_model(D, F, L, flips_per_level, false);
    int d = 0;
    for (int s = 0; s < sets; ++s) {
        std::vector<int> at((size_t)L, 0);
        const int n = 2 + (int)(rnd() % (uint32_t)(most - 1));
        for (int i = 0; i < n;) {
            const int l = 1 + (int)(rnd() % (uint32_t)(L - 1));
            if (!at[(size_t)l]) at[(size_t)l] = 1, ++i;
        }
        for (int i = 0; i < 40 && d < D; ++i, d += 1 + (int)(rnd() % 3u)) {
            uint32_t bit = (m.level[(size_t)(d >> 5)] >> (d & 31)) & 1u;
            for (int l = 1; l < L; ++l) {
                bit ^= (uint32_t)at[(size_t)l];
                uint32_t &word = m.level[(size_t)l * m.W + (d >> 5)];
                word = (word & ~(1u << (d & 31))) | (bit << (d & 31));
            }
        }
    }
    return m;
}

static int bit_of(const std::vector<uint32_t> &t, size_t row, int W, int d) { return (int)((t[row * W + (d >> 5)] >> (d & 31)) & 1u); }

// Eq. (1) bit by bit
static void encode_definition(const Model &m, const std::vector<int> &q, std::vector<uint32_t> *hv) {
    hv->assign((size_t)m.W, 0u);
    for (int d = 0; d < m.D; ++d) {
        int count = 0;
        for (int f = 0; f < m.F; ++f) count += bit_of(m.item, (size_t)f, m.W, d) ^ bit_of(m.level, (size_t)q[(size_t)f], m.W, d);
        if (m.votes != m.F) count += bit_of(m.tie, 0, m.W, d);
        if (2 * count > m.votes) (*hv)[(size_t)d >> 5] |= 1u << (d & 31);
    }
}

// the row every sample gets at the level-invariant dimensions (hdc_create takes it from one encoded sample)
static void constant_row(const Model &m, const std::vector<std::vector<int>> &by_tau,
                         const std::vector<hdc::FlipChain> &chains, std::vector<uint32_t> *row) {
    std::vector<int> q((size_t)m.F, 0);
    encode_definition(m, q, row);
    for (size_t t = 1; t < by_tau.size(); ++t)
        for (int d : by_tau[t]) (*row)[(size_t)d >> 5] &= ~(1u << (d & 31));
    for (const hdc::FlipChain &ch : chains)
        for (int d : ch.dims) (*row)[(size_t)d >> 5] &= ~(1u << (d & 31));
}

#define FAIL(...)            \
    do {                     \
        printf(__VA_ARGS__); \
        printf("\n");        \
        return false;        \
    } while (0)

// encode_contract.hip's use of its tables: bit = [2 <U, B> - |U| <= kc], placed through src_of;
// with chains, the running value R = <U, B> - |U| / 2 - kc / 2 - 1 / 4 of a chain's first tile,
// then <U, B> - |U| / 2 - R at every further one, the bit its sign at the last (inverted where flagged)
static bool check_contract(const Model &m, const std::vector<std::vector<int>> &by_tau,
                           const std::vector<hdc::FlipChain> &chains, const std::vector<uint32_t> &crow, int v, int samples) {
    const int steps = ((m.F + 63) / 64 + 1) / 2 * 2;
    hdc::CtTables T;
    hdc::build_contract_tables(m.view(), by_tau, chains, steps, v, &T);
    if (T.chained != !chains.empty()) FAIL("chained flag");
    const int S = 1 << v, tiles = (int)T.tau_of.size();
    if ((int)T.range_tile.size() != S + 1 || T.range_tile[0] != 0 || T.range_tile[(size_t)S] != tiles) FAIL("range table");
    if (T.kc.size() != (size_t)tiles * 32 || T.bt.size() != (size_t)tiles * steps * 64) FAIL("table sizes");
    for (int s = 0; s < samples; ++s) {
        std::vector<int> q((size_t)m.F);
        for (int f = 0; f < m.F; ++f) q[(size_t)f] = s == 0 ? 0 : s == 1 ? m.L - 1 : (int)(rnd() % (uint32_t)m.L);
        std::vector<uint32_t> want;
        encode_definition(m, q, &want);
        // every tile's 32 columns
        std::vector<uint8_t> colbit((size_t)tiles * 32, 0);
        std::vector<float> run(32, 0.0f);
        bool open = false;   // inside a chain
        for (int t = 0; t < tiles; ++t) {
            const int entry = T.tau_of[(size_t)t];
            const int tau = T.chained ? entry & hdc::kCtTauMask : entry;
            const bool first = !T.chained || (entry & hdc::kCtFirst), last = !T.chained || (entry & hdc::kCtLast);
            const bool invert = T.chained && (entry & hdc::kCtInvert);
            if (first == open) FAIL("tile %d: chain flags out of order", t);
            for (int r = 0; r <= S; ++r)
                if (T.range_tile[(size_t)r] == t && open) FAIL("tile %d: a chain runs across two ranges", t);
            open = !last;
            if (tau < 1 || tau >= m.L) FAIL("threshold %d of tile %d", tau, t);
            int nu = 0;
            for (int f = 0; f < m.F; ++f) nu += q[(size_t)f] >= tau;
            for (int j = 0; j < 32; ++j) {
                int dot = 0;
                for (int f = 0; f < m.F; ++f) {
                    if (q[(size_t)f] < tau) continue;
                    const int k = f >> 6, h = (f >> 5) & 1, p = hdc::feature_bit(f);
                    const uint32_t word = hdc::reverse3_host(T.bt[((size_t)t * steps + k) * 64 + h * 32 + j]);   // (its own inverse)
                    dot += (int)((word >> p) & 1u);
                }
                const float a = (float)dot - 0.5f * (float)nu;
                run[(size_t)j] = first ? a - 0.5f * T.kc[(size_t)t * 32 + j] - 0.25f : a - run[(size_t)j];
                if (last) colbit[(size_t)t * 32 + j] = (run[(size_t)j] < 0.0f) != invert;
            }
        }
        if (open) FAIL("the last chain is not closed");
        for (int r = 0; r < S; ++r) {
            const int w_lo = (int)((int64_t)r * m.W >> v), w_hi = (int)((int64_t)(r + 1) * m.W >> v);
            const int t0 = T.range_tile[(size_t)r], t1 = T.range_tile[(size_t)r + 1];
            if (t1 - t0 > T.range_max) FAIL("range_max");
            for (int w = w_lo; w < w_hi; ++w) {
                uint32_t got = crow[(size_t)w];
                for (int b = 0; b < 32; ++b) {
                    const uint32_t at = T.src_of[(size_t)b * m.W + w];
                    if (at == 0xffffffffu) continue;
                    if (at >= (uint32_t)(t1 - t0) * 32) FAIL("column %u of word %d bit %d outside its range's tiles", at, w, b);
                    got |= (uint32_t)colbit[(size_t)t0 * 32 + at] << b;
                }
                if (got != want[(size_t)w]) FAIL("contract: D=%d F=%d L=%d split %d sample %d word %d: %08x, definition %08x", m.D, m.F, m.L, v, s, w, got, want[(size_t)w]);
            }
        }
    }
    return true;
}

// encode_wide.hip's use of its tables: bit = [sum over all slots of U * sample value * model value < 0]
static bool check_wide(const Model &m, const std::vector<std::vector<int>> &by_tau, const std::vector<uint32_t> &crow,
                       int max_steps, int tiles_per_item, int samples, bool expect_fit) {
    hdc::WdTables T;
    hdc::build_wide_tables(m.view(), by_tau, max_steps, tiles_per_item, &T);
    if (!T.steps) {
        if (expect_fit) FAIL("wide: D=%d F=%d L=%d was expected to fit %d steps", m.D, m.F, m.L, max_steps);
        return true;
    }
    if (T.steps % 2 || T.steps * 64 <= m.F || T.steps > max_steps) FAIL("wide: steps %d", T.steps);
    std::vector<uint32_t> src2;
    if (!hdc::wide_place_table(T, crow.data(), m.D, m.W, &src2)) FAIL("wide: placement table");
    const int n_items = (int)(T.items.size() / 4);
    if (T.bx.size() != (size_t)T.tiles * (T.steps / 2) * 64 * 4) FAIL("wide: operand table size");
    for (int s = 0; s < samples; ++s) {
        std::vector<int> q((size_t)m.F);
        for (int f = 0; f < m.F; ++f) q[(size_t)f] = s == 0 ? 0 : s == 1 ? m.L - 1 : (int)(rnd() % (uint32_t)m.L);
        std::vector<uint32_t> want;
        encode_definition(m, q, &want);
        std::vector<uint8_t> col((size_t)T.cols + 2, 0);
        col[(size_t)T.cols + 1] = 1;
        int next_col = 0, next_tile = 0;
        for (int it = 0; it < n_items; ++it) {
            const int tau = T.items[(size_t)4 * it], tile0 = T.items[(size_t)4 * it + 1], nd = T.items[(size_t)4 * it + 2],
                      col0 = T.items[(size_t)4 * it + 3];
            if (tau < 1 || tau >= m.L || nd < 1 || nd > 16 * tiles_per_item || tile0 != next_tile || col0 != next_col) FAIL("wide: item %d", it);
            next_tile += (nd + 15) / 16, next_col += nd;
            for (int i = 0; i < nd; ++i) {
                const int t = tile0 + i / 16, j = i & 15;
                float acc = 0.0f;
                for (int f = 0; f < T.steps * 64; ++f) {
                    const bool u = f < m.F ? q[(size_t)f] >= tau : true;   // (slots past F: bin number all ones)
                    if (!u) continue;
                    // (the kernel's lane 16 b + j of matrix instruction mi: column j, the 32 slots of block b of its 128)
                    const int mi = f / 128, blk = (f % 128) / 32, p = hdc::feature_bit(f);
                    const uint32_t word = T.bx[(((size_t)t * (T.steps / 2) + mi) * 64 + 16 * blk + j) * 4 + (p & 3)];
                    acc += hdc::wd_sample_value(f) * hdc::fp4_value((word >> (4 * (p >> 2))) & 15u);
                }
                if (acc == 0.0f) FAIL("wide: a sum of exactly zero (the threshold slots must leave a half)");
                col[(size_t)col0 + i] = acc < 0.0f;
            }
        }
        if (next_col != T.cols || next_tile != T.tiles) FAIL("wide: totals");
        for (int w = 0; w < m.W; ++w) {
            uint32_t got = 0;
            for (int b = 0; b < 32; ++b) {
                const uint32_t pair = src2[(size_t)(b >> 1) * m.W + w];
                const uint32_t at = b & 1 ? pair >> 16 : pair & 0xffffu;
                if (at > (uint32_t)T.cols + 1) FAIL("wide: column %u of word %d bit %d", at, w, b);
                got |= (uint32_t)col[at] << b;
            }
            if (got != want[(size_t)w]) FAIL("wide: D=%d F=%d L=%d sample %d word %d: %08x, definition %08x", m.D, m.F, m.L, s, w, got, want[(size_t)w]);
        }
    }
    return true;
}

int main() {
    struct Shape {
        int D, F, L, flips;
        bool wide_fits;
    };
    const Shape shapes[] = {
        {1000, 100, 16, 33, true},     // D / (2 (L - 1)) flips per level: half of the dimensions vary; even F: the tie vector votes
        {2049, 31, 64, 16, true},      // odd F, a partial last word
        {513, 64, 4, 171, true},       // every dimension flips once; F fills a step exactly: the threshold takes two more
        {700, 342, 64, 5, true},       // the long stream's feature count, 42 spare slots
        {300, 383, 8, 20, true},       // one spare slot in six steps cannot carry the thresholds: eight steps
        {96, 4, 2, 40, true},          // the smallest model
        {640, 129, 256, 2, true},      // many thresholds of two dimensions
        {1500, 617, 64, 11, true},     // ten steps: five tiles of a threshold per work item
    };
    long checked = 0;
    for (const Shape &sh : shapes) {
        const Model m = make_model(sh.D, sh.F, sh.L, sh.flips, false);
        std::vector<std::vector<int>> by_tau, by_tau2;
        std::vector<hdc::FlipChain> chains;
        if (!hdc::flip_thresholds(m.view(), &by_tau) || !hdc::flip_chains(m.view(), &by_tau2, &chains)) {
            printf("D=%d F=%d L=%d: thresholds refused\n", sh.D, sh.F, sh.L);
            return 1;
        }
        if (!chains.empty() || by_tau != by_tau2) {
            printf("D=%d F=%d L=%d: the two readings of the thresholds differ\n", sh.D, sh.F, sh.L);
            return 1;
        }
        std::vector<uint32_t> crow;
        constant_row(m, by_tau, chains, &crow);
        for (int v = 0; v < 3 && (1 << v) <= m.W; ++v)
            if (!check_contract(m, by_tau, chains, crow, v, 6)) return 1;
        if (!check_wide(m, by_tau, crow, 10, 5, 6, sh.wide_fits)) return 1;
        if (!check_wide(m, by_tau, crow, 10, 3, 4, sh.wide_fits)) return 1;
        if (!check_wide(m, by_tau, crow, 6, 5, 2, false)) return 1;   // (the six-step limit: fits or is refused, never wrong)
        ++checked;
    }
    {   // a dimension that flips and flips back: refused by the reading that wants single flips, a chain for the other
        const Model m = make_model(400, 20, 8, 10, true);
        std::vector<std::vector<int>> by_tau;
        std::vector<hdc::FlipChain> chains;
        if (hdc::flip_thresholds(m.view(), &by_tau)) {
            printf("a dimension that flips twice was accepted\n");
            return 1;
        }
        if (!hdc::flip_chains(m.view(), &by_tau, &chains) || chains.size() != 1 || chains[0].dims != std::vector<int>{3} ||
            chains[0].taus != std::vector<int>{2, 3}) {
            printf("the dimension that flips twice is not the one chain\n");
            return 1;
        }
        std::vector<uint32_t> crow;
        constant_row(m, by_tau, chains, &crow);
        for (int v = 0; v < 3; ++v)
            if (!check_contract(m, by_tau, chains, crow, v, 8)) return 1;
        ++checked;
    }
    // dimensions that flip 2 to 8 times, in sets that share their levels, beside the single flips
    const struct {
        int D, F, L, flips, sets, most;
    } chained[] = {{1000, 100, 16, 20, 6, 4}, {2049, 31, 64, 10, 12, 8}, {700, 342, 64, 5, 5, 3}, {300, 64, 4, 50, 3, 3},
                   {96, 4, 3, 10, 1, 2}, {1500, 617, 9, 40, 20, 8}};
    for (const auto &sh : chained) {
        const Model m = make_chain_model(sh.D, sh.F, sh.L, sh.flips, sh.sets, sh.most);
        std::vector<std::vector<int>> by_tau;
        std::vector<hdc::FlipChain> chains;
        if (!hdc::flip_chains(m.view(), &by_tau, &chains) || chains.empty()) {
            printf("chained D=%d F=%d L=%d: no chains\n", sh.D, sh.F, sh.L);
            return 1;
        }
        for (const hdc::FlipChain &ch : chains)
            if (ch.taus.size() < 2 || (int)ch.taus.size() > hdc::kCtMaxChain || ch.dims.empty()) {
                printf("chained D=%d: a chain of %zu levels and %zu dimensions\n", sh.D, ch.taus.size(), ch.dims.size());
                return 1;
            }
        std::vector<uint32_t> crow;
        constant_row(m, by_tau, chains, &crow);
        for (int v = 0; v < 3 && (1 << v) <= m.W; ++v)
            if (!check_contract(m, by_tau, chains, crow, v, 8)) return 1;
        ++checked;
    }
    {   // more flips than the contraction follows: refused
        Model m = make_model(400, 20, 12, 10, false);
        for (int l = 0; l < m.L; ++l) m.level[(size_t)l * m.W] = (m.level[(size_t)l * m.W] & ~1u) | (uint32_t)(l & 1);
        std::vector<std::vector<int>> by_tau;
        std::vector<hdc::FlipChain> chains;
        if (hdc::flip_chains(m.view(), &by_tau, &chains)) {
            printf("a dimension that flips eleven times was accepted\n");
            return 1;
        }
    }
    printf("OK %ld models\n", checked);
    return 0;
}
