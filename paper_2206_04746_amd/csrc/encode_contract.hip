// ID-Level encoding (arXiv 2206.04746, Sec. III Eq. 1) as a contraction over the features, on the
// matrix cores.  Same bits as encode_kernel; taken for level tables in which every dimension that
// varies along the levels flips exactly once (the construction of Sec. III: neighbouring level
// vectors differ in a few more dimensions each), with at most 256 levels and 896 features, and
// for tables with dimensions that flip several times where these share their levels (below).
//
// For a dimension d that flips once let t_d be the first level whose bit differs from level 0's, and
// B[f][d] = item[f][d] ^ level[0][d].  The vote of feature f is B[f][d] ^ [q_f >= t_d], so the
// number of votes is
//     count[d] = sum_f B[f][d] + |U| - 2 * <U, B[.][d]>,     U_f = [q_f >= t_d],
// a constant of the model, the number of features at or above the threshold, and a dot product of
// two bit vectors over the features.  All dimensions with the same threshold share U: for a tile
// of 32 samples and 32 such dimensions the dot products are one v_mfma_f32_32x32x64_f8f6f4 per 64
// features, on 4-bit floats whose bits are the vectors'
// bits IN PLACE (a nibble with one bit set is 0.5, 1 or 2; the other operand is stored with the
// bits of every nibble reversed, so that every product is 1 or 0; see search_mfma.hip, which
// uses the same operands).  U itself comes from the quantised features kept as bit planes over the
// features: [q >= t] for 32 features at once is one 3-input bit operation per plane.
//
// A block takes 32 samples.  It quantises them first, a thread per four neighbouring features of a
// sample, and leaves the bin numbers in LDS a byte each; from these come the bit planes of all 32
// samples (32 bytes per lane and MFMA step, three rounds of masked swaps among eight words).
// Models of up to 4 MFMA steps run with eight waves, each of which builds all planes in its own
// registers; from 6 steps on a block has twelve waves (168 registers each), which share the work
// and read the planes from LDS at every threshold.  (Before: a ballot per plane over a wave of 64
// features of one sample, 55 instructions per 64 bin numbers against 6 + 9 now, and the block
// waited 16 k clocks instead of 8 k for its operands.)  The waves split the tiles of dimensions.
// The bits come out with
// a dimension per lane and a sample per register: a lane strings the 16 bits of its registers
// together (the sign of a fused multiply-add, shifted in by v_alignbit) and leaves them in LDS as
// the word "dimension (tile, column) of 16 samples".  When all tiles are done, thread w collects,
// for each of the 32 bits of word w of a row, that bit's word over the samples (a table names the
// tile and column of every varying bit; one LDS read per bit serves all 32 samples), transposes
// the 32 x 32 bits in registers, adds the model's constant bits and writes word w of the 32 rows.
// With few samples (fewer blocks of 32 than a quarter or half of the CUs) a row's words are split
// into 4 or 2 ranges and a block takes 32 samples and one range: its tiles are the range's
// dimensions (a table set per way of splitting), it places only the range's words, and it still
// quantises all features of its samples.  Rows of more than 512 words are always split (a thread
// places one word of its block's range), which takes the kernel to D = 65536.
// Dimensions that flip more than once (up to 8 times) are followed too, where enough of them flip
// at the same levels to fill tiles: with t_1 < t_2 < ... the levels at which such a dimension
// changes, its level bit is level0 ^ [q >= t_1] ^ [q >= t_2] ^ ..., the vote of a feature
// B ^ ([q >= t_1] - [q >= t_2] + ...), and the count the single-flip sums of its thresholds with
// alternating sign.  Its 32-dimension group takes one tile per threshold, one after the other in
// the same wave; the accumulators carry the running value from tile to tile, negated each time
// (-R + <U_i, B> - |U_i| / 2), and the bits come out of the last tile, inverted where the tiles
// are even in number and their thresholds ascend (the host lets every other group of a chain
// descend, with the start value to match, so that neighbouring tiles share a threshold and its
// masks).  (kChain; a model without such dimensions runs the kernel without it.)
// (Tried first: an LDS atomic OR per bit into images of the rows, six times the time of the MFMAs;
// then the wave's ballots as words over the dimensions and a gather per (bit, sample), LDS bank
// conflicts making it four times the time of the MFMAs.)
#include "hdc_internal.h"
#include "bundle.h"
#include "contract_tables.h"

#include <algorithm>
#include <vector>

namespace hdc {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v8i __attribute__((ext_vector_type(8)));
typedef float v16f __attribute__((ext_vector_type(16)));

constexpr int kCtWaves = 8;        // waves per block at least (the kernel runs with 8 or 12)
constexpr int kCtPlanes = 8;      // most bit planes of a bin number: L <= 256 (a model has ceil(log2 L) of them)
constexpr int kCtMaxSteps = 14;   // MFMAs per tile: 64 features each
constexpr int kCtSamples = 32;    // samples per block and job
// A model with chains is taken while its tiles, a chain's counted one and a quarter times (most
// bring a new threshold), are at most (24 + F / 34) / 10 times the tiles its varying dimensions
// would fill: measured at D = 10000 on 65536 samples against the vector kernel, whose time grows
// with F (617 features, 30 % of the dimensions in chains of 2 to 8, 3.3 times; 100 features,
// chains of 2 to 4, 2.7 times: see the measurements where prepare_contract is described).
constexpr int chain_work_tenths(int F) { return 24 + F / 34; }

template <typename T>
static int upload(T **dst, const std::vector<T> &src) {
    void *ptr = nullptr;
    hipError_t e = hipMalloc(&ptr, src.size() * sizeof(T) + 256);
    if (e == hipErrorOutOfMemory) {
        (void)hipGetLastError();
        return HDC_ENOMEM;
    }
    if (e != hipSuccess) return hip_fail(e, "hipMalloc");
    *dst = reinterpret_cast<T *>(ptr);
    e = hipMemcpy(ptr, src.data(), src.size() * sizeof(T), hipMemcpyHostToDevice);
    return e == hipSuccess ? HDC_OK : hip_fail(e, "hipMemcpy");
}

// ---- host: tables of the model -----------------------------------------------------------------
// Leaves c->ct_ready false when the model is not of the shape described above (or on any doubt);
// only a failed allocation or copy is an error.
int prepare_contract(hdc_ctx_impl *c, const uint32_t *item, const uint32_t *level, const uint32_t *tie) {
    const hdc_params &p = c->p;
    const int W = c->W, F = p.F, L = p.L;
    c->ct_ready = false;
    c->ct_min_split = -1;
    if (!c->expand_d || L < 2 || L > (1 << kCtPlanes) || F > 64 * kCtMaxSteps || F < 4 || W > 4 * kCtWaves * kWave) return HDC_OK;   // four features per load; a thread per word of a quarter of a row at least
    const int steps = ((F + 63) / 64 + 1) / 2 * 2;   // the kernel is built for even counts; a step past F meets zeros
    const ModelView model = {p.D, W, F, L, c->votes, item, level, tie};
    std::vector<std::vector<int>> by_tau;
    std::vector<FlipChain> chains;
    if (!flip_chains(model, &by_tau, &chains)) return HDC_OK;   // a dimension that flips more often than the kernel follows
    if (!chains.empty()) {
        // A chain's tiles are as many as its thresholds per 32 dimensions, full or not: where the
        // dimensions that flip more than once do not share their levels (a random table), the tiles
        // are many and nearly empty, and the vector kernel is the faster one.
        int64_t varying = 0, tiles4 = 0;   // tiles in quarters
        for (const std::vector<int> &dims : by_tau) varying += (int64_t)dims.size(), tiles4 += 4 * (((int64_t)dims.size() + 31) / 32);
        for (const FlipChain &ch : chains)
            varying += (int64_t)ch.dims.size(), tiles4 += 5 * (int64_t)ch.taus.size() * (((int64_t)ch.dims.size() + 31) / 32);
        if (tiles4 * 10 > 4 * chain_work_tenths(F) * ((varying + 31) / 32)) return HDC_OK;
    }
    for (int v = 0; v < 3; ++v) {   // the row's words in 1 << v ranges, a block per (32 samples, range)
        const int S = 1 << v;
        if (W < S) break;   // every range of words has a word
        if ((W + S - 1) / S > kCtWaves * kWave) continue;   // and a thread for each of its words
        CtTables tabs;
        build_contract_tables(model, by_tau, chains, steps, v, &tabs);
        const std::vector<int32_t> &tau_of = tabs.tau_of, &range_tile = tabs.range_tile;
        const std::vector<uint32_t> &src_of = tabs.src_of, &bt = tabs.bt;
        const std::vector<float> &kc = tabs.kc;
        const int range_max = tabs.range_max;
        if (tau_of.empty()) return HDC_OK;
        // a wave keeps its tiles' thresholds a lane each (with chains its share of the tiles ends a chain's length later at most)
        if (range_max > kCtWaves * (kWave - (chains.empty() ? 0 : kCtMaxChain))) continue;
        c->ct_tiles[v] = (int)tau_of.size();
        c->ct_range_max[v] = range_max;
        for (int r = 0; r <= 4; ++r) c->ct_range[v][r] = range_tile[(size_t)std::min(r, S)];
        int rc = upload(&c->ct_tau_d[v], tau_of);
        if (rc == HDC_OK) rc = upload(&c->ct_col_d[v], src_of);
        if (rc == HDC_OK) rc = upload(&c->ct_k_d[v], kc);
        if (rc == HDC_OK) rc = upload(&c->ct_bt_d[v], bt);
        if (rc != HDC_OK) return rc;
        if (c->ct_min_split < 0) c->ct_min_split = v;
        c->ct_max_split = v;
    }
    if (c->ct_min_split < 0) return HDC_OK;
    c->ct_steps = steps;
    c->ct_chained = !chains.empty();
    c->ct_ready = true;
    return HDC_OK;
}

// Both operands as 4-bit floats (format code 4), no block scales; 16 bytes of each are used.
__device__ __forceinline__ v16f mfma_fp4(v4i a, v4i b, v16f c) {
    const v8i a8 = {a[0], a[1], a[2], a[3], 0, 0, 0, 0}, b8 = {b[0], b[1], b[2], b[3], 0, 0, 0, 0};
    return __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(a8, b8, c, 4, 4, 0, 0, 0, 0);
}

struct CtRanges {
    int t[5];   // first tile of each of up to four ranges of words, and the end of the last
};

typedef uint32_t ct_u32x4_a4 __attribute__((ext_vector_type(4), aligned(4)));   // a global load of 16 bytes at any word
typedef uint32_t ct_u32x4 __attribute__((ext_vector_type(4)));

// Dynamic LDS: the job's bin numbers, a byte each, [sample][KS * 64 + 16] (the 16 spread the rows
// over the banks), then per (tile, column) the bits of the job's 32 samples [T * 32] (two 16-bit
// halves, one per lane half).
template <int KS, int NB, bool kU8, int NW, bool kChain>
__global__ __launch_bounds__(NW *kWave) void encode_contract_kernel(
    const void *__restrict__ feats, int64_t N, int F, int L, const float *__restrict__ lo,
    const float *__restrict__ scale, int W, int split, const CtRanges range_tile,
    const uint32_t *__restrict__ bt, const uint32_t *__restrict__ src_of, const float *__restrict__ kc,
    const int32_t *__restrict__ tau, const uint32_t *__restrict__ const_row, uint32_t *__restrict__ hv) {
    extern __shared__ __attribute__((aligned(16))) uint32_t pl_lds[];
    constexpr int kQuads = KS * 16;                                  // groups of four features per sample
    constexpr int kPerRound = NW * kWave / kQuads;             // samples the block quantises at a time
    constexpr int kRounds = (kCtSamples + kPerRound - 1) / kPerRound;
    constexpr int kRowBytes = KS * 64 + 16;
    // From 12 steps on the planes do not fit the registers next to the operands: the waves share
    // their construction and leave them in LDS, [step][planes 0..3 | 4..7][lane] of four words.
    constexpr bool kPlanesInLds = KS > 10 || NW > 8;
    ct_u32x4 *planes = reinterpret_cast<ct_u32x4 *>(pl_lds + kCtSamples * kRowBytes / 4);
    uint32_t *over = pl_lds + kCtSamples * kRowBytes / 4 + (kPlanesInLds ? KS * 2 * kWave * 4 : 0);
    uint16_t *over16 = reinterpret_cast<uint16_t *>(over);
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int lane = threadIdx.x & (kWave - 1);
    const int j = lane & 31, h = lane >> 5;
    // every lane's read address for the value of lane 4 * h of its own half (see u_of below)
    const int u_addr = (4 * h) * 4;
    // this thread's four features when the block quantises (the same in every round) and its sample of a round
    const int f0 = 4 * ((int)threadIdx.x % kQuads), s_in = (int)threadIdx.x / kQuads;
    const int fq = min(f0, F - 4);                 // what it loads: four features that exist (F >= 4: the host sees to that)
    const int q_shift = 8 * min(f0 - fq, 3);       // and where its own first feature's bin number is in them
    uint32_t keep = 0;   // the bytes of its word that are features at all
#pragma unroll
    for (int i = 0; i < 4; ++i)
        if (f0 + i < F) keep |= 0xffu << (8 * i);

    // A unit of work: 32 samples and one of the 1 << split ranges of a row's words.
    const int64_t units = ((N + kCtSamples - 1) / kCtSamples) << split;
    for (int64_t unit = blockIdx.x; unit < units; unit += gridDim.x) {   // block-uniform
        const int64_t job = unit >> split;
        const int range = (int)(unit & ((1 << split) - 1));
        // (the bounds come with the kernel's arguments: a table in memory would put a load in front of every job)
        const int t_first = range == 0 ? range_tile.t[0] : range == 1 ? range_tile.t[1] : range == 2 ? range_tile.t[2] : range_tile.t[3];
        const int t_end = range == 0 ? range_tile.t[1] : range == 1 ? range_tile.t[2] : range == 2 ? range_tile.t[3] : range_tile.t[4];
        const int w_first = (int)((int64_t)range * W >> split), w_end = (int)((int64_t)(range + 1) * W >> split);
        // the wave's tiles (at most 64: the host sees to that) and their thresholds, a tile per lane
        int t_lo = t_first + (int)((int64_t)wave * (t_end - t_first) / NW);
        int t_hi = t_first + (int)((int64_t)(wave + 1) * (t_end - t_first) / NW);
        if constexpr (kChain) {   // a chain's tiles stay in one wave: both ends move on to the next tile that starts one
            while (t_lo < t_end && !(tau[t_lo] & kCtFirst)) ++t_lo;
            while (t_hi < t_end && !(tau[t_hi] & kCtFirst)) ++t_hi;
        }
        // The job's bin numbers.  A thread takes four neighbouring features of a sample with one 16-byte
        // load, kPerRound samples to a round, and leaves the four bin numbers as one word in LDS.  No
        // branches around the loads (all of a thread's rounds are in flight together): the group that
        // straddles F, and those past it, load the row's last four features and shift the word.
        {
            const int64_t first = job * kCtSamples;
            uint32_t raw[kRounds][4];
            float lo_f[4], sc_f[4];
#pragma unroll
            for (int r = 0; r < kRounds; ++r) {   // (rows past N, and the threads with no sample in this round: some row that exists)
                const int64_t at = first + min(r * kPerRound + s_in, kCtSamples - 1);
                const int64_t n = at < N ? at : N - 1;
                if (kU8) {
                    const uint8_t *row = reinterpret_cast<const uint8_t *>(feats) + n * F + fq;
#pragma unroll
                    for (int i = 0; i < 4; ++i) raw[r][i] = row[i];
                } else {
                    const ct_u32x4_a4 v = *reinterpret_cast<const ct_u32x4_a4 *>(reinterpret_cast<const uint32_t *>(feats) + n * F + fq);
                    raw[r][0] = v[0], raw[r][1] = v[1], raw[r][2] = v[2], raw[r][3] = v[3];
                }
            }
            {   // the features' ranges after the features (index opaque: lifted out of the job loop, the block's
                // first feature loads would wait for these)
                int fqo = fq;
                asm volatile("" : "+v"(fqo));
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    lo_f[i] = kU8 ? 0.0f : lo[fqo + i];
                    sc_f[i] = kU8 ? 0.0f : scale[fqo + i];
                }
            }
            __builtin_amdgcn_sched_barrier(0);   // (or the first round is worked on before the others are asked for)
#pragma unroll
            for (int r = 0; r < kRounds; ++r) {
                const int sn = r * kPerRound + s_in;
                uint32_t word = 0;
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    uint32_t q;
                    if (kU8) {
                        q = (raw[r][i] * (uint32_t)L) >> 8;
                    } else {   // bin_f32 without its branches: NaN and negatives go to 0 through the maximum
                        const float t = __fmul_rn(__fsub_rn(__builtin_bit_cast(float, raw[r][i]), lo_f[i]), sc_f[i]);
                        q = (uint32_t)(int)fminf(fmaxf(t, 0.0f), (float)(L - 1));
                    }
                    word |= q << (8 * i);
                }
                if (s_in < kPerRound && sn < kCtSamples) pl_lds[(sn * kRowBytes + f0) >> 2] = (word >> q_shift) & keep;
            }
        }
        __syncthreads();
        // The bin numbers as bit planes over the features, made by every wave for itself and kept in
        // registers (up to 10 MFMA steps; beyond, see kPlanesInLds): lane (sample j,
        // half h) reads its 32 bytes of MFMA step k and moves bit b of byte i of word m to bit
        // 8 i + m of plane b (word index and bit index trade three of their bits, one per round).
        const int tau_mine = t_lo + lane < t_hi ? tau[t_lo + lane] : 0;   // (on its way while the planes are made)
        auto planes_of = [&](const int k, uint32_t (&x)[8]) {
            const ct_u32x4 *src = reinterpret_cast<const ct_u32x4 *>(
                reinterpret_cast<const uint8_t *>(pl_lds) + j * kRowBytes + k * 64 + h * 32);
            const ct_u32x4 v0 = src[0], v1 = src[1];
            x[0] = v0[0], x[1] = v0[1], x[2] = v0[2], x[3] = v0[3], x[4] = v1[0], x[5] = v1[1], x[6] = v1[2], x[7] = v1[3];
#pragma unroll
            for (int stage = 0; stage < 3; ++stage) {
                const int sh = 1 << stage;
                const uint32_t m = stage == 0 ? 0x55555555u : stage == 1 ? 0x33333333u : 0x0f0f0f0fu;
#pragma unroll
                for (int i = 0; i < 8; ++i)
                    if ((i & sh) == 0) {
                        const uint32_t a = x[i], b = x[i + sh];
                        x[i] = (a & m) | ((b << sh) & ~m);
                        x[i + sh] = ((a >> sh) & m) | (b & ~m);
                    }
            }
        };
        uint32_t pln[kPlanesInLds ? 1 : KS][NB];
        if constexpr (kPlanesInLds) {
#pragma unroll
            for (int k0 = 0; k0 < KS; k0 += NW) {
                const int k = k0 + wave;
                if (k < KS) {   // wave-uniform
                    uint32_t x[8];
                    planes_of(k, x);
                    planes[(k * 2 + 0) * kWave + lane] = ct_u32x4{x[0], x[1], x[2], x[3]};
                    if (NB > 4) planes[(k * 2 + 1) * kWave + lane] = ct_u32x4{x[4], x[5], x[6], x[7]};
                }
            }
            __syncthreads();
        } else {
#pragma unroll
            for (int k = 0; k < KS; ++k) {
                uint32_t x[8];
                planes_of(k, x);
#pragma unroll
                for (int b = 0; b < NB; ++b) pln[k][b] = x[b];
            }
        }

        int cur_tau = 0;
        v4i a[KS];
        float u_of[16];   // -|U| / 2 of the sample that accumulator register r belongs to
        uint32_t btw[KS];
        float k_mine = 0.0f;
        if (t_lo < t_hi) {
#pragma unroll
            for (int k = 0; k < KS; ++k) btw[k] = bt[((size_t)t_lo * KS + k) * 64 + lane];
            k_mine = kc[t_lo * 32 + j];
        }
        v16f acc;
        if constexpr (kChain) {
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[r] = 0.0f;
        }
        for (int t = t_lo; t < t_hi; ++t) {
            const int entry = __builtin_amdgcn_readlane(tau_mine, t - t_lo);
            const int tt = kChain ? entry & kCtTauMask : entry;
            if (tt != cur_tau) {   // wave-uniform: the samples' [q >= tt] over the features, their masks, their counts
                cur_tau = tt;
                uint32_t cnt = 0;
#pragma unroll
                for (int k = 0; k < KS; ++k) {
                    uint32_t ge = 0xffffffffu;
                    uint32_t qp[8];
                    if constexpr (kPlanesInLds) {
                        const ct_u32x4 p0 = planes[(k * 2 + 0) * kWave + lane];
                        const ct_u32x4 p1 = NB > 4 ? planes[(k * 2 + 1) * kWave + lane] : ct_u32x4{0u, 0u, 0u, 0u};
                        qp[0] = p0[0], qp[1] = p0[1], qp[2] = p0[2], qp[3] = p0[3], qp[4] = p1[0], qp[5] = p1[1], qp[6] = p1[2], qp[7] = p1[3];
                    } else {
#pragma unroll
                        for (int b = 0; b < NB; ++b) qp[b] = pln[k][b];
                    }
#pragma unroll
                    for (int b = 0; b < NB; ++b) {
                        const uint32_t q = qp[b];
                        const uint32_t tb = (tt >> b) & 1 ? 0xffffffffu : 0u;   // wave-uniform
                        ge = __builtin_amdgcn_bitop3_b32(q, ge, tb, 0xD4);      // tb ? q & ge : q | ge
                    }
                    cnt += __popc(ge);
                    a[k] = v4i{(int)(ge & 0x11111111u), (int)(ge & 0x22222222u), (int)(ge & 0x44444444u),
                               (int)((ge >> 1) & 0x44444444u)};
                }
                cnt += (uint32_t)__shfl_xor((int)cnt, 32, kWave);   // both halves of a sample's features
                // register r of a lane belongs to sample 8 * (r / 4) + 4 * h + r % 4 of the job
                const int neg = __builtin_bit_cast(int, -0.5f * (float)cnt);
#pragma unroll
                for (int r = 0; r < 16; ++r)
                    u_of[r] = __builtin_bit_cast(float, __builtin_amdgcn_ds_bpermute(u_addr + (8 * (r >> 2) + (r & 3)) * 4, neg));
            }
            // The bit of (sample, dimension) is [2 <U,B> - |U| <= K], i.e. the sign of <U,B> - K / 2 - |U| / 2 -
            // 0.25 (multiples of a half but for the quarter): the accumulators start at what follows <U,B>.
            // (a chain's further tiles: what follows <U,B> there, less the running value)
            if (!kChain || (entry & kCtFirst)) {
                const float start = -0.5f * k_mine - 0.25f;
#pragma unroll
                for (int r = 0; r < 16; ++r) acc[r] = start + u_of[r];
            } else {
#pragma unroll
                for (int r = 0; r < 16; ++r) acc[r] = u_of[r] - acc[r];
            }
#pragma unroll
            for (int k = 0; k < KS; ++k) {
                const uint32_t m = btw[k];
                const v4i b = {(int)(m & 0x44444444u), (int)(m & 0x22222222u), (int)(m & 0x11111111u),
                               (int)((m >> 3) & 0x11111111u)};
                acc = mfma_fp4(a[k], b, acc);
            }
            {   // the next tile's operands and constants (past the wave's last tile: the same again)
                const int tn = t + 1 < t_hi ? t + 1 : t;
#pragma unroll
                for (int k = 0; k < KS; ++k) btw[k] = bt[((size_t)tn * KS + k) * 64 + lane];
            }
            if (!kChain || (entry & kCtLast)) {   // wave-uniform
                // register 0's bit ends up highest
                uint32_t bits = 0;
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const float d = acc[r];   // (a copy: __builtin_bit_cast applied to the vector element itself reads element 0)
                    bits = __builtin_amdgcn_alignbit(bits, __builtin_bit_cast(uint32_t, d), 31);
                }
                if (kChain && (entry & kCtInvert)) bits = ~bits;
                over16[(size_t)((t - t_first) * 32 + j) * 2 + h] = (uint16_t)bits;
            }
            k_mine = kc[(t + 1 < t_hi ? t + 1 : t) * 32 + j];
        }
        // (this thread's entries of the bit table are asked for before the barrier, not after it)
        uint32_t x[32];
        uint32_t cbits;
        {
            int w = min(w_first + (int)threadIdx.x, w_end - 1);   // this thread's word of a row
            // (opaque to the compiler, or it lifts these 32 loads out of the job loop: a block with one
            // job would then wait for them before it starts, and hold 32 registers throughout)
            asm volatile("" : "+v"(w));
#pragma unroll
            for (int b = 0; b < 32; ++b) x[b] = src_of[(size_t)b * W + w];   // (~0: a constant of the model)
            cbits = const_row[w];
        }
        __builtin_amdgcn_sched_barrier(0);
        __syncthreads();

        // Word w of the job's rows.  Bit p of a word of `over` is the sample of register 15 - p of
        // lane half 0 (p < 16) or register 31 - p of half 1.
        if (w_first + (int)threadIdx.x < w_end) {
#pragma unroll
            for (int b = 0; b < 32; ++b) x[b] = x[b] != 0xffffffffu ? over[x[b]] : 0u;
            // x[b] bit p  ->  x[p] bit b
#pragma unroll
            for (int stage = 0; stage < 5; ++stage) {
                const int k = 16 >> stage;
                const uint32_t m = stage == 0 ? 0x0000ffffu : stage == 1 ? 0x00ff00ffu : stage == 2 ? 0x0f0f0f0fu
                                 : stage == 3 ? 0x33333333u : 0x55555555u;
#pragma unroll
                for (int i = 0; i < 32; ++i)
                    if ((i & k) == 0) {
                        const uint32_t tsw = ((x[i] >> k) ^ x[i + k]) & m;
                        x[i + k] ^= tsw;
                        x[i] ^= tsw << k;
                    }
            }
            const int64_t first = job * kCtSamples;
#pragma unroll
            for (int p = 0; p < 32; ++p) {
                const int r = p < 16 ? 15 - p : 31 - p;
                const int sn = 8 * (r >> 2) + (p < 16 ? 0 : 4) + (r & 3);
                if (first + sn < N) hv[(first + sn) * W + w_first + threadIdx.x] = x[p] | cbits;
            }
        }
        __syncthreads();
    }
}

constexpr int kCtSplitWork = 1024;         // MFMAs per 32 samples from which a row's words are split over blocks
// A block takes 32 samples and is a chain of some 60 k clocks whatever the call's size: below these
// counts the vector kernels are as fast (measured as whole calls, three launches against one:
// 512 samples of the 617-feature shape 36 us against 28, 128 samples 29 against 26).
constexpr int64_t kCtMinSamples = 1024;        // models whose words are not split over blocks
constexpr int64_t kCtMinSamplesSplit = 256;    // models whose words are

template <int KS, int NB, bool kU8, bool kChain>
static int launch_contract(hdc_ctx_impl *c, const void *x, int64_t n, uint32_t *out, hipStream_t s) {
    // With few samples, several blocks per 32 of them, each with a range of the row's words -- where
    // the tiles are most of a block's work (every block quantises its 32 samples in full, and ranges
    // make more, emptier tiles: with 300 MFMAs per 32 samples the split was 8 % slower, with 1900 25 % faster).
    const int64_t jobs = (n + kCtSamples - 1) / kCtSamples;
    int v = jobs * 4 <= c->num_cus ? 2 : jobs * 2 <= c->num_cus ? 1 : 0;
    if (c->ct_tiles[c->ct_min_split] * c->ct_steps < kCtSplitWork) v = 0;
    v = std::max(c->ct_min_split, std::min(v, c->ct_max_split));   // (wide rows are always split: a thread per word of a range)
    // Twelve waves where the tiles are most of the work (a third wave per SIMD fills more of the gaps
    // between matrix and vector instructions: 3 to 6 % on the 342- to 784-feature shapes), eight
    // for small models (100 features: 3 % slower with twelve).  The limits the host applies to the
    // tables are those of eight.
    constexpr int NW = KS >= 6 ? 12 : kCtWaves;
    constexpr bool kPlanesInLds = KS > 10 || NW > 8;
    auto kern = encode_contract_kernel<KS, NB, kU8, NW, kChain>;
    const size_t lds = (size_t)kCtSamples * (KS * 64 + 16) + (kPlanesInLds ? (size_t)KS * 2 * kWave * 16 : 0) +
                       (size_t)c->ct_range_max[v] * 32 * 4;
    if (lds > 64 * 1024)
        HDC_HIP(hipFuncSetAttribute(reinterpret_cast<const void *>(kern), hipFuncAttributeMaxDynamicSharedMemorySize,
                                    (int)lds));
    const int64_t blocks = std::min<int64_t>(jobs << v, (int64_t)c->num_cus);
    CtRanges rt;
    for (int r = 0; r <= 4; ++r) rt.t[r] = c->ct_range[v][r];
    hipLaunchKernelGGL(kern, dim3((unsigned)blocks), dim3(NW * kWave), lds, s, x, n, c->p.F, c->p.L, c->lo_d,
                       c->scale_d, c->W, v, rt, c->ct_bt_d[v], c->ct_col_d[v], c->ct_k_d[v],
                       c->ct_tau_d[v], c->expand_d + (size_t)7 * c->W, out);
    HDC_HIP(hipGetLastError());
    return HDC_OK;
}

// The kernel is built for an even number of steps and for 6 or 8 bit planes (L <= 64, L <= 256).
template <int NB, bool kU8, bool kChain>
static int launch_contract_steps(hdc_ctx_impl *c, const void *x, int64_t n, uint32_t *out, hipStream_t s) {
    switch (c->ct_steps) {
    case 2: return launch_contract<2, NB, kU8, kChain>(c, x, n, out, s);
    case 4: return launch_contract<4, NB, kU8, kChain>(c, x, n, out, s);
    case 6: return launch_contract<6, NB, kU8, kChain>(c, x, n, out, s);
    case 8: return launch_contract<8, NB, kU8, kChain>(c, x, n, out, s);
    case 10: return launch_contract<10, NB, kU8, kChain>(c, x, n, out, s);
    case 12: return launch_contract<12, NB, kU8, kChain>(c, x, n, out, s);
    default: return launch_contract<14, NB, kU8, kChain>(c, x, n, out, s);
    }
}

template <bool kChain>
static int launch_contract_planes(hdc_ctx_impl *c, const void *x, int64_t n, uint32_t *out, hipStream_t s) {
    const bool u8 = c->p.feat_dtype == HDC_U8;
    if (c->p.L <= 64)
        return u8 ? launch_contract_steps<6, true, kChain>(c, x, n, out, s) : launch_contract_steps<6, false, kChain>(c, x, n, out, s);
    return u8 ? launch_contract_steps<8, true, kChain>(c, x, n, out, s) : launch_contract_steps<8, false, kChain>(c, x, n, out, s);
}

// Encodes with the contraction if the model and the call are of its shape; false otherwise (then
// nothing was launched).
bool try_encode_contract(hdc_ctx_impl *c, const void *feats, int64_t N, uint32_t *hv, hipStream_t s, int *rc) {
    if (!c->ct_ready) return false;
    const bool splits = c->ct_max_split > 0 && c->ct_tiles[c->ct_min_split] * c->ct_steps >= kCtSplitWork;
    if (N < (splits ? kCtMinSamplesSplit : kCtMinSamples)) return false;
    ProfScope prof(c, HDC_K_ENCODE_CONTRACT, s);
    *rc = c->ct_chained ? launch_contract_planes<true>(c, feats, N, hv, s) : launch_contract_planes<false>(c, feats, N, hv, s);
    return true;
}

}  // namespace hdc
