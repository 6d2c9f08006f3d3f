// ID-Level encoding (arXiv 2206.04746, Sec. III Eq. 1) as a contraction over the features on the
// matrix cores, for long streams of samples and models of at most 640 feature slots: the form of
// encode_contract.hip rearranged so that the vector unit has less to do per matrix instruction.
//
// As there, a dimension d that flips once along the levels, at level t_d, gets from feature f the
// vote B[f][d] ^ [q_f >= t_d] with B = item ^ level[0], and with U_f = [q_f >= t_d]
//     count[d] = sum_f B[f][d] - sum_f U_f (2 B[f][d] - 1).
// The second sum is a dot product of a 0/1 vector with a +-1 vector: on 4-bit floats the sample
// side is a nibble with one bit set (0.5, 1 or 2, the bits of U in place), the model side is
// the reciprocal of that with the sign of 2 B - 1, every product is +-1 and the fp32 sums are
// exact.  What the vote threshold and the constant sum_f B need is added by the contraction
// itself: the feature slots between F and the next multiple of 64 are given U = 1 for every
// sample (their bin number is all ones) and model-side values that add up to -(K_d + 1/2),
// K_d = sum_f B[f][d] + tie_d - ceil(votes / 2).  The accumulators start at zero (an inline
// constant of the instruction) and the encoded bit is their sign: no per-sample count of U, no
// start values, no compare.
//
// A block of eight waves takes a job of G groups of 32 samples (G = 4, or 2 where the LDS does not
// hold four), a job after the other:
//   Q  it loads and quantises the job (cache hits: the lines were touched while the previous
//      job's rows were written), leaves the bin numbers in LDS a byte each, and turns them into
//      bit planes over the features, [group][step] of 64 lanes x NB words, in LDS;
//   T  a wave takes a threshold and up to five tiles of 16 of its dimensions at a time.  The
//      tiles' model-side operands come ready-made from memory, 16 bytes a lane (L2 hits: every
//      block reads the same table), and stay in registers for the G groups.  The matrix
//      instruction is the 16 samples x 16 dimensions x 128 feature slots one: per group, half
//      group and 128 slots the wave reads the planes, forms [q >= t] with one 3-input bit
//      operation per plane and the four operand words with five more instructions, and issues
//      an instruction per tile: 11 vector instructions per five matrix instructions of 16
//      clocks (the 32 x 32 x 64 instruction, 32 clocks, got three per operand: a threshold's 79
//      or 80 dimensions at D = 10000, L = 64 left its third tile of 32 half empty; 19 per
//      matrix instruction in encode_contract.hip).  The signs of a lane's 8 accumulators of a
//      tile, strung together, are a byte of the word "dimension x 32 samples", left in LDS;
//   P  a wave places 64 words of a group's 32 rows at a time: a lane collects the 32 words of
//      its row word (a table names the column of every bit; constant bits of the model point at
//      an all-zero or all-one word), transposes 32 x 32 bits in registers and writes the word
//      of the 32 rows.
// What bounds it (342 features, 128 samples a job): T takes 25, P 9 and Q 3 us of a job's 45.
// In T a SIMD's two waves issue, per threshold and group, 30 matrix instructions (16 clocks each,
// one at a time per SIMD) and 106 vector instructions (66 for the operands, 40 to string the
// signs together), 904 clocks if counted one after the other, and that sum is what they take.
// A wave issues in order, so its own two kinds never overlap, and its SIMD partner's overlap
// little (a replica of the loop, with parts taken away, gives the same sum; spreading the sign
// work over the steps with a second set of accumulators, wave priorities around the matrix
// instructions, plane reads two steps ahead and barriers that wait for the LDS only changed
// nothing).
#include "hdc_internal.h"
#include "contract_tables.h"

#include <algorithm>
#include <cstdlib>
#include <type_traits>
#include <vector>

namespace hdc {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v8i __attribute__((ext_vector_type(8)));
typedef float v4f __attribute__((ext_vector_type(4)));
typedef uint32_t wd_u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t wd_u32x2 __attribute__((ext_vector_type(2)));
typedef uint32_t wd_u32x6 __attribute__((ext_vector_type(6)));
typedef uint32_t wd_u32x4_a4 __attribute__((ext_vector_type(4), aligned(4)));   // a global load of 16 bytes at any word

// Waves per block: two per group of a job.  Four groups: eight waves, a block per compute unit (two
// waves per SIMD, 256 registers each).  Two groups: four waves, and two blocks per compute unit where
// the LDS holds both, so that one block's tile phase fills the other's loads and stores.
constexpr int wd_waves_of(int groups) { return 2 * groups; }
// Tiles of 16 dimensions of one threshold a wave works on at a time: their model-side operands
// stay in registers (4 a tile and matrix instruction of 128 feature slots).  Five tiles hold the
// dimensions of a threshold of the usual models (79 or 80 at D = 10000, L = 64); a threshold
// with more is several items.
constexpr int kWdTiles = 5;
constexpr int kWdTilesLong = 5;      // ... of models of more than 6 steps
constexpr int wd_tiles_of(int steps) { return steps > 6 ? kWdTilesLong : kWdTiles; }
// Steps of 64 feature slots per tile at most, two to a matrix instruction.
constexpr int kWdMaxSteps = 10;
constexpr size_t kWdLdsLimit = 160 * 1024;

// ---- host: tables of the model (built in contract_tables.h) ------------------------------------
template <typename T>
static int wd_upload(T **dst, const std::vector<T> &src) {
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

size_t wide_lds_bytes(int steps, int nb, int groups, int ovs) {
    const size_t planes = (size_t)groups * steps * kWave * (16 + (nb > 6 ? 16 : 8));
    const size_t over = (size_t)groups * ovs * 4;
    const size_t bins = (size_t)groups * 32 * (steps * 64 + 16);
    return 16 + planes + std::max(over, bins);
}

// Leaves c->wd_ready false when the model is not of the kernel's shape; only a failed allocation
// or copy is an error.  Needs c->expand_d (the constant bits of the level-invariant dimensions).
int prepare_wide(hdc_ctx_impl *c, const uint32_t *item, const uint32_t *level, const uint32_t *tie) {
    const hdc_params &p = c->p;
    const int W = c->W, F = p.F, L = p.L;
    c->wd_ready = false;
    if (!c->expand_d || L < 2 || L > 256 || F < 4 || F > 64 * kWdMaxSteps || W > 512) return HDC_OK;
    const ModelView model = {p.D, W, F, L, c->votes, item, level, tie};
    std::vector<std::vector<int>> by_tau;
    if (!flip_thresholds(model, &by_tau)) return HDC_OK;   // a dimension that flips twice rules the model out
    WdTables tabs;
    build_wide_tables(model, by_tau, kWdMaxSteps, kWdTiles, &tabs);
    if (tabs.steps && wd_tiles_of(tabs.steps) != kWdTiles)   // (the steps come out the same)
        build_wide_tables(model, by_tau, kWdMaxSteps, wd_tiles_of(tabs.steps), &tabs);
    if (!tabs.steps) return HDC_OK;
    const int steps = tabs.steps, cols = tabs.cols;
    const int nb = L <= 64 ? 6 : 8;
    const std::vector<int32_t> &items = tabs.items;
    const std::vector<uint32_t> &bx = tabs.bx;
    // constant bits of the model: the all-zero word at column `cols`, the all-one word after it
    std::vector<uint32_t> const_row((size_t)W), src2;
    {
        hipError_t e = hipMemcpy(const_row.data(), c->expand_d + (size_t)7 * W, (size_t)W * 4, hipMemcpyDeviceToHost);
        if (e != hipSuccess) return hip_fail(e, "hipMemcpy");
    }
    if (!wide_place_table(tabs, const_row.data(), p.D, W, &src2)) return HDC_OK;   // (16-bit column numbers; the LDS limit is far below)
    const int ovs = cols + 2;
    int groups = 0;
    for (int g : {4, 2})
        if (!groups && wide_lds_bytes(steps, nb, g, ovs) + 64 <= kWdLdsLimit) groups = g;
    if (!groups) return HDC_OK;
    if (steps > 6 && groups != 4) return HDC_OK;   // (measured: with two groups a job the other kernel is faster for such models)
    int rc = wd_upload(&c->wd_items_d, items);
    if (rc == HDC_OK) rc = wd_upload(&c->wd_bx_d, bx);
    if (rc == HDC_OK) rc = wd_upload(&c->wd_src_d, src2);
    if (rc != HDC_OK) return rc;
    c->wd_steps = steps;
    c->wd_nb = nb;
    c->wd_groups = groups;
    c->wd_items = (int)(items.size() / 4);
    c->wd_tiles = tabs.tiles;
    c->wd_ovs = ovs;
    c->wd_ready = true;
    return HDC_OK;
}

// Both operands as 4-bit floats (format code 4), no block scales; 16 bytes of each are used.
// 16 samples x 16 dimensions x 128 feature slots: lane 16 b + i brings sample i (first operand) or
// dimension i (second) against the 32 slots of block b; it gets back dimension i of samples
// 4 b .. 4 b + 3.
__device__ __forceinline__ v4f wd_mfma(v4i a, wd_u32x4 b, v4f c) {
    const v8i a8 = {a[0], a[1], a[2], a[3], 0, 0, 0, 0};
    const v8i b8 = {(int)b[0], (int)b[1], (int)b[2], (int)b[3], 0, 0, 0, 0};
    return __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(a8, b8, c, 4, 4, 0, 0, 0, 0);
}


// Dynamic LDS: the planes [G * KS][64 lanes] of 16 bytes (planes 0..3), then of 8 or 16 bytes (planes
// 4..), then a region that holds first the job's bin numbers, a byte each, [sample][KS * 64 + 16]
// (the 16 spread the rows over the banks), and later per group and column the bits of the
// group's 32 samples, [G][ovs] words, the last two of each group all zeros and all ones.
template <int KS, int NB, bool kU8, int G>
__global__ __launch_bounds__(wd_waves_of(G) * kWave, 2) void encode_wide_kernel(
    const void *__restrict__ feats, int64_t N, int F, int L, const float *__restrict__ lo,
    const float *__restrict__ scale, int W, const int4 *__restrict__ items, int n_items,
    const wd_u32x4 *__restrict__ bx, const uint32_t *__restrict__ src_of, int ovs, int stagger, uint32_t *__restrict__ hv) {
    extern __shared__ __attribute__((aligned(16))) uint32_t wd_lds[];
    constexpr int kWdWaves = wd_waves_of(G), kWdThreads = kWdWaves * kWave;
    constexpr int kSamples = 32 * G;
    constexpr int kQuads = KS * 16;                              // groups of four features per sample row, pad slots included
    constexpr int kPerRound = kWdThreads / kQuads;               // samples the block loads at a time
    constexpr int kRounds = (kSamples + kPerRound - 1) / kPerRound;
    constexpr int kBatch = kRounds <= 26 ? kRounds : (kRounds + 1) / 2;   // rounds in flight together (their registers)
    constexpr int kRowBytes = KS * 64 + 16;
    constexpr int kRawRegs = kU8 ? 1 : 4;
    // 128-byte lines of the next job's features a thread asks for ahead of time: all of them up to
    // three per thread (192 KB a block); of longer feature rows only that much, since what a
    // compute unit can count on in its die's L2 (4 MB for 32 units, the model's tables in it as
    // well) is less than a job (617 features: 316 KB; asking for all of it was 2 to 4 % slower than
    // for none, the counters showing the lines fetched twice)
    constexpr int kTouches = std::min(3, (kSamples * KS * 64 * (kU8 ? 1 : 4) / 128 + kWdThreads - 1) / kWdThreads);
    constexpr int TB = wd_tiles_of(KS);
    uint32_t *ticket = wd_lds;   // the next item of the tile phase (16 bytes in front of the planes)
    wd_u32x4 *planes_a = reinterpret_cast<wd_u32x4 *>(wd_lds + 4);
    typedef typename std::conditional<(NB > 6), wd_u32x4, wd_u32x2>::type plane_b_t;
    plane_b_t *planes_b = reinterpret_cast<plane_b_t *>(wd_lds + 4 + G * KS * kWave * 4);
    uint32_t *over = wd_lds + 4 + G * KS * kWave * (4 + (NB > 6 ? 4 : 2));
    uint8_t *over8 = reinterpret_cast<uint8_t *>(over);
    const uint8_t *bins = reinterpret_cast<const uint8_t *>(over);
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int lane = threadIdx.x & (kWave - 1);
    const int j = lane & 31, h = lane >> 5;
    static_assert(KS % 2 == 0, "two steps of 64 feature slots to a matrix instruction");
    constexpr int KH = KS / 2;          // matrix instructions per tile and half group
    // In the tile phase lane 16 b + i stands for sample i of a half group and the 32 feature slots
    // of block b of a matrix instruction: step b / 2, half b % 2 of the planes
    const int jc = lane & 15, kq = lane >> 4;
    const int plane_lane = (kq >> 1) * kWave + (kq & 1) * 32 + jc;

    wd_u32x4 bm[TB][KH];
    const int64_t jobs = (N + kSamples - 1) / kSamples;
    // All blocks start together and a job takes every block the same time, so for their first ten
    // jobs or so (until they have drifted apart by themselves) the whole chip loads, computes and
    // stores in step, and the loads and stores of 256 blocks at once queue up behind each other.
    // Blocks therefore start up to half a job apart (measured on 1M samples: 4 % of the launch).
    // The wait ends with the clock, and after a bounded number of naps whatever the clock does.
    if (stagger > 0) {
        const uint64_t t0 = wall_clock64();
        const uint64_t ticks = (uint64_t)((blockIdx.x >> 3) & 7) * (uint64_t)stagger;   // 10 ns each; neighbours in a die start apart
        for (int nap = 0; nap < 20000 && wall_clock64() - t0 < ticks; ++nap) __builtin_amdgcn_s_sleep(8);
    }
    for (int64_t job = blockIdx.x; job < jobs; job += gridDim.x) {   // block-uniform
        // ---- Q: bin numbers, a byte each; slots past F get all ones (U = 1 at every threshold).
        // A thread takes four neighbouring features (the same in every round) of kPerRound samples
        // a round, all rounds in flight together (cache hits but for a block's first job: the lines
        // were asked for while the previous job's rows were written).  Every thread loads in every
        // round (those without a feature or a sample of their own: something that exists).
        {
            if (threadIdx.x == 0) *ticket = kWdWaves;   // (every wave starts on item `wave`)
            int tid = threadIdx.x;
            asm volatile("" : "+v"(tid));   // (opaque: what follows is worked out per job, not kept in registers across the phases)
            const int f0 = 4 * (tid % kQuads), s_in = tid / kQuads;
            const bool feats_mine = f0 < F;                               // (slots past F are not features)
            const int fq = min(f0, F - 4);                                // what it loads: four features that exist
            const int q_shift = 8 * min(max(f0 - fq, 0), 3);              // where its own first feature's bin number is in them
            uint32_t keep = 0;                                            // the bytes of its word that are features
#pragma unroll
            for (int i = 0; i < 4; ++i)
                if (f0 + i < F) keep |= 0xffu << (8 * i);
            const int64_t first = job * kSamples;
            const int last = (int)min((int64_t)(kSamples - 1), N - 1 - first);   // (rows past N: the last row)
            const uint8_t *base = reinterpret_cast<const uint8_t *>(feats) + first * F * (kU8 ? 1 : 4);
            float lo_f[4], sc_f[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                lo_f[i] = kU8 ? 0.0f : lo[fq + i];
                sc_f[i] = kU8 ? 0.0f : scale[fq + i];
            }
#pragma unroll
            for (int r0 = 0; r0 < kRounds; r0 += kBatch) {   // (one turn up to 384 feature slots; the turns one after the other)
                uint32_t raw[kBatch][kRawRegs];
#pragma unroll
                for (int rr = 0; rr < kBatch; ++rr) {
                    const int sn = min((r0 + rr) * kPerRound + s_in, last);
                    if (kU8) {
                        const uint8_t *row = base + (sn * F + fq);
                        raw[rr][0] = (uint32_t)row[0] | ((uint32_t)row[1] << 8) | ((uint32_t)row[2] << 16) | ((uint32_t)row[3] << 24);
                    } else {
                        const wd_u32x4_a4 v = *reinterpret_cast<const wd_u32x4_a4 *>(base + (size_t)(uint32_t)((sn * F + fq) * 4));
#pragma unroll
                        for (int i = 0; i < 4; ++i) raw[rr][i] = v[i];
                    }
                }
                if (s_in < kPerRound) {
#pragma unroll
                    for (int rr = 0; rr < kBatch; ++rr) {
                        const int sn = (r0 + rr) * kPerRound + s_in;
                        uint32_t word = 0;
                        if (feats_mine) {
#pragma unroll
                            for (int i = 0; i < 4; ++i) {
                                uint32_t q;
                                if (kU8) {
                                    q = (((raw[rr][0] >> (8 * i)) & 0xffu) * (uint32_t)L) >> 8;
                                } else {   // the bin rule without its branches: NaN and negatives go to 0 through the maximum
                                    const float t = __fmul_rn(__fsub_rn(__builtin_bit_cast(float, raw[rr][i]), lo_f[i]), sc_f[i]);
                                    q = (uint32_t)(int)fminf(fmaxf(t, 0.0f), (float)(L - 1));
                                }
                                word |= q << (8 * i);
                            }
                            word = (word >> q_shift) & keep;
                        }
                        if (sn < kSamples) over[(sn * kRowBytes + f0) >> 2] = word | ~keep;
                    }
                }
                __builtin_amdgcn_sched_barrier(0);
            }
        }
        __syncthreads();
        // The bin numbers as bit planes over the features: lane (sample j, half h) reads its 32 bytes of
        // step k of group g and moves bit b of byte i of word m to bit 8 i + m of plane b (word index
        // and bit index trade three of their bits, one per round).
#pragma unroll 1
        for (int task = wave; task < G * KS; task += kWdWaves) {
            const int g = task / KS, k = task - g * KS;
            const wd_u32x4 *from = reinterpret_cast<const wd_u32x4 *>(bins + (g * 32 + j) * kRowBytes + k * 64 + h * 32);
            const wd_u32x4 v0 = from[0], v1 = from[1];
            uint32_t x[8] = {v0[0], v0[1], v0[2], v0[3], v1[0], v1[1], v1[2], v1[3]};
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
            planes_a[task * kWave + lane] = wd_u32x4{x[0], x[1], x[2], x[3]};
            if constexpr (NB > 6) planes_b[task * kWave + lane] = wd_u32x4{x[4], x[5], x[6], x[7]};
            else planes_b[task * kWave + lane] = wd_u32x2{x[4], x[5]};
        }
        __syncthreads();
        if (threadIdx.x < 2 * G) over[(threadIdx.x >> 1) * ovs + ovs - 2 + (threadIdx.x & 1)] = (threadIdx.x & 1) ? 0xffffffffu : 0u;

        // ---- T: a threshold and up to TB tiles of 16 of its dimensions per wave and turn.  The tiles'
        // model-side operands stay in registers for the G groups; while the last group is worked
        // on, each is replaced by the next item's as soon as its last instruction has been issued
        // (those of the first matrix instruction, wanted first, wait in registers of their own
        // from the item's start: 1 % of the kernel).
        // The items are dealt out by a counter: the SIMD favours its older wave, which would be
        // through a fixed share early and leave the younger one to finish alone (1.95 -> 1.75 ms per
        // million samples).  Units of an item and half of the groups, to shorten the wait for the
        // last wave, were slower (1.90 ms): every unit fetches its tiles' operands again.
        {
            constexpr int kSplit = 1, kUnitGroups = G;   // units per item, groups per unit
            const int n_units = n_items * kSplit;
            int unit = wave;
            auto claim = [&]() {
                uint32_t got = 0;
                if (lane == 0) got = atomicAdd(ticket, 1u);
                return (int)__builtin_amdgcn_readfirstlane(got);
            };
            int unit_next = claim();
            int4 item = items[min(unit / kSplit, n_items - 1)];
            if (unit < n_units) {
                const int tile0 = __builtin_amdgcn_readfirstlane(item.y), nt = (__builtin_amdgcn_readfirstlane(item.z) + 15) >> 4;
#pragma unroll
                for (int t = 0; t < TB; ++t)
#pragma unroll
                    for (int k = 0; k < KH; ++k) bm[t][k] = bx[((size_t)(tile0 + min(t, nt - 1)) * KH + k) * kWave + lane];
            }
#pragma unroll 1
            for (; unit < n_units; unit = unit_next, unit_next = claim()) {
                const int g0 = (unit % kSplit) * kUnitGroups;
                const int tau = __builtin_amdgcn_readfirstlane(item.x);
                const int nd = __builtin_amdgcn_readfirstlane(item.z), col0 = __builtin_amdgcn_readfirstlane(item.w);
                const int nt = (nd + 15) >> 4;
                const int un = unit_next < n_units ? unit_next : unit;   // (after the wave's last unit: the same again, unused)
                const int g0_n = (un % kSplit) * kUnitGroups;
                item = items[un / kSplit];
                const int tile0_n = __builtin_amdgcn_readfirstlane(item.y), nt_n = (__builtin_amdgcn_readfirstlane(item.z) + 15) >> 4;
                const wd_u32x4 *bn[TB];
#pragma unroll
                for (int t = 0; t < TB; ++t) bn[t] = bx + (size_t)(tile0_n + min(t, nt_n - 1)) * KH * kWave + lane;
                // the next item's operands of the first matrix instruction are asked for now, a whole
                // item ahead (those of the others replace this item's in its last group, a group ahead)
                wd_u32x4 b0n[TB];
#pragma unroll
                for (int t = 0; t < TB; ++t) b0n[t] = bn[t][0];
                uint32_t tb[NB];
#pragma unroll
                for (int b = 0; b < NB; ++b) tb[b] = (tau >> b) & 1 ? 0xffffffffu : 0u;   // wave-uniform
                wd_u32x4 pa = planes_a[g0 * KS * kWave + plane_lane];
                plane_b_t pb = planes_b[g0 * KS * kWave + plane_lane];
                // One group of 32 samples, as two halves of 16, against the item's NT tiles (a
                // constant here: no branch in the loop); the last group also fetches the next
                // item's operands, each as soon as its last instruction has been issued.
                auto group = [&](const int g, auto nt_c, auto last_c) {
                    constexpr int NT = decltype(nt_c)::value;
                    constexpr bool kLast = decltype(last_c)::value;
                    v4f acc[NT][2];
                    const wd_u32x4 *pa_at = planes_a + (kLast ? g0_n : g + 1) * KS * kWave + plane_lane;   // where the planes after this group's are
                    const plane_b_t *pb_at = planes_b + (kLast ? g0_n : g + 1) * KS * kWave + plane_lane;
                    const wd_u32x4 *pa_in = planes_a + g * KS * kWave + plane_lane;
                    const plane_b_t *pb_in = planes_b + g * KS * kWave + plane_lane;
#pragma unroll
                    for (int k = 0; k < KH; ++k) {
#pragma unroll
                        for (int rh = 0; rh < 2; ++rh) {
                            // the samples' [q >= tau] over the lane's 32 feature slots, from the least significant plane up
                            uint32_t qp[8] = {pa[0], pa[1], pa[2], pa[3], pb[0], pb[1], 0u, 0u};
                            if constexpr (NB > 6) qp[6] = pb[2], qp[7] = pb[3];
                            if (rh == 0) {   // the next turn's planes: the other half group, then the next two steps
                                pa = pa_in[2 * k * kWave + 16];
                                pb = pb_in[2 * k * kWave + 16];
                            } else if (k + 1 < KH) {
                                pa = pa_in[2 * (k + 1) * kWave];
                                pb = pb_in[2 * (k + 1) * kWave];
                            } else {
                                pa = pa_at[0];
                                pb = pb_at[0];
                            }
                            uint32_t ge = 0xffffffffu;
#pragma unroll
                            for (int b = 0; b < NB; ++b) ge = __builtin_amdgcn_bitop3_b32(qp[b], ge, tb[b], 0xD4);   // tb ? q & ge : q | ge
                            const v4i a = {(int)(ge & 0x11111111u), (int)(ge & 0x22222222u), (int)(ge & 0x44444444u),
                                           (int)((ge >> 1) & 0x44444444u)};
#pragma unroll
                            for (int t = 0; t < NT; ++t) {
                                if (k == 0) acc[t][rh] = wd_mfma(a, bm[t][k], v4f{0, 0, 0, 0});
                                else acc[t][rh] = wd_mfma(a, bm[t][k], acc[t][rh]);
                            }
                        }
                        if constexpr (kLast) {
                            if (k > 0) {
#pragma unroll
                                for (int t = 0; t < TB; ++t) bm[t][k] = bn[t][k * kWave];
                            }
                        }
                    }
                    // the signs strung together, the first half group's first register highest: bit
                    // 7 - (4 rh + r) of the lane's byte is sample 16 rh + 4 kq + r of the group
#pragma unroll
                    for (int t = 0; t < NT; ++t) {
                        uint32_t bits = 0;
#pragma unroll
                        for (int rh = 0; rh < 2; ++rh)
#pragma unroll
                            for (int r = 0; r < 4; ++r) {
                                const float d = acc[t][rh][r];
                                bits = __builtin_amdgcn_alignbit(bits, __builtin_bit_cast(uint32_t, d), 31);
                            }
                        if (16 * t + jc < nd) over8[((size_t)(g * ovs + col0 + 16 * t + jc) << 2) + kq] = (uint8_t)bits;
                    }
                };
                auto run = [&](auto nt_c) {
#pragma unroll 1
                    for (int g = g0; g < g0 + kUnitGroups - 1; ++g) group(g, nt_c, std::false_type{});
                    group(g0 + kUnitGroups - 1, nt_c, std::true_type{});
                };
                if (nt <= 1) run(std::integral_constant<int, 1>{});
                else if (nt == 2) run(std::integral_constant<int, 2>{});
                else if (nt == 3 && TB > 3) run(std::integral_constant<int, 3>{});
                else run(std::integral_constant<int, TB>{});
#pragma unroll
                for (int t = 0; t < TB; ++t) bm[t][0] = b0n[t];
            }
        }
        __syncthreads();

        // ---- P: a wave places 64 words of a group's 32 rows at a time: lane l, word w = 64 c + l, reads
        // the 32 entries of `over` that its table names (asked for a chunk ahead), transposes 32 x 32
        // bits in registers and writes word w of the 32 rows.  Wave v takes group v % G and every
        // (waves / G)-th chunk of 64 words, which gives each SIMD the same number of chunks.  The next
        // job's features are asked for here (a word of every 128 bytes), so that they are in the
        // cache when the job starts.
        {
            const int64_t first = job * kSamples;
            constexpr int kChunkStep = kWdWaves / G;
            int lane_p = lane;
            asm volatile("" : "+v"(lane_p));   // (opaque: the offsets below are worked out per job, not kept in registers across the phases)
            const int g = wave % G;
            const int chunks = (W + kWave - 1) / kWave;
            constexpr int kMaxChunks = (8 + kChunkStep - 1) / kChunkStep;   // rows of up to 512 words (the host sees to that)
            uint32_t from[kMaxChunks][16];   // all of the wave's table entries first: nothing else is in flight yet
            uint32_t touched = 0;
#pragma unroll
            for (int ci = 0; ci < kMaxChunks; ++ci) {
                // (a uniform base and a 32-bit offset per lane: no 64-bit address per load to keep)
                const uint32_t off = 4u * (uint32_t)min((wave / G + ci * kChunkStep) * kWave + lane_p, W - 1);
#pragma unroll
                for (int i = 0; i < 16; ++i)
                    from[ci][i] = *reinterpret_cast<const uint32_t *>(reinterpret_cast<const uint8_t *>(src_of + (size_t)i * W) + off);
            }
            {
                const int64_t nj = min(job + (int64_t)gridDim.x, jobs - 1);   // (after the last job: once more)
                const uint32_t *base = reinterpret_cast<const uint32_t *>(reinterpret_cast<const uint8_t *>(feats) + nj * kSamples * F * (kU8 ? 1 : 4));
                const int64_t words = (min((int64_t)kSamples, N - nj * kSamples) * F * (kU8 ? 1 : 4)) >> 2;
                const int64_t lines = (words + 31) >> 5;
#pragma unroll
                for (int i = 0; i < kTouches; ++i) {
                    const int64_t at = min((int64_t)(threadIdx.x + i * kWdThreads), lines - 1) * 32;
                    touched ^= base[min(at, words - 1)];
                }
            }
            const bool whole = first + kSamples <= N;   // block-uniform: no row of the job is past N
#pragma unroll
            for (int ci = 0; ci < kMaxChunks; ++ci) {
                const int c = wave / G + ci * kChunkStep;
                if (c >= chunks) break;   // wave-uniform
                const int w = min(c * kWave + lane_p, W - 1);
                uint32_t x[32];
#pragma unroll
                for (int i = 0; i < 16; ++i) {
                    x[2 * i] = over[g * ovs + (from[ci][i] & 0xffffu)];
                    x[2 * i + 1] = over[g * ovs + (from[ci][i] >> 16)];
                }
                // x[b] bit p  ->  x[p] bit b: halves and bytes trade places by byte permutes, the finer
                // stages by masked merges
#pragma unroll
                for (int i = 0; i < 16; ++i) {
                    const uint32_t lo = x[i], hi = x[i + 16];
                    x[i] = __builtin_amdgcn_perm(hi, lo, 0x05040100u);
                    x[i + 16] = __builtin_amdgcn_perm(hi, lo, 0x07060302u);
                }
#pragma unroll
                for (int i = 0; i < 32; ++i)
                    if ((i & 8) == 0) {
                        const uint32_t lo = x[i], hi = x[i + 8];
                        x[i] = __builtin_amdgcn_perm(hi, lo, 0x06020400u);
                        x[i + 8] = __builtin_amdgcn_perm(hi, lo, 0x07030501u);
                    }
#pragma unroll
                for (int stage = 2; stage < 5; ++stage) {
                    const int k = 16 >> stage;
                    const uint32_t m = stage == 2 ? 0x0f0f0f0fu : stage == 3 ? 0x33333333u : 0x55555555u;
#pragma unroll
                    for (int i = 0; i < 32; ++i)
                        if ((i & k) == 0) {
                            const uint32_t lo = x[i], hi = x[i + k];
                            x[i] = (lo & m) | ((hi << k) & ~m);
                            x[i + k] = ((lo >> k) & m) | (hi & ~m);
                        }
                }
                // bit p of a word of `over`: byte p / 8 came from the lanes of feature block p / 8, whose
                // registers hold samples 4 (p / 8) .. + 3 of either half group; bit 7 - (4 rh + r) of the byte is
                // register r of half group rh.
                // The rows go past the caches (streaming stores): a long stream's rows are read again
                // only after many more have been written, and kept in the L2 they push out the next
                // job's features and leave the kernel that reads the rows next a cache full of lines
                // to write back (the accumulating pass over 1M rows: 274 -> 225 us).
                if (c * kWave + lane_p < W) {
                    uint8_t *out = reinterpret_cast<uint8_t *>(hv + (first + 32 * g) * W);   // wave-uniform
#pragma unroll
                    for (int p = 0; p < 32; ++p) {
                        const int sn = 16 * ((7 - (p & 7)) >> 2) + 4 * (p >> 3) + ((7 - (p & 7)) & 3);
                        if (whole || first + 32 * g + sn < N) __builtin_nontemporal_store(x[p], reinterpret_cast<uint32_t *>(out + 4u * (uint32_t)(sn * W + w)));
                    }
                }
                __builtin_amdgcn_sched_barrier(0);   // (a chunk after the other: their registers are the same)
            }
            if (touched == 0x9e3779b9u && N < 0) hv[0] = touched;   // (never: keeps the loads above)
        }
        __syncthreads();
    }
}

template <int KS, int NB, bool kU8, int G>
static int launch_wide(hdc_ctx_impl *c, const void *x, int64_t n, uint32_t *out, hipStream_t s) {
    auto kern = encode_wide_kernel<KS, NB, kU8, G>;
    const size_t lds = wide_lds_bytes(KS, NB, G, c->wd_ovs);
    if (lds > 64 * 1024)
        HDC_HIP(hipFuncSetAttribute(reinterpret_cast<const void *>(kern), hipFuncAttributeMaxDynamicSharedMemorySize,
                                    (int)lds));
    const int64_t jobs = (n + 32 * G - 1) / (32 * G);
    const int per_cu = G == 2 && 2 * (lds + 1024) <= kWdLdsLimit ? 2 : 1;
    const int64_t blocks = std::min<int64_t>(jobs, (int64_t)c->num_cus * per_cu);
    // Start offsets between blocks (see the kernel): a sixteenth of a job's time per step, eight steps, from ten
    // jobs per block on.  A job takes about 3.2 times what its matrix instructions take alone
    // (7.6 ns each, four SIMDs).
    int stagger = 0;
    if (jobs >= 10 * blocks) {
        const double job_us = (double)c->wd_tiles * KS * G * 0.0076 / 4.0 * 3.2;
        stagger = (int)std::min(job_us * 100.0 / 16.0, 1000.0);   // in 10 ns; at most 10 us a step
    }
    hipLaunchKernelGGL(kern, dim3((unsigned)blocks), dim3(wd_waves_of(G) * kWave), lds, s, x, n, c->p.F, c->p.L, c->lo_d,
                       c->scale_d, c->W, reinterpret_cast<const int4 *>(c->wd_items_d), c->wd_items,
                       reinterpret_cast<const wd_u32x4 *>(c->wd_bx_d), c->wd_src_d, c->wd_ovs, stagger, out);
    HDC_HIP(hipGetLastError());
    return HDC_OK;
}

template <int NB, bool kU8, int G>
static int launch_wide_steps(hdc_ctx_impl *c, const void *x, int64_t n, uint32_t *out, hipStream_t s) {
    switch (c->wd_steps) {
    case 2: return launch_wide<2, NB, kU8, G>(c, x, n, out, s);
    case 4: return launch_wide<4, NB, kU8, G>(c, x, n, out, s);
    case 6: return launch_wide<6, NB, kU8, G>(c, x, n, out, s);
    case 8: return launch_wide<8, NB, kU8, G>(c, x, n, out, s);
    default: return launch_wide<10, NB, kU8, G>(c, x, n, out, s);
    }
}

// The kernel is taken when the jobs of 32 G samples fill the chip's blocks, which work through
// their jobs one after the other, to seven tenths at least (so from one job per compute unit on;
// 1.2 jobs per unit would be two rounds for the price of 1.2).
bool try_encode_wide(hdc_ctx_impl *c, const void *feats, int64_t N, uint32_t *hv, hipStream_t s, int *rc) {
    if (!c->wd_ready) return false;
    const int64_t jobs = (N + 32 * c->wd_groups - 1) / (32 * c->wd_groups);
    const int64_t rounds = (jobs + c->num_cus - 1) / c->num_cus;
    if (jobs < c->num_cus || jobs * 10 < rounds * c->num_cus * 7) return false;
    ProfScope prof(c, HDC_K_ENCODE_WIDE, s);
    const bool u8 = c->p.feat_dtype == HDC_U8;
    if (c->wd_groups == 4) {
        if (c->wd_nb == 6) *rc = u8 ? launch_wide_steps<6, true, 4>(c, feats, N, hv, s) : launch_wide_steps<6, false, 4>(c, feats, N, hv, s);
        else *rc = u8 ? launch_wide_steps<8, true, 4>(c, feats, N, hv, s) : launch_wide_steps<8, false, 4>(c, feats, N, hv, s);
    } else {
        if (c->wd_nb == 6) *rc = u8 ? launch_wide_steps<6, true, 2>(c, feats, N, hv, s) : launch_wide_steps<6, false, 2>(c, feats, N, hv, s);
        else *rc = u8 ? launch_wide_steps<8, true, 2>(c, feats, N, hv, s) : launch_wide_steps<8, false, 2>(c, feats, N, hv, s);
    }
    return true;
}

}  // namespace hdc

