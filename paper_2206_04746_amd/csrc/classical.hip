// Classical training (arXiv 2206.04746, Sec. III): acc[c][d] += hv[n][d] for c = label[n],
// and the majority vote that turns the sums into class vectors.
//
// The per-dimension sum down a column of packed rows is the paper's "vertical summation"
// (Sec. IV-B2).  Here it needs no transposition: a lane owns one 32-bit word column and
// keeps the 32 counts bit-sliced (plane i = bit i of each count); adding rows is carry-save
// arithmetic with v_bitop3_b32 full adders, a few VALU ops per streamed word, so the kernel
// stays HBM-bound.  Rows of up to 320 words and up to four classes: a block takes a run of
// consecutive rows, orders them by class by itself in LDS and gives each of its 16 waves a
// share to read as whole rows (accumulate_local_kernel: no grouping pass, no wave waits for
// another while it streams; rows of up to 640 words go through it twice, a half of every
// row each time).  More classes: the rows are first grouped by class (a counting
// sort of the labels, only the row indices move) and a block takes a run of rows of ONE class
// (accumulate_rows_kernel, the same streaming).  Wider rows: grouped as well; a block's waves
// cover the slices of 64 word columns side by side (so rows are read as whole contiguous
// lines) times a few row groups, meeting at a barrier every 16 rows (accumulate_kernel).  The
// waves' bit-sliced counts are added through LDS and written out as 16-bit partial sums, one
// row of partials per block and class.  A second, tiny kernel adds the partial
// rows of each class into acc.  (Flushing blocks straight into acc with atomics was measured at
// 10-25 G atomics/s, several times slower than streaming the rows themselves.)  Everything is
// integer addition, so any order gives the same bits.
#include "hdc_internal.h"

namespace hdc {

constexpr int kAccWaves = 16;      // most waves per accumulate block (slices x row groups)
constexpr int kWavePlanes = 11;    // a wave counts at most 2040 rows
constexpr int kBlockPlanes = 12;   // a block counts at most 4088 rows
constexpr int kGroupThreads = 1024;
constexpr int64_t kSmallN = 32768;   // up to here one block groups the rows in one launch

typedef const uint32_t __attribute__((address_space(4))) *const_u32_ptr;

// ---- grouping rows by class ----------------------------------------------------------
// cnt[c] = rows with label c (c < C); off = exclusive prefix of cnt (row offsets into perm);
// blk = exclusive prefix of ceil(cnt / block_rows) (work list of the accumulate kernel).
// Run by the first wave of a block: lane l owns a contiguous chunk of classes and the chunk
// totals are prefix-summed across the wave.  cnt_s may alias cnt.
__device__ __forceinline__ void scan_counts(const uint32_t *cnt_s, int C, uint32_t block_rows,
                                            uint32_t *cnt, uint32_t *off, uint32_t *blk, uint32_t *off_s,
                                            int64_t *class_n) {
    const int lane = threadIdx.x;
    if (lane >= kWave) return;
    const int per = (C + kWave - 1) / kWave;
    const int c0 = min(lane * per, C), c1 = min(c0 + per, C);
    uint32_t so = 0, sb = 0;
    for (int c = c0; c < c1; ++c) {
        so += cnt_s[c];
        sb += (cnt_s[c] + block_rows - 1) / block_rows;
    }
    uint32_t po = so, pb = sb;   // inclusive wave scan
#pragma unroll
    for (int d = 1; d < kWave; d <<= 1) {
        const uint32_t to = __shfl_up(po, d, kWave), tb = __shfl_up(pb, d, kWave);
        if (lane >= d) {
            po += to;
            pb += tb;
        }
    }
    uint32_t o = po - so, b = pb - sb;
    for (int c = c0; c < c1; ++c) {
        const uint32_t k = cnt_s[c];
        off[c] = o;
        blk[c] = b;
        if (off_s) off_s[c] = o;
        cnt[c] = k;
        class_n[c] += (int64_t)k;
        o += k;
        b += (k + block_rows - 1) / block_rows;
    }
    if (lane == kWave - 1) {
        off[C] = po;
        blk[C] = pb;
    }
}

// Small batches: one block counts, scans and scatters in a single launch.
__global__ __launch_bounds__(kGroupThreads) void group_small_kernel(
    const int32_t *__restrict__ labels, int N, int C, uint32_t block_rows, uint32_t *cnt, uint32_t *off,
    uint32_t *blk, uint32_t *perm, int64_t *class_n) {
    extern __shared__ uint32_t sm[];   // cnt_s[C + 1] | off_s[C + 1] (then the scatter cursors)
    uint32_t *cnt_s = sm, *off_s = sm + (C + 1);
    for (int i = threadIdx.x; i <= C; i += kGroupThreads) cnt_s[i] = 0;
    __syncthreads();
    for (int n = threadIdx.x; n < N; n += kGroupThreads) {
        const int32_t y = labels[n];
        if (y >= 0 && y < C) atomicAdd(&cnt_s[y], 1u);
    }
    __syncthreads();
    scan_counts(cnt_s, C, block_rows, cnt, off, blk, off_s, class_n);
    __syncthreads();
    for (int n = threadIdx.x; n < N; n += kGroupThreads) {
        const int32_t y = labels[n];
        if (y >= 0 && y < C) perm[atomicAdd(&off_s[y], 1u)] = (uint32_t)n;
    }
}

// Large batches: count and scatter over many blocks.  The per-class totals and cursors live in
// cur[0..C), cur[C + 1] counts the blocks that are through; all of them are zero between launches:
// the block that finds itself last (a ticket from the counter) takes the totals out with exchanges
// that leave zeros, so no launch is needed to clear them, and does the launch's serial part (the
// scan over the classes).  These words are only ever touched by device-wide atomics, and a block
// takes its ticket after its own atomics have returned their values, so the last block's
// exchanges see every addition; nothing else is passed between blocks, and no fence is used (a
// device-wide release writes back the whole L2 of the block's die: 20 us here after an encode).
// One stream at a time per context, as for all of the training scratch.
__device__ __forceinline__ bool last_block_done(uint32_t *done, uint32_t *flag_s) {
    __syncthreads();
    if (threadIdx.x == 0) {
        const uint32_t t = atomicAdd(done, 1u);
        const bool last = t == gridDim.x - 1;
        if (last) atomicExch(done, 0u);   // (nobody else touches it again in this launch)
        *flag_s = last;
    }
    __syncthreads();
    return *flag_s != 0;
}

// Count the labels; the last block scans the totals into cnt / off / blk and adds them to class_n.
__global__ __launch_bounds__(256) void count_labels_kernel(const int32_t *__restrict__ labels,
                                                            int64_t N, int C, uint32_t block_rows,
                                                            uint32_t *cur, uint32_t *cnt, uint32_t *off,
                                                            uint32_t *blk, int64_t *class_n) {
    extern __shared__ uint32_t h[];   // h[C], then the flag
    for (int i = threadIdx.x; i < C; i += 256) h[i] = 0;
    __syncthreads();
    for (int64_t n = (int64_t)blockIdx.x * 256 + threadIdx.x; n < N; n += (int64_t)gridDim.x * 256) {
        const int32_t y = labels[n];
        if (y >= 0 && y < C) atomicAdd(&h[y], 1u);
    }
    __syncthreads();
    for (int i = threadIdx.x; i < C; i += 256)
        if (h[i]) {
            const uint32_t was = atomicAdd(&cur[i], h[i]);
            asm volatile("" ::"v"(was));   // (waited for: the addition is done before the block's ticket is taken)
        }
    if (!last_block_done(cur + C + 1, h + C)) return;
    for (int i = threadIdx.x; i < C; i += 256) h[i] = atomicExch(&cur[i], 0u);
    __syncthreads();
    scan_counts(h, C, block_rows, cnt, off, blk, nullptr, class_n);
}

// Each block handles contiguous runs of labels: local histogram, ONE global atomic per class to
// reserve the run's range in perm, then local ranks from LDS cursors.  The last block clears the
// cursors.
constexpr int kScatterRun = 4096;
__global__ __launch_bounds__(256) void scatter_rows_kernel(const int32_t *__restrict__ labels,
                                                            int64_t N, int C,
                                                            const uint32_t *__restrict__ off,
                                                            uint32_t *cur, uint32_t *perm) {
    extern __shared__ uint32_t h[];   // h[C]: count, then the run's next free slot per class; then the flag
    for (int64_t run0 = (int64_t)blockIdx.x * kScatterRun; run0 < N;
         run0 += (int64_t)gridDim.x * kScatterRun) {
        const int64_t run1 = min(run0 + (int64_t)kScatterRun, N);
        for (int i = threadIdx.x; i < C; i += 256) h[i] = 0;
        __syncthreads();
        for (int64_t n = run0 + threadIdx.x; n < run1; n += 256) {
            const int32_t y = labels[n];
            if (y >= 0 && y < C) atomicAdd(&h[y], 1u);
        }
        __syncthreads();
        for (int i = threadIdx.x; i < C; i += 256) {
            const uint32_t k = h[i];
            h[i] = k ? off[i] + atomicAdd(&cur[i], k) : 0u;
        }
        __syncthreads();
        for (int64_t n = run0 + threadIdx.x; n < run1; n += 256) {
            const int32_t y = labels[n];
            if (y >= 0 && y < C) perm[atomicAdd(&h[y], 1u)] = (uint32_t)n;
        }
        __syncthreads();
    }
    if (!last_block_done(cur + C + 1, h + C)) return;
    for (int i = threadIdx.x; i < C; i += 256) atomicExch(&cur[i], 0u);
}

// One or two classes: no totals are needed before the rows are placed.  Class 0 fills perm from
// the front, class 1 from the back (the order inside a class does not matter to a sum), so one
// launch counts and scatters; the last block writes cnt / off / blk and adds to class_n.  A
// block's threads hold the 16384 labels of its run in registers (all loads in flight together);
// wave ballots count the classes and rank the rows, one atomic per class reserves the run's
// ranges.
constexpr int kTwoPer = 64;                 // labels per thread: few blocks, since every block's three atomics
constexpr int kTwoRun = 256 * kTwoPer;      // on the same words are served one after the other (about 30 ns each)
__global__ __launch_bounds__(256) void group_two_kernel(const int32_t *__restrict__ labels, int64_t N, int C,
                                                         uint32_t block_rows, uint32_t *cur, uint32_t *cnt,
                                                         uint32_t *off, uint32_t *blk, uint32_t *perm,
                                                         int64_t *class_n) {
    __shared__ uint32_t wsum[4], base_s[2], flag_s;
    const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x >> 6;
    const uint64_t below = ((uint64_t)1 << lane) - 1;
    for (int64_t run0 = (int64_t)blockIdx.x * kTwoRun; run0 < N; run0 += (int64_t)gridDim.x * kTwoRun) {
        // label i of a thread is number i * 256 + thread of the run: neighbouring lanes, neighbouring labels
        int32_t y[kTwoPer];
#pragma unroll
        for (int i = 0; i < kTwoPer; ++i) {
            const int64_t n = run0 + i * 256 + threadIdx.x;
            y[i] = n < N ? labels[n] : -1;
        }
        uint32_t mine = 0;   // the wave's rows of class 0 | of class 1 << 16 (wave-uniform)
#pragma unroll
        for (int i = 0; i < kTwoPer; ++i)
            mine += (uint32_t)__popcll(__ballot(y[i] == 0)) + ((uint32_t)__popcll(__ballot(y[i] == 1 && C > 1)) << 16);
        if (lane == 0) wsum[wave] = mine;
        __syncthreads();
        uint32_t before = 0, total = 0;
#pragma unroll
        for (int w = 0; w < 4; ++w) {
            if (w < wave) before += wsum[w];
            total += wsum[w];
        }
        if (threadIdx.x < 2) {
            const uint32_t k = threadIdx.x == 0 ? (total & 0xffffu) : (total >> 16);
            base_s[threadIdx.x] = k ? atomicAdd(&cur[threadIdx.x], k) : 0u;
        }
        __syncthreads();
        // the wave's rows in the order (step, lane): the rows of a class in one step go to neighbouring places
        uint32_t at0 = base_s[0] + (before & 0xffffu), at1 = base_s[1] + (before >> 16);
#pragma unroll
        for (int i = 0; i < kTwoPer; ++i) {
            const uint64_t m0 = __ballot(y[i] == 0), m1 = __ballot(y[i] == 1 && C > 1);
            const uint32_t row = (uint32_t)(run0 + i * 256 + threadIdx.x);
            if (y[i] == 0) perm[at0 + (uint32_t)__popcll(m0 & below)] = row;
            else if (y[i] == 1 && C > 1) perm[(uint32_t)N - 1u - (at1 + (uint32_t)__popcll(m1 & below))] = row;
            at0 += (uint32_t)__popcll(m0);
            at1 += (uint32_t)__popcll(m1);
        }
        __syncthreads();   // (wsum and base_s are written again in the next run)
    }
    if (!last_block_done(cur + C + 1, &flag_s)) return;
    if (threadIdx.x == 0) {
        const uint32_t k0 = atomicExch(&cur[0], 0u), k1 = C > 1 ? atomicExch(&cur[1], 0u) : 0u;
        const uint32_t b0 = (k0 + block_rows - 1) / block_rows, b1 = (k1 + block_rows - 1) / block_rows;
        cnt[0] = k0, off[0] = 0, blk[0] = 0;
        class_n[0] += (int64_t)k0;
        if (C > 1) {
            cnt[1] = k1, off[1] = (uint32_t)N - k1, blk[1] = b0;
            class_n[1] += (int64_t)k1;
            off[2] = (uint32_t)N, blk[2] = b0 + b1;
        } else {
            off[1] = k0, blk[1] = b0;
        }
    }
}

// ---- vertical count ------------------------------------------------------------------
// grid.x = work item (block of rows of one class; an upper bound, surplus blocks exit),
// grid.y = chunk of `spb` slices of 64 word columns.  The block's waves form rg row groups x
// spb slices: waves of one row group read the SAME rows side by side, so every row is fetched
// as one contiguous run by one CU (whole cache lines, no refetch by other CUs); row group g
// streams rows [g * rb, (g + 1) * rb) of the item.  Dynamic LDS: the merge area
// [(rg - 1) * spb][kWavePlanes][64].
__global__ __launch_bounds__(1024) void accumulate_kernel(
    const uint32_t *__restrict__ hv, const uint32_t *__restrict__ perm,
    const uint32_t *__restrict__ cnt, const uint32_t *__restrict__ off,
    const uint32_t *__restrict__ blk, int C, int W, int Wp, int rb, int spb, int rg,
    uint32_t *__restrict__ partial) {
    extern __shared__ uint32_t merge[];
    const uint32_t item = blockIdx.x;
    if (item >= blk[C]) return;
    // class of this work item: last c with blk[c] <= item (blk is non-decreasing)
    int lo = 0, hi = C - 1;
    while (lo < hi) {
        const int mid = (lo + hi + 1) >> 1;
        if (blk[mid] <= item) lo = mid; else hi = mid - 1;
    }
    const int c = lo;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int lane = threadIdx.x & (kWave - 1);
    const int group = wave / spb;          // row group
    const int sl = wave - group * spb;     // slice within the block
    const int col = (blockIdx.y * spb + sl) * kSliceWords + lane;
    const uint32_t first = (item - blk[c]) * (uint32_t)(rg * rb) + (uint32_t)(group * rb);
    const uint32_t total = cnt[c];
    const uint32_t rows = first < total ? min((uint32_t)rb, total - first) : 0u;
    const bool in_range = col < W;

    const_u32_ptr idx = (const_u32_ptr)(uintptr_t)(perm + off[c] + first);   // wave-uniform
    uint32_t pl[kBlockPlanes];
#pragma unroll
    for (int i = 0; i < kBlockPlanes; ++i) pl[i] = 0;

    // eight rows at a time, the next eight already in flight while these are counted
    auto load8 = [&](uint32_t r0, uint32_t (&x)[8]) {
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            x[j] = 0;
            if (r0 + j < rows && in_range) {   // the row test is wave-uniform
                const uint32_t *row = hv + (int64_t)idx[r0 + j] * W;
                x[j] = __builtin_nontemporal_load(row + col);
            }
        }
    };
    auto add8 = [&](const uint32_t (&x)[8]) {
        uint32_t a, b, p, c2a, c2b, c3;
        p = pl[0]; a = maj3(p, x[0], x[1]); p = xor3(p, x[0], x[1]);
        b = maj3(p, x[2], x[3]); p = xor3(p, x[2], x[3]); pl[0] = p;
        p = pl[1]; c2a = maj3(p, a, b); pl[1] = xor3(p, a, b);
        p = pl[0]; a = maj3(p, x[4], x[5]); p = xor3(p, x[4], x[5]);
        b = maj3(p, x[6], x[7]); p = xor3(p, x[6], x[7]); pl[0] = p;
        p = pl[1]; c2b = maj3(p, a, b); pl[1] = xor3(p, a, b);
        p = pl[2]; c3 = maj3(p, c2a, c2b); pl[2] = xor3(p, c2a, c2b);
#pragma unroll
        for (int i = 3; i < kWavePlanes; ++i) {
            const uint32_t t = pl[i] & c3;
            pl[i] ^= c3;
            c3 = t;
        }
    };
    // All waves of the block make the same number of trips (those of row group 0, which has the
    // most rows; a wave past its own rows loads nothing and adds zeros) and meet at a barrier
    // every trip.  Without it the waves that read neighbouring slices of the same rows drift
    // apart by more rows than the L2 keeps, and every cache line that straddles two slices
    // (rows are not multiples of the line size) is fetched from HBM twice: measured, 27 % more
    // bytes fetched than the rows hold.
    const uint32_t first0 = (item - blk[c]) * (uint32_t)(rg * rb);
    const uint32_t trips_rows = first0 < total ? min((uint32_t)rb, total - first0) : 0u;   // block-uniform
    uint32_t xa[8], xb[8];
    load8(0, xa);
    for (uint32_t r0 = 0; r0 < trips_rows; r0 += 16) {
        __syncthreads();
        load8(r0 + 8, xb);
        add8(xa);
        load8(r0 + 16, xa);
        add8(xb);
    }

    // add the row groups' counts: groups 1.. park their planes in LDS, group 0 sums and flushes
    if (group > 0) {
        uint32_t *dst = merge + (size_t)((group - 1) * spb + sl) * (kWavePlanes * kWave) + lane;
#pragma unroll
        for (int i = 0; i < kWavePlanes; ++i) dst[i * kWave] = pl[i];
    }
    __syncthreads();
    if (group != 0) return;
    if (col >= Wp) return;   // (wave-uniform: the last chunk of slices may reach past the row, and a partial row has Wp columns)
    for (int g = 0; g < rg - 1; ++g) {
        const uint32_t *src = merge + (size_t)(g * spb + sl) * (kWavePlanes * kWave) + lane;
        uint32_t carry = 0;
#pragma unroll
        for (int i = 0; i < kWavePlanes; ++i) {
            const uint32_t a = pl[i], b = src[i * kWave];
            pl[i] = xor3(a, b, carry);
            carry = maj3(a, b, carry);
        }
        pl[kWavePlanes] ^= carry;   // top plane: the block total stays below 2^12
    }
    // this lane's 32 counts as 16 dwords of two 16-bit sums each (pad columns store zeros)
    uint4 *dst = reinterpret_cast<uint4 *>(partial + ((size_t)item * Wp + col) * 16);
#pragma unroll
    for (int q4 = 0; q4 < 4; ++q4) {
        uint32_t w[4];
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            const int b0 = (q4 * 4 + k) * 2;
            uint32_t v = 0;
#pragma unroll
            for (int i = 0; i < kBlockPlanes; ++i)
                v |= (((pl[i] >> b0) & 1u) << i) | (((pl[i] >> (b0 + 1)) & 1u) << (16 + i));
            w[k] = v;
        }
        dst[q4] = make_uint4(w[0], w[1], w[2], w[3]);
    }
}

// ---- vertical count, a wave per row (rows of up to 320 words) -----------------------------------
// grid.x = work item as above.  The block's 16 waves take a sixteenth of the item's rows each, a
// contiguous run; a wave reads whole rows, a lane KPL words of each (word_of below), eight
// rows at a time (count_rows), and keeps a set of count planes per word position; the waves
// never wait for one another: no barrier in the stream.  A wave counts at most 248 rows (eight
// planes); the waves' counts meet in LDS in two rounds (waves 8..15 into 0..7, then 1..7
// into 0), and the block total, twelve planes, goes back through LDS so that KPL waves turn a
// position each into 16-bit sums.  Dynamic LDS: 8 x KPL x 9 planes of 64 words.
constexpr int kRowsWaves = 16;
constexpr int kRowsPlanes = 8;                      // a wave counts at most 255 rows ...
constexpr int kRowsPerWaveMax = 248;                // ... in steps of 8

// eight words into a position's count planes (carry-save: seven full adders, then a ripple from plane 3)
__device__ __forceinline__ void count8(uint32_t *q, const uint32_t *x) {
    uint32_t a, b, p, c2a, c2b, c3;
    p = q[0]; a = maj3(p, x[0], x[1]); p = xor3(p, x[0], x[1]);
    b = maj3(p, x[2], x[3]); p = xor3(p, x[2], x[3]); q[0] = p;
    p = q[1]; c2a = maj3(p, a, b); q[1] = xor3(p, a, b);
    p = q[0]; a = maj3(p, x[4], x[5]); p = xor3(p, x[4], x[5]);
    b = maj3(p, x[6], x[7]); p = xor3(p, x[6], x[7]); q[0] = p;
    p = q[1]; c2b = maj3(p, a, b); q[1] = xor3(p, a, b);
    p = q[2]; c3 = maj3(p, c2a, c2b); q[2] = xor3(p, c2a, c2b);
#pragma unroll
    for (int i = 3; i < kRowsPlanes; ++i) {
        const uint32_t t = q[i] & c3;
        q[i] ^= c3;
        c3 = t;
    }
}

// Which words of a row a lane holds, position k = 0 .. KPL - 1.  Plain: word k * 64 + lane.
// Quad (rows of 257 to 320 words): words 4 * lane + k for k < 4, which one 16-byte load
// brings, and word 256 + lane for k = 4.
template <bool QUAD>
__device__ __forceinline__ int word_of(const int k, const int lane) {
    return QUAD ? (k < 4 ? 4 * lane + k : 4 * kWave + lane) : k * kWave + lane;
}
typedef uint32_t u32x4_a4 __attribute__((ext_vector_type(4), aligned(4)));   // (rows start at any word)

// A wave counts `nrows` rows into its planes, eight rows at a time.  rows8(r0, last, row) gives
// the addresses of rows r0 .. r0 + 7 of the wave's run, none past `last` (wave-uniform
// values).  A batch is asked for in one burst, row after row, so that the memory sees a row's
// pieces together, and counted as it comes in; while the burst is under way the next batch's
// addresses are worked out.  The wave's own loads and counting overlap little; those of the
// block's other 15 waves do.  (Measured on 1M rows of 313 words: asking for the next batch
// slice by slice while this one is counted, 32 to 38 loads always in flight, was 10 % slower
// than the burst; a burst that goes through the batch position by position, eight rows'
// first 256 bytes, then their second, 8 % slower than row by row; 16-byte loads 2.5 % faster
// than 4-byte ones.)  Nothing is conditional about the loads and no loaded word is used before
// its turn to be counted (either would make the wave wait for every load at once): the up to
// seven rows left over come as one more batch of eight, the surplus a repeat of the last row,
// masked.  Lanes past the end of a row read its last word; the caller drops their counts.
template <int KPL, bool QUAD, typename Rows8>
__device__ __forceinline__ void count_rows(uint32_t (&pl)[KPL][kRowsPlanes], const uint32_t nrows, const int lane,
                                           const int W, Rows8 rows8) {
    static_assert(!QUAD || KPL == 5, "the quad layout is for rows of 257 to 320 words");
    int at[KPL];
#pragma unroll
    for (int k = 0; k < KPL; ++k) at[k] = min(word_of<QUAD>(k, lane), W - 1);
    uint32_t x[KPL][8];
    const uint32_t *row[8];
    auto ask = [&]() {
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            if constexpr (QUAD) {
                const u32x4_a4 q = __builtin_nontemporal_load(reinterpret_cast<const u32x4_a4 *>(row[j] + 4 * lane));
                x[0][j] = q.x, x[1][j] = q.y, x[2][j] = q.z, x[3][j] = q.w;
                x[4][j] = __builtin_nontemporal_load(row[j] + at[4]);
            } else {
#pragma unroll
                for (int k = 0; k < KPL; ++k) x[k][j] = __builtin_nontemporal_load(row[j] + at[k]);
            }
        }
    };
    const uint32_t full = nrows & ~7u;
    if (full > 0) rows8(0u, full - 1, row);
    for (uint32_t r0 = 0; r0 < full; r0 += 8) {
        ask();
        __builtin_amdgcn_sched_barrier(0);
        rows8(min(r0 + 8, full - 8), full - 1, row);   // (after the last batch: the same again, unused)
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int k = 0; k < KPL; ++k) count8(pl[k], x[k]);
    }
    if (nrows > full) {   // wave-uniform
        rows8(full, nrows - 1, row);
        ask();
#pragma unroll
        for (int k = 0; k < KPL; ++k) {
#pragma unroll
            for (int j = 0; j < 8; ++j) x[k][j] = full + j < nrows ? x[k][j] : 0u;
            count8(pl[k], x[k]);
        }
    }
}

// x[b] bit p  ->  x[p] bit b (32 x 32 bits per lane): halves and bytes trade places by byte
// permutes, the finer stages by masked merges.  Registers known to be zero cost nothing.
__device__ __forceinline__ void transpose32(uint32_t (&x)[32]) {
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
}

// The 16 waves' counts (eight planes per lane and word position; pl's ninth plane comes in zero)
// meet in LDS: waves 8..15 park theirs and waves 0..7 add them to their own (nine planes), park
// the sums in the same slots, and then wave k adds up position k of the eight slots - and of
// `extra`, one more count of at most 248 parked elsewhere in LDS in the same layout (block-
// uniform, may be null) - into the block total, twelve planes, turns the planes into 32 counts
// by a bit transposition and writes them as 16-bit sums, 32 dimensions per lane as 16 dwords
// (pad columns store zeros), at dst + word_of(k, lane) * 16.  All threads of the block call it;
// two barriers inside, and the caller keeps the slots untouched until every wave is through
// (a barrier, or the kernel's end).  merge: 8 slots of KPL x 9 planes of 64 words.  (Adding the
// eight sums up in wave 0 alone, every position, and turning planes into sums bit by bit took
// 14 us per call and block; this form about 4.)
template <int KPL, bool QUAD>
__device__ __forceinline__ void merge_and_store(uint32_t (&pl)[KPL][9], uint32_t *merge, const int wave,
                                                const int lane, const int Wp, uint32_t *dst_row,
                                                const uint32_t *extra = nullptr) {
    constexpr int kSlot = KPL * 9 * kWave;
    if (wave >= 8) {
        uint32_t *dst = merge + (size_t)(wave - 8) * kSlot + lane;
#pragma unroll
        for (int k = 0; k < KPL; ++k)
#pragma unroll
            for (int i = 0; i < kRowsPlanes; ++i) dst[(k * 9 + i) * kWave] = pl[k][i];
    }
    __syncthreads();
    if (wave < 8) {   // at most 496 rows: nine planes, back into the slot they came from
        uint32_t *slot = merge + (size_t)wave * kSlot + lane;
#pragma unroll
        for (int k = 0; k < KPL; ++k) {
            uint32_t carry = 0;
#pragma unroll
            for (int i = 0; i < kRowsPlanes; ++i) {
                const uint32_t a = pl[k][i], b = slot[(k * 9 + i) * kWave];
                slot[(k * 9 + i) * kWave] = xor3(a, b, carry);
                carry = maj3(a, b, carry);
            }
            slot[(k * 9 + kRowsPlanes) * kWave] = carry;
        }
    }
    __syncthreads();
    if (wave >= KPL) return;
    const int col = word_of<QUAD>(wave, lane);
    uint32_t x[32];
#pragma unroll
    for (int i = 0; i < 32; ++i) x[i] = 0;
    auto add = [&](const uint32_t *from, const int planes) {   // x += position `wave` of a parked count
        const uint32_t *src = from + (size_t)(wave * 9) * kWave + lane;
        uint32_t carry = 0;
#pragma unroll
        for (int i = 0; i < 12; ++i) {
            const uint32_t a = x[i], b = i < planes ? src[i * kWave] : 0u;
            x[i] = xor3(a, b, carry);
            carry = maj3(a, b, carry);
        }
    };
#pragma unroll
    for (int w = 0; w < 8; ++w) add(merge + (size_t)w * kSlot, 9);
    if (extra) add(extra, kRowsPlanes);   // (the block total stays below 2^12)
    if (col >= Wp) return;
    transpose32(x);   // x[p] = the count of the word's dimension p
    uint4 *dst = reinterpret_cast<uint4 *>(dst_row + (size_t)col * 16);
#pragma unroll
    for (int q4 = 0; q4 < 4; ++q4)
        dst[q4] = make_uint4(x[8 * q4] | (x[8 * q4 + 1] << 16), x[8 * q4 + 2] | (x[8 * q4 + 3] << 16),
                             x[8 * q4 + 4] | (x[8 * q4 + 5] << 16), x[8 * q4 + 6] | (x[8 * q4 + 7] << 16));
}

template <int KPL, bool QUAD>
__global__ __launch_bounds__(kRowsWaves *kWave) void accumulate_rows_kernel(
    const uint32_t *__restrict__ hv, const uint32_t *__restrict__ perm, const uint32_t *__restrict__ cnt,
    const uint32_t *__restrict__ off, const uint32_t *__restrict__ blk, int C, int W, int Wp, int rpw,
    uint32_t *__restrict__ partial) {
    extern __shared__ uint32_t merge[];
    const uint32_t item = blockIdx.x;
    if (item >= blk[C]) return;
    int lo = 0, hi = C - 1;   // class of this work item: last c with blk[c] <= item (blk is non-decreasing)
    while (lo < hi) {
        const int mid = (lo + hi + 1) >> 1;
        if (blk[mid] <= item) lo = mid; else hi = mid - 1;
    }
    const int c = lo;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int lane = threadIdx.x & (kWave - 1);
    const uint32_t first = __builtin_amdgcn_readfirstlane((item - blk[c]) * (uint32_t)(kRowsWaves * rpw) + (uint32_t)(wave * rpw));
    const uint32_t total = __builtin_amdgcn_readfirstlane(cnt[c]);
    // (wave-uniform, and said so: the row numbers below then come by scalar loads)
    const uint32_t rows = __builtin_amdgcn_readfirstlane(first < total ? min((uint32_t)rpw, total - first) : 0u);
    const_u32_ptr idx = (const_u32_ptr)(uintptr_t)(perm + __builtin_amdgcn_readfirstlane(off[c]) + first);

    uint32_t pl[KPL][kRowsPlanes];
#pragma unroll
    for (int k = 0; k < KPL; ++k)
#pragma unroll
        for (int i = 0; i < kRowsPlanes; ++i) pl[k][i] = 0;
    count_rows<KPL, QUAD>(pl, rows, lane, W, [&](const uint32_t r0, const uint32_t last, const uint32_t *(&row)[8]) {
#pragma unroll
        for (int j = 0; j < 8; ++j) row[j] = hv + (int64_t)idx[min(r0 + (uint32_t)j, last)] * W;
    });
    uint32_t t[KPL][9];
#pragma unroll
    for (int k = 0; k < KPL; ++k)
#pragma unroll
        for (int i = 0; i < 9; ++i) t[k][i] = (i < kRowsPlanes && word_of<QUAD>(k, lane) < W) ? pl[k][i] : 0u;
    merge_and_store<KPL, QUAD>(t, merge, wave, lane, Wp, partial + (size_t)item * Wp * 16);
}

// ---- vertical count of a few classes without grouping the rows first ----------------------------
// Up to kLocalMaxC classes.  grid.x = blocks of 16 * rpw consecutive rows (rpw at most 248).  The
// block orders its rows by class by itself: a wave reads the labels of its rpw rows, a lane four
// of them, and counts the classes with ballots; after a barrier every wave knows where its rows
// of each class go in the block's list (LDS, 16-bit row offsets, class after class) and writes
// them there.  Then the list is dealt out again, rpw entries per wave, so that a wave's run
// holds one class except where a class ends inside it: the wave counts a class's stretch as
// accumulate_rows_kernel does (the batch's eight row numbers come from the list with one LDS
// read and eight readlanes) and, where more of its run follows, parks that count in the class's
// own LDS slot (a class ends in one wave only) and starts again.  No wave waits for another
// until all have streamed.  The classes are then merged one after the other, a wave giving
// the count it still holds to its class and zeros to the others, the parked count going in
// as a seventeenth; the class's partial row is item c * gridDim.x + block.  Rows whose label
// is outside [0, C) are on no list.  Saved against grouped rows: the grouping launch and the
// trip of the row numbers through memory.
// labels == nullptr: every row is of class 0 (the vertical sum on its own).  Block 0 writes the
// work list of the reduction (blk[c] = c * gridDim.x); class_n[c] grows by the block's rows of c.
// Dynamic LDS: (8 + C - 1) x KPL x 9 planes of 64 words.
constexpr int kLocalMaxC = 4;
template <int KPL, bool QUAD>
__global__ __launch_bounds__(kRowsWaves *kWave) void accumulate_local_kernel(
    const uint32_t *__restrict__ hv, const int32_t *__restrict__ labels, uint32_t n, int C, int W, int Wp, int rpw,
    uint32_t *__restrict__ partial, uint32_t *__restrict__ blk, unsigned long long *class_n, int stride) {
    // (W, Wp: the words this launch counts, which start at hv; stride: the words from a row to the next)
    extern __shared__ uint32_t merge[];
    __shared__ uint16_t list_s[kRowsWaves * 256];
    __shared__ uint32_t wc_s[kRowsWaves][kLocalMaxC], used_s[kLocalMaxC];
    constexpr int kSlotWords = KPL * 9 * kWave;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int lane = threadIdx.x & (kWave - 1);
    const uint32_t block_first = blockIdx.x * (uint32_t)(kRowsWaves * rpw);
    const uint32_t first = __builtin_amdgcn_readfirstlane(block_first + (uint32_t)(wave * rpw));
    const uint32_t rows = __builtin_amdgcn_readfirstlane(first < n ? min((uint32_t)rpw, n - first) : 0u);
    if (blockIdx.x == 0 && threadIdx.x <= (unsigned)C) blk[threadIdx.x] = threadIdx.x * gridDim.x;
    if (threadIdx.x < kLocalMaxC) used_s[threadIdx.x] = 0;
    int32_t y[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const uint32_t r = (uint32_t)(j * kWave + lane);
        y[j] = r < rows ? (labels ? labels[(size_t)first + r] : 0) : -1;
    }
    for (int c = 0; c < C; ++c) {
        uint32_t k = 0;
#pragma unroll
        for (int j = 0; j < 4; ++j) k += (uint32_t)__popcll(__ballot(y[j] == c));
        if (lane == 0) wc_s[wave][c] = k;
    }
    __syncthreads();
    uint32_t bnd[kLocalMaxC + 1];   // where the classes start in the block's list (block-uniform)
    bnd[0] = 0;
    {
        const uint64_t below = ((uint64_t)1 << lane) - 1;
#pragma unroll
        for (int c = 0; c < kLocalMaxC; ++c) {
            uint32_t before = 0, total = 0;
            if (c < C) {
                for (int w = 0; w < kRowsWaves; ++w) {
                    const uint32_t k = wc_s[w][c];
                    before += w < wave ? k : 0u;
                    total += k;
                }
                uint32_t at = bnd[c] + before;
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const uint64_t m = __ballot(y[j] == c);
                    if (y[j] == c) list_s[at + (uint32_t)__popcll(m & below)] = (uint16_t)(wave * rpw + j * kWave + lane);
                    at += (uint32_t)__popcll(m);
                }
                if (class_n && threadIdx.x == 0 && total) atomicAdd(class_n + c, (unsigned long long)total);
            }
            bnd[c + 1] = __builtin_amdgcn_readfirstlane(bnd[c] + total);
        }
    }
    __syncthreads();
    uint32_t mine[KPL];   // (a lane past the row's end read the last word again: its counts are dropped)
#pragma unroll
    for (int k = 0; k < KPL; ++k) mine[k] = word_of<QUAD>(k, lane) < W ? 0xffffffffu : 0u;
    uint32_t pl[KPL][kRowsPlanes];
#pragma unroll
    for (int k = 0; k < KPL; ++k)
#pragma unroll
        for (int i = 0; i < kRowsPlanes; ++i) pl[k][i] = 0;
    int mine_c = -1;     // the class of the count the wave holds at the end
    const uint32_t run0 = (uint32_t)(wave * rpw), run1 = min(run0 + (uint32_t)rpw, bnd[kLocalMaxC]);
#pragma unroll
    for (int c = 0; c < kLocalMaxC; ++c) {
        const uint32_t s0 = max(run0, bnd[c]), s1 = min(run1, bnd[c + 1]);
        if (c >= C || s0 >= s1) continue;   // wave-uniform
        const uint16_t *lst = list_s + s0;
        count_rows<KPL, QUAD>(pl, s1 - s0, lane, W, [&](const uint32_t r0, const uint32_t last, const uint32_t *(&row)[8]) {
            const uint32_t v = lst[min(r0 + (uint32_t)(lane & 7), last)];   // one LDS read, eight readlanes
#pragma unroll
            for (int j = 0; j < 8; ++j)
                row[j] = hv + (int64_t)(block_first + (uint32_t)__builtin_amdgcn_readlane((int)v, j)) * stride;
        });
        if (run1 > bnd[c + 1]) {   // more of the run follows: this class's count waits in its slot
            uint32_t *dst = merge + (size_t)(8 + c) * kSlotWords + lane;
#pragma unroll
            for (int k = 0; k < KPL; ++k)
#pragma unroll
                for (int i = 0; i < kRowsPlanes; ++i) {
                    dst[(k * 9 + i) * kWave] = pl[k][i] & mine[k];
                    pl[k][i] = 0;
                }
            if (lane == 0) used_s[c] = 1;
        } else {
            mine_c = c;
        }
    }
    __syncthreads();
    for (int c = 0; c < C; ++c) {
        uint32_t t[KPL][9];
#pragma unroll
        for (int k = 0; k < KPL; ++k)
#pragma unroll
            for (int i = 0; i < 9; ++i) t[k][i] = (i < kRowsPlanes && mine_c == c) ? (pl[k][i] & mine[k]) : 0u;
        const uint32_t *extra = used_s[c] ? merge + (size_t)(8 + c) * kSlotWords : nullptr;
        merge_and_store<KPL, QUAD>(t, merge, wave, lane, Wp, partial + ((size_t)c * gridDim.x + blockIdx.x) * Wp * 16, extra);
        __syncthreads();   // (the totals in LDS have been read before the next class parks there)
    }
}

// ---- small batches: grouping, counting and the update of acc in one launch ----------------------
// Up to kFusedMaxN rows.  grid = (C, slices of 64 word columns), 16 waves per block.  A block takes
// class c and one slice: it lists the rows of the class in LDS by itself (every block reads the few
// thousand labels; a wave appends its matches with one LDS atomic), its 16 waves count a sixteenth
// of those rows each with the same bit-sliced adders as accumulate_kernel (a couple of 8-row
// batches per wave), the 16 counts are added pairwise through LDS in four rounds, and all waves
// together turn the planes into integers and add them to acc[c][the slice's 2048 dimensions],
// which this block alone owns (coalesced 8-byte read-modify-writes, the old values fetched at the
// start).  Three launches and two scratch round trips less than the general path; fourteen
// planes hold any count up to the row limit, whatever the class sizes.
constexpr int kFusedMaxN = 8192;
constexpr int kFusedPlanes = 14;
static_assert(kFusedMaxN < (1 << kFusedPlanes), "a class may hold every row");
constexpr size_t kFusedSlotWords = (size_t)kAccWaves * kFusedPlanes * kWave;   // one plane set per wave

__global__ __launch_bounds__(kAccWaves *kWave) void accumulate_small_kernel(
    const uint32_t *__restrict__ hv, const int32_t *__restrict__ labels, int N, int W, int D, int32_t *acc,
    int64_t *class_n) {
    extern __shared__ uint32_t sm[];   // plane sets [16][kFusedPlanes][64], then the row list (u16)
    __shared__ uint32_t count;
    uint16_t *list = reinterpret_cast<uint16_t *>(sm + kFusedSlotWords);
    const int c = blockIdx.x;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int lane = threadIdx.x & (kWave - 1);
    if (threadIdx.x == 0) count = 0;
    __syncthreads();
    {   // a thread's labels all at once (the loads are independent), then the appends
        constexpr int kPer = kFusedMaxN / (kAccWaves * kWave);
        int lab[kPer];
#pragma unroll
        for (int k = 0; k < kPer; ++k) {
            const int i = threadIdx.x + k * kAccWaves * kWave;
            lab[k] = i < N ? labels[i] : -1;
        }
#pragma unroll
        for (int k = 0; k < kPer; ++k) {
            const bool hit = lab[k] == c;
            const uint64_t m = __ballot(hit);
            if (m) {   // uniform: one atomic per wave reserves room for its matches (any order: integer sums)
                uint32_t base = 0;
                if (lane == 0) base = atomicAdd(&count, (uint32_t)__popcll(m));
                base = __builtin_amdgcn_readfirstlane(base);
                const uint32_t rank = __builtin_amdgcn_mbcnt_hi((uint32_t)(m >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)m, 0u));
                if (hit) list[base + rank] = (uint16_t)(threadIdx.x + k * kAccWaves * kWave);
            }
        }
    }
    __syncthreads();
    const uint32_t total = count;
    if (total == 0) return;   // uniform
    if (blockIdx.y == 0 && threadIdx.x == 0) class_n[c] += (int64_t)total;

    // the two accumulators this lane will add to at the end, on their way while the rows are counted:
    // wave g finishes word columns 4g .. 4g+3 of the slice, lane l bits 2 (l % 16), +1 of column l / 16
    const int fcol = blockIdx.y * kSliceWords + wave * 4 + (lane >> 4);
    const int fbit = (lane & 15) * 2;
    const int64_t fd = (int64_t)fcol * 32 + fbit;
    int32_t *fdst = acc + (int64_t)c * D + fd;
    const bool pair = (D & 1) == 0 && (reinterpret_cast<uintptr_t>(acc) & 7u) == 0 && fd + 1 < D;
    int2 old2 = make_int2(0, 0);
    if (pair) {
        old2 = *reinterpret_cast<const int2 *>(fdst);
    } else {
        if (fd < D) old2.x = fdst[0];
        if (fd + 1 < D) old2.y = fdst[1];
    }

    const int col = blockIdx.y * kSliceWords + lane;
    const bool in_range = col < W;
    const uint32_t rb = ((total + kAccWaves - 1) / kAccWaves + 7) / 8 * 8;
    const uint32_t first = (uint32_t)wave * rb;
    const uint32_t rows = first < total ? min(rb, total - first) : 0u;

    uint32_t pl[kFusedPlanes];
#pragma unroll
    for (int i = 0; i < kFusedPlanes; ++i) pl[i] = 0;
    auto load8 = [&](uint32_t r0, uint32_t(&x)[8]) {
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            x[j] = 0;
            if (r0 + j < rows && in_range) x[j] = hv[(int64_t)list[first + r0 + j] * W + col];   // row test: uniform
        }
    };
    auto add8 = [&](const uint32_t(&x)[8]) {
        uint32_t a, b, p, c2a, c2b, c3;
        p = pl[0]; a = maj3(p, x[0], x[1]); p = xor3(p, x[0], x[1]);
        b = maj3(p, x[2], x[3]); p = xor3(p, x[2], x[3]); pl[0] = p;
        p = pl[1]; c2a = maj3(p, a, b); pl[1] = xor3(p, a, b);
        p = pl[0]; a = maj3(p, x[4], x[5]); p = xor3(p, x[4], x[5]);
        b = maj3(p, x[6], x[7]); p = xor3(p, x[6], x[7]); pl[0] = p;
        p = pl[1]; c2b = maj3(p, a, b); pl[1] = xor3(p, a, b);
        p = pl[2]; c3 = maj3(p, c2a, c2b); pl[2] = xor3(p, c2a, c2b);
#pragma unroll
        for (int i = 3; i < kFusedPlanes; ++i) {
            const uint32_t t = pl[i] & c3;
            pl[i] ^= c3;
            c3 = t;
        }
    };
    uint32_t xa[8], xb[8];
    load8(0, xa);
    for (uint32_t r0 = 0; r0 < rows; r0 += 16) {
        load8(r0 + 8, xb);
        add8(xa);
        load8(r0 + 16, xa);
        add8(xb);
    }

    // 16 plane sets -> 1: the upper half of the waves still in play parks its planes, the lower
    // half adds them (ripple-carry adders on the planes; the class total fits, so the last carry
    // is zero).  Every wave has a set of its own in LDS, so one barrier per round is enough.
    uint32_t *mine = sm + (size_t)wave * kFusedPlanes * kWave + lane;
#pragma unroll
    for (int stride = kAccWaves / 2; stride >= 1; stride >>= 1) {
        if (wave >= stride && wave < 2 * stride) {
#pragma unroll
            for (int i = 0; i < kFusedPlanes; ++i) mine[i * kWave] = pl[i];
        }
        __syncthreads();
        if (wave < stride) {
            const uint32_t *src = mine + (size_t)stride * kFusedPlanes * kWave;
            uint32_t carry = 0;
#pragma unroll
            for (int i = 0; i < kFusedPlanes; ++i) {
                const uint32_t a = pl[i], b = src[i * kWave];
                pl[i] = xor3(a, b, carry);
                carry = maj3(a, b, carry);
            }
        }
    }
    if (wave == 0) {
#pragma unroll
        for (int i = 0; i < kFusedPlanes; ++i) mine[i * kWave] = pl[i];
    }
    __syncthreads();
    // all waves: planes of set 0 -> two integers per lane -> acc
    uint32_t v0 = 0, v1 = 0;
    const uint32_t *fin = sm + (wave * 4 + (lane >> 4));
#pragma unroll
    for (int i = 0; i < kFusedPlanes; ++i) {
        const uint32_t p = fin[i * kWave] >> fbit;
        v0 |= (p & 1u) << i;
        v1 |= ((p >> 1) & 1u) << i;
    }
    if (pair) {
        *reinterpret_cast<int2 *>(fdst) = make_int2(old2.x + (int)v0, old2.y + (int)v1);
    } else {
        if (fd < D) fdst[0] = old2.x + (int)v0;
        if (fd + 1 < D) fdst[1] = old2.y + (int)v1;
    }
}

// acc[c][d] += sum over the class's partial rows.  grid = (dimension pairs / 256, C, K): the
// K parts of a class's item range are combined with atomics only when K > 1.
__global__ __launch_bounds__(256) void reduce_partials_kernel(const uint32_t *__restrict__ partial,
                                                               const uint32_t *__restrict__ blk, int Wp,
                                                               int D, int K, int32_t *acc, int d0) {
    const int c = blockIdx.y;
    const int pair = blockIdx.x * 256 + threadIdx.x;   // dims 2*pair, 2*pair + 1
    if (pair >= Wp * 16) return;
    const uint32_t i0 = blk[c], i1 = blk[c + 1];
    const uint32_t per = (i1 - i0 + K - 1) / K;
    const uint32_t a = min(i0 + blockIdx.z * per, i1), b = min(a + per, i1);
    uint32_t s0 = 0, s1 = 0;
    const uint32_t *src = partial + (size_t)a * Wp * 16 + pair;
    const size_t step = (size_t)Wp * 16;
    uint32_t it = a;
    for (; it + 4 <= b; it += 4, src += 4 * step) {   // four independent loads in flight
        const uint32_t v0 = src[0], v1 = src[step], v2 = src[2 * step], v3 = src[3 * step];
        s0 += (v0 & 0xffffu) + (v1 & 0xffffu) + (v2 & 0xffffu) + (v3 & 0xffffu);
        s1 += (v0 >> 16) + (v1 >> 16) + (v2 >> 16) + (v3 >> 16);
    }
    for (; it < b; ++it, src += step) {
        const uint32_t v = *src;
        s0 += v & 0xffffu;
        s1 += v >> 16;
    }
    const int d = d0 + pair * 2;   // (d0: the first dimension of the partial rows, even)
    int32_t *dst = acc + (int64_t)c * D + d;
    if (K == 1) {
        if (d < D && s0) dst[0] += (int32_t)s0;
        if (d + 1 < D && s1) dst[1] += (int32_t)s1;
    } else {
        if (d < D && s0) atomicAdd(&dst[0], (int32_t)s0);
        if (d + 1 < D && s1) atomicAdd(&dst[1], (int32_t)s1);
    }
}

// Shape of the accumulate launch: slices per block, row groups per block, how many blocks the
// chip holds at once, and for a chunk of n rows the rows per wave.  Rows per wave are chosen so
// that the whole chunk is ONE round of blocks (a second, nearly empty round would double the
// time), capped so that a block's count fits its planes, and a multiple of the 8-row step.
struct AccPlan {
    bool rows;        // rows of at most 320 words: the wave-per-row kernel (rg = its 16 waves, rb = rows per wave)
    int spb, rg, ychunks;
    int64_t cap;      // blocks per launch that run at once, minus the C possible partial blocks
    int64_t rb_max;   // most rows per wave
    int64_t rows_max; // most rows one launch takes in a single round
};
constexpr int kRowsMaxKpl = 5;   // word positions per lane the wave-per-row kernel is built for (its registers)
// Rows up to here go through accumulate_local, the wider ones of them in two column slices.  More
// slices lose to the slice-per-wave kernel: every pass opens the same memory pages again for a
// shorter piece of each row (1 M-row-equivalents at C = 2: D = 20000 333 -> 247 us, 16384 233 -> 220,
// 14000 274 -> 253; three slices at D = 28000 263 -> 274, four at 32768 251 -> 266).
constexpr int kLocalMaxWords = 2 * kRowsMaxKpl * kSliceWords;
static size_t rows_lds(int kpl) { return (size_t)8 * kpl * 9 * kWave * sizeof(uint32_t); }
// (the 16-byte layout where the rows have 257 to 320 words)
static const void *rows_kernel(int kpl, int W) {
    switch (kpl) {
    case 1: return reinterpret_cast<const void *>(accumulate_rows_kernel<1, false>);
    case 2: return reinterpret_cast<const void *>(accumulate_rows_kernel<2, false>);
    case 3: return reinterpret_cast<const void *>(accumulate_rows_kernel<3, false>);
    case 4: return reinterpret_cast<const void *>(accumulate_rows_kernel<4, false>);
    default: return W > 4 * kWave ? reinterpret_cast<const void *>(accumulate_rows_kernel<5, true>)
                                  : reinterpret_cast<const void *>(accumulate_rows_kernel<5, false>);
    }
}
static const void *local_kernel(int kpl, int W) {
    switch (kpl) {
    case 1: return reinterpret_cast<const void *>(accumulate_local_kernel<1, false>);
    case 2: return reinterpret_cast<const void *>(accumulate_local_kernel<2, false>);
    case 3: return reinterpret_cast<const void *>(accumulate_local_kernel<3, false>);
    case 4: return reinterpret_cast<const void *>(accumulate_local_kernel<4, false>);
    default: return W > 4 * kWave ? reinterpret_cast<const void *>(accumulate_local_kernel<5, true>)
                                  : reinterpret_cast<const void *>(accumulate_local_kernel<5, false>);
    }
}
static int plan_static(hdc_ctx_impl *c, AccPlan *p) {
    const int nslices = c->Wp / kSliceWords;
    p->rows = nslices <= kRowsMaxKpl;
    if (p->rows) {
        p->spb = 1, p->rg = kRowsWaves, p->ychunks = 1;
        int bpc = c->acc_bpc;
        if (bpc == 0) {
            if (rows_lds(nslices) > 64 * 1024)
                HDC_HIP(hipFuncSetAttribute(rows_kernel(nslices, c->W), hipFuncAttributeMaxDynamicSharedMemorySize, (int)rows_lds(nslices)));
            HDC_HIP(hipOccupancyMaxActiveBlocksPerMultiprocessor(&bpc, rows_kernel(nslices, c->W), kRowsWaves * kWave, rows_lds(nslices)));
            if (bpc < 1) bpc = 1;
            c->acc_bpc = bpc;
        }
        p->cap = (int64_t)c->num_cus * bpc - c->p.C;
        if (p->cap < 1) p->cap = 1;
        p->rb_max = kRowsPerWaveMax;
        p->rows_max = c->perm_rows;   // (any number of whole rounds of blocks in one launch, see plan_rb)
        return HDC_OK;
    }
    p->spb = nslices < kAccWaves ? nslices : kAccWaves;
    p->rg = kAccWaves / p->spb;
    p->ychunks = (nslices + p->spb - 1) / p->spb;
    int bpc = c->acc_bpc;
    if (bpc == 0) {   // asked once per context: the block shape depends on D alone
        const size_t lds = (size_t)(p->rg - 1) * p->spb * kWavePlanes * kWave * sizeof(uint32_t);
        HDC_HIP(hipOccupancyMaxActiveBlocksPerMultiprocessor(
            &bpc, reinterpret_cast<const void *>(accumulate_kernel), p->spb * p->rg * kWave, lds));
        if (bpc < 1) bpc = 1;
        c->acc_bpc = bpc;
    }
    p->cap = (int64_t)c->num_cus * bpc / p->ychunks - c->p.C;
    if (p->cap < 1) p->cap = 1;
    p->rb_max = (4088 / p->rg) / 8 * 8;
    if (p->rb_max > 2040) p->rb_max = 2040;
    p->rows_max = p->cap * p->rg * p->rb_max;
    if (p->rows_max > c->perm_rows) p->rows_max = c->perm_rows;
    return HDC_OK;
}
static int64_t plan_rb(const AccPlan &p, int64_t n) {
    // The wave-per-row kernel takes more rows than one round of full blocks holds as several
    // rounds of equal, smaller blocks in the same launch (a last round of a few full blocks
    // would take as long as a whole one).
    const int64_t rounds = p.rows ? (n + p.rg * p.cap * p.rb_max - 1) / (p.rg * p.cap * p.rb_max) : 1;
    int64_t rb = ((n + p.rg * p.cap * rounds - 1) / (p.rg * p.cap * rounds) + 7) / 8 * 8;
    return rb < 16 ? 16 : (rb > p.rb_max ? p.rb_max : rb);
}

int64_t classical_max_items(hdc_ctx_impl *c) {
    AccPlan p;
    if (plan_static(c, &p) != HDC_OK) return -1;
    // full blocks of one round plus at most one partial block per class, with some slack
    return p.cap + 2 * (int64_t)c->p.C + 16 + c->perm_rows / (p.rg * p.rb_max);
}

// acc += the partial rows of each class (blk in the context's scratch lists them); the rows are
// Wp words wide (0: the model's) and start at word w0 of the model's rows.
static int reduce_partials(hdc_ctx_impl *c, int classes, int32_t *acc, hipStream_t s, int Wp = 0, int w0 = 0) {
    if (Wp == 0) Wp = c->Wp;
    // enough threads for the reduction: split a class's partial rows K ways when C is small
    const int pairs = Wp * 16;
    int K = (int)((262144 + (int64_t)classes * pairs - 1) / ((int64_t)classes * pairs));
    K = K < 1 ? 1 : (K > 16 ? 16 : K);
    hipLaunchKernelGGL(reduce_partials_kernel, dim3((unsigned)((pairs + 255) / 256), (unsigned)classes, (unsigned)K),
                       dim3(256), 0, s, c->partial_d, c->cls_blk_d, Wp, c->p.D, K, acc, 32 * w0);
    HDC_HIP(hipGetLastError());
    return HDC_OK;
}

// The accumulate + reduce launches for n rows already grouped into `classes` classes (perm,
// cnt, off, blk in the context's scratch); acc [classes][D] is added to.
static int accumulate_grouped(hdc_ctx_impl *c, const AccPlan &plan, const uint32_t *hv0, int64_t n,
                              int classes, int64_t rb, int32_t *acc, hipStream_t s) {
    const int spb = plan.spb, rg = plan.rg, ychunks = plan.ychunks;
    const int rb32 = (int)rb;
    const uint32_t block_rows = (uint32_t)(rg * rb);
    const int64_t items = (n + block_rows - 1) / block_rows + classes;
    if (items > c->partial_items) return HDC_ELIMIT;   // cannot happen: sized for the worst case
    const size_t lds = (size_t)(rg - 1) * spb * kWavePlanes * kWave * sizeof(uint32_t);
    if (plan.rows) {
        const int kpl = c->Wp / kSliceWords;
        if (rows_lds(kpl) > 64 * 1024)   // (per launch: the limit belongs to the function, not to a context)
            HDC_HIP(hipFuncSetAttribute(rows_kernel(kpl, c->W), hipFuncAttributeMaxDynamicSharedMemorySize, (int)rows_lds(kpl)));
        ProfScope prof(c, HDC_K_ACCUMULATE, s);
        void *args[] = {(void *)&hv0, (void *)&c->perm_d, (void *)&c->cls_cnt_d, (void *)&c->cls_off_d, (void *)&c->cls_blk_d,
                        (void *)&classes, (void *)&c->W, (void *)&c->Wp, (void *)&rb32, (void *)&c->partial_d};
        HDC_HIP(hipLaunchKernel(rows_kernel(kpl, c->W), dim3((unsigned)items), dim3(kRowsWaves * kWave), args, rows_lds(kpl), s));
    } else {
        ProfScope prof(c, HDC_K_ACCUMULATE, s);
        hipLaunchKernelGGL(accumulate_kernel, dim3((unsigned)items, (unsigned)ychunks), dim3(spb * rg * kWave),
                           lds, s, hv0, c->perm_d, c->cls_cnt_d, c->cls_off_d, c->cls_blk_d, classes, c->W,
                           c->Wp, (int)rb, spb, rg, c->partial_d);
    }
    return reduce_partials(c, classes, acc, s);
}

// Rows of at most 320 words and at most kLocalMaxC classes: no grouping, accumulate_local_kernel
// on the rows as they lie (labels == nullptr: one class) and the reduction.  A launch takes as
// many rows as its blocks' partial rows (classes per block) fit the scratch; as in plan_rb, more
// rows than one round of full blocks holds run as equal rounds of smaller blocks.
static int accumulate_local(hdc_ctx_impl *c, const uint32_t *hv, const int32_t *labels, int64_t N,
                            int classes, int32_t *acc, int64_t *class_n, hipStream_t s) {
    // Rows of more than 320 words (up to 640: the callers see to that) are taken in two column
    // slices of equal width (a multiple of four words), a pass of the same kernel per slice: a
    // wave then reads a kilobyte or more of a row in one piece, and the labels once per slice.
    const int nsl = (c->W + kRowsMaxKpl * kSliceWords - 1) / (kRowsMaxKpl * kSliceWords);
    const int ws = nsl == 1 ? c->W : ((c->W + nsl - 1) / nsl + 3) / 4 * 4;
    const int kpl = (ws + kSliceWords - 1) / kSliceWords;
    const void *fn = local_kernel(kpl, ws);
    const size_t lds = rows_lds(kpl) / 8 * (8 + classes - 1);   // (a slot more per class that can end inside a wave's run)
    const bool raise = lds + 16 * 1024 > 64 * 1024;     // (the kernel has some static LDS of its own)
    if (raise) HDC_HIP(hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
    int &held = c->acc_local_bpc[classes > 1];   // (the LDS of a block grows with the classes: one answer for the sum on its own, one for training)
    if (held == 0) {
        int bpc = 0;
        HDC_HIP(hipOccupancyMaxActiveBlocksPerMultiprocessor(&bpc, fn, kRowsWaves * kWave, lds));
        held = bpc < 1 ? 1 : bpc;
    }
    const int64_t most = c->partial_items / classes;   // blocks a launch may have (the scratch is sized for partial rows of the model's width)
    if (most < 1) return HDC_ELIMIT;                   // cannot happen: the scratch holds a row per class and more
    int64_t cap = (int64_t)c->num_cus * held;
    if (cap > most) cap = most;
    const int64_t round_rows = cap * kRowsWaves * kRowsPerWaveMax;
    const int64_t rows_max = most / cap * round_rows;
    for (int64_t n0 = 0; n0 < N; n0 += rows_max) {
        const int64_t n = (N - n0 < rows_max) ? N - n0 : rows_max;
        const int64_t rounds = (n + round_rows - 1) / round_rows;
        int64_t rpw = ((n + kRowsWaves * cap * rounds - 1) / (kRowsWaves * cap * rounds) + 7) / 8 * 8;
        rpw = rpw < 16 ? 16 : (rpw > kRowsPerWaveMax ? kRowsPerWaveMax : rpw);
        const int64_t blocks = (n + kRowsWaves * rpw - 1) / (kRowsWaves * rpw);
        if (blocks > most) return HDC_ELIMIT;          // cannot happen: blocks <= cap * rounds <= most
        const int32_t *lab0 = labels ? labels + n0 : nullptr;
        const uint32_t n32 = (uint32_t)n;
        const int rpw32 = (int)rpw;
        for (int sl = 0; sl < nsl; ++sl) {
            const int w0 = sl * ws;
            int w_sl = c->W - w0 < ws ? c->W - w0 : ws;
            int wp_sl = (w_sl + kSliceWords - 1) / kSliceWords * kSliceWords;
            const uint32_t *hv0 = hv + (size_t)n0 * c->W + w0;
            unsigned long long *cn = sl == 0 ? reinterpret_cast<unsigned long long *>(class_n) : nullptr;   // (the rows are counted once)
            {
                ProfScope prof(c, HDC_K_ACCUMULATE, s);
                void *args[] = {(void *)&hv0, (void *)&lab0, (void *)&n32, (void *)&classes, (void *)&w_sl, (void *)&wp_sl,
                                (void *)&rpw32, (void *)&c->partial_d, (void *)&c->cls_blk_d, (void *)&cn, (void *)&c->W};
                HDC_HIP(hipLaunchKernel(fn, dim3((unsigned)blocks), dim3(kRowsWaves * kWave), args, lds, s));
            }
            const int rc = reduce_partials(c, classes, acc, s, wp_sl, w0);
            if (rc != HDC_OK) return rc;
        }
    }
    return HDC_OK;
}

int launch_train_classical(hdc_ctx_impl *c, const uint32_t *hv, const int32_t *labels, int64_t N,
                           int32_t *acc, int64_t *class_n, hipStream_t s) {
    const int C = c->p.C;
    AccPlan plan;
    const int prc = plan_static(c, &plan);
    if (prc != HDC_OK) return prc;
    if (N <= kFusedMaxN) {
        const size_t lds = kFusedSlotWords * sizeof(uint32_t) + (size_t)(N + 1) / 2 * 2 * sizeof(uint16_t);
        if (lds > 64 * 1024)   // (per launch: the limit belongs to the function, and another context may have set a smaller one)
            HDC_HIP(hipFuncSetAttribute(reinterpret_cast<const void *>(accumulate_small_kernel),
                                        hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
        ProfScope prof(c, HDC_K_ACCUMULATE, s);
        hipLaunchKernelGGL(accumulate_small_kernel, dim3((unsigned)C, (unsigned)(c->Wp / kSliceWords)),
                           dim3(kAccWaves * kWave), lds, s, hv, labels, (int)N, c->W, c->p.D, acc, class_n);
        HDC_HIP(hipGetLastError());
        return HDC_OK;
    }
    if (C <= kLocalMaxC && c->W <= kLocalMaxWords) return accumulate_local(c, hv, labels, N, C, acc, class_n, s);
    for (int64_t n0 = 0; n0 < N; n0 += plan.rows_max) {
        const int64_t n = (N - n0 < plan.rows_max) ? N - n0 : plan.rows_max;
        const uint32_t *hv0 = hv + (size_t)n0 * c->W;
        const int32_t *lab0 = labels + n0;
        const int64_t rb = plan_rb(plan, n);
        const uint32_t block_rows = (uint32_t)(plan.rg * rb);
        if (n <= kSmallN) {
            hipLaunchKernelGGL(group_small_kernel, dim3(1), dim3(kGroupThreads), (size_t)(2 * C + 2) * 4, s,
                               lab0, (int)n, C, block_rows, c->cls_cnt_d, c->cls_off_d, c->cls_blk_d,
                               c->perm_d, class_n);
        } else {
            const int64_t runs = (n + kScatterRun - 1) / kScatterRun;
            const unsigned nb = (unsigned)(runs > 4096 ? 4096 : runs);
            if (C <= 2) {
                const unsigned nb2 = (unsigned)((n + kTwoRun - 1) / kTwoRun);
                hipLaunchKernelGGL(group_two_kernel, dim3(nb2), dim3(256), 0, s, lab0, n, C, block_rows, c->cls_cur_d,
                                   c->cls_cnt_d, c->cls_off_d, c->cls_blk_d, c->perm_d, class_n);
            } else {
                hipLaunchKernelGGL(count_labels_kernel, dim3(nb), dim3(256), (size_t)(C + 1) * 4, s, lab0, n, C,
                                   block_rows, c->cls_cur_d, c->cls_cnt_d, c->cls_off_d, c->cls_blk_d, class_n);
                hipLaunchKernelGGL(scatter_rows_kernel, dim3(nb), dim3(256), (size_t)(C + 1) * 4, s, lab0, n, C,
                                   c->cls_off_d, c->cls_cur_d, c->perm_d);
            }
        }
        const int rc = accumulate_grouped(c, plan, hv0, n, C, rb, acc, s);
        if (rc != HDC_OK) return rc;
    }
    return HDC_OK;
}

// ---- vertical summation on its own (Sec. IV-B2) --------------------------------------------
// out[d] = number of rows with dimension d set: the class count with every row in one class.
// The grouping step degenerates to the identity permutation.
__global__ __launch_bounds__(256) void group_all_kernel(uint32_t n, uint32_t block_rows, uint32_t *cnt,
                                                         uint32_t *off, uint32_t *blk, uint32_t *perm) {
    const uint32_t i = blockIdx.x * 256 + threadIdx.x;
    if (i < n) perm[i] = i;
    if (i == 0) {
        cnt[0] = n;
        off[0] = 0;
        off[1] = n;
        blk[0] = 0;
        blk[1] = (n + block_rows - 1) / block_rows;
    }
}

__global__ __launch_bounds__(256) void zero_i32_kernel(int32_t *p, int64_t n) {
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i < n) p[i] = 0;
}

int launch_vsum(hdc_ctx_impl *c, const uint32_t *hv, int64_t N, int32_t *out, hipStream_t s) {
    AccPlan plan;
    const int prc = plan_static(c, &plan);
    if (prc != HDC_OK) return prc;
    hipLaunchKernelGGL(zero_i32_kernel, dim3((unsigned)((c->p.D + 255) / 256)), dim3(256), 0, s, out,
                       (int64_t)c->p.D);
    if (c->W <= kLocalMaxWords) return accumulate_local(c, hv, nullptr, N, 1, out, nullptr, s);
    for (int64_t n0 = 0; n0 < N; n0 += plan.rows_max) {
        const int64_t n = (N - n0 < plan.rows_max) ? N - n0 : plan.rows_max;
        const int64_t rb = plan_rb(plan, n);
        hipLaunchKernelGGL(group_all_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s, (uint32_t)n,
                           (uint32_t)(plan.rg * rb), c->cls_cnt_d, c->cls_off_d, c->cls_blk_d, c->perm_d);
        const int rc = accumulate_grouped(c, plan, hv + (size_t)n0 * c->W, n, 1, rb, out, s);
        if (rc != HDC_OK) return rc;
    }
    HDC_HIP(hipGetLastError());
    return HDC_OK;
}

// ---- vertical summation without a context and without any allocation ------------------------
// For callers that cannot allocate (HIP graph capture, serving loops, harnesses that forbid it):
// the kernels of launch_vsum with their scratch (the identity permutation, the work list and the
// blocks' partial count rows) in a static device array instead of a context's buffers.  Rows are
// taken kStaticRows at a time, which bounds the scratch; the launches of one call, and of calls
// on one stream, follow each other on the stream and so share the array safely; calls that
// overlap on one GPU (two streams) race on it.
constexpr int kStaticMaxD = 16384;                 // 512 words per row
constexpr int64_t kStaticRows = 262144;            // rows per round of launches
constexpr int64_t kStaticItems = 192;              // partial rows a round can produce (see vsum_static below)
constexpr size_t kStaticPermWords = (size_t)kStaticRows;
constexpr size_t kStaticListWords = 64;            // cnt[2], off[2], blk[2] of the one "class", padded
constexpr size_t kStaticPartialWords = (size_t)kStaticItems * (kStaticMaxD / 32) * 16;
constexpr size_t kStaticWords = kStaticPermWords + kStaticListWords + kStaticPartialWords;   // 7.3 MB
static __device__ __align__(256) uint32_t scratch[kStaticWords];

constexpr int kStaticMaxDevices = 64;
struct StaticDevice {
    uint32_t *ptr;   // this device's copy of `scratch` (the array's name is no device address on the host)
    int num_cus;
    int bpc[kAccWaves + 1];   // blocks of accumulate_kernel a CU holds, by slices per block (0 = not asked yet)
};
static StaticDevice g_static[kStaticMaxDevices];
static bool g_static_ready[kStaticMaxDevices];

int vsum_static(int32_t D, const uint32_t *hv, int64_t N, int32_t *out, hipStream_t s) {
    int dev = -1;
    HDC_HIP(hipGetDevice(&dev));
    if (dev < 0 || dev >= kStaticMaxDevices) return HDC_ELIMIT;
    StaticDevice &sd = g_static[dev];
    if (!g_static_ready[dev]) {   // once per device, with that device current
        void *ptr = nullptr;
        HDC_HIP(hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)));
        HDC_HIP(hipDeviceGetAttribute(&sd.num_cus, hipDeviceAttributeMultiprocessorCount, dev));
        if (!ptr || sd.num_cus < 1) return HDC_EHIP;
        sd.ptr = static_cast<uint32_t *>(ptr);
        for (int &b : sd.bpc) b = 0;
        g_static_ready[dev] = true;
    }
    const int W = (D + 31) / 32, Wp = (W + kSliceWords - 1) / kSliceWords * kSliceWords;
    const int nslices = Wp / kSliceWords;
    const int spb = nslices < kAccWaves ? nslices : kAccWaves, rg = kAccWaves / spb;
    const int ychunks = (nslices + spb - 1) / spb;
    const size_t lds = (size_t)(rg - 1) * spb * kWavePlanes * kWave * sizeof(uint32_t);
    if (sd.bpc[spb] == 0) {
        int bpc = 0;
        HDC_HIP(hipOccupancyMaxActiveBlocksPerMultiprocessor(&bpc, reinterpret_cast<const void *>(accumulate_kernel),
                                                             spb * rg * kWave, lds));
        sd.bpc[spb] = bpc < 1 ? 1 : bpc;
    }
    uint32_t *perm = sd.ptr, *cnt = perm + kStaticPermWords, *off = cnt + 2, *blk = off + 2;
    uint32_t *partial = cnt + kStaticListWords;
    // rows per wave so that a round of rows is one round of blocks, within what a block's planes count
    int64_t cap = (int64_t)sd.num_cus * sd.bpc[spb] / ychunks - 1;
    cap = cap < 1 ? 1 : (cap > kStaticItems - 2 ? kStaticItems - 2 : cap);
    int64_t rb_max = (4088 / rg) / 8 * 8;
    rb_max = rb_max > 2040 ? 2040 : rb_max;
    hipLaunchKernelGGL(zero_i32_kernel, dim3((unsigned)((D + 255) / 256)), dim3(256), 0, s, out, (int64_t)D);
    for (int64_t n0 = 0; n0 < N; n0 += kStaticRows) {
        const int64_t n = N - n0 < kStaticRows ? N - n0 : kStaticRows;
        int64_t rb = ((n + rg * cap - 1) / (rg * cap) + 7) / 8 * 8;
        rb = rb < 16 ? 16 : (rb > rb_max ? rb_max : rb);
        const uint32_t block_rows = (uint32_t)(rg * rb);
        const int64_t items = (n + block_rows - 1) / block_rows + 1;
        if (items > kStaticItems) return HDC_ELIMIT;   // (262144 rows in blocks of at least 2040 rows: 130 items at most)
        hipLaunchKernelGGL(group_all_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s, (uint32_t)n, block_rows,
                           cnt, off, blk, perm);
        hipLaunchKernelGGL(accumulate_kernel, dim3((unsigned)items, (unsigned)ychunks), dim3(spb * rg * kWave), lds, s,
                           hv + (size_t)n0 * W, perm, cnt, off, blk, 1, W, Wp, (int)rb, spb, rg, partial);
        const int pairs = Wp * 16;
        int K = (int)((262144 + (int64_t)pairs - 1) / pairs);
        K = K < 1 ? 1 : (K > 16 ? 16 : K);
        hipLaunchKernelGGL(reduce_partials_kernel, dim3((unsigned)((pairs + 255) / 256), 1u, (unsigned)K), dim3(256), 0, s,
                           partial, blk, Wp, D, K, out, 0);
    }
    HDC_HIP(hipGetLastError());
    return HDC_OK;
}

// ---- majority vote to class vectors ----------------------------------------------------
// One lane per dimension; a wave's 64 decisions are gathered with a ballot into two words.
__global__ __launch_bounds__(256) void binarize_classical_kernel(const int32_t *__restrict__ acc,
                                                                  const int64_t *__restrict__ class_n,
                                                                  const uint32_t *__restrict__ tie,
                                                                  int D, int W, uint32_t *class_hv) {
    const int c = blockIdx.y;
    const int d = blockIdx.x * blockDim.x + threadIdx.x;
    bool bit = false;
    if (d < D) {
        const int64_t twice = 2 * (int64_t)acc[(int64_t)c * D + d];
        const int64_t n = class_n[c];
        bit = twice > n ? true : twice < n ? false : ((tie[d >> 5] >> (d & 31)) & 1u);
    }
    const uint64_t m = __ballot(bit);
    const int lane = threadIdx.x & (kWave - 1);
    const int w = d >> 5;
    if ((lane & 31) == 0 && w < W)
        class_hv[(int64_t)c * W + w] = (uint32_t)(lane ? (m >> 32) : m);
}

int launch_binarize_classical(hdc_ctx_impl *c, const int32_t *acc, const int64_t *class_n,
                              uint32_t *class_hv, hipStream_t s) {
    const unsigned bx = (unsigned)((c->W * 32 + 255) / 256);
    hipLaunchKernelGGL(binarize_classical_kernel, dim3(bx, (unsigned)c->p.C), dim3(256), 0, s, acc,
                       class_n, c->tie_d, c->p.D, c->W, class_hv);
    HDC_HIP(hipGetLastError());
    return HDC_OK;
}

}  // namespace hdc
