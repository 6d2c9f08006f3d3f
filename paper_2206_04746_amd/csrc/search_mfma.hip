// Hamming-distance inference on the matrix cores (arXiv 2206.04746, Sec. III: nearest class vector
// by Hamming distance; Sec. IV-B2 for the summation it replaces).
//
// dist[n][c] = popcount(x_n) + popcount(m_c) - 2 * <x_n, m_c>, the last term a dot product of 0/1
// vectors: over a long stream of queries and seven or more classes that is a dense contraction
// (N x C x D), and the vector unit's two instructions per (word, class) bound the other kernels
// well below the rate at which the rows arrive from HBM.  Here the contraction runs as
// v_mfma_f32_32x32x64_f8f6f4 on 4-bit floats, the fastest operand type of the matrix cores:
// M = 32 class slots, N = 32 queries, K = 64 four-bit elements = two 32-bit words of every query,
// one from each half of its row.
//
// No bit is unpacked.  An element of K stands for one bit of a word, but it holds that bit IN
// PLACE: a 4-bit float (sign, two exponent bits, one mantissa bit) with a single bit set is 0.5,
// 1 or 2 for bits 0, 1, 2, so the query operand for bit p of every nibble is x & (0x11111111 << p):
// four masks per word, 16 bytes per lane, one MFMA.  The class operand carries the reciprocal
// weight: the class words are stored with bits 0..2 of every nibble reversed, so that
// m' & (0x11111111 << (2 - p)) is worth 2, 1 or 0.5 where the query's is worth 0.5, 1 or 2, and
// every product is 1 or 0.  Bit 3 is the sign bit and on its own means (minus) zero: it is moved
// down one place on the query side ((x >> 1) & 0x44444444, worth 2) and down to the mantissa on
// the class side ((m' >> 3) & 0x11111111, worth 0.5).  The fp32 accumulators hold <x, m> exactly
// (whole numbers below 2^24).  Which element of K a (lane, register, nibble) feeds is the same
// for both operands, and any pairing of equal positions gives the same sum, so nothing here
// depends on the order of K inside the instruction.
//
// A lane feeds class slot (lane % 32) to the first operand and query (lane % 32) to the second;
// the two halves of the wave take the two halves of a row.  A block of eight waves works on 64
// consecutive rows (two tiles of 32 queries) at a time and splits their words eight ways: wave v
// takes words [v * 4P, (v + 1) * 4P) of both halves of every row.  Together the waves read the
// 64 rows - 80 KB of consecutive memory at D = 10000 - within one pass, so every cache line comes
// from HBM once; a wave that walked through rows of its own in slices would come back to each
// line long after it had left the cache.  The wave fetches its slices with coalesced 16-byte
// loads, parks them in an LDS area of its own and reads them back a row half per lane (reading
// them from memory that way directly - every lane a row of its own - costs more in the texture
// path than the MFMAs take); the loads for the block's next 64 rows are in flight while it
// computes.  A wave's slice of the class vectors never changes: each lane keeps the 4P words of
// its class slot in registers for the whole launch, and their four masks are formed once per step
// for both tiles.
//
// The accumulators come back with the query on the lane and the class slot on the register (and
// the wave half).  Each wave writes its partial dot products (at most 64 * 4P each: two to a
// 32-bit word) to its LDS area; after a barrier wave w adds up, over the eight waves, four
// registers of one tile, turns them into keys (distance, class) and takes their minimum; after
// a second barrier 64 threads take the minimum over the four register groups.  Slot 31 holds an
// all-ones class: its dot product is popcount(x), needed only when distances are written out.
// Hence 31 classes to a pass where distances are asked for, 32 where not.  More classes (up to 124) take up to four passes over the same row
// images, each with class words of its own in registers; the running minimum of a query's keys
// stays in the reducing wave's registers between the passes, and the partial sums of consecutive
// passes go to two LDS areas used in turn, so that a pass costs one barrier.  Rows too long for
// 64 images in LDS (D above 10240 or so) are taken 32 at a time, one tile of queries per job,
// with one pass.  Beyond what one launch holds the classes are dealt out over several launches:
// all but the last leave a query's best key so far in pred[], all but the first start from it.
#include "hdc_internal.h"

#include <algorithm>
#include <climits>

namespace hdc {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v8i __attribute__((ext_vector_type(8)));
typedef float v16f __attribute__((ext_vector_type(16)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4_a4 __attribute__((ext_vector_type(4), aligned(4)));

constexpr int kMfmaWaves = 8;    // per block: two per SIMD, one block per CU
constexpr int kSlots = 32;       // class slots of an MFMA (its M)
constexpr int kTile = 32;        // queries of an MFMA (its N)
constexpr int kMaxTiles = 2;     // tiles of queries a block carries at a time: two, or one where the rows are long
constexpr int kOnes = kSlots - 1;              // the slot of the all-ones class
constexpr int pass_classes(bool with_dist) { return with_dist ? kOnes : kSlots; }   // classes of a pass: the all-ones class takes a slot only where distances are written
constexpr int kMaxPasses = 4;
constexpr int kRegs = 4;                       // accumulator registers a wave reduces (of one tile): two packed words per lane
constexpr int kGroups = 16 / kRegs;            // such groups per tile; wave w reduces group w % 4 of tile w / 4
constexpr int partial_bytes(int tiles) { return tiles * 8 * kWave * 4; }   // a wave's partial dot products, two to a word

// Host and device agree on the geometry of a row: the first half is s0 words (a multiple of 4, so
// that both halves start on a 16-byte boundary of the row), each wave takes 4P words of each half,
// and a row's image in LDS is row_bytes long (an odd number of 16-byte units: the 16-byte reads of
// 8 neighbouring lanes, a row each, then fall into different banks).
struct RowGeo {
    int s0, pieces, row_bytes, tiles, passes;
    size_t lds_bytes;
};
static inline RowGeo row_geo(int W, int tiles, int passes) {
    RowGeo g;
    g.tiles = tiles;
    g.passes = passes;
    g.s0 = ((W + 1) / 2 + 3) / 4 * 4;
    g.pieces = (g.s0 / 4 + kMfmaWaves - 1) / kMfmaWaves;
    const int units = (W + 3) / 4;
    g.row_bytes = 16 * (units | 1);
    // the last wave's slice of the second half may reach past the last row's image: one more image of slack
    g.lds_bytes = (size_t)(2 * kSlots * passes + 2 * tiles * kGroups * kTile) * 4 + (size_t)(tiles * kTile + 1) * g.row_bytes +
                  (size_t)(passes > 1 ? 2 : 1) * kMfmaWaves * partial_bytes(tiles);
    return g;
}

// bits 0..2 of every nibble reversed, bit 3 in place
__device__ __forceinline__ uint32_t reverse3(uint32_t m) {
    return (m & 0xaaaaaaaau) | ((m & 0x11111111u) << 2) | ((m >> 2) & 0x11111111u);
}

// Both operands as 4-bit floats (format code 4), no block scales; 16 bytes of each are used.
__device__ __forceinline__ v16f mfma(v4i a, v4i b, v16f c) {
    const v8i a8 = {a[0], a[1], a[2], a[3], 0, 0, 0, 0}, b8 = {b[0], b[1], b[2], b[3], 0, 0, 0, 0};
    return __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(a8, b8, c, 4, 4, 0, 0, 0, 0);
}

// Dynamic LDS: popcount(m_c) [32 a pass], key bases of as many, keys [tiles][4 groups][32 queries], popcount(x) parts of
// the same shape, the images of the job's rows (and one of slack), then the waves' partial sums
// (two areas where there are several passes).
template <int P, int kTiles, int kPasses, bool kDist>
__global__ __launch_bounds__(kMfmaWaves *kWave) void search_mfma_kernel(
    const uint32_t *__restrict__ hv, int64_t N, const uint32_t *__restrict__ class_hv, int C, int W, int D,
    int s0, int row_bytes, uint32_t *__restrict__ dist, int32_t *__restrict__ pred, int c0, int Cn, int keys_in,
    int keys_out) {
    // this launch: classes c0 .. c0 + Cn - 1 of the C; keys_in: pred[] holds the best key of the
    // classes before c0; keys_out: leave the key there, not the class
    constexpr int kJob = kTile * kTiles;
    constexpr int kPassClasses = pass_classes(kDist);
    constexpr int kWaveRows = kJob / kMfmaWaves;   // rows of a job a wave fetches
    constexpr int kPartialBytes = partial_bytes(kTiles);
    constexpr int kAreaBytes = kMfmaWaves * kPartialBytes;
    constexpr int kSteps = 4 * P;      // words of a row half per wave = MFMA steps per job and pass
    constexpr int kLoads = kTiles * P; // 16-byte loads per lane per job: a wave's rows of at most 16P pieces over 64 lanes
    extern __shared__ uint32_t popc_m[];
    int *base_tab = reinterpret_cast<int *>(popc_m + kSlots * kPasses);   // [pass][group][wave half][register]
    int *keyq = base_tab + kSlots * kPasses;
    int *popx = keyq + kTiles * kGroups * kTile;
    char *rows = reinterpret_cast<char *>(popx + kTiles * kGroups * kTile);
    char *partials = rows + (size_t)(kJob + 1) * row_bytes;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int lane = threadIdx.x & (kWave - 1);
    const int q = lane & (kTile - 1), h = lane >> 5;
    const uint32_t tail = (D & 31) ? (1u << (D & 31)) - 1u : 0xffffffffu;

    // The lane's class words: words h * s0 + wave * 4P + s of the class its slot q stands for in
    // each pass, zero where that is outside the half (the row words they meet there are other
    // words or no words at all).
    // The slices of the waves and halves cover every word of a class once, so popcount(m_c) is
    // the sum of the lanes' counts over their own words: no second reading of the class vectors.
    uint32_t cw[kPasses][kSteps];
    for (int j = threadIdx.x; j < kSlots * kPasses; j += kMfmaWaves * kWave) popc_m[j] = 0;
    __syncthreads();
#pragma unroll
    for (int p = 0; p < kPasses; ++p) {
        const int cls = p * kPassClasses + q;    // counted from c0
        const bool real = q < kPassClasses && cls < Cn;
        uint32_t ones = 0;
#pragma unroll
        for (int s = 0; s < kSteps; ++s) {
            const int w = h * s0 + wave * kSteps + s;
            uint32_t m = 0;
            if (w < (h ? W : s0)) {
                if (real) m = class_hv[(int64_t)(c0 + cls) * W + w];
                else if (kDist && q == kOnes && p == 0) m = w == W - 1 ? tail : 0xffffffffu;
            }
            ones += __popc(m);
            cw[p][s] = reverse3(m);
        }
        if (real) atomicAdd(&popc_m[cls], ones);
    }
    __syncthreads();

    // Which class slot each accumulator register of a lane belongs to, asked of the instruction
    // itself: five elements of K carry the bits of the slot number on the class side (as 1, 1, 4,
    // 4, 4) against 1, 2, 1, 2, 4 on the query side, products 1, 2, 4, 8, 16.  In the reduction
    // wave w handles kRegs registers of one tile (group w % kGroups of tile w / kGroups): their
    // slots and key bases ((popcount(m) << 10) | class; slots without a class start so high that
    // no dot product brings them below a real one).
    const int rg = wave % kGroups, rt = wave / kGroups;
    const bool reduces = rt < kTiles;     // wave-uniform: with one tile waves 4 to 7 have nothing to reduce
    int slot_of[kRegs], base_of[kRegs];      // the bases of the first pass; with several passes all of them are in LDS
    {
        const int bits = (q & 1 ? 0x2 : 0) | (q & 2 ? 0x20 : 0) | (q & 4 ? 0x600 : 0) | (q & 8 ? 0x6000 : 0) |
                         (q & 16 ? 0x60000 : 0);
        const v4i a = {h == 0 ? bits : 0, 0, 0, 0}, b = {h == 0 ? 0x64242 : 0, 0, 0, 0};
        v16f z;
#pragma unroll
        for (int r = 0; r < 16; ++r) z[r] = 0.0f;
        z = mfma(a, b, z);
#pragma unroll
        for (int j = 0; j < kRegs; ++j) {
            float v = 0.0f;
#pragma unroll
            for (int g = 0; g < kGroups; ++g) v = rg == g ? z[g * kRegs + j] : v;
            slot_of[j] = (int)v;
#pragma unroll
            for (int p = 0; p < kPasses; ++p) {
                const int cls = p * kPassClasses + slot_of[j];
                const int base =
                    slot_of[j] < kPassClasses && cls < Cn ? (int)((popc_m[cls] << 10) | (uint32_t)(c0 + cls)) : INT_MAX;
                if (p == 0) base_of[j] = base;
                if (kPasses > 1 && rt == 0 && q == 0) base_tab[((p * kGroups + rg) * 2 + h) * kRegs + j] = base;
            }
        }
        if (kPasses > 1) __syncthreads();
    }

    // The lane's share of a job's fetch.  Wave v brings a job's rows 8v .. 8v + 7 (4v .. 4v + 3
    // where it has one tile): their whole 16-byte pieces, piece after piece over the lanes (load i:
    // piece number i * 64 + lane of the rows' W / 4 each; numbers past the end repeat the last
    // piece), and, where W is no multiple of 4,
    // the one to three words left over, a word per lane.  One register per load: the word's offset
    // from the job's first word in bits 0..15, the 16-byte unit of the images from bit 16.
    const int whole = W / 4;
    uint32_t load_of[kLoads];
#pragma unroll
    for (int i = 0; i < kLoads; ++i) {
        const int id = min(i * kWave + lane, kWaveRows * whole - 1);
        const int r = wave * kWaveRows + id / whole, pc = id % whole;
        load_of[i] = (uint32_t)(r * W + 4 * pc) | ((uint32_t)(r * (row_bytes / 16) + pc) << 16);
    }
    const int left = W - 4 * whole;                  // 0..3 words
    const int lr = wave * kWaveRows + (lane >> 2) % kWaveRows, lj = min(lane & 3, max(left - 1, 0));
    const int left_word = lr * W + 4 * whole + lj;   // lanes past the words left over repeat the last one
    char *left_at = rows + lr * row_bytes + (4 * whole + lj) * 4;

    const char *take_at = rows + q * row_bytes + (h * s0 + wave * kSteps) * 4;
    const int tile_bytes = kTile * row_bytes;
    auto bases = [&](int(&base)[kRegs], int p) {   // of the lane's registers in pass p
        if constexpr (kPasses > 1) {
            const int4 b = *reinterpret_cast<const int4 *>(base_tab + ((p * kGroups + rg) * 2 + h) * kRegs);
            base[0] = b.x, base[1] = b.y, base[2] = b.z, base[3] = b.w;
        } else {
#pragma unroll
            for (int j = 0; j < kRegs; ++j) base[j] = base_of[j];
        }
    };
    char *mine = partials + wave * kPartialBytes;

    const int64_t jobs = (N + kJob - 1) / kJob;
    const int64_t last_word = N * W - 1;
    u32x4_a4 f[kLoads];
    uint32_t f_left = 0;
    auto fetch = [&](int64_t job) {   // rows past N read the last row's last words
        const int64_t first = job * kJob * W;
#pragma unroll
        for (int i = 0; i < kLoads; ++i) {
            const int64_t at = first + (load_of[i] & 0xffffu);
            f[i] = *reinterpret_cast<const u32x4_a4 *>(hv + (at + 3 <= last_word ? at : last_word - 3));
        }
        if (left) {   // the same for every thread of the launch
            const int64_t at = first + left_word;
            f_left = hv[at <= last_word ? at : last_word];
        }
    };
    // Several passes: a row's distances are many, and lanes that each write single words of 32
    // rows reach a fraction of the memory's rate.  They meet in the second area of the partial
    // sums (row pitch odd) after the job's last barrier and leave as whole rows after the next
    // job's first one, under its matrix instructions; that area is next written in that job's
    // second pass, a barrier later.
    constexpr bool kStaged = kDist && kPasses > 1;
    int *stage = reinterpret_cast<int *>(partials + kAreaBytes);
    const int stage_pitch = Cn | 1;
    static_assert(!kStaged || kJob * (kMaxPasses * kOnes + 1) * 4 <= kAreaBytes, "a job's distances fit an area");
    auto rows_out = [&](int64_t of_job) {   // wave v: rows v, v + 8, ...; four rows read before the first of them is written
        constexpr int kCols = (kPasses * kPassClasses + kWave - 1) / kWave;
        constexpr int kAtOnce = 4;
        uint32_t *out = dist + (of_job * kJob + wave) * C + c0;
        const int64_t rows_left = N - of_job * kJob - wave;    // this wave's rows: those with i * 8 below this
#pragma unroll 1
        for (int i0 = 0; i0 < kWaveRows; i0 += kAtOnce) {
            int v[kAtOnce][kCols];
#pragma unroll
            for (int i = 0; i < kAtOnce; ++i)
#pragma unroll
                for (int cc = 0; cc < kCols; ++cc)
                    v[i][cc] = stage[(wave + (i0 + i) * kMfmaWaves) * stage_pitch + min(lane + cc * kWave, Cn - 1)];
#pragma unroll
            for (int i = 0; i < kAtOnce; ++i)
#pragma unroll
                for (int cc = 0; cc < kCols; ++cc)
                    if ((i0 + i) * kMfmaWaves < rows_left && lane + cc * kWave < Cn)
                        out[(int64_t)(i0 + i) * kMfmaWaves * C + lane + cc * kWave] = (uint32_t)v[i][cc];
        }
    };
    int64_t staged = -1;    // the job whose distances wait there (block-uniform)

    fetch(blockIdx.x);
    for (int64_t job = blockIdx.x; job < jobs; job += gridDim.x) {   // block-uniform
        // (every wave has taken the previous job's words: it has passed that job's second barrier)
#pragma unroll
        for (int i = 0; i < kLoads; ++i) *reinterpret_cast<u32x4 *>(rows + (load_of[i] >> 16) * 16) = f[i];
        if (left) *reinterpret_cast<uint32_t *>(left_at) = f_left;
        __syncthreads();
        fetch(job + gridDim.x);                 // past the last job it reads the buffer's last words
        __builtin_amdgcn_sched_barrier(0);      // the loads go out before the MFMAs, not after
        if constexpr (kStaged) {
            if (staged >= 0) rows_out(staged);
        }

        // the lane's words come out of the images a piece (four steps) ahead of their use
        auto take = [&](u32x4(&x)[kTiles], int k) {
#pragma unroll
            for (int t = 0; t < kTiles; ++t) x[t] = *reinterpret_cast<const u32x4 *>(take_at + t * tile_bytes + k * 16);
        };
        int key = INT_MAX;
        int dot[kPasses][kRegs];
        // Two passes go through the row images together: the query-side masks of a word are formed
        // once for both, their partial sums go to the two areas at once, and one barrier serves
        // both.  (Three and four passes go one at a time: two more sets of accumulators would not
        // fit beside their class words.)
        constexpr int kTogether = kPasses == 2 ? 2 : 1;
#pragma unroll
        for (int p0 = 0; p0 < kPasses; p0 += kTogether) {
            v16f acc[kTogether][kTiles];
#pragma unroll
            for (int i = 0; i < kTogether; ++i)
#pragma unroll
                for (int t = 0; t < kTiles; ++t)
#pragma unroll
                    for (int r = 0; r < 16; ++r) acc[i][t][r] = 0.0f;
            u32x4 x[2][kTiles];
            take(x[0], 0);
#pragma unroll
            for (int k = 0; k < P; ++k) {
                if (k + 1 < P) take(x[(k + 1) & 1], k + 1);
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    v4i b[kTiles];
#pragma unroll
                    for (int t = 0; t < kTiles; ++t) {
                        const uint32_t xw = x[k & 1][t][e];
                        b[t] = v4i{(int)(xw & 0x11111111u), (int)(xw & 0x22222222u), (int)(xw & 0x44444444u),
                                   (int)((xw >> 1) & 0x44444444u)};
                    }
#pragma unroll
                    for (int i = 0; i < kTogether; ++i) {
                        uint32_t c = cw[p0 + i][4 * k + e];
                        // With one pass over two tiles the compiler keeps all the masks of the class words
                        // in registers over the whole launch; the other forms have no room for that
                        // (it would spill them in this loop), so there the word is made opaque here.
                        if constexpr (kPasses > 1 || kTiles == 1 || P > 5) asm volatile("" : "+v"(c));
                        const v4i a = {(int)(c & 0x44444444u), (int)(c & 0x22222222u), (int)(c & 0x11111111u),
                                       (int)((c >> 3) & 0x11111111u)};
#pragma unroll
                        for (int t = 0; t < kTiles; ++t) acc[i][t] = mfma(a, b[t], acc[i][t]);
                    }
                }
            }

            // partial dot products, registers 2i and 2i + 1 in one word: [tile][group of four registers][lane][2 words];
            // pass p takes area p % 2
#pragma unroll
            for (int i = 0; i < kTogether; ++i) {
                uint32_t *out = reinterpret_cast<uint32_t *>(mine + ((p0 + i) & 1) * kAreaBytes);
#pragma unroll
                for (int t = 0; t < kTiles; ++t)
#pragma unroll
                    for (int g = 0; g < kGroups; ++g) {
                        uint32_t pk[2];
#pragma unroll
                        for (int j = 0; j < 2; ++j)
                            pk[j] = (uint32_t)acc[i][t][kRegs * g + 2 * j] | ((uint32_t)acc[i][t][kRegs * g + 2 * j + 1] << 16);
                        *reinterpret_cast<uint2 *>(out + ((t * kGroups + g) * kWave + lane) * 2) = make_uint2(pk[0], pk[1]);
                    }
            }
            __syncthreads();
            // (the pass after the next writes this area again: every wave has then passed the next
            // pass's barrier, or the job's last one, and so has read what it needs here)

            if (reduces) {
#pragma unroll
                for (int i = 0; i < kTogether; ++i) {
                    const int p = p0 + i, area = (p & 1) * kAreaBytes;
                    // the halves of a word add up separately: eight partials stay far below 2^16
                    uint2 sum = make_uint2(0u, 0u);
#pragma unroll
                    for (int v = 0; v < kMfmaWaves; ++v) {
                        const uint2 part = *reinterpret_cast<const uint2 *>(
                            reinterpret_cast<const uint32_t *>(partials + area + v * kPartialBytes) +
                            ((rt * kGroups + rg) * kWave + lane) * 2);
                        sum.x += part.x;
                        sum.y += part.y;
                    }
                    dot[p][0] = (int)(sum.x & 0xffffu);
                    dot[p][1] = (int)(sum.x >> 16);
                    dot[p][2] = (int)(sum.y & 0xffffu);
                    dot[p][3] = (int)(sum.y >> 16);
                    int base[kRegs];
                    bases(base, p);
#pragma unroll
                    for (int j = 0; j < kRegs; ++j) key = min(key, base[j] - (dot[p][j] << 11));   // the key takes 2048 * dot off
                }
            }
        }
        if (reduces) {
            key = min(key, __shfl_xor(key, 32, kWave));
            if (h == 0) keyq[(rt * kGroups + rg) * kTile + q] = key;
            if (kDist) {
                int part = 0;
#pragma unroll
                for (int j = 0; j < kRegs; ++j) part += slot_of[j] == kOnes ? dot[0][j] : 0;
                part += __shfl_xor(part, 32, kWave);
                if (h == 0) popx[(rt * kGroups + rg) * kTile + q] = part;
            }
        }
        __syncthreads();

        if (threadIdx.x < kJob) {
            const int t = threadIdx.x >> 5, qq = threadIdx.x & (kTile - 1);
            int k = keyq[(t * kGroups + 0) * kTile + qq];
#pragma unroll
            for (int g = 1; g < kGroups; ++g) k = min(k, keyq[(t * kGroups + g) * kTile + qq]);
            const int64_t n = job * kJob + threadIdx.x;
            if (n < N) {
                if (keys_in) k = min(k, pred[n]);
                pred[n] = keys_out ? k : k & 1023;
            }
        }
        if constexpr (kStaged) {
            if (reduces) {
                int popc_x = 0;
#pragma unroll
                for (int g = 0; g < kGroups; ++g) popc_x += popx[(rt * kGroups + g) * kTile + q];
#pragma unroll
                for (int p = 0; p < kPasses; ++p) {
                    int base[kRegs];
                    bases(base, p);
#pragma unroll
                    for (int j = 0; j < kRegs; ++j)
                        if (base[j] != INT_MAX)
                            stage[(rt * kTile + q) * stage_pitch + p * kPassClasses + slot_of[j]] =
                                popc_x + (base[j] >> 10) - 2 * dot[p][j];
                }
            }
            staged = job;
        } else if (kDist && reduces) {
            int popc_x = 0;
#pragma unroll
            for (int g = 0; g < kGroups; ++g) popc_x += popx[(rt * kGroups + g) * kTile + q];
            const int64_t n = job * kJob + rt * kTile + q;
            if (n < N) {
#pragma unroll
                for (int j = 0; j < kRegs; ++j)
                    if (base_of[j] != INT_MAX)
                        dist[n * C + (base_of[j] & 1023)] = (uint32_t)(popc_x + (base_of[j] >> 10) - 2 * dot[0][j]);
            }
        }
    }
    if constexpr (kStaged) {
        if (staged >= 0) {
            __syncthreads();
            rows_out(staged);
        }
    }
}

constexpr int64_t kMfmaQueries = 20480;        // from here on with 9 to 12 classes (measured against the vector kernels at D = 10000)
constexpr int64_t kMfmaQueriesMany = 8192;     // and from here on with 13 or more: 10000 queries x 26 classes 19 -> 12 us (below, a block's set-up -- its class words -- outweighs its one or two jobs: 4096 x 100 classes 20 us on the vector kernel, 35 here)

// What one launch is given: its classes and what pred[] holds before and after it.
struct ClassSpan {
    int c0, n, keys_in, keys_out;
};

template <int P, int kTiles, int kPasses>
static int launch_mfma(hdc_ctx_impl *c, const RowGeo &g, const ClassSpan &cs, const uint32_t *hv, int64_t N,
                       const uint32_t *class_hv, uint32_t *dist, int32_t *pred, hipStream_t s) {
    const void *kern = dist ? reinterpret_cast<const void *>(search_mfma_kernel<P, kTiles, kPasses, true>)
                            : reinterpret_cast<const void *>(search_mfma_kernel<P, kTiles, kPasses, false>);
    if (g.lds_bytes > 64 * 1024)
        HDC_HIP(hipFuncSetAttribute(kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)g.lds_bytes));
    constexpr int kJob = kTile * kTiles;
    const int64_t jobs = (N + kJob - 1) / kJob;
    const int64_t blocks = std::min<int64_t>(256, jobs);
    {
        ProfScope prof(c, HDC_K_SEARCH, s);
        if (dist)
            hipLaunchKernelGGL((search_mfma_kernel<P, kTiles, kPasses, true>), dim3((unsigned)blocks),
                               dim3(kMfmaWaves * kWave), g.lds_bytes, s, hv, N, class_hv, c->p.C, c->W, c->p.D, g.s0,
                               g.row_bytes, dist, pred, cs.c0, cs.n, cs.keys_in, cs.keys_out);
        else
            hipLaunchKernelGGL((search_mfma_kernel<P, kTiles, kPasses, false>), dim3((unsigned)blocks),
                               dim3(kMfmaWaves * kWave), g.lds_bytes, s, hv, N, class_hv, c->p.C, c->W, c->p.D, g.s0,
                               g.row_bytes, dist, pred, cs.c0, cs.n, cs.keys_in, cs.keys_out);
    }
    HDC_HIP(hipGetLastError());
    return HDC_OK;
}

template <int P>
static int launch_passes(hdc_ctx_impl *c, const RowGeo &g, const ClassSpan &cs, const uint32_t *hv, int64_t N,
                         const uint32_t *class_hv, uint32_t *dist, int32_t *pred, hipStream_t s) {
    switch (g.passes) {
    case 1: return launch_mfma<P, 2, 1>(c, g, cs, hv, N, class_hv, dist, pred, s);
    case 2: return launch_mfma<P, 2, 2>(c, g, cs, hv, N, class_hv, dist, pred, s);
    case 3: return launch_mfma<P, 2, 3>(c, g, cs, hv, N, class_hv, dist, pred, s);
    default: return launch_mfma<P, 2, 4>(c, g, cs, hv, N, class_hv, dist, pred, s);
    }
}

static int launch_span(hdc_ctx_impl *c, const RowGeo &g, const ClassSpan &cs, const uint32_t *hv, int64_t N,
                       const uint32_t *class_hv, uint32_t *dist, int32_t *pred, hipStream_t s) {
    if (g.tiles == 2) {
        switch (g.pieces) {
        case 1: return launch_passes<1>(c, g, cs, hv, N, class_hv, dist, pred, s);
        case 2: return launch_passes<2>(c, g, cs, hv, N, class_hv, dist, pred, s);
        case 3: return launch_passes<3>(c, g, cs, hv, N, class_hv, dist, pred, s);
        case 4: return launch_passes<4>(c, g, cs, hv, N, class_hv, dist, pred, s);
        case 5: return launch_passes<5>(c, g, cs, hv, N, class_hv, dist, pred, s);
        case 6: return launch_mfma<6, 2, 1>(c, g, cs, hv, N, class_hv, dist, pred, s);   // (one pass: see try_search_mfma)
        default: return launch_mfma<7, 2, 1>(c, g, cs, hv, N, class_hv, dist, pred, s);
        }
    }
    switch ((g.pieces + 1) / 2) {    // an odd count takes the next even one: its last slices meet zero class words
    case 3: return launch_mfma<6, 1, 1>(c, g, cs, hv, N, class_hv, dist, pred, s);
    case 4: return launch_mfma<8, 1, 1>(c, g, cs, hv, N, class_hv, dist, pred, s);
    case 5: return launch_mfma<10, 1, 1>(c, g, cs, hv, N, class_hv, dist, pred, s);
    case 6: return launch_mfma<12, 1, 1>(c, g, cs, hv, N, class_hv, dist, pred, s);
    case 7: return launch_mfma<14, 1, 1>(c, g, cs, hv, N, class_hv, dist, pred, s);
    default: return launch_mfma<16, 1, 1>(c, g, cs, hv, N, class_hv, dist, pred, s);
    }
}

// Takes the search if it is of the shape this kernel is for; returns false otherwise.
bool try_search_mfma(hdc_ctx_impl *c, const uint32_t *hv, int64_t N, const uint32_t *class_hv,
                     uint32_t *dist, int32_t *pred, hipStream_t s, int *rc) {
    const int C = c->p.C, W = c->W;
    // fewer classes: the row-per-16-lanes kernel is as fast or faster (this one takes the same time for
    // any number of classes of a pass: at D = 10000, 0.25 ms for a million queries, 0.29 ms with distances)
    if (N < (C >= 13 ? kMfmaQueriesMany : kMfmaQueries) || C < 9 || W < 4) return false;
    static_assert(HDC_MAX_C <= 1024, "a key keeps the class in ten bits");
    // D up to 10240: two tiles of queries per job and up to four passes a launch; up to 32768: a
    // tile per job (the class words of such a row fill the registers) and one pass a launch
    const int pieces = row_geo(W, 1, 1).pieces;
    if (pieces > 16) return false;
    const int kPassClasses = pass_classes(dist != nullptr);
    const int passes = (C + kPassClasses - 1) / kPassClasses;
    // (D up to 14336 and one pass: two tiles still fit, the registers and the LDS)
    const int tiles = pieces <= 5 || (pieces <= 7 && passes == 1 && row_geo(W, 2, 1).lds_bytes <= 160 * 1024) ? 2 : 1;
    const int launch_passes_max = tiles == 2 && pieces <= 5 ? kMaxPasses : 1;
    const int launches = (passes + launch_passes_max - 1) / launch_passes_max;
    if (row_geo(W, tiles, std::min(passes, launch_passes_max)).lds_bytes > 160 * 1024) return false;
    for (int i = 0, p0 = 0; i < launches; ++i) {
        const int np = passes / launches + (i < passes % launches ? 1 : 0);   // as equal as they come
        const ClassSpan cs = {p0 * kPassClasses, std::min(C - p0 * kPassClasses, np * kPassClasses), i > 0,
                              i + 1 < launches};
        *rc = launch_span(c, row_geo(W, tiles, np), cs, hv, N, class_hv, dist, pred, s);
        if (*rc != HDC_OK) return true;
        p0 += np;
    }
    return true;
}

}  // namespace hdc
