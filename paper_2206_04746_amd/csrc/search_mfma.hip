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
// the two halves of the wave take the two halves of a row, so a lane needs only its own half of
// its own query's row.  Reading it from there directly (every lane a row of its own) costs more
// in the texture path than the MFMAs take, so a wave fetches 64 bytes of 128 row halves at a time
// with coalesced 16-byte loads (4 lanes per 64 bytes), parks them in an LDS area of its own and
// reads them back a row half per lane; the loads of the next 64 bytes - or of the next 64
// queries - are in flight while the MFMAs of this chunk run.  The class words come from LDS too (one
// word per lane per step) and their eight masks are formed once for the kTiles tiles of 32
// queries that a wave carries at a time.  The accumulators come back with the query on the lane
// and the class slot on the register (and the wave half), so the nearest class is a minimum over
// the lane's own 16 registers plus one exchange between the halves.  Slot 31 holds an all-ones
// class: its dot product is popcount(x), needed only when distances are written out.  Hence
// C <= 31.
#include "hdc_internal.h"

#include <algorithm>
#include <climits>

namespace hdc {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v8i __attribute__((ext_vector_type(8)));
typedef float v16f __attribute__((ext_vector_type(16)));
typedef uint32_t u32x4_a4 __attribute__((ext_vector_type(4), aligned(4)));

constexpr int kMfmaWaves = 8;    // per block: two per SIMD, one block per CU
constexpr int kSlots = 32;       // class slots of an MFMA (its M)
constexpr int kTile = 32;        // queries of an MFMA (its N)
constexpr int kTiles = 2;        // tiles a wave carries at a time
constexpr int kJob = kTile * kTiles;
constexpr int kChunk = 16;       // words of a row half a lane holds at a time (64 bytes)
constexpr int kPieces = kChunk / 4;
constexpr int kOnes = kSlots - 1;   // the slot of the all-ones class
// A wave's LDS area: [tile][half][row] segments of 64 bytes, 80 bytes apart (the 16-byte reads of
// 8 neighbouring lanes then fall into 32 different banks).
constexpr int kSegBytes = 80;
constexpr int kHalfBytes = kTile * kSegBytes;                 // 2560: the 32 rows of one (tile, half)
constexpr int kWaveBytes = kTiles * 2 * kHalfBytes;           // 10240
constexpr int kFetches = kTiles * 2 * kTile * kChunk * 4 / (kWave * 16);   // 8 loads of 16 bytes per lane per chunk
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

// bits 0..2 of every nibble reversed, bit 3 in place
__device__ __forceinline__ uint32_t reverse3(uint32_t m) {
    return (m & 0xaaaaaaaau) | ((m & 0x11111111u) << 2) | ((m >> 2) & 0x11111111u);
}

// Both operands as 4-bit floats (format code 4), no block scales; 16 bytes of each are used.
__device__ __forceinline__ v16f mfma(v4i a, v4i b, v16f c) {
    const v8i a8 = {a[0], a[1], a[2], a[3], 0, 0, 0, 0}, b8 = {b[0], b[1], b[2], b[3], 0, 0, 0, 0};
    return __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(a8, b8, c, 4, 4, 0, 0, 0, 0);
}

__device__ __forceinline__ void wave_sync_lds() {   // LDS written by some lanes of the wave, read by others
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

// Fetch number i of a chunk covers 16 row halves: tile i / 4, half (i / 2) % 2, rows 16 * (i % 2)
// + lane / 4, the lane taking piece lane % 4 (four words) of the 64 bytes.  rows[t][e] is the
// lane's row of tile t in the upper (e = 1) or lower 16.  A piece that would cross the end of the
// row is moved back to the row's last 16 bytes (the class words in LDS are laid out to match).
struct Fetched {
    u32x4_a4 v[kFetches];
};
__device__ __forceinline__ void fetch_chunk(Fetched &f, const uint32_t *(&rows)[kTiles][2], int c, int s0,
                                            int W, int lane) {
    int w[2];
#pragma unroll
    for (int hh = 0; hh < 2; ++hh) w[hh] = min(hh * s0 + c * kChunk + 4 * (lane & 3), W - 4);
#pragma unroll
    for (int i = 0; i < kFetches; ++i)
        f.v[i] = *reinterpret_cast<const u32x4_a4 *>(rows[i / 4][i % 2] + w[(i / 2) % 2]);
}
__device__ __forceinline__ void park_chunk(const Fetched &f, char *area, int lane) {
    char *at = area + (lane >> 2) * kSegBytes + (lane & 3) * 16;
#pragma unroll
    for (int i = 0; i < kFetches; ++i) *reinterpret_cast<u32x4 *>(at + i * (kHalfBytes / 2)) = f.v[i];
}

struct RowChunk {   // the lane's 16 words of its half of its row, for each tile
    u32x4 x[kTiles][kPieces];
};
__device__ __forceinline__ void take_chunk(RowChunk &r, const char *area, int q, int h) {
    const char *at = area + h * kHalfBytes + q * kSegBytes;
#pragma unroll
    for (int t = 0; t < kTiles; ++t)
#pragma unroll
        for (int k = 0; k < kPieces; ++k) r.x[t][k] = *reinterpret_cast<const u32x4 *>(at + t * 2 * kHalfBytes + k * 16);
}

// kChunk steps: the class words cl[0], cl[32], ... against the chunk's words
__device__ __forceinline__ void run_chunk(const RowChunk &r, const uint32_t *cl, v16f (&acc)[kTiles]) {
#pragma unroll
    for (int s = 0; s < kChunk; ++s) {
        const uint32_t cw = cl[s * kSlots];
        const v4i a = {(int)(cw & 0x44444444u), (int)(cw & 0x22222222u), (int)(cw & 0x11111111u),
                       (int)((cw >> 3) & 0x11111111u)};
#pragma unroll
        for (int t = 0; t < kTiles; ++t) {
            const uint32_t xw = r.x[t][s / 4][s % 4];
            const v4i b = {(int)(xw & 0x11111111u), (int)(xw & 0x22222222u), (int)(xw & 0x44444444u),
                           (int)((xw >> 1) & 0x44444444u)};
            acc[t] = mfma(a, b, acc[t]);
        }
    }
}

// Dynamic LDS: class words [2 halves][spad steps][32 slots], popcount(m_c) [32], then every wave's
// area for row segments.
template <bool kDist>
__global__ __launch_bounds__(kMfmaWaves *kWave) void search_mfma_kernel(
    const uint32_t *__restrict__ hv, int64_t N, const uint32_t *__restrict__ class_hv, int C, int W, int D,
    int spad, uint32_t *__restrict__ dist, int32_t *__restrict__ pred) {
    extern __shared__ uint32_t cls[];
    uint32_t *popc_m = cls + 2 * spad * kSlots;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int lane = threadIdx.x & (kWave - 1);
    const int q = lane & (kTile - 1), h = lane >> 5;
    const int s0 = (W + 1) / 2;                  // words of the first half of a row; the second has W - s0
    const uint32_t tail = (D & 31) ? (1u << (D & 31)) - 1u : 0xffffffffu;

    // The class word a lane meets at step s of half hh is the one its query word of that step was
    // read from: word `first + s` of the row, or, in a piece moved back from the end of the row (see
    // load_chunk), a word of the row's last four.  A moved piece counts only the words that no
    // earlier piece of the half holds; a step whose word lies outside the half counts nothing.
    for (int idx = threadIdx.x; idx < 2 * spad * kSlots; idx += kMfmaWaves * kWave) {
        const int j = idx & (kSlots - 1), hs = idx / kSlots;
        const int hh = hs >= spad, s = hs - hh * spad;
        const int unmoved = hh * s0 + (s & ~3);
        const int w = min(unmoved, W - 4) + (s & 3);
        uint32_t m = 0;
        if (w >= unmoved && w < (hh ? W : s0)) {
            if (j < C) m = class_hv[(int64_t)j * W + w];
            else if (j == kOnes) m = w == W - 1 ? tail : 0xffffffffu;
        }
        cls[idx] = reverse3(m);
    }
    for (int j = wave; j < C; j += kMfmaWaves) {
        uint32_t n = 0;
        for (int w = lane; w < W; w += kWave) n += __popc(class_hv[(int64_t)j * W + w]);
#pragma unroll
        for (int sft = 1; sft < kWave; sft <<= 1) n += (uint32_t)__shfl_xor((int)n, sft, kWave);
        if (lane == 0) popc_m[j] = n;
    }
    __syncthreads();

    // Which class slot each accumulator register of this lane belongs to, asked of the
    // instruction itself: five elements of K carry the bits of the slot number on the class side
    // (as 1, 1, 4, 4, 4) against 1, 2, 1, 2, 4 on the query side, products 1, 2, 4, 8, 16.
    int slot[16];
    {
        const int bits = (q & 1 ? 0x2 : 0) | (q & 2 ? 0x20 : 0) | (q & 4 ? 0x600 : 0) | (q & 8 ? 0x6000 : 0) |
                         (q & 16 ? 0x60000 : 0);
        const v4i a = {h == 0 ? bits : 0, 0, 0, 0}, b = {h == 0 ? 0x64242 : 0, 0, 0, 0};
        v16f z;
#pragma unroll
        for (int r = 0; r < 16; ++r) z[r] = 0.0f;
        z = mfma(a, b, z);
#pragma unroll
        for (int r = 0; r < 16; ++r) slot[r] = (int)z[r];
    }
    // key of (register r, dot product d): (popcount(m) - 2 d) * 1024 + class, signed; slots without
    // a class start so high that no dot product brings them below a real one
    int base[16];
#pragma unroll
    for (int r = 0; r < 16; ++r)
        base[r] = slot[r] < C ? (int)((popc_m[slot[r]] << 10) | (uint32_t)slot[r]) : INT_MAX;

    const int nc = spad / kChunk;
    const int64_t jobs = (N + kJob - 1) / kJob;
    const int64_t stride = (int64_t)gridDim.x * kMfmaWaves;
    int64_t job = (int64_t)blockIdx.x * kMfmaWaves + wave;
    if (job >= jobs) return;   // wave-uniform; there is no block-wide barrier below

    char *area = reinterpret_cast<char *>(popc_m + kSlots) + wave * kWaveBytes;
    const uint32_t *cl = cls + (size_t)h * spad * kSlots + q;
    auto rows_of = [&](int64_t jb, const uint32_t *(&rows)[kTiles][2]) {   // rows past N read row N - 1
#pragma unroll
        for (int t = 0; t < kTiles; ++t)
#pragma unroll
            for (int e = 0; e < 2; ++e) {
                const int64_t n = jb * kJob + t * kTile + e * 16 + (lane >> 2);
                rows[t][e] = hv + (n < N ? n : N - 1) * W;
            }
    };
    const uint32_t *rows[kTiles][2], *rows_next[kTiles][2];
    rows_of(job, rows);
    rows_of(job + stride, rows_next);
    Fetched f;
    fetch_chunk(f, rows, 0, s0, W, lane);
    for (;;) {
        int64_t n_of[kTiles];
#pragma unroll
        for (int t = 0; t < kTiles; ++t) n_of[t] = job * kJob + t * kTile + q;
        v16f acc[kTiles];
#pragma unroll
        for (int t = 0; t < kTiles; ++t)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[t][r] = 0.0f;

        for (int c = 0; c < nc; ++c) {
            wave_sync_lds();              // every lane has taken the previous chunk
            park_chunk(f, area, lane);
            wave_sync_lds();
            // the next fetch is never under a condition: after the last chunk it is the first chunk of
            // the wave's next 64 queries (rows past N clamp, so a wave without a next job reads row N - 1)
            const bool last = c + 1 == nc;
            const uint32_t *from[kTiles][2];
#pragma unroll
            for (int t = 0; t < kTiles; ++t)
#pragma unroll
                for (int e = 0; e < 2; ++e) from[t][e] = last ? rows_next[t][e] : rows[t][e];
            fetch_chunk(f, from, last ? 0 : c + 1, s0, W, lane);
            __builtin_amdgcn_sched_barrier(0);   // the loads go out before the MFMAs of this chunk, not after
            RowChunk x;
            take_chunk(x, area, q, h);
            run_chunk(x, cl + (size_t)c * kChunk * kSlots, acc);
        }

#pragma unroll
        for (int t = 0; t < kTiles; ++t) {
            // the key takes 2048 * dot off
            int dot[16];
#pragma unroll
            for (int r = 0; r < 16; ++r) dot[r] = (int)acc[t][r];
            int key = INT_MAX;
#pragma unroll
            for (int r = 0; r < 16; ++r) key = min(key, base[r] - (dot[r] << 11));
            key = min(key, __shfl_xor(key, 32, kWave));
            if (h == (t & 1) && n_of[t] < N) pred[n_of[t]] = key & 1023;
            if (kDist) {
                int popc_x = 0;
#pragma unroll
                for (int r = 0; r < 16; ++r) popc_x += slot[r] == kOnes ? dot[r] : 0;
                popc_x += __shfl_xor(popc_x, 32, kWave);
                if (n_of[t] < N) {
#pragma unroll
                    for (int r = 0; r < 16; ++r)
                        if (slot[r] < C)
                            dist[n_of[t] * C + slot[r]] = (uint32_t)(popc_x + (base[r] >> 10) - 2 * dot[r]);
                }
            }
        }
        job += stride;
        if (job >= jobs) break;
#pragma unroll
        for (int t = 0; t < kTiles; ++t)
#pragma unroll
            for (int e = 0; e < 2; ++e) rows[t][e] = rows_next[t][e];
        rows_of(job + stride, rows_next);
    }
}

constexpr int64_t kMfmaQueries = 32768;   // from here on there is a job for most waves of the chip

// Takes the search if it is of the shape this kernel is for; returns false otherwise.
bool try_search_mfma(hdc_ctx_impl *c, const uint32_t *hv, int64_t N, const uint32_t *class_hv,
                     uint32_t *dist, int32_t *pred, hipStream_t s, int *rc) {
    const int C = c->p.C, W = c->W;
    if (N < kMfmaQueries || C < 7 || C > kOnes || W < 4) return false;
    const int steps = (W + 1) / 2;
    const int spad = (steps + kChunk - 1) / kChunk * kChunk;
    const size_t lds = ((size_t)2 * spad * kSlots + kSlots) * 4 + (size_t)kMfmaWaves * kWaveBytes;
    if (lds > 160 * 1024) return false;   // D up to about 19000
    *rc = [&]() -> int {
        const void *kern = dist ? reinterpret_cast<const void *>(search_mfma_kernel<true>)
                                : reinterpret_cast<const void *>(search_mfma_kernel<false>);
        if (lds > 64 * 1024)
            HDC_HIP(hipFuncSetAttribute(kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
        const int64_t jobs = (N + kJob - 1) / kJob;
        const int64_t blocks = std::min<int64_t>(256, (jobs + kMfmaWaves - 1) / kMfmaWaves);
        {
            ProfScope prof(c, HDC_K_SEARCH, s);
            if (dist)
                hipLaunchKernelGGL(search_mfma_kernel<true>, dim3((unsigned)blocks), dim3(kMfmaWaves * kWave), lds, s,
                                   hv, N, class_hv, C, W, c->p.D, spad, dist, pred);
            else
                hipLaunchKernelGGL(search_mfma_kernel<false>, dim3((unsigned)blocks), dim3(kMfmaWaves * kWave), lds, s,
                                   hv, N, class_hv, C, W, c->p.D, spad, dist, pred);
        }
        HDC_HIP(hipGetLastError());
        return HDC_OK;
    }();
    return true;
}

}  // namespace hdc
