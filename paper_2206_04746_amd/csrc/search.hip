// Hamming-distance inference (arXiv 2206.04746, Sec. III): dist[n][c] = popcount(hv[n] XOR
// class_hv[c]) summed over the words of a row, pred[n] = nearest class (lowest index on ties).
// This is the paper's "horizontal summation" (Sec. IV-B2); v_bcnt_u32_b32 adds the popcount
// of a word straight into a 32-bit accumulator, so no narrow partial accumulators are needed.
//
// Layout of the work: a wave streams kRows query rows at a time, lane l holding words
// l, l+64, ... of each row (coalesced 256-byte reads).  The class vectors sit in LDS; for a
// group of G classes every lane forms its partial distance for (row, class): kRows*G values
// per lane, each to be summed over the 64 lanes.  They are summed together, halving the number
// of live values at every step: at the step for lane bit b, value i keeps going in the lanes
// whose bit b is clear, value i + n/2 in the others, each lane adding what its partner (lane ^
// 2^b) holds of the value it keeps.  For bits 5 and 4 that is one v_permlane32_swap /
// v_permlane16_swap (new in gfx950: two registers trade half of their rows) plus one add per
// PAIR of values; for bits 3..0 two DPP adds and a select per pair.  When one value is left the
// remaining bits are plain folds.  About 2.5 ops per value instead of a 6-step reduction each;
// lane l ends up with the total of value l >> (6 - log2(kRows*G)).
#include "hdc_internal.h"

namespace hdc {

constexpr int kSearchWaves = 4;
constexpr int kRows = 4;      // query rows a wave handles at a time

// acc + popcount(x) in one instruction.  Written out because the compiler, given __popc(x) + acc
// in a chain, counts every word against zero and adds the counts up with extra instructions.
__device__ __forceinline__ uint32_t bcnt_acc(uint32_t x, uint32_t acc) {
    uint32_t r;
    asm("v_bcnt_u32_b32 %0, %1, %2" : "=v"(r) : "v"(x), "v"(acc));
    return r;
}

template <int CTRL>
__device__ __forceinline__ uint32_t dpp(uint32_t v) {
    return (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, CTRL, 0xF, 0xF, true);
}
// what lane ^ 2^BIT holds of v, BIT = 3..0
template <int BIT>
__device__ __forceinline__ uint32_t partner(uint32_t v) {
    if (BIT == 3) return dpp<0x128>(v);                                          // row_ror:8
    if (BIT == 2) return (uint32_t)__builtin_amdgcn_ds_swizzle((int)v, 0x101F);  // swap groups of 4 lanes
    if (BIT == 1) return dpp<0x4E>(v);                                           // quad_perm 2,3,0,1
    return dpp<0xB1>(v);                                                         // quad_perm 1,0,3,2
}

// The steps for lane bits BIT..0 on n live values.
template <int BIT, int NV>
struct FoldLow {
    static __device__ __forceinline__ uint32_t run(uint32_t *v, int lane) {
        if (NV > 1) {
            constexpr int H = NV > 1 ? NV / 2 : 1;
            const bool upper = (lane >> BIT) & 1;
#pragma unroll
            for (int i = 0; i < H; ++i) {
                const uint32_t a = v[i] + partner<BIT>(v[i]);
                const uint32_t b = v[i + H] + partner<BIT>(v[i + H]);
                v[i] = upper ? b : a;
            }
            return FoldLow<BIT - 1, H>::run(v, lane);
        } else {
            v[0] += partner<BIT>(v[0]);
            return FoldLow<BIT - 1, 1>::run(v, lane);
        }
    }
};
template <int NV>
struct FoldLow<-1, NV> {
    static __device__ __forceinline__ uint32_t run(uint32_t *v, int) { return v[0]; }
};

// Sums each of the NV >= 4 values over the wave; lane l returns the total of value l >> (6 - log2 NV).
template <int NV>
__device__ __forceinline__ uint32_t fold_values(uint32_t (&v)[NV], int lane) {
    static_assert(NV >= 4 && NV <= 64 && (NV & (NV - 1)) == 0, "a power of two between 4 and 64");
    constexpr int H = NV / 2, Q = NV / 4;
#pragma unroll
    for (int i = 0; i < H; ++i) {   // lane bit 5: lanes 32..63 of v[i] trade places with lanes 0..31 of v[i + H]
        const auto r = __builtin_amdgcn_permlane32_swap(v[i], v[i + H], false, false);
        v[i] = r[0] + r[1];
    }
#pragma unroll
    for (int i = 0; i < Q; ++i) {   // lane bit 4: odd rows of 16 lanes of v[i] trade places with even rows of v[i + Q]
        const auto r = __builtin_amdgcn_permlane16_swap(v[i], v[i + Q], false, false);
        v[i] = r[0] + r[1];
    }
    return FoldLow<3, Q>::run(v, lane);
}

// minimum over the 16 lanes of a row (kRows == 4: each query row owns one row of lanes)
__device__ __forceinline__ uint32_t row_min(uint32_t k) {
    k = min(k, dpp<0x128>(k));
    k = min(k, dpp<0x124>(k));
    k = min(k, dpp<0x122>(k));
    return min(k, dpp<0x121>(k));
}

// This lane's words of kRows query rows starting at row n0 (rows past N repeat row N - 1, columns
// past W read as zero).  Clamped addresses and a select instead of a branch around each load: all
// loads are in flight together.
template <int WPL, bool kStream>
__device__ __forceinline__ void load_rows(const uint32_t *__restrict__ hv, int64_t n0, int64_t N, int W, int lane,
                                          uint32_t (&x)[kRows][WPL]) {
#pragma unroll
    for (int r = 0; r < kRows; ++r) {
        const int64_t n = (n0 + r < N) ? n0 + r : N - 1;
        const uint32_t *row = hv + n * W;
#pragma unroll
        for (int j = 0; j < WPL; ++j) {
            const int w = lane + j * kWave;
            const uint32_t v = kStream ? __builtin_nontemporal_load(row + (w < W ? w : W - 1)) : row[w < W ? w : W - 1];
            x[r][j] = w < W ? v : 0u;
        }
    }
}

// Distances of the wave's kRows rows to the classes c0 .. c0 + G - 1 (those below c_end), totals as
// fold_values leaves them.  word(c, j) is class c's word for this lane's j-th column.
template <int WPL, int G, typename WordFn>
__device__ __forceinline__ uint32_t group_totals(const uint32_t (&x)[kRows][WPL], int c0, int c_end, int lane,
                                                 WordFn word) {
    uint32_t v[kRows * G];
#pragma unroll
    for (int g = 0; g < G; ++g) {
        uint32_t part[kRows];
#pragma unroll
        for (int r = 0; r < kRows; ++r) part[r] = 0;
        if (c0 + g < c_end) {   // wave-uniform
#pragma unroll
            for (int j = 0; j < WPL; ++j) {
                const uint32_t mw = word(c0 + g, j);
#pragma unroll
                for (int r = 0; r < kRows; ++r) part[r] = bcnt_acc(x[r][j] ^ mw, part[r]);
            }
        }
#pragma unroll
        for (int r = 0; r < kRows; ++r) v[r * G + g] = part[r];
    }
    return fold_values<kRows * G>(v, lane);
}

template <int G>
struct Owner {   // which (row, class of the group) a lane finalises, and whether it is the one that writes
    static constexpr int kShift = G == 16 ? 0 : G == 8 ? 1 : G == 4 ? 2 : G == 2 ? 3 : 4;
    int r_of, g_of;
    bool writes;
    __device__ __forceinline__ explicit Owner(int lane) {
        const int idx = lane >> kShift;
        r_of = idx / G;
        g_of = idx % G;
        writes = (lane & ((1 << kShift) - 1)) == 0;
    }
};

// Dynamic LDS: class vectors [C][Wl] (Wl = words per lane * 64, pad words zero).
template <int WPL, int G>
__global__ __launch_bounds__(kSearchWaves * kWave) void search_kernel(
    const uint32_t *__restrict__ hv, int64_t N, const uint32_t *__restrict__ class_hv, int C, int W,
    uint32_t *__restrict__ dist, int32_t *__restrict__ pred) {
    extern __shared__ uint32_t cls[];
    constexpr int Wl = WPL * kWave;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int lane = threadIdx.x & (kWave - 1);

    for (int i = threadIdx.x; i < C * Wl; i += kSearchWaves * kWave) {
        const int c = i / Wl, w = i - c * Wl;
        cls[i] = w < W ? class_hv[(int64_t)c * W + w] : 0u;
    }
    __syncthreads();

    const int64_t tiles = (N + kRows - 1) / kRows;
    const Owner<G> own(lane);
    for (int64_t t = (int64_t)blockIdx.x * kSearchWaves + wave; t < tiles;
         t += (int64_t)gridDim.x * kSearchWaves) {
        const int64_t n0 = t * kRows;
        uint32_t x[kRows][WPL];
        load_rows<WPL, true>(hv, n0, N, W, lane, x);   // a million queries pass once: not worth caching
        uint32_t best_key = 0xffffffffu;
        for (int c0 = 0; c0 < C; c0 += G) {
            const uint32_t total = group_totals<WPL, G>(
                x, c0, C, lane, [&](int c, int j) { return cls[(size_t)c * Wl + j * kWave + lane]; });
            const int cidx = c0 + own.g_of;
            const int64_t n = n0 + own.r_of;
            if (cidx < C && n < N) {
                if (dist && own.writes) dist[n * C + cidx] = total;
                const uint32_t key = (total << 10) | (uint32_t)cidx;   // D < 2^21, C <= 1024
                best_key = min(best_key, key);
            }
        }
        // minimum over the lanes of each row; the key orders by distance, then class
        best_key = row_min(best_key);
        if ((lane & 15) == 0 && n0 + own.r_of < N) pred[n0 + own.r_of] = (int32_t)(best_key & 1023u);
    }
}

// ---- a row per 16 lanes --------------------------------------------------------------------
// Second layout for long streams of queries, taken when a row fills 16 lanes well: lane i of a
// row's 16 lanes holds the 16-byte pieces i, i + 16, ... of the row (KPL pieces), so a wave still
// streams kRows rows at a time, now with 16-byte loads, and every lane works for ONE row.  A
// partial distance then has to be summed over 16 lanes instead of 64, and a lane carries G values
// instead of kRows * G: the fold costs about a quarter of what it costs in search_kernel, which
// is what bounds that kernel from about ten classes on.  The price is in LDS traffic: the class
// words are read per row, i.e. four times per wave (16-byte reads, the four rows reading the same
// addresses).
//
// Rows are 4-byte aligned only and the last piece of a row may be short; a lane whose piece
// would cross the end of the row reads the row's LAST 16 bytes instead and keeps the words that
// belong to its own piece (none, for a piece wholly past the end), so no read leaves the row.
// The class vectors are staged in LDS in the same piece order, with zeros where a lane keeps
// nothing.  Needs W >= 4.
typedef uint32_t u32x4_a4 __attribute__((ext_vector_type(4), aligned(4)));   // a piece in a row
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));                  // a piece in LDS (16-byte aligned)

constexpr int kRowLanes = kWave / kRows;   // 16

// first word the lane's piece `piece` is read from, and which of the four words it keeps
__device__ __forceinline__ int piece_start(int piece, int W) { return 4 * piece + 3 < W ? 4 * piece : W - 4; }
__device__ __forceinline__ bool piece_keeps(int piece, int start, int j, int W) {
    return start + j >= 4 * piece && start + j < W && start + j < 4 * piece + 4;
}

template <int KPL, int G>
__global__ __launch_bounds__(kSearchWaves * kWave) void search_rows16_kernel(
    const uint32_t *__restrict__ hv, int64_t N, const uint32_t *__restrict__ class_hv, int C, int W,
    uint32_t *__restrict__ dist, int32_t *__restrict__ pred) {
    extern __shared__ uint32_t cls[];    // [C][KPL][16 lanes][4 words]
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int lane = threadIdx.x & (kWave - 1);
    const int i = lane & (kRowLanes - 1), r = lane / kRowLanes;

    for (int idx = threadIdx.x; idx < C * KPL * kWave; idx += kSearchWaves * kWave) {
        const int c = idx / (KPL * kWave), rem = idx - c * (KPL * kWave);
        const int piece = (rem >> 2) % kRowLanes + kRowLanes * (rem / kWave), j = rem & 3;
        const int start = piece_start(piece, W);
        cls[idx] = piece_keeps(piece, start, j, W) ? class_hv[(int64_t)c * W + start + j] : 0u;
    }
    __syncthreads();

    // only the lane's last piece can be short or past the end
    constexpr int kLast = KPL - 1;
    const int last_piece = i + kRowLanes * kLast;
    const int last_start = piece_start(last_piece, W);
    uint32_t keep[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) keep[j] = piece_keeps(last_piece, last_start, j, W) ? 0xffffffffu : 0u;

    constexpr int kShift = G == 16 ? 0 : G == 8 ? 1 : G == 4 ? 2 : 3;   // lane i ends with value i >> kShift
    const int g_of = i >> kShift;
    const bool writes = (i & ((1 << kShift) - 1)) == 0;
    const u32x4 *cls4 = reinterpret_cast<const u32x4 *>(cls);

    const int64_t tiles = (N + kRows - 1) / kRows;
    for (int64_t t = (int64_t)blockIdx.x * kSearchWaves + wave; t < tiles;
         t += (int64_t)gridDim.x * kSearchWaves) {
        const int64_t n = t * kRows + r;
        const uint32_t *row = hv + (n < N ? n : N - 1) * W;
        u32x4_a4 x[KPL];
#pragma unroll
        for (int k = 0; k < kLast; ++k)
            x[k] = __builtin_nontemporal_load(reinterpret_cast<const u32x4_a4 *>(row + 4 * (i + kRowLanes * k)));
        x[kLast] = __builtin_nontemporal_load(reinterpret_cast<const u32x4_a4 *>(row + last_start));
#pragma unroll
        for (int j = 0; j < 4; ++j) x[kLast][j] &= keep[j];

        uint32_t best_key = 0xffffffffu;
        for (int c0 = 0; c0 < C; c0 += G) {
            uint32_t v[G];
#pragma unroll
            for (int g = 0; g < G; ++g) {
                uint32_t part = 0;
                if (c0 + g < C) {   // wave-uniform
                    const u32x4 *m = cls4 + ((size_t)(c0 + g) * KPL) * kRowLanes + i;
#pragma unroll
                    for (int k = 0; k < KPL; ++k) {
                        const u32x4 mw = m[k * kRowLanes];
#pragma unroll
                        for (int j = 0; j < 4; ++j) part = bcnt_acc(x[k][j] ^ mw[j], part);
                    }
                }
                v[g] = part;
            }
            const uint32_t total = FoldLow<3, G>::run(v, lane);
            const int cidx = c0 + g_of;
            if (cidx < C && n < N) {
                if (dist && writes) dist[n * C + cidx] = total;
                best_key = min(best_key, (total << 10) | (uint32_t)cidx);   // D < 2^21, C <= 1024
            }
        }
        best_key = row_min(best_key);
        if (i == 0 && n < N) pred[n] = (int32_t)(best_key & 1023u);
    }
}

// ---- few queries ----------------------------------------------------------------------------
constexpr int kGroup = 16;    // classes per reduction round of the few-query kernel; kRows * kGroup == 64
constexpr int kXchStride = 17;
constexpr int kXchWords = kWave * kXchStride;

// Few queries: the kernel above would fill only a fraction of the chip (one tile of kRows rows per
// wave, every block first staging all class vectors in LDS).  Here a block takes ONE tile and
// its kSearchWaves waves split the classes between them, reading the class words straight from
// global memory (the class vectors are a few tens of KB: cache hits after the first blocks).
// A launch of this size is over in a few microseconds and runs its code once per block, so the
// code is kept small (a loop over the classes, not the unrolled groups of search_kernel, whose
// instructions alone take longer to fetch on a cold instruction cache than this kernel runs): per
// class two DPP adds fold each quad of lanes, the 16 quad sums of every (row, class) value go
// through LDS once (stride 17, conflict-free) and lane v adds up the 16 partials of value v.  The
// waves' best keys meet in LDS.
template <int WPL>
__global__ __launch_bounds__(kSearchWaves * kWave) void search_few_kernel(
    const uint32_t *__restrict__ hv, int64_t N, const uint32_t *__restrict__ class_hv, int C, int W,
    uint32_t *__restrict__ dist, int32_t *__restrict__ pred) {
    __shared__ uint32_t xch_all[kSearchWaves * kXchWords];
    __shared__ uint32_t keys[kSearchWaves][kRows];
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int lane = threadIdx.x & (kWave - 1);
    uint32_t *xch = xch_all + wave * kXchWords;
    const int r_of = lane / kGroup, g_of = lane % kGroup;
    const int64_t n0 = (int64_t)blockIdx.x * kRows;
    // this wave's classes: a contiguous share
    const int per = (C + kSearchWaves - 1) / kSearchWaves;
    const int c_lo = min(wave * per, C), c_hi = min(c_lo + per, C);

    uint32_t x[kRows][WPL];
    load_rows<WPL, false>(hv, n0, N, W, lane, x);
    uint32_t best_key = 0xffffffffu;
    for (int c0 = c_lo; c0 < c_hi; c0 += kGroup) {
        const int gcount = min(kGroup, c_hi - c0);
        for (int g = 0; g < gcount; ++g) {
            const uint32_t *m = class_hv + (int64_t)(c0 + g) * W;
            uint32_t part[kRows];
#pragma unroll
            for (int r = 0; r < kRows; ++r) part[r] = 0;
            uint32_t mw[WPL];   // clamped addresses and a select: the loads are in flight together
#pragma unroll
            for (int j = 0; j < WPL; ++j) {
                const int w = lane + j * kWave;
                const uint32_t v = m[w < W ? w : W - 1];
                mw[j] = w < W ? v : 0u;
            }
#pragma unroll
            for (int j = 0; j < WPL; ++j)
#pragma unroll
                for (int r = 0; r < kRows; ++r) part[r] = bcnt_acc(x[r][j] ^ mw[j], part[r]);
#pragma unroll
            for (int r = 0; r < kRows; ++r) {
                uint32_t v = part[r];
                v += dpp<0xB1>(v);
                v += dpp<0x4E>(v);
                if ((lane & 3) == 0) xch[(r * kGroup + g) * kXchStride + (lane >> 2)] = v;
            }
        }
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
        uint32_t total = 0;
        if (g_of < gcount) {
            const uint32_t *src = xch + lane * kXchStride;
#pragma unroll
            for (int l = 0; l < kWave / 4; ++l) total += src[l];
        }
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
        const int cidx = c0 + g_of;
        const int64_t n = n0 + r_of;
        if (g_of < gcount && n < N) {
            if (dist) dist[n * C + cidx] = total;
            best_key = min(best_key, (total << 10) | (uint32_t)cidx);
        }
    }
#pragma unroll
    for (int sft = 1; sft < kGroup; sft <<= 1)
        best_key = min(best_key, (uint32_t)__shfl_xor((int)best_key, sft, kWave));
    if (g_of == 0) keys[wave][r_of] = best_key;   // 0xffffffff from a wave without classes
    __syncthreads();
    if (threadIdx.x < kRows && n0 + threadIdx.x < N) {
        uint32_t k = keys[0][threadIdx.x];
#pragma unroll
        for (int w = 1; w < kSearchWaves; ++w) k = min(k, keys[w][threadIdx.x]);
        pred[n0 + threadIdx.x] = (int32_t)(k & 1023u);
    }
}

// Rows too long for a wave's registers (more than 16 words per lane, D > 32768): the shape of
// search_few_kernel - a block per tile of kRows rows, its waves splitting the classes, class words
// from global memory - with the row words read again for every class instead of held in registers.
// Not a fast path: it exists so that no dimension the other entry points take is refused here.
__global__ __launch_bounds__(kSearchWaves * kWave) void search_long_kernel(
    const uint32_t *__restrict__ hv, int64_t N, const uint32_t *__restrict__ class_hv, int C, int W,
    uint32_t *__restrict__ dist, int32_t *__restrict__ pred) {
    __shared__ uint32_t xch_all[kSearchWaves * kXchWords];
    __shared__ uint32_t keys[kSearchWaves][kRows];
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int lane = threadIdx.x & (kWave - 1);
    uint32_t *xch = xch_all + wave * kXchWords;
    const int r_of = lane / kGroup, g_of = lane % kGroup;
    const int64_t n0 = (int64_t)blockIdx.x * kRows;
    const int per = (C + kSearchWaves - 1) / kSearchWaves;
    const int c_lo = min(wave * per, C), c_hi = min(c_lo + per, C);
    const uint32_t *row[kRows];
#pragma unroll
    for (int r = 0; r < kRows; ++r) row[r] = hv + ((n0 + r < N) ? n0 + r : N - 1) * W;

    uint32_t best_key = 0xffffffffu;
    for (int c0 = c_lo; c0 < c_hi; c0 += kGroup) {
        const int gcount = min(kGroup, c_hi - c0);
        for (int g = 0; g < gcount; ++g) {
            const uint32_t *m = class_hv + (int64_t)(c0 + g) * W;
            uint32_t part[kRows];
#pragma unroll
            for (int r = 0; r < kRows; ++r) part[r] = 0;
            for (int w = lane; w < W; w += kWave) {
                const uint32_t mw = m[w];
#pragma unroll
                for (int r = 0; r < kRows; ++r) part[r] = bcnt_acc(row[r][w] ^ mw, part[r]);
            }
#pragma unroll
            for (int r = 0; r < kRows; ++r) {
                uint32_t v = part[r];
                v += dpp<0xB1>(v);
                v += dpp<0x4E>(v);
                if ((lane & 3) == 0) xch[(r * kGroup + g) * kXchStride + (lane >> 2)] = v;
            }
        }
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
        uint32_t total = 0;
        if (g_of < gcount) {
            const uint32_t *src = xch + lane * kXchStride;
#pragma unroll
            for (int l = 0; l < kWave / 4; ++l) total += src[l];
        }
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
        const int cidx = c0 + g_of;
        const int64_t n = n0 + r_of;
        if (g_of < gcount && n < N) {
            if (dist) dist[n * C + cidx] = total;
            best_key = min(best_key, (total << 10) | (uint32_t)cidx);
        }
    }
#pragma unroll
    for (int sft = 1; sft < kGroup; sft <<= 1)
        best_key = min(best_key, (uint32_t)__shfl_xor((int)best_key, sft, kWave));
    if (g_of == 0) keys[wave][r_of] = best_key;
    __syncthreads();
    if (threadIdx.x < kRows && n0 + threadIdx.x < N) {
        uint32_t k = keys[0][threadIdx.x];
#pragma unroll
        for (int w = 1; w < kSearchWaves; ++w) k = min(k, keys[w][threadIdx.x]);
        pred[n0 + threadIdx.x] = (int32_t)(k & 1023u);
    }
}

constexpr int64_t kFewQueries = 8192;   // below this the one-tile-per-block kernel is used

template <int WPL, int G>
static int launch_search_shape(hdc_ctx_impl *c, const uint32_t *hv, int64_t N, const uint32_t *class_hv,
                               uint32_t *dist, int32_t *pred, hipStream_t s) {
    // class vectors too many for LDS: the few-query kernel reads them from global memory and is
    // correct for any number of queries
    const size_t lds = (size_t)c->p.C * WPL * kWave * 4;
    if (N < kFewQueries || lds > 160 * 1024) {
        ProfScope prof(c, HDC_K_SEARCH, s);
        hipLaunchKernelGGL(search_few_kernel<WPL>, dim3((unsigned)((N + kRows - 1) / kRows)),
                           dim3(kSearchWaves * kWave), 0, s, hv, N, class_hv, c->p.C, c->W, dist, pred);
        HDC_HIP(hipGetLastError());
        return HDC_OK;
    }
    auto kern = search_kernel<WPL, G>;
    if (lds > 64 * 1024)
        HDC_HIP(hipFuncSetAttribute(reinterpret_cast<const void *>(kern),
                                    hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
    const int64_t tiles = (N + kRows - 1) / kRows;
    int64_t blocks = (tiles + kSearchWaves - 1) / kSearchWaves;
    if (blocks > 256 * 16) blocks = 256 * 16;   // persistent-style grid, a few blocks per CU
    {
        ProfScope prof(c, HDC_K_SEARCH, s);
        hipLaunchKernelGGL(kern, dim3((unsigned)blocks), dim3(kSearchWaves * kWave), lds, s, hv, N,
                           class_hv, c->p.C, c->W, dist, pred);
    }
    HDC_HIP(hipGetLastError());
    return HDC_OK;
}

// Classes per reduction round: few classes take a narrow group (fewer idle values in the fold, fewer
// registers: measured, 8 beats 16 up to 16 classes); rows of many words per lane take at most 8, to
// keep kRows * G partials plus the rows in registers.
template <int WPL>
static int launch_search_wpl(hdc_ctx_impl *c, const uint32_t *hv, int64_t N, const uint32_t *class_hv,
                             uint32_t *dist, int32_t *pred, hipStream_t s) {
    const int share = c->p.C;
    if (share <= 2) return launch_search_shape<WPL, 2>(c, hv, N, class_hv, dist, pred, s);
    if (share <= 16 || WPL > 6) return launch_search_shape<WPL, 8>(c, hv, N, class_hv, dist, pred, s);
    return launch_search_shape<WPL, 16>(c, hv, N, class_hv, dist, pred, s);
}

template <int KPL, int G>
static int launch_rows16_shape(hdc_ctx_impl *c, const uint32_t *hv, int64_t N, const uint32_t *class_hv,
                               uint32_t *dist, int32_t *pred, hipStream_t s) {
    const size_t lds = (size_t)c->p.C * KPL * kWave * 4;
    auto kern = search_rows16_kernel<KPL, G>;
    if (lds > 64 * 1024)
        HDC_HIP(hipFuncSetAttribute(reinterpret_cast<const void *>(kern),
                                    hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
    const int64_t tiles = (N + kRows - 1) / kRows;
    int64_t blocks = (tiles + kSearchWaves - 1) / kSearchWaves;
    if (blocks > 256 * 16) blocks = 256 * 16;
    {
        ProfScope prof(c, HDC_K_SEARCH, s);
        hipLaunchKernelGGL(kern, dim3((unsigned)blocks), dim3(kSearchWaves * kWave), lds, s, hv, N,
                           class_hv, c->p.C, c->W, dist, pred);
    }
    HDC_HIP(hipGetLastError());
    return HDC_OK;
}

template <int KPL>
static int launch_rows16(hdc_ctx_impl *c, const uint32_t *hv, int64_t N, const uint32_t *class_hv,
                         uint32_t *dist, int32_t *pred, hipStream_t s) {
    if (c->p.C <= 2) return launch_rows16_shape<KPL, 2>(c, hv, N, class_hv, dist, pred, s);
    if (c->p.C <= 8) return launch_rows16_shape<KPL, 8>(c, hv, N, class_hv, dist, pred, s);
    return launch_rows16_shape<KPL, 16>(c, hv, N, class_hv, dist, pred, s);
}

// The row-per-16-lanes kernel when the stream is long, the pieces of a row fill the lanes of an
// instantiated size to 85 % or more, and the class vectors fit in LDS; returns false otherwise.
static bool try_rows16(hdc_ctx_impl *c, const uint32_t *hv, int64_t N, const uint32_t *class_hv,
                       uint32_t *dist, int32_t *pred, hipStream_t s, int *rc) {
    if (N < kFewQueries || c->W < 4) return false;
    const int pieces = (c->W + 3) / 4;
    const int need = (pieces + kRowLanes - 1) / kRowLanes;
    static const int sizes[] = {1, 2, 3, 4, 5, 6, 8, 12, 16};
    int kpl = 0;
    for (int sz : sizes)
        if (sz >= need) { kpl = sz; break; }
    if (!kpl || pieces * 100 < 85 * kRowLanes * kpl) return false;
    if (c->W < 4 * kRowLanes * (kpl - 1)) return false;   // the kernel takes all but a lane's last piece as whole
    if ((size_t)c->p.C * kpl * kWave * 4 > 160 * 1024) return false;
    switch (kpl) {
    case 1: *rc = launch_rows16<1>(c, hv, N, class_hv, dist, pred, s); break;
    case 2: *rc = launch_rows16<2>(c, hv, N, class_hv, dist, pred, s); break;
    case 3: *rc = launch_rows16<3>(c, hv, N, class_hv, dist, pred, s); break;
    case 4: *rc = launch_rows16<4>(c, hv, N, class_hv, dist, pred, s); break;
    case 5: *rc = launch_rows16<5>(c, hv, N, class_hv, dist, pred, s); break;
    case 6: *rc = launch_rows16<6>(c, hv, N, class_hv, dist, pred, s); break;
    case 8: *rc = launch_rows16<8>(c, hv, N, class_hv, dist, pred, s); break;
    case 12: *rc = launch_rows16<12>(c, hv, N, class_hv, dist, pred, s); break;
    default: *rc = launch_rows16<16>(c, hv, N, class_hv, dist, pred, s); break;
    }
    return true;
}

int launch_search(hdc_ctx_impl *c, const uint32_t *hv, int64_t N, const uint32_t *class_hv,
                  uint32_t *dist, int32_t *pred, hipStream_t s) {
    {
        int rc = HDC_OK;
        if (try_search_mfma(c, hv, N, class_hv, dist, pred, s, &rc)) return rc;
        if (try_rows16(c, hv, N, class_hv, dist, pred, s, &rc)) return rc;
    }
    // words per lane, rounded up to an instantiated size (a whole row lives in registers)
    const int wpl = (c->W + kWave - 1) / kWave;
    if (wpl <= 1) return launch_search_wpl<1>(c, hv, N, class_hv, dist, pred, s);
    if (wpl <= 2) return launch_search_wpl<2>(c, hv, N, class_hv, dist, pred, s);
    if (wpl <= 3) return launch_search_wpl<3>(c, hv, N, class_hv, dist, pred, s);
    if (wpl <= 4) return launch_search_wpl<4>(c, hv, N, class_hv, dist, pred, s);
    if (wpl <= 5) return launch_search_wpl<5>(c, hv, N, class_hv, dist, pred, s);
    if (wpl <= 6) return launch_search_wpl<6>(c, hv, N, class_hv, dist, pred, s);
    if (wpl <= 8) return launch_search_wpl<8>(c, hv, N, class_hv, dist, pred, s);
    if (wpl <= 12) return launch_search_wpl<12>(c, hv, N, class_hv, dist, pred, s);
    if (wpl <= 16) return launch_search_wpl<16>(c, hv, N, class_hv, dist, pred, s);
    {   // D > 32768
        ProfScope prof(c, HDC_K_SEARCH, s);
        hipLaunchKernelGGL(search_long_kernel, dim3((unsigned)((N + kRows - 1) / kRows)), dim3(kSearchWaves * kWave), 0,
                           s, hv, N, class_hv, c->p.C, c->W, dist, pred);
    }
    HDC_HIP(hipGetLastError());
    return HDC_OK;
}

}  // namespace hdc
