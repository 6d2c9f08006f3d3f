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

int launch_search(hdc_ctx_impl *c, const uint32_t *hv, int64_t N, const uint32_t *class_hv,
                  uint32_t *dist, int32_t *pred, hipStream_t s) {
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
