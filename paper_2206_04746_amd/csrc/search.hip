// Hamming-distance inference (arXiv 2206.04746, Sec. III): dist[n][c] = popcount(hv[n] XOR
// class_hv[c]) summed over the words of a row, pred[n] = nearest class (lowest index on ties).
// This is the paper's "horizontal summation" (Sec. IV-B2); v_bcnt_u32_b32 adds the popcount
// of a word straight into a 32-bit accumulator, so no narrow partial accumulators are needed.
//
// Layout of the work: a wave streams kRows query rows at a time, lane l holding words
// l, l+64, ... of each row (coalesced 256-byte reads).  The class vectors sit in LDS; for a
// group of kGroup classes every lane forms its partial distance for (row, class).  The
// kRows*kGroup = 64 values are reduced over the 64 lanes in two stages: two DPP adds fold
// each quad of lanes, then the 16 quad sums of every value go through LDS once (stride 17,
// conflict-free) and lane v adds up the 16 partials of value v - a few ops per (row, class)
// instead of a full 6-step cross-lane reduction for each.
#include "hdc_internal.h"

namespace hdc {

constexpr int kSearchWaves = 4;
constexpr int kRows = 4;      // query rows a wave handles at a time
constexpr int kGroup = 16;    // classes per reduction round; kRows * kGroup == 64

constexpr int kXchStride = 17;
constexpr int kXchWords = kWave * kXchStride;

// lane i gets `v` from lane i^1 (quad_perm 1,0,3,2) or i^2 (quad_perm 2,3,0,1)
__device__ __forceinline__ uint32_t quad_xor1(uint32_t v) {
    return (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0xB1, 0xF, 0xF, true);
}
__device__ __forceinline__ uint32_t quad_xor2(uint32_t v) {
    return (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x4E, 0xF, 0xF, true);
}

// Dynamic LDS: class vectors [C][Wl] (Wl = words per lane * 64, pad words zero), then per
// wave a [64][17] exchange area.
template <int WPL>
__global__ __launch_bounds__(kSearchWaves * kWave) void search_kernel(
    const uint32_t *__restrict__ hv, int64_t N, const uint32_t *__restrict__ class_hv, int C, int W,
    uint32_t *__restrict__ dist, int32_t *__restrict__ pred) {
    extern __shared__ uint32_t smem[];
    constexpr int Wl = WPL * kWave;
    uint32_t *cls = smem;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int lane = threadIdx.x & (kWave - 1);
    uint32_t *xch = smem + (size_t)C * Wl + wave * kXchWords;

    for (int i = threadIdx.x; i < C * Wl; i += kSearchWaves * kWave) {
        const int c = i / Wl, w = i - c * Wl;
        cls[i] = w < W ? class_hv[(int64_t)c * W + w] : 0u;
    }
    __syncthreads();

    const int64_t tiles = (N + kRows - 1) / kRows;
    const int r_of = lane / kGroup;   // which of the kRows rows this lane finalises
    const int g_of = lane % kGroup;   // which class of the group
    for (int64_t t = (int64_t)blockIdx.x * kSearchWaves + wave; t < tiles;
         t += (int64_t)gridDim.x * kSearchWaves) {
        const int64_t n0 = t * kRows;
        uint32_t x[kRows][WPL];
#pragma unroll
        for (int r = 0; r < kRows; ++r) {
            const int64_t n = (n0 + r < N) ? n0 + r : N - 1;
            const uint32_t *row = hv + n * W;
#pragma unroll
            for (int j = 0; j < WPL; ++j) {
                const int w = lane + j * kWave;
                x[r][j] = w < W ? row[w] : 0u;
            }
        }
        uint32_t best_key = 0xffffffffu;
        for (int c0 = 0; c0 < C; c0 += kGroup) {
            const int gcount = min(kGroup, C - c0);
            for (int g = 0; g < gcount; ++g) {
                const uint32_t *m = cls + (size_t)(c0 + g) * Wl + lane;
                uint32_t part[kRows];
#pragma unroll
                for (int r = 0; r < kRows; ++r) part[r] = 0;
#pragma unroll
                for (int j = 0; j < WPL; ++j) {
                    const uint32_t mw = m[j * kWave];
#pragma unroll
                    for (int r = 0; r < kRows; ++r) part[r] += __popc(x[r][j] ^ mw);
                }
#pragma unroll
                for (int r = 0; r < kRows; ++r) {
                    uint32_t v = part[r];
                    v += quad_xor1(v);
                    v += quad_xor2(v);
                    if ((lane & 3) == 0) xch[(r * kGroup + g) * kXchStride + (lane >> 2)] = v;
                }
            }
            // lane v = r*kGroup + g sums the 16 quad sums of value v.  Writer and reader are
            // the same wave, whose LDS accesses execute in program order: the fences only
            // stop the compiler from moving the reads above the writes (and the next
            // round's writes above these reads).
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
                const uint32_t key = (total << 10) | (uint32_t)cidx;   // D < 2^21, C <= 1024
                best_key = min(best_key, key);
            }
        }
        // minimum over the kGroup lanes of each row; the key orders by distance, then class
#pragma unroll
        for (int sft = 1; sft < kGroup; sft <<= 1)
            best_key = min(best_key, (uint32_t)__shfl_xor((int)best_key, sft, kWave));
        if (g_of == 0 && n0 + r_of < N) pred[n0 + r_of] = (int32_t)(best_key & 1023u);
    }
}

// Few queries: the kernel above would fill only a fraction of the chip (one tile of kRows rows per
// wave, every block first staging all class vectors in LDS).  Here a block takes ONE tile and
// its kSearchWaves waves split the classes between them, reading the class words straight from
// global memory (the class vectors are a few tens of KB: cache hits after the first blocks).
// The arithmetic and the reduction inside a wave are those of search_kernel; the waves' best keys
// meet in LDS.
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
#pragma unroll
    for (int r = 0; r < kRows; ++r) {
        const int64_t n = (n0 + r < N) ? n0 + r : N - 1;
        const uint32_t *row = hv + n * W;
#pragma unroll
        for (int j = 0; j < WPL; ++j) {
            const int w = lane + j * kWave;
            x[r][j] = w < W ? row[w] : 0u;
        }
    }
    uint32_t best_key = 0xffffffffu;
    for (int c0 = c_lo; c0 < c_hi; c0 += kGroup) {
        const int gcount = min(kGroup, c_hi - c0);
        for (int g = 0; g < gcount; ++g) {
            const uint32_t *m = class_hv + (int64_t)(c0 + g) * W;
            uint32_t part[kRows];
#pragma unroll
            for (int r = 0; r < kRows; ++r) part[r] = 0;
#pragma unroll
            for (int j = 0; j < WPL; ++j) {
                const int w = lane + j * kWave;
                const uint32_t mw = w < W ? m[w] : 0u;
#pragma unroll
                for (int r = 0; r < kRows; ++r) part[r] += __popc(x[r][j] ^ mw);
            }
#pragma unroll
            for (int r = 0; r < kRows; ++r) {
                uint32_t v = part[r];
                v += quad_xor1(v);
                v += quad_xor2(v);
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

constexpr int64_t kFewQueries = 8192;   // below this the one-tile-per-block kernel is used

template <int WPL>
static int launch_search_wpl(hdc_ctx_impl *c, const uint32_t *hv, int64_t N, const uint32_t *class_hv,
                             uint32_t *dist, int32_t *pred, hipStream_t s) {
    if (N < kFewQueries) {
        ProfScope prof(c, HDC_K_SEARCH, s);
        hipLaunchKernelGGL(search_few_kernel<WPL>, dim3((unsigned)((N + kRows - 1) / kRows)),
                           dim3(kSearchWaves * kWave), 0, s, hv, N, class_hv, c->p.C, c->W, dist, pred);
        HDC_HIP(hipGetLastError());
        return HDC_OK;
    }
    const size_t lds = ((size_t)c->p.C * WPL * kWave + (size_t)kSearchWaves * kXchWords) * 4;
    if (lds > 160 * 1024) return HDC_ELIMIT;
    auto kern = search_kernel<WPL>;
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
    return HDC_ELIMIT;   // D > 32768
}

}  // namespace hdc
