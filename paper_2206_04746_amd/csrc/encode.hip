// ID-Level encoding (arXiv 2206.04746, Sec. III, Eq. 1) for gfx950:
//   hv[n][d] = majority_f( item[f][d] XOR level[bin(x[n][f])][d] ).
//
// Two kernels per chunk of samples:
//   quantize_kernel  features -> one bin index byte per (sample, feature)   (HBM-bound, tiny)
//   encode_kernel    bind + bundle + majority + pack                        (VALU-bound)
//
// encode_kernel keeps the per-dimension vote counts bit-sliced: a lane owns one 32-bit word
// column (32 dimensions) and holds the count of every dimension as P bit planes, plane i
// carrying bit i of all 32 counts.  Adding two bound words to a plane is one full adder =
// two v_bitop3_b32 (sum, carry), so a feature costs one XOR (bind) plus about one full adder
// (bundle).  The counters start at a bias chosen so that the top plane of the final count IS
// the majority bit; ties cannot occur because the device item table carries the tie vector
// as an extra vote whenever the number of features is even.
#include "hdc_internal.h"

namespace hdc {

// ---------------------------------------------------------------- bin index (Sec. III)
// fp32: t = (x - lo) * scale with two separately rounded operations, floor, clamp to
// [0, L-1]; anything not >= 0 (negative, NaN) -> 0.   u8: (x * L) >> 8.
__device__ __forceinline__ uint32_t bin_f32(float x, float lo, float scale, int L) {
    float t = __fmul_rn(__fsub_rn(x, lo), scale);
    if (!(t >= 0.0f)) return 0u;
    if (t >= (float)L) return (uint32_t)(L - 1);
    return (uint32_t)(int)t;
}

// One thread produces the four bin bytes of features 4g..4g+3 of one sample; features at
// or beyond F (the tie-vote row and the pad rows of the device item table) get bin 0.
template <bool kU8>
__global__ __launch_bounds__(256) void quantize_kernel(const void *__restrict__ feats, int64_t N,
                                                        int F, int Fp, int L,
                                                        const float *__restrict__ lo,
                                                        const float *__restrict__ scale,
                                                        uint32_t *__restrict__ q4) {
    const int groups = Fp >> 2;
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= N * groups) return;
    const int64_t n = i / groups;
    const int f0 = (int)(i - n * groups) << 2;
    uint32_t packed = 0;
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        const int f = f0 + k;
        uint32_t b = 0;
        if (f < F) {
            if (kU8) {
                b = ((uint32_t) reinterpret_cast<const uint8_t *>(feats)[n * F + f] * (uint32_t)L) >> 8;
            } else {
                b = bin_f32(reinterpret_cast<const float *>(feats)[n * F + f], lo[f], scale[f], L);
            }
        }
        packed |= b << (8 * k);
    }
    q4[i] = packed;
}

// ------------------------------------------------------------- bundling (Eq. 1's sum)
// Adds the 2^LV bound words of features J0 .. J0+2^LV-1 into planes 0..LV-1 and returns the
// carry of weight 2^LV.  Depth-first, so only one pending carry per level is alive.
template <int LV, int J0>
struct Tree {
    static __device__ __forceinline__ uint32_t run(uint32_t *pl, const uint32_t *id,
                                                   const uint32_t *lv_lane, const uint32_t *qw) {
        const uint32_t a = Tree<LV - 1, J0>::run(pl, id, lv_lane, qw);
        const uint32_t b = Tree<LV - 1, J0 + (1 << (LV - 1))>::run(pl, id, lv_lane, qw);
        const uint32_t p = pl[LV - 1];
        pl[LV - 1] = xor3(p, a, b);
        return maj3(p, a, b);
    }
};
template <int J0>
struct Tree<1, J0> {
    static __device__ __forceinline__ uint32_t bound(const uint32_t *id, const uint32_t *lv_lane,
                                                     const uint32_t *qw, int j) {
        const uint32_t bin = (qw[j >> 2] >> (8 * (j & 3))) & 0xffu;   // wave-uniform
        return id[j] ^ lv_lane[bin * kSliceWords];                     // bind (XOR)
    }
    static __device__ __forceinline__ uint32_t run(uint32_t *pl, const uint32_t *id,
                                                   const uint32_t *lv_lane, const uint32_t *qw) {
        const uint32_t x0 = bound(id, lv_lane, qw, J0);
        const uint32_t x1 = bound(id, lv_lane, qw, J0 + 1);
        const uint32_t p = pl[0];
        pl[0] = xor3(p, x0, x1);
        return maj3(p, x0, x1);
    }
};

typedef const uint32_t __attribute__((address_space(4))) *const_u32_ptr;
constexpr int kEncodeWaves = 4;   // waves per block of encode_kernel

// Block = kEncodeWaves waves, all on the same slice of 64 word columns (one column per lane);
// each wave carries S samples through all Fp features.  Dynamic LDS: level[L][64].
template <int S, int P>
__global__ __launch_bounds__(kEncodeWaves * kWave) void encode_kernel(const uint8_t *__restrict__ q,
                                                      const uint32_t *__restrict__ item,
                                                      const uint32_t *__restrict__ level,
                                                      uint32_t *__restrict__ hv, int N, int Fp, int L,
                                                      int W, int Wp, uint32_t bias) {
    extern __shared__ uint32_t lv[];
    const int slice = blockIdx.x;
    const int tile = blockIdx.y;
    const int lane = threadIdx.x & (kWave - 1);
    const int col = slice * kSliceWords + lane;

    for (int i = threadIdx.x; i < L * kSliceWords; i += kEncodeWaves * kWave)
        lv[i] = level[(int64_t)(i >> 6) * Wp + slice * kSliceWords + (i & 63)];
    __syncthreads();

    // kEncodeWaves is a compile-time constant on purpose: a block size read from the dispatch
    // packet makes the compiler treat the sample index as divergent and the bin loads as vector.
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int n_base = (tile * kEncodeWaves + wave) * S;
    if (n_base >= N) return;

    uint32_t pl[S][P];
#pragma unroll
    for (int s = 0; s < S; ++s)
#pragma unroll
        for (int i = 0; i < P; ++i) pl[s][i] = ((bias >> i) & 1u) ? 0xffffffffu : 0u;

    // The bin bytes are wave-uniform and were written by an earlier kernel: read them through
    // the constant address space so they arrive by scalar loads, off the vector pipeline.
    const_u32_ptr qrow[S];
#pragma unroll
    for (int s = 0; s < S; ++s) {
        const int n = min(n_base + s, N - 1);   // a ragged last wave recomputes row N-1
        qrow[s] = (const_u32_ptr)(uintptr_t)(q + (int64_t)n * Fp);
    }
    const uint32_t *lv_lane = lv + lane;

    for (int f0 = 0; f0 < Fp; f0 += kFeatBlock) {
        uint32_t id[kFeatBlock];
#pragma unroll
        for (int j = 0; j < kFeatBlock; ++j) {
            const uint32_t *row = item + (int64_t)(f0 + j) * Wp;   // uniform base, lane offset
            id[j] = row[col];
        }
#pragma unroll
        for (int s = 0; s < S; ++s) {
            uint32_t qw[kFeatBlock / 4];
#pragma unroll
            for (int k = 0; k < kFeatBlock / 4; ++k) qw[k] = qrow[s][(f0 >> 2) + k];
            uint32_t c = Tree<5, 0>::run(pl[s], id, lv_lane, qw);   // carry of weight 32
#pragma unroll
            for (int i = 5; i < P; ++i) {                            // ripple it upward
                const uint32_t t = pl[s][i] & c;
                pl[s][i] ^= c;
                c = t;
            }
        }
    }

    if (col < W) {
#pragma unroll
        for (int s = 0; s < S; ++s)
            if (n_base + s < N) hv[(int64_t)(n_base + s) * W + col] = pl[s][P - 1];
    }
}

template <int S, int P>
static int launch_encode_sp(hdc_ctx_impl *c, int N, uint32_t *hv, uint32_t bias, hipStream_t s) {
    const int nslices = c->Wp / kSliceWords;
    const int waves = kEncodeWaves;
    const int tiles = (N + waves * S - 1) / (waves * S);
    const size_t lds = (size_t)c->p.L * kSliceWords * sizeof(uint32_t);
    hipLaunchKernelGGL((encode_kernel<S, P>), dim3((unsigned)nslices, (unsigned)tiles), dim3(waves * kWave), lds, s,
                       c->q_d, c->item_d, c->level_d, hv, N, c->Fp, c->p.L, c->W, c->Wp, bias);
    return HDC_OK;
}

int launch_encode(hdc_ctx_impl *c, const void *feats, int64_t N, uint32_t *hv, hipStream_t s) {
    // Majority of `votes` (odd) inputs: count >= thr.  With P-1 = ceil(log2(thr)) and the
    // counters starting at 2^(P-1) - thr, bit P-1 of the final count is the answer and the
    // count never reaches 2^P.
    const uint32_t thr = ((uint32_t)c->votes + 1u) / 2u;
    int top = 0;
    while ((1u << top) < thr) ++top;
    int P = top + 1;
    P = P <= 6 ? 6 : P <= 8 ? 8 : P <= 10 ? 10 : P <= 12 ? 12 : 16;
    const uint32_t bias = (1u << (P - 1)) - thr;

    for (int64_t n0 = 0; n0 < N; n0 += c->q_rows) {
        const int64_t n = (N - n0 < c->q_rows) ? N - n0 : c->q_rows;
        const size_t esz = c->p.feat_dtype == HDC_U8 ? 1 : 4;
        const void *x = reinterpret_cast<const uint8_t *>(feats) + (size_t)n0 * c->p.F * esz;
        const int64_t items = n * (c->Fp >> 2);
        const unsigned qblocks = (unsigned)((items + 255) / 256);
        if (c->p.feat_dtype == HDC_U8)
            hipLaunchKernelGGL(quantize_kernel<true>, dim3(qblocks), dim3(256), 0, s, x, n, c->p.F,
                               c->Fp, c->p.L, c->lo_d, c->scale_d, reinterpret_cast<uint32_t *>(c->q_d));
        else
            hipLaunchKernelGGL(quantize_kernel<false>, dim3(qblocks), dim3(256), 0, s, x, n, c->p.F,
                               c->Fp, c->p.L, c->lo_d, c->scale_d, reinterpret_cast<uint32_t *>(c->q_d));
        uint32_t *out = hv + (size_t)n0 * c->W;
        switch (P) {
            case 6: launch_encode_sp<4, 6>(c, (int)n, out, bias, s); break;
            case 8: launch_encode_sp<4, 8>(c, (int)n, out, bias, s); break;
            case 10: launch_encode_sp<4, 10>(c, (int)n, out, bias, s); break;
            case 12: launch_encode_sp<4, 12>(c, (int)n, out, bias, s); break;
            default: launch_encode_sp<4, 16>(c, (int)n, out, bias, s); break;
        }
        HDC_HIP(hipGetLastError());
    }
    return HDC_OK;
}

}  // namespace hdc
