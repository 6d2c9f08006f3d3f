// ID-Level encoding (arXiv 2206.04746, Sec. III, Eq. 1) for gfx950:
//   hv[n][d] = majority_f( item[f][d] XOR level[bin(x[n][f])][d] ).
//
// Two kernels per chunk of samples:
//   quantize_kernel  features -> one 16-bit level-row offset per (sample, feature)  (tiny)
//   encode_kernel    bind + bundle + majority + pack                        (VALU-bound)
//
// encode_kernel keeps the per-dimension vote counts bit-sliced: a lane owns one 32-bit word
// column (32 dimensions) and holds the count of every dimension as P bit planes, plane i
// carrying bit i of all 32 counts.  Adding two bound words to a plane is one full adder =
// two v_bitop3_b32 (sum, carry), so a feature costs one XOR (bind) plus about one full adder
// (bundle).  The counters start at a bias chosen so that the top plane of the final count IS
// the majority bit; ties cannot occur because the device item table carries the tie vector
// as an extra vote whenever the number of features is even.
#include "bundle.h"

namespace hdc {

// One thread produces the entries of features 4g..4g+3 for kQuantRows consecutive samples
// (the per-feature range is loaded once and reused down the rows).  An entry is the byte
// offset of the bin's row in the LDS level slice (bin * 256, fits 16 bits for L <= 256);
// features at or beyond F (the tie-vote row and the pad rows of the device item table) get
// bin 0.  grid = (feature groups / 64, row tiles).
constexpr int kQuantRows = 8;
template <bool kU8>
__global__ __launch_bounds__(64) void quantize_kernel(const void *__restrict__ feats, int64_t N,
                                                       int F, int Fp, int L,
                                                       const float *__restrict__ lo,
                                                       const float *__restrict__ scale,
                                                       uint2 *__restrict__ q4) {
    const int groups = Fp >> 2;
    const int g = blockIdx.x * 64 + threadIdx.x;
    if (g >= groups) return;
    const int f0 = g << 2;
    float lo4[4] = {0.f, 0.f, 0.f, 0.f}, sc4[4] = {0.f, 0.f, 0.f, 0.f};
    if (!kU8) {
#pragma unroll
        for (int k = 0; k < 4; ++k)
            if (f0 + k < F) {
                lo4[k] = lo[f0 + k];
                sc4[k] = scale[f0 + k];
            }
    }
    const int64_t r0 = (int64_t)blockIdx.y * kQuantRows;
    // All loads first, with clamped indices (a value loaded for a row or feature that does not
    // exist is dropped below): nothing conditional stands between the 4 * kQuantRows loads, so
    // they are all in flight together.
    float xf[kQuantRows][4];
    uint32_t xb[kQuantRows][4];
#pragma unroll
    for (int r = 0; r < kQuantRows; ++r) {
        const int64_t n = r0 + r < N ? r0 + r : N - 1;
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            const int f = f0 + k < F ? f0 + k : F - 1;
            if (kU8)
                xb[r][k] = reinterpret_cast<const uint8_t *>(feats)[n * F + f];
            else
                xf[r][k] = reinterpret_cast<const float *>(feats)[n * F + f];
        }
    }
#pragma unroll
    for (int r = 0; r < kQuantRows; ++r) {
        uint32_t packed[2] = {0u, 0u};
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            uint32_t b = kU8 ? (xb[r][k] * (uint32_t)L) >> 8 : bin_f32(xf[r][k], lo4[k], sc4[k], L);
            if (f0 + k >= F) b = 0;
            packed[k >> 1] |= (b * (kSliceWords * 4u)) << (16 * (k & 1));
        }
        if (r0 + r < N) q4[(r0 + r) * groups + g] = make_uint2(packed[0], packed[1]);
    }
}

// Block = WAVES waves, all on the same slice of 64 word columns (one column per lane, level
// slice [L][64] in dynamic LDS; the level-row offsets the quantiser wrote are absolute LDS byte
// addresses, which holds because this kernel has no static LDS, so its dynamic LDS starts at
// address 0 - the launcher checks that).  Blocks are persistent: the grid is what the chip
// holds at once and every wave walks over several units of S samples of its slice, so the
// level slice is loaded once per block whatever the batch size.  A unit runs the features 16
// at a time: 16 ID words are loaded once and serve all S samples.
//
// Carries: a 16-vote tree leaves a carry of weight 16; two of them meet in plane 4, two of
// those in plane 5, and only every 64 features does a carry ripple through the upper planes.
template <int S, int P, int WAVES>
__global__ __launch_bounds__(WAVES * kWave) void encode_kernel(
    const uint16_t *__restrict__ q, const uint32_t *__restrict__ item,
    const uint32_t *__restrict__ level, uint32_t *__restrict__ hv, int N, int Fp, int L, int W,
    uint32_t bias) {
    static_assert(P >= 8, "planes 4 and 5 take the deferred carries");
    extern __shared__ uint32_t lv[];
    const int slice = blockIdx.x;
    const int lane = threadIdx.x & (kWave - 1);
    const int col = slice * kSliceWords + lane;

    {   // this slice of the level table is one contiguous run of L * 64 words
        const uint32_t *src = level + (size_t)slice * L * kSliceWords;
        for (int i = threadIdx.x; i < L * kSliceWords; i += WAVES * kWave) lv[i] = src[i];
    }
    __syncthreads();

    // (address = wave-uniform base of the half-block + this lane's byte offset + j * 256 as an
    // immediate: no per-row address arithmetic)
    const uint32_t lane_bytes = (uint32_t)lane * 4u;
    const char *item_slice = reinterpret_cast<const char *>(item + (size_t)slice * Fp * kSliceWords);
    auto load_ids = [&](int f, uint32_t (&id)[16]) {
        const char *base = item_slice + (size_t)f * (kSliceWords * 4);
#pragma unroll
        for (int j = 0; j < 16; ++j)
            id[j] = *reinterpret_cast<const uint32_t *>(base + j * (kSliceWords * 4) + lane_bytes);
    };

    // units of S samples are dealt round-robin to the waves of this slice (all units cost the
    // same, so a static deal balances as well as a work queue and needs no atomics).  WAVES is
    // a template constant on purpose: derived from blockDim, the compiler would treat the
    // sample index as divergent and fetch the bin offsets with vector loads.
    const int units = (N + S - 1) / S;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int stride = (int)gridDim.y * WAVES;
    for (int u = (int)blockIdx.y * WAVES + wave; u < units; u += stride) {
        const int n_base = u * S;

        uint32_t pl[S][P];
#pragma unroll
        for (int s = 0; s < S; ++s)
#pragma unroll
            for (int i = 0; i < P; ++i) pl[s][i] = ((bias >> i) & 1u) ? 0xffffffffu : 0u;

        // The bin offsets are wave-uniform and were written by an earlier kernel: read them
        // through the constant address space so they arrive by scalar loads.
        const_u32_ptr qrow[S];
#pragma unroll
        for (int s = 0; s < S; ++s) {
            const int n = min(n_base + s, N - 1);   // a ragged last unit recomputes row N-1
            qrow[s] = (const_u32_ptr)(uintptr_t)(q + (int64_t)n * Fp);
        }
        // one half-block: bind 16 features of every sample with their level rows and bundle
        // them; c16[s] receives the carry of weight 16
        auto half_block = [&](int f, uint32_t (&c16)[S]) {
            uint32_t id[16];
            load_ids(f, id);
#pragma unroll
            for (int s = 0; s < S; ++s) {
                uint32_t qpair[8];
#pragma unroll
                for (int k = 0; k < 8; ++k) qpair[k] = qrow[s][(f >> 1) + k];
                uint32_t x[16];
                gather16(x, qpair);
#pragma unroll
                for (int j = 0; j < 16; ++j) x[j] ^= id[j];  // bind (XOR)
                c16[s] = Tree<4, 0>::run(pl[s], x);          // bundle 16 votes
                // Pin the step's results here (empty volatile asm, no instruction): the asm
                // statements keep their order, so the tree above cannot be sunk below the next
                // gather, which would keep several samples' 16 bound words alive at once.
                asm volatile("" : "+v"(c16[s]), "+v"(pl[s][0]), "+v"(pl[s][1]), "+v"(pl[s][2]), "+v"(pl[s][3]));
            }
        };

        // two pairs (64 features) per trip: their weight-32 carries meet in plane 5 and only the
        // weight-64 carry ripples up
        auto pair_carry = [&](int f, uint32_t (&c32)[S]) {
            uint32_t ca[S], cb[S];
            half_block(f, ca);
            half_block(f + 16, cb);
#pragma unroll
            for (int s = 0; s < S; ++s) {
                const uint32_t p4 = pl[s][4];
                pl[s][4] = xor3(p4, ca[s], cb[s]);
                c32[s] = maj3(p4, ca[s], cb[s]);
            }
        };
        int f0 = 0;
        for (; f0 + 64 <= Fp; f0 += 64) {
            uint32_t ea[S], eb[S];
            pair_carry(f0, ea);
            pair_carry(f0 + 32, eb);
#pragma unroll
            for (int s = 0; s < S; ++s) {
                const uint32_t p5 = pl[s][5];
                pl[s][5] = xor3(p5, ea[s], eb[s]);
                ripple<6, P>(pl[s], maj3(p5, ea[s], eb[s]));
            }
        }
        if (f0 + 32 <= Fp) {   // one pair left over
            uint32_t ea[S];
            pair_carry(f0, ea);
            f0 += 32;
#pragma unroll
            for (int s = 0; s < S; ++s) ripple<5, P>(pl[s], ea[s]);
        }
        if (f0 < Fp) {   // Fp is an odd multiple of 16: the last half-block has no partner
            uint32_t ca[S];
            half_block(f0, ca);
#pragma unroll
            for (int s = 0; s < S; ++s) ripple<4, P>(pl[s], ca[s]);
        }

        if (col < W) {
#pragma unroll
            for (int s = 0; s < S; ++s)
                if (n_base + s < N) hv[(int64_t)(n_base + s) * W + col] = pl[s][P - 1];
        }
    }
}

// Few samples: with a sample (or a few) per wave there are not enough waves to keep the vector
// units busy, and a lone wave runs at the pace of its dependent instructions.  Here the WAVES waves
// of a block share ONE sample of the block's slice: wave w bundles its share of the half-blocks of
// 16 features into planes of its own (wave 0's start at the bias), waves 1.. park theirs in LDS,
// and wave 0 adds them up (ripple-carry over the planes) and stores the majority word.  One
// barrier per sample: the merge area behind the level slice is double-buffered by sample parity.
// Every wave of a block makes the same trips, so the barrier is reached by all.
template <int P, int WAVES>
__global__ __launch_bounds__(WAVES * kWave) void encode_split_kernel(
    const uint16_t *__restrict__ q, const uint32_t *__restrict__ item,
    const uint32_t *__restrict__ level, uint32_t *__restrict__ hv, int N, int Fp, int L, int W,
    uint32_t bias) {
    extern __shared__ uint32_t lv[];   // level slice [L][64] at address 0, then merge [2][WAVES - 1][P][64]
    const int slice = blockIdx.x;
    const int lane = threadIdx.x & (kWave - 1);
    const int col = slice * kSliceWords + lane;
    {
        const uint32_t *src = level + (size_t)slice * L * kSliceWords;
        for (int i = threadIdx.x; i < L * kSliceWords; i += WAVES * kWave) lv[i] = src[i];
    }
    __syncthreads();
    uint32_t *merge = lv + (size_t)L * kSliceWords;

    const uint32_t lane_bytes = (uint32_t)lane * 4u;
    const char *item_slice = reinterpret_cast<const char *>(item + (size_t)slice * Fp * kSliceWords);
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int nhb = Fp / kFeatBlock;                      // half-blocks of 16 features
    const int hb0 = wave * nhb / WAVES, hb1 = (wave + 1) * nhb / WAVES;

    int parity = 0;
    for (int n = blockIdx.y; n < N; n += (int)gridDim.y, parity ^= 1) {
        uint32_t pl[P];
#pragma unroll
        for (int i = 0; i < P; ++i) pl[i] = (wave == 0 && ((bias >> i) & 1u)) ? 0xffffffffu : 0u;
        const_u32_ptr qrow = (const_u32_ptr)(uintptr_t)(q + (int64_t)n * Fp);
        for (int hb = hb0; hb < hb1; ++hb) {
            const int f = hb * kFeatBlock;
            const char *base = item_slice + (size_t)f * (kSliceWords * 4);
            uint32_t id[16];
#pragma unroll
            for (int j = 0; j < 16; ++j)
                id[j] = *reinterpret_cast<const uint32_t *>(base + j * (kSliceWords * 4) + lane_bytes);
            uint32_t qpair[8];
#pragma unroll
            for (int k = 0; k < 8; ++k) qpair[k] = qrow[(f >> 1) + k];
            uint32_t x[16];
            gather16(x, qpair);
#pragma unroll
            for (int j = 0; j < 16; ++j) x[j] ^= id[j];
            ripple<4, P>(pl, Tree<4, 0>::run(pl, x));
        }
        if (wave > 0) {
            uint32_t *dst = merge + ((size_t)(parity * (WAVES - 1) + wave - 1) * P) * kSliceWords + lane;
#pragma unroll
            for (int i = 0; i < P; ++i) dst[i * kSliceWords] = pl[i];
        }
        __syncthreads();
        if (wave == 0) {
#pragma unroll 1
            for (int w = 0; w < WAVES - 1; ++w) {
                const uint32_t *src = merge + ((size_t)(parity * (WAVES - 1) + w) * P) * kSliceWords + lane;
                uint32_t carry = 0;
#pragma unroll
                for (int i = 0; i < P; ++i) {
                    const uint32_t a = pl[i], b = src[i * kSliceWords];
                    pl[i] = xor3(a, b, carry);
                    carry = maj3(a, b, carry);
                }
            }
            if (col < W) hv[(int64_t)n * W + col] = pl[P - 1];
        }
    }
}

typedef void (*encode_fn)(const uint16_t *, const uint32_t *, const uint32_t *, uint32_t *, int, int, int,
                          int, uint32_t);
struct EncodeVariant {
    encode_fn fn;
    int S, P, waves;
};
#define HDC_VARIANTS(P) \
    {encode_kernel<1, P, 4>, 1, P, 4}, {encode_kernel<2, P, 4>, 2, P, 4}, {encode_kernel<4, P, 4>, 4, P, 4}, \
    {encode_kernel<1, P, 8>, 1, P, 8}, {encode_kernel<2, P, 8>, 2, P, 8}, {encode_kernel<4, P, 8>, 4, P, 8}
static const EncodeVariant kVariants[] = {HDC_VARIANTS(8), HDC_VARIANTS(10), HDC_VARIANTS(12), HDC_VARIANTS(16)};
#undef HDC_VARIANTS

// `item`, `level`, W, Wp: the full tables of the context or its compact ones; hv has rows of W words.
static int launch_encode_kernel(hdc_ctx_impl *c, const uint32_t *item, const uint32_t *level, int W, int Wp,
                                int P, int N, uint32_t *hv, uint32_t bias, hipStream_t s) {
    const int nslices = Wp / kSliceWords;
    const int waves = c->p.L > 128 ? 8 : 4;   // a big level slice: fewer, larger blocks per CU
    // small batches take 2-sample or 1-sample units so that there are enough of them for 1024
    // SIMDs (measured crossovers: about 3 four-sample units, 2.5 two-sample units per SIMD)
    const int S = ((int64_t)((N + 3) / 4) * nslices >= 3072) ? 4 : ((int64_t)((N + 1) / 2) * nslices >= 2560) ? 2 : 1;
    const size_t lds = (size_t)c->p.L * kSliceWords * sizeof(uint32_t);
    // Too few samples for a sample per wave: the waves of a block share one (measured against the
    // one-sample units: faster up to about 2000 sample-slices; 16 waves per sample for a handful
    // of samples - a single sample encodes in 8 us instead of 21 - and 8 beyond).
    if (S == 1 && (int64_t)N * nslices <= 2048) {
        const int which = (int64_t)N * nslices <= 256 ? 1 : 0;
        const int kSplitWaves = which ? 16 : 8;
#define HDC_SPLIT(W_) (P == 8 ? encode_split_kernel<8, W_> : P == 10 ? encode_split_kernel<10, W_> \
                       : P == 12 ? encode_split_kernel<12, W_> : encode_split_kernel<16, W_>)
        encode_fn fn = which ? HDC_SPLIT(16) : HDC_SPLIT(8);
#undef HDC_SPLIT
        const size_t lds_split = lds + (size_t)2 * (kSplitWaves - 1) * P * kSliceWords * sizeof(uint32_t);
        // (the limit belongs to the function, not to a context: another context may have set a smaller one since)
        if (lds_split > 64 * 1024)
            HDC_HIP(hipFuncSetAttribute(reinterpret_cast<const void *>(fn), hipFuncAttributeMaxDynamicSharedMemorySize,
                                        (int)lds_split));
        if (c->enc_split_bpc[which] == 0 || c->enc_split_L[which] != c->p.L) {
            hipFuncAttributes attr;
            HDC_HIP(hipFuncGetAttributes(&attr, reinterpret_cast<const void *>(fn)));
            if (attr.sharedSizeBytes != 0) return HDC_ELIMIT;
            int n = 0;
            HDC_HIP(hipOccupancyMaxActiveBlocksPerMultiprocessor(&n, reinterpret_cast<const void *>(fn),
                                                                 kSplitWaves * kWave, lds_split));
            c->enc_split_bpc[which] = n < 1 ? 1 : n;
            c->enc_split_L[which] = c->p.L;
        }
        int per_slice = (c->num_cus * c->enc_split_bpc[which]) / nslices;
        if (per_slice < 1) per_slice = 1;
        if (per_slice > N) per_slice = N;
        const int k = (N + per_slice - 1) / per_slice;   // samples per block, evened out
        per_slice = (N + k - 1) / k;
        ProfScope prof(c, HDC_K_ENCODE, s);
        hipLaunchKernelGGL(fn, dim3((unsigned)nslices, (unsigned)per_slice), dim3(kSplitWaves * kWave), lds_split, s,
                           c->q_d, item, level, hv, N, c->Fp, c->p.L, W, bias);
        return HDC_OK;
    }
    const EncodeVariant *v = nullptr;
    for (const EncodeVariant &k : kVariants)
        if (k.S == S && k.P == P && k.waves == waves) v = &k;
    if (!v) return HDC_ELIMIT;
    // Per variant, once per context: no static LDS allowed (the level-row offsets are absolute LDS
    // addresses), and how many blocks of it a CU holds (registers and LDS).
    static_assert(sizeof(kVariants) / sizeof(kVariants[0]) <= sizeof(c->enc_bpc) / sizeof(c->enc_bpc[0]),
                  "one slot per variant");
    int &bpc = c->enc_bpc[v - kVariants];
    if (bpc == 0 || c->enc_bpc_L[v - kVariants] != c->p.L) {
        hipFuncAttributes attr;
        HDC_HIP(hipFuncGetAttributes(&attr, reinterpret_cast<const void *>(v->fn)));
        if (attr.sharedSizeBytes != 0) return HDC_ELIMIT;
        int n = 0;
        HDC_HIP(hipOccupancyMaxActiveBlocksPerMultiprocessor(&n, reinterpret_cast<const void *>(v->fn),
                                                             waves * kWave, lds));
        bpc = n < 1 ? 1 : n;
        c->enc_bpc_L[v - kVariants] = c->p.L;
    }
    // persistent grid: at most what the chip holds at once, sized so that the deal comes out
    // even - every wave gets k units (the last few k-1), never some waves one unit more than
    // the rest of a nearly idle chip
    const int units = (N + S - 1) / S;
    int max_waves = (c->num_cus * bpc) / nslices * waves;
    if (max_waves < waves) max_waves = waves;
    const int k = (units + max_waves - 1) / max_waves;          // units per wave
    const int need_waves = (units + k - 1) / k;
    const int per_slice = (need_waves + waves - 1) / waves;
    ProfScope prof(c, HDC_K_ENCODE, s);
    hipLaunchKernelGGL(v->fn, dim3((unsigned)nslices, (unsigned)per_slice), dim3(waves * kWave), lds, s,
                       c->q_d, item, level, hv, N, c->Fp, c->p.L, W, bias);
    return HDC_OK;
}

// ---- spreading compact hypervectors back over all dimensions ---------------------------------
// One lane per output word w.  The bits of w that vary are a run of the compact row starting at
// bit tab[0][w]; they are spread to the set bits of tab[1][w] by five shift-and-merge stages
// (a bit's distance to its place, in binary: stage i moves the bits whose distance has bit i
// set by 2^i, highest first; tab[2 + i][w] marks where they land), and the model's constant
// bits tab[7][w] fill the rest.  A thread keeps its word's eight table entries in registers and
// walks down the rows.
constexpr int kExpandRows = 4;
__global__ __launch_bounds__(kExpandRows *kWave) void expand_kernel(const uint32_t *__restrict__ hvc, int64_t N, int Wc,
                                                                    int W, const uint32_t *__restrict__ tab,
                                                                    uint32_t *__restrict__ hv) {
    const int w = blockIdx.x * kWave + (threadIdx.x & (kWave - 1));
    if (w >= W) return;
    const uint32_t off = tab[w], keep = tab[W + w], cst = tab[7 * W + w];
    uint32_t stage[5];
#pragma unroll
    for (int i = 0; i < 5; ++i) stage[i] = tab[(2 + i) * W + w];
    const int i0 = (int)(off >> 5), sh = (int)(off & 31u);
    for (int64_t n = (int64_t)blockIdx.y * kExpandRows + (threadIdx.x >> 6); n < N;
         n += (int64_t)gridDim.y * kExpandRows) {
        uint32_t x = 0;
        if (keep) {
            const uint32_t *row = hvc + n * Wc;
            const uint32_t lo = i0 < Wc ? row[i0] : 0u, hi = i0 + 1 < Wc ? row[i0 + 1] : 0u;
            x = sh ? (lo >> sh) | (hi << (32 - sh)) : lo;
#pragma unroll
            for (int i = 4; i >= 0; --i) x = (x & ~stage[i]) | ((x << (1 << i)) & stage[i]);
        }
        hv[n * W + w] = (x & keep) | cst;
    }
}

// Majority of `votes` (odd) inputs: count >= thr.  With P-1 = ceil(log2(thr)) and the counters
// starting at bias = 2^(P-1) - thr, bit P-1 of the final count is the answer and the count
// never reaches 2^P.  P is rounded up to a plane count the kernels are built for.
void majority_planes(const hdc_ctx_impl *c, int *P_out, uint32_t *bias_out) {
    const uint32_t thr = ((uint32_t)c->votes + 1u) / 2u;
    int top = 0;
    while ((1u << top) < thr) ++top;
    int P = top + 1;
    P = P <= 8 ? 8 : P <= 10 ? 10 : P <= 12 ? 12 : 16;
    *P_out = P;
    *bias_out = (1u << (P - 1)) - thr;
}

// n compact rows in the context's staging buffer -> n full rows at `out`.
void launch_expand(hdc_ctx_impl *c, int64_t n, uint32_t *out, hipStream_t s) {
    int64_t gy = (n + kExpandRows - 1) / kExpandRows;
    if (gy > 2048) gy = 2048;
    hipLaunchKernelGGL(expand_kernel, dim3((unsigned)((c->W + kWave - 1) / kWave), (unsigned)gy),
                       dim3(kExpandRows * kWave), 0, s, c->hvc_d, n, c->Wc, c->W, c->expand_d, out);
}

int launch_encode(hdc_ctx_impl *c, const void *feats, int64_t N, uint32_t *hv, hipStream_t s) {
    {
        int rc = HDC_OK;
        if (try_encode_wide(c, feats, N, hv, s, &rc)) return rc;
        if (try_encode_contract(c, feats, N, hv, s, &rc)) return rc;
    }
    int P;
    uint32_t bias;
    majority_planes(c, &P, &bias);

    for (int64_t n0 = 0; n0 < N; n0 += c->q_rows) {
        const int64_t n = (N - n0 < c->q_rows) ? N - n0 : c->q_rows;
        const size_t esz = c->p.feat_dtype == HDC_U8 ? 1 : 4;
        const void *x = reinterpret_cast<const uint8_t *>(feats) + (size_t)n0 * c->p.F * esz;
        {
            ProfScope prof(c, HDC_K_QUANTIZE, s);
            const dim3 qgrid((unsigned)(((c->Fp >> 2) + 63) / 64), (unsigned)((n + kQuantRows - 1) / kQuantRows));
            uint2 *q4 = reinterpret_cast<uint2 *>(c->q_d);
            if (c->p.feat_dtype == HDC_U8)
                hipLaunchKernelGGL(quantize_kernel<true>, qgrid, dim3(64), 0, s, x, n, c->p.F, c->Fp, c->p.L,
                                   c->lo_d, c->scale_d, q4);
            else
                hipLaunchKernelGGL(quantize_kernel<false>, qgrid, dim3(64), 0, s, x, n, c->p.F, c->Fp, c->p.L,
                                   c->lo_d, c->scale_d, q4);
        }
        uint32_t *out = hv + (size_t)n0 * c->W;
        if (!c->compact) {
            const int rc = launch_encode_kernel(c, c->item_d, c->level_d, c->W, c->Wp, P, (int)n, out, bias, s);
            if (rc != HDC_OK) return rc;
        } else {
            if (c->Wc > 0) {
                const int rc = launch_encode_kernel(c, c->citem_d, c->clevel_d, c->Wc, c->Wcp, P, (int)n, c->hvc_d,
                                                    bias, s);
                if (rc != HDC_OK) return rc;
            }
            launch_expand(c, n, out, s);
        }
        HDC_HIP(hipGetLastError());
    }
    return HDC_OK;
}

}  // namespace hdc
