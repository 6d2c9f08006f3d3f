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

// One thread produces the entries of features 4g..4g+3 of one sample.  An entry is the byte
// offset of the bin's row in the LDS level slice (bin * 256, fits 16 bits for L <= 256);
// features at or beyond F (the tie-vote row and the pad rows of the device item table) get
// bin 0.
template <bool kU8>
__global__ __launch_bounds__(256) void quantize_kernel(const void *__restrict__ feats, int64_t N,
                                                        int F, int Fp, int L,
                                                        const float *__restrict__ lo,
                                                        const float *__restrict__ scale,
                                                        uint2 *__restrict__ q4) {
    const int groups = Fp >> 2;
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= N * groups) return;
    const int64_t n = i / groups;
    const int f0 = (int)(i - n * groups) << 2;
    uint32_t packed[2] = {0u, 0u};
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
        packed[k >> 1] |= (b * (kSliceWords * 4u)) << (16 * (k & 1));
    }
    q4[i] = make_uint2(packed[0], packed[1]);
}

// ------------------------------------------------------------- bundling (Eq. 1's sum)
typedef const uint32_t __attribute__((address_space(4))) *const_u32_ptr;

// Level words of 16 features for this lane's column, fetched from the LDS level slice.
// qpair[k] holds the LDS byte offsets (bin * 256) of features 2k and 2k+1 as two u16.  The
// row offset is wave-uniform, so it goes through M0 and ds_read_addtid_b32 (address = M0 +
// lane * 4): no vector ALU work is spent on addresses.  One wait state separates a write of
// M0 from the LDS instruction that reads it.
//
// The trailing s_waitcnt makes the outputs valid before the asm statement ends.
__device__ __forceinline__ void gather16(uint32_t (&x)[16], const uint32_t (&qpair)[8]) {
    asm volatile(
        "s_and_b32 m0, %16, 0xffff\n\ts_nop 0\n\tds_read_addtid_b32 %0\n\t"
        "s_lshr_b32 m0, %16, 16\n\ts_nop 0\n\tds_read_addtid_b32 %1\n\t"
        "s_and_b32 m0, %17, 0xffff\n\ts_nop 0\n\tds_read_addtid_b32 %2\n\t"
        "s_lshr_b32 m0, %17, 16\n\ts_nop 0\n\tds_read_addtid_b32 %3\n\t"
        "s_and_b32 m0, %18, 0xffff\n\ts_nop 0\n\tds_read_addtid_b32 %4\n\t"
        "s_lshr_b32 m0, %18, 16\n\ts_nop 0\n\tds_read_addtid_b32 %5\n\t"
        "s_and_b32 m0, %19, 0xffff\n\ts_nop 0\n\tds_read_addtid_b32 %6\n\t"
        "s_lshr_b32 m0, %19, 16\n\ts_nop 0\n\tds_read_addtid_b32 %7\n\t"
        "s_and_b32 m0, %20, 0xffff\n\ts_nop 0\n\tds_read_addtid_b32 %8\n\t"
        "s_lshr_b32 m0, %20, 16\n\ts_nop 0\n\tds_read_addtid_b32 %9\n\t"
        "s_and_b32 m0, %21, 0xffff\n\ts_nop 0\n\tds_read_addtid_b32 %10\n\t"
        "s_lshr_b32 m0, %21, 16\n\ts_nop 0\n\tds_read_addtid_b32 %11\n\t"
        "s_and_b32 m0, %22, 0xffff\n\ts_nop 0\n\tds_read_addtid_b32 %12\n\t"
        "s_lshr_b32 m0, %22, 16\n\ts_nop 0\n\tds_read_addtid_b32 %13\n\t"
        "s_and_b32 m0, %23, 0xffff\n\ts_nop 0\n\tds_read_addtid_b32 %14\n\t"
        "s_lshr_b32 m0, %23, 16\n\ts_nop 0\n\tds_read_addtid_b32 %15\n\t"
        "s_waitcnt lgkmcnt(0)"
        : "=&v"(x[0]), "=&v"(x[1]), "=&v"(x[2]), "=&v"(x[3]), "=&v"(x[4]), "=&v"(x[5]), "=&v"(x[6]),
          "=&v"(x[7]), "=&v"(x[8]), "=&v"(x[9]), "=&v"(x[10]), "=&v"(x[11]), "=&v"(x[12]),
          "=&v"(x[13]), "=&v"(x[14]), "=&v"(x[15])
        : "s"(qpair[0]), "s"(qpair[1]), "s"(qpair[2]), "s"(qpair[3]), "s"(qpair[4]), "s"(qpair[5]),
          "s"(qpair[6]), "s"(qpair[7])
        : "scc", "memory");
}
// Adds the 2^LV bound words x[J0 .. J0+2^LV-1] into planes 0..LV-1 and returns the carry of
// weight 2^LV.  Depth-first, so only one pending carry per level is alive.
template <int LV, int J0>
struct Tree {
    static __device__ __forceinline__ uint32_t run(uint32_t *pl, const uint32_t *x) {
        const uint32_t a = Tree<LV - 1, J0>::run(pl, x);
        const uint32_t b = Tree<LV - 1, J0 + (1 << (LV - 1))>::run(pl, x);
        const uint32_t p = pl[LV - 1];
        pl[LV - 1] = xor3(p, a, b);
        return maj3(p, a, b);
    }
};
template <int J0>
struct Tree<1, J0> {
    static __device__ __forceinline__ uint32_t run(uint32_t *pl, const uint32_t *x) {
        const uint32_t p = pl[0];
        pl[0] = xor3(p, x[J0], x[J0 + 1]);
        return maj3(p, x[J0], x[J0 + 1]);
    }
};

// Carry `c` of weight 2^FROM rippled into planes FROM..P-1 (half adders).
template <int FROM, int P>
__device__ __forceinline__ void ripple(uint32_t *pl, uint32_t c) {
#pragma unroll
    for (int i = FROM; i < P; ++i) {
        const uint32_t t = pl[i] & c;
        pl[i] ^= c;
        c = t;
    }
}

// Block = WAVES waves, all on the same slice of 64 word columns (one column per lane, level
// slice [L][64] in dynamic LDS; the level-row offsets the quantiser wrote are absolute LDS
// byte addresses, which holds because this kernel has no static LDS, so its dynamic LDS starts
// at address 0 - the launcher checks that).  The waves form WAVES/FS groups; a group carries S samples through all Fp features,
// 16 at a time, its FS waves each taking a contiguous share of the features and adding their
// bit-sliced partial counts together through LDS at the end.  FS > 1 makes the work units
// smaller, which is what a small batch needs to fill 1024 SIMDs; FS = 1 has no merge at all.
template <int S, int P, int WAVES, int FS>
__global__ __launch_bounds__(WAVES * kWave) void encode_kernel(
    const uint16_t *__restrict__ q, const uint32_t *__restrict__ item,
    const uint32_t *__restrict__ level, uint32_t *__restrict__ hv, int N, int Fp, int L, int W, int Wp,
    uint32_t bias) {
    extern __shared__ uint32_t lv[];
    constexpr int GROUPS = WAVES / FS;
    const int slice = blockIdx.x;
    const int tile = blockIdx.y;
    const int lane = threadIdx.x & (kWave - 1);
    const int col = slice * kSliceWords + lane;

    {   // this slice of the level table is one contiguous run of L * 64 words
        const uint32_t *src = level + (size_t)slice * L * kSliceWords;
        for (int i = threadIdx.x; i < L * kSliceWords; i += WAVES * kWave) lv[i] = src[i];
    }
    __syncthreads();

    // WAVES is a compile-time constant on purpose: a block size read from the dispatch packet
    // makes the compiler treat the sample index as divergent and the bin loads as vector loads.
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int group = wave / FS;
    const int part = wave % FS;
    const int n_base = (tile * GROUPS + group) * S;
    const bool live = n_base < N;
    if (FS == 1 && !live) return;   // with FS > 1 every wave must reach the merge barriers

    // Only the first wave of a group starts from the bias; the others add plain partial counts.
    const uint32_t my_bias = part == 0 ? bias : 0u;
    uint32_t pl[S][P];
#pragma unroll
    for (int s = 0; s < S; ++s)
#pragma unroll
        for (int i = 0; i < P; ++i) pl[s][i] = ((my_bias >> i) & 1u) ? 0xffffffffu : 0u;

    // The bin offsets are wave-uniform and were written by an earlier kernel: read them through
    // the constant address space so they arrive by scalar loads, off the vector pipeline.
    const_u32_ptr qrow[S];
#pragma unroll
    for (int s = 0; s < S; ++s) {
        const int n = min(n_base + s, N - 1);   // a ragged last group recomputes row N-1
        qrow[s] = (const_u32_ptr)(uintptr_t)(q + (int64_t)n * Fp);
    }

    // This wave's share of the features: a contiguous run of 32-feature pairs (the last share
    // also takes the unpaired half-block, if Fp is an odd multiple of 16).
    const int pairs = Fp >> 5;
    const int per = (pairs + FS - 1) / FS;
    int f0 = min(part * per, pairs) << 5;
    const int f_end = (part == FS - 1) ? Fp : (min((part + 1) * per, pairs) << 5);

    // ID rows are loaded one half-block ahead of their use (ida / idb alternate), so their
    // latency hides behind the arithmetic of the half-block before.
    // (address = wave-uniform base of the half-block in SGPRs + this lane's byte offset +
    // j * 256 as an immediate: no vector address arithmetic, no address registers)
    const uint32_t lane_bytes = (uint32_t)lane * 4u;
    const char *item_slice = reinterpret_cast<const char *>(item + (size_t)slice * Fp * kSliceWords);
    auto load_ids = [&](int f, uint32_t (&id)[16]) {
        const char *base = item_slice + (size_t)f * (kSliceWords * 4);
#pragma unroll
        for (int j = 0; j < 16; ++j)
            id[j] = *reinterpret_cast<const uint32_t *>(base + j * (kSliceWords * 4) + lane_bytes);
    };
    // the S samples of one half-block: bind 16 features with their level rows and bundle
    // them; c16[s] receives the carry of weight 16
    auto half_block = [&](int f, const uint32_t (&id)[16], uint32_t (&c16)[S]) {
#pragma unroll
        for (int s = 0; s < S; ++s) {
            uint32_t qpair[8];
#pragma unroll
            for (int k = 0; k < 8; ++k) qpair[k] = qrow[s][(f >> 1) + k];
            uint32_t x[16];
            gather16(x, qpair);
#pragma unroll
            for (int j = 0; j < 16; ++j) x[j] ^= id[j];     // bind (XOR)
            c16[s] = Tree<4, 0>::run(pl[s], x);              // bundle 16 votes
            // Keep the samples in program order: the gathers are volatile and cannot move, so
            // pinning the results here (empty volatile asm, no instruction) stops the compiler
            // from sinking this sample's arithmetic below the next gathers, which would hold
            // S * 16 landing registers alive at once.
            asm volatile("" : "+v"(c16[s]), "+v"(pl[s][0]), "+v"(pl[s][1]), "+v"(pl[s][2]), "+v"(pl[s][3]));
        }
    };

    if (live && f0 < f_end) {
        uint32_t ida[16], idb[16];
        load_ids(f0, ida);
        for (; f0 + 32 <= f_end; f0 += 32) {
            uint32_t ca[S], cb[S];
            load_ids(f0 + 16, idb);
            half_block(f0, ida, ca);
            if (f0 + 32 < f_end) load_ids(f0 + 32, ida);
            half_block(f0 + 16, idb, cb);
#pragma unroll
            for (int s = 0; s < S; ++s) {
                const uint32_t p = pl[s][4];
                pl[s][4] = xor3(p, ca[s], cb[s]);
                ripple<5, P>(pl[s], maj3(p, ca[s], cb[s]));
            }
        }
        if (f0 < f_end) {   // the unpaired last half-block; its IDs are already in flight
            uint32_t ca[S];
            half_block(f0, ida, ca);
#pragma unroll
            for (int s = 0; s < S; ++s) ripple<4, P>(pl[s], ca[s]);
        }
    }

    if (FS > 1) {
        // Sum the FS partial counts of every sample: waves 1..FS-1 of a group park their planes
        // in LDS (behind the level slice), wave 0 adds them with P full adders each.
        uint32_t *mbuf = lv + L * kSliceWords + group * ((FS - 1) * P * kWave);
#pragma unroll
        for (int s = 0; s < S; ++s) {
            if (part > 0) {
#pragma unroll
                for (int i = 0; i < P; ++i) mbuf[((part - 1) * P + i) * kWave + lane] = pl[s][i];
            }
            __syncthreads();
            if (part == 0) {
#pragma unroll
                for (int r = 0; r < FS - 1; ++r) {
                    uint32_t carry = 0;
#pragma unroll
                    for (int i = 0; i < P; ++i) {
                        const uint32_t a = pl[s][i], b2 = mbuf[(r * P + i) * kWave + lane];
                        pl[s][i] = xor3(a, b2, carry);
                        carry = maj3(a, b2, carry);
                    }
                }
            }
            __syncthreads();
        }
    }

    if (part == 0 && live && col < W) {
#pragma unroll
        for (int s = 0; s < S; ++s)
            if (n_base + s < N) hv[(int64_t)(n_base + s) * W + col] = pl[s][P - 1];
    }
}

template <int S, int P, int WAVES, int FS>
static int launch_encode_spwf(hdc_ctx_impl *c, int N, uint32_t *hv, uint32_t bias, hipStream_t s) {
    constexpr int GROUPS = WAVES / FS;
    const int nslices = c->Wp / kSliceWords;
    const int tiles = (N + GROUPS * S - 1) / (GROUPS * S);
    const size_t lds = ((size_t)c->p.L * kSliceWords + (FS > 1 ? (size_t)GROUPS * (FS - 1) * P * kWave : 0)) *
                       sizeof(uint32_t);
    static int static_lds = -1;   // level-row offsets are absolute: no static LDS allowed
    if (static_lds < 0) {
        hipFuncAttributes attr;
        if (hipFuncGetAttributes(&attr, reinterpret_cast<const void *>(encode_kernel<S, P, WAVES, FS>)) !=
            hipSuccess)
            return HDC_EHIP;
        static_lds = (int)attr.sharedSizeBytes;
    }
    if (static_lds != 0) return HDC_ELIMIT;
    ProfScope prof(c, HDC_K_ENCODE, s);
    hipLaunchKernelGGL((encode_kernel<S, P, WAVES, FS>), dim3((unsigned)nslices, (unsigned)tiles),
                       dim3(WAVES * kWave), lds, s, c->q_d, c->item_d, c->level_d, hv, N, c->Fp, c->p.L,
                       c->W, c->Wp, bias);
    return HDC_OK;
}

template <int S, int P>
static int launch_encode_sp(hdc_ctx_impl *c, int N, uint32_t *hv, uint32_t bias, hipStream_t s) {
    // Work units needed to give every SIMD of the chip a few waves; below that, split the
    // features of a sample group over the waves of a block (smaller units, one LDS merge).
    const int64_t units = (int64_t)((N + S - 1) / S) * (c->Wp / kSliceWords);
    const bool split = units < 4 * 1024 * 4 && (c->Fp >> 5) >= 8;
    // a large level table leaves room for few blocks per CU: use bigger blocks then
    if (c->p.L > 128) {
        if (split) return launch_encode_spwf<S, P, 8, 4>(c, N, hv, bias, s);
        return launch_encode_spwf<S, P, 8, 1>(c, N, hv, bias, s);
    }
    if (split) return launch_encode_spwf<S, P, 4, 4>(c, N, hv, bias, s);
    return launch_encode_spwf<S, P, 4, 1>(c, N, hv, bias, s);
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
        {
            ProfScope prof(c, HDC_K_QUANTIZE, s);
            uint2 *q4 = reinterpret_cast<uint2 *>(c->q_d);
            if (c->p.feat_dtype == HDC_U8)
                hipLaunchKernelGGL(quantize_kernel<true>, dim3(qblocks), dim3(256), 0, s, x, n, c->p.F,
                                   c->Fp, c->p.L, c->lo_d, c->scale_d, q4);
            else
                hipLaunchKernelGGL(quantize_kernel<false>, dim3(qblocks), dim3(256), 0, s, x, n, c->p.F,
                                   c->Fp, c->p.L, c->lo_d, c->scale_d, q4);
        }
        uint32_t *out = hv + (size_t)n0 * c->W;
        int rc;
        switch (P) {
            case 6: rc = launch_encode_sp<4, 6>(c, (int)n, out, bias, s); break;
            case 8: rc = launch_encode_sp<4, 8>(c, (int)n, out, bias, s); break;
            case 10: rc = launch_encode_sp<4, 10>(c, (int)n, out, bias, s); break;
            case 12: rc = launch_encode_sp<4, 12>(c, (int)n, out, bias, s); break;
            default: rc = launch_encode_sp<4, 16>(c, (int)n, out, bias, s); break;
        }
        if (rc != HDC_OK) return rc;
        HDC_HIP(hipGetLastError());
    }
    return HDC_OK;
}

}  // namespace hdc
