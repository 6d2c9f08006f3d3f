// ID-Level encoding (arXiv 2206.04746, Sec. III, Eq. 1) for inputs whose features mostly fall
// into bin 0 (images with a dark background, say).  Same result as encode_kernel, less work:
//
//   count[d] = sum_f item[f][d] ^ level[bin_f][d]
//            = sum_f b_f[d]  +  sum_{f: bin_f != 0} ( (b_f[d] ^ e_bin[d]) - b_f[d] ),
//   b_f = item[f] ^ level[0]   (the vote of feature f when it sits in bin 0),
//   e_q = level[q] ^ level[0]  (where bin q's level vector differs from bin 0's).
//
// The first sum is a constant of the model (kept bit-sliced, bias included); the second runs
// over the listed features only.  A listed feature adds 1 + delta, delta = e & (b ? -1 : +1),
// a two-bit number (low bit ~e, high bit e & ~b); the ones are taken back by starting the
// counters at  base - (number of listed entries)  modulo 2^P.  Adding the low bit to plane 0
// and forming the weight-2 carry are two v_bitop3_b32 on (plane 0, e, b); the 16 carries of a
// block of 16 entries go through the usual carry-save tree on planes 1..4.  About 4.6 lane-ops
// per listed (feature, word) against 3 per (feature, word) of the dense kernel, so the lists
// pay off below roughly 60 % listed features.
//
// Three kernels per chunk: sparse_lists_kernel (quantise, list the features not in bin 0),
// encode_sparse_kernel (bundle), expand_kernel when the tables are the compact ones.
#include "bundle.h"

namespace hdc {

// Scalar loads are asked for a block ahead of their use: wait_scalar_loads() at the top of a trip
// (for what was issued a trip ago) and pin_schedule() after new loads have been issued keep the
// compiler from moving either next to the other.
__device__ __forceinline__ void wait_scalar_loads() {
    __builtin_amdgcn_sched_barrier(0);
    __builtin_amdgcn_s_waitcnt(0xC07F);   // lgkmcnt(0)
}
__device__ __forceinline__ void pin_schedule() { __builtin_amdgcn_sched_barrier(0); }

// ---- tables, derived on the device from the tables the dense kernel uses ------------------------
// dst[slice][r][64] = src[slice][r][64] ^ ref[slice][0][64]
__global__ __launch_bounds__(256) void xor_row0_kernel(const uint32_t *__restrict__ src,
                                                       const uint32_t *__restrict__ ref, int rows, int ref_rows,
                                                       int nslices, uint32_t *__restrict__ dst) {
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= (int64_t)nslices * rows * kSliceWords) return;
    const int w = (int)(i % kSliceWords);
    const int slice = (int)(i / ((int64_t)rows * kSliceWords));
    dst[i] = src[i] ^ ref[(size_t)slice * ref_rows * kSliceWords + w];
}

// base[slice][i][lane] = plane i of ( bias + sum over all Fp rows of b[slice][f][lane] ): what the
// dense kernel's counters hold for a sample whose every feature is in bin 0.
__global__ __launch_bounds__(kWave) void base_planes_kernel(const uint32_t *__restrict__ b, int Fp, int P,
                                                             uint32_t bias, uint32_t *__restrict__ base) {
    const int slice = blockIdx.x, lane = threadIdx.x;
    const uint32_t *col = b + (size_t)slice * Fp * kSliceWords + lane;
    uint32_t pl[16];
#pragma unroll
    for (int i = 0; i < 16; ++i) pl[i] = ((bias >> i) & 1u) ? 0xffffffffu : 0u;
    for (int f = 0; f < Fp; ++f) {
        uint32_t c = col[(size_t)f * kSliceWords];
#pragma unroll
        for (int i = 0; i < 16; ++i) {   // ripple one vote through the planes
            const uint32_t t = pl[i] & c;
            pl[i] ^= c;
            c = t;
        }
    }
    for (int i = 0; i < P; ++i) base[((size_t)slice * P + i) * kSliceWords + lane] = pl[i];
}

// ---- lists ----------------------------------------------------------------------------------------
// One wave per sample.  The features whose bin is not 0 are listed in ascending order as two
// parallel rows: qa[n][k] = bin * 256 (u16, the byte offset of the bin's row in the LDS slice, as
// the dense kernel's quantiser writes it) and fb[n][k] = f * 256 (the byte offset of the feature's
// row in a slice of b).  The list is padded with (feature 0, bin 0) entries - which add exactly the
// 1 that is taken back for every entry - to a multiple of 16; blocks[n] = entries / 16.
constexpr int kListWaves = 4;
template <bool kU8>
__global__ __launch_bounds__(kListWaves *kWave) void sparse_lists_kernel(
    const void *__restrict__ feats, int64_t N, int F, int Fp, int L, const float *__restrict__ lo,
    const float *__restrict__ scale, uint16_t *__restrict__ qa, uint32_t *__restrict__ fb,
    uint32_t *__restrict__ blocks) {
    const int lane = threadIdx.x & (kWave - 1);
    const int64_t n = (int64_t)blockIdx.x * kListWaves + (threadIdx.x >> 6);
    if (n >= N) return;
    uint16_t *qrow = qa + n * Fp;
    uint32_t *frow = fb + n * Fp;
    int listed = 0;
    constexpr int kAhead = 8;   // feature chunks of 64 whose values are fetched together
    for (int f0 = 0; f0 < F; f0 += kAhead * kWave) {
        // all loads first, at clamped indices (what is fetched for f >= F is dropped below)
        float xf[kAhead];
        uint32_t xb[kAhead];
#pragma unroll
        for (int u = 0; u < kAhead; ++u) {
            const int f = min(f0 + u * kWave + lane, F - 1);
            if (kU8)
                xb[u] = reinterpret_cast<const uint8_t *>(feats)[n * F + f];
            else
                xf[u] = reinterpret_cast<const float *>(feats)[n * F + f];
        }
        float lo_u[kAhead], sc_u[kAhead];
        if (!kU8) {
#pragma unroll
            for (int u = 0; u < kAhead; ++u) {
                const int f = min(f0 + u * kWave + lane, F - 1);
                lo_u[u] = lo[f];
                sc_u[u] = scale[f];
            }
        }
#pragma unroll
        for (int u = 0; u < kAhead; ++u) {
            const int f = f0 + u * kWave + lane;
            uint32_t bin = kU8 ? (xb[u] * (uint32_t)L) >> 8 : bin_f32(xf[u], lo_u[u], sc_u[u], L);
            if (f >= F) bin = 0;
            const uint64_t hits = __ballot(bin != 0);
            if (bin != 0) {
                const int k = listed + __popcll(hits & ((1ull << lane) - 1ull));
                qrow[k] = (uint16_t)(bin * (kSliceWords * 4u));
                frow[k] = (uint32_t)f * (kSliceWords * 4u);
            }
            listed += __popcll(hits);
        }
    }
    const int padded = (listed + 15) & ~15;   // <= Fp, which is a multiple of 16 and >= F
    if (listed + lane < padded) {
        qrow[listed + lane] = 0;
        frow[listed + lane] = 0;
    }
    if (lane == 0) blocks[n] = (uint32_t)(padded >> 4);
}

// ---- bundling -------------------------------------------------------------------------------------
// Same block shape as encode_kernel: WAVES waves on one slice of 64 word columns, the slice of e
// in dynamic LDS (no static LDS: the listed bin offsets are absolute LDS addresses), persistent
// blocks, samples dealt round-robin to the waves.  Rows of b come from global memory (L1 / L2, the
// table is a few hundred KB): one 64-bit add per listed entry forms the lane's address from the
// wave-uniform row offset.  (Buffer loads that take the row offset as their scalar offset need no
// such add but measured 9 % slower: the kernel is bound by the issue of these loads, about one per
// 5 clocks per CU, not by the vector ALU.)  The rows of the next block of 16 entries are requested
// before the current block is bundled.
template <int P, int WAVES>
__global__ __launch_bounds__(WAVES *kWave) void encode_sparse_kernel(
    const uint16_t *__restrict__ qa, const uint32_t *__restrict__ fb, const uint32_t *__restrict__ blocks,
    const uint32_t *__restrict__ b, const uint32_t *__restrict__ e, const uint32_t *__restrict__ base,
    uint32_t *__restrict__ hv, int N, int Fp, int L, int W) {
    static_assert(P >= 8, "planes 1..4 take the tree, plane 5 its carry");
    extern __shared__ uint32_t lv[];
    const int slice = blockIdx.x;
    const int lane = threadIdx.x & (kWave - 1);
    const int col = slice * kSliceWords + lane;
    {
        const uint32_t *src = e + (size_t)slice * L * kSliceWords;
        for (int i = threadIdx.x; i < L * kSliceWords; i += WAVES * kWave) lv[i] = src[i];
    }
    __syncthreads();

    // this lane's column of this slice of b; a listed row offset f * 256 (f < F) stays inside it
    const char *bcol = reinterpret_cast<const char *>(b + (size_t)slice * Fp * kSliceWords + lane);
    uint32_t start[P];
#pragma unroll
    for (int i = 0; i < P; ++i) start[i] = base[((size_t)slice * P + i) * kSliceWords + lane];

    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int stride = (int)gridDim.y * WAVES;
    for (int n = (int)blockIdx.y * WAVES + wave; n < N; n += stride) {
        const_u32_ptr qrow = (const_u32_ptr)(uintptr_t)(qa + (int64_t)n * Fp);
        const_u32_ptr frow = (const_u32_ptr)(uintptr_t)(fb + (int64_t)n * Fp);
        const int nb = (int)((const_u32_ptr)(uintptr_t)blocks)[n];

        // counters start at base - 16 * nb (mod 2^P): add the wave-uniform constant plane by plane
        uint32_t pl[P];
        {
            const uint32_t k = (0u - 16u * (uint32_t)nb) & ((1u << P) - 1u);
            uint32_t carry = 0;
#pragma unroll
            for (int i = 0; i < P; ++i) {
                const uint32_t kb = 0u - ((k >> i) & 1u);
                pl[i] = xor3(start[i], kb, carry);
                carry = maj3(start[i], kb, carry);
            }
        }

        // Entry block `blk` of this sample (clamped: a block past the last repeats it, and what is
        // fetched for it is dropped): its 16 row offsets / its 8 pairs of bin offsets, by scalar loads.
        auto offsets_of = [&](int blk, uint32_t (&so)[16]) {
            const int at = (blk < nb ? blk : nb - 1) * 16;
#pragma unroll
            for (int j = 0; j < 16; ++j) so[j] = frow[at + j];
        };
        auto bins_of = [&](int blk, uint32_t (&qp)[8]) {
            const int at = (blk < nb ? blk : nb - 1) * 8;
#pragma unroll
            for (int k = 0; k < 8; ++k) qp[k] = qrow[at + k];
        };
        // request the 16 rows of b at the byte offsets `so`
        auto request = [&](const uint32_t (&so)[16], uint32_t (&w)[16]) {
#pragma unroll
            for (int j = 0; j < 16; ++j)
                w[j] = *reinterpret_cast<const uint32_t *>(bcol + so[j]);
        };
        // bundle an entry block: bin offsets qp, rows of b in w
        auto bundle = [&](const uint32_t (&x)[16], const uint32_t (&w)[16]) {
            uint32_t c2[16];
            uint32_t p0 = pl[0];
#pragma unroll
            for (int j = 0; j < 16; ++j) {
                // p0 + (1 + delta): sum bit ~(p0 ^ e); carry of weight 2 = (e & ~b) | (p0 & ~e)
                c2[j] = __builtin_amdgcn_bitop3_b32(p0, x[j], w[j], 0x74);
                p0 = __builtin_amdgcn_bitop3_b32(p0, x[j], w[j], 0xC3);
            }
            pl[0] = p0;
            ripple<5, P>(pl, Tree<4, 0>::run(pl + 1, c2));
        };

        if (nb > 0) {
            // Two blocks per trip (A even, B odd), nothing conditional inside.  Everything a block
            // needs is asked for a block or more ahead: its row offsets two blocks ahead (scalar
            // loads), its rows of b one block ahead (buffer loads at those offsets), its bin
            // offsets two blocks ahead.  Scalar loads are issued right after a gather has waited
            // on the LDS counter, so the next such wait finds them long done.
            uint32_t wa[16], wb[16], so_a[16], so_b[16], qa_[8], qb_[8], x[16];
            offsets_of(0, so_a);
            offsets_of(1, so_b);
            bins_of(0, qa_);
            bins_of(1, qb_);
            request(so_a, wa);              // (waits for so_a)
            offsets_of(2, so_a);
            pin_schedule();
            int blk = 0;
            for (; blk + 1 < nb; blk += 2) {
                wait_scalar_loads();
                request(so_b, wb);          // rows of block blk + 1
                gather16(x, qa_);           // e rows of block blk
                offsets_of(blk + 3, so_b);
                bins_of(blk + 2, qa_);
                pin_schedule();
                bundle(x, wa);
                request(so_a, wa);          // rows of block blk + 2
                gather16(x, qb_);           // e rows of block blk + 1
                offsets_of(blk + 4, so_a);
                bins_of(blk + 3, qb_);
                pin_schedule();
                bundle(x, wb);
            }
            if (blk < nb) {
                gather16(x, qa_);
                bundle(x, wa);
            }
        }
        if (col < W) hv[(int64_t)n * W + col] = pl[P - 1];
    }
}

typedef void (*sparse_fn)(const uint16_t *, const uint32_t *, const uint32_t *, const uint32_t *, const uint32_t *,
                          const uint32_t *, uint32_t *, int, int, int, int);
struct SparseVariant {
    sparse_fn fn;
    int P, waves;
};
#define HDC_SPARSE(P) {encode_sparse_kernel<P, 4>, P, 4}, {encode_sparse_kernel<P, 8>, P, 8}
static const SparseVariant kSparse[] = {HDC_SPARSE(8), HDC_SPARSE(10), HDC_SPARSE(12), HDC_SPARSE(16)};
#undef HDC_SPARSE

// First use: scratch for the lists and the three derived tables.
static int prepare_sparse(hdc_ctx_impl *c, int P, uint32_t bias, hipStream_t s) {
    if (c->sp_ready) return HDC_OK;
    const bool compact = c->compact;
    if (compact && c->Wc == 0) {   // nothing varies: the dense path already writes constants only
        c->sp_ready = true;
        return HDC_OK;
    }
    const uint32_t *item = compact ? c->citem_d : c->item_d;
    const uint32_t *level = compact ? c->clevel_d : c->level_d;
    const int Wp = compact ? c->Wcp : c->Wp;
    const int nslices = Wp / kSliceWords;
    HDC_HIP(hipSetDevice(c->device));
    auto alloc = [&](void **p, size_t bytes) -> int {
        const hipError_t e = hipMalloc(p, bytes + 256);
        if (e == hipErrorOutOfMemory) {
            (void)hipGetLastError();
            return HDC_ENOMEM;
        }
        HDC_HIP(e);
        return HDC_OK;
    };
    int rc = alloc(reinterpret_cast<void **>(&c->sp_b_d), (size_t)c->Fp * Wp * 4);
    if (rc == HDC_OK) rc = alloc(reinterpret_cast<void **>(&c->sp_e_d), (size_t)c->p.L * Wp * 4);
    if (rc == HDC_OK) rc = alloc(reinterpret_cast<void **>(&c->sp_base_d), (size_t)nslices * P * kSliceWords * 4);
    if (rc == HDC_OK) rc = alloc(reinterpret_cast<void **>(&c->sp_fb_d), (size_t)c->q_rows * c->Fp * 4);
    if (rc == HDC_OK) rc = alloc(reinterpret_cast<void **>(&c->sp_blocks_d), (size_t)c->q_rows * 4);
    if (rc != HDC_OK) {   // all or nothing: a later call starts over
        uint32_t **owned[] = {&c->sp_b_d, &c->sp_e_d, &c->sp_base_d, &c->sp_fb_d, &c->sp_blocks_d};
        for (uint32_t **p : owned) {
            if (*p) (void)hipFree(*p);
            *p = nullptr;
        }
        return rc;
    }
    const int64_t nb = (int64_t)c->Fp * Wp, ne = (int64_t)c->p.L * Wp;
    hipLaunchKernelGGL(xor_row0_kernel, dim3((unsigned)((nb + 255) / 256)), dim3(256), 0, s, item, level, c->Fp,
                       c->p.L, nslices, c->sp_b_d);
    hipLaunchKernelGGL(xor_row0_kernel, dim3((unsigned)((ne + 255) / 256)), dim3(256), 0, s, level, level, c->p.L,
                       c->p.L, nslices, c->sp_e_d);
    hipLaunchKernelGGL(base_planes_kernel, dim3((unsigned)nslices), dim3(kWave), 0, s, c->sp_b_d, c->Fp, P, bias,
                       c->sp_base_d);
    HDC_HIP(hipGetLastError());
    c->sp_ready = true;
    return HDC_OK;
}

// Scratch and derived tables of hdc_encode_sparse (a no-op when they are there).
int reserve_sparse(hdc_ctx_impl *c, hipStream_t s) {
    int P;
    uint32_t bias;
    majority_planes(c, &P, &bias);
    return prepare_sparse(c, P, bias, s);
}

int launch_encode_sparse(hdc_ctx_impl *c, const void *feats, int64_t N, uint32_t *hv, hipStream_t s) {
    int P;
    uint32_t bias;
    majority_planes(c, &P, &bias);
    const int prc = prepare_sparse(c, P, bias, s);
    if (prc != HDC_OK) return prc;
    const bool compact = c->compact;
    if (compact && c->Wc == 0) return launch_encode(c, feats, N, hv, s);
    const int W = compact ? c->Wc : c->W, Wp = compact ? c->Wcp : c->Wp;
    const int nslices = Wp / kSliceWords;
    const int waves = c->p.L > 128 ? 8 : 4;
    const SparseVariant *v = nullptr;
    for (const SparseVariant &k : kSparse)
        if (k.P == P && k.waves == waves) v = &k;
    if (!v) return HDC_ELIMIT;
    const size_t lds = (size_t)c->p.L * kSliceWords * sizeof(uint32_t);
    if (c->sp_bpc == 0) {
        hipFuncAttributes attr;
        HDC_HIP(hipFuncGetAttributes(&attr, reinterpret_cast<const void *>(v->fn)));
        if (attr.sharedSizeBytes != 0) return HDC_ELIMIT;
        int n = 0;
        HDC_HIP(hipOccupancyMaxActiveBlocksPerMultiprocessor(&n, reinterpret_cast<const void *>(v->fn),
                                                             waves * kWave, lds));
        c->sp_bpc = n < 1 ? 1 : n;
    }
    for (int64_t n0 = 0; n0 < N; n0 += c->q_rows) {
        const int64_t n = (N - n0 < c->q_rows) ? N - n0 : c->q_rows;
        const size_t esz = c->p.feat_dtype == HDC_U8 ? 1 : 4;
        const void *x = reinterpret_cast<const uint8_t *>(feats) + (size_t)n0 * c->p.F * esz;
        {
            ProfScope prof(c, HDC_K_QUANTIZE, s);
            const dim3 grid((unsigned)((n + kListWaves - 1) / kListWaves));
            if (c->p.feat_dtype == HDC_U8)
                hipLaunchKernelGGL(sparse_lists_kernel<true>, grid, dim3(kListWaves * kWave), 0, s, x, n, c->p.F,
                                   c->Fp, c->p.L, c->lo_d, c->scale_d, c->q_d, c->sp_fb_d, c->sp_blocks_d);
            else
                hipLaunchKernelGGL(sparse_lists_kernel<false>, grid, dim3(kListWaves * kWave), 0, s, x, n, c->p.F,
                                   c->Fp, c->p.L, c->lo_d, c->scale_d, c->q_d, c->sp_fb_d, c->sp_blocks_d);
        }
        uint32_t *out = hv + (size_t)n0 * c->W;
        {
            int max_waves = (c->num_cus * c->sp_bpc) / nslices * waves;
            if (max_waves < waves) max_waves = waves;
            const int64_t k = (n + max_waves - 1) / max_waves;   // samples per wave
            const int64_t need_waves = (n + k - 1) / k;
            const int per_slice = (int)((need_waves + waves - 1) / waves);
            ProfScope prof(c, HDC_K_ENCODE, s);
            hipLaunchKernelGGL(v->fn, dim3((unsigned)nslices, (unsigned)per_slice), dim3(waves * kWave), lds, s,
                               c->q_d, c->sp_fb_d, c->sp_blocks_d, c->sp_b_d, c->sp_e_d, c->sp_base_d,
                               compact ? c->hvc_d : out, (int)n, c->Fp, c->p.L, W);
        }
        if (compact) launch_expand(c, n, out, s);
        HDC_HIP(hipGetLastError());
    }
    return HDC_OK;
}

}  // namespace hdc
