// Classical training (arXiv 2206.04746, Sec. III): acc[c][d] += hv[n][d] for c = label[n],
// and the majority vote that turns the sums into class vectors.
//
// The per-dimension sum down a column of packed rows is the paper's "vertical summation"
// (Sec. IV-B2).  Here it needs no transposition: a lane owns one 32-bit word column and
// keeps the 32 counts bit-sliced (plane i = bit i of each count); adding rows is carry-save
// arithmetic with v_bitop3_b32 full adders, about 3 VALU ops per streamed word, so the kernel
// stays HBM-bound.  Rows are first grouped by class (a counting sort of the labels, only the
// row indices move), then every wave streams up to kRowBlock rows of ONE class and flushes
// its counters to acc with integer atomics - sums of integers, so any order gives the same
// bits.
#include "hdc_internal.h"

namespace hdc {

constexpr int kRowBlock = 2040;   // rows per wave before a flush (count fits kPlanes bits)
constexpr int kPlanes = 11;

// ---- grouping rows by class ----------------------------------------------------------
// cnt[c] = rows with label c; cnt[C] = rows with a label outside [0, C) (skipped later).
__global__ void clear_counts_kernel(uint32_t *cnt, uint32_t *cur, int C) {
    for (int i = threadIdx.x; i <= C; i += blockDim.x) {
        cnt[i] = 0;
        if (i < C) cur[i] = 0;
    }
}

__global__ __launch_bounds__(256) void count_labels_kernel(const int32_t *__restrict__ labels,
                                                            int64_t N, int C, uint32_t *cnt) {
    extern __shared__ uint32_t h[];
    for (int i = threadIdx.x; i <= C; i += blockDim.x) h[i] = 0;
    __syncthreads();
    for (int64_t n = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; n < N;
         n += (int64_t)gridDim.x * blockDim.x) {
        const int32_t y = labels[n];
        atomicAdd(&h[(y >= 0 && y < C) ? y : C], 1u);
    }
    __syncthreads();
    for (int i = threadIdx.x; i <= C; i += blockDim.x)
        if (h[i]) atomicAdd(&cnt[i], h[i]);
}

// One block: exclusive prefix of the class counts (row offsets into perm) and of the
// per-class row-block counts (work list of the accumulate kernel); class_n += counts.
__global__ void scan_counts_kernel(const uint32_t *cnt, uint32_t *off, uint32_t *blk, int C,
                                   int64_t *class_n) {
    if (threadIdx.x == 0) {
        uint32_t o = 0, b = 0;
        for (int c = 0; c < C; ++c) {
            off[c] = o;
            blk[c] = b;
            o += cnt[c];
            b += (cnt[c] + kRowBlock - 1) / kRowBlock;
        }
        off[C] = o;
        blk[C] = b;
    }
    for (int c = threadIdx.x; c < C; c += blockDim.x) class_n[c] += (int64_t)cnt[c];
}

__global__ __launch_bounds__(256) void scatter_rows_kernel(const int32_t *__restrict__ labels,
                                                            int64_t N, int C,
                                                            const uint32_t *__restrict__ off,
                                                            uint32_t *cur, uint32_t *perm) {
    for (int64_t n = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; n < N;
         n += (int64_t)gridDim.x * blockDim.x) {
        const int32_t y = labels[n];
        if (y >= 0 && y < C) perm[off[y] + atomicAdd(&cur[y], 1u)] = (uint32_t)n;
    }
}

// ---- vertical count ------------------------------------------------------------------
typedef const uint32_t __attribute__((address_space(4))) *const_u32_ptr;
constexpr int kAccWaves = 4;

// grid.x = row-block index in the work list (an upper bound; surplus blocks exit),
// grid.y = group of kAccWaves word slices.  A wave = one slice of 64 word columns.
__global__ __launch_bounds__(kAccWaves * kWave) void accumulate_kernel(
    const uint32_t *__restrict__ hv, const uint32_t *__restrict__ perm,
    const uint32_t *__restrict__ cnt, const uint32_t *__restrict__ off,
    const uint32_t *__restrict__ blk, int C, int W, int D, int32_t *acc) {
    const uint32_t item = blockIdx.x;
    if (item >= blk[C]) return;
    // class of this work item: last c with blk[c] <= item (blk is non-decreasing)
    int lo = 0, hi = C - 1;
    while (lo < hi) {
        const int mid = (lo + hi + 1) >> 1;
        if (blk[mid] <= item) lo = mid; else hi = mid - 1;
    }
    const int c = lo;
    const uint32_t first = (item - blk[c]) * kRowBlock;
    const uint32_t rows = min((uint32_t)kRowBlock, cnt[c] - first);
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int lane = threadIdx.x & (kWave - 1);
    const int col = (blockIdx.y * kAccWaves + wave) * kSliceWords + lane;
    if (col >= W) return;

    const_u32_ptr idx = (const_u32_ptr)(uintptr_t)(perm + off[c] + first);   // wave-uniform
    uint32_t pl[kPlanes];
#pragma unroll
    for (int i = 0; i < kPlanes; ++i) pl[i] = 0;

    for (uint32_t r0 = 0; r0 < rows; r0 += 8) {
        uint32_t x[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            x[j] = 0;
            if (r0 + j < rows) {   // uniform
                const uint32_t *row = hv + (int64_t)idx[r0 + j] * W;
                x[j] = row[col];
            }
        }
        uint32_t a, b, p, c2a, c2b, c3;
        p = pl[0]; a = maj3(p, x[0], x[1]); p = xor3(p, x[0], x[1]);
        b = maj3(p, x[2], x[3]); p = xor3(p, x[2], x[3]); pl[0] = p;
        p = pl[1]; c2a = maj3(p, a, b); pl[1] = xor3(p, a, b);
        p = pl[0]; a = maj3(p, x[4], x[5]); p = xor3(p, x[4], x[5]);
        b = maj3(p, x[6], x[7]); p = xor3(p, x[6], x[7]); pl[0] = p;
        p = pl[1]; c2b = maj3(p, a, b); pl[1] = xor3(p, a, b);
        p = pl[2]; c3 = maj3(p, c2a, c2b); pl[2] = xor3(p, c2a, c2b);
#pragma unroll
        for (int i = 3; i < kPlanes; ++i) {
            const uint32_t t = pl[i] & c3;
            pl[i] ^= c3;
            c3 = t;
        }
    }

    int32_t *dst = acc + (int64_t)c * D + (int64_t)col * 32;
    const int valid = min(32, D - col * 32);
    for (int b = 0; b < valid; ++b) {
        uint32_t v = 0;
#pragma unroll
        for (int i = 0; i < kPlanes; ++i) v |= ((pl[i] >> b) & 1u) << i;
        if (v) atomicAdd(&dst[b], (int32_t)v);
    }
}

int launch_train_classical(hdc_ctx_impl *c, const uint32_t *hv, const int32_t *labels, int64_t N,
                           int32_t *acc, int64_t *class_n, hipStream_t s) {
    const int C = c->p.C;
    for (int64_t n0 = 0; n0 < N; n0 += c->perm_rows) {
        const int64_t n = (N - n0 < c->perm_rows) ? N - n0 : c->perm_rows;
        const uint32_t *hv0 = hv + (size_t)n0 * c->W;
        const int32_t *lab0 = labels + n0;
        const unsigned gb = (unsigned)((n + 256 * 8 - 1) / (256 * 8));
        const unsigned nb = gb < 1 ? 1 : (gb > 2048 ? 2048 : gb);
        hipLaunchKernelGGL(clear_counts_kernel, dim3(1), dim3(256), 0, s, c->cls_cnt_d, c->cls_cur_d, C);
        hipLaunchKernelGGL(count_labels_kernel, dim3(nb), dim3(256), (size_t)(C + 1) * 4, s, lab0, n, C,
                           c->cls_cnt_d);
        hipLaunchKernelGGL(scan_counts_kernel, dim3(1), dim3(256), 0, s, c->cls_cnt_d, c->cls_off_d,
                           c->cls_blk_d, C, class_n);
        hipLaunchKernelGGL(scatter_rows_kernel, dim3(nb), dim3(256), 0, s, lab0, n, C, c->cls_off_d,
                           c->cls_cur_d, c->perm_d);
        const unsigned items = (unsigned)((n + kRowBlock - 1) / kRowBlock) + (unsigned)C;
        const unsigned slice_groups = (unsigned)((c->Wp / kSliceWords + kAccWaves - 1) / kAccWaves);
        {
            ProfScope prof(c, HDC_K_ACCUMULATE, s);
            hipLaunchKernelGGL(accumulate_kernel, dim3(items, slice_groups), dim3(kAccWaves * kWave), 0,
                               s, hv0, c->perm_d, c->cls_cnt_d, c->cls_off_d, c->cls_blk_d, C, c->W,
                               c->p.D, acc);
        }
        HDC_HIP(hipGetLastError());
    }
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
