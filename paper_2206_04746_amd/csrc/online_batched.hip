// Batched online training (arXiv 2206.04746, Sec. VI-D2; update rules of Sec. III, Eqs. 2-3).
//
// With the class accumulators frozen over a batch, the chain of hdc_train_online breaks into
// three data-parallel steps per batch:
//   forward   dot[n][c] = <acc[c], s_n>   for every sample of the batch        (C x D x B FMAs)
//   weights   cosines, prediction and the two fp32 weights of each sample      (tiny)
//   backward  delta[c][d] = sum over the batch of the weighted +-s_n, then
//             acc = float(double(acc) + delta) and the new squared norms       (<= 2 x D x B adds)
// All sums are fp64.  Dimensions sit on lanes in both big steps (64 consecutive dimensions of a
// sample are exactly one 64-bit lane mask, so the +-1 of a lane is one v_cndmask on the mask);
// fp64 FMA on the vector unit has the same peak as the fp64 matrix path on this chip, so there
// is nothing to gain from MFMA here.
#include <type_traits>

#include "hdc_internal.h"

namespace hdc {

typedef const uint32_t __attribute__((address_space(4))) *kptr_u32;

// One record per sample of the batch, written by the weights step, read by the backward step.
struct OnlineWeight {
    int32_t y;      // label, or -1: sample skipped
    int32_t pred;   // predicted class if it differs from y, else -1
    float w_y;      // float(1 - cos_y)
    float w_p;      // float(lr * (1 - cos_pred))
};
typedef const OnlineWeight __attribute__((address_space(4))) *kptr_w;

constexpr int kFwdWaves = 4;     // waves per forward block
constexpr int kFwdGroups = 16;   // 64-dimension groups per forward slice
constexpr int kFwdClasses = 2;   // classes per forward wave
constexpr int kBwdMaxWaves = 16;
constexpr int kBwdSlots = 256;   // (waves x classes) rows of 64 doubles in the backward LDS: 128 KB

__device__ __forceinline__ double dpp_f64(double v, const int sel) {
    const int lo = __double2loint(v), hi = __double2hiint(v);
    int mlo, mhi;
    switch (sel) {
        case 0: mlo = __builtin_amdgcn_update_dpp(0, lo, 0xB1, 0xF, 0xF, true);    // quad_perm 1,0,3,2
                mhi = __builtin_amdgcn_update_dpp(0, hi, 0xB1, 0xF, 0xF, true); break;
        case 1: mlo = __builtin_amdgcn_update_dpp(0, lo, 0x4E, 0xF, 0xF, true);    // quad_perm 2,3,0,1
                mhi = __builtin_amdgcn_update_dpp(0, hi, 0x4E, 0xF, 0xF, true); break;
        case 2: mlo = __builtin_amdgcn_update_dpp(0, lo, 0x141, 0xF, 0xF, true);   // row_half_mirror
                mhi = __builtin_amdgcn_update_dpp(0, hi, 0x141, 0xF, 0xF, true); break;
        default: mlo = __builtin_amdgcn_update_dpp(0, lo, 0x140, 0xF, 0xF, true);  // row_mirror
                 mhi = __builtin_amdgcn_update_dpp(0, hi, 0x140, 0xF, 0xF, true); break;
    }
    return __hiloint2double(mhi, mlo);
}

// Sum over the 64 lanes, result in every lane (fixed order).
__device__ __forceinline__ double wave_sum_f64(double v) {
    v += dpp_f64(v, 0);
    v += dpp_f64(v, 1);
    v += dpp_f64(v, 2);
    v += dpp_f64(v, 3);
    v += __shfl_xor(v, 16, kWave);
    v += __shfl_xor(v, 32, kWave);
    return v;
}

// +1.0 in the lanes whose bit of the 64-bit mask is set, -1.0 in the others.  The mask lives
// in a scalar register pair, which is the form v_cndmask takes its lane select in.
__device__ __forceinline__ double lane_sign(uint64_t mask) {
    int hi;
    const int neg = (int)0xBFF00000u, pos = 0x3FF00000;
    asm("v_cndmask_b32_e64 %0, %1, %2, %3" : "=v"(hi) : "v"(neg), "v"(pos), "s"(mask));
    return __hiloint2double(hi, 0);
}

// 64-bit lane mask of dimension group `g` (dimensions 64 g .. 64 g + 63) of one sample row.
// `row` and `g` are wave-uniform: scalar loads.  With FULL the caller guarantees that both
// words lie inside the row; otherwise words past the row read as zero (the load itself is
// clamped to the row, so that it stays unconditional).
template <bool FULL>
__device__ __forceinline__ uint64_t group_mask(kptr_u32 row, int g, int W) {
    if (FULL) return (uint64_t)row[2 * g] | ((uint64_t)row[2 * g + 1] << 32);
    const int i0 = 2 * g, i1 = 2 * g + 1;
    const uint32_t lo = row[i0 < W ? i0 : W - 1], hi = row[i1 < W ? i1 : W - 1];
    return (uint64_t)(i0 < W ? lo : 0u) | ((uint64_t)(i1 < W ? hi : 0u) << 32);
}

// ---- forward: partial dot products ---------------------------------------------------------
// grid (slices, class chunks, sample tiles).  A wave keeps acc[c0 .. c0+CC)[its 64 KPT
// dimensions] in registers as fp64 and walks `spw` samples; per sample and class it leaves one
// partial dot product part[slice][n][c].
template <int CC, int KPT>
__global__ __launch_bounds__(kFwdWaves *kWave) void online_fwd_kernel(
    const uint32_t *__restrict__ hv, int64_t nb, const float *__restrict__ acc, int D, int W, int C,
    int spw, double *__restrict__ part) {
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int slice = blockIdx.x;
    const int c0 = blockIdx.y * CC;
    const int64_t n0 = ((int64_t)blockIdx.z * kFwdWaves + wave) * spw;
    if (n0 >= nb) return;   // the kernel has no barrier
    const int64_t n1 = n0 + spw < nb ? n0 + spw : nb;

    double v[CC][KPT];
#pragma unroll
    for (int j = 0; j < CC; ++j)
#pragma unroll
        for (int k = 0; k < KPT; ++k) {
            const int d = (slice * KPT + k) * kWave + lane;
            v[j][k] = (c0 + j < C && d < D) ? (double)acc[(int64_t)(c0 + j) * D + d] : 0.0;
        }

    auto walk = [&](auto full) {
        constexpr bool FULL = decltype(full)::value;
        for (int64_t n = n0; n < n1; ++n) {
            kptr_u32 row = (kptr_u32)(hv + n * W);
            double p[CC];
#pragma unroll
            for (int j = 0; j < CC; ++j) p[j] = 0.0;
#pragma unroll
            for (int k = 0; k < KPT; ++k) {
                const double sgn = lane_sign(group_mask<FULL>(row, slice * KPT + k, W));
#pragma unroll
                for (int j = 0; j < CC; ++j) p[j] = fma(v[j][k], sgn, p[j]);
            }
#pragma unroll
            for (int j = 0; j < CC; ++j) {
                const double t = wave_sum_f64(p[j]);
                if (lane == 0 && c0 + j < C) part[((int64_t)slice * nb + n) * C + c0 + j] = t;
            }
        }
    };
    if ((slice + 1) * KPT * 2 <= W)
        walk(std::true_type{});
    else
        walk(std::false_type{});
}

// ---- weights ---------------------------------------------------------------------------------
// One thread per sample: finishes the dot products (slices in ascending order), cosines against
// the frozen rows, prediction (lowest class among equals) and the two weights.
__global__ __launch_bounds__(256) void online_weights_kernel(
    const double *__restrict__ part, int slices, int64_t nb, const int32_t *__restrict__ labels,
    const double *__restrict__ normpart, int G, int C, double root_d, float lr,
    OnlineWeight *__restrict__ out) {
    extern __shared__ double nrm[];   // [C] squared norms of the frozen rows
    for (int c = threadIdx.x; c < C; c += blockDim.x) {
        double s = 0.0;
        for (int g = 0; g < G; ++g) s += normpart[(int64_t)c * G + g];
        nrm[c] = s;
    }
    __syncthreads();
    const int64_t n = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (n >= nb) return;
    const int y = labels[n];
    OnlineWeight r;
    r.y = -1;
    r.pred = -1;
    r.w_y = 0.0f;
    r.w_p = 0.0f;
    if (y >= 0 && y < C) {
        double best = 0.0, cos_y = 0.0;
        int pred = 0;
        for (int c = 0; c < C; ++c) {
            double dot = 0.0;
            for (int s = 0; s < slices; ++s) dot += part[((int64_t)s * nb + n) * C + c];
            const double nn = nrm[c];
            const double cs = nn == 0.0 ? 0.0 : dot / (sqrt(nn) * root_d);
            if (c == 0 || cs > best) {
                best = cs;
                pred = c;
            }
            if (c == y) cos_y = cs;
        }
        r.y = y;
        r.pred = pred != y ? pred : -1;
        r.w_y = (float)(1.0 - cos_y);
        r.w_p = (float)((double)lr * (1.0 - best));
    }
    out[n] = r;
}

// ---- backward: batch sum, update, new norms ----------------------------------------------------
// One block per group of 64 dimensions; its waves split the batch into contiguous runs.  A wave
// adds the weighted +-1 of each of its samples into its own LDS rows (one row of 64 doubles
// per class of the window [c_lo, c_lo + c_n)), in sample order; after the barrier the rows of
// the waves are added in wave order, the accumulators take the sum in one rounding, and the
// squared norm of this block's 64 elements of each row goes to normpart[c][g].
__global__ __launch_bounds__(kBwdMaxWaves *kWave) void online_bwd_kernel(
    const uint32_t *__restrict__ hv, const OnlineWeight *__restrict__ wts, int64_t B, float *acc,
    int D, int W, int c_lo, int c_n, int G, double *__restrict__ normpart) {
    extern __shared__ double rows[];   // [waves][c_n][64]
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int nw = blockDim.x >> 6;
    const int g = blockIdx.x;
    double *mine = rows + (int64_t)wave * c_n * kWave;
    for (int c = 0; c < c_n; ++c) mine[c * kWave + lane] = 0.0;

    const int64_t per = (B + nw - 1) / nw;
    const int64_t n0 = wave * per;
    const int64_t n1 = n0 + per < B ? n0 + per : B;
    kptr_w rec = (kptr_w)wts;
    for (int64_t n = n0; n < n1; ++n) {
        const int y = rec[n].y;
        if (y < 0) continue;
        const int pred = rec[n].pred;
        const int yy = y - c_lo, pp = pred - c_lo;
        const bool hit_y = yy >= 0 && yy < c_n;
        const bool hit_p = pred >= 0 && pp >= 0 && pp < c_n;
        if (!hit_y && !hit_p) continue;
        const double sgn = lane_sign(group_mask<false>((kptr_u32)(hv + n * W), g, W));
        if (hit_y) mine[yy * kWave + lane] += (double)rec[n].w_y * sgn;
        if (hit_p) mine[pp * kWave + lane] -= (double)rec[n].w_p * sgn;
    }
    __syncthreads();

    const int d = g * kWave + lane;
    for (int c = wave; c < c_n; c += nw) {
        double s = 0.0;
        for (int w = 0; w < nw; ++w) s += rows[((int64_t)w * c_n + c) * kWave + lane];
        double q = 0.0;
        if (d < D) {
            float *a = acc + (int64_t)(c_lo + c) * D + d;
            const float nv = (float)((double)*a + s);
            *a = nv;
            q = (double)nv * (double)nv;
        }
        q = wave_sum_f64(q);
        if (lane == 0) normpart[(int64_t)(c_lo + c) * G + g] = q;
    }
}

// ---- host side ---------------------------------------------------------------------------------
static int grow(void **p, size_t *have, size_t want) {
    if (*have >= want) return HDC_OK;
    if (*p) HDC_HIP(hipFree(*p));   // waits for the device: nothing still reads the old buffer
    *p = nullptr;
    *have = 0;
    const hipError_t e = hipMalloc(p, want + 256);
    if (e == hipErrorOutOfMemory) {
        (void)hipGetLastError();
        return HDC_ENOMEM;
    }
    HDC_HIP(e);
    *have = want;
    return HDC_OK;
}

static int launch_bwd(hdc_ctx_impl *c, const uint32_t *hv, const OnlineWeight *wts, int64_t B, float *acc,
                      int G, double *normpart, hipStream_t s) {
    const int C = c->p.C;
    for (int c_lo = 0; c_lo < C; c_lo += kBwdSlots) {
        const int c_n = C - c_lo < kBwdSlots ? C - c_lo : kBwdSlots;
        int nw = kBwdSlots / c_n;
        if (nw > kBwdMaxWaves) nw = kBwdMaxWaves;
        while (nw > 1 && (int64_t)(nw / 2) * 4 >= B) nw /= 2;   // at least a few samples per wave
        const size_t lds = (size_t)nw * c_n * kWave * sizeof(double);
        ProfScope prof(c, HDC_K_ONLINE_BWD, s);
        hipLaunchKernelGGL(online_bwd_kernel, dim3((unsigned)G), dim3((unsigned)nw * kWave), lds, s, hv, wts,
                           B, acc, c->p.D, c->W, c_lo, c_n, G, normpart);
        HDC_HIP(hipGetLastError());
    }
    return HDC_OK;
}

int launch_train_online_batched(hdc_ctx_impl *c, const uint32_t *hv, const int32_t *labels, int64_t N,
                                int32_t epochs, float lr, int64_t batch, float *acc, hipStream_t s) {
    const int C = c->p.C, D = c->p.D, W = c->W;
    const int G = (D + kWave - 1) / kWave;
    const int slices = (G + kFwdGroups - 1) / kFwdGroups;
    const int chunks = (C + kFwdClasses - 1) / kFwdClasses;
    if (batch > N) batch = N;

    // forward + weights run over sub-batches of at most `sb` samples (bounds the partial buffer)
    int64_t sb = (int64_t)(256u << 20) / ((int64_t)slices * C * (int64_t)sizeof(double));
    if (sb > 4096) sb = 4096;
    if (sb < 64) sb = 64;
    if (sb > batch) sb = batch;
    {
        void *p = c->ob_part_d;
        HDC_HIP(hipSetDevice(c->device));
        int rc = grow(&p, &c->ob_part_bytes, (size_t)slices * sb * C * sizeof(double));
        c->ob_part_d = static_cast<double *>(p);
        if (rc != HDC_OK) return rc;
        p = c->ob_wts_d;
        rc = grow(&p, &c->ob_wts_bytes, (size_t)batch * sizeof(OnlineWeight));
        c->ob_wts_d = p;
        if (rc != HDC_OK) return rc;
        p = c->ob_norm_d;
        rc = grow(&p, &c->ob_norm_bytes, (size_t)C * G * sizeof(double));
        c->ob_norm_d = static_cast<double *>(p);
        if (rc != HDC_OK) return rc;
    }
    double *part = c->ob_part_d;
    OnlineWeight *wts = static_cast<OnlineWeight *>(c->ob_wts_d);
    double *normpart = c->ob_norm_d;
    if (!c->ob_attr_set) {
        HDC_HIP(hipFuncSetAttribute(reinterpret_cast<const void *>(online_bwd_kernel),
                                    hipFuncAttributeMaxDynamicSharedMemorySize,
                                    (int)(kBwdSlots * kWave * sizeof(double))));
        c->ob_attr_set = true;
    }

    // squared norms of the rows as handed in: a backward step over an empty batch
    int rc = launch_bwd(c, hv, wts, 0, acc, G, normpart, s);
    if (rc != HDC_OK) return rc;
    const double root_d = sqrt((double)D);
    for (int32_t e = 0; e < epochs; ++e)
        for (int64_t b0 = 0; b0 < N; b0 += batch) {
            const int64_t B = b0 + batch < N ? batch : N - b0;
            for (int64_t s0 = 0; s0 < B; s0 += sb) {
                const int64_t nb = s0 + sb < B ? sb : B - s0;
                int64_t spw = (nb * slices * chunks + 2047) / 2048;
                if (spw < 1) spw = 1;
                if (spw > 64) spw = 64;
                const int64_t tiles = (nb + kFwdWaves * spw - 1) / (kFwdWaves * spw);
                {
                    ProfScope prof(c, HDC_K_ONLINE_FWD, s);
                    hipLaunchKernelGGL((online_fwd_kernel<kFwdClasses, kFwdGroups>),
                                       dim3((unsigned)slices, (unsigned)chunks, (unsigned)tiles),
                                       dim3(kFwdWaves * kWave), 0, s, hv + (b0 + s0) * W, nb, acc, D, W, C,
                                       (int)spw, part);
                }
                HDC_HIP(hipGetLastError());
                hipLaunchKernelGGL(online_weights_kernel, dim3((unsigned)((nb + 255) / 256)), dim3(256),
                                   (size_t)C * sizeof(double), s, part, slices, nb, labels + b0 + s0, normpart,
                                   G, C, root_d, lr, wts + s0);
                HDC_HIP(hipGetLastError());
            }
            rc = launch_bwd(c, hv + b0 * W, wts, B, acc, G, normpart, s);
            if (rc != HDC_OK) return rc;
        }
    return HDC_OK;
}

}  // namespace hdc
