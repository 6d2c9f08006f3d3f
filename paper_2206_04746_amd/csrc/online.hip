// Online training (arXiv 2206.04746, Sec. III, Eqs. 2-3 and the caption of Fig. 1).
//
// The method is a dependency chain over the samples: every step needs the class
// accumulators left by the step before ("cannot be highly parallelized", Sec. VI-D2).  What
// is parallel is the work inside one step - C dot products over D dimensions and at most two
// row updates - so one persistent workgroup of 1024 threads walks the chain and spreads the
// D dimensions over its lanes.  Thread t owns dimensions t, t+1024, ... in every phase, so a
// thread only ever re-reads accumulator elements it wrote itself; the only communication per
// step is the block-wide reduction of the C dot products (and of the squared norms of the one
// or two rows that changed).  Dot products and norms are summed in fp64, the weights are
// rounded once to fp32 and each accumulator element takes one fp32 add per update.
#include "hdc_internal.h"

namespace hdc {

constexpr int kOnlineThreads = 1024;
constexpr int kOnlineWaves = kOnlineThreads / kWave;

__device__ __forceinline__ double wave_sum(double v) {
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, kWave);
    return v;
}

// LDS doubles: nrm[C] | cosv[C] | red[kOnlineWaves][C]
__global__ __launch_bounds__(kOnlineThreads) void online_kernel(
    const uint32_t *__restrict__ hv, const int32_t *__restrict__ labels, int64_t N, int epochs,
    float lr, float *acc, int D, int W, int C, double root_d) {
    extern __shared__ double sm[];
    double *nrm = sm;
    double *cosv = sm + C;
    double *red = sm + 2 * C;
    const int tid = threadIdx.x;
    const int lane = tid & (kWave - 1);
    const int wave = tid >> 6;

    // squared norms of the rows as handed in
    for (int c = 0; c < C; ++c) {
        double p = 0.0;
        for (int d = tid; d < D; d += kOnlineThreads) {
            const double v = (double)acc[(int64_t)c * D + d];
            p += v * v;
        }
        p = wave_sum(p);
        if (lane == 0) red[wave * C + c] = p;
    }
    __syncthreads();
    for (int c = tid; c < C; c += kOnlineThreads) {
        double s = 0.0;
        for (int w = 0; w < kOnlineWaves; ++w) s += red[w * C + c];
        nrm[c] = s;
    }
    __syncthreads();

    for (int e = 0; e < epochs; ++e) {
        for (int64_t n = 0; n < N; ++n) {
            const int y = labels[n];
            if (y < 0 || y >= C) continue;   // uniform
            const uint32_t *h = hv + n * W;
            // bit k of `bits` = the sample's bit in this thread's k-th dimension (D <= 32768)
            uint32_t bits = 0;
            for (int d = tid, k = 0; d < D; d += kOnlineThreads, ++k)
                bits |= ((h[d >> 5] >> (d & 31)) & 1u) << k;

            // ---- similarity of the sample to every class, from the rows as they are now
            for (int c = 0; c < C; ++c) {
                const float *m = acc + (int64_t)c * D;
                double p = 0.0;
                for (int d = tid, k = 0; d < D; d += kOnlineThreads, ++k) {
                    const double v = (double)m[d];
                    p += ((bits >> k) & 1u) ? v : -v;
                }
                p = wave_sum(p);
                if (lane == 0) red[wave * C + c] = p;
            }
            __syncthreads();
            for (int c = tid; c < C; c += kOnlineThreads) {
                double dot = 0.0;
                for (int w = 0; w < kOnlineWaves; ++w) dot += red[w * C + c];
                const double nn = nrm[c];
                cosv[c] = nn == 0.0 ? 0.0 : dot / (sqrt(nn) * root_d);
            }
            __syncthreads();
            int pred = 0;
            double best = cosv[0];
            for (int c = 1; c < C; ++c) {
                const double v = cosv[c];
                if (v > best) { best = v; pred = c; }
            }
            const float w_y = (float)(1.0 - cosv[y]);
            const float w_p = (float)((double)lr * (1.0 - best));
            const bool wrong = pred != y;

            // ---- updates (Eq. 2 always, Eq. 3 only after a wrong prediction) and new norms
            float *my = acc + (int64_t)y * D;
            float *mp = acc + (int64_t)pred * D;
            double py = 0.0, pp = 0.0;
            for (int d = tid, k = 0; d < D; d += kOnlineThreads, ++k) {
                const bool bit = (bits >> k) & 1u;
                const float ny = __fadd_rn(my[d], bit ? w_y : -w_y);
                my[d] = ny;
                py += (double)ny * (double)ny;
                if (wrong) {
                    const float np = __fadd_rn(mp[d], bit ? -w_p : w_p);
                    mp[d] = np;
                    pp += (double)np * (double)np;
                }
            }
            py = wave_sum(py);
            pp = wave_sum(pp);
            if (lane == 0) {
                red[wave * 2] = py;
                red[wave * 2 + 1] = pp;
            }
            __syncthreads();
            if (tid == 0) {
                double sy = 0.0, sp = 0.0;
                for (int w = 0; w < kOnlineWaves; ++w) {
                    sy += red[w * 2];
                    sp += red[w * 2 + 1];
                }
                nrm[y] = sy;
                if (wrong) nrm[pred] = sp;
            }
            __syncthreads();
        }
    }
}

int launch_train_online(hdc_ctx_impl *c, const uint32_t *hv, const int32_t *labels, int64_t N,
                        int32_t epochs, float lr, float *acc, hipStream_t s) {
    const int C = c->p.C;
    if (c->p.D > 32 * kOnlineThreads) return HDC_ELIMIT;   // a thread keeps its sample bits in one word
    const size_t lds = (size_t)(2 + kOnlineWaves) * (C < 2 ? 2 : C) * sizeof(double);
    auto kern = online_kernel;
    if (lds > 64 * 1024)
        HDC_HIP(hipFuncSetAttribute(reinterpret_cast<const void *>(kern),
                                    hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
    {
        ProfScope prof(c, HDC_K_ONLINE, s);
        hipLaunchKernelGGL(kern, dim3(1), dim3(kOnlineThreads), lds, s, hv, labels, N, (int)epochs, lr,
                           acc, c->p.D, c->W, C, sqrt((double)c->p.D));
    }
    HDC_HIP(hipGetLastError());
    return HDC_OK;
}

// class bit = sign of the accumulator, exactly zero -> tie bit.  One lane per dimension.
__global__ __launch_bounds__(256) void binarize_online_kernel(const float *__restrict__ acc,
                                                               const uint32_t *__restrict__ tie,
                                                               int D, int W, uint32_t *class_hv) {
    const int c = blockIdx.y;
    const int d = blockIdx.x * blockDim.x + threadIdx.x;
    bool bit = false;
    if (d < D) {
        const float a = acc[(int64_t)c * D + d];
        bit = a > 0.0f ? true : a < 0.0f ? false : ((tie[d >> 5] >> (d & 31)) & 1u);
    }
    const uint64_t m = __ballot(bit);
    const int lane = threadIdx.x & (kWave - 1);
    const int w = d >> 5;
    if ((lane & 31) == 0 && w < W)
        class_hv[(int64_t)c * W + w] = (uint32_t)(lane ? (m >> 32) : m);
}

int launch_binarize_online(hdc_ctx_impl *c, const float *acc, uint32_t *class_hv, hipStream_t s) {
    const unsigned bx = (unsigned)((c->W * 32 + 255) / 256);
    hipLaunchKernelGGL(binarize_online_kernel, dim3(bx, (unsigned)c->p.C), dim3(256), 0, s, acc,
                       c->tie_d, c->p.D, c->W, class_hv);
    HDC_HIP(hipGetLastError());
    return HDC_OK;
}

}  // namespace hdc
