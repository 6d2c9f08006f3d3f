// Online training (arXiv 2206.04746, Sec. III, Eqs. 2-3 and the caption of Fig. 1).
//
// The method is a dependency chain over the samples: every step needs the class
// accumulators left by the step before (Sec. VI-D2 notes that this rules out parallelism over
// the samples).  What
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

// ---- register-resident variant ---------------------------------------------------------
// Same algorithm, but the accumulators never leave the registers during the call: thread t
// holds acc[c][t + 1024 k] for c < CMAX, k < KPT.  Per step: prefetch the next sample's bits,
// C dot products (fp64 partial sums per thread, DPP butterfly per wave, 16 wave sums through
// LDS), thread c finishes cos_c, then the one or two row updates, whose new squared norms ride
// along to the next step's barrier.  Two block barriers per step.
__device__ __forceinline__ double dpp_shuffle_f64(double v, const int ctrl_sel) {
    // helper for wave_sum_dpp: moves both halves of a double with the same DPP control
    const int lo = __double2loint(v), hi = __double2hiint(v);
    int mlo, mhi;
    switch (ctrl_sel) {
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

// Sum over the 64 lanes, result in every lane.  Rows of 16 lanes fold with DPP (no LDS), the
// four row sums are exchanged with two lane permutes.
__device__ __forceinline__ double wave_sum_dpp(double v) {
    v += dpp_shuffle_f64(v, 0);
    v += dpp_shuffle_f64(v, 1);
    v += dpp_shuffle_f64(v, 2);
    v += dpp_shuffle_f64(v, 3);
    v += __shfl_xor(v, 16, kWave);
    v += __shfl_xor(v, 32, kWave);
    return v;
}

// Sum over the 64 lanes, valid in lane 63 only: four DPP folds inside each row of 16 lanes, then
// the row totals travel by row broadcast (lane 15 of a row into the next row, lane 31 into rows
// 2 and 3) - no LDS round trips, which matters where one wave works alone.
__device__ __forceinline__ double dpp_row_bcast_f64(double v, const int which) {
    const int lo = __double2loint(v), hi = __double2hiint(v);
    int mlo, mhi;
    if (which == 15) {   // row_bcast:15 into rows 1 and 3
        mlo = __builtin_amdgcn_update_dpp(0, lo, 0x142, 0xA, 0xF, false);
        mhi = __builtin_amdgcn_update_dpp(0, hi, 0x142, 0xA, 0xF, false);
    } else {             // row_bcast:31 into rows 2 and 3
        mlo = __builtin_amdgcn_update_dpp(0, lo, 0x143, 0xC, 0xF, false);
        mhi = __builtin_amdgcn_update_dpp(0, hi, 0x143, 0xC, 0xF, false);
    }
    return __hiloint2double(mhi, mlo);
}
__device__ __forceinline__ double wave_sum_to_lane63(double v) {
    v += dpp_shuffle_f64(v, 0);
    v += dpp_shuffle_f64(v, 1);
    v += dpp_shuffle_f64(v, 2);
    v += dpp_shuffle_f64(v, 3);
    v += dpp_row_bcast_f64(v, 15);
    v += dpp_row_bcast_f64(v, 31);
    return v;
}

// x / (sqrt(nn) * root_d) for nn > 0 without the long IEEE square root and division: the
// hardware reciprocal square root estimate refined by two Newton steps (error about one unit in
// the last place), inv_root_d = 1 / sqrt(D) from the host.
__device__ __forceinline__ double cosine_of(double dot, double nn, double inv_root_d) {
    double r = __builtin_amdgcn_rsq(nn);
    r = r * fma(-0.5 * nn * r, r, 1.5);
    r = r * fma(-0.5 * nn * r, r, 1.5);
    return dot * r * inv_root_d;
}

template <int CMAX, int KPT>
__global__ __launch_bounds__(kOnlineThreads) void online_reg_kernel(
    const uint32_t *__restrict__ hv, const int32_t *__restrict__ labels, int64_t N, int epochs,
    float lr, float *acc, int D, int W, int C, double root_d) {
    __shared__ double nrm[CMAX];
    __shared__ double cosv[CMAX];
    __shared__ double red[kOnlineWaves][CMAX];
    __shared__ double red2[kOnlineWaves][2];
    const int tid = threadIdx.x;
    const int lane = tid & (kWave - 1);
    const int wave = tid >> 6;

    // which dimensions this thread owns, and the hv word / bit of each
    float m[CMAX][KPT];
#pragma unroll
    for (int c = 0; c < CMAX; ++c)
#pragma unroll
        for (int k = 0; k < KPT; ++k) {
            const int d = tid + k * kOnlineThreads;
            m[c][k] = (c < C && d < D) ? acc[(int64_t)c * D + d] : 0.0f;
        }
    // squared norms of the rows as handed in
#pragma unroll
    for (int c = 0; c < CMAX; ++c) {
        double p = 0.0;
#pragma unroll
        for (int k = 0; k < KPT; ++k) p += (double)m[c][k] * (double)m[c][k];
        p = wave_sum_dpp(p);
        if (lane == 0) red[wave][c] = p;
    }
    __syncthreads();
    if (tid < CMAX) {
        double s = 0.0;
        for (int w = 0; w < kOnlineWaves; ++w) s += red[w][tid];
        nrm[tid] = s;
    }
    __syncthreads();   // red[] is rewritten by the first step
    // no row has pending norm partials yet
    int upd_y = -1, upd_p = -1;

    auto load_bits = [&](int64_t n) {
        uint32_t bits = 0;
        const uint32_t *h = hv + n * W;
#pragma unroll
        for (int k = 0; k < KPT; ++k) {
            const int d = tid + k * kOnlineThreads;
            if (d < D) bits |= ((h[d >> 5] >> (d & 31)) & 1u) << k;
        }
        return bits;
    };

    const int64_t steps = (int64_t)epochs * N;
    uint32_t bits_next = steps > 0 ? load_bits(0) : 0u;
    int y_next = steps > 0 ? labels[0] : 0;
    int64_t n = 0;
    for (int64_t step = 0; step < steps; ++step) {
        const uint32_t bits = bits_next;
        const int y = y_next;
        const int64_t n1 = (n + 1 == N) ? 0 : n + 1;
        if (step + 1 < steps) {   // next sample's bits and label travel while this step computes
            bits_next = load_bits(n1);
            y_next = labels[n1];
        }
        n = n1;
        if (y < 0 || y >= C) continue;   // uniform

        // ---- similarity of the sample to every class, from the rows as they are now
#pragma unroll
        for (int c = 0; c < CMAX; ++c) {
            if (c < C) {
                double p = 0.0;
#pragma unroll
                for (int k = 0; k < KPT; ++k) {
                    const double v = (double)m[c][k];
                    p += ((bits >> k) & 1u) ? v : -v;
                }
                p = wave_sum_dpp(p);
                if (lane == 0) red[wave][c] = p;
            }
        }
        __syncthreads();
        if (tid < C) {
            // rows changed by the previous step first get their new squared norm
            if (tid == upd_y || tid == upd_p) {
                double s = 0.0;
                const int which = tid == upd_y ? 0 : 1;
                for (int w = 0; w < kOnlineWaves; ++w) s += red2[w][which];
                nrm[tid] = s;
            }
            double dot = 0.0;
            for (int w = 0; w < kOnlineWaves; ++w) dot += red[w][tid];
            const double nn = nrm[tid];
            cosv[tid] = nn == 0.0 ? 0.0 : dot / (sqrt(nn) * root_d);
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
        double py = 0.0, pp = 0.0;
#pragma unroll
        for (int c = 0; c < CMAX; ++c) {
            if (c == y) {
#pragma unroll
                for (int k = 0; k < KPT; ++k) {
                    if (tid + k * kOnlineThreads < D) {
                        const float v = __fadd_rn(m[c][k], ((bits >> k) & 1u) ? w_y : -w_y);
                        m[c][k] = v;
                        py += (double)v * (double)v;
                    }
                }
            } else if (wrong && c == pred) {
#pragma unroll
                for (int k = 0; k < KPT; ++k) {
                    if (tid + k * kOnlineThreads < D) {
                        const float v = __fadd_rn(m[c][k], ((bits >> k) & 1u) ? -w_p : w_p);
                        m[c][k] = v;
                        pp += (double)v * (double)v;
                    }
                }
            }
        }
        py = wave_sum_dpp(py);
        pp = wave_sum_dpp(pp);
        if (lane == 0) {
            red2[wave][0] = py;
            red2[wave][1] = pp;
        }
        upd_y = y;
        upd_p = wrong ? pred : -1;
        // red2 is read after the next step's first barrier and rewritten after its second
    }

#pragma unroll
    for (int c = 0; c < CMAX; ++c)
#pragma unroll
        for (int k = 0; k < KPT; ++k) {
            const int d = tid + k * kOnlineThreads;
            if (c < C && d < D) acc[(int64_t)c * D + d] = m[c][k];
        }
}

// ---- register-resident variant for few classes --------------------------------------------
// As above, but the block-wide sums go through LDS in two stages instead of a butterfly per
// value in every wave: each thread parks its per-class partial dot product (and, from the
// update of the step before, its partial squared norms of the one or two rows that changed) in
// LDS; after the barrier wave c alone adds up column c (16 loads per lane, one butterfly),
// refreshes the norm of row c if that row changed, and its first lane finishes cos_c.  All
// threads then read the C cosines, decide and update their own elements.  Two barriers per
// step; the per-thread partial dot product is KPT FMAs per class on a +-1.0 built from the
// sample's bit (two integer ops per element, shared by the classes).  Needs C + 2 <= 16 waves.
template <int CMAX, int KPT>
__global__ __launch_bounds__(kOnlineThreads) void online_lds_kernel(
    const uint32_t *__restrict__ tbits, int64_t N, int epochs, float lr, float *acc, int D, int C,
    double inv_root_d) {
    static_assert(CMAX + 2 <= kOnlineWaves, "one wave per column");
    extern __shared__ double part_dyn[];   // [CMAX + 2][1024] columns: C dot products, then norm(y), norm(pred)
    auto part_at = [&](int col) { return part_dyn + col * kOnlineThreads; };
    __shared__ double nrm[CMAX];
    __shared__ double cosv[CMAX];
    const int tid = threadIdx.x;
    const int lane = tid & (kWave - 1);
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);

    float m[CMAX][KPT];
#pragma unroll
    for (int c = 0; c < CMAX; ++c)
#pragma unroll
        for (int k = 0; k < KPT; ++k) {
            const int d = tid + k * kOnlineThreads;
            m[c][k] = (c < C && d < D) ? acc[(int64_t)c * D + d] : 0.0f;
        }
    // squared norms of the rows as handed in, through the same two stages
#pragma unroll
    for (int c = 0; c < CMAX; ++c) {
        double p = 0.0;
#pragma unroll
        for (int k = 0; k < KPT; ++k) p += (double)m[c][k] * (double)m[c][k];
        part_at(c)[tid] = p;
    }
    __syncthreads();
    if (wave < C) {
        double s = 0.0;
#pragma unroll
        for (int i = 0; i < kOnlineWaves; ++i) s += part_at(wave)[lane + i * kWave];
        s = wave_sum_dpp(s);
        if (lane == 0) nrm[wave] = s;
    }
    __syncthreads();
    int upd_y = -1, upd_p = -1;   // rows whose norm partials wait in columns CMAX, CMAX + 1

    // low 16 bits of a thread's word: bit k = the sample's bit in the thread's k-th dimension;
    // high 16 bits: label + 1, or 0 for a label outside [0, C).  Prepared by online_bits_kernel,
    // so a step costs one coalesced load per thread.
    static_assert(KPT <= 16, "sample bits share a word with the label");
    auto load_word = [&](int64_t n) { return tbits[n * kOnlineThreads + tid]; };

    // A sample's word (bits and label) is fetched two steps before its step: a first read comes
    // from beyond the L2 and takes longer than one step.
    const int64_t steps = (int64_t)epochs * N;
    int64_t nf = 0;   // sample index of the next fetch
    auto fetch = [&]() {
        const uint32_t w = load_word(nf);   // harmless when it runs past the last step: in bounds, unused
        nf = (nf + 1 == N) ? 0 : nf + 1;
        return w;
    };
    // Two steps per trip, each with a register of its own for the prefetched word; a word is
    // taken apart at the top of its step and its register reloaded at once, for the step two
    // ahead - nothing is copied, so nothing waits for a load that has just been issued.
    uint32_t word_a = fetch(), word_b = fetch();
    auto one_step = [&](uint32_t &word) {
        const uint32_t bits = word & 0xffffu;
        const int y = __builtin_amdgcn_readfirstlane((int)(word >> 16)) - 1;   // -1: label out of range
        word = fetch();
        if (y < 0) return;   // uniform

        // ---- stage 1: this thread's share of every dot product
        {
            // +1.0 where the bit is set, -1.0 where it is not: sign bit = inverted sample bit
            const uint32_t inv = ~bits;
            int sgn_hi[KPT];
#pragma unroll
            for (int k = 0; k < KPT; ++k) sgn_hi[k] = (int)(((inv << (31 - k)) & 0x80000000u) | 0x3FF00000u);
#pragma unroll
            for (int c = 0; c < CMAX; ++c) {
                if (c < C) {
                    double p = 0.0;
#pragma unroll
                    for (int k = 0; k < KPT; ++k) p = fma((double)m[c][k], __hiloint2double(sgn_hi[k], 0), p);
                    part_at(c)[tid] = p;
                }
            }
        }
        __syncthreads();
        // ---- stage 2: wave c finishes column c
        if (wave < C) {
            // (8 loads in flight at a time: the registers of this stage are allocated in every
            // wave, next to the accumulators; two running sums halve the chain of additions)
            const double *colp = part_at(wave) + lane;
            double d0 = 0.0, d1 = 0.0;
#pragma unroll 4
            for (int i = 0; i < kOnlineWaves; i += 2) {
                d0 += colp[i * kWave];
                d1 += colp[(i + 1) * kWave];
            }
            double dot = d0 + d1;
            const int col = wave == upd_y ? CMAX : (wave == upd_p ? CMAX + 1 : -1);   // uniform
            double nn = 0.0;
            if (col >= 0) {
                const double *np = part_at(col) + lane;
                double n0 = 0.0, n1 = 0.0;
#pragma unroll 4
                for (int i = 0; i < kOnlineWaves; i += 2) {
                    n0 += np[i * kWave];
                    n1 += np[(i + 1) * kWave];
                }
                nn = wave_sum_to_lane63(n0 + n1);
            }
            dot = wave_sum_to_lane63(dot);
            if (lane == kWave - 1) {
                if (col >= 0) nrm[wave] = nn; else nn = nrm[wave];
                cosv[wave] = nn == 0.0 ? 0.0 : cosine_of(dot, nn, inv_root_d);
            }
        }
        __syncthreads();
        // ---- stage 3: decision and updates (Eq. 2 always, Eq. 3 only after a wrong prediction)
        int pred = 0;
        double best = cosv[0];
        for (int c = 1; c < C; ++c) {
            const double v = cosv[c];
            if (v > best) { best = v; pred = c; }
        }
        const float w_y = (float)(1.0 - cosv[y]);
        const float w_p = (float)((double)lr * (1.0 - best));
        const bool wrong = pred != y;
        double py = 0.0, pp = 0.0;
#pragma unroll
        for (int c = 0; c < CMAX; ++c) {
            if (c == y) {
#pragma unroll
                for (int k = 0; k < KPT; ++k) {
                    if (tid + k * kOnlineThreads < D) {
                        const float v = __fadd_rn(m[c][k], ((bits >> k) & 1u) ? w_y : -w_y);
                        m[c][k] = v;
                        py = fma((double)v, (double)v, py);
                    }
                }
            } else if (wrong && c == pred) {
#pragma unroll
                for (int k = 0; k < KPT; ++k) {
                    if (tid + k * kOnlineThreads < D) {
                        const float v = __fadd_rn(m[c][k], ((bits >> k) & 1u) ? -w_p : w_p);
                        m[c][k] = v;
                        pp = fma((double)v, (double)v, pp);
                    }
                }
            }
        }
        part_at(CMAX)[tid] = py;
        part_at(CMAX + 1)[tid] = pp;
        upd_y = y;
        upd_p = wrong ? pred : -1;
        // the norm columns are read after the next step's first barrier and rewritten after its
        // second; cosv is rewritten after the next step's first barrier
    };
    for (int64_t step = 0; step < steps; step += 2) {
        one_step(word_a);
        if (step + 1 < steps) one_step(word_b);
    }

#pragma unroll
    for (int c = 0; c < CMAX; ++c)
#pragma unroll
        for (int k = 0; k < KPT; ++k) {
            const int d = tid + k * kOnlineThreads;
            if (c < C && d < D) acc[(int64_t)c * D + d] = m[c][k];
        }
}

// tbits[n][t]: low half = bits of sample n in the dimensions thread t owns (t, t + 1024, ...),
// bit k for the k-th of them (D <= 16384); high half = label + 1, 0 if the label is outside
// [0, C).  One block per sample.
__global__ __launch_bounds__(kOnlineThreads) void online_bits_kernel(const uint32_t *__restrict__ hv,
                                                                      const int32_t *__restrict__ labels, int C,
                                                                      int D, int W, uint32_t *__restrict__ tbits) {
    const int tid = threadIdx.x;
    const uint32_t *h = hv + (int64_t)blockIdx.x * W;
    const int y = labels[blockIdx.x];
    uint32_t word = (y >= 0 && y < C) ? (uint32_t)(y + 1) << 16 : 0u;
    for (int d = tid, k = 0; d < D; d += kOnlineThreads, ++k) word |= ((h[d >> 5] >> (d & 31)) & 1u) << k;
    tbits[(int64_t)blockIdx.x * kOnlineThreads + tid] = word;
}

constexpr int64_t kOnlineChunk = 16384;   // samples whose per-thread bit words are prepared at a time (64 MB)

// The per-thread sample words of the LDS variant of hdc_train_online (64 MB; a no-op when there).
int reserve_online(hdc_ctx_impl *c) {
    if (c->on_bits_d) return HDC_OK;
    HDC_HIP(hipSetDevice(c->device));
    const hipError_t e = hipMalloc(reinterpret_cast<void **>(&c->on_bits_d),
                                   (size_t)kOnlineChunk * kOnlineThreads * sizeof(uint32_t));
    if (e == hipErrorOutOfMemory) {
        (void)hipGetLastError();
        return HDC_ENOMEM;
    }
    HDC_HIP(e);
    return HDC_OK;
}

template <int CMAX, int KPT>
static int launch_online_lds(hdc_ctx_impl *c, const uint32_t *hv, const int32_t *labels, int64_t N,
                             int32_t epochs, float lr, float *acc, hipStream_t s) {
    auto kern = online_lds_kernel<CMAX, KPT>;
    const size_t lds = (size_t)(CMAX + 2) * kOnlineThreads * sizeof(double);
    static_assert(CMAX < (int)(sizeof(c->on_attr_set) / sizeof(c->on_attr_set[0])), "flag per CMAX");
    if (!c->on_attr_set[CMAX] && lds > 64 * 1024) {
        HDC_HIP(hipFuncSetAttribute(reinterpret_cast<const void *>(kern),
                                    hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
        c->on_attr_set[CMAX] = true;
    }
    {
        const int rc = reserve_online(c);
        if (rc != HDC_OK) return rc;
    }
    // A set that fits one chunk is prepared once and walked `epochs` times by one launch; a
    // longer one is walked chunk by chunk, every epoch (the accumulators rest in memory between
    // launches, which changes nothing: they are fp32 there and in the registers).
    const bool one = N <= kOnlineChunk;
    for (int32_t e = 0; e < (one ? 1 : epochs); ++e)
        for (int64_t n0 = 0; n0 < N; n0 += kOnlineChunk) {
            const int64_t n = N - n0 < kOnlineChunk ? N - n0 : kOnlineChunk;
            hipLaunchKernelGGL(online_bits_kernel, dim3((unsigned)n), dim3(kOnlineThreads), 0, s, hv + n0 * c->W,
                               labels + n0, c->p.C, c->p.D, c->W, c->on_bits_d);
            ProfScope prof(c, HDC_K_ONLINE, s);
            hipLaunchKernelGGL(kern, dim3(1), dim3(kOnlineThreads), lds, s, c->on_bits_d, n, one ? (int)epochs : 1,
                               lr, acc, c->p.D, c->p.C, 1.0 / sqrt((double)c->p.D));
        }
    HDC_HIP(hipGetLastError());
    return HDC_OK;
}

template <int CMAX, int KPT>
static int launch_online_reg(hdc_ctx_impl *c, const uint32_t *hv, const int32_t *labels, int64_t N,
                             int32_t epochs, float lr, float *acc, hipStream_t s) {
    ProfScope prof(c, HDC_K_ONLINE, s);
    hipLaunchKernelGGL((online_reg_kernel<CMAX, KPT>), dim3(1), dim3(kOnlineThreads), 0, s, hv, labels, N,
                       (int)epochs, lr, acc, c->p.D, c->W, c->p.C, sqrt((double)c->p.D));
    HDC_HIP(hipGetLastError());
    return HDC_OK;
}

int launch_train_online(hdc_ctx_impl *c, const uint32_t *hv, const int32_t *labels, int64_t N,
                        int32_t epochs, float lr, float *acc, hipStream_t s) {
    const int C = c->p.C;
    // a thread keeps its sample bits in one word: beyond 32768 dimensions the batched trainer runs
    // with batches of one sample, which is the same method (slower: three launches per sample)
    if (c->p.D > 32 * kOnlineThreads) return launch_train_online_batched(c, hv, labels, N, epochs, lr, 1, acc, s);
    // Register-resident kernel when C x (dimensions per thread) fits the register file.
    const int kpt = (c->p.D + kOnlineThreads - 1) / kOnlineThreads;
#define HDC_ONLINE_LDS_CASE(CM, KP) \
    if (C <= CM && kpt <= KP) return launch_online_lds<CM, KP>(c, hv, labels, N, epochs, lr, acc, s)
    HDC_ONLINE_LDS_CASE(8, 2);
    HDC_ONLINE_LDS_CASE(4, 4);
    HDC_ONLINE_LDS_CASE(12, 4);
    HDC_ONLINE_LDS_CASE(2, 10);
    HDC_ONLINE_LDS_CASE(6, 10);
#undef HDC_ONLINE_LDS_CASE
#define HDC_ONLINE_CASE(CM, KP) \
    if (C <= CM && kpt <= KP) return launch_online_reg<CM, KP>(c, hv, labels, N, epochs, lr, acc, s)
    HDC_ONLINE_CASE(8, 1);
    HDC_ONLINE_CASE(32, 1);
    HDC_ONLINE_CASE(80, 1);
    HDC_ONLINE_CASE(8, 2);
    HDC_ONLINE_CASE(40, 2);
    HDC_ONLINE_CASE(4, 4);
    HDC_ONLINE_CASE(20, 4);
    HDC_ONLINE_CASE(2, 10);
    HDC_ONLINE_CASE(6, 10);
    HDC_ONLINE_CASE(2, 16);
#undef HDC_ONLINE_CASE
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
