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
constexpr int kBwdMaxWaves = 16;
constexpr int kBwdUnroll = 8;    // samples per trip of the backward loop
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

// mem += v on an LDS double that only this lane touches; nothing is returned, so the wave does
// not wait for it (ds_add_f64).
__device__ __forceinline__ void lds_add(double *mem, double v) {
    (void)__hip_atomic_fetch_add(mem, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WAVEFRONT);
}

// 64-bit lane mask of dimension group `g` (dimensions 64 g .. 64 g + 63) of one sample row.
// `row` and `g` are wave-uniform: scalar loads.  SAFE = 2: both words lie inside the row;
// SAFE = 1: the low word does, the high word may be the first word past the row (odd W) and
// then reads as zero; SAFE = 0: either may lie past the row.  A load that might leave the row
// is clamped to it, so that it stays unconditional.
template <int SAFE>
__device__ __forceinline__ uint64_t group_mask(kptr_u32 row, int g, int W) {
    const int i0 = 2 * g, i1 = 2 * g + 1;
    const uint32_t lo = SAFE >= 1 ? row[i0] : row[i0 < W ? i0 : W - 1];
    const uint32_t hi = SAFE >= 2 ? row[i1] : row[i1 < W ? i1 : W - 1];
    return (uint64_t)((SAFE >= 1 || i0 < W) ? lo : 0u) | ((uint64_t)((SAFE >= 2 || i1 < W) ? hi : 0u) << 32);
}

// Scalar loads return in any order, so the only wait there is for them is "all of them".  A
// loop that wants the next trip's scalar operands in flight while it computes therefore waits
// at the top of a trip (for the loads issued a trip ago), issues the next loads, and pins them
// above the arithmetic.
__device__ __forceinline__ void wait_scalar_loads() {
    __builtin_amdgcn_sched_barrier(0);    // keeps the wait below the arithmetic of the trip before
    __builtin_amdgcn_s_waitcnt(0xC07F);   // lgkmcnt(0)
}
__device__ __forceinline__ void pin_schedule() { __builtin_amdgcn_sched_barrier(0); }

// ---- forward: partial dot products ---------------------------------------------------------
// grid (slices, class chunks, sample tiles).  A wave keeps acc[c0 .. c0+CC)[its 64 KPT
// dimensions] in registers as fp64 and walks `spw` samples, NS at a time; per sample and class
// it leaves one partial dot product part[slice][n][c].  Per sample and group of 64 dimensions:
// one v_cndmask for the signs, CC FMAs.  The NS * CC = 16 per-lane sums of a trip are reduced
// over the lanes together: each lane parks its 16 values in the wave's LDS tile, then lane
// (j, r) adds up value j of source lanes 16 r .. 16 r + 15 and two lane exchanges fold the four
// r.  That is ~4 issue slots per value instead of ~20 for a butterfly per value.  The masks of
// the next sample are loaded (scalar) while the current one computes.
constexpr int kFwdVals = 16;                 // values reduced per trip = NS * CC
constexpr int kFwdStride = kWave + 1;        // doubles per value row in the LDS tile (+1: banks)

template <int CC, int KPT>
__global__ __launch_bounds__(kFwdWaves *kWave) void online_fwd_kernel(
    const uint32_t *__restrict__ hv, int64_t nb, const float *__restrict__ acc, int D, int W, int C,
    int spw, double *__restrict__ part) {
    constexpr int NS = kFwdVals / CC;
    __shared__ double xch[kFwdWaves][kFwdVals * kFwdStride];
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int slice = blockIdx.x;
    const int c0 = blockIdx.y * CC;
    const int64_t n0 = ((int64_t)blockIdx.z * kFwdWaves + wave) * spw;
    const int64_t n1 = n0 + spw < nb ? n0 + spw : nb;
    double *buf = xch[wave];

    // The last slice is shifted back to end with the last group, so that its 2 KPT words are
    // (but for the word after an odd W) inside the row like everyone else's; the groups it
    // shares with the slice before it count there, not here.
    const int G = (D + kWave - 1) / kWave;
    const int g_own = slice * KPT;
    const int g_base = (g_own + KPT <= G || G < KPT) ? g_own : G - KPT;

    // The block's waves all work on the same slice of the class rows: it is fetched once per
    // block (every thread a few elements; clamped addresses, values dropped afterwards, so that
    // all loads are in flight together) and handed to the waves through LDS.  At launch every
    // block on the chip asks for the same few hundred KB at once, so fewer requests count.
    float *stage = reinterpret_cast<float *>(&xch[0][0]);   // CC * KPT * 64 floats; the tiles are not in use yet
    static_assert(sizeof(float) * CC * KPT * kWave <= sizeof(xch), "staging area");
    {
        constexpr int kPerThread = CC * KPT * kWave / (kFwdWaves * kWave);
        float x[kPerThread];
#pragma unroll
        for (int i = 0; i < kPerThread; ++i) {
            const int e = threadIdx.x + i * kFwdWaves * kWave;   // (j, k, lane) flattened
            const int j = e / (KPT * kWave), k = (e / kWave) % KPT;
            const int d = (g_base + k) * kWave + (e % kWave);
            const int cc = c0 + j < C ? c0 + j : C - 1, dd = d < D ? d : D - 1;
            x[i] = acc[(int64_t)cc * D + dd];
            if (!(c0 + j < C && d < D && g_base + k >= g_own)) x[i] = 0.0f;
        }
#pragma unroll
        for (int i = 0; i < kPerThread; ++i) stage[threadIdx.x + i * kFwdWaves * kWave] = x[i];
    }
    __syncthreads();
    double v[CC][KPT];
#pragma unroll
    for (int j = 0; j < CC; ++j)
#pragma unroll
        for (int k = 0; k < KPT; ++k) v[j][k] = (double)stage[(j * KPT + k) * kWave + lane];
    __syncthreads();        // the staging area becomes the waves' reduction tiles
    if (n0 >= nb) return;   // no block barrier below this line

    auto walk = [&](auto safe) {
        constexpr int SAFE = decltype(safe)::value;
        auto masks = [&](int64_t n, uint64_t(&m)[KPT]) {
            kptr_u32 row = (kptr_u32)(hv + n * W);
#pragma unroll
            for (int k = 0; k < KPT; ++k)
                m[k] = k + 1 < KPT || SAFE == 2 ? group_mask<(SAFE > 0 ? 2 : 0)>(row, g_base + k, W)
                                                : group_mask<SAFE>(row, g_base + k, W);
        };
        uint64_t nxt[KPT];
        masks(n0, nxt);
        for (int64_t n = n0; n < n1; n += NS) {
            double p[NS][CC];
#pragma unroll
            for (int u = 0; u < NS; ++u) {
                uint64_t cur[KPT];
                wait_scalar_loads();
#pragma unroll
                for (int k = 0; k < KPT; ++k) cur[k] = nxt[k];
                // rows past the wave's last sample repeat it; their sums are not stored
                masks(n + u + 1 < n1 ? n + u + 1 : n1 - 1, nxt);
                pin_schedule();
#pragma unroll
                for (int j = 0; j < CC; ++j) p[u][j] = 0.0;
#pragma unroll
                for (int k = 0; k < KPT; ++k) {
                    const double sgn = lane_sign(cur[k]);
#pragma unroll
                    for (int j = 0; j < CC; ++j) p[u][j] = fma(v[j][k], sgn, p[u][j]);
                }
            }
            // all lanes -> lane (value, quarter): through the wave's LDS tile
#pragma unroll
            for (int u = 0; u < NS; ++u)
#pragma unroll
                for (int j = 0; j < CC; ++j) buf[(u * CC + j) * kFwdStride + lane] = p[u][j];
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
            const int val = lane & (kFwdVals - 1), quarter = lane >> 4;
            const double *src = buf + val * kFwdStride + quarter * 16;
            double t = 0.0;
#pragma unroll
            for (int i = 0; i < 16; ++i) t += src[i];
            t += __shfl_xor(t, 16, kWave);
            t += __shfl_xor(t, 32, kWave);
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();   // the tile is rewritten by the next trip
            const int u = val / CC, j = val % CC;
            if (lane < kFwdVals && n + u < n1 && c0 + j < C)
                part[((int64_t)slice * nb + n + u) * C + c0 + j] = t;
        }
    };
    if ((g_base + KPT) * 2 <= W)
        walk(std::integral_constant<int, 2>{});
    else if ((g_base + KPT) * 2 - 1 <= W)
        walk(std::integral_constant<int, 1>{});
    else
        walk(std::integral_constant<int, 0>{});
}

// ---- finishing the dot products: cosines and their argmax --------------------------------------
// Threads work in groups of `cp` lanes (a power of two <= 64, >= C when C <= 64) per sample;
// lane lc of a group takes classes lc, lc + cp, ...  For each it adds the slice partials in
// ascending slice order (independent loads), forms cos = dot / (|row| sqrt(D)) (0 for a zero
// row), optionally stores it, and keeps its best; a butterfly over the group then leaves in every
// lane the largest cosine and the lowest class that has it.  *cos_y receives cos of class y
// (summed over the group: exactly one lane holds it).
__device__ __forceinline__ void finish_cosines(const double *__restrict__ part, int slices, int64_t nb, int64_t n,
                                               bool live, int C, const double *nrm, double root_d, int cp, int lc,
                                               int y, float *cos_out, double *best_out, int *pred_out,
                                               double *cos_y) {
    double best = -2.0, cy = 0.0;   // cosines lie in [-1, 1]
    int pred = 0x7fffffff;
    if (live)
        for (int c = lc; c < C; c += cp) {
            double dot = 0.0;
            for (int s = 0; s < slices; ++s) dot += part[((int64_t)s * nb + n) * C + c];
            const double nn = nrm[c];
            const double cs = nn == 0.0 ? 0.0 : dot / (sqrt(nn) * root_d);
            if (cos_out) cos_out[n * C + c] = (float)cs;
            if (cs > best) {   // classes ascend within a lane: the first of equals stays
                best = cs;
                pred = c;
            }
            if (c == y) cy = cs;
        }
    for (int off = cp >> 1; off > 0; off >>= 1) {
        const double ob = __shfl_xor(best, off, kWave);
        const int op = __shfl_xor(pred, off, kWave);
        cy += __shfl_xor(cy, off, kWave);
        if (ob > best || (ob == best && op < pred)) {
            best = ob;
            pred = op;
        }
    }
    *best_out = best;
    *pred_out = pred;
    *cos_y = cy;
}

// lanes per sample for C classes
static int cosine_group(int C) {
    int cp = 1;
    while (cp < C && cp < kWave) cp <<= 1;
    return cp;
}

// ---- weights (and the transposed sample bits for the backward step) -----------------------------
// Blocks [0, wblocks): cp lanes per sample finish the dot products (finish_cosines), cosines
// against the frozen rows, prediction (lowest class among equals) and the two
// weights, as a record per sample and, for few classes, also as a dense row of signed fp64
// coefficients (+w_y at y, -w_p at a wrong prediction, 0 elsewhere).  Blocks from wblocks on do an unrelated job that needs no launch of its own: each
// turns a tile of 64 samples x 32 words of hv into colmask, the 64-bit lane mask of dimension
// group g of sample n stored group-major (or gw adjacent groups interleaved per sample), so
// that the backward step, which works on one or a few groups of all samples, reads its masks
// contiguously instead of 8 bytes out of every 4 W-byte row.
constexpr int kTileSamples = 64;
constexpr int kTileGroups = 16;

__global__ __launch_bounds__(256) void online_weights_kernel(
    const double *__restrict__ part, int slices, int64_t nb, const int32_t *__restrict__ labels,
    const double *__restrict__ normpart, int G, int C, double root_d, float lr,
    OnlineWeight *__restrict__ out, double *__restrict__ coef, int CB, int cp, int wblocks,
    const uint32_t *__restrict__ hv, int W, uint64_t *__restrict__ colmask, int64_t ld, int gw,
    uint32_t *reset) {
    extern __shared__ double nrm[];   // [C] squared norms of the frozen rows
    __shared__ uint32_t tile[kTileSamples][2 * kTileGroups + 1];
    const int t = threadIdx.x;
    if (reset && blockIdx.x == 0 && t == 0) *reset = 0;   // the row counter of online_lists_kernel, which runs next
    if ((int)blockIdx.x >= wblocks) {
        const int idx = blockIdx.x - wblocks;
        const int stiles = (int)(ld / kTileSamples);
        const int64_t ns = (int64_t)(idx % stiles) * kTileSamples;
        const int g0 = (idx / stiles) * kTileGroups;
#pragma unroll
        for (int r = 0; r < 8; ++r) {
            const int sm = r * 8 + (t >> 5), w = 2 * g0 + (t & 31);
            tile[sm][t & 31] = (ns + sm < nb && w < W) ? hv[(ns + sm) * W + w] : 0u;
        }
        __syncthreads();
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int gg = (t >> 6) + 4 * i, sm = t & 63;
            const int g = g0 + gg;
            if (g < G)   // layout [g / gw][n][g % gw]: gw = 1 is group-major, gw > 1 interleaves gw groups
                colmask[((int64_t)(g / gw) * ld + ns + sm) * gw + g % gw] =
                    (uint64_t)tile[sm][2 * gg] | ((uint64_t)tile[sm][2 * gg + 1] << 32);
        }
        return;
    }
    // squared norm of row c: a wave per class, lanes stride over the groups (fixed order)
    for (int c = t >> 6; c < C; c += 4) {
        double s = 0.0;
        for (int g = t & 63; g < G; g += kWave) s += normpart[(int64_t)c * G + g];
        s = wave_sum_f64(s);
        if ((t & 63) == 0) nrm[c] = s;
    }
    __syncthreads();
    const int spb = 256 / cp, lc = t % cp;
    const int64_t n = (int64_t)blockIdx.x * spb + t / cp;
    const bool inside = n < nb;
    const int y = inside ? labels[n] : -1;
    const bool live = inside && y >= 0 && y < C;
    double best, cos_y;
    int pred;
    finish_cosines(part, slices, nb, n, live, C, nrm, root_d, cp, lc, y, nullptr, &best, &pred, &cos_y);
    OnlineWeight r;
    r.y = live ? y : -1;
    r.pred = (live && pred != y) ? pred : -1;
    r.w_y = live ? (float)(1.0 - cos_y) : 0.0f;
    r.w_p = live ? (float)((double)lr * (1.0 - best)) : 0.0f;
    if (inside && lc == 0) out[n] = r;
    // the same two weights as a dense row of CB signed fp64 coefficients (small C only; CB <= cp
    // or the lanes loop); rows from nb up to the padded length are zero, so that they add nothing
    if (coef && n < ld)
        for (int j = lc; j < CB; j += cp)
            coef[n * CB + j] = j == r.y ? (double)r.w_y : j == r.pred ? -(double)r.w_p : 0.0;
}

// ---- backward: batch sum, update, new norms ----------------------------------------------------
// One block per group of 64 dimensions; its waves split the nb samples into contiguous runs.  A
// wave adds the weighted +-1 of each of its samples into its own LDS rows (one row of 64
// doubles per class of the window [c_lo, c_lo + c_n)), in sample order; after the barrier the
// rows of the waves are added in wave order.  A batch longer than one launch covers is summed
// over several launches through `carry` (fp64 [C][D]: read unless `first`, written unless
// `last`).  On the last one the accumulators take the sum in one rounding and the squared norm
// of this block's 64 elements of each row goes to normpart[c][g].
//
// Where the sum of a wave lives depends on C.  CB > 0 (C <= CB <= 16): in registers, one fp64
// per class; every sample is one FMA per class with the dense coefficient row from the weights
// step, which arrives by scalar loads (an FMA with a zero coefficient leaves the sum as it is).
// CB == 0: in the LDS rows themselves, one ds_add_f64 per weight of a sample - about 30
// cycles of the LDS pipe each, which the 16 waves of a block share, so it only wins when a
// dense row would be long.
typedef const uint64_t __attribute__((address_space(4))) *kptr_u64;
typedef const double __attribute__((address_space(4))) *kptr_f64;

template <int CB>
__global__ __launch_bounds__(kBwdMaxWaves *kWave) void online_bwd_kernel(
    const uint64_t *__restrict__ colmask, int64_t ld, const OnlineWeight *__restrict__ wts,
    const double *__restrict__ coef, int64_t nb, float *acc, int D, int c_lo, int c_n, int G,
    double *carry, int first, int last, double *__restrict__ normpart, int gpb, int64_t bs,
    double *__restrict__ partial, int c_all) {
    extern __shared__ double rows[];   // [waves][c_n][64]
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int nw = blockDim.x >> 6;
    // wave = (run, group): the block covers gpb adjacent groups and nw / gpb runs of samples.
    // Waves of one run read the same coefficient rows (one fetch into the CU's scalar cache).
    const int runs = nw / gpb;
    const int gi = wave % gpb, run = wave / gpb;
    const int g = blockIdx.x * gpb + gi;
    double *mine = rows + (int64_t)wave * c_n * kWave;

    // the block's samples [b_lo, b_hi), split into runs of whole trips, so that a trip's 8
    // masks are one aligned 64-byte load (bs is a multiple of 8)
    const int64_t b_lo = (int64_t)blockIdx.y * bs;
    const int64_t b_hi = b_lo + bs < nb ? b_lo + bs : nb;
    const int64_t span = b_hi > b_lo ? b_hi - b_lo : 0;
    const int64_t per = ((span + runs - 1) / runs + kBwdUnroll - 1) / kBwdUnroll * kBwdUnroll;
    const int64_t n0 = b_lo + run * per;
    const int64_t n1 = g >= G ? n0 : (n0 + per < b_hi ? n0 + per : b_hi);   // a group past the last: no samples
    kptr_u64 col = (kptr_u64)(colmask + (int64_t)(g < G ? g : G - 1) * ld);
    // All buffers are readable up to the next multiple of 64 samples; entries past nb are
    // ignored.
    if constexpr (CB > 0) {
        // samples per trip: two trips' operands (T masks + T * CB coefficients) fit the SGPRs
        constexpr int T = CB <= 4 ? 4 : 16 / CB;
        double delta[CB];
#pragma unroll
        for (int j = 0; j < CB; ++j) delta[j] = 0.0;
        kptr_f64 cf = (kptr_f64)coef;
        auto fetch = [&](int64_t n, uint64_t(&m)[T], double(&k)[T][CB]) {
#pragma unroll
            for (int u = 0; u < T; ++u) {
                m[u] = col[n + u];
#pragma unroll
                for (int j = 0; j < CB; ++j) k[u][j] = cf[(n + u) * CB + j];
            }
        };
        // no test for n + u < n1 inside a trip: coefficient rows from nb up to the next
        // multiple of 64 are zero, and a run ends at a multiple of 8 or at nb
        auto add = [&](const uint64_t(&m)[T], const double(&k)[T][CB]) {
#pragma unroll
            for (int u = 0; u < T; ++u) {
                const double sgn = lane_sign(m[u]);
#pragma unroll
                for (int j = 0; j < CB; ++j) delta[j] = fma(k[u][j], sgn, delta[j]);
            }
        };
        // A run is a whole number of kBwdUnroll-sample rounds and every trip of a round is
        // executed: samples from nb up to the end of the round have zero coefficients.  The
        // fetch after a run's last trip is redirected to the run's start (in bounds, unused).
        constexpr int U = kBwdUnroll / T;
        const int64_t n_end = (n1 + kBwdUnroll - 1) / kBwdUnroll * kBwdUnroll;   // end of the last round
        uint64_t mn[T];
        double kn[T][CB];
        if (n0 < n1) fetch(n0, mn, kn);
        for (int64_t n = n0; n < n1; n += kBwdUnroll) {
#pragma unroll
            for (int q = 0; q < U; ++q) {
                uint64_t mc[T];
                double kc[T][CB];
                wait_scalar_loads();
#pragma unroll
                for (int u = 0; u < T; ++u) {
                    mc[u] = mn[u];
#pragma unroll
                    for (int j = 0; j < CB; ++j) kc[u][j] = kn[u][j];
                }
                const int64_t nn = n + (q + 1) * T;
                fetch(nn < n_end ? nn : n0, mn, kn);
                pin_schedule();
                add(mc, kc);
            }
        }
#pragma unroll
        for (int j = 0; j < CB; ++j)
            if (j < c_n) mine[j * kWave + lane] = delta[j];
    } else {
        for (int c = 0; c < c_n; ++c) mine[c * kWave + lane] = 0.0;
        kptr_w rec = (kptr_w)wts;
        // kBwdUnroll samples per trip: their scalar loads are in flight together, and the LDS
        // adds return nothing, so a trip never waits on the LDS.  LDS operations of one wave
        // complete in issue order: two samples of the same class add in sample order.
        for (int64_t n = n0; n < n1; n += kBwdUnroll) {
            OnlineWeight r[kBwdUnroll];
            uint64_t m[kBwdUnroll];
#pragma unroll
            for (int u = 0; u < kBwdUnroll; ++u) {
                r[u].y = rec[n + u].y;
                r[u].pred = rec[n + u].pred;
                r[u].w_y = rec[n + u].w_y;
                r[u].w_p = rec[n + u].w_p;
                m[u] = col[n + u];
            }
#pragma unroll
            for (int u = 0; u < kBwdUnroll; ++u) {
                const bool live = n + u < n1 && r[u].y >= 0;
                const int yy = r[u].y - c_lo, pp = r[u].pred - c_lo;
                const bool hit_y = live && yy >= 0 && yy < c_n;
                const bool hit_p = live && r[u].pred >= 0 && pp >= 0 && pp < c_n;
                const double sgn = lane_sign(m[u]);
                if (hit_y) lds_add(&mine[yy * kWave + lane], (double)r[u].w_y * sgn);
                if (hit_p) lds_add(&mine[pp * kWave + lane], -((double)r[u].w_p * sgn));
            }
        }
    }
    __syncthreads();

    // (class, group) pairs of the block, dealt to the waves; runs are added in run order
    for (int idx = wave; idx < c_n * gpb; idx += nw) {
        const int c = idx / gpb, g2 = blockIdx.x * gpb + idx % gpb;
        if (g2 >= G) continue;
        const int d = g2 * kWave + lane;
        const int64_t at = (int64_t)(c_lo + c) * D + d;
        double s = (!partial && !first && d < D) ? carry[at] : 0.0;
        for (int r = 0; r < runs; ++r) s += rows[((int64_t)(r * gpb + idx % gpb) * c_n + c) * kWave + lane];
        if (partial) {   // this block's share of the batch sum; online_apply_kernel does the rest
            if (d < D) partial[((int64_t)blockIdx.y * c_all + c_lo + c) * D + d] = s;
            continue;
        }
        if (!last) {
            if (d < D) carry[at] = s;
            continue;
        }
        double q = 0.0;
        if (d < D) {
            const float nv = (float)((double)acc[at] + s);
            acc[at] = nv;
            q = (double)nv * (double)nv;
        }
        q = wave_sum_f64(q);
        if (lane == 0) normpart[(int64_t)(c_lo + c) * G + g2] = q;
    }
}

// Backward sums for many samples (the split path): a wave owns GW adjacent groups (64 GW
// dimensions) for its run of samples, so every coefficient that arrives through the scalar
// cache - which delivers only about a dword per clock to a CU - feeds GW FMAs per lane instead
// of one.  Block = 16 runs of one group column; grid (columns, shares).  Per sample: one scalar
// load of CB coefficients, one of GW masks (colmask interleaved by GW), GW v_cndmask + CB * GW
// FMAs; the next sample's operands are in flight meanwhile.  The 16 runs are then added in run
// order through LDS, class by class, into this block's share of the batch sum.
template <int CB, int GW>
__global__ __launch_bounds__(kBwdMaxWaves *kWave) void online_bwd_wide_kernel(
    const uint64_t *__restrict__ colmask, int64_t ld, const double *__restrict__ coef, int64_t nb, int D, int C,
    int64_t bs, double *__restrict__ partial) {
    __shared__ double buf[kBwdMaxWaves][GW * kWave];
    const int lane = threadIdx.x & (kWave - 1);
    const int run = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int colx = blockIdx.x;
    const int64_t b_lo = (int64_t)blockIdx.y * bs;
    const int64_t b_hi = b_lo + bs < nb ? b_lo + bs : nb;
    const int64_t span = b_hi > b_lo ? b_hi - b_lo : 0;
    const int64_t per = (span + kBwdMaxWaves - 1) / kBwdMaxWaves;
    const int64_t n0 = b_lo + run * per;
    const int64_t n1 = n0 + per < b_hi ? n0 + per : b_hi;
    kptr_u64 col = (kptr_u64)(colmask + (int64_t)colx * ld * GW);
    kptr_f64 cf = (kptr_f64)coef;

    double delta[CB][GW];
#pragma unroll
    for (int j = 0; j < CB; ++j)
#pragma unroll
        for (int i = 0; i < GW; ++i) delta[j][i] = 0.0;
    auto fetch = [&](int64_t n, uint64_t(&m)[GW], double(&k)[CB]) {
#pragma unroll
        for (int i = 0; i < GW; ++i) m[i] = col[n * GW + i];
#pragma unroll
        for (int j = 0; j < CB; ++j) k[j] = cf[n * CB + j];
    };
    uint64_t mn[GW];
    double kn[CB];
    if (n0 < n1) fetch(n0, mn, kn);
    for (int64_t n = n0; n < n1; ++n) {
        uint64_t mc[GW];
        double kc[CB];
        wait_scalar_loads();
#pragma unroll
        for (int i = 0; i < GW; ++i) mc[i] = mn[i];
#pragma unroll
        for (int j = 0; j < CB; ++j) kc[j] = kn[j];
        fetch(n + 1 < n1 ? n + 1 : n0, mn, kn);   // past the run: its start again (in bounds, unused)
        pin_schedule();
#pragma unroll
        for (int i = 0; i < GW; ++i) {
            const double sgn = lane_sign(mc[i]);
#pragma unroll
            for (int j = 0; j < CB; ++j) delta[j][i] = fma(kc[j], sgn, delta[j][i]);
        }
        pin_schedule();   // the register copies of the loop-carried operands stay below the arithmetic
    }
    // runs -> block sum, one class at a time through the LDS tile
    const int t = threadIdx.x;
#pragma unroll
    for (int j = 0; j < CB; ++j) {
        if (j < C) {   // uniform over the block
#pragma unroll
            for (int i = 0; i < GW; ++i) buf[run][i * kWave + lane] = delta[j][i];
            __syncthreads();
            if (t < GW * kWave) {
                double sum = 0.0;
#pragma unroll
                for (int r = 0; r < kBwdMaxWaves; ++r) sum += buf[r][t];
                const int d = colx * GW * kWave + t;
                if (d < D) partial[((int64_t)blockIdx.y * C + j) * D + d] = sum;
            }
            __syncthreads();
        }
    }
}

// Second half of a backward step whose samples were split over several blocks per group:
// delta = the blocks' shares in block order (plus the carry of earlier launches of the same
// batch), then the update and the norm partials exactly as in online_bwd_kernel.
// grid (G, ceil(C / 4)), one wave per (class, group).
__global__ __launch_bounds__(256) void online_apply_kernel(const double *__restrict__ partial, int shares,
                                                           float *acc, int D, int C, int G, double *carry,
                                                           int first, int last, double *__restrict__ normpart,
                                                           const uint32_t *__restrict__ slots) {
    const int lane = threadIdx.x & (kWave - 1);
    const int c = blockIdx.y * 4 + (threadIdx.x >> 6), g = blockIdx.x;
    if (c >= C) return;
    const int d = g * kWave + lane;
    const int64_t at = (int64_t)c * D + d;
    double s = 0.0;
    if (d < D) {
        if (!first) s = carry[at];
        if (slots) {   // the list path: class c owns rows slots[C + c] .. + slots[2 C + c] - 1 of `partial`
            const uint32_t r0 = slots[C + c], rn = slots[2 * C + c];
            uint32_t y = 0;
            for (; y + 4 <= rn; y += 4) {   // four rows in flight; added in row order
                const double *p = partial + (int64_t)(r0 + y) * D + d;
                const double a0 = p[0], a1 = p[D], a2 = p[2 * (int64_t)D], a3 = p[3 * (int64_t)D];
                s += a0;
                s += a1;
                s += a2;
                s += a3;
            }
            for (; y < rn; ++y) s += partial[(int64_t)(r0 + y) * D + d];
        } else {
            for (int y = 0; y < shares; ++y) s += partial[((int64_t)y * C + c) * D + d];
        }
    }
    if (!last) {
        if (d < D) carry[at] = s;
        return;
    }
    double q = 0.0;
    if (d < D) {
        const float nv = (float)((double)acc[at] + s);
        acc[at] = nv;
        q = (double)nv * (double)nv;
    }
    q = wave_sum_f64(q);
    if (lane == 0) normpart[(int64_t)c * G + g] = q;
}

// ---- backward by class lists ---------------------------------------------------------------------
// A sample changes at most two rows (its label's, always, and a wrong prediction's), so the batch
// sum of row c only needs the samples that name c: about (1 + error rate) N / C of them, whatever C
// is - where the dense forms above multiply every sample into every class.
//
// online_lists_kernel, a block per class: the samples whose record names the class, in sample
// order, as (sample index, signed weight) pairs; the 16 waves take contiguous runs of samples,
// count their hits, and after a prefix over the waves write them in place.  meta[c] = entries of
// class c; the class then takes ceil(entries / kListItem) consecutive rows of the share buffer
// (meta[C + c] = first row, meta[2 C + c] = rows) from a counter bumped by one atomic per class, and
// puts one (class, item) word per row into the work list behind it.  The order in which classes
// get their rows varies from run to run; the sums do not, each row is added up by one block in
// list order and a class's rows are added in row order.
constexpr int kListItem = 128;   // entries per work item (one wave's run)
__global__ __launch_bounds__(1024) void online_lists_kernel(const OnlineWeight *__restrict__ wts, int64_t nb, int C,
                                                            int64_t ld, uint32_t *__restrict__ list_n,
                                                            double *__restrict__ list_w, uint32_t *meta) {
    __shared__ uint32_t wave_hits[16];
    __shared__ uint32_t row0;
    const int c = blockIdx.x;
    const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x >> 6;
    const int64_t per = (nb + 15) / 16;
    const int64_t n0 = wave * per, n1 = n0 + per < nb ? n0 + per : nb;
    uint32_t hits = 0;
    for (int64_t n = n0 + lane; n < n1 + lane; n += kWave) {   // every lane makes the same trips
        const bool in = n < n1;
        const OnlineWeight r = in ? wts[n] : OnlineWeight{-1, -1, 0.f, 0.f};
        hits += (uint32_t)__popcll(__ballot(in && (r.y == c || r.pred == c)));
    }
    if (lane == 0) wave_hits[wave] = hits;
    __syncthreads();
    uint32_t before = 0, total = 0;
    for (int w = 0; w < 16; ++w) {
        if (w < wave) before += wave_hits[w];
        total += wave_hits[w];
    }
    uint32_t *ln = list_n + (int64_t)c * ld;
    double *lw = list_w + (int64_t)c * ld;
    uint32_t at = before;
    for (int64_t n = n0 + lane; n < n1 + lane; n += kWave) {
        const bool in = n < n1;
        const OnlineWeight r = in ? wts[n] : OnlineWeight{-1, -1, 0.f, 0.f};
        const bool hit = in && (r.y == c || r.pred == c);
        const uint64_t m = __ballot(hit);
        if (hit) {
            const uint32_t k = at + (uint32_t)__popcll(m & ((1ull << lane) - 1ull));
            ln[k] = (uint32_t)n;
            lw[k] = r.y == c ? (double)r.w_y : -(double)r.w_p;
        }
        at += (uint32_t)__popcll(m);
    }
    const uint32_t rows = (total + kListItem - 1) / kListItem;
    if (threadIdx.x == 0) {
        row0 = rows ? atomicAdd(meta + 3 * C, rows) : 0u;
        meta[c] = total;
        meta[C + c] = row0;
        meta[2 * C + c] = rows;
    }
    __syncthreads();
    for (uint32_t j = threadIdx.x; j < rows; j += 1024) meta[3 * C + 1 + row0 + j] = ((uint32_t)c << 16) | j;
}

// online_bwd_list_kernel, grid (columns of GW dimension groups, work items), kListWaves waves per
// block: work item (class c, run j) = entries [j * kListItem, ...) of class c's list, a quarter
// per wave (a wave's pace is set by the two scalar-load round trips per eight entries - sample
// index and weight, then that sample's lane masks from colmask - so the run is short and spread
// over waves rather than long).  A wave adds weight * (+-1) of each of its entries into GW * 64
// fp64 sums in registers; the waves' sums meet in LDS, are added in wave order and go to row
// meta[C + c] + j of the share buffer.
constexpr int kListWaves = 4;
template <int GW>
__global__ __launch_bounds__(kListWaves *kWave) void online_bwd_list_kernel(
    const uint64_t *__restrict__ colmask, int64_t ld, const uint32_t *__restrict__ list_n,
    const double *__restrict__ list_w, const uint32_t *__restrict__ meta, int C, int D,
    double *__restrict__ partial) {
    __shared__ double buf[kListWaves][GW * kWave];
    const uint32_t items = meta[3 * C];
    if (blockIdx.y >= items) return;   // block-uniform
    const uint32_t word = meta[3 * C + 1 + blockIdx.y];
    const int c = (int)(word >> 16);
    const uint32_t j = word & 0xffffu;
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    constexpr uint32_t kPerWave = kListItem / kListWaves;
    const uint32_t end = min((j + 1) * (uint32_t)kListItem, meta[c]);
    const uint32_t e0 = min(j * kListItem + wave * kPerWave, end), e1 = min(e0 + kPerWave, end);
    const int colx = blockIdx.x;
    kptr_u32 ln = (kptr_u32)(list_n + (int64_t)c * ld);
    kptr_f64 lw = (kptr_f64)(list_w + (int64_t)c * ld);
    kptr_u64 col = (kptr_u64)(colmask + (int64_t)colx * ld * GW);
    double sum[GW];
#pragma unroll
    for (int i = 0; i < GW; ++i) sum[i] = 0.0;
    for (uint32_t e = e0; e < e1; e += 8) {
        // eight entries at a time; past the run's end the last entry repeats with weight zero
        uint32_t n[8];
        double w[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            const uint32_t at = min(e + u, e1 - 1);
            n[u] = ln[at];
            w[u] = e + u < e1 ? lw[at] : 0.0;
        }
        uint64_t m[8][GW];
#pragma unroll
        for (int u = 0; u < 8; ++u)
#pragma unroll
            for (int i = 0; i < GW; ++i) m[u][i] = col[(int64_t)n[u] * GW + i];
#pragma unroll
        for (int u = 0; u < 8; ++u)
#pragma unroll
            for (int i = 0; i < GW; ++i) sum[i] = fma(w[u], lane_sign(m[u][i]), sum[i]);
    }
#pragma unroll
    for (int i = 0; i < GW; ++i) buf[wave][i * kWave + lane] = sum[i];
    __syncthreads();
    double *dst = partial + (int64_t)(meta[C + c] + j) * D;
    for (int t = threadIdx.x; t < GW * kWave; t += kListWaves * kWave) {
        double total = 0.0;
#pragma unroll
        for (int w = 0; w < kListWaves; ++w) total += buf[w][t];
        const int d = colx * GW * kWave + t;
        if (d < D) dst[d] = total;
    }
}

// ---- squared norms of given rows, and cosine inference ---------------------------------------
// normpart[c][g] = sum of acc[c][d]^2 over the 64 dimensions of group g, with the arithmetic of
// the backward step's epilogue.  grid (G, ceil(C / 4)), one wave per (class, group).
__global__ __launch_bounds__(256) void online_norm_kernel(const float *__restrict__ acc, int D, int C, int G,
                                                          double *__restrict__ normpart) {
    const int lane = threadIdx.x & (kWave - 1);
    const int c = blockIdx.y * 4 + (threadIdx.x >> 6), g = blockIdx.x;
    if (c >= C) return;
    const int d = g * kWave + lane;
    double q = 0.0;
    if (d < D) {
        const double v = (double)acc[(int64_t)c * D + d];
        q = v * v;
    }
    q = wave_sum_f64(q);
    if (lane == 0) normpart[(int64_t)c * G + g] = q;
}

// Cosine-similarity inference (Sec. III): cp lanes per sample finish the dot products of
// the forward step into cosines (finish_cosines); cos_out [nb][C] fp32 (optional), pred = lowest class with the
// largest cosine (compared in fp64).
__global__ __launch_bounds__(256) void cosine_finish_kernel(
    const double *__restrict__ part, int slices, int64_t nb, const double *__restrict__ normpart, int G, int C,
    double root_d, int cp, float *__restrict__ cos_out, int32_t *__restrict__ pred_out) {
    extern __shared__ double nrm[];   // [C]
    const int t = threadIdx.x;
    for (int c = t >> 6; c < C; c += 4) {
        double s = 0.0;
        for (int g = t & 63; g < G; g += kWave) s += normpart[(int64_t)c * G + g];
        s = wave_sum_f64(s);
        if ((t & 63) == 0) nrm[c] = s;
    }
    __syncthreads();
    const int spb = 256 / cp, lc = t % cp;
    const int64_t n = (int64_t)blockIdx.x * spb + t / cp;
    double best, cos_y;
    int pred;
    finish_cosines(part, slices, nb, n, n < nb, C, nrm, root_d, cp, lc, -1, cos_out, &best, &pred, &cos_y);
    if (n < nb && lc == 0) pred_out[n] = pred;
}

// ---- host side ---------------------------------------------------------------------------------
template <typename T>
static int grow(T **p, size_t *have, size_t want) {
    if (*have >= want) return HDC_OK;
    if (*p) HDC_HIP(hipFree(*p));   // waits for the device: nothing still reads the old buffer
    *p = nullptr;
    *have = 0;
    const hipError_t e = hipMalloc(reinterpret_cast<void **>(p), want + 256);
    if (e == hipErrorOutOfMemory) {
        (void)hipGetLastError();
        return HDC_ENOMEM;
    }
    HDC_HIP(e);
    *have = want;
    return HDC_OK;
}

// Width of the dense coefficient rows of the backward step, 0 = none (LDS sums).
static int bwd_dense_width(int C) { return C <= 2 ? 2 : C <= 4 ? 4 : C <= 8 ? 8 : C <= 16 ? 16 : 0; }

constexpr int kBwdSplitMin = 2048;   // from this many samples on, the samples of a group are split over blocks

// Groups per wave of the split path: 64 registers of sums (CB classes x GW groups x fp64).
static int bwd_group_width(int C) { return bwd_dense_width(C) == 16 ? 2 : 4; }

// How many blocks share the samples of one group column: one round of blocks, one per CU.
static int bwd_shares(const hdc_ctx_impl *c, int G, int64_t nb) {
    if (bwd_dense_width(c->p.C) == 0 || nb < kBwdSplitMin) return 1;
    const int gw = bwd_group_width(c->p.C);
    const int cols = (G + gw - 1) / gw;
    int64_t shares = c->num_cus / cols;
    const int64_t most = nb / 256;                                   // at least 256 samples per block
    const int64_t fit = (int64_t)(64u << 20) / ((int64_t)c->p.C * c->p.D * (int64_t)sizeof(double));
    if (shares > most) shares = most;
    if (shares > fit) shares = fit;
    if (shares > 64) shares = 64;
    return shares < 1 ? 1 : (int)shares;
}

// More than 16 classes (no dense coefficient rows) and at least 1024 samples in the piece: the
// backward step goes by class lists (measured at 26 classes: equal at 512 samples, 1.07x faster at
// 1024, 1.45x at 8192; for up to 16 classes the dense forms are as fast or faster).
static bool bwd_by_lists(int C, int64_t nb) { return C > 16 && nb >= 1024; }
constexpr int kListGroups = 4;   // dimension groups per wave of online_bwd_list_kernel
static int64_t list_rows(int64_t nb, int C) { return 2 * nb / kListItem + C + 1; }   // most share rows

static int launch_bwd(hdc_ctx_impl *c, int64_t ld, int64_t nb, float *acc, int G, bool first, bool last,
                      hipStream_t s) {
    const int C = c->p.C;
    const OnlineWeight *wts = static_cast<const OnlineWeight *>(c->ob_wts_d);
    if (bwd_by_lists(C, nb)) {
        ProfScope prof(c, HDC_K_ONLINE_BWD, s);
        hipLaunchKernelGGL(online_lists_kernel, dim3((unsigned)C), dim3(1024), 0, s, wts, nb, C, ld, c->ob_ln_d,
                           c->ob_lw_d, c->ob_meta_d);
        hipLaunchKernelGGL(online_bwd_list_kernel<kListGroups>,
                           dim3((unsigned)((G + kListGroups - 1) / kListGroups), (unsigned)list_rows(nb, C)),
                           dim3(kListWaves * kWave),
                           0, s, c->ob_col_d, ld, c->ob_ln_d, c->ob_lw_d, c->ob_meta_d, C, c->p.D, c->ob_share_d);
        hipLaunchKernelGGL(online_apply_kernel, dim3((unsigned)G, (unsigned)((C + 3) / 4)), dim3(256), 0, s,
                           c->ob_share_d, 0, acc, c->p.D, C, G, c->ob_carry_d, first ? 1 : 0, last ? 1 : 0,
                           c->ob_norm_d, c->ob_meta_d);
        HDC_HIP(hipGetLastError());
        return HDC_OK;
    }
    const int shares = bwd_shares(c, G, nb);
    if (shares > 1) {
        // dense sums, a column of bwd_group_width() groups per block, `shares` blocks per column; the
        // blocks' sums meet in online_apply_kernel
        const int gw = bwd_group_width(C);
        const int64_t bs = (nb + shares - 1) / shares;
        const int used = (int)((nb + bs - 1) / bs);
        const dim3 grid((unsigned)((G + gw - 1) / gw), (unsigned)used), block(kBwdMaxWaves * kWave);
        {
            ProfScope prof(c, HDC_K_ONLINE_BWD, s);
#define HDC_BWD(CB, GW)                                                                                     \
    hipLaunchKernelGGL((online_bwd_wide_kernel<CB, GW>), grid, block, 0, s, c->ob_col_d, ld, c->ob_coef_d, nb, \
                       c->p.D, C, bs, c->ob_share_d)
            switch (bwd_dense_width(C)) {
                case 2: HDC_BWD(2, 4); break;
                case 4: HDC_BWD(4, 4); break;
                case 8: HDC_BWD(8, 4); break;
                default: HDC_BWD(16, 2); break;
            }
#undef HDC_BWD
            HDC_HIP(hipGetLastError());
            hipLaunchKernelGGL(online_apply_kernel, dim3((unsigned)G, (unsigned)((C + 3) / 4)), dim3(256), 0, s,
                               c->ob_share_d, used, acc, c->p.D, C, G, c->ob_carry_d, first ? 1 : 0, last ? 1 : 0,
                               c->ob_norm_d, static_cast<const uint32_t *>(nullptr));
        }
        HDC_HIP(hipGetLastError());
        return HDC_OK;
    }
    for (int c_lo = 0; c_lo < C; c_lo += kBwdSlots) {
        const int c_n = C - c_lo < kBwdSlots ? C - c_lo : kBwdSlots;
        int nw = kBwdSlots / c_n;
        if (nw > kBwdMaxWaves) nw = kBwdMaxWaves;
        while (nw > 1 && (int64_t)(nw / 2) * kBwdUnroll >= nb) nw /= 2;   // no wave without a trip
        const size_t lds = (size_t)nw * c_n * kWave * sizeof(double);
        const dim3 grid((unsigned)G), block((unsigned)nw * kWave);
        const int64_t bs = (nb + kBwdUnroll - 1) / kBwdUnroll * kBwdUnroll;   // one block takes all samples
        ProfScope prof(c, HDC_K_ONLINE_BWD, s);
#define HDC_BWD(CB)                                                                                          \
    hipLaunchKernelGGL(online_bwd_kernel<CB>, grid, block, lds, s, c->ob_col_d, ld, wts, c->ob_coef_d, nb, acc, \
                       c->p.D, c_lo, c_n, G, c->ob_carry_d, first ? 1 : 0, last ? 1 : 0, c->ob_norm_d, 1, bs,  \
                       static_cast<double *>(nullptr), C)
        switch (bwd_dense_width(C)) {
            case 2: HDC_BWD(2); break;
            case 4: HDC_BWD(4); break;
            case 8: HDC_BWD(8); break;
            case 16: HDC_BWD(16); break;
            default: HDC_BWD(0); break;
        }
#undef HDC_BWD
        HDC_HIP(hipGetLastError());
    }
    return HDC_OK;
}

// Shape of the forward launch for C classes and D dimensions.
struct FwdShape {
    bool wide;     // 4 classes x 8 groups per wave instead of 2 x 16
    int slices, chunks, ns;
};
static FwdShape fwd_shape(int C, int G) {
    FwdShape f;
    // whichever wastes fewer class slots (relative cost per class slot and 16 groups: 71 : 62
    // issue slots at 2 : 4 classes)
    f.wide = ((C + 3) / 4) * 125 < ((C + 1) / 2) * 71;
    const int cc = f.wide ? 4 : 2, groups = f.wide ? 8 : 16;
    f.slices = (G + groups - 1) / groups;
    f.chunks = (C + cc - 1) / cc;
    f.ns = kFwdVals / cc;
    return f;
}

// Most samples one forward launch takes: bounds the partial-dot-product scratch to 256 MB.
static int64_t fwd_sub_batch(const FwdShape &f, int C, int64_t limit) {
    int64_t sb = (int64_t)(256u << 20) / ((int64_t)f.slices * C * (int64_t)sizeof(double));
    if (sb > 8192) sb = 8192;
    if (sb < 64) sb = 64;
    return sb > limit ? limit : sb;
}

static int launch_fwd(hdc_ctx_impl *c, const FwdShape &f, const uint32_t *rows, int64_t nb, const float *acc,
                      hipStream_t s) {
    // about four waves per SIMD when there is that much work; whole trips per wave
    int64_t spw = (nb * f.slices * f.chunks + 4095) / 4096;
    spw = (spw + f.ns - 1) / f.ns * f.ns;
    if (spw > 64) spw = 64;
    const int64_t tiles = (nb + kFwdWaves * spw - 1) / (kFwdWaves * spw);
    const dim3 grid((unsigned)f.slices, (unsigned)f.chunks, (unsigned)tiles);
    ProfScope prof(c, HDC_K_ONLINE_FWD, s);
    if (f.wide)
        hipLaunchKernelGGL((online_fwd_kernel<4, 8>), grid, dim3(kFwdWaves * kWave), 0, s, rows, nb, acc, c->p.D,
                           c->W, c->p.C, (int)spw, c->ob_part_d);
    else
        hipLaunchKernelGGL((online_fwd_kernel<2, 16>), grid, dim3(kFwdWaves * kWave), 0, s, rows, nb, acc, c->p.D,
                           c->W, c->p.C, (int)spw, c->ob_part_d);
    HDC_HIP(hipGetLastError());
    return HDC_OK;
}

static int launch_norm(hdc_ctx_impl *c, const float *acc, int G, hipStream_t s) {
    hipLaunchKernelGGL(online_norm_kernel, dim3((unsigned)G, (unsigned)((c->p.C + 3) / 4)), dim3(256), 0, s, acc,
                       c->p.D, c->p.C, G, c->ob_norm_d);
    HDC_HIP(hipGetLastError());
    return HDC_OK;
}

// Scratch of hdc_train_online_batched for batches of up to `batch` samples (grown if smaller; a
// no-op, without any synchronisation, when it is there already).
int reserve_online_batched(hdc_ctx_impl *c, int64_t batch) {
    const int C = c->p.C, D = c->p.D;
    const int G = (D + kWave - 1) / kWave;
    const FwdShape f = fwd_shape(C, G);
    const int64_t sb = fwd_sub_batch(f, C, batch);
    const int64_t ld = (sb + kTileSamples - 1) / kTileSamples * kTileSamples;
    HDC_HIP(hipSetDevice(c->device));
    int rc = grow(&c->ob_part_d, &c->ob_part_bytes, (size_t)f.slices * sb * C * sizeof(double));
    if (rc == HDC_OK) rc = grow(&c->ob_wts_d, &c->ob_wts_bytes, (size_t)ld * sizeof(OnlineWeight));
    if (rc == HDC_OK) rc = grow(&c->ob_col_d, &c->ob_col_bytes, (size_t)(G + 3) * ld * sizeof(uint64_t));
    const int cb = bwd_dense_width(C);
    if (rc == HDC_OK && cb) rc = grow(&c->ob_coef_d, &c->ob_coef_bytes, (size_t)ld * cb * sizeof(double));
    if (rc == HDC_OK) rc = grow(&c->ob_norm_d, &c->ob_norm_bytes, (size_t)C * G * sizeof(double));
    if (rc == HDC_OK && batch > sb)
        rc = grow(&c->ob_carry_d, &c->ob_carry_bytes, (size_t)C * D * sizeof(double));
    const int shares = bwd_shares(c, G, sb);
    size_t share_bytes = shares > 1 ? (size_t)shares * C * D * sizeof(double) : 0;
    if (bwd_by_lists(C, sb)) {
        const size_t rows = (size_t)list_rows(sb, C);
        if (rows * D * sizeof(double) > share_bytes) share_bytes = rows * D * sizeof(double);
        if (rc == HDC_OK) rc = grow(&c->ob_ln_d, &c->ob_ln_bytes, (size_t)C * ld * sizeof(uint32_t));
        if (rc == HDC_OK) rc = grow(&c->ob_lw_d, &c->ob_lw_bytes, (size_t)C * ld * sizeof(double));
        if (rc == HDC_OK) rc = grow(&c->ob_meta_d, &c->ob_meta_bytes, (3 * (size_t)C + 1 + rows) * sizeof(uint32_t));
    }
    if (rc == HDC_OK && share_bytes) rc = grow(&c->ob_share_d, &c->ob_share_bytes, share_bytes);
    return rc;
}

// Scratch of hdc_search_cosine for calls of up to `queries` queries.
int reserve_search_cosine(hdc_ctx_impl *c, int64_t queries) {
    const int C = c->p.C, G = (c->p.D + kWave - 1) / kWave;
    const FwdShape f = fwd_shape(C, G);
    const int64_t sb = fwd_sub_batch(f, C, queries);
    HDC_HIP(hipSetDevice(c->device));
    int rc = grow(&c->ob_part_d, &c->ob_part_bytes, (size_t)f.slices * sb * C * sizeof(double));
    if (rc == HDC_OK) rc = grow(&c->ob_norm_d, &c->ob_norm_bytes, (size_t)C * G * sizeof(double));
    return rc;
}

int launch_train_online_batched(hdc_ctx_impl *c, const uint32_t *hv, const int32_t *labels, int64_t N,
                                int32_t epochs, float lr, int64_t batch, float *acc, hipStream_t s) {
    const int C = c->p.C, D = c->p.D, W = c->W;
    const int G = (D + kWave - 1) / kWave;
    const FwdShape f = fwd_shape(C, G);
    if (batch > N) batch = N;

    // A batch is worked off in pieces of at most `sb` samples (forward, weights, backward each);
    // sb bounds the scratch: partial dot products and transposed masks.
    const int64_t sb = fwd_sub_batch(f, C, batch);
    const int cb = bwd_dense_width(C);
    int rc = reserve_online_batched(c, batch);
    if (rc != HDC_OK) return rc;
    if (!c->ob_attr_set) {
        const void *kernels[] = {reinterpret_cast<const void *>(online_bwd_kernel<0>),
                                 reinterpret_cast<const void *>(online_bwd_kernel<2>),
                                 reinterpret_cast<const void *>(online_bwd_kernel<4>),
                                 reinterpret_cast<const void *>(online_bwd_kernel<8>),
                                 reinterpret_cast<const void *>(online_bwd_kernel<16>)};
        for (const void *k : kernels)
            HDC_HIP(hipFuncSetAttribute(k, hipFuncAttributeMaxDynamicSharedMemorySize,
                                        (int)(kBwdSlots * kWave * sizeof(double))));
        c->ob_attr_set = true;
    }

    rc = launch_norm(c, acc, G, s);   // squared norms of the rows as handed in
    if (rc != HDC_OK) return rc;
    const double root_d = sqrt((double)D);
    const int ttiles = (G + kTileGroups - 1) / kTileGroups;
    for (int32_t e = 0; e < epochs; ++e)
        for (int64_t b0 = 0; b0 < N; b0 += batch) {
            const int64_t B = b0 + batch < N ? batch : N - b0;
            for (int64_t s0 = 0; s0 < B; s0 += sb) {
                const int64_t nb = s0 + sb < B ? sb : B - s0;
                const uint32_t *rows = hv + (b0 + s0) * W;
                rc = launch_fwd(c, f, rows, nb, acc, s);
                if (rc != HDC_OK) return rc;
                const int64_t ld_used = (nb + kTileSamples - 1) / kTileSamples * kTileSamples;
                const int cp = cosine_group(C);
                const int wblocks = (int)((ld_used + 256 / cp - 1) / (256 / cp));
                const int tblocks = (int)(ld_used / kTileSamples) * ttiles;
                hipLaunchKernelGGL(online_weights_kernel, dim3((unsigned)(wblocks + tblocks)), dim3(256),
                                   (size_t)C * sizeof(double), s, c->ob_part_d, f.slices, nb, labels + b0 + s0,
                                   c->ob_norm_d, G, C, root_d, lr, static_cast<OnlineWeight *>(c->ob_wts_d),
                                   cb && !bwd_by_lists(C, nb) ? c->ob_coef_d : nullptr, cb, cp, wblocks, rows, W,
                                   c->ob_col_d, ld_used,
                                   bwd_by_lists(C, nb) ? kListGroups : bwd_shares(c, G, nb) > 1 ? bwd_group_width(C) : 1,
                                   bwd_by_lists(C, nb) ? c->ob_meta_d + 3 * C : nullptr);
                HDC_HIP(hipGetLastError());
                rc = launch_bwd(c, ld_used, nb, acc, G, s0 == 0, s0 + nb == B, s);
                if (rc != HDC_OK) return rc;
            }
        }
    return HDC_OK;
}

int launch_search_cosine(hdc_ctx_impl *c, const uint32_t *hv, int64_t N, const float *acc, float *cos_out,
                         int32_t *pred, hipStream_t s) {
    const int C = c->p.C, D = c->p.D, W = c->W;
    const int G = (D + kWave - 1) / kWave;
    const FwdShape f = fwd_shape(C, G);
    const int64_t sb = fwd_sub_batch(f, C, N);
    int rc = reserve_search_cosine(c, N);
    if (rc != HDC_OK) return rc;
    rc = launch_norm(c, acc, G, s);
    if (rc != HDC_OK) return rc;
    const double root_d = sqrt((double)D);
    for (int64_t n0 = 0; n0 < N; n0 += sb) {
        const int64_t nb = n0 + sb < N ? sb : N - n0;
        rc = launch_fwd(c, f, hv + n0 * W, nb, acc, s);
        if (rc != HDC_OK) return rc;
        const int cp = cosine_group(C);
        hipLaunchKernelGGL(cosine_finish_kernel, dim3((unsigned)((nb + 256 / cp - 1) / (256 / cp))), dim3(256),
                           (size_t)C * sizeof(double), s, c->ob_part_d, f.slices, nb, c->ob_norm_d, G, C, root_d, cp,
                           cos_out ? cos_out + n0 * C : nullptr, pred + n0);
        HDC_HIP(hipGetLastError());
    }
    return HDC_OK;
}

}  // namespace hdc
