// The paper's stand-alone hypervector primitives (arXiv 2206.04746, Sec. IV-B1 and IV-B2): bit
// packing and unpacking, and the horizontal sum.  (The vertical sum lives with classical
// training, whose counting kernel it is.)  All three stream their input once: HBM-bound.
#include "hdc_internal.h"

namespace hdc {

// Streams that are read or written once go past the caches ("nt": measured, unpack writes at 7.4
// instead of 4.9 TB/s with it).
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
__device__ __forceinline__ uint4 nt_load16(const uint8_t *p) {
    const u32x4 v = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(p));
    return make_uint4(v.x, v.y, v.z, v.w);
}

// 4 bytes -> 4 bits: bit i of the result = (byte i of x != 0).
__device__ __forceinline__ uint32_t nibble_of_bytes(uint32_t x) {
    const uint32_t nz = (((x & 0x7f7f7f7fu) + 0x7f7f7f7fu) | x) & 0x80808080u;   // bit 7 of every non-zero byte
    // bits 0, 8, 16, 24 of (nz >> 7) land on bits 28..31 of the product, one term each
    return ((nz >> 7) * 0x10204080u) >> 28;
}

// 4 bits -> 4 bytes of 0 / 1: byte i of the result = bit i of nib.
__device__ __forceinline__ uint32_t bytes_of_nibble(uint32_t nib) {
    return (nib * 0x00204081u) & 0x01010101u;
}

// Aligned matrices whose D is a multiple of 16: one thread per 16 input bytes, consecutive threads
// on consecutive chunks (a row's chunks padded to an even count so that the two halves of a word
// sit in neighbouring lanes); the odd lane hands its 16 bits to the even one, which stores the
// word.  Every cache line is read by one load instruction, so the loads can go past the caches.
constexpr int kPackAhead = 4;   // chunks per thread, all requested before the first is used
__global__ __launch_bounds__(256) void pack16_kernel(const uint8_t *__restrict__ bits, int64_t N, int D, int W,
                                                     uint32_t *__restrict__ hv) {
    const int cpr = D >> 4, pitch = (cpr + 1) & ~1;
    const int64_t t0 = (int64_t)blockIdx.x * (256 * kPackAhead) + threadIdx.x;
    int64_t n[kPackAhead];
    int c[kPackAhead];
    uint4 a[kPackAhead];
#pragma unroll
    for (int k = 0; k < kPackAhead; ++k) {
        const int64_t t = t0 + k * 256;
        n[k] = t / pitch;
        c[k] = (int)(t - n[k] * pitch);
        // a slot that is padding or past the matrix re-reads chunk 0 of the last row (in bounds, unused)
        const bool real = n[k] < N && c[k] < cpr;
        a[k] = nt_load16(bits + (real ? n[k] : N - 1) * D + 16 * (real ? c[k] : 0));
    }
#pragma unroll
    for (int k = 0; k < kPackAhead; ++k) {
        const bool real = n[k] < N && c[k] < cpr;
        uint32_t half = nibble_of_bytes(a[k].x) | nibble_of_bytes(a[k].y) << 4 | nibble_of_bytes(a[k].z) << 8 |
                        nibble_of_bytes(a[k].w) << 12;
        if (!real) half = 0;
        const uint32_t other = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)half, 0xB1, 0xF, 0xF, true);   // lane ^ 1
        if (real && (c[k] & 1) == 0) hv[n[k] * W + (c[k] >> 1)] = half | other << 16;
    }
}

// Any D and alignment: one thread per output word, byte loads.
__global__ __launch_bounds__(256) void pack_kernel(const uint8_t *__restrict__ bits, int64_t N, int D, int W,
                                                   uint32_t *__restrict__ hv) {
    const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (idx >= N * W) return;
    const int64_t n = idx / W;
    const int w = (int)(idx - n * W);
    const uint8_t *src = bits + n * D + 32 * w;
    const int left = D - 32 * w;   // > 0
    const int m = left < 32 ? left : 32;
    uint32_t word = 0;
    for (int i = 0; i < m; ++i) word |= (uint32_t)(src[i] != 0) << i;
    hv[idx] = word;
}

// Aligned matrices whose D is a multiple of 16: one thread per 16 output bytes.  Chunk g of the
// byte matrix (bytes 16 g .. 16 g + 15) is half a word of row g / (D / 16), and consecutive
// threads write consecutive chunks, so a store instruction covers one contiguous kilobyte (a
// thread per word, two stores 32 bytes apart, fills every cache line in two halves and ran at
// three quarters of this rate).
__global__ __launch_bounds__(256) void unpack16_kernel(const uint32_t *__restrict__ hv, int64_t N, int D, int W,
                                                       uint4 *__restrict__ bits16) {
    const int cpr = D >> 4;   // chunks per row
    const int64_t g = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (g >= N * cpr) return;
    const int64_t n = g / cpr;
    const int c = (int)(g - n * cpr);
    const uint32_t half = (hv[n * W + (c >> 1)] >> (16 * (c & 1))) & 0xffffu;
    uint4 o;
    o.x = bytes_of_nibble(half & 15u);
    o.y = bytes_of_nibble((half >> 4) & 15u);
    o.z = bytes_of_nibble((half >> 8) & 15u);
    o.w = bytes_of_nibble(half >> 12);
    u32x4 v;
    v.x = o.x; v.y = o.y; v.z = o.z; v.w = o.w;
    __builtin_nontemporal_store(v, reinterpret_cast<u32x4 *>(bits16 + g));
}

// Any D and alignment: one thread per word, byte stores.
__global__ __launch_bounds__(256) void unpack_kernel(const uint32_t *__restrict__ hv, int64_t N, int D, int W,
                                                     uint8_t *__restrict__ bits) {
    const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (idx >= N * W) return;
    const int64_t n = idx / W;
    const int w = (int)(idx - n * W);
    const uint32_t word = hv[idx];
    uint8_t *dst = bits + n * D + 32 * w;
    const int left = D - 32 * w;
    const int m = left < 32 ? left : 32;
    for (int i = 0; i < m; ++i) dst[i] = (uint8_t)((word >> i) & 1u);
}

// Horizontal sum: a wave takes kHsumRows consecutive rows at a time, lanes stride over the words
// of all of them together (kHsumRows independent loads per step, several steps unrolled, so a
// lane has a dozen loads in flight), v_bcnt accumulates per row, one butterfly per row at the end.
constexpr int kHsumWaves = 4;
constexpr int kHsumRows = 4;
__global__ __launch_bounds__(kHsumWaves *kWave) void hsum_kernel(const uint32_t *__restrict__ hv, int64_t N,
                                                                  int W, int32_t *__restrict__ out) {
    const int lane = threadIdx.x & (kWave - 1);
    const int64_t n0 = ((int64_t)blockIdx.x * kHsumWaves + (threadIdx.x >> 6)) * kHsumRows;
    if (n0 >= N) return;
    const uint32_t *row[kHsumRows];
    uint32_t s[kHsumRows];
#pragma unroll
    for (int r = 0; r < kHsumRows; ++r) {
        row[r] = hv + (n0 + r < N ? n0 + r : N - 1) * W;   // surplus rows repeat the last one, unused
        s[r] = 0;
    }
#pragma unroll 4
    for (int w = lane; w < W; w += kWave)
#pragma unroll
        for (int r = 0; r < kHsumRows; ++r) s[r] += __popc(row[r][w]);
#pragma unroll
    for (int r = 0; r < kHsumRows; ++r) {
#pragma unroll
        for (int off = 32; off > 0; off >>= 1) s[r] += __shfl_xor(s[r], off, kWave);
        if (lane == 0 && n0 + r < N) out[n0 + r] = (int32_t)s[r];
    }
}

static inline bool vec_ok(const void *p, int D) {
    return (D & 15) == 0 && (reinterpret_cast<uintptr_t>(p) & 15u) == 0;
}

int launch_pack(hdc_ctx_impl *c, const uint8_t *bits, int64_t N, uint32_t *hv, hipStream_t s) {
    if (vec_ok(bits, c->p.D)) {
        const int64_t slots = N * (((c->p.D >> 4) + 1) & ~1);
        hipLaunchKernelGGL(pack16_kernel, dim3((unsigned)((slots + 256 * kPackAhead - 1) / (256 * kPackAhead))), dim3(256), 0, s, bits, N, c->p.D,
                           c->W, hv);
    } else {
        const int64_t words = N * c->W;
        hipLaunchKernelGGL(pack_kernel, dim3((unsigned)((words + 255) / 256)), dim3(256), 0, s, bits, N, c->p.D,
                           c->W, hv);
    }
    HDC_HIP(hipGetLastError());
    return HDC_OK;
}

int launch_unpack(hdc_ctx_impl *c, const uint32_t *hv, int64_t N, uint8_t *bits, hipStream_t s) {
    if (vec_ok(bits, c->p.D)) {
        const int64_t chunks = N * (c->p.D >> 4);
        hipLaunchKernelGGL(unpack16_kernel, dim3((unsigned)((chunks + 255) / 256)), dim3(256), 0, s, hv, N, c->p.D,
                           c->W, reinterpret_cast<uint4 *>(bits));
    } else {
        const int64_t words = N * c->W;
        hipLaunchKernelGGL(unpack_kernel, dim3((unsigned)((words + 255) / 256)), dim3(256), 0, s, hv, N, c->p.D,
                           c->W, bits);
    }
    HDC_HIP(hipGetLastError());
    return HDC_OK;
}

int launch_hsum(hdc_ctx_impl *c, const uint32_t *hv, int64_t N, int32_t *out, hipStream_t s) {
    hipLaunchKernelGGL(hsum_kernel, dim3((unsigned)((N + kHsumWaves * kHsumRows - 1) / (kHsumWaves * kHsumRows))),
                       dim3(kHsumWaves * kWave), 0,
                       s, hv, N, c->W, out);
    HDC_HIP(hipGetLastError());
    return HDC_OK;
}

}  // namespace hdc
