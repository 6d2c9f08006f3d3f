// The paper's stand-alone hypervector primitives (arXiv 2206.04746, Sec. IV-B1 and IV-B2): bit
// packing and unpacking, and the horizontal sum.  (The vertical sum lives with classical
// training, whose counting kernel it is.)  All three stream their input once: HBM-bound.
#include "hdc_internal.h"

namespace hdc {

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

// One thread per output word.  VEC: D is a multiple of 16 and the byte matrix is 16-byte
// aligned, so a word's 32 (or, for the last word of a row, 16) bytes are one or two uint4.
template <bool VEC>
__global__ __launch_bounds__(256) void pack_kernel(const uint8_t *__restrict__ bits, int64_t N, int D, int W,
                                                   uint32_t *__restrict__ hv) {
    const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (idx >= N * W) return;
    const int64_t n = idx / W;
    const int w = (int)(idx - n * W);
    const uint8_t *src = bits + n * D + 32 * w;
    const int left = D - 32 * w;   // > 0
    uint32_t word = 0;
    if (VEC) {
        const uint4 a = *reinterpret_cast<const uint4 *>(src);
        word = nibble_of_bytes(a.x) | nibble_of_bytes(a.y) << 4 | nibble_of_bytes(a.z) << 8 |
               nibble_of_bytes(a.w) << 12;
        if (left >= 32) {
            const uint4 b = *reinterpret_cast<const uint4 *>(src + 16);
            word |= nibble_of_bytes(b.x) << 16 | nibble_of_bytes(b.y) << 20 | nibble_of_bytes(b.z) << 24 |
                    nibble_of_bytes(b.w) << 28;
        }
    } else {
        const int m = left < 32 ? left : 32;
        for (int i = 0; i < m; ++i) word |= (uint32_t)(src[i] != 0) << i;
    }
    hv[idx] = word;
}

template <bool VEC>
__global__ __launch_bounds__(256) void unpack_kernel(const uint32_t *__restrict__ hv, int64_t N, int D, int W,
                                                     uint8_t *__restrict__ bits) {
    const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (idx >= N * W) return;
    const int64_t n = idx / W;
    const int w = (int)(idx - n * W);
    const uint32_t word = hv[idx];
    uint8_t *dst = bits + n * D + 32 * w;
    const int left = D - 32 * w;
    if (VEC) {
        uint4 a, b;
        a.x = bytes_of_nibble(word & 15u);
        a.y = bytes_of_nibble((word >> 4) & 15u);
        a.z = bytes_of_nibble((word >> 8) & 15u);
        a.w = bytes_of_nibble((word >> 12) & 15u);
        *reinterpret_cast<uint4 *>(dst) = a;
        if (left >= 32) {
            b.x = bytes_of_nibble((word >> 16) & 15u);
            b.y = bytes_of_nibble((word >> 20) & 15u);
            b.z = bytes_of_nibble((word >> 24) & 15u);
            b.w = bytes_of_nibble(word >> 28);
            *reinterpret_cast<uint4 *>(dst + 16) = b;
        }
    } else {
        const int m = left < 32 ? left : 32;
        for (int i = 0; i < m; ++i) dst[i] = (uint8_t)((word >> i) & 1u);
    }
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
    const int64_t words = N * c->W;
    const dim3 grid((unsigned)((words + 255) / 256));
    if (vec_ok(bits, c->p.D))
        hipLaunchKernelGGL(pack_kernel<true>, grid, dim3(256), 0, s, bits, N, c->p.D, c->W, hv);
    else
        hipLaunchKernelGGL(pack_kernel<false>, grid, dim3(256), 0, s, bits, N, c->p.D, c->W, hv);
    HDC_HIP(hipGetLastError());
    return HDC_OK;
}

int launch_unpack(hdc_ctx_impl *c, const uint32_t *hv, int64_t N, uint8_t *bits, hipStream_t s) {
    const int64_t words = N * c->W;
    const dim3 grid((unsigned)((words + 255) / 256));
    if (vec_ok(bits, c->p.D))
        hipLaunchKernelGGL(unpack_kernel<true>, grid, dim3(256), 0, s, hv, N, c->p.D, c->W, bits);
    else
        hipLaunchKernelGGL(unpack_kernel<false>, grid, dim3(256), 0, s, hv, N, c->p.D, c->W, bits);
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
