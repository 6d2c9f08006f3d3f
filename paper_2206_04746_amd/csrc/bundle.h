// Device helpers shared by the encoding kernels (arXiv 2206.04746, Sec. III, Eq. 1): the bin rule,
// the LDS gather of level rows and the bit-sliced carry-save adders that bundle bound words.
#ifndef HDC_BUNDLE_H
#define HDC_BUNDLE_H

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

// ------------------------------------------------------------- bundling (Eq. 1's sum)
typedef const uint32_t __attribute__((address_space(4))) *const_u32_ptr;

// Level words of 16 features for this lane's column come from the LDS level slice.  The row
// offset is wave-uniform, so it goes through M0 and ds_read_addtid_b32 (address = M0 + lane*4):
// no vector ALU work is spent on addresses.  One wait state separates a write of M0 from the
// LDS instruction that reads it.  q[k] holds the LDS byte offsets (bin * 256) of features 2k
// and 2k+1 as two u16.  The 16 level words arrive in compiler-allocated registers and the asm
// statement ends with the wait, so nothing is in flight outside it.  No "memory" clobber: the
// level slice is read-only after the barrier that publishes it (a volatile asm cannot cross
// that barrier), and without the clobber the compiler may fetch the next bin offsets early.
__device__ __forceinline__ void gather16(uint32_t (&x)[16], const uint32_t (&q)[8]) {
#define HDC_G2(qs, a, b)                                                      \
    "s_and_b32 m0, " qs ", 0xffff\n\ts_nop 0\n\tds_read_addtid_b32 " a "\n\t" \
    "s_lshr_b32 m0, " qs ", 16\n\ts_nop 0\n\tds_read_addtid_b32 " b "\n\t"
    asm volatile(HDC_G2("%16", "%0", "%1") HDC_G2("%17", "%2", "%3") HDC_G2("%18", "%4", "%5")
                 HDC_G2("%19", "%6", "%7") HDC_G2("%20", "%8", "%9") HDC_G2("%21", "%10", "%11")
                 HDC_G2("%22", "%12", "%13") HDC_G2("%23", "%14", "%15") "s_waitcnt lgkmcnt(0)"
                 : "=&v"(x[0]), "=&v"(x[1]), "=&v"(x[2]), "=&v"(x[3]), "=&v"(x[4]), "=&v"(x[5]), "=&v"(x[6]),
                   "=&v"(x[7]), "=&v"(x[8]), "=&v"(x[9]), "=&v"(x[10]), "=&v"(x[11]), "=&v"(x[12]),
                   "=&v"(x[13]), "=&v"(x[14]), "=&v"(x[15])
                 : "s"(q[0]), "s"(q[1]), "s"(q[2]), "s"(q[3]), "s"(q[4]), "s"(q[5]), "s"(q[6]), "s"(q[7])
                 : "scc");
#undef HDC_G2
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

}  // namespace hdc

#endif  // HDC_BUNDLE_H
