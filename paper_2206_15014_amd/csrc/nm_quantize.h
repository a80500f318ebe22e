// The scalar quantiser of Sec. 3.3 (Eq. 5, offset 0) as the kernels evaluate it: a correctly
// rounded fp32 quotient, round half to even, symmetric clamp.  Shared by the weight compressor
// and the activation quantiser so that both take the same decision on every input.
#ifndef NM_QUANTIZE_H
#define NM_QUANTIZE_H

#include <hip/hip_runtime.h>

namespace nm {

// The correctly rounded fp32 quotient w / s for many w and one s.  RECIP = false: the division
// operator.  RECIP = true: the same value from y = RN(1 / s), computed once per row: q0 = RN(w y)
// is within 1.5 ulp of w / s (y and the product each carry half an ulp of their own); one
// residual step, q1 = RN(q0 + RN(w - s q0) y), lands within half an ulp plus a 2^-24th of an ulp,
// i.e. on one of the two neighbours of w / s; and for such a q1 the residual w - s q1 is exact in
// one fused multiply-add and q2 = RN(q1 + (w - s q1) y) is RN(w / s) itself when y is the
// correctly rounded reciprocal (Markstein's theorem on fused-multiply-add division) - five
// operations in place of the eleven of the division sequence.  Valid without overflow, underflow
// or subnormal y; the caller takes this route only for 2^-60 <= s <= 2^60, where |w| <= 127 s
// keeps every intermediate normal or, for quotients far below one half, irrelevant to the code.
template <bool RECIP>
struct Divisor {
    float s, y;
    __device__ __forceinline__ float quotient(float w) const
    {
        if constexpr (RECIP) {
            const float q0 = __fmul_rn(w, y);
            const float q1 = __fmaf_rn(__fmaf_rn(-s, q0, w), y, q0);
            return __fmaf_rn(__fmaf_rn(-s, q1, w), y, q1);
        } else {
            return __fdiv_rn(w, s);
        }
    }
};

// Eq. 5 with offset 0: correctly rounded fp32 quotient, round half to even, symmetric clamp.
template <int BITS, bool RECIP>
__device__ __forceinline__ int quantize(float w, const Divisor<RECIP>& d)
{
    constexpr float QMAX = (float)((1 << (BITS - 1)) - 1);
    float r = rintf(d.quotient(w));
    r = fminf(fmaxf(r, -QMAX), QMAX);
    return (int)r;
}

}  // namespace nm

#endif
