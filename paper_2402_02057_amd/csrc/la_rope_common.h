// Rotary position embedding, the arithmetic shared by the pass of its own (la_step_rope), by the
// attention kernel that rotates its query rows (and, on request, the step keys) on the way in and
// by the append that rotates the key rows it copies: written out operation by operation, so that
// all of them give the same bits.
#pragma once
#include <hip/hip_runtime.h>

namespace la {

// Pair (a, b) turned by the angle with cosine c and sine s: (a c - b s, b c + a s), each with one
// product rounded and one fused multiply-add, in fp32.
__device__ __forceinline__ void rope_pair(float a, float b, float c, float s, float& ra, float& rb)
{
    const float bs = b * s, as = a * s;
    ra = __builtin_fmaf(a, c, -bs);
    rb = __builtin_fmaf(b, c, as);
}

// Eight pairs held in two 16-byte vectors of a row (xa, xb), with the eight cosines and sines of
// the pairs.  interleaved == false: pair e is (xa[e], xb[e]) (the vectors are pieces c and
// c + head_dim/16 of the row); true: the sixteen elements are the pairs (0,1), (2,3), ...
template <class V8>
__device__ __forceinline__ void rope_eight_pairs(const V8& xa, const V8& xb, const float (&co)[8],
                                                 const float (&si)[8], bool interleaved, V8& ya, V8& yb)
{
    if (interleaved) {
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            const float a = e < 4 ? (float)xa[2 * e] : (float)xb[2 * e - 8];
            const float b = e < 4 ? (float)xa[2 * e + 1] : (float)xb[2 * e - 7];
            float ra, rb;
            rope_pair(a, b, co[e], si[e], ra, rb);
            if (e < 4) { ya[2 * e] = (__bf16)ra; ya[2 * e + 1] = (__bf16)rb; }
            else { yb[2 * e - 8] = (__bf16)ra; yb[2 * e - 7] = (__bf16)rb; }
        }
    } else {
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            float ra, rb;
            rope_pair((float)xa[e], (float)xb[e], co[e], si[e], ra, rb);
            ya[e] = (__bf16)ra;
            yb[e] = (__bf16)rb;
        }
    }
}

}  // namespace la
