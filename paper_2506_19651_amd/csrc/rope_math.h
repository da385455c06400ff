// Rotation arithmetic of the RoPE step (Sec. "Position Encoding"), shared by the stand-alone RoPE
// kernel, the cos/sin table kernel and the attention kernel's fused query rotation, so that a query
// rotated on the fly has exactly the bits pevlm_rope_seq would have stored.  Every contraction is
// written out (fma) so that the result does not depend on the surrounding code.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace pevlm {

struct RopeFreq {
    double inv_freq[64];  // rope_base^(-2i/D), i < D/2
};

// cos / sin of pos * inv_freq: the angle is formed in fp64 and reduced to [-pi, pi] before the fp32
// (bf16 tensors) or fp64 (fp32 tensors) sine and cosine.
template <bool WIDE>
__device__ __forceinline__ void rope_cos_sin(double pos, double inv_freq, float &c, float &s)
{
    const double two_pi = 6.283185307179586476925286766559;
    const double theta = pos * inv_freq;
    const double r = fma(-two_pi, rint(theta / two_pi), theta);
    if (WIDE) {
        double sd, cd;
        sincos(r, &sd, &cd);
        s = (float)sd;
        c = (float)cd;
    } else {
        sincosf((float)r, &s, &c);
    }
}

// (a, b) = (x[i], x[i + D/2]) turned by the angle whose cosine and sine are c, s
__device__ __forceinline__ void rope_rotate(float a, float b, float c, float s, float &lo, float &hi)
{
    lo = __builtin_fmaf(a, c, -(b * s));
    hi = __builtin_fmaf(b, c, a * s);
}

typedef __attribute__((ext_vector_type(2))) __bf16 rope_bf16x2;

// two fp32 values -> packed bf16 pair, round to nearest even (x0 in the low half)
__device__ __forceinline__ uint32_t rope_pack_bf16(float x0, float x1)
{
    rope_bf16x2 v;
    v[0] = (__bf16)x0;
    v[1] = (__bf16)x1;
    return __builtin_bit_cast(uint32_t, v);
}

}  // namespace pevlm
