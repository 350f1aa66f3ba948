// Power-of-two scalings of the fp16 value path, derived from per-head statistics.  Used by the conversion
// pre-pass and by the main kernel, which must agree bit for bit.
//
// Per (batch, head), stats[8] = { max|V|, max|tV|, max row norm^2 of Q, of tQ, of K, of tK, 0, 0 }.
//   V16  = fp16(V  * 2^-eV)   with max|V16|  in [2^13, 2^14)
//   tV16 = fp16(tV * 2^-eA)
//   H~16 = fp16(H~ * 2^(eV - eA))
// so that the O accumulator holds 2^-eV O~ and the A+B accumulator holds 2^-eA (A + B).  eA is the smallest
// exponent that keeps both |tV16| < 2^14 and |H~16| <= P~ * 2^8, using the Cauchy-Schwarz bound
// |tS scale - ctr| <= 2 scale (|tq||k| + |q||tk|) for the tangent scores.  The row norms come from a sample of
// the rows (every 16th and the last), so this is an estimate of that bound, which itself is loose by an order of
// magnitude on ordinary data.  Scores smaller than it only lose headroom; should a tangent score exceed what the
// scale allows, H~16 overflows to inf, which the main kernel detects at the end of its sweep, and the tile is redone
// by the bf16-pair kernel: a wrong estimate costs time, never correctness.
#pragma once
#include <hip/hip_runtime.h>

namespace attn_jvp {

struct F16Scales {
    int eV, eA;
};

__host__ __device__ inline int ilogb_pos(float x) {   // floor(log2 x) for finite x > 0 (denormals -> -127)
    union { float f; unsigned u; } c;
    c.f = x;
    return (int)((c.u >> 23) & 0xff) - 127;
}

__host__ __device__ inline F16Scales f16_scales(const float* st, float scale) {
    F16Scales r;
    const float mV = st[0], mT = st[1];
    r.eV = mV > 0.f ? ilogb_pos(mV) - 13 : 0;
    const float umax = 2.f * fabsf(scale) * (sqrtf(st[3]) * sqrtf(st[4]) + sqrtf(st[2]) * sqrtf(st[5]));
    int eA = -1000;
    if (umax > 0.f && umax < 3.0e38f) eA = r.eV + ilogb_pos(umax) + 1 - 8;
    if (mT > 0.f) {
        const int eT = ilogb_pos(mT) - 13;
        eA = eT > eA ? eT : eA;
    }
    if (eA == -1000) eA = r.eV;          // no tangent anywhere: any value works
    // keep 2^(eV - eA) and the epilogue factors inside the float range
    if (eA < r.eV - 60) eA = r.eV - 60;
    if (eA > r.eV + 60) eA = r.eV + 60;
    r.eA = eA;
    return r;
}

}  // namespace attn_jvp
