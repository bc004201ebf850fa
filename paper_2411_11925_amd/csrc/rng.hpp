// Counter-based generator of the sampler: Philox-4x32-10 (Salmon et al., SC'11)
// plus fixed-sequence fp32 transforms to uniforms and normals.
//
// Counter = (row_lo, row_hi, slot | stream << 16, block); key = (seed_lo, seed_hi).
// One counter gives four 32-bit words.  Uniform: (w >> 9 + 1/2) * 2^-23, exact in
// fp32.  Normals: Box-Muller on word pairs (0,1) and (2,3), each evaluated by the
// operation sequence below in IEEE fp32 with no fused multiply-add, so any
// conforming implementation reproduces the same bit patterns:
//   u1 = uniform(w_a);  split u1 = m*2^e, m in [1,2); if m > SQRT2: m*=0.5, e+=1
//   s = (m-1)/(m+1); s2 = s*s; p = ((C9*s2 + C7)*s2 + C5)*s2 + C3
//   ln u1 = float(e)*LN2 + (2*s)*(s2*p + 1);  r = sqrt(-2 * ln u1)
//   k = w_b >> 9; quarter = k >> 21; f = (float(k & 0x1FFFFF) + 1/2) * 2^-21
//   g = f > 1/2 ? 1 - f : f;  y = g*HALFPI;  y2 = y*y
//   sin = y*((((S9*y2 + S7)*y2 + S5)*y2 + S3)*y2 + 1)
//   cos = ((((K10*y2 + K8)*y2 + K6)*y2 + K4)*y2 + K2)*y2 + 1
//   f > 1/2 swaps sin and cos; the quarter rotates (cos,sin) by 90 degrees each.
//   n0 = r*cos(angle), n1 = r*sin(angle)
// Constants are given as fp32 bit patterns.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace csd {

struct Words4 { uint32_t w0, w1, w2, w3; };

__device__ __forceinline__ Words4 philox4x32_10(uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3,
                                                uint32_t k0, uint32_t k1) {
#pragma unroll
    for (int r = 0; r < 10; ++r) {
        const uint32_t hi0 = __umulhi(0xD2511F53u, c0), lo0 = 0xD2511F53u * c0;
        const uint32_t hi1 = __umulhi(0xCD9E8D57u, c2), lo1 = 0xCD9E8D57u * c2;
        const uint32_t n0 = hi1 ^ c1 ^ k0, n2 = hi0 ^ c3 ^ k1;
        c0 = n0; c1 = lo1; c2 = n2; c3 = lo0;
        k0 += 0x9E3779B9u; k1 += 0xBB67AE85u;
    }
    return Words4{c0, c1, c2, c3};
}

__device__ __forceinline__ Words4 philox_at(uint64_t seed, uint64_t row, uint32_t slot,
                                            uint32_t stream, uint32_t block) {
    return philox4x32_10((uint32_t)row, (uint32_t)(row >> 32), (slot & 0xFFFFu) | (stream << 16), block,
                         (uint32_t)seed, (uint32_t)(seed >> 32));
}

__device__ __forceinline__ float uniform23(uint32_t w) {
#pragma clang fp contract(off)
    return ((float)(w >> 9) + 0.5f) * __uint_as_float(0x34000000u);   // 2^-23
}

__device__ __forceinline__ void normal_pair(uint32_t wa, uint32_t wb, float& n0, float& n1) {
#pragma clang fp contract(off)
    const float u1 = uniform23(wa);
    const uint32_t bits = __float_as_uint(u1);
    int e = (int)(bits >> 23) - 127;
    float m = __uint_as_float((bits & 0x007FFFFFu) | 0x3F800000u);
    if (m > __uint_as_float(0x3FB504F3u)) { m = m * 0.5f; e += 1; }
    const float s = __fdiv_rn(m - 1.0f, m + 1.0f);
    const float s2 = s * s;
    float p = __uint_as_float(0x3DE38E39u);            // 1/9
    p = p * s2; p = p + __uint_as_float(0x3E124925u);  // 1/7
    p = p * s2; p = p + __uint_as_float(0x3E4CCCCDu);  // 1/5
    p = p * s2; p = p + __uint_as_float(0x3EAAAAABu);  // 1/3
    float w = s2 * p; w = w + 1.0f;
    const float lnm = (2.0f * s) * w;
    float lnu = (float)e * __uint_as_float(0x3F317218u);   // ln 2
    lnu = lnu + lnm;
    const float r = __builtin_sqrtf(-2.0f * lnu);   // correctly rounded (not the 1-ulp native sqrt)

    const uint32_t k = wb >> 9;
    const uint32_t quarter = k >> 21;
    const float f = ((float)(k & 0x001FFFFFu) + 0.5f) * __uint_as_float(0x35000000u);  // 2^-21
    const bool hi = f > 0.5f;
    const float g = hi ? 1.0f - f : f;
    const float y = g * __uint_as_float(0x3FC90FDBu);      // pi/2
    const float y2 = y * y;
    float ps = __uint_as_float(0x3638EF1Du);               // 1/9!
    ps = ps * y2; ps = ps + __uint_as_float(0xB9500D01u);  // -1/7!
    ps = ps * y2; ps = ps + __uint_as_float(0x3C088889u);  // 1/5!
    ps = ps * y2; ps = ps + __uint_as_float(0xBE2AAAABu);  // -1/3!
    ps = ps * y2; ps = ps + 1.0f;
    float sn = y * ps;
    float pc = __uint_as_float(0xB493F27Eu);               // -1/10!
    pc = pc * y2; pc = pc + __uint_as_float(0x37D00D01u);  // 1/8!
    pc = pc * y2; pc = pc + __uint_as_float(0xBAB60B61u);  // -1/6!
    pc = pc * y2; pc = pc + __uint_as_float(0x3D2AAAABu);  // 1/4!
    pc = pc * y2; pc = pc + -0.5f;
    pc = pc * y2;
    float cs = pc + 1.0f;
    if (hi) { const float tmp = sn; sn = cs; cs = tmp; }
    float c, sv;
    switch (quarter) {
        case 0: c = cs; sv = sn; break;
        case 1: c = -sn; sv = cs; break;
        case 2: c = -cs; sv = -sn; break;
        default: c = sn; sv = -cs; break;
    }
    n0 = r * c;
    n1 = r * sv;
}

// four standard normals: elements 4*block .. 4*block+3 of the row's draw
__device__ __forceinline__ void normals4(uint64_t seed, uint64_t row, uint32_t slot, uint32_t stream,
                                         uint32_t block, float out[4]) {
    const Words4 w = philox_at(seed, row, slot, stream, block);
    normal_pair(w.w0, w.w1, out[0], out[1]);
    normal_pair(w.w2, w.w3, out[2], out[3]);
}

__device__ __forceinline__ float uniform_at(uint64_t seed, uint64_t row, uint32_t slot, uint32_t stream) {
    return uniform23(philox_at(seed, row, slot, stream, 0).w0);
}

}  // namespace csd
