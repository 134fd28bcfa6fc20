// Arithmetic of the input transforms of a linear layer (device code shared by
// the standalone kernels and the persistent decode kernel): RMSNorm with an
// optional residual add in front, and SiLU(gate) * up.  Paper: kernel table
// (RMS-norm and SiLU-multiply kernels of the decode path); the formulas are the
// usual ones.  Every result is rounded to bf16 once, to nearest even.
#pragma once

#include "nvq_internal.h"

namespace nvq {

#if defined(__HIPCC__)

// a + b of two bf16 numbers, rounded to bf16 once.  The sum is formed in
// binary32 and rounded again to bf16; with an 8-bit significand that is the
// same as rounding the exact sum once (double rounding is innocuous for sums,
// products, quotients and roots when the wider format has at least 2 * 8 + 2
// bits of significand: Figueroa, "When is double rounding innocuous?", 1995).
__device__ __forceinline__ uint32_t add_bf16_bits(uint32_t a, uint32_t b) {
    return float_to_bf16_bits(bf16_bits_to_float(a) + bf16_bits_to_float(b));
}

// Eight bf16 values (one uint4) at a time.
__device__ __forceinline__ uint4 add_bf16x8(const uint4 &a, const uint4 &b) {
    const uint32_t av[4] = {a.x, a.y, a.z, a.w}, bv[4] = {b.x, b.y, b.z, b.w};
    uint32_t o[4];
#pragma unroll
    for (int d = 0; d < 4; ++d)
        o[d] = pack_bf16x2(bf16_bits_to_float(av[d] & 0xffffu) + bf16_bits_to_float(bv[d] & 0xffffu),
                           bf16_bits_to_float(av[d] >> 16) + bf16_bits_to_float(bv[d] >> 16));
    return make_uint4(o[0], o[1], o[2], o[3]);
}

__device__ __forceinline__ float sumsq_bf16x8(const uint4 &h) {
    const uint32_t hv[4] = {h.x, h.y, h.z, h.w};
    float s = 0.0f;
#pragma unroll
    for (int d = 0; d < 4; ++d) {
        const float lo = bf16_bits_to_float(hv[d] & 0xffffu), hi = bf16_bits_to_float(hv[d] >> 16);
        s = fmaf(lo, lo, s);
        s = fmaf(hi, hi, s);
    }
    return s;
}

// 1 / sqrt(mean of squares + eps) from the sum of squares of K values.
__device__ __forceinline__ float rms_scale(float sumsq, int K, float eps) {
    return 1.0f / sqrtf(sumsq / (float)K + eps);
}

// bf16(h * r * gamma), eight at a time.
__device__ __forceinline__ uint4 scale_bf16x8(const uint4 &h, float r, const uint4 &gamma) {
    const uint32_t hv[4] = {h.x, h.y, h.z, h.w}, gv[4] = {gamma.x, gamma.y, gamma.z, gamma.w};
    uint32_t o[4];
#pragma unroll
    for (int d = 0; d < 4; ++d) {
        const float lo = bf16_bits_to_float(hv[d] & 0xffffu) * r * bf16_bits_to_float(gv[d] & 0xffffu);
        const float hi = bf16_bits_to_float(hv[d] >> 16) * r * bf16_bits_to_float(gv[d] >> 16);
        o[d] = pack_bf16x2(lo, hi);
    }
    return make_uint4(o[0], o[1], o[2], o[3]);
}

// g / (1 + exp(-g)) * u with the hardware's exp2 and reciprocal (each good to
// about one unit of binary32; the argument of exp2 adds |g| * 2^-24 relative):
// far below the bf16 rounding that follows, a handful of instructions instead
// of some forty.  Where this runs every workgroup evaluates the whole vector
// before its first weight row, so the instructions are time on the critical path.
__device__ __forceinline__ float silu_mul_one(float g, float u) {
    const float e = __builtin_amdgcn_exp2f(g * -1.44269504088896341f);
    return g * __builtin_amdgcn_rcpf(1.0f + e) * u;
}

// bf16(silu(g) * u), eight at a time.
__device__ __forceinline__ uint4 silu_mul_bf16x8(const uint4 &g, const uint4 &u) {
    const uint32_t gv[4] = {g.x, g.y, g.z, g.w}, uv[4] = {u.x, u.y, u.z, u.w};
    uint32_t o[4];
#pragma unroll
    for (int d = 0; d < 4; ++d) {
        const float lo = silu_mul_one(bf16_bits_to_float(gv[d] & 0xffffu),
                                      bf16_bits_to_float(uv[d] & 0xffffu));
        const float hi = silu_mul_one(bf16_bits_to_float(gv[d] >> 16),
                                      bf16_bits_to_float(uv[d] >> 16));
        o[d] = pack_bf16x2(lo, hi);
    }
    return make_uint4(o[0], o[1], o[2], o[3]);
}

#endif  // __HIPCC__

// Internal launchers (validated arguments; enqueue only).  One workgroup per
// token; K % 8 == 0.
int launch_rms_norm(const uint16_t *x, const uint16_t *res, const uint16_t *gamma, float eps, int M,
                    int K, uint16_t *out, uint16_t *h_out, hipStream_t st);
int launch_silu_mul(const uint16_t *g, const uint16_t *u, int M, int K, uint16_t *out,
                    hipStream_t st);

}  // namespace nvq
