// Pieces shared by the matrix-core kernels for small batches: the operand
// types of the 16x16x32 MFMAs, the 4x4 dword transpose across the four 16-lane
// rows of a wave, and per precision (W4A8, W4A16) how activations are loaded,
// brought into operand order and multiplied.  Paper: the W4A8 / W4A16 kernel
// descriptions and the deferred correction of the constant nibble offset.
#pragma once

#include "nvq_internal.h"

namespace nvq {

typedef int int4v __attribute__((ext_vector_type(4)));
typedef float float4v __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef unsigned uint2v __attribute__((ext_vector_type(2)));
typedef unsigned uint4v __attribute__((ext_vector_type(4)));

// Pointers that come out of a table in memory are generic to the compiler;
// every access here is to global memory, and saying so keeps the loads off the
// slower flat path.
template <typename T>
__device__ __forceinline__ const __attribute__((address_space(1))) T *as_global(const void *p) {
    return (const __attribute__((address_space(1))) T *)p;
}

__device__ __forceinline__ void store_global(void *y, int y_dtype, int64_t idx, float v) {
    if (y_dtype == NVQ_F32)
        ((__attribute__((address_space(1))) float *)y)[idx] = v;
    else
        ((__attribute__((address_space(1))) uint16_t *)y)[idx] = float_to_bf16_bits(v);
}

// Weights are loaded through the caches: a wave reads 64 bytes of each of 16
// rows per load and its neighbours read the other halves of the same 128-byte
// lines a little later; with non-temporal loads a third of the lines was
// fetched from HBM twice.
__device__ __forceinline__ uint4v load_stream(const uint4 *p) {
    return *as_global<uint4v>(p);
}

// r[j] of lane-row kb holds element (kb, j) of a 4x4 matrix of dwords (one
// matrix per lane column n); afterwards r[i] of lane-row kb holds (i, kb).
__device__ __forceinline__ void transpose_rows(uint32_t (&r)[4]) {
    const uint2v a = __builtin_amdgcn_permlane32_swap(r[0], r[2], false, false);
    const uint2v b = __builtin_amdgcn_permlane32_swap(r[1], r[3], false, false);
    const uint2v c = __builtin_amdgcn_permlane16_swap(a.x, b.x, false, false);
    const uint2v d = __builtin_amdgcn_permlane16_swap(a.y, b.y, false, false);
    r[0] = c.x;
    r[1] = c.y;
    r[2] = d.x;
    r[3] = d.y;
}

template <int PREC>
struct Act;

// int8 codes: 8 bytes per lane and MFMA.
template <>
struct Act<NVQ_W4A8> {
    typedef long operand;
    static constexpr int kBytes = 1;
    // Raw activations of a column (4 groups x 32 codes = 128 bytes per token):
    // lane (m, kb) loads the two halves of group kb of token m.
    static constexpr int kRaw = 2;
    static constexpr int kLaneBytes = 32;  // byte offset of lane-row kb: kb * 32
    __device__ static void load(const char *p, uint4v (&raw)[kRaw]) {
        raw[0] = *as_global<uint4v>(p);
        raw[1] = *as_global<uint4v>(p + 16);
    }
    // Operands of groups 0..3: dword kb of each half (codes 4kb..4kb+3 and
    // 16+4kb..16+4kb+3), the choice the weight operand makes.
    template <int NRAW>
    __device__ static void operands(const uint4v (&raw)[NRAW], operand (&a)[4]) {
        uint32_t lo[4] = {raw[0].x, raw[0].y, raw[0].z, raw[0].w};
        uint32_t hi[4] = {raw[1].x, raw[1].y, raw[1].z, raw[1].w};
        transpose_rows(lo);
        transpose_rows(hi);
#pragma unroll
        for (int i = 0; i < 4; ++i) a[i] = (long)((uint64_t)lo[i] | ((uint64_t)hi[i] << 32));
    }
    __device__ static operand weights(uint32_t v) {
        const uint32_t lo = v & 0x0f0f0f0fu, hi = (v >> 4) & 0x0f0f0f0fu;
        return (long)((uint64_t)lo | ((uint64_t)hi << 32));
    }
    __device__ static int4v offset(operand a) {
        const int4v z = {0, 0, 0, 0};
        return __builtin_amdgcn_mfma_i32_16x16x32_i8(a, (long)0xf8f8f8f8f8f8f8f8ull, z, 0, 0, 0);
    }
    __device__ static float4v product(operand a, operand b, int4v c, int4v &raw) {
        raw = __builtin_amdgcn_mfma_i32_16x16x32_i8(a, b, c, 0, 0, 0);
        const float4v f = {(float)raw.x, (float)raw.y, (float)raw.z, (float)raw.w};
        return f;
    }
    typedef int4v offset_t;
};

// bf16 activations: 16 bytes per lane and MFMA.
template <>
struct Act<NVQ_W4A16> {
    typedef bf16x8 operand;
    static constexpr int kBytes = 2;
    // Raw activations of a column (4 groups x 32 bf16 = 256 bytes per token):
    // lane (m, kb) loads the 16-byte piece kb of each group of token m, so one
    // load instruction reads 64 contiguous bytes per token.
    static constexpr int kRaw = 4;
    static constexpr int kLaneBytes = 16;
    __device__ static void load(const char *p, uint4v (&raw)[kRaw]) {
#pragma unroll
        for (int i = 0; i < 4; ++i) raw[i] = *as_global<uint4v>(p + 64 * i);
    }
    // Lane-row kb needs activations 4kb..4kb+3 and 16+4kb..16+4kb+3 of a group:
    // the first or second half of piece kb/2 and of piece 2 + kb/2.  For the
    // first dwords of the halves, x and z of the four pieces: a permlane16 swap
    // gives rows (x0 z0 x2 z2) and (x1 z1 x3 z3), a permlane32 swap of those
    // (x0 z0 x1 z1) and (x2 z2 x3 z3); the same for the second dwords y and w.
    template <int NRAW>
    __device__ static void operands(const uint4v (&raw)[NRAW], operand (&a)[4]) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const uint2v xz = __builtin_amdgcn_permlane16_swap(raw[i].x, raw[i].z, false, false);
            const uint2v x = __builtin_amdgcn_permlane32_swap(xz.x, xz.y, false, false);
            const uint2v yw = __builtin_amdgcn_permlane16_swap(raw[i].y, raw[i].w, false, false);
            const uint2v y = __builtin_amdgcn_permlane32_swap(yw.x, yw.y, false, false);
            a[i] = __builtin_bit_cast(bf16x8, make_uint4(x.x, y.x, x.y, y.y));
        }
    }
    __device__ static operand weights(uint32_t v) {
        constexpr uint32_t kMagic = 0x43434343u;  // high byte of bf16(128 + n)
        const uint32_t lo = v & 0x0f0f0f0fu, hi = (v >> 4) & 0x0f0f0f0fu;
        // byte permute: selector 0-3 picks a byte of the second operand, 4-7 of the first
        const uint4 b = make_uint4(__builtin_amdgcn_perm(kMagic, lo, 0x04010400u),
                                   __builtin_amdgcn_perm(kMagic, lo, 0x04030402u),
                                   __builtin_amdgcn_perm(kMagic, hi, 0x04010400u),
                                   __builtin_amdgcn_perm(kMagic, hi, 0x04030402u));
        return __builtin_bit_cast(bf16x8, b);
    }
    __device__ static float4v offset(operand a) {
        const float4v z = {0.0f, 0.0f, 0.0f, 0.0f};
        constexpr uint32_t kNeg136 = 0xc308c308u;  // bf16(-136) twice
        const uint4 c = make_uint4(kNeg136, kNeg136, kNeg136, kNeg136);
        return __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, __builtin_bit_cast(bf16x8, c), z, 0, 0,
                                                       0);
    }
    __device__ static float4v product(operand a, operand b, float4v c, int4v &raw) {
        (void)raw;
        return __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b, c, 0, 0, 0);
    }
    typedef float4v offset_t;
};

}  // namespace nvq
