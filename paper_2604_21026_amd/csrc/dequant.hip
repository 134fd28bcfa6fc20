// nvq_dequant_bf16: packed int4 weights -> dense bf16 weights for the prefill /
// large-batch path, where the product is a real contraction and a dense GEMM
// takes over.  Paper: kernel table, the dequantisation kernel that materialises
// 16-bit weights for the library GEMM (its 16-bit type is F16, ours bf16).
//
// out[n][k] = bf16(code * scale).  The product of a 4-bit code and an fp16
// scale is exact in binary32, so the one rounding (to nearest even) is the one
// to bf16 and a CPU run of the same rule gives equal bits.
//
// Four lanes per group of 32 weights: lane q of the four produces weights
// 8q .. 8q+7 (one 16-byte store, so a wave writes 1 KiB of contiguous output
// per instruction) from the 8 bytes that hold them: the low nibbles of bytes
// 0-7 (q = 0) or 8-15 (q = 1), or the high nibbles of the same bytes (q = 2, 3).
#include "nvq_internal.h"

namespace nvq {

__global__ __launch_bounds__(256) void dequant_bf16_kernel(const uint2 *__restrict__ qw,
                                                           const uint16_t *__restrict__ scales,
                                                           int64_t groups,
                                                           uint4 *__restrict__ out) {
    const int64_t t = (int64_t)blockIdx.x * 256 + threadIdx.x;
    const int64_t g = t >> 2;
    const int q = (int)(t & 3);
    if (g >= groups) return;
    const uint2 b = qw[g * 2 + (q & 1)];
    const float s = half_bits_to_float(scales[g]);
    const int shift = (q >> 1) * 4;
    const uint32_t w[2] = {(b.x >> shift) & 0x0f0f0f0fu, (b.y >> shift) & 0x0f0f0f0fu};
    uint32_t o[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const int c0 = (int)((w[j >> 1] >> (16 * (j & 1))) & 0xffu) - 8;
        const int c1 = (int)((w[j >> 1] >> (16 * (j & 1) + 8)) & 0xffu) - 8;
        o[j] = pack_bf16x2((float)c0 * s, (float)c1 * s);
    }
    // written once, read later by another kernel: keep it out of the way of the weights
    typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
    const u32x4 v = {o[0], o[1], o[2], o[3]};
    __builtin_nontemporal_store(v, reinterpret_cast<u32x4 *>(out) + t);
}

}  // namespace nvq

extern "C" int nvq_dequant_bf16(const uint8_t *qweight, const uint16_t *scales, int64_t N,
                                int64_t K, uint16_t *out_bf16, void *stream) {
    if (!qweight || !scales || !out_bf16) return NVQ_ERR_INVALID_ARG;
    if (N <= 0 || K <= 0 || (K % 32) != 0 || K > NVQ_MAX_K) return NVQ_ERR_SHAPE;
    if (!nvq::aligned(qweight, 16) || !nvq::aligned(scales, 2) || !nvq::aligned(out_bf16, 16))
        return NVQ_ERR_ALIGN;
    const int64_t groups = N * (K / 32);
    const int64_t blocks = (groups * 4 + 255) / 256;
    if (blocks > 0x7fffffffLL) return NVQ_ERR_SHAPE;
    hipLaunchKernelGGL(nvq::dequant_bf16_kernel, dim3((unsigned)blocks), dim3(256), 0,
                       (hipStream_t)stream, reinterpret_cast<const uint2 *>(qweight), scales,
                       groups, reinterpret_cast<uint4 *>(out_bf16));
    NVQ_HIP_TRY(hipGetLastError());
    return NVQ_OK;
}
