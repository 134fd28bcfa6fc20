// nvq_pack_int4: fp32 weights -> planar int4 codes + fp16 group scales.
// Block format after the paper's W4A8 section (32 weights, one fp16 scale,
// nibbles centred at 8); scale rule absmax / 7, round-half-to-even, IEEE
// division so that a CPU implementation of the same rule gives the same bytes.
//
// Eight lanes own one group of 32 weights (one float4 each), so a wave reads
// 1 KiB of consecutive weights per load.  Lanes 0-3 of a team hold the low
// nibbles of the 16 output bytes, lanes 4-7 the high nibbles; one cross-lane
// exchange merges them and lanes 0-3 store one dword each.
#include "nvq_internal.h"

namespace nvq {

__global__ __launch_bounds__(256) void pack_int4_kernel(const float4 *__restrict__ W,
                                                        int64_t total_groups,
                                                        uint32_t *__restrict__ qw,
                                                        uint16_t *__restrict__ scales) {
    const int sub = threadIdx.x & 7;
    int64_t gid = (int64_t)blockIdx.x * 32 + (threadIdx.x >> 3);
    const bool valid = gid < total_groups;
    if (!valid) gid = total_groups - 1;  // keep the whole team in the exchange below

    const float4 w = W[gid * 8 + sub];
    float amax = fmaxf(fmaxf(fabsf(w.x), fabsf(w.y)), fmaxf(fabsf(w.z), fabsf(w.w)));
    amax = fmaxf(amax, __shfl_xor(amax, 1, 64));
    amax = fmaxf(amax, __shfl_xor(amax, 2, 64));
    amax = fmaxf(amax, __shfl_xor(amax, 4, 64));

    const float s32 = amax / 7.0f;
    const _Float16 sh = (_Float16)s32;  // round to nearest even
    const float s = (float)sh;
    const bool live = (s != 0.0f) && !__builtin_isinf(s);

    auto code = [&](float v) -> uint32_t {
        if (!live) return 8u;
        float r = rintf(v / s);
        r = fminf(fmaxf(r, -8.0f), 7.0f);
        return (uint32_t)((int)r + 8);
    };
    const uint32_t mine = code(w.x) | (code(w.y) << 8) | (code(w.z) << 16) | (code(w.w) << 24);
    const uint32_t other = __shfl_xor(mine, 4, 64);
    if (valid) {
        if (sub < 4) qw[gid * 4 + sub] = mine | (other << 4);
        if (sub == 0) scales[gid] = __builtin_bit_cast(uint16_t, sh);
    }
}

}  // namespace nvq

extern "C" int nvq_pack_int4(const float *W, int64_t N, int64_t K, int group, uint8_t *qweight,
                             uint16_t *scales, void *stream) {
    if (!W || !qweight || !scales) return NVQ_ERR_INVALID_ARG;
    if (group != 32) return NVQ_ERR_UNSUPPORTED;
    if (N <= 0 || K <= 0 || (K % 32) != 0 || K > NVQ_MAX_K) return NVQ_ERR_SHAPE;
    if (!nvq::aligned(W, 16) || !nvq::aligned(qweight, 16) || !nvq::aligned(scales, 2))
        return NVQ_ERR_ALIGN;
    const int64_t groups = N * (K / 32);
    const int64_t blocks = (groups + 31) / 32;
    if (blocks > 0x7fffffffLL) return NVQ_ERR_SHAPE;
    hipLaunchKernelGGL(nvq::pack_int4_kernel, dim3((unsigned)blocks), dim3(256), 0,
                       (hipStream_t)stream, reinterpret_cast<const float4 *>(W), groups,
                       reinterpret_cast<uint32_t *>(qweight), scales);
    NVQ_HIP_TRY(hipGetLastError());
    return NVQ_OK;
}
