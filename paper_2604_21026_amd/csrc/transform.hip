// nvq_rms_norm_bf16 / nvq_silu_mul_bf16: the two elementwise neighbours of the
// decode linears as kernels of their own (paper: kernel table, RMS-norm kernel
// "single-pass, shared memory" and SiLU-multiply kernel).  The persistent decode
// kernel applies the same arithmetic while it prepares a layer's input; these
// kernels serve the per-phase path and callers outside the walker.
//
// One workgroup per token, a lane handles eight consecutive values per step.
#include "transform.h"

namespace nvq {

constexpr int kTransformThreads = 256;

__global__ __launch_bounds__(kTransformThreads) void rms_norm_kernel(
    const uint4 *__restrict__ x, const uint4 *__restrict__ res, const uint4 *__restrict__ gamma,
    float eps, int K, uint4 *__restrict__ out, uint4 *__restrict__ h_out) {
    __shared__ float red[kTransformThreads / 64];
    const int m = blockIdx.x, chunks = K / 8;
    const uint4 *xr = x + (int64_t)m * chunks;
    const uint4 *rr = res ? res + (int64_t)m * chunks : nullptr;
    float ss = 0.0f;
    for (int c = threadIdx.x; c < chunks; c += kTransformThreads) {
        uint4 h = xr[c];
        if (rr) h = add_bf16x8(h, rr[c]);
        if (h_out) h_out[(int64_t)m * chunks + c] = h;
        ss += sumsq_bf16x8(h);
    }
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) ss += __shfl_xor(ss, off, 64);
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = ss;
    __syncthreads();
    ss = red[0];
#pragma unroll
    for (int i = 1; i < kTransformThreads / 64; ++i) ss += red[i];
    const float r = rms_scale(ss, K, eps);
    for (int c = threadIdx.x; c < chunks; c += kTransformThreads) {
        uint4 h = xr[c];
        if (rr) h = add_bf16x8(h, rr[c]);
        out[(int64_t)m * chunks + c] = scale_bf16x8(h, r, gamma[c]);
    }
}

__global__ __launch_bounds__(kTransformThreads) void silu_mul_kernel(const uint4 *__restrict__ g,
                                                                     const uint4 *__restrict__ u,
                                                                     int64_t chunks,
                                                                     uint4 *__restrict__ out) {
    const int64_t c = (int64_t)blockIdx.x * kTransformThreads + threadIdx.x;
    if (c < chunks) out[c] = silu_mul_bf16x8(g[c], u[c]);
}

int launch_rms_norm(const uint16_t *x, const uint16_t *res, const uint16_t *gamma, float eps, int M,
                    int K, uint16_t *out, uint16_t *h_out, hipStream_t st) {
    hipLaunchKernelGGL(rms_norm_kernel, dim3(M), dim3(kTransformThreads), 0, st,
                       reinterpret_cast<const uint4 *>(x), reinterpret_cast<const uint4 *>(res),
                       reinterpret_cast<const uint4 *>(gamma), eps, K,
                       reinterpret_cast<uint4 *>(out), reinterpret_cast<uint4 *>(h_out));
    NVQ_HIP_TRY(hipGetLastError());
    return NVQ_OK;
}

int launch_silu_mul(const uint16_t *g, const uint16_t *u, int M, int K, uint16_t *out,
                    hipStream_t st) {
    const int64_t chunks = (int64_t)M * K / 8;
    hipLaunchKernelGGL(silu_mul_kernel,
                       dim3((unsigned)((chunks + kTransformThreads - 1) / kTransformThreads)),
                       dim3(kTransformThreads), 0, st, reinterpret_cast<const uint4 *>(g),
                       reinterpret_cast<const uint4 *>(u), chunks, reinterpret_cast<uint4 *>(out));
    NVQ_HIP_TRY(hipGetLastError());
    return NVQ_OK;
}

}  // namespace nvq

extern "C" int nvq_rms_norm_bf16(const uint16_t *x, const uint16_t *res, const uint16_t *gamma,
                                 float eps, int M, int K, uint16_t *out, uint16_t *h_out,
                                 void *stream) {
    if (!x || !gamma || !out) return NVQ_ERR_INVALID_ARG;
    if (M <= 0 || M > NVQ_MAX_M || K <= 0 || (K % 32) != 0 || K > NVQ_MAX_K) return NVQ_ERR_SHAPE;
    if (!(eps >= 0.0f)) return NVQ_ERR_INVALID_ARG;
    if (!nvq::aligned(x, 16) || !nvq::aligned(res, 16) || !nvq::aligned(gamma, 16) ||
        !nvq::aligned(out, 16) || !nvq::aligned(h_out, 16))
        return NVQ_ERR_ALIGN;
    return nvq::launch_rms_norm(x, res, gamma, eps, M, K, out, h_out, (hipStream_t)stream);
}

extern "C" int nvq_silu_mul_bf16(const uint16_t *g, const uint16_t *u, int M, int K, uint16_t *out,
                                 void *stream) {
    if (!g || !u || !out) return NVQ_ERR_INVALID_ARG;
    if (M <= 0 || M > NVQ_MAX_M || K <= 0 || (K % 32) != 0 || K > NVQ_MAX_K) return NVQ_ERR_SHAPE;
    if (!nvq::aligned(g, 16) || !nvq::aligned(u, 16) || !nvq::aligned(out, 16))
        return NVQ_ERR_ALIGN;
    return nvq::launch_silu_mul(g, u, M, K, out, (hipStream_t)stream);
}
