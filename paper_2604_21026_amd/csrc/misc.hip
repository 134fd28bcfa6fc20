// Status strings, error bookkeeping, the routing-rule host helper and the two
// measurement kernels (streaming read, plain copy).
#include <stdio.h>
#include <string.h>

#include "nvq_internal.h"

namespace nvq {

static thread_local char g_hip_error[256] = "";

void set_hip_error(hipError_t e, const char *where) {
    snprintf(g_hip_error, sizeof g_hip_error, "%s: %s", where, hipGetErrorString(e));
}

int device_cu_count() {
    static int cached[64] = {0};
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return 256;
    if (cached[dev] == 0) {
        int cu = 0;
        if (hipDeviceGetAttribute(&cu, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess ||
            cu <= 0)
            cu = 256;
        cached[dev] = cu;
    }
    return cached[dev];
}

// Streaming read for the machine's HBM ceiling: one workgroup of 256 lanes per
// compute unit, every lane with six non-temporal 128-bit loads in flight (24 KiB
// per compute unit), grid-strided; it sums what it reads so that the loads
// cannot be dropped and adds one word per wave to *out.  Measured on an MI355X
// over 4 GiB: 7.43 TB/s.  More in flight is slower (two workgroups x 6 loads:
// 6.8, four x 8: 5.6 TB/s), fewer too (one x 4: 6.4); plain instead of
// non-temporal loads lose another 10 %.
constexpr int kReadUnroll = 6;
constexpr int kReadWgPerCu = 1;
typedef uint32_t read_u32x4 __attribute__((ext_vector_type(4)));
__global__ __launch_bounds__(256) void stream_read_kernel(const read_u32x4 *__restrict__ src,
                                                          size_t n16,
                                                          unsigned long long *__restrict__ out) {
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    uint32_t acc = 0;
    for (; i + (kReadUnroll - 1) * stride < n16; i += kReadUnroll * stride) {
        read_u32x4 v[kReadUnroll];
#pragma unroll
        for (int k = 0; k < kReadUnroll; ++k) v[k] = __builtin_nontemporal_load(src + i + k * stride);
#pragma unroll
        for (int k = 0; k < kReadUnroll; ++k) acc += v[k].x ^ v[k].y ^ v[k].z ^ v[k].w;
    }
    for (; i < n16; i += stride) {
        const read_u32x4 a = __builtin_nontemporal_load(src + i);
        acc += a.x ^ a.y ^ a.z ^ a.w;
    }
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) acc += __shfl_xor(acc, off, 64);
    if ((threadIdx.x & 63) == 0) atomicAdd(out, (unsigned long long)acc);
}

__global__ __launch_bounds__(256) void stream_copy_kernel(uint4 *__restrict__ dst,
                                                          const uint4 *__restrict__ src,
                                                          size_t n16) {
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n16; i += stride)
        dst[i] = src[i];
}

}  // namespace nvq

extern "C" const char *nvq_status_string(int status) {
    switch (status) {
        case NVQ_OK: return "ok";
        case NVQ_ERR_INVALID_ARG: return "invalid argument";
        case NVQ_ERR_SHAPE: return "unsupported shape";
        case NVQ_ERR_ALIGN: return "misaligned pointer";
        case NVQ_ERR_UNSUPPORTED: return "unsupported request";
        case NVQ_ERR_HIP: return "HIP runtime error";
        case NVQ_ERR_WORKSPACE: return "workspace missing, misaligned or too small";
        default: return "unknown status";
    }
}

extern "C" const char *nvq_last_hip_error(void) { return nvq::g_hip_error; }

extern "C" int nvq_precision_from_scores(const double *scores, int L, double tau, double eps,
                                         int32_t *out) {
    if (!scores || !out) return NVQ_ERR_INVALID_ARG;
    if (L <= 0) return NVQ_ERR_SHAPE;
    double lo = scores[0], hi = scores[0];
    for (int i = 1; i < L; ++i) {
        lo = scores[i] < lo ? scores[i] : lo;
        hi = scores[i] > hi ? scores[i] : hi;
    }
    const double range = hi - lo;
    for (int i = 0; i < L; ++i) {
        const double shat = range < eps ? 0.0 : (scores[i] - lo) / range;
        out[i] = shat >= tau ? NVQ_W4A16 : NVQ_W4A8;
    }
    return NVQ_OK;
}

extern "C" int nvq_stream_read(const void *src, size_t bytes, void *out, void *stream) {
    if (!src || !out) return NVQ_ERR_INVALID_ARG;
    if (bytes == 0 || bytes % 16) return NVQ_ERR_SHAPE;
    if (!nvq::aligned(src, 16) || !nvq::aligned(out, 8)) return NVQ_ERR_ALIGN;
    const int grid = nvq::device_cu_count() * nvq::kReadWgPerCu;
    hipLaunchKernelGGL(nvq::stream_read_kernel, dim3(grid), dim3(256), 0, (hipStream_t)stream,
                       reinterpret_cast<const nvq::read_u32x4 *>(src), bytes / 16,
                       reinterpret_cast<unsigned long long *>(out));
    NVQ_HIP_TRY(hipGetLastError());
    return NVQ_OK;
}

extern "C" int nvq_stream_copy(void *dst, const void *src, size_t bytes, void *stream) {
    if (!src || !dst) return NVQ_ERR_INVALID_ARG;
    if (bytes == 0 || bytes % 16) return NVQ_ERR_SHAPE;
    if (!nvq::aligned(src, 16) || !nvq::aligned(dst, 16)) return NVQ_ERR_ALIGN;
    const int grid = nvq::device_cu_count() * 8;
    hipLaunchKernelGGL(nvq::stream_copy_kernel, dim3(grid), dim3(256), 0, (hipStream_t)stream,
                       reinterpret_cast<uint4 *>(dst), reinterpret_cast<const uint4 *>(src),
                       bytes / 16);
    NVQ_HIP_TRY(hipGetLastError());
    return NVQ_OK;
}
