// The calibration statistics of the paper's Algorithm 1 (Monte Carlo activation
// profiling): per layer and token two magnitudes, Euclidean norms of output
// vectors of the layer's linears (query and value projections side by side;
// the feed-forward block's output), averaged into one score per layer, which
// nvq_precision_from_scores turns into the precision map.  Not on the decode
// path: it runs once per model, over a few calibration prompts.
#include "nvq_internal.h"

namespace nvq {

namespace {

constexpr int kNormThreads = 256;

template <typename T>
__device__ __forceinline__ float load_value(const T *p, int64_t i);
template <>
__device__ __forceinline__ float load_value<float>(const float *p, int64_t i) {
    return p[i];
}
template <>
__device__ __forceinline__ float load_value<uint16_t>(const uint16_t *p, int64_t i) {
    return bf16_bits_to_float(p[i]);
}

// One workgroup per token: the sum of squares of its row of a and of b.
template <typename T>
__global__ __launch_bounds__(kNormThreads) void token_norms_kernel(
    const T *__restrict__ a, int Na, const T *__restrict__ b, int Nb, float *__restrict__ out) {
    __shared__ float red[kNormThreads / 64];
    const int64_t m = blockIdx.x;
    float sum = 0.0f;
    for (int n = threadIdx.x; n < Na; n += kNormThreads) {
        const float v = load_value(a, m * Na + n);
        sum = fmaf(v, v, sum);
    }
    for (int n = threadIdx.x; n < Nb; n += kNormThreads) {
        const float v = load_value(b, m * Nb + n);
        sum = fmaf(v, v, sum);
    }
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) sum += __shfl_xor(sum, off, 64);
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = sum;
    __syncthreads();
    if (threadIdx.x == 0) {
        float total = red[0];
#pragma unroll
        for (int i = 1; i < kNormThreads / 64; ++i) total += red[i];
        out[m] = sqrtf(total);
    }
}

}  // namespace

}  // namespace nvq

extern "C" int nvq_token_norms(const void *a, int Na, const void *b, int Nb, int M, int dtype,
                               float *out, void *stream) {
    using namespace nvq;
    if (!a || !out || (Nb > 0 && !b)) return NVQ_ERR_INVALID_ARG;
    if (dtype != NVQ_F32 && dtype != NVQ_BF16) return NVQ_ERR_INVALID_ARG;
    if (Na <= 0 || Nb < 0 || M <= 0) return NVQ_ERR_SHAPE;
    const size_t al = dtype == NVQ_F32 ? 4 : 2;
    if (!aligned(a, al) || (Nb > 0 && !aligned(b, al)) || !aligned(out, 4)) return NVQ_ERR_ALIGN;
    const hipStream_t st = (hipStream_t)stream;
    if (dtype == NVQ_F32)
        hipLaunchKernelGGL(token_norms_kernel<float>, dim3(M), dim3(kNormThreads), 0, st,
                           reinterpret_cast<const float *>(a), Na,
                           reinterpret_cast<const float *>(b), Nb, out);
    else
        hipLaunchKernelGGL(token_norms_kernel<uint16_t>, dim3(M), dim3(kNormThreads), 0, st,
                           reinterpret_cast<const uint16_t *>(a), Na,
                           reinterpret_cast<const uint16_t *>(b), Nb, out);
    NVQ_HIP_TRY(hipGetLastError());
    return NVQ_OK;
}

extern "C" int nvq_mcap_scores(const float *a_attn, const float *a_ffn, const int *prompt_len, int k,
                               int L, double *scores) {
    if (!a_attn || !a_ffn || !prompt_len || !scores) return NVQ_ERR_INVALID_ARG;
    if (k <= 0 || L <= 0) return NVQ_ERR_SHAPE;
    int64_t T = 0;
    for (int j = 0; j < k; ++j) {
        if (prompt_len[j] <= 0) return NVQ_ERR_SHAPE;
        T += prompt_len[j];
    }
    for (int i = 0; i < L; ++i) {
        const float *aa = a_attn + (int64_t)i * T, *af = a_ffn + (int64_t)i * T;
        double mean_of_means = 0.0;
        int64_t t0 = 0;
        for (int j = 0; j < k; ++j) {
            double sum = 0.0;
            for (int64_t t = t0; t < t0 + prompt_len[j]; ++t) sum += (double)aa[t] + (double)af[t];
            mean_of_means += sum / prompt_len[j];
            t0 += prompt_len[j];
        }
        scores[i] = mean_of_means / k;
    }
    return NVQ_OK;
}
