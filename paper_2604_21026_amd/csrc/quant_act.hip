// nvq_quant_act_i8: bf16 activations -> int8 codes, fp32 scale(s) and the
// per-32 code sums that the W4A8 GEMV's deferred correction needs.
// Paper, appendix "F16 -> Q8 Activation Quantization": s = amax / 127,
// q = round(x / s), clamp to [-127, 127].  Rounding is half-to-even and the
// division is IEEE binary32, so a CPU run of the same rule gives equal codes.
//
// One workgroup per token.  A thread handles chunks of 8 consecutive values
// (one 128-bit load); four neighbouring lanes therefore cover one group of 32
// and reduce its code sum (and, for per-group scales, its absmax) with two
// cross-lane exchanges.  Pass 1 finds the token's absmax, pass 2 re-reads the
// (cache-resident) row and quantises.
#include "nvq_internal.h"

namespace nvq {

constexpr int kQuantThreads = 256;

__device__ __forceinline__ float chunk_absmax(const uint4 &v) {
    const uint32_t w[4] = {v.x, v.y, v.z, v.w};
    float a = 0.0f;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        a = fmaxf(a, fabsf(bf16_bits_to_float(w[i] & 0xffffu)));
        a = fmaxf(a, fabsf(bf16_bits_to_float(w[i] >> 16)));
    }
    return a;
}

__device__ __forceinline__ int quant_one(float x, float s) {
    float r = rintf(x / s);
    r = fminf(fmaxf(r, -127.0f), 127.0f);
    return (int)r;
}

// Byte offset, in the operand image of the persistent small-batch kernel, of
// the 16-byte piece that holds input e (a multiple of 8) of token m: KiB blocks
// per (token tile, 128-input column, piece), 16 bytes per (kb, token) in them.
// PIECES = 2 for int8 codes (piece = a half of group kb of the column), 4 for
// bf16 (piece i = inputs 32 i .. 32 i + 31, split over kb by eights).
template <int PIECES>
__device__ __forceinline__ size_t image_offset(int K, int m, int e) {
    const int c = e >> 7, off = e & 127;
    const int kb = PIECES == 2 ? off >> 5 : (off & 31) >> 3;
    const int piece = PIECES == 2 ? (off & 31) >> 4 : off >> 5;
    const size_t block = ((size_t)(m >> 4) * (K >> 7) + c) * PIECES + piece;
    return block * 1024 + (size_t)(kb * 16 + (m & 15)) * 16 + (PIECES == 2 ? (off & 8) : 0);
}

// Token m of one [M][K] input, by one workgroup.  IMAGE: the codes go to the
// operand image `xq` instead of the [M][K] matrix, and no code sums are kept.
template <bool PER_GROUP, bool IMAGE = false>
__device__ __forceinline__ void quant_token(const uint4 *__restrict__ x, int K, int m,
                                            int8_t *__restrict__ xq, float *__restrict__ xscale,
                                            int32_t *__restrict__ xgsum) {
    const int chunks = K / 8;  // multiple of 4
    const int G = K / 32;
    const uint4 *xr = x + (int64_t)m * chunks;
    uint2 *qr = reinterpret_cast<uint2 *>(xq + (IMAGE ? 0 : (int64_t)m * K));
    int32_t *gs = IMAGE ? nullptr : xgsum + (int64_t)m * G;

    float s_tok = 0.0f;
    if (!PER_GROUP) {
        __shared__ float red[kQuantThreads / 64];
        float a = 0.0f;
        for (int c = threadIdx.x; c < chunks; c += kQuantThreads) a = fmaxf(a, chunk_absmax(xr[c]));
#pragma unroll
        for (int off = 32; off > 0; off >>= 1) a = fmaxf(a, __shfl_xor(a, off, 64));
        if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = a;
        __syncthreads();
        a = red[0];
#pragma unroll
        for (int i = 1; i < kQuantThreads / 64; ++i) a = fmaxf(a, red[i]);
        s_tok = a / 127.0f;
        if (threadIdx.x == 0) xscale[m] = s_tok;
    }

    // chunks is a multiple of 4 and the stride a multiple of 4, so the four
    // lanes of a team are valid or invalid together.
    for (int c = threadIdx.x; c < chunks; c += kQuantThreads) {
        const uint4 v = xr[c];
        float s = s_tok;
        if (PER_GROUP) {
            float a = chunk_absmax(v);
            a = fmaxf(a, __shfl_xor(a, 1, 64));
            a = fmaxf(a, __shfl_xor(a, 2, 64));
            s = a / 127.0f;
            if ((c & 3) == 0) xscale[(int64_t)m * G + (c >> 2)] = s;
        }
        const uint32_t w[4] = {v.x, v.y, v.z, v.w};
        int q[8];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            q[2 * i] = (s != 0.0f) ? quant_one(bf16_bits_to_float(w[i] & 0xffffu), s) : 0;
            q[2 * i + 1] = (s != 0.0f) ? quant_one(bf16_bits_to_float(w[i] >> 16), s) : 0;
        }
        int sum = 0;
#pragma unroll
        for (int i = 0; i < 8; ++i) sum += q[i];
        uint2 out;
        out.x = (uint32_t)(q[0] & 0xff) | ((uint32_t)(q[1] & 0xff) << 8) |
                ((uint32_t)(q[2] & 0xff) << 16) | ((uint32_t)(q[3] & 0xff) << 24);
        out.y = (uint32_t)(q[4] & 0xff) | ((uint32_t)(q[5] & 0xff) << 8) |
                ((uint32_t)(q[6] & 0xff) << 16) | ((uint32_t)(q[7] & 0xff) << 24);
        if (IMAGE) {
            *reinterpret_cast<uint2 *>(xq + image_offset<2>(K, m, 8 * c)) = out;
            continue;
        }
        qr[c] = out;
        sum += __shfl_xor(sum, 1, 64);
        sum += __shfl_xor(sum, 2, 64);
        if ((c & 3) == 0) gs[c >> 2] = sum;
    }
}

template <bool PER_GROUP>
__global__ __launch_bounds__(kQuantThreads) void quant_act_kernel(
    const uint4 *__restrict__ x, int K, int8_t *__restrict__ xq, float *__restrict__ xscale,
    int32_t *__restrict__ xgsum) {
    quant_token<PER_GROUP>(x, K, blockIdx.x, xq, xscale, xgsum);
}

// Per-token scales, the inputs of many phases in one grid.
__global__ __launch_bounds__(kQuantThreads) void quant_act_group_kernel(
    const GroupPhase *__restrict__ tab, const uint16_t *__restrict__ jobs, int M) {
    const int job = blockIdx.x / M, m = blockIdx.x - job * M;
    const GroupPhase &P = tab[jobs[job]];
    quant_token<false>(reinterpret_cast<const uint4 *>(P.x_bf16), P.G * 32, m, P.xq, P.xscale,
                       P.xgsum);
}

// Operand images of many phases in one grid: quantised codes (W4A8) or a
// rearranged copy of the bf16 inputs (W4A16).
__global__ __launch_bounds__(kQuantThreads) void operand_image_group_kernel(
    const GroupPhase *__restrict__ tab, const uint16_t *__restrict__ jobs, int M) {
    const int job = blockIdx.x / M, m = blockIdx.x - job * M;
    const GroupPhase &P = tab[jobs[job]];
    const int K = P.G * 32;
    const uint4 *x = reinterpret_cast<const uint4 *>(P.x_bf16);
    if (P.precision == NVQ_W4A8) {
        quant_token<false, true>(x, K, m, reinterpret_cast<int8_t *>(P.xa), P.xscale, nullptr);
    } else {
        const uint4 *xr = x + (int64_t)m * (K / 8);
        for (int c = threadIdx.x; c < K / 8; c += kQuantThreads)
            *reinterpret_cast<uint4 *>(P.xa + image_offset<4>(K, m, 8 * c)) = xr[c];
    }
}

int launch_quant_act_group(const GroupPhase *tab, const uint16_t *jobs, int njobs, int M,
                           bool image, hipStream_t st) {
    if (njobs <= 0) return NVQ_OK;
    if (image)
        hipLaunchKernelGGL(operand_image_group_kernel, dim3(njobs * M), dim3(kQuantThreads), 0, st,
                           tab, jobs, M);
    else
        hipLaunchKernelGGL(quant_act_group_kernel, dim3(njobs * M), dim3(kQuantThreads), 0, st,
                           tab, jobs, M);
    NVQ_HIP_TRY(hipGetLastError());
    return NVQ_OK;
}

int launch_quant_act(const uint16_t *x, int M, int K, int act_group, int8_t *xq, float *xscale,
                     int32_t *xgsum, hipStream_t st) {
    if (act_group == 0)
        hipLaunchKernelGGL(quant_act_kernel<false>, dim3(M), dim3(kQuantThreads), 0, st,
                           reinterpret_cast<const uint4 *>(x), K, xq, xscale, xgsum);
    else
        hipLaunchKernelGGL(quant_act_kernel<true>, dim3(M), dim3(kQuantThreads), 0, st,
                           reinterpret_cast<const uint4 *>(x), K, xq, xscale, xgsum);
    NVQ_HIP_TRY(hipGetLastError());
    return NVQ_OK;
}

}  // namespace nvq

extern "C" int nvq_quant_act_i8(const uint16_t *x_bf16, int M, int K, int act_group, int8_t *xq,
                                float *xscale, int32_t *xgsum, void *stream) {
    if (!x_bf16 || !xq || !xscale || !xgsum) return NVQ_ERR_INVALID_ARG;
    if (act_group != 0 && act_group != 32) return NVQ_ERR_INVALID_ARG;
    if (M <= 0 || M > NVQ_MAX_M || K <= 0 || (K % 32) != 0 || K > NVQ_MAX_K) return NVQ_ERR_SHAPE;
    if (!nvq::aligned(x_bf16, 16) || !nvq::aligned(xq, 16) || !nvq::aligned(xscale, 4) ||
        !nvq::aligned(xgsum, 4))
        return NVQ_ERR_ALIGN;
    return nvq::launch_quant_act(x_bf16, M, K, act_group, xq, xscale, xgsum, (hipStream_t)stream);
}
