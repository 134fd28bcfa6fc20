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

// Token m of one [M][K] input, by one workgroup.
template <bool PER_GROUP>
__device__ __forceinline__ void quant_token(const uint4 *__restrict__ x, int K, int m,
                                            int8_t *__restrict__ xq, float *__restrict__ xscale,
                                            int32_t *__restrict__ xgsum) {
    const int chunks = K / 8;  // multiple of 4
    const int G = K / 32;
    const uint4 *xr = x + (int64_t)m * chunks;
    uint2 *qr = reinterpret_cast<uint2 *>(xq + (int64_t)m * K);
    int32_t *gs = xgsum + (int64_t)m * G;

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

// ---- operand images of the persistent small-batch kernel ---------------------
// Per tile of 16 tokens, 128-input column c and piece i one KiB whose 16 bytes
// number 16 * kb + n are, for token n of the tile, the int8 codes 32 * kb +
// 16 * i .. + 15 of the column (W4A8, two pieces) or the bf16 inputs 32 * i +
// 8 * kb .. + 7 of the column (W4A16, four pieces): the order in which a wave
// of the matrix-core kernel loads its activation operands.  Two grids: the
// per-token scales of the W4A8 phases first, then the images, a wave writing
// whole KiB pieces (one workgroup per token, as for the [M][K] codes, would
// write 8 or 16 bytes here and there into lines shared with 15 other
// workgroups).

// Per-token scale of token m of every W4A8 job (the other jobs' workgroups leave).
__global__ __launch_bounds__(kQuantThreads) void token_scale_group_kernel(
    const GroupPhase *__restrict__ tab, const uint16_t *__restrict__ jobs, int M) {
    const int job = blockIdx.x / M, m = blockIdx.x - job * M;
    const GroupPhase &P = tab[jobs[job]];
    if (P.precision != NVQ_W4A8) return;
    __shared__ float red[kQuantThreads / 64];
    const int chunks = P.G * 4;
    const uint4 *xr = reinterpret_cast<const uint4 *>(P.x_bf16) + (int64_t)m * chunks;
    float a = 0.0f;
    for (int c = threadIdx.x; c < chunks; c += kQuantThreads) a = fmaxf(a, chunk_absmax(xr[c]));
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) a = fmaxf(a, __shfl_xor(a, off, 64));
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = a;
    __syncthreads();
    if (threadIdx.x == 0) {
        a = red[0];
#pragma unroll
        for (int i = 1; i < kQuantThreads / 64; ++i) a = fmaxf(a, red[i]);
        P.xscale[m] = a / 127.0f;
    }
}

constexpr int kImageColumns = 8;  // columns of 128 inputs per workgroup (two per wave)

__device__ __forceinline__ uint32_t quant_pack4(uint32_t w0, uint32_t w1, float s) {
    const int q0 = (s != 0.0f) ? quant_one(bf16_bits_to_float(w0 & 0xffffu), s) : 0;
    const int q1 = (s != 0.0f) ? quant_one(bf16_bits_to_float(w0 >> 16), s) : 0;
    const int q2 = (s != 0.0f) ? quant_one(bf16_bits_to_float(w1 & 0xffffu), s) : 0;
    const int q3 = (s != 0.0f) ? quant_one(bf16_bits_to_float(w1 >> 16), s) : 0;
    return (uint32_t)(q0 & 0xff) | ((uint32_t)(q1 & 0xff) << 8) | ((uint32_t)(q2 & 0xff) << 16) |
           ((uint32_t)(q3 & 0xff) << 24);
}

// img_units[u] names the phase of grid unit u; a unit is a token tile times
// kImageColumns columns of that phase.  Token slots past M are left as they are.
__global__ __launch_bounds__(kQuantThreads) void operand_image_group_kernel(
    const GroupPhase *__restrict__ tab, const uint16_t *__restrict__ img_units, int M) {
    const GroupPhase &P = tab[img_units[blockIdx.x]];
    const int local = blockIdx.x - P.img_begin;
    const int C4 = P.G >> 2, cblocks = (C4 + kImageColumns - 1) / kImageColumns;
    const int mt = local / cblocks, cb = local - mt * cblocks;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int n = lane & 15, kb = lane >> 4;
    const int m = mt * 16 + n;
    if (m >= M) return;
    const uint16_t *xr = P.x_bf16 + (int64_t)m * (P.G * 32);
    if (P.precision == NVQ_W4A8) {
        const float s = P.xscale[m];
        for (int c = cb * kImageColumns + wave; c < C4 && c < (cb + 1) * kImageColumns; c += 4) {
#pragma unroll
            for (int i = 0; i < 2; ++i) {
                const uint4 *src = reinterpret_cast<const uint4 *>(xr + c * 128 + 32 * kb + 16 * i);
                const uint4 v0 = src[0], v1 = src[1];
                const uint4 out = make_uint4(quant_pack4(v0.x, v0.y, s), quant_pack4(v0.z, v0.w, s),
                                             quant_pack4(v1.x, v1.y, s), quant_pack4(v1.z, v1.w, s));
                *reinterpret_cast<uint4 *>(P.xa + ((size_t)(mt * C4 + c) * 2 + i) * 1024 +
                                           lane * 16) = out;
            }
        }
    } else {
        for (int c = cb * kImageColumns + wave; c < C4 && c < (cb + 1) * kImageColumns; c += 4) {
#pragma unroll
            for (int i = 0; i < 4; ++i)
                *reinterpret_cast<uint4 *>(P.xa + ((size_t)(mt * C4 + c) * 4 + i) * 1024 +
                                           lane * 16) =
                    *reinterpret_cast<const uint4 *>(xr + c * 128 + 32 * i + 8 * kb);
        }
    }
}

int image_units(int M, int K) { return ((M + 15) / 16) * ((K / 128 + kImageColumns - 1) / kImageColumns); }

int launch_operand_images(const GroupPhase *tab, const uint16_t *jobs, int njobs,
                          const uint16_t *img_units, int nimg, int M, hipStream_t st) {
    if (njobs <= 0 || nimg <= 0) return NVQ_OK;
    hipLaunchKernelGGL(token_scale_group_kernel, dim3(njobs * M), dim3(kQuantThreads), 0, st, tab,
                       jobs, M);
    NVQ_HIP_TRY(hipGetLastError());
    hipLaunchKernelGGL(operand_image_group_kernel, dim3(nimg), dim3(kQuantThreads), 0, st, tab,
                       img_units, M);
    NVQ_HIP_TRY(hipGetLastError());
    return NVQ_OK;
}

int launch_quant_act_group(const GroupPhase *tab, const uint16_t *jobs, int njobs, int M,
                           hipStream_t st) {
    if (njobs <= 0) return NVQ_OK;
    hipLaunchKernelGGL(quant_act_group_kernel, dim3(njobs * M), dim3(kQuantThreads), 0, st, tab, jobs,
                       M);
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
