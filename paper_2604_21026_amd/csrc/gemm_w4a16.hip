// nvq_gemm_w4a16: the prefill / large-batch product.  Paper: kernel table (the
// weights are dequantised to 16-bit values, a dense GEMM follows) and the
// remark in the limitations that large batches are bound by compute.  Here the
// two are one kernel: Y[m][n] = sum_k X[m][k] * Wd[n][k] with Wd[n][k] =
// bf16(code[n][k] * scale[n][k/32]) (what nvq_dequant_bf16 stores), bf16 x bf16
// products accumulated in fp32 on the matrix cores; the dense weights never
// exist in memory, a wave dequantises the nibbles it is about to multiply.
//
// v_mfma_f32_32x32x16_bf16: operand A = 32 tokens x 16 inputs, operand B = 16
// inputs x 32 weight rows, lane (i, b) = (lane % 32, lane / 32) supplies eight
// inputs of token / row i.  Which eight is free as long as both operands agree:
// for step s of a quantisation group lane (i, b) takes inputs 16 s + 8 b ..
// + 7, that is 16 contiguous bytes of the activations and, of the group's 16
// packed bytes, the low (s = 0) or high (s = 1) nibbles of bytes 8 b .. 8 b + 7:
// one 8-byte load per lane, row and group.  Nibble -> fp32 (byte convert),
// one FMA with the group's scale ((n - 8) * s is exact), round to bf16.
//
// A workgroup of four waves owns 256 tokens x 128 weight rows, a wave 128 x 64
// (4 x 2 MFMA tiles, 128 accumulator registers); a wave's dequantised operand
// serves its four token tiles.  Activations pass through LDS (rows padded to
// 80 bytes: 16 lanes reading 16 bytes each then cover all 64 banks), double
// buffered, one barrier per group of 32 inputs; the next group's activations
// and packed weights are requested before the current group is multiplied.
#include "nvq_internal.h"

namespace nvq {

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef float floatx2 __attribute__((ext_vector_type(2)));

constexpr int kGemmTokens = 256;  // per workgroup
constexpr int kGemmRows = 128;
constexpr int kGemmThreads = 256;
constexpr int kXRowBytes = 80;  // 32 bf16 + 16 bytes of padding

__device__ __forceinline__ uint32_t pack_bf16(float a, float b) {
    const floatx2 f = {a, b};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(f, bf16x2));  // nearest even
}

// Eight weights of a lane: the nibbles of two dwords (already masked to
// 0x0f0f0f0f) times the scale, as bf16.  neg8s = -8 * s.
__device__ __forceinline__ bf16x8 dequant8(uint32_t n0, uint32_t n1, float s, float neg8s) {
    float w[8];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        w[i] = fmaf((float)((n0 >> (8 * i)) & 0xffu), s, neg8s);
        w[4 + i] = fmaf((float)((n1 >> (8 * i)) & 0xffu), s, neg8s);
    }
    const uint4 p = make_uint4(pack_bf16(w[0], w[1]), pack_bf16(w[2], w[3]), pack_bf16(w[4], w[5]),
                               pack_bf16(w[6], w[7]));
    return __builtin_bit_cast(bf16x8, p);
}

template <bool F32>
__global__ __launch_bounds__(kGemmThreads) void gemm_w4a16_kernel(
    const uint2 *__restrict__ qw, const uint16_t *__restrict__ sc, int N, int G,
    const uint4 *__restrict__ x, int M, void *__restrict__ y) {
    __shared__ __attribute__((aligned(16))) unsigned char xs[2][kGemmTokens * kXRowBytes];

    const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
    const int wm = wave >> 1, wn = wave & 1;
    const int li = lane & 31, lb = lane >> 5;
    const int m0 = blockIdx.y * kGemmTokens, n0 = blockIdx.x * kGemmRows;

    // staging: thread t copies the 64 bytes of token m0 + t (the last token
    // again past the end: those results are not stored)
    const int mt = m0 + t < M ? m0 + t : M - 1;
    const uint4 *xrow = x + (size_t)mt * (size_t)(G * 4);
    // the lane's weight rows, one per row tile (the last row again past the end)
    const uint2 *qrow[2];
    const uint16_t *srow[2];
#pragma unroll
    for (int rt = 0; rt < 2; ++rt) {
        const int n = n0 + wn * 64 + rt * 32 + li;
        const int nc = n < N ? n : N - 1;
        qrow[rt] = qw + (size_t)nc * (size_t)(G * 2) + lb;
        srow[rt] = sc + (size_t)nc * (size_t)G;
    }

    floatx16 acc[4][2];
#pragma unroll
    for (int tt = 0; tt < 4; ++tt)
#pragma unroll
        for (int rt = 0; rt < 2; ++rt)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[tt][rt][r] = 0.0f;

    // requests in flight: the activations of the group after next (in
    // registers until they are staged) and the packed weights of the next group
    uint4 xn0, xn1, xn2, xn3;
    uint2 wn0, wn1;
    uint16_t sn0, sn1;
#define NVQ_REQUEST_X(g_)          \
    do {                           \
        xn0 = xrow[4 * (g_)];      \
        xn1 = xrow[4 * (g_) + 1];  \
        xn2 = xrow[4 * (g_) + 2];  \
        xn3 = xrow[4 * (g_) + 3];  \
    } while (0)
#define NVQ_REQUEST_W(g_)          \
    do {                           \
        wn0 = qrow[0][2 * (g_)];   \
        wn1 = qrow[1][2 * (g_)];   \
        sn0 = srow[0][(g_)];       \
        sn1 = srow[1][(g_)];       \
    } while (0)
#define NVQ_STAGE_X(buf_)                                                            \
    do {                                                                             \
        uint4 *dst_ = reinterpret_cast<uint4 *>(&xs[(buf_)][t * kXRowBytes]);        \
        dst_[0] = xn0;                                                               \
        dst_[1] = xn1;                                                               \
        dst_[2] = xn2;                                                               \
        dst_[3] = xn3;                                                               \
    } while (0)

    NVQ_REQUEST_X(0);
    NVQ_REQUEST_W(0);
    NVQ_STAGE_X(0);
    if (G > 1) NVQ_REQUEST_X(1);
    __syncthreads();

    for (int g = 0; g < G; ++g) {
        const int cur = g & 1;
        const uint2 wcur[2] = {wn0, wn1};
        const float s0 = half_bits_to_float(sn0), s1 = half_bits_to_float(sn1);
        if (g + 1 < G) NVQ_REQUEST_W(g + 1);

        // operand B: [row tile][step]
        bf16x8 b[2][2];
        {
            const float sv[2] = {s0, s1};
#pragma unroll
            for (int rt = 0; rt < 2; ++rt) {
                const float neg8s = -8.0f * sv[rt];
                b[rt][0] = dequant8(wcur[rt].x & 0x0f0f0f0fu, wcur[rt].y & 0x0f0f0f0fu, sv[rt], neg8s);
                b[rt][1] = dequant8((wcur[rt].x >> 4) & 0x0f0f0f0fu, (wcur[rt].y >> 4) & 0x0f0f0f0fu,
                                    sv[rt], neg8s);
            }
        }
#pragma unroll
        for (int tt = 0; tt < 4; ++tt) {
            const unsigned char *row = &xs[cur][(wm * 128 + tt * 32 + li) * kXRowBytes + 16 * lb];
            const bf16x8 a0 = __builtin_bit_cast(bf16x8, *reinterpret_cast<const uint4 *>(row));
            const bf16x8 a1 = __builtin_bit_cast(bf16x8, *reinterpret_cast<const uint4 *>(row + 32));
#pragma unroll
            for (int rt = 0; rt < 2; ++rt) {
                acc[tt][rt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a0, b[rt][0], acc[tt][rt], 0, 0, 0);
                acc[tt][rt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a1, b[rt][1], acc[tt][rt], 0, 0, 0);
            }
        }
        if (g + 1 < G) {
            NVQ_STAGE_X(cur ^ 1);  // everyone left this buffer before the last barrier
            if (g + 2 < G) NVQ_REQUEST_X(g + 2);
        }
        __syncthreads();
    }

#undef NVQ_REQUEST_X
#undef NVQ_REQUEST_W
#undef NVQ_STAGE_X

    // result tile: lane (j, b) holds weight row j; register r holds token
    // 8 * (r / 4) + 4 * b + r % 4
#pragma unroll
    for (int tt = 0; tt < 4; ++tt)
#pragma unroll
        for (int rt = 0; rt < 2; ++rt) {
            const int n = n0 + wn * 64 + rt * 32 + li;
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int m = m0 + wm * 128 + tt * 32 + 8 * (r >> 2) + 4 * lb + (r & 3);
                if (m < M && n < N) {
                    if (F32)
                        reinterpret_cast<float *>(y)[(size_t)m * N + n] = acc[tt][rt][r];
                    else
                        reinterpret_cast<uint16_t *>(y)[(size_t)m * N + n] =
                            float_to_bf16_bits(acc[tt][rt][r]);
                }
            }
        }
}

}  // namespace

}  // namespace nvq

extern "C" int nvq_gemm_w4a16(const uint8_t *qweight, const uint16_t *scales, int64_t N, int64_t K,
                              const uint16_t *x_bf16, int64_t M, void *y, int y_dtype,
                              void *stream) {
    using namespace nvq;
    if (!qweight || !scales || !x_bf16 || !y) return NVQ_ERR_INVALID_ARG;
    if (y_dtype != NVQ_F32 && y_dtype != NVQ_BF16) return NVQ_ERR_INVALID_ARG;
    if (N <= 0 || M <= 0 || K <= 0 || (K % 32) != 0 || K > NVQ_MAX_K || N > (1 << 24) ||
        M > (1 << 24))
        return NVQ_ERR_SHAPE;
    if (!aligned(qweight, 16) || !aligned(scales, 2) || !aligned(x_bf16, 16) ||
        !aligned(y, y_dtype == NVQ_F32 ? 4 : 2))
        return NVQ_ERR_ALIGN;
    const dim3 grid((unsigned)((N + kGemmRows - 1) / kGemmRows),
                    (unsigned)((M + kGemmTokens - 1) / kGemmTokens)),
        block(kGemmThreads);
    if (grid.y > 65535u) return NVQ_ERR_SHAPE;
    const uint2 *qw = reinterpret_cast<const uint2 *>(qweight);
    const uint4 *x = reinterpret_cast<const uint4 *>(x_bf16);
    if (y_dtype == NVQ_F32)
        hipLaunchKernelGGL(gemm_w4a16_kernel<true>, grid, block, 0, (hipStream_t)stream, qw, scales,
                           (int)N, (int)(K / 32), x, (int)M, y);
    else
        hipLaunchKernelGGL(gemm_w4a16_kernel<false>, grid, block, 0, (hipStream_t)stream, qw, scales,
                           (int)N, (int)(K / 32), x, (int)M, y);
    NVQ_HIP_TRY(hipGetLastError());
    return NVQ_OK;
}
