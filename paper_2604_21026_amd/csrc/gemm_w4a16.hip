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
// inputs of token / row i.  Which eight is free as long as both operands agree,
// and since the scale is folded into the bf16 weight an MFMA may mix two
// quantisation groups: the kernel advances by pairs of groups (64 inputs), lane
// (i, b) takes its eight inputs from group 2 p + b of pair p, inputs 8 s .. 8 s
// + 7 of that group in MFMA step s = 0..3.  For the activations that is 16
// contiguous bytes; for the weights the lane loads the group's 16 packed bytes
// once (adjacent to the other lane's group: 32 contiguous bytes per row) and
// step s uses the low (s < 2) or high nibbles of bytes 8 (s % 2) .. + 7.
// Nibble -> fp32 (byte convert), one FMA with the group's scale ((n - 8) * s is
// exact), round to bf16.
//
// A workgroup of four waves owns 256 tokens x 128 weight rows, a wave 128 x 64
// (4 x 2 MFMA tiles, 128 accumulator registers); a wave's dequantised operand
// serves its four token tiles.  Activations pass through LDS (rows of 128 bytes
// padded to 144: 16 lanes reading 16 bytes each then cover all 64 banks),
// double buffered, eight neighbouring threads staging a token's 128 bytes; one
// barrier per pair of groups.  The next pair's activations and packed weights
// are requested before the current pair is multiplied.
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
constexpr int kXRowBytes = 144;  // 64 bf16 + 16 bytes of padding

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
    const uint4 *__restrict__ qw, const uint16_t *__restrict__ sc, int N, int G,
    const uint4 *__restrict__ x, int M, void *__restrict__ y) {
    __shared__ __attribute__((aligned(16))) unsigned char xs[2][kGemmTokens * kXRowBytes];

    const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
    const int wm = wave >> 1, wn = wave & 1;
    const int li = lane & 31, lb = lane >> 5;
    const int m0 = blockIdx.y * kGemmTokens, n0 = blockIdx.x * kGemmRows;
    const int P = (G + 1) >> 1;  // pairs of groups

    // Staging: eight neighbouring threads copy the 128 bytes of a token and
    // pair (one cache line), thread t those of tokens m0 + t / 8 + 32 i (the
    // last token again past the end: those results are not stored).
    const uint4 *xrow[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        const int m = m0 + (t >> 3) + 32 * i;
        xrow[i] = x + (size_t)(m < M ? m : M - 1) * (size_t)(G * 4);
    }
    // The lane's weight rows, one per row tile (the last row again past the end).
    const uint4 *qrow[2];
    const uint16_t *srow[2];
#pragma unroll
    for (int rt = 0; rt < 2; ++rt) {
        const int n = n0 + wn * 64 + rt * 32 + li;
        const int nc = n < N ? n : N - 1;
        qrow[rt] = qw + (size_t)nc * (size_t)G;
        srow[rt] = sc + (size_t)nc * (size_t)G;
    }

    floatx16 acc[4][2];
#pragma unroll
    for (int tt = 0; tt < 4; ++tt)
#pragma unroll
        for (int rt = 0; rt < 2; ++rt)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[tt][rt][r] = 0.0f;

    // In flight between pairs: the activations and the packed weights of the
    // next pair.  An odd number of groups: the missing group of the last pair is
    // the last group again, with scale 0 (all its weights 0).
    uint4 xn0, xn1, xn2, xn3, xn4, xn5, xn6, xn7, wn0, wn1;
    uint32_t hn0, hn1;
#define NVQ_REQUEST(p_)                                                              \
    do {                                                                             \
        {                                                                            \
            const int gx_ = 2 * (p_) + ((t >> 2) & 1);                               \
            const int cx_ = 4 * (gx_ < G ? gx_ : G - 1) + (t & 3);                   \
            xn0 = xrow[0][cx_];                                                      \
            xn1 = xrow[1][cx_];                                                      \
            xn2 = xrow[2][cx_];                                                      \
            xn3 = xrow[3][cx_];                                                      \
            xn4 = xrow[4][cx_];                                                      \
            xn5 = xrow[5][cx_];                                                      \
            xn6 = xrow[6][cx_];                                                      \
            xn7 = xrow[7][cx_];                                                      \
        }                                                                            \
        const int gw_ = 2 * (p_) + lb;                                               \
        const int gc_ = gw_ < G ? gw_ : G - 1;                                       \
        wn0 = qrow[0][gc_];                                                          \
        wn1 = qrow[1][gc_];                                                          \
        hn0 = gw_ < G ? (uint32_t)srow[0][gc_] : 0u;                                 \
        hn1 = gw_ < G ? (uint32_t)srow[1][gc_] : 0u;                                 \
    } while (0)
#define NVQ_STAGE_X(buf_)                                                            \
    do {                                                                             \
        unsigned char *dst_ = &xs[(buf_)][(t >> 3) * kXRowBytes + 16 * (t & 7)];     \
        *reinterpret_cast<uint4 *>(dst_) = xn0;                                      \
        *reinterpret_cast<uint4 *>(dst_ + 32 * kXRowBytes) = xn1;                    \
        *reinterpret_cast<uint4 *>(dst_ + 64 * kXRowBytes) = xn2;                    \
        *reinterpret_cast<uint4 *>(dst_ + 96 * kXRowBytes) = xn3;                    \
        *reinterpret_cast<uint4 *>(dst_ + 128 * kXRowBytes) = xn4;                   \
        *reinterpret_cast<uint4 *>(dst_ + 160 * kXRowBytes) = xn5;                   \
        *reinterpret_cast<uint4 *>(dst_ + 192 * kXRowBytes) = xn6;                   \
        *reinterpret_cast<uint4 *>(dst_ + 224 * kXRowBytes) = xn7;                   \
    } while (0)

    NVQ_REQUEST(0);
    NVQ_STAGE_X(0);
    uint4 wc0 = wn0, wc1 = wn1;
    uint32_t hc0 = hn0, hc1 = hn1;
    NVQ_REQUEST((P > 1 ? 1 : 0));
    __syncthreads();

    for (int p = 0; p < P; ++p) {
        const int cur = p & 1;
        // next pair: stage what was requested during the pair before, ask for the one after
        const uint4 wnext0 = wn0, wnext1 = wn1;
        const uint32_t hnext0 = hn0, hnext1 = hn1;
        NVQ_STAGE_X(cur ^ 1);  // everyone left this buffer before the last barrier
        {
            const int p2 = p + 2 < P ? p + 2 : P - 1;
            NVQ_REQUEST(p2);
        }
        const uint4 wc[2] = {wc0, wc1};
        const float sv[2] = {half_bits_to_float((uint16_t)hc0), half_bits_to_float((uint16_t)hc1)};
        const float m8[2] = {-8.0f * sv[0], -8.0f * sv[1]};
#pragma unroll
        for (int st = 0; st < 4; ++st) {
            bf16x8 b[2];
#pragma unroll
            for (int rt = 0; rt < 2; ++rt) {
                const uint32_t d0 = (st & 1) ? wc[rt].z : wc[rt].x, d1 = (st & 1) ? wc[rt].w : wc[rt].y;
                b[rt] = (st < 2) ? dequant8(d0 & 0x0f0f0f0fu, d1 & 0x0f0f0f0fu, sv[rt], m8[rt])
                                 : dequant8((d0 >> 4) & 0x0f0f0f0fu, (d1 >> 4) & 0x0f0f0f0fu, sv[rt],
                                            m8[rt]);
            }
#pragma unroll
            for (int tt = 0; tt < 4; ++tt) {
                const unsigned char *row =
                    &xs[cur][(wm * 128 + tt * 32 + li) * kXRowBytes + 64 * lb + 16 * st];
                const bf16x8 a = __builtin_bit_cast(bf16x8, *reinterpret_cast<const uint4 *>(row));
#pragma unroll
                for (int rt = 0; rt < 2; ++rt)
                    acc[tt][rt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b[rt], acc[tt][rt], 0, 0, 0);
            }
        }
        wc0 = wnext0;
        wc1 = wnext1;
        hc0 = hnext0;
        hc1 = hnext1;
        __syncthreads();
    }

#undef NVQ_REQUEST
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
    const uint4 *qw = reinterpret_cast<const uint4 *>(qweight);
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
