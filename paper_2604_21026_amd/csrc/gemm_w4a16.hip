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
// serves its four token tiles.  Activations and packed weights pass through
// LDS (rows padded to 80 bytes: 16 lanes reading 16 bytes each then cover all
// 64 banks), both double buffered, the activations group by group, the weights
// four groups at a time (64 contiguous bytes per row and load).  A wave holds
// the operands of the group it multiplies in registers and, while the matrix
// core works, reads the next group's activations from LDS and dequantises the
// next group's weights; memory is asked for a group's activations three groups
// ahead.  One barrier per group of 32 inputs.
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
constexpr int kWRowBytes = 80;  // four groups of 16 packed bytes + 16 bytes of padding

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
    const uint4 *__restrict__ x, int M, void *__restrict__ y, int scales_by_four) {
    __shared__ __attribute__((aligned(16))) unsigned char xs[2][kGemmTokens * kXRowBytes];
    __shared__ __attribute__((aligned(16))) unsigned char wq[2][kGemmRows * kWRowBytes];
    __shared__ __attribute__((aligned(8))) uint16_t ws[2][kGemmRows][4];

    const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
    const int wm = wave >> 1, wn = wave & 1;
    const int li = lane & 31, lb = lane >> 5;
    const int m0 = blockIdx.y * kGemmTokens, n0 = blockIdx.x * kGemmRows;

    // Staging, activations: four neighbouring threads copy the 64 bytes of a
    // token and group (one request to the cache per token and load), thread t
    // those of tokens m0 + t / 4 + 64 i (the last token again past the end: those
    // results are not stored).
    const uint4 *xrow[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int m = m0 + (t >> 2) + 64 * i;
        xrow[i] = x + (size_t)(m < M ? m : M - 1) * (size_t)(G * 4) + (t & 3);
    }
    // Staging, weights: four groups (128 inputs) at a time, so that four
    // neighbouring threads copy 64 contiguous bytes of a row (a load per lane,
    // row and group asks the cache for a line per 8 bytes and was what bound the
    // kernel); thread t the 16 bytes of group 4 j + t % 4 of rows t / 4 and
    // t / 4 + 64, and thread t < 128 the four scales of row t.
    const uint4 *wrow[2];
#pragma unroll
    for (int i = 0; i < 2; ++i) {
        const int n = n0 + (t >> 2) + 64 * i;
        wrow[i] = qw + (size_t)(n < N ? n : N - 1) * (size_t)G;
    }
    const int ns = n0 + (t & 127);
    const uint16_t *srow = sc + (size_t)(ns < N ? ns : N - 1) * (size_t)G;

    floatx16 acc[4][2];
#pragma unroll
    for (int tt = 0; tt < 4; ++tt)
#pragma unroll
        for (int rt = 0; rt < 2; ++rt)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[tt][rt][r] = 0.0f;

    // In flight: the activations of the group after next and the weights of the
    // four groups after the next four, in registers until they are staged.
    uint4 xn0, xn1, xn2, xn3, wq0, wq1;
    uint2 wsc;
#define NVQ_REQUEST_X(g_)          \
    do {                           \
        xn0 = xrow[0][4 * (g_)];   \
        xn1 = xrow[1][4 * (g_)];   \
        xn2 = xrow[2][4 * (g_)];   \
        xn3 = xrow[3][4 * (g_)];   \
    } while (0)
#define NVQ_STAGE_X(buf_)                                                            \
    do {                                                                             \
        unsigned char *dst_ = &xs[(buf_)][(t >> 2) * kXRowBytes + 16 * (t & 3)];     \
        *reinterpret_cast<uint4 *>(dst_) = xn0;                                      \
        *reinterpret_cast<uint4 *>(dst_ + 64 * kXRowBytes) = xn1;                    \
        *reinterpret_cast<uint4 *>(dst_ + 128 * kXRowBytes) = xn2;                   \
        *reinterpret_cast<uint4 *>(dst_ + 192 * kXRowBytes) = xn3;                   \
    } while (0)
    // groups past the end are clamped to the last one (their products are not formed)
#define NVQ_REQUEST_W(j_)                                                            \
    do {                                                                             \
        const int gq_ = 4 * (j_) + (t & 3) < G ? 4 * (j_) + (t & 3) : G - 1;         \
        wq0 = wrow[0][gq_];                                                          \
        wq1 = wrow[1][gq_];                                                          \
        if (t < 128) {                                                               \
            if (scales_by_four) {                                                    \
                const int gs_ = 4 * (j_) < G ? 4 * (j_) : G - 4;                     \
                wsc = *reinterpret_cast<const uint2 *>(srow + gs_);                  \
            } else {                                                                 \
                uint32_t h_[4];                                                      \
                _Pragma("unroll") for (int i_ = 0; i_ < 4; ++i_)                     \
                    h_[i_] = srow[4 * (j_) + i_ < G ? 4 * (j_) + i_ : G - 1];        \
                wsc = make_uint2(h_[0] | (h_[1] << 16), h_[2] | (h_[3] << 16));      \
            }                                                                        \
        }                                                                            \
    } while (0)
#define NVQ_STAGE_W(buf_)                                                            \
    do {                                                                             \
        unsigned char *dst_ = &wq[(buf_)][(t >> 2) * kWRowBytes + 16 * (t & 3)];     \
        *reinterpret_cast<uint4 *>(dst_) = wq0;                                      \
        *reinterpret_cast<uint4 *>(dst_ + 64 * kWRowBytes) = wq1;                    \
        if (t < 128) *reinterpret_cast<uint2 *>(&ws[(buf_)][t][0]) = wsc;            \
    } while (0)
    // operand A of one group: [token tile][step], from LDS buffer buf_
#define NVQ_READ_A(a_, buf_)                                                                       \
    do {                                                                                           \
        _Pragma("unroll") for (int tt = 0; tt < 4; ++tt) {                                         \
            const unsigned char *row_ =                                                            \
                &xs[(buf_)][(wm * 128 + tt * 32 + li) * kXRowBytes + 16 * lb];                     \
            a_[tt][0] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const uint4 *>(row_));        \
            a_[tt][1] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const uint4 *>(row_ + 32));   \
        }                                                                                          \
    } while (0)
    // operand B of group g_: [row tile][step], from the staged words and scales
#define NVQ_DEQUANT(b_, g_)                                                                        \
    do {                                                                                           \
        const int wb_ = ((g_) >> 2) & 1, gi_ = (g_) & 3;                                           \
        _Pragma("unroll") for (int rt = 0; rt < 2; ++rt) {                                         \
            const int r_ = wn * 64 + rt * 32 + li;                                                 \
            const uint2 w_ =                                                                       \
                *reinterpret_cast<const uint2 *>(&wq[wb_][r_ * kWRowBytes + 16 * gi_ + 8 * lb]);   \
            const float s_ = half_bits_to_float(ws[wb_][r_][gi_]);                                 \
            const float m_ = -8.0f * s_;                                                           \
            b_[rt][0] = dequant8(w_.x & 0x0f0f0f0fu, w_.y & 0x0f0f0f0fu, s_, m_);                  \
            b_[rt][1] = dequant8((w_.x >> 4) & 0x0f0f0f0fu, (w_.y >> 4) & 0x0f0f0f0fu, s_, m_);    \
        }                                                                                          \
    } while (0)

    // One group of 32 inputs.  The MFMAs of group g take their operands from
    // registers (ac_, bc_); while the matrix core works, the wave fetches the
    // activations of group g + 1 from LDS (an_) and dequantises its weights
    // (bn_).  Before that the activations of group g + 2 go to the LDS buffer
    // that group g's were read from during the group before (buffer g % 2 holds
    // group g) and memory is asked for group g + 3; every fourth group the
    // weights of the next four groups are staged the same way (buffer
    // (g / 4) % 2; group g + 1's were staged at least one group ago).
#define NVQ_GROUP(g_, ac_, bc_, an_, bn_)                                                          \
    do {                                                                                           \
        const int cur_ = (g_) & 1;                                                                 \
        NVQ_STAGE_X(cur_);                                                                         \
        {                                                                                          \
            const int g3_ = (g_) + 3 < G ? (g_) + 3 : G - 1;                                       \
            NVQ_REQUEST_X(g3_);                                                                    \
        }                                                                                          \
        if (((g_) & 3) == 0) {                                                                     \
            NVQ_STAGE_W((((g_) >> 2) + 1) & 1);                                                    \
            NVQ_REQUEST_W(((g_) >> 2) + 2);                                                        \
        }                                                                                          \
        /* the two MFMAs into one accumulator are eight MFMAs apart */                            \
        _Pragma("unroll") for (int st = 0; st < 2; ++st)                                           \
            _Pragma("unroll") for (int tt = 0; tt < 4; ++tt)                                       \
                _Pragma("unroll") for (int rt = 0; rt < 2; ++rt)                                   \
            acc[tt][rt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ac_[tt][st], bc_[rt][st],        \
                                                                  acc[tt][rt], 0, 0, 0);           \
        NVQ_READ_A(an_, cur_ ^ 1);                                                                 \
        NVQ_DEQUANT(bn_, ((g_) + 1 < G ? (g_) + 1 : G - 1));                                       \
        __syncthreads();                                                                           \
    } while (0)

    bf16x8 aA[4][2], aB[4][2], bA[2][2], bB[2][2];
    {
        const int g1 = G > 1 ? 1 : G - 1, g2 = G > 2 ? 2 : G - 1;
        NVQ_REQUEST_X(0);
        NVQ_REQUEST_W(0);
        NVQ_STAGE_X(0);
        NVQ_STAGE_W(0);
        NVQ_REQUEST_X(g1);
        NVQ_REQUEST_W(1);
        __syncthreads();
        NVQ_READ_A(aA, 0);
        NVQ_DEQUANT(bA, 0);
        NVQ_STAGE_X(1);
        NVQ_REQUEST_X(g2);
        __syncthreads();
    }
    // here: aA, bA = group 0; LDS: activations of group 1, weights of groups
    // 0..3; registers: activations of group 2, weights of groups 4..7

    for (int g = 0; g < G; g += 2) {
        NVQ_GROUP(g, aA, bA, aB, bB);
        if (g + 1 < G) NVQ_GROUP(g + 1, aB, bB, aA, bA);
    }

#undef NVQ_GROUP
#undef NVQ_DEQUANT
#undef NVQ_READ_A
#undef NVQ_REQUEST_X
#undef NVQ_REQUEST_W
#undef NVQ_STAGE_X
#undef NVQ_STAGE_W

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
    // four scales of a row in one 8-byte load
    const int by_four = (K % 128) == 0 && aligned(scales, 8) ? 1 : 0;
    const uint4 *x = reinterpret_cast<const uint4 *>(x_bf16);
    if (y_dtype == NVQ_F32)
        hipLaunchKernelGGL(gemm_w4a16_kernel<true>, grid, block, 0, (hipStream_t)stream, qw, scales,
                           (int)N, (int)(K / 32), x, (int)M, y, by_four);
    else
        hipLaunchKernelGGL(gemm_w4a16_kernel<false>, grid, block, 0, (hipStream_t)stream, qw, scales,
                           (int)N, (int)(K / 32), x, (int)M, y, by_four);
    NVQ_HIP_TRY(hipGetLastError());
    return NVQ_OK;
}
