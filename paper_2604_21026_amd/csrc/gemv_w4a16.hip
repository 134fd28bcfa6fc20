// nvq_gemv_w4a16: int4 weights x bf16 activations, fp32 accumulate.
// Paper: the W4A16 branch of the per-layer precision dispatch (kernel table:
// in-register dequantisation, cross-lane reduction, no integer dot product).
//
// Dequantisation never leaves the registers and costs one bit operation per
// two weights: a nibble n placed in the low mantissa bits of the bf16 pattern
// 0x4300 is the number 128 + n exactly, so a byte permute turns two nibble
// bytes into a bf16 pair (128 + n0, 128 + n1) that feeds the packed bf16 dot
// instruction against two activations.  The constant 136 = 128 + 8 that this
// adds to every signed code is removed per group of 32 by preloading the
// accumulator with -136 * sum(x_group), the floating-point twin of the
// paper's deferred bias correction.  Every product (128+n)*x is exact in
// fp32; only the order of fp32 additions differs from a wide reference.
//
// Batch 1 (fast path): decomposition as in gemv_tile.h with the lane's bf16
// activations register-resident (16 dwords per owned group).  Two to 32
// tokens go to the matrix-core kernel (gemv_mfma.hip), other cases to the
// generic kernel.
#include "gemv_tile.h"

namespace nvq {

typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));

__device__ __forceinline__ float dot2_bf16(uint32_t a, uint32_t b, float c) {
    return __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2_t, a),
                                           __builtin_bit_cast(bf16x2_t, b), c, false);
}

// x[j] holds activations (2j, 2j+1) of the group as a bf16 pair.
__device__ __forceinline__ float block_dot_bf16(const uint4 &w, const uint32_t (&x)[16], float acc) {
    const uint32_t wv[4] = {w.x, w.y, w.z, w.w};
    constexpr uint32_t kMagic = 0x43434343u;  // high byte of bf16(128 + n)
#pragma unroll
    for (int d = 0; d < 4; ++d) {
        const uint32_t lo = wv[d] & 0x0f0f0f0fu;         // elements 4d .. 4d+3, one per byte
        const uint32_t hi = (wv[d] >> 4) & 0x0f0f0f0fu;  // elements 16+4d .. 16+4d+3
        // byte permute: selector 0-3 picks a byte of the second operand,
        // 4-7 a byte of the first
        const uint32_t l01 = __builtin_amdgcn_perm(kMagic, lo, 0x04010400u);
        const uint32_t l23 = __builtin_amdgcn_perm(kMagic, lo, 0x04030402u);
        const uint32_t h01 = __builtin_amdgcn_perm(kMagic, hi, 0x04010400u);
        const uint32_t h23 = __builtin_amdgcn_perm(kMagic, hi, 0x04030402u);
        acc = dot2_bf16(l01, x[2 * d], acc);
        acc = dot2_bf16(l23, x[2 * d + 1], acc);
        acc = dot2_bf16(h01, x[8 + 2 * d], acc);
        acc = dot2_bf16(h23, x[8 + 2 * d + 1], acc);
    }
    return acc;
}

// -136 * (sum of the 32 activations of a group), fp32.
__device__ __forceinline__ float group_offset(const uint32_t (&x)[16]) {
    float s = 0.0f;
#pragma unroll
    for (int j = 0; j < 16; ++j) s = dot2_bf16(0x3f803f80u, x[j], s);  // (1, 1) . (x0, x1)
    return -136.0f * s;
}

template <int GPL, int LPR>
__global__ __launch_bounds__(256) void gemv_w4a16_m1_kernel(GemvSegs S, int G,
                                                            const uint4 *__restrict__ x) {
    constexpr int U = tile_rows(GPL);
    constexpr int TEAMS = 256 / LPR;
    const int lane = threadIdx.x % LPR;
    const int v = blockIdx.x * TEAMS + threadIdx.x / LPR;
    const int V = gridDim.x * TEAMS;
    const int tiles = (S.total_rows + U - 1) / U;

    uint32_t xr[GPL][16];
    float off[GPL];
    int gc[GPL];
#pragma unroll
    for (int i = 0; i < GPL; ++i) {
        const int g = i * LPR + lane;
        const bool ok = g < G;
        gc[i] = ok ? g : 0;
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const uint4 a = x[gc[i] * 4 + q];
            xr[i][4 * q + 0] = ok ? a.x : 0u;
            xr[i][4 * q + 1] = ok ? a.y : 0u;
            xr[i][4 * q + 2] = ok ? a.z : 0u;
            xr[i][4 * q + 3] = ok ? a.w : 0u;
        }
        off[i] = group_offset(xr[i]);
    }

    uint4 wb[U][GPL];
    uint16_t sb[U][GPL];
    auto load_tile = [&](int t, uint4(&w)[U][GPL], uint16_t(&s)[U][GPL]) {
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const RowRef r = locate_row(S, t * U + u, G);
#pragma unroll
            for (int i = 0; i < GPL; ++i) {
                w[u][i] = stream_load16(r.qw + gc[i]);  // read once: non-temporal, whole lines
                s[u][i] = r.sc[gc[i]];
            }
        }
    };

    int t = v;
    if (t < tiles) load_tile(t, wb, sb);
    for (; t < tiles; t += V) {
        uint4 wn[U][GPL] = {};
        uint16_t sn[U][GPL] = {};
        if (t + V < tiles) load_tile(t + V, wn, sn);

#pragma unroll
        for (int u = 0; u < U; ++u) {
            const RowRef r = locate_row(S, t * U + u, G);
            float sum = 0.0f;
#pragma unroll
            for (int i = 0; i < GPL; ++i) {
                const float acc = block_dot_bf16(wb[u][i], xr[i], off[i]);
                sum = fmaf(half_bits_to_float(sb[u][i]), acc, sum);
            }
            sum = group_sum<LPR>(sum);
            if (lane == 0 && r.valid) store_out(r.y, r.y_dtype, r.n, sum);
        }
#pragma unroll
        for (int u = 0; u < U; ++u)
#pragma unroll
            for (int i = 0; i < GPL; ++i) {
                wb[u][i] = wn[u][i];
                sb[u][i] = sn[u][i];
            }
    }
}

// Generic kernel: one wave per row, lanes stride over the groups, tokens in
// chunks of MT, activations read from memory.
template <int MT>
__global__ __launch_bounds__(256) void gemv_w4a16_generic_kernel(GemvSegs S, int G, int M,
                                                                 const uint4 *__restrict__ x) {
    const int lane = threadIdx.x & 63;
    const int wave = blockIdx.x * 4 + (threadIdx.x >> 6);
    const int waves = gridDim.x * 4;
    for (int row = wave; row < S.total_rows; row += waves) {
        const RowRef r = locate_row(S, row, G);
        for (int m0 = 0; m0 < M; m0 += MT) {
            float sum[MT];
#pragma unroll
            for (int mm = 0; mm < MT; ++mm) sum[mm] = 0.0f;
            for (int g = lane; g < G; g += 64) {
                const uint4 w = r.qw[g];
                const float sw = half_bits_to_float(r.sc[g]);
#pragma unroll
                for (int mm = 0; mm < MT; ++mm) {
                    const int m = m0 + mm;
                    if (m < M) {
                        const int64_t xg = ((int64_t)m * G + g) * 4;
                        uint32_t xv[16];
#pragma unroll
                        for (int q = 0; q < 4; ++q) {
                            const uint4 a = x[xg + q];
                            xv[4 * q + 0] = a.x;
                            xv[4 * q + 1] = a.y;
                            xv[4 * q + 2] = a.z;
                            xv[4 * q + 3] = a.w;
                        }
                        const float acc = block_dot_bf16(w, xv, group_offset(xv));
                        sum[mm] = fmaf(sw, acc, sum[mm]);
                    }
                }
            }
#pragma unroll
            for (int mm = 0; mm < MT; ++mm) {
                const int m = m0 + mm;
                const float tot = group_sum<64>(sum[mm]);
                if (lane == 0 && m < M) store_out(r.y, r.y_dtype, (int64_t)m * r.N + r.n, tot);
            }
        }
    }
}

template <int GPL, int LPR>
static int launch_m1(const GemvSegs &S, int G, const uint16_t *x, hipStream_t st) {
    constexpr int U = tile_rows(GPL);
    const int tiles = (S.total_rows + U - 1) / U;
    const dim3 grid(gemv_grid(tiles, 256 / LPR, kM1WgPerCu)), block(256);
    hipLaunchKernelGGL((gemv_w4a16_m1_kernel<GPL, LPR>), grid, block, 0, st, S, G,
                       reinterpret_cast<const uint4 *>(x));
    NVQ_HIP_TRY(hipGetLastError());
    return NVQ_OK;
}

int launch_gemv_w4a16(const GemvSegs &S, int K, const uint16_t *x, int M, hipStream_t st) {
    const int G = K / 32;
    if (M == 1 && G <= 512) {
        if (G % 32 == 0 && G % 64 != 0 && G <= 96) {
            if (G == 32) return launch_m1<1, 32>(S, G, x, st);
            return launch_m1<3, 32>(S, G, x, st);
        }
        switch ((G + 63) / 64) {
            case 1: return launch_m1<1, 64>(S, G, x, st);
            case 2: return launch_m1<2, 64>(S, G, x, st);
            case 3: return launch_m1<3, 64>(S, G, x, st);
            case 4: return launch_m1<4, 64>(S, G, x, st);
            case 5: return launch_m1<5, 64>(S, G, x, st);
            case 6: return launch_m1<6, 64>(S, G, x, st);
            case 7: return launch_m1<7, 64>(S, G, x, st);
            default: return launch_m1<8, 64>(S, G, x, st);
        }
    }
    if (gemv_mfma_supported(S, K, M)) return launch_gemv_mfma(S, K, NVQ_W4A16, x, nullptr, M, st);
    const dim3 grid(gemv_grid(S.total_rows, 4, 8)), block(256);
    hipLaunchKernelGGL((gemv_w4a16_generic_kernel<4>), grid, block, 0, st, S, G, M,
                       reinterpret_cast<const uint4 *>(x));
    NVQ_HIP_TRY(hipGetLastError());
    return NVQ_OK;
}

}  // namespace nvq

extern "C" int nvq_gemv_w4a16(const uint8_t *qweight, const uint16_t *scales, int N, int K,
                              const uint16_t *x_bf16, int M, void *y, int y_dtype, void *stream) {
    if (!qweight || !scales || !x_bf16 || !y) return NVQ_ERR_INVALID_ARG;
    if (y_dtype != NVQ_F32 && y_dtype != NVQ_BF16) return NVQ_ERR_INVALID_ARG;
    if (N <= 0 || M <= 0 || M > NVQ_MAX_M || K <= 0 || (K % 32) != 0 || K > NVQ_MAX_K)
        return NVQ_ERR_SHAPE;
    if (!nvq::aligned(qweight, 16) || !nvq::aligned(scales, 2) || !nvq::aligned(x_bf16, 16) ||
        !nvq::aligned(y, y_dtype == NVQ_F32 ? 4 : 2))
        return NVQ_ERR_ALIGN;
    nvq::GemvSegs S = {};
    S.qw[0] = reinterpret_cast<const uint4 *>(qweight);
    S.sc[0] = scales;
    S.y[0] = y;
    S.N[0] = N;
    S.row_end[0] = N;
    S.y_dtype[0] = y_dtype;
    S.nseg = 1;
    S.total_rows = N;
    return nvq::launch_gemv_w4a16(S, K, x_bf16, M, (hipStream_t)stream);
}
