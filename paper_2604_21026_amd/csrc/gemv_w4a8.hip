// nvq_gemv_w4a8: int4 weights x int8 activations, int32 block accumulators,
// fp32 rescale.  Paper: W4A8 kernel description and appendix "W4A8 dp4a
// Matrix-Vector Product".
//
// The unsigned nibbles go straight into the packed signed-int8 dot
// instruction (0..15 is a valid int8) and the constant offset is removed
// with the paper's deferred correction: acc = sum nib*q - 8*sum q, where
// sum q per block comes from the activation quantisation step.  The
// accumulator is preloaded with -8*sum q, so the correction costs nothing in
// the loop.
//
// Batch 1 (fast path): see gemv_tile.h for the lane/row decomposition; the
// int8 codes of the lane's groups are register-resident, the loop body per
// 32 weights is one 128-bit load, 12 bit operations, 8 dot4, one convert and
// one FMA.  Two to 32 tokens with a per-token scale go to the matrix-core
// kernel (gemv_mfma.hip); any other case takes the generic kernel, which
// re-reads activations from memory.
#include "gemv_tile.h"

namespace nvq {

__device__ __forceinline__ int block_dot_i8(const uint4 &w, const uint32_t (&x)[8], int acc) {
    const uint32_t wv[4] = {w.x, w.y, w.z, w.w};
#pragma unroll
    for (int d = 0; d < 4; ++d) {
        const uint32_t lo = wv[d] & 0x0f0f0f0fu;         // elements 4d .. 4d+3
        const uint32_t hi = (wv[d] >> 4) & 0x0f0f0f0fu;  // elements 16+4d .. 16+4d+3
        acc = __builtin_amdgcn_sdot4((int)lo, (int)x[d], acc, false);
        acc = __builtin_amdgcn_sdot4((int)hi, (int)x[4 + d], acc, false);
    }
    return acc;
}

template <int GPL, int LPR, bool PER_GROUP, bool DEBUG>
__global__ __launch_bounds__(256) void gemv_w4a8_m1_kernel(GemvSegs S, int G,
                                                           const uint4 *__restrict__ xq,
                                                           const float *__restrict__ xscale,
                                                           const int32_t *__restrict__ xgsum) {
    constexpr int U = tile_rows(GPL);
    constexpr int TEAMS = 256 / LPR;
    const int lane = threadIdx.x % LPR;
    const int v = blockIdx.x * TEAMS + threadIdx.x / LPR;
    const int V = gridDim.x * TEAMS;
    const int tiles = (S.total_rows + U - 1) / U;

    // Activation codes of the groups this lane owns, for the whole kernel.
    uint32_t xr[GPL][8];
    int neg8[GPL];
    float xsg[GPL];
    int gc[GPL];
    bool ok[GPL];
#pragma unroll
    for (int i = 0; i < GPL; ++i) {
        const int g = i * LPR + lane;
        ok[i] = g < G;
        gc[i] = ok[i] ? g : 0;
        const uint4 a = xq[gc[i] * 2], b = xq[gc[i] * 2 + 1];
        const uint32_t t[8] = {a.x, a.y, a.z, a.w, b.x, b.y, b.z, b.w};
#pragma unroll
        for (int d = 0; d < 8; ++d) xr[i][d] = ok[i] ? t[d] : 0u;
        neg8[i] = ok[i] ? -8 * xgsum[gc[i]] : 0;
        xsg[i] = PER_GROUP ? xscale[gc[i]] : 1.0f;
    }
    const float xs = PER_GROUP ? 1.0f : xscale[0];

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
                const int acc = block_dot_i8(wb[u][i], xr[i], neg8[i]);
                if (DEBUG) {
                    if (r.valid && ok[i] && r.dbg) r.dbg[(int64_t)r.n * G + gc[i]] = acc;
                }
                float sw = half_bits_to_float(sb[u][i]);
                if (PER_GROUP) sw *= xsg[i];
                sum = fmaf(sw, (float)acc, sum);
            }
            sum = group_sum<LPR>(sum);
            if (lane == 0 && r.valid) store_out(r.y, r.y_dtype, r.n, sum * xs);
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
// chunks of MT.  Activations are read from memory (cache-resident).
template <int MT, bool PER_GROUP, bool DEBUG>
__global__ __launch_bounds__(256) void gemv_w4a8_generic_kernel(
    GemvSegs S, int G, int M, const uint4 *__restrict__ xq, const float *__restrict__ xscale,
    const int32_t *__restrict__ xgsum) {
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
                        const int64_t xg = (int64_t)m * G + g;
                        const uint4 a = xq[xg * 2], b = xq[xg * 2 + 1];
                        const uint32_t x[8] = {a.x, a.y, a.z, a.w, b.x, b.y, b.z, b.w};
                        const int acc = block_dot_i8(w, x, -8 * xgsum[xg]);
                        if (DEBUG) {
                            if (r.dbg) r.dbg[((int64_t)m * r.N + r.n) * G + g] = acc;
                        }
                        const float s = PER_GROUP ? sw * xscale[xg] : sw;
                        sum[mm] = fmaf(s, (float)acc, sum[mm]);
                    }
                }
            }
#pragma unroll
            for (int mm = 0; mm < MT; ++mm) {
                const int m = m0 + mm;
                const float tot = group_sum<64>(sum[mm]);
                if (lane == 0 && m < M)
                    store_out(r.y, r.y_dtype, (int64_t)m * r.N + r.n,
                              PER_GROUP ? tot : tot * xscale[m]);
            }
        }
    }
}

template <int GPL, int LPR>
static int launch_m1(const GemvSegs &S, int G, const int8_t *xq, const float *xscale,
                     const int32_t *xgsum, bool per_group, bool debug, hipStream_t st) {
    constexpr int U = tile_rows(GPL);
    const int tiles = (S.total_rows + U - 1) / U;
    const dim3 grid(gemv_grid(tiles, 256 / LPR, kM1WgPerCu)), block(256);
    const uint4 *x4 = reinterpret_cast<const uint4 *>(xq);
#define NVQ_GO(PG, DBG)                                                                        \
    hipLaunchKernelGGL((gemv_w4a8_m1_kernel<GPL, LPR, PG, DBG>), grid, block, 0, st, S, G, x4, \
                       xscale, xgsum)
    if (per_group) {
        if (debug) NVQ_GO(true, true); else NVQ_GO(true, false);
    } else {
        if (debug) NVQ_GO(false, true); else NVQ_GO(false, false);
    }
#undef NVQ_GO
    NVQ_HIP_TRY(hipGetLastError());
    return NVQ_OK;
}

int launch_gemv_w4a8(const GemvSegs &S, int K, const int8_t *xq, const float *xscale,
                     const int32_t *xgsum, int act_group, int M, hipStream_t st) {
    const int G = K / 32;
    const bool pg = act_group == 32;
    bool debug = false;
    for (int i = 0; i < S.nseg; ++i) debug |= S.dbg[i] != nullptr;
    if (M == 1 && G <= 512) {
        if (G % 32 == 0 && G % 64 != 0 && G <= 96) {
            if (G == 32) return launch_m1<1, 32>(S, G, xq, xscale, xgsum, pg, debug, st);
            return launch_m1<3, 32>(S, G, xq, xscale, xgsum, pg, debug, st);
        }
        switch ((G + 63) / 64) {
            case 1: return launch_m1<1, 64>(S, G, xq, xscale, xgsum, pg, debug, st);
            case 2: return launch_m1<2, 64>(S, G, xq, xscale, xgsum, pg, debug, st);
            case 3: return launch_m1<3, 64>(S, G, xq, xscale, xgsum, pg, debug, st);
            case 4: return launch_m1<4, 64>(S, G, xq, xscale, xgsum, pg, debug, st);
            case 5: return launch_m1<5, 64>(S, G, xq, xscale, xgsum, pg, debug, st);
            case 6: return launch_m1<6, 64>(S, G, xq, xscale, xgsum, pg, debug, st);
            case 7: return launch_m1<7, 64>(S, G, xq, xscale, xgsum, pg, debug, st);
            default: return launch_m1<8, 64>(S, G, xq, xscale, xgsum, pg, debug, st);
        }
    }
    if (!pg && gemv_mfma_supported(S, K, M))
        return launch_gemv_mfma(S, K, NVQ_W4A8, xq, xscale, M, st);
    const dim3 grid(gemv_grid(S.total_rows, 4, 8)), block(256);
    const uint4 *x4 = reinterpret_cast<const uint4 *>(xq);
#define NVQ_GO(PG, DBG)                                                                      \
    hipLaunchKernelGGL((gemv_w4a8_generic_kernel<4, PG, DBG>), grid, block, 0, st, S, G, M, \
                       x4, xscale, xgsum)
    if (pg) {
        if (debug) NVQ_GO(true, true); else NVQ_GO(true, false);
    } else {
        if (debug) NVQ_GO(false, true); else NVQ_GO(false, false);
    }
#undef NVQ_GO
    NVQ_HIP_TRY(hipGetLastError());
    return NVQ_OK;
}

}  // namespace nvq

extern "C" int nvq_gemv_w4a8(const uint8_t *qweight, const uint16_t *scales, int N, int K,
                             const int8_t *xq, const float *xscale, const int32_t *xgsum,
                             int act_group, int M, void *y, int y_dtype, int32_t *acc_debug,
                             void *stream) {
    if (!qweight || !scales || !xq || !xscale || !xgsum || !y) return NVQ_ERR_INVALID_ARG;
    if (act_group != 0 && act_group != 32) return NVQ_ERR_INVALID_ARG;
    if (y_dtype != NVQ_F32 && y_dtype != NVQ_BF16) return NVQ_ERR_INVALID_ARG;
    if (N <= 0 || M <= 0 || M > NVQ_MAX_M || K <= 0 || (K % 32) != 0 || K > NVQ_MAX_K)
        return NVQ_ERR_SHAPE;
    if (!nvq::aligned(qweight, 16) || !nvq::aligned(scales, 2) || !nvq::aligned(xq, 16) ||
        !nvq::aligned(xscale, 4) || !nvq::aligned(xgsum, 4) ||
        !nvq::aligned(y, y_dtype == NVQ_F32 ? 4 : 2) || !nvq::aligned(acc_debug, 4))
        return NVQ_ERR_ALIGN;
    nvq::GemvSegs S = {};
    S.qw[0] = reinterpret_cast<const uint4 *>(qweight);
    S.sc[0] = scales;
    S.y[0] = y;
    S.dbg[0] = acc_debug;
    S.N[0] = N;
    S.row_end[0] = N;
    S.y_dtype[0] = y_dtype;
    S.nseg = 1;
    S.total_rows = N;
    return nvq::launch_gemv_w4a8(S, K, xq, xscale, xgsum, act_group, M, (hipStream_t)stream);
}
