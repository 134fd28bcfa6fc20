// Small-batch (2 <= M <= 32 tokens) W4A8 and W4A16 products on the matrix
// cores.  Paper: the W4A8 / W4A16 kernel descriptions and the remark in the
// limitations that batch > 1 moves the product towards compute; the weights
// are still read once per step, so the kernel stays bound by HBM.
//
// One 16x16x32 MFMA covers exactly one quantisation group: 16 tokens x 32
// inputs (operand A) times 32 inputs x 16 weight rows (operand B).  Lane
// (n, kb) = (lane % 16, lane / 16) supplies eight of the 32 inputs of weight
// row n; which eight is free as long as the activation operand uses the same
// choice, so the lane takes dword kb of the group's 16 bytes as they lie in
// memory: its low nibbles are inputs 4kb..4kb+3 and its high nibbles inputs
// 16+4kb..16+4kb+3.  The result tile puts weight row n in lane n of every
// 16-lane row and tokens 4kb..4kb+3 in the lane's four registers, so one
// fp16 weight scale per lane and group rescales the tile (convert + FMA per
// output for W4A8, FMA per output for W4A16).
//
// Nibbles enter the MFMA unsigned (W4A8: bytes 0..15; W4A16: the bf16 numbers
// 128 + n, a nibble under the byte 0x43).  The constant offset (8, or 136) is
// removed with the paper's deferred correction, itself an MFMA: the
// activation operand times a constant operand (all -8, or all -136) yields
// -8 * sum(q) or -136 * sum(x) of the group for every output of the tile and
// is the accumulator input of the weight MFMAs, shared by the R row tiles a
// wave processes together.
//
// Memory: lane (n, kb) loads the 16 bytes of group 4c + kb of row n, so a
// wave reads 64 contiguous bytes of 16 rows per load; a 4x4 transpose across
// the four 16-lane rows (two permlane32 and two permlane16 swaps) then gives
// the lane dword kb of groups 4c..4c+3.  The activation operands are loaded
// the same way, 16 bytes per lane with whole 64-byte runs per token and
// instruction, and brought into operand order with the same swaps: narrower
// loads that fetch each lane's operand bytes directly touch four times as many
// cache lines per instruction and were bound by the L1 lookup rate.
//
// A workgroup owns 16 * R consecutive rows; its W (8 or 16) waves split K by
// 64-byte columns, each requests all loads of a pass of B columns before the
// first MFMA, and the partial tiles are summed through LDS in wave order.
#include "gemv_tile.h"
#include "mfma_act.h"

namespace nvq {

namespace {

// One 64-byte column (four groups) of the lane's row in each of R row tiles,
// and the lane's activation operands for the four groups.
template <int PREC, int R, int MT>
struct Column {
    uint4v w[R];  // group 4c + kb of row n
    uint2 s[R];   // fp16 scales of groups 4c .. 4c+3 of row n
    uint4v a[MT][Act<PREC>::kRaw];
};

// A workgroup of W waves owns 16 * R consecutive rows at a time; wave w takes
// the columns w, w + W, ... of those rows, B columns per pass: every load of a
// pass is requested before the first MFMA, so a wave has B * R KiB of weights
// in flight and the compute units overlap the passes of their resident waves.
//
// mfma_units works through the units unit_first, unit_first + unit_step, ...
// of one phase (a unit = 16 * R rows); `red` is W x (R * MT * 4) x 64 floats
// of LDS.
template <int PREC, int R, int MT, int W, int B, bool DEBUG>
__device__ __forceinline__ void mfma_units(const GemvSegs &S, int G, int M,
                                           const char *__restrict__ xin,
                                           const float *__restrict__ xscale, int unit_first,
                                           int unit_step, float (*red)[R * MT * 4][64]) {
    typedef Act<PREC> A;
    constexpr int kTile = R * MT * 4;  // result registers per lane

    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    const int n = lane & 15, kb = lane >> 4;
    const int C4 = G >> 2;
    const uint32_t row_bytes = (uint32_t)G * 32 * A::kBytes;
    const int units = (S.total_rows + 16 * R - 1) / (16 * R);

    // Byte offset of the lane's part of group 0 for its token in each token
    // tile.  Tokens past M read token 0: an MFMA keeps tokens apart and the
    // results of those tokens are never stored.
    uint32_t xoff[MT];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
        const int m = mt * 16 + n;
        xoff[mt] = (m < M ? m : 0) * row_bytes + kb * A::kLaneBytes;
    }
    // Per-token activation scale of the lane's result registers (W4A8).
    float xs[MT][4];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
        for (int jj = 0; jj < 4; ++jj) {
            const int m = mt * 16 + kb * 4 + jj;
            xs[mt][jj] = (PREC == NVQ_W4A8 && m < M) ? as_global<float>(xscale)[m] : 1.0f;
        }

    for (int unit = unit_first; unit < units; unit += unit_step) {
        RowRef rr[R];
#pragma unroll
        for (int r = 0; r < R; ++r) rr[r] = locate_row(S, (unit * R + r) * 16 + n, G);

        float f[R][MT][4];
#pragma unroll
        for (int r = 0; r < R; ++r)
#pragma unroll
            for (int mt = 0; mt < MT; ++mt)
#pragma unroll
                for (int jj = 0; jj < 4; ++jj) f[r][mt][jj] = 0.0f;

        for (int c0 = w; c0 < C4; c0 += W * B) {
            Column<PREC, R, MT> col[B];
#pragma unroll
            for (int b = 0; b < B; ++b) {
                const int c = c0 + b * W;
                const bool ok = c < C4;  // (wave-uniform)
                const int cc = ok ? c : C4 - 1;
                const char *xcol = xin + (size_t)cc * (128 * A::kBytes);
#pragma unroll
                for (int mt = 0; mt < MT; ++mt) A::load(xcol + xoff[mt], col[b].a[mt]);
#pragma unroll
                for (int r = 0; r < R; ++r) {
                    col[b].w[r] = load_stream(rr[r].qw + 4 * cc + kb);
                    const uint2v sc = *as_global<uint2v>(rr[r].sc + 4 * cc);
                    // a column past the end of the row contributes zero
                    col[b].s[r] = make_uint2(ok ? sc.x : 0u, ok ? sc.y : 0u);
                }
            }
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int b = 0; b < B; ++b) {
                const int c = c0 + b * W;
                uint32_t q[R][4];
                float sw[R][4];
#pragma unroll
                for (int r = 0; r < R; ++r) {
                    q[r][0] = col[b].w[r].x;
                    q[r][1] = col[b].w[r].y;
                    q[r][2] = col[b].w[r].z;
                    q[r][3] = col[b].w[r].w;
                    transpose_rows(q[r]);
                    sw[r][0] = half_bits_to_float((uint16_t)(col[b].s[r].x & 0xffffu));
                    sw[r][1] = half_bits_to_float((uint16_t)(col[b].s[r].x >> 16));
                    sw[r][2] = half_bits_to_float((uint16_t)(col[b].s[r].y & 0xffffu));
                    sw[r][3] = half_bits_to_float((uint16_t)(col[b].s[r].y >> 16));
                }
                typename A::operand act[MT][4];
#pragma unroll
                for (int mt = 0; mt < MT; ++mt) A::operands(col[b].a[mt], act[mt]);
#pragma unroll
                for (int i = 0; i < 4; ++i) {
#pragma unroll
                    for (int mt = 0; mt < MT; ++mt) {
                        const typename A::operand a = act[mt][i];
                        const typename A::offset_t off = A::offset(a);
#pragma unroll
                        for (int r = 0; r < R; ++r) {
                            int4v raw;
                            const float4v p = A::product(a, A::weights(q[r][i]), off, raw);
                            f[r][mt][0] = fmaf(sw[r][i], p.x, f[r][mt][0]);
                            f[r][mt][1] = fmaf(sw[r][i], p.y, f[r][mt][1]);
                            f[r][mt][2] = fmaf(sw[r][i], p.z, f[r][mt][2]);
                            f[r][mt][3] = fmaf(sw[r][i], p.w, f[r][mt][3]);
                            if (DEBUG && PREC == NVQ_W4A8) {
                                if (rr[r].valid && rr[r].dbg && c < C4) {
                                    const int acc[4] = {raw.x, raw.y, raw.z, raw.w};
#pragma unroll
                                    for (int jj = 0; jj < 4; ++jj) {
                                        const int m = mt * 16 + kb * 4 + jj;
                                        if (m < M)
                                            rr[r].dbg[((int64_t)m * rr[r].N + rr[r].n) * G + 4 * c +
                                                      i] = acc[jj];
                                    }
                                }
                            }
                        }
                    }
                }
            }
            __builtin_amdgcn_sched_barrier(0);
        }

        // Sum the K slices of the waves in wave order.
#pragma unroll
        for (int r = 0; r < R; ++r)
#pragma unroll
            for (int mt = 0; mt < MT; ++mt)
#pragma unroll
                for (int jj = 0; jj < 4; ++jj)
                    red[w][(r * MT + mt) * 4 + jj][lane] = f[r][mt][jj] * xs[mt][jj];
        __syncthreads();
#pragma unroll
        for (int pass = 0; pass < (kTile + W - 1) / W; ++pass) {
            const int reg = pass * W + w;
            if (reg < kTile) {
                float sum = 0.0f;
#pragma unroll
                for (int k = 0; k < W; ++k) sum += red[k][reg][lane];
                const int r = reg / (MT * 4), mt = (reg >> 2) % MT, jj = reg & 3;
                const int m = mt * 16 + kb * 4 + jj;
                const RowRef o = locate_row(S, (unit * R + r) * 16 + n, G);
                if (o.valid && m < M) store_global(o.y, o.y_dtype, (int64_t)m * o.N + o.n, sum);
            }
        }
        __syncthreads();
    }
}

template <int PREC, int R, int MT, int W, int B, bool DEBUG>
__global__ __launch_bounds__(W * 64) void gemv_mfma_kernel(
    GemvSegs S, int G, int M, const char *__restrict__ xin, const float *__restrict__ xscale) {
    __shared__ float red[W][R * MT * 4][64];
    mfma_units<PREC, R, MT, W, B, DEBUG>(S, G, M, xin, xscale, blockIdx.x, gridDim.x, red);
}

// Grouped launch: the row tiles of many phases in one grid, one tile per
// workgroup.  unit_phase[u] names the phase of grid unit u.
constexpr int kGroupWaves = 4;
template <int MT, int R>
__global__ __launch_bounds__(kGroupWaves * 64) void gemv_mfma_group_kernel(
    const GroupPhase *__restrict__ tab, const uint16_t *__restrict__ unit_phase, int M) {
    __shared__ float red[kGroupWaves][R * MT * 4][64];
    const int u = blockIdx.x;
    const GroupPhase &P = tab[unit_phase[u]];
    const int unit = u - P.unit_begin;
    // one pass of the unit loop: the step is larger than any unit count
    if (P.precision == NVQ_W4A8)
        mfma_units<NVQ_W4A8, R, MT, kGroupWaves, 2, false>(
            P.segs, P.G, M, reinterpret_cast<const char *>(P.xq), P.xscale, unit, 1 << 30, red);
    else
        mfma_units<NVQ_W4A16, R, MT, kGroupWaves, 2, false>(
            P.segs, P.G, M, reinterpret_cast<const char *>(P.x_bf16), nullptr, unit, 1 << 30, red);
}

template <int PREC, int R, int MT, int W, int B, bool DEBUG>
int launch_one(const GemvSegs &S, int G, int M, const void *x, const float *xscale,
               hipStream_t st) {
    const int units = (S.total_rows + 16 * R - 1) / (16 * R);
    const int cap = device_cu_count() * 8;
    const dim3 grid(units < cap ? units : cap), block(W * 64);
    hipLaunchKernelGGL((gemv_mfma_kernel<PREC, R, MT, W, B, DEBUG>), grid, block, 0, st, S, G, M,
                       reinterpret_cast<const char *>(x), xscale);
    NVQ_HIP_TRY(hipGetLastError());
    return NVQ_OK;
}

template <int PREC>
int launch_prec(const GemvSegs &S, int G, int M, const void *x, const float *xscale, bool debug,
                hipStream_t st) {
    const bool wide = M > 16;
    // Eight waves share a row tile, so that a compute unit holds two or three
    // workgroups whose load and compute passes overlap; sixteen when there are
    // too few tiles for that and each wave still gets two columns (K >= 4096).
    const int tiles = (S.total_rows + 15) / 16;
    const bool many = (G >> 2) >= 32 && tiles <= 2 * device_cu_count();
#define NVQ_GO(MT, W, DBG) return launch_one<PREC, 1, MT, W, 2, DBG>(S, G, M, x, xscale, st)
    if (debug) {  // accumulator dump, same summation order as the plain kernel
        if (wide) { if (many) NVQ_GO(2, 16, true); else NVQ_GO(2, 8, true); }
        if (many) NVQ_GO(1, 16, true); else NVQ_GO(1, 8, true);
    }
    if (wide) { if (many) NVQ_GO(2, 16, false); else NVQ_GO(2, 8, false); }
    if (many) NVQ_GO(1, 16, false); else NVQ_GO(1, 8, false);
#undef NVQ_GO
}

}  // namespace

bool gemv_mfma_supported(const GemvSegs &S, int K, int M) {
    if (M < 2 || M > 32 || K % 128 != 0) return false;
    for (int i = 0; i < S.nseg; ++i)
        if (!aligned(S.sc[i], 8)) return false;
    return true;
}

int launch_gemv_mfma_group(const GroupPhase *tab, const uint16_t *unit_phase, int nunits, int M,
                           hipStream_t st) {
    if (nunits <= 0) return NVQ_OK;
    const dim3 grid(nunits), block(kGroupWaves * 64);
    if (M > 16)
        hipLaunchKernelGGL((gemv_mfma_group_kernel<2, 2>), grid, block, 0, st, tab, unit_phase, M);
    else
        hipLaunchKernelGGL((gemv_mfma_group_kernel<1, 2>), grid, block, 0, st, tab, unit_phase, M);
    NVQ_HIP_TRY(hipGetLastError());
    return NVQ_OK;
}

int launch_gemv_mfma(const GemvSegs &S, int K, int precision, const void *x, const float *xscale,
                     int M, hipStream_t st) {
    bool debug = false;
    for (int i = 0; i < S.nseg; ++i) debug |= S.dbg[i] != nullptr;
    if (precision == NVQ_W4A8)
        return launch_prec<NVQ_W4A8>(S, K / 32, M, x, xscale, debug, st);
    return launch_prec<NVQ_W4A16>(S, K / 32, M, x, nullptr, false, st);
}

}  // namespace nvq
