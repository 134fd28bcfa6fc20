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
// the lane dword kb of groups 4c..4c+3.  A workgroup owns 16 * R consecutive
// rows; its eight waves split K by 64-byte columns and their partial tiles
// are summed through LDS in a fixed order.
#include "gemv_tile.h"

namespace nvq {

namespace {

typedef int int4v __attribute__((ext_vector_type(4)));
typedef float float4v __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef unsigned uint2v __attribute__((ext_vector_type(2)));
typedef unsigned uint4v __attribute__((ext_vector_type(4)));

constexpr int kMfmaWaves = 8;

__device__ __forceinline__ uint4v load_stream(const uint4 *p) {
    return __builtin_nontemporal_load(reinterpret_cast<const uint4v *>(p));
}

// r[j] of lane-row kb holds element (kb, j) of a 4x4 matrix of dwords (one
// matrix per lane column n); afterwards r[i] of lane-row kb holds (i, kb).
__device__ __forceinline__ void transpose_rows(uint32_t (&r)[4]) {
    const uint2v a = __builtin_amdgcn_permlane32_swap(r[0], r[2], false, false);
    const uint2v b = __builtin_amdgcn_permlane32_swap(r[1], r[3], false, false);
    const uint2v c = __builtin_amdgcn_permlane16_swap(a.x, b.x, false, false);
    const uint2v d = __builtin_amdgcn_permlane16_swap(a.y, b.y, false, false);
    r[0] = c.x;
    r[1] = c.y;
    r[2] = d.x;
    r[3] = d.y;
}

template <int PREC>
struct Act;

// int8 codes: 8 bytes per lane and MFMA.
template <>
struct Act<NVQ_W4A8> {
    typedef long operand;
    static constexpr int kBytes = 1;
    __device__ static operand load(const char *p, bool ok) {
        const uint32_t lo = *reinterpret_cast<const uint32_t *>(p);
        const uint32_t hi = *reinterpret_cast<const uint32_t *>(p + 16);
        const uint64_t v = (uint64_t)lo | ((uint64_t)hi << 32);
        return ok ? (long)v : 0l;
    }
    __device__ static operand weights(uint32_t v) {
        const uint32_t lo = v & 0x0f0f0f0fu, hi = (v >> 4) & 0x0f0f0f0fu;
        return (long)((uint64_t)lo | ((uint64_t)hi << 32));
    }
    __device__ static int4v offset(operand a) {
        const int4v z = {0, 0, 0, 0};
        return __builtin_amdgcn_mfma_i32_16x16x32_i8(a, (long)0xf8f8f8f8f8f8f8f8ull, z, 0, 0, 0);
    }
    __device__ static float4v product(operand a, operand b, int4v c, int4v &raw) {
        raw = __builtin_amdgcn_mfma_i32_16x16x32_i8(a, b, c, 0, 0, 0);
        const float4v f = {(float)raw.x, (float)raw.y, (float)raw.z, (float)raw.w};
        return f;
    }
    typedef int4v offset_t;
};

// bf16 activations: 16 bytes per lane and MFMA.
template <>
struct Act<NVQ_W4A16> {
    typedef bf16x8 operand;
    static constexpr int kBytes = 2;
    __device__ static operand load(const char *p, bool ok) {
        const uint2 lo = *reinterpret_cast<const uint2 *>(p);
        const uint2 hi = *reinterpret_cast<const uint2 *>(p + 32);
        uint4 v = make_uint4(lo.x, lo.y, hi.x, hi.y);
        if (!ok) v = make_uint4(0, 0, 0, 0);
        return __builtin_bit_cast(bf16x8, v);
    }
    __device__ static operand weights(uint32_t v) {
        constexpr uint32_t kMagic = 0x43434343u;  // high byte of bf16(128 + n)
        const uint32_t lo = v & 0x0f0f0f0fu, hi = (v >> 4) & 0x0f0f0f0fu;
        // byte permute: selector 0-3 picks a byte of the second operand, 4-7 of the first
        const uint4 b = make_uint4(__builtin_amdgcn_perm(kMagic, lo, 0x04010400u),
                                   __builtin_amdgcn_perm(kMagic, lo, 0x04030402u),
                                   __builtin_amdgcn_perm(kMagic, hi, 0x04010400u),
                                   __builtin_amdgcn_perm(kMagic, hi, 0x04030402u));
        return __builtin_bit_cast(bf16x8, b);
    }
    __device__ static float4v offset(operand a) {
        const float4v z = {0.0f, 0.0f, 0.0f, 0.0f};
        constexpr uint32_t kNeg136 = 0xc308c308u;  // bf16(-136) twice
        const uint4 c = make_uint4(kNeg136, kNeg136, kNeg136, kNeg136);
        return __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, __builtin_bit_cast(bf16x8, c), z, 0, 0,
                                                       0);
    }
    __device__ static float4v product(operand a, operand b, float4v c, int4v &raw) {
        (void)raw;
        return __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b, c, 0, 0, 0);
    }
    typedef float4v offset_t;
};

// One 64-byte column (four groups) of the lane's row in each of R row tiles.
template <int R>
struct Column {
    uint4v w[R];  // group 4c + kb of row n
    uint2 s[R];   // fp16 scales of groups 4c .. 4c+3 of row n
};

template <int PREC, int R, int MT, bool DEBUG>
__global__ __launch_bounds__(kMfmaWaves * 64) void gemv_mfma_kernel(
    GemvSegs S, int G, int M, const char *__restrict__ xin, const float *__restrict__ xscale) {
    typedef Act<PREC> A;
    constexpr int kTile = R * MT * 4;  // result registers per lane
    __shared__ float red[kMfmaWaves][kTile][64];

    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    const int n = lane & 15, kb = lane >> 4;
    const int C4 = G >> 2;
    const int64_t row_bytes = (int64_t)G * 32 * A::kBytes;
    const int units = (S.total_rows + 16 * R - 1) / (16 * R);

    // The lane's token in each token tile and where its part of a group starts.
    const char *xrow[MT];
    bool xok[MT];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
        const int m = mt * 16 + n;
        xok[mt] = m < M;
        xrow[mt] = xin + (xok[mt] ? m : 0) * row_bytes + kb * 4 * A::kBytes;
    }

    for (int unit = blockIdx.x; unit < units; unit += gridDim.x) {
        RowRef rr[R];
#pragma unroll
        for (int r = 0; r < R; ++r) rr[r] = locate_row(S, (unit * R + r) * 16 + n, G);

        float f[R][MT][4];
#pragma unroll
        for (int r = 0; r < R; ++r)
#pragma unroll
            for (int mt = 0; mt < MT; ++mt)
#pragma unroll
                for (int j = 0; j < 4; ++j) f[r][mt][j] = 0.0f;

        auto fetch = [&](int c, Column<R> &col) {
#pragma unroll
            for (int r = 0; r < R; ++r) {
                col.w[r] = load_stream(rr[r].qw + 4 * c + kb);
                col.s[r] = *reinterpret_cast<const uint2 *>(rr[r].sc + 4 * c);
            }
        };

        Column<R> cur;
        if (w < C4) fetch(w, cur);
        for (int c = w; c < C4; c += kMfmaWaves) {
            Column<R> nxt = cur;
            if (c + kMfmaWaves < C4) fetch(c + kMfmaWaves, nxt);

            uint32_t t[R][4];
            float sw[R][4];
#pragma unroll
            for (int r = 0; r < R; ++r) {
                t[r][0] = cur.w[r].x;
                t[r][1] = cur.w[r].y;
                t[r][2] = cur.w[r].z;
                t[r][3] = cur.w[r].w;
                transpose_rows(t[r]);
                sw[r][0] = half_bits_to_float((uint16_t)(cur.s[r].x & 0xffffu));
                sw[r][1] = half_bits_to_float((uint16_t)(cur.s[r].x >> 16));
                sw[r][2] = half_bits_to_float((uint16_t)(cur.s[r].y & 0xffffu));
                sw[r][3] = half_bits_to_float((uint16_t)(cur.s[r].y >> 16));
            }
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int g = 4 * c + i;
#pragma unroll
                for (int mt = 0; mt < MT; ++mt) {
                    const typename A::operand a =
                        A::load(xrow[mt] + (int64_t)g * 32 * A::kBytes, xok[mt]);
                    const typename A::offset_t off = A::offset(a);
#pragma unroll
                    for (int r = 0; r < R; ++r) {
                        int4v raw;
                        const float4v p = A::product(a, A::weights(t[r][i]), off, raw);
                        f[r][mt][0] = fmaf(sw[r][i], p.x, f[r][mt][0]);
                        f[r][mt][1] = fmaf(sw[r][i], p.y, f[r][mt][1]);
                        f[r][mt][2] = fmaf(sw[r][i], p.z, f[r][mt][2]);
                        f[r][mt][3] = fmaf(sw[r][i], p.w, f[r][mt][3]);
                        if (DEBUG && PREC == NVQ_W4A8) {
                            if (rr[r].valid && rr[r].dbg) {
                                const int acc[4] = {raw.x, raw.y, raw.z, raw.w};
#pragma unroll
                                for (int j = 0; j < 4; ++j) {
                                    const int m = mt * 16 + kb * 4 + j;
                                    if (m < M)
                                        rr[r].dbg[((int64_t)m * rr[r].N + rr[r].n) * G + g] =
                                            acc[j];
                                }
                            }
                        }
                    }
                }
            }
            cur = nxt;
        }

        // Sum the eight K slices in wave order.
#pragma unroll
        for (int r = 0; r < R; ++r)
#pragma unroll
            for (int mt = 0; mt < MT; ++mt)
#pragma unroll
                for (int j = 0; j < 4; ++j) red[w][(r * MT + mt) * 4 + j][lane] = f[r][mt][j];
        __syncthreads();
        for (int e = threadIdx.x; e < kTile * 64; e += kMfmaWaves * 64) {
            const int reg = e >> 6, l = e & 63;
            float sum = 0.0f;
#pragma unroll
            for (int q = 0; q < kMfmaWaves; ++q) sum += red[q][reg][l];
            const int r = reg / (MT * 4), mt = (reg >> 2) % MT, j = reg & 3;
            const int m = mt * 16 + (l >> 4) * 4 + j;
            const RowRef o = locate_row(S, (unit * R + r) * 16 + (l & 15), G);
            if (o.valid && m < M) {
                if (PREC == NVQ_W4A8) sum *= xscale[m];
                store_out(o.y, o.y_dtype, (int64_t)m * o.N + o.n, sum);
            }
        }
        __syncthreads();
    }
}

template <int PREC, int R, int MT, bool DEBUG>
int launch_one(const GemvSegs &S, int G, int M, const void *x, const float *xscale,
               hipStream_t st) {
    const int units = (S.total_rows + 16 * R - 1) / (16 * R);
    const int cap = device_cu_count() * 4;
    const dim3 grid(units < cap ? units : cap), block(kMfmaWaves * 64);
    hipLaunchKernelGGL((gemv_mfma_kernel<PREC, R, MT, DEBUG>), grid, block, 0, st, S, G, M,
                       reinterpret_cast<const char *>(x), xscale);
    NVQ_HIP_TRY(hipGetLastError());
    return NVQ_OK;
}

template <int PREC>
int launch_prec(const GemvSegs &S, int G, int M, const void *x, const float *xscale, bool debug,
                hipStream_t st) {
    const bool wide = M > 16;
    if (debug)  // accumulator dump: one row tile per workgroup
        return wide ? launch_one<PREC, 1, 2, true>(S, G, M, x, xscale, st)
                    : launch_one<PREC, 1, 1, true>(S, G, M, x, xscale, st);
    // Row tiles per workgroup: share the activation operand between as many
    // tiles as still leaves two workgroups for every compute unit.
    const int tiles = (S.total_rows + 15) / 16;
    const int want = 2 * device_cu_count();
    const int R = tiles >= 4 * want ? 4 : tiles >= 2 * want ? 2 : 1;
#define NVQ_GO(RR)                                                              \
    return wide ? launch_one<PREC, RR, 2, false>(S, G, M, x, xscale, st)       \
                : launch_one<PREC, RR, 1, false>(S, G, M, x, xscale, st)
    if (R == 4) NVQ_GO(4);
    if (R == 2) NVQ_GO(2);
    NVQ_GO(1);
#undef NVQ_GO
}

}  // namespace

bool gemv_mfma_supported(const GemvSegs &S, int K, int M) {
    if (M < 2 || M > 32 || K % 128 != 0) return false;
    for (int i = 0; i < S.nseg; ++i)
        if (!aligned(S.sc[i], 8)) return false;
    return true;
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
