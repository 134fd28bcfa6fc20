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
// Two kernels.  The one with wide tiles (256 x 256 per workgroup, second half of
// this file) runs when K is a multiple of 256 and the output has at least 32
// such tiles; the other one, described here, takes everything else.
//
// A workgroup of four waves owns 256 tokens x 128 weight rows, a wave 128 x 64
// (4 x 2 MFMA tiles, 128 accumulator registers); a wave's dequantised operand
// serves its four token tiles.  Activations pass through LDS (rows of 128 bytes
// padded to 144: 16 lanes reading 16 bytes each then cover all 64 banks),
// double buffered, eight neighbouring threads staging a token's 128 bytes; one
// barrier per pair of groups.  The next pair's activations and packed weights
// are requested before the current pair is multiplied.
#include "nvq_internal.h"

#include <cstdlib>

namespace nvq {

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef float floatx2 __attribute__((ext_vector_type(2)));
typedef unsigned uint4v __attribute__((ext_vector_type(4)));

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


// ---- wide tiles --------------------------------------------------------------
// 256 tokens x 256 weight rows per workgroup, four waves, one per SIMD with the
// whole register file (the 8 x 2 accumulator tiles of a wave fill 256
// registers): a wave multiplies all 256 tokens by its own 64 rows, so that a
// weight is dequantised once per workgroup and serves eight MFMAs.  K must be a
// multiple of 256 (a pair of groups per step, blocks of four pairs below).
//
// Everything comes from global memory straight into LDS, 16 bytes per lane:
//  - the activations of a pair of groups (256 tokens x 128 bytes, three buffers
//    shared by the waves; 1 KiB = eight whole lines per load instruction);
//  - the packed weights of a wave's 64 rows for two pairs (64 bytes per row:
//    16 half lines per instruction, two buffers per wave) and their scales for
//    four pairs (16 bytes per row, two buffers per wave).  Loaded by the lane
//    that needs them (lane i = row i, 16 bytes of one group) a load instruction
//    touches 32 lines for 1 KiB and the wave stands still while it is taken
//    apart: with the weight loads pointed at one row the kernel ran 25-30 %
//    faster, which is what the detour through LDS is for.
// A row's 16-byte pieces are stored permuted so that the 16 lanes of a quarter
// wave, reading the same piece of 16 consecutive rows, touch every LDS bank once:
// piece c of activation row r at position c ^ ((r / 2) % 8), piece c of weight
// row r at position c ^ ((r / 4) % 4).
typedef __attribute__((address_space(3))) void *lds_void_ptr;

constexpr int kWideTokens = 256, kWideRows = 256;
constexpr int kWideBuf = kWideTokens * 128;  // bytes of one activation buffer
constexpr int kWideBw = 64 * 64;             // a wave's packed weights of two pairs
constexpr int kWideBs = 64 * 16;             // a wave's scales of four pairs
constexpr int kWideLds = 3 * kWideBuf + 4 * 2 * (kWideBw + kWideBs);

// s_waitcnt immediate that waits for vmcnt <= n only
constexpr int wide_vmcnt(int n) { return (n & 15) | ((n >> 4) << 14) | 0x0f70; }

template <bool F32>
__global__ __launch_bounds__(kGemmThreads) __attribute__((amdgpu_waves_per_eu(1, 1))) void
gemm_w4a16_wide_kernel(const unsigned char *__restrict__ qw, const unsigned char *__restrict__ sc,
                       int N, int G, const unsigned char *__restrict__ x, int M,
                       void *__restrict__ y) {
    __shared__ __attribute__((aligned(1024))) unsigned char lds[kWideLds];
    unsigned char *const xa = lds;
    const int t = threadIdx.x, lane = t & 63;
    const int wave = __builtin_amdgcn_readfirstlane(t >> 6);
    unsigned char *const bw = lds + 3 * kWideBuf + wave * 2 * kWideBw;
    unsigned char *const bs = lds + 3 * kWideBuf + 4 * 2 * kWideBw + wave * 2 * kWideBs;
    const int li = lane & 31, lb = lane >> 5;
    // Tiles in token-major order, weight rows fastest.  (Giving each XCD, with its
    // own L2, a contiguous eighth of the tiles, so that its workgroups share one or
    // two token tiles, changed the time by -1..+3 %; starting every workgroup at a
    // different place along K made it 3-7 % slower; reading the inputs from LDS two
    // steps ahead instead of one changed nothing.)
    const int nx = (N + kWideRows - 1) / kWideRows;
    const int tile = (int)blockIdx.x;
    const int m0 = (tile / nx) * kWideTokens, n0 = (tile % nx) * kWideRows;
    const int P = G >> 1;  // pairs of groups, a multiple of 4

    // Activation loads: instruction j of this wave fills rows 8 (8 wave + j) ..
    // + 7 of a buffer, lane l the position l % 8 of row l / 8 of those (rows past
    // the last token: the last token again; those results are not stored).
    // Addresses are a base common to the wave plus a 32-bit offset per lane (the
    // form a load instruction takes without any address arithmetic in the lanes).
    const unsigned char *const xbase = x + (size_t)m0 * (size_t)(G * 64);
    uint32_t xo[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) {
        const int r = 8 * (8 * wave + j) + (lane >> 3);
        const int c = (lane & 7) ^ ((r >> 1) & 7);
        const int rc = m0 + r < M ? r : M - 1 - m0;
        xo[j] = (uint32_t)rc * (uint32_t)(G * 64) + 16u * (uint32_t)c;
    }
    auto issue_a1 = [&](unsigned char *buf, int p, int j) {
        __builtin_amdgcn_global_load_lds((const void *)(xbase + (size_t)p * 128 + xo[j]),
                                         (lds_void_ptr)(buf + (8 * wave + j) * 1024), 16, 0, 0);
    };
    // Weight loads: instruction j fills rows 16 j .. + 15 of a weight buffer, lane l
    // the position l % 4 of row l / 4 of those (rows past the last one: the last one
    // again).  Scale load: lane l the 16 bytes of row l.
    const int nw = n0 + wave * 64 < N ? n0 + wave * 64 : N - 1;  // the wave's first row
    const unsigned char *const qbase = qw + (size_t)nw * (size_t)(G * 16);
    const unsigned char *const sbase = sc + (size_t)nw * (size_t)(G * 2);
    uint32_t qo[4], so;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const int r = 16 * j + (lane >> 2);
        const int c = (lane & 3) ^ ((r >> 2) & 3);
        const int rc = nw + r < N ? r : N - 1 - nw;
        qo[j] = (uint32_t)rc * (uint32_t)(G * 16) + 16u * (uint32_t)c;
    }
    so = (uint32_t)(nw + lane < N ? lane : N - 1 - nw) * (uint32_t)(G * 2);
    // block b2 = pairs 2 b2, 2 b2 + 1 into weight buffer `sel`; block b4 = pairs 4 b4 .. + 3
    auto issue_bw1 = [&](int b2, int sel, int j) {
        __builtin_amdgcn_global_load_lds((const void *)(qbase + (size_t)b2 * 64 + qo[j]),
                                         (lds_void_ptr)(bw + sel * kWideBw + j * 1024), 16, 0, 0);
    };
    auto issue_bs = [&](int b4, int sel) {
        __builtin_amdgcn_global_load_lds((const void *)(sbase + (size_t)b4 * 16 + so),
                                         (lds_void_ptr)(bs + sel * kWideBs), 16, 0, 0);
    };

    floatx16 acc[8][2];
#pragma unroll
    for (int tt = 0; tt < 8; ++tt)
#pragma unroll
        for (int rt = 0; rt < 2; ++rt)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[tt][rt][r] = 0.0f;

    // The lane's LDS positions.  Activations: row li of a token tile, piece 4 lb +
    // st in MFMA step st.  Weights: row li of a row tile, the group lb of the first
    // pair of a block (the second pair: the position ^ 2); scales: row li, group lb
    // of the first pair of a block of four.
    const uint32_t xa0 = (uint32_t)(uintptr_t)xa;
    uint32_t apos[4];
#pragma unroll
    for (int st = 0; st < 4; ++st) apos[st] = li * 128 + 16 * ((4 * lb + st) ^ ((li >> 1) & 7));
    const uint32_t bwpos = (uint32_t)(uintptr_t)bw + li * 64 + 16 * (lb ^ ((li >> 2) & 3));
    const uint32_t bspos = (uint32_t)(uintptr_t)bs + li * 16 + 2 * lb;

    // The loop is a chain of MFMA steps (four per pair of groups, 16 inputs per
    // lane half each).  Everything else is dealt between the sixteen MFMAs of a
    // step, a little after each, so that the matrix core never waits for more
    // than a few instructions: the eight LDS reads of the next step's inputs, the
    // conversion of the next step's sixteen weights (byte -> fp32, one FMA with
    // the scale, every other time the rounding of two to bf16), in step 1 the LDS
    // reads of the next pair's packed weights, in step 2 their unpacking and in
    // step 3 the loads from global memory.  The step after step 3 is step 0 of the
    // next pair.  LDS accesses are written as instructions with their own waits:
    // before an LDS access it knows of, the compiler waits for every load in flight.
    struct BRaw {  // the lane's packed weights and scales of a pair, per row tile
        uint4v w[2];
        uint32_t h[2];
    };
    struct Nibbles {  // one nibble per byte, [row tile][low, high][dword]; the high ones times 16
        uint32_t d[2][2][4];
        float s[2][2];  // scale for the low nibbles, scale / 16 for the high ones
        float m8[2];    // -8 * scale
    };
    // piece k of 10: the low and high nibbles of a dword (k < 8), the scale of a row tile
    auto unpack1 = [&](const BRaw &b, Nibbles &nb, int k) {
        if (k < 8) {
            const int rt = k >> 2, i = k & 3;
            const uint32_t d = b.w[rt][i];
            nb.d[rt][0][i] = d & 0x0f0f0f0fu;
            nb.d[rt][1][i] = d & 0xf0f0f0f0u;
            // the bytes are converted one by one; seen through, the compiler
            // extracts each nibble from d again with an instruction of its own
            asm("" : "+v"(nb.d[rt][0][i]));
            asm("" : "+v"(nb.d[rt][1][i]));
        } else {
            const int rt = k - 8;
            nb.s[rt][0] = half_bits_to_float((uint16_t)b.h[rt]);
            nb.s[rt][1] = 0.0625f * nb.s[rt][0];  // exact
            nb.m8[rt] = -8.0f * nb.s[rt][0];
        }
    };
    // weight i (0..15) of MFMA step st: row tile i / 8, input i % 8 of the step
    auto weight = [&](const Nibbles &nb, int st, int i) -> float {
        const int rt = i >> 3, e = i & 7;
        const uint32_t d = nb.d[rt][st >> 1][2 * (st & 1) + (e >> 2)];
        return fmaf((float)((d >> (8 * (e & 3))) & 0xffu), nb.s[rt][st >> 1], nb.m8[rt]);
    };
    auto read_input = [&](uint32_t addr, int tt, uint4v &a) {
        switch (tt) {
#define NVQ_RD(t_) case t_: asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(a) : "v"(addr), "n"(t_ * 4096)); break;
            NVQ_RD(0) NVQ_RD(1) NVQ_RD(2) NVQ_RD(3) NVQ_RD(4) NVQ_RD(5) NVQ_RD(6) NVQ_RD(7)
#undef NVQ_RD
        }
    };
    // piece 0, 1: the packed weights of row tile 0, 1 (32 rows = 2 KiB further); 2, 3: the scales
    auto read_b1 = [&](uint32_t waddr, uint32_t saddr, BRaw &b, int piece) {
        switch (piece) {
            case 0: asm volatile("ds_read_b128 %0, %1" : "=v"(b.w[0]) : "v"(waddr)); break;
            case 1: asm volatile("ds_read_b128 %0, %1 offset:2048" : "=v"(b.w[1]) : "v"(waddr)); break;
            case 2: asm volatile("ds_read_u16 %0, %1" : "=v"(b.h[0]) : "v"(saddr)); break;
            case 3: asm volatile("ds_read_u16 %0, %1 offset:512" : "=v"(b.h[1]) : "v"(saddr)); break;
        }
    };
    uint4v a[2][8];
    uint32_t bo[2][2][4];  // [step parity][row tile] bf16 x 8
    BRaw braw;             // of the next pair
    Nibbles nba, nbb;      // of the pair being multiplied and of the next one, in turn
    auto arrived = [&](uint4v (&v)[8]) {
        asm volatile("s_waitcnt lgkmcnt(0)"
                     : "+v"(v[0]), "+v"(v[1]), "+v"(v[2]), "+v"(v[3]), "+v"(v[4]), "+v"(v[5]),
                       "+v"(v[6]), "+v"(v[7]), "+v"(braw.w[0]), "+v"(braw.w[1]), "+v"(braw.h[0]),
                       "+v"(braw.h[1]));
    };

    // The loads from global memory that belong to pair p: the activations of pair p +
    // 3 (eight instructions), for even p before them the weight block p / 2 + 2
    // (four), for p % 4 == 0 before those the scale block p / 4 + 1 (one): a list of
    // `kind` = 13, 8, 12 or 8 instructions.  They are dealt over four steps (step 3
    // of pair p, where the buffer of pair p becomes free, and steps 0..2 of pair p +
    // 1), a quarter of the list each, one every fourth MFMA: a load instruction holds
    // up the wave that issues it while the address unit is busy, and the four waves
    // of a workgroup issue theirs at the same time.
    auto load_op = [&](int kind, int quarter, int m, unsigned char *abuf, int pa, int b2, int wsel,
                       int b4, int ssel) {
        const int first = kind == 13 ? (quarter == 0 ? 0 : 1 + 3 * quarter) : (kind / 4) * quarter;
        const int count = kind == 13 ? (quarter == 0 ? 4 : 3) : kind / 4;
        if (m >= count) return;
        int k = first + m;
        if (kind == 13) {
            if (k == 0) {
                issue_bs(b4, ssel);
                return;
            }
            k -= 1;
        }
        if (kind >= 12) {
            if (k < 4) {
                issue_bw1(b2, wsel, k);
                return;
            }
            k -= 4;
        }
        issue_a1(abuf, pa, k);
    };

    // Step `st` of the pair in registers (a[st % 2], bo[st % 2]) while the operands
    // of step `nst` of the pair at `nbuf` with the nibbles `wn` are made.  extra =
    // 1: also reads the next pair's packed weights from LDS (at waddr / saddr);
    // extra = 2: also unpacks them into wnext.  Every step issues a quarter of a list
    // of loads (kind, quarter): the activations of pair pa into abuf, the weight
    // block b2 into buffer wsel, the scale block b4 into buffer ssel.
    auto step = [&](int st, uint32_t nbuf, const Nibbles &wn, Nibbles &wnext, int nst, int extra,
                    uint32_t waddr, uint32_t saddr, int kind, int quarter, unsigned char *abuf, int pa,
                    int b2, int wsel, int b4, int ssel) {
        const int c = st & 1, n = c ^ 1;
        const uint32_t addr = nbuf + apos[nst];
        float prev = 0.0f;
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            const int tt = i >> 1, rt = i & 1;
            acc[tt][rt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(
                __builtin_bit_cast(bf16x8, a[c][tt]),
                __builtin_bit_cast(bf16x8, make_uint4(bo[c][rt][0], bo[c][rt][1], bo[c][rt][2], bo[c][rt][3])),
                acc[tt][rt], 0, 0, 0);
            if (i < 8) read_input(addr, i, a[n][i]);
            const float w = weight(wn, nst, i);
            if (i & 1) bo[n][i >> 3][(i & 7) >> 1] = pack_bf16(prev, w);
            prev = w;
            if (extra == 1 && i >= 8 && i < 12) read_b1(waddr, saddr, braw, i - 8);
            if (extra == 2 && i >= 4 && i < 14) unpack1(braw, wnext, i - 4);
            if ((i & 3) == 2) load_op(kind, quarter, i >> 2, abuf, pa, b2, wsel, b4, ssel);
            __builtin_amdgcn_sched_barrier(0);
        }
        arrived(a[n]);
    };

#define NVQ_PIN asm volatile("" ::: "memory")
    // Before the loop: the activations of pairs 0 and 1 and the first quarter of
    // those of pair 2 (the rest follows in steps 0..2 of pair 0, as in every turn of
    // the loop), the weights of pairs 0..3 and their scales; pair 0 unpacked and its
    // first operands in registers.
    const int last2 = (P >> 1) - 1, last4 = (P >> 2) - 1;
    auto pair_or_last = [&](int q) { return q < P ? q : P - 1; };
    issue_bs(0, 0);
#pragma unroll
    for (int j = 0; j < 4; ++j) issue_bw1(0, 0, j);
#pragma unroll
    for (int j = 0; j < 4; ++j) issue_bw1(1 < last2 ? 1 : last2, 1, j);
#pragma unroll
    for (int q = 0; q < 2; ++q)
#pragma unroll
        for (int j = 0; j < 8; ++j) issue_a1(xa + q * kWideBuf, pair_or_last(q), j);
#pragma unroll
    for (int j = 0; j < 2; ++j) issue_a1(xa + 2 * kWideBuf, pair_or_last(2), j);
    NVQ_PIN;
    __builtin_amdgcn_s_waitcnt(wide_vmcnt(0));
    __builtin_amdgcn_s_barrier();
    NVQ_PIN;
#pragma unroll
    for (int piece = 0; piece < 4; ++piece) read_b1(bwpos, bspos, braw, piece);
#pragma unroll
    for (int tt = 0; tt < 8; ++tt) read_input(xa0 + apos[0], tt, a[0][tt]);
    arrived(a[0]);
#pragma unroll
    for (int k = 0; k < 10; ++k) unpack1(braw, nba, k);
    {
        float prev = 0.0f;
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            const float w = weight(nba, 0, i);
            if (i & 1) bo[0][i >> 3][(i & 7) >> 1] = pack_bf16(prev, w);
            prev = w;
        }
    }

    // Four pairs per turn (a block of scales, two blocks of weights); pair p = 4 k +
    // i has a list of 13, 8, 12, 8 loads for i = 0..3.  The wait before step 3 of pair
    // p lets the list of pair p - 1 (begun in step 3 of that pair, ended in step 2 of
    // this one) stay in flight and ends all older loads: A(p + 1), read right after the
    // barrier, is in the list of pair p - 2, and the weights and scales of pair p + 2,
    // read from LDS in step 1 of pair p + 1, are in that of pair p - 2 or older.
    int cur = 0, prv = 2 * kWideBuf;  // byte offsets of the activation buffers of pairs p and p - 1
    int ssel = 0;                     // scale buffer of the pairs 4 k .. 4 k + 3
    for (int p = 0; p < P; p += 4) {
        // i_: place of the pair in the turn; kprev_, kind_: the lists of pairs p - 1 and p
#define NVQ_PAIR(i_, kprev_, kind_, nb, nnb)                                                     \
    do {                                                                                         \
        const int q_ = (i_) + 1; /* the next pair's place in its blocks */                       \
        const uint32_t waddr_ = (bwpos + ((q_ >> 1) & 1) * kWideBw) ^ ((q_ & 1) * 32);           \
        const uint32_t saddr_ = bspos + (((q_ >> 2) ? ssel ^ 1 : ssel)) * kWideBs + (q_ & 3) * 4; \
        const int nxt_ = cur + kWideBuf == 3 * kWideBuf ? 0 : cur + kWideBuf;                    \
        /* the list of the pair before: its activations go to that pair's buffer */             \
        const int pp_ = p + (i_) - 1;                                                            \
        const int pa_ = pair_or_last(pp_ + 3);                                                   \
        const int pb2_ = (pp_ >> 1) + 2 < last2 ? (pp_ >> 1) + 2 : last2;                        \
        const int pb4_ = (p >> 2) + 1 < last4 ? (p >> 2) + 1 : last4;                            \
        const int pws_ = (((i_) + 3) >> 1) & 1; /* ((i - 1) / 2) % 2 for i = 1..3 */             \
        step(0, xa0 + cur, nb, nnb, 1, 0, 0, 0, kprev_, 1, xa + prv, pa_, pb2_, pws_, pb4_,      \
             ssel ^ 1);                                                                          \
        step(1, xa0 + cur, nb, nnb, 2, 1, waddr_, saddr_, kprev_, 2, xa + prv, pa_, pb2_, pws_,  \
             pb4_, ssel ^ 1);                                                                    \
        step(2, xa0 + cur, nb, nnb, 3, 2, 0, 0, kprev_, 3, xa + prv, pa_, pb2_, pws_, pb4_,      \
             ssel ^ 1);                                                                          \
        __builtin_amdgcn_s_waitcnt(wide_vmcnt(kprev_));                                          \
        __builtin_amdgcn_s_barrier();                                                            \
        NVQ_PIN;                                                                                 \
        {                                                                                        \
            const int b2_ = ((p + (i_)) >> 1) + 2;                                               \
            step(3, xa0 + nxt_, nnb, nb, 0, 0, 0, 0, kind_, 0, xa + cur, pair_or_last(p + (i_) + 3), \
                 b2_ < last2 ? b2_ : last2, ((i_) >> 1) & 1, pb4_, ssel ^ 1);                    \
        }                                                                                        \
        NVQ_PIN;                                                                                 \
        prv = cur;                                                                               \
        cur = nxt_;                                                                              \
    } while (0)
        NVQ_PAIR(0, 8, 13, nba, nbb);
        NVQ_PAIR(1, 13, 8, nbb, nba);
        NVQ_PAIR(2, 8, 12, nba, nbb);
        NVQ_PAIR(3, 12, 8, nbb, nba);
#undef NVQ_PAIR
        ssel ^= 1;
    }
#undef NVQ_PIN
    // no load into LDS may outlive the wave
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");

    // Result tile: lane (j, b) holds weight row j; register r holds token
    // 8 * (r / 4) + 4 * b + r % 4 of a 32 x 32 tile.
    if (!F32 && (N & 7) == 0 && (reinterpret_cast<uintptr_t>(y) & 15) == 0) {
        // bf16 results pass through LDS (free now), so that they leave as whole
        // 128-byte lines, 16 bytes per lane, instead of 2 bytes per lane: a wave's
        // 256 tokens x 64 rows in 32 KiB, a row of 128 bytes per token with its
        // 16-byte pieces permuted (piece c at position c ^ ((token / 4) % 8): the two
        // halves of the wave write tokens four apart).
        __builtin_amdgcn_s_barrier();  // every wave has left the loop: nothing reads or fills LDS
        unsigned char *const out = lds + wave * (kWideTokens * 128);
#pragma unroll
        for (int tt = 0; tt < 8; ++tt)
#pragma unroll
            for (int rt = 0; rt < 2; ++rt)
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int tok = tt * 32 + 8 * (r >> 2) + 4 * lb + (r & 3);
                    const int nl = rt * 32 + li;
                    const int pos = (nl >> 3) ^ ((tok >> 2) & 7);
                    *reinterpret_cast<uint16_t *>(out + tok * 128 + pos * 16 + (nl & 7) * 2) =
                        float_to_bf16_bits(acc[tt][rt][r]);
                }
        // the wave reads back what it wrote itself
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
        const int nb0 = n0 + wave * 64;
#pragma unroll 4
        for (int i = 0; i < 32; ++i) {
            const int idx = i * 64 + lane;
            const int tok = idx >> 3, pos = idx & 7;
            const int c = pos ^ ((tok >> 2) & 7);
            const uint4 v = *reinterpret_cast<const uint4 *>(out + tok * 128 + pos * 16);
            const int m = m0 + tok, n = nb0 + c * 8;
            if (m < M && n < N)
                *reinterpret_cast<uint4 *>(reinterpret_cast<uint16_t *>(y) + (size_t)m * N + n) = v;
        }
        return;
    }
#pragma unroll
    for (int tt = 0; tt < 8; ++tt)
#pragma unroll
        for (int rt = 0; rt < 2; ++rt) {
            const int n = n0 + wave * 64 + rt * 32 + li;
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int m = m0 + tt * 32 + 8 * (r >> 2) + 4 * lb + (r & 3);
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
    // The wide tiles need K % 256 == 0 and enough tiles to occupy the machine; the
    // environment variable NVQ_GEMM_TILE (wide | narrow) overrides the choice where
    // both kernels can run (used by the tests to reach both on small shapes).
    const int64_t tiles = ((N + kWideRows - 1) / kWideRows) * ((M + kWideTokens - 1) / kWideTokens);
    // (its loads move 16 bytes of scales at a time: the scales 16-byte aligned, too)
    const bool can_wide = (K % 256) == 0 && aligned(scales, 16);
    bool wide = can_wide && tiles >= 32;
    if (const char *force = getenv("NVQ_GEMM_TILE")) {
        if (force[0] == 'w' && can_wide) wide = true;
        if (force[0] == 'n') wide = false;
    }
    if (wide) {
        if (tiles > (int64_t)0x7fffffff) return NVQ_ERR_SHAPE;
        const dim3 wgrid((unsigned)tiles);
        const unsigned char *xb = reinterpret_cast<const unsigned char *>(x_bf16);
        const unsigned char *sb = reinterpret_cast<const unsigned char *>(scales);
        if (y_dtype == NVQ_F32)
            hipLaunchKernelGGL(gemm_w4a16_wide_kernel<true>, wgrid, dim3(kGemmThreads), 0,
                               (hipStream_t)stream, qweight, sb, (int)N, (int)(K / 32), xb, (int)M, y);
        else
            hipLaunchKernelGGL(gemm_w4a16_wide_kernel<false>, wgrid, dim3(kGemmThreads), 0,
                               (hipStream_t)stream, qweight, sb, (int)N, (int)(K / 32), xb, (int)M, y);
        NVQ_HIP_TRY(hipGetLastError());
        return NVQ_OK;
    }
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
