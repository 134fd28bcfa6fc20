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
// weight is dequantised once per workgroup and serves eight MFMAs.  The
// activations of a pair of groups (256 rows of 128 bytes) go from global memory
// straight into LDS, 16 bytes per lane and 1 KiB per load instruction; three
// buffers, loads two pairs ahead of the multiplication, one barrier per pair.
// A row's eight 16-byte pieces are stored permuted (piece c of row r at
// position c ^ ((r / 2) % 8)): the 16 lanes of a quarter wave, reading the same
// piece of 16 consecutive rows, then touch every LDS bank once.
typedef __attribute__((address_space(3))) void *lds_void_ptr;

constexpr int kWideTokens = 256, kWideRows = 256;
constexpr int kWideBuf = kWideTokens * 128;  // bytes of one activation buffer

// s_waitcnt immediate that waits for vmcnt <= n only
constexpr int wide_vmcnt(int n) { return (n & 15) | ((n >> 4) << 14) | 0x0f70; }

template <bool F32>
__global__ __launch_bounds__(kGemmThreads) __attribute__((amdgpu_waves_per_eu(1, 1))) void
gemm_w4a16_wide_kernel(const uint4 *__restrict__ qw, const uint16_t *__restrict__ sc, int N, int G,
                       const unsigned char *__restrict__ x, int M, void *__restrict__ y) {
    __shared__ __attribute__((aligned(1024))) unsigned char xa[4 * kWideBuf];

    const int t = threadIdx.x, lane = t & 63;
    const int wave = __builtin_amdgcn_readfirstlane(t >> 6);
    const int li = lane & 31, lb = lane >> 5;
    // Tiles in token-major order, weight rows fastest.  (Giving each XCD, with its
    // own L2, a contiguous eighth of the tiles, so that its workgroups share one or
    // two token tiles, was 7 % slower; so was starting every workgroup at a
    // different place along K.)
    const int nx = (N + kWideRows - 1) / kWideRows, ny = (M + kWideTokens - 1) / kWideTokens;
    const int tile = (int)blockIdx.x;
    if (tile >= nx * ny) return;
    const int m0 = (tile / nx) * kWideTokens, n0 = (tile % nx) * kWideRows;
    const int P = (G + 1) >> 1;  // pairs of groups
    const bool odd = (G & 1) != 0;

    // Activation loads: instruction j of this wave fills rows 8 (8 wave + j) ..
    // + 7 of a buffer, lane l the position l % 8 of row l / 8 of those: piece
    // (l % 8) ^ ((row / 2) % 8) of that token's 128 bytes (rows past the last
    // token: the last token again; those results are not stored).  In the
    // missing second group of an odd last pair the first group is read again
    // (its weights count as 0).
    const unsigned char *xg[8];
    int tailfix[2];
#pragma unroll
    for (int j = 0; j < 8; ++j) {
        const int r = 8 * (8 * wave + j) + (lane >> 3);
        const int c = (lane & 7) ^ ((r >> 1) & 7);
        const int m = m0 + r < M ? m0 + r : M - 1;
        xg[j] = x + (size_t)m * (size_t)(G * 64) + 16 * c;
        if (j < 2) tailfix[j] = c >= 4 ? -64 : 0;  // c depends on j through its parity only
    }
    auto issue_a1 = [&](unsigned char *buf, int p, int j) {
        const bool fix = odd && p == P - 1;
        const unsigned char *g = xg[j] + (size_t)p * 128 + (fix ? tailfix[j & 1] : 0);
        __builtin_amdgcn_global_load_lds((const void *)g, (lds_void_ptr)(buf + (8 * wave + j) * 1024),
                                         16, 0, 0);
    };
    auto issue_a = [&](unsigned char *buf, int p) {
#pragma unroll
        for (int j = 0; j < 8; ++j) issue_a1(buf, p, j);
    };

    // The lane's weight rows, one per row tile (the last row again past the end).
    const uint4 *qrow[2];
    const uint16_t *srow[2];
#pragma unroll
    for (int rt = 0; rt < 2; ++rt) {
        const int n = n0 + wave * 64 + rt * 32 + li;
        const int nc = n < N ? n : N - 1;
        qrow[rt] = qw + (size_t)nc * (size_t)G;
        srow[rt] = sc + (size_t)nc * (size_t)G;
    }
    struct BRaw {
        uint4v w[2];
        uint32_t h[2];
        uint32_t hmask;  // 0 for the missing group of an odd last pair
    };
    // piece 0, 2: the packed weights of row tile 0, 1; piece 1, 3: their scales
    auto request_b1 = [&](BRaw &b, int p, bool live, int piece) {
        const int g = 2 * p + lb;
        const int gc = g < G ? g : G - 1;
        const int rt = piece >> 1;
        if ((piece & 1) == 0)
            asm volatile("global_load_dwordx4 %0, %1, off" : "=v"(b.w[rt]) : "v"(qrow[rt] + gc));
        else
            // Loaded in any case (a branch here would split the loop's body) and
            // masked when used.  Both as instructions: the compiler would wait for
            // every load in flight where these are used (and pack the two 16-bit
            // values into one register at the end of the loop's body, waiting for
            // them there).  The wait before the barrier covers them.
            asm volatile("global_load_ushort %0, %1, off" : "=v"(b.h[rt]) : "v"(srow[rt] + gc));
        b.hmask = (g < G && live) ? 0xffffu : 0u;
    };
    auto request_b = [&](BRaw &b, int p, bool live) {
#pragma unroll
        for (int piece = 0; piece < 4; ++piece) request_b1(b, p, live, piece);
    };

    floatx16 acc[8][2];
#pragma unroll
    for (int tt = 0; tt < 8; ++tt)
#pragma unroll
        for (int rt = 0; rt < 2; ++rt)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[tt][rt][r] = 0.0f;

    // the lane's position in a row of a buffer per MFMA step, and its row of tile 0
    int apos[4];
#pragma unroll
    for (int st = 0; st < 4; ++st) apos[st] = li * 128 + 16 * ((4 * lb + st) ^ ((li >> 1) & 7));

    // The loop is a chain of MFMA steps (four per pair of groups, 16 inputs per
    // lane half each).  Everything else is dealt between the sixteen MFMAs of a
    // step, a little after each, so that the matrix core never waits for more
    // than a few instructions: the eight LDS reads of the next step's inputs, the
    // conversion of the next step's sixteen weights (byte -> fp32, one FMA with
    // the scale, every other time the rounding of two to bf16), in step 2 the
    // unpacking of the next pair's nibbles and in step 3 the twelve global loads
    // of the pairs ahead (a load instruction can hold up the wave for tens of
    // cycles).  The step after step 3 is step 0 of the next pair.  Four buffers:
    // pair q lives in buffer q % 4; when pair p + 3 is loaded (step 3 of pair p)
    // every wave has passed the barrier of pair p and with it pair p - 1.
    struct Nibbles {  // a pair's weights of the lane: one nibble per byte, [row tile][low, high][dword]
        uint32_t d[2][2][4];
        uint32_t h[2];  // fp16 scale bits
        float m8[2];    // -8 * scale
    };
    // piece k of 10: the low and high nibbles of a dword (k < 8), the scale of a row tile
    auto unpack1 = [&](const BRaw &b, Nibbles &nb, int k) {
        if (k < 8) {
            const int rt = k >> 2, i = k & 3;
            const uint32_t d = b.w[rt][i];
            nb.d[rt][0][i] = d & 0x0f0f0f0fu;
            nb.d[rt][1][i] = (d >> 4) & 0x0f0f0f0fu;
            // the bytes are converted one by one; seen through, the compiler
            // extracts each nibble from d again with an instruction of its own
            asm("" : "+v"(nb.d[rt][0][i]));
            asm("" : "+v"(nb.d[rt][1][i]));
        } else {
            const int rt = k - 8;
            nb.h[rt] = b.h[rt] & b.hmask;
            nb.m8[rt] = -8.0f * half_bits_to_float((uint16_t)nb.h[rt]);
        }
    };
    // weight i (0..15) of MFMA step st: row tile i / 8, input i % 8 of the step
    auto weight = [&](const Nibbles &nb, int st, int i) -> float {
        const int rt = i >> 3, e = i & 7;
        const uint32_t d = nb.d[rt][st >> 1][2 * (st & 1) + (e >> 2)];
        return fmaf((float)((d >> (8 * (e & 3))) & 0xffu), half_bits_to_float((uint16_t)nb.h[rt]),
                    nb.m8[rt]);
    };
    // LDS reads are written as instructions with their own wait: before an LDS
    // read it knows of, the compiler waits for every load in flight, the loads
    // into LDS of the pairs ahead included.
    auto read_input = [&](uint32_t addr, int tt, uint4v &a) {
        switch (tt) {
#define NVQ_RD(t_) case t_: asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(a) : "v"(addr), "n"(t_ * 4096)); break;
            NVQ_RD(0) NVQ_RD(1) NVQ_RD(2) NVQ_RD(3) NVQ_RD(4) NVQ_RD(5) NVQ_RD(6) NVQ_RD(7)
#undef NVQ_RD
        }
    };
    auto arrived = [&](uint4v (&a)[8]) {
        asm volatile("s_waitcnt lgkmcnt(0)"
                     : "+v"(a[0]), "+v"(a[1]), "+v"(a[2]), "+v"(a[3]), "+v"(a[4]), "+v"(a[5]),
                       "+v"(a[6]), "+v"(a[7]));
    };
    uint4v a[2][8];
    uint32_t bo[2][2][4];  // [step parity][row tile] bf16 x 8
    BRaw bset[2];          // the packed weights of pair q wait in set q % 2 (in flight, then landed)
    Nibbles nb, nnb;       // of the pair being multiplied and of the next one

    // Step `st` of the pair in registers (a[st % 2], bo[st % 2]) while the operands
    // of step `nst` of the pair in LDS at `nbuf` with the nibbles `wn` are made.
    // extra = 1: also unpacks `bs` into nnb; extra = 2: also loads the weights of
    // pair pb into `bs` and the activations of pair pa into the buffer at abuf.
    auto step = [&](int st, uint32_t nbuf, const Nibbles &wn, int nst, int extra, BRaw &bs, int pb,
                    bool pb_live, unsigned char *abuf, int pa) {
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
            if (extra == 1 && i >= 4 && i < 14) unpack1(bs, nnb, i - 4);
            if (extra == 2 && i >= 2 && i < 6) request_b1(bs, pb, pb_live, i - 2);
            if (extra == 2 && i >= 6 && i < 14) issue_a1(abuf, pa, i - 6);
            __builtin_amdgcn_sched_barrier(0);
        }
        arrived(a[n]);
    };

    // Order of the loads, kept by compiler barriers: B(0) A(0) B(1) A(1) B(2) A(2),
    // then in step 3 of pair p: B(p + 3) A(p + 3).  Before step 2 of pair p, A(p + 1)
    // and B(p + 1) are needed; the twelve loads of B(p + 2) and A(p + 2) are the only
    // younger ones.  Pairs past the last one (an odd number of pairs is rounded up:
    // the loop takes two at a time, one per set of weight registers) read the last
    // pair again with scale 0.
#define NVQ_PIN asm volatile("" ::: "memory")
    const uint32_t xa0 = (uint32_t)(uintptr_t)xa;
    auto pair_or_last = [&](int q) { return q < P ? q : P - 1; };
    request_b(bset[0], 0, true);
    NVQ_PIN;
    issue_a(xa, 0);
    NVQ_PIN;
    request_b(bset[1], pair_or_last(1), 1 < P);
    NVQ_PIN;
    issue_a(xa + kWideBuf, pair_or_last(1));
    NVQ_PIN;
    __builtin_amdgcn_s_waitcnt(wide_vmcnt(12));
    __builtin_amdgcn_s_barrier();
    NVQ_PIN;
    asm volatile("" : "+v"(bset[0].h[0]), "+v"(bset[0].h[1]), "+v"(bset[0].w[0]), "+v"(bset[0].w[1]));
#pragma unroll
    for (int k = 0; k < 10; ++k) unpack1(bset[0], nb, k);
    NVQ_PIN;
    request_b(bset[0], pair_or_last(2), 2 < P);
    NVQ_PIN;
    issue_a(xa + 2 * kWideBuf, pair_or_last(2));
    NVQ_PIN;
#pragma unroll
    for (int tt = 0; tt < 8; ++tt) read_input(xa0 + apos[0], tt, a[0][tt]);
    {
        float prev = 0.0f;
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            const float w = weight(nb, 0, i);
            if (i & 1) bo[0][i >> 3][(i & 7) >> 1] = pack_bf16(prev, w);
            prev = w;
        }
    }
    arrived(a[0]);

    int cur = 0;  // byte offset of the buffer of pair p
    // one pair; `bs` is the set of pair p + 1 (and then of pair p + 3)
    auto pair = [&](int p, BRaw &bs) {
        const int nxt = (cur + kWideBuf) & (4 * kWideBuf - 1), fill = (cur + 3 * kWideBuf) & (4 * kWideBuf - 1);
        step(0, xa0 + cur, nb, 1, 0, bs, 0, false, xa, 0);
        step(1, xa0 + cur, nb, 2, 0, bs, 0, false, xa, 0);
        __builtin_amdgcn_s_waitcnt(wide_vmcnt(12));
        __builtin_amdgcn_s_barrier();
        NVQ_PIN;
        // the weights were loaded behind the compiler's back: no use before the wait
        asm volatile("" : "+v"(bs.h[0]), "+v"(bs.h[1]), "+v"(bs.w[0]), "+v"(bs.w[1]));
        step(2, xa0 + cur, nb, 3, 1, bs, 0, false, xa, 0);
        step(3, xa0 + nxt, nnb, 0, 2, bs, pair_or_last(p + 3), p + 3 < P, xa + fill, pair_or_last(p + 3));
        nb = nnb;
        cur = nxt;
    };
    for (int p = 0; p < P; p += 2) {
        pair(p, bset[1]);
        pair(p + 1, bset[0]);
    }
#undef NVQ_PIN
    // No load may outlive the loop: the loads into LDS must not outlive the wave, and
    // the registers of the last weight loads (the compiler does not know that they
    // are still being written) stay reserved up to this wait.
    asm volatile("s_waitcnt vmcnt(0)" ::"v"(bset[0].w[0]), "v"(bset[0].w[1]), "v"(bset[0].h[0]),
                 "v"(bset[0].h[1]), "v"(bset[1].w[0]), "v"(bset[1].w[1]), "v"(bset[1].h[0]),
                 "v"(bset[1].h[1])
                 : "memory");

    // result tile: lane (j, b) holds weight row j; register r holds token
    // 8 * (r / 4) + 4 * b + r % 4
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
    const bool wide = getenv("NVQ_GEMM_WIDE") != nullptr;
    if (wide) {
        const int64_t tiles = ((N + kWideRows - 1) / kWideRows) * ((M + kWideTokens - 1) / kWideTokens);
        const dim3 wgrid((unsigned)(((tiles + 7) / 8) * 8));
        const unsigned char *xb = reinterpret_cast<const unsigned char *>(x_bf16);
        const uint4 *qww = reinterpret_cast<const uint4 *>(qweight);
        if (y_dtype == NVQ_F32)
            hipLaunchKernelGGL(gemm_w4a16_wide_kernel<true>, wgrid, dim3(kGemmThreads), 0,
                               (hipStream_t)stream, qww, scales, (int)N, (int)(K / 32), xb, (int)M, y);
        else
            hipLaunchKernelGGL(gemm_w4a16_wide_kernel<false>, wgrid, dim3(kGemmThreads), 0,
                               (hipStream_t)stream, qww, scales, (int)N, (int)(K / 32), xb, (int)M, y);
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
