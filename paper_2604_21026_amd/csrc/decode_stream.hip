// Persistent streaming kernel for a whole decode step at batch 1.
//
// Why: one decode step is a chain of ~130 phases (q/k/v, o, gate/up, down per
// block) of 1-10 us each at HBM speed.  Launching a kernel per phase leaves
// the memory system idle at every boundary; the paper removes its launch
// bubbles with graph capture (paragraph "CUDA graph capture for decode").
// Here the whole layer list runs in ONE launch, and, because weights never
// depend on activations, every wave keeps fetching the weights of the coming
// phases while the current phase is being set up.
//
// Structure.  One workgroup per compute unit, all co-resident: kStreamWaves
// streaming waves (three per SIMD) and one loader wave.  Each streaming wave
// owns a contiguous range of rows in every phase (possibly none: a phase too
// short to give every wave a dozen chunks deals its rows in larger units to
// fewer waves, and a wave passes the phases that give it nothing without a
// look, by a skip table the host prepares; a wave issues one instruction per
// 6-10 cycles, and taking part in a phase costs it some 250 of them) and sees
// its work as one flat sequence of 1 KiB chunks (64 groups x 16 B of one
// weight row) across all phases.  Chunks are fetched with non-temporal global->LDS loads into a
// per-wave ring of kSlots slots and consumed in order; a slot is refilled as
// soon as its chunk has been taken out, independent of phase boundaries, and
// the ring is first filled before anything else happens in the kernel.  The
// fp16 scales travel the same way (one 2-byte load per lane and chunk).  Ring
// loads are the only vector-memory loads of a wave on the fast path, issued
// two per chunk, so the number of loads in flight behind a chunk is a
// compile-time constant and one `s_waitcnt vmcnt(n)` tells when it has landed.
//
// Activations.  A phase's input is needed by every wave in a prepared form,
// the "image": int8 codes (W4A8) or bf16 values (W4A16) laid out in planes of
// G x 16 bytes, plus per group the constant of the deferred offset correction
// (-8*sum(codes) or -136*sum(x)), plus the scale(s).  For a phase that depends
// on no earlier phase the image is built ONCE per step, in global memory, by
// one workgroup in a prologue (instead of once per compute unit) and announced
// through a flag word of its own; there is no grid-wide barrier.  The loader
// wave copies images from there into a circular LDS area up to kLookahead
// phases ahead and announces them through an LDS word; streaming waves report
// the phases they have finished through one LDS word each, which tells the
// loader when a region may be overwritten.  On this path the streaming waves
// never meet at a barrier, so they may drift apart and absorb each other's
// jitter.  A dependent phase builds its image in LDS from the raw input after
// its wait, all streaming waves together, with workgroup barriers.
//
// A lane meets the same few groups in every row of a phase (group i*64+lane
// for chunk i of the row), so for rows of up to four chunks it takes their
// activations out of the image once per phase and keeps them in registers;
// only longer rows read them from LDS per chunk.  Reading them per chunk made
// LDS, not HBM, the bound of the W4A16 phases (64 bytes per lane and chunk).
//
// Two or three streaming waves share a SIMD and the hardware favours the
// oldest whenever several can issue, which lets it refill its ring sooner and
// leaves the others behind; the wave priority therefore rotates from phase to
// phase.
//
// Ordering.  The host marks, per phase, the latest earlier phase whose
// buffers it conflicts with.  Such a phase takes its input only after every
// workgroup has published that phase (one flag word per workgroup, no
// atomics), and its input is read after the wait instead of being streamed
// ahead.  A bounded spin turns a stuck wait (e.g. the grid not co-resident)
// into an error status instead of a hang.
//
// Mail.  Where a phase's input is exactly the bf16 output of one earlier phase
// (the o projection into the next norm, gate and up into SiLU-multiply, down
// into the next block: every link of a real decode step), flags are not used at
// all.  The producing waves post each result a second time as a 32-bit word
// that carries the tag of this walk next to the bf16 value, with write-through
// stores and without waiting for them; the consuming waves poll those words,
// each its share of the vector, until all of them carry the tag.  Every word is
// its own flag, so no store has to be waited for, no fence and no workgroup
// barrier stand on the producer's side, and the consumer's wait and its fetch
// of the data are one and the same trip to memory.  (With flags a dependent
// phase cost 14 us: the producer drains its loads to learn that its stores are
// done, meets its workgroup, writes back its L2 and raises the flag; the
// consumer polls 256 flags, invalidates its L2, meets its workgroup and only
// then asks for the data.)
#include <type_traits>

#include "decode_stream.h"
#include "transform.h"

namespace nvq {

namespace {

typedef __attribute__((address_space(3))) void *lds_void_ptr;
// The phase table is read through the constant address space: it does not
// change during the kernel, and only such loads are certain to become scalar
// loads (a vector load would join the ring's vmcnt queue and be waited for
// with vmcnt(0)).
typedef const __attribute__((address_space(4))) StreamPhase CPhase;
typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2_t __attribute__((ext_vector_type(2)));

constexpr int kSlots = 3;                 // ring slots per wave (1 KiB weights + 256 B scales):
                                          // 36 KiB in flight per compute unit.  4, 5 and 6 stream
                                          // no faster on 1B-, 3B- and 8B-shaped steps (2 is 1-4 %
                                          // slower), and a dependent chain, which computes at the
                                          // pace of its slowest wave, is 3 % faster with 3 than 6
constexpr int kOpsPerChunk = 2;            // scale load + weight load
constexpr int kXChunkElems = 512;          // bf16 values per input chunk
constexpr int kMaxXShare = (kStreamMaxK / kXChunkElems + kStreamWaves - 1) / kStreamWaves;  // 4

constexpr uint32_t kSpinLimit = 4u << 20;  // polls before a wait gives up (seconds)
constexpr uint32_t kMailSpinLimit = 1u << 20;  // likewise for mail (a poll is a trip to memory)
constexpr int kLookahead = 3;              // phases the loader wave may run ahead (6 and 12: no faster)

// s_waitcnt immediate that waits for vmcnt <= n only (gfx9 encoding:
// vmcnt[3:0] | expcnt[6:4] | lgkmcnt[11:8] | vmcnt[5:4] at [15:14]).
constexpr int vmcnt_imm(int n) { return (n & 15) | ((n >> 4) << 14) | 0x0f70; }

struct Shared {
    uint4 ring[kStreamWaves][kSlots][64];
    uint32_t sring[kStreamWaves][kSlots][64];  // one dword per lane: zero-extended fp16 scale
    uint4 area[kStreamImageArea / 16];  // activation images of consecutive phases (circular)
    float amax_part[kStreamWaves];
    float sumsq_part[kStreamWaves];
    uint32_t progress[kStreamWaves];  // phases finished by each streaming wave
    uint32_t img_ready;               // images of phases < img_ready are in LDS
    int abort;
};

// ---- LDS access as instructions ---------------------------------------------
// While global->LDS loads are in flight the compiler guards every LDS access
// it knows of with a full vmcnt(0) wait, which would drain the ring each time.
// The kernel's LDS traffic is therefore written as instructions, with explicit
// waits.
__device__ __forceinline__ uint32_t lds_addr(const void *p) {
    return (uint32_t)(uintptr_t)p;  // LDS pointers are 32-bit offsets
}
__device__ __forceinline__ void lds_barrier() {
    // every LDS access issued so far has completed before anyone passes
    asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
}
__device__ __forceinline__ uint4 lds_read16(uint32_t addr) {
    u32x4_t v;
    asm volatile("ds_read_b128 %0, %1\n\ts_waitcnt lgkmcnt(0)" : "=v"(v) : "v"(addr) : "memory");
    return make_uint4(v.x, v.y, v.z, v.w);
}
__device__ __forceinline__ uint32_t lds_read4(uint32_t addr) {
    uint32_t v;
    asm volatile("ds_read_b32 %0, %1\n\ts_waitcnt lgkmcnt(0)" : "=v"(v) : "v"(addr) : "memory");
    return v;
}
// an LDS word that every lane reads from the same address, as a scalar: the
// compiler cannot see through the instruction, and control flow that depended
// on a per-lane value would push the wave-uniform stream state into vector
// registers
__device__ __forceinline__ uint32_t lds_read4_uniform(uint32_t addr) {
    return (uint32_t)__builtin_amdgcn_readfirstlane((int)lds_read4(addr));
}
__device__ __forceinline__ void lds_write4(uint32_t addr, uint32_t v) {
    asm volatile("ds_write_b32 %0, %1" : : "v"(addr), "v"(v) : "memory");
}
__device__ __forceinline__ void lds_write8(uint32_t addr, uint32_t lo, uint32_t hi) {
    u32x2_t v = {lo, hi};
    asm volatile("ds_write_b64 %0, %1" : : "v"(addr), "v"(v) : "memory");
}
__device__ __forceinline__ void lds_write16(uint32_t addr, const uint4 &d) {
    u32x4_t v = {d.x, d.y, d.z, d.w};
    asm volatile("ds_write_b128 %0, %1" : : "v"(addr), "v"(v) : "memory");
}

// ---- cross-lane helpers (data-parallel-primitive moves, no LDS traffic) ------
template <int CTRL, int ROW_MASK>
__device__ __forceinline__ float dpp_move(float x) {
    return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), CTRL,
                                                                 ROW_MASK, 0xf, false));
}
// total valid in lane 63
__device__ __forceinline__ float wave_sum_to_lane63(float v) {
    v += dpp_move<0xb1, 0xf>(v);   // quad_perm [1,0,3,2]
    v += dpp_move<0x4e, 0xf>(v);   // quad_perm [2,3,0,1]
    v += dpp_move<0x141, 0xf>(v);  // row_half_mirror
    v += dpp_move<0x140, 0xf>(v);  // row_mirror: every lane of a row of 16 holds the row sum
    v += dpp_move<0x142, 0xa>(v);  // row_bcast15 into rows 1 and 3
    v += dpp_move<0x143, 0xc>(v);  // row_bcast31 into rows 2 and 3
    return v;
}
// maximum of non-negative values, valid in lane 63 (0 is the neutral element)
__device__ __forceinline__ float wave_max_to_lane63(float v) {
    v = fmaxf(v, dpp_move<0xb1, 0xf>(v));
    v = fmaxf(v, dpp_move<0x4e, 0xf>(v));
    v = fmaxf(v, dpp_move<0x141, 0xf>(v));
    v = fmaxf(v, dpp_move<0x140, 0xf>(v));
    v = fmaxf(v, dpp_move<0x142, 0xa>(v));
    v = fmaxf(v, dpp_move<0x143, 0xc>(v));
    return v;
}
// sum / max over each aligned group of four lanes, valid in all four
__device__ __forceinline__ float quad_sum(float v) {
    v += dpp_move<0xb1, 0xf>(v);
    v += dpp_move<0x4e, 0xf>(v);
    return v;
}
__device__ __forceinline__ int quad_sum(int v) {
    v += __builtin_amdgcn_update_dpp(0, v, 0xb1, 0xf, 0xf, false);
    v += __builtin_amdgcn_update_dpp(0, v, 0x4e, 0xf, 0xf, false);
    return v;
}
__device__ __forceinline__ float quad_max(float v) {
    v = fmaxf(v, dpp_move<0xb1, 0xf>(v));
    v = fmaxf(v, dpp_move<0x4e, 0xf>(v));
    return v;
}

// Byte p of the wave's row of the skip table, as a scalar load.
typedef const __attribute__((address_space(4))) uint32_t CSkipWord;
__device__ __forceinline__ int phase_skip(CSkipWord *row, int p) {
    return (int)((row[p >> 2] >> ((p & 3) * 8)) & 0xffu);
}

// ---- the issue side: where the wave's next chunk comes from -------------------
// All fields are wave-uniform.  A run is a sequence of chunks at a constant
// pointer stride: consecutive weight rows inside one matrix (a single row
// when K is no multiple of 2048).
struct Issue {
    const char *q;      // next chunk: 64 x 16 bytes
    const char *s;      // its 64 scales (2 bytes each)
    uint32_t qstep, sstep;  // pointer advance per chunk, in bytes (unsigned: two scalar adds)
    int left;           // chunks left in the run
    int tail;           // valid lanes in the run's last chunk (64 = all)
    int p;              // phase of the run
    int part;           // 0: row range of phase p not yet set up
    int row, row_stop;  // weight rows of phase p not yet turned into runs
};

__device__ __forceinline__ void issue_next_run(Issue &c, CPhase *tab, CSkipWord *skips, int nphase,
                                               int w, int gw, const uint4 *dummy) {
    for (;;) {
        if (c.p >= nphase) {
            // past the last phase: dummy chunks keep the load count constant
            c.q = reinterpret_cast<const char *>(dummy);
            c.s = reinterpret_cast<const char *>(dummy);
            c.qstep = c.sstep = 0;
            c.left = 1 << 30;
            c.tail = 64;
            return;
        }
        CPhase &ph = tab[c.p];
        if (c.part == 0) {
            c.part = 1;
            int first, count;
            stream_wave_rows(ph.rows_base, ph.rows_extra, ph.rows_rot,
                             ph.spread ? w * (int)gridDim.x + (gw - w) / kStreamWaves : gw,
                             (int)gridDim.x * kStreamWaves, first, count);
            c.row = first * ph.row_unit;
            c.row_stop = c.row + count * ph.row_unit;  // (the last unit of a phase may be short)
            c.row_stop = c.row_stop < ph.total_rows ? c.row_stop : ph.total_rows;
        }
        if (c.row < c.row_stop) {
            int first = 0, end = ph.row_end[0];
            const uint4 *q = ph.qw[0];
            const uint16_t *s = ph.sc[0];
#pragma unroll
            for (int k = 1; k < kMaxSeg; ++k)
                if (k < ph.nseg && c.row >= ph.row_end[k - 1]) {
                    first = ph.row_end[k - 1];
                    end = ph.row_end[k];
                    q = ph.qw[k];
                    s = ph.sc[k];
                }
            // rows in pairs: an even number of rows of 96 groups is a whole number
            // of chunks (segments hold an even number of rows, so does the range)
            const bool pairs = ph.pair_stream != 0;
            const bool ragged = (ph.G & 63) != 0 && !pairs;
            int rows = (c.row_stop < end ? c.row_stop : end) - c.row;
            if (ragged) rows = 1;
            const int64_t off = (int64_t)(c.row - first) * ph.G;
            c.q = reinterpret_cast<const char *>(q + off);
            c.s = reinterpret_cast<const char *>(s + off);
            c.qstep = 64 * 16;
            c.sstep = 64 * 2;
            c.left = pairs ? rows / 2 * (2 * kStreamPairG / 64) : rows * ph.gpl;
            c.tail = ragged ? ph.G - (ph.gpl - 1) * 64 : 64;
            c.row += rows;
            return;
        }
        ++c.p;
        if (c.p < nphase) c.p += phase_skip(skips, c.p);  // phases without rows for this wave
        c.part = 0;
    }
}

// Issue the two loads of the next chunk into ring slot `slot`.
__device__ __forceinline__ void issue_chunk(Issue &c, CPhase *tab, CSkipWord *skips, int nphase,
                                            Shared &sh, int w, int gw, int slot, int lane,
                                            const uint4 *dummy) {
    const int valid = c.left == 1 ? c.tail : 64;
    if (valid >= 64) {
        __builtin_amdgcn_global_load_lds((const void *)(c.s + lane * 2),
                                         (lds_void_ptr)&sh.sring[w][slot][0], 2, 0, 2);
        __builtin_amdgcn_global_load_lds((const void *)(c.q + lane * 16),
                                         (lds_void_ptr)&sh.ring[w][slot][0], 16, 0, 2);
    } else {
        // lanes past the end issue nothing; lane 0 is always valid, so both
        // loads are issued and the load count stays exact
        if (lane < valid)
            __builtin_amdgcn_global_load_lds((const void *)(c.s + lane * 2),
                                             (lds_void_ptr)&sh.sring[w][slot][0], 2, 0, 2);
        if (lane < valid)
            __builtin_amdgcn_global_load_lds((const void *)(c.q + lane * 16),
                                             (lds_void_ptr)&sh.ring[w][slot][0], 16, 0, 2);
    }
    c.q += c.qstep;
    c.s += c.sstep;
    if (--c.left == 0) issue_next_run(c, tab, skips, nphase, w, gw, dummy);
}

// ---- arithmetic of one chunk ----------------------------------------------------
__device__ __forceinline__ int dot_w4a8(const u32x4_t &w, const u32x4_t &xlo, const u32x4_t &xhi,
                                        int acc) {
#pragma unroll
    for (int d = 0; d < 4; ++d) {
        const uint32_t lo = w[d] & 0x0f0f0f0fu;         // elements 4d .. 4d+3
        const uint32_t hi = (w[d] >> 4) & 0x0f0f0f0fu;  // elements 16+4d .. 16+4d+3
        acc = __builtin_amdgcn_sdot4((int)lo, (int)xlo[d], acc, false);
        acc = __builtin_amdgcn_sdot4((int)hi, (int)xhi[d], acc, false);
    }
    return acc;
}

typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
__device__ __forceinline__ float dot2_bf16(uint32_t a, uint32_t b, float c) {
    return __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2_t, a),
                                           __builtin_bit_cast(bf16x2_t, b), c, false);
}

// x[k] holds elements 8k .. 8k+7 of the group as four bf16 pairs.  A nibble n
// under the high byte 0x43 is the bf16 number 128 + n; `off` = -136 * sum(x)
// removes the constant.  Two accumulator chains keep the dots independent.
__device__ __forceinline__ float dot_w4a16(const u32x4_t &w, const u32x4_t (&x)[4], float off) {
    constexpr uint32_t kMagic = 0x43434343u;
    float a0 = off, a1 = 0.0f;
#pragma unroll
    for (int d = 0; d < 4; ++d) {
        const uint32_t lo = w[d] & 0x0f0f0f0fu;
        const uint32_t hi = (w[d] >> 4) & 0x0f0f0f0fu;
        // byte permute: selector 0-3 picks a byte of the second operand, 4-7 of the first
        const uint32_t l01 = __builtin_amdgcn_perm(kMagic, lo, 0x04010400u);
        const uint32_t l23 = __builtin_amdgcn_perm(kMagic, lo, 0x04030402u);
        const uint32_t h01 = __builtin_amdgcn_perm(kMagic, hi, 0x04010400u);
        const uint32_t h23 = __builtin_amdgcn_perm(kMagic, hi, 0x04030402u);
        // elements 4d..4d+3 live in x[d/2] words 2(d%2), 2(d%2)+1; 16+4d.. in x[2+d/2]
        a0 = dot2_bf16(l01, x[d >> 1][2 * (d & 1)], a0);
        a1 = dot2_bf16(l23, x[d >> 1][2 * (d & 1) + 1], a1);
        a0 = dot2_bf16(h01, x[2 + (d >> 1)][2 * (d & 1)], a0);
        a1 = dot2_bf16(h23, x[2 + (d >> 1)][2 * (d & 1) + 1], a1);
    }
    return a0 + a1;
}

// ---- activation images ---------------------------------------------------------
// Byte layout of an image (identical in global memory and in LDS):
//   W4A8 : plane 0 (codes of elements 0..15 of each group, G x 16 B), plane 1
//          (elements 16..31), aux[G] int32 = -8*sum(codes), then for per-group
//          scales xsg[G] fp32, then the per-token scale (fp32, 16 B reserved);
//   W4A16: planes 0..3 (elements 8q..8q+7 as bf16, G x 16 B each), aux[G] fp32
//          = -136*sum(x).
template <bool PER_GROUP>
struct ImgLayout {
    int aux, xsg, stok;  // byte offsets
    __device__ __forceinline__ ImgLayout(bool w4a8, int G) {
        aux = (w4a8 ? 32 : 64) * G;
        xsg = aux + 4 * G;
        stok = xsg + (PER_GROUP ? 4 * G : 0);
    }
};

struct LdsWriter {
    uint32_t base;
    __device__ __forceinline__ void w4(int off, uint32_t v) const { lds_write4(base + off, v); }
    __device__ __forceinline__ void w8(int off, uint32_t lo, uint32_t hi) const {
        lds_write8(base + off, lo, hi);
    }
    __device__ __forceinline__ void w16(int off, const uint4 &v) const {
        lds_write16(base + off, v);
    }
};
struct GlobalWriter {
    char *base;
    __device__ __forceinline__ void w4(int off, uint32_t v) const {
        *reinterpret_cast<uint32_t *>(base + off) = v;
    }
    __device__ __forceinline__ void w8(int off, uint32_t lo, uint32_t hi) const {
        *reinterpret_cast<uint2 *>(base + off) = make_uint2(lo, hi);
    }
    __device__ __forceinline__ void w16(int off, const uint4 &v) const {
        *reinterpret_cast<uint4 *>(base + off) = v;
    }
};

__device__ __forceinline__ float chunk_absmax(const uint4 &v) {
    const uint32_t wv[4] = {v.x, v.y, v.z, v.w};
    float a = 0.0f;
#pragma unroll
    for (int d = 0; d < 4; ++d) {
        a = fmaxf(a, fabsf(bf16_bits_to_float(wv[d] & 0xffffu)));
        a = fmaxf(a, fabsf(bf16_bits_to_float(wv[d] >> 16)));
    }
    return a;
}

// One lane's eight consecutive bf16 values (a quarter of group g; the four
// lanes of a group sit next to each other) go into the image.  Quantisation
// follows the paper's appendix "F16 -> Q8 Activation Quantization":
// q = round(x / s) clamped to [-127, 127], round half to even, IEEE division.
template <bool PER_GROUP, class Writer>
__device__ __forceinline__ void image_put(const Writer &wr, const ImgLayout<PER_GROUP> &L,
                                          bool w4a8, int G, int g, int lane, const uint4 &raw,
                                          float s_tok) {
    const int quarter = lane & 3;
    const bool valid = g < G;
    const uint32_t wv[4] = {raw.x, raw.y, raw.z, raw.w};
    if (w4a8) {
        float s = s_tok;
        if (PER_GROUP) {
            s = quad_max(chunk_absmax(raw)) / 127.0f;
            if (valid && quarter == 0) wr.w4(L.xsg + g * 4, __float_as_uint(s));
        }
        // One division per scale instead of one per value: t = x * fl(1 / s) is within
        // 2^-15 of the correctly rounded quotient fl(x / s) (|x / s| <= 127: two
        // roundings of 2^-24 relative, and the quotient's own), so unless t lies within
        // 2^-14 of a half-integer, rounding t gives the integer that rounding the
        // quotient gives; where it does (an exact tie, say) the lane divides after all.
        // A scale too small for its reciprocal takes the division for every value.
        const bool by_reciprocal = s >= 0x1p-100f;
        const float inv_s = by_reciprocal ? 1.0f / s : 0.0f;
        // (one test for the lane's eight values: the lanes with a value near a tie redo
        // all eight by division, one lane in a thousand)
        float x[8], r[8];
        bool redo = !by_reciprocal;
#pragma unroll
        for (int d = 0; d < 4; ++d) {
            x[2 * d] = bf16_bits_to_float(wv[d] & 0xffffu);
            x[2 * d + 1] = bf16_bits_to_float(wv[d] >> 16);
        }
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const float t = x[i] * inv_s;
            r[i] = rintf(t);
            redo = redo || fabsf(t - r[i]) > 0.5f - 0x1p-14f;
        }
        if (redo) {
#pragma unroll
            for (int i = 0; i < 8; ++i) r[i] = rintf(x[i] / s);
        }
        uint32_t out[2] = {0, 0};
        int qsum = 0;
#pragma unroll
        for (int d = 0; d < 4; ++d) {
            int q0 = 0, q1 = 0;
            if (s != 0.0f) {
                q0 = (int)fminf(fmaxf(r[2 * d], -127.0f), 127.0f);
                q1 = (int)fminf(fmaxf(r[2 * d + 1], -127.0f), 127.0f);
            }
            qsum += q0 + q1;
            out[d >> 1] |= ((uint32_t)(q0 & 0xff) | ((uint32_t)(q1 & 0xff) << 8)) << (16 * (d & 1));
        }
        qsum = quad_sum(qsum);
        if (valid) {
            wr.w8((quarter >> 1) * (G * 16) + g * 16 + (quarter & 1) * 8, out[0], out[1]);
            if (quarter == 0) wr.w4(L.aux + g * 4, (uint32_t)(-8 * qsum));
        }
    } else {
        float part = 0.0f;
#pragma unroll
        for (int d = 0; d < 4; ++d) part = dot2_bf16(0x3f803f80u, wv[d], part);
        part = quad_sum(part);
        if (valid) {
            wr.w16(quarter * (G * 16) + g * 16, raw);
            if (quarter == 0) wr.w4(L.aux + g * 4, __float_as_uint(-136.0f * part));
        }
    }
}

// Optional per-phase timestamps (100 MHz wall clock) taken by wave 0 of
// workgroup 0; slot meanings are documented with nvq_plan_trace.
constexpr int kTraceSlots = 8;
struct Trace {
    unsigned long long *buf;  // nullptr: off
    int wgs, nphase;          // workgroups that record (the first `wgs`), phases per workgroup
};
__device__ __forceinline__ void trace_mark(const Trace &trace, int wg, int w, int lane, int p,
                                           int slot) {
    if (trace.buf && wg < trace.wgs && w == 0 && lane == 0)
        trace.buf[((size_t)wg * trace.nphase + p) * kTraceSlots + slot] = wall_clock64();
}

// ---- mail --------------------------------------------------------------------
// Post eight consecutive bf16 values (piece j of 512, lane's share) in every
// replica of a mailbox.
__device__ __forceinline__ void mail_post8_one(uint32_t *mail, uint32_t stride, int r, int j,
                                               int lane, const uint4 &v, uint32_t tag_hi) {
    const u32x4_t a = {tag_hi | (v.x & 0xffffu), tag_hi | (v.x >> 16), tag_hi | (v.y & 0xffffu),
                       tag_hi | (v.y >> 16)};
    const u32x4_t b = {tag_hi | (v.z & 0xffffu), tag_hi | (v.z >> 16), tag_hi | (v.w & 0xffffu),
                       tag_hi | (v.w >> 16)};
    uint32_t *p = mail + (size_t)r * stride + (size_t)j * 512 + lane * 4;
    // (the s_nop: a store of more than 8 bytes reads its data registers a few cycles after it
    // issues, and the compiler, which does not see into the statement, may let the next
    // instruction overwrite them)
    asm volatile("global_store_dwordx4 %0, %1, off sc1\n\t"
                 "global_store_dwordx4 %0, %2, off offset:1024 sc1\n\ts_nop 3"
                 :
                 : "v"(p), "v"(a), "v"(b)
                 : "memory");
}

// The same in every replica.
__device__ __forceinline__ void mail_post8(uint32_t *mail, uint32_t stride, int j, int lane,
                                           const uint4 &v, uint32_t tag_hi) {
    for (int r = 0; r < kMailReplicas; ++r) mail_post8_one(mail, stride, r, j, lane, v, tag_hi);
}

// Word of value v in a mailbox (see StreamPhase).
__device__ __forceinline__ int mail_word(int v) {
    return (v & ~511) + ((v >> 2) & 1) * 256 + ((v >> 3) & 63) * 4 + (v & 3);
}

// Collect this wave's pieces (w, w + kStreamWaves, ...) of one or two K-value
// operands from their mailboxes (mail1 may be nullptr): poll until every word
// carries the tag.  The loads bypass the caches that other compute units do not
// share (device scope) and a word is written whole, so a word with the right tag
// holds this walk's value.  A lane asks again only for what it is still missing.
// Returns false if the wait
// was given up (abort raised, status set) or another wave raised abort; the
// outputs are then undefined.
__device__ __forceinline__ uint32_t mail_bad(const u32x4_t &a, const u32x4_t &b, uint32_t tag_hi) {
    return ((a.x ^ tag_hi) | (a.y ^ tag_hi) | (a.z ^ tag_hi) | (a.w ^ tag_hi) | (b.x ^ tag_hi) |
            (b.y ^ tag_hi) | (b.z ^ tag_hi) | (b.w ^ tag_hi)) >> 16;
}
// low halves of two words side by side
__device__ __forceinline__ uint4 mail_pack(const u32x4_t &a, const u32x4_t &b) {
    return make_uint4(__builtin_amdgcn_perm(a.y, a.x, 0x05040100u),
                      __builtin_amdgcn_perm(a.w, a.z, 0x05040100u),
                      __builtin_amdgcn_perm(b.y, b.x, 0x05040100u),
                      __builtin_amdgcn_perm(b.w, b.z, 0x05040100u));
}

// NP pieces of NO operands at a time (the registers of a wave hold three
// piece-operands in flight next to everything else, not six).
template <int NP, int NO, int NK>
__device__ __forceinline__ bool mail_poll(const uint32_t *mail0, const uint32_t *mail1, int K,
                                          int nxc, int w, int lane, uint32_t tag_hi,
                                          uint4 (&out0)[NK], uint4 (&out1)[NK], uint32_t abort_a,
                                          uint32_t *status, int where) {
    // bit NO * k + o of `need`: this lane's share of piece k of operand o has not come yet
    uint32_t need = 0;
#pragma unroll
    for (int k = 0; k < NP; ++k) {
        const int j = w + k * kStreamWaves;
        int idx = j * 64 + lane;
        asm volatile("" : "+v"(idx));
        if (j < nxc && idx < K / 8) need |= ((1u << NO) - 1u) << (NO * k);
    }
    uint32_t spins = 0;
    while (__any(need != 0)) {
        u32x4_t a[NP][NO], b[NP][NO];
#pragma unroll
        for (int k = 0; k < NP; ++k) {
#pragma unroll
            for (int o = 0; o < NO; ++o) {
                a[k][o] = b[k][o] = u32x4_t{0, 0, 0, 0};
                if (need & (1u << (NO * k + o))) {
                    const uint32_t *p =
                        (o == 0 ? mail0 : mail1) + (size_t)(w + k * kStreamWaves) * 512 + lane * 4;
                    asm volatile("global_load_dwordx4 %0, %2, off sc1\n\t"
                                 "global_load_dwordx4 %1, %2, off offset:1024 sc1"
                                 : "+v"(a[k][o]), "+v"(b[k][o])
                                 : "v"(p)
                                 : "memory");
                }
            }
        }
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
#pragma unroll
        for (int k = 0; k < NP; ++k) {
#pragma unroll
            for (int o = 0; o < NO; ++o) {
                asm volatile("" : "+v"(a[k][o]), "+v"(b[k][o]));  // nothing is used before that wait
                const uint32_t bit = 1u << (NO * k + o);
                if ((need & bit) && mail_bad(a[k][o], b[k][o], tag_hi) == 0) {
                    need &= ~bit;
                    (o == 0 ? out0[k] : out1[k]) = mail_pack(a[k][o], b[k][o]);
                }
            }
        }
        if (!__any(need != 0)) break;
        if (lds_read4_uniform(abort_a)) return false;
        if (++spins > kMailSpinLimit) {
            if (lane == 0) {
                lds_write4(abort_a, 1u);
                __hip_atomic_store(status, 5u | ((uint32_t)where << 8), __ATOMIC_RELAXED,
                                   __HIP_MEMORY_SCOPE_AGENT);
            }
            return false;
        }
        __builtin_amdgcn_s_sleep(1);
    }
    return true;
}

template <int NK>
__device__ __forceinline__ bool mail_fetch(const uint32_t *mail0, const uint32_t *mail1, int K,
                                           int nxc, int w, int lane, uint32_t tag_hi,
                                           uint4 (&out0)[NK], uint4 (&out1)[NK], uint32_t abort_a,
                                           uint32_t *status, int where, const Trace &trace,
                                           int wg) {
    if (nxc <= kStreamWaves && mail1)  // one piece per wave: both operands at once
        return mail_poll<1, 2>(mail0, mail1, K, nxc, w, lane, tag_hi, out0, out1, abort_a, status,
                               where);
    if (!mail_poll<NK, 1>(mail0, nullptr, K, nxc, w, lane, tag_hi, out0, out1, abort_a, status,
                          where))
        return false;
    trace_mark(trace, wg, w, lane, where / 2, 4);  // (operands fetched one after the other)
    return !mail1 || mail_poll<NK, 1>(mail1, nullptr, K, nxc, w, lane, tag_hi, out1, out0, abort_a,
                                      status, where + 1);
}

// Build the image of phase `ph` from its raw input, all waves of the workgroup
// together: wave w handles the 512-value pieces w, w + waves, ...  The phase's
// input transform (RMSNorm with residual add, SiLU-multiply; paper: kernel
// table) is applied on the way, so it costs no launch and no pass over memory;
// `h_wg`: this workgroup's number for the dealing of the residual sum's stores (-1:
// it stores all of it).  Operands that
// have a mailbox (MAIL) are polled out of it instead of being loaded.  With
// `entry_barrier` (phases built after a wait) the workgroup meets once after the
// operands have arrived: from then on every wave has left the previous phase
// (the image region may be written) and all see the same abort word; false is
// returned if it is set.  The caller guarantees that sh.amax_part and
// sh.sumsq_part are free; up to two more barriers are used inside (sum of
// squares for RMSNorm; absmax exchange for W4A8 with a per-token scale).
template <bool PER_GROUP, bool MAIL, class Writer>
__device__ __forceinline__ bool image_build(const Writer &wr, CPhase &ph, Shared &sh, int w,
                                            int lane, int h_wg, bool entry_barrier,
                                            uint32_t tag_hi, uint32_t mail_stride, uint32_t abort_a,
                                            uint32_t *status, int p, const Trace &trace, int wg) {
    const int in_op = ph.in_op;
    if (w >= kStreamWaves) {  // the loader wave only keeps the barrier count
        if (entry_barrier) {
            lds_barrier();
            if (lds_read4_uniform(abort_a)) return false;
        }
        if (in_op == NVQ_IN_RMSNORM) lds_barrier();
        if (ph.precision == NVQ_W4A8 && !PER_GROUP) lds_barrier();
        return true;
    }
    const bool w4a8 = ph.precision == NVQ_W4A8;
    const int G = ph.G, K = ph.K;
    const ImgLayout<PER_GROUP> L(w4a8, G);
    const int nxc = (K + kXChunkElems - 1) / kXChunkElems;
    const uint4 *x = reinterpret_cast<const uint4 *>(ph.x);
    const uint4 *x2 = reinterpret_cast<const uint4 *>(ph.x2);
    uint4 xsh[kMaxXShare], x2sh[kMaxXShare];
    float ss = 0.0f;
    // All requests first (the input, then the second operand of the transform), so
    // that they are in flight together: issued piece by piece between the uses, a
    // wave's two or three pieces cost it two or three trips to memory in a row.
    const bool second = in_op == NVQ_IN_SILU_MUL || (in_op == NVQ_IN_RMSNORM && x2 != nullptr);
    const uint32_t *mail_x = nullptr, *mail_x2 = nullptr;
    if constexpr (MAIL) {
        // the replica of this workgroup's XCD
        const size_t mine = (size_t)(wg & (kMailReplicas - 1)) * mail_stride;
        mail_x = ph.mail_x ? ph.mail_x + mine : nullptr;
        mail_x2 = second && ph.mail_x2 ? ph.mail_x2 + mine : nullptr;
    }
#pragma unroll
    for (int k = 0; k < kMaxXShare; ++k) {
        const int j = w + k * kStreamWaves;
        int idx = j * 64 + lane;
        asm volatile("" : "+v"(idx));  // computed here, not kept through the kernel
        xsh[k] = make_uint4(0, 0, 0, 0);
        if (!mail_x && j < nxc && idx < K / 8) xsh[k] = x[idx];
    }
#pragma unroll
    for (int k = 0; k < kMaxXShare; ++k) {
        const int j = w + k * kStreamWaves;
        int idx = j * 64 + lane;
        asm volatile("" : "+v"(idx));
        x2sh[k] = make_uint4(0, 0, 0, 0);
        if (second && !mail_x2 && j < nxc && idx < K / 8) x2sh[k] = x2[idx];
    }
    if constexpr (MAIL) {
        // (both at once if both come by mail; a result of false shows in the abort word)
        if (mail_x)
            mail_fetch(mail_x, mail_x2, K, nxc, w, lane, tag_hi, xsh, x2sh, abort_a, status, 2 * p,
                       trace, wg);
        else if (mail_x2)
            mail_fetch(mail_x2, nullptr, K, nxc, w, lane, tag_hi, x2sh, xsh, abort_a, status,
                       2 * p + 1, trace, wg);
    }
    // with mail the norm weights are requested as soon as the operands have come (not
    // before: the registers are needed for the wait), so that they arrive while the
    // workgroup meets and adds up the squares
    uint4 gsh[MAIL ? kMaxXShare : 1];
    if constexpr (MAIL) {
        const uint4 *gamma = reinterpret_cast<const uint4 *>(ph.gamma);
#pragma unroll
        for (int k = 0; k < kMaxXShare; ++k) {
            const int j = w + k * kStreamWaves;
            int idx = j * 64 + lane;
            asm volatile("" : "+v"(idx));
            gsh[k] = make_uint4(0, 0, 0, 0);
            if (in_op == NVQ_IN_RMSNORM && j < nxc && idx < K / 8) gsh[k] = gamma[idx];
        }
    }
    if (entry_barrier) {
        trace_mark(trace, wg, w, lane, p, 5);  // this wave's share of the operands has arrived
        lds_barrier();
        if (lds_read4_uniform(abort_a)) return false;
        trace_mark(trace, wg, w, lane, p, 3);  // ... and everybody's
    }
#pragma unroll
    for (int k = 0; k < kMaxXShare; ++k) {
        const int j = w + k * kStreamWaves;
        int idx = j * 64 + lane;
        asm volatile("" : "+v"(idx));
        if (j < nxc && idx < K / 8) {
            if (in_op == NVQ_IN_SILU_MUL) {
                xsh[k] = silu_mul_bf16x8(xsh[k], x2sh[k]);
            } else if (in_op == NVQ_IN_RMSNORM) {
                if (x2) {
                    xsh[k] = add_bf16x8(xsh[k], x2sh[k]);
                    if (ph.h_out) {
                        // Who stores the sum: the one workgroup that builds the image (h_wg
                        // < 0: prologue), else the work is dealt out, piece j to workgroup
                        // 8 j for the caller's buffer and to workgroups 8 j + r for replica
                        // r of the mailbox (one workgroup doing all of it finished every
                        // such phase 2 us behind the others, which then waited for it)
                        const int nwg = (int)gridDim.x;
                        int r = h_wg - j * kMailReplicas % nwg;
                        r = r < 0 ? r + nwg : r;
                        if (h_wg < 0 || r == 0) reinterpret_cast<uint4 *>(ph.h_out)[idx] = xsh[k];
                        if constexpr (MAIL) {
                            if (ph.mail_h) {
                                if (h_wg < 0)
                                    mail_post8(ph.mail_h, mail_stride, j, lane, xsh[k], tag_hi);
                                else if (r < kMailReplicas)
                                    mail_post8_one(ph.mail_h, mail_stride, r, j, lane, xsh[k],
                                                   tag_hi);
                            }
                        }
                    }
                }
                ss += sumsq_bf16x8(xsh[k]);
            }
        }
    }
    if (in_op == NVQ_IN_RMSNORM) {
        ss = wave_sum_to_lane63(ss);
        if (lane == 63) lds_write4(lds_addr(&sh.sumsq_part[w]), __float_as_uint(ss));
        lds_barrier();
        float tot = 0.0f;
#pragma unroll
        for (int k = 0; k < kStreamWaves; k += 4) {
            const uint4 a = lds_read16(lds_addr(&sh.sumsq_part[k]));
            tot += __uint_as_float(a.x);
            tot += __uint_as_float(a.y);
            tot += __uint_as_float(a.z);
            tot += __uint_as_float(a.w);
        }
        const float r = rms_scale(tot, K, ph.eps);
        // (without mail, requesting the norm weights together with the input: 16 more
        // live registers here and no gain, they come out of the L2)
        const uint4 *gamma = reinterpret_cast<const uint4 *>(ph.gamma);
#pragma unroll
        for (int k = 0; k < kMaxXShare; ++k) {
            const int j = w + k * kStreamWaves;
            const int idx = j * 64 + lane;
            if (j < nxc && idx < K / 8)
                xsh[k] = scale_bf16x8(xsh[k], r, MAIL ? gsh[MAIL ? k : 0] : gamma[idx]);
        }
    }
    float amax = 0.0f;
#pragma unroll
    for (int k = 0; k < kMaxXShare; ++k) amax = fmaxf(amax, chunk_absmax(xsh[k]));
    float s_tok = 0.0f;
    if (w4a8 && !PER_GROUP) {
        amax = wave_max_to_lane63(amax);
        if (lane == 63) lds_write4(lds_addr(&sh.amax_part[w]), __float_as_uint(amax));
        lds_barrier();
        float m = 0.0f;
#pragma unroll
        for (int k = 0; k < kStreamWaves; k += 4) {
            const uint4 a = lds_read16(lds_addr(&sh.amax_part[k]));
            m = fmaxf(m, fmaxf(fmaxf(__uint_as_float(a.x), __uint_as_float(a.y)),
                               fmaxf(__uint_as_float(a.z), __uint_as_float(a.w))));
        }
        s_tok = m / 127.0f;
        if (w == 0 && lane == 0) wr.w4(L.stok, __float_as_uint(s_tok));
    }
#pragma unroll
    for (int k = 0; k < kMaxXShare; ++k) {
        const int j = w + k * kStreamWaves;
        if (j < nxc)
            image_put<PER_GROUP>(wr, L, w4a8, G, j * 16 + (lane >> 2), lane, xsh[k], s_tok);
    }
    return true;
}

// ---- per-wave stream state ---------------------------------------------------------
struct Stream {
    Issue ic;
    uint32_t slot;  // ring slot of the next chunk in stream order
};

// Wave 0: spin until every workgroup's flag has reached `target`.
__device__ __forceinline__ bool wait_flags(const uint32_t *flags, int nwg, uint32_t target,
                                           int lane) {
    uint32_t spins = 0;
    for (;;) {
        bool all = true;
        for (int f0 = 0; f0 < nwg; f0 += 256) {  // four independent loads per lane
            uint32_t v[4];
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                int f = f0 + j * 64 + lane;
                // (opaque, so that the four addresses are computed here and not kept in
                // registers through the whole kernel)
                asm volatile("" : "+v"(f));
                v[j] = f < nwg ? __hip_atomic_load(flags + f, __ATOMIC_RELAXED,
                                                   __HIP_MEMORY_SCOPE_AGENT)
                               : target;
            }
#pragma unroll
            for (int j = 0; j < 4; ++j) all = all && (int32_t)(v[j] - target) >= 0;
        }
        if (__all(all)) return true;
        if (++spins > kSpinLimit) return false;
        __builtin_amdgcn_s_sleep(1);
    }
}

// PAIRS: the table has phases whose rows are streamed in pairs (pair_stream).  A
// kernel of its own, because the mere presence of that path costs the others
// some 7 % on lists of many short phases (the compiler's register assignment
// for the code they share).
// MAIL: some phase posts or reads mail; likewise a kernel of its own.
template <bool PER_GROUP, bool PAIRS, bool MAIL>
__global__ __launch_bounds__(kStreamThreads, 1) void decode_stream_kernel(
    const StreamPhase *__restrict__ tab_generic, const uint8_t *__restrict__ skips_generic,
    int nphase, int nimages, uint32_t *__restrict__ flags, uint32_t *__restrict__ status, uint32_t flag_base,
    const uint4 *__restrict__ dummy, unsigned long long *__restrict__ trace_buf, int trace_wgs,
    uint32_t mail_tag_hi, uint32_t mail_stride) {
    const Trace trace = {trace_buf, trace_wgs, nphase};
    __shared__ Shared sh;
    CPhase *tab = (CPhase *)tab_generic;
    // wave index, made provably wave-uniform; wave 0 also talks to the other workgroups
    const int w = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int lane = threadIdx.x & 63;
    const int wg = blockIdx.x;
    const int nwg = gridDim.x;
    // The wave's place in the two orders rows are dealt in (StreamPhase::spread).
    // For the dealing the workgroups are counted XCD by XCD (workgroup b runs on XCD
    // b mod 8): the compute units of an XCD then stream neighbouring parts of a
    // matrix (8B step 0.655 -> 0.645 ms).
    const int wgd = (nwg & 7) == 0 ? (wg & 7) * (nwg >> 3) + (wg >> 3) : wg;
    const int gw = wgd * kStreamWaves + w;
    const int gw_spread = w * nwg + wgd;
    const uint32_t abort_a = lds_addr(&sh.abort);
    if (threadIdx.x == 0) lds_write4(abort_a, 0u);
    trace_mark(trace, wg, w, lane, 0, 5);  // kernel entered

    // The streaming waves request their first chunks at once: weights depend on
    // nothing, so the ring fills while the prologue below prepares the images.
    // this wave's row of the skip table (the loader wave has none and looks at every phase)
    CSkipWord *skips = (CSkipWord *)(skips_generic + (size_t)(w < kStreamWaves ? gw : 0) *
                                                         (size_t)stream_skip_stride(nphase));
    // the workgroup's row behind the waves' rows: byte p != 0 = no wave of it works in phase p
    CSkipWord *wg_passes =
        (CSkipWord *)(skips_generic + ((size_t)nwg * kStreamWaves + (size_t)wgd) *
                                          (size_t)stream_skip_stride(nphase));
    Stream st;
    st.ic.p = 0;
    st.ic.part = 0;
    st.ic.left = 0;
    st.slot = 0;
    if (w < kStreamWaves) {
        st.ic.p = phase_skip(skips, 0);
        issue_next_run(st.ic, tab, skips, nphase, w, gw, dummy);
        for (int u = 0; u < kSlots; ++u)  // fill the ring
            issue_chunk(st.ic, tab, skips, nphase, sh, w, gw, u, lane, dummy);
    }

    // ---- prologue: images of the phases that depend on no earlier phase, one
    // ---- workgroup per phase, each announced through the phase's flag word as
    // ---- soon as it is stored (the loader waves wait for the images they copy,
    // ---- nobody waits for all of them)
    uint32_t *const img_flags = flags + kStreamImageFlags;
    auto flag_copy = [&](int r) -> uint32_t * {
        return r == 0 ? flags : flags + kStreamFlagCopies + (r - 1) * kStreamMaxWg;
    };

    if (nimages > 0) {
        for (int p = wg; p < nphase; p += nwg) {
            CPhase &ph = tab[p];
            if (ph.img) {
                const GlobalWriter wr = {reinterpret_cast<char *>(const_cast<uint4 *>(ph.img))};
                image_build<PER_GROUP, MAIL>(wr, ph, sh, w, lane, -1, false, mail_tag_hi, mail_stride,
                                             abort_a, status, p, trace, wg);
                __builtin_amdgcn_s_waitcnt(vmcnt_imm(0));  // this wave's image stores have completed
                lds_barrier();                             // (and sh.amax_part may be reused)
                if (w == 0) {
                    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "agent");
                    if (lane == 0)
                        __hip_atomic_store(img_flags + p, flag_base + 1u, __ATOMIC_RELAXED,
                                           __HIP_MEMORY_SCOPE_AGENT);
                }
            }
        }
    }
    trace_mark(trace, wg, w, lane, 0, 3);  // prologue done
    const uint32_t area_base = lds_addr(sh.area);
    const uint32_t progress_a = lds_addr(&sh.progress[0]);
    const uint32_t ready_a = lds_addr(&sh.img_ready);
    if (threadIdx.x < kStreamWaves) lds_write4(progress_a + threadIdx.x * 4, 0u);
    if (threadIdx.x == 0) lds_write4(ready_a, 0u);
    lds_barrier();

    if (w == kStreamWaves) {
        // ================= loader wave =================
        // Copies prepared images into LDS ahead of the streaming waves and
        // mirrors every workgroup barrier they execute.
        int q = 0;         // first phase whose image has not been dealt with
        int pending = -1;  // phase whose image has been requested but not yet announced
        // The requested image has landed: announce it.
        auto flush = [&]() {
            if (pending >= 0) {
                __builtin_amdgcn_s_waitcnt(vmcnt_imm(0));
                if (lane == 0) lds_write4(ready_a, (uint32_t)(pending + 1));
                pending = -1;
            }
        };
        // Has the prologue of some workgroup stored the image of phase i yet?  The
        // answer is needed for every image once; lane j looks at phase i + j, and
        // everything up to the first missing image is remembered.  Blocks (bounded)
        // until phase i itself is stored; false on abort.
        int stored = 0;  // the images of all phases < stored are known to be stored
        auto image_stored = [&](int i) -> bool {
            uint32_t spins = 0;
            while (i >= stored) {
                flush();  // (its loads would otherwise be waited for with the flag loads)
                const int j = stored + lane;
                bool ok = true;
                if (j < nphase && tab_generic[j].img != nullptr)
                    ok = __hip_atomic_load(img_flags + j, __ATOMIC_RELAXED,
                                           __HIP_MEMORY_SCOPE_AGENT) == flag_base + 1u;
                const uint64_t missing = ~__builtin_amdgcn_ballot_w64(ok);
                const int run = missing ? __builtin_ctzll(missing) : 64;
                if (run > 0) {
                    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");
                    stored += run;
                    continue;
                }
                if (lds_read4_uniform(abort_a)) return false;
                if (++spins > kSpinLimit) {
                    lds_write4(abort_a, 1u);
                    __hip_atomic_store(status, 2u | ((uint32_t)i << 8), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                    return false;
                }
                __builtin_amdgcn_s_sleep(4);
            }
            return true;
        };
        // Request the image of independent phase q (blocks until its LDS region
        // is free: every wave has finished phase img_need) and announce the one
        // requested before it, so that two images are in flight.  False on abort.
        auto load_image = [&]() -> bool {
            CPhase &pq = tab[q];
            const uint32_t need = (uint32_t)(pq.img_need + 1);
            uint32_t spins = 0;
            for (;;) {
                uint32_t m = 0xffffffffu;
#pragma unroll
                for (int k = 0; k < kStreamWaves; k += 4) {
                    const uint4 a = lds_read16(progress_a + 4 * k);
                    m = m < a.x ? m : a.x;
                    m = m < a.y ? m : a.y;
                    m = m < a.z ? m : a.z;
                    m = m < a.w ? m : a.w;
                }
                if ((uint32_t)__builtin_amdgcn_readfirstlane((int)m) >= need) break;
                flush();  // the waves may be waiting for exactly that image
                if (lds_read4_uniform(abort_a)) return false;
                if (++spins > kSpinLimit) {
                    lds_write4(abort_a, 1u);
                    __hip_atomic_store(status, 3u | ((uint32_t)q << 8), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                    return false;
                }
                __builtin_amdgcn_s_sleep(2);
            }
            if (!image_stored(q)) return false;
            const uint32_t dst = (uint32_t)pq.img_lds;
            const int chunks = pq.img_chunks;
            for (int j = 0; j < chunks; ++j)
                __builtin_amdgcn_global_load_lds(
                    (const void *)(pq.img + j * 64 + lane),
                    (lds_void_ptr)(reinterpret_cast<char *>(sh.area) + dst + j * 1024), 16, 0, 0);
            if (pending >= 0) {
                // loads return in order: the older image is complete when at most
                // the `chunks` loads just issued are outstanding
                switch (chunks) {
#define NVQ_W(n) case n: __builtin_amdgcn_s_waitcnt(vmcnt_imm(n)); break;
                    NVQ_W(1) NVQ_W(2) NVQ_W(3) NVQ_W(4) NVQ_W(5) NVQ_W(6) NVQ_W(7) NVQ_W(8)
                    NVQ_W(9) NVQ_W(10) NVQ_W(11) NVQ_W(12) NVQ_W(13) NVQ_W(14) NVQ_W(15) NVQ_W(16)
                    NVQ_W(17) NVQ_W(18) NVQ_W(19) NVQ_W(20) NVQ_W(21) NVQ_W(22) NVQ_W(23) NVQ_W(24)
                    NVQ_W(25) NVQ_W(26) NVQ_W(27) NVQ_W(28) NVQ_W(29) NVQ_W(30) NVQ_W(31)
#undef NVQ_W
                    default: __builtin_amdgcn_s_waitcnt(vmcnt_imm(0)); break;
                }
                if (lane == 0) lds_write4(ready_a, (uint32_t)(pending + 1));
            }
            pending = q;
            ++q;
            return true;
        };
        bool live = true;
        for (int p = 0; p < nphase && live; ++p) {
            CPhase &ph = tab[p];
            if (ph.dep) {
                flush();
                if (ph.wait_phase >= 0) lds_barrier();  // flags seen
                const LdsWriter wr = {0};
                // barrier count only; false: abort raised
                if (!image_build<PER_GROUP, MAIL>(wr, ph, sh, w, lane, 0, true, 0u, 0u, abort_a,
                                                  status, p, trace, wg))
                    break;
                lds_barrier();  // image complete
                q = p + 1;
            }
            // Run ahead of the streaming waves.  Only regions that free up
            // without a barrier of phase p or later may be waited for here:
            // the streaming waves may need this wave at such a barrier first.
            for (;;) {
                // images of phases in which no wave of this workgroup works are not loaded
                while (q < nphase && phase_skip(wg_passes, q) != 0) ++q;
                if (!(live && q < nphase && q <= p + kLookahead && !tab[q].dep &&
                      tab[q].img_need < p))
                    break;
                live = load_image();
            }
            if (ph.publish && live) {
                flush();
                lds_barrier();
            }
        }
        flush();
        return;
    }

    // ================= streaming waves =================
    const uint32_t ring_base = lds_addr(&sh.ring[w][0][0]) + lane * 16;
    const uint32_t sring_base = lds_addr(&sh.sring[w][0][0]) + lane * 4;


    // Take the next chunk of the stream out of the ring (16 bytes and one
    // scale per lane) and refill its slot at once.  When a chunk is taken, the
    // other kSlots - 1 slots all hold younger chunks (the previous slot was
    // refilled when its chunk was taken), so that many may stay in flight.
    auto pop_chunk = [&](uint32_t &scale_bits) -> uint4 {
        __builtin_amdgcn_s_waitcnt(vmcnt_imm(kOpsPerChunk * (kSlots - 1)));
        u32x4_t v;
        uint32_t sb;
        asm volatile("ds_read_b128 %0, %2\n\tds_read_b32 %1, %3\n\ts_waitcnt lgkmcnt(0)"
                     : "=&v"(v), "=&v"(sb)
                     : "v"(ring_base + st.slot * 1024u), "v"(sring_base + st.slot * 256u)
                     : "memory");
        scale_bits = sb;
        issue_chunk(st.ic, tab, skips, nphase, sh, w, gw, (int)st.slot, lane, dummy);
        st.slot = st.slot + 1 == kSlots ? 0 : st.slot + 1;
        return make_uint4(v.x, v.y, v.z, v.w);
    };

    // This wave has finished every phase before `done`: the loader wave may reuse the
    // room of their images.
    auto note_progress = [&](uint32_t done) {
        if (lane == 0) lds_write4(progress_a + w * 4, done);
    };

    bool aborted = false;
    uint32_t ready_seen = 0;     // sh.img_ready as requested on entering an independent phase
    bool ready_pending = false;  // ... and not yet looked at
    for (int p = 0; p < nphase && !aborted; ++p) {
        {
            // phases in which this wave has no rows and nobody meets at a barrier are
            // passed without a look; the loader learns that they are done with
            const int pass = phase_skip(skips, p);
            if (pass > 0) {
                p += pass;
                note_progress((uint32_t)(p < nphase ? p : nphase));
                if (p >= nphase) break;
            }
        }
        CPhase &ph = tab[p];
        const int G = ph.G;
        const bool w4a8 = ph.precision == NVQ_W4A8;
        const ImgLayout<PER_GROUP> L(w4a8, G);
        const uint32_t img = area_base + (uint32_t)ph.img_lds;
        trace_mark(trace, wg, w, lane, p, 0);

        if (ph.dep) {
            // ---- dependent phase.  Through the flags: wait until every workgroup has
            // ---- published phase wait_phase.  Then build the image from the raw input
            // ---- (or from the mail, whose arrival is the wait), all together
            if (ph.wait_phase >= 0) {
                if (w == 0) {
                    const bool ok = wait_flags(flag_copy(wg & (kFlagReplicas - 1)), nwg,
                                               flag_base + 2u + (uint32_t)ph.wait_phase, lane);
                    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");
                    if (!ok && lane == 0) {
                        lds_write4(abort_a, 1u);
                        __hip_atomic_store(status, 1u | ((uint32_t)p << 8), __ATOMIC_RELAXED,
                                           __HIP_MEMORY_SCOPE_AGENT);
                    }
                }
                lds_barrier();  // satisfied (or abort raised)
            }
            trace_mark(trace, wg, w, lane, p, 1);
            const LdsWriter wr = {img};
            if (!image_build<PER_GROUP, MAIL>(wr, ph, sh, w, lane, wg, true, mail_tag_hi,
                                              mail_stride, abort_a, status, p, trace, wg))
                break;
            trace_mark(trace, wg, w, lane, p, 2);
            lds_barrier();  // the image is complete
            ready_pending = false;
        } else {
            // ---- independent phase: the loader wave announces the image.  The word is
            // ---- only requested here; it is looked at after the wait that the wave's
            // ---- first reads of the image need anyway (LDS serves a wave's requests
            // ---- in order, so reads issued after it saw the image if it says so)
            trace_mark(trace, wg, w, lane, p, 1);
            asm volatile("ds_read_b32 %0, %1" : "=v"(ready_seen) : "v"(ready_a) : "memory");
            ready_pending = true;
        }
        // Waves w, w + 4, w + 8 share a SIMD; rotate their priorities so that none
        // of them is favoured for long (see the header).  (In phases that end with
        // everybody waiting for the slowest wave: equal priorities, or the oldest wave
        // first, cost 7 % of a dependent step; the youngest first is as good as rotating.)
        switch (((w >> 2) + p) % 3) {
            case 0: __builtin_amdgcn_s_setprio(0); break;
            case 1: __builtin_amdgcn_s_setprio(1); break;
            default: __builtin_amdgcn_s_setprio(2); break;
        }

        // ---- this wave's weight rows ---------------------------------------------------
        const int gpl = ph.gpl;
        int r0, nrows;
        stream_wave_rows(ph.rows_base, ph.rows_extra, ph.rows_rot, ph.spread ? gw_spread : gw,
                         nwg * kStreamWaves, r0, nrows);
        r0 *= ph.row_unit;
        nrows *= ph.row_unit;
        if (r0 + nrows > ph.total_rows) nrows = ph.total_rows - r0;  // a short last unit
        // In a phase that somebody waits for, the waves with a unit more than the others
        // go first on their SIMD: the phase ends when they do.
        if (ph.spread && ph.rows_extra > 0 && nrows > ph.rows_base * ph.row_unit)
            __builtin_amdgcn_s_setprio(3);
        const int r1 = r0 + nrows;
        uint32_t xs_bits = 0x3f800000u;  // per-token activation scale (W4A8), else 1
        const uint32_t plane = (uint32_t)G * 16u;
        // Requested with the first activations, valid after the wait that follows them.
        auto request_xs = [&]() {
            if (w4a8 && !PER_GROUP)
                asm volatile("ds_read_b32 %0, %1" : "=v"(xs_bits) : "v"(img + L.stok) : "memory");
        };
        // After that wait: did the word requested on entering the phase say that the
        // image is there?  If not, waits for it (bounded) and returns false once: the
        // reads have to be issued again.  On abort `aborted` is set (and true returned).
        auto image_ready = [&]() -> bool {
            if (!ready_pending) return true;
            ready_pending = false;
            if ((uint32_t)__builtin_amdgcn_readfirstlane((int)ready_seen) >= (uint32_t)(p + 1))
                return true;
            uint32_t spins = 0;
            while (lds_read4_uniform(ready_a) < (uint32_t)(p + 1)) {
                if (lds_read4_uniform(abort_a) || ++spins > kSpinLimit) {
                    aborted = true;
                    if (lane == 0) {
                        lds_write4(abort_a, 1u);
                        __hip_atomic_store(status, 4u | ((uint32_t)p << 8), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                    }
                    return true;
                }
                __builtin_amdgcn_s_sleep(1);
            }
            return false;
        };
        float yv = 0.0f;  // results of up to 64 rows, one per lane, until they are stored

        // The lane's activations of group g = i * 64 + lane (clamped to a valid group)
        // out of the LDS image; nothing is waited for.
        auto request_group = [&](int g, u32x4_t(&x)[4], uint32_t &aux, uint32_t &sgbits, bool &ok) {
            ok = g < G;
            const uint32_t ga = img + (ok ? g : 0) * 16;
            const uint32_t aux_a = img + L.aux + (ok ? g : 0) * 4;
            if (w4a8) {
                asm volatile("ds_read_b128 %0, %3\n\tds_read_b128 %1, %4\n\tds_read_b32 %2, %5"
                             : "=&v"(x[0]), "=&v"(x[1]), "=&v"(aux)
                             : "v"(ga), "v"(ga + plane), "v"(aux_a)
                             : "memory");
                if (PER_GROUP)
                    asm volatile("ds_read_b32 %0, %1"
                                 : "=&v"(sgbits)
                                 : "v"(img + L.xsg + (ok ? g : 0) * 4)
                                 : "memory");
            } else {
                asm volatile("ds_read_b128 %0, %5\n\tds_read_b128 %1, %6\n\tds_read_b128 %2, %7\n\t"
                             "ds_read_b128 %3, %8\n\tds_read_b32 %4, %9"
                             : "=&v"(x[0]), "=&v"(x[1]), "=&v"(x[2]), "=&v"(x[3]), "=&v"(aux)
                             : "v"(ga), "v"(ga + plane), "v"(ga + 2 * plane), "v"(ga + 3 * plane),
                               "v"(aux_a)
                             : "memory");
            }
        };
        auto request_x = [&](int i, u32x4_t(&x)[4], uint32_t &aux, uint32_t &sgbits, bool &ok) {
            request_group(i * 64 + lane, x, aux, sgbits, ok);
        };
        // One chunk against the lane's activations of its group, added to `sum`.
        auto chunk_term = [&](float sum, const uint4 &wq, uint32_t sbits, const u32x4_t(&x)[4],
                              uint32_t aux, uint32_t sgbits, bool ok) -> float {
            const u32x4_t wv = {wq.x, wq.y, wq.z, wq.w};
            float sw = ok ? half_bits_to_float((uint16_t)sbits) : 0.0f;
            if (w4a8) {
                const int acc = dot_w4a8(wv, x[0], x[1], (int)aux);
                if (PER_GROUP) sw *= __uint_as_float(sgbits);
                return fmaf(sw, (float)acc, sum);
            }
            return fmaf(sw, dot_w4a16(wv, x, __uint_as_float(aux)), sum);
        };
        // End of row `row`: reduce over the lanes, park the result in lane
        // (row - r0) % 64, store once per 64 rows.
        auto finish_row = [&](int row, float sum) {
            const float tot = __builtin_bit_cast(
                float,
                __builtin_amdgcn_readlane(__builtin_bit_cast(int, wave_sum_to_lane63(sum)), 63));
            const int k = row - r0;
            if (lane == (k & 63)) yv = tot * __uint_as_float(xs_bits);
            if ((k & 63) == 63 || row == r1 - 1) {
                const int r = row - (k & 63) + lane;
                if (r <= row) {
                    int first = 0;
                    void *y = ph.y[0];
                    int dt = ph.y_dtype[0];
                    uint32_t *mail = nullptr;
                    if constexpr (MAIL) mail = ph.mail_y[0];
#pragma unroll
                    for (int sgm = 1; sgm < kMaxSeg; ++sgm)
                        if (sgm < ph.nseg && r >= ph.row_end[sgm - 1]) {
                            first = ph.row_end[sgm - 1];
                            y = ph.y[sgm];
                            dt = ph.y_dtype[sgm];
                            if constexpr (MAIL) mail = ph.mail_y[sgm];
                        }
                    store_out(y, dt, r - first, yv);
                    if constexpr (MAIL) {
                        // the same bf16 value once more, tagged, for the phases that read it
                        if (mail) {
                            uint32_t *at = mail + mail_word(r - first);
                            const uint32_t word = mail_tag_hi | float_to_bf16_bits(yv);
                            for (int rep = 0; rep < kMailReplicas; ++rep, at += mail_stride)
                                __hip_atomic_store(at, word, __ATOMIC_RELAXED,
                                                   __HIP_MEMORY_SCOPE_AGENT);
                        }
                    }
                }
            }
        };
        // Rows of at most kRegGpl chunks: the lane meets the same GPL groups in
        // every row, so their activations are taken out of the image once per
        // phase and stay in registers.  (Reading them per chunk makes LDS the
        // bound of the W4A16 phases: 64 bytes per lane and chunk on top of the
        // ring's 20.)
        auto rows_in_registers = [&](auto gpl_const) {
            constexpr int GPL = decltype(gpl_const)::value;
            u32x4_t x[GPL][4];
            uint32_t aux[GPL], sgb[GPL];
            bool ok[GPL];
            do {
                request_xs();
#pragma unroll
                for (int i = 0; i < GPL; ++i) {
                    x[i][2] = x[i][3] = u32x4_t{0, 0, 0, 0};
                    sgb[i] = 0;
                    request_x(i, x[i], aux[i], sgb[i], ok[i]);
                }
                asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
                asm volatile("" : "+v"(xs_bits), "+v"(ready_seen));
#pragma unroll
                for (int i = 0; i < GPL; ++i)  // nothing may be scheduled (or copied) before that wait
                    asm volatile(""
                                 : "+v"(x[i][0]), "+v"(x[i][1]), "+v"(x[i][2]), "+v"(x[i][3]),
                                   "+v"(aux[i]), "+v"(sgb[i]));
            } while (!image_ready());
            if (!ph.dep) trace_mark(trace, wg, w, lane, p, 2);
            if (aborted) return;
            for (int row = r0; row < r0 + nrows; ++row) {
                float sum = 0.0f;
#pragma unroll
                for (int i = 0; i < GPL; ++i) {
                    uint32_t sbits;
                    const uint4 wq = pop_chunk(sbits);
                    sum = chunk_term(sum, wq, sbits, x[i], aux[i], sgb[i], ok[i]);
                }
                finish_row(row, sum);
            }
        };
        // Rows of 96 groups in pairs (A, B): three chunks, the lanes of the first hold
        // groups 0..63 of A, those of the second groups 64..95 of A and 0..31 of B,
        // those of the third groups 32..95 of B; the lane's three groups stay in
        // registers for the phase.
        auto row_pairs = [&]() {
            u32x4_t x[3][4];
            uint32_t aux[3], sgb[3];
            bool ok[3];
            const bool first_half = lane < 32;
            do {
                request_xs();
#pragma unroll
                for (int i = 0; i < 3; ++i) {
                    x[i][2] = x[i][3] = u32x4_t{0, 0, 0, 0};
                    sgb[i] = 0;
                    const int g = i == 0 ? lane : i == 1 ? (first_half ? 64 + lane : lane - 32) : 32 + lane;
                    request_group(g, x[i], aux[i], sgb[i], ok[i]);
                }
                asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
                asm volatile("" : "+v"(xs_bits), "+v"(ready_seen));
#pragma unroll
                for (int i = 0; i < 3; ++i)
                    asm volatile(""
                                 : "+v"(x[i][0]), "+v"(x[i][1]), "+v"(x[i][2]), "+v"(x[i][3]),
                                   "+v"(aux[i]), "+v"(sgb[i]));
            } while (!image_ready());
            if (!ph.dep) trace_mark(trace, wg, w, lane, p, 2);
            if (aborted) return;
            for (int row = r0; row < r1; row += 2) {
                uint32_t sbits;
                uint4 wq = pop_chunk(sbits);
                float sum_a = chunk_term(0.0f, wq, sbits, x[0], aux[0], sgb[0], true);
                wq = pop_chunk(sbits);
                const float mid = chunk_term(0.0f, wq, sbits, x[1], aux[1], sgb[1], true);
                sum_a += first_half ? mid : 0.0f;
                float sum_b = first_half ? 0.0f : mid;
                wq = pop_chunk(sbits);
                sum_b = chunk_term(sum_b, wq, sbits, x[2], aux[2], sgb[2], true);
                finish_row(row, sum_a);
                finish_row(row + 1, sum_b);
            }
        };
        // (a wave without rows in this phase never looks at the image)
        if (nrows > 0 && ph.pair_stream != 0) {
            // (the host pairs rows only with per-token activation scales: with a
            // scale per group the wave's registers do not hold this path as well)
            if constexpr (!PER_GROUP && PAIRS) row_pairs();
        } else if (nrows > 0) switch (gpl) {
            case 1: rows_in_registers(std::integral_constant<int, 1>()); break;
            case 2: rows_in_registers(std::integral_constant<int, 2>()); break;
            case 4: rows_in_registers(std::integral_constant<int, 4>()); break;
            default: {
                // rows of three chunks, and longer ones: the first kHeldGpl groups of the lane stay in
                // registers as above, the others come out of the image for every
                // chunk (the registers of a wave hold no more)
                constexpr int kHeldGpl = 3;
                u32x4_t hx[kHeldGpl][4];
                uint32_t haux[kHeldGpl], hsgb[kHeldGpl];
                bool hok[kHeldGpl];
                do {
                    request_xs();
#pragma unroll
                    for (int i = 0; i < kHeldGpl; ++i) {
                        hx[i][2] = hx[i][3] = u32x4_t{0, 0, 0, 0};
                        hsgb[i] = 0;
                        request_x(i, hx[i], haux[i], hsgb[i], hok[i]);
                    }
                    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
                    asm volatile("" : "+v"(xs_bits), "+v"(ready_seen));
#pragma unroll
                    for (int i = 0; i < kHeldGpl; ++i)
                        asm volatile(""
                                     : "+v"(hx[i][0]), "+v"(hx[i][1]), "+v"(hx[i][2]),
                                       "+v"(hx[i][3]), "+v"(haux[i]), "+v"(hsgb[i]));
                } while (!image_ready());
                if (!ph.dep) trace_mark(trace, wg, w, lane, p, 2);
                if (aborted) break;
                for (int row = r0; row < r1; ++row) {
                    float sum = 0.0f;
#pragma unroll
                    for (int i = 0; i < kHeldGpl; ++i) {
                        uint32_t sbits;
                        const uint4 wq = pop_chunk(sbits);
                        sum = chunk_term(sum, wq, sbits, hx[i], haux[i], hsgb[i], hok[i]);
                    }
                    for (int i = kHeldGpl; i < gpl; ++i) {
                        u32x4_t x[4];
                        x[2] = x[3] = u32x4_t{0, 0, 0, 0};
                        uint32_t aux, sgbits = 0;
                        bool ok;
                        request_x(i, x, aux, sgbits, ok);
                        uint32_t sbits;
                        const uint4 wq = pop_chunk(sbits);  // its lgkmcnt(0) also covers the reads above
                        // nothing below may be scheduled (or copied) before that wait
                        asm volatile(""
                                     : "+v"(x[0]), "+v"(x[1]), "+v"(x[2]), "+v"(x[3]), "+v"(aux),
                                       "+v"(sgbits));
                        sum = chunk_term(sum, wq, sbits, x, aux, sgbits, ok);
                    }
                    finish_row(row, sum);
                }
            }
        }
        if (aborted) break;
        // this wave no longer reads the phase's image
        note_progress((uint32_t)(p + 1));
        trace_mark(trace, wg, w, lane, p, 7);
        if (trace.buf && wg < trace.wgs && lane == 0)  // the last of the workgroup's waves
            __hip_atomic_fetch_max(&trace.buf[((size_t)wg * trace.nphase + p) * kTraceSlots + 6],
                                   wall_clock64(), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);

        if (ph.publish) {
            // a later phase reads or overwrites what this one touched: make the
            // workgroup's outputs visible device-wide, then raise its flag
            __builtin_amdgcn_s_waitcnt(vmcnt_imm(0));  // this wave's stores have completed
            lds_barrier();
            if (w == 0) {
                trace_mark(trace, wg, w, lane, p, 3);
                __builtin_amdgcn_fence(__ATOMIC_RELEASE, "agent");
                if (lane < kFlagReplicas)  // one store instruction, a lane per copy
                    __hip_atomic_store(flag_copy(lane) + wg, flag_base + 2u + (uint32_t)p,
                                       __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                trace_mark(trace, wg, w, lane, p, 4);
            }
        }
    }
    __builtin_amdgcn_s_waitcnt(vmcnt_imm(0));  // no load may outlive the wave
}

}  // namespace

namespace {
// The instantiations that are launched: per-group scales never pair rows.
template <bool PER_GROUP, bool PAIRS, bool MAIL>
bool fits_a_compute_unit() {
    int n = 0;
    return hipOccupancyMaxActiveBlocksPerMultiprocessor(
               &n, decode_stream_kernel<PER_GROUP, PAIRS, MAIL>, kStreamThreads, 0) == hipSuccess &&
           n >= 1;
}
}  // namespace

int stream_grid_limit() {
    static int cached = -1;
    if (cached < 0) {
        // every instantiation that may be launched must fit a compute unit
        const bool ok = fits_a_compute_unit<false, false, false>() &&
                        fits_a_compute_unit<true, false, false>() &&
                        fits_a_compute_unit<false, true, false>() &&
                        fits_a_compute_unit<false, false, true>() &&
                        fits_a_compute_unit<true, false, true>() &&
                        fits_a_compute_unit<false, true, true>();
        cached = ok ? device_cu_count() : 0;
    }
    return cached;
}

namespace {
template <bool PER_GROUP, bool PAIRS, bool MAIL>
void launch_variant(const StreamPhase *tab_dev, const uint8_t *skips, int nphase, int nimages,
                    uint32_t *flags, uint32_t *status, uint32_t flag_base, const uint4 *dummy,
                    int nwg, unsigned long long *trace, int trace_wgs, uint32_t mail_tag_hi,
                    uint32_t mail_stride, hipStream_t st) {
    hipLaunchKernelGGL((decode_stream_kernel<PER_GROUP, PAIRS, MAIL>), dim3(nwg),
                       dim3(kStreamThreads), 0, st, tab_dev, skips, nphase, nimages, flags, status,
                       flag_base, dummy, trace, trace_wgs, mail_tag_hi, mail_stride);
}
}  // namespace

int launch_decode_stream(const StreamPhase *tab_dev, const uint8_t *skips, int nphase, int nimages,
                         int act_group, bool pairs, bool mail, uint32_t mail_tag,
                         uint32_t mail_stride, uint32_t *flags, uint32_t *status, uint32_t flag_base, const void *dummy, int nwg,
                         unsigned long long *trace, int trace_wgs, hipStream_t st) {
    const uint4 *d = reinterpret_cast<const uint4 *>(dummy);
    if (mail && (mail_tag == 0 || mail_tag > 0xffffu)) return NVQ_ERR_INVALID_ARG;
    const uint32_t tag_hi = mail_tag << 16;
    const bool per_group = act_group == 32;
    if (per_group && pairs) return NVQ_ERR_INVALID_ARG;  // rows are not paired with per-group scales
#define NVQ_LAUNCH(PG, PR, ML)                                                                   \
    launch_variant<PG, PR, ML>(tab_dev, skips, nphase, nimages, flags, status, flag_base, d, nwg, \
                               trace, trace_wgs, tag_hi, mail_stride, st)
    if (per_group) {
        if (mail) NVQ_LAUNCH(true, false, true); else NVQ_LAUNCH(true, false, false);
    } else if (pairs) {
        if (mail) NVQ_LAUNCH(false, true, true); else NVQ_LAUNCH(false, true, false);
    } else {
        if (mail) NVQ_LAUNCH(false, false, true); else NVQ_LAUNCH(false, false, false);
    }
#undef NVQ_LAUNCH
    NVQ_HIP_TRY(hipGetLastError());
    return NVQ_OK;
}

}  // namespace nvq
