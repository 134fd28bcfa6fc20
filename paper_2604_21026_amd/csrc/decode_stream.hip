// Persistent streaming kernel for a whole decode step at batch 1.
//
// Why: one decode step is a chain of ~130 dependent phases (q/k/v, o, gate/up,
// down per block) of 1-10 us each at HBM speed.  Launching a kernel per phase
// leaves the memory system idle at every boundary; the paper removes its
// launch bubbles with graph capture (paragraph "CUDA graph capture for
// decode").  Here the whole layer list runs in ONE launch, and, because
// weights never depend on activations, every wave keeps fetching the weights
// of the coming phases while it waits for the current phase's input.
//
// Structure of a workgroup (one per compute unit, all co-resident):
//   * kStreamWaves streaming waves.  Each owns a contiguous range of rows in
//     every phase and sees its work as one flat sequence of 1 KiB chunks
//     (64 groups x 16 B of one weight row) across all phases.  Chunks are
//     fetched with non-temporal global->LDS loads into a per-wave ring of
//     kSlots slots and consumed in order; the ring is refilled as soon as a
//     pair of slots has been consumed, independent of phase boundaries.
//     The fp16 scales travel the same way (one dword load per lane serves a
//     pair of chunks).  A streaming wave issues no other vector-memory
//     operation, so the number of loads in flight behind any chunk is a
//     compile-time constant and one `s_waitcnt vmcnt(n)` tells when a pair of
//     chunks has landed.
//   * control duties, carried by wave 0 between its own rows.  It alone talks
//     to global memory besides the weight stream: it waits until every
//     workgroup has finished the previous phase (one flag word per workgroup,
//     no atomics), copies the phase's input vector into LDS, and after a
//     phase that others depend on publishes its own flag.  Every wave writes
//     its own output rows (one store instruction per 64 rows).  Its extra memory operations queue behind its ring loads,
//     which only makes the ring's counted waits conservative.
//   Activation quantisation (W4A8 phases) is done by the streaming waves
//   cooperatively out of LDS, once per workgroup per phase.
//
// Ordering: the host marks, per phase, the latest earlier phase whose buffers
// it depends on (its input overlaps that phase's outputs, or its outputs
// overlap that phase's input or outputs).  Such a phase reads its input only
// after every workgroup has published the phase it depends on; a phase that
// depends on nothing has its input fetched one phase ahead.  A bounded spin
// turns a stuck wait (e.g. the grid not co-resident) into an error status
// instead of a hang.
#include "decode_stream.h"

namespace nvq {

namespace {

typedef __attribute__((address_space(3))) void *lds_void_ptr;

constexpr int kSlots = 10;            // 1 KiB weight slots per wave
constexpr int kUnits = kSlots / 2;    // a unit = two chunks + their scales = 3 loads
constexpr int kOpsPerUnit = 3;
constexpr int kXStageBytes = kStreamMaxK * 2;  // bf16 input vector
constexpr uint32_t kSpinLimit = 4u << 20;      // polls before giving up (seconds)

// s_waitcnt immediate that waits for vmcnt <= n only (gfx9 encoding:
// vmcnt[3:0] | expcnt[6:4] | lgkmcnt[11:8] | vmcnt[5:4] at [15:14]).
constexpr int vmcnt_imm(int n) { return (n & 15) | ((n >> 4) << 14) | 0x0f70; }

struct Shared {
    uint4 ring[kStreamWaves][kSlots][64];
    uint32_t sring[kStreamWaves][kUnits][64];
    uint4 xstage[2][kXStageBytes / 16];  // input vectors of phases p (p & 1) and p + 1
    float xsg[kStreamMaxK / 32];         // per-group activation scales (act_group 32)
    float amax_part[kStreamWaves];
    int abort;
};

__device__ __forceinline__ void lds_barrier() {
    // every LDS access issued so far has completed before anyone passes
    asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
}

__device__ __forceinline__ uint32_t lds_addr(const void *p) {
    return (uint32_t)(uintptr_t)p;  // LDS pointers are 32-bit offsets
}

// LDS reads of a streaming wave are written as instructions: the compiler
// would otherwise put a full vmcnt(0) wait in front of every LDS read while
// global->LDS loads are in flight, and drain the weight ring each time.
typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));
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

// LDS writes likewise (the compiler also guards them with vmcnt(0)).  The
// data reaches LDS before the next lds_barrier(), which waits for lgkmcnt(0).
__device__ __forceinline__ void lds_write4(uint32_t addr, uint32_t v) {
    asm volatile("ds_write_b32 %0, %1" : : "v"(addr), "v"(v) : "memory");
}
__device__ __forceinline__ void lds_write8(uint32_t addr, uint32_t lo, uint32_t hi) {
    typedef uint32_t u32x2_t __attribute__((ext_vector_type(2)));
    u32x2_t v = {lo, hi};
    asm volatile("ds_write_b64 %0, %1" : : "v"(addr), "v"(v) : "memory");
}

// Position in a streaming wave's flat chunk sequence (all fields uniform).
struct Cursor {
    int p, nphase;
    int row, row_stop, i, gpl, G;
    int seg, seg_end;
    const uint4 *qrow;
    const uint16_t *srow;
};

__device__ __forceinline__ void cursor_set_segment(Cursor &c, const StreamPhase &ph) {
    int seg = 0, first = 0;
#pragma unroll
    for (int s = 1; s < kMaxSeg; ++s)
        if (s < ph.nseg && c.row >= ph.row_end[s - 1]) {
            seg = s;
            first = ph.row_end[s - 1];
        }
    const uint4 *q = ph.qw[0];
    const uint16_t *sc = ph.sc[0];
    int end = ph.row_end[0];
#pragma unroll
    for (int s = 1; s < kMaxSeg; ++s)
        if (seg == s) {
            q = ph.qw[s];
            sc = ph.sc[s];
            end = ph.row_end[s];
        }
    c.seg = seg;
    c.seg_end = end;
    c.qrow = q + (int64_t)(c.row - first) * c.G;
    c.srow = sc + (int64_t)(c.row - first) * c.G;
}

// Enter phase c.p (skipping phases in which this wave owns no rows).
__device__ __forceinline__ void cursor_enter(Cursor &c, const StreamPhase *tab, int gw) {
    while (c.p < c.nphase) {
        const StreamPhase &ph = tab[c.p];
        const int r0 = gw * ph.rows_per_wave;
        int r1 = r0 + ph.rows_per_wave;
        r1 = r1 < ph.total_rows ? r1 : ph.total_rows;
        if (r0 < r1) {
            c.row = r0;
            c.row_stop = r1;
            c.i = 0;
            c.gpl = ph.gpl;
            c.G = ph.G;
            cursor_set_segment(c, ph);
            return;
        }
        ++c.p;
    }
}

__device__ __forceinline__ void cursor_advance(Cursor &c, const StreamPhase *tab, int gw) {
    if (++c.i < c.gpl) return;
    c.i = 0;
    ++c.row;
    c.qrow += c.G;
    c.srow += c.G;
    if (c.row == c.row_stop) {
        ++c.p;
        cursor_enter(c, tab, gw);
    } else if (c.row == c.seg_end) {
        cursor_set_segment(c, tab[c.p]);
    }
}

// Issue the three loads of one unit into unit slot `us` of this wave's ring.
// Past the end of the stream the loads re-read a dummy line so that the
// number of loads in flight stays constant.
__device__ __forceinline__ void issue_unit(Cursor &c, const StreamPhase *tab, int gw, Shared &sh,
                                           int w, int us, int lane, const uint4 *dummy) {
    const bool a_ok = c.p < c.nphase;
    const uint4 *qa = a_ok ? c.qrow + c.i * 64 : dummy;
    const uint32_t *sa = a_ok ? reinterpret_cast<const uint32_t *>(c.srow + c.i * 64)
                              : reinterpret_cast<const uint32_t *>(dummy);
    const int ga = a_ok ? c.G - c.i * 64 : 64;  // valid groups in chunk A
    if (a_ok) cursor_advance(c, tab, gw);
    const bool b_ok = c.p < c.nphase;
    const uint4 *qb = b_ok ? c.qrow + c.i * 64 : dummy;
    const uint32_t *sb = b_ok ? reinterpret_cast<const uint32_t *>(c.srow + c.i * 64)
                              : reinterpret_cast<const uint32_t *>(dummy);
    const int gb = b_ok ? c.G - c.i * 64 : 64;
    if (b_ok) cursor_advance(c, tab, gw);

    // scales: lanes 0-31 fetch chunk A's 32 dwords, lanes 32-63 chunk B's
    const int hl = lane & 31;
    const bool upper = lane >= 32;
    const uint32_t *sp = (upper ? sb : sa) + hl;
    if (2 * hl < (upper ? gb : ga))
        __builtin_amdgcn_global_load_lds((const void *)sp, (lds_void_ptr)&sh.sring[w][us][0], 4, 0,
                                         2);
    if (lane < ga)
        __builtin_amdgcn_global_load_lds((const void *)(qa + lane),
                                         (lds_void_ptr)&sh.ring[w][2 * us][0], 16, 0, 2);
    if (lane < gb)
        __builtin_amdgcn_global_load_lds((const void *)(qb + lane),
                                         (lds_void_ptr)&sh.ring[w][2 * us + 1][0], 16, 0, 2);
}

// ---- arithmetic of one chunk ----------------------------------------------
__device__ __forceinline__ int dot_w4a8(const uint4 &w, const uint32_t (&x)[8], int acc) {
    const uint32_t wv[4] = {w.x, w.y, w.z, w.w};
#pragma unroll
    for (int d = 0; d < 4; ++d) {
        const uint32_t lo = wv[d] & 0x0f0f0f0fu;
        const uint32_t hi = (wv[d] >> 4) & 0x0f0f0f0fu;
        acc = __builtin_amdgcn_sdot4((int)lo, (int)x[d], acc, false);
        acc = __builtin_amdgcn_sdot4((int)hi, (int)x[4 + d], acc, false);
    }
    return acc;
}

typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
__device__ __forceinline__ float dot2_bf16(uint32_t a, uint32_t b, float c) {
    return __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2_t, a),
                                           __builtin_bit_cast(bf16x2_t, b), c, false);
}

// Two accumulator chains so that consecutive dot instructions are independent.
__device__ __forceinline__ float dot_w4a16(const uint4 &w, const uint32_t (&x)[16], float off) {
    const uint32_t wv[4] = {w.x, w.y, w.z, w.w};
    constexpr uint32_t kMagic = 0x43434343u;
    float a0 = off, a1 = 0.0f;
#pragma unroll
    for (int d = 0; d < 4; ++d) {
        const uint32_t lo = wv[d] & 0x0f0f0f0fu;
        const uint32_t hi = (wv[d] >> 4) & 0x0f0f0f0fu;
        const uint32_t l01 = __builtin_amdgcn_perm(kMagic, lo, 0x04010400u);
        const uint32_t l23 = __builtin_amdgcn_perm(kMagic, lo, 0x04030402u);
        const uint32_t h01 = __builtin_amdgcn_perm(kMagic, hi, 0x04010400u);
        const uint32_t h23 = __builtin_amdgcn_perm(kMagic, hi, 0x04030402u);
        a0 = dot2_bf16(l01, x[2 * d], a0);
        a1 = dot2_bf16(l23, x[2 * d + 1], a1);
        a0 = dot2_bf16(h01, x[8 + 2 * d], a0);
        a1 = dot2_bf16(h23, x[8 + 2 * d + 1], a1);
    }
    return a0 + a1;
}

// Sum over the 64 lanes with data-parallel-primitive moves only (no LDS
// traffic); the total is valid in lane 63.
template <int CTRL, int ROW_MASK>
__device__ __forceinline__ float dpp_move(float x) {
    return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), CTRL,
                                                                 ROW_MASK, 0xf, false));
}
__device__ __forceinline__ float wave_sum_to_lane63(float v) {
    v += dpp_move<0xb1, 0xf>(v);   // quad_perm [1,0,3,2]
    v += dpp_move<0x4e, 0xf>(v);   // quad_perm [2,3,0,1]
    v += dpp_move<0x141, 0xf>(v);  // row_half_mirror
    v += dpp_move<0x140, 0xf>(v);  // row_mirror: every lane of a row of 16 holds the row sum
    v += dpp_move<0x142, 0xa>(v);  // row_bcast15 into rows 1 and 3
    v += dpp_move<0x143, 0xc>(v);  // row_bcast31 into rows 2 and 3
    return v;
}

// ---- consuming one phase ----------------------------------------------------
struct StreamState {
    Cursor ic;       // issue cursor
    uint32_t rslot;  // ring slot of the next chunk to read from LDS (chunks are read in order)
    uint32_t uslot;  // unit slot the next refill goes to
};

// One chunk as it sits in registers between its LDS read and its use.
template <bool WITH_X>
struct ChunkRegs {
    u32x4_t w;
    uint32_t s;
    u32x4_t x[WITH_X ? 4 : 1];
};

template <int PREC, int GPL, bool PER_GROUP>
__device__ __forceinline__ void consume_phase(const StreamPhase &ph, const StreamPhase *tab,
                                              StreamState &st, Shared &sh, int w, int gw, int lane,
                                              const uint4 *dummy, float xs_token,
                                              uint32_t stage /* LDS address of the input */) {
    constexpr int XR = PREC == NVQ_W4A8 ? 8 : 16;
    // Activations stay in registers for the whole phase unless that would take
    // more than 64 registers (bf16 activations of more than four chunks); then
    // they are re-read from the LDS stage together with each weight chunk.
    constexpr bool XREG = PREC == NVQ_W4A8 || GPL <= 4;
    constexpr int NX = XREG ? GPL : 1;
    uint32_t xr[NX][XR];
    int neg8[GPL];
    float xoff[GPL];
    float xsg[GPL];
    uint32_t xaddr[GPL];  // LDS address of the lane's group in the stage (!XREG)
    bool okv[GPL];        // the lane's group exists (false past the end of a ragged row)
#pragma unroll
    for (int i = 0; i < GPL; ++i) {
        const int g = i * 64 + lane;
        const bool ok = g < ph.G;
        const int gc = ok ? g : 0;
        okv[i] = ok;
        const uint32_t src = stage + gc * (XR * 4);
        xaddr[i] = src;
        uint32_t t[XR];
#pragma unroll
        for (int q = 0; q < XR / 4; ++q) {
            const uint4 a = lds_read16(src + q * 16);
            t[4 * q + 0] = ok ? a.x : 0u;
            t[4 * q + 1] = ok ? a.y : 0u;
            t[4 * q + 2] = ok ? a.z : 0u;
            t[4 * q + 3] = ok ? a.w : 0u;
        }
        if constexpr (PREC == NVQ_W4A8) {
            int sum = 0;
#pragma unroll
            for (int d = 0; d < 8; ++d) sum = __builtin_amdgcn_sdot4(0x01010101, (int)t[d], sum, false);
            neg8[i] = -8 * sum;
            xsg[i] = PER_GROUP ? __uint_as_float(lds_read4(lds_addr(sh.xsg) + gc * 4)) : 1.0f;
        } else {
            float sum = 0.0f;
#pragma unroll
            for (int j = 0; j < 16; ++j) sum = dot2_bf16(0x3f803f80u, t[j], sum);
            xoff[i] = -136.0f * sum;
        }
        if constexpr (XREG) {
#pragma unroll
            for (int d = 0; d < XR; ++d) xr[i][d] = t[d];
        }
    }
    // Lanes past the end of a ragged row (K no multiple of 2048) read ring
    // slots that no load has written: their scale is forced to zero and their
    // activations are zero, so whatever bits sit there contribute exactly 0.
    const int r0 = gw * ph.rows_per_wave;
    int r1 = r0 + ph.rows_per_wave;
    r1 = r1 < ph.total_rows ? r1 : ph.total_rows;
    if (r0 >= r1) return;
    const uint32_t ring_base = lds_addr(&sh.ring[w][0][0]) + lane * 16;
    const uint32_t sring_base = lds_addr(&sh.sring[w][0][0]) + lane * 2;

    ChunkRegs<!XREG> nxt;
    // Start the LDS reads of the next chunk in stream order; i_next is its
    // position in its row.  Entering a new unit first waits until the unit has
    // landed: at that point every unit but the one being read and the one
    // still to be refilled is in flight behind it.
    auto fetch = [&](int i_next) {
        const uint32_t slot = st.rslot;
        if ((slot & 1u) == 0) __builtin_amdgcn_s_waitcnt(vmcnt_imm(kOpsPerUnit * (kUnits - 2)));
        asm volatile("ds_read_b128 %0, %2\n\tds_read_u16 %1, %3"
                     : "=&v"(nxt.w), "=&v"(nxt.s)
                     : "v"(ring_base + slot * 1024u), "v"(sring_base + slot * 128u)
                     : "memory");
        if constexpr (!XREG) {
            asm volatile("ds_read_b128 %0, %4\n\tds_read_b128 %1, %4 offset:16\n\t"
                         "ds_read_b128 %2, %4 offset:32\n\tds_read_b128 %3, %4 offset:48"
                         : "=&v"(nxt.x[0]), "=&v"(nxt.x[1]), "=&v"(nxt.x[2]), "=&v"(nxt.x[3])
                         : "v"(xaddr[i_next])
                         : "memory");
        }
        st.rslot = slot + 1 == kSlots ? 0 : slot + 1;
    };
    // Wait for the reads started by fetch().  The registers are tied to the
    // wait so that no use (and no copy) of them can be scheduled before it; the
    // wait sits in the same iteration as the fetch, never across the loop
    // back-edge, where the compiler may insert register copies.
    auto landed = [&]() {
        if constexpr (XREG) {
            asm volatile("s_waitcnt lgkmcnt(0)" : "+v"(nxt.w), "+v"(nxt.s) : : "memory");
        } else {
            asm volatile("s_waitcnt lgkmcnt(0)"
                         : "+v"(nxt.w), "+v"(nxt.s), "+v"(nxt.x[0]), "+v"(nxt.x[1]), "+v"(nxt.x[2]),
                           "+v"(nxt.x[3])
                         : : "memory");
        }
    };
    fetch(0);
    landed();

    float yv = 0.0f;  // results of up to 64 rows, one per lane, until they are stored
    for (int row = r0; row < r1; ++row) {
        float sum = 0.0f;
#pragma unroll
        for (int i = 0; i < GPL; ++i) {
            const ChunkRegs<!XREG> cur = nxt;
            // slot the current chunk came from = the one before rslot
            const uint32_t cslot = st.rslot == 0 ? kSlots - 1 : st.rslot - 1;
            const bool more = !(i == GPL - 1 && row == r1 - 1);
            if (more) fetch(i == GPL - 1 ? 0 : i + 1);

            const uint4 wv = make_uint4(cur.w.x, cur.w.y, cur.w.z, cur.w.w);
            float sw = okv[i] ? half_bits_to_float((uint16_t)cur.s) : 0.0f;
            if constexpr (PREC == NVQ_W4A8) {
                const int acc = dot_w4a8(wv, xr[i], neg8[i]);
                if (PER_GROUP) sw *= xsg[i];
                sum = fmaf(sw, (float)acc, sum);
            } else if constexpr (XREG) {
                sum = fmaf(sw, dot_w4a16(wv, xr[i], xoff[i]), sum);
            } else {
                uint32_t xv[16];
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    xv[4 * q + 0] = cur.x[q].x;
                    xv[4 * q + 1] = cur.x[q].y;
                    xv[4 * q + 2] = cur.x[q].z;
                    xv[4 * q + 3] = cur.x[q].w;
                }
                const float part = dot_w4a16(wv, xv, xoff[i]);
                sum = fmaf(sw, okv[i] ? part : 0.0f, sum);
            }
            if (cslot & 1u) {  // second chunk of a unit used up: refill the unit's two slots
                issue_unit(st.ic, tab, gw, sh, w, (int)st.uslot, lane, dummy);
                st.uslot = st.uslot + 1 == kUnits ? 0 : st.uslot + 1;
            }
            if (more) landed();
        }
        sum = wave_sum_to_lane63(sum);
        // park the row's result in lane (row - r0) % 64; one store per 64 rows
        const float tot =
            __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, sum), 63));
        const int k = row - r0;
        if (lane == (k & 63)) yv = PREC == NVQ_W4A8 ? tot * xs_token : tot;
        if ((k & 63) == 63 || row == r1 - 1) {
            const int r = row - (k & 63) + lane;  // the row this lane holds
            if (r <= row) {
                int first = 0;
                void *y = ph.y[0];
                int dt = ph.y_dtype[0];
#pragma unroll
                for (int sgm = 1; sgm < kMaxSeg; ++sgm)
                    if (sgm < ph.nseg && r >= ph.row_end[sgm - 1]) {
                        first = ph.row_end[sgm - 1];
                        y = ph.y[sgm];
                        dt = ph.y_dtype[sgm];
                    }
                store_out(y, dt, r - first, yv);
            }
        }
    }
}

// Quantise the staged bf16 input in place (streaming waves, cooperatively).
// On return xstage holds K int8 codes; returns the per-token scale (1 when the
// scales are per group).
template <bool PER_GROUP>
__device__ __forceinline__ float quantise_stage(const StreamPhase &ph, Shared &sh, int w, int lane,
                                                uint32_t stage) {
    const int t = w * 64 + lane;             // 0 .. kStreamWaves*64-1
    constexpr int NT = kStreamWaves * 64;
    constexpr int MAXC = (kStreamMaxK / 8 + NT - 1) / NT;  // chunks of 8 values per lane
    const int chunks = ph.K / 8;
    uint4 raw[MAXC];
    float amax = 0.0f;
#pragma unroll
    for (int k = 0; k < MAXC; ++k) {
        const int c = t + k * NT;
        raw[k] = make_uint4(0, 0, 0, 0);
        if (k * NT < chunks) {  // uniform: this round holds data for some lane
            if (c < chunks) raw[k] = lds_read16(stage + c * 16);
            const uint32_t wv[4] = {raw[k].x, raw[k].y, raw[k].z, raw[k].w};
#pragma unroll
            for (int d = 0; d < 4; ++d) {
                amax = fmaxf(amax, fabsf(bf16_bits_to_float(wv[d] & 0xffffu)));
                amax = fmaxf(amax, fabsf(bf16_bits_to_float(wv[d] >> 16)));
            }
        }
    }
    float s_tok = 0.0f;
    if (!PER_GROUP) {
#pragma unroll
        for (int off = 32; off > 0; off >>= 1) amax = fmaxf(amax, __shfl_xor(amax, off, 64));
        if (lane == 0) lds_write4(lds_addr(&sh.amax_part[w]), __float_as_uint(amax));
    }
    lds_barrier();  // everyone has read its raw values; partial maxima are visible
    if (!PER_GROUP) {
        float a = 0.0f;
#pragma unroll
        for (int i = 0; i < kStreamWaves; ++i)
            a = fmaxf(a, __uint_as_float(lds_read4(lds_addr(&sh.amax_part[i]))));
        s_tok = a / 127.0f;
    }
    const uint32_t qstage = stage;
#pragma unroll
    for (int k = 0; k < MAXC; ++k) {
        if (k * NT >= chunks) break;
        const int c = t + k * NT;
        const uint32_t wv[4] = {raw[k].x, raw[k].y, raw[k].z, raw[k].w};
        float s = s_tok;
        if (PER_GROUP) {
            float a = 0.0f;
#pragma unroll
            for (int d = 0; d < 4; ++d) {
                a = fmaxf(a, fabsf(bf16_bits_to_float(wv[d] & 0xffffu)));
                a = fmaxf(a, fabsf(bf16_bits_to_float(wv[d] >> 16)));
            }
            a = fmaxf(a, __shfl_xor(a, 1, 64));
            a = fmaxf(a, __shfl_xor(a, 2, 64));
            s = a / 127.0f;
            if (c < chunks && (c & 3) == 0) lds_write4(lds_addr(&sh.xsg[c >> 2]), __float_as_uint(s));
        }
        uint32_t out[2] = {0, 0};
#pragma unroll
        for (int d = 0; d < 4; ++d) {
            int q0 = 0, q1 = 0;
            if (s != 0.0f) {
                float r0 = rintf(bf16_bits_to_float(wv[d] & 0xffffu) / s);
                float r1 = rintf(bf16_bits_to_float(wv[d] >> 16) / s);
                q0 = (int)fminf(fmaxf(r0, -127.0f), 127.0f);
                q1 = (int)fminf(fmaxf(r1, -127.0f), 127.0f);
            }
            out[d >> 1] |= ((uint32_t)(q0 & 0xff) | ((uint32_t)(q1 & 0xff) << 8)) << (16 * (d & 1));
        }
        if (c < chunks) lds_write8(qstage + c * 8, out[0], out[1]);
    }
    lds_barrier();  // codes (and group scales) are visible
    return PER_GROUP ? 1.0f : s_tok;  // group scales are applied per chunk instead
}

template <int PREC, bool PER_GROUP>
__device__ __forceinline__ void consume_dispatch(const StreamPhase &ph, const StreamPhase *tab,
                                                 StreamState &st, Shared &sh, int w, int gw,
                                                 int lane, const uint4 *dummy, float xs,
                                                 uint32_t stage) {
    switch (ph.gpl) {
        case 1: consume_phase<PREC, 1, PER_GROUP>(ph, tab, st, sh, w, gw, lane, dummy, xs, stage); break;
        case 2: consume_phase<PREC, 2, PER_GROUP>(ph, tab, st, sh, w, gw, lane, dummy, xs, stage); break;
        case 3: consume_phase<PREC, 3, PER_GROUP>(ph, tab, st, sh, w, gw, lane, dummy, xs, stage); break;
        case 4: consume_phase<PREC, 4, PER_GROUP>(ph, tab, st, sh, w, gw, lane, dummy, xs, stage); break;
        case 5: consume_phase<PREC, 5, PER_GROUP>(ph, tab, st, sh, w, gw, lane, dummy, xs, stage); break;
        case 6: consume_phase<PREC, 6, PER_GROUP>(ph, tab, st, sh, w, gw, lane, dummy, xs, stage); break;
        default: consume_phase<PREC, 7, PER_GROUP>(ph, tab, st, sh, w, gw, lane, dummy, xs, stage); break;
    }
}

// Optional per-phase timestamps (100 MHz wall clock) of workgroup 0:
// trace[p][0..4] control wave: wait begin, flags seen, input staged, phase
// computed, outputs published; trace[p][5..7] streaming wave 0: input seen,
// activations ready, own rows done.
constexpr int kTraceSlots = 8;
__device__ __forceinline__ void trace_mark(unsigned long long *trace, int wg, int lane, int p,
                                           int slot) {
    if (trace && wg == 0 && lane == 0) trace[p * kTraceSlots + slot] = wall_clock64();
}

template <bool PER_GROUP>
__global__ __launch_bounds__(kStreamThreads, 1) void decode_stream_kernel(
    const StreamPhase *__restrict__ tab, int nphase, uint32_t *__restrict__ flags,
    uint32_t *__restrict__ status, uint32_t flag_base, const uint4 *__restrict__ dummy,
    unsigned long long *__restrict__ trace) {
    __shared__ Shared sh;
    // wave index, made provably wave-uniform; wave 0 also carries the control duties
    const int w = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int lane = threadIdx.x & 63;
    const int wg = blockIdx.x;
    const int nwg = gridDim.x;
    if (threadIdx.x == 0) sh.abort = 0;

    const int gw = wg * kStreamWaves + w;
    StreamState st;
    st.ic.p = 0;
    st.ic.nphase = nphase;
    cursor_enter(st.ic, tab, gw);
    st.rslot = 0;
    st.uslot = 0;
    for (int u = 0; u < kUnits; ++u)  // fill the ring
        issue_unit(st.ic, tab, gw, sh, w, u, lane, dummy);

    // Stage the input vector of phase q (bf16, K values) with global->LDS
    // loads, all in flight at once; completion is awaited later with vmcnt(0).
    auto stage_input = [&](int q) {
        const StreamPhase &pq = tab[q];
        const uint4 *xsrc = reinterpret_cast<const uint4 *>(pq.x);
        const int n16 = pq.K / 8;
        for (int c0 = 0; c0 < n16; c0 += 64)
            if (c0 + lane < n16)
                __builtin_amdgcn_global_load_lds((const void *)(xsrc + c0 + lane),
                                                 (lds_void_ptr)&sh.xstage[q & 1][c0], 16, 0, 0);
    };
    bool staged = false;  // wave 0: the current phase's input is already on its way

    for (int p = 0; p < nphase; ++p) {
        const StreamPhase &ph = tab[p];
        const uint32_t stage = lds_addr(&sh.xstage[p & 1][0]);
        if (w == 0) {
            // ---- control duty 1: honour the phase's dependency, have its input in LDS ----
            bool ok = true;
            trace_mark(trace, wg, lane, p, 0);
            if (ph.wait_phase >= 0) {
                // every workgroup must have published phase wait_phase
                const uint32_t target = flag_base + (uint32_t)ph.wait_phase + 1u;
                uint32_t spins = 0;
                for (;;) {
                    bool all = true;
                    for (int f0 = 0; f0 < nwg; f0 += 256) {  // four independent loads per lane
                        uint32_t v[4];
#pragma unroll
                        for (int j = 0; j < 4; ++j) {
                            const int f = f0 + j * 64 + lane;
                            v[j] = f < nwg ? __hip_atomic_load(flags + f, __ATOMIC_RELAXED,
                                                               __HIP_MEMORY_SCOPE_AGENT)
                                           : target;
                        }
#pragma unroll
                        for (int j = 0; j < 4; ++j) all = all && (int32_t)(v[j] - target) >= 0;
                    }
                    if (__all(all)) break;
                    if (++spins > kSpinLimit) {
                        ok = false;
                        break;
                    }
                    __builtin_amdgcn_s_sleep(1);
                }
                __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");
            }
            trace_mark(trace, wg, lane, p, 1);
            if (ok) {
                if (!staged) stage_input(p);
                __builtin_amdgcn_s_waitcnt(vmcnt_imm(0));
            } else if (lane == 0) {
                lds_write4(lds_addr(&sh.abort), 1u);
                __hip_atomic_store(status, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            }
            trace_mark(trace, wg, lane, p, 2);
        }
        // B1: this phase's input is staged (or abort raised); every wave has
        // left the previous phase, so the other stage buffer is free
        lds_barrier();
        if (lds_read4(lds_addr(&sh.abort))) break;
        if (w == 0) {
            trace_mark(trace, wg, lane, p, 5);
            // start fetching the next phase's input now if it depends on nothing
            staged = p + 1 < nphase && tab[p + 1].wait_phase < 0;
            if (staged) stage_input(p + 1);
        }
        float xs = 1.0f;
        if (ph.precision == NVQ_W4A8) {
            xs = quantise_stage<PER_GROUP>(ph, sh, w, lane, stage);  // B2, B3 inside
            if (w == 0) trace_mark(trace, wg, lane, p, 6);
            consume_dispatch<NVQ_W4A8, PER_GROUP>(ph, tab, st, sh, w, gw, lane, dummy, xs, stage);
        } else {
            if (w == 0) trace_mark(trace, wg, lane, p, 6);
            consume_dispatch<NVQ_W4A16, false>(ph, tab, st, sh, w, gw, lane, dummy, xs, stage);
        }
        if (w == 0) trace_mark(trace, wg, lane, p, 7);
        if (ph.publish) {
            // a later phase reads or overwrites what this one touched: make the
            // workgroup's outputs visible device-wide, then raise its flag
            __builtin_amdgcn_s_waitcnt(vmcnt_imm(0));  // this wave's stores have completed
            lds_barrier();                             // B4
            if (w == 0) {
                trace_mark(trace, wg, lane, p, 3);
                __builtin_amdgcn_fence(__ATOMIC_RELEASE, "agent");
                if (lane == 0)
                    __hip_atomic_store(flags + wg, flag_base + (uint32_t)p + 1u, __ATOMIC_RELAXED,
                                       __HIP_MEMORY_SCOPE_AGENT);
                trace_mark(trace, wg, lane, p, 4);
            }
        }
    }
    __builtin_amdgcn_s_waitcnt(vmcnt_imm(0));  // no load may outlive the wave
}

}  // namespace

int stream_grid_limit() {
    static int cached = -1;
    if (cached < 0) {
        int per_cu = 0;
        if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, decode_stream_kernel<false>,
                                                         kStreamThreads, 0) != hipSuccess)
            per_cu = 0;
        cached = per_cu >= 1 ? device_cu_count() : 0;
    }
    return cached;
}

int launch_decode_stream(const StreamPhase *tab_dev, int nphase, int act_group, uint32_t *flags,
                         uint32_t *status, uint32_t flag_base, const void *dummy, int nwg,
                         unsigned long long *trace, hipStream_t st) {
    const dim3 grid(nwg), block(kStreamThreads);
    if (act_group == 32)
        hipLaunchKernelGGL(decode_stream_kernel<true>, grid, block, 0, st, tab_dev, nphase, flags,
                           status, flag_base, reinterpret_cast<const uint4 *>(dummy), trace);
    else
        hipLaunchKernelGGL(decode_stream_kernel<false>, grid, block, 0, st, tab_dev, nphase, flags,
                           status, flag_base, reinterpret_cast<const uint4 *>(dummy), trace);
    NVQ_HIP_TRY(hipGetLastError());
    return NVQ_OK;
}

}  // namespace nvq
