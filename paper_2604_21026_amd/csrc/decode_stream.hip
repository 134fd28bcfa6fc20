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
// Structure.  One workgroup of kStreamWaves waves per compute unit, all
// co-resident.  Each wave owns a contiguous range of rows in every phase and
// sees its work as one flat sequence of 1 KiB chunks across all phases:
//   - per phase, first its share of the phase's input vector (512 bf16 values
//     per chunk, chunks dealt round-robin to the waves of the workgroup),
//   - then its weight rows (64 groups x 16 B of one row per chunk).
// Chunks are fetched with non-temporal global->LDS loads into a per-wave ring
// of kSlots slots and consumed in order; a slot is refilled as soon as its
// chunk has been taken out, independent of phase boundaries.  The fp16 scales
// travel the same way (one 2-byte load per lane and chunk).  Ring loads are
// the only vector-memory loads of a wave on the fast path, issued two per
// chunk, so the number of loads in flight behind a chunk is a compile-time
// constant and one `s_waitcnt vmcnt(n)` tells when it has landed.
//
// Per phase the workgroup prepares the input once: each wave takes its share
// out of its ring, the waves agree on the absmax (W4A8), quantise or copy
// their shares into an LDS buffer laid out in 16-byte planes, and store per
// group the constant that the deferred offset correction needs.  Then every
// wave walks its weight chunks; the lane's activations of a chunk's group
// come from that LDS buffer.
//
// Ordering.  The host marks, per phase, the latest earlier phase whose
// buffers it conflicts with.  Such a phase takes its input only after every
// workgroup has published that phase (one flag word per workgroup, no
// atomics), and its input is read after the wait instead of being streamed
// ahead.  A bounded spin turns a stuck wait (e.g. the grid not co-resident)
// into an error status instead of a hang.
#include "decode_stream.h"

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

constexpr int kSlots = 12;                 // ring slots per wave (1 KiB weights + 256 B scales)
constexpr int kOpsPerChunk = 2;            // scale load + weight load
constexpr int kMaxG = kStreamMaxK / 32;    // 448 groups
constexpr int kXChunkElems = 512;          // bf16 values per input chunk
constexpr int kMaxXShare = (kStreamMaxK / kXChunkElems + kStreamWaves - 1) / kStreamWaves;  // 4
constexpr uint32_t kSpinLimit = 4u << 20;  // polls before a wait gives up (seconds)

// s_waitcnt immediate that waits for vmcnt <= n only (gfx9 encoding:
// vmcnt[3:0] | expcnt[6:4] | lgkmcnt[11:8] | vmcnt[5:4] at [15:14]).
constexpr int vmcnt_imm(int n) { return (n & 15) | ((n >> 4) << 14) | 0x0f70; }

struct Shared {
    uint4 ring[kStreamWaves][kSlots][64];
    uint32_t sring[kStreamWaves][kSlots][64];  // one dword per lane: zero-extended fp16 scale
    uint4 xbuf[kStreamMaxK * 2 / 16];  // the phase's activations in planes of G x 16 bytes
    uint32_t xaux[kMaxG];              // per group: -8*sum(codes) (int) or -136*sum(x) (float)
    float xsg[kMaxG];                  // per-group activation scales (act_group 32)
    float amax_part[kStreamWaves];
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

// ---- the issue side: where the wave's next chunk comes from -------------------
// All fields are wave-uniform.  A run is a sequence of chunks at a constant
// pointer stride: the wave's share of a phase's input, or consecutive weight
// rows inside one matrix (a single row when K is no multiple of 2048).
struct Issue {
    const uint4 *q;     // next chunk: 64 x 16 bytes
    const uint16_t *s;  // its 64 scales (the dummy line for input chunks)
    int qstep, sstep;   // pointer advance per chunk, in elements
    int left;           // chunks left in the run
    int tail;           // valid lanes in the run's last chunk (64 = all)
    int p;              // phase of the run
    int part;           // 0: input share issued next, 1: weight rows
    int row, row_stop;  // weight rows of phase p not yet turned into runs
};

__device__ __forceinline__ void issue_next_run(Issue &c, CPhase *tab, int nphase, int w,
                                               int gw, const uint4 *dummy) {
    for (;;) {
        if (c.p >= nphase) {
            // past the last phase: dummy chunks keep the load count constant
            c.q = dummy;
            c.s = reinterpret_cast<const uint16_t *>(dummy);
            c.qstep = c.sstep = 0;
            c.left = 1 << 30;
            c.tail = 64;
            return;
        }
        CPhase &ph = tab[c.p];
        if (c.part == 0) {
            // the wave's share of the input vector: chunks w, w + waves, ...
            c.part = 1;
            c.row = gw * ph.rows_per_wave;
            const int stop = c.row + ph.rows_per_wave;
            c.row_stop = stop < ph.total_rows ? stop : ph.total_rows;
            const int nxc = (ph.K + kXChunkElems - 1) / kXChunkElems;
            if (w < nxc) {
                const int n = (nxc - w + kStreamWaves - 1) / kStreamWaves;
                const int last = w + (n - 1) * kStreamWaves;
                const int tail = ph.K / 8 - last * 64;  // 16-byte pieces left for the last chunk
                const bool ahead = ph.wait_phase < 0;   // else the input is read after the wait
                c.q = ahead ? reinterpret_cast<const uint4 *>(ph.x) + w * 64 : dummy;
                c.s = reinterpret_cast<const uint16_t *>(dummy);
                c.qstep = ahead ? kStreamWaves * 64 : 0;
                c.sstep = 0;
                c.left = n;
                c.tail = ahead && tail < 64 ? tail : 64;
                return;
            }
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
            const bool ragged = (ph.G & 63) != 0;
            int rows = (c.row_stop < end ? c.row_stop : end) - c.row;
            if (ragged) rows = 1;
            const int64_t off = (int64_t)(c.row - first) * ph.G;
            c.q = q + off;
            c.s = s + off;
            c.qstep = c.sstep = 64;
            c.left = rows * ph.gpl;
            c.tail = ragged ? ph.G - (ph.gpl - 1) * 64 : 64;
            c.row += rows;
            return;
        }
        ++c.p;
        c.part = 0;
    }
}

// Issue the two loads of the next chunk into ring slot `slot`.
__device__ __forceinline__ void issue_chunk(Issue &c, CPhase *tab, int nphase,
                                            Shared &sh, int w, int gw, int slot, int lane,
                                            const uint4 *dummy) {
    const int valid = c.left == 1 ? c.tail : 64;
    if (valid >= 64) {
        __builtin_amdgcn_global_load_lds((const void *)(c.s + lane),
                                         (lds_void_ptr)&sh.sring[w][slot][0], 2, 0, 2);
        __builtin_amdgcn_global_load_lds((const void *)(c.q + lane),
                                         (lds_void_ptr)&sh.ring[w][slot][0], 16, 0, 2);
    } else {
        // lanes past the end issue nothing; lane 0 is always valid, so both
        // loads are issued and the load count stays exact
        if (lane < valid)
            __builtin_amdgcn_global_load_lds((const void *)(c.s + lane),
                                             (lds_void_ptr)&sh.sring[w][slot][0], 2, 0, 2);
        if (lane < valid)
            __builtin_amdgcn_global_load_lds((const void *)(c.q + lane),
                                             (lds_void_ptr)&sh.ring[w][slot][0], 16, 0, 2);
    }
    c.q += c.qstep;
    c.s += c.sstep;
    if (--c.left == 0) issue_next_run(c, tab, nphase, w, gw, dummy);
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

// ---- per-wave stream state ---------------------------------------------------------
struct Stream {
    Issue ic;
    uint32_t slot;  // ring slot of the next chunk in stream order
};

// Optional per-phase timestamps (100 MHz wall clock) taken by wave 0 of
// workgroup 0; slot meanings are documented with nvq_plan_trace.
constexpr int kTraceSlots = 8;
__device__ __forceinline__ void trace_mark(unsigned long long *trace, int wg, int w, int lane,
                                           int p, int slot) {
    if (trace && wg == 0 && w == 0 && lane == 0) trace[p * kTraceSlots + slot] = wall_clock64();
}

template <bool PER_GROUP>
__global__ __launch_bounds__(kStreamThreads, 1) void decode_stream_kernel(
    const StreamPhase *__restrict__ tab_generic, int nphase, uint32_t *__restrict__ flags,
    uint32_t *__restrict__ status, uint32_t flag_base, const uint4 *__restrict__ dummy,
    unsigned long long *__restrict__ trace) {
    __shared__ Shared sh;
    CPhase *tab = (CPhase *)tab_generic;
    // wave index, made provably wave-uniform; wave 0 also talks to the other workgroups
    const int w = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int lane = threadIdx.x & 63;
    const int wg = blockIdx.x;
    const int nwg = gridDim.x;
    const int gw = wg * kStreamWaves + w;
    if (threadIdx.x == 0) lds_write4(lds_addr(&sh.abort), 0u);

    const uint32_t ring_base = lds_addr(&sh.ring[w][0][0]) + lane * 16;
    const uint32_t sring_base = lds_addr(&sh.sring[w][0][0]) + lane * 4;
    const uint32_t xbuf_base = lds_addr(sh.xbuf);
    const uint32_t xaux_base = lds_addr(sh.xaux);
    const uint32_t xsg_base = lds_addr(sh.xsg);

    Stream st;
    st.ic.p = 0;
    st.ic.part = 0;
    st.ic.left = 0;
    issue_next_run(st.ic, tab, nphase, w, gw, dummy);
    st.slot = 0;
    for (int u = 0; u < kSlots; ++u)  // fill the ring
        issue_chunk(st.ic, tab, nphase, sh, w, gw, u, lane, dummy);

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
        issue_chunk(st.ic, tab, nphase, sh, w, gw, (int)st.slot, lane, dummy);
        st.slot = st.slot + 1 == kSlots ? 0 : st.slot + 1;
        return make_uint4(v.x, v.y, v.z, v.w);
    };

    for (int p = 0; p < nphase; ++p) {
        CPhase &ph = tab[p];
        const int G = ph.G;
        const int K = ph.K;
        const bool w4a8 = ph.precision == NVQ_W4A8;
        trace_mark(trace, wg, w, lane, p, 0);

        // ---- dependency: wait until every workgroup has published phase wait_phase ----
        const bool dependent = ph.wait_phase >= 0;
        if (dependent) {
            if (w == 0) {
                const uint32_t target = flag_base + (uint32_t)ph.wait_phase + 1u;
                uint32_t spins = 0;
                bool ok = true;
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
                if (!ok && lane == 0) {
                    lds_write4(lds_addr(&sh.abort), 1u);
                    __hip_atomic_store(status, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                }
            }
            lds_barrier();  // the dependency is satisfied (or abort raised) for the whole workgroup
            if (lds_read4(lds_addr(&sh.abort))) break;
        }
        trace_mark(trace, wg, w, lane, p, 1);

        // ---- this wave's share of the input vector: chunks w, w + waves, ... -----------
        const int nxc = (K + kXChunkElems - 1) / kXChunkElems;
        uint4 xsh[kMaxXShare];
        float amax = 0.0f;
#pragma unroll
        for (int k = 0; k < kMaxXShare; ++k) {
            xsh[k] = make_uint4(0, 0, 0, 0);
            const int j = w + k * kStreamWaves;  // chunk index (uniform)
            if (j < nxc) {
                uint32_t unused;
                uint4 v = pop_chunk(unused);  // a dummy chunk when the phase is dependent
                const bool valid = j * 64 + lane < K / 8;
                if (dependent)
                    v = valid ? reinterpret_cast<const uint4 *>(ph.x)[j * 64 + lane]
                              : make_uint4(0, 0, 0, 0);
                if (!valid) v = make_uint4(0, 0, 0, 0);
                xsh[k] = v;
                const uint32_t wv[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
                for (int d = 0; d < 4; ++d) {
                    amax = fmaxf(amax, fabsf(bf16_bits_to_float(wv[d] & 0xffffu)));
                    amax = fmaxf(amax, fabsf(bf16_bits_to_float(wv[d] >> 16)));
                }
            }
        }
        if (w4a8 && !PER_GROUP) {
            amax = wave_max_to_lane63(amax);
            if (lane == 63) lds_write4(lds_addr(&sh.amax_part[w]), __float_as_uint(amax));
        }
        trace_mark(trace, wg, w, lane, p, 2);
        // B1: every wave has left the previous phase (the activation buffer is
        // free) and, for W4A8, the partial maxima are visible
        lds_barrier();
        trace_mark(trace, wg, w, lane, p, 5);

        float s_tok = 0.0f;
        if (w4a8 && !PER_GROUP) {
            const uint4 a = lds_read16(lds_addr(&sh.amax_part[0]));
            const uint4 b = lds_read16(lds_addr(&sh.amax_part[4]));
            float m = fmaxf(fmaxf(__uint_as_float(a.x), __uint_as_float(a.y)),
                            fmaxf(__uint_as_float(a.z), __uint_as_float(a.w)));
            m = fmaxf(m, fmaxf(fmaxf(__uint_as_float(b.x), __uint_as_float(b.y)),
                               fmaxf(__uint_as_float(b.z), __uint_as_float(b.w))));
            s_tok = m / 127.0f;
        }
        // Each lane holds 8 consecutive values = a quarter of group g; the four
        // lanes of a group sit next to each other.
        const int quarter = lane & 3;
#pragma unroll
        for (int k = 0; k < kMaxXShare; ++k) {
            const int j = w + k * kStreamWaves;
            if (j < nxc) {
                const int g = j * 16 + (lane >> 2);
                const bool valid = g < G;
                const uint32_t wv[4] = {xsh[k].x, xsh[k].y, xsh[k].z, xsh[k].w};
                if (w4a8) {
                    float s = s_tok;
                    if (PER_GROUP) {
                        float a = 0.0f;
#pragma unroll
                        for (int d = 0; d < 4; ++d) {
                            a = fmaxf(a, fabsf(bf16_bits_to_float(wv[d] & 0xffffu)));
                            a = fmaxf(a, fabsf(bf16_bits_to_float(wv[d] >> 16)));
                        }
                        s = quad_max(a) / 127.0f;
                        if (valid && quarter == 0) lds_write4(xsg_base + g * 4, __float_as_uint(s));
                    }
                    uint32_t out[2] = {0, 0};
                    int qsum = 0;
#pragma unroll
                    for (int d = 0; d < 4; ++d) {
                        int q0 = 0, q1 = 0;
                        if (s != 0.0f) {
                            const float r0 = rintf(bf16_bits_to_float(wv[d] & 0xffffu) / s);
                            const float r1 = rintf(bf16_bits_to_float(wv[d] >> 16) / s);
                            q0 = (int)fminf(fmaxf(r0, -127.0f), 127.0f);
                            q1 = (int)fminf(fmaxf(r1, -127.0f), 127.0f);
                        }
                        qsum += q0 + q1;
                        out[d >> 1] |= ((uint32_t)(q0 & 0xff) | ((uint32_t)(q1 & 0xff) << 8))
                                       << (16 * (d & 1));
                    }
                    qsum = quad_sum(qsum);
                    if (valid) {
                        // codes of elements 0..15 in plane 0, 16..31 in plane 1
                        lds_write8(xbuf_base + (quarter >> 1) * (G * 16) + g * 16 + (quarter & 1) * 8,
                                   out[0], out[1]);
                        if (quarter == 0) lds_write4(xaux_base + g * 4, (uint32_t)(-8 * qsum));
                    }
                } else {
                    float part = 0.0f;
#pragma unroll
                    for (int d = 0; d < 4; ++d) part = dot2_bf16(0x3f803f80u, wv[d], part);
                    part = quad_sum(part);
                    if (valid) {
                        // elements 8q..8q+7 in plane q
                        lds_write16(xbuf_base + quarter * (G * 16) + g * 16, xsh[k]);
                        if (quarter == 0)
                            lds_write4(xaux_base + g * 4, __float_as_uint(-136.0f * part));
                    }
                }
            }
        }
        lds_barrier();  // B2: the activations of the phase are in place
        trace_mark(trace, wg, w, lane, p, 6);

        // ---- this wave's weight rows ---------------------------------------------------
        const int gpl = ph.gpl;
        const int r0 = gw * ph.rows_per_wave;
        int r1 = r0 + ph.rows_per_wave;
        r1 = r1 < ph.total_rows ? r1 : ph.total_rows;
        const int nchunks = r1 > r0 ? (r1 - r0) * gpl : 0;
        const float xs = (w4a8 && !PER_GROUP) ? s_tok : 1.0f;
        const uint32_t plane = (uint32_t)G * 16u;
        int i = 0;        // chunk position inside the row
        int row = r0;
        float sum = 0.0f;
        float yv = 0.0f;  // results of up to 64 rows, one per lane, until they are stored
        for (int c = 0; c < nchunks; ++c) {
            // the lane's group of this chunk and its activations
            const int g = i * 64 + lane;
            const bool ok = g < G;
            const uint32_t ga = xbuf_base + (ok ? g : 0) * 16;
            const uint32_t aux_a = xaux_base + (ok ? g : 0) * 4;
            u32x4_t xa, xb, xc = {0, 0, 0, 0}, xd = {0, 0, 0, 0};
            uint32_t aux, sgbits = 0;
            if (w4a8) {
                asm volatile("ds_read_b128 %0, %3\n\tds_read_b128 %1, %4\n\tds_read_b32 %2, %5"
                             : "=&v"(xa), "=&v"(xb), "=&v"(aux)
                             : "v"(ga), "v"(ga + plane), "v"(aux_a)
                             : "memory");
                if (PER_GROUP)
                    asm volatile("ds_read_b32 %0, %1"
                                 : "=&v"(sgbits)
                                 : "v"(xsg_base + (ok ? g : 0) * 4)
                                 : "memory");
            } else {
                asm volatile("ds_read_b128 %0, %5\n\tds_read_b128 %1, %6\n\tds_read_b128 %2, %7\n\t"
                             "ds_read_b128 %3, %8\n\tds_read_b32 %4, %9"
                             : "=&v"(xa), "=&v"(xb), "=&v"(xc), "=&v"(xd), "=&v"(aux)
                             : "v"(ga), "v"(ga + plane), "v"(ga + 2 * plane), "v"(ga + 3 * plane),
                               "v"(aux_a)
                             : "memory");
            }
            uint32_t sbits;
            const uint4 wq = pop_chunk(sbits);  // its lgkmcnt(0) also covers the reads above
            // nothing below may be scheduled (or copied) before that wait
            asm volatile("" : "+v"(xa), "+v"(xb), "+v"(xc), "+v"(xd), "+v"(aux), "+v"(sgbits));
            const u32x4_t wv = {wq.x, wq.y, wq.z, wq.w};
            float sw = ok ? half_bits_to_float((uint16_t)sbits) : 0.0f;
            if (w4a8) {
                const int acc = dot_w4a8(wv, xa, xb, (int)aux);
                if (PER_GROUP) sw *= __uint_as_float(sgbits);
                sum = fmaf(sw, (float)acc, sum);
            } else {
                const u32x4_t xq[4] = {xa, xb, xc, xd};
                sum = fmaf(sw, dot_w4a16(wv, xq, __uint_as_float(aux)), sum);
            }
            if (++i == gpl) {
                // end of a row: reduce, park the result in lane (row - r0) % 64
                i = 0;
                const float tot = __builtin_bit_cast(
                    float, __builtin_amdgcn_readlane(
                               __builtin_bit_cast(int, wave_sum_to_lane63(sum)), 63));
                sum = 0.0f;
                const int k = row - r0;
                if (lane == (k & 63)) yv = tot * xs;
                if ((k & 63) == 63 || row == r1 - 1) {  // one store per 64 rows
                    const int r = row - (k & 63) + lane;
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
                ++row;
            }
        }
        trace_mark(trace, wg, w, lane, p, 7);

        if (ph.publish) {
            // a later phase reads or overwrites what this one touched: make the
            // workgroup's outputs visible device-wide, then raise its flag
            __builtin_amdgcn_s_waitcnt(vmcnt_imm(0));  // this wave's stores have completed
            lds_barrier();
            if (w == 0) {
                trace_mark(trace, wg, w, lane, p, 3);
                __builtin_amdgcn_fence(__ATOMIC_RELEASE, "agent");
                if (lane == 0)
                    __hip_atomic_store(flags + wg, flag_base + (uint32_t)p + 1u, __ATOMIC_RELAXED,
                                       __HIP_MEMORY_SCOPE_AGENT);
                trace_mark(trace, wg, w, lane, p, 4);
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
