// Small-batch (2 <= M <= 32 tokens) products on the matrix cores, as one
// persistent grid per batch of independent phases.  Paper: the W4A8 / W4A16
// kernel descriptions; the arithmetic is that of the per-tile kernel
// (gemv_mfma.hip), what differs is how the weights reach the waves.
//
// A short-lived workgroup per row tile loads, waits, computes and reduces, and
// the few of them that fit a compute unit do not cover the memory latency.
// Here the waves stay: a team (a loader wave and W consumer waves) works off
// groups of consecutive units of the batch (a unit = R consecutive 16-row
// tiles of some phase), dealt so that the teams of an XCD advance through the
// phases together (RingWalk).  A team splits into
//   * one loader wave that copies the weights and scales of the units, column
//     by column (a column = four groups = 64 bytes of each of the 16 rows of a
//     tile), straight from global memory into LDS rings, one ring per consumer
//     wave, running ahead across unit boundaries as far as the rings allow;
//   * W = 4 consumer waves; a step is four consecutive columns of the unit,
//     one per wave (K is a multiple of 512), so the waves advance together.
//     Wave w reads column 4i + w of step i from its ring, loads the
//     activations of the column itself (they come from the L2 cache, and the
//     request for the next column is made before the current one is
//     multiplied), feeds the MFMAs and, at the end of a unit, adds the W
//     partial tiles through LDS in wave order.
// Per step the loader issues 2 x 4 weight loads of 1 KiB (8 rows x 128 bytes)
// and one scale load (32 rows x 32 bytes: the 16 scales of the step's four
// columns).  Its loads are the only ones it has in flight and complete in
// order, so "the oldest step not yet announced has arrived" is an exact vmcnt
// wait; while the ring is full it announces step after step (`landed`), and a
// consumer advances its `consumed` count once a step is in its registers; the
// loader reuses a slot when every wave has consumed it.  All waits are bounded: a wave that gives up sets the abort
// word, every wave then runs to the end without waiting, and the host finds
// the status word set.
#include "gemv_tile.h"
#include "mfma_act.h"

namespace nvq {

namespace {

typedef __attribute__((address_space(3))) void *lds_void_ptr;
// The tables do not change during the kernel; read through the constant
// address space they become scalar loads, which the loader needs: a vector
// load would join its queue of ring loads and be waited for with vmcnt(0).
typedef const __attribute__((address_space(4))) GroupPhase CGroup;
typedef const __attribute__((address_space(4))) uint32_t CWord;

constexpr int kRingWaves = 4;    // consumer waves per team (W)
constexpr int kRingBundle = 3;   // units whose row tiles share the activation operands
constexpr int kRingSteps = 4;    // ring capacity in steps (all may be in flight)
constexpr int kTeamThreads = (kRingWaves + 1) * 64;  // a team: the consumers and their loader
constexpr int kRingR = 2;        // row tiles per unit (the scale load fills 64 lanes)
constexpr uint32_t kRingSpinLimit = 1u << 24;

constexpr int ring_vmcnt_imm(int n) { return (n & 15) | ((n >> 4) << 14) | 0x0f70; }

template <int MT>
struct RingShared {
    // [step][row tile][column pair][row half]: 8 rows x 128 bytes (two columns)
    // per KiB, in the lane order of the loader (ring_lane_of)
    uint4 ring[kRingSteps][kRingR][2][2][64];
    uint4 sring[kRingSteps][64];  // lane (r, n, half): scales of columns 4i+2half, 4i+2half+1
    float red[2][kRingWaves][kRingR * MT * 4][64];   // partial tiles, by unit parity
    alignas(16) uint32_t consumed[kRingWaves];  // steps each wave has copied into registers
    uint32_t landed;                // steps that have arrived in the rings
    uint32_t done;                  // partial tiles written so far (all units)
    uint32_t abort;
};

// LDS words the waves signal through, as instructions: the compiler must not
// cache them, and in the loader it would guard each access with vmcnt(0).
__device__ __forceinline__ uint32_t ring_lds_addr(const void *p) { return (uint32_t)(uintptr_t)p; }
__device__ __forceinline__ uint32_t ring_read_word(uint32_t addr) {
    uint32_t v;
    asm volatile("ds_read_b32 %0, %1\n\ts_waitcnt lgkmcnt(0)" : "=v"(v) : "v"(addr) : "memory");
    return (uint32_t)__builtin_amdgcn_readfirstlane((int)v);
}
typedef uint32_t ring_u32x4 __attribute__((ext_vector_type(4)));
// the smallest of four consecutive words (16-byte aligned), wave-uniform
__device__ __forceinline__ uint32_t ring_read_min4(uint32_t addr) {
    ring_u32x4 v;
    asm volatile("ds_read_b128 %0, %1\n\ts_waitcnt lgkmcnt(0)" : "=v"(v) : "v"(addr) : "memory");
    const uint32_t a = v.x < v.y ? v.x : v.y, b = v.z < v.w ? v.z : v.w;
    return (uint32_t)__builtin_amdgcn_readfirstlane((int)(a < b ? a : b));
}
__device__ __forceinline__ void ring_write_word(uint32_t addr, uint32_t v) {
    asm volatile("ds_write_b32 %0, %1" : : "v"(addr), "v"(v) : "memory");
}
__device__ __forceinline__ void ring_add_word(uint32_t addr, uint32_t v) {
    asm volatile("ds_add_u32 %0, %1" : : "v"(addr), "v"(v) : "memory");
}

// Wait until the word at `addr` has reached `want` (counts only grow) and
// return what it holds.  Gives up after kRingSpinLimit polls or when another
// wave has given up.
__device__ __forceinline__ uint32_t ring_wait(uint32_t addr, uint32_t want, uint32_t abort_addr,
                                              bool &dead) {
    if (dead) return want;
    uint32_t spins = 0, seen;
    while ((int32_t)((seen = ring_read_word(addr)) - want) < 0) {
        __builtin_amdgcn_s_sleep(1);
        if ((++spins & 1023u) == 0 && (ring_read_word(abort_addr) != 0 || spins >= kRingSpinLimit)) {
            ring_write_word(abort_addr, 1u);
            dead = true;
            return want;
        }
    }
    return seen;
}

// ---- the loader wave --------------------------------------------------------
// Where piece `piece` (16 bytes, 0..7) of row n (0..15) of a two-column block
// lies in its KiB: the loader's lane order.  Rows are rotated against each
// other by one piece and neighbouring rows swapped in the second row half, so
// that the 16 lanes that read the same piece of the 16 rows hit 16 different
// groups of LDS banks.
__device__ __forceinline__ int ring_lane_of(int n, int piece) {
    const int q = n & 7, h = n >> 3;
    return 8 * (q ^ h) + ((piece + q) & 7);
}

// The loader's loads are the only ones it has in flight and they complete in
// order: with `outstanding` steps of OPS loads each not yet announced, the
// oldest has arrived when at most (outstanding - 1) * OPS loads are pending.
template <int OPS>
__device__ __forceinline__ void ring_wait_oldest(uint32_t outstanding) {
    if (outstanding >= 4)
        __builtin_amdgcn_s_waitcnt(ring_vmcnt_imm(3 * OPS));
    else if (outstanding == 3)
        __builtin_amdgcn_s_waitcnt(ring_vmcnt_imm(2 * OPS));
    else if (outstanding == 2)
        __builtin_amdgcn_s_waitcnt(ring_vmcnt_imm(OPS));
    else
        __builtin_amdgcn_s_waitcnt(ring_vmcnt_imm(0));
}

// A team's way through its part of the batch.  The batch is cut into parts
// of equal weight bytes, one per XCD (workgroup g runs on XCD g mod 8: the
// compute units of an XCD share an L2 cache), and the teams of an XCD take the
// part's groups of U units in turn: team q the groups q, q + teams, ...  So
// the teams of an XCD advance through the phases together and the operand
// image they all read is one phase's, which stays in their L2; a group that
// crosses a phase boundary is worked off as two bundles.
struct RingWalk {
    int a;       // first unit of the current group
    int u;       // next unit to work on
    int u_end;   // end of the current group
    int p;       // phase of unit u (when u < u_end)
    int part_end, stride;
};

template <int U>
__device__ __forceinline__ void ring_walk_settle(RingWalk &wk, CGroup *tab) {
    if (wk.u >= wk.u_end) {
        wk.a += wk.stride;
        wk.u = wk.a;
        const int e = wk.a + U;
        wk.u_end = e < wk.part_end ? e : wk.part_end;
    }
    if (wk.u < wk.u_end)
        while (wk.u >= tab[wk.p].unit_begin + tab[wk.p].unit_count) ++wk.p;  // phases have units
}

template <int U>
__device__ __forceinline__ RingWalk ring_walk_begin(CGroup *tab, int part_begin, int part_end,
                                                    int p, int q, int teams) {
    RingWalk wk;
    wk.part_end = part_end;
    wk.stride = teams * U;
    wk.a = part_begin + q * U;
    wk.u = wk.a;
    const int e = wk.a + U;
    wk.u_end = e < part_end ? e : part_end;
    wk.p = p;
    if (wk.u < wk.u_end)
        while (wk.u >= tab[wk.p].unit_begin + tab[wk.p].unit_count) ++wk.p;
    return wk;
}

// Units a team works on together: up to U consecutive units of one phase, so
// that the activation operands of a column serve U * R row tiles.
template <int U>
__device__ __forceinline__ int bundle_units(int u, int u_end, int phase_end) {
    int cnt = u_end - u;
    cnt = cnt < phase_end - u ? cnt : phase_end - u;
    return cnt < U ? cnt : U;
}

template <int MT, int U>
__device__ __forceinline__ void ring_loader(CGroup *tab, RingWalk wk, RingShared<MT> &sh,
                                            int lane, bool &dead) {
    constexpr int W = kRingWaves, S = kRingSteps, R = kRingR;
    constexpr int kOps = R * W + 1;  // loads per step
    static_assert(W == 4, "one 16-byte read fetches every wave's count");
    static_assert(S == 4 && kOps * (S - 1) < 64, "ring_wait_oldest covers up to four steps");
    // A load moves whole 128-byte lines: eight rows x two columns, the eight
    // lanes 8q .. 8q + 7 one line.  (64-byte halves of a line fetched by two
    // loads a little apart came from HBM twice too often: rows a power of two
    // bytes apart fall into few sets of the first-level cache, and the line was
    // gone before its second half was asked for.)  Lane 8l + j of the load for
    // row half h holds row 8h + q, q = l xor h, and of it piece (j - q) mod 8;
    // see ring_lane_of.
    const int lq = lane >> 3;
    const int sr = lane >> 5, sn = (lane >> 1) & 15, shalf = lane & 1;
    const uint32_t abort_addr = ring_lds_addr(&sh.abort);
    const uint32_t landed_addr = ring_lds_addr(&sh.landed);
    const uint32_t consumed_addr = ring_lds_addr(&sh.consumed[0]);
    uint32_t T = 0;         // steps issued
    uint32_t published = 0; // steps announced to the consumers
    uint32_t cons_min = 0;  // a lower bound of every wave's consumed count

    while (wk.u < wk.u_end) {
        CGroup &P = tab[wk.p];
        const int u = wk.u;
        const int G = P.G, steps = G >> 4;
        const int cnt = bundle_units<U>(u, wk.u_end, P.unit_begin + P.unit_count);
        const uint4 *gq[U][R][2], *gs[U];
#pragma unroll
        for (int j = 0; j < U; ++j) {
            const int unit = u - P.unit_begin + (j < cnt ? j : 0);
#pragma unroll
            for (int r = 0; r < R; ++r)
#pragma unroll
                for (int h = 0; h < 2; ++h)
                    gq[j][r][h] = locate_row(P.segs, (unit * R + r) * 16 + 8 * h + (lq ^ h), G).qw +
                                  (((lane & 7) - (lq ^ h)) & 7);
            // 16 bytes = the 8 scales of two columns
            gs[j] = reinterpret_cast<const uint4 *>(
                        locate_row(P.segs, (unit * R + sr) * 16 + sn, G).sc) +
                    shalf;
        }
        for (int i = 0; i < steps; ++i) {
#pragma unroll
            for (int j = 0; j < U; ++j) {
                if (j >= cnt) continue;
                // No free slot: announce what has arrived in the meantime (the
                // oldest load first; the wait returns at once if it is there),
                // then watch the consumers.
                uint32_t spins = 0;
                while (T - cons_min >= (uint32_t)S && !dead) {
                    if (published < T) {
                        ring_wait_oldest<kOps>(T - published);
                        ring_write_word(landed_addr, ++published);
                        cons_min = ring_read_min4(consumed_addr);
                        continue;
                    }
                    cons_min = ring_read_min4(consumed_addr);
                    if (T - cons_min < (uint32_t)S) break;
                    __builtin_amdgcn_s_sleep(1);
                    if ((++spins & 1023u) == 0 &&
                        (ring_read_word(abort_addr) != 0 || spins >= kRingSpinLimit)) {
                        ring_write_word(abort_addr, 1u);
                        dead = true;
                    }
                }
                if (!dead) {  // else no further loads; the consumers no longer wait
                    const int slot = (int)(T % S);
#pragma unroll
                    for (int r = 0; r < R; ++r)
#pragma unroll
                        for (int cp = 0; cp < 2; ++cp)
#pragma unroll
                            for (int h = 0; h < 2; ++h)
                                __builtin_amdgcn_global_load_lds(
                                    (const void *)(gq[j][r][h] + 16 * i + 8 * cp),
                                    (lds_void_ptr)&sh.ring[slot][r][cp][h][0], 16, 0, 2);
                    __builtin_amdgcn_global_load_lds((const void *)(gs[j] + 2 * i),
                                                     (lds_void_ptr)&sh.sring[slot][0], 16, 0, 0);
                }
                ++T;
            }
        }
        wk.u += cnt;
        ring_walk_settle<U>(wk, tab);
    }
    // what is still in flight
    __builtin_amdgcn_s_waitcnt(ring_vmcnt_imm(0));
    ring_write_word(landed_addr, T);
}

// ---- the consumer waves -----------------------------------------------------
// What a consumer needs of a unit (wave-uniform).
struct RingUnit {
    int phase, unit, G, C4, precision;
    const char *xin;
};

__device__ __forceinline__ RingUnit ring_unit(CGroup *tab, int p, int u) {
    RingUnit d;
    CGroup &P = tab[p];
    d.phase = p;
    d.unit = u - P.unit_begin;
    d.G = P.G;
    d.C4 = d.G >> 2;
    d.precision = P.precision;
    d.xin = P.xa;
    return d;
}

// Request the activations of column c from a phase's operand image: per token
// tile the lane's 16 bytes of each KiB piece (two for int8 codes, four for
// bf16), 64 lanes x 16 contiguous bytes per load.  lane_off is the lane's byte
// offset in a piece (ring_lane_offset).
// Lane (n, kb) = (lane % 16, lane / 16) holds token n of a tile.  With fewer
// than 16 tokens the lanes of the missing ones read the slot of token
// n mod 2^ceil(log2 M) instead (an MFMA keeps tokens apart and their results
// are never stored), so that a load touches M / 16 of a piece only.
__device__ __forceinline__ int ring_lane_offset(int lane, int M) {
    int mask = 15;
    if (M <= 8) mask = 7;
    if (M <= 4) mask = 3;
    if (M <= 2) mask = 1;
    return ((lane >> 4) * 16 + (lane & 15 & mask)) * 16;
}

template <int MT>
__device__ __forceinline__ void ring_request_a(const char *xin, int C4, int precision, int c,
                                               int lane_off, uint4v (&raw)[MT][4]) {
    const int pieces = precision == NVQ_W4A8 ? 2 : 4;
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
        const char *p = xin + ((size_t)(mt * C4 + c) * pieces) * 1024 + lane_off;
        raw[mt][0] = *as_global<uint4v>(p);
        raw[mt][1] = *as_global<uint4v>(p + 1024);
        if (pieces == 4) {
            raw[mt][2] = *as_global<uint4v>(p + 2048);
            raw[mt][3] = *as_global<uint4v>(p + 3072);
        }
    }
}

// The columns of a bundle of `cnt` units that belong to this wave.  `raw` holds
// the activations of the first of them on entry and of the first column of the
// next bundle on exit.
template <int PREC, int MT, int U>
__device__ __forceinline__ void ring_bundle_columns(const RingUnit &d, int cnt, const RingUnit &nxt,
                                                    bool has_next, uint32_t &k,
                                                    uint32_t &landed, int M,
                                                    RingShared<MT> &sh, int w, int lane,
                                                    int lane_off, bool &dead,
                                                    uint4v (&raw)[MT][4],
                                                    float (&f)[U][kRingR][MT][4]) {
    typedef Act<PREC> A;
    constexpr int W = kRingWaves, S = kRingSteps, R = kRingR;
    const int n = lane & 15, kb = lane >> 4;
    const uint32_t abort_addr = ring_lds_addr(&sh.abort);
    const uint32_t landed_addr = ring_lds_addr(&sh.landed);
    const uint32_t consumed_addr = ring_lds_addr(&sh.consumed[w]);

    for (int c = w; c < d.C4; c += W) {
        // operands of this column, then the request for the following one
        typename A::operand act[MT][4];
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) A::operands(raw[mt], act[mt]);
        // one request site for "the next column of this bundle" and "the first
        // column of the next bundle": loads issued on two paths into the same
        // registers would be waited for where the paths join
        {
            const bool more = c + W < d.C4;
            const char *xin = more ? d.xin : nxt.xin;
            const int c4 = more ? d.C4 : nxt.C4, prec = more ? d.precision : nxt.precision;
            const int cn = more ? c + W : w;
            if (more || has_next) ring_request_a<MT>(xin, c4, prec, cn, lane_off, raw);
        }
#pragma unroll
        for (int j = 0; j < U; ++j) {
            if (j >= cnt) continue;
            // the loader is usually ahead: ask again only past what was seen
            if ((int32_t)(landed - (k + 1)) < 0)
                landed = ring_wait(landed_addr, k + 1, abort_addr, dead);
            const int slot = (int)(k % S);
            // Dword kb of each of the column's four 16-byte groups of row n: what the MFMA's
            // weight operand of group i wants in lane (n, kb), read as four words (one 16-byte
            // read per lane would bring group kb's four dwords instead, and four cross-lane
            // swaps would have to transpose them: the vector ALU is what bounds this kernel,
            // the local memory is not).
            uint32_t q[R][4];
            uint2 sc[R];
#pragma unroll
            for (int r = 0; r < R; ++r) {
#pragma unroll
                for (int i = 0; i < 4; ++i)
                    q[r][i] = reinterpret_cast<const uint32_t *>(
                        &sh.ring[slot][r][w >> 1][n >> 3][ring_lane_of(n, 4 * (w & 1) + i)])[kb];
                // the wave's column is the first or second half of 16-byte piece w / 2
                sc[r] = reinterpret_cast<const uint2 *>(
                    &sh.sring[slot][(r * 16 + n) * 2 + (w >> 1)])[w & 1];
            }
            // the slot is free once these reads have been carried out; LDS serves
            // a wave's requests in order, so the write below comes after them
            asm volatile("" ::: "memory");
            ++k;
            if (lane == 0) ring_write_word(consumed_addr, k);

            float sw[R][4];
#pragma unroll
            for (int r = 0; r < R; ++r) {
                sw[r][0] = half_bits_to_float((uint16_t)(sc[r].x & 0xffffu));
                sw[r][1] = half_bits_to_float((uint16_t)(sc[r].x >> 16));
                sw[r][2] = half_bits_to_float((uint16_t)(sc[r].y & 0xffffu));
                sw[r][3] = half_bits_to_float((uint16_t)(sc[r].y >> 16));
            }
#pragma unroll
            for (int i = 0; i < 4; ++i) {
#pragma unroll
                for (int mt = 0; mt < MT; ++mt) {
                    // the correction term, recomputed per unit: an MFMA is cheaper
                    // than the registers that would keep it
                    const typename A::offset_t off = A::offset(act[mt][i]);
#pragma unroll
                    for (int r = 0; r < R; ++r) {
                        int4v acc;
                        const float4v p = A::product(act[mt][i], A::weights(q[r][i]), off, acc);
                        f[j][r][mt][0] = fmaf(sw[r][i], p.x, f[j][r][mt][0]);
                        f[j][r][mt][1] = fmaf(sw[r][i], p.y, f[j][r][mt][1]);
                        f[j][r][mt][2] = fmaf(sw[r][i], p.z, f[j][r][mt][2]);
                        f[j][r][mt][3] = fmaf(sw[r][i], p.w, f[j][r][mt][3]);
                    }
                }
            }
        }
    }
}

template <int MT, int U>
__device__ __forceinline__ void ring_consumer(CGroup *tab, RingWalk wk, int M,
                                              RingShared<MT> &sh, int w, int lane, bool &dead) {
    constexpr int W = kRingWaves, R = kRingR;
    constexpr int kTile = R * MT * 4;
    const int n = lane & 15, kb = lane >> 4;
    const uint32_t abort_addr = ring_lds_addr(&sh.abort);
    const uint32_t done_addr = ring_lds_addr(&sh.done);
    if (wk.u >= wk.u_end) return;

    uint32_t k = 0;       // steps this wave has consumed
    uint32_t landed = 0;  // steps known to have arrived
    uint32_t units_done = 0;
    RingUnit cur = ring_unit(tab, wk.p, wk.u);
    uint4v raw[MT][4];
    const int lane_off = ring_lane_offset(lane, M);
    ring_request_a<MT>(cur.xin, cur.C4, cur.precision, w, lane_off, raw);
    float xs[MT][4];  // per-token activation scale of the lane's result registers (W4A8)
    bool fresh = true;

    while (wk.u < wk.u_end) {
        CGroup &P = tab[cur.phase];
        const int cnt = bundle_units<U>(wk.u, wk.u_end, P.unit_begin + P.unit_count);
        RingWalk nw = wk;
        nw.u += cnt;
        ring_walk_settle<U>(nw, tab);
        const bool has_next = nw.u < nw.u_end;
        RingUnit nxt = cur;
        if (has_next) {
            if (nw.p == cur.phase)
                nxt.unit = nw.u - P.unit_begin;
            else
                nxt = ring_unit(tab, nw.p, nw.u);
        }
        if (fresh) {
#pragma unroll
            for (int mt = 0; mt < MT; ++mt)
#pragma unroll
                for (int jj = 0; jj < 4; ++jj) {
                    const int m = mt * 16 + kb * 4 + jj;
                    xs[mt][jj] = (cur.precision == NVQ_W4A8 && m < M)
                                     ? as_global<float>(P.xscale)[m]
                                     : 1.0f;
                }
        }

        float f[U][R][MT][4];
#pragma unroll
        for (int j = 0; j < U; ++j)
#pragma unroll
            for (int r = 0; r < R; ++r)
#pragma unroll
                for (int mt = 0; mt < MT; ++mt)
#pragma unroll
                    for (int jj = 0; jj < 4; ++jj) f[j][r][mt][jj] = 0.0f;

        if (cur.precision == NVQ_W4A8)
            ring_bundle_columns<NVQ_W4A8, MT, U>(cur, cnt, nxt, has_next, k, landed, M, sh, w, lane, lane_off, dead,
                                                 raw, f);
        else
            ring_bundle_columns<NVQ_W4A16, MT, U>(cur, cnt, nxt, has_next, k, landed, M, sh, w, lane, lane_off, dead,
                                                  raw, f);

        // unit by unit, add the K slices of the waves in wave order
#pragma unroll
        for (int j = 0; j < U; ++j) {
            if (j >= cnt) continue;
            const int par = (int)(units_done & 1u);
#pragma unroll
            for (int r = 0; r < R; ++r)
#pragma unroll
                for (int mt = 0; mt < MT; ++mt)
#pragma unroll
                    for (int jj = 0; jj < 4; ++jj)
                        sh.red[par][w][(r * MT + mt) * 4 + jj][lane] = f[j][r][mt][jj] * xs[mt][jj];
            asm volatile("" ::: "memory");
            if (lane == 0) ring_add_word(done_addr, 1u);
            ++units_done;
            ring_wait(done_addr, units_done * (uint32_t)W, abort_addr, dead);
            if (!dead) {
#pragma unroll
                for (int pass = 0; pass < (kTile + W - 1) / W; ++pass) {
                    const int reg = pass * W + w;
                    if (reg < kTile) {
                        float sum = 0.0f;
#pragma unroll
                        for (int i = 0; i < W; ++i) sum += sh.red[par][i][reg][lane];
                        const int r = reg / (MT * 4), mt = (reg >> 2) % MT, jj = reg & 3;
                        const int m = mt * 16 + kb * 4 + jj;
                        const RowRef o =
                            locate_row(P.segs, ((cur.unit + j) * R + r) * 16 + n, cur.G);
                        if (o.valid && m < M)
                            store_global(o.y, o.y_dtype, (int64_t)m * o.N + o.n, sum);
                    }
                }
            }
        }
        fresh = nxt.phase != cur.phase;
        cur = nxt;
        wk = nw;
    }
}

// TEAMS teams share a workgroup (and nothing else): one workgroup per compute
// unit holds all the LDS, which several smaller workgroups could not divide
// among themselves as well.  part_tab holds nparts + 1 unit indices, the cuts
// of the batch into parts, then nparts + 1 phase indices, the phase of the unit
// at each cut; workgroup g serves part g mod nparts (see RingWalk).
template <int MT, int TEAMS, int U>
__global__ __launch_bounds__(TEAMS *kTeamThreads) void gemv_mfma_ring_kernel(
    const GroupPhase *__restrict__ tab_, const uint32_t *__restrict__ part_tab_, int nparts, int M,
    uint32_t *__restrict__ status) {
    __shared__ RingShared<MT> shared[TEAMS];
    CGroup *tab = (CGroup *)tab_;
    CWord *part_tab = (CWord *)part_tab_;
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    const int t = wave / (kRingWaves + 1), w = wave - t * (kRingWaves + 1);
    RingShared<MT> &sh = shared[t];
    if (w == 0 && lane < kRingWaves) sh.consumed[lane] = 0;
    if (w == 0 && lane == 0) {
        sh.landed = 0;
        sh.done = 0;
        sh.abort = 0;
    }
    __syncthreads();
    const int part = (int)blockIdx.x % nparts;
    // workgroups of this part: those g < grid with g mod nparts == part
    const int part_wgs = ((int)gridDim.x - 1 - part) / nparts + 1;
    const RingWalk wk = ring_walk_begin<U>(tab, (int)part_tab[part], (int)part_tab[part + 1],
                                           (int)part_tab[nparts + 1 + part],
                                           ((int)blockIdx.x / nparts) * TEAMS + t, part_wgs * TEAMS);
    bool dead = false;
    if (w == kRingWaves) __builtin_amdgcn_s_setprio(3);  // the loader's few instructions go first
    if (w == kRingWaves)
        ring_loader<MT, U>(tab, wk, sh, lane, dead);
    else
        ring_consumer<MT, U>(tab, wk, M, sh, w, lane, dead);
    if (dead && lane == 0) __hip_atomic_store(status, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

}  // namespace

// A step is four columns (512 inputs), and the scale load moves 16 bytes per lane.
bool gemv_mfma_ring_supported(const GemvSegs &S, int K) {
    if (K % (128 * kRingWaves) != 0) return false;
    for (int i = 0; i < S.nseg; ++i)
        if (!aligned(S.sc[i], 16)) return false;
    return true;
}

int ring_teams_per_workgroup(int M) { return M > 16 ? 2 : 3; }
int ring_bundle_units(int M) { return M > 16 ? 1 : kRingBundle; }

// One workgroup per compute unit at most: three teams (52 KiB of LDS each) up
// to 16 tokens, two (68 KiB each) beyond; fewer workgroups if the batch has
// fewer groups of units than that many teams.
int ring_grid(int M, int nunits) {
    const int per_wg = ring_teams_per_workgroup(M) * ring_bundle_units(M);
    const int want = (nunits + per_wg - 1) / per_wg, cap = device_cu_count();
    return want < cap ? want : cap;
}
// Parts the batch is cut into: one per XCD (eight; workgroups go to the XCDs in
// turn), fewer for a grid of fewer workgroups.
int ring_parts(int grid) { return grid < 8 ? grid : 8; }

// part_tab: nparts + 1 unit indices (the cuts of the batch), then nparts + 1
// phase indices (the phase of each cut's unit), in device memory.
int launch_gemv_mfma_ring(const GroupPhase *tab, const uint32_t *part_tab, int nparts, int grid,
                          int M, uint32_t *status, hipStream_t st) {
    if (nparts <= 0 || grid <= 0) return NVQ_OK;
    const int tpw = ring_teams_per_workgroup(M);
    const dim3 g(grid), block(tpw * kTeamThreads);
    if (M > 16)
        hipLaunchKernelGGL((gemv_mfma_ring_kernel<2, 2, 1>), g, block, 0, st, tab, part_tab, nparts,
                           M, status);
    else
        hipLaunchKernelGGL((gemv_mfma_ring_kernel<1, 3, kRingBundle>), g, block, 0, st, tab,
                           part_tab, nparts, M, status);
    NVQ_HIP_TRY(hipGetLastError());
    return NVQ_OK;
}

}  // namespace nvq
