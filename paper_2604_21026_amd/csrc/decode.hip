// nvq_decode_linears / nvq_plan_*: walk the linear layers of one decode step
// under a per-layer precision map.  Paper: routing rule of the
// precision-dispatch section (W4A16 if the layer's normalised score reaches
// the threshold, else W4A8); activation codes are computed once per input and
// reused by every projection that reads it; the step is issued without
// per-kernel host round trips (paragraph on graph capture for decode).
//
// The host groups consecutive entries that read the same input with the same
// precision into a phase (q/k/v, gate/up; at most four matrices per phase).
// Batch 1 runs the whole list in one launch of the persistent streaming
// kernel (decode_stream.hip).  Other batch sizes, and shapes the streaming
// kernel does not take, run on the caller's stream as launches per phase (one
// quantisation launch per W4A8 phase and one fused GEMV launch), or, for 2..32
// tokens of shapes the matrix-core kernel takes, as two launches per batch of
// mutually independent phases (one grid quantises, one multiplies).
#include <algorithm>
#include <mutex>
#include <new>
#include <vector>

#include "decode_stream.h"
#include "transform.h"

namespace nvq {

namespace {

size_t round_up(size_t v, size_t a) { return (v + a - 1) / a * a; }


// Workspace layout (offsets from a 256-byte aligned base).
struct Workspace {
    uint16_t *xt;       // [M][maxK]           transformed input (per-phase launches)
    int8_t *xq;         // [M][maxK]           activation codes (per-phase launches)
    float *xscale;      // [M][maxK/32]
    int32_t *xgsum;     // [M][maxK/32]
    StreamPhase *tab;   // [n]                 phase table of the streaming kernel
    uint32_t *flags;    // [kStreamMaxWg]      one word per workgroup
    uint32_t *status;   // [64]                word 0: a wait timed out
    uint32_t *imgflags; // [n]                 one word per phase (follows the status words)
    void *dummy;        // 1 KiB               target of the ring's filler loads
    char *images;       // prepared activation images of the streaming kernel
    uint8_t *skips;     // skip table of the streaming kernel (M = 1): a row per streaming wave
    GroupPhase *gtab;   // [n]                 phase table of the grouped small-batch launches
    uint16_t *gjobs;    // [n]                 W4A8 phases, batch after batch
    uint16_t *gunits;   // [group_units]       phase of every 16-row tile, batch after batch
    uint32_t *gteams;   // [n][2][kRingMaxParts + 1]  per batch: the parts of the ring kernel's XCDs
    uint16_t *gimgs;    // [group_images]      phase of every operand image unit, batch after batch
    char *gquant;       // per-phase activation codes, scales and code sums
    uint32_t *mail;     // mailboxes of the streaming kernel (M = 1): tagged copies of outputs
    size_t bytes;
};

// Sizes that depend on the layer list (upper bounds: every entry its own phase).
struct ListSizes {
    int maxK;
    size_t image_bytes;  // activation images of the streaming kernel (M = 1)
    size_t group_units;  // 16-row tiles of all entries (M > 1)
    size_t group_quant;  // codes + scales + code sums of all W4A8 entries (M > 1)
    size_t group_images; // operand image units of all entries (M > 1)
    bool transforms;     // some entry has an input transform
    size_t mail_words;   // mailboxes for every output and residual sum (M = 1)
};

// Activations of a phase in the order the persistent small-batch kernel loads
// them: token tiles of 16, whole KiB per (tile, 128-input column, piece).
size_t operand_image_bytes(int M, int K, int precision) {
    return (size_t)((M + 15) / 16) * 16 * K * (precision == NVQ_W4A8 ? 1 : 2);
}

size_t quant_bytes(int M, int K) {
    return round_up((size_t)M * K, 256) + round_up((size_t)M * 4, 256) +
           round_up((size_t)M * (K / 32) * 4, 256);
}

static_assert(kStreamMaxWg * 4 == NVQ_WORKSPACE_STATUS_OFFSET, "the header states the offset");

Workspace carve(void *base, int M, int n, const ListSizes &ls) {
    const int maxK = ls.maxK;
    const size_t image_bytes = ls.image_bytes;
    Workspace w;
    char *b = reinterpret_cast<char *>(base);
    const size_t G = (size_t)maxK / 32;
    size_t off = 0;
    auto take = [&](size_t bytes) {
        char *p = b + off;
        off += round_up(bytes, 256);
        return p;
    };
    // the flag block comes first: the status word has a fixed place in every workspace
    w.flags = reinterpret_cast<uint32_t *>(take(kStreamMaxWg * 4));
    w.status = reinterpret_cast<uint32_t *>(take(256));
    take((size_t)(kFlagReplicas - 1) * kStreamMaxWg * 4);  // the other copies of the flags
    w.imgflags = reinterpret_cast<uint32_t *>(take((size_t)(n > 0 ? n : 1) * 4));
    w.xt = reinterpret_cast<uint16_t *>(take(ls.transforms ? (size_t)M * maxK * 2 : 0));
    w.xq = reinterpret_cast<int8_t *>(take((size_t)M * maxK));
    w.xscale = reinterpret_cast<float *>(take((size_t)M * G * 4));
    w.xgsum = reinterpret_cast<int32_t *>(take((size_t)M * G * 4));
    w.tab = reinterpret_cast<StreamPhase *>(take((size_t)(n > 0 ? n : 1) * sizeof(StreamPhase)));
    w.dummy = take(1024);
    w.images = take(image_bytes);
    w.skips = reinterpret_cast<uint8_t *>(
        take(M == 1 ? (size_t)kStreamMaxWg * (kStreamWaves + 1) * (size_t)stream_skip_stride(n) : 0));
    const size_t nn = (size_t)(n > 0 ? n : 1);
    w.gtab = reinterpret_cast<GroupPhase *>(take(M > 1 ? nn * sizeof(GroupPhase) : 0));
    w.gjobs = reinterpret_cast<uint16_t *>(take(M > 1 ? nn * 2 : 0));
    w.gunits = reinterpret_cast<uint16_t *>(take(M > 1 ? ls.group_units * 2 : 0));
    w.gteams = reinterpret_cast<uint32_t *>(take(M > 1 ? nn * 2 * (kRingMaxParts + 1) * 4 : 0));
    w.gimgs = reinterpret_cast<uint16_t *>(take(M > 1 ? ls.group_images * 2 : 0));
    w.gquant = take(M > 1 ? ls.group_quant : 0);
    w.mail = reinterpret_cast<uint32_t *>(
        take(M == 1 ? stream_mail_stride(ls.mail_words) * kMailReplicas * 4 : 0));
    w.bytes = off;
    return w;
}

int check_layers(const nvq_linear *L, int n, int M, int act_group, ListSizes *sizes) {
    if (!L || n < 0) return NVQ_ERR_INVALID_ARG;
    if (act_group != 0 && act_group != 32) return NVQ_ERR_INVALID_ARG;
    if (M <= 0 || M > NVQ_MAX_M) return NVQ_ERR_SHAPE;
    int mk = 32;
    size_t ib = 0, gu = 0, gq = 0, gi = 0, mw = 0;
    bool tr = false;
    for (int i = 0; i < n; ++i) {
        const nvq_linear &e = L[i];
        if (!e.qweight || !e.scales || !e.x_bf16 || !e.y) return NVQ_ERR_INVALID_ARG;
        if (e.precision != NVQ_W4A8 && e.precision != NVQ_W4A16) return NVQ_ERR_INVALID_ARG;
        if (e.in_op == NVQ_IN_RMSNORM) {
            if (!e.gamma_bf16 || !(e.eps >= 0.0f)) return NVQ_ERR_INVALID_ARG;
        } else if (e.in_op == NVQ_IN_SILU_MUL) {
            if (!e.x2_bf16) return NVQ_ERR_INVALID_ARG;
        } else if (e.in_op != NVQ_IN_PLAIN) {
            return NVQ_ERR_INVALID_ARG;
        }
        if (e.in_op != NVQ_IN_PLAIN &&
            (!aligned(e.x2_bf16, 16) || !aligned(e.gamma_bf16, 16) || !aligned(e.h_out_bf16, 16)))
            return NVQ_ERR_ALIGN;
        tr = tr || e.in_op != NVQ_IN_PLAIN;
        if (e.y_dtype != NVQ_F32 && e.y_dtype != NVQ_BF16) return NVQ_ERR_INVALID_ARG;
        if (e.N <= 0 || e.K <= 0 || (e.K % 32) != 0 || e.K > NVQ_MAX_K) return NVQ_ERR_SHAPE;
        if (!aligned(e.qweight, 16) || !aligned(e.scales, 2) || !aligned(e.x_bf16, 16) ||
            !aligned(e.y, e.y_dtype == NVQ_F32 ? 4 : 2))
            return NVQ_ERR_ALIGN;
        if (e.K > mk) mk = e.K;
        // upper bound: every entry its own phase with a prepared image
        if (e.K <= kStreamMaxK) ib += (size_t)stream_image_bytes(e.K, e.precision, act_group);
        gu += (size_t)(e.N + 15) / 16 + 1;
        // codes, scales and code sums (W4A8), or the operand image of the
        // persistent small-batch kernel (either precision)
        const size_t image = operand_image_bytes(M, e.K, e.precision) + round_up((size_t)M * 4, 256);
        const size_t plain = e.precision == NVQ_W4A8 ? quant_bytes(M, e.K) : 0;
        gq += image > plain ? image : plain;
        gi += (size_t)image_units(M, e.K);
        // upper bound: every bf16 output and every residual sum has a mailbox
        if (e.y_dtype == NVQ_BF16) mw += stream_mail_words(e.N);
        if (e.in_op == NVQ_IN_RMSNORM && e.x2_bf16 && e.h_out_bf16) mw += stream_mail_words(e.K);
    }
    sizes->maxK = mk;
    sizes->image_bytes = ib;
    sizes->group_units = gu;
    sizes->group_quant = gq;
    sizes->group_images = gi;
    sizes->transforms = tr;
    sizes->mail_words = mw;
    return NVQ_OK;
}

// Consecutive entries with the same input, K and precision, at most kMaxSeg.
struct Phase {
    int first, count;
};

// The input transform of an entry (none: every field compares equal to none).
bool same_transform(const nvq_linear &a, const nvq_linear &b) {
    if (a.in_op != b.in_op) return false;
    if (a.in_op == NVQ_IN_PLAIN) return true;
    return a.x2_bf16 == b.x2_bf16 && a.gamma_bf16 == b.gamma_bf16 && a.eps == b.eps &&
           a.h_out_bf16 == b.h_out_bf16;
}

std::vector<Phase> group_phases(const nvq_linear *L, int n) {
    std::vector<Phase> out;
    int i = 0;
    while (i < n) {
        int j = i + 1;
        while (j < n && j - i < kMaxSeg && L[j].x_bf16 == L[i].x_bf16 && L[j].K == L[i].K &&
               L[j].precision == L[i].precision && same_transform(L[i], L[j]))
            ++j;
        out.push_back({i, j - i});
        i = j;
    }
    return out;
}

// True if phase b reads the same input as phase a with the same precision
// (a phase split only because it had more than kMaxSeg matrices).
bool same_input(const nvq_linear *L, const Phase &a, const Phase &b) {
    return L[a.first].x_bf16 == L[b.first].x_bf16 && L[a.first].K == L[b.first].K &&
           L[a.first].precision == L[b.first].precision &&
           same_transform(L[a.first], L[b.first]);
}

GemvSegs make_segs(const nvq_linear *L, const Phase &ph) {
    GemvSegs S = {};
    int rows = 0;
    for (int k = 0; k < ph.count; ++k) {
        const nvq_linear &e = L[ph.first + k];
        S.qw[k] = reinterpret_cast<const uint4 *>(e.qweight);
        S.sc[k] = e.scales;
        S.y[k] = e.y;
        S.dbg[k] = nullptr;
        S.N[k] = e.N;
        rows += e.N;
        S.row_end[k] = rows;
        S.y_dtype[k] = e.y_dtype;
    }
    S.nseg = ph.count;
    S.total_rows = rows;
    return S;
}

// One launch (or two) per phase on the caller's stream.
int walk_per_phase(const nvq_linear *L, const std::vector<Phase> &phases, int M, int act_group,
                   const Workspace &ws, hipStream_t st) {
    for (size_t p = 0; p < phases.size(); ++p) {
        const Phase &ph = phases[p];
        const nvq_linear &e0 = L[ph.first];
        const bool w4a8 = e0.precision == NVQ_W4A8;
        const bool fresh = !(p > 0 && same_input(L, phases[p - 1], ph));
        const uint16_t *x = e0.x_bf16;
        if (e0.in_op != NVQ_IN_PLAIN) {
            // the transformed input of the previous phase is still in ws.xt if it was the same
            if (fresh) {
                const int t = e0.in_op == NVQ_IN_RMSNORM
                                  ? launch_rms_norm(e0.x_bf16, e0.x2_bf16, e0.gamma_bf16, e0.eps, M,
                                                    e0.K, ws.xt, e0.h_out_bf16, st)
                                  : launch_silu_mul(e0.x_bf16, e0.x2_bf16, M, e0.K, ws.xt, st);
                if (t != NVQ_OK) return t;
            }
            x = ws.xt;
        }
        if (w4a8 && fresh) {
            const int q = launch_quant_act(x, M, e0.K, act_group, ws.xq, ws.xscale, ws.xgsum, st);
            if (q != NVQ_OK) return q;
        }
        const GemvSegs S = make_segs(L, ph);
        const int g = w4a8 ? launch_gemv_w4a8(S, e0.K, ws.xq, ws.xscale, ws.xgsum, act_group, M, st)
                           : launch_gemv_w4a16(S, e0.K, x, M, st);
        if (g != NVQ_OK) return g;
    }
    return NVQ_OK;
}

struct Range {
    uintptr_t lo, hi;
};
bool overlap(const Range &a, const Range &b) { return a.lo < b.hi && b.lo < a.hi; }

// What a phase reads (input, second operand and norm weights) and what it
// writes (every layer's output, the residual sum).
void phase_ranges(const nvq_linear *L, const Phase &ph, int M, std::vector<Range> *in,
                  std::vector<Range> *out) {
    const nvq_linear &e0 = L[ph.first];
    const size_t xbytes = (size_t)M * e0.K * 2;
    in->push_back({(uintptr_t)e0.x_bf16, (uintptr_t)e0.x_bf16 + xbytes});
    if (e0.in_op != NVQ_IN_PLAIN) {
        if (e0.x2_bf16) in->push_back({(uintptr_t)e0.x2_bf16, (uintptr_t)e0.x2_bf16 + xbytes});
        if (e0.gamma_bf16)
            in->push_back({(uintptr_t)e0.gamma_bf16, (uintptr_t)e0.gamma_bf16 + (size_t)e0.K * 2});
        if (e0.in_op == NVQ_IN_RMSNORM && e0.x2_bf16 && e0.h_out_bf16)
            out->push_back({(uintptr_t)e0.h_out_bf16, (uintptr_t)e0.h_out_bf16 + xbytes});
    }
    for (int k = 0; k < ph.count; ++k) {
        const nvq_linear &e = L[ph.first + k];
        const size_t bytes = (size_t)M * e.N * (e.y_dtype == NVQ_F32 ? 4 : 2);
        out->push_back({(uintptr_t)e.y, (uintptr_t)e.y + bytes});
    }
}

// The layers of a phase run concurrently and read their input while outputs
// are already being stored: no output of a phase may overlap anything the phase
// reads, or another of its outputs.
int check_phase_hazards(const nvq_linear *L, const std::vector<Phase> &phases, int M) {
    for (const Phase &ph : phases) {
        std::vector<Range> in, out;
        phase_ranges(L, ph, M, &in, &out);
        for (size_t a = 0; a < out.size(); ++a) {
            for (const Range &r : in)
                if (overlap(out[a], r)) return NVQ_ERR_INVALID_ARG;
            for (size_t b = a + 1; b < out.size(); ++b)
                if (overlap(out[a], out[b])) return NVQ_ERR_INVALID_ARG;
        }
    }
    return NVQ_OK;
}

// The order the persistent kernel takes the phases in (batch 1).  A phase that
// reads what its predecessor writes starts with everybody waiting for the
// predecessor's slowest wave and for the results to travel.  Where the phase
// after it conflicts with neither of the two, that one goes first: the waves
// that are done early then have work, and the wait has passed when they get
// there.  (A decode step whose attention runs elsewhere has one such phase per
// block, the o projection.)  Phases that do not conflict may run in any order,
// so every result is what the list's own order gives.
bool phases_conflict(const nvq_linear *L, const Phase &a, const Phase &b, int M) {
    std::vector<Range> ain, aout, bin, bout;
    phase_ranges(L, a, M, &ain, &aout);
    phase_ranges(L, b, M, &bin, &bout);
    for (const Range &y : aout) {
        for (const Range &x : bin)
            if (overlap(y, x)) return true;
        for (const Range &z : bout)
            if (overlap(y, z)) return true;
    }
    for (const Range &y : bout)
        for (const Range &x : ain)
            if (overlap(y, x)) return true;
    return false;
}

void schedule_phases(const nvq_linear *L, std::vector<Phase> *phases, int M, bool ordered) {
    if (M != 1 || ordered) return;
    std::vector<Phase> &ph = *phases;
    for (size_t p = 1; p + 1 < ph.size(); ++p) {
        if (phases_conflict(L, ph[p - 1], ph[p], M) && !phases_conflict(L, ph[p], ph[p + 1], M) &&
            !phases_conflict(L, ph[p - 1], ph[p + 1], M)) {
            std::swap(ph[p], ph[p + 1]);
            ++p;  // the phase that waits stays where it is now
        }
    }
}

// Mail links (batch 1, persistent kernel).  An input operand (x, or x2 of a
// transform) of phase p is linked if the latest earlier phase that writes any
// of its bytes writes exactly that vector as one bf16 output (y of one of its
// layers with N = K of p, or its residual sum): then p takes the operand from
// the mailbox that phase posts it in, never from the caller's buffer.
struct OperandLink {
    int phase;  // producing phase, or -1: not linked
    int seg;    // its layer (segment of the phase), or kMaxSeg: its residual sum
};
struct PhaseLinks {
    OperandLink x, x2;
};

OperandLink find_link(const nvq_linear *L, const std::vector<Phase> &phases, size_t p,
                      const uint16_t *operand) {
    const OperandLink none = {-1, 0};
    if (!operand) return none;
    const nvq_linear &e0 = L[phases[p].first];
    const Range r = {(uintptr_t)operand, (uintptr_t)operand + (size_t)e0.K * 2};
    for (size_t q = p; q-- > 0;) {
        const Phase &pq = phases[q];
        const nvq_linear &q0 = L[pq.first];
        OperandLink hit = none;
        int overlaps = 0;
        for (int k = 0; k < pq.count; ++k) {
            const nvq_linear &e = L[pq.first + k];
            const Range y = {(uintptr_t)e.y,
                             (uintptr_t)e.y + (size_t)e.N * (e.y_dtype == NVQ_F32 ? 4 : 2)};
            if (!overlap(y, r)) continue;
            ++overlaps;
            if (y.lo == r.lo && y.hi == r.hi && e.y_dtype == NVQ_BF16) hit = {(int)q, k};
        }
        if (q0.in_op == NVQ_IN_RMSNORM && q0.x2_bf16 && q0.h_out_bf16) {
            const Range h = {(uintptr_t)q0.h_out_bf16, (uintptr_t)q0.h_out_bf16 + (size_t)q0.K * 2};
            if (overlap(h, r)) {
                ++overlaps;
                if (h.lo == r.lo && h.hi == r.hi) hit = {(int)q, kMaxSeg};
            }
        }
        if (overlaps == 0) continue;          // an older phase may have written it
        return overlaps == 1 ? hit : none;     // the latest writer decides
    }
    return none;
}

std::vector<PhaseLinks> find_links(const nvq_linear *L, const std::vector<Phase> &phases, int M,
                                   bool ordered) {
    std::vector<PhaseLinks> links(phases.size(), PhaseLinks{{-1, 0}, {-1, 0}});
    if (M != 1 || ordered) return links;
    for (size_t p = 1; p < phases.size(); ++p) {
        const nvq_linear &e0 = L[phases[p].first];
        links[p].x = find_link(L, phases, p, e0.x_bf16);
        const bool second = e0.in_op == NVQ_IN_SILU_MUL || (e0.in_op == NVQ_IN_RMSNORM && e0.x2_bf16);
        if (second) links[p].x2 = find_link(L, phases, p, e0.x2_bf16);
    }
    return links;
}

// Per phase the latest earlier phase it conflicts with (it reads what that
// phase wrote, or writes what that phase read or wrote), or -1; with `ordered`
// every phase depends on its predecessor.  Operands that arrive by mail
// (`links`) are not read from memory and take no part in this.
std::vector<int> phase_deps(const nvq_linear *L, const std::vector<Phase> &phases, int M,
                            bool ordered, const std::vector<PhaseLinks> *links = nullptr) {
    const size_t P = phases.size();
    std::vector<int> deps(P, -1);
    std::vector<std::vector<Range>> xin(P), yout(P);  // what a phase reads and writes
    for (size_t p = 0; p < P; ++p) {
        phase_ranges(L, phases[p], M, &xin[p], &yout[p]);
        if (!links) continue;
        const nvq_linear &e0 = L[phases[p].first];
        auto drop = [&](const uint16_t *operand) {
            for (size_t i = 0; i < xin[p].size(); ++i)
                if (xin[p][i].lo == (uintptr_t)operand) {
                    xin[p].erase(xin[p].begin() + (long)i);
                    return;
                }
        };
        if ((*links)[p].x.phase >= 0) drop(e0.x_bf16);
        if ((*links)[p].x2.phase >= 0) drop(e0.x2_bf16);
    }
    for (size_t p = 1; p < P; ++p) {
        int dep = ordered ? (int)p - 1 : -1;
        for (size_t q = 0; q < p && !ordered; ++q) {
            bool hit = false;
            for (const Range &yq : yout[q]) {
                for (const Range &xp : xin[p]) hit = hit || overlap(xp, yq);  // read after write
                for (const Range &yp : yout[p]) hit = hit || overlap(yp, yq);  // write after write
            }
            for (const Range &yp : yout[p])
                for (const Range &xq : xin[q]) hit = hit || overlap(yp, xq);  // write after read
            if (hit) dep = (int)q;
        }
        deps[p] = dep;
    }
    return deps;
}

// Small batches on the matrix cores, grouped: phases that do not depend on
// each other form a batch, and a batch is two launches: one grid quantises the
// inputs of all its W4A8 phases, one grid holds the row tiles of all its
// phases.  Empty if some phase does not qualify for the matrix-core kernel.
struct GroupBatch {
    int job_first, njobs;    // range in the job list
    int unit_first, nunits;  // range in the unit list
    int img_first, nimg;     // range in the image unit list
    int part_first, nparts;  // the batch's table in the part list (2 * (nparts + 1) words)
    int grid;                // workgroups of the persistent kernel
};
struct GroupPlan {
    bool ring;  // the persistent kernel serves the list: every phase has a job and an operand image
    std::vector<GroupPhase> tab;
    std::vector<uint16_t> jobs, units, imgs;
    std::vector<uint32_t> parts;  // per batch: nparts + 1 unit cuts, then the phases at the cuts
    std::vector<GroupBatch> batches;
};

// Cut the units of a batch into contiguous parts of (nearly) equal weight
// bytes, one per XCD of the persistent kernel's grid; a unit of phase p weighs
// G_p.
void cut_batch(GroupPlan &gp, GroupBatch &b, int M) {
    b.grid = ring_grid(M, b.nunits);
    const int nparts = ring_parts(b.grid);
    b.part_first = (int)gp.parts.size();
    b.nparts = nparts;
    if (nparts <= 0) return;
    uint64_t total = 0;
    for (int u = 0; u < b.nunits; ++u) total += (uint64_t)gp.tab[gp.units[(size_t)b.unit_first + u]].G;
    std::vector<uint32_t> cut((size_t)nparts + 1), phase((size_t)nparts + 1);
    uint64_t before = 0;  // weight of the units before u
    int t = 0;
    for (int u = 0; u < b.nunits; ++u) {
        // part t starts at the first unit whose predecessors weigh t / nparts of the batch
        while (t < nparts && before * (uint64_t)nparts >= (uint64_t)t * total) {
            cut[(size_t)t] = (uint32_t)u;
            phase[(size_t)t] = gp.units[(size_t)b.unit_first + u];
            ++t;
        }
        before += (uint64_t)gp.tab[gp.units[(size_t)b.unit_first + u]].G;
    }
    for (; t <= nparts; ++t) {
        cut[(size_t)t] = (uint32_t)b.nunits;
        phase[(size_t)t] = gp.units[(size_t)b.unit_first + b.nunits - 1];
    }
    gp.parts.insert(gp.parts.end(), cut.begin(), cut.end());
    gp.parts.insert(gp.parts.end(), phase.begin(), phase.end());
}

GroupPlan group_plan(const nvq_linear *L, const std::vector<Phase> &phases, int M, int act_group,
                     bool ordered, const Workspace &ws) {
    GroupPlan gp;
    gp.ring = false;
    if (M < 2 || act_group != 0 || phases.size() > 65535) return gp;
    for (const Phase &ph : phases)
        if (L[ph.first].in_op != NVQ_IN_PLAIN ||
            !gemv_mfma_supported(make_segs(L, ph), L[ph.first].K, M))
            return gp;
    gp.ring = true;
    for (const Phase &ph : phases)
        gp.ring = gp.ring && gemv_mfma_ring_supported(make_segs(L, ph), L[ph.first].K);
    const std::vector<int> deps = phase_deps(L, phases, M, ordered);
    size_t qoff = 0;
    GroupBatch cur = {0, 0, 0, 0, 0, 0, 0, 0, 0};
    int batch_first = 0;
    for (size_t p = 0; p < phases.size(); ++p) {
        const nvq_linear &e0 = L[phases[p].first];
        if (deps[p] >= batch_first) {  // depends on a phase of the open batch: close it
            cut_batch(gp, cur, M);
            gp.batches.push_back(cur);
            cur = {(int)gp.jobs.size(), 0, (int)gp.units.size(), 0, (int)gp.imgs.size(), 0, 0, 0, 0};
            batch_first = (int)p;
        }
        GroupPhase g = {};
        g.segs = make_segs(L, phases[p]);
        g.x_bf16 = e0.x_bf16;
        g.G = e0.K / 32;
        g.precision = e0.precision;
        g.unit_begin = cur.nunits;
        if (gp.ring) {
            char *b = ws.gquant + qoff;
            g.xa = b;
            g.xscale = reinterpret_cast<float *>(b + operand_image_bytes(M, e0.K, e0.precision));
            qoff += operand_image_bytes(M, e0.K, e0.precision) + round_up((size_t)M * 4, 256);
            gp.jobs.push_back((uint16_t)p);
            ++cur.njobs;
            g.img_begin = cur.nimg;
            const int iu = image_units(M, e0.K);
            gp.imgs.insert(gp.imgs.end(), (size_t)iu, (uint16_t)p);
            cur.nimg += iu;
        } else if (e0.precision == NVQ_W4A8) {
            char *b = ws.gquant + qoff;
            g.xq = reinterpret_cast<int8_t *>(b);
            g.xscale = reinterpret_cast<float *>(b + round_up((size_t)M * e0.K, 256));
            g.xgsum = reinterpret_cast<int32_t *>(b + round_up((size_t)M * e0.K, 256) +
                                                  round_up((size_t)M * 4, 256));
            qoff += quant_bytes(M, e0.K);
            gp.jobs.push_back((uint16_t)p);
            ++cur.njobs;
        }
        const int rows_per_unit = 16 * group_row_tiles(M);
        const int units = (g.segs.total_rows + rows_per_unit - 1) / rows_per_unit;
        g.unit_count = units;
        gp.units.insert(gp.units.end(), (size_t)units, (uint16_t)p);
        cur.nunits += units;
        gp.tab.push_back(g);
    }
    cut_batch(gp, cur, M);
    gp.batches.push_back(cur);
    return gp;
}

// Start of the cyclic run of `len` entries of `load` with the smallest sum
// (the first such run).
int lightest_window(const std::vector<uint64_t> &load, int len) {
    const int n = (int)load.size();
    if (len <= 0 || len >= n) return 0;
    uint64_t sum = 0;
    for (int j = 0; j < len; ++j) sum += load[(size_t)j];
    uint64_t best = sum;
    int at = 0;
    for (int s = 1; s < n; ++s) {
        sum += load[(size_t)(s + len - 1) % n] - load[(size_t)s - 1];
        if (sum < best) {
            best = sum;
            at = s;
        }
    }
    return at;
}

// Phase table for the streaming kernel; empty if some phase does not qualify.
// Each phase records the latest earlier phase it conflicts with (it reads what
// that phase wrote, or writes what that phase read or wrote); with `ordered`
// every phase is made to depend on its predecessor.
// `mail`: start of the mailbox area in the workspace (words are handed out from
// it; *mail_words receives how many).
std::vector<StreamPhase> stream_table(const nvq_linear *L, const std::vector<Phase> &phases, int M,
                                      int act_group, int nwg, bool ordered, char *images,
                                      int *nimages, std::vector<uint8_t> *skips = nullptr,
                                      uint32_t *mail = nullptr, size_t *mail_words = nullptr) {
    std::vector<StreamPhase> tab;
    if (mail_words) *mail_words = 0;
    if (M != 1 || nwg <= 0 || nwg > kStreamMaxWg) return tab;
    const int waves = nwg * kStreamWaves;
    // bytes of extra rows dealt to each wave so far: the extra rows of a phase
    // go to the run of waves that has received the least
    std::vector<uint64_t> extra_bytes((size_t)waves, 0);
    const std::vector<PhaseLinks> links = find_links(L, phases, M, ordered);
    const std::vector<int> deps = phase_deps(L, phases, M, ordered, &links);
    // a phase someone waits for, through the flags or by mail; a phase that waits
    std::vector<char> published(phases.size(), 0), waits(phases.size(), 0);
    for (size_t p = 1; p < phases.size(); ++p) {
        if (deps[p] >= 0) published[(size_t)deps[p]] = 1;
        if (links[p].x.phase >= 0) published[(size_t)links[p].x.phase] = 1;
        if (links[p].x2.phase >= 0) published[(size_t)links[p].x2.phase] = 1;
        waits[p] = deps[p] >= 0 || links[p].x.phase >= 0 || links[p].x2.phase >= 0;
    }
    size_t pi = 0;
    for (const Phase &ph : phases) {
        const size_t p_index = pi++;
        const nvq_linear &e0 = L[ph.first];
        const int G = e0.K / 32;
        if (e0.K > kStreamMaxK) return {};
        StreamPhase sp = {};
        sp.in_op = e0.in_op;
        sp.eps = e0.eps;
        sp.x2 = e0.in_op != NVQ_IN_PLAIN ? e0.x2_bf16 : nullptr;
        sp.gamma = e0.in_op == NVQ_IN_RMSNORM ? e0.gamma_bf16 : nullptr;
        sp.h_out = e0.in_op == NVQ_IN_RMSNORM && e0.x2_bf16 ? e0.h_out_bf16 : nullptr;
        int rows = 0;
        for (int k = 0; k < ph.count; ++k) {
            const nvq_linear &e = L[ph.first + k];
            sp.qw[k] = reinterpret_cast<const uint4 *>(e.qweight);
            sp.sc[k] = e.scales;
            sp.y[k] = e.y;
            rows += e.N;
            sp.row_end[k] = rows;
            sp.y_dtype[k] = e.y_dtype;
        }
        sp.x = e0.x_bf16;
        sp.nseg = ph.count;
        sp.total_rows = rows;
        sp.K = e0.K;
        sp.G = G;
        sp.gpl = (G + 63) / 64;
        sp.precision = e0.precision;
        sp.row_unit = 1;
        sp.pair_stream = 0;
        sp.spread = waits[p_index] || published[p_index];
        if (G == kStreamPairG && act_group != 32) {
            bool even = true;
            for (int k = 0; k < ph.count; ++k) even = even && L[ph.first + k].N % 2 == 0;
            if (even) sp.row_unit = sp.pair_stream = 2;
        }
        // A phase with fewer rows than would give every wave kStreamThinChunks
        // chunks deals them in larger units to fewer waves: what a wave spends per
        // phase it takes part in (descriptor, image, addresses of its run, the row
        // sums) is then spent once per that many chunks, and the other waves pass.
        // Only where nobody waits for the phase and it waits for nobody: there the
        // waves are free to drift apart and the bytes even out over the phases.
        if (!waits[p_index] && !published[p_index]) {
            const int half_chunks_per_row = sp.pair_stream ? 3 : 2 * sp.gpl;  // in half chunks
            int unit = sp.row_unit;
            while (unit * half_chunks_per_row < 2 * kStreamThinChunks) unit += sp.row_unit;
            if (unit > sp.row_unit && (int64_t)rows < (int64_t)unit * waves) sp.row_unit = unit;
        }
        const int units = (rows + sp.row_unit - 1) / sp.row_unit;  // the last one may be short
        sp.rows_base = units / waves;
        sp.rows_extra = units - sp.rows_base * waves;
        sp.rows_rot = 0;  // set below
        sp.wait_phase = -1;
        sp.publish = 0;
        sp.dep = waits[p_index];
        sp.mail_x = sp.mail_x2 = nullptr;
        sp.mail_h = nullptr;
        for (int k = 0; k < kMaxSeg; ++k) sp.mail_y[k] = nullptr;
        sp.img = nullptr;
        sp.img_chunks = 0;
        tab.push_back(sp);
    }
    const size_t P = tab.size();
    // Which waves get a phase's extra units (a cyclic run of waves, rows_rot its
    // start).  Two ways, the one that leaves the heaviest wave lighter wins: the run
    // that has received the fewest bytes so far, or simply the run after the
    // previous phase's.
    {
        std::vector<int> rot[2];
        uint64_t heaviest[2];
        for (int way = 0; way < 2; ++way) {
            std::fill(extra_bytes.begin(), extra_bytes.end(), 0);
            rot[way].resize(P);
            int next = 0;
            std::vector<uint64_t> view((size_t)waves);
            for (size_t p = 0; p < P; ++p) {
                const int extra = tab[p].rows_extra;
                // extra_bytes is indexed workgroup * kStreamWaves + wave; position j of
                // the phase's dealing order is that wave:
                auto wave_at = [&](int j) {
                    return tab[p].spread ? (size_t)(j % nwg) * kStreamWaves + (size_t)(j / nwg)
                                         : (size_t)j;
                };
                int at = next;
                if (way == 0) {
                    for (int j = 0; j < waves; ++j) view[(size_t)j] = extra_bytes[wave_at(j)];
                    at = lightest_window(view, extra);
                }
                if (extra > 0) next = (next + extra) % waves;
                rot[way][p] = at;
                for (int j = 0; j < extra; ++j)
                    extra_bytes[wave_at((at + j) % waves)] +=
                        (uint64_t)tab[p].G * 18 * tab[p].row_unit;
            }
            heaviest[way] = *std::max_element(extra_bytes.begin(), extra_bytes.end());
        }
        const int way = heaviest[1] < heaviest[0] ? 1 : 0;
        for (size_t p = 0; p < P; ++p) tab[p].rows_rot = rot[way][p];
    }
    for (size_t p = 1; p < P; ++p) {
        tab[p].wait_phase = deps[p];
        if (deps[p] >= 0) tab[deps[p]].publish = 1;
    }
    // Mailboxes: one per linked output, shared by the phases that read it.
    {
        size_t used = 0;
        auto box = [&](const OperandLink &l) -> uint32_t * {
            StreamPhase &src = tab[(size_t)l.phase];
            uint32_t *&slot = l.seg == kMaxSeg ? src.mail_h : src.mail_y[l.seg];
            if (!slot) {
                // (never followed on the host; without a workspace only counted)
                slot = (mail ? mail : reinterpret_cast<uint32_t *>(uintptr_t(4096))) + used;
                const int n = l.seg == kMaxSeg ? src.K
                                               : src.row_end[l.seg] - (l.seg ? src.row_end[l.seg - 1] : 0);
                used += stream_mail_words(n);
            }
            return slot;
        };
        for (size_t p = 1; p < P; ++p) {
            if (links[p].x.phase >= 0) tab[p].mail_x = box(links[p].x);
            if (links[p].x2.phase >= 0) tab[p].mail_x2 = box(links[p].x2);
        }
        if (mail_words) *mail_words = used;
    }
    // The skip table: a wave passes, without looking at them, the phases that give it
    // no rows and have no barrier (nobody waits for them, they wait for nobody).
    if (skips) {
        const int stride = stream_skip_stride((int)P);
        skips->assign((size_t)(waves + nwg) * stride, 0);
        std::vector<uint8_t> active((size_t)waves);
        for (size_t pp = P; pp-- > 0;) {
            const StreamPhase &sp = tab[pp];
            const bool skippable = !sp.dep && !sp.publish;  // no barrier in the phase
            for (int j = 0; j < waves; ++j) {
                int jj = j - sp.rows_rot;
                jj = jj < 0 ? jj + waves : jj;
                const size_t g = sp.spread ? (size_t)(j % nwg) * kStreamWaves + (size_t)(j / nwg)
                                           : (size_t)j;
                active[g] = !skippable || sp.rows_base > 0 || jj < sp.rows_extra;
            }
            for (int g = 0; g < waves; ++g) {
                uint8_t *row = skips->data() + (size_t)g * stride;
                if (active[(size_t)g]) {
                    row[pp] = 0;
                } else {
                    const int next = pp + 1 < P ? row[pp + 1] : 0;
                    row[pp] = (uint8_t)(next >= 255 ? 255 : next + 1);
                }
            }
            for (int wgi = 0; wgi < nwg; ++wgi) {
                bool any = false;
                for (int k = 0; k < kStreamWaves; ++k)
                    any = any || active[(size_t)wgi * kStreamWaves + k];
                (*skips)[(size_t)(waves + wgi) * stride + pp] = any ? 0 : 1;
            }
        }
    }
    // Activation images.  A phase that waits for nothing gets its image
    // prepared in global memory.  In LDS the images of consecutive phases are
    // laid out one after the other in a circular area; img_need names the
    // latest phase whose image a new one overwrites (every wave must have
    // finished that phase before the new image may be loaded).
    size_t off = 0;
    int count = 0;
    struct Live {
        int phase, lo, hi;
    };
    std::vector<Live> live;
    int cursor = 0;
    for (size_t p = 0; p < P; ++p) {
        const int bytes = stream_image_bytes(tab[p].K, tab[p].precision, act_group);
        if (!tab[p].dep) {
            tab[p].img = reinterpret_cast<const uint4 *>(images + off);
            tab[p].img_chunks = bytes / 1024;
            off += (size_t)bytes;
            ++count;
        }
        if (cursor + bytes > kStreamImageArea) cursor = 0;
        int need = -1;
        std::vector<Live> keep;
        for (const Live &l : live) {
            if (l.lo < cursor + bytes && cursor < l.hi)
                need = l.phase > need ? l.phase : need;
            else
                keep.push_back(l);
        }
        live.swap(keep);
        live.push_back({(int)p, cursor, cursor + bytes});
        tab[p].img_lds = cursor;
        // Images are loaded in phase order, so what an earlier image had to wait
        // for has been waited for: the requirement is a running maximum (a region
        // dropped from `live` above may still be partly in use).
        if (p > 0 && tab[p - 1].img_need > need) need = tab[p - 1].img_need;
        tab[p].img_need = need;
        cursor += bytes;
    }
    *nimages = count;
    return tab;
}

__global__ void fill_u32_kernel(uint32_t *p, int n, uint32_t v) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i] = v;
}

}  // namespace

}  // namespace nvq

namespace nvq {
constexpr int kDescribeWords = 16;  // words per phase written by nvq_plan_describe
}

struct nvq_plan {
    std::vector<nvq_linear> layers;
    std::vector<nvq::Phase> phases;
    nvq::Workspace ws;
    int M, act_group;
    int nwg;           // workgroups of the streaming kernel, 0 = per-phase launches
    int nphase;        // entries of the device phase table
    int nwaits;        // phases that wait for an earlier phase (streaming kernel)
    int nimages;       // phases whose activation image is prepared in the prologue
    std::vector<nvq::GroupBatch> batches;  // grouped small-batch launches (empty: not used)
    bool ring;         // grouped launches use the persistent ring kernel
    uint32_t runs;     // walks issued so far (advances the flag base)
    bool pairs;        // some phase of the streaming table deals its rows in pairs
    bool mail;         // some phase of the streaming table posts or reads mail
    int nmail;         // phases that take an operand from a mailbox
    size_t mail_stride;  // words between the replicas of a mailbox
    unsigned long long *trace;  // device buffer for per-phase timestamps, or nullptr
    int trace_wgs;     // workgroups that record there
};

extern "C" size_t nvq_decode_workspace_bytes(const nvq_linear *layers, int n, int M,
                                             int act_group) {
    nvq::ListSizes ls;
    if (nvq::check_layers(layers, n, M, act_group, &ls) != NVQ_OK) return 0;
    return nvq::carve(nullptr, M, n, ls).bytes;
}

extern "C" int nvq_plan_create(const nvq_linear *layers, int n, int M, int act_group, int flags,
                               void *workspace, size_t workspace_bytes, void *stream,
                               nvq_plan **plan_out) {
    using namespace nvq;
    if (!plan_out || (flags & ~NVQ_PLAN_ORDERED)) return NVQ_ERR_INVALID_ARG;
    *plan_out = nullptr;
    ListSizes ls;
    const int rc = check_layers(layers, n, M, act_group, &ls);
    if (rc != NVQ_OK) return rc;
    if (!workspace || !aligned(workspace, 256)) return NVQ_ERR_WORKSPACE;
    const Workspace ws = carve(workspace, M, n, ls);
    if (workspace_bytes < ws.bytes) return NVQ_ERR_WORKSPACE;
    nvq_plan *pl = new (std::nothrow) nvq_plan();
    if (!pl) return NVQ_ERR_UNSUPPORTED;
    pl->layers.assign(layers, layers + n);
    pl->phases = group_phases(pl->layers.data(), n);
    schedule_phases(pl->layers.data(), &pl->phases, M, (flags & NVQ_PLAN_ORDERED) != 0);
    if (check_phase_hazards(pl->layers.data(), pl->phases, M) != NVQ_OK) {
        delete pl;
        return NVQ_ERR_INVALID_ARG;
    }
    pl->ws = ws;
    pl->M = M;
    pl->act_group = act_group;
    pl->runs = 0;
    pl->pairs = false;
    pl->mail = false;
    pl->nmail = 0;
    pl->mail_stride = 0;
    pl->trace = nullptr;
    pl->trace_wgs = 0;
    pl->nwg = 0;
    pl->nphase = 0;
    pl->nwaits = 0;
    pl->nimages = 0;
    pl->ring = false;
    hipStream_t st = (hipStream_t)stream;
    const int nwg = n > 0 ? stream_grid_limit() : 0;
    int nimages = 0;
    std::vector<uint8_t> skips;
    size_t mail_words = 0;
    const std::vector<StreamPhase> tab =
        stream_table(pl->layers.data(), pl->phases, M, act_group, nwg,
                     (flags & NVQ_PLAN_ORDERED) != 0, ws.images, &nimages, &skips, ws.mail,
                     &mail_words);
    if (!tab.empty()) {
        for (const StreamPhase &sp : tab) {
            pl->pairs = pl->pairs || sp.pair_stream != 0;
            pl->nmail += sp.mail_x || sp.mail_x2;
        }
        pl->mail = mail_words > 0;
        pl->mail_stride = stream_mail_stride(ls.mail_words);
        // pageable source: the copy has left the host buffer when the call returns
        hipError_t e = hipMemcpyAsync(ws.tab, tab.data(), tab.size() * sizeof(StreamPhase),
                                      hipMemcpyHostToDevice, st);
        if (e == hipSuccess)
            e = hipMemcpyAsync(ws.skips, skips.data(), skips.size(), hipMemcpyHostToDevice, st);
        if (e == hipSuccess) {
            const int words = kStreamImageFlags + n;  // workgroup flags, status, image flags
            hipLaunchKernelGGL(fill_u32_kernel, dim3((words + 255) / 256), dim3(256), 0, st, ws.flags,
                               words, 0u);
            e = hipGetLastError();
        }
        if (e == hipSuccess && mail_words > 0) {
            // no word of any replica carries a tag yet (tags start at 1)
            const size_t all = pl->mail_stride * kMailReplicas;
            if (all > 0x7fffffffu) {
                delete pl;
                return NVQ_ERR_UNSUPPORTED;
            }
            hipLaunchKernelGGL(fill_u32_kernel, dim3((unsigned)((all + 255) / 256)), dim3(256), 0, st,
                               ws.mail, (int)all, 0u);
            e = hipGetLastError();
        }
        if (e != hipSuccess) {
            set_hip_error(e, "nvq_plan_create");
            delete pl;
            return NVQ_ERR_HIP;
        }
        pl->nwg = nwg;
        pl->nphase = (int)tab.size();
        pl->nimages = nimages;
        for (const StreamPhase &sp : tab) pl->nwaits += sp.dep;
    } else if (n > 0) {
        const GroupPlan gp = group_plan(pl->layers.data(), pl->phases, M, act_group,
                                        (flags & NVQ_PLAN_ORDERED) != 0, ws);
        if (!gp.tab.empty()) {
            // pageable sources: the copies have left the host buffers when the calls return
            hipError_t e = hipMemcpyAsync(ws.gtab, gp.tab.data(), gp.tab.size() * sizeof(GroupPhase),
                                          hipMemcpyHostToDevice, st);
            if (e == hipSuccess && !gp.jobs.empty())
                e = hipMemcpyAsync(ws.gjobs, gp.jobs.data(), gp.jobs.size() * 2,
                                   hipMemcpyHostToDevice, st);
            if (e == hipSuccess)
                e = hipMemcpyAsync(ws.gunits, gp.units.data(), gp.units.size() * 2,
                                   hipMemcpyHostToDevice, st);
            if (e == hipSuccess && !gp.imgs.empty())
                e = hipMemcpyAsync(ws.gimgs, gp.imgs.data(), gp.imgs.size() * 2,
                                   hipMemcpyHostToDevice, st);
            if (e == hipSuccess && !gp.parts.empty())
                e = hipMemcpyAsync(ws.gteams, gp.parts.data(), gp.parts.size() * 4,
                                   hipMemcpyHostToDevice, st);
            if (e == hipSuccess) {
                hipLaunchKernelGGL(fill_u32_kernel, dim3(1), dim3(64), 0, st, ws.status, 1, 0u);
                e = hipGetLastError();
            }
            if (e != hipSuccess) {
                set_hip_error(e, "nvq_plan_create");
                delete pl;
                return NVQ_ERR_HIP;
            }
            pl->batches = gp.batches;
            pl->nwaits = (int)gp.batches.size() - 1;
            pl->ring = gp.ring;
        }
    }
    *plan_out = pl;
    return NVQ_OK;
}

extern "C" int nvq_plan_run(nvq_plan *pl, void *stream) {
    using namespace nvq;
    if (!pl) return NVQ_ERR_INVALID_ARG;
    hipStream_t st = (hipStream_t)stream;
    if (pl->layers.empty()) return NVQ_OK;
    if (pl->nwg > 0) {
        const uint32_t base = pl->runs * (uint32_t)(pl->nphase + 2);
        const uint32_t tag = pl->runs % 65535u + 1u;  // 1..65535, never that of the walk before
        ++pl->runs;
        return launch_decode_stream(pl->ws.tab, pl->ws.skips, pl->nphase, pl->nimages, pl->act_group,
                                    pl->pairs, pl->mail, tag, (uint32_t)pl->mail_stride,
                                    pl->ws.flags, pl->ws.status, base,
                                    pl->ws.dummy, pl->nwg, pl->trace, pl->trace_wgs, st);
    }
    if (!pl->batches.empty()) {
        for (const GroupBatch &b : pl->batches) {
            int rc = pl->ring ? launch_operand_images(pl->ws.gtab, pl->ws.gjobs + b.job_first, b.njobs,
                                                      pl->ws.gimgs + b.img_first, b.nimg, pl->M, st)
                              : launch_quant_act_group(pl->ws.gtab, pl->ws.gjobs + b.job_first,
                                                       b.njobs, pl->M, st);
            if (rc != NVQ_OK) return rc;
            rc = pl->ring ? launch_gemv_mfma_ring(pl->ws.gtab, pl->ws.gteams + b.part_first, b.nparts,
                                                  b.grid, pl->M, pl->ws.status, st)
                          : launch_gemv_mfma_group(pl->ws.gtab, pl->ws.gunits + b.unit_first,
                                                   b.nunits, pl->M, st);
            if (rc != NVQ_OK) return rc;
        }
        return NVQ_OK;
    }
    return walk_per_phase(pl->layers.data(), pl->phases, pl->M, pl->act_group, pl->ws, st);
}

extern "C" int nvq_plan_info(const nvq_plan *pl, int *streaming, int *phases, int *waits) {
    if (!pl) return NVQ_ERR_INVALID_ARG;
    if (streaming) *streaming = pl->nwg > 0 ? 1 : pl->batches.empty() ? 0 : pl->ring ? 3 : 2;
    if (phases) *phases = (int)pl->phases.size();
    if (waits) *waits = pl->nwaits;
    return NVQ_OK;
}

extern "C" int nvq_plan_describe(const nvq_linear *layers, int n, int M, int act_group, int flags,
                                 int workgroups, int32_t *out, int out_words) {
    using namespace nvq;
    if (!out || out_words < 0 || workgroups <= 0 || (flags & ~NVQ_PLAN_ORDERED))
        return NVQ_ERR_INVALID_ARG;
    ListSizes ls;
    const int rc = check_layers(layers, n, M, act_group, &ls);
    if (rc != NVQ_OK) return rc;
    std::vector<Phase> phases = group_phases(layers, n);
    schedule_phases(layers, &phases, M, (flags & NVQ_PLAN_ORDERED) != 0);
    if (check_phase_hazards(layers, phases, M) != NVQ_OK) return NVQ_ERR_INVALID_ARG;
    const bool ordered = (flags & NVQ_PLAN_ORDERED) != 0;
    int nimages = 0;
    const std::vector<StreamPhase> tab =
        stream_table(layers, phases, M, act_group, workgroups, ordered,
                     reinterpret_cast<char *>(uintptr_t(4096)) /* never followed */, &nimages);
    const std::vector<int> deps = phase_deps(layers, phases, M, ordered);
    const int need = 2 + (int)phases.size() * kDescribeWords;
    if (out_words < need) return NVQ_ERR_WORKSPACE;
    out[0] = (int32_t)phases.size();
    out[1] = tab.empty() ? 0 : workgroups * kStreamWaves;
    for (size_t p = 0; p < phases.size(); ++p) {
        int32_t *o = out + 2 + p * kDescribeWords;
        o[0] = phases[p].first;
        o[1] = phases[p].count;
        o[2] = tab.empty() ? deps[p] : tab[p].wait_phase;
        for (int k = 3; k < kDescribeWords; ++k) o[k] = 0;
        if (!tab.empty()) {
            const StreamPhase &sp = tab[p];
            o[3] = sp.publish;
            o[4] = sp.total_rows;
            o[5] = sp.rows_base;
            o[6] = sp.rows_extra;
            o[7] = sp.rows_rot;
            o[8] = sp.img_lds;
            o[9] = sp.img_need;
            o[10] = stream_image_bytes(sp.K, sp.precision, act_group);
            o[11] = sp.img ? 1 : 0;
            o[12] = sp.row_unit;
            o[13] = sp.pair_stream;
            o[14] = sp.spread;
            bool posts = sp.mail_h != nullptr;
            for (int k = 0; k < kMaxSeg; ++k) posts = posts || sp.mail_y[k] != nullptr;
            o[15] = (sp.mail_x ? 1 : 0) + (sp.mail_x2 ? 2 : 0) + (posts ? 4 : 0);
        }
    }
    return NVQ_OK;
}

extern "C" int nvq_plan_describe_skips(const nvq_linear *layers, int n, int M, int act_group,
                                       int flags, int workgroups, uint8_t *out, size_t out_bytes,
                                       int *stride) {
    using namespace nvq;
    if (!out || !stride || workgroups <= 0 || (flags & ~NVQ_PLAN_ORDERED))
        return NVQ_ERR_INVALID_ARG;
    ListSizes ls;
    const int rc = check_layers(layers, n, M, act_group, &ls);
    if (rc != NVQ_OK) return rc;
    std::vector<Phase> phases = group_phases(layers, n);
    schedule_phases(layers, &phases, M, (flags & NVQ_PLAN_ORDERED) != 0);
    if (check_phase_hazards(layers, phases, M) != NVQ_OK) return NVQ_ERR_INVALID_ARG;
    int nimages = 0;
    std::vector<uint8_t> skips;
    const std::vector<StreamPhase> tab =
        stream_table(layers, phases, M, act_group, workgroups, (flags & NVQ_PLAN_ORDERED) != 0,
                     reinterpret_cast<char *>(uintptr_t(4096)) /* never followed */, &nimages,
                     &skips);
    *stride = tab.empty() ? 0 : stream_skip_stride((int)tab.size());
    if (out_bytes < skips.size()) return NVQ_ERR_WORKSPACE;
    std::copy(skips.begin(), skips.end(), out);
    return NVQ_OK;
}

extern "C" int nvq_plan_describe_batches(const nvq_linear *layers, int n, int M, int act_group,
                                         int flags, int32_t *out, int out_words) {
    using namespace nvq;
    if (!out || out_words < 2 || (flags & ~NVQ_PLAN_ORDERED)) return NVQ_ERR_INVALID_ARG;
    ListSizes ls;
    const int rc = check_layers(layers, n, M, act_group, &ls);
    if (rc != NVQ_OK) return rc;
    const std::vector<Phase> phases = group_phases(layers, n);
    if (check_phase_hazards(layers, phases, M) != NVQ_OK) return NVQ_ERR_INVALID_ARG;
    Workspace none = {};  // pointers into it are computed, never followed
    const GroupPlan gp = group_plan(layers, phases, M, act_group, (flags & NVQ_PLAN_ORDERED) != 0,
                                    none);
    out[0] = gp.tab.empty() ? 0 : (int32_t)gp.batches.size();
    out[1] = gp.ring ? 1 : 0;
    if (gp.tab.empty()) return NVQ_OK;
    constexpr int kWords = 6 + 2 * (kRingMaxParts + 1);
    if (out_words < 2 + (int)gp.batches.size() * kWords) return NVQ_ERR_WORKSPACE;
    for (size_t b = 0; b < gp.batches.size(); ++b) {
        const GroupBatch &gb = gp.batches[b];
        int32_t *o = out + 2 + b * kWords;
        for (int k = 0; k < kWords; ++k) o[k] = -1;
        o[0] = gb.nunits > 0 ? gp.units[(size_t)gb.unit_first] : -1;
        o[1] = gb.nunits > 0 ? gp.units[(size_t)gb.unit_first + gb.nunits - 1] : -1;
        o[2] = gb.nunits;
        o[3] = gb.njobs;
        o[4] = gb.grid;
        o[5] = gb.nparts;
        for (int k = 0; k <= gb.nparts && gb.nparts > 0; ++k) {
            o[6 + k] = (int32_t)gp.parts[(size_t)gb.part_first + k];
            o[6 + kRingMaxParts + 1 + k] = (int32_t)gp.parts[(size_t)gb.part_first + gb.nparts + 1 + k];
        }
    }
    return NVQ_OK;
}

extern "C" int nvq_plan_trace(nvq_plan *pl, uint64_t *buf, size_t bytes) {
    if (!pl) return NVQ_ERR_INVALID_ARG;
    const size_t one = (size_t)pl->nphase * nvq::kStreamTraceSlots * 8;
    if (buf && (bytes < one || !nvq::aligned(buf, 8))) return NVQ_ERR_WORKSPACE;
    pl->trace = reinterpret_cast<unsigned long long *>(buf);
    // room for every workgroup: all of them record, else the first one only
    pl->trace_wgs = buf ? (pl->nwg > 0 && bytes >= one * (size_t)pl->nwg ? pl->nwg : 1) : 0;
    return NVQ_OK;
}

extern "C" int nvq_plan_status(nvq_plan *pl, void *stream, int *timed_out) {
    if (!pl || !timed_out) return NVQ_ERR_INVALID_ARG;
    uint32_t v = 0;
    if (pl->nwg > 0 || pl->ring) {
        NVQ_HIP_TRY(hipStreamSynchronize((hipStream_t)stream));
        NVQ_HIP_TRY(hipMemcpy(&v, pl->ws.status, 4, hipMemcpyDeviceToHost));
    }
    *timed_out = (int)v;
    return NVQ_OK;
}

extern "C" void nvq_plan_destroy(nvq_plan *pl) { delete pl; }

extern "C" int nvq_decode_linears(const nvq_linear *layers, int n, int M, int act_group,
                                  void *workspace, size_t workspace_bytes, void *stream) {
    if (n == 0) {
        nvq::ListSizes ls;
        return nvq::check_layers(layers, n, M, act_group, &ls);
    }
    nvq_plan *pl = nullptr;
    int rc = nvq_plan_create(layers, n, M, act_group, NVQ_PLAN_DEFAULT, workspace, workspace_bytes,
                             stream, &pl);
    if (rc != NVQ_OK) return rc;
    rc = nvq_plan_run(pl, stream);
    nvq_plan_destroy(pl);
    return rc;
}

extern "C" int nvq_decode_status(const void *workspace, void *stream, int *timed_out) {
    if (!workspace || !timed_out || !nvq::aligned(workspace, 256)) return NVQ_ERR_INVALID_ARG;
    uint32_t v = 0;
    NVQ_HIP_TRY(hipStreamSynchronize((hipStream_t)stream));
    NVQ_HIP_TRY(hipMemcpy(&v, static_cast<const char *>(workspace) + NVQ_WORKSPACE_STATUS_OFFSET, 4,
                          hipMemcpyDeviceToHost));
    *timed_out = (int)v;
    return NVQ_OK;
}

// ---- the walk for callers that cannot allocate ------------------------------
namespace nvq {
namespace {

// Activation codes, scales and code sums of the phase being run (and its
// transformed input): the scratch memory of the per-phase launches.  One copy
// per GPU, held until the process ends; its address on a device is looked up
// once, with that device current.
static __device__ __align__(256) unsigned char scratch[NVQ_STATIC_SCRATCH_BYTES];

constexpr int kMaxDevices = 64;
void *g_scratch_ptr[kMaxDevices];  // per device, nullptr until looked up
std::mutex g_scratch_mutex;

int scratch_for_current_device(void **out) {
    int dev = 0;
    NVQ_HIP_TRY(hipGetDevice(&dev));
    if (dev < 0 || dev >= kMaxDevices) return NVQ_ERR_UNSUPPORTED;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void *p = nullptr;
        NVQ_HIP_TRY(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
        if (!p || !aligned(p, 256)) return NVQ_ERR_HIP;
        g_scratch_ptr[dev] = p;
    }
    *out = g_scratch_ptr[dev];
    return NVQ_OK;
}

}  // namespace
}  // namespace nvq

extern "C" int nvq_decode_linears_static(const nvq_linear *layers, int n, int M, int act_group,
                                         void *stream) {
    using namespace nvq;
    ListSizes ls;
    const int rc = check_layers(layers, n, M, act_group, &ls);
    if (rc != NVQ_OK) return rc;
    if (n == 0) return NVQ_OK;
    const std::vector<Phase> phases = group_phases(layers, n);
    if (check_phase_hazards(layers, phases, M) != NVQ_OK) return NVQ_ERR_INVALID_ARG;
    // the part of the workspace that launches per phase use
    const size_t G = (size_t)ls.maxK / 32;
    const size_t xt_bytes = round_up(ls.transforms ? (size_t)M * ls.maxK * 2 : 0, 256);
    const size_t xq_bytes = round_up((size_t)M * ls.maxK, 256);
    const size_t gs_bytes = round_up((size_t)M * G * 4, 256);
    if (xt_bytes + xq_bytes + 2 * gs_bytes > (size_t)NVQ_STATIC_SCRATCH_BYTES)
        return NVQ_ERR_WORKSPACE;
    void *base = nullptr;
    const int sc = scratch_for_current_device(&base);
    if (sc != NVQ_OK) return sc;
    Workspace ws = {};
    char *b = static_cast<char *>(base);
    ws.xt = reinterpret_cast<uint16_t *>(b);
    ws.xq = reinterpret_cast<int8_t *>(b + xt_bytes);
    ws.xscale = reinterpret_cast<float *>(b + xt_bytes + xq_bytes);
    ws.xgsum = reinterpret_cast<int32_t *>(b + xt_bytes + xq_bytes + gs_bytes);
    // every phase writes what it reads from the scratch before reading it
    // (transform, quantisation), so nothing has to be cleared between calls
    return walk_per_phase(layers, phases, M, act_group, ws, (hipStream_t)stream);
}
