// Interface between the host-side walker and the persistent streaming kernel.
#pragma once

#include "nvq_internal.h"

namespace nvq {

constexpr int kStreamWaves = 12;  // streaming waves per workgroup (three per SIMD)
constexpr int kStreamThreads = (kStreamWaves + 1) * 64;  // plus the loader wave
constexpr int kStreamMaxK = 14336;     // widest input an activation image holds
constexpr int kStreamImageMax = 31744;  // largest image, padded to whole KiB (bf16, K = 14336)
constexpr int kStreamImageArea = 59392; // LDS bytes that hold the images of consecutive phases
constexpr int kStreamMaxWg = 1024;      // flag words reserved for workgroups
// Layout of the flag words: [0, kStreamMaxWg) one per workgroup, then 64 status
// words, then kFlagReplicas - 1 more copies of the workgroup flags (a workgroup
// raises its flag in every copy and polls the copy of its XCD: 256 workgroups
// polling the same kilobyte made the memory channel that holds it the bound of
// the wait), then one word per phase ("the prepared image of this phase is
// stored").
constexpr int kFlagReplicas = 8;
constexpr int kStreamFlagCopies = kStreamMaxWg + 64;  // copies 1 .. kFlagReplicas - 1
constexpr int kStreamImageFlags = kStreamFlagCopies + (kFlagReplicas - 1) * kStreamMaxWg;
// Skip table: one row of skip_stride(phases) bytes per streaming wave (workgroup *
// kStreamWaves + wave); byte p = how many phases from p on the wave may pass
// without a look (it has no rows in them and they have no barriers), at most 255.
// Then one row per workgroup: byte p = 1 if all its waves pass phase p (the loader
// wave does not fetch that phase's image), else 0.
constexpr int stream_skip_stride(int nphase) { return (nphase + 4 + 3) / 4 * 4; }
constexpr int kStreamPairG = 96;  // groups per row for which rows are streamed in pairs
// Chunks a wave should at least get from a phase it works on (measured on 1B-, 3B-
// and 8B-shaped steps: 4 -> 8 -> 12 gains at every step, flat from 12 to 16, 24 and
// more lose again).
constexpr int kStreamThinChunks = 12;

// One phase = up to four weight matrices that read the same input vector.
// Lives in device memory; every field is read wave-uniformly.
struct StreamPhase {
    const uint4 *qw[kMaxSeg];
    const uint16_t *sc[kMaxSeg];
    void *y[kMaxSeg];
    int row_end[kMaxSeg];  // first row after segment i (rows numbered across segments)
    int y_dtype[kMaxSeg];
    const uint16_t *x;     // bf16 [K]
    // what stands between x and the layer (NVQ_IN_*): RMSNorm of x (+ x2) times
    // gamma, with the sum stored to h_out, or SiLU(x) * x2
    const uint16_t *x2, *gamma;
    uint16_t *h_out;
    int in_op;
    float eps;
    int nseg, total_rows;
    int K, G, gpl;         // G = K/32, gpl = ceil(G/64) <= 7
    int precision;         // NVQ_W4A8 | NVQ_W4A16
    // Rows are dealt to the W = workgroups * kStreamWaves waves as evenly as whole
    // rows allow.  Workgroups count XCD by XCD here (of a grid of a multiple of 8,
    // workgroup b is number (b mod 8) * grid / 8 + b / 8), and so do the rows of the
    // skip table.  wave = workgroup * kStreamWaves + wave in the workgroup, or, with
    // spread = 1, wave in the workgroup * workgroups + workgroup: then neighbours sit
    // on different compute units and the waves that get a phase's extra rows are
    // spread evenly over them, which a phase that others wait for needs (it ends with
    // its busiest compute unit; 18 % of the step time of a dependent chain), while
    // independent phases stream faster (5 %) with a compute unit's waves on
    // neighbouring rows.  Wave j' = (wave - rows_rot) mod W takes rows_base units
    // of rows, one more if j' < rows_extra, in order of j'.  The host chooses
    // rows_rot per phase so that the extra units go to the waves that have
    // received the fewest bytes so far, or simply to the run of waves after the
    // previous phase's, whichever leaves the heaviest wave of the table lighter.
    int rows_base, rows_extra, rows_rot;
    // A unit is row_unit neighbouring rows (the last unit of the phase may be
    // short): 1, or more where an independent phase is too short to give every
    // wave kStreamThinChunks chunks.  pair_stream = 2 with G = 96, where a row is
    // one and a half chunks: rows 2i and 2i + 1 are streamed as three full chunks,
    // the middle one half of each row, instead of four chunks of which two are
    // half empty; it needs an even number of rows in every segment, per-token
    // activation scales and an even row_unit.  Otherwise 0.
    int row_unit, pair_stream;
    int spread;
    int wait_phase;        // latest earlier phase this one waits for through the flags, or -1
    int publish;           // 1 if a later phase waits for this one through the flags
    // Mail: an input operand that is exactly the bf16 output (or residual sum) of
    // one earlier phase is not read from the caller's buffer.  The producing waves
    // also post every value as a 32-bit word (tag << 16 | bf16 bits) in a mailbox of
    // the workspace, with write-through stores and without waiting for anything; the
    // consumers poll the words themselves until all carry the tag of this walk.  A
    // word is its own flag, so no fence, no flag and no wait on the producer's side
    // are needed, and the consumer's first look at the data is its wait.
    // Word order inside a mailbox: values in pieces of 512; value 8 l + e of a piece
    // (l < 64, e < 8) is word (e / 4) * 256 + 4 l + e % 4 of the piece, so that lane l
    // of a wave collects its eight values with two fully coalesced 16-byte loads.
    // Every mailbox exists kMailReplicas times, stream_mail_stride words apart; the
    // producers post to all of them, a consumer polls the replica of its XCD
    // (workgroup number modulo 8).  All 256 workgroups polling the same lines made
    // the few memory channels that hold them the bound of the wait; with replicas
    // the same requests spread over eight times as many.  The pointers below name
    // replica 0.
    const uint32_t *mail_x, *mail_x2;  // mailboxes this phase reads x / x2 from, or nullptr
    uint32_t *mail_y[kMaxSeg];         // where the outputs of segment i are also posted, or nullptr
    uint32_t *mail_h;                  // where the residual sum is also posted, or nullptr
    int dep;               // 1 if the phase builds its image itself after waiting (flags or mail)
    int img_chunks;        // KiB chunks of the prepared image (0 if built in the kernel)
    int img_lds;           // byte offset of the phase's image inside the LDS image area
    int img_need;          // latest phase whose image this one overwrites in LDS, or -1
    const uint4 *img;      // prepared image in global memory, or nullptr
};

// Workgroups the streaming kernel may be launched with (all must be
// co-resident): the number of compute units, or 0 if the kernel does not fit.
int stream_grid_limit();

#if defined(__HIPCC__)
// First row and row count of wave `gw` (of `waves`) in a phase.
__device__ __forceinline__ void stream_wave_rows(int rows_base, int rows_extra, int rows_rot,
                                                 int gw, int waves, int &first, int &count) {
    int j = gw - rows_rot;
    j = j < 0 ? j + waves : j;
    const int more = j < rows_extra ? j : rows_extra;
    first = j * rows_base + more;
    count = rows_base + (j < rows_extra ? 1 : 0);
}

#endif

// Words of a mailbox for `n` values (whole pieces of 512).
static inline size_t stream_mail_words(int n) { return ((size_t)n + 511) / 512 * 512; }
// Replicas of every mailbox, and the distance in words between two replicas of
// an area that holds `words` words of mailboxes (an odd number of 256-byte units
// on top of whole 16 KiB, so that replicas do not fall on the same memory channels).
constexpr int kMailReplicas = 8;
static inline size_t stream_mail_stride(size_t words) {
    return words == 0 ? 0 : (words + 4095) / 4096 * 4096 + 33 * 64;
}

// Bytes of the activation image of a layer with K inputs, padded to whole KiB.
static inline int stream_image_bytes(int K, int precision, int act_group) {
    const int G = K / 32;
    const int raw = precision == NVQ_W4A8 ? 36 * G + (act_group == 32 ? 4 * G : 0) + 16 : 68 * G;
    return (raw + 1023) / 1024 * 1024;
}

// Enqueue one walk.  `flags` holds one word per workgroup, the status words
// (`status` = flags + kStreamMaxWg; word 0 is set to a code if a wait gave up) and
// one word per phase; all persist between runs of the same table, with
// `flag_base` advanced by nphase + 2 per run (image word = base + 1: the
// phase's image is stored; workgroup word = base + 2 + p: phase p published).  `nimages` = phases with a prepared
// image (0 skips the prologue).  `dummy` is any valid
// 1 KiB of device memory.  `trace` is nullptr or trace_wgs * nphase * 8 words
// that receive the per-phase timestamps of the first trace_wgs workgroups (of the
// phases their first wave does not pass).  `skips`: the skip table, nwg * (kStreamWaves + 1) rows.  `pairs` says that some phase of
// the table streams its rows in pairs (pair_stream): the kernel variant that has
// that path is launched.  `mail`: some phase of the table posts or reads mail (the
// kernel variant with that path); `mail_tag` (1..65535) is the tag of this walk:
// it must differ from the tag of the walk before it on the same mailboxes, and a
// mailbox is cleared to zero before its first use; `mail_stride`: words between
// the replicas of a mailbox.
int launch_decode_stream(const StreamPhase *tab_dev, const uint8_t *skips, int nphase, int nimages,
                         int act_group, bool pairs, bool mail, uint32_t mail_tag,
                         uint32_t mail_stride, uint32_t *flags,
                         uint32_t *status, uint32_t flag_base, const void *dummy, int nwg,
                         unsigned long long *trace, int trace_wgs, hipStream_t st);

// Timestamps written per phase when a trace buffer is given (see the kernel).
constexpr int kStreamTraceSlots = 8;

}  // namespace nvq
