// Row-tile bookkeeping shared by the two batch-1 GEMV kernels.
//
// Work decomposition (both kernels): a "team" of LPR lanes (64 or 32) owns a
// whole weight row at a time.  Lane l of the team owns the groups
// g = i*LPR + l, i < GPL, of every row, so that one load instruction of the
// team reads LPR consecutive 16-byte groups (1 KiB or 512 B of one row), and
// the activation values of those groups stay in the lane's registers for the
// whole kernel.  Teams walk row tiles of U rows in a grid-stride loop and
// fetch the next tile before computing the current one.
#pragma once

#include "nvq_internal.h"

namespace nvq {

// 16 bytes that are read once (weights): a non-temporal load.
__device__ __forceinline__ uint4 stream_load16(const uint4 *p) {
    typedef uint32_t u32x4_nt __attribute__((ext_vector_type(4)));
    const u32x4_nt v = __builtin_nontemporal_load(reinterpret_cast<const u32x4_nt *>(p));
    return make_uint4(v.x, v.y, v.z, v.w);
}

struct RowRef {
    const uint4 *qw;     // first group of the row
    const uint16_t *sc;  // first scale of the row
    void *y;             // output vector of the row's segment
    int32_t *dbg;        // accumulator dump of the row's segment (or nullptr)
    int N;               // rows in the segment
    int n;               // row index inside the segment
    int y_dtype;
    bool valid;
};

// Map a global row number to its segment.  Rows past the end are clamped to
// the last row so that loads stay in bounds; `valid` masks the stores.  SEGS is
// a (possibly address-space qualified) GemvSegs.
template <typename SEGS>
__device__ __forceinline__ RowRef locate_row(SEGS &S, int row, int G) {
    RowRef r;
    r.valid = row < S.total_rows;
    if (!r.valid) row = S.total_rows - 1;
    // select chain instead of indexing: the segment table lives in kernel
    // arguments and a dynamic index would force it through scratch memory
    int first = 0;
    r.qw = S.qw[0];
    r.sc = S.sc[0];
    r.y = S.y[0];
    r.dbg = S.dbg[0];
    r.N = S.N[0];
    r.y_dtype = S.y_dtype[0];
#pragma unroll
    for (int i = 1; i < kMaxSeg; ++i) {
        if (i < S.nseg && row >= S.row_end[i - 1]) {
            first = S.row_end[i - 1];
            r.qw = S.qw[i];
            r.sc = S.sc[i];
            r.y = S.y[i];
            r.dbg = S.dbg[i];
            r.N = S.N[i];
            r.y_dtype = S.y_dtype[i];
        }
    }
    r.n = row - first;
    r.qw += (int64_t)r.n * G;
    r.sc += (int64_t)r.n * G;
    return r;
}

// Rows per tile for a given groups-per-lane count: about eight 16-byte loads
// per lane per tile.
// Resident workgroups per compute unit of the batch-1 kernels (measured on a 295 MB
// layer: 2 -> 3 workgroups 68 -> 60 us, 4 and 6 no better).
constexpr int kM1WgPerCu = 3;
constexpr int tile_rows(int gpl) { return gpl <= 1 ? 8 : gpl <= 2 ? 4 : gpl <= 4 ? 2 : 1; }

// Grid size for a batch-1 GEMV: enough workgroups of `teams_per_wg` teams to
// give every tile a team, at most `wg_per_cu` resident workgroups per
// compute unit (the kernels are grid-stride beyond that).
static inline int gemv_grid(int tiles, int teams_per_wg, int wg_per_cu) {
    int want = (tiles + teams_per_wg - 1) / teams_per_wg;
    const int cus = device_cu_count();
    if (want < 1) want = 1;
    if (want <= cus * wg_per_cu) return want;
    // A whole number k of workgroups per compute unit; the work takes ceil(want / grid)
    // rounds, and a round costs a compute unit k / efficiency(k) (measured: two resident
    // workgroups stream at 0.85, one at 0.6 of the rate of three or more).  1024
    // workgroups' worth of tiles are better served by 512 (two even rounds) than by
    // 768 (two rounds, the second a third full).
    int best = cus;
    double best_cost = 1e30;
    for (int k = 1; k <= wg_per_cu; ++k) {
        const double eff = k == 1 ? 0.6 : k == 2 ? 0.85 : 1.0;
        const int rounds = (want + cus * k - 1) / (cus * k);
        const double cost = rounds * (k / eff);
        if (cost < best_cost) {
            best_cost = cost;
            best = cus * k;
        }
    }
    return best;
}

}  // namespace nvq
