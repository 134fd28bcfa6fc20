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
constexpr int tile_rows(int gpl) { return gpl <= 1 ? 8 : gpl <= 2 ? 4 : gpl <= 4 ? 2 : 1; }

// Grid size for a batch-1 GEMV: enough workgroups of `teams_per_wg` teams to
// give every tile a team, capped at `wg_per_cu` resident workgroups per
// compute unit (the kernels are grid-stride beyond that).
static inline int gemv_grid(int tiles, int teams_per_wg, int wg_per_cu) {
    int want = (tiles + teams_per_wg - 1) / teams_per_wg;
    int cap = device_cu_count() * wg_per_cu;
    if (want < 1) want = 1;
    return want < cap ? want : cap;
}

}  // namespace nvq
