// Internal declarations shared by the translation units of libnvq (host side
// and gfx950 device helpers).  Not installed; the public ABI is include/nvq.h.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "nvq.h"

namespace nvq {

// ---- host helpers ---------------------------------------------------------
void set_hip_error(hipError_t e, const char *where);
int device_cu_count();  // compute units of the current device (cached)

#define NVQ_HIP_TRY(expr)                                   \
    do {                                                    \
        hipError_t e_ = (expr);                             \
        if (e_ != hipSuccess) {                             \
            ::nvq::set_hip_error(e_, #expr);                \
            return NVQ_ERR_HIP;                             \
        }                                                   \
    } while (0)

static inline bool aligned(const void *p, size_t a) {
    return (reinterpret_cast<uintptr_t>(p) & (a - 1)) == 0;
}

// Up to four weight matrices that read the same input can be served by one
// GEMV launch (q/k/v, gate/up).  Rows are numbered consecutively across the
// segments; row_end[i] is the first row after segment i.
constexpr int kMaxSeg = 4;
struct GemvSegs {
    const uint4 *qw[kMaxSeg];     // [N_i][G] one uint4 = one group of 32 nibbles
    const uint16_t *sc[kMaxSeg];  // [N_i][G] fp16 bits
    void *y[kMaxSeg];             // [M][N_i]
    int32_t *dbg[kMaxSeg];        // [M][N_i][G] or nullptr
    int N[kMaxSeg];
    int row_end[kMaxSeg];
    int y_dtype[kMaxSeg];
    int nseg;
    int total_rows;
};

// Internal launchers (validated arguments; enqueue only).
int launch_quant_act(const uint16_t *x, int M, int K, int act_group, int8_t *xq, float *xscale,
                     int32_t *xgsum, hipStream_t st);
int launch_gemv_w4a8(const GemvSegs &segs, int K, const int8_t *xq, const float *xscale,
                     const int32_t *xgsum, int act_group, int M, hipStream_t st);
int launch_gemv_w4a16(const GemvSegs &segs, int K, const uint16_t *x, int M, hipStream_t st);
// Matrix-core path for 2 <= M <= 32 tokens (per-token activation scale, K a
// multiple of 128, scale rows 8-byte aligned); `x` is the int8 codes or the
// bf16 activations according to `precision`.
bool gemv_mfma_supported(const GemvSegs &segs, int K, int M);
int launch_gemv_mfma(const GemvSegs &segs, int K, int precision, const void *x,
                     const float *xscale, int M, hipStream_t st);

// One phase of a grouped small-batch launch (lives in device memory): the
// activation quantisation of all its tokens (W4A8) and the matrix-core product
// of its row tiles run in grids shared with the other phases of its batch.
struct GroupPhase {
    GemvSegs segs;           // accumulator dumps unused
    const uint16_t *x_bf16;  // [M][K] input
    int8_t *xq;              // [M][K]   codes      (W4A8 phases, workspace)
    float *xscale;           // [M]      scales
    int32_t *xgsum;          // [M][K/32] code sums
    char *xa;                // operand image of the persistent kernel (either precision, workspace)
    int G, precision;
    int unit_begin;          // first grid unit of the phase in its batch
    int unit_count;          // its units
    int img_begin;           // first image unit of the phase in its batch (launch_operand_images)
};
// jobs[j] names the phase whose M tokens grid blocks j*M .. j*M+M-1 quantise.
int launch_quant_act_group(const GroupPhase *tab, const uint16_t *jobs, int njobs, int M,
                           hipStream_t st);
// The operand images `xa` of the phases named in `jobs` (per-token scales of
// the W4A8 ones first, then the images: img_units[u] names the phase of image
// unit u, a token tile times eight 128-input columns; image_units(M, K) of
// them per phase, numbered from GroupPhase::img_begin).  Per tile of 16
// tokens, column c and piece i one KiB whose 16 bytes number 16 * kb + n are,
// for token n of the tile, the int8 codes 32 * kb + 16 * i .. + 15 of the
// column (W4A8, two pieces; xscale as in launch_quant_act_group, no code sums)
// or the bf16 inputs 32 * i + 8 * kb .. + 7 of the column, copied (W4A16, four
// pieces).  Token slots past M are left as they are.
int image_units(int M, int K);
int launch_operand_images(const GroupPhase *tab, const uint16_t *jobs, int njobs,
                          const uint16_t *img_units, int nimg, int M, hipStream_t st);
// unit_phase[u] names the phase of grid unit u; a unit is group_row_tiles(M)
// consecutive 16-row tiles, which share their activation operands (as many as
// fit the registers next to one or two token tiles).
static inline int group_row_tiles(int M) { (void)M; return 2; }
int launch_gemv_mfma_group(const GroupPhase *tab, const uint16_t *unit_phase, int nunits, int M,
                           hipStream_t st);
// The same work as one persistent grid of teams (a loader wave feeding four
// consumer waves through LDS rings); needs K % 512 == 0 and 16-byte aligned
// scale rows in every phase, and the operand images of launch_quant_act_group.
// The batch is cut into `nparts` = ring_parts(grid) parts of equal weight bytes
// that the workgroups of one XCD each work off together; part_tab (device
// memory): nparts + 1 unit indices, the cuts, then nparts + 1 phase indices,
// the phase of the unit at each cut.  A wait inside the kernel that gives up
// sets *status.
constexpr int kRingMaxParts = 8;
bool gemv_mfma_ring_supported(const GemvSegs &segs, int K);
int ring_grid(int M, int nunits);
int ring_parts(int grid);
int launch_gemv_mfma_ring(const GroupPhase *tab, const uint32_t *part_tab, int nparts, int grid,
                          int M, uint32_t *status, hipStream_t st);

// ---- device helpers -------------------------------------------------------
#if defined(__HIPCC__)

__device__ __forceinline__ float bf16_bits_to_float(uint32_t h) {
    return __uint_as_float(h << 16);
}

// fp32 -> bf16 bits, round to nearest even: the hardware's conversion
// (v_cvt_pk_bf16_f32, one instruction for two values).
__device__ __forceinline__ uint16_t float_to_bf16_bits(float f) {
    return __builtin_bit_cast(uint16_t, (__bf16)f);
}
typedef __bf16 nvq_bf16x2 __attribute__((ext_vector_type(2)));
// ... two at a time, `lo` in the low half of the word.
__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {
    const nvq_bf16x2 v = {(__bf16)lo, (__bf16)hi};
    return __builtin_bit_cast(uint32_t, v);
}

__device__ __forceinline__ float half_bits_to_float(uint16_t h) {
    _Float16 v = __builtin_bit_cast(_Float16, h);
    return (float)v;
}

// Sum across the LPR lanes of an aligned lane group; every lane gets the sum.
template <int LPR>
__device__ __forceinline__ float group_sum(float v) {
#pragma unroll
    for (int off = LPR / 2; off > 0; off >>= 1) v += __shfl_xor(v, off, 64);
    return v;
}

__device__ __forceinline__ void store_out(void *y, int y_dtype, int64_t idx, float v) {
    if (y_dtype == NVQ_F32)
        reinterpret_cast<float *>(y)[idx] = v;
    else
        reinterpret_cast<uint16_t *>(y)[idx] = float_to_bf16_bits(v);
}

#endif  // __HIPCC__

}  // namespace nvq
