// nvq_decode_linears: walk the linear layers of one decode step under a
// per-layer precision map.  Paper: routing rule of the precision-dispatch
// section (W4A16 if the layer's normalised score reaches the threshold, else
// W4A8); activation codes are computed once per input and reused by every
// projection that reads it.
//
// The host groups consecutive entries that read the same input with the same
// precision into a phase (q/k/v, gate/up) and serves a phase with one fused
// GEMV launch over up to four weight matrices.  Launches are only enqueued,
// never waited for, so a caller can record the whole walk into a HIP graph.
#include "nvq_internal.h"

namespace nvq {

struct Workspace {
    int8_t *xq;
    float *xscale;
    int32_t *xgsum;
    size_t bytes;
};

static size_t round_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

// Scratch for the activation codes of the widest layer.
static Workspace carve(void *base, int maxK, int M) {
    Workspace w;
    const size_t G = (size_t)maxK / 32;
    size_t off = 0;
    w.xq = reinterpret_cast<int8_t *>(reinterpret_cast<char *>(base) + off);
    off += round_up((size_t)M * maxK, 256);
    w.xscale = reinterpret_cast<float *>(reinterpret_cast<char *>(base) + off);
    off += round_up((size_t)M * G * 4, 256);
    w.xgsum = reinterpret_cast<int32_t *>(reinterpret_cast<char *>(base) + off);
    off += round_up((size_t)M * G * 4, 256);
    w.bytes = off;
    return w;
}

static int check_layers(const nvq_linear *L, int n, int M, int act_group, int *maxK) {
    if (!L || n < 0) return NVQ_ERR_INVALID_ARG;
    if (act_group != 0 && act_group != 32) return NVQ_ERR_INVALID_ARG;
    if (M <= 0 || M > NVQ_MAX_M) return NVQ_ERR_SHAPE;
    int mk = 32;
    for (int i = 0; i < n; ++i) {
        const nvq_linear &e = L[i];
        if (!e.qweight || !e.scales || !e.x_bf16 || !e.y) return NVQ_ERR_INVALID_ARG;
        if (e.precision != NVQ_W4A8 && e.precision != NVQ_W4A16) return NVQ_ERR_INVALID_ARG;
        if (e.y_dtype != NVQ_F32 && e.y_dtype != NVQ_BF16) return NVQ_ERR_INVALID_ARG;
        if (e.N <= 0 || e.K <= 0 || (e.K % 32) != 0 || e.K > NVQ_MAX_K) return NVQ_ERR_SHAPE;
        if (!aligned(e.qweight, 16) || !aligned(e.scales, 2) || !aligned(e.x_bf16, 16) ||
            !aligned(e.y, e.y_dtype == NVQ_F32 ? 4 : 2))
            return NVQ_ERR_ALIGN;
        if (e.K > mk) mk = e.K;
    }
    *maxK = mk;
    return NVQ_OK;
}

}  // namespace nvq

extern "C" size_t nvq_decode_workspace_bytes(const nvq_linear *layers, int n, int M,
                                             int act_group) {
    int maxK = 0;
    if (nvq::check_layers(layers, n, M, act_group, &maxK) != NVQ_OK) return 0;
    return nvq::carve(nullptr, maxK, M).bytes;
}

extern "C" int nvq_decode_linears(const nvq_linear *layers, int n, int M, int act_group,
                                  void *workspace, size_t workspace_bytes, void *stream) {
    using namespace nvq;
    int maxK = 0;
    const int rc = check_layers(layers, n, M, act_group, &maxK);
    if (rc != NVQ_OK) return rc;
    if (n == 0) return NVQ_OK;
    if (!workspace || !aligned(workspace, 256)) return NVQ_ERR_WORKSPACE;
    const Workspace ws = carve(workspace, maxK, M);
    if (workspace_bytes < ws.bytes) return NVQ_ERR_WORKSPACE;
    hipStream_t st = (hipStream_t)stream;

    int i = 0;
    while (i < n) {
        // a phase: consecutive entries with the same input, K and precision
        int j = i + 1;
        while (j < n && layers[j].x_bf16 == layers[i].x_bf16 && layers[j].K == layers[i].K &&
               layers[j].precision == layers[i].precision)
            ++j;
        const int K = layers[i].K;
        if (layers[i].precision == NVQ_W4A8) {
            const int q = launch_quant_act(layers[i].x_bf16, M, K, act_group, ws.xq, ws.xscale,
                                           ws.xgsum, st);
            if (q != NVQ_OK) return q;
        }
        for (int b = i; b < j; b += kMaxSeg) {
            GemvSegs S = {};
            int rows = 0;
            const int e = b + kMaxSeg < j ? b + kMaxSeg : j;
            for (int s = b; s < e; ++s) {
                const int k = s - b;
                S.qw[k] = reinterpret_cast<const uint4 *>(layers[s].qweight);
                S.sc[k] = layers[s].scales;
                S.y[k] = layers[s].y;
                S.dbg[k] = nullptr;
                S.N[k] = layers[s].N;
                rows += layers[s].N;
                S.row_end[k] = rows;
                S.y_dtype[k] = layers[s].y_dtype;
            }
            S.nseg = e - b;
            S.total_rows = rows;
            const int g = layers[i].precision == NVQ_W4A8
                              ? launch_gemv_w4a8(S, K, ws.xq, ws.xscale, ws.xgsum, act_group, M, st)
                              : launch_gemv_w4a16(S, K, layers[i].x_bf16, M, st);
            if (g != NVQ_OK) return g;
        }
        i = j;
    }
    return NVQ_OK;
}
