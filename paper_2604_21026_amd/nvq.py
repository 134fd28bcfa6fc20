"""Thin ctypes binding over libnvq.so (C ABI in include/nvq.h).

Argument marshalling only: torch supplies device memory and the current
stream, every computation happens in the library's HIP kernels.  There is no
fallback: if libnvq.so is missing, loading fails with an error.
"""
import ctypes as C
import os
from typing import List, Optional, Sequence

import torch

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "libnvq.so")

F32, BF16 = 0, 1
W4A8, W4A16 = 0, 1
MAX_M = 32
PLAN_ORDERED = 1
IN_PLAIN, IN_RMSNORM, IN_SILU_MUL = 0, 1, 2

EXPORTS = (
    "nvq_status_string", "nvq_last_hip_error", "nvq_pack_int4", "nvq_quant_act_i8",
    "nvq_gemv_w4a16", "nvq_gemv_w4a8", "nvq_decode_workspace_bytes", "nvq_decode_linears",
    "nvq_decode_status", "nvq_decode_linears_static",
    "nvq_plan_create", "nvq_plan_run", "nvq_plan_info", "nvq_plan_status", "nvq_plan_trace",
    "nvq_plan_destroy", "nvq_plan_describe", "nvq_plan_describe_batches",
    "nvq_plan_describe_skips",
    "nvq_dequant_bf16", "nvq_gemm_w4a16", "nvq_rms_norm_bf16", "nvq_silu_mul_bf16", "nvq_precision_from_scores", "nvq_token_norms", "nvq_mcap_scores", "nvq_stream_read", "nvq_stream_copy",
)


class NvqError(RuntimeError):
    def __init__(self, status: int, what: str, detail: str = ""):
        self.status = status
        super().__init__("%s failed: status %d (%s)%s" % (what, status, _status_string(status),
                                                          (": " + detail) if detail else ""))


class Linear(C.Structure):
    """Mirror of `nvq_linear`."""
    _fields_ = [("qweight", C.c_void_p), ("scales", C.c_void_p), ("N", C.c_int32),
                ("K", C.c_int32), ("x_bf16", C.c_void_p), ("y", C.c_void_p),
                ("y_dtype", C.c_int32), ("precision", C.c_int32), ("in_op", C.c_int32),
                ("eps", C.c_float), ("x2_bf16", C.c_void_p), ("gamma_bf16", C.c_void_p),
                ("h_out_bf16", C.c_void_p)]


_lib = None


def lib() -> C.CDLL:
    """Load libnvq.so (built beforehand by paper_2604_21026_amd.build)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise FileNotFoundError(
            "%s not found: build it with `python -m paper_2604_21026_amd.build`" % LIB_PATH)
    L = C.CDLL(LIB_PATH)
    vp, ci, i64, sz = C.c_void_p, C.c_int, C.c_int64, C.c_size_t
    L.nvq_status_string.restype = C.c_char_p
    L.nvq_status_string.argtypes = [ci]
    L.nvq_last_hip_error.restype = C.c_char_p
    L.nvq_last_hip_error.argtypes = []
    L.nvq_pack_int4.argtypes = [vp, i64, i64, ci, vp, vp, vp]
    L.nvq_dequant_bf16.argtypes = [vp, vp, i64, i64, vp, vp]
    L.nvq_gemm_w4a16.argtypes = [vp, vp, i64, i64, vp, i64, vp, ci, vp]
    L.nvq_rms_norm_bf16.argtypes = [vp, vp, vp, C.c_float, ci, ci, vp, vp, vp]
    L.nvq_silu_mul_bf16.argtypes = [vp, vp, ci, ci, vp, vp]
    L.nvq_quant_act_i8.argtypes = [vp, ci, ci, ci, vp, vp, vp, vp]
    L.nvq_gemv_w4a16.argtypes = [vp, vp, ci, ci, vp, ci, vp, ci, vp]
    L.nvq_gemv_w4a8.argtypes = [vp, vp, ci, ci, vp, vp, vp, ci, ci, vp, ci, vp, vp]
    L.nvq_decode_workspace_bytes.restype = sz
    L.nvq_decode_workspace_bytes.argtypes = [vp, ci, ci, ci]
    L.nvq_decode_linears.argtypes = [vp, ci, ci, ci, vp, sz, vp]
    L.nvq_decode_status.argtypes = [vp, vp, C.POINTER(ci)]
    L.nvq_decode_linears_static.argtypes = [vp, ci, ci, ci, vp]
    L.nvq_plan_create.argtypes = [vp, ci, ci, ci, ci, vp, sz, vp, C.POINTER(vp)]
    L.nvq_plan_run.argtypes = [vp, vp]
    L.nvq_plan_info.argtypes = [vp, C.POINTER(ci), C.POINTER(ci), C.POINTER(ci)]
    L.nvq_plan_status.argtypes = [vp, vp, C.POINTER(ci)]
    L.nvq_plan_trace.argtypes = [vp, vp, sz]
    L.nvq_plan_destroy.argtypes = [vp]
    L.nvq_plan_describe.argtypes = [vp, ci, ci, ci, ci, ci, vp, ci]
    L.nvq_plan_describe_batches.argtypes = [vp, ci, ci, ci, ci, vp, ci]
    L.nvq_plan_describe_skips.argtypes = [vp, ci, ci, ci, ci, ci, vp, sz, vp]
    L.nvq_plan_destroy.restype = None
    L.nvq_precision_from_scores.argtypes = [vp, ci, C.c_double, C.c_double, vp]
    L.nvq_token_norms.argtypes = [vp, ci, vp, ci, ci, ci, vp, vp]
    L.nvq_mcap_scores.argtypes = [vp, vp, vp, ci, ci, vp]
    L.nvq_stream_read.argtypes = [vp, sz, vp, vp]
    L.nvq_stream_copy.argtypes = [vp, vp, sz, vp]
    for f in ("nvq_pack_int4", "nvq_quant_act_i8", "nvq_gemv_w4a16", "nvq_gemv_w4a8",
              "nvq_decode_linears", "nvq_decode_status", "nvq_decode_linears_static",
              "nvq_precision_from_scores", "nvq_stream_read",
              "nvq_stream_copy", "nvq_plan_create", "nvq_plan_run", "nvq_plan_info",
              "nvq_plan_status", "nvq_plan_trace"):
        getattr(L, f).restype = ci
    _lib = L
    return L


def _status_string(status: int) -> str:
    return lib().nvq_status_string(status).decode()


def _check(status: int, what: str):
    if status != 0:
        detail = lib().nvq_last_hip_error().decode() if status == 5 else ""
        raise NvqError(status, what, detail)


def _stream() -> int:
    return torch.cuda.current_stream().cuda_stream


def _dev(t: torch.Tensor, dtype, name: str) -> int:
    if not t.is_cuda:
        raise ValueError("%s must be a device tensor" % name)
    if t.dtype != dtype:
        raise ValueError("%s must be %s, got %s" % (name, dtype, t.dtype))
    if not t.is_contiguous():
        raise ValueError("%s must be contiguous" % name)
    return t.data_ptr()


def _y_dtype(dtype) -> int:
    if dtype == torch.float32:
        return F32
    if dtype == torch.bfloat16:
        return BF16
    raise ValueError("output dtype must be float32 or bfloat16")


# ---- entry points (same names as the C ABI) ----------------------------------
def pack_int4(W: torch.Tensor, group: int = 32):
    """W fp32 [N,K] (device) -> qweight u8 [N,K/2], scales int16 (fp16 bits) [N,K/32]."""
    N, K = W.shape
    q = torch.empty((N, K // 2), dtype=torch.uint8, device=W.device)
    s = torch.empty((N, K // 32), dtype=torch.int16, device=W.device)
    _check(lib().nvq_pack_int4(_dev(W, torch.float32, "W"), N, K, group, q.data_ptr(),
                               s.data_ptr(), _stream()), "nvq_pack_int4")
    return q, s


def dequant_bf16_into(qweight: torch.Tensor, scales: torch.Tensor, out: torch.Tensor):
    """qweight u8 [N,K/2], scales int16 (fp16 bits) [N,K/32] -> dense bf16 weights in out [N,K]."""
    N, K = qweight.shape[0], qweight.shape[1] * 2
    if tuple(out.shape) != (N, K):
        raise ValueError("out: shape mismatch")
    _check(lib().nvq_dequant_bf16(_dev(qweight, torch.uint8, "qweight"),
                                  _dev(scales, torch.int16, "scales"), N, K,
                                  _dev(out, torch.bfloat16, "out"), _stream()), "nvq_dequant_bf16")
    return out


def dequant_bf16(qweight: torch.Tensor, scales: torch.Tensor) -> torch.Tensor:
    N, K = qweight.shape[0], qweight.shape[1] * 2
    return dequant_bf16_into(qweight, scales,
                             torch.empty((N, K), dtype=torch.bfloat16, device=qweight.device))


def rms_norm(x: torch.Tensor, gamma: torch.Tensor, eps: float, res: Optional[torch.Tensor] = None):
    """x, res bf16 [M,K], gamma bf16 [K] -> (out bf16 [M,K], h bf16 [M,K] or None)."""
    M, K = x.shape
    out = torch.empty_like(x)
    h = torch.empty_like(x) if res is not None else None
    _check(lib().nvq_rms_norm_bf16(_dev(x, torch.bfloat16, "x"),
                                   _dev(res, torch.bfloat16, "res") if res is not None else None,
                                   _dev(gamma, torch.bfloat16, "gamma"), float(eps), M, K,
                                   out.data_ptr(), h.data_ptr() if h is not None else None,
                                   _stream()), "nvq_rms_norm_bf16")
    return out, h


def silu_mul(g: torch.Tensor, u: torch.Tensor) -> torch.Tensor:
    """g, u bf16 [M,K] -> bf16(silu(g) * u)."""
    M, K = g.shape
    out = torch.empty_like(g)
    _check(lib().nvq_silu_mul_bf16(_dev(g, torch.bfloat16, "g"), _dev(u, torch.bfloat16, "u"), M, K,
                                   out.data_ptr(), _stream()), "nvq_silu_mul_bf16")
    return out


def quant_act_i8(x: torch.Tensor, act_group: int = 0, out=None):
    """x bf16 [M,K] -> xq i8 [M,K], xscale f32 [M] or [M,K/32], xgsum i32 [M,K/32]
    (`out`: the three tensors to write into, as returned by an earlier call)."""
    M, K = x.shape
    if out is not None:
        xq, xs, gs = out
    else:
        xq = torch.empty((M, K), dtype=torch.int8, device=x.device)
        xs = torch.empty((M,) if act_group == 0 else (M, K // 32), dtype=torch.float32,
                         device=x.device)
        gs = torch.empty((M, K // 32), dtype=torch.int32, device=x.device)
    _check(lib().nvq_quant_act_i8(_dev(x, torch.bfloat16, "x"), M, K, act_group, xq.data_ptr(),
                                  xs.data_ptr(), gs.data_ptr(), _stream()), "nvq_quant_act_i8")
    return xq, xs, gs


def gemv_w4a16(qweight, scales, x, out_dtype=torch.float32, out: Optional[torch.Tensor] = None):
    N, K = qweight.shape[0], qweight.shape[1] * 2
    M = x.shape[0]
    if x.shape[1] != K or tuple(scales.shape) != (N, K // 32):
        raise ValueError("shape mismatch")
    y = out if out is not None else torch.empty((M, N), dtype=out_dtype, device=x.device)
    _check(lib().nvq_gemv_w4a16(_dev(qweight, torch.uint8, "qweight"),
                                _dev(scales, torch.int16, "scales"), N, K,
                                _dev(x, torch.bfloat16, "x"), M, _dev(y, y.dtype, "y"),
                                _y_dtype(y.dtype), _stream()), "nvq_gemv_w4a16")
    return y


def gemm_w4a16(qweight, scales, x, out_dtype=torch.float32, out: Optional[torch.Tensor] = None):
    """Prefill / large-batch product: x bf16 [M,K] -> y [M,N] (weights rounded to bf16)."""
    N, K = qweight.shape[0], qweight.shape[1] * 2
    M = x.shape[0]
    if x.shape[1] != K or tuple(scales.shape) != (N, K // 32):
        raise ValueError("shape mismatch")
    y = out if out is not None else torch.empty((M, N), dtype=out_dtype, device=x.device)
    _check(lib().nvq_gemm_w4a16(_dev(qweight, torch.uint8, "qweight"),
                                _dev(scales, torch.int16, "scales"), N, K,
                                _dev(x, torch.bfloat16, "x"), M, _dev(y, y.dtype, "y"),
                                _y_dtype(y.dtype), _stream()), "nvq_gemm_w4a16")
    return y


def gemv_w4a8(qweight, scales, xq, xscale, xgsum, act_group: int = 0,
              out_dtype=torch.float32, want_acc: bool = False,
              out: Optional[torch.Tensor] = None):
    N, K = qweight.shape[0], qweight.shape[1] * 2
    M = xq.shape[0]
    if xq.shape[1] != K or tuple(scales.shape) != (N, K // 32):
        raise ValueError("shape mismatch")
    y = out if out is not None else torch.empty((M, N), dtype=out_dtype, device=xq.device)
    acc = (torch.empty((M, N, K // 32), dtype=torch.int32, device=xq.device)
           if want_acc else None)
    _check(lib().nvq_gemv_w4a8(_dev(qweight, torch.uint8, "qweight"),
                               _dev(scales, torch.int16, "scales"), N, K,
                               _dev(xq, torch.int8, "xq"), _dev(xscale, torch.float32, "xscale"),
                               _dev(xgsum, torch.int32, "xgsum"), act_group, M,
                               _dev(y, y.dtype, "y"), _y_dtype(y.dtype),
                               acc.data_ptr() if want_acc else None, _stream()),
           "nvq_gemv_w4a8")
    return (y, acc) if want_acc else y


class DecodeList:
    """A host-side `nvq_linear[]` plus the tensors it points to and its workspace."""

    def __init__(self, entries: Sequence[dict], M: int, act_group: int = 0,
                 ordered: bool = False):
        self.M, self.act_group = M, act_group
        self.ordered = ordered
        self.n = len(entries)
        self.arr = (Linear * max(self.n, 1))()
        self.keep: List[torch.Tensor] = []
        dev = None
        for i, e in enumerate(entries):
            q, s, x, y = e["qweight"], e["scales"], e["x"], e["y"]
            N, K = q.shape[0], q.shape[1] * 2
            if tuple(x.shape) != (M, K) or tuple(y.shape) != (M, N):
                raise ValueError("entry %d: shape mismatch" % i)
            op = int(e.get("in_op", IN_PLAIN))
            x2, gamma, h = e.get("x2"), e.get("gamma"), e.get("h_out")
            if x2 is not None and tuple(x2.shape) != (M, K):
                raise ValueError("entry %d: x2 shape mismatch" % i)
            if h is not None and tuple(h.shape) != (M, K):
                raise ValueError("entry %d: h_out shape mismatch" % i)
            if gamma is not None and tuple(gamma.shape) != (K,):
                raise ValueError("entry %d: gamma shape mismatch" % i)
            self.arr[i] = Linear(_dev(q, torch.uint8, "qweight"), _dev(s, torch.int16, "scales"),
                                 N, K, _dev(x, torch.bfloat16, "x"), _dev(y, y.dtype, "y"),
                                 _y_dtype(y.dtype), int(e["precision"]), op,
                                 float(e.get("eps", 0.0)),
                                 _dev(x2, torch.bfloat16, "x2") if x2 is not None else None,
                                 _dev(gamma, torch.bfloat16, "gamma") if gamma is not None else None,
                                 _dev(h, torch.bfloat16, "h_out") if h is not None else None)
            self.keep += [q, s, x, y, x2, gamma, h]
            dev = q.device
        need = lib().nvq_decode_workspace_bytes(C.byref(self.arr), self.n, M, act_group)
        if self.n and need == 0:
            raise NvqError(1, "nvq_decode_workspace_bytes")
        self.workspace = torch.empty(max(need, 256), dtype=torch.uint8, device=dev or "cuda")

    def run(self):
        """One walk through nvq_decode_linears (uploads the phase table each call)."""
        _check(lib().nvq_decode_linears(C.byref(self.arr), self.n, self.M, self.act_group,
                                        self.workspace.data_ptr(), self.workspace.numel(),
                                        _stream()), "nvq_decode_linears")

    def run_static(self):
        """One walk through nvq_decode_linears_static (no workspace, launches only)."""
        _check(lib().nvq_decode_linears_static(C.byref(self.arr), self.n, self.M, self.act_group,
                                               _stream()), "nvq_decode_linears_static")

    def timed_out(self) -> bool:
        """Synchronises; True if a wait inside the last walk on this workspace gave up."""
        t = C.c_int()
        _check(lib().nvq_decode_status(self.workspace.data_ptr(), _stream(), C.byref(t)),
               "nvq_decode_status")
        return bool(t.value)

    # ---- plan: prepared once, run many times ----
    def plan(self):
        if getattr(self, "_plan", None) is None:
            h = C.c_void_p()
            _check(lib().nvq_plan_create(C.byref(self.arr), self.n, self.M, self.act_group,
                                         PLAN_ORDERED if self.ordered else 0,
                                         self.workspace.data_ptr(), self.workspace.numel(),
                                         _stream(), C.byref(h)), "nvq_plan_create")
            self._plan = h
        return self._plan

    def run_plan(self):
        _check(lib().nvq_plan_run(self.plan(), _stream()), "nvq_plan_run")

    def plan_info(self):
        s, p, w = C.c_int(), C.c_int(), C.c_int()
        _check(lib().nvq_plan_info(self.plan(), C.byref(s), C.byref(p), C.byref(w)),
               "nvq_plan_info")
        return {"streaming": s.value == 1, "grouped": s.value in (2, 3),
                "persistent_grouped": s.value == 3, "phases": p.value, "waits": w.value}

    def plan_timed_out(self) -> bool:
        t = C.c_int()
        _check(lib().nvq_plan_status(self.plan(), _stream(), C.byref(t)), "nvq_plan_status")
        self.status_code = t.value      # which wait gave up, and in which phase (see nvq.h)
        return bool(t.value)

    def trace(self, buf: Optional[torch.Tensor]):
        """Attach (or detach with None) an int64 device tensor of phases*8 timestamps."""
        self._trace = buf
        _check(lib().nvq_plan_trace(self.plan(), buf.data_ptr() if buf is not None else None,
                                    buf.numel() * 8 if buf is not None else 0), "nvq_plan_trace")

    def close(self):
        if getattr(self, "_plan", None) is not None:
            lib().nvq_plan_destroy(self._plan)
            self._plan = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


def plan_describe_batches(linears: Sequence[Linear], M: int, ordered: bool = False):
    """Host-side planning of the grouped small-batch launches (no device needed):
    (persistent kernel used, [dict per batch])."""
    n = len(linears)
    arr = (Linear * max(n, 1))(*linears)
    per = 6 + 2 * 9
    words = 2 + max(n, 1) * per
    out = (C.c_int32 * words)()
    _check(lib().nvq_plan_describe_batches(C.byref(arr), n, M, 0, PLAN_ORDERED if ordered else 0,
                                           out, words), "nvq_plan_describe_batches")
    res = []
    for b in range(out[0]):
        o = out[2 + b * per:2 + (b + 1) * per]
        nparts = o[5]
        res.append(dict(first_phase=o[0], last_phase=o[1], units=o[2], jobs=o[3], grid=o[4],
                        parts=nparts, cuts=list(o[6:6 + nparts + 1]),
                        cut_phases=list(o[15:15 + nparts + 1])))
    return bool(out[1]), res


DESCRIBE_FIELDS = ("first", "count", "wait", "publish", "rows", "rows_base", "rows_extra",
                   "rows_rot", "img_lds", "img_need", "img_bytes", "img_prepared", "row_unit",
                   "pair_stream", "spread", "mail")


def plan_describe(linears: Sequence[Linear], M: int, act_group: int = 0, ordered: bool = False,
                  workgroups: int = 256):
    """Host-side planning of a walk (no device needed): (streaming waves or 0, [dict per
    phase]).  `linears` are `Linear` structs; their pointers are compared, never followed."""
    n = len(linears)
    arr = (Linear * max(n, 1))(*linears)
    words = 2 + n * len(DESCRIBE_FIELDS)
    out = (C.c_int32 * words)()
    _check(lib().nvq_plan_describe(C.byref(arr), n, M, act_group, PLAN_ORDERED if ordered else 0,
                                   workgroups, out, words), "nvq_plan_describe")
    k = len(DESCRIBE_FIELDS)
    return int(out[1]), [dict(zip(DESCRIBE_FIELDS, out[2 + p * k:2 + (p + 1) * k]))
                          for p in range(out[0])]


def plan_describe_skips(linears: Sequence[Linear], M: int, act_group: int = 0,
                        ordered: bool = False, workgroups: int = 256):
    """The skip table of the batch-1 persistent kernel (no device needed): a uint8 array
    [workgroups * 13][phases + padding]: rows workgroup * 12 + streaming wave, then one row per
    workgroup; or None."""
    import numpy as np
    n = len(linears)
    arr = (Linear * max(n, 1))(*linears)
    rows = workgroups * 13
    cap = rows * (n + 8)
    out = np.zeros(cap, np.uint8)
    stride = C.c_int(0)
    _check(lib().nvq_plan_describe_skips(C.byref(arr), n, M, act_group,
                                         PLAN_ORDERED if ordered else 0, workgroups,
                                         out.ctypes.data, cap, C.byref(stride)),
           "nvq_plan_describe_skips")
    if stride.value == 0:
        return None
    return out[:rows * stride.value].reshape(rows, stride.value)


def decode_linears(entries: Sequence[dict], M: int, act_group: int = 0) -> DecodeList:
    """Run one walk over `entries` (dicts with qweight, scales, x, y, precision)."""
    dl = DecodeList(entries, M, act_group)
    dl.run()
    return dl


def token_norms(a: torch.Tensor, b: Optional[torch.Tensor] = None) -> torch.Tensor:
    """Per-token Euclidean norm of the rows of a (and b side by side): f32 [M]."""
    M, Na = a.shape
    Nb = 0 if b is None else b.shape[1]
    if b is not None and (b.shape[0] != M or b.dtype != a.dtype):
        raise ValueError("b: shape or dtype mismatch")
    out = torch.empty(M, dtype=torch.float32, device=a.device)
    _check(lib().nvq_token_norms(_dev(a, a.dtype, "a"), Na,
                                 _dev(b, a.dtype, "b") if b is not None else None, Nb, M,
                                 _y_dtype(a.dtype), _dev(out, torch.float32, "out"), _stream()),
           "nvq_token_norms")
    return out


def mcap_scores(a_attn, a_ffn, prompt_len: Sequence[int]):
    """Algorithm 1's score line (host): a_attn, a_ffn float32 [L][T] -> list of L scores."""
    import numpy as np
    aa = np.ascontiguousarray(a_attn, dtype=np.float32)
    af = np.ascontiguousarray(a_ffn, dtype=np.float32)
    if aa.ndim != 2 or aa.shape != af.shape or sum(prompt_len) != aa.shape[1]:
        raise ValueError("shape mismatch")
    pl = (C.c_int * len(prompt_len))(*[int(v) for v in prompt_len])
    out = (C.c_double * aa.shape[0])()
    _check(lib().nvq_mcap_scores(aa.ctypes.data, af.ctypes.data, pl, len(prompt_len), aa.shape[0],
                                 out), "nvq_mcap_scores")
    return list(out)


def precision_from_scores(scores: Sequence[float], tau: float = 0.7, eps: float = 1e-12):
    n = len(scores)
    s = (C.c_double * n)(*[float(v) for v in scores])
    out = (C.c_int32 * n)()
    _check(lib().nvq_precision_from_scores(s, n, tau, eps, out), "nvq_precision_from_scores")
    return list(out)


def stream_read(buf: torch.Tensor, sink: torch.Tensor):
    _check(lib().nvq_stream_read(buf.data_ptr(), buf.numel() * buf.element_size(),
                                 sink.data_ptr(), _stream()), "nvq_stream_read")


def stream_copy(dst: torch.Tensor, src: torch.Tensor):
    _check(lib().nvq_stream_copy(dst.data_ptr(), src.data_ptr(),
                                 src.numel() * src.element_size(), _stream()), "nvq_stream_copy")
