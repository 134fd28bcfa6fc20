"""ctypes front end of the CPU oracle (oracle/nvq_oracle.c).

TEST INFRASTRUCTURE ONLY: imported by tests/, the smoke check and the
benchmark's cpu_baseline leg.  It never imports the GPU package, and the GPU
package never imports it.  Arrays are numpy; bf16 and fp16 values travel as
uint16 bit patterns.
"""
import ctypes as C
import os

import numpy as np

from . import build as _build

_lib = None


class OracleError(RuntimeError):
    pass


class _Linear(C.Structure):
    _fields_ = [("qweight", C.c_void_p), ("scales", C.c_void_p),
                ("N", C.c_int64), ("K", C.c_int64),
                ("x", C.c_void_p), ("y", C.c_void_p), ("precision", C.c_int),
                ("in_op", C.c_int), ("x2", C.c_void_p), ("gamma", C.c_void_p),
                ("eps", C.c_double), ("h_out", C.c_void_p), ("xt", C.c_void_p)]


IN_PLAIN, IN_RMSNORM, IN_SILU_MUL = 0, 1, 2


def lib():
    global _lib
    if _lib is None:
        path = _build.build()
        L = C.CDLL(path)
        L.orc_bf16_to_float.restype = C.c_float
        L.orc_bf16_to_float.argtypes = [C.c_uint16]
        L.orc_float_to_bf16.restype = C.c_uint16
        L.orc_float_to_bf16.argtypes = [C.c_float]
        L.orc_half_to_float.restype = C.c_float
        L.orc_half_to_float.argtypes = [C.c_uint16]
        L.orc_float_to_half.restype = C.c_uint16
        L.orc_float_to_half.argtypes = [C.c_float]
        vp, i64, ci = C.c_void_p, C.c_int64, C.c_int
        L.orc_pack_int4.argtypes = [vp, i64, i64, vp, vp]
        L.orc_dequant_int4.argtypes = [vp, vp, i64, i64, vp]
        L.orc_dequant_bf16.argtypes = [vp, vp, i64, i64, vp]
        L.orc_dequant_bf16.restype = C.c_int
        L.orc_quant_act_i8.argtypes = [vp, i64, i64, ci, vp, vp, vp]
        L.orc_gemv_w4a8.argtypes = [vp, vp, i64, i64, vp, vp, ci, i64, vp, vp]
        L.orc_w4a8_acc_deferred.argtypes = [vp, i64, i64, vp, vp, i64, vp]
        L.orc_gemv_w4a16.argtypes = [vp, vp, i64, i64, vp, i64, vp]
        L.orc_decode_linears.argtypes = [vp, i64, i64, ci, vp, vp]
        L.orc_double_to_bf16.restype = C.c_uint16
        L.orc_double_to_bf16.argtypes = [C.c_double]
        L.orc_rms_norm.argtypes = [vp, vp, vp, C.c_double, i64, i64, vp, vp]
        L.orc_rms_norm.restype = C.c_int
        L.orc_silu_mul.argtypes = [vp, vp, i64, i64, vp]
        L.orc_silu_mul.restype = C.c_int
        L.orc_precision_from_scores.argtypes = [vp, i64, C.c_double, C.c_double, vp, vp]
        L.orc_token_norms.argtypes = [vp, i64, vp, i64, i64, ci, vp]
        L.orc_token_norms.restype = C.c_int
        L.orc_mcap_scores.argtypes = [vp, vp, vp, i64, i64, vp]
        L.orc_mcap_scores.restype = C.c_int
        for f in ("orc_pack_int4", "orc_dequant_int4", "orc_quant_act_i8", "orc_gemv_w4a8",
                  "orc_w4a8_acc_deferred", "orc_gemv_w4a16", "orc_decode_linears",
                  "orc_precision_from_scores"):
            getattr(L, f).restype = C.c_int
        _lib = L
    return _lib


def _p(a):
    return a.ctypes.data_as(C.c_void_p)


def _chk(rc, what):
    if rc != 0:
        raise OracleError("%s failed with oracle status %d" % (what, rc))


def _arr(a, dtype, ndim=None):
    a = np.ascontiguousarray(a, dtype=dtype)
    if ndim is not None and a.ndim != ndim:
        raise ValueError("expected %d-d array" % ndim)
    return a


# ---- number formats --------------------------------------------------------
def half_to_float(bits):
    return lib().orc_half_to_float(int(bits))


def float_to_half(f):
    return lib().orc_float_to_half(float(np.float32(f)))


def bf16_to_float(bits):
    return lib().orc_bf16_to_float(int(bits))


def float_to_bf16(f):
    return lib().orc_float_to_bf16(float(np.float32(f)))


# ---- the path ---------------------------------------------------------------
def pack_int4(W, allow_range_error=False):
    """W fp32 [N,K] -> (qweight u8 [N,K/2], scales u16 [N,K/32])."""
    W = _arr(W, np.float32, 2)
    N, K = W.shape
    q = np.empty((N, K // 2), np.uint8)
    s = np.empty((N, K // 32), np.uint16)
    rc = lib().orc_pack_int4(_p(W), N, K, _p(q), _p(s))
    if not (allow_range_error and rc == 3):
        _chk(rc, "pack_int4")
    return q, s


def dequant_int4(qweight, scales):
    """-> float64 [N,K] with Wd = code * scale."""
    q = _arr(qweight, np.uint8, 2)
    s = _arr(scales, np.uint16, 2)
    N, K = q.shape[0], q.shape[1] * 2
    Wd = np.empty((N, K), np.float64)
    _chk(lib().orc_dequant_int4(_p(q), _p(s), N, K, _p(Wd)), "dequant_int4")
    return Wd


def dequant_bf16(qweight, scales):
    """-> uint16 (bf16 bits) [N,K] with value bf16_rne(code * scale)."""
    q = _arr(qweight, np.uint8, 2)
    s = _arr(scales, np.uint16, 2)
    N, K = q.shape[0], q.shape[1] * 2
    out = np.empty((N, K), np.uint16)
    _chk(lib().orc_dequant_bf16(_p(q), _p(s), N, K, _p(out)), "dequant_bf16")
    return out


def gemm_w4a16_dense(qweight, scales, x_bf16):
    """Prefill / large-batch product (paper: kernel table, the weights are dequantised to 16-bit
    values and a dense GEMM follows): Y = X * Wd^T with Wd the bf16 weights of dequant_bf16 and
    X the bf16 activations [M,K]; every product is exact in float64, the sum is float64.
    -> float64 [M,N]."""
    wd = dequant_bf16(qweight, scales).astype(np.uint32) << 16
    x = _arr(x_bf16, np.uint16, 2).astype(np.uint32) << 16
    return x.view(np.float32).astype(np.float64) @ wd.view(np.float32).astype(np.float64).T


def quant_act_i8(x_bf16, act_group=0):
    """x u16(bf16 bits) [M,K] -> (xq i8 [M,K], xscale f32 [M] or [M,K/32], xgsum i32 [M,K/32])."""
    x = _arr(x_bf16, np.uint16, 2)
    M, K = x.shape
    xq = np.empty((M, K), np.int8)
    xs = np.empty((M,) if act_group == 0 else (M, K // 32), np.float32)
    gs = np.empty((M, K // 32), np.int32)
    _chk(lib().orc_quant_act_i8(_p(x), M, K, act_group, _p(xq), _p(xs), _p(gs)), "quant_act_i8")
    return xq, xs, gs


def gemv_w4a8(qweight, scales, xq, xscale, act_group=0, want_acc=False):
    """-> y float64 [M,N] (and acc int32 [M,N,K/32])."""
    q = _arr(qweight, np.uint8, 2)
    s = _arr(scales, np.uint16, 2)
    xq = _arr(xq, np.int8, 2)
    xs = _arr(xscale, np.float32)
    N, K = q.shape[0], q.shape[1] * 2
    M = xq.shape[0]
    assert xq.shape[1] == K and s.shape == (N, K // 32)
    y = np.empty((M, N), np.float64)
    acc = np.empty((M, N, K // 32), np.int32) if want_acc else None
    _chk(lib().orc_gemv_w4a8(_p(q), _p(s), N, K, _p(xq), _p(xs), act_group, M, _p(y),
                             _p(acc) if want_acc else None), "gemv_w4a8")
    return (y, acc) if want_acc else y


def w4a8_acc_deferred(qweight, xq, xgsum):
    q = _arr(qweight, np.uint8, 2)
    xq = _arr(xq, np.int8, 2)
    gs = _arr(xgsum, np.int32, 2)
    N, K = q.shape[0], q.shape[1] * 2
    M = xq.shape[0]
    acc = np.empty((M, N, K // 32), np.int32)
    _chk(lib().orc_w4a8_acc_deferred(_p(q), N, K, _p(xq), _p(gs), M, _p(acc)), "w4a8_acc_deferred")
    return acc


def gemv_w4a16(qweight, scales, x_bf16):
    """-> y float64 [M,N]."""
    q = _arr(qweight, np.uint8, 2)
    s = _arr(scales, np.uint16, 2)
    x = _arr(x_bf16, np.uint16, 2)
    N, K = q.shape[0], q.shape[1] * 2
    M = x.shape[0]
    assert x.shape[1] == K and s.shape == (N, K // 32)
    y = np.empty((M, N), np.float64)
    _chk(lib().orc_gemv_w4a16(_p(q), _p(s), N, K, _p(x), M, _p(y)), "gemv_w4a16")
    return y


def rms_norm(x_bf16, gamma_bf16, eps, res_bf16=None):
    """x, res u16(bf16) [M,K], gamma u16 [K] -> (out u16 [M,K], h u16 [M,K] or None):
    out = bf16(h * gamma / sqrt(mean(h^2) + eps)), h = bf16(x + res) (or x)."""
    x = _arr(x_bf16, np.uint16, 2)
    g = _arr(gamma_bf16, np.uint16, 1)
    M, K = x.shape
    assert g.shape == (K,)
    out = np.empty((M, K), np.uint16)
    r = h = None
    if res_bf16 is not None:
        r = _arr(res_bf16, np.uint16, 2)
        assert r.shape == (M, K)
        h = np.empty((M, K), np.uint16)
    _chk(lib().orc_rms_norm(_p(x), _p(r) if r is not None else None, _p(g), float(eps), M, K,
                            _p(out), _p(h) if h is not None else None), "rms_norm")
    return out, h


def silu_mul(g_bf16, u_bf16):
    """g, u u16(bf16) [M,K] -> u16 [M,K]: bf16(silu(g) * u)."""
    g = _arr(g_bf16, np.uint16, 2)
    u = _arr(u_bf16, np.uint16, 2)
    assert g.shape == u.shape
    out = np.empty(g.shape, np.uint16)
    _chk(lib().orc_silu_mul(_p(g), _p(u), g.shape[0], g.shape[1], _p(out)), "silu_mul")
    return out


def decode_linears(layers, M, act_group=0):
    """layers: list of dicts {qweight, scales, x, precision[, in_op, x2, gamma, eps]};
    returns list of y float64 [M,N].  With in_op the layer's input is first transformed
    (IN_RMSNORM: rms_norm(x, gamma, eps, res=x2); IN_SILU_MUL: silu_mul(x, x2)); an entry dict
    with in_op IN_RMSNORM and x2 receives the key "h" (u16 [M,K]) = bf16(x + x2)."""
    n = len(layers)
    arr = (_Linear * max(n, 1))()
    keep = []
    ys = []
    maxK = 32
    for i, L in enumerate(layers):
        q = _arr(L["qweight"], np.uint8, 2)
        s = _arr(L["scales"], np.uint16, 2)
        x = _arr(L["x"], np.uint16, 2)
        N, K = q.shape[0], q.shape[1] * 2
        assert x.shape == (M, K)
        y = np.empty((M, N), np.float64)
        keep += [q, s, x]
        ys.append(y)
        maxK = max(maxK, K)
        op = int(L.get("in_op", 0))
        x2 = g = h = xt = None
        if op != 0:
            xt = np.empty((M, K), np.uint16)
            if L.get("x2") is not None:
                x2 = _arr(L["x2"], np.uint16, 2)
                assert x2.shape == (M, K)
            if op == IN_RMSNORM:
                g = _arr(L["gamma"], np.uint16, 1)
                assert g.shape == (K,)
                if x2 is not None:
                    h = np.empty((M, K), np.uint16)
                    L["h"] = h
            keep += [xt, x2, g, h]
        ptr = lambda a: a.ctypes.data if a is not None else None
        arr[i] = _Linear(q.ctypes.data, s.ctypes.data, N, K, x.ctypes.data, y.ctypes.data,
                         int(L["precision"]), op, ptr(x2), ptr(g), float(L.get("eps", 0.0)),
                         ptr(h), ptr(xt))
    sq = np.empty(M * maxK, np.int8)
    ss = np.empty(M * maxK // 32, np.float32)
    _chk(lib().orc_decode_linears(C.byref(arr), n, M, act_group, _p(sq), _p(ss)), "decode_linears")
    return ys


def token_norms(a, b=None):
    """Per-token Euclidean norm of the rows of a [M,Na] (float32, or uint16 = bf16 bits), with
    the rows of b [M,Nb] appended if given (Algorithm 1's magnitudes).  -> float64 [M]."""
    dt = 1 if np.asarray(a).dtype == np.uint16 else 0
    a = _arr(a, np.uint16 if dt else np.float32, 2)
    M, Na = a.shape
    Nb = 0
    if b is not None:
        b = _arr(b, np.uint16 if dt else np.float32, 2)
        Nb = b.shape[1]
    out = np.empty(M, np.float64)
    _chk(lib().orc_token_norms(_p(a), Na, _p(b) if b is not None else None, Nb, M, dt, _p(out)),
         "token_norms")
    return out


def mcap_scores(a_attn, a_ffn, prompt_len):
    """Algorithm 1's score line.  a_attn, a_ffn float64 [L,T], prompt_len ints summing to T."""
    aa = _arr(a_attn, np.float64, 2)
    af = _arr(a_ffn, np.float64, 2)
    pl = _arr(prompt_len, np.int64, 1)
    s = np.empty(aa.shape[0], np.float64)
    _chk(lib().orc_mcap_scores(_p(aa), _p(af), _p(pl), pl.shape[0], aa.shape[0], _p(s)),
         "mcap_scores")
    return s


def precision_from_scores(scores, tau=0.7, eps=1e-12):
    """-> (uint8 [L]: 1 = W4A16, 0 = W4A8; normalised scores float64 [L])."""
    s = _arr(scores, np.float64, 1)
    out = np.empty(s.shape[0], np.uint8)
    shat = np.empty(s.shape[0], np.float64)
    _chk(lib().orc_precision_from_scores(_p(s), s.shape[0], tau, eps, _p(out), _p(shat)),
         "precision_from_scores")
    return out, shat
