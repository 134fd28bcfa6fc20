"""Independent numpy helpers used only to pin the oracle (never as expected
values for the GPU path: those come from oracle/ alone).  They restate the
packed layout with array operations instead of the oracle's scalar loops, so a
wrong index or nibble order in the oracle shows up as a disagreement."""
import numpy as np


def unpack_codes(qweight: np.ndarray) -> np.ndarray:
    """u8 [N, K/2] -> signed codes int32 [N, K] (layout: byte g*16+j holds
    element 32g+j in its low nibble and element 32g+16+j in its high nibble)."""
    N, half = qweight.shape
    G = half // 16
    b = qweight.reshape(N, G, 16).astype(np.int32)
    lo = (b & 15) - 8
    hi = (b >> 4) - 8
    return np.concatenate([lo, hi], axis=2).reshape(N, G * 32)


def half_bits_to_f64(bits: np.ndarray) -> np.ndarray:
    return bits.astype(np.uint16).view(np.float16).astype(np.float64)


def bf16_bits_to_f64(bits: np.ndarray) -> np.ndarray:
    u = bits.astype(np.uint16).astype(np.uint32) << 16
    return u.view(np.float32).astype(np.float64)


def dequant(qweight: np.ndarray, scales: np.ndarray) -> np.ndarray:
    codes = unpack_codes(qweight).astype(np.float64)
    s = half_bits_to_f64(scales)
    return codes * np.repeat(s, 32, axis=1)


def rel_l2(a: np.ndarray, b: np.ndarray) -> float:
    a = np.asarray(a, np.float64).ravel()
    b = np.asarray(b, np.float64).ravel()
    d = np.linalg.norm(a - b)
    n = np.linalg.norm(b)
    return float(d / n) if n > 0 else float(d)
