"""Seeded synthetic inputs for the decode-linear workloads.

This module holds input generation only: shapes, random draws, the outlier
recipe, the precision-map draw.  None of the method's arithmetic (no
quantisation, no packing, no dot products) lives here, so the CPU oracle's
tests and the GPU path's tests can both use it without sharing any of the
code under test.  The real Llama checkpoints behind the paper's throughput
table are not available; layers of the same shapes with N(0, 0.02) weights
and N(0, 1) activations (1% of channels scaled by 20) stand in for them.
"""
from dataclasses import dataclass
from typing import Dict, List, Tuple

import torch

BASE_SEED = 20260421

# name -> (n_blocks, hidden, kv_dim, ffn, vocab or 0).  Shapes are written
# K -> N: q/o hidden->hidden, k/v hidden->kv_dim, gate/up hidden->ffn,
# down ffn->hidden.
MODELS: Dict[str, Tuple[int, int, int, int, int]] = {
    "llama-1b": (16, 2048, 512, 8192, 0),
    "llama-3b": (28, 3072, 1024, 8192, 0),
    "llama-8b": (32, 4096, 1024, 14336, 128256),
}

SLOTS = ("q", "k", "v", "o", "gate", "up", "down")


@dataclass
class LinearSpec:
    name: str
    block: int          # transformer block index; -1 for lm_head
    slot: int           # index into SLOTS; 7 for lm_head
    N: int
    K: int
    phase: int          # entries with equal phase read the same input


def model_linears(model: str, with_lm_head: bool = None) -> List[LinearSpec]:
    """The ordered list of linears of one decode step.  Phases per block:
    (q,k,v) share an input, o, (gate,up) share an input, down."""
    nb, h, kv, ffn, vocab = MODELS[model]
    if with_lm_head is None:
        with_lm_head = vocab > 0
    out: List[LinearSpec] = []
    ph = 0
    for b in range(nb):
        for slot, (N, K, dph) in enumerate([(h, h, 0), (kv, h, 0), (kv, h, 0), (h, h, 1),
                                             (ffn, h, 2), (ffn, h, 2), (h, ffn, 3)]):
            out.append(LinearSpec("blk%d.%s" % (b, SLOTS[slot]), b, slot, N, K, ph + dph))
        ph += 4
    if with_lm_head and vocab:
        out.append(LinearSpec("lm_head", -1, 7, vocab, h, ph))
    return out


def weight_bytes(N: int, K: int) -> int:
    """Packed size: 4-bit codes plus one 16-bit scale per 32 weights."""
    return N * K // 2 + N * (K // 32) * 2


def _gen(seed: int, device) -> torch.Generator:
    g = torch.Generator(device=device)
    g.manual_seed(int(seed))
    return g


def make_weight(seed: int, N: int, K: int, device="cpu", sigma: float = 0.02) -> torch.Tensor:
    """fp32 [N, K] ~ N(0, sigma)."""
    w = torch.randn((N, K), generator=_gen(seed, device), device=device, dtype=torch.float32)
    return w.mul_(sigma)


def outlier_channels(K: int, seed: int = BASE_SEED) -> torch.Tensor:
    """floor(0.01 K) channel indices, one fixed set per K."""
    n = K // 100
    perm = torch.randperm(K, generator=_gen(seed + 700_000 + K, "cpu"))
    return perm[:n].sort().values


def make_activation(seed: int, M: int, K: int, outliers: bool = True, device="cpu") -> torch.Tensor:
    """bf16 [M, K] ~ N(0, 1); with outliers, 1% of channels are scaled by 20."""
    x = torch.randn((M, K), generator=_gen(seed, "cpu"), dtype=torch.float32)
    if outliers:
        idx = outlier_channels(K)
        x[:, idx] *= 20.0
    return x.to(torch.bfloat16).to(device)


def make_precision_map(n_blocks: int, n_w4a16: int, seed: int = BASE_SEED) -> List[int]:
    """Per-block precision bits with exactly n_w4a16 blocks set to 1 (W4A16)."""
    perm = torch.randperm(n_blocks, generator=_gen(seed + 900_000, "cpu"))
    bits = [0] * n_blocks
    for i in perm[:n_w4a16].tolist():
        bits[i] = 1
    return bits


def tensor_seed(block: int, slot: int, seed: int = BASE_SEED) -> int:
    return seed + 1000 * (block + 1) + slot


def activation_seed(phase: int, seed: int = BASE_SEED) -> int:
    return seed + 500_000 + phase


def bf16_bits(x: torch.Tensor) -> torch.Tensor:
    """Reinterpret a bf16 tensor as int16 bit patterns (no arithmetic)."""
    return x.view(torch.int16)
