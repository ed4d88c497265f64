"""Seeded synthetic inputs for the fused LM-head + Gumbel-max sampling path.

This module only *makes inputs*: bf16 hidden states, bf16 LM-head weights,
per-row temperatures and per-row seeds, at the shapes and value distributions of
the workload configurations (random bf16 tensors at model shapes, as in the
paper's kernel microbenchmarks, Section "Setup").  It contains none of the
method's arithmetic (no matmul, no Philox, no Gumbel transform, no argmax), so it
can serve both the CPU oracle and the HIP path without coupling them.

Every array is a pure function of (config name, B): the generator is numpy's
SeedSequence-keyed PCG64, drawn in fixed-size row chunks so the result does not
depend on how many threads filled it.

bf16 values are carried as ``numpy.uint16`` bit patterns (numpy has no bf16).
"""
from __future__ import annotations

from concurrent.futures import ThreadPoolExecutor
from dataclasses import dataclass, field
from typing import Optional, Sequence

import numpy as np

_CHUNK_ROWS = 1024  # rows per independently seeded chunk (fixed: part of the recipe)
_TAG_H, _TAG_W, _TAG_TAU = 1, 2, 3


@dataclass(frozen=True)
class Workload:
    """One workload configuration (shapes, value recipe, temperatures, seeds)."""

    name: str
    D: int
    V: int
    batch_sizes: Sequence[int]
    data_seed: int
    w_row_scale: float = 1.0          # W ~ N(0, w_row_scale^2 / D)
    tau_mode: str = "const"           # "const" | "uniform" | "cycle"
    tau_values: Sequence[float] = (1.0,)
    per_row_seeds: bool = False       # row b draws with seed b (else one seed for all rows)
    seed: int = 0
    vocab_tile: int = 128
    note: str = ""
    extra: dict = field(default_factory=dict)


WORKLOADS = {
    # B=1, tiny: the oracle finishes in well under a second.
    "C1": Workload("C1", D=256, V=4096, batch_sizes=(1,), data_seed=1001,
                   note="tiny: hidden ~N(0,1), W ~N(0,1/D), tau=1, seed 0, vocab tile 128"),
    # Llama-3-8B-shaped LM head, bandwidth-bound decode regime.
    "C2": Workload("C2", D=4096, V=128256, batch_sizes=(1, 2, 4, 8, 16), data_seed=1002,
                   per_row_seeds=True, note="Llama-3-8B-shaped LM head, tau=1, per-row seeds"),
    # Qwen-style large vocabulary, per-row temperature U[0.5, 1.5].
    "C3": Workload("C3", D=3584, V=152064, batch_sizes=(32, 64, 128), data_seed=1003,
                   tau_mode="uniform", tau_values=(0.5, 1.5), per_row_seeds=True,
                   note="Qwen-style vocab, tau ~ U[0.5,1.5], seeds 0..B-1"),
    # Compute-leaning, peaky logits (std ~ 4), many near-ties.
    "C4": Workload("C4", D=8192, V=128256, batch_sizes=(256,), data_seed=1004,
                   w_row_scale=4.0, tau_values=(0.7,),
                   note="W rows scaled x4 so logits have std ~4; tau=0.7"),
    # Wide hidden sweep with cycled temperatures.
    "C5": Workload("C5", D=7168, V=129280, batch_sizes=(1, 8, 64, 256, 512), data_seed=1005,
                   tau_mode="cycle", tau_values=(0.3, 1.0, 2.0),
                   note="wide hidden sweep; tau cycled {0.3,1,2} by row"),
}


def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round float32 to bfloat16 (round-to-nearest-even); returns uint16 bit patterns."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    bits = x.view(np.uint32)
    rounding = ((bits >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF)
    return ((bits + rounding) >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(bits: np.ndarray) -> np.ndarray:
    """Widen bf16 bit patterns (uint16) to float32 exactly."""
    b = np.ascontiguousarray(bits, dtype=np.uint16).astype(np.uint32) << np.uint32(16)
    return b.view(np.float32)


def _normal_bf16(rows: int, cols: int, std: float, seed_words: Sequence[int],
                 threads: int = 8) -> np.ndarray:
    """[rows, cols] bf16 bits of N(0, std^2), chunk c seeded by (seed_words..., c)."""
    out = np.empty((rows, cols), dtype=np.uint16)
    nchunks = (rows + _CHUNK_ROWS - 1) // _CHUNK_ROWS

    def fill(c: int) -> None:
        r0 = c * _CHUNK_ROWS
        r1 = min(rows, r0 + _CHUNK_ROWS)
        rng = np.random.default_rng([int(s) for s in seed_words] + [c])
        x = rng.standard_normal((r1 - r0, cols), dtype=np.float32)
        if std != 1.0:
            x *= np.float32(std)
        out[r0:r1] = f32_to_bf16_bits(x)

    if nchunks <= 1 or threads <= 1:
        for c in range(nchunks):
            fill(c)
    else:
        with ThreadPoolExecutor(max_workers=threads) as ex:
            list(ex.map(fill, range(nchunks)))
    return out


def make_hidden(wl: Workload, B: int) -> np.ndarray:
    """Hidden states H [B, D], bf16 bits, ~N(0,1).  Row b is the same for every B."""
    return _normal_bf16(B, wl.D, 1.0, (wl.data_seed, _TAG_H))


def make_weights(wl: Workload, V: Optional[int] = None, threads: int = 8) -> np.ndarray:
    """LM-head weights W [V, D], bf16 bits, ~N(0, w_row_scale^2 / D)."""
    V = wl.V if V is None else V
    std = wl.w_row_scale / float(np.sqrt(wl.D))
    return _normal_bf16(V, wl.D, std, (wl.data_seed, _TAG_W), threads=threads)


def make_temperature(wl: Workload, B: int) -> np.ndarray:
    """Per-row temperature [B] float32."""
    if wl.tau_mode == "const":
        return np.full(B, wl.tau_values[0], dtype=np.float32)
    if wl.tau_mode == "uniform":
        lo, hi = wl.tau_values
        rng = np.random.default_rng([wl.data_seed, _TAG_TAU])
        return rng.uniform(lo, hi, size=B).astype(np.float32)
    if wl.tau_mode == "cycle":
        vals = np.asarray(wl.tau_values, dtype=np.float32)
        return vals[np.arange(B) % len(vals)]
    raise ValueError(wl.tau_mode)


def make_row_seeds(wl: Workload, B: int) -> Optional[np.ndarray]:
    """Per-row 64-bit seeds (row b -> seed b) or None when the config uses one seed."""
    if not wl.per_row_seeds:
        return None
    return np.arange(B, dtype=np.uint64)


def make_small(D: int, V: int, B: int, data_seed: int, w_row_scale: float = 1.0):
    """Ad-hoc small case (H, W) with the same value recipe, for tile/ragged-shape tests."""
    H = _normal_bf16(B, D, 1.0, (data_seed, _TAG_H), threads=1)
    W = _normal_bf16(V, D, w_row_scale / float(np.sqrt(D)), (data_seed, _TAG_W), threads=1)
    return H, W


def quantize_e4m3(W_bits: np.ndarray):
    """Input preparation for the FP8-weight path: bf16 weights [V, D] -> (codes uint8 [V, D],
    scale float32 [V]) with one scale per row, scale = max|w| / 448 (448 = largest E4M3 value) and
    round-to-nearest-even onto the OCP E4M3 grid.  The rounding is torch's float8_e4m3fn cast."""
    import torch
    Wf = torch.from_numpy(bf16_bits_to_f32(W_bits))
    amax = Wf.abs().amax(dim=1).clamp_min(1e-30)
    scale = (amax / 448.0).to(torch.float32)
    q = (Wf / scale[:, None]).clamp(-448.0, 448.0).to(torch.float8_e4m3fn)
    return q.view(torch.uint8).numpy().copy(), scale.numpy().copy()


def quantize_mxfp4(W_bits: np.ndarray):
    """Input preparation for the MXFP4-weight path: bf16 weights [V, D] (D % 32 == 0) ->
    (codes uint8 [V, D/2], two E2M1 codes per byte with the even element in the low nibble;
    scales uint8 [V, D/32], E8M0).  Per block of 32: scale exponent = floor(log2(max|w|)) - 2 (the
    largest E2M1 magnitude is 6 = 1.5 * 2^2), elements rounded to the nearest E2M1 magnitude
    (ties to the even code), saturating at 6."""
    V, D = W_bits.shape
    assert D % 32 == 0
    grid = np.array([0.0, 0.5, 1.0, 1.5, 2.0, 3.0, 4.0, 6.0], dtype=np.float32)
    mid = (grid[:-1] + grid[1:]) / 2          # decision points between neighbouring magnitudes
    packed = np.empty((V, D // 2), dtype=np.uint8)
    scales = np.empty((V, D // 32), dtype=np.uint8)
    for r0 in range(0, V, 2048):              # row chunks keep the temporaries small
        Wf = bf16_bits_to_f32(W_bits[r0:r0 + 2048])
        rows = Wf.shape[0]
        blocks = Wf.reshape(rows, D // 32, 32)
        amax = np.abs(blocks).max(axis=2)
        exp = np.where(amax > 0, np.floor(np.log2(np.where(amax > 0, amax, 1.0))) - 2, -127.0)
        exp = np.clip(exp, -127, 125).astype(np.float32)
        scaled = (np.abs(blocks) / np.exp2(exp)[:, :, None]).astype(np.float32)
        # nearest magnitude; a value exactly on a decision point goes to the even code
        code = np.searchsorted(mid, scaled.reshape(-1), side="left").astype(np.uint8)
        on_mid = code < 7
        on_mid &= scaled.reshape(-1) == mid[np.minimum(code, 6)]
        code = np.where(on_mid & (code % 2 == 1), code + 1, code).astype(np.uint8)
        code = code.reshape(rows, D)
        code |= (Wf < 0).astype(np.uint8) << 3
        packed[r0:r0 + rows] = code[:, 0::2] | (code[:, 1::2] << 4)
        scales[r0:r0 + rows] = (exp + 127).astype(np.uint8)
    return packed, scales


def to_device_bf16(bits: np.ndarray):
    """bf16 bit patterns (uint16) -> torch.bfloat16 tensor on the current GPU (a plain upload)."""
    import torch
    return torch.from_numpy(np.ascontiguousarray(bits).view(np.int16)).view(torch.bfloat16).cuda()


def to_device_seeds(seeds: Optional[np.ndarray]):
    """uint64 seeds -> device tensor carrying the same 64-bit patterns (torch has no uint64 math)."""
    import torch
    if seeds is None:
        return None
    return torch.from_numpy(np.ascontiguousarray(seeds, dtype=np.uint64).view(np.int64)).cuda()
