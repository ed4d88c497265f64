"""Byte and element counts of one call (measurement arithmetic for ``bench.py`` and the tests; no
part of the library or of the oracle)."""
from __future__ import annotations

VOCAB_TILE = 128     # vocabulary ids per stage-1 candidate
LOGITS_CHUNK = 1024  # ids per workgroup of the stand-alone Gumbel-max kernel of the unfused path


def io_model_bytes(B: int, D: int, V: int, fused: bool = True, w_bytes_per_row: int | None = None) -> int:
    """Algorithmic HBM bytes of one call (the paper's IO cost model, Section "IO Cost Model and
    Predicted Speedup", in bytes: bf16 W and H, fp32 logits, 8-byte candidates and outputs).
    fused:    2 V D + 2 B D + 2 * 8 B T + 8 B
    unfused:  2 V D + 2 B D + 2 * 4 B V + 2 * 8 B TC + 8 B      (TC = ceil(V / 1024))
    w_bytes_per_row replaces 2 D for lower-precision weights."""
    T = (V + VOCAB_TILE - 1) // VOCAB_TILE
    wrow = 2 * D if w_bytes_per_row is None else w_bytes_per_row
    base = V * wrow + 2 * B * D + 8 * B
    if fused:
        return base + 2 * 8 * B * T
    TC = (V + LOGITS_CHUNK - 1) // LOGITS_CHUNK
    return base + 2 * 4 * B * V + 2 * 8 * B * TC


def stage1_bytes(B: int, D: int, V: int, w_bytes_per_row: int | None = None) -> int:
    """Algorithmic bytes of one stage-1 launch: W once, H once, candidates written."""
    T = (V + VOCAB_TILE - 1) // VOCAB_TILE
    wrow = 2 * D if w_bytes_per_row is None else w_bytes_per_row
    return V * wrow + 2 * B * D + 8 * B * T


def io_model_speedup_elements(B: int, D: int, V: int) -> float:
    """M_baseline / M_fused of the paper's IO cost model, in element counts as printed there:
    (VD + DB + 2VB + B) / (VD + DB + B)."""
    return (V * D + D * B + 2 * V * B + B) / (V * D + D * B + B)
