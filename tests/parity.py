"""Acceptance rule for GPU-vs-oracle comparisons (shared by the GPU tests and the smoke check).

A row passes when the GPU index equals the oracle index.  Otherwise it passes only as a
near-tie: the oracle's top-two perturbed scores differ by less than
tol = 1e-3 * (1 + |s_max|) and the oracle's own score of the GPU's pick is within tol of the
maximum.  In every case the GPU's reported value must match the oracle's score of the GPU's
pick to 2e-3 / min(tau, 1) + tol (the per-logit budget of 2e-3, carried through the 1/tau scale).
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Optional, Sequence

import numpy as np


from fs_workloads import to_device_bf16, to_device_seeds  # noqa: F401  (re-exported for the tests)


@dataclass
class Verdict:
    rows: int = 0
    exact: int = 0
    near_ties: int = 0
    failures: list = field(default_factory=list)
    max_val_err: float = 0.0

    @property
    def ok(self) -> bool:
        return not self.failures

    def __str__(self) -> str:
        return (f"rows={self.rows} exact={self.exact} near_ties={self.near_ties} "
                f"failures={len(self.failures)} max_val_err={self.max_val_err:.3g}")


def judge(orc, H, W, tau, gpu_idx, gpu_val, ref, *, seed=0, row_seeds=None, row_ids=None,
          row_offset=0, vocab_offset=0, rows: Optional[Sequence[int]] = None,
          bias=None, allowed_words=None) -> Verdict:
    """ref = oracle.sample(...) over the rows being judged (same order as `rows`, which index
    into H / gpu_idx; default all rows).  row_ids gives the global row word per judged row."""
    B = H.shape[0]
    rows = list(range(B)) if rows is None else list(rows)
    v = Verdict()
    for k, b in enumerate(rows):
        v.rows += 1
        s1, s2 = float(ref["top1"][k]), float(ref["top2"][k])
        i1 = int(ref["idx"][k])
        gi, gv = int(gpu_idx[b]), float(gpu_val[b])
        tol = 1e-3 * (1.0 + abs(s1)) if np.isfinite(s1) else 0.0
        t = float(tau[b])
        seed_b = int(row_seeds[b]) if row_seeds is not None else int(seed)
        row_word = int(row_ids[k]) if row_ids is not None else row_offset + b
        if i1 < 0:   # nothing finite in this row: both must say so
            if gi != -1 or gv != -np.inf:
                v.failures.append((b, "expected idx -1 / -inf", gi, gv))
            else:
                v.exact += 1
            continue
        if gi < vocab_offset or gi >= vocab_offset + W.shape[0]:
            v.failures.append((b, "index out of range", gi, gv))
            continue
        if bias is None and allowed_words is None:
            s_pick = orc.score_at(H, W, b, gi - vocab_offset, t, seed_b, row_word, gi)
        else:   # full transform: (y + bias) / tau, -inf when the id is masked for this row
            arow = None if allowed_words is None else (allowed_words if allowed_words.ndim == 1 else allowed_words[b])
            s_pick = orc.score_at_full(H, W, b, gi - vocab_offset, t, seed_b, row_word, gi, bias=bias,
                                       allowed_row=arow)
        val_tol = 2e-3 / min(t, 1.0) + tol
        err = abs(gv - s_pick)
        v.max_val_err = max(v.max_val_err, err)
        if not err <= val_tol:
            v.failures.append((b, "value mismatch", gi, gv, s_pick, val_tol))
            continue
        if gi == i1:
            v.exact += 1
        elif (s1 - s2) < tol and (s1 - s_pick) < tol:
            v.near_ties += 1
        else:
            v.failures.append((b, "wrong index", gi, i1, s1, s2, s_pick, tol))
    return v
