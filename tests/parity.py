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
          bias=None, allowed_words=None, w8_scale=False, w4_scales=None) -> Verdict:
    """w8_scale: not False when W holds FP8 (E4M3) codes; then it is the per-row scale array or None.
    w4_scales: the E8M0 scale bytes when W holds MXFP4 codes.
    ref = oracle.sample(...) over the rows being judged (same order as `rows`, which index
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
        if gi < vocab_offset or gi >= vocab_offset + W.shape[0]:   # W.shape[0] = V for every weight format
            v.failures.append((b, "index out of range", gi, gv))
            continue
        if w4_scales is not None:
            s_pick = orc.score_at_w4(H, W, w4_scales, b, gi - vocab_offset, t, seed_b, row_word, gi)
        elif w8_scale is not False:
            s_pick = orc.score_at_w8(H, W, w8_scale, b, gi - vocab_offset, t, seed_b, row_word, gi)
        elif bias is None and allowed_words is None:
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


def lse_tol(tau, lse) -> float:
    """Tolerance of a log-sum-exp of transformed logits: the per-logit budget carried through 1/tau,
    plus fp32 rounding of the accumulation."""
    a = abs(float(lse)) if np.isfinite(lse) else 0.0
    return 2e-3 / min(float(tau), 1.0) + 1e-5 * a + 1e-4


def judge_grouped(orc, mode, ref, H, W, tau, gpu_idx, gpu_lse, gpu_L, gpu_z, *, g, seed=0,
                  row_seeds=None, row_offset=0, vocab_offset=0, bias=None, allowed_words=None) -> Verdict:
    """Grouped variants against oracle.sample_grouped(...) (`ref`), row by row.

    What is unique is compared exactly: the per-group local samples z_k (up to near-ties of the
    in-group perturbed scores, judged like the main path) and, given those, the chosen group.
    The group log-masses and the log-normaliser are compared to lse_tol.  A group decision that
    sits within tolerance of its threshold in the oracle's fp64 arithmetic may go either way:
      parallel: any group whose perturbed log-mass is within 1e-3 (1 + |max|) of the maximum;
      online:   decision k is uncertain when |u_k - p_k| <= 1e-3 p_k / min(tau, 1) + 1e-6; the
                valid answers are the last certainly accepted group and every uncertain group
                after it.
    """
    B = H.shape[0]
    m = ref["L"].shape[1]
    v = Verdict()
    for b in range(B):
        v.rows += 1
        t = float(tau[b])
        seed_b = int(row_seeds[b]) if row_seeds is not None else int(seed)
        row_word = row_offset + b
        arow = None if allowed_words is None else (allowed_words if allowed_words.ndim == 1 else allowed_words[b])
        bad = False
        for k in range(m):
            Lr, Lg = float(ref["L"][b, k]), float(gpu_L[b, k])
            zr, zg = int(ref["zk"][b, k]), int(gpu_z[b, k])
            if not np.isfinite(Lr):
                if Lg != -np.inf or zg != -1:
                    v.failures.append((b, k, "zero-mass group mismatch", Lg, zg)); bad = True
                continue
            if not abs(Lg - Lr) <= lse_tol(t, Lr):
                v.failures.append((b, k, "group log-mass", Lg, Lr)); bad = True
            if zg != zr:
                s1, s2 = float(ref["s1"][b, k]), float(ref["s2"][b, k])
                tol = 1e-3 * (1.0 + abs(s1))
                lo = vocab_offset + k * g
                in_group = lo <= zg < min(lo + g, vocab_offset + W.shape[0])
                s_pick = orc.score_at_full(H, W, b, zg - vocab_offset, t, seed_b, row_word, zg, bias=bias,
                                           allowed_row=arow) if in_group else -np.inf
                if not (in_group and (s1 - s2) < tol and (s1 - s_pick) < tol):
                    v.failures.append((b, k, "local sample", zg, zr, s1, s2)); bad = True
        lr, lg = float(ref["lse"][b]), float(gpu_lse[b])
        if np.isfinite(lr):
            if not abs(lg - lr) <= lse_tol(t, lr):
                v.failures.append((b, "log-normaliser", lg, lr)); bad = True
        elif lg != -np.inf:
            v.failures.append((b, "log-normaliser of an empty row", lg)); bad = True
        gi, ri = int(gpu_idx[b]), int(ref["idx"][b])
        if ri < 0 or gi < 0:
            if gi != ri:
                v.failures.append((b, "empty row mismatch", gi, ri)); bad = True
            elif not bad:
                v.exact += 1
            continue
        kg = (gi - vocab_offset) // g
        if not (0 <= kg < m) or gi != int(gpu_z[b, kg]):
            v.failures.append((b, "index is not the chosen group's local sample", gi, kg)); continue
        kr = (ri - vocab_offset) // g
        if mode == 0:
            outer = ref["outer"][b]
            top = float(outer[kr])
            valid = {k for k in range(m) if top - float(outer[k]) < 1e-3 * (1.0 + abs(top))}
        else:
            u, p = ref["outer"][b], ref["p"][b]
            tolk = 1e-3 * p / min(t, 1.0) + 1e-6
            certain = [k for k in range(m) if np.isfinite(p[k]) and u[k] < p[k] - tolk[k]]
            last = max(certain) if certain else -1
            valid = {k for k in range(m) if np.isfinite(p[k]) and abs(u[k] - p[k]) <= tolk[k] and k > last}
            if last >= 0:
                valid.add(last)
        if kg == kr and not bad:
            v.exact += 1
        elif kg in valid and not bad:
            v.near_ties += 1
        elif not bad:
            v.failures.append((b, "wrong group", kg, kr, sorted(valid)[:8]))
    return v
