"""ctypes front end of the CPU oracle (``fs_oracle.c``).

TEST INFRASTRUCTURE ONLY: imported by ``tests/``, by ``__graft_entry__.smoke()`` and by the
``cpu_baseline`` leg of ``bench.py``.  The product package never imports this module, and this
module never imports the product package.

``build()`` compiles ``fs_oracle.c`` with gcc into ``liboracle.so`` next to this file;
``lib()`` loads it (building it first if it is missing).
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from typing import Optional

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "fs_oracle.c")
_SO = os.path.join(_HERE, "liboracle.so")
_lib = None


def build(force: bool = True) -> str:
    """Compile the oracle.  Plain x86-64 code (no -march=native): the .so travels between hosts."""
    if force or not os.path.exists(_SO) or os.path.getmtime(_SO) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-std=c11", "-fPIC", "-shared", "-fopenmp", "-ffp-contract=off",
               "-Wall", "-Wextra", "-o", _SO, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _SO


_u16p = np.ctypeslib.ndpointer(dtype=np.uint16, flags="C_CONTIGUOUS")
_f64p = np.ctypeslib.ndpointer(dtype=np.float64, flags="C_CONTIGUOUS")
_f32p = np.ctypeslib.ndpointer(dtype=np.float32, flags="C_CONTIGUOUS")
_i64p = np.ctypeslib.ndpointer(dtype=np.int64, flags="C_CONTIGUOUS")
_i32p = np.ctypeslib.ndpointer(dtype=np.int32, flags="C_CONTIGUOUS")
_u32p = np.ctypeslib.ndpointer(dtype=np.uint32, flags="C_CONTIGUOUS")


def lib():
    global _lib
    if _lib is not None:
        return _lib
    build(force=False)
    L = C.CDLL(_SO)
    L.fso_philox4x32_10.argtypes = [_u32p, _u32p, _u32p]
    L.fso_philox4x32_10.restype = None
    L.fso_random_word.argtypes = [C.c_uint64, C.c_int64, C.c_int64]
    L.fso_random_word.restype = C.c_uint32
    L.fso_uniform_x.argtypes = [C.c_uint32]
    L.fso_uniform_x.restype = C.c_float
    L.fso_gumbel_from_word.argtypes = [C.c_uint32]
    L.fso_gumbel_from_word.restype = C.c_double
    L.fso_gumbel.argtypes = [C.c_uint64, C.c_int64, C.c_int64]
    L.fso_gumbel.restype = C.c_double
    L.fso_logit.argtypes = [_u16p, _u16p, C.c_int64, C.c_int64, C.c_int64]
    L.fso_logit.restype = C.c_double
    L.fso_logits.argtypes = [_u16p, _u16p, C.c_int64, C.c_int64, C.c_int64, _f64p]
    L.fso_logits.restype = C.c_int
    L.fso_gumbel_max_row.argtypes = [_f64p, C.c_int64, C.c_double, C.c_uint64, C.c_int64, C.c_int64,
                                     C.POINTER(C.c_int64), C.POINTER(C.c_double),
                                     C.POINTER(C.c_int64), C.POINTER(C.c_double)]
    L.fso_gumbel_max_row.restype = None
    L.fso_score_at.argtypes = [_u16p, _u16p, C.c_int64, C.c_int64, C.c_int64, C.c_double,
                               C.c_uint64, C.c_int64, C.c_int64]
    L.fso_score_at.restype = C.c_double
    L.fso_sample.argtypes = [_u16p, _u16p, C.c_int64, C.c_int64, C.c_int64, _f32p, C.c_uint64,
                             C.c_void_p, C.c_int64, C.c_void_p, C.c_int64, _i32p, _f32p, _f64p,
                             _i64p, _f64p]
    L.fso_sample.restype = C.c_int
    L.fso_sample_tiled.argtypes = [_u16p, _u16p, C.c_int64, C.c_int64, C.c_int64, _f32p, C.c_uint64,
                                   C.c_void_p, C.c_int64, C.c_int64, C.c_int64, _f64p, _i64p,
                                   _i32p, _f32p]
    L.fso_sample_tiled.restype = C.c_int
    L.fso_draw_counts.argtypes = [_f64p, C.c_int64, C.c_double, C.c_uint64, C.c_int64, C.c_int64,
                                  C.c_int, _i64p, C.c_void_p]
    L.fso_draw_counts.restype = None
    L.fso_softmax.argtypes = [_f64p, C.c_int64, C.c_double, _f64p, C.POINTER(C.c_double)]
    L.fso_softmax.restype = None
    L.fso_gumbel_from_words.argtypes = [_u32p, C.c_int64, _f64p, C.c_void_p]
    L.fso_gumbel_from_words.restype = None
    L.fso_random_words.argtypes = [C.c_uint64, C.c_int64, C.c_int64, C.c_int64, _u32p]
    L.fso_random_words.restype = None
    L.fso_transform_row.argtypes = [_f64p, C.c_int64, C.c_double, C.c_void_p, C.c_void_p, _f64p]
    L.fso_transform_row.restype = None
    L.fso_gumbel_max_transformed.argtypes = [_f64p, C.c_int64, C.c_uint64, C.c_int64, C.c_int64,
                                             C.POINTER(C.c_int64), C.POINTER(C.c_double),
                                             C.POINTER(C.c_int64), C.POINTER(C.c_double)]
    L.fso_gumbel_max_transformed.restype = None
    L.fso_log_sum_exp.argtypes = [_f64p, C.c_int64]
    L.fso_log_sum_exp.restype = C.c_double
    L.fso_sample_full.argtypes = [_u16p, _u16p, C.c_int64, C.c_int64, C.c_int64, _f32p, C.c_uint64,
                                  C.c_void_p, C.c_int64, C.c_void_p, C.c_int64, C.c_void_p, C.c_void_p,
                                  C.c_int64, _i32p, _f32p, _f64p, _f64p, _i64p, _f64p]
    L.fso_sample_full.restype = C.c_int
    L.fso_score_at_full.argtypes = [_u16p, _u16p, C.c_int64, C.c_int64, C.c_int64, C.c_double,
                                    C.c_uint64, C.c_int64, C.c_int64, C.c_void_p, C.c_void_p]
    L.fso_score_at_full.restype = C.c_double
    L.fso_num_threads.argtypes = []
    L.fso_num_threads.restype = C.c_int
    _u8p = np.ctypeslib.ndpointer(dtype=np.uint8, flags="C_CONTIGUOUS")
    L.fso_e4m3_to_double.argtypes = [C.c_uint8]
    L.fso_e4m3_to_double.restype = C.c_double
    L.fso_logit_w8.argtypes = [_u16p, _u8p, C.c_void_p, C.c_int64, C.c_int64, C.c_int64]
    L.fso_logit_w8.restype = C.c_double
    L.fso_logits_w8.argtypes = [_u16p, _u8p, C.c_void_p, C.c_int64, C.c_int64, C.c_int64, _f64p]
    L.fso_logits_w8.restype = C.c_int
    L.fso_sample_w8.argtypes = [_u16p, _u8p, C.c_void_p, C.c_int64, C.c_int64, C.c_int64, _f32p, C.c_uint64,
                                C.c_void_p, C.c_int64, C.c_void_p, C.c_int64, _i32p, _f32p, _f64p, _i64p, _f64p]
    L.fso_sample_w8.restype = C.c_int
    L.fso_score_at_w8.argtypes = [_u16p, _u8p, C.c_void_p, C.c_int64, C.c_int64, C.c_int64, C.c_double,
                                  C.c_uint64, C.c_int64, C.c_int64]
    L.fso_score_at_w8.restype = C.c_double
    L.fso_e2m1_to_double.argtypes = [C.c_uint8]
    L.fso_e2m1_to_double.restype = C.c_double
    L.fso_e8m0_to_double.argtypes = [C.c_uint8]
    L.fso_e8m0_to_double.restype = C.c_double
    L.fso_logits_w4.argtypes = [_u16p, _u8p, _u8p, C.c_int64, C.c_int64, C.c_int64, _f64p]
    L.fso_logits_w4.restype = C.c_int
    L.fso_sample_w4.argtypes = [_u16p, _u8p, _u8p, C.c_int64, C.c_int64, C.c_int64, _f32p, C.c_uint64,
                                C.c_void_p, C.c_int64, C.c_void_p, C.c_int64, _i32p, _f32p, _f64p, _i64p, _f64p]
    L.fso_sample_w4.restype = C.c_int
    L.fso_score_at_w4.argtypes = [_u16p, _u8p, _u8p, C.c_int64, C.c_int64, C.c_int64, C.c_double,
                                  C.c_uint64, C.c_int64, C.c_int64]
    L.fso_score_at_w4.restype = C.c_double
    L.fso_group_word.argtypes = [C.c_uint64, C.c_int64, C.c_int64, C.c_uint32]
    L.fso_group_word.restype = C.c_uint32
    L.fso_group_stats.argtypes = [_f64p, C.c_int64, C.c_int64, C.c_uint64, C.c_int64, C.c_int64,
                                  _i64p, _f64p, _f64p, _f64p]
    L.fso_group_stats.restype = None
    L.fso_group_choose_parallel.argtypes = [_f64p, C.c_int64, C.c_uint64, C.c_int64, C.c_int64, _f64p]
    L.fso_group_choose_parallel.restype = C.c_int64
    L.fso_group_choose_online.argtypes = [_f64p, C.c_int64, C.c_uint64, C.c_int64, C.c_int64, _f64p,
                                          _f64p, C.POINTER(C.c_double)]
    L.fso_group_choose_online.restype = C.c_int64
    L.fso_sample_grouped.argtypes = [_u16p, _u16p, C.c_int64, C.c_int64, C.c_int64, _f32p, C.c_uint64,
                                     C.c_void_p, C.c_int64, C.c_void_p, C.c_int64, C.c_void_p,
                                     C.c_void_p, C.c_int64, C.c_int64, C.c_int, _i32p, _f64p, _i64p,
                                     _f64p, _f64p, _f64p, _f64p, _f64p]
    L.fso_sample_grouped.restype = C.c_int
    L.fso_grouped_draw_counts.argtypes = [_f64p, C.c_int64, C.c_int64, C.c_int, C.c_uint64, C.c_int64,
                                          C.c_int64, _i64p]
    L.fso_grouped_draw_counts.restype = None
    L.fso_topk_row.argtypes = [_f64p, C.c_int64, C.c_int64, C.c_int64, _f64p, _i64p, C.POINTER(C.c_double)]
    L.fso_topk_row.restype = C.c_int
    L.fso_top_p_cut.argtypes = [_f64p, C.c_int64, C.c_double, C.POINTER(C.c_double)]
    L.fso_top_p_cut.restype = C.c_int64
    L.fso_sample_topk.argtypes = [_u16p, _u16p, C.c_int64, C.c_int64, C.c_int64, _f32p, C.c_uint64, C.c_void_p,
                                  C.c_int64, C.c_int64, C.c_int64, C.c_double, C.c_int, _i32p, _f32p, _f64p, _i64p,
                                  _i64p, _f64p, _f64p, _f64p, _f64p]
    L.fso_sample_topk.restype = C.c_int
    _lib = L
    return L


# ----------------------------------------------------------------------------- numpy wrappers

def philox4x32_10(ctr, key) -> np.ndarray:
    ctr = np.ascontiguousarray(ctr, dtype=np.uint32)
    key = np.ascontiguousarray(key, dtype=np.uint32)
    out = np.zeros(4, dtype=np.uint32)
    lib().fso_philox4x32_10(ctr, key, out)
    return out


def random_word(seed: int, row: int, vocab_id: int) -> int:
    return int(lib().fso_random_word(seed, row, vocab_id))


def random_words(seed: int, row: int, v0: int, n: int) -> np.ndarray:
    out = np.empty(n, dtype=np.uint32)
    lib().fso_random_words(seed, row, v0, n, out)
    return out


def uniform_x(r: int) -> float:
    return float(lib().fso_uniform_x(r))


def gumbel_from_word(r: int) -> float:
    return float(lib().fso_gumbel_from_word(r))


def gumbel_from_words(r: np.ndarray):
    r = np.ascontiguousarray(r, dtype=np.uint32)
    g = np.empty(r.size, dtype=np.float64)
    x = np.empty(r.size, dtype=np.float32)
    lib().fso_gumbel_from_words(r, r.size, g, x.ctypes.data_as(C.c_void_p))
    return g, x


def gumbel(seed: int, row: int, vocab_id: int) -> float:
    return float(lib().fso_gumbel(seed, row, vocab_id))


def logit(H: np.ndarray, W: np.ndarray, b: int, i: int) -> float:
    return float(lib().fso_logit(H, W, H.shape[1], b, i))


def logits(H: np.ndarray, W: np.ndarray) -> np.ndarray:
    B, D = H.shape
    V = W.shape[0]
    assert W.shape[1] == D
    Y = np.empty((B, V), dtype=np.float64)
    lib().fso_logits(H, W, B, D, V, Y)
    return Y


def gumbel_max_row(y: np.ndarray, tau: float, seed: int, row: int, vocab_offset: int = 0):
    """Streaming Gumbel-max over one row of raw logits -> (idx, val, idx2, val2)."""
    y = np.ascontiguousarray(y, dtype=np.float64)
    i1, i2 = C.c_int64(), C.c_int64()
    m1, m2 = C.c_double(), C.c_double()
    lib().fso_gumbel_max_row(y, y.size, float(tau), seed, row, vocab_offset,
                             C.byref(i1), C.byref(m1), C.byref(i2), C.byref(m2))
    return i1.value, m1.value, i2.value, m2.value


def score_at(H, W, b_local: int, i_local: int, tau: float, seed: int, row: int, vocab_id: int) -> float:
    return float(lib().fso_score_at(H, W, H.shape[1], b_local, i_local, float(tau), seed, row, vocab_id))


def _opt_ptr(a: Optional[np.ndarray], dtype):
    if a is None:
        return None, None
    a = np.ascontiguousarray(a, dtype=dtype)
    return a, a.ctypes.data_as(C.c_void_p)


def sample(H, W, tau, seed: int = 0, row_seeds=None, row_offset: int = 0, row_ids=None,
           vocab_offset: int = 0):
    """Full path.  Returns dict(idx, val, top1, idx2, top2, threads)."""
    B, D = H.shape
    V = W.shape[0]
    tau = np.ascontiguousarray(tau, dtype=np.float32)
    assert tau.shape == (B,)
    rs, rs_p = _opt_ptr(row_seeds, np.uint64)
    ri, ri_p = _opt_ptr(row_ids, np.int64)
    out_idx = np.empty(B, dtype=np.int32)
    out_val = np.empty(B, dtype=np.float32)
    top1 = np.empty(B, dtype=np.float64)
    idx2 = np.empty(B, dtype=np.int64)
    top2 = np.empty(B, dtype=np.float64)
    nt = lib().fso_sample(H, W, B, D, V, tau, seed, rs_p, row_offset, ri_p, vocab_offset,
                          out_idx, out_val, top1, idx2, top2)
    if nt < 0:
        raise MemoryError("oracle: out of memory")
    return dict(idx=out_idx, val=out_val, top1=top1, idx2=idx2, top2=top2, threads=nt)


def sample_tiled(H, W, tau, tile: int, seed: int = 0, row_seeds=None, row_offset: int = 0,
                 vocab_offset: int = 0):
    """Two-stage form with vocabulary tile size `tile`.  Returns dict(idx, val, cand_val, cand_idx)."""
    B, D = H.shape
    V = W.shape[0]
    T = (V + tile - 1) // tile
    tau = np.ascontiguousarray(tau, dtype=np.float32)
    rs, rs_p = _opt_ptr(row_seeds, np.uint64)
    cand_val = np.empty((B, T), dtype=np.float64)
    cand_idx = np.empty((B, T), dtype=np.int64)
    out_idx = np.empty(B, dtype=np.int32)
    out_val = np.empty(B, dtype=np.float32)
    nt = lib().fso_sample_tiled(H, W, B, D, V, tau, seed, rs_p, row_offset, vocab_offset, tile,
                                cand_val, cand_idx, out_idx, out_val)
    if nt < 0:
        raise MemoryError("oracle: out of memory")
    return dict(idx=out_idx, val=out_val, cand_val=cand_val, cand_idx=cand_idx)


def draw_counts(y, tau: float, seed: int, ndraws: int, by_row: bool = True, row0: int = 0,
                return_vals: bool = False):
    y = np.ascontiguousarray(y, dtype=np.float64)
    counts = np.zeros(y.size, dtype=np.int64)
    vals = np.empty(ndraws, dtype=np.float64) if return_vals else None
    vp = vals.ctypes.data_as(C.c_void_p) if return_vals else None
    lib().fso_draw_counts(y, y.size, float(tau), seed, row0, ndraws, 1 if by_row else 0, counts, vp)
    return (counts, vals) if return_vals else counts


def softmax(y, tau: float = 1.0):
    y = np.ascontiguousarray(y, dtype=np.float64)
    p = np.empty_like(y)
    lse = C.c_double()
    lib().fso_softmax(y, y.size, float(tau), p, C.byref(lse))
    return p, lse.value


def pack_allowed(allowed_bool: np.ndarray) -> np.ndarray:
    """Pack a boolean array [..., V] (True = allowed) into 32-bit words [..., ceil(V/32)],
    bit i%32 of word i/32.  Pure data layout, no method arithmetic."""
    a = np.asarray(allowed_bool, dtype=bool)
    V = a.shape[-1]
    nw = (V + 31) // 32
    pad = np.zeros(a.shape[:-1] + (nw * 32,), dtype=bool)
    pad[..., :V] = a
    bits = pad.reshape(a.shape[:-1] + (nw, 32)).astype(np.uint64)
    words = (bits << np.arange(32, dtype=np.uint64)).sum(axis=-1)
    return np.ascontiguousarray(words.astype(np.uint32))


def transform_row(y, tau: float, bias=None, allowed_words=None) -> np.ndarray:
    y = np.ascontiguousarray(y, dtype=np.float64)
    z = np.empty_like(y)
    b, bp = _opt_ptr(bias, np.float32)
    a, ap = _opt_ptr(allowed_words, np.uint32)
    lib().fso_transform_row(y, y.size, float(tau), bp, ap, z)
    return z


def gumbel_max_transformed(z, seed: int, row: int, vocab_offset: int = 0):
    z = np.ascontiguousarray(z, dtype=np.float64)
    i1, i2 = C.c_int64(), C.c_int64()
    m1, m2 = C.c_double(), C.c_double()
    lib().fso_gumbel_max_transformed(z, z.size, seed, row, vocab_offset, C.byref(i1), C.byref(m1),
                                     C.byref(i2), C.byref(m2))
    return i1.value, m1.value, i2.value, m2.value


def log_sum_exp(z) -> float:
    z = np.ascontiguousarray(z, dtype=np.float64)
    return float(lib().fso_log_sum_exp(z, z.size))


def sample_full(H, W, tau, seed: int = 0, row_seeds=None, row_offset: int = 0, row_ids=None,
                vocab_offset: int = 0, bias=None, allowed_words=None):
    """Full transform + log-normaliser.  allowed_words: None, [nw] (shared) or [B, nw] uint32."""
    B, D = H.shape
    V = W.shape[0]
    tau = np.ascontiguousarray(tau, dtype=np.float32)
    rs, rs_p = _opt_ptr(row_seeds, np.uint64)
    ri, ri_p = _opt_ptr(row_ids, np.int64)
    bb, bb_p = _opt_ptr(bias, np.float32)
    aw, aw_p = _opt_ptr(allowed_words, np.uint32)
    stride = 0
    if aw is not None and aw.ndim == 2:
        assert aw.shape[0] == B
        stride = aw.shape[1]
    out_idx = np.empty(B, dtype=np.int32)
    out_val = np.empty(B, dtype=np.float32)
    lse = np.empty(B, dtype=np.float64)
    top1 = np.empty(B, dtype=np.float64)
    idx2 = np.empty(B, dtype=np.int64)
    top2 = np.empty(B, dtype=np.float64)
    nt = lib().fso_sample_full(H, W, B, D, V, tau, seed, rs_p, row_offset, ri_p, vocab_offset, bb_p, aw_p,
                               stride, out_idx, out_val, lse, top1, idx2, top2)
    if nt < 0:
        raise MemoryError("oracle: out of memory")
    return dict(idx=out_idx, val=out_val, lse=lse, top1=top1, idx2=idx2, top2=top2, threads=nt)


def score_at_full(H, W, b_local, i_local, tau, seed, row, vocab_id, bias=None, allowed_row=None) -> float:
    bb, bb_p = _opt_ptr(bias, np.float32)
    ar, ar_p = _opt_ptr(allowed_row, np.uint32)
    return float(lib().fso_score_at_full(H, W, H.shape[1], b_local, i_local, float(tau), seed, row,
                                         vocab_id, bb_p, ar_p))


def e4m3_to_double(code: int) -> float:
    return float(lib().fso_e4m3_to_double(int(code) & 0xFF))


def logits_w8(H, W8, scale=None) -> np.ndarray:
    B, D = H.shape
    V = W8.shape[0]
    sc, sc_p = _opt_ptr(scale, np.float32)
    Y = np.empty((B, V), dtype=np.float64)
    lib().fso_logits_w8(H, W8, sc_p, B, D, V, Y)
    return Y


def sample_w8(H, W8, scale, tau, seed: int = 0, row_seeds=None, row_offset: int = 0, row_ids=None,
              vocab_offset: int = 0):
    """Default path on FP8 (E4M3) weights with per-row scales.  Returns dict(idx, val, top1, idx2, top2)."""
    B, D = H.shape
    V = W8.shape[0]
    tau = np.ascontiguousarray(tau, dtype=np.float32)
    sc, sc_p = _opt_ptr(scale, np.float32)
    rs, rs_p = _opt_ptr(row_seeds, np.uint64)
    ri, ri_p = _opt_ptr(row_ids, np.int64)
    out_idx = np.empty(B, dtype=np.int32)
    out_val = np.empty(B, dtype=np.float32)
    top1 = np.empty(B, dtype=np.float64)
    idx2 = np.empty(B, dtype=np.int64)
    top2 = np.empty(B, dtype=np.float64)
    nt = lib().fso_sample_w8(H, W8, sc_p, B, D, V, tau, seed, rs_p, row_offset, ri_p, vocab_offset,
                             out_idx, out_val, top1, idx2, top2)
    if nt < 0:
        raise MemoryError("oracle: out of memory")
    return dict(idx=out_idx, val=out_val, top1=top1, idx2=idx2, top2=top2, threads=nt)


def score_at_w8(H, W8, scale, b_local, i_local, tau, seed, row, vocab_id) -> float:
    sc, sc_p = _opt_ptr(scale, np.float32)
    return float(lib().fso_score_at_w8(H, W8, sc_p, H.shape[1], b_local, i_local, float(tau), seed, row, vocab_id))


def e2m1_to_double(nibble: int) -> float:
    return float(lib().fso_e2m1_to_double(int(nibble) & 0xF))


def e8m0_to_double(e: int) -> float:
    return float(lib().fso_e8m0_to_double(int(e) & 0xFF))


def logits_w4(H, W4, S) -> np.ndarray:
    B, D = H.shape
    V = W4.shape[0]
    Y = np.empty((B, V), dtype=np.float64)
    lib().fso_logits_w4(H, W4, S, B, D, V, Y)
    return Y


def sample_w4(H, W4, S, tau, seed: int = 0, row_seeds=None, row_offset: int = 0, row_ids=None,
              vocab_offset: int = 0):
    """Default path on MXFP4 weights (E2M1 codes, two per byte, one E8M0 scale per 32 elements)."""
    B, D = H.shape
    V = W4.shape[0]
    assert W4.shape == (V, D // 2) and S.shape == (V, D // 32)
    tau = np.ascontiguousarray(tau, dtype=np.float32)
    rs, rs_p = _opt_ptr(row_seeds, np.uint64)
    ri, ri_p = _opt_ptr(row_ids, np.int64)
    out_idx = np.empty(B, dtype=np.int32)
    out_val = np.empty(B, dtype=np.float32)
    top1 = np.empty(B, dtype=np.float64)
    idx2 = np.empty(B, dtype=np.int64)
    top2 = np.empty(B, dtype=np.float64)
    nt = lib().fso_sample_w4(H, W4, S, B, D, V, tau, seed, rs_p, row_offset, ri_p, vocab_offset,
                             out_idx, out_val, top1, idx2, top2)
    if nt < 0:
        raise MemoryError("oracle: out of memory")
    return dict(idx=out_idx, val=out_val, top1=top1, idx2=idx2, top2=top2, threads=nt)


def score_at_w4(H, W4, S, b_local, i_local, tau, seed, row, vocab_id) -> float:
    return float(lib().fso_score_at_w4(H, W4, S, H.shape[1], b_local, i_local, float(tau), seed, row, vocab_id))


GROUPED_PARALLEL, GROUPED_ONLINE = 0, 1


def group_word(seed: int, row: int, group_id: int, stream: int) -> int:
    return int(lib().fso_group_word(seed, row, group_id, stream))


def group_stats(z, g: int, seed: int, row: int, vocab_offset: int = 0):
    """Per-group local sample, its top-two perturbed scores and the group log-mass of one row."""
    z = np.ascontiguousarray(z, dtype=np.float64)
    m = (z.size + g - 1) // g
    zk = np.empty(m, dtype=np.int64)
    s1, s2, L = (np.empty(m, dtype=np.float64) for _ in range(3))
    lib().fso_group_stats(z, z.size, g, seed, row, vocab_offset, zk, s1, s2, L)
    return dict(zk=zk, s1=s1, s2=s2, L=L)


def group_choose_parallel(L, seed: int, row: int, group_offset: int = 0):
    L = np.ascontiguousarray(L, dtype=np.float64)
    score = np.empty_like(L)
    k = lib().fso_group_choose_parallel(L, L.size, seed, row, group_offset, score)
    return int(k), score


def group_choose_online(L, seed: int, row: int, group_offset: int = 0):
    L = np.ascontiguousarray(L, dtype=np.float64)
    u, p = np.empty_like(L), np.empty_like(L)
    lse = C.c_double()
    k = lib().fso_group_choose_online(L, L.size, seed, row, group_offset, u, p, C.byref(lse))
    return int(k), u, p, lse.value


def sample_grouped(H, W, tau, g: int, mode: int, seed: int = 0, row_seeds=None, row_offset: int = 0,
                   row_ids=None, vocab_offset: int = 0, bias=None, allowed_words=None):
    """Grouped variants (mode GROUPED_PARALLEL / GROUPED_ONLINE) with groups of g ids.
    Returns idx, lse and the per-group diagnostics zk, s1, s2, L, outer, p (each [B, m])."""
    B, D = H.shape
    V = W.shape[0]
    assert vocab_offset % g == 0
    m = (V + g - 1) // g
    tau = np.ascontiguousarray(tau, dtype=np.float32)
    rs, rs_p = _opt_ptr(row_seeds, np.uint64)
    ri, ri_p = _opt_ptr(row_ids, np.int64)
    bb, bb_p = _opt_ptr(bias, np.float32)
    aw, aw_p = _opt_ptr(allowed_words, np.uint32)
    stride = 0
    if aw is not None and aw.ndim == 2:
        assert aw.shape[0] == B
        stride = aw.shape[1]
    out_idx = np.empty(B, dtype=np.int32)
    lse = np.empty(B, dtype=np.float64)
    zk = np.empty((B, m), dtype=np.int64)
    s1, s2, L, outer, p = (np.full((B, m), np.nan, dtype=np.float64) for _ in range(5))
    nt = lib().fso_sample_grouped(H, W, B, D, V, tau, seed, rs_p, row_offset, ri_p, vocab_offset, bb_p,
                                  aw_p, stride, g, mode, out_idx, lse, zk, s1, s2, L, outer, p)
    if nt < 0:
        raise MemoryError("oracle: out of memory")
    return dict(idx=out_idx, lse=lse, zk=zk, s1=s1, s2=s2, L=L, outer=outer, p=p, threads=nt)


def grouped_draw_counts(z, g: int, mode: int, seed: int, ndraws: int, row0: int = 0) -> np.ndarray:
    z = np.ascontiguousarray(z, dtype=np.float64)
    counts = np.zeros(z.size, dtype=np.int64)
    lib().fso_grouped_draw_counts(z, z.size, g, mode, seed, row0, ndraws, counts)
    return counts


def num_threads() -> int:
    return int(lib().fso_num_threads())


# ----------------------------------------------------------------------------- truncated supports

TOPK_TRUNCATE, TOPK_GUMBEL = 0, 1


def topk_row(key, k: int, vocab_offset: int = 0):
    """The k largest keys of a row by a full sort -> (keys [k], ids [k], (k+1)-th key)."""
    key = np.ascontiguousarray(key, dtype=np.float64)
    ok = np.empty(k, dtype=np.float64)
    oi = np.empty(k, dtype=np.int64)
    nxt = C.c_double()
    if lib().fso_topk_row(key, key.size, k, vocab_offset, ok, oi, C.byref(nxt)) != 0:
        raise MemoryError("oracle: out of memory")
    return ok, oi, nxt.value


def top_p_cut(z_sorted, top_p: float):
    """Nucleus rule on candidates in descending order -> (number kept, mass of the kept prefix without its last)."""
    z = np.ascontiguousarray(z_sorted, dtype=np.float64)
    mb = C.c_double()
    n = lib().fso_top_p_cut(z, z.size, float(top_p), C.byref(mb))
    return int(n), mb.value


def sample_topk(H, W, tau, k: int, top_p: float = 1.0, mode: int = TOPK_TRUNCATE, seed: int = 0, row_seeds=None,
                row_offset: int = 0, vocab_offset: int = 0):
    """Top-k / nucleus draw (mode TOPK_TRUNCATE) or Gumbel-top-k (mode TOPK_GUMBEL).  Returns
    dict(idx, val, top_key [B,k], top_id [B,k], n_kept, kth1, mass_before, top1, top2, threads)."""
    B, D = H.shape
    V = W.shape[0]
    tau = np.ascontiguousarray(tau, dtype=np.float32)
    rs, rs_p = _opt_ptr(row_seeds, np.uint64)
    out_idx = np.empty(B, dtype=np.int32)
    out_val = np.empty(B, dtype=np.float32)
    top_key = np.empty((B, k), dtype=np.float64)
    top_id = np.empty((B, k), dtype=np.int64)
    n_kept = np.empty(B, dtype=np.int64)
    kth1 = np.empty(B, dtype=np.float64)
    mass_before = np.empty(B, dtype=np.float64)
    top1 = np.empty(B, dtype=np.float64)
    top2 = np.empty(B, dtype=np.float64)
    nt = lib().fso_sample_topk(H, W, B, D, V, tau, seed, rs_p, row_offset, vocab_offset, k, float(top_p), int(mode),
                               out_idx, out_val, top_key, top_id, n_kept, kth1, mass_before, top1, top2)
    if nt < 0:
        raise MemoryError("oracle: out of memory")
    return dict(idx=out_idx, val=out_val, top_key=top_key, top_id=top_id, n_kept=n_kept, kth1=kth1,
                mass_before=mass_before, top1=top1, top2=top2, threads=nt)
