"""Thin Python binding of the C ABI in ``include/flash_sample.h`` (ctypes; argument marshalling
only -- every step of the method runs in the HIP kernels of ``libflashsample.so``).

PyTorch is used for device memory and streams, nothing else.  There is no CPU fallback: if the
library is missing or a call fails, an exception is raised.

Functions mirror the C names (``EXPORTS`` lists every symbol of the header): ``flash_sample``,
``flash_sample_ex``, ``flash_sample_static``, ``flash_sample_full``, ``flash_sample_grouped``,
``flash_group_choose``, ``flash_sample_w8``, ``flash_sample_w4``, the stages ``flash_sample_stage1`` /
``flash_sample_stage2``, the comparison path ``flash_sample_unfused`` / ``flash_lm_head_logits`` /
``flash_gumbel_argmax_logits`` and the debug taps.  The measurement aids of
``include/flash_sample_measure.h`` are bound in ``paper_2603_15854_amd.measure``.

Every tensor argument is checked for device, dtype, contiguity and length before its pointer is
handed over: the C side cannot see any of these.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libflashsample.so")

FS_OK = 0
FS_ERR_NULL, FS_ERR_SHAPE, FS_ERR_ALIGN, FS_ERR_WORKSPACE, FS_ERR_HIP, FS_ERR_UNSUPPORTED = 1, 2, 3, 4, 5, 6
FS_ERR_DEVICE, FS_ERR_SCRATCH_LIMIT = 7, 8
FS_VOCAB_TILE = 128
FS_FLAG_NONE, FS_FLAG_GREEDY, FS_FLAG_EXACT_LOG = 0, 1, 2
FS_VARIANT_AUTO, FS_VARIANT_SPLITK, FS_VARIANT_TILED2 = 0, 2, 7
FS_STATIC_SCRATCH_BYTES = 8 << 20

# every symbol include/flash_sample.h declares
EXPORTS = (
    "flash_sample_num_tiles", "flash_sample_workspace_bytes", "flash_sample", "flash_sample_ex",
    "flash_sample_static",
    "flash_sample_full", "flash_sample_full_workspace_bytes",
    "flash_sample_topk", "flash_sample_topk_unfused", "flash_sample_topk_workspace_bytes",
    "flash_sample_grouped", "flash_sample_num_groups", "flash_group_choose",
    "flash_sample_w8", "flash_sample_e4m3_decode", "flash_sample_w4", "flash_sample_mxfp4_decode",
    "flash_sample_stage1", "flash_sample_stage2", "flash_sample_unfused", "flash_lm_head_logits",
    "flash_gumbel_argmax_logits", "flash_sample_noise", "flash_sample_gumbel_transform",
    "fs_status_string",
)
# every symbol include/flash_sample_measure.h declares
MEASURE_EXPORTS = ("flash_measure_stream_probe", "flash_measure_kernel_choice")


def FS_VARIANT(v: int) -> int:
    return (v & 0xFF) << 8


def FS_TUNE_WGS_PER_CU(n: int) -> int:
    return (n & 0xF) << 16


FS_TUNE_TILE_SHAPE = FS_TUNE_WGS_PER_CU


class FlashSampleError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {fs_status_string(status)} (status {status})")


_lib = None


def lib():
    """Load libflashsample.so (built by ``python -m paper_2603_15854_amd.build``)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise FileNotFoundError(
            f"{LIB_PATH} is missing: build it with `python -m paper_2603_15854_amd.build` "
            "(there is no fallback path)")
    # One HIP runtime per process, and it has to be the one torch brings: the tensors this binding is
    # handed are allocated by it.  The library names the runtime by its soname only, so whichever copy
    # is loaded first serves both; loading this library before torch would put torch on the system's
    # copy (every launch then fails with a HIP error).
    import torch  # noqa: F401
    L = C.CDLL(LIB_PATH)
    vp, i32, i64, u32, u64, sz = C.c_void_p, C.c_int, C.c_int64, C.c_uint32, C.c_uint64, C.c_size_t
    L.flash_sample_num_tiles.argtypes = [i32]
    L.flash_sample_num_tiles.restype = i32
    L.flash_measure_kernel_choice.argtypes = [i32, i32, i32, i32]
    L.flash_measure_kernel_choice.restype = i32
    L.flash_sample_workspace_bytes.argtypes = [i32, i32]
    L.flash_sample_workspace_bytes.restype = sz
    L.flash_sample.argtypes = [vp, vp, i32, i32, i32, vp, u64, vp, vp]
    L.flash_sample.restype = i32
    L.flash_sample_ex.argtypes = [vp, vp, i32, i32, i32, vp, u64, vp, i64, C.c_int32, vp, vp, vp, sz, vp, u32]
    L.flash_sample_ex.restype = i32
    L.flash_sample_static.argtypes = [vp, vp, i32, i32, i32, vp, u64, vp, i64, C.c_int32, vp, vp, vp, u32]
    L.flash_sample_static.restype = i32
    L.flash_sample_full_workspace_bytes.argtypes = [i32, i32]
    L.flash_sample_full_workspace_bytes.restype = sz
    L.flash_sample_full.argtypes = [vp, vp, i32, i32, i32, vp, u64, vp, i64, C.c_int32, vp, vp, i64,
                                    vp, vp, vp, vp, sz, vp, u32]
    L.flash_sample_full.restype = i32
    L.flash_sample_topk_workspace_bytes.argtypes = [i32, i32, i32]
    L.flash_sample_topk_workspace_bytes.restype = sz
    L.flash_sample_topk.argtypes = [vp, vp, i32, i32, i32, vp, u64, vp, i64, C.c_int32, i32, C.c_float, i32,
                                    vp, vp, vp, vp, vp, vp, sz, vp, u32]
    L.flash_sample_topk.restype = i32
    L.flash_sample_topk_unfused.argtypes = [vp, vp, i32, i32, i32, vp, u64, vp, i64, C.c_int32, i32, C.c_float, i32,
                                            vp, vp, vp, vp, vp, vp, vp, sz, vp, u32]
    L.flash_sample_topk_unfused.restype = i32
    L.flash_sample_num_groups.argtypes = [i32, i32]
    L.flash_sample_num_groups.restype = i32
    L.flash_sample_grouped.argtypes = [vp, vp, i32, i32, i32, vp, u64, vp, i64, C.c_int32, vp, vp, i64,
                                       i32, i32, vp, vp, vp, vp, vp, sz, vp, u32]
    L.flash_sample_grouped.restype = i32
    L.flash_group_choose.argtypes = [vp, vp, i32, i32, i32, u64, vp, i64, i64, vp, vp, vp]
    L.flash_group_choose.restype = i32
    L.flash_sample_w8.argtypes = [vp, vp, vp, i32, i32, i32, vp, u64, vp, i64, C.c_int32, vp, vp, vp, vp, sz, vp, u32]
    L.flash_sample_w8.restype = i32
    L.flash_sample_w4.argtypes = [vp, vp, vp, i32, i32, i32, vp, u64, vp, i64, C.c_int32, vp, vp, vp, vp, sz, vp, u32]
    L.flash_sample_w4.restype = i32
    L.flash_sample_mxfp4_decode.argtypes = [vp, vp, i32, vp, vp]
    L.flash_sample_mxfp4_decode.restype = i32
    L.flash_sample_e4m3_decode.argtypes = [vp, i32, vp, vp]
    L.flash_sample_e4m3_decode.restype = i32
    L.flash_sample_stage1.argtypes = [vp, vp, i32, i32, i32, vp, u64, vp, i64, C.c_int32, vp, vp, vp, vp, u32]
    L.flash_sample_stage1.restype = i32
    L.flash_sample_stage2.argtypes = [vp, vp, i32, i32, vp, vp, vp]
    L.flash_sample_stage2.restype = i32
    L.flash_sample_unfused.argtypes = [vp, vp, i32, i32, i32, vp, u64, vp, i64, C.c_int32, vp, vp, vp, vp, sz, vp, u32]
    L.flash_sample_unfused.restype = i32
    L.flash_lm_head_logits.argtypes = [vp, vp, i32, i32, i32, vp, vp, u32]
    L.flash_lm_head_logits.restype = i32
    L.flash_gumbel_argmax_logits.argtypes = [vp, i32, i32, vp, u64, vp, i64, C.c_int32, vp, vp, vp, sz, vp]
    L.flash_gumbel_argmax_logits.restype = i32
    L.flash_sample_noise.argtypes = [u64, i64, C.c_int32, i32, vp, vp]
    L.flash_sample_noise.restype = i32
    L.flash_sample_gumbel_transform.argtypes = [vp, i32, vp, vp, u32]
    L.flash_sample_gumbel_transform.restype = i32
    L.flash_measure_stream_probe.argtypes = [vp, vp, sz, vp, vp]
    L.flash_measure_stream_probe.restype = i32
    L.fs_status_string.argtypes = [i32]
    L.fs_status_string.restype = C.c_char_p
    _lib = L
    return L


def fs_status_string(status: int) -> str:
    return lib().fs_status_string(int(status)).decode()


def flash_sample_num_tiles(V: int) -> int:
    return int(lib().flash_sample_num_tiles(int(V)))


def flash_sample_workspace_bytes(B: int, V: int) -> int:
    return int(lib().flash_sample_workspace_bytes(int(B), int(V)))


# ----------------------------------------------------------------------------- marshalling

def _ptr(t, dtype=None, numel: Optional[int] = None, name: str = "tensor") -> Optional[int]:
    """Device pointer of a torch tensor (None -> NULL) after checking what the C side cannot see:
    device, contiguity, and -- when given -- dtype and the minimum number of elements."""
    if t is None:
        return None
    if not t.is_cuda:
        raise ValueError(f"{name}: expected a device tensor")
    if not t.is_contiguous():
        raise ValueError(f"{name}: expected a contiguous tensor")
    if dtype is not None:
        ok = t.dtype in dtype if isinstance(dtype, (tuple, list)) else t.dtype == dtype
        if not ok:
            raise ValueError(f"{name}: expected dtype {dtype}, got {t.dtype}")
    if numel is not None and t.numel() < numel:
        raise ValueError(f"{name}: expected at least {numel} elements, got {t.numel()}")
    return t.data_ptr()


def _f32(t, n, name):
    import torch
    return _ptr(t, torch.float32, n, name)


def _i32(t, n, name):
    import torch
    return _ptr(t, torch.int32, n, name)


def _seeds(t, n):
    """row_seeds: 64-bit patterns, carried as int64 (torch has no uint64 arithmetic)."""
    import torch
    return _ptr(t, (torch.int64, torch.uint64), n, "row_seeds")


def _stream_ptr(stream) -> Optional[int]:
    import torch
    if stream is None:
        stream = torch.cuda.current_stream()
    return stream.cuda_stream or None


def _check(status: int, where: str) -> None:
    if status != FS_OK:
        raise FlashSampleError(status, where)


def _shapes(hidden, W):
    import torch
    if hidden.dtype != torch.bfloat16 or W.dtype != torch.bfloat16:
        raise ValueError("hidden and W must be bfloat16")
    if hidden.dim() != 2 or W.dim() != 2 or hidden.shape[1] != W.shape[1]:
        raise ValueError("hidden must be [B, D] and W [V, D]")
    return hidden.shape[0], hidden.shape[1], W.shape[0]


def _outputs(B, device, out_idx, out_val):
    import torch
    if out_idx is None:
        out_idx = torch.empty(B, dtype=torch.int32, device=device)
    if out_val is None:
        out_val = torch.empty(B, dtype=torch.float32, device=device)
    _i32(out_idx, B, "out_idx")
    _f32(out_val, B, "out_val")
    return out_idx, out_val


def _scratch(need: int, device, workspace, stream):
    """The caller's workspace, or a fresh one.  A fresh one is a temporary: when the call runs on a
    stream other than torch's current one the allocator is told (record_stream), so the block is
    not handed out again while the kernels still use it."""
    import torch
    if workspace is None:
        workspace = torch.empty(max(need, 256), dtype=torch.uint8, device=device)
        if stream is not None and stream != torch.cuda.current_stream():
            workspace.record_stream(stream)
    _ptr(workspace, None, None, "workspace")
    return workspace, workspace.numel() * workspace.element_size()


def _workspace(B, V, device, workspace, stream=None):
    return _scratch(flash_sample_workspace_bytes(B, V), device, workspace, stream)


# ----------------------------------------------------------------------------- entry points

def flash_sample(hidden, W, temperature, seed: int = 0, out_idx=None, out_val=None):
    """i*_b ~ Cat(softmax(hidden_b W^T / temperature_b)); returns (out_idx int32 [B], out_val fp32 [B]).
    Runs on the null stream (the C entry point's contract)."""
    B, D, V = _shapes(hidden, W)
    out_idx, out_val = _outputs(B, hidden.device, out_idx, out_val)
    st = lib().flash_sample(_ptr(hidden), _ptr(W), B, D, V, _f32(temperature, B, "temperature"), int(seed),
                            _ptr(out_idx), _ptr(out_val))
    _check(st, "flash_sample")
    return out_idx, out_val


def flash_sample_ex(hidden, W, temperature, seed: int = 0, row_seeds=None, row_offset: int = 0,
                    vocab_offset: int = 0, out_idx=None, out_val=None, workspace=None, stream=None,
                    flags: int = 0):
    B, D, V = _shapes(hidden, W)
    out_idx, out_val = _outputs(B, hidden.device, out_idx, out_val)
    workspace, ws_bytes = _workspace(B, V, hidden.device, workspace, stream)
    st = lib().flash_sample_ex(_ptr(hidden), _ptr(W), B, D, V, _f32(temperature, B, "temperature"), int(seed),
                               _seeds(row_seeds, B), int(row_offset), int(vocab_offset), _ptr(out_idx),
                               _ptr(out_val), _ptr(workspace), ws_bytes, _stream_ptr(stream), int(flags))
    _check(st, "flash_sample_ex")
    return out_idx, out_val


def flash_sample_static(hidden, W, temperature, out_idx, out_val, seed: int = 0, row_seeds=None,
                        row_offset: int = 0, vocab_offset: int = 0, stream=None, flags: int = 0):
    """flash_sample_ex on the library's built-in scratch: no allocation anywhere, so the caller
    passes the outputs too.  Calls that overlap on one device race on the scratch."""
    B, D, V = _shapes(hidden, W)
    st = lib().flash_sample_static(_ptr(hidden), _ptr(W), B, D, V, _f32(temperature, B, "temperature"),
                                   int(seed), _seeds(row_seeds, B), int(row_offset), int(vocab_offset),
                                   _i32(out_idx, B, "out_idx"), _f32(out_val, B, "out_val"),
                                   _stream_ptr(stream), int(flags))
    _check(st, "flash_sample_static")
    return out_idx, out_val


def flash_sample_full_workspace_bytes(B: int, V: int) -> int:
    return int(lib().flash_sample_full_workspace_bytes(int(B), int(V)))


def _mask_args(allowed, B, V):
    """(pointer, stride in words) of an allowed-id bit mask: [ceil(V/32)] shared or [B, >= ceil(V/32)]."""
    import torch
    if allowed is None:
        return None, 0
    words = (V + 31) // 32
    if allowed.dim() == 2:
        if allowed.shape[0] < B or allowed.shape[1] < words:
            raise ValueError("allowed: expected [B, >= ceil(V/32)] words")
        return _ptr(allowed, (torch.int32, torch.uint32), None, "allowed"), allowed.shape[1]
    return _ptr(allowed, (torch.int32, torch.uint32), words, "allowed"), 0


def flash_sample_full(hidden, W, temperature, seed: int = 0, row_seeds=None, row_offset: int = 0,
                      vocab_offset: int = 0, bias=None, allowed=None, want_lse: bool = True,
                      out_idx=None, out_val=None, out_lse=None, workspace=None, stream=None, flags: int = 0):
    """Draw with bias / allowed-id mask / log-normaliser.  `allowed` is an int32 tensor of bit words,
    [ceil(V/32)] (shared by all rows) or [B, >= ceil(V/32)].  Returns (out_idx, out_val, out_lse)."""
    import torch
    B, D, V = _shapes(hidden, W)
    out_idx, out_val = _outputs(B, hidden.device, out_idx, out_val)
    if want_lse and out_lse is None:
        out_lse = torch.empty(B, dtype=torch.float32, device=hidden.device)
    mask_ptr, stride = _mask_args(allowed, B, V)
    workspace, ws_bytes = _scratch(flash_sample_full_workspace_bytes(B, V), hidden.device, workspace, stream)
    st = lib().flash_sample_full(_ptr(hidden), _ptr(W), B, D, V, _f32(temperature, B, "temperature"), int(seed),
                                 _seeds(row_seeds, B), int(row_offset), int(vocab_offset), _f32(bias, V, "bias"),
                                 mask_ptr, int(stride), _ptr(out_idx), _ptr(out_val), _f32(out_lse, B, "out_lse"),
                                 _ptr(workspace), ws_bytes, _stream_ptr(stream), int(flags))
    _check(st, "flash_sample_full")
    return out_idx, out_val, out_lse


def flash_sample_w8(hidden, W8, w_scale, temperature, seed: int = 0, row_seeds=None, row_offset: int = 0,
                    vocab_offset: int = 0, logits=None, out_idx=None, out_val=None, workspace=None,
                    stream=None, flags: int = 0):
    """Draw on FP8 (E4M3) weights: W8 is a uint8 tensor [V, D], w_scale fp32 [V] or None."""
    import torch
    if hidden.dtype != torch.bfloat16 or W8.dtype != torch.uint8:
        raise ValueError("hidden must be bfloat16 and W8 uint8")
    if hidden.dim() != 2 or W8.dim() != 2 or hidden.shape[1] != W8.shape[1]:
        raise ValueError("hidden must be [B, D] and W8 [V, D]")
    B, D, V = hidden.shape[0], hidden.shape[1], W8.shape[0]
    out_idx, out_val = _outputs(B, hidden.device, out_idx, out_val)
    workspace, ws_bytes = _workspace(B, V, hidden.device, workspace, stream)
    st = lib().flash_sample_w8(_ptr(hidden), _ptr(W8), _f32(w_scale, V, "w_scale"), B, D, V,
                               _f32(temperature, B, "temperature"), int(seed),
                               _seeds(row_seeds, B), int(row_offset), int(vocab_offset), _f32(logits, B * V, "logits"),
                               _ptr(out_idx), _ptr(out_val), _ptr(workspace), ws_bytes, _stream_ptr(stream),
                               int(flags))
    _check(st, "flash_sample_w8")
    return out_idx, out_val


def flash_sample_w4(hidden, W4, w_scales, temperature, seed: int = 0, row_seeds=None, row_offset: int = 0,
                    vocab_offset: int = 0, logits=None, out_idx=None, out_val=None, workspace=None,
                    stream=None, flags: int = 0):
    """Draw on MXFP4 weights: W4 uint8 [V, D/2] (two E2M1 codes per byte), w_scales uint8 [V, D/32]."""
    import torch
    if hidden.dtype != torch.bfloat16 or W4.dtype != torch.uint8 or w_scales.dtype != torch.uint8:
        raise ValueError("hidden must be bfloat16, W4 and w_scales uint8")
    B, D, V = hidden.shape[0], hidden.shape[1], W4.shape[0]
    if W4.dim() != 2 or W4.shape[1] * 2 != D or tuple(w_scales.shape) != (V, D // 32):
        raise ValueError("W4 must be [V, D/2] and w_scales [V, D/32]")
    out_idx, out_val = _outputs(B, hidden.device, out_idx, out_val)
    workspace, ws_bytes = _workspace(B, V, hidden.device, workspace, stream)
    st = lib().flash_sample_w4(_ptr(hidden), _ptr(W4), _ptr(w_scales), B, D, V,
                               _f32(temperature, B, "temperature"), int(seed),
                               _seeds(row_seeds, B), int(row_offset), int(vocab_offset), _f32(logits, B * V, "logits"),
                               _ptr(out_idx), _ptr(out_val), _ptr(workspace), ws_bytes, _stream_ptr(stream),
                               int(flags))
    _check(st, "flash_sample_w4")
    return out_idx, out_val


def flash_sample_mxfp4_decode(codes, scales, out=None, stream=None):
    """codes: uint8 tensor of 4 * n8 bytes (eight codes per dword), scales: uint8 [n8]."""
    import torch
    n8 = scales.numel()
    if out is None:
        out = torch.empty(8 * n8, dtype=torch.float32, device=codes.device)
    _check(lib().flash_sample_mxfp4_decode(_ptr(codes, torch.uint8, 4 * n8, "codes"), _ptr(scales, torch.uint8),
                                           n8, _f32(out, 8 * n8, "out"), _stream_ptr(stream)),
           "flash_sample_mxfp4_decode")
    return out


def flash_sample_e4m3_decode(codes, out=None, stream=None):
    import torch
    n = codes.numel()
    if out is None:
        out = torch.empty(n, dtype=torch.float32, device=codes.device)
    _check(lib().flash_sample_e4m3_decode(_ptr(codes, torch.uint8), n, _f32(out, n, "out"), _stream_ptr(stream)),
           "flash_sample_e4m3_decode")
    return out


FS_GROUPED_PARALLEL, FS_GROUPED_ONLINE = 0, 1
FS_TOPK_TRUNCATE, FS_TOPK_GUMBEL = 0, 1
FS_TOPK_MAX_K = 64


def flash_sample_topk_workspace_bytes(B: int, V: int, k: int) -> int:
    return int(lib().flash_sample_topk_workspace_bytes(int(B), int(V), int(k)))


def flash_sample_topk(hidden, W, temperature, k: int, top_p: float = 1.0, mode: int = FS_TOPK_TRUNCATE, seed: int = 0,
                      row_seeds=None, row_offset: int = 0, vocab_offset: int = 0, fused: bool = True, logits=None,
                      out_idx=None, out_val=None, topk_val=None, topk_idx=None, n_kept=None, workspace=None, stream=None,
                      flags: int = 0):
    """Top-k / nucleus draw (FS_TOPK_TRUNCATE) or Gumbel-top-k (FS_TOPK_GUMBEL).  fused=False runs the
    comparison form over stored logits.  Returns (out_idx, out_val, topk_val [B,k], topk_idx [B,k], n_kept [B])."""
    import torch
    B, D, V = _shapes(hidden, W)
    out_idx, out_val = _outputs(B, hidden.device, out_idx, out_val)
    tv = torch.empty((B, k), dtype=torch.float32, device=hidden.device) if topk_val is None else topk_val
    ti = torch.empty((B, k), dtype=torch.int32, device=hidden.device) if topk_idx is None else topk_idx
    nk = torch.empty(B, dtype=torch.int32, device=hidden.device) if n_kept is None else n_kept
    workspace, ws_bytes = _scratch(flash_sample_topk_workspace_bytes(B, V, k), hidden.device, workspace, stream)
    common = (_ptr(hidden), _ptr(W), B, D, V, _f32(temperature, B, "temperature"), int(seed), _seeds(row_seeds, B),
              int(row_offset), int(vocab_offset), int(k), float(top_p), int(mode))
    tail = (_ptr(out_idx), _ptr(out_val), _ptr(tv), _ptr(ti), _ptr(nk), _ptr(workspace), ws_bytes, _stream_ptr(stream),
            int(flags))
    tail = (tail[0], tail[1], _f32(tv, B * k, "topk_val"), _i32(ti, B * k, "topk_idx"), _i32(nk, B, "n_kept")) + tail[5:]
    if fused:
        st = lib().flash_sample_topk(*common, *tail)
        _check(st, "flash_sample_topk")
    else:
        if logits is None:
            logits = torch.empty((B, V), dtype=torch.float32, device=hidden.device)
        st = lib().flash_sample_topk_unfused(*common, _f32(logits, B * V, "logits"), *tail)
        _check(st, "flash_sample_topk_unfused")
    return out_idx, out_val, tv, ti, nk


def flash_sample_num_groups(V: int, group_tiles: int) -> int:
    return int(lib().flash_sample_num_groups(int(V), int(group_tiles)))


def flash_sample_grouped(hidden, W, temperature, group_tiles: int = 1, mode: int = FS_GROUPED_PARALLEL,
                         seed: int = 0, row_seeds=None, row_offset: int = 0, vocab_offset: int = 0,
                         bias=None, allowed=None, want_groups: bool = False, out_idx=None, out_lse=None,
                         workspace=None, stream=None, flags: int = 0):
    """Grouped draw (groups of 128 * group_tiles ids).  Returns (out_idx, out_lse, group_log_mass,
    group_sample); the last two are [B, m] tensors when want_groups, else None."""
    import torch
    B, D, V = _shapes(hidden, W)
    if out_idx is None:
        out_idx = torch.empty(B, dtype=torch.int32, device=hidden.device)
    if out_lse is None:
        out_lse = torch.empty(B, dtype=torch.float32, device=hidden.device)
    gl = gs = None
    if want_groups:
        m = flash_sample_num_groups(V, group_tiles)
        gl = torch.empty((B, m), dtype=torch.float32, device=hidden.device)
        gs = torch.empty((B, m), dtype=torch.int32, device=hidden.device)
    mask_ptr, stride = _mask_args(allowed, B, V)
    workspace, ws_bytes = _scratch(flash_sample_full_workspace_bytes(B, V), hidden.device, workspace, stream)
    st = lib().flash_sample_grouped(_ptr(hidden), _ptr(W), B, D, V, _f32(temperature, B, "temperature"), int(seed),
                                    _seeds(row_seeds, B), int(row_offset), int(vocab_offset), _f32(bias, V, "bias"),
                                    mask_ptr, int(stride), int(group_tiles), int(mode),
                                    _i32(out_idx, B, "out_idx"), _f32(out_lse, B, "out_lse"), _ptr(gl), _ptr(gs),
                                    _ptr(workspace), ws_bytes, _stream_ptr(stream), int(flags))
    _check(st, "flash_sample_grouped")
    return out_idx, out_lse, gl, gs


def flash_group_choose(group_log_mass, group_sample, mode: int = FS_GROUPED_PARALLEL, seed: int = 0,
                       row_seeds=None, row_offset: int = 0, group_offset: int = 0, out_idx=None,
                       out_lse=None, stream=None):
    """Group choice from per-group (log-mass, sample) pairs, [B, m] each.  Returns (out_idx, out_lse)."""
    import torch
    B, m = group_log_mass.shape
    if out_idx is None:
        out_idx = torch.empty(B, dtype=torch.int32, device=group_log_mass.device)
    if out_lse is None:
        out_lse = torch.empty(B, dtype=torch.float32, device=group_log_mass.device)
    st = lib().flash_group_choose(_f32(group_log_mass, B * m, "group_log_mass"),
                                  _i32(group_sample, B * m, "group_sample"), B, m, int(mode), int(seed),
                                  _seeds(row_seeds, B), int(row_offset), int(group_offset),
                                  _i32(out_idx, B, "out_idx"), _f32(out_lse, B, "out_lse"), _stream_ptr(stream))
    _check(st, "flash_group_choose")
    return out_idx, out_lse


def flash_sample_stage1(hidden, W, temperature, seed: int = 0, row_seeds=None, row_offset: int = 0,
                        vocab_offset: int = 0, cand_val=None, cand_idx=None, logits=None,
                        want_candidates: bool = True, stream=None, flags: int = 0):
    """Stage 1 alone.  Returns (cand_val [B,T] fp32, cand_idx [B,T] int32) (None, None if not wanted)."""
    import torch
    B, D, V = _shapes(hidden, W)
    T = flash_sample_num_tiles(V)
    if want_candidates:
        if cand_val is None:
            cand_val = torch.empty((B, T), dtype=torch.float32, device=hidden.device)
        if cand_idx is None:
            cand_idx = torch.empty((B, T), dtype=torch.int32, device=hidden.device)
    st = lib().flash_sample_stage1(_ptr(hidden), _ptr(W), B, D, V, _f32(temperature, B, "temperature"), int(seed),
                                   _seeds(row_seeds, B), int(row_offset), int(vocab_offset),
                                   _f32(cand_val, B * T, "cand_val"), _i32(cand_idx, B * T, "cand_idx"),
                                   _f32(logits, B * V, "logits"), _stream_ptr(stream), int(flags))
    _check(st, "flash_sample_stage1")
    return cand_val, cand_idx


def flash_sample_stage2(cand_val, cand_idx, out_idx=None, out_val=None, stream=None):
    B, T = cand_val.shape
    out_idx, out_val = _outputs(B, cand_val.device, out_idx, out_val)
    st = lib().flash_sample_stage2(_f32(cand_val, B * T, "cand_val"), _i32(cand_idx, B * T, "cand_idx"), B, T,
                                   _ptr(out_idx), _ptr(out_val), _stream_ptr(stream))
    _check(st, "flash_sample_stage2")
    return out_idx, out_val


def flash_sample_unfused(hidden, W, temperature, seed: int = 0, row_seeds=None, row_offset: int = 0,
                         vocab_offset: int = 0, logits=None, out_idx=None, out_val=None,
                         workspace=None, stream=None, flags: int = 0):
    import torch
    B, D, V = _shapes(hidden, W)
    if logits is None:
        logits = torch.empty((B, V), dtype=torch.float32, device=hidden.device)
    out_idx, out_val = _outputs(B, hidden.device, out_idx, out_val)
    workspace, ws_bytes = _workspace(B, V, hidden.device, workspace, stream)
    st = lib().flash_sample_unfused(_ptr(hidden), _ptr(W), B, D, V, _f32(temperature, B, "temperature"), int(seed),
                                    _seeds(row_seeds, B), int(row_offset), int(vocab_offset),
                                    _f32(logits, B * V, "logits"),
                                    _ptr(out_idx), _ptr(out_val), _ptr(workspace), ws_bytes,
                                    _stream_ptr(stream), int(flags))
    _check(st, "flash_sample_unfused")
    return out_idx, out_val, logits


def flash_lm_head_logits(hidden, W, logits=None, stream=None, flags: int = 0):
    import torch
    B, D, V = _shapes(hidden, W)
    if logits is None:
        logits = torch.empty((B, V), dtype=torch.float32, device=hidden.device)
    st = lib().flash_lm_head_logits(_ptr(hidden), _ptr(W), B, D, V, _f32(logits, B * V, "logits"),
                                    _stream_ptr(stream), int(flags))
    _check(st, "flash_lm_head_logits")
    return logits


def flash_gumbel_argmax_logits(logits, temperature, seed: int = 0, row_seeds=None, row_offset: int = 0,
                               vocab_offset: int = 0, out_idx=None, out_val=None, workspace=None,
                               stream=None):
    B, V = logits.shape
    out_idx, out_val = _outputs(B, logits.device, out_idx, out_val)
    workspace, ws_bytes = _workspace(B, V, logits.device, workspace, stream)
    st = lib().flash_gumbel_argmax_logits(_f32(logits, B * V, "logits"), B, V, _f32(temperature, B, "temperature"),
                                          int(seed), _seeds(row_seeds, B), int(row_offset), int(vocab_offset),
                                          _ptr(out_idx), _ptr(out_val), _ptr(workspace), ws_bytes,
                                          _stream_ptr(stream))
    _check(st, "flash_gumbel_argmax_logits")
    return out_idx, out_val


def flash_sample_noise(seed: int, row: int, v0: int, n: int, device="cuda", stream=None):
    import torch
    g = torch.empty(n, dtype=torch.float32, device=device)
    st = lib().flash_sample_noise(int(seed), int(row), int(v0), int(n), _ptr(g), _stream_ptr(stream))
    _check(st, "flash_sample_noise")
    return g


def flash_sample_gumbel_transform(words, stream=None, flags: int = 0):
    import torch
    g = torch.empty(words.numel(), dtype=torch.float32, device=words.device)
    st = lib().flash_sample_gumbel_transform(_ptr(words, (torch.int32, torch.uint32), None, "words"), words.numel(),
                                             _ptr(g), _stream_ptr(stream), int(flags))
    _check(st, "flash_sample_gumbel_transform")
    return g
