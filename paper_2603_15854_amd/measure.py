"""Binding of ``include/flash_sample_measure.h``: measurement aids that live in the same shared
library as the sampler but are no part of the method (argument marshalling only)."""
from __future__ import annotations

from . import _check, _ptr, _stream_ptr, lib


def flash_measure_kernel_choice(B: int, D: int, V: int, compute_units: int = 256) -> int:
    return int(lib().flash_measure_kernel_choice(int(B), int(D), int(V), int(compute_units)))


def flash_measure_stream_probe(src, dst=None, sink=None, stream=None) -> None:
    nbytes = src.numel() * src.element_size()
    st = lib().flash_measure_stream_probe(_ptr(dst), _ptr(src), nbytes, _ptr(sink), _stream_ptr(stream))
    _check(st, "flash_measure_stream_probe")
