"""Grouped per-label DC-CGAN training step on gfx950: thin ctypes binding over the C-ABI library."""
from .binding import (GanConfig, Gan, GanError, lib_path, load_library, FP32, BF16, make_config)  # noqa: F401
