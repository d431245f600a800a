"""Streaming-rollout frame update on MI355X: thin Python binding over libsr.so.

Every step of the path runs in the library's HIP kernels; this package only
marshals arguments.  PyTorch is used for device memory and streams."""
from .binding import (SrError, SrGraph, analyze, count_valid_patterns, tableau, equally_model_parallel,  # noqa: F401
                      pattern_count_bounds, lib_path, load_library, SR_F32, SR_BF16, EXPORTS)
