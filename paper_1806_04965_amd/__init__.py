"""Streaming-rollout frame update on MI355X: thin Python binding over libsr.so.

Every step of the path runs in the library's HIP kernels; this package only
marshals arguments.  PyTorch is used for device memory and streams."""
from .binding import (SrError, SrGraph, analyze, count_valid_patterns, lib_path, load_library,  # noqa: F401
                      SR_F32, SR_BF16, EXPORTS)
