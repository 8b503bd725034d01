"""PQk-means iteration on AMD MI355X: thin Python binding over the C ABI of libpqkm.so.

The functions here carry the names of the C entry points (include/pqkm.h) and only marshal
arguments: torch tensors supply device memory, the current torch stream supplies the HIP
stream.  Every step of the path runs in the library's HIP kernels; there is no CPU fallback
-- a missing library raises at import of the first call.
"""
from .binding import (NOALLOC_SCRATCH_BYTES, PqkmError, assign, assign_indexed, assign_noalloc, check, build_tables, decode, encode, fit, fit_until, fit_until_workspace_bytes, lib_path, load, profile_read, profile_read_steps, set_option,
                      status_string, update, update_naive, workspace_bytes)

__all__ = ["NOALLOC_SCRATCH_BYTES", "PqkmError", "assign", "assign_indexed", "assign_noalloc", "check", "build_tables", "decode", "encode", "fit", "fit_until", "fit_until_workspace_bytes", "lib_path", "load", "profile_read", "profile_read_steps", "set_option",
           "status_string", "update", "update_naive", "workspace_bytes"]
