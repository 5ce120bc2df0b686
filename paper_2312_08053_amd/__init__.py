"""MI355X-native Kimad+ compression step: thin ctypes binding over libkimad.so.

All arithmetic of the method runs in the HIP kernels behind the C ABI of
``include/kimad.h``; this package only marshals arguments.  PyTorch supplies
device memory and the stream.  There is no CPU fallback: a missing library is an
error.
"""
from .binding import (KimadError, Plan, lib, kimad_workspace_bytes, kimad_plan_create,
                      kimad_plan_destroy, kimad_profile, kimad_allocate, kimad_allocate_static, kimad_compress_ef,
                      kimad_step, kimad_error_at, kimad_uniform_sizes, kimad_payload_layer_counts, kimad_server_apply, kimad_budget_bytes, kimad_strerror, kimad_version, KIMAD_REUSE_PROFILE,
                      KIMAD_CFG_CLASSIC_PROFILE,
                      EXPORTED_SYMBOLS, LIB_PATH)

__all__ = ["KimadError", "Plan", "lib", "kimad_workspace_bytes", "kimad_plan_create",
           "kimad_plan_destroy", "kimad_profile", "kimad_allocate", "kimad_allocate_static", "kimad_compress_ef",
           "kimad_step", "kimad_error_at", "kimad_uniform_sizes", "kimad_payload_layer_counts", "kimad_server_apply", "kimad_budget_bytes", "kimad_strerror", "kimad_version", "KIMAD_REUSE_PROFILE", "KIMAD_CFG_CLASSIC_PROFILE",
           "EXPORTED_SYMBOLS", "LIB_PATH"]
