"""Sparse ternary GEMM  Y = X W + b  (W in {-1,0,+1}, TCSC format) for one AMD MI355X.

Python binding of libtstgemm.so: argument marshalling only, every step of the computation
runs in the HIP library.  PyTorch supplies device memory and streams.
"""
from .binding import (TstgemmError, Tcsc, library_path, tcsc_build, tcsc_from_arrays, tcsc_to_dense, tcsc_dims,
                      tcsc_arrays, tcsc_device_bytes, tcsc_layout, tcsc_upload, tstgemm, tstgemm_signed, tstgemm_packed, tcsc_signed_arrays, tcsc_packed_codes,
                      tcsc_select_forms, tstgemm_workspace_bytes, tstgemm_noalloc, NOALLOC_SCRATCH_BYTES, tstgemm_probe_lds_read,
                      tstgemm_probe_stream_read, tstgemm_probe_tile_copy, tcsc_destroy, tcsc_strerror,
                      FORM_ROWSETS, FORM_CUTS, FORM_LISTS16, FORM_SIGNED, FORM_PACKED, FORM_WORKSPACE, FORM_ALL)

__all__ = ["TstgemmError", "Tcsc", "library_path", "tcsc_build", "tcsc_from_arrays", "tcsc_to_dense", "tcsc_dims",
           "tcsc_arrays", "tcsc_device_bytes", "tcsc_layout", "tcsc_upload", "tstgemm", "tstgemm_signed", "tstgemm_packed",
           "tcsc_signed_arrays", "tcsc_packed_codes", "tcsc_select_forms", "tstgemm_workspace_bytes", "tstgemm_noalloc", "NOALLOC_SCRATCH_BYTES",
           "tstgemm_probe_lds_read", "tstgemm_probe_stream_read", "tstgemm_probe_tile_copy", "tcsc_destroy", "tcsc_strerror",
           "FORM_ROWSETS", "FORM_CUTS", "FORM_LISTS16", "FORM_SIGNED", "FORM_PACKED", "FORM_WORKSPACE", "FORM_ALL"]
