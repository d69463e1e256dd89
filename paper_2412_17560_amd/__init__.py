"""MI355X-native GQSA group-sparse, group-quantised GEMV (paper Sec. 3.2, 3.5).

Thin ctypes binding over libgqsa.so (C ABI declared in include/gqsa.h).  The
binding only marshals arguments: every step of the hot path runs in the HIP
kernels.  PyTorch is used by callers for device memory and streams only.
"""
from .binding import (  # noqa: F401
    GqsaError,
    GqsaHandle,
    gqsa_copy,
    gqsa_default_partition,
    gqsa_dense_f16_gemv,
    gqsa_export,
    gqsa_build_panels,
    gqsa_export_device_blob,
    gqsa_export_panel_blob,
    gqsa_free,
    gqsa_gemv,
    gqsa_gemv_multi,
    gqsa_gemv_static,
    gqsa_import,
    gqsa_info,
    gqsa_launch_floor,
    gqsa_load,
    gqsa_pack,
    gqsa_pack_device,
    gqsa_pack_hessian,
    gqsa_pack_rows,
    gqsa_partition,
    gqsa_save,
    gqsa_set_partition,
    gqsa_set_partition_aligned,
    gqsa_set_partition_rows,
    gqsa_status_string,
    gqsa_stream_read,
    gqsa_stream_read_workgroups,
    gqsa_upload,
    library_path,
)
