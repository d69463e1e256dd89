"""ctypes marshalling for libgqsa.so -- same names as the C ABI, no arithmetic here."""
from __future__ import annotations

import ctypes as C
import os

import numpy as np

from . import build as _build

_LIB = None


class GqsaError(RuntimeError):
    def __init__(self, status: int, what: str):
        super().__init__(f"{what}: {gqsa_status_string(status)} (status {status})")
        self.status = status


class _Info(C.Structure):
    _fields_ = [("N", C.c_int64), ("K", C.c_int64), ("G", C.c_int32), ("bits", C.c_int32),
                ("nnz_groups", C.c_int64), ("values_bytes", C.c_int64), ("n_blocks", C.c_int64),
                ("n_workgroups", C.c_int32), ("waves_per_workgroup", C.c_int32),
                ("needs_fixup", C.c_int32), ("span_tiles", C.c_int32), ("n_empty_rows", C.c_int64),
                ("device_bytes", C.c_int64), ("algorithmic_bytes", C.c_int64),
                ("on_device", C.c_int32), ("panel_integer_zeros", C.c_int32), ("panel_bytes", C.c_int64),
                ("tile_blocks", C.c_int32), ("tile_lanes", C.c_int32), ("span_per_worker", C.c_int32),
                ("reserved0", C.c_int32)]


def library_path() -> str:
    return _build.LIB


def _lib():
    global _LIB
    if _LIB is not None:
        return _LIB
    # PyTorch ships its own HIP runtime (same SONAME as the system one).  Streams and device
    # pointers handed to libgqsa come from PyTorch, so both must live in ONE runtime: import
    # torch first, and the loader resolves libgqsa's libamdhip64 to the copy already mapped.
    # (A host-only build named by GQSA_LIBRARY has no HIP runtime to share.)
    if not _build.HOST_ONLY:
        import torch  # noqa: F401
    path = _build.LIB
    if not os.path.exists(path):
        _build.build()           # nothing built yet: build once, in-tree
    if not os.path.exists(path):
        raise ImportError(f"libgqsa.so is missing at {path}; run `python -m paper_2412_17560_amd.build`")
    lib = C.CDLL(path)
    vp, i64, i32 = C.c_void_p, C.c_int64, C.c_int
    lib.gqsa_pack.restype = C.c_int
    lib.gqsa_pack.argtypes = [vp, i64, i64, i32, i32, C.c_double, C.POINTER(vp)]
    lib.gqsa_pack_rows.restype = C.c_int
    lib.gqsa_pack_rows.argtypes = [vp, i64, i64, i32, i32, vp, C.POINTER(vp)]
    lib.gqsa_pack_hessian.restype = C.c_int
    lib.gqsa_pack_hessian.argtypes = [vp, i64, i64, i32, i32, C.c_double, vp, C.POINTER(vp)]
    lib.gqsa_pack_device.restype = C.c_int
    lib.gqsa_pack_device.argtypes = [vp, i64, i64, i32, i32, C.c_double, vp, vp, vp, C.POINTER(vp)]
    lib.gqsa_save.restype = C.c_int
    lib.gqsa_save.argtypes = [vp, C.c_char_p]
    lib.gqsa_load.restype = C.c_int
    lib.gqsa_load.argtypes = [C.c_char_p, C.POINTER(vp)]
    lib.gqsa_import.restype = C.c_int
    lib.gqsa_import.argtypes = [vp, vp, vp, vp, vp, i64, i64, i32, i32, C.POINTER(vp)]
    lib.gqsa_set_partition.restype = C.c_int
    lib.gqsa_set_partition.argtypes = [vp, i32, i32]
    lib.gqsa_build_panels.restype = C.c_int
    lib.gqsa_build_panels.argtypes = [vp]
    lib.gqsa_export_panel_blob.restype = C.c_int
    lib.gqsa_export_panel_blob.argtypes = [vp, vp, C.c_size_t]
    lib.gqsa_set_partition_aligned.restype = C.c_int
    lib.gqsa_set_partition_aligned.argtypes = [vp, i32, i32, i32]
    lib.gqsa_upload.restype = C.c_int
    lib.gqsa_upload.argtypes = [vp]
    lib.gqsa_gemv.restype = C.c_int
    lib.gqsa_gemv.argtypes = [vp, vp, vp, i32, vp]
    lib.gqsa_gemv_static.restype = C.c_int
    lib.gqsa_gemv_static.argtypes = [vp, vp, vp, i32, vp]
    lib.gqsa_default_partition.restype = C.c_int
    lib.gqsa_default_partition.argtypes = [vp, i64, i64, i32, i32, C.POINTER(C.c_int32 * 6)]
    lib.gqsa_set_partition_rows.restype = C.c_int
    lib.gqsa_set_partition_rows.argtypes = [vp, i32, i32, i32, i32, i32]
    lib.gqsa_gemv_panels.restype = C.c_int
    lib.gqsa_gemv_panels.argtypes = [vp, vp, vp, i32, vp]
    lib.gqsa_gemv_multi.restype = C.c_int
    lib.gqsa_gemv_multi.argtypes = [C.POINTER(vp), i32, vp, C.POINTER(vp), i32, vp]
    lib.gqsa_info.restype = C.c_int
    lib.gqsa_info.argtypes = [vp, C.POINTER(_Info)]
    lib.gqsa_export.restype = C.c_int
    lib.gqsa_export.argtypes = [vp, vp, vp, vp, vp, vp]
    lib.gqsa_export_device_blob.restype = C.c_int
    lib.gqsa_export_device_blob.argtypes = [vp, vp, C.c_size_t]
    lib.gqsa_free.restype = None
    lib.gqsa_free.argtypes = [vp]
    lib.gqsa_status_string.restype = C.c_char_p
    lib.gqsa_status_string.argtypes = [C.c_int]
    lib.gqsa_dense_f16_gemv.restype = C.c_int
    lib.gqsa_dense_f16_gemv.argtypes = [vp, vp, vp, i64, i64, i32, vp]
    lib.gqsa_stream_read.restype = C.c_int
    lib.gqsa_stream_read.argtypes = [vp, C.c_size_t, vp, vp]
    lib.gqsa_copy.restype = C.c_int
    lib.gqsa_copy.argtypes = [vp, vp, C.c_size_t, vp]
    lib.gqsa_launch_floor.restype = C.c_int
    lib.gqsa_launch_floor.argtypes = [i32, i32, vp, vp]
    lib.gqsa_stream_read_workgroups.restype = C.c_int
    lib.gqsa_stream_read_workgroups.argtypes = []
    _LIB = lib
    return lib


def gqsa_status_string(status: int) -> str:
    return _lib().gqsa_status_string(int(status)).decode()


def _check(status: int, what: str):
    if status != 0:
        raise GqsaError(status, what)


class GqsaHandle:
    """Owns one gqsa_handle_t; freed on gqsa_free() or garbage collection."""

    def __init__(self, ptr: int):
        self.ptr = C.c_void_p(ptr)

    def __del__(self):
        try:
            gqsa_free(self)
        except Exception:
            pass


def _np_ptr(a):
    return None if a is None else C.c_void_p(a.ctypes.data)


def gqsa_pack(W: np.ndarray, G: int = 16, bits: int = 4, sparsity: float = 0.5) -> GqsaHandle:
    W = np.ascontiguousarray(W, dtype=np.float32)
    if W.ndim != 2:
        raise ValueError("W must be [N, K]")
    out = C.c_void_p()
    _check(_lib().gqsa_pack(_np_ptr(W), W.shape[0], W.shape[1], G, bits, float(sparsity),
                            C.byref(out)), "gqsa_pack")
    return GqsaHandle(out.value)


def gqsa_pack_hessian(W: np.ndarray, hinv_diag: np.ndarray, G: int = 16, bits: int = 4,
                      sparsity: float = 0.5) -> GqsaHandle:
    W = np.ascontiguousarray(W, dtype=np.float32)
    d = np.ascontiguousarray(hinv_diag, dtype=np.float32)
    if W.ndim != 2 or d.shape != (W.shape[1],):
        raise ValueError("W must be [N, K] and hinv_diag [K]")
    out = C.c_void_p()
    _check(_lib().gqsa_pack_hessian(_np_ptr(W), W.shape[0], W.shape[1], G, bits, float(sparsity),
                                    _np_ptr(d), C.byref(out)), "gqsa_pack_hessian")
    return GqsaHandle(out.value)


def gqsa_pack_device(W, G: int = 16, bits: int = 4, sparsity: float = 0.5, keep_per_row=None, hinv_diag=None,
                     stream=None) -> GqsaHandle:
    """gqsa_pack / gqsa_pack_rows / gqsa_pack_hessian on the GPU: W a float32 device tensor [N, K],
    hinv_diag a float32 device tensor [K] or None, keep_per_row a host int32 array [N] or None."""
    if W.dim() != 2:
        raise ValueError("W must be [N, K]")
    keep = None
    if keep_per_row is not None:
        keep = np.ascontiguousarray(keep_per_row, dtype=np.int32)
        if keep.shape != (W.shape[0],):
            raise ValueError("keep_per_row must be [N]")
    if hinv_diag is not None and tuple(hinv_diag.shape) != (W.shape[1],):
        raise ValueError("hinv_diag must be [K]")
    out = C.c_void_p()
    _check(_lib().gqsa_pack_device(_dev_ptr(W, "torch.float32", "W"), W.shape[0], W.shape[1], G, bits, float(sparsity),
                                   _np_ptr(keep) if keep is not None else None,
                                   _dev_ptr(hinv_diag, "torch.float32", "hinv_diag") if hinv_diag is not None else None,
                                   _stream_ptr(stream), C.byref(out)), "gqsa_pack_device")
    return GqsaHandle(out.value)


def gqsa_save(h: GqsaHandle, path: str) -> None:
    _check(_lib().gqsa_save(h.ptr, os.fsencode(path)), "gqsa_save")


def gqsa_load(path: str) -> GqsaHandle:
    out = C.c_void_p()
    _check(_lib().gqsa_load(os.fsencode(path), C.byref(out)), "gqsa_load")
    return GqsaHandle(out.value)


def gqsa_pack_rows(W: np.ndarray, keep_per_row: np.ndarray, G: int = 16, bits: int = 4) -> GqsaHandle:
    W = np.ascontiguousarray(W, dtype=np.float32)
    keep = np.ascontiguousarray(keep_per_row, dtype=np.int32)
    if W.ndim != 2 or keep.shape != (W.shape[0],):
        raise ValueError("W must be [N, K] and keep_per_row [N]")
    out = C.c_void_p()
    _check(_lib().gqsa_pack_rows(_np_ptr(W), W.shape[0], W.shape[1], G, bits, _np_ptr(keep),
                                 C.byref(out)), "gqsa_pack_rows")
    return GqsaHandle(out.value)


def gqsa_import(rowIndex, groups, values, scales_f16, zeros_f16, N: int, K: int, G: int = 16,
                bits: int = 4) -> GqsaHandle:
    ri = np.ascontiguousarray(rowIndex, dtype=np.int32)
    gr = np.ascontiguousarray(groups, dtype=np.int32)
    va = np.ascontiguousarray(values, dtype=np.uint8)
    sc = np.ascontiguousarray(scales_f16, dtype=np.uint16)
    ze = np.ascontiguousarray(zeros_f16, dtype=np.uint16)
    if ri.shape != (N + 1,):
        raise ValueError("rowIndex must have N+1 entries")
    nnz = int(ri[-1])
    if gr.size != nnz or sc.size != nnz or ze.size != nnz or va.size != nnz * G * bits // 8:
        raise ValueError("array sizes do not match rowIndex[N]")
    out = C.c_void_p()
    _check(_lib().gqsa_import(_np_ptr(ri), _np_ptr(gr), _np_ptr(va), _np_ptr(sc), _np_ptr(ze),
                              N, K, G, bits, C.byref(out)), "gqsa_import")
    return GqsaHandle(out.value)


def gqsa_set_partition(h: GqsaHandle, n_workgroups: int, waves_per_workgroup: int = 16) -> None:
    _check(_lib().gqsa_set_partition(h.ptr, int(n_workgroups), int(waves_per_workgroup)),
           "gqsa_set_partition")


def gqsa_set_partition_aligned(h: GqsaHandle, span_tiles: int, n_workgroups: int = 0,
                               waves_per_workgroup: int = 4) -> None:
    _check(_lib().gqsa_set_partition_aligned(h.ptr, int(span_tiles), int(n_workgroups), int(waves_per_workgroup)),
           "gqsa_set_partition_aligned")


def gqsa_set_partition_rows(h: GqsaHandle, tile_blocks: int, tile_lanes: int = 64, tiles_per_worker: int = 1,
                            n_workgroups: int = 0, waves_per_workgroup: int = 4) -> None:
    _check(_lib().gqsa_set_partition_rows(h.ptr, int(tile_blocks), int(tile_lanes), int(tiles_per_worker),
                                          int(n_workgroups), int(waves_per_workgroup)), "gqsa_set_partition_rows")


def gqsa_build_panels(h: GqsaHandle) -> None:
    _check(_lib().gqsa_build_panels(h.ptr), "gqsa_build_panels")


def gqsa_export_panel_blob(h: GqsaHandle) -> bytes:
    n = gqsa_info(h)["panel_bytes"]
    buf = np.zeros(max(n, 1), dtype=np.uint8)
    _check(_lib().gqsa_export_panel_blob(h.ptr, _np_ptr(buf), n), "gqsa_export_panel_blob")
    return buf[:n].tobytes()


def gqsa_upload(h: GqsaHandle) -> None:
    _check(_lib().gqsa_upload(h.ptr), "gqsa_upload")


def gqsa_info(h: GqsaHandle) -> dict:
    info = _Info()
    _check(_lib().gqsa_info(h.ptr, C.byref(info)), "gqsa_info")
    return {name: getattr(info, name) for name, _ in _Info._fields_ if not name.startswith("reserved")}


def gqsa_export(h: GqsaHandle) -> dict:
    info = gqsa_info(h)
    nnz = info["nnz_groups"]
    ri = np.zeros(info["N"] + 1, dtype=np.int32)
    gr = np.zeros(nnz, dtype=np.int32)
    va = np.zeros(info["values_bytes"], dtype=np.uint8)
    sc = np.zeros(nnz, dtype=np.uint16)
    ze = np.zeros(nnz, dtype=np.uint16)
    _check(_lib().gqsa_export(h.ptr, _np_ptr(ri), _np_ptr(gr) if nnz else None,
                              _np_ptr(va) if nnz else None, _np_ptr(sc) if nnz else None,
                              _np_ptr(ze) if nnz else None), "gqsa_export")
    return {"rowIndex": ri, "groups": gr, "values": va, "scales": sc, "zeros": ze}


def gqsa_export_device_blob(h: GqsaHandle) -> bytes:
    n = gqsa_info(h)["device_bytes"]
    buf = np.zeros(n, dtype=np.uint8)
    _check(_lib().gqsa_export_device_blob(h.ptr, _np_ptr(buf), n), "gqsa_export_device_blob")
    return buf.tobytes()


def gqsa_free(h: GqsaHandle) -> None:
    if h.ptr is not None and h.ptr.value:
        _lib().gqsa_free(h.ptr)
        h.ptr = C.c_void_p()


def _stream_ptr(stream):
    if stream is None:
        import torch
        stream = torch.cuda.current_stream()
    return C.c_void_p(getattr(stream, "cuda_stream", stream))


def _dev_ptr(t, dtype_name: str, what: str):
    import torch
    if not isinstance(t, torch.Tensor) or not t.is_cuda or not t.is_contiguous():
        raise ValueError(f"{what} must be a contiguous device tensor")
    if str(t.dtype) != dtype_name:
        raise ValueError(f"{what} must be {dtype_name}")
    return C.c_void_p(t.data_ptr())


def gqsa_default_partition(rowIndex, K: int, G: int = 16, bits: int = 4):
    """(n_workgroups, waves_per_workgroup, span_tiles, tile_blocks, tile_lanes, span_per_worker) the library would
    choose for these row pointers."""
    ri = np.ascontiguousarray(rowIndex, dtype=np.int32)
    out = (C.c_int32 * 6)()
    _check(_lib().gqsa_default_partition(C.c_void_p(ri.ctypes.data), ri.size - 1, K, G, bits, C.byref(out)),
           "gqsa_default_partition")
    return tuple(int(v) for v in out)


def gqsa_partition(h: GqsaHandle):
    """The handle's partition, in the order of gqsa_default_partition."""
    info = gqsa_info(h)
    return tuple(info[k] for k in ("n_workgroups", "waves_per_workgroup", "span_tiles", "tile_blocks", "tile_lanes",
                                   "span_per_worker"))


def gqsa_gemv_static(h: GqsaHandle, x, y, stream=None):
    """gqsa_gemv without any allocation: y must be given, the handle must be on the device."""
    info = gqsa_info(h)
    if x.dim() != 2 or x.shape[1] != info["K"] or tuple(y.shape) != (x.shape[0], info["N"]):
        raise ValueError("x must be [batch, K] and y [batch, N]")
    _check(_lib().gqsa_gemv_static(h.ptr, _dev_ptr(x, "torch.float16", "x"), _dev_ptr(y, "torch.float16", "y"),
                                   x.shape[0], _stream_ptr(stream)), "gqsa_gemv_static")
    return y


def gqsa_gemv(h: GqsaHandle, x, y=None, stream=None, panels: bool = False):
    """y[batch,N] (fp16, device) = W^ x[batch,K]; enqueues on `stream` (default: torch's current).
    panels=True: gqsa_gemv_panels (the second image, whatever the batch)."""
    import torch
    info = gqsa_info(h)
    if x.dim() == 1:
        x = x.unsqueeze(0)
    batch = x.shape[0]
    if x.shape[1] != info["K"]:
        raise ValueError("x must be [batch, K]")
    if y is None:
        y = torch.empty((batch, info["N"]), dtype=torch.float16, device=x.device)
    if tuple(y.shape) != (batch, info["N"]):
        raise ValueError("y must be [batch, N]")
    fn = _lib().gqsa_gemv_panels if panels else _lib().gqsa_gemv
    _check(fn(h.ptr, _dev_ptr(x, "torch.float16", "x"), _dev_ptr(y, "torch.float16", "y"), batch,
              _stream_ptr(stream)), "gqsa_gemv_panels" if panels else "gqsa_gemv")
    return y


def gqsa_gemv_multi(hs, x, ys=None, stream=None):
    """ys[i][batch,N_i] = W^_i x for several matrices sharing x, in one launch."""
    import torch
    infos = [gqsa_info(h) for h in hs]
    if x.dim() == 1:
        x = x.unsqueeze(0)
    batch = x.shape[0]
    if any(x.shape[1] != inf["K"] for inf in infos):
        raise ValueError("x must be [batch, K] for every matrix")
    if ys is None:
        ys = [torch.empty((batch, inf["N"]), dtype=torch.float16, device=x.device) for inf in infos]
    if len(ys) != len(hs) or any(tuple(y.shape) != (batch, inf["N"]) for y, inf in zip(ys, infos)):
        raise ValueError("ys[i] must be [batch, N_i]")
    n = len(hs)
    harr = (C.c_void_p * n)(*[h.ptr.value for h in hs])
    yarr = (C.c_void_p * n)(*[_dev_ptr(y, "torch.float16", "y").value for y in ys])
    _check(_lib().gqsa_gemv_multi(harr, n, _dev_ptr(x, "torch.float16", "x"), yarr, batch,
                                  _stream_ptr(stream)), "gqsa_gemv_multi")
    return ys


def gqsa_dense_f16_gemv(W, x, y=None, stream=None):
    import torch
    if x.dim() == 1:
        x = x.unsqueeze(0)
    N, K = W.shape
    batch = x.shape[0]
    if y is None:
        y = torch.empty((batch, N), dtype=torch.float16, device=x.device)
    _check(_lib().gqsa_dense_f16_gemv(_dev_ptr(W, "torch.float16", "W"),
                                      _dev_ptr(x, "torch.float16", "x"),
                                      _dev_ptr(y, "torch.float16", "y"), N, K, batch,
                                      _stream_ptr(stream)), "gqsa_dense_f16_gemv")
    return y


def gqsa_stream_read_workgroups() -> int:
    return int(_lib().gqsa_stream_read_workgroups())


def gqsa_copy(dst, src, stream=None) -> None:
    nbytes = src.numel() * src.element_size()
    if dst.numel() * dst.element_size() != nbytes:
        raise ValueError("dst and src must have the same size")
    _check(_lib().gqsa_copy(C.c_void_p(dst.data_ptr()), C.c_void_p(src.data_ptr()), nbytes,
                            _stream_ptr(stream)), "gqsa_copy")


def gqsa_launch_floor(n_workgroups: int, lds_bytes: int, sink, stream=None) -> None:
    _check(_lib().gqsa_launch_floor(int(n_workgroups), int(lds_bytes), C.c_void_p(sink.data_ptr()),
                                    _stream_ptr(stream)), "gqsa_launch_floor")


def gqsa_stream_read(buf, sink, stream=None) -> None:
    nbytes = buf.numel() * buf.element_size()
    _check(_lib().gqsa_stream_read(C.c_void_p(buf.data_ptr()), nbytes, C.c_void_p(sink.data_ptr()),
                                   _stream_ptr(stream)), "gqsa_stream_read")
