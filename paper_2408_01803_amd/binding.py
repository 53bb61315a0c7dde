"""ctypes binding of libstb (include/stb.h).  Argument marshalling only: every step of the path runs
inside the library.  The functions carry the names of the C entry points; `PackedMatrix` is a small
holder for a packed image on the host and its copy in HBM.

PyTorch is used for device memory and streams only.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional, Sequence

import numpy as np

_PKG = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_PKG, "libstb.so")

STB_BLOCK = 128
STB_MAX_BATCH = 32
STB_PLANE_ALIGN = 256

STB_OK, STB_EINVAL, STB_ENULL, STB_EALIGN, STB_ENONFINITE, STB_EHIP, STB_EUNSUPPORTED, STB_ETOOBIG = 0, -1, -2, -3, -4, -5, -6, -7
STB_GEMV_STATIC_SCRATCH_BYTES = 8 * 1024 * 1024


class StbError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        msg = _lib().stb_strerror(status).decode() if _LIB is not None else str(status)
        if status == STB_EHIP:
            msg += f" [hip error {_lib().stb_last_hip_error()}]"
        super().__init__(f"{where}: {msg} ({status})")


class stb_cfg_t(C.Structure):
    _fields_ = [("n_out", C.c_int32), ("k_in", C.c_int32), ("N", C.c_int32), ("M", C.c_int32),
                ("block", C.c_int32), ("n_salient", C.c_int32), ("region_mode", C.c_int32)]


class stb_layout_t(C.Structure):
    _fields_ = (
        [("cfg", stb_cfg_t)]
        + [(name, C.c_int32) for name in (
            "n_salient_pad", "n_blocks", "kind", "n_row_tiles", "n_super", "sal_chunks", "max_sal_block",
            "max_sal_half")]
        + [(name, C.c_int64) for name in (
            "mask_stride", "sign_stride", "region_stride", "res_stride",
            "mask_bytes", "sign_bytes", "region_bytes", "res_bytes",
            "scales_bytes", "res_scale_bytes", "salmap_bytes", "salprefix_bytes", "saltab_bytes",
            "total_bytes",
            "off_mask", "off_sign", "off_region", "off_res", "off_scales", "off_res_scale",
            "off_salmap", "off_salprefix", "off_saltab",
            "image_bytes")]
        + [(name, C.c_void_p) for name in (
            "mask", "sign", "region", "res_sign", "sal_bitmap", "sal_block_prefix", "sal_tab",
            "scales", "res_scale")]
        + [("res_t_bytes", C.c_int64), ("off_res_t", C.c_int64), ("res_t", C.c_void_p)]
    )


STB_KIND_ROWMAJOR, STB_KIND_TILED = 0, 1

PLANE_FIELDS = (("mask", "off_mask", "mask_bytes"), ("sign", "off_sign", "sign_bytes"),
                ("region", "off_region", "region_bytes"), ("res_sign", "off_res", "res_bytes"),
                ("scales", "off_scales", "scales_bytes"), ("res_scale", "off_res_scale", "res_scale_bytes"),
                ("sal_bitmap", "off_salmap", "salmap_bytes"),
                ("sal_block_prefix", "off_salprefix", "salprefix_bytes"))

_LIB = None

EXPORTS = ("stb_layout_sizes", "stb_layout_bind", "stb_tiled_sizes", "stb_tile", "stb_untile", "stb_tile_device", "stb_pack", "stb_pack_obc", "stb_hessian_factor", "stb_pack_obc_hybrid", "stb_pack_obc_hybrid_workspace_bytes", "stb_pack_device", "stb_pack_device_workspace_bytes", "stb_unpack", "stb_salient_columns", "stb_salient_columns_hc", "stb_layer_l2_norm", "stb_layer_nm_assignment", "stb_code24_export", "stb_code24_import", "stb_code24_index", "stb_dequant", "stb_gemv",
           "stb_gemv_static", "stb_gemv_workspace_bytes", "stb_gemv_batched", "stb_gemv_batched_workspace_bytes", "stb_gemm", "stb_gemm_workspace_bytes", "stb_probe_read", "stb_probe_mfma", "stb_set_kernel_override", "stb_strerror", "stb_last_hip_error")


def _lib():
    """Loads libstb.so.  There is no fallback: a missing library is an error."""
    global _LIB
    if _LIB is not None:
        return _LIB
    if not os.path.exists(LIB_PATH):
        raise ImportError(f"{LIB_PATH} is missing: run `python -c 'import __graft_entry__ as g; g.build()'` "
                          "(or paper_2408_01803_amd/build.py) first")
    # The device tensors that callers pass come from PyTorch, whose wheel carries its own copy of the HIP runtime.  It
    # has to be in the process before this library is, so that the library's kernels resolve to that same runtime
    # (loaded the other way round, two runtimes coexist and every launch fails with "no device").
    try:
        import torch  # noqa: F401
    except ImportError:
        pass
    lib = C.CDLL(LIB_PATH)
    P = C.POINTER
    lib.stb_layout_sizes.argtypes = [P(stb_cfg_t), P(stb_layout_t)]
    lib.stb_layout_bind.argtypes = [P(stb_layout_t), C.c_void_p]
    lib.stb_tiled_sizes.argtypes = [P(stb_cfg_t), P(stb_layout_t)]
    lib.stb_tile.argtypes = [P(stb_layout_t), P(stb_layout_t)]
    lib.stb_untile.argtypes = [P(stb_layout_t), P(stb_layout_t)]
    lib.stb_tile_device.argtypes = [P(stb_layout_t), P(stb_layout_t), C.c_void_p]
    lib.stb_tile_device.restype = C.c_int
    lib.stb_pack.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, P(stb_layout_t), C.c_int32]
    lib.stb_pack_obc.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, P(stb_layout_t), C.c_int32]
    lib.stb_pack_obc.restype = C.c_int
    lib.stb_hessian_factor.argtypes = [C.c_void_p, C.c_int32, C.c_int32, C.c_double, C.c_void_p, C.c_void_p, C.c_int32]
    lib.stb_hessian_factor.restype = C.c_int
    lib.stb_pack_obc_hybrid.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, P(stb_layout_t), C.c_int32,
                                        C.c_void_p, C.c_int64, C.c_void_p]
    lib.stb_pack_obc_hybrid.restype = C.c_int
    lib.stb_pack_obc_hybrid_workspace_bytes.argtypes = [P(stb_cfg_t)]
    lib.stb_pack_obc_hybrid_workspace_bytes.restype = C.c_int64
    lib.stb_pack_device_workspace_bytes.argtypes = [P(stb_cfg_t), C.c_int32]
    lib.stb_pack_device_workspace_bytes.restype = C.c_int64
    lib.stb_pack_device.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, P(stb_layout_t), C.c_int32, C.c_void_p, C.c_int64,
                                    C.c_void_p]
    lib.stb_pack_device.restype = C.c_int
    lib.stb_unpack.argtypes = [P(stb_layout_t), C.c_void_p]
    lib.stb_salient_columns.argtypes = [C.c_void_p, C.c_int32, C.c_int32, C.c_void_p, C.c_double, C.c_int32,
                                        C.c_void_p, P(C.c_int32)]
    lib.stb_salient_columns.restype = C.c_int
    lib.stb_salient_columns_hc.argtypes = [C.c_void_p, C.c_int32, C.c_int32, C.c_void_p, C.c_int32, C.c_void_p, P(C.c_int32)]
    lib.stb_salient_columns_hc.restype = C.c_int
    lib.stb_layer_l2_norm.argtypes = [C.c_void_p, C.c_int64, P(C.c_double)]
    lib.stb_layer_l2_norm.restype = C.c_int
    lib.stb_layer_nm_assignment.argtypes = [C.c_void_p, C.c_int32, C.c_double, C.c_int32, C.c_void_p]
    lib.stb_layer_nm_assignment.restype = C.c_int
    lib.stb_code24_export.argtypes = [P(stb_layout_t), C.c_void_p, C.c_void_p]
    lib.stb_code24_export.restype = C.c_int
    lib.stb_code24_import.argtypes = [P(stb_layout_t), C.c_void_p, C.c_void_p]
    lib.stb_code24_import.restype = C.c_int
    lib.stb_code24_index.argtypes = [P(stb_layout_t), C.c_void_p, C.c_void_p]
    lib.stb_code24_index.restype = C.c_int
    lib.stb_dequant.argtypes = [P(stb_layout_t), C.c_void_p, C.c_void_p]
    lib.stb_gemv.argtypes = [P(stb_layout_t), C.c_void_p, C.c_int32, C.c_void_p, C.c_int32, C.c_void_p,
                             C.c_int64, C.c_void_p]
    lib.stb_gemv_static.argtypes = [P(stb_layout_t), C.c_void_p, C.c_int32, C.c_void_p, C.c_int32, C.c_void_p]
    lib.stb_gemv_static.restype = C.c_int
    lib.stb_gemv_workspace_bytes.argtypes = [P(stb_cfg_t), C.c_int32]
    lib.stb_gemv_workspace_bytes.restype = C.c_int64
    lib.stb_gemv_batched.argtypes = [C.c_int32, P(P(stb_layout_t)), P(C.c_void_p), C.c_int32,
                                     P(C.c_void_p), C.c_int32, C.c_void_p, C.c_int64, C.c_void_p]
    lib.stb_gemv_batched_workspace_bytes.argtypes = [C.c_int32, P(P(stb_cfg_t)), C.c_int32]
    lib.stb_gemv_batched_workspace_bytes.restype = C.c_int64
    lib.stb_gemm.argtypes = [P(stb_layout_t), C.c_void_p, C.c_int32, C.c_void_p, C.c_int32,
                             C.c_void_p, C.c_int64, C.c_void_p]
    lib.stb_gemm_workspace_bytes.argtypes = [P(stb_layout_t), C.c_int32]
    lib.stb_gemm_workspace_bytes.restype = C.c_int64
    lib.stb_probe_read.argtypes = [C.c_void_p, C.c_int64, C.c_void_p, C.c_void_p]
    lib.stb_probe_read.restype = C.c_int
    lib.stb_probe_mfma.argtypes = [C.c_int32, C.c_int32, C.c_int32, C.c_int32, C.c_void_p, C.c_void_p]
    lib.stb_probe_mfma.restype = C.c_int
    lib.stb_set_kernel_override.argtypes = [C.c_int32, C.c_int32, C.c_int32, C.c_int32]
    lib.stb_set_kernel_override.restype = C.c_int
    lib.stb_strerror.argtypes = [C.c_int]
    lib.stb_strerror.restype = C.c_char_p
    lib.stb_last_hip_error.restype = C.c_int
    for name in ("stb_layout_sizes", "stb_layout_bind", "stb_tiled_sizes", "stb_tile", "stb_untile", "stb_pack", "stb_unpack", "stb_dequant",
                 "stb_gemv", "stb_gemv_batched", "stb_gemm"):
        getattr(lib, name).restype = C.c_int
    _LIB = lib
    return lib


def _check(status: int, where: str):
    if status != STB_OK:
        raise StbError(int(status), where)


def make_cfg(n_out: int, k_in: int, N: int, M: int, n_salient: int, region_mode: int = 0) -> stb_cfg_t:
    return stb_cfg_t(n_out, k_in, N, M, STB_BLOCK, n_salient, region_mode)


def aligned_bytes(nbytes: int, align: int = STB_PLANE_ALIGN) -> np.ndarray:
    """Zero-filled uint8 host buffer whose address is a multiple of `align`."""
    raw = np.zeros(nbytes + align, dtype=np.uint8)
    off = (-raw.ctypes.data) % align
    return raw[off:off + nbytes]


# ---- entry points, same names as the C ABI -----------------------------------------------------
def stb_layout_sizes(cfg: stb_cfg_t) -> stb_layout_t:
    out = stb_layout_t()
    _check(_lib().stb_layout_sizes(C.byref(cfg), C.byref(out)), "stb_layout_sizes")
    return out


def stb_hessian_factor(X, lam: float, n_threads: int = 0):
    """(Hc, xnorm) for calibration activations X (r x k fp32, host): see stb_hessian_factor in stb.h."""
    X = np.ascontiguousarray(X, dtype=np.float32)
    r, k = X.shape
    Hc = np.empty((k, k), dtype=np.float64)
    xnorm = np.empty(k, dtype=np.float32)
    _check(_lib().stb_hessian_factor(X.ctypes.data_as(C.c_void_p), r, k, C.c_double(lam), Hc.ctypes.data_as(C.c_void_p),
                                     xnorm.ctypes.data_as(C.c_void_p), n_threads), "stb_hessian_factor")
    return Hc, xnorm


def stb_layout_bind(layout: stb_layout_t, base_ptr: int) -> stb_layout_t:
    _check(_lib().stb_layout_bind(C.byref(layout), C.c_void_p(base_ptr)), "stb_layout_bind")
    return layout


def stb_tiled_sizes(cfg: stb_cfg_t) -> stb_layout_t:
    out = stb_layout_t()
    _check(_lib().stb_tiled_sizes(C.byref(cfg), C.byref(out)), "stb_tiled_sizes")
    return out


def stb_tile(src_rowmajor: stb_layout_t, dst_tiled: stb_layout_t) -> None:
    _check(_lib().stb_tile(C.byref(src_rowmajor), C.byref(dst_tiled)), "stb_tile")


def stb_untile(src_tiled: stb_layout_t, dst_rowmajor: stb_layout_t) -> None:
    _check(_lib().stb_untile(C.byref(src_tiled), C.byref(dst_rowmajor)), "stb_untile")


def stb_tile_device(src_rowmajor_dev: stb_layout_t, dst_tiled_dev: stb_layout_t, stream: Optional[int] = None) -> None:
    _check(_lib().stb_tile_device(C.byref(src_rowmajor_dev), C.byref(dst_tiled_dev), C.c_void_p(_stream_ptr(stream))),
           "stb_tile_device")


def stb_pack(W: np.ndarray, xnorm: np.ndarray, sal_bitmap: np.ndarray, layout: stb_layout_t,
             n_threads: int = 0) -> None:
    W = np.ascontiguousarray(W, dtype=np.float32)
    xnorm = np.ascontiguousarray(xnorm, dtype=np.float32)
    sal_bitmap = np.ascontiguousarray(sal_bitmap, dtype=np.uint32)
    assert W.shape == (layout.cfg.n_out, layout.cfg.k_in) and xnorm.shape == (layout.cfg.k_in,)
    assert sal_bitmap.shape == (layout.cfg.k_in // 32,)
    _check(_lib().stb_pack(W.ctypes.data, xnorm.ctypes.data, sal_bitmap.ctypes.data, C.byref(layout),
                           n_threads), "stb_pack")


def stb_pack_obc(W: np.ndarray, Hc: Optional[np.ndarray], xnorm: np.ndarray, sal_bitmap: np.ndarray,
                 layout: stb_layout_t, n_threads: int = 0) -> None:
    W = np.ascontiguousarray(W, dtype=np.float32)
    xnorm = np.ascontiguousarray(xnorm, dtype=np.float32)
    sal_bitmap = np.ascontiguousarray(sal_bitmap, dtype=np.uint32)
    k = layout.cfg.k_in
    assert W.shape == (layout.cfg.n_out, k) and xnorm.shape == (k,) and sal_bitmap.shape == (k // 32,)
    if Hc is not None:
        Hc = np.ascontiguousarray(Hc, dtype=np.float64)
        assert Hc.shape == (k, k)
    _check(_lib().stb_pack_obc(W.ctypes.data, None if Hc is None else Hc.ctypes.data, xnorm.ctypes.data,
                               sal_bitmap.ctypes.data, C.byref(layout), n_threads), "stb_pack_obc")


def stb_pack_obc_hybrid_workspace_bytes(cfg: stb_cfg_t) -> int:
    r = int(_lib().stb_pack_obc_hybrid_workspace_bytes(C.byref(cfg)))
    if r < 0:
        _check(r, "stb_pack_obc_hybrid_workspace_bytes")
    return r


def stb_pack_obc_hybrid(W: np.ndarray, Hc: Optional[np.ndarray], xnorm: np.ndarray, sal_bitmap: np.ndarray,
                        layout: stb_layout_t, n_threads: int = 0, workspace=None, stream: Optional[int] = None) -> None:
    """stb_pack_obc with the compensation update on the GPU; `workspace`: uint8 device tensor (allocated if None)."""
    W = np.ascontiguousarray(W, dtype=np.float32)
    xnorm = np.ascontiguousarray(xnorm, dtype=np.float32)
    sal_bitmap = np.ascontiguousarray(sal_bitmap, dtype=np.uint32)
    k = layout.cfg.k_in
    assert W.shape == (layout.cfg.n_out, k) and xnorm.shape == (k,) and sal_bitmap.shape == (k // 32,)
    if Hc is not None:
        Hc = np.ascontiguousarray(Hc, dtype=np.float64)
        assert Hc.shape == (k, k)
        if workspace is None:
            workspace = new_device_scratch(stb_pack_obc_hybrid_workspace_bytes(layout.cfg))
    _check(_lib().stb_pack_obc_hybrid(W.ctypes.data, None if Hc is None else Hc.ctypes.data, xnorm.ctypes.data,
                                      sal_bitmap.ctypes.data, C.byref(layout), n_threads,
                                      None if workspace is None else workspace.data_ptr(),
                                      0 if workspace is None else workspace.numel(),
                                      _stream_ptr(stream) if Hc is not None else None), "stb_pack_obc_hybrid")


def stb_pack_device_workspace_bytes(cfg: stb_cfg_t, si_per_block: bool = False) -> int:
    r = int(_lib().stb_pack_device_workspace_bytes(C.byref(cfg), int(bool(si_per_block))))
    if r < 0:
        _check(r, "stb_pack_device_workspace_bytes")
    return r


def stb_pack_device(W, xnorm, sal_bitmap, out_dev: stb_layout_t, si_per_block: bool = False, workspace=None,
                    stream: Optional[int] = None) -> None:
    """W, xnorm, sal_bitmap: CUDA tensors (float32 [n][k], float32 [k], int32 [k/32]); out_dev: row-major layout bound
    to device memory; workspace: uint8 CUDA tensor from new_device_scratch."""
    import torch
    cfg = out_dev.cfg
    assert W.is_cuda and W.dtype == torch.float32 and W.is_contiguous() and tuple(W.shape) == (cfg.n_out, cfg.k_in)
    assert xnorm.is_cuda and xnorm.dtype == torch.float32 and xnorm.is_contiguous() and xnorm.numel() == cfg.k_in
    assert sal_bitmap.is_cuda and sal_bitmap.dtype == torch.int32 and sal_bitmap.numel() == cfg.k_in // 32
    _check(_lib().stb_pack_device(W.data_ptr(), xnorm.data_ptr(), sal_bitmap.data_ptr(), C.byref(out_dev),
                                  int(bool(si_per_block)), workspace.data_ptr() if workspace is not None else None,
                                  workspace.numel() if workspace is not None else 0, _stream_ptr(stream)),
           "stb_pack_device")


def stb_unpack(layout: stb_layout_t) -> np.ndarray:
    out = np.empty((layout.cfg.n_out, layout.cfg.k_in), dtype=np.float32)
    _check(_lib().stb_unpack(C.byref(layout), out.ctypes.data), "stb_unpack")
    return out


def stb_salient_columns(W: np.ndarray, xnorm: np.ndarray, lam: float, max_per_block: int) -> np.ndarray:
    """sal_bitmap (k/32 uint32 words) of the columns that Alg. 2 "Salient" picks, block by block."""
    W = np.ascontiguousarray(W, dtype=np.float32)
    xnorm = np.ascontiguousarray(xnorm, dtype=np.float32)
    n, k = W.shape
    if xnorm.shape != (k,):
        raise ValueError("xnorm must have k entries")
    out = np.zeros(max(k // 32, 1), dtype=np.uint32)
    count = C.c_int32(0)
    _check(_lib().stb_salient_columns(W.ctypes.data, n, k, xnorm.ctypes.data, float(lam), int(max_per_block),
                                      out.ctypes.data, C.byref(count)), "stb_salient_columns")
    return out


def stb_salient_columns_hc(W: np.ndarray, Hc: np.ndarray, max_per_block: int) -> np.ndarray:
    """sal_bitmap of the columns that Alg. 2 "Salient" picks with the diagonal of the factor Hc (k x k float64)."""
    W = np.ascontiguousarray(W, dtype=np.float32)
    Hc = np.ascontiguousarray(Hc, dtype=np.float64)
    n, k = W.shape
    if Hc.shape != (k, k):
        raise ValueError("Hc must be k x k")
    out = np.zeros(max(k // 32, 1), dtype=np.uint32)
    count = C.c_int32(0)
    _check(_lib().stb_salient_columns_hc(W.ctypes.data, n, k, Hc.ctypes.data, int(max_per_block), out.ctypes.data,
                                         C.byref(count)), "stb_salient_columns_hc")
    return out


def stb_layer_l2_norm(W: np.ndarray) -> float:
    W = np.ascontiguousarray(W, dtype=np.float32)
    out = C.c_double(0.0)
    _check(_lib().stb_layer_l2_norm(W.ctypes.data, W.size, C.byref(out)), "stb_layer_l2_norm")
    return float(out.value)


def stb_layer_nm_assignment(omegas, r_target: float, M: int = 8) -> np.ndarray:
    om = np.ascontiguousarray(omegas, dtype=np.float64)
    out = np.zeros(om.size, dtype=np.int32)
    _check(_lib().stb_layer_nm_assignment(om.ctypes.data, om.size, float(r_target), int(M), out.ctypes.data),
           "stb_layer_nm_assignment")
    return out


def stb_code24_export(layout: stb_layout_t):
    """(E, V): the meta index [n][k/16] uint16 and the sign bytes [n][k/16] uint8 of a row-major 2:4 host layout."""
    n, k16 = layout.cfg.n_out, layout.cfg.k_in // 16
    E = np.empty((n, k16), dtype=np.uint16)
    V = np.empty((n, k16), dtype=np.uint8)
    _check(_lib().stb_code24_export(C.byref(layout), E.ctypes.data, V.ctypes.data), "stb_code24_export")
    return E, V


def stb_code24_import(layout: stb_layout_t, E: np.ndarray, V: np.ndarray) -> None:
    n, k16 = layout.cfg.n_out, layout.cfg.k_in // 16
    if E.shape != (n, k16) or V.shape != (n, k16) or E.dtype != np.uint16 or V.dtype != np.uint8:
        raise ValueError("E must be uint16 [n][k/16] and V uint8 [n][k/16]")
    E = np.ascontiguousarray(E)
    V = np.ascontiguousarray(V)
    _check(_lib().stb_code24_import(C.byref(layout), E.ctypes.data, V.ctypes.data), "stb_code24_import")


def _stream_ptr(stream) -> int:
    if stream is None:
        import torch
        return torch.cuda.current_stream().cuda_stream
    return int(getattr(stream, "cuda_stream", stream))


def stb_code24_index(layout_dev: stb_layout_t, E_dev, stream=None) -> None:
    _check(_lib().stb_code24_index(C.byref(layout_dev), C.c_void_p(E_dev.data_ptr()),
                                   C.c_void_p(_stream_ptr(stream))), "stb_code24_index")


def stb_dequant(layout_dev: stb_layout_t, out_dev, stream=None) -> None:
    _check(_lib().stb_dequant(C.byref(layout_dev), C.c_void_p(out_dev.data_ptr()),
                              C.c_void_p(_stream_ptr(stream))), "stb_dequant")


def _ws(workspace):
    if workspace is None:
        return C.c_void_p(0), 0
    return C.c_void_p(workspace.data_ptr()), workspace.numel() * workspace.element_size()


def stb_gemv_workspace_bytes(cfg: stb_cfg_t, B: int) -> int:
    r = _lib().stb_gemv_workspace_bytes(C.byref(cfg), B)
    if r < 0:
        raise StbError(int(r), "stb_gemv_workspace_bytes")
    return int(r)


def stb_gemv(layout_dev: stb_layout_t, x_dev, B: int, y_dev, y_fp32: bool = False, workspace=None,
             stream=None) -> None:
    ws_ptr, ws_bytes = _ws(workspace)
    _check(_lib().stb_gemv(C.byref(layout_dev), C.c_void_p(x_dev.data_ptr()), B,
                           C.c_void_p(y_dev.data_ptr()), int(y_fp32), ws_ptr, ws_bytes,
                           C.c_void_p(_stream_ptr(stream))), "stb_gemv")


def stb_gemv_static(layout_dev: stb_layout_t, x_dev, B: int, y_dev, y_fp32: bool = False, stream=None) -> None:
    _check(_lib().stb_gemv_static(C.byref(layout_dev), C.c_void_p(x_dev.data_ptr()), B,
                                  C.c_void_p(y_dev.data_ptr()), int(y_fp32), C.c_void_p(_stream_ptr(stream))),
           "stb_gemv_static")


def stb_gemv_batched(layouts_dev: Sequence[stb_layout_t], xs_dev, B: int, ys_dev, y_fp32: bool = False,
                     workspace=None, stream=None) -> None:
    n = len(layouts_dev)
    LP = C.POINTER(stb_layout_t)
    lay = (LP * n)(*[C.pointer(l) for l in layouts_dev])
    xs = (C.c_void_p * n)(*[x.data_ptr() for x in xs_dev])
    ys = (C.c_void_p * n)(*[y.data_ptr() for y in ys_dev])
    ws_ptr, ws_bytes = _ws(workspace)
    _check(_lib().stb_gemv_batched(n, lay, xs, B, ys, int(y_fp32), ws_ptr, ws_bytes,
                                   C.c_void_p(_stream_ptr(stream))), "stb_gemv_batched")


def stb_gemv_batched_workspace_bytes(cfgs: Sequence[stb_cfg_t], B: int) -> int:
    n = len(cfgs)
    CP = C.POINTER(stb_cfg_t)
    arr = (CP * n)(*[C.pointer(c) for c in cfgs])
    r = _lib().stb_gemv_batched_workspace_bytes(n, arr, B)
    if r < 0:
        raise StbError(int(r), "stb_gemv_batched_workspace_bytes")
    return int(r)


def stb_gemm_workspace_bytes(layout: stb_layout_t, T: int) -> int:
    r = _lib().stb_gemm_workspace_bytes(C.byref(layout), T)
    if r < 0:
        raise StbError(int(r), "stb_gemm_workspace_bytes")
    return int(r)


def stb_gemm(layout_dev: stb_layout_t, X_dev, T: int, Y_dev, y_fp32: bool = False, workspace=None,
             stream=None) -> None:
    ws_ptr, ws_bytes = _ws(workspace)
    _check(_lib().stb_gemm(C.byref(layout_dev), C.c_void_p(X_dev.data_ptr()), T,
                           C.c_void_p(Y_dev.data_ptr()), int(y_fp32), ws_ptr, ws_bytes,
                           C.c_void_p(_stream_ptr(stream))), "stb_gemm")


def stb_probe_read(src_dev, nbytes: int, sink_dev, stream=None) -> None:
    _check(_lib().stb_probe_read(C.c_void_p(src_dev.data_ptr()), nbytes, C.c_void_p(sink_dev.data_ptr()),
                                 C.c_void_p(_stream_ptr(stream))), "stb_probe_read")


def stb_probe_mfma(kind: int, valu: int, steps: int, n_workgroups: int, sink_dev, stream=None) -> None:
    _check(_lib().stb_probe_mfma(kind, valu, steps, n_workgroups, C.c_void_p(sink_dev.data_ptr()),
                                 C.c_void_p(_stream_ptr(stream))), "stb_probe_mfma")


def stb_set_kernel_override(gemv_kernel: int = 0, gemv_visits: int = 0, gemv_splits: int = 0, gemm_kernel: int = 0) -> None:
    _check(_lib().stb_set_kernel_override(gemv_kernel, gemv_visits, gemv_splits, gemm_kernel), "stb_set_kernel_override")


GEMV_THIN = 1
GEMM_DENSE, GEMM_DENSE32, GEMM_SPARSE16, GEMM_SHARED = 1, 2, 3, 4


def new_device_scratch(nbytes: int, device="cuda:0", zero: bool = False):
    """256-byte aligned uint8 device tensor of `nbytes` bytes (None for 0)."""
    import torch
    if nbytes == 0:
        return None
    make = torch.zeros if zero else torch.empty
    raw = make(nbytes + STB_PLANE_ALIGN, dtype=torch.uint8, device=device)
    off = (-raw.data_ptr()) % STB_PLANE_ALIGN
    return raw[off:off + nbytes]


# ---- holder --------------------------------------------------------------------------------------
class PackedMatrix:
    """A packed image on the host (numpy, 256-byte aligned) and, after `to_device`, its copy in HBM."""

    def __init__(self, cfg: stb_cfg_t):
        self.cfg = cfg
        self.host_layout = stb_layout_sizes(cfg)
        self.host_image = aligned_bytes(self.host_layout.image_bytes)
        stb_layout_bind(self.host_layout, self.host_image.ctypes.data)
        self.dev_layout: Optional[stb_layout_t] = None
        self.dev_image = None

    @classmethod
    def pack(cls, W, xnorm, sal_bitmap, N: int, M: int, region_mode: int = 0, n_threads: int = 0):
        n, k = W.shape
        sal_bitmap = np.ascontiguousarray(sal_bitmap, dtype=np.uint32)
        S = int(np.unpackbits(sal_bitmap.view(np.uint8)).sum())
        pm = cls(make_cfg(n, k, N, M, S, region_mode))
        stb_pack(W, xnorm, sal_bitmap, pm.host_layout, n_threads)
        return pm

    @classmethod
    def pack_obc(cls, W, Hc, xnorm, sal_bitmap, N: int, M: int, region_mode: int = 0, n_threads: int = 0):
        n, k = W.shape
        sal_bitmap = np.ascontiguousarray(sal_bitmap, dtype=np.uint32)
        S = int(np.unpackbits(sal_bitmap.view(np.uint8)).sum())
        pm = cls(make_cfg(n, k, N, M, S, region_mode))
        stb_pack_obc(W, Hc, xnorm, sal_bitmap, pm.host_layout, n_threads)
        return pm

    @classmethod
    def pack_obc_hybrid(cls, W, Hc, xnorm, sal_bitmap, N: int, M: int, region_mode: int = 0, n_threads: int = 0):
        n, k = W.shape
        sal_bitmap = np.ascontiguousarray(sal_bitmap, dtype=np.uint32)
        S = int(np.unpackbits(sal_bitmap.view(np.uint8)).sum())
        pm = cls(make_cfg(n, k, N, M, S, region_mode))
        stb_pack_obc_hybrid(W, Hc, xnorm, sal_bitmap, pm.host_layout, n_threads)
        return pm

    @property
    def packed_bytes(self) -> int:
        return int(self.host_layout.total_bytes)

    def plane(self, name: str) -> np.ndarray:
        """Bytes of one plane of the host image (a view)."""
        for pname, off, size in PLANE_FIELDS:
            if pname == name:
                o, s = getattr(self.host_layout, off), getattr(self.host_layout, size)
                return self.host_image[o:o + s]
        raise KeyError(name)

    def planes(self) -> dict:
        return {name: self.plane(name) for name, _, _ in PLANE_FIELDS}

    def unpack(self) -> np.ndarray:
        return stb_unpack(self.host_layout)

    def tiled(self):
        """(layout, image) of the tiled device order on the host, built once by stb_tile."""
        if getattr(self, "_tiled", None) is None:
            lay = stb_tiled_sizes(self.cfg)
            img = aligned_bytes(lay.image_bytes)
            stb_layout_bind(lay, img.ctypes.data)
            stb_tile(self.host_layout, lay)
            self._tiled = (lay, img)
        return self._tiled

    def host_pair(self, tiled: bool):
        return self.tiled() if tiled else (self.host_layout, self.host_image)

    def to_device(self, device="cuda:0", tiled: bool = False):
        """Copies the row-major (tiled=False) or tiled image to HBM and binds `dev_layout` to it."""
        import torch
        lay, img = self.host_pair(tiled)
        self.dev_image = torch.empty(lay.image_bytes + STB_PLANE_ALIGN, dtype=torch.uint8, device=device)
        off = (-self.dev_image.data_ptr()) % STB_PLANE_ALIGN
        view = self.dev_image[off:off + lay.image_bytes]
        view.copy_(torch.from_numpy(img))
        self.dev_layout = self.clone_layout_for(view.data_ptr(), tiled)
        self.workspace = self.new_workspace(device)
        return self

    def new_workspace(self, device="cuda:0"):
        """Zero-filled stb_gemv scratch for this matrix (None if the shape needs none), 256-byte aligned."""
        return new_device_scratch(stb_gemv_workspace_bytes(self.cfg, STB_MAX_BATCH), device, zero=True)

    def new_gemm_workspace(self, T: int, device="cuda:0"):
        """stb_gemm scratch for T tokens against the layout that is on the device (None if none is needed)."""
        return new_device_scratch(stb_gemm_workspace_bytes(self.dev_layout, T), device)

    def clone_layout_for(self, base_ptr: int, tiled: bool = False) -> stb_layout_t:
        """Layout struct of the same matrix bound to another copy of the image (host or device)."""
        src, _ = self.host_pair(tiled)
        lay = stb_layout_t()
        C.memmove(C.byref(lay), C.byref(src), C.sizeof(stb_layout_t))
        return stb_layout_bind(lay, base_ptr)
