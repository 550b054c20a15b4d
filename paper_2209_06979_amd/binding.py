"""Thin Python binding over the C ABI of libmagicube.so (see include/magicube.h).

Argument marshalling only: every step of the path runs in the library's HIP kernels.
PyTorch supplies device memory (tensors) and the current stream, nothing else.  If the
shared library is missing the import fails -- there is no fallback implementation.
"""
from __future__ import annotations

import ctypes
import os
from ctypes import POINTER, c_char_p, c_float, c_int, c_int32, c_int64, c_size_t, c_void_p

import numpy as np
import torch  # noqa: F401  -- must come first: the library then binds to the HIP runtime torch ships

_PKG = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_PKG, "libmagicube.so")

MC_OK, MC_EINVAL, MC_EUNSUPPORTED, MC_EALIGN, MC_EHIP, MC_ENOMEM, MC_ERANGE = 0, -1, -2, -3, -4, -5, -6
PREC = {"L8R8": 0, "L8R4": 1, "L4R4": 2, "L16R8": 3, "L16R16": 4, "L16R4": 5, "L12R4": 6}
LHS_BITS = {"L8R8": 8, "L8R4": 8, "L4R4": 4, "L16R8": 16, "L16R16": 16, "L16R4": 16, "L12R4": 12}
RHS_BITS = {"L8R8": 8, "L8R4": 4, "L4R4": 4, "L16R8": 8, "L16R16": 16, "L16R4": 4, "L12R4": 4}


def _container_bits(bits: int) -> int:
    """Bits an element occupies in memory (a 12-bit value travels as int16)."""
    return 16 if bits == 12 else bits
CHUNK = 64


class Layout(ctypes.Structure):
    _fields_ = [("P", c_int32), ("nvec", c_int64), ("nslots", c_int64), ("vals_bytes", c_int64)]


class BlockedLayout(ctypes.Structure):
    _fields_ = [("nblk", c_int32), ("nchunks", c_int64), ("vals_bytes", c_int64)]


KBLOCK = 1024


class MergedLayout(ctypes.Structure):
    _fields_ = [("group", c_int32), ("P", c_int32), ("nvec", c_int64)]


class Options(ctypes.Structure):
    """mc_options: kernel-variant choices of one call; all zero = automatic."""
    _fields_ = [("spmm_row_tile_bytes", c_int), ("spmm_waves", c_int), ("spmm_stages", c_int), ("spmm_splitting", c_int),
                ("spmm_slab", c_int), ("spmm_slab_waves", c_int), ("spmm_slab_panels", c_int), ("sddmm_waves", c_int), ("softmax_variant", c_int), ("attention_mode", c_int),
                ("spmm_merge", c_int)]


class MagicubeError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        detail = lib.mc_last_error_detail().decode() if status == MC_EHIP else ""
        super().__init__(f"{where}: {lib.mc_strerror(status).decode()} ({status}) {detail}".rstrip())


def _load() -> ctypes.CDLL:
    if not os.path.exists(LIB_PATH):
        raise ImportError(
            f"{LIB_PATH} is missing: build it first (python -m paper_2209_06979_amd.build); "
            "there is no CPU fallback")
    L = ctypes.CDLL(LIB_PATH)
    i32p = POINTER(c_int32)
    L.mc_strerror.argtypes = [c_int]; L.mc_strerror.restype = c_char_p
    L.mc_version.argtypes = []; L.mc_version.restype = c_char_p
    L.mc_last_error_detail.argtypes = []; L.mc_last_error_detail.restype = c_char_p
    L.mc_layout_query.argtypes = [c_int, c_int, c_int, c_int, i32p, POINTER(Layout)]
    L.mc_pack_host.argtypes = [c_int, c_int, c_int, c_int, i32p, i32p, c_void_p, i32p, i32p, c_void_p]
    L.mc_unpack_host.argtypes = [c_int, c_int, c_int, c_int, i32p, i32p, c_void_p, i32p, i32p, c_void_p]
    L.mc_blocked_query.argtypes = [c_int, c_int, c_int, c_int, i32p, i32p, POINTER(BlockedLayout)]
    L.mc_pack_blocked_host.argtypes = [c_int, c_int, c_int, c_int, i32p, i32p, c_void_p, i32p, c_void_p, c_void_p, i32p]
    L.mc_mat_create.argtypes = [c_int, c_int, c_int, c_int, i32p, i32p, c_void_p, c_void_p, POINTER(c_void_p)]
    L.mc_mat_set_values_device.argtypes = [c_void_p, c_void_p, c_void_p]
    L.mc_mat_destroy.argtypes = [c_void_p]; L.mc_mat_destroy.restype = None
    L.mc_mat_info.argtypes = [c_void_p, POINTER(c_int), POINTER(c_int), POINTER(c_int), POINTER(c_int),
                              POINTER(c_int64), POINTER(c_int64)]
    L.mc_spmm.argtypes = [c_void_p, c_void_p, c_int, c_int, c_int, c_void_p, c_int, c_void_p]
    L.mc_spmm_flags.argtypes = [c_void_p, c_void_p, c_int, c_int, c_int, ctypes.c_uint, c_void_p, c_int, c_void_p]
    L.mc_sddmm.argtypes = [c_void_p, c_int, c_void_p, c_int, c_int, c_void_p, c_int, c_void_p, c_void_p]
    L.mc_sddmm_flags.argtypes = [c_void_p, c_int, c_void_p, c_int, c_int, c_void_p, c_int, ctypes.c_uint, c_void_p, c_void_p]
    L.mc_sparse_softmax.argtypes = [c_void_p, c_int, c_void_p, c_float, c_float, c_void_p, c_void_p]
    L.mc_attention_workspace_bytes.argtypes = [c_int, c_void_p]; L.mc_attention_workspace_bytes.restype = c_size_t
    L.mc_sparse_attention.argtypes = [c_void_p, c_void_p, c_void_p, c_int, c_int, c_int, c_void_p,
                                      c_float, c_float, c_float, c_float, c_void_p, c_void_p, c_size_t, c_void_p]
    L.mc_sparse_attention_strided.argtypes = [c_void_p, c_void_p, c_void_p, c_int, c_int, c_int, c_int64, c_int64,
                                              c_void_p, c_float, c_float, c_float, c_float, c_void_p, c_void_p,
                                              c_size_t, c_void_p]
    L.mc_sparse_softmax_bits.argtypes = [c_void_p, c_int, c_void_p, c_float, c_float, c_int, c_void_p, c_void_p]
    L.mc_attention_workspace_bytes_bits.argtypes = [c_int, c_void_p, c_int]
    L.mc_attention_workspace_bytes_bits.restype = c_size_t
    L.mc_sparse_attention_bits.argtypes = [c_void_p, c_void_p, c_void_p, c_int, c_int, c_int, c_int64, c_int64,
                                           c_void_p, c_int, c_int, c_float, c_float, c_float, c_float, c_void_p,
                                           c_void_p, c_size_t, c_void_p]
    L.mc_probe_gather_sink_len.argtypes = [c_void_p, c_int, c_int]; L.mc_probe_gather_sink_len.restype = c_int64
    L.mc_probe_gather.argtypes = [c_void_p, c_void_p, c_int, c_int, c_int, c_void_p, c_void_p]
    L.mc_sparse_attention_batched.argtypes = [c_void_p, c_void_p, c_void_p, c_int, c_int, c_int, c_int, c_int64, c_int64,
                                              c_int64, c_void_p, c_int, c_int, c_float, c_float, c_float, c_float,
                                              c_void_p, c_void_p, c_size_t, c_void_p]
    L.mc_sparse_attention_out.argtypes = [c_void_p, c_void_p, c_void_p, c_int, c_int, c_int, c_int, c_int64, c_int64,
                                          c_int64, c_void_p, c_int, c_int, c_float, c_float, c_float, c_float, c_int,
                                          c_void_p, c_void_p, c_size_t, c_void_p]
    L.mc_spmm_dequant.argtypes = [c_void_p, c_void_p, c_int, c_int, c_int, ctypes.c_uint, c_float, c_int, c_void_p, c_int,
                                  c_void_p]
    L.mc_sddmm_dequant.argtypes = [c_void_p, c_int, c_void_p, c_int, c_int, c_void_p, c_int, ctypes.c_uint, c_float, c_int,
                                   c_void_p, c_void_p]
    L.mc_sparse_softmax_to_mat.argtypes = [c_void_p, c_void_p, c_float, c_float, c_void_p]
    L.mc_spmm_form.argtypes = [c_void_p, c_int, c_int, POINTER(Options)]
    L.mc_mat_merged_info.argtypes = [c_void_p, POINTER(c_int), POINTER(c_int64)]
    L.mc_merged_query.argtypes = [c_int, c_int, c_int, c_int, i32p, i32p, c_int, POINTER(MergedLayout)]
    L.mc_merge_host.argtypes = [c_int, c_int, c_int, c_int, i32p, i32p, c_void_p, c_int, i32p, i32p, c_void_p, i32p]
    L.mc_probe_mfma.argtypes = [c_int, c_int, c_void_p, c_void_p]
    L.mc_probe_spmm_phases_len.argtypes = [c_void_p, c_int]; L.mc_probe_spmm_phases_len.restype = c_int64
    L.mc_probe_spmm_phases.argtypes = [c_void_p, c_void_p, c_int, c_int, c_void_p, c_int, c_void_p, c_void_p]
    L.mc_sddmm_to_mat.argtypes = [c_void_p, c_int, c_void_p, c_int, c_int, c_int, c_float, c_void_p, c_void_p]
    L.mc_absmax.argtypes = [c_void_p, c_int64, c_void_p, c_void_p]
    L.mc_quantize.argtypes = [c_void_p, c_int64, c_float, c_int, c_void_p, c_void_p]
    L.mc_options_init.argtypes = [POINTER(Options)]; L.mc_options_init.restype = None
    L.mc_set_thread_options.argtypes = [POINTER(Options)]
    L.mc_get_thread_options.argtypes = [POINTER(Options)]
    L.mc_spmm_ex.argtypes = [c_void_p, c_void_p, c_int, c_int, c_int, ctypes.c_uint, POINTER(Options), c_void_p, c_int, c_void_p]
    L.mc_sddmm_ex.argtypes = [c_void_p, c_int, c_void_p, c_int, c_int, c_void_p, c_int, ctypes.c_uint, POINTER(Options),
                              c_void_p, c_void_p]
    L.mc_sparse_attention_ex.argtypes = [c_void_p, c_void_p, c_void_p, c_int, c_int, c_int, c_int, c_int64, c_int64,
                                         c_int64, c_void_p, c_int, c_int, c_float, c_float, c_float, c_float, c_int,
                                         POINTER(Options), c_void_p, c_void_p, c_size_t, c_void_p]
    L.mc_sparse_attention_static.argtypes = [c_void_p, c_void_p, c_void_p, c_int, c_int, c_int, c_int, c_int64, c_int64,
                                             c_int64, c_void_p, c_int, c_int, c_float, c_float, c_float, c_float, c_int,
                                             POINTER(Options), c_void_p, c_void_p]
    L.mc_attention_workspace_needed.argtypes = [c_int, c_int, c_void_p, c_int, POINTER(Options)]
    L.mc_attention_workspace_needed.restype = c_size_t
    L.mc_set_spmm_variant.argtypes = [c_int, c_int]
    L.mc_set_attention_mode.argtypes = [c_int]
    L.mc_set_spmm_splitting.argtypes = [c_int]
    L.mc_set_spmm_stages.argtypes = [c_int]
    L.mc_set_sddmm_variant.argtypes = [c_int]
    L.mc_set_softmax_variant.argtypes = [c_int]
    for name in ("mc_layout_query", "mc_pack_host", "mc_unpack_host", "mc_mat_create", "mc_mat_set_values_device",
                 "mc_mat_info", "mc_spmm", "mc_spmm_flags", "mc_sddmm", "mc_sddmm_flags", "mc_sparse_softmax", "mc_sparse_softmax_bits", "mc_sparse_attention",
                 "mc_sparse_attention_strided", "mc_sparse_attention_bits", "mc_sparse_attention_batched", "mc_probe_gather",
                 "mc_absmax", "mc_quantize", "mc_sparse_attention_out", "mc_spmm_dequant", "mc_sddmm_dequant", "mc_sparse_softmax_to_mat",
                 "mc_set_spmm_variant", "mc_set_attention_mode", "mc_set_sddmm_variant", "mc_set_spmm_splitting", "mc_set_spmm_stages",
                 "mc_set_softmax_variant", "mc_set_thread_options", "mc_get_thread_options", "mc_spmm_ex", "mc_sddmm_ex",
                 "mc_sparse_attention_ex", "mc_sparse_attention_static", "mc_blocked_query", "mc_pack_blocked_host", "mc_sddmm_to_mat", "mc_probe_mfma", "mc_spmm_form",
                 "mc_mat_merged_info", "mc_merged_query", "mc_merge_host", "mc_probe_spmm_phases"):
        getattr(L, name).restype = c_int
    return L


lib = _load()


def _check(status: int, where: str) -> None:
    if status != MC_OK:
        raise MagicubeError(status, where)


def _i32(a) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.int32)


def _p32(a: np.ndarray):
    return a.ctypes.data_as(POINTER(c_int32))


def _stream() -> int:
    return torch.cuda.current_stream().cuda_stream


# ------------------------------------------------------------------ host format ----
def layout_query(M, K, V, lhs_bits, row_ptr) -> Layout:
    rp = _i32(row_ptr)
    if rp.shape[0] < 1 or (M > 0 and V > 0 and M % V == 0 and rp.shape[0] != M // V + 1):
        raise MagicubeError(MC_EINVAL, "layout_query(row_ptr length)")
    lay = Layout()
    _check(lib.mc_layout_query(M, K, V, lhs_bits, _p32(rp), ctypes.byref(lay)), "mc_layout_query")
    return lay


def pack_host(M, K, V, lhs_bits, row_ptr, col_idx, values):
    """Interchange arrays -> (panel_ptr, slot_idx, slot_vals) host arrays in device format."""
    rp, ci = _i32(row_ptr), _i32(col_idx)
    lay = layout_query(M, K, V, lhs_bits, rp)
    if ci.shape[0] != lay.nvec:
        raise MagicubeError(MC_EINVAL, "pack_host(col_idx length)")
    panel_ptr = np.zeros(2 * lay.P, np.int32)
    slot_idx = np.zeros(max(lay.nslots, 1), np.int32)
    slot_vals = np.zeros(max(lay.vals_bytes, 1), np.uint8)
    vals = None if values is None else np.ascontiguousarray(values)
    _check(lib.mc_pack_host(M, K, V, lhs_bits, _p32(rp), _p32(ci),
                            None if vals is None else vals.ctypes.data, _p32(panel_ptr), _p32(slot_idx),
                            slot_vals.ctypes.data), "mc_pack_host")
    return panel_ptr, slot_idx[:lay.nslots], slot_vals[:lay.vals_bytes]


def pack_blocked_host(M, K, V, lhs_bits, row_ptr, col_idx, values):
    """Interchange arrays -> (nblk, blk_ptr, blk_rows, blk_vals, blk_src): the K-blocked variant of the format."""
    rp, ci = _i32(row_ptr), _i32(col_idx)
    if rp.shape[0] < 1 or (M > 0 and V > 0 and M % V == 0 and rp.shape[0] != M // V + 1) or ci.shape[0] != int(rp[-1]):
        raise MagicubeError(MC_EINVAL, "pack_blocked_host(array lengths)")
    bl = BlockedLayout()
    _check(lib.mc_blocked_query(M, K, V, lhs_bits, _p32(rp), _p32(ci), ctypes.byref(bl)), "mc_blocked_query")
    P = M // V
    blk_ptr = np.zeros(P * bl.nblk + 1, np.int32)
    blk_rows = np.zeros(max(bl.nchunks * CHUNK, 1), np.uint16)
    blk_src = np.zeros(max(bl.nchunks * CHUNK, 1), np.int32)
    blk_vals = np.zeros(max(bl.vals_bytes, 1), np.uint8)
    vals = None if values is None else np.ascontiguousarray(values)
    _check(lib.mc_pack_blocked_host(M, K, V, lhs_bits, _p32(rp), _p32(ci), None if vals is None else vals.ctypes.data,
                                    _p32(blk_ptr), blk_rows.ctypes.data, blk_vals.ctypes.data, _p32(blk_src)),
           "mc_pack_blocked_host")
    return bl.nblk, blk_ptr, blk_rows[:bl.nchunks * CHUNK], blk_vals[:bl.vals_bytes], blk_src[:bl.nchunks * CHUNK]


def merge_host(M, K, V, lhs_bits, row_ptr, col_idx, values, group):
    """Interchange arrays -> (m_row_ptr, m_col_idx, m_values, m_src): `group` consecutive panels as one panel of
    V * group rows at the union of their columns (m_values: bytes in interchange order, None for a pattern)."""
    rp, ci = _i32(row_ptr), _i32(col_idx)
    if rp.shape[0] < 1 or (M > 0 and V > 0 and M % V == 0 and rp.shape[0] != M // V + 1) or ci.shape[0] != int(rp[-1]):
        raise MagicubeError(MC_EINVAL, "merge_host(array lengths)")
    ml = MergedLayout()
    _check(lib.mc_merged_query(M, K, V, lhs_bits, _p32(rp), _p32(ci), group, ctypes.byref(ml)), "mc_merged_query")
    m_row_ptr = np.zeros(ml.P + 1, np.int32)
    m_col_idx = np.zeros(max(ml.nvec, 1), np.int32)
    m_src = np.zeros(max(ml.nvec * group, 1), np.int32)
    vals = None if values is None else np.ascontiguousarray(values)
    nbytes = ml.nvec * group * V * _container_bits(lhs_bits) // 8
    m_values = None if vals is None else np.zeros(max(nbytes, 1), np.uint8)
    _check(lib.mc_merge_host(M, K, V, lhs_bits, _p32(rp), _p32(ci), None if vals is None else vals.ctypes.data, group,
                             _p32(m_row_ptr), _p32(m_col_idx), None if m_values is None else m_values.ctypes.data, _p32(m_src)),
           "mc_merge_host")
    return m_row_ptr, m_col_idx[:ml.nvec], (None if m_values is None else m_values[:nbytes]), m_src[:ml.nvec * group]


def unpack_host(M, K, V, lhs_bits, panel_ptr, slot_idx, slot_vals):
    pp, si = _i32(panel_ptr), _i32(slot_idx)
    P = M // V
    nvec = int(sum(int(pp[2 * p + 1]) - int(pp[2 * p]) for p in range(P)))
    row_ptr = np.zeros(P + 1, np.int32)
    col_idx = np.zeros(max(nvec, 1), np.int32)
    values = np.zeros(max(nvec * V * max(_container_bits(lhs_bits), 8) // 8, 1), np.uint8)
    sv = np.ascontiguousarray(slot_vals, dtype=np.uint8)
    _check(lib.mc_unpack_host(M, K, V, lhs_bits, _p32(pp), _p32(si), sv.ctypes.data if lhs_bits else None,
                              _p32(row_ptr), _p32(col_idx), values.ctypes.data), "mc_unpack_host")
    return row_ptr, col_idx[:nvec], values[:nvec * V * _container_bits(lhs_bits) // 8]


# ---------------------------------------------------------------- device objects ----
class SparseMatrix:
    """Device-resident vector-sparse matrix or mask (owns an mc_mat handle)."""

    def __init__(self, M, K, V, row_ptr, col_idx, values=None, lhs_bits=0):
        rp, ci = _i32(row_ptr), _i32(col_idx)
        if M > 0 and V > 0 and M % V == 0 and rp.shape[0] != M // V + 1:
            raise MagicubeError(MC_EINVAL, "SparseMatrix(row_ptr length)")
        if rp.shape[0] and ci.shape[0] != int(rp[-1]):
            raise MagicubeError(MC_EINVAL, "SparseMatrix(col_idx length)")
        vals = None if values is None else np.ascontiguousarray(values)
        if vals is not None and vals.nbytes != ci.shape[0] * V * _container_bits(lhs_bits) // 8:
            raise MagicubeError(MC_EINVAL, "SparseMatrix(values size)")
        h = c_void_p()
        _check(lib.mc_mat_create(M, K, V, lhs_bits if vals is not None else 0, _p32(rp), _p32(ci),
                                 None if vals is None else vals.ctypes.data, _stream(), ctypes.byref(h)),
               "mc_mat_create")
        self.handle = h
        self.M, self.K, self.V, self.lhs_bits = M, K, V, (lhs_bits if vals is not None else 0)
        nvec, nslots = c_int64(), c_int64()
        _check(lib.mc_mat_info(h, None, None, None, None, ctypes.byref(nvec), ctypes.byref(nslots)), "mc_mat_info")
        self.nvec, self.nslots = nvec.value, nslots.value
        grp, mnvec = c_int(), c_int64()
        _check(lib.mc_mat_merged_info(h, ctypes.byref(grp), ctypes.byref(mnvec)), "mc_mat_merged_info")
        self.merge_group, self.merged_nvec = grp.value, mnvec.value   # 0: the operand has no merged copy

    def set_values(self, values_dev) -> None:
        """values_dev: device tensor, nvec*V elements in interchange (vector-major) order."""
        assert values_dev.is_cuda and values_dev.is_contiguous()
        assert values_dev.numel() * values_dev.element_size() == self.nvec * self.V * _container_bits(self.lhs_bits) // 8
        _check(lib.mc_mat_set_values_device(self.handle, values_dev.data_ptr(), _stream()), "mc_mat_set_values_device")

    def close(self) -> None:
        if getattr(self, "handle", None):
            lib.mc_mat_destroy(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


def set_thread_options(options: Options | None) -> None:
    """Defaults of the calling thread for calls made without ``options=`` (None: automatic)."""
    _check(lib.mc_set_thread_options(None if options is None else ctypes.byref(options)), "mc_set_thread_options")


def get_thread_options() -> Options:
    o = Options()
    _check(lib.mc_get_thread_options(ctypes.byref(o)), "mc_get_thread_options")
    return o


def set_spmm_variant(bytes_per_row_tile: int = 0, waves: int = 0) -> None:
    _check(lib.mc_set_spmm_variant(bytes_per_row_tile, waves), "mc_set_spmm_variant")


def set_spmm_stages(stages: int = 2) -> None:
    _check(lib.mc_set_spmm_stages(stages), "mc_set_spmm_stages")


def set_spmm_splitting(enable: bool = True) -> None:
    _check(lib.mc_set_spmm_splitting(1 if enable else 0), "mc_set_spmm_splitting")


def set_sddmm_variant(waves: int = -1) -> None:
    _check(lib.mc_set_sddmm_variant(waves), "mc_set_sddmm_variant")


def set_softmax_variant(variant: int = 0) -> None:
    _check(lib.mc_set_softmax_variant(variant), "mc_set_softmax_variant")


def set_attention_mode(mode: int = 0) -> None:
    _check(lib.mc_set_attention_mode(mode), "mc_set_attention_mode")


def spmm(A: SparseMatrix, B, prec: str, out=None, lhs_unsigned: bool = False, rhs_unsigned: bool = False,
         options: Options | None = None):
    """C = A * B (int32, M x N).  B: device tensor (K, N) int8, (K, N/2) uint8 for R4, (K, N) int16 for R16.
    lhs_unsigned / rhs_unsigned: read the 8- or 4-bit operand as non-negative values.
    options: kernel-variant choices of this call (None: the calling thread's defaults)."""
    assert B.is_cuda and B.dim() == 2 and B.stride(1) == 1
    rbits = RHS_BITS[prec]
    N = B.shape[1] * B.element_size() * 8 // rbits
    ldb = B.stride(0) * B.element_size() * 8 // rbits
    if out is None:
        out = torch.empty((A.M, N), dtype=torch.int32, device=B.device)
    assert out.is_cuda and out.dtype == torch.int32 and out.shape == (A.M, N) and out.stride(1) == 1
    flags = (1 if lhs_unsigned else 0) | (2 if rhs_unsigned else 0)
    if options is not None:
        _check(lib.mc_spmm_ex(A.handle, B.data_ptr(), N, ldb, PREC[prec], flags, ctypes.byref(options), out.data_ptr(),
                              out.stride(0), _stream()), "mc_spmm_ex")
        return out
    _check(lib.mc_spmm_flags(A.handle, B.data_ptr(), N, ldb, PREC[prec], flags, out.data_ptr(), out.stride(0), _stream()),
           "mc_spmm_flags")
    return out


OUT_TYPE = {torch.float32: 0, torch.float16: 1}


def spmm_form(A: SparseMatrix, N: int, prec: str, options: Options | None = None) -> str:
    """The form mc_spmm_ex would take for this operand: "gather" or "lds" (K-blocks of B resident in LDS)."""
    r = lib.mc_spmm_form(A.handle, N, PREC[prec], ctypes.byref(options) if options is not None else None)
    if r < 0:
        _check(r, "mc_spmm_form")
    return "lds" if r & 1 else "gather"


def spmm_on_merged(A: SparseMatrix, N: int, prec: str, options: Options | None = None) -> bool:
    """Whether mc_spmm_ex would run on the operand's merged copy (panels sharing the MFMA's 16 rows)."""
    r = lib.mc_spmm_form(A.handle, N, PREC[prec], ctypes.byref(options) if options is not None else None)
    if r < 0:
        _check(r, "mc_spmm_form")
    return bool(r & 2)


def spmm_dequant(A: SparseMatrix, B, prec: str, scale: float, out_dtype=torch.float32, out=None,
                 lhs_unsigned: bool = False, rhs_unsigned: bool = False):  # kernel variants: the thread's options
    """C = scale * (A * B) as fp32 or fp16 (M x N): SpMM with the dequantisation fused into the kernel."""
    assert B.is_cuda and B.dim() == 2 and B.stride(1) == 1
    rbits = RHS_BITS[prec]
    N = B.shape[1] * B.element_size() * 8 // rbits
    ldb = B.stride(0) * B.element_size() * 8 // rbits
    if out is None:
        out = torch.empty((A.M, N), dtype=out_dtype, device=B.device)
    assert out.is_cuda and out.dtype == out_dtype and out.shape == (A.M, N) and out.stride(1) == 1
    flags = (1 if lhs_unsigned else 0) | (2 if rhs_unsigned else 0)
    _check(lib.mc_spmm_dequant(A.handle, B.data_ptr(), N, ldb, PREC[prec], flags, float(scale), OUT_TYPE[out_dtype],
                               out.data_ptr(), out.stride(0), _stream()), "mc_spmm_dequant")
    return out


def probe_gather(A: SparseMatrix, B, prec: str, sink=None):
    """Only the gather of spmm(A, B, prec) (a measurement aid); returns the per-workgroup sink."""
    assert B.is_cuda and B.dim() == 2 and B.stride(1) == 1
    rbits = RHS_BITS[prec]
    N = B.shape[1] * B.element_size() * 8 // rbits
    if sink is None:
        sink = torch.zeros(int(lib.mc_probe_gather_sink_len(A.handle, N, PREC[prec])), dtype=torch.int32, device=B.device)
    _check(lib.mc_probe_gather(A.handle, B.data_ptr(), N, B.stride(0) * B.element_size() * 8 // rbits, PREC[prec],
                               sink.data_ptr(), _stream()), "mc_probe_gather")
    return sink


def probe_spmm_phases(A: SparseMatrix, B, out=None, trace=None):
    """The L8-R8 SpMM in its 128-byte-tile, two-wave, two-chunks-in-flight form with ten clock readings per wave
    (a measurement aid); returns (C, trace) with trace an int64 tensor of shape (waves, 10), 100 MHz ticks."""
    assert B.is_cuda and B.dim() == 2 and B.stride(1) == 1 and B.element_size() == 1
    N = B.shape[1]
    if out is None:
        out = torch.empty((A.M, N), dtype=torch.int32, device=B.device)
    if trace is None:
        trace = torch.zeros((int(lib.mc_probe_spmm_phases_len(A.handle, N)) // 10, 10), dtype=torch.int64, device=B.device)
    _check(lib.mc_probe_spmm_phases(A.handle, B.data_ptr(), N, B.stride(0), out.data_ptr(), out.stride(0), trace.data_ptr(),
                                    _stream()), "mc_probe_spmm_phases")
    return out, trace


def probe_mfma(workgroups: int, iters: int, sink=None):
    """Only MFMAs (a measurement aid): workgroups * 4 waves * iters * 8 instructions of 32768 int8 operations each."""
    if sink is None:
        sink = torch.empty(workgroups * 256, dtype=torch.int32, device="cuda")
    _check(lib.mc_probe_mfma(workgroups, iters, sink.data_ptr(), _stream()), "mc_probe_mfma")
    return sink


def sddmm(Q, Kmat, mask: SparseMatrix, prec: str, out=None, lhs_unsigned: bool = False, rhs_unsigned: bool = False,
          options: Options | None = None):
    """S (nvec*V int32, interchange order) = (Q * Kmat^T) at the mask's stored vectors."""
    assert Q.is_cuda and Kmat.is_cuda and Q.dim() == 2 and Kmat.dim() == 2
    assert Q.stride(1) == 1 and Kmat.stride(1) == 1 and Q.shape[1] == Kmat.shape[1]
    bits = LHS_BITS[prec]
    Kd = Q.shape[1] * Q.element_size() * 8 // bits
    assert Q.element_size() == Kmat.element_size()
    if out is None:
        out = torch.empty(mask.nvec * mask.V, dtype=torch.int32, device=Q.device)
    assert out.is_cuda and out.dtype == torch.int32 and out.numel() == mask.nvec * mask.V and out.is_contiguous()
    flags = (1 if lhs_unsigned else 0) | (2 if rhs_unsigned else 0)
    if options is not None:
        _check(lib.mc_sddmm_ex(Q.data_ptr(), Q.stride(0) * Q.element_size() * 8 // bits, Kmat.data_ptr(),
                               Kmat.stride(0) * Kmat.element_size() * 8 // bits, Kd, mask.handle, PREC[prec], flags,
                               ctypes.byref(options), out.data_ptr(), _stream()), "mc_sddmm_ex")
        return out
    _check(lib.mc_sddmm_flags(Q.data_ptr(), Q.stride(0) * Q.element_size() * 8 // bits, Kmat.data_ptr(),
                              Kmat.stride(0) * Kmat.element_size() * 8 // bits, Kd,
                              mask.handle, PREC[prec], flags, out.data_ptr(), _stream()), "mc_sddmm_flags")
    return out


def sddmm_dequant(Q, Kmat, mask: SparseMatrix, prec: str, scale: float, out_dtype=torch.float32, out=None,
                  lhs_unsigned: bool = False, rhs_unsigned: bool = False):
    """scale * (Q * Kmat^T) at the mask's stored vectors as nvec*V fp32 or fp16 values (interchange order)."""
    assert Q.is_cuda and Kmat.is_cuda and Q.dim() == 2 and Kmat.dim() == 2
    assert Q.stride(1) == 1 and Kmat.stride(1) == 1 and Q.shape[1] == Kmat.shape[1]
    bits = LHS_BITS[prec]
    Kd = Q.shape[1] * Q.element_size() * 8 // bits
    assert Q.element_size() == Kmat.element_size()
    if out is None:
        out = torch.empty(mask.nvec * mask.V, dtype=out_dtype, device=Q.device)
    assert out.is_cuda and out.dtype == out_dtype and out.numel() == mask.nvec * mask.V and out.is_contiguous()
    flags = (1 if lhs_unsigned else 0) | (2 if rhs_unsigned else 0)
    _check(lib.mc_sddmm_dequant(Q.data_ptr(), Q.stride(0) * Q.element_size() * 8 // bits, Kmat.data_ptr(),
                                Kmat.stride(0) * Kmat.element_size() * 8 // bits, Kd, mask.handle, PREC[prec], flags,
                                float(scale), OUT_TYPE[out_dtype], out.data_ptr(), _stream()), "mc_sddmm_dequant")
    return out


def sddmm_to_mat(Q, Kmat, P: SparseMatrix, prec: str, scale: float) -> None:
    """(Q * Kmat^T) at P's pattern, re-quantised to P's 8- or 16-bit integers and written into P's device values."""
    assert Q.is_cuda and Kmat.is_cuda and Q.dim() == 2 and Kmat.dim() == 2
    assert Q.stride(1) == 1 and Kmat.stride(1) == 1 and Q.shape[1] == Kmat.shape[1] and Q.element_size() == Kmat.element_size()
    bits = LHS_BITS[prec]
    Kd = Q.shape[1] * Q.element_size() * 8 // bits
    _check(lib.mc_sddmm_to_mat(Q.data_ptr(), Q.stride(0) * Q.element_size() * 8 // bits, Kmat.data_ptr(),
                               Kmat.stride(0) * Kmat.element_size() * 8 // bits, Kd, PREC[prec], float(scale), P.handle,
                               _stream()), "mc_sddmm_to_mat")


def absmax(x, out=None):
    """max |x| of a contiguous fp32 device tensor, as a one-element device tensor."""
    assert x.is_cuda and x.dtype == torch.float32 and x.is_contiguous()
    if out is None:
        out = torch.empty(1, dtype=torch.float32, device=x.device)
    _check(lib.mc_absmax(x.data_ptr(), x.numel(), out.data_ptr(), _stream()), "mc_absmax")
    return out


def quantize(x, scale: float, bits: int = 8, out=None):
    """Symmetric quantisation of a contiguous fp32 device tensor: int8 codes of the same shape, or
    (bits=4) uint8 with half the last dimension, two codes per byte."""
    assert x.is_cuda and x.dtype == torch.float32 and x.is_contiguous()
    if out is None:
        if bits == 4:
            out = torch.empty(x.shape[:-1] + (x.shape[-1] // 2,), dtype=torch.uint8, device=x.device)
        else:
            out = torch.empty(x.shape, dtype=torch.int8, device=x.device)
    assert out.is_cuda and out.is_contiguous()
    if out.numel() * (2 if bits == 4 else 1) != x.numel() and bits in (4, 8):
        raise MagicubeError(MC_EINVAL, "quantize(out size)")
    _check(lib.mc_quantize(x.data_ptr(), x.numel(), float(scale), bits, out.data_ptr(), _stream()), "mc_quantize")
    return out


def sparse_softmax(mask: SparseMatrix, S, score_scale: float, inv_s_p: float, out=None, code_bits: int = 8):
    """Integer codes (int8, or int16 for code_bits=16) of the row softmax over the stored
    entries; S: (batch, nvec*V) int32."""
    assert S.is_cuda and S.dtype == torch.int32 and S.is_contiguous()
    n = mask.nvec * mask.V
    S2 = S.reshape(-1, n) if n else S.reshape(S.shape[0] if S.dim() > 1 else 1, 0)
    dt = torch.int16 if code_bits == 16 else torch.int8
    if out is None:
        out = torch.empty(S2.shape, dtype=dt, device=S.device)
    assert out.is_cuda and out.dtype == dt and out.is_contiguous() and out.numel() == S2.numel()
    _check(lib.mc_sparse_softmax_bits(mask.handle, S2.shape[0], S2.data_ptr(), score_scale, inv_s_p, code_bits,
                                      out.data_ptr(), _stream()), "mc_sparse_softmax_bits")
    return out.reshape(S.shape)


def sparse_softmax_to_mat(P: SparseMatrix, S, score_scale: float, inv_s_p: float) -> None:
    """Softmax of one score set (nvec*V int32) written as integer codes straight into P's device values."""
    assert S.is_cuda and S.dtype == torch.int32 and S.is_contiguous() and S.numel() == P.nvec * P.V
    _check(lib.mc_sparse_softmax_to_mat(P.handle, S.data_ptr(), float(score_scale), float(inv_s_p), _stream()),
           "mc_sparse_softmax_to_mat")


def attention_workspace_bytes(heads: int, mask: SparseMatrix, p_bits: int = 8) -> int:
    return int(lib.mc_attention_workspace_bytes_bits(heads, mask.handle, p_bits))


def attention_workspace_needed(heads: int, dk: int, mask: SparseMatrix, p_bits: int = 8, options: Options | None = None) -> int:
    """Bytes of workspace the layer will really use (0 when the fused kernel takes it)."""
    return int(lib.mc_attention_workspace_needed(heads, dk, mask.handle, p_bits,
                                                 None if options is None else ctypes.byref(options)))


STATIC_SCRATCH_BYTES = 16 << 20


def sparse_attention_static(Q8, K8, V8, mask: SparseMatrix, s_q, s_k, s_v, s_p, out, p_bits: int = 8, qkv_bits: int = 8,
                            options: Options | None = None):
    """sparse_attention for callers that cannot allocate: no workspace argument (the library's own per-GPU array
    holds the intermediates) and a caller-provided ``out``.  This wrapper allocates nothing on the device either."""
    epb = 8 // qkv_bits
    batched = Q8.dim() == 4
    batch = Q8.shape[0] if batched else 1
    heads, L, dkb = Q8.shape[-3:]
    dk = dkb * epb
    st = tuple(x * epb for x in Q8.stride()[:-1])
    bs, hs, ts = (st if batched else (0,) + st)
    for t in (Q8, K8, V8):
        assert t.is_cuda and t.element_size() == 1 and t.shape == Q8.shape and t.stride() == Q8.stride() and t.stride(-1) == 1
    assert out.is_cuda and out.dtype in OUT_TYPE and out.shape == tuple(Q8.shape[:-1]) + (dk,) and out.stride() == st + (1,)
    _check(lib.mc_sparse_attention_static(Q8.data_ptr(), K8.data_ptr(), V8.data_ptr(), batch, heads, L, dk, bs, hs, ts,
                                          mask.handle, p_bits, qkv_bits, float(s_q), float(s_k), float(s_v), float(s_p),
                                          OUT_TYPE[out.dtype], None if options is None else ctypes.byref(options),
                                          out.data_ptr(), _stream()), "mc_sparse_attention_static")
    return out


def sparse_attention(Q8, K8, V8, mask: SparseMatrix, s_q, s_k, s_v, s_p, out=None, workspace=None,
                     p_bits: int = 8, qkv_bits: int = 8, out_dtype=torch.float32, options: Options | None = None):
    """Quantized sparse self-attention; Q8/K8/V8: (heads, L, dk) or (batch, heads, L, dk) int8
    device tensors, or for qkv_bits=4 uint8 tensors of half the last dimension with two 4-bit
    values per byte.  p_bits is the width of the re-quantised softmax output (8 or 16);
    out_dtype is torch.float32 or torch.float16.

    Any layout with unit stride along dk is accepted as long as the three tensors (and
    ``out``) share it; a (heads, L, dk) view of a token-major (L, heads, dk) buffer, i.e.
    ``x.permute(1, 0, 2)``, selects the fast two-heads-per-request path.
    """
    epb = 8 // qkv_bits                       # elements per byte
    batched = Q8.dim() == 4
    batch = Q8.shape[0] if batched else 1
    heads, L, dkb = Q8.shape[-3:]
    dk = dkb * epb
    st = tuple(x * epb for x in Q8.stride()[:-1])     # strides in elements
    bs, hs, ts = (st if batched else (0,) + st)
    for t in (Q8, K8, V8):
        assert t.is_cuda and t.element_size() == 1 and t.shape == Q8.shape and t.stride() == Q8.stride() and t.stride(-1) == 1
    oshape = tuple(Q8.shape[:-1]) + (dk,)
    if out is None:
        out = torch.empty_strided(oshape, st + (1,), dtype=out_dtype, device=Q8.device)   # the inputs' layout
    assert out.is_cuda and out.dtype == out_dtype and out.shape == oshape and out.stride() == st + (1,)
    if workspace is None:
        need = attention_workspace_needed(heads, dk, mask, p_bits, options)
        workspace = torch.empty(need, dtype=torch.uint8, device=Q8.device) if need else None
    ws_ptr, ws_bytes = (None, 0) if workspace is None else (workspace.data_ptr(), workspace.numel() * workspace.element_size())
    assert workspace is None or (workspace.is_cuda and workspace.is_contiguous())
    if options is not None:
        _check(lib.mc_sparse_attention_ex(Q8.data_ptr(), K8.data_ptr(), V8.data_ptr(), batch, heads, L, dk, bs, hs, ts,
                                          mask.handle, p_bits, qkv_bits, float(s_q), float(s_k), float(s_v), float(s_p),
                                          OUT_TYPE[out_dtype], ctypes.byref(options), out.data_ptr(), ws_ptr, ws_bytes,
                                          _stream()), "mc_sparse_attention_ex")
        return out
    _check(lib.mc_sparse_attention_out(Q8.data_ptr(), K8.data_ptr(), V8.data_ptr(), batch, heads, L, dk, bs, hs, ts,
                                       mask.handle, p_bits, qkv_bits, float(s_q), float(s_k), float(s_v), float(s_p),
                                       OUT_TYPE[out_dtype], out.data_ptr(), ws_ptr, ws_bytes, _stream()),
           "mc_sparse_attention_out")
    return out
