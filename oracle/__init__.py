"""CPU oracle for the quantized vector-sparse SpMM / SDDMM / sparse-attention path.

TEST INFRASTRUCTURE ONLY.  Nothing here is part of the product: only the tests,
``__graft_entry__.smoke()`` and the ``cpu_baseline`` leg of ``bench.py`` may import it.
It shares no code with the HIP path and never imports the GPU package.

What it holds
-------------
* ``spmm_dense`` / ``sddmm_dense``: thin ctypes wrappers over ``magicube_oracle.c``,
  the plain int64-accumulating definitions of SpMM (Section 4.2) and SDDMM
  (Section 4.3) on a dense matrix with its zeros materialised plus one "stored" flag
  per (row panel, column).
* helpers that turn the interchange data (BCRS with V x 1 blocks, Section 4.1; packed
  int4; int16) into those dense operands, written here independently of the GPU side.
* the integer-splitting identities of Section 4.4 (unsigned and signed emulation).
* ``attention``: the quantized sparse self-attention layer of Section 5.3 in fp64.

Parity pins for every function live in ``tests/test_oracle_pins.py``.  The only
convention not fixed by the paper is the static scale of the re-quantised softmax
output (``s_p``); it is an input here, so nothing in this file is "parity unpinned".
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "magicube_oracle.c")
_LIB = os.path.join(_HERE, "liboracle.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile the C oracle with gcc (``-O2 -fopenmp``); returns the library path."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(
            ["gcc", "-O2", "-fopenmp", "-shared", "-fPIC", "-o", _LIB, _SRC])
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        lib = ctypes.CDLL(_LIB)
        i32p = ctypes.POINTER(ctypes.c_int32)
        u8p = ctypes.POINTER(ctypes.c_uint8)
        lib.mco_spmm.argtypes = [ctypes.c_int] * 4 + [i32p, u8p, i32p, i32p]
        lib.mco_spmm.restype = ctypes.c_int
        lib.mco_sddmm.argtypes = [ctypes.c_int] * 4 + [i32p, i32p, u8p, i32p]
        lib.mco_sddmm.restype = ctypes.c_int
        lib.mco_num_threads.restype = ctypes.c_int
        lib.mco_set_num_threads.argtypes = [ctypes.c_int]
        _lib = lib
    return _lib


def num_threads() -> int:
    return int(_load().mco_num_threads())


def set_num_threads(n: int) -> None:
    _load().mco_set_num_threads(int(n))


def _i32(a):
    a = np.ascontiguousarray(a, dtype=np.int32)
    return a, a.ctypes.data_as(ctypes.POINTER(ctypes.c_int32))


def _u8(a):
    a = np.ascontiguousarray(a, dtype=np.uint8)
    return a, a.ctypes.data_as(ctypes.POINTER(ctypes.c_uint8))


# --------------------------------------------------------------------------- #
# Plain definitions (C)                                                        #
# --------------------------------------------------------------------------- #
def spmm_dense(A, stored, B, V: int) -> np.ndarray:
    """C[i][j] = sum_k stored[i//V][k] * A[i][k] * B[k][j]  (SpMM, Section 4.2).

    A: (M, K) ints, stored: (M//V, K) flags, B: (K, N) ints.  Exact; raises
    OverflowError if a result does not fit int32.
    """
    A, pa = _i32(A)
    B, pb = _i32(B)
    stored, ps = _u8(stored)
    M, K = A.shape
    K2, N = B.shape
    assert K2 == K and M % V == 0 and stored.shape == (M // V, K)
    C = np.empty((M, N), dtype=np.int32)
    rc = _load().mco_spmm(M, K, N, V, pa, ps, pb, C.ctypes.data_as(ctypes.POINTER(ctypes.c_int32)))
    if rc:
        raise OverflowError("SpMM result does not fit int32")
    return C


def sddmm_dense(Q, Kmat, stored, V: int) -> np.ndarray:
    """(Q @ Kmat.T) read at the stored vectors (SDDMM, Section 4.3).

    Q: (M, Kd), Kmat: (Nc, Kd), stored: (M//V, Nc).  Returns the 1-D int32 array of
    V values per stored vector: panels ascending, columns ascending inside a panel,
    the V rows of the vector consecutive.
    """
    Q, pq = _i32(Q)
    Kmat, pk = _i32(Kmat)
    stored, ps = _u8(stored)
    M, Kd = Q.shape
    Nc, Kd2 = Kmat.shape
    assert Kd2 == Kd and M % V == 0 and stored.shape == (M // V, Nc)
    nvec = int(np.count_nonzero(stored))
    S = np.empty(nvec * V, dtype=np.int32)
    rc = _load().mco_sddmm(M, Kd, Nc, V, pq, pk, ps, S.ctypes.data_as(ctypes.POINTER(ctypes.c_int32)))
    if rc:
        raise OverflowError("SDDMM result does not fit int32")
    return S


# --------------------------------------------------------------------------- #
# Interchange data -> dense operands                                           #
# --------------------------------------------------------------------------- #
def unpack_int4(packed, unsigned: bool = False) -> np.ndarray:
    """4-bit values from bytes, along the last axis.

    Byte j holds element 2j in bits 3:0 and element 2j+1 in bits 7:4, each a
    two's-complement value in [-8, 7] (or, with ``unsigned``, a value in [0, 15]).
    Returns int32 with the last axis doubled.
    """
    p = np.asarray(packed).view(np.uint8).astype(np.int32)
    lo = p & 15
    hi = (p >> 4) & 15
    if not unsigned:
        lo = np.where(lo >= 8, lo - 16, lo)
        hi = np.where(hi >= 8, hi - 16, hi)
    out = np.empty(p.shape[:-1] + (p.shape[-1] * 2,), dtype=np.int32)
    out[..., 0::2] = lo
    out[..., 1::2] = hi
    return out


def pack_int4(q) -> np.ndarray:
    """Inverse of ``unpack_int4`` for values in [-8, 7] (or [0, 15]): two 4-bit values per byte along the
    last axis, element 2j in bits 3:0 and element 2j+1 in bits 7:4 of byte j.  Returns uint8 with the
    last axis halved."""
    q = np.asarray(q).astype(np.int64)
    if q.shape[-1] % 2:
        raise ValueError("the last axis must hold an even number of 4-bit values")
    if q.size and (q.min() < -8 or q.max() > 15):
        raise ValueError("value outside four bits")
    return ((q[..., 0::2] & 15) | ((q[..., 1::2] & 15) << 4)).astype(np.uint8)


def stored_flags(M: int, K: int, V: int, row_ptr, col_idx) -> np.ndarray:
    """(M//V, K) uint8 flags of the stored vectors of a BCRS pattern with V x 1 blocks."""
    P = M // V
    row_ptr = np.asarray(row_ptr, dtype=np.int64)
    col_idx = np.asarray(col_idx, dtype=np.int64)
    flags = np.zeros((P, K), dtype=np.uint8)
    for p in range(P):
        cols = col_idx[row_ptr[p]:row_ptr[p + 1]]
        flags[p, cols] = 1
    return flags


def vector_values_as_int(values, nvec: int, V: int, bits: int, unsigned: bool = False) -> np.ndarray:
    """(nvec, V) int32 from vector-major stored values of the given width.

    bits=8: int8; bits=16: int16; bits=12: int16 container restricted to 12-bit values;
    bits=4: two elements per byte along the V axis.
    """
    if unsigned and bits not in (4, 8):
        raise ValueError("unsigned operands are defined here for 4 and 8 bits")
    if bits == 8:
        return np.asarray(values).view(np.uint8 if unsigned else np.int8).reshape(nvec, V).astype(np.int32)
    if bits == 16 or bits == 12:
        vv = np.asarray(values).view(np.int16).reshape(nvec, V).astype(np.int32)
        if bits == 12 and vv.size and (vv.min() < -2048 or vv.max() > 2047):
            raise ValueError("12-bit operand outside [-2048, 2047]")
        return vv
    if bits == 4:
        return unpack_int4(np.asarray(values).view(np.uint8).reshape(nvec, V // 2), unsigned)
    raise ValueError("bits must be 4, 8, 12 or 16")


def bcrs_to_dense(M: int, K: int, V: int, row_ptr, col_idx, vec_vals) -> tuple[np.ndarray, np.ndarray]:
    """Dense (M, K) int32 matrix with zeros materialised, and the stored flags.

    ``vec_vals`` is (nvec, V): the dense V x 1 blocks in BCRS order (Section 4.1).
    """
    row_ptr = np.asarray(row_ptr, dtype=np.int64)
    col_idx = np.asarray(col_idx, dtype=np.int64)
    vec_vals = np.asarray(vec_vals, dtype=np.int32)
    A = np.zeros((M, K), dtype=np.int32)
    for p in range(M // V):
        lo, hi = row_ptr[p], row_ptr[p + 1]
        A[p * V:(p + 1) * V, col_idx[lo:hi]] = vec_vals[lo:hi].T
    return A, stored_flags(M, K, V, row_ptr, col_idx)


# Table of supported precisions (Section 4.4).  A 12-bit operand travels in an int16
# container and must lie in [-2048, 2047].
_LHS_BITS = {"L8R8": 8, "L8R4": 8, "L4R4": 4, "L16R8": 16, "L16R16": 16, "L16R4": 16, "L12R4": 12}
_RHS_BITS = {"L8R8": 8, "L8R4": 4, "L4R4": 4, "L16R8": 8, "L16R16": 16, "L16R4": 4, "L12R4": 4}


def dense_rhs_as_int(B, bits: int, unsigned: bool = False) -> np.ndarray:
    """Row-major dense operand as int32; bits=4 means two elements per byte along a row,
    bits=16 little-endian int16 elements."""
    if unsigned and bits not in (4, 8):
        raise ValueError("unsigned operands are defined here for 4 and 8 bits")
    if bits == 8:
        return np.asarray(B).view(np.uint8 if unsigned else np.int8).astype(np.int32)
    if bits == 16:
        return np.asarray(B).view(np.int16).astype(np.int32)
    if bits == 4:
        return unpack_int4(np.asarray(B).view(np.uint8), unsigned)
    raise ValueError("bits must be 4, 8 or 16")


def spmm(M, K, V, row_ptr, col_idx, values, B, prec: str, lhs_unsigned: bool = False,
         rhs_unsigned: bool = False) -> np.ndarray:
    """SpMM from interchange data: widen every operand to int, then ``spmm_dense``.

    Lx-Ry names the operand widths (Table "precision supported" of the paper); the
    oracle never splits planes -- mixed precision is just integers of other ranges, and an
    unsigned operand (Section 4.4.1) is the same bytes read as non-negative values.
    """
    nvec = len(col_idx)
    vv = vector_values_as_int(values, nvec, V, _LHS_BITS[prec], lhs_unsigned)
    A, flags = bcrs_to_dense(M, K, V, row_ptr, col_idx, vv)
    return spmm_dense(A, flags, dense_rhs_as_int(B, _RHS_BITS[prec], rhs_unsigned), V)


def sddmm(M, Nc, V, row_ptr, col_idx, Q, Kmat, prec: str, lhs_unsigned: bool = False,
          rhs_unsigned: bool = False) -> np.ndarray:
    """SDDMM from interchange data; Q and Kmat are row-major (packed along Kd for int4)."""
    bits = _LHS_BITS[prec]
    if bits not in (4, 8, 16) or _RHS_BITS[prec] != bits:
        raise ValueError("SDDMM is defined here for L8R8, L4R4 and L16R16")
    flags = stored_flags(M, Nc, V, row_ptr, col_idx)
    return sddmm_dense(dense_rhs_as_int(Q, bits, lhs_unsigned), dense_rhs_as_int(Kmat, bits, rhs_unsigned), flags, V)


# Largest magnitude of a re-quantised SDDMM result: symmetric, 8 bits: 127; 16 bits: 32639 (the same convention
# as P_CODE_MAX: the largest value a two-signed-byte operand can hold).
S_CODE_MAX = {8: 127, 16: 32639}


def requantize_scores(S, scale, bits: int = 8) -> np.ndarray:
    """Integer codes of SDDMM results that feed a following SpMM as its sparse operand (Section 4.3 lets the
    SDDMM write the format of the next operator, whose operands are 8- or 16-bit integers):
    code = clamp(rint(S * scale), -S_CODE_MAX, S_CODE_MAX), ties to even.

    The decision is taken in the kernel's precision, binary32 (the paper fixes none): the int32 score is
    converted to fp32 (round to nearest even), multiplied by the fp32 scale with ONE rounding, and that
    product is rounded to an integer.  numpy's float32 arithmetic is IEEE and does exactly this."""
    x = np.asarray(S).astype(np.int64).astype(np.float32) * np.float32(scale)
    q = np.clip(np.rint(x), -S_CODE_MAX[bits], S_CODE_MAX[bits])
    return q.astype(np.int8 if bits == 8 else np.int16)


# --------------------------------------------------------------------------- #
# Integer splitting (Section 4.4)                                              #
# --------------------------------------------------------------------------- #
def split_unsigned(a, low_bits: int):
    """a = a0 + 2**low_bits * a1 with a0 the low bits (unsigned) -- unsigned emulation."""
    a = np.asarray(a, dtype=np.int64)
    return a & ((1 << low_bits) - 1), a >> low_bits


def split_signed(a, low_bits: int):
    """Two's-complement split: low part unsigned, high part signed (arithmetic shift)."""
    a = np.asarray(a, dtype=np.int64)
    return a & ((1 << low_bits) - 1), a >> low_bits


def split_balanced(a, low_bits: int):
    """a = lo + 2**low_bits * hi with lo in [-2**(low_bits-1), 2**(low_bits-1)) (both signed)."""
    a = np.asarray(a, dtype=np.int64)
    half = 1 << (low_bits - 1)
    hi = (a + half) >> low_bits
    return a - (hi << low_bits), hi


# --------------------------------------------------------------------------- #
# Quantized sparse attention (Section 5.3)                                     #
# --------------------------------------------------------------------------- #
def quantize_per_tensor(x, bits: int = 8):
    """Symmetric quantisation with one scale: qmax = 2**(bits-1) - 1, s = max|x|/qmax,
    q = rint(x/s) in [-qmax, qmax] (returned as int8, one value per element, not packed)."""
    x = np.asarray(x, dtype=np.float64)
    qmax = (1 << (bits - 1)) - 1
    s = np.float32(np.max(np.abs(x)) / qmax)
    q = np.clip(np.rint(x / np.float64(s)), -qmax, qmax).astype(np.int8)
    return q, s


def sparse_softmax(S, row_ptr, V: int, scale: float) -> np.ndarray:
    """Row softmax over the stored entries only, in fp64.

    S: V values per stored vector (SDDMM output order).  Row (p, v) owns the entries
    S[(row_ptr[p] + i) * V + v].  x = S * scale; p = exp(x - max) / sum.
    Masked-out positions are excluded from the softmax (they are not stored).
    """
    S = np.asarray(S)
    row_ptr = np.asarray(row_ptr, dtype=np.int64)
    out = np.zeros(S.shape, dtype=np.float64)
    for p in range(len(row_ptr) - 1):
        lo, hi = row_ptr[p] * V, row_ptr[p + 1] * V
        if hi == lo:
            continue
        x = S[lo:hi].astype(np.float64).reshape(-1, V) * np.float64(scale)
        e = np.exp(x - x.max(axis=0, keepdims=True))
        out[lo:hi] = (e / e.sum(axis=0, keepdims=True)).reshape(-1)
    return out


def dequantize(acc, scale, out_bits: int = 32) -> np.ndarray:
    """Fused dequantisation of an integer result (Section 5.3): the exact integer times the real
    scale (an fp32 number), computed in fp64 and rounded ONCE, to nearest even, to the output
    type: fp32 (out_bits 32) or fp16 (out_bits 16; magnitudes of 65520 and above become inf)."""
    if out_bits not in (16, 32):
        raise ValueError("out_bits must be 16 or 32")
    x = np.asarray(acc).astype(np.float64) * np.float64(np.float32(scale))
    with np.errstate(over="ignore"):
        return x.astype(np.float32 if out_bits == 32 else np.float16)


# Largest code of the re-quantised softmax output.  8 bits: the int8 maximum.  16 bits: 32639, a
# CONVENTION of this build and not a statement of the paper (which fixes no code range for its
# "16b" layers): it is the largest value whose split into two SIGNED bytes (hi = (c + 128) >> 8)
# still fits, i.e. the limit of a signed x signed matrix unit fed a two-plane operand.  The
# ceiling is only reached when s_p is chosen below 1/32639; with the default s_p = 1/32639 the
# clamp is inactive and the codes are rint(p / s_p) as for any other static scale.
P_CODE_MAX = {8: 127, 16: 32639}


def requantize_probabilities(p, s_p: float, bits: int = 8) -> np.ndarray:
    """Integer codes of softmax outputs: clamp(rint(p / s_p), 0, P_CODE_MAX[bits]), ties to even."""
    q = np.clip(np.rint(np.asarray(p, dtype=np.float64) / np.float64(s_p)), 0, P_CODE_MAX[bits])
    return q.astype(np.int8 if bits == 8 else np.int16)


def attention(Q8, K8, V8, row_ptr, col_idx, V: int, s_q, s_k, s_v, s_p, p_bits: int = 8, qkv_bits: int = 8,
              out_bits: int = 64):
    """Quantized self-attention with a vector-sparse mask shared by all heads.

    Q8, K8, V8: (heads, L, dk) int8, or for qkv_bits=4 (heads, L, dk/2) bytes with two
    4-bit values each.  Per head: integer SDDMM(Q, K^T) at the mask -> dequantise with
    s_q*s_k/sqrt(dk) -> softmax over the stored entries -> re-quantisation to p_bits-bit
    codes with the static scale s_p -> integer SpMM with V -> scale s_p*s_v.  The paper's
    "xb-yb" variants (Section 5.3 / end-to-end latency figure) are p_bits=x, qkv_bits=y.
    Returns (O (heads, L, dk), scores int32, probabilities fp64, integer codes), the last
    three as (heads, nvec*V) in SDDMM output order.  O is fp64, or with out_bits 32 / 16 the
    fp64 value rounded once to fp32 / fp16 (the paper's output type).
    """
    if qkv_bits == 4:
        Q8, K8, V8 = (unpack_int4(np.asarray(t).view(np.uint8)) for t in (Q8, K8, V8))
    elif qkv_bits != 8:
        raise ValueError("qkv_bits must be 4 or 8")
    Q8 = np.asarray(Q8)
    heads, L, dk = Q8.shape
    flags = stored_flags(L, L, V, row_ptr, col_idx)
    scale = np.float64(np.float32(s_q)) * np.float64(np.float32(s_k)) / np.sqrt(np.float64(dk))
    nvec = len(col_idx)
    O = np.empty((heads, L, dk), dtype=np.float64)
    scores = np.empty((heads, nvec * V), dtype=np.int32)
    probs = np.empty((heads, nvec * V), dtype=np.float64)
    codes = np.empty((heads, nvec * V), dtype=np.int8 if p_bits == 8 else np.int16)
    for h in range(heads):
        scores[h] = sddmm_dense(Q8[h].astype(np.int32), np.asarray(K8[h]).astype(np.int32), flags, V)
        probs[h] = sparse_softmax(scores[h], row_ptr, V, scale)
        codes[h] = requantize_probabilities(probs[h], s_p, p_bits)
        A, _ = bcrs_to_dense(L, L, V, row_ptr, col_idx, codes[h].reshape(nvec, V))
        C = spmm_dense(A, flags, np.asarray(V8[h]).astype(np.int32), V)
        O[h] = C.astype(np.float64) * (np.float64(np.float32(s_p)) * np.float64(np.float32(s_v)))
    if out_bits != 64:
        with np.errstate(over="ignore"):
            O = O.astype({32: np.float32, 16: np.float16}[out_bits])
    return O, scores, probs, codes
