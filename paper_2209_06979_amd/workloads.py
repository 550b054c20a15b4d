"""Seeded synthetic inputs shaped like the paper's workloads.

This module only draws random patterns and values (NumPy PCG64, fixed seeds).  It
holds none of the method's arithmetic (not even the quantisation of the layer's inputs)
and is the one piece shared by the GPU tests, the benchmark and the CPU oracle's tests.

The paper evaluates on DLMC matrices dilated to V x 1 vectors (Section 5) and on a
sparse-Transformer attention layer (Section 5.3).  Neither data set is available, so
these generators stand in for them: same shapes, vector lengths, sparsity levels and
value ranges, with a uniformly random pattern of exactly round((1 - s) * K) stored
vectors in every row panel.
"""
from __future__ import annotations

import numpy as np

BASE_SEED = 22090697900


def seed_for(config: int, index: int = 0) -> int:
    """Seed of input ``index`` of benchmark configuration ``config``."""
    return BASE_SEED + 1000 * int(config) + int(index)


def vectors_per_panel(K: int, sparsity: float) -> int:
    return int(np.floor((1.0 - sparsity) * K + 0.5))


def vector_sparse_pattern(M: int, K: int, V: int, sparsity: float, seed: int,
                          keep_diagonal: bool = False):
    """Random 1-D-block pattern: (row_ptr[M/V + 1], col_idx[nvec]) as int32.

    Every panel of V rows stores exactly ``vectors_per_panel(K, sparsity)`` column
    vectors, chosen uniformly without replacement and listed in ascending order.
    With ``keep_diagonal`` the V columns p*V .. p*V+V-1 of panel p are always among
    them (attention masks: every softmax row then contains its own position).
    """
    assert M % V == 0
    P = M // V
    keep = vectors_per_panel(K, sparsity)
    rng = np.random.default_rng(seed)
    cols = np.empty((P, keep), dtype=np.int32)
    for p in range(P):
        if keep_diagonal:
            diag = np.arange(p * V, min(p * V + V, K), dtype=np.int64)
            assert keep >= len(diag)
            others = np.setdiff1d(np.arange(K, dtype=np.int64), diag, assume_unique=True)
            pick = rng.choice(others, size=keep - len(diag), replace=False)
            c = np.concatenate([diag, pick])
        else:
            c = rng.choice(K, size=keep, replace=False)
        cols[p] = np.sort(c)
    row_ptr = (np.arange(P + 1, dtype=np.int64) * keep).astype(np.int32)
    return row_ptr, cols.reshape(-1)


def ragged_pattern(M: int, K: int, V: int, counts, seed: int):
    """Pattern with a given number of stored vectors per panel (may be 0)."""
    P = M // V
    counts = np.asarray(counts, dtype=np.int64)
    assert counts.shape == (P,) and counts.max(initial=0) <= K
    rng = np.random.default_rng(seed)
    cols = [np.sort(rng.choice(K, size=int(c), replace=False)).astype(np.int32) for c in counts]
    row_ptr = np.concatenate([[0], np.cumsum(counts)]).astype(np.int32)
    col_idx = np.concatenate(cols).astype(np.int32) if P else np.zeros(0, np.int32)
    return row_ptr, col_idx


def uniform_int8(shape, seed: int, lo: int = -128, hi: int = 127) -> np.ndarray:
    rng = np.random.default_rng(seed)
    return rng.integers(lo, hi + 1, size=shape, dtype=np.int64).astype(np.int8)


def uniform_int16(shape, seed: int, lo: int = -2048, hi: int = 2047) -> np.ndarray:
    rng = np.random.default_rng(seed)
    return rng.integers(lo, hi + 1, size=shape, dtype=np.int64).astype(np.int16)


def uniform_packed_int4(shape_bytes, seed: int) -> np.ndarray:
    """Uniform bytes: every byte is a pair of uniform 4-bit two's-complement values."""
    rng = np.random.default_rng(seed)
    return rng.integers(0, 256, size=shape_bytes, dtype=np.int64).astype(np.uint8)


def normal_fp32(shape, seed: int) -> np.ndarray:
    rng = np.random.default_rng(seed)
    return rng.standard_normal(size=shape).astype(np.float32)


def spmm_case(M, K, N, V, sparsity, prec: str, seed: int):
    """One SpMM problem: pattern, vector-major LHS values and the dense RHS.

    prec: "L8R8" | "L8R4" | "L4R4" | "L16R8" | "L16R16" | "L16R4" | "L12R4".  int4 operands
    are packed two per byte (LHS along the V axis of a vector, RHS along a row); 16-bit and
    12-bit operands are int16 arrays drawn from [-2048, 2047] so that exact sums fit int32.
    """
    row_ptr, col_idx = vector_sparse_pattern(M, K, V, sparsity, seed)
    nvec = len(col_idx)
    if prec == "L4R4":
        vals = uniform_packed_int4((nvec, V // 2), seed + 1)
    elif prec in ("L16R8", "L16R16", "L16R4", "L12R4"):
        vals = uniform_int16((nvec, V), seed + 1)
    else:
        vals = uniform_int8((nvec, V), seed + 1)
    if prec in ("L8R4", "L4R4", "L16R4", "L12R4"):
        B = uniform_packed_int4((K, N // 2), seed + 2)
    elif prec == "L16R16":
        B = uniform_int16((K, N), seed + 2)
    else:
        B = uniform_int8((K, N), seed + 2)
    return dict(M=M, K=K, N=N, V=V, prec=prec, row_ptr=row_ptr, col_idx=col_idx, values=vals, B=B)


def sddmm_case(M, Nc, Kd, V, sparsity, prec: str, seed: int):
    """One SDDMM problem: mask pattern, Q (M x Kd) and Kmat (Nc x Kd), row-major."""
    row_ptr, col_idx = vector_sparse_pattern(M, Nc, V, sparsity, seed)
    if prec == "L4R4":
        Q = uniform_packed_int4((M, Kd // 2), seed + 1)
        Kmat = uniform_packed_int4((Nc, Kd // 2), seed + 2)
    elif prec == "L16R16":
        Q = uniform_int16((M, Kd), seed + 1)
        Kmat = uniform_int16((Nc, Kd), seed + 2)
    else:
        Q = uniform_int8((M, Kd), seed + 1)
        Kmat = uniform_int8((Nc, Kd), seed + 2)
    return dict(M=M, Nc=Nc, Kd=Kd, V=V, prec=prec, row_ptr=row_ptr, col_idx=col_idx, Q=Q, Kmat=Kmat)


def attention_case(heads, L, dk, V, sparsity, seed: int):
    """fp32 N(0,1) projections and a mask with the diagonal blocks kept."""
    row_ptr, col_idx = vector_sparse_pattern(L, L, V, sparsity, seed, keep_diagonal=True)
    return dict(heads=heads, L=L, dk=dk, V=V, row_ptr=row_ptr, col_idx=col_idx,
                q=normal_fp32((heads, L, dk), seed + 1),
                k=normal_fp32((heads, L, dk), seed + 2),
                v=normal_fp32((heads, L, dk), seed + 3))
