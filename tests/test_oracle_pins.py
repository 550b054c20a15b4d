"""Pins for the CPU oracle: each one ties an oracle function to something other than
itself -- brute force on tiny inputs, a library routine on a special case, a closed
form, an invariant, or a value printed in the paper (tests/golden/)."""
import os

import numpy as np
import pytest
import torch

import oracle
from paper_2209_06979_amd import workloads as wl
import input_prep as prep

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _tiny(M, K, N, V, density, seed, lo=-128, hi=127):
    rng = np.random.default_rng(seed)
    P = M // V
    flags = (rng.random((P, K)) < density).astype(np.uint8)
    A = rng.integers(lo, hi + 1, size=(M, K)).astype(np.int32)
    A *= np.repeat(flags, V, axis=0).astype(np.int32)
    B = rng.integers(-128, 128, size=(K, N)).astype(np.int32)
    return A, flags, B


# ------------------------------------------------------------------ SpMM ----
@pytest.mark.parametrize("V", [1, 2, 4, 8])
def test_spmm_bruteforce_triple_loop(V):
    """Zeros materialised, plain python loops over i, j, k (no mask needed then)."""
    M, K, N = 2 * V, 7, 5
    A, flags, B = _tiny(M, K, N, V, 0.5, 11 + V)
    want = [[sum(int(A[i][k]) * int(B[k][j]) for k in range(K)) for j in range(N)] for i in range(M)]
    got = oracle.spmm_dense(A, flags, B, V)
    assert got.dtype == np.int32 and got.tolist() == want


def test_spmm_flags_gate_the_sum():
    """Entries outside the stored vectors must not contribute even if nonzero."""
    V, M, K, N = 4, 8, 9, 3
    rng = np.random.default_rng(5)
    A = rng.integers(-128, 128, size=(M, K)).astype(np.int32)      # fully dense values
    flags = (rng.random((M // V, K)) < 0.4).astype(np.uint8)
    B = rng.integers(-128, 128, size=(K, N)).astype(np.int32)
    masked = A * np.repeat(flags, V, axis=0)
    want = masked.astype(np.int64) @ B.astype(np.int64)
    assert np.array_equal(oracle.spmm_dense(A, flags, B, V), want)
    assert not np.array_equal(want, A.astype(np.int64) @ B.astype(np.int64))


def test_spmm_sparsity_zero_is_library_matmul():
    V, M, K, N = 8, 64, 96, 48
    A, flags, B = _tiny(M, K, N, V, 1.1, 3)
    assert flags.all()
    assert np.array_equal(oracle.spmm_dense(A, flags, B, V), A.astype(np.int64) @ B.astype(np.int64))
    t = torch.from_numpy(A).to(torch.int64) @ torch.from_numpy(B).to(torch.int64)
    assert np.array_equal(oracle.spmm_dense(A, flags, B, V), t.numpy())


def test_spmm_not_transposed_or_swapped():
    """Asymmetric shapes and a one-hot probe: C[i][j] picks A[i][k0] * B[k0][j]."""
    V, M, K, N = 2, 4, 3, 5
    A = np.zeros((M, K), np.int32); A[3, 1] = 7
    flags = np.zeros((M // V, K), np.uint8); flags[1, 1] = 1
    B = np.arange(K * N, dtype=np.int32).reshape(K, N) - 6
    C = oracle.spmm_dense(A, flags, B, V)
    want = np.zeros((M, N), np.int64); want[3] = 7 * B[1]
    assert np.array_equal(C, want)


def test_spmm_closed_forms():
    V, M, K, N = 8, 32, 40, 16
    A, flags, _ = _tiny(M, K, N, V, 0.3, 9)
    ones = np.ones((K, N), np.int32)
    C = oracle.spmm_dense(A, flags, ones, V)
    assert np.array_equal(C, np.repeat(A.sum(axis=1, keepdims=True), N, axis=1))
    # one stored vector per panel holding the unit vector e_v: row p*V+v gathers B[col]
    B = np.random.default_rng(1).integers(-128, 128, size=(K, N)).astype(np.int32)
    A1 = np.zeros((M, K), np.int32); f1 = np.zeros((M // V, K), np.uint8)
    for p in range(M // V):
        col, v = (5 * p + 3) % K, p % V
        f1[p, col] = 1; A1[p * V + v, col] = 1
    C1 = oracle.spmm_dense(A1, f1, B, V)
    for p in range(M // V):
        for v in range(V):
            want = B[(5 * p + 3) % K] if v == p % V else np.zeros(N, np.int32)
            assert np.array_equal(C1[p * V + v], want)


def test_spmm_linearity():
    V, M, K, N = 4, 16, 24, 8
    A, flags, B = _tiny(M, K, N, V, 0.5, 21, lo=-60, hi=60)
    A2, _, B2 = _tiny(M, K, N, V, 0.5, 22, lo=-60, hi=60)
    A2 *= np.repeat(flags, V, axis=0).astype(np.int32)
    f = oracle.spmm_dense
    assert np.array_equal(f(A, flags, B + B2, V), f(A, flags, B, V) + f(A, flags, B2, V))
    assert np.array_equal(f(A + A2, flags, B, V), f(A, flags, B, V) + f(A2, flags, B, V))
    assert np.array_equal(f(3 * A, flags, B, V), 3 * f(A, flags, B, V))


def test_spmm_overflow_is_reported():
    V, K = 2, 4
    A = np.full((2, K), 2**30, np.int32); flags = np.ones((1, K), np.uint8)
    B = np.full((K, 1), 2, np.int32)
    with pytest.raises(OverflowError):
        oracle.spmm_dense(A, flags, B, V)
    B[:] = 0; B[0, 0] = 1
    assert oracle.spmm_dense(A, flags, B, V)[0, 0] == 2**30


def test_bcrs_to_dense_and_vector_order_invariance():
    """Vectors may be listed in any order inside a panel; the product does not change."""
    V, M, K, N = 4, 12, 10, 6
    rp, ci = wl.ragged_pattern(M, K, V, [3, 0, 5], 17)
    vals = wl.uniform_int8((len(ci), V), 18)
    A, flags = oracle.bcrs_to_dense(M, K, V, rp, ci, vals)
    # independent construction with python loops
    A_ref = np.zeros((M, K), np.int64)
    for p in range(M // V):
        for i in range(rp[p], rp[p + 1]):
            for v in range(V):
                A_ref[p * V + v, ci[i]] = vals[i, v]
    assert np.array_equal(A, A_ref)
    assert flags.sum() == len(ci) and flags[1].sum() == 0
    B = wl.uniform_int8((K, N), 19)
    C = oracle.spmm(M, K, V, rp, ci, vals, B, "L8R8")
    assert np.array_equal(C, A_ref @ B.astype(np.int64))
    assert not C[V:2 * V].any()                      # empty panel -> zero rows
    rng = np.random.default_rng(3)
    ci2, vals2 = ci.copy(), vals.copy()
    for p in range(M // V):
        perm = rng.permutation(rp[p + 1] - rp[p]) + rp[p]
        ci2[rp[p]:rp[p + 1]] = ci[perm]; vals2[rp[p]:rp[p + 1]] = vals[perm]
    assert np.array_equal(oracle.spmm(M, K, V, rp, ci2, vals2, B, "L8R8"), C)


# ----------------------------------------------------------------- SDDMM ----
def test_sddmm_bruteforce_and_order():
    V, M, Nc, Kd = 2, 6, 5, 3
    rng = np.random.default_rng(2)
    Q = rng.integers(-128, 128, size=(M, Kd)).astype(np.int32)
    Kmat = rng.integers(-128, 128, size=(Nc, Kd)).astype(np.int32)
    flags = np.array([[1, 0, 1, 0, 0], [0, 0, 0, 0, 0], [0, 1, 1, 0, 1]], np.uint8)
    want = []
    for p in range(M // V):
        for c in range(Nc):
            if flags[p][c]:
                for v in range(V):
                    want.append(sum(int(Q[p * V + v][k]) * int(Kmat[c][k]) for k in range(Kd)))
    assert oracle.sddmm_dense(Q, Kmat, flags, V).tolist() == want


@pytest.mark.parametrize("V", [2, 4, 8])
def test_sddmm_is_dense_product_at_mask_positions(V):
    M, Nc, Kd = 8 * V, 40, 32
    c = wl.sddmm_case(M, Nc, Kd, V, 0.7, "L8R8", 100 + V)
    dense = c["Q"].astype(np.int64) @ c["Kmat"].astype(np.int64).T          # library routine
    S = oracle.sddmm(M, Nc, V, c["row_ptr"], c["col_idx"], c["Q"], c["Kmat"], "L8R8")
    S = S.reshape(-1, V)
    for p in range(M // V):
        for i in range(c["row_ptr"][p], c["row_ptr"][p + 1]):
            assert np.array_equal(S[i], dense[p * V:(p + 1) * V, c["col_idx"][i]])


def test_sddmm_full_mask_is_library_matmul():
    V, M, Nc, Kd = 4, 16, 12, 20
    rng = np.random.default_rng(8)
    Q = rng.integers(-128, 128, size=(M, Kd)).astype(np.int32)
    Kmat = rng.integers(-128, 128, size=(Nc, Kd)).astype(np.int32)
    S = oracle.sddmm_dense(Q, Kmat, np.ones((M // V, Nc), np.uint8), V)
    dense = (torch.from_numpy(Q).long() @ torch.from_numpy(Kmat).long().T).numpy()
    # S[p][c][v] -> dense[p*V+v][c]
    got = S.reshape(M // V, Nc, V).transpose(0, 2, 1).reshape(M, Nc)
    assert np.array_equal(got, dense)


# ------------------------------------------------- nibbles and planes ----
def _golden_rows():
    rows = []
    with open(os.path.join(GOLDEN, "split_examples.txt")) as f:
        for line in f:
            if line.strip() and not line.startswith("#"):
                kind, val, bits, low_bits, lo, hi = line.split()
                rows.append((kind, int(val), bits, int(low_bits), int(lo), int(hi)))
    return rows


def test_split_matches_the_papers_worked_examples():
    rows = _golden_rows()
    assert len(rows) == 2
    for kind, val, bits, low_bits, lo, hi in rows:
        # the printed bit pattern is the 8-bit encoding of the printed value
        assert int(bits, 2) == val % 256
        fn = oracle.split_unsigned if kind == "unsigned" else oracle.split_signed
        got_lo, got_hi = fn(val, low_bits)
        assert (int(got_lo), int(got_hi)) == (lo, hi)
        assert lo + (hi << low_bits) == val


def test_unpack_int4_convention():
    # 0xED: bits 3:0 = 1101 -> -3 (element 0), bits 7:4 = 1110 -> -2 (element 1);
    # the high nibble read signed is the -2 of the paper's signed example.
    assert oracle.unpack_int4(np.array([0xED], np.uint8)).tolist() == [-3, -2]
    assert oracle.unpack_int4(np.array([0x70, 0x08], np.uint8)).tolist() == [0, 7, -8, 0]
    allb = np.arange(256, dtype=np.uint8)
    u = oracle.unpack_int4(allb).reshape(256, 2)
    assert u.min() == -8 and u.max() == 7
    assert np.array_equal((u[:, 0] & 15) | ((u[:, 1] & 15) << 4), np.arange(256))


@pytest.mark.parametrize("split", ["textbook", "balanced"])
def test_plane_split_identity_16bit(split):
    """(hi << 8) * B + lo * B == A16 * B with int64 sums, for both ways of splitting."""
    V, M, K, N = 8, 16, 64, 8
    rng = np.random.default_rng(77)
    flags = (rng.random((M // V, K)) < 0.5).astype(np.uint8)
    A16 = rng.integers(-32768, 32640, size=(M, K)).astype(np.int32) * np.repeat(flags, V, axis=0)
    A16[0, :4] = [-32768, 32639, -129, 127]
    A16[0, :4] *= flags[0, :4]
    B = rng.integers(-128, 128, size=(K, N)).astype(np.int32)
    lo, hi = (oracle.split_signed if split == "textbook" else oracle.split_balanced)(A16, 8)
    assert np.array_equal(lo + (hi << 8), A16)
    if split == "textbook":
        assert lo.min() >= 0 and lo.max() <= 255 and hi.min() >= -128 and hi.max() <= 127
    else:
        assert lo.min() >= -128 and lo.max() <= 127 and hi.min() >= -128 and hi.max() <= 127
    full = A16.astype(np.int64) @ B.astype(np.int64)
    assert np.array_equal(oracle.spmm_dense(A16, flags, B, V), full)
    c_hi = oracle.spmm_dense(hi.astype(np.int32), flags, B, V).astype(np.int64)
    c_lo = oracle.spmm_dense(lo.astype(np.int32), flags, B, V).astype(np.int64)
    assert np.array_equal((c_hi << 8) + c_lo, full)


def test_low_precision_cases_equal_widened_int8_cases():
    V, M, K, N = 8, 32, 48, 32
    c = wl.spmm_case(M, K, N, V, 0.5, "L4R4", 31)
    nvec = len(c["col_idx"])
    # widen by hand with an independent formula: sign-extend each nibble via int8 shifts
    def widen(packed):
        p = packed.astype(np.uint8)
        lo = (np.left_shift(p, 4).astype(np.uint8).view(np.int8) >> 4).astype(np.int8)
        hi = (p.view(np.int8) >> 4).astype(np.int8)
        return np.stack([lo, hi], axis=-1).reshape(p.shape[:-1] + (-1,))
    A8, B8 = widen(c["values"]), widen(c["B"])
    assert A8.shape == (nvec, V) and B8.shape == (K, N)
    want = oracle.spmm(M, K, V, c["row_ptr"], c["col_idx"], A8, B8, "L8R8")
    assert np.array_equal(oracle.spmm(M, K, V, c["row_ptr"], c["col_idx"], c["values"], c["B"], "L4R4"), want)
    assert np.array_equal(oracle.spmm(M, K, V, c["row_ptr"], c["col_idx"], A8, c["B"], "L8R4"), want)
    s = wl.sddmm_case(M, K, 64, V, 0.5, "L4R4", 32)
    want = oracle.sddmm(M, K, V, s["row_ptr"], s["col_idx"], widen(s["Q"]), widen(s["Kmat"]), "L8R8")
    assert np.array_equal(oracle.sddmm(M, K, V, s["row_ptr"], s["col_idx"], s["Q"], s["Kmat"], "L4R4"), want)


def test_l16r8_from_interchange_data():
    V, M, K, N = 8, 16, 32, 16
    c = wl.spmm_case(M, K, N, V, 0.5, "L16R8", 41)
    A, flags = oracle.bcrs_to_dense(M, K, V, c["row_ptr"], c["col_idx"], c["values"])
    want = A.astype(np.int64) @ c["B"].astype(np.int64)
    assert np.array_equal(oracle.spmm(M, K, V, c["row_ptr"], c["col_idx"], c["values"], c["B"], "L16R8"), want)


@pytest.mark.parametrize("prec", ["L16R16", "L16R4", "L12R4"])
def test_wide_spmm_precisions_from_interchange_data(prec):
    """Python-integer loops over the stored vectors only, operands widened by hand."""
    V, M, K, N = 4, 8, 12, 32
    c = wl.spmm_case(M, K, N, V, 0.5, prec, 43)
    vals = c["values"].astype(np.int64)                       # (nvec, V) int16 container
    if prec == "L16R16":
        Bw = [[int(x) for x in row] for row in c["B"]]
    else:                                                     # nibbles: low first, two's complement
        Bw = [[(((b >> sh) & 15) ^ 8) - 8 for b in row.tolist() for sh in (0, 4)] for row in c["B"]]
    want = [[0] * N for _ in range(M)]
    for p in range(M // V):
        for i in range(c["row_ptr"][p], c["row_ptr"][p + 1]):
            k = int(c["col_idx"][i])
            for v in range(V):
                for n in range(N):
                    want[p * V + v][n] += int(vals[i, v]) * Bw[k][n]
    got = oracle.spmm(M, K, V, c["row_ptr"], c["col_idx"], c["values"], c["B"], prec)
    assert got.tolist() == want


def test_l12_rejects_wider_values():
    V, M, K, N = 4, 8, 12, 32
    c = wl.spmm_case(M, K, N, V, 0.5, "L12R4", 44)
    bad = c["values"].copy()
    bad[0, 0] = 2048
    with pytest.raises(ValueError):
        oracle.spmm(M, K, V, c["row_ptr"], c["col_idx"], bad, c["B"], "L12R4")


def test_l16r16_is_the_four_plane_sum():
    """Section 4.4 with both operands split: A = Ah*256 + Al, B = Bh*256 + Bl (high parts signed,
    low parts unsigned) gives C = (Ch_h << 16) + ((Ch_l + Cl_h) << 8) + Cl_l, planes multiplied by
    the library matmul."""
    V, M, K, N = 8, 16, 40, 16
    c = wl.spmm_case(M, K, N, V, 0.5, "L16R16", 45)
    vals = c["values"].copy()
    vals.reshape(-1)[:4] = [-2048, 2047, -1, 255]
    A, flags = oracle.bcrs_to_dense(M, K, V, c["row_ptr"], c["col_idx"], vals)
    al, ah = oracle.split_signed(A, 8)
    bl, bh = oracle.split_signed(c["B"], 8)
    want = ((ah @ bh) << 16) + (((ah @ bl) + (al @ bh)) << 8) + (al @ bl)
    assert np.array_equal(oracle.spmm(M, K, V, c["row_ptr"], c["col_idx"], vals, c["B"], "L16R16"), want)


def test_sddmm_l16r16_against_library_matmul_and_loops():
    V, M, Nc, Kd = 4, 8, 12, 16
    c = wl.sddmm_case(M, Nc, Kd, V, 0.5, "L16R16", 46)
    got = oracle.sddmm(M, Nc, V, c["row_ptr"], c["col_idx"], c["Q"], c["Kmat"], "L16R16")
    full = torch.from_numpy(c["Q"].astype(np.int64)) @ torch.from_numpy(c["Kmat"].astype(np.int64)).T
    want = []
    for p in range(M // V):
        for i in range(c["row_ptr"][p], c["row_ptr"][p + 1]):
            for v in range(V):
                want.append(int(full[p * V + v, int(c["col_idx"][i])]))
    assert got.tolist() == want
    q, k = c["Q"].tolist(), c["Kmat"].tolist()
    i = int(c["row_ptr"][1])                                   # first vector of panel 1, row v = 2
    assert got[i * V + 2] == sum(a * b for a, b in zip(q[V + 2], k[int(c["col_idx"][i])]))


@pytest.mark.parametrize("prec", ["L8R8", "L8R4", "L4R4"])
@pytest.mark.parametrize("lu,ru", [(True, True), (True, False), (False, True)])
def test_unsigned_operands_by_integer_loops(prec, lu, ru):
    """Section 4.4.1: the same bytes read as non-negative values; loops over the stored vectors."""
    V, M, K, N = 4, 8, 12, 32
    c = wl.spmm_case(M, K, N, V, 0.5, prec, 47)
    def lhs(i, v):
        if prec == "L4R4":
            b = int(c["values"][i, v // 2]); x = (b >> (4 * (v % 2))) & 15
            return x if lu else (x ^ 8) - 8
        x = int(c["values"].view(np.uint8)[i, v])
        return x if lu else (x ^ 128) - 128
    def rhs(k, n):
        if prec in ("L8R4", "L4R4"):
            b = int(c["B"][k, n // 2]); x = (b >> (4 * (n % 2))) & 15
            return x if ru else (x ^ 8) - 8
        x = int(c["B"].view(np.uint8)[k, n])
        return x if ru else (x ^ 128) - 128
    want = [[0] * N for _ in range(M)]
    for p in range(M // V):
        for i in range(c["row_ptr"][p], c["row_ptr"][p + 1]):
            for v in range(V):
                for n in range(N):
                    want[p * V + v][n] += lhs(i, v) * rhs(int(c["col_idx"][i]), n)
    got = oracle.spmm(M, K, V, c["row_ptr"], c["col_idx"], c["values"], c["B"], prec, lhs_unsigned=lu, rhs_unsigned=ru)
    assert got.tolist() == want
    if lu and ru:
        assert got.min() >= 0


def test_unsigned_plane_emulation_identity():
    """The paper's unsigned example (Section 4.4.1): an unsigned 8-bit A as two unsigned 4-bit planes,
    C = C0 + 16 * C1, planes multiplied by the library matmul; 237 = 13 + 16 * 14."""
    lo, hi = oracle.split_unsigned(np.array([237]), 4)
    assert (int(lo[0]), int(hi[0])) == (13, 14)
    V, M, K, N = 8, 16, 24, 32
    c = wl.spmm_case(M, K, N, V, 0.5, "L8R4", 48)
    A, flags = oracle.bcrs_to_dense(M, K, V, c["row_ptr"], c["col_idx"], c["values"].view(np.uint8).astype(np.int32))
    Bu = oracle.unpack_int4(c["B"], unsigned=True)
    a0, a1 = oracle.split_unsigned(A, 4)
    want = (a0 @ Bu.astype(np.int64)) + 16 * (a1 @ Bu.astype(np.int64))
    got = oracle.spmm(M, K, V, c["row_ptr"], c["col_idx"], c["values"], c["B"], "L8R4", lhs_unsigned=True, rhs_unsigned=True)
    assert np.array_equal(got, want)


@pytest.mark.parametrize("prec", ["L8R8", "L4R4"])
def test_unsigned_sddmm_against_library_matmul(prec):
    V, M, Nc, Kd = 4, 8, 12, 32
    c = wl.sddmm_case(M, Nc, Kd, V, 0.5, prec, 49)
    if prec == "L4R4":
        Qu, Ku = oracle.unpack_int4(c["Q"], True), oracle.unpack_int4(c["Kmat"], True)
        assert Qu.min() >= 0 and Qu.max() == 15
    else:
        Qu, Ku = c["Q"].view(np.uint8).astype(np.int64), c["Kmat"].view(np.uint8).astype(np.int64)
    full = torch.from_numpy(Qu.astype(np.int64)) @ torch.from_numpy(Ku.astype(np.int64)).T
    want = []
    for p in range(M // V):
        for i in range(c["row_ptr"][p], c["row_ptr"][p + 1]):
            for v in range(V):
                want.append(int(full[p * V + v, int(c["col_idx"][i])]))
    got = oracle.sddmm(M, Nc, V, c["row_ptr"], c["col_idx"], c["Q"], c["Kmat"], prec, lhs_unsigned=True, rhs_unsigned=True)
    assert got.tolist() == want


# ------------------------------------------------------------ attention ----
def test_softmax_rows_sum_to_one_and_uniform_case():
    V = 8
    rp = np.array([0, 3, 3, 10], np.int32)
    rng = np.random.default_rng(4)
    S = rng.integers(-2000, 2000, size=10 * V).astype(np.int32)
    p = oracle.sparse_softmax(S, rp, V, 0.01).reshape(10, V)
    assert np.allclose(p[0:3].sum(axis=0), 1.0, atol=1e-14)
    assert np.allclose(p[3:10].sum(axis=0), 1.0, atol=1e-14)
    S[:] = 123
    p = oracle.sparse_softmax(S, rp, V, 0.5).reshape(10, V)
    assert np.allclose(p[0:3], 1 / 3) and np.allclose(p[3:], 1 / 7)


def test_requantize_rounding():
    p = np.array([0.0, 0.5 / 127, 1.5 / 127, 2.5 / 127, 1.0, 0.49999 / 127])
    # exact ties cannot be represented exactly in binary; check neighbours and ends
    q = oracle.requantize_probabilities(np.array([0.0, 1.0, 0.3 / 127, 0.7 / 127, 63.4 / 127]), 1 / 127)
    assert q.tolist() == [0, 127, 0, 1, 63]
    assert oracle.requantize_probabilities(np.array([2.0]), 1 / 127).tolist() == [127]
    assert oracle.requantize_probabilities(np.array([2.5, 3.5]), 1.0).tolist() == [2, 4]  # ties to even
    del p


def test_quantizer_hand_worked_values_and_bounds():
    """Symmetric per-tensor quantisation (Section 5.3, first step) on values worked out by hand: with max|x| = 2
    the 8-bit scale is 2/127 and x/s = 63.5 x; the 4-bit scale is 2/7 and x/s = 3.5 x."""
    x = np.array([-2.0, -1.01, 0.3, 0.52, 2.0, 0.0], np.float32)
    q8, s8 = oracle.quantize_per_tensor(x, 8)
    assert s8 == np.float32(2.0 / 127.0) and q8.tolist() == [-127, -64, 19, 33, 127, 0]
    q4, s4 = oracle.quantize_per_tensor(x, 4)
    assert s4 == np.float32(2.0 / 7.0) and q4.tolist() == [-7, -4, 1, 2, 7, 0]
    y = wl.normal_fp32((2, 64, 16), 5)
    q, s = oracle.quantize_per_tensor(y)
    assert np.abs(q).max() == 127
    assert np.max(np.abs(q * np.float64(s) - y)) <= 0.5 * s + 1e-7


def test_pack_int4_explicit_bytes_and_round_trip():
    """Element 2j sits in bits 3:0 and element 2j+1 in bits 7:4 of byte j, two's complement."""
    assert oracle.pack_int4(np.array([1, 2, -1, 7, -8, 0])).tolist() == [0x21, 0x7F, 0x08]
    allb = np.arange(256, dtype=np.uint8).reshape(128, 2)
    assert np.array_equal(oracle.pack_int4(oracle.unpack_int4(allb)), allb)
    q = np.random.default_rng(3).integers(-8, 8, size=(5, 3, 8))
    assert np.array_equal(oracle.unpack_int4(oracle.pack_int4(q)), q)
    with pytest.raises(ValueError):
        oracle.pack_int4(np.array([1, 2, 3]))
    with pytest.raises(ValueError):
        oracle.pack_int4(np.array([16, 0]))
    packed, s = prep.quantize_inputs_int4(np.array([[-2.0, 0.3, 0.52, 2.0]], np.float32))
    assert packed.tolist() == [[0x19, 0x72]] and s == np.float32(2.0 / 7.0)


def test_attention_against_dense_torch_reference():
    """Second, independent route: dense fp64 attention in torch with -inf at masked
    positions and the same fake-quantisation steps."""
    heads, L, dk, V = 2, 64, 16, 8
    c = wl.attention_case(heads, L, dk, V, 0.75, 900)
    q8, s_q = prep.quantize_inputs_int8(c["q"]); k8, s_k = prep.quantize_inputs_int8(c["k"])
    v8, s_v = prep.quantize_inputs_int8(c["v"])
    s_p = np.float32(1.0 / 127.0)
    O, scores, probs, codes = oracle.attention(q8, k8, v8, c["row_ptr"], c["col_idx"], V, s_q, s_k, s_v, s_p)
    flags = oracle.stored_flags(L, L, V, c["row_ptr"], c["col_idx"])
    keep = torch.from_numpy(np.repeat(flags, V, axis=0).astype(bool))
    assert bool(keep.diagonal().all())
    for h in range(heads):
        Sd = torch.from_numpy(q8[h]).double() @ torch.from_numpy(k8[h]).double().T
        x = Sd * (float(s_q) * float(s_k) / np.sqrt(dk))
        x = x.masked_fill(~keep, float("-inf"))
        Pd = torch.softmax(x, dim=1)
        Pq = torch.clamp(torch.round(Pd / float(s_p)), 0, 127)
        Od = (Pq @ torch.from_numpy(v8[h]).double()) * (float(s_p) * float(s_v))
        assert np.allclose(O[h], Od.numpy(), rtol=0, atol=1e-12)
        # stored probabilities are the dense ones at the mask positions
        pr = probs[h].reshape(-1, V)
        for p in range(L // V):
            for i in range(c["row_ptr"][p], c["row_ptr"][p + 1]):
                assert np.allclose(pr[i], Pd[p * V:(p + 1) * V, c["col_idx"][i]].numpy(), atol=1e-15)
    # quantised attention stays close to the unquantised fp64 attention on the same mask
    for h in range(heads):
        x = (torch.from_numpy(c["q"][h]).double() @ torch.from_numpy(c["k"][h]).double().T) / np.sqrt(dk)
        ref = torch.softmax(x.masked_fill(~keep, float("-inf")), dim=1) @ torch.from_numpy(c["v"][h]).double()
        assert np.max(np.abs(O[h] - ref.numpy())) < 0.15


def _half_bits_by_hand(x) -> int:
    """IEEE binary16 bit pattern of a finite double or exact Fraction, rounded to nearest even,
    by integer arithmetic on exact fractions (no library conversion)."""
    from fractions import Fraction
    import math
    x = Fraction(x)
    sign = 0x8000 if x < 0 else 0
    f = abs(x)
    if f >= Fraction(65520):                                 # half-way between 65504 and 2^16 rounds to inf
        return sign | 0x7c00
    if f == 0:
        return sign
    e = max(math.floor(math.log2(f)) if f >= Fraction(1, 1 << 14) else -14, -14)
    while f >= Fraction(2) ** (e + 1):                       # guard against log2 rounding
        e += 1
    while e > -14 and f < Fraction(2) ** e:
        e -= 1
    ulp = Fraction(2) ** (e - 10)
    n, r = divmod(f, ulp)
    n = int(n)
    if r > ulp / 2 or (r == ulp / 2 and n % 2 == 1):
        n += 1
    # n counts ulps: normal numbers have n in [1024, 2048]; 2048 carries into the next exponent
    if e == -14 and n < 1024:
        return sign | n                                      # subnormal (or zero)
    if n == 2048:
        n, e = 1024, e + 1
    return sign | ((e + 15) << 10) | (n - 1024)


def test_dequantize_rounds_once_to_nearest_even():
    """fp16 and fp32 outputs of the fused dequantisation: bit patterns against a by-hand
    rounding of the exact product, and against struct's 'e' / 'f' packers."""
    import struct
    from fractions import Fraction
    rng = np.random.default_rng(77)
    acc = np.concatenate([rng.integers(-2**31, 2**31, 400), rng.integers(-70000, 70000, 400),
                          [0, 1, -1, 2049, 2051, -2049, 4098, 65519, 65520, -65520, 2**31 - 1, -2**31]]).astype(np.int64)
    for scale in (1.0, np.float32(0.001), np.float32(1 / 127 / 127), np.float32(2.0 ** -24), np.float32(3e-8)):
        h = oracle.dequantize(acc, scale, 16)
        f = oracle.dequantize(acc, scale, 32)
        assert h.dtype == np.float16 and f.dtype == np.float32
        for a_, hb, fb in zip(acc.tolist(), h.view(np.uint16).tolist(), f.view(np.uint32).tolist()):
            exact = Fraction(a_) * Fraction(float(np.float32(scale)))   # no rounding at all
            assert hb == _half_bits_by_hand(exact), (a_, scale)
            if abs(exact) < 65520:
                assert hb == struct.unpack("<H", struct.pack("<e", float(exact)))[0]
            assert fb == struct.unpack("<I", struct.pack("<f", float(exact)))[0]
    # ties: 2049 is half-way between 2048 and 2050 -> even mantissa (2048); 2051 -> 2052
    assert oracle.dequantize(np.array([2049, 2051, 4098]), 1.0, 16).tolist() == [2048.0, 2052.0, 4096.0]
    assert np.isinf(oracle.dequantize(np.array([65520]), 1.0, 16)[0]) and oracle.dequantize(np.array([65519]), 1.0, 16)[0] == 65504


def test_attention_output_types_are_single_roundings():
    heads, L, dk, V = 2, 64, 16, 8
    c = wl.attention_case(heads, L, dk, V, 0.75, 902)
    (q, s_q), (k, s_k), (v, s_v) = (prep.quantize_inputs_int8(c[n]) for n in "qkv")
    args = (q, k, v, c["row_ptr"], c["col_idx"], V, s_q, s_k, s_v, np.float32(1 / 127))
    O64 = oracle.attention(*args)[0]
    O16 = oracle.attention(*args, out_bits=16)[0]
    O32 = oracle.attention(*args, out_bits=32)[0]
    assert O64.dtype == np.float64 and O16.dtype == np.float16 and O32.dtype == np.float32
    hb = [_half_bits_by_hand(x) for x in O64.reshape(-1).tolist()]
    assert O16.reshape(-1).view(np.uint16).tolist() == hb
    assert np.array_equal(O32, O64.astype(np.float32))
    assert np.abs(O16.astype(np.float64) - O64).max() <= 2.0 ** -11 * np.abs(O64).max()


def test_requantize_16_bit_codes():
    q = oracle.requantize_probabilities(np.array([0.0, 1.0, 2.0, 100.4 / 32639, 100.6 / 32639]), 1 / 32639, 16)
    assert q.dtype == np.int16 and q.tolist() == [0, 32639, 32639, 100, 101]
    lo, hi = oracle.split_balanced(np.array([32639]), 8)      # the largest code still splits into signed bytes
    assert hi[0] == 127 and lo[0] == 127
    lo, hi = oracle.split_balanced(np.array([32640]), 8)
    assert hi[0] == 128                                        # ... and the next one does not


@pytest.mark.parametrize("p_bits,qkv_bits", [(16, 8), (8, 4)])
def test_attention_variants_against_dense_torch_reference(p_bits, qkv_bits):
    """The 16b-8b and 8b-4b variants of the layer, by the dense masked route in torch."""
    heads, L, dk, V = 2, 64, 16, 8
    c = wl.attention_case(heads, L, dk, V, 0.75, 901)
    if qkv_bits == 4:
        (q, s_q), (k, s_k), (v, s_v) = (prep.quantize_inputs_int4(c[n]) for n in "qkv")
        # unpack by an independent formula: sign-extend nibbles with int8 shifts
        def widen(p):
            lo = (np.left_shift(p, 4).astype(np.uint8).view(np.int8) >> 4)
            hi = (p.view(np.int8) >> 4)
            return np.stack([lo, hi], axis=-1).reshape(p.shape[:-1] + (-1,)).astype(np.int8)
        qi, ki, vi = widen(q), widen(k), widen(v)
        for t, (tq, ts) in zip("qkv", ((qi, s_q), (ki, s_k), (vi, s_v))):
            oq, os_ = oracle.quantize_per_tensor(c[t], 4)
            assert os_ == ts and np.array_equal(oq, tq) and np.abs(tq).max() == 7
    else:
        (q, s_q), (k, s_k), (v, s_v) = (prep.quantize_inputs_int8(c[n]) for n in "qkv")
        qi, ki, vi = q, k, v
    pmax = {8: 127, 16: 32639}[p_bits]
    s_p = np.float32(1.0 / pmax)
    O, scores, probs, codes = oracle.attention(q, k, v, c["row_ptr"], c["col_idx"], V, s_q, s_k, s_v, s_p,
                                               p_bits=p_bits, qkv_bits=qkv_bits)
    assert codes.dtype == (np.int8 if p_bits == 8 else np.int16) and codes.max() <= pmax and codes.min() >= 0
    flags = oracle.stored_flags(L, L, V, c["row_ptr"], c["col_idx"])
    keep = torch.from_numpy(np.repeat(flags, V, axis=0).astype(bool))
    for h in range(heads):
        Sd = torch.from_numpy(qi[h]).double() @ torch.from_numpy(ki[h]).double().T
        x = (Sd * (float(s_q) * float(s_k) / np.sqrt(dk))).masked_fill(~keep, float("-inf"))
        Pq = torch.clamp(torch.round(torch.softmax(x, dim=1) / float(s_p)), 0, pmax)
        Od = (Pq @ torch.from_numpy(vi[h]).double()) * (float(s_p) * float(s_v))
        assert np.allclose(O[h], Od.numpy(), rtol=0, atol=1e-12)
    if p_bits == 16:   # finer codes: closer to the layer with unquantised probabilities than the 8-bit codes are
        O8 = oracle.attention(q, k, v, c["row_ptr"], c["col_idx"], V, s_q, s_k, s_v, np.float32(1 / 127))[0]
        for h in range(heads):
            Sd = torch.from_numpy(qi[h]).double() @ torch.from_numpy(ki[h]).double().T
            x = (Sd * (float(s_q) * float(s_k) / np.sqrt(dk))).masked_fill(~keep, float("-inf"))
            ref = (torch.softmax(x, dim=1) @ torch.from_numpy(vi[h]).double()).numpy() * float(s_v)
            assert np.abs(O[h] - ref).max() < 0.05 * np.abs(O8[h] - ref).max()


# ------------------------------------------------------------ generators ----
def test_generators_are_seeded_and_exact():
    rp, ci = wl.vector_sparse_pattern(64, 512, 8, 0.8, wl.seed_for(1))
    rp2, ci2 = wl.vector_sparse_pattern(64, 512, 8, 0.8, wl.seed_for(1))
    assert np.array_equal(ci, ci2) and np.array_equal(rp, rp2)
    assert wl.vectors_per_panel(512, 0.8) == 102 and len(ci) == 8 * 102
    assert wl.vectors_per_panel(4096, 0.9) == 410 and wl.vectors_per_panel(4096, 0.98) == 82
    for p in range(8):
        seg = ci[rp[p]:rp[p + 1]]
        assert np.all(np.diff(seg) > 0) and seg.min() >= 0 and seg.max() < 512
    rp, ci = wl.vector_sparse_pattern(64, 64, 8, 0.5, 3, keep_diagonal=True)
    for p in range(8):
        assert set(range(8 * p, 8 * p + 8)) <= set(ci[rp[p]:rp[p + 1]].tolist())


def test_requantize_scores_hand_worked_and_exact_route():
    """SDDMM results turned into the next SpMM's integer operand (Section 4.3): explicit values with exact binary
    products (ties go to even, the clamp is symmetric), and a second route through exact rational arithmetic
    wherever the fp32 product is exact."""
    from fractions import Fraction
    S = np.array([0, 1, 3, 5, -1, -3, 7, 254, 255, -255, 1000, -100000], np.int32)
    assert oracle.requantize_scores(S, 0.5).tolist() == [0, 0, 2, 2, 0, -2, 4, 127, 127, -127, 127, -127]
    assert oracle.requantize_scores(S, 0.5, 16).tolist() == [0, 0, 2, 2, 0, -2, 4, 127, 128, -128, 500, -32639]
    assert oracle.requantize_scores(np.array([65278, 65279, 70000]), 0.5, 16).tolist() == [32639, 32639, 32639]
    # scale 2^-k, scores below 2^24: the fp32 product is exact, so rint of the exact rational must agree
    rng = np.random.default_rng(9)
    S = rng.integers(-(1 << 23), 1 << 23, size=4000).astype(np.int32)
    for k in (3, 10, 17):
        want = []
        for v in S.tolist():
            q = Fraction(v, 1 << k)
            f = q.numerator // q.denominator
            r = q - f
            n = f + (1 if r > Fraction(1, 2) or (r == Fraction(1, 2) and f % 2) else 0)
            want.append(max(-32639, min(32639, n)))
        assert oracle.requantize_scores(S, 2.0 ** -k, 16).tolist() == want
    # scores beyond 2^24 are first rounded to fp32 (to even): 2^24 + 1 -> 2^24
    assert oracle.requantize_scores(np.array([(1 << 24) + 1, (1 << 24) + 3]), 2.0 ** -10, 16).tolist() == [16384, 16384]
    assert oracle.requantize_scores(np.array([5]), 0.1).dtype == np.int8 and oracle.requantize_scores(np.array([5]), 0.1, 16).dtype == np.int16
