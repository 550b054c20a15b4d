"""GPU parity of unsigned 8- and 4-bit operands (Section 4.4.1) against the CPU oracle: bit-exact."""
import numpy as np
import pytest

from paper_2209_06979_amd import workloads as wl
from gpu_util import run_spmm_gpu, run_spmm_oracle

pytestmark = pytest.mark.gpu

SIGNS = [(True, True), (True, False), (False, True)]
PRECS = ["L8R8", "L8R4", "L4R4"]


def _spmm(case, variant=(0, 0)):
    print(f"spmm case M={case['M']} K={case['K']} N={case['N']} V={case['V']} {case['prec']} "
          f"unsigned=({case.get('lhs_unsigned')}, {case.get('rhs_unsigned')}) variant={variant}", flush=True)
    got, want = run_spmm_gpu(case, variant), run_spmm_oracle(case)
    bad = np.argwhere(got != want)
    assert bad.size == 0, f"{len(bad)} mismatches, first at {bad[0]}: got {got[tuple(bad[0])]} want {want[tuple(bad[0])]}"


def _case(M, K, N, V, s, prec, seed, lu, ru):
    c = wl.spmm_case(M, K, N, V, s, prec, seed)
    c["lhs_unsigned"], c["rhs_unsigned"] = lu, ru
    return c


@pytest.mark.parametrize("prec", PRECS)
@pytest.mark.parametrize("lu,ru", SIGNS)
@pytest.mark.parametrize("V", [2, 4, 8])
def test_spmm_unsigned_small(prec, lu, ru, V):
    _spmm(_case(16 * V, 640, 256, V, 0.75, prec, 5000 + V, lu, ru))


@pytest.mark.parametrize("bnb", [64, 128, 256])
@pytest.mark.parametrize("waves", [1, 2, 4, 8])
@pytest.mark.parametrize("prec", PRECS)
def test_spmm_unsigned_every_tile_variant(bnb, waves, prec):
    N = 320 if prec == "L8R8" else 384
    _spmm(_case(64, 1024, N, 8, 0.7, prec, 5100 + bnb + waves, True, True), (bnb, waves))


@pytest.mark.parametrize("prec", PRECS)
@pytest.mark.parametrize("lu,ru", SIGNS)
def test_spmm_unsigned_ragged_and_empty_panels(prec, lu, ru):
    V, K, N = 8, 700, 192
    counts = [0, 1, 15, 16, 17, 63, 64, 65, 127, 128, 129, 0, 300, 700, 2, 0]
    M = V * len(counts)
    rp, ci = wl.ragged_pattern(M, K, V, counts, 5201)
    nvec = len(ci)
    vals = wl.uniform_packed_int4((nvec, V // 2), 5202) if prec == "L4R4" else wl.uniform_int8((nvec, V), 5202)
    B = wl.uniform_int8((K, N), 5203) if prec == "L8R8" else wl.uniform_packed_int4((K, N // 2), 5203)
    case = dict(M=M, K=K, N=N, V=V, prec=prec, row_ptr=rp, col_idx=ci, values=vals, B=B, lhs_unsigned=lu, rhs_unsigned=ru)
    for variant in [(0, 0), (64, 4), (128, 2)]:
        _spmm(case, variant)


def test_spmm_unsigned_extreme_values():
    """Every operand at its largest value: 255 * 255 and 15 * 15 per term."""
    V, M, K, N = 8, 16, 512, 64
    rp, ci = wl.vector_sparse_pattern(M, K, V, 0.0, 5)
    full8 = np.full((len(ci), V), -1, np.int8)
    _spmm(dict(M=M, K=K, N=N, V=V, prec="L8R8", row_ptr=rp, col_idx=ci, values=full8, B=np.full((K, N), -1, np.int8),
               lhs_unsigned=True, rhs_unsigned=True))
    full4 = np.full((len(ci), V // 2), 0xFF, np.uint8)
    _spmm(dict(M=M, K=K, N=N, V=V, prec="L4R4", row_ptr=rp, col_idx=ci, values=full4, B=np.full((K, N // 2), 0xFF, np.uint8),
               lhs_unsigned=True, rhs_unsigned=True))
    _spmm(dict(M=M, K=K, N=N, V=V, prec="L8R4", row_ptr=rp, col_idx=ci, values=full8, B=np.zeros((K, N // 2), np.uint8),
               lhs_unsigned=True, rhs_unsigned=True))


@pytest.mark.parametrize("prec", PRECS)
def test_spmm_unsigned_full_size_4096(prec):
    _spmm(_case(4096, 4096, 256, 8, 0.9, prec, wl.seed_for(2, 77), True, True))


def test_unsigned_is_refused_for_wide_operands():
    import torch
    from paper_2209_06979_amd import binding as mc
    c = wl.spmm_case(16, 64, 32, 8, 0.5, "L16R8", 5301)
    A = mc.SparseMatrix(c["M"], c["K"], c["V"], c["row_ptr"], c["col_idx"], c["values"], 16)
    with pytest.raises(mc.MagicubeError) as e:
        mc.spmm(A, torch.from_numpy(c["B"]).cuda(), "L16R8", lhs_unsigned=True)
    assert e.value.status == mc.MC_EUNSUPPORTED
    A.close()


# -------------------------------------------------------------------- SDDMM ----
def _sddmm(case, variants=(-1,)):
    from gpu_util import run_sddmm_gpu, run_sddmm_oracle
    want = run_sddmm_oracle(case)
    for waves in variants:      # -1: automatic; 0: operands straight from memory; 1..8: waves of the LDS-staged kernel
        print(f"sddmm case M={case['M']} Nc={case['Nc']} Kd={case['Kd']} V={case['V']} {case['prec']} "
              f"unsigned=({case.get('lhs_unsigned')}, {case.get('rhs_unsigned')}) waves={waves}", flush=True)
        got = run_sddmm_gpu(case, waves)
        assert got.shape == want.shape
        bad = np.flatnonzero(got != want)
        assert bad.size == 0, f"{len(bad)} mismatches, first at {bad[0]}: got {got[bad[0]]} want {want[bad[0]]}"


@pytest.mark.parametrize("prec", ["L8R8", "L4R4"])
@pytest.mark.parametrize("lu,ru", SIGNS)
@pytest.mark.parametrize("V", [2, 4, 8])
@pytest.mark.parametrize("Kd", [64, 96, 256, 1056])
def test_sddmm_unsigned(prec, lu, ru, V, Kd):
    c = wl.sddmm_case(16 * V, 300, Kd, V, 0.7, prec, 5400 + V + Kd)
    c["lhs_unsigned"], c["rhs_unsigned"] = lu, ru
    _sddmm(c, variants=(-1, 0, 1, 2, 4, 8))


@pytest.mark.parametrize("prec,Kd", [("L8R8", 128), ("L8R8", 512), ("L8R8", 1024), ("L4R4", 128), ("L4R4", 512), ("L4R4", 1024),
                                     ("L4R4", 2048)])
@pytest.mark.parametrize("lu,ru", SIGNS)
def test_sddmm_unsigned_every_staged_row_length(prec, Kd, lu, ru):
    """Rows of 64 .. 1024 bytes run on the LDS-staged kernel (512 and 1024 in passes), also with unsigned operands."""
    c = wl.sddmm_case(64, 300, Kd, 8, 0.5, prec, 5450 + Kd)
    c["lhs_unsigned"], c["rhs_unsigned"] = lu, ru
    _sddmm(c, variants=(-1, 0, 2, 8))


@pytest.mark.parametrize("prec", ["L8R8", "L4R4"])
def test_sddmm_unsigned_ragged_and_extremes(prec):
    V, Nc, Kd = 8, 500, 128
    counts = [0, 1, 15, 16, 17, 63, 64, 65, 0, 129, 500, 3]
    M = V * len(counts)
    rp, ci = wl.ragged_pattern(M, Nc, V, counts, 5501)
    nb = Kd // 2 if prec == "L4R4" else Kd
    Q, Km = np.full((M, nb), 0xFF, np.uint8), np.full((Nc, nb), 0xFF, np.uint8)     # every operand at its maximum
    Q[::3] = wl.uniform_packed_int4((len(Q[::3]), nb), 5502)
    _sddmm(dict(M=M, Nc=Nc, Kd=Kd, V=V, prec=prec, row_ptr=rp, col_idx=ci, Q=Q, Kmat=Km, lhs_unsigned=True, rhs_unsigned=True))


@pytest.mark.parametrize("prec", ["L8R8", "L4R4"])
def test_sddmm_unsigned_full_size_4096(prec):
    c = wl.sddmm_case(4096, 4096, 256, 8, 0.9, prec, wl.seed_for(3, 77))
    c["lhs_unsigned"], c["rhs_unsigned"] = True, True
    _sddmm(c)
