"""GPU parity of the SpMM form that keeps K-blocks of B resident in LDS (Section 4.2's product, computed without
re-fetching B rows per stored vector) against the CPU oracle, element by element, through the C ABI."""
import numpy as np
import pytest

from paper_2209_06979_amd import workloads as wl
from gpu_util import torch_dev, run_spmm_oracle

pytestmark = pytest.mark.gpu

PRECS = ["L8R8", "L8R4", "L4R4", "L16R8", "L16R4", "L12R4"]


def _forced():
    from paper_2209_06979_amd import binding as mc
    o = mc.Options()
    o.spmm_slab = 1
    return o


def _run(case, options=None, dequant=None):
    """Runs one problem with the LDS-resident form forced (the K-blocked copy is built because the creating thread
    asks for it) and returns the whole output."""
    import torch
    from paper_2209_06979_amd import binding as mc
    o = options or _forced()
    mc.set_thread_options(o)
    try:
        A = mc.SparseMatrix(case["M"], case["K"], case["V"], case["row_ptr"], case["col_idx"], case["values"],
                            mc.LHS_BITS[case["prec"]])
        B = torch_dev(case["B"])
        if dequant is None:
            out = torch.full((case["M"], case["N"]), -7777777, dtype=torch.int32, device="cuda")
            mc.spmm(A, B, case["prec"], out=out, options=o)
        else:
            scale, dt = dequant
            out = torch.full((case["M"], case["N"]), float("nan"), dtype=dt, device="cuda")
            mc.spmm_dequant(A, B, case["prec"], scale, dt, out=out)      # takes the thread's options
        torch.cuda.synchronize()
        A.close()
        return out.cpu().numpy()
    finally:
        mc.set_thread_options(None)


def _check(case, tag=""):
    print(f"slab spmm {case['prec']} M={case['M']} K={case['K']} N={case['N']} V={case['V']} {tag}", flush=True)
    got, want = _run(case), run_spmm_oracle(case)
    bad = np.argwhere(got != want)
    assert len(bad) == 0, f"{len(bad)} mismatches, first at {bad[:5].tolist()}"


@pytest.mark.parametrize("prec", PRECS)
@pytest.mark.parametrize("V", [2, 4, 8])
def test_every_precision_and_vector_length(prec, V):
    """Three K-blocks, the last one partial; several column tiles with a ragged last one for the 8-bit B."""
    N = {"L8R8": 144, "L16R8": 144}.get(prec, 160)            # 144 bytes / 80 bytes of nibbles per row: 2.25 / 1.25 tiles
    _check(wl.spmm_case(64 * V, 2500, N, V, 0.5, prec, 8100 + V))


@pytest.mark.parametrize("prec", ["L8R8", "L4R4", "L16R8"])
def test_ragged_and_empty_panels(prec):
    V, K = 8, 3000
    counts = [0, 1, 63, 64, 65, 130, 0, 17, 1500, 3000, 2, 0, 700, 64, 128, 5]
    rp, ci = wl.ragged_pattern(V * len(counts), K, V, counts, 8200)
    c = wl.spmm_case(V * len(counts), K, 128, V, 0.5, prec, 8201)
    c["row_ptr"], c["col_idx"] = rp, ci
    nvec = len(ci)
    c["values"] = (wl.uniform_packed_int4((nvec, V // 2), 8202) if prec == "L4R4" else
                   wl.uniform_int16((nvec, V), 8202) if prec == "L16R8" else wl.uniform_int8((nvec, V), 8202))
    _check(c, "ragged")


@pytest.mark.parametrize("K", [64, 1024, 1025, 2048, 5000])
def test_block_boundaries_of_k(K):
    """K below, at and just above one block; a whole number of blocks; five blocks."""
    _check(wl.spmm_case(256, K, 64, 8, 0.6, "L8R8", 8300 + K))
    _check(wl.spmm_case(128, K, 64, 4, 0.3, "L8R4", 8301 + K))


@pytest.mark.parametrize("shape", [(8, 8), (16, 8), (40, 8), (120, 8), (512, 8), (2048, 2), (4096, 2), (8, 2)])
def test_work_splits(shape):
    """Few panels (several waves share a panel), exactly as many as waves, and many panels per wave (the
    accumulators of up to four panels live in a wave's registers; more panels mean more workgroups)."""
    M, V = shape
    _check(wl.spmm_case(M, 2048, 256, V, 0.5, "L8R8", 8400 + M), "work split")
    _check(wl.spmm_case(M, 2048, 256, V, 0.5, "L4R4", 8401 + M), "work split")


def test_extreme_values_wrap_free():
    """All operands at their extremes: the int32 sums of the largest case still fit (4096 * 128 * 128)."""
    V, K, N = 8, 2048, 64
    c = wl.spmm_case(64, K, N, V, 0.0, "L8R8", 8500)
    c["values"][:] = -128
    c["B"][:] = -128
    _check(c, "extremes")
    c = wl.spmm_case(64, K, N, V, 0.0, "L16R8", 8501)
    c["values"][:] = 32639
    c["values"][::3] = -32768
    c["B"][:] = 127
    c["B"][::2] = -128
    K2 = 256                                                   # 256 * 32768 * 128 = 2^30: fits
    c2 = wl.spmm_case(64, K2, N, V, 0.0, "L16R8", 8502)
    c2["values"][:] = np.where(np.arange(c2["values"].size).reshape(c2["values"].shape) % 2, 32639, -32768)
    _check(c2, "16-bit extremes")


@pytest.mark.parametrize("prec", ["L8R8", "L16R4"])
def test_fused_dequantisation_outputs(prec):
    """fp32 and fp16 outputs of the same kernel: equal to the oracle's single rounding wherever the integer fits 24
    bits (these sizes do), the fp16 output equal to the kernel's fp32 output rounded once."""
    import torch
    import oracle
    c = wl.spmm_case(256, 2048, 128, 8, 0.5, prec, 8600)
    want_int = run_spmm_oracle(c)
    assert np.abs(want_int).max() < (1 << 24)
    scale = np.float32(3.1e-4)
    f32 = _run(c, dequant=(float(scale), torch.float32))
    assert np.array_equal(f32, oracle.dequantize(want_int, scale, 32))
    f16 = _run(c, dequant=(float(scale), torch.float16))
    assert np.array_equal(f16.view(np.uint16), f32.astype(np.float16).view(np.uint16))


def test_values_replaced_on_the_device_reach_the_blocked_copy():
    import torch
    from paper_2209_06979_amd import binding as mc
    for prec in ("L8R8", "L4R4", "L16R8"):
        c = wl.spmm_case(256, 2500, 64, 8, 0.5, prec, 8700)
        o = _forced()
        mc.set_thread_options(o)
        try:
            A = mc.SparseMatrix(c["M"], c["K"], 8, c["row_ptr"], c["col_idx"], c["values"], mc.LHS_BITS[prec])
            new = np.ascontiguousarray(np.roll(c["values"], 3, axis=0))
            A.set_values(torch_dev(new))
            out = torch.full((256, 64), -7777777, dtype=torch.int32, device="cuda")
            mc.spmm(A, torch_dev(c["B"]), prec, out=out, options=o)
            torch.cuda.synchronize()
            A.close()
        finally:
            mc.set_thread_options(None)
        c2 = dict(c, values=new)
        assert np.array_equal(out.cpu().numpy(), run_spmm_oracle(c2)), prec


def test_softmax_written_values_fall_back_to_the_gather_form():
    """mc_sparse_softmax_to_mat writes the panel format only; a following SpMM must not use the stale blocked copy."""
    import torch
    import oracle
    from paper_2209_06979_amd import binding as mc
    V, L = 8, 512
    rp, ci = wl.vector_sparse_pattern(L, L, V, 0.5, 8800)
    nvec = len(ci)
    o = _forced()
    mc.set_thread_options(o)
    try:
        P = mc.SparseMatrix(L, L, V, rp, ci, np.zeros((nvec, V), np.int8), 8)
        S = np.random.default_rng(8801).integers(-3000, 3000, size=nvec * V).astype(np.int32)
        mc.sparse_softmax_to_mat(P, torch_dev(S), 1e-3, 127.0)
        B = wl.uniform_int8((L, 64), 8802)
        out = mc.spmm(P, torch_dev(B), "L8R8", options=o)
        torch.cuda.synchronize()
        codes = mc.sparse_softmax(P, torch_dev(S.reshape(1, -1)), 1e-3, 127.0).cpu().numpy().reshape(nvec, V)
        P.close()
    finally:
        mc.set_thread_options(None)
    want = oracle.spmm(L, L, V, rp, ci, codes, B, "L8R8")      # exact product of the GPU's own codes
    assert np.array_equal(out.cpu().numpy(), want)


@pytest.mark.parametrize("V,s,N,prec", [(8, 0.5, 512, "L8R8"), (2, 0.5, 256, "L8R8"), (4, 0.7, 512, "L8R4"), (8, 0.5, 256, "L16R8"),
                                        (2, 0.7, 128, "L4R4")])
def test_full_size_points_of_the_sweep_grid(V, s, N, prec):
    """4096 x 4096 points of the precision sweep, whole output against the oracle, in the automatic configuration
    (which takes the LDS-resident form at these points) and with the form forced."""
    import torch
    from paper_2209_06979_amd import binding as mc
    c = wl.spmm_case(4096, 4096, N, V, s, prec, wl.seed_for(2, 1))
    want = run_spmm_oracle(c)
    got = _run(c)
    assert np.array_equal(got, want)
    A = mc.SparseMatrix(4096, 4096, V, c["row_ptr"], c["col_idx"], c["values"], mc.LHS_BITS[prec])
    out = torch.full((4096, N), -7777777, dtype=torch.int32, device="cuda")
    mc.spmm(A, torch_dev(c["B"]), prec, out=out)
    torch.cuda.synchronize()
    A.close()
    assert np.array_equal(out.cpu().numpy(), want)
