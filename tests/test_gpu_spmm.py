"""GPU parity of SpMM (all precisions) against the CPU oracle: bit-exact int32."""
import numpy as np
import pytest

from paper_2209_06979_amd import workloads as wl
from gpu_util import run_spmm_gpu, run_spmm_oracle

pytestmark = pytest.mark.gpu

PRECS = ["L8R8", "L8R4", "L4R4", "L16R8"]


def _check(case, variant=(0, 0)):
    print(f"spmm case M={case['M']} K={case['K']} N={case['N']} V={case['V']} {case['prec']} variant={variant}",
          flush=True)
    got = run_spmm_gpu(case, variant)
    want = run_spmm_oracle(case)
    assert got.dtype == np.int32 and got.shape == want.shape
    bad = np.argwhere(got != want)
    assert bad.size == 0, f"{len(bad)} mismatches, first at {bad[0]}: got {got[tuple(bad[0])]} want {want[tuple(bad[0])]}"


def test_config1_l8r8_512():
    """BASELINE config 1: 512x512, V=8, 80 % of vectors zero, N=128."""
    _check(wl.spmm_case(512, 512, 128, 8, 0.8, "L8R8", wl.seed_for(1)))


@pytest.mark.parametrize("prec", PRECS)
@pytest.mark.parametrize("V", [2, 4, 8])
def test_small_all_precisions_and_vector_lengths(prec, V):
    # 3 chunks of 64 per panel (one ragged), several row tiles
    _check(wl.spmm_case(16 * V, 640, 256, V, 0.75, prec, 500 + V))


@pytest.mark.parametrize("bnb", [64, 128, 256])
@pytest.mark.parametrize("waves", [1, 2, 4, 8])
@pytest.mark.parametrize("prec", PRECS)
def test_every_tile_variant(bnb, waves, prec):
    N = 320 if prec in ("L8R8", "L16R8") else 384   # ragged last row tile for 128- and 256-byte tiles
    _check(wl.spmm_case(64, 1024, N, 8, 0.7, prec, 600 + bnb + waves), (bnb, waves))


@pytest.mark.parametrize("prec", PRECS)
def test_ragged_panels_and_empty_panels(prec):
    V, K, N = 8, 700, 192
    counts = [0, 1, 15, 16, 17, 63, 64, 65, 127, 128, 129, 0, 300, 700, 2, 0]
    M = V * len(counts)
    rp, ci = wl.ragged_pattern(M, K, V, counts, 71)
    nvec = len(ci)
    vals = {"L4R4": lambda: wl.uniform_packed_int4((nvec, V // 2), 72),
            "L16R8": lambda: wl.uniform_int16((nvec, V), 72)}.get(prec, lambda: wl.uniform_int8((nvec, V), 72))()
    B = wl.uniform_packed_int4((K, N // 2), 73) if prec in ("L8R4", "L4R4") else wl.uniform_int8((K, N), 73)
    case = dict(M=M, K=K, N=N, V=V, prec=prec, row_ptr=rp, col_idx=ci, values=vals, B=B)
    for variant in [(0, 0), (64, 4), (128, 2)]:
        _check(case, variant)


@pytest.mark.parametrize("N", [16, 32, 48, 80, 144])
def test_narrow_and_odd_widths(N):
    _check(wl.spmm_case(32, 256, N, 8, 0.5, "L8R8", 800 + N))
    _check(wl.spmm_case(32, 256, 2 * N, 4, 0.5, "L8R4", 900 + N))


def test_extreme_values_saturate_nothing():
    """All operands at -128 / most negative int4: the largest magnitudes the MFMA sees."""
    V, M, K, N = 8, 16, 512, 64
    rp, ci = wl.vector_sparse_pattern(M, K, V, 0.0, 5)
    vals = np.full((len(ci), V), -128, np.int8)
    B = np.full((K, N), -128, np.int8)
    _check(dict(M=M, K=K, N=N, V=V, prec="L8R8", row_ptr=rp, col_idx=ci, values=vals, B=B))
    v4 = np.full((len(ci), V // 2), 0x88, np.uint8)
    B4 = np.full((K, N // 2), 0x88, np.uint8)
    _check(dict(M=M, K=K, N=N, V=V, prec="L4R4", row_ptr=rp, col_idx=ci, values=v4, B=B4))
    v16 = np.full((len(ci), V), -32768, np.int16)
    B1 = np.full((K, N), 127, np.int8)
    _check(dict(M=M, K=K, N=N, V=V, prec="L16R8", row_ptr=rp, col_idx=ci, values=v16, B=B1))
    v16[:] = 32639
    _check(dict(M=M, K=K, N=N, V=V, prec="L16R8", row_ptr=rp, col_idx=ci, values=v16, B=B1))


def test_strided_operands_and_repeatability():
    import torch
    from paper_2209_06979_amd import binding as mc
    import oracle
    c = wl.spmm_case(64, 512, 128, 8, 0.8, "L8R8", 44)
    A = mc.SparseMatrix(c["M"], c["K"], c["V"], c["row_ptr"], c["col_idx"], c["values"], 8)
    Bbig = torch.zeros((c["K"], 160), dtype=torch.int8, device="cuda")
    Bbig[:, :128] = torch.from_numpy(c["B"]).cuda()
    Cbig = torch.full((c["M"], 132), 5, dtype=torch.int32, device="cuda")
    want = oracle.spmm(c["M"], c["K"], c["V"], c["row_ptr"], c["col_idx"], c["values"], c["B"], "L8R8")
    for _ in range(3):
        mc.spmm(A, Bbig[:, :128], "L8R8", out=Cbig[:, :128])
        torch.cuda.synchronize()
        got = Cbig.cpu().numpy()
        assert np.array_equal(got[:, :128], want) and (got[:, 128:] == 5).all()
    # argument checks that need a live handle
    with pytest.raises(mc.MagicubeError) as e:
        mc.spmm(A, Bbig[:, :128], "L16R8")
    assert e.value.status == mc.MC_EINVAL
    with pytest.raises(mc.MagicubeError) as e:
        mc.spmm(A, Bbig[:, 1:129], "L8R8")
    assert e.value.status == mc.MC_EALIGN
    with pytest.raises(mc.MagicubeError) as e:
        mc.spmm(A, Bbig[:, :120], "L8R8")
    assert e.value.status == mc.MC_EINVAL
    A.close()


@pytest.mark.parametrize("prec,V,s,N", [("L8R8", 8, 0.9, 256), ("L8R8", 2, 0.5, 128), ("L8R4", 4, 0.98, 512),
                                        ("L4R4", 8, 0.7, 512), ("L16R8", 8, 0.9, 256)])
def test_full_size_4096(prec, V, s, N):
    """BASELINE configs 2 and 4 at full size, whole output compared."""
    seed = wl.seed_for(4 if prec == "L16R8" else 2, int(s * 100) + V)
    _check(wl.spmm_case(4096, 4096, N, V, s, prec, seed))


def test_set_values_device_round_trip():
    import torch
    from paper_2209_06979_amd import binding as mc
    import oracle
    for prec in PRECS:
        c = wl.spmm_case(64, 512, 128, 8, 0.6, prec, 300)
        bits = mc.LHS_BITS[prec]
        zeros = np.zeros_like(c["values"])
        A = mc.SparseMatrix(c["M"], c["K"], c["V"], c["row_ptr"], c["col_idx"], zeros, bits)
        A.set_values(torch.from_numpy(np.ascontiguousarray(c["values"]).view(np.uint8)).cuda())
        C = mc.spmm(A, torch.from_numpy(c["B"]).cuda(), prec)
        torch.cuda.synchronize()
        assert np.array_equal(C.cpu().numpy(), run_spmm_oracle(c)), prec
        A.close()


SWEEP = [(prec, V, s, N)
         for prec in PRECS for V, s, N in [(8, 0.5, 128), (8, 0.7, 512), (8, 0.95, 256), (4, 0.8, 256), (2, 0.9, 512),
                                           (4, 0.5, 128), (2, 0.98, 128)]]


@pytest.mark.parametrize("prec,V,s,N", SWEEP)
def test_config2_sweep_points_full_size(prec, V, s, N):
    """A spread of BASELINE config 2 grid points (4096 x 4096; V, sparsity, N, precision), whole output compared,
    in the launch configuration the library picks by itself (the one bench.py times)."""
    _check(wl.spmm_case(4096, 4096, N, V, s, prec, wl.seed_for(2, 1000 + int(s * 100) + 10 * V + N)))


def test_ablation_shape_and_tall_matrix():
    """The shape of the paper's ablation matrix (Section 5.1: M=256, K=2304, N=512) and a tall, very sparse one."""
    for prec in PRECS:
        _check(wl.spmm_case(256, 2304, 512, 8, 0.7, prec, 77))
    _check(wl.spmm_case(32768, 8192, 64, 8, 0.99, "L8R8", 78))
    _check(wl.spmm_case(16384, 1024, 1024, 4, 0.9, "L8R4", 79))


@pytest.mark.parametrize("prec", ["L8R8", "L8R4"])
def test_dense_operand_spanning_more_than_4_gib(prec):
    """Rows of B a mebibyte apart: the last row starts beyond 2^32 bytes, which takes the kernel form with
    64-bit row offsets (one chunk in flight)."""
    import torch
    from paper_2209_06979_amd import binding as mc
    K, ld = 4097, (1 << 20) + 16
    c = wl.spmm_case(256, K - 1, 128, 8, 0.9, prec, 7400)
    # the patterns of the generator address K - 1 columns; one more vector per panel names the last row
    rp = c["row_ptr"] + np.arange(len(c["row_ptr"]), dtype=np.int32)
    ci = np.concatenate([np.r_[c["col_idx"][a:b], K - 1] for a, b in zip(c["row_ptr"][:-1], c["row_ptr"][1:])]).astype(np.int32)
    vals = np.concatenate([np.concatenate([c["values"][a:b], c["values"][a:a + 1]]) for a, b in zip(c["row_ptr"][:-1], c["row_ptr"][1:])])
    Bh = np.concatenate([c["B"], c["B"][:1]])
    case = dict(c, K=K, row_ptr=rp, col_idx=ci, values=np.ascontiguousarray(vals), B=Bh)
    want = run_spmm_oracle(case)
    A = mc.SparseMatrix(256, K, 8, rp, ci, case["values"], mc.LHS_BITS[prec])
    big = torch.empty((K, ld), dtype=torch.from_numpy(Bh).dtype, device="cuda")
    assert big.element_size() == 1 and (K - 1) * ld > 1 << 32
    Bv = big[:, :Bh.shape[1]]
    Bv.copy_(torch.from_numpy(Bh).cuda())
    print(f"spmm {prec} with B rows {ld} bytes apart", flush=True)
    got = mc.spmm(A, Bv, prec)
    torch.cuda.synchronize()
    assert np.array_equal(got.cpu().numpy(), want)
    A.close()
    del big


@pytest.mark.parametrize("prec", ["L8R8", "L4R4", "L16R8"])
def test_large_dimensions(prec):
    """16384 x 16384 at 98 % sparsity (2048 panels, K four times the sweep's) and a tall 32768 x 4096 one with V = 2."""
    _check(wl.spmm_case(16384, 16384, 128, 8, 0.98, prec, 7200))
    _check(wl.spmm_case(32768, 4096, 64, 2, 0.95, prec, 7201))


@pytest.mark.parametrize("prec", PRECS)
@pytest.mark.parametrize("M,K,N,s", [(128, 4096, 512, 0.5), (256, 2304, 512, 0.7), (1024, 4096, 256, 0.7), (8, 4096, 256, 0.0)])
def test_few_panels_take_narrow_tiles(prec, M, K, N, s):
    """Fewer panels than compute units: the automatic choice narrows the row tiles (same results)."""
    _check(wl.spmm_case(M, K, N, 8, s, prec, 7100 + M))


def test_phase_probe_computes_the_product_and_stamps_every_wave_in_order():
    """The instrumented instantiation of the SpMM kernel: the same product as the oracle's, and per wave ten clock
    readings that never run backwards; operands outside its one kernel form are refused."""
    import torch
    from paper_2209_06979_amd import binding as mc
    V, K, N = 8, 900, 320                                      # 2.5 tiles of 128 bytes
    counts = [0, 1, 63, 64, 65, 129, 300, 512, 7, 0, 450]
    M = V * len(counts)
    rp, ci = wl.ragged_pattern(M, K, V, counts, 181)
    c = dict(M=M, K=K, N=N, V=V, prec="L8R8", row_ptr=rp, col_idx=ci, values=wl.uniform_int8((len(ci), V), 182),
             B=wl.uniform_int8((K, N), 183))
    A = mc.SparseMatrix(M, K, V, rp, ci, c["values"], 8)
    out = torch.full((M, N), -7777777, dtype=torch.int32, device="cuda")
    _, trace = mc.probe_spmm_phases(A, torch.from_numpy(c["B"]).cuda(), out=out)
    torch.cuda.synchronize()
    A.close()
    assert np.array_equal(out.cpu().numpy(), run_spmm_oracle(c))
    t = trace.cpu().numpy()
    assert t.shape == (len(counts) * 3 * 2, 10) and (t > 0).all()
    assert (np.diff(t, axis=1) >= 0).all()
    assert t.max() - t.min() < 100_000                         # all within a millisecond of each other (100 MHz ticks)
    long_panels = mc.SparseMatrix(8, K, V, [0, 600], np.arange(600, dtype=np.int32), wl.uniform_int8((600, V), 184), 8)
    with pytest.raises(mc.MagicubeError) as e:                 # 10 chunks: more than two waves keep in flight
        mc.probe_spmm_phases(long_panels, torch.from_numpy(c["B"]).cuda())
    assert e.value.status == mc.MC_EUNSUPPORTED
    long_panels.close()


@pytest.mark.parametrize("bnb,waves", [(64, 1), (128, 2), (256, 4)])
def test_gather_probe_fetches_the_rows_spmm_would(bnb, waves):
    """The gather-only measurement kernel: every workgroup reports the first word of its staged rows."""
    import torch
    from paper_2209_06979_amd import binding as mc
    V, K, N = 8, 700, 320
    counts = [0, 1, 63, 64, 65, 129, 300, 700]
    M = V * len(counts)
    rp, ci = wl.ragged_pattern(M, K, V, counts, 171)
    B = wl.uniform_int8((K, N), 172)
    A = mc.SparseMatrix(M, K, V, rp, ci, wl.uniform_int8((len(ci), V), 173), 8)
    mc.set_spmm_variant(bnb, waves)
    try:
        sink = mc.probe_gather(A, torch.from_numpy(B).cuda(), "L8R8")
        torch.cuda.synchronize()
    finally:
        mc.set_spmm_variant(0, 0)
        A.close()
    sink = sink.cpu().numpy()
    ntiles = (N + bnb - 1) // bnb
    for p, n in enumerate(counts):
        for t in range(ntiles):
            if n == 0:
                want = 0
            else:
                nch = (n + 63) // 64
                c_last = (nch - 1) // waves * waves            # last chunk of wave 0
                col = ci[rp[p] + c_last * 64]
                want = int(B[col, t * bnb:t * bnb + 4].copy().view(np.int32)[0])
            assert sink[p * ntiles + t] == want, (p, t)


@pytest.mark.parametrize("prec", PRECS + ["L16R16", "L16R4"])
def test_very_unequal_panels_are_split_into_work_items(prec):
    """A few panels many times longer than the rest: the library cuts them into several work items whose
    partial results are added with integer atomics.  Same result with the splitting turned off."""
    from paper_2209_06979_amd import binding as mc
    V, K, N = 8, 2048, 192
    counts = [30] * 40 + [2048, 1500, 0, 1] + [50] * 20
    M = V * len(counts)
    rp, ci = wl.ragged_pattern(M, K, V, counts, 181)
    nvec = len(ci)
    if prec == "L4R4":
        vals = wl.uniform_packed_int4((nvec, V // 2), 182)
    elif prec.startswith("L16"):
        vals = wl.uniform_int16((nvec, V), 182, -512, 511)
    else:
        vals = wl.uniform_int8((nvec, V), 182)
    if prec.endswith("R4"):
        B = wl.uniform_packed_int4((K, N // 2), 183)
    elif prec.endswith("R16"):
        B = wl.uniform_int16((K, N), 183, -512, 511)
    else:
        B = wl.uniform_int8((K, N), 183)
    case = dict(M=M, K=K, N=N, V=V, prec=prec, row_ptr=rp, col_idx=ci, values=vals, B=B)
    for variant in [(0, 0), (64, 1), (128, 4)]:
        _check(case, variant)
    mc.set_spmm_splitting(False)
    try:
        _check(case)
    finally:
        mc.set_spmm_splitting(True)
    if prec == "L8R8":
        case["lhs_unsigned"] = case["rhs_unsigned"] = True
        _check(case)


@pytest.mark.parametrize("prec", ["L8R8", "L8R4", "L4R4"])
def test_config2_whole_grid_full_size(prec):
    """Every point of BASELINE config 2 for one precision: V in {2,4,8} x sparsity in {0.5 .. 0.98} x
    N in {128,256,512} at 4096 x 4096, whole outputs compared (54 points per precision)."""
    import torch
    from paper_2209_06979_amd import binding as mc
    for V in (2, 4, 8):
        for s in (0.5, 0.7, 0.8, 0.9, 0.95, 0.98):
            # one pattern and one set of A values per (V, s); B per N
            base = wl.spmm_case(4096, 4096, 512, V, s, prec, wl.seed_for(2, 2000 + int(s * 100) + 10 * V))
            A = mc.SparseMatrix(4096, 4096, V, base["row_ptr"], base["col_idx"], base["values"], mc.LHS_BITS[prec])
            for N in (128, 256, 512):
                nb = N // 2 if prec != "L8R8" else N
                Bh = np.ascontiguousarray(base["B"][:, :nb])
                print(f"config 2: {prec} V={V} s={s} N={N}", flush=True)
                got = mc.spmm(A, torch.from_numpy(Bh).cuda(), prec).cpu().numpy()
                want = run_spmm_oracle(dict(base, N=N, B=Bh))
                assert np.array_equal(got, want), (prec, V, s, N)
            A.close()


@pytest.mark.parametrize("prec", PRECS + ["L16R16", "L16R4"])
def test_one_and_two_chunks_in_flight_agree(prec):
    """The kernel form with two chunks of gathered rows in flight per wave (default where it applies) and the
    one-chunk form, on panels short enough for the former and on longer ones."""
    from paper_2209_06979_amd import binding as mc
    for s, N in ((0.9, 256), (0.97, 128), (0.6, 256)):
        case = wl.spmm_case(256, 2048, N, 8, s, prec, 195)
        for stages in (1, 2):
            mc.set_spmm_stages(stages)
            try:
                for variant in [(0, 0), (64, 1), (128, 2), (256, 8)]:
                    _check(case, variant)
            finally:
                mc.set_spmm_stages(2)


@pytest.mark.parametrize("prec", PRECS)
@pytest.mark.parametrize("V", [2, 8])
def test_matrix_without_any_stored_vector(prec, V):
    """Every panel empty (a valid, all-zero sparse operand with no value buffer at all): C must be
    written as zeros, and replacing the (zero) values from the device is a no-op."""
    import torch
    from paper_2209_06979_amd import binding as mc
    M, K, N = 8 * V, 64, 64
    rp, ci = wl.ragged_pattern(M, K, V, np.zeros(M // V, np.int64), 75)
    vals = np.zeros((0, V // 2 if prec == "L4R4" else V), {"L16R8": np.int16, "L4R4": np.uint8}.get(prec, np.int8))
    B = wl.uniform_packed_int4((K, N // 2), 76) if prec in ("L8R4", "L4R4") else wl.uniform_int8((K, N), 76)
    case = dict(M=M, K=K, N=N, V=V, prec=prec, row_ptr=rp, col_idx=ci, values=vals, B=B)
    _check(case)
    A = mc.SparseMatrix(M, K, V, rp, ci, vals, mc.LHS_BITS[prec])
    A.set_values(torch.zeros(0, dtype=torch.int8, device="cuda"))
    out = mc.spmm_dequant(A, torch.from_numpy(B).cuda(), prec, 0.5, torch.float16)
    torch.cuda.synchronize()
    assert out.shape == (M, N) and not out.any()
    A.close()
