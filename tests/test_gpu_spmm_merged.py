"""GPU parity of the SpMM on an operand's merged copy (consecutive panels sharing one panel of 8 or 16 rows at the
union of their columns: the same product as Section 4.2's, fewer rows of B fetched) against the CPU oracle, element
by element, through the C ABI; with the copy forced, forbidden and chosen automatically."""
import numpy as np
import pytest

from paper_2209_06979_amd import workloads as wl
from gpu_util import torch_dev, run_spmm_oracle

pytestmark = pytest.mark.gpu

PRECS = ["L8R8", "L8R4", "L4R4", "L16R8", "L16R16", "L16R4", "L12R4"]


def _opts(merge, slab=0, tile=0, waves=0):
    from paper_2209_06979_amd import binding as mc
    o = mc.Options()
    o.spmm_merge, o.spmm_slab, o.spmm_row_tile_bytes, o.spmm_waves = merge, slab, tile, waves
    return o


def _values(prec, nvec, V, seed):
    if prec == "L4R4":
        return wl.uniform_packed_int4((nvec, V // 2), seed)
    if prec in ("L16R8", "L16R16", "L16R4", "L12R4"):
        return wl.uniform_int16((nvec, V), seed)
    return wl.uniform_int8((nvec, V), seed)


def _run(case, options, create_options=None, dequant=None, flags=(False, False), new_values=None):
    """One problem on an operand created under create_options (default: the call's options, so that a forced copy
    is also built); returns the whole output and whether the call ran on the merged copy."""
    import torch
    from paper_2209_06979_amd import binding as mc
    mc.set_thread_options(create_options or options)
    try:
        A = mc.SparseMatrix(case["M"], case["K"], case["V"], case["row_ptr"], case["col_idx"], case["values"],
                            mc.LHS_BITS[case["prec"]])
    finally:
        mc.set_thread_options(None)
    try:
        if new_values is not None:
            A.set_values(torch_dev(new_values))
        B = torch_dev(case["B"])
        if dequant is None:
            out = torch.full((case["M"], case["N"]), -7777777, dtype=torch.int32, device="cuda")
            mc.spmm(A, B, case["prec"], out=out, options=options, lhs_unsigned=flags[0], rhs_unsigned=flags[1])
        else:
            scale, dt = dequant
            out = torch.full((case["M"], case["N"]), float("nan"), dtype=dt, device="cuda")
            mc.set_thread_options(options)
            try:
                mc.spmm_dequant(A, B, case["prec"], scale, dt, out=out)      # takes the thread's options
            finally:
                mc.set_thread_options(None)
        torch.cuda.synchronize()
        on_merged = mc.spmm_on_merged(A, case["N"], case["prec"], options) and not any(flags)
        return out.cpu().numpy(), on_merged, A.merge_group
    finally:
        A.close()


def _check(case, tag="", **kw):
    print(f"merged spmm {case['prec']} M={case['M']} K={case['K']} N={case['N']} V={case['V']} {tag}", flush=True)
    want = run_spmm_oracle(case)
    got, on_merged, group = _run(case, _opts(1), **kw)
    bad = np.argwhere(got != want)
    assert len(bad) == 0, f"merged: {len(bad)} mismatches, first at {bad[:5].tolist()}"
    return on_merged, group


@pytest.mark.parametrize("prec", PRECS)
@pytest.mark.parametrize("V", [2, 4, 8])
def test_every_precision_and_vector_length(prec, V):
    """Panels whose number is not a multiple of the group (the last merged panel runs past the matrix), rows of
    2.25 tiles (1.25 for nibbles)."""
    N = {"L8R8": 144, "L16R8": 144, "L16R16": 72}.get(prec, 160)
    panels = 37
    on_merged, group = _check(wl.spmm_case(panels * V, 700, N, V, 0.6, prec, 9100 + V))
    rows = 16 if prec in ("L8R8", "L8R4", "L4R4") else 8
    assert group == (rows // V if rows // V >= 2 else 0)
    assert on_merged == (group != 0)


@pytest.mark.parametrize("prec", ["L8R8", "L4R4", "L16R8", "L8R4"])
@pytest.mark.parametrize("V", [2, 4, 8])
def test_ragged_and_empty_panels(prec, V):
    K = 3000
    counts = [0, 1, 63, 64, 65, 130, 0, 17, 1500, 3000, 2, 0, 700, 64, 128, 5, 0, 0, 0, 0, 0, 0, 0, 0, 1, 0, 0, 0, 0, 0, 0, 0, 33]
    rp, ci = wl.ragged_pattern(V * len(counts), K, V, counts, 9200 + V)
    c = wl.spmm_case(V * len(counts), K, 128, V, 0.5, prec, 9201)
    c["row_ptr"], c["col_idx"] = rp, ci
    c["values"] = _values(prec, len(ci), V, 9202)
    _check(c, "ragged")


@pytest.mark.parametrize("tile,waves", [(64, 1), (64, 4), (128, 1), (128, 2), (128, 8), (256, 2), (256, 4)])
@pytest.mark.parametrize("stages", [1, 2])
def test_sixteen_row_panels_in_every_tile_variant(tile, waves, stages):
    """The gather kernel stages a 16-row tile in two halves: every tile width, wave count and both pipelining forms."""
    import torch
    from paper_2209_06979_amd import binding as mc
    for prec, V in (("L8R8", 2), ("L8R4", 4), ("L4R4", 8)):
        if tile == 256 and prec != "L8R8":
            continue
        c = wl.spmm_case(40 * V, 900, 320 if prec == "L8R8" else 640, V, 0.7, prec, 9300 + tile + waves)
        o = _opts(1, tile=tile, waves=waves)
        o.spmm_stages = stages
        got, on_merged, group = _run(c, o)
        assert on_merged and group * V == 16
        assert np.array_equal(got, run_spmm_oracle(c)), (prec, tile, waves, stages)


@pytest.mark.parametrize("prec", ["L8R8", "L8R4", "L4R4", "L16R8", "L16R4"])
@pytest.mark.parametrize("V", [2, 4])
def test_lds_resident_form_on_the_merged_copy(prec, V):
    """The merged copy has a K-blocked copy of its own; forced, the LDS-resident form runs on 16-row (or 8-row) panels."""
    from paper_2209_06979_amd import binding as mc
    c = wl.spmm_case(64 * V + 2 * V, 2500, 160, V, 0.4, prec, 9400 + V)
    o = _opts(1, slab=1)
    got, on_merged, _ = _run(c, o)
    assert on_merged
    assert np.array_equal(got, run_spmm_oracle(c))
    for ppw in (1, 2, 4):
        if ppw == 4 and prec != "L8R8" and prec != "L16R8":
            continue
        o = _opts(1, slab=1)
        o.spmm_slab_panels, o.spmm_slab_waves = ppw, 3
        got, _, _ = _run(c, o)
        assert np.array_equal(got, run_spmm_oracle(c)), ppw


def test_forbidden_and_automatic_agree_with_forced():
    c = wl.spmm_case(2048, 2048, 256, 2, 0.5, "L8R8", 9500)
    want = run_spmm_oracle(c)
    got_never, on_never, group_never = _run(c, _opts(-1))
    assert not on_never and group_never == 0               # the copy is not even built on a thread that forbids it
    got_never2, on_never2, group2 = _run(c, _opts(-1), create_options=_opts(0))
    assert not on_never2 and group2 == 8                   # built, but this call may not use it
    got_auto, on_auto, _ = _run(c, _opts(0))
    assert on_auto                                         # a dense V = 2 operand: the copy saves 3/4 of the fetches
    for got in (got_never, got_never2, got_auto):
        assert np.array_equal(got, want)
    sparse = wl.spmm_case(2048, 2048, 64, 8, 0.98, "L8R8", 9501)
    got, on_merged, group = _run(sparse, _opts(0))
    assert group == 2 and not on_merged                    # nothing to gain: the automatic choice keeps the operand as it is
    assert np.array_equal(got, run_spmm_oracle(sparse))


def test_unsigned_operands_keep_to_the_unmerged_operand_when_sixteen_rows_leave_no_spare_row():
    c = wl.spmm_case(64 * 4, 1200, 128, 4, 0.5, "L8R8", 9600)
    c["lhs_unsigned"], c["rhs_unsigned"] = True, True
    got, on_merged, group = _run(c, _opts(1), flags=(True, True))
    assert group == 4 and not on_merged
    assert np.array_equal(got, run_spmm_oracle(c))


@pytest.mark.parametrize("prec", ["L8R8", "L4R4", "L16R8"])
def test_values_replaced_on_the_device_reach_the_merged_copy(prec):
    V = 4
    c = wl.spmm_case(50 * V, 2500, 64, V, 0.5, prec, 9700)
    new = np.ascontiguousarray(np.roll(c["values"], 5, axis=0))
    for slab in (0, 1):
        got, on_merged, _ = _run(c, _opts(1, slab=slab), new_values=new)
        assert on_merged
        assert np.array_equal(got, run_spmm_oracle(dict(c, values=new))), (prec, slab)


def test_softmax_written_values_do_not_reach_a_stale_merged_copy():
    """mc_sparse_softmax_to_mat writes the panel format only; the SpMM after it must read that, not the merged copy."""
    import torch
    import oracle
    from paper_2209_06979_amd import binding as mc
    V, L = 8, 512
    rp, ci = wl.vector_sparse_pattern(L, L, V, 0.5, 9800)
    nvec = len(ci)
    o = _opts(1)
    mc.set_thread_options(o)
    try:
        P = mc.SparseMatrix(L, L, V, rp, ci, np.zeros((nvec, V), np.int8), 8)
    finally:
        mc.set_thread_options(None)
    assert P.merge_group == 2
    S = np.random.default_rng(9801).integers(-3000, 3000, size=nvec * V).astype(np.int32)
    mc.sparse_softmax_to_mat(P, torch_dev(S), 1e-3, 127.0)
    B = wl.uniform_int8((L, 64), 9802)
    out = mc.spmm(P, torch_dev(B), "L8R8", options=o)
    torch.cuda.synchronize()
    assert not mc.spmm_on_merged(P, 64, "L8R8", o)
    codes = mc.sparse_softmax(P, torch_dev(S.reshape(1, -1)), 1e-3, 127.0).cpu().numpy().reshape(nvec, V)
    P.close()
    assert np.array_equal(out.cpu().numpy(), oracle.spmm(L, L, V, rp, ci, codes, B, "L8R8"))


@pytest.mark.parametrize("prec", ["L8R8", "L16R4"])
def test_fused_dequantisation_outputs(prec):
    import torch
    import oracle
    c = wl.spmm_case(36 * 4, 2048, 128, 4, 0.5, prec, 9900)
    want_int = run_spmm_oracle(c)
    assert np.abs(want_int).max() < (1 << 24)
    scale = np.float32(3.1e-4)
    f32, on_merged, _ = _run(c, _opts(1), dequant=(float(scale), torch.float32))
    assert on_merged
    assert np.array_equal(f32, oracle.dequantize(want_int, scale, 32))
    f16, _, _ = _run(c, _opts(1), dequant=(float(scale), torch.float16))
    assert np.array_equal(f16.view(np.uint16), f32.astype(np.float16).view(np.uint16))


def test_very_unequal_panels_are_cut_into_work_items_on_the_merged_copy_too():
    V, K = 2, 4096
    counts = [4000] * 8 + [20] * 504
    rp, ci = wl.ragged_pattern(V * len(counts), K, V, counts, 9950)
    c = wl.spmm_case(V * len(counts), K, 128, V, 0.5, "L8R8", 9951)
    c["row_ptr"], c["col_idx"] = rp, ci
    c["values"] = wl.uniform_int8((len(ci), V), 9952)
    _check(c, "skewed")


@pytest.mark.parametrize("V,s,N,prec", [(2, 0.5, 256, "L8R8"), (4, 0.7, 512, "L8R4"), (2, 0.9, 256, "L4R4"), (4, 0.8, 256, "L16R8"),
                                        (8, 0.5, 512, "L8R8")])
def test_full_size_points_of_the_sweep_grid(V, s, N, prec):
    """4096 x 4096 points of the precision sweep, whole output against the oracle: merged copy forced, and the
    automatic configuration (which takes the merged copy at these points)."""
    c = wl.spmm_case(4096, 4096, N, V, s, prec, wl.seed_for(2, 1))
    want = run_spmm_oracle(c)
    got, on_merged, _ = _run(c, _opts(1))
    assert on_merged and np.array_equal(got, want)
    got, on_merged, _ = _run(c, _opts(0))
    assert on_merged and np.array_equal(got, want)


@pytest.mark.parametrize("prec", ["L8R8", "L4R4", "L16R8"])
def test_large_dimensions(prec):
    """A tall 32768 x 4096 operand with V = 2 (2048 merged panels, or 4096 of 8 rows) and a 16384 x 16384 one with V = 4."""
    _check(wl.spmm_case(32768, 4096, 64, 2, 0.95, prec, 9960))
    _check(wl.spmm_case(16384, 16384, 128, 4, 0.98, prec, 9961))
