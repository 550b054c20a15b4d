"""GPU parity of the emulated wide precisions (table of supported precisions, Section 4.4):
SpMM L16-R16 / L16-R4 / L12-R4 and SDDMM L16-R16, bit-exact against the CPU oracle."""
import numpy as np
import pytest

from paper_2209_06979_amd import workloads as wl
import input_prep as prep
from gpu_util import run_spmm_gpu, run_spmm_oracle, run_sddmm_gpu, run_sddmm_oracle

pytestmark = pytest.mark.gpu

WIDE = ["L16R16", "L16R4", "L12R4"]


def _spmm(case, variant=(0, 0)):
    print(f"spmm case M={case['M']} K={case['K']} N={case['N']} V={case['V']} {case['prec']} variant={variant}",
          flush=True)
    got, want = run_spmm_gpu(case, variant), run_spmm_oracle(case)
    assert got.dtype == np.int32 and got.shape == want.shape
    bad = np.argwhere(got != want)
    assert bad.size == 0, f"{len(bad)} mismatches, first at {bad[0]}: got {got[tuple(bad[0])]} want {want[tuple(bad[0])]}"


def _sddmm(case, variants=(-1,)):
    want = run_sddmm_oracle(case)
    for waves in variants:
        print(f"sddmm case M={case['M']} Nc={case['Nc']} Kd={case['Kd']} V={case['V']} {case['prec']} waves={waves}",
              flush=True)
        got = run_sddmm_gpu(case, waves)
        assert got.shape == want.shape
        bad = np.flatnonzero(got != want)
        assert bad.size == 0, f"{len(bad)} mismatches, first at {bad[0]}: got {got[bad[0]]} want {want[bad[0]]}"


def _rhs(prec, K, N, seed, lo=-2048, hi=2047):
    if prec == "L16R16":
        return wl.uniform_int16((K, N), seed, lo, hi)
    return wl.uniform_packed_int4((K, N // 2), seed)


# --------------------------------------------------------------------- SpMM ----
@pytest.mark.parametrize("prec", WIDE)
@pytest.mark.parametrize("V", [2, 4, 8])
def test_spmm_small(prec, V):
    _spmm(wl.spmm_case(16 * V, 640, 256, V, 0.75, prec, 2000 + V))


@pytest.mark.parametrize("bnb", [64, 128, 256])
@pytest.mark.parametrize("waves", [1, 2, 4, 8])
@pytest.mark.parametrize("prec", WIDE)
def test_spmm_every_tile_variant(bnb, waves, prec):
    N = 168 if prec == "L16R16" else 384    # 336- / 192-byte rows: ragged last tile for 128- and 256-byte tiles
    _spmm(wl.spmm_case(64, 1024, N, 8, 0.7, prec, 2100 + bnb + waves), (bnb, waves))


@pytest.mark.parametrize("prec", WIDE)
def test_spmm_ragged_and_empty_panels(prec):
    V, K, N = 8, 700, 192
    counts = [0, 1, 15, 16, 17, 63, 64, 65, 127, 128, 129, 0, 300, 700, 2, 0]
    M = V * len(counts)
    rp, ci = wl.ragged_pattern(M, K, V, counts, 2201)
    case = dict(M=M, K=K, N=N, V=V, prec=prec, row_ptr=rp, col_idx=ci,
                values=wl.uniform_int16((len(ci), V), 2202), B=_rhs(prec, K, N, 2203))
    for variant in [(0, 0), (64, 4), (128, 2)]:
        _spmm(case, variant)


@pytest.mark.parametrize("N", [8, 24, 40, 136])
def test_spmm_l16r16_narrow_widths(N):
    _spmm(wl.spmm_case(32, 256, N, 8, 0.5, "L16R16", 2300 + N))
    _spmm(wl.spmm_case(16, 256, N, 4, 0.5, "L16R16", 2350 + N))


def test_spmm_l16r16_full_int16_range():
    """B takes every int16 value (its low byte is used unsigned); A up to the split's limit."""
    V, K, N = 8, 512, 64
    counts = [1] * 8 + [3] * 4 + [16] * 4
    M = V * len(counts)
    rp, ci = wl.ragged_pattern(M, K, V, counts, 2401)
    nvec = len(ci)
    B = wl.uniform_int16((K, N), 2402, -32768, 32767)
    B[ci[0], :4] = [-32768, 32767, -1, 255]
    vals = wl.uniform_int16((nvec, V), 2403, -2048, 2047)
    vals[:8] = wl.uniform_int16((8, V), 2404, -32768, 32639)       # panels with a single vector: no overflow
    vals[0, :4] = [-32768, 32639, -129, 128]
    _spmm(dict(M=M, K=K, N=N, V=V, prec="L16R16", row_ptr=rp, col_idx=ci, values=vals, B=B))


def test_spmm_r4_large_plane_sums():
    """Most negative operands everywhere: each plane sum is shifted before the planes are combined."""
    V, M, K, N = 8, 16, 2048, 64
    rp, ci = wl.vector_sparse_pattern(M, K, V, 0.0, 5)
    vals = np.full((len(ci), V), -2048, np.int16)
    B4 = np.full((K, N // 2), 0x88, np.uint8)
    for prec in ("L16R4", "L12R4"):
        _spmm(dict(M=M, K=K, N=N, V=V, prec=prec, row_ptr=rp, col_idx=ci, values=vals, B=B4))
    vals[:] = 16000                          # C = 16000 * 7 * 2048 = 2.3e8 fits int32, 16 * C would not
    _spmm(dict(M=M, K=K, N=N, V=V, prec="L16R4", row_ptr=rp, col_idx=ci, values=vals, B=np.full_like(B4, 0x77)))


def test_l12_values_are_range_checked():
    from paper_2209_06979_amd import binding as mc
    c = wl.spmm_case(16, 64, 32, 8, 0.5, "L12R4", 2501)
    bad = c["values"].copy()
    bad[0, 0] = -2049
    with pytest.raises(mc.MagicubeError) as e:
        mc.SparseMatrix(c["M"], c["K"], c["V"], c["row_ptr"], c["col_idx"], bad, 12)
    assert e.value.status == mc.MC_ERANGE
    A = mc.SparseMatrix(c["M"], c["K"], c["V"], c["row_ptr"], c["col_idx"], c["values"], 12)
    import torch
    B = torch.from_numpy(c["B"]).cuda()
    with pytest.raises(mc.MagicubeError):      # a 12-bit matrix is not a 16-bit one
        mc.spmm(A, B, "L16R4")
    A.close()


@pytest.mark.parametrize("prec", WIDE)
def test_spmm_full_size_4096(prec):
    _spmm(wl.spmm_case(4096, 4096, 256, 8, 0.9, prec, wl.seed_for(4, 7)))


def test_set_values_device_16bit_then_l16r16():
    import torch
    import oracle
    from paper_2209_06979_amd import binding as mc
    c = wl.spmm_case(64, 512, 64, 8, 0.6, "L16R16", 2601)
    A = mc.SparseMatrix(c["M"], c["K"], c["V"], c["row_ptr"], c["col_idx"], np.zeros_like(c["values"]), 16)
    A.set_values(torch.from_numpy(c["values"]).cuda())
    got = mc.spmm(A, torch.from_numpy(c["B"]).cuda(), "L16R16").cpu().numpy()
    A.close()
    assert np.array_equal(got, oracle.spmm(c["M"], c["K"], c["V"], c["row_ptr"], c["col_idx"], c["values"], c["B"], "L16R16"))


# -------------------------------------------------------------------- SDDMM ----
@pytest.mark.parametrize("V", [2, 4, 8])
@pytest.mark.parametrize("Kd", [32, 64, 128, 256])
def test_sddmm_l16r16_small(V, Kd):
    _sddmm(wl.sddmm_case(16 * V, 300, Kd, V, 0.7, "L16R16", 3000 + V + Kd), variants=(-1, 0, 1, 2, 4, 8))


@pytest.mark.parametrize("Kd", [8, 24, 72, 200, 520])
def test_sddmm_l16r16_odd_reduction_lengths(Kd):
    _sddmm(wl.sddmm_case(64, 200, Kd, 8, 0.5, "L16R16", 3100 + Kd))


def test_sddmm_l16r16_ragged_and_extreme_values():
    V, Nc, Kd = 8, 500, 64
    counts = [0, 1, 15, 16, 17, 63, 64, 65, 0, 129, 500, 3]
    M = V * len(counts)
    rp, ci = wl.ragged_pattern(M, Nc, V, counts, 3201)
    Q = wl.uniform_int16((M, Kd), 3202)
    Km = wl.uniform_int16((Nc, Kd), 3203, -16, 15)
    # one extreme element per row: the products stay below 2**30 + small
    Q[:, 5] = np.where(np.arange(M) % 2 == 0, -32768, 32639)
    Km[:, 5] = np.where(np.arange(Nc) % 3 == 0, 32639, -32768)
    _sddmm(dict(M=M, Nc=Nc, Kd=Kd, V=V, prec="L16R16", row_ptr=rp, col_idx=ci, Q=Q, Kmat=Km), variants=(-1, 0, 2, 8))


@pytest.mark.parametrize("Kd,s", [(64, 0.9), (256, 0.9), (128, 0.7)])
def test_sddmm_l16r16_full_size_4096(Kd, s):
    _sddmm(wl.sddmm_case(4096, 4096, Kd, 8, s, "L16R16", wl.seed_for(3, 500 + Kd)))


# ------------------------------------------------- attention "xb-yb" variants ----
def _attention_variant_check(heads, L, dk, sparsity, seed, p_bits, qkv_bits, token_major=False, mode=0, s_p=None):
    """The layer with p_bits-bit softmax codes and qkv_bits-bit Q/K/V against the oracle, with the
    same tie protocol as the 8b-8b layer: 1e-3, plus one code step for every entry whose
    re-quantisation sits on a rounding boundary within fp32 accuracy."""
    import torch
    import oracle
    from paper_2209_06979_amd import binding as mc
    from test_gpu_sddmm import _tie_ambiguous, _layout
    V = 8
    c = wl.attention_case(heads, L, dk, V, sparsity, seed)
    quant = prep.quantize_inputs_int4 if qkv_bits == 4 else prep.quantize_inputs_int8
    (q, s_q), (k, s_k), (v, s_v) = (quant(c[n]) for n in "qkv")
    s_p = np.float32(1.0 / oracle.P_CODE_MAX[p_bits]) if s_p is None else np.float32(s_p)
    vmax = 7 if qkv_bits == 4 else 127
    print(f"attention {p_bits}b-{qkv_bits}b heads={heads} L={L} dk={dk} s={sparsity} token_major={token_major} mode={mode}",
          flush=True)
    mask = mc.SparseMatrix(L, L, V, c["row_ptr"], c["col_idx"])
    out = _layout(np.full((heads, L, dk), np.nan, np.float32), token_major)
    mc.set_attention_mode(mode)
    try:
        O = mc.sparse_attention(_layout(q, token_major), _layout(k, token_major), _layout(v, token_major), mask,
                                s_q, s_k, s_v, s_p, out=out, p_bits=p_bits, qkv_bits=qkv_bits)
        torch.cuda.synchronize()
    finally:
        mc.set_attention_mode(0)
    O = O.cpu().numpy().astype(np.float64)
    mask.close()
    want, scores, probs, codes = oracle.attention(q, k, v, c["row_ptr"], c["col_idx"], V, s_q, s_k, s_v, s_p,
                                                  p_bits=p_bits, qkv_bits=qkv_bits)
    amb = _tie_ambiguous(probs, s_p).reshape(heads, -1, V)
    rp = c["row_ptr"]
    n_amb_rows = np.zeros((heads, L), np.int64)
    for p in range(L // V):
        n_amb_rows[:, p * V:(p + 1) * V] = amb[:, rp[p]:rp[p + 1], :].sum(axis=1)
    tol = 1e-3 + n_amb_rows[:, :, None] * float(s_p) * float(s_v) * vmax
    err = np.abs(O - want)
    assert (err <= tol).all(), f"max err {err.max()} (ambiguous entries: {int(amb.sum())})"
    clean = n_amb_rows == 0
    if p_bits == 8:
        assert clean.mean() > (0.9 if float(s_p) >= 1 / 127.001 else 0.5)   # finer scales: larger p / s_p, more near-ties
    else:
        # a 16-bit code step is worth s_p * s_v * 127 ~ 1e-7 .. 1e-6 of output: many rows hold an entry
        # near a rounding boundary, but the plain bound must then hold without any allowance
        assert err.max() < 1e-3
    print(f"  max abs err {err.max():.3e}; clean rows {clean.mean():.3f} max err {err[clean].max():.3e}", flush=True)


@pytest.mark.parametrize("p_bits,qkv_bits,dk", [(16, 8, 32), (16, 8, 96), (8, 4, 32), (8, 4, 96), (16, 4, 32), (16, 4, 96), (8, 4, 64)])
@pytest.mark.parametrize("token_major", [False, True])
def test_attention_variants_head_dimensions_below_the_tile(p_bits, qkv_bits, dk, token_major):
    """16-bit codes and 4-bit inputs with rows shorter than the fused kernel's tile (4-bit inputs: head dimensions
    that are multiples of 32)."""
    _attention_variant_check(2, 512, dk, 0.8, 4300 + dk, p_bits, qkv_bits, token_major)
    _attention_variant_check(1, 2048, dk, 0.6, 4310 + dk, p_bits, qkv_bits, token_major)   # 819 vectors: two waves


@pytest.mark.parametrize("p_bits,qkv_bits", [(16, 8), (8, 4), (16, 4)])
@pytest.mark.parametrize("token_major", [False, True])
@pytest.mark.parametrize("mode", [0, 1, 5])                   # automatic / kernel pipeline / two heads per workgroup
def test_attention_variants_small(p_bits, qkv_bits, token_major, mode):
    _attention_variant_check(2, 256, 64, 0.75, 4000, p_bits, qkv_bits, token_major, mode)   # one chunk per panel
    _attention_variant_check(3, 512, 32, 0.9, 4001, p_bits, qkv_bits, token_major, mode)    # dk = 32: pipeline
    _attention_variant_check(2, 1024, 64, 0.6, 4002, p_bits, qkv_bits, token_major, mode)   # 7 chunks, ragged tail
    _attention_variant_check(2, 2048, 64, 0.75, 4004, p_bits, qkv_bits, token_major, mode)  # 512 vectors: longest fused panel
    _attention_variant_check(1, 2048, 128, 0.7, 4003, p_bits, qkv_bits, token_major, mode)  # 614 vectors, dk 128


@pytest.mark.parametrize("token_major", [False, True])
@pytest.mark.parametrize("mode", [0, 3, 4])
def test_attention_16bit_codes_head_dimension_128(token_major, mode):
    """Two planes of codes with rows of 128 bytes (the fused kernel's largest LDS footprint)."""
    _attention_variant_check(2, 256, 128, 0.75, 4010, 16, 8, token_major, mode)
    _attention_variant_check(2, 1024, 128, 0.6, 4011, 16, 8, token_major, mode)
    _attention_variant_check(1, 2048, 128, 0.4, 4012, 16, 8, token_major, mode)   # 20 chunks: four waves in every mode


@pytest.mark.parametrize("p_bits", [8, 16])
@pytest.mark.parametrize("token_major", [False, True])
@pytest.mark.parametrize("mode", [0, 2, 3, 4])
def test_attention_4bit_inputs_head_dimension_128(p_bits, token_major, mode):
    """Rows of 64 bytes of nibbles: two MFMA steps per score tile, eight column tiles of output."""
    _attention_variant_check(2, 256, 128, 0.75, 4020, p_bits, 4, token_major, mode)
    _attention_variant_check(4, 1024, 128, 0.6, 4021, p_bits, 4, token_major, mode)   # 7 chunks, ragged tail
    _attention_variant_check(1, 2048, 128, 0.4, 4022, p_bits, 4, token_major, mode)   # 20 chunks: four waves in every mode


@pytest.mark.parametrize("mode", [0, 3, 4])   # 3, 4: two heads per workgroup whatever the size of the launch
@pytest.mark.parametrize("p_bits,qkv_bits,dk", [(8, 8, 64), (16, 8, 64), (8, 4, 64), (8, 4, 128)])
def test_attention_two_heads_per_workgroup_sharing_long_panels(p_bits, qkv_bits, dk, mode):
    """Token-major tensors with panels of more than 512 vectors: pairs of waves (one wave per head) share the
    chunks of a panel and every wave goes through the chunk loops as often as the busiest pair."""
    for heads, L, sp, seed in ((2, 2048, 0.6, 4500),    # 13 chunks: pairs with 7 and 6
                               (2, 1024, 0.45, 4503),   # 9 chunks: 5 and 4
                               (4, 2048, 0.4, 4501),    # 20 chunks: four pairs with 5 each
                               (2, 2048, 0.17, 4504),   # 27 chunks: 7, 7, 7, 6
                               (2, 2048, 0.0, 4502)):   # 32 chunks: the longest fused panel
        _attention_variant_check(heads, L, dk, sp, seed, p_bits, qkv_bits, True, mode)


@pytest.mark.parametrize("p_bits,qkv_bits", [(16, 8), (8, 4)])
@pytest.mark.parametrize("mode", [0, 1, 6])
def test_attention_variants_config5_shape(p_bits, qkv_bits, mode):
    """The 16b-8b and 8b-4b variants at 8 heads, L=4096, dk=64, 90 % vector sparsity."""
    _attention_variant_check(8, 4096, 64, 0.9, wl.seed_for(5, 1), p_bits, qkv_bits, mode=mode)


@pytest.mark.parametrize("p_bits,qkv_bits", [(8, 8), (16, 8), (8, 4)])
@pytest.mark.parametrize("token_major", [False, True])
@pytest.mark.parametrize("mode", [0, 1, 3, 5])
def test_attention_codes_saturate_at_the_largest_code(p_bits, qkv_bits, token_major, mode):
    """A softmax scale finer than 1 / (largest code): every probability above code_max * s_p must
    become the largest code (127 or 32639), not wrap or run on to 255 / 65535."""
    s_p = 1.0 / (4 * {8: 127, 16: 32639}[p_bits])
    _attention_variant_check(2, 256, 64, 0.9, 4400, p_bits, qkv_bits, token_major, mode, s_p=s_p)   # few entries per row: large p
    _attention_variant_check(2, 1024, 64, 0.6, 4401, p_bits, qkv_bits, token_major, mode, s_p=s_p)


@pytest.mark.parametrize("p_bits,qkv_bits", [(16, 8), (8, 4), (16, 4)])
def test_attention_variants_long_panels_and_forced_wave_counts(p_bits, qkv_bits):
    _attention_variant_check(2, 2048, 64, 0.6, 4300, p_bits, qkv_bits)            # 13 chunks: two waves per (panel, head)
    _attention_variant_check(1, 2048, 64, 0.3, 4301, p_bits, qkv_bits)            # 23 chunks: four waves
    _attention_variant_check(2, 1024, 64, 0.6, 4302, p_bits, qkv_bits, mode=3)    # 7 chunks on two waves
    _attention_variant_check(2, 256, 64, 0.75, 4303, p_bits, qkv_bits, True, 4)   # one chunk on four waves


def test_attention_16b8b_ragged_rows():
    """16-bit codes in the fused kernel with panels of very different lengths (empty ones give zeros)."""
    import torch
    import oracle
    from paper_2209_06979_amd import binding as mc
    V, L, dk, heads = 8, 512, 64, 2
    counts = np.r_[[0, 1, 2, 15, 16, 17, 63, 64, 65, 127, 128, 129, 300, 511, 512, 0], np.full(L // V - 16, 40)]
    rp, ci = wl.ragged_pattern(L, L, V, counts, 4200)
    (q, s_q), (k, s_k), (v, s_v) = (prep.quantize_inputs_int8(wl.normal_fp32((heads, L, dk), 4201 + i)) for i in range(3))
    s_p = np.float32(1 / 32639)
    want = oracle.attention(q, k, v, rp, ci, V, s_q, s_k, s_v, s_p, p_bits=16)[0]
    mask = mc.SparseMatrix(L, L, V, rp, ci)
    O = mc.sparse_attention(torch.from_numpy(q).cuda(), torch.from_numpy(k).cuda(), torch.from_numpy(v).cuda(), mask,
                            s_q, s_k, s_v, s_p, p_bits=16)
    torch.cuda.synchronize()
    O = O.cpu().numpy().astype(np.float64)
    mask.close()
    assert np.abs(O - want).max() < 1e-3
    assert not O[:, :8].any() and not O[:, 15 * 8:16 * 8].any()


def test_sparse_softmax_16_bit_codes():
    import torch
    import oracle
    from paper_2209_06979_amd import binding as mc
    from test_gpu_sddmm import _tie_ambiguous
    V, L = 8, 512
    rp, ci = wl.ragged_pattern(L, L, V, np.r_[[1, 2, 0, 64, 300], np.full(L // V - 5, 51)], 4101)
    nnz = len(ci) * V
    S = np.random.default_rng(4102).integers(-60000, 60000, size=(3, nnz)).astype(np.int32)
    scale = np.float32(2.5e-4)
    mask = mc.SparseMatrix(L, L, V, rp, ci)
    codes = mc.sparse_softmax(mask, torch.from_numpy(S).cuda(), float(scale), 32639.0, code_bits=16)
    torch.cuda.synchronize()
    codes = codes.cpu().numpy()
    assert codes.dtype == np.int16 and codes.max() == 32639     # the single-entry rows: p = 1
    for b in range(3):
        p = oracle.sparse_softmax(S[b], rp, V, scale)
        want = oracle.requantize_probabilities(p, 1 / 32639, 16)
        amb = _tie_ambiguous(p, 1 / 32639)
        diff = codes[b].astype(np.int32) - want.astype(np.int32)
        assert (diff[~amb] == 0).all(), f"{np.count_nonzero(diff[~amb])} code mismatches away from ties"
        assert (np.abs(diff[amb]) <= 1).all()
        assert amb.mean() < 0.05
    mask.close()


@pytest.mark.parametrize("mode", [0, 3])   # 3: two heads per workgroup on token-major tensors whatever the size of the launch
@pytest.mark.parametrize("L,dk,sparsity", [(1536, 64, 0.5), (2048, 64, 0.3), (1536, 128, 0.5)])
def test_attention_batched_long_panels_equal_item_by_item(L, dk, sparsity, mode):
    """Batches whose panels need two or four waves per (panel, head), in both tensor orders."""
    import torch
    from paper_2209_06979_amd import binding as mc
    B, heads, V = 2, 2, 8
    c = wl.attention_case(B * heads, L, dk, V, sparsity, 4450 + dk)
    (q, s_q), (k, s_k), (v, s_v) = (prep.quantize_inputs_int8(c[n]) for n in "qkv")
    s_p = np.float32(1.0 / 127.0)
    mask = mc.SparseMatrix(L, L, V, c["row_ptr"], c["col_idx"])
    try:
        for token_major in (False, True):
            def dev(t):
                x = torch.from_numpy(np.ascontiguousarray(t)).cuda().reshape(B, heads, L, -1)
                return x.permute(0, 2, 1, 3).contiguous().permute(0, 2, 1, 3) if token_major else x
            qd, kd, vd = dev(q), dev(k), dev(v)
            print(f"batched attention L={L} dk={dk} s={sparsity} token_major={token_major} mode={mode}", flush=True)
            mc.set_attention_mode(mode)
            O = mc.sparse_attention(qd, kd, vd, mask, s_q, s_k, s_v, s_p)
            torch.cuda.synchronize()
            assert O.shape == (B, heads, L, dk) and bool(torch.isfinite(O).all())
            for b in range(B):
                Ob = mc.sparse_attention(qd[b], kd[b], vd[b], mask, s_q, s_k, s_v, s_p)
                torch.cuda.synchronize()
                if mode == 0:
                    # the automatic choice gives a smaller launch more waves per (panel, head): the softmax
                    # sums may be added in another order, and a code next to a rounding boundary may move
                    d = (O[b] - Ob).abs()
                    assert float((d > 1e-6).float().mean()) < 0.02 and float(d.max()) < 0.05
                else:
                    assert torch.equal(O[b], Ob), b
            # and the single items against the kernel pipeline, up to the order of the fp32 sums
            mc.set_attention_mode(1)
            Op = mc.sparse_attention(qd[0], kd[0], vd[0], mask, s_q, s_k, s_v, s_p)
            torch.cuda.synchronize()
            mc.set_attention_mode(0)
            d = (O[0] - Op).abs()
            assert float((d > 1e-6).float().mean()) < 0.02 and float(d.max()) < 0.05
    finally:
        mc.set_attention_mode(0)
        mask.close()


@pytest.mark.parametrize("mode", [0, 1, 6])
@pytest.mark.parametrize("p_bits,qkv_bits", [(8, 8), (16, 8), (8, 4)])
def test_attention_batched_equals_item_by_item(p_bits, qkv_bits, mode):
    """A batch sharing one mask, in the (batch, L, heads, dk) layout of a projection's output and in the
    contiguous (batch, heads, L, dk) one: every item must equal the single-item call bit for bit (the
    panels here have two chunks, which leaves the automatic choice nothing to vary with the launch size)."""
    import torch
    from paper_2209_06979_amd import binding as mc
    B, heads, L, dk, V = 3, 4, 512, 64, 8
    c = wl.attention_case(B * heads, L, dk, V, 0.8, 4400)
    quant = prep.quantize_inputs_int4 if qkv_bits == 4 else prep.quantize_inputs_int8
    (q, s_q), (k, s_k), (v, s_v) = (quant(c[n]) for n in "qkv")
    s_p = np.float32(1.0 / (32639.0 if p_bits == 16 else 127.0))
    mask = mc.SparseMatrix(L, L, V, c["row_ptr"], c["col_idx"])
    mc.set_attention_mode(mode)
    try:
        for token_major in (False, True):
            def dev(t):
                x = torch.from_numpy(np.ascontiguousarray(t)).cuda().reshape(B, heads, L, -1)
                return x.permute(0, 2, 1, 3).contiguous().permute(0, 2, 1, 3) if token_major else x
            qd, kd, vd = dev(q), dev(k), dev(v)
            print(f"batched attention {p_bits}b-{qkv_bits}b mode={mode} token_major={token_major}", flush=True)
            O = mc.sparse_attention(qd, kd, vd, mask, s_q, s_k, s_v, s_p, p_bits=p_bits, qkv_bits=qkv_bits)
            torch.cuda.synchronize()
            assert O.shape == (B, heads, L, dk) and bool(torch.isfinite(O).all())
            for b in range(B):
                Ob = mc.sparse_attention(qd[b], kd[b], vd[b], mask, s_q, s_k, s_v, s_p, p_bits=p_bits, qkv_bits=qkv_bits)
                torch.cuda.synchronize()
                assert torch.equal(O[b], Ob), b
    finally:
        mc.set_attention_mode(0)
        mask.close()
