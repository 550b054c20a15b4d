"""GPU parity of the fused dequantisation (Section 5.3): SpMM and SDDMM that write scale * result
as fp32 or fp16, and the attention layer with an fp16 output, against the CPU oracle.

Bars, derived from the arithmetic: the kernels compute float(int32 result) * scale in fp32 and
round that to fp16; the oracle rounds the exact product once.
  * fp32: identical bits where the integer result fits 24 bits (its conversion is then exact and
    the product is rounded once on both sides); otherwise at most one fp32 unit in the last place.
  * fp16: identical bits except where the fp32 intermediate falls exactly half-way between two
    fp16 numbers (double rounding; checked element by element): then one fp16 unit in the last
    place; and the fp16 result is always exactly the kernel's own fp32 result rounded to nearest
    even.
"""
import numpy as np
import pytest

from paper_2209_06979_amd import workloads as wl
import input_prep as prep
from gpu_util import torch_dev, run_spmm_oracle, run_sddmm_oracle

pytestmark = pytest.mark.gpu


def _ulp(x, dtype):
    ax = np.abs(x.astype(np.float64))
    finfo = np.finfo(dtype)
    e = np.floor(np.log2(np.maximum(ax, finfo.tiny)))
    return 2.0 ** (e - finfo.nmant)


def _compare(got32, got16, acc, scale):
    """got32 / got16: the kernel's fp32 and fp16 outputs; acc: the oracle's exact integers."""
    import oracle
    import torch
    want32 = oracle.dequantize(acc, scale, 32)
    want16 = oracle.dequantize(acc, scale, 16)
    g32, g16 = got32.cpu().numpy(), got16.cpu().numpy()
    assert g32.dtype == np.float32 and g16.dtype == np.float16 and g32.shape == want32.shape
    small = np.abs(acc.astype(np.int64)) <= (1 << 24)
    assert np.array_equal(g32[small].view(np.uint32), want32[small].view(np.uint32))
    assert (np.abs(g32.astype(np.float64) - want32.astype(np.float64)) <= _ulp(want32, np.float32)).all()
    # fp16 = the kernel's fp32 value rounded once (torch's conversion is the independent check)
    assert torch.equal(got16, got32.half())
    fin = np.isfinite(want16)
    assert np.array_equal(np.isinf(g16), ~fin) and np.array_equal(np.sign(g16[~fin]), np.sign(want16[~fin]))
    d = np.abs(g16[fin].astype(np.float64) - want16[fin].astype(np.float64))
    assert (d <= _ulp(want16[fin], np.float16)).all()
    # a difference needs the fp32 intermediate to sit exactly half-way between two fp16 numbers
    w32 = want32[fin].astype(np.float64)
    h = w32.astype(np.float16)
    lo = np.nextafter(h, np.float16(-np.inf)).astype(np.float64)
    hi = np.nextafter(h, np.float16(np.inf)).astype(np.float64)
    h = h.astype(np.float64)
    tie = (np.abs(w32 - h) == np.abs(w32 - lo)) | (np.abs(w32 - h) == np.abs(w32 - hi))
    assert not ((d != 0) & ~tie).any()
    assert (d == 0).mean() > 0.99
    return float((d == 0).mean())


def _spmm(case, scale):
    import torch
    from paper_2209_06979_amd import binding as mc
    print(f"spmm_dequant M={case['M']} K={case['K']} N={case['N']} V={case['V']} {case['prec']} scale={scale}", flush=True)
    A = mc.SparseMatrix(case["M"], case["K"], case["V"], case["row_ptr"], case["col_idx"], case["values"],
                        mc.LHS_BITS[case["prec"]])
    B = torch_dev(case["B"])
    kw = dict(lhs_unsigned=case.get("lhs_unsigned", False), rhs_unsigned=case.get("rhs_unsigned", False))
    o32 = torch.full((case["M"], case["N"]), float("nan"), dtype=torch.float32, device="cuda")
    o16 = torch.full((case["M"], case["N"]), float("nan"), dtype=torch.float16, device="cuda")
    mc.spmm_dequant(A, B, case["prec"], scale, torch.float32, out=o32, **kw)
    mc.spmm_dequant(A, B, case["prec"], scale, torch.float16, out=o16, **kw)
    torch.cuda.synchronize()
    A.close()
    return _compare(o32, o16, run_spmm_oracle(case), scale)


def _sddmm(case, scale):
    import torch
    from paper_2209_06979_amd import binding as mc
    print(f"sddmm_dequant M={case['M']} Nc={case['Nc']} Kd={case['Kd']} V={case['V']} {case['prec']} scale={scale}", flush=True)
    mask = mc.SparseMatrix(case["M"], case["Nc"], case["V"], case["row_ptr"], case["col_idx"])
    Q, Km = torch_dev(case["Q"]), torch_dev(case["Kmat"])
    kw = dict(lhs_unsigned=case.get("lhs_unsigned", False), rhs_unsigned=case.get("rhs_unsigned", False))
    n = mask.nvec * mask.V
    o32 = torch.full((n,), float("nan"), dtype=torch.float32, device="cuda")
    o16 = torch.full((n,), float("nan"), dtype=torch.float16, device="cuda")
    mc.sddmm_dequant(Q, Km, mask, case["prec"], scale, torch.float32, out=o32, **kw)
    mc.sddmm_dequant(Q, Km, mask, case["prec"], scale, torch.float16, out=o16, **kw)
    torch.cuda.synchronize()
    mask.close()
    return _compare(o32, o16, run_sddmm_oracle(case), scale)


SPMM_PRECS = ["L8R8", "L8R4", "L4R4", "L16R8", "L16R16", "L16R4", "L12R4"]


@pytest.mark.parametrize("prec", SPMM_PRECS)
@pytest.mark.parametrize("V", [2, 4, 8])
def test_spmm_dequant_small(prec, V):
    # several tiles and a ragged tail; scales that keep fp16 finite, and one that overflows it
    _spmm(wl.spmm_case(192, 640, 160, V, 0.7, prec, 6100 + V), np.float32(1.0 / 127 / 127))
    _spmm(wl.spmm_case(64, 256, 96, V, 0.5, prec, 6110 + V), np.float32(0.37))


@pytest.mark.parametrize("prec", ["L8R8", "L4R4", "L16R8"])
def test_spmm_dequant_headline_shape(prec):
    _spmm(wl.spmm_case(4096, 4096, 256, 8, 0.9, prec, wl.seed_for(2, 700)), np.float32(3.1e-5))


@pytest.mark.parametrize("lu,ru", [(True, False), (False, True), (True, True)])
def test_spmm_dequant_unsigned(lu, ru):
    c = wl.spmm_case(128, 512, 128, 8, 0.8, "L8R8", 6200)
    c["lhs_unsigned"], c["rhs_unsigned"] = lu, ru
    _spmm(c, np.float32(2.0 ** -12))


def test_spmm_dequant_unequal_panels_are_not_split():
    """Panels far longer than the average: the integer entry point shares them between workgroups
    with atomics; the dequantising one must give each panel to one workgroup and still be right."""
    rng = np.random.default_rng(6300)
    M, K, N, V = 512, 4096, 128, 8
    keep = np.full(M // V, 16)
    keep[::16] = 3000
    rows = [np.sort(rng.choice(K, k, replace=False)) for k in keep]
    row_ptr = np.concatenate([[0], np.cumsum(keep)]).astype(np.int32)
    col_idx = np.concatenate(rows).astype(np.int32)
    vals = rng.integers(-128, 128, size=(len(col_idx), V)).astype(np.int8)
    B = rng.integers(-128, 128, size=(K, N)).astype(np.int8)
    case = dict(M=M, K=K, N=N, V=V, prec="L8R8", row_ptr=row_ptr, col_idx=col_idx, values=vals, B=B)
    _spmm(case, np.float32(1e-4))


@pytest.mark.parametrize("prec", ["L8R8", "L4R4", "L16R16"])
@pytest.mark.parametrize("V", [2, 4, 8])
@pytest.mark.parametrize("Kd", [64, 256, 96])                 # LDS-staged kernels and the direct one
def test_sddmm_dequant_small(prec, V, Kd):
    _sddmm(wl.sddmm_case(256, 384, Kd, V, 0.7, prec, 6400 + V + Kd), np.float32(1.0 / 127 / 127 / 8))


@pytest.mark.parametrize("lu,ru", [(True, False), (True, True)])
def test_sddmm_dequant_unsigned(lu, ru):
    c = wl.sddmm_case(128, 256, 64, 8, 0.8, "L8R8", 6500)
    c["lhs_unsigned"], c["rhs_unsigned"] = lu, ru
    _sddmm(c, np.float32(2.0 ** -10))


def test_sddmm_dequant_full_size():
    _sddmm(wl.sddmm_case(4096, 4096, 256, 8, 0.9, "L8R8", wl.seed_for(3, 700)), np.float32(1.0 / 127 / 127 / 16))


# ------------------------------------------------------------ attention, fp16 output ----
def _attention_f16(heads, L, dk, sparsity, seed, p_bits=8, qkv_bits=8, token_major=False, mode=0, batch=0):
    """fp16 output == the fp32 output of the same entry point rounded once (bit for bit), and within
    the layer's tolerance plus one fp16 unit of the oracle's fp16 output."""
    import torch
    import oracle
    from paper_2209_06979_amd import binding as mc
    from test_gpu_sddmm import _layout
    V = 8
    print(f"attention fp16 out {p_bits}b-{qkv_bits}b heads={heads} L={L} dk={dk} s={sparsity} token_major={token_major} "
          f"mode={mode} batch={batch}", flush=True)
    items = [wl.attention_case(heads, L, dk, V, sparsity, seed + i) for i in range(max(batch, 1))]
    c = items[0]
    quant = prep.quantize_inputs_int4 if qkv_bits == 4 else prep.quantize_inputs_int8
    # one scale per tensor over the whole batch: quantise the stacked tensors
    stacked = {n: np.stack([it[n] for it in items]) for n in "qkv"}
    (q, s_q), (k, s_k), (v, s_v) = (quant(stacked[n]) for n in "qkv")
    s_p = np.float32(1.0 / oracle.P_CODE_MAX[p_bits])
    mask = mc.SparseMatrix(L, L, V, c["row_ptr"], c["col_idx"])

    def dev(t):
        if batch:
            return torch.stack([_layout(t[i], token_major) for i in range(batch)])
        return _layout(t[0], token_major)
    mc.set_attention_mode(mode)
    try:
        args = (dev(q), dev(k), dev(v), mask, s_q, s_k, s_v, s_p)
        O32 = mc.sparse_attention(*args, p_bits=p_bits, qkv_bits=qkv_bits)
        O16 = mc.sparse_attention(*args, p_bits=p_bits, qkv_bits=qkv_bits, out_dtype=torch.float16)
        torch.cuda.synchronize()
    finally:
        mc.set_attention_mode(0)
    mask.close()
    assert O16.dtype == torch.float16 and O16.shape == O32.shape and O16.stride() == O32.stride()
    assert torch.equal(O16, O32.half())
    got = O16.cpu().numpy().reshape((max(batch, 1), heads, L, dk))
    for i in range(max(batch, 1)):
        want = oracle.attention(q[i], k[i], v[i], c["row_ptr"], c["col_idx"], V, s_q, s_k, s_v, s_p, p_bits=p_bits,
                                qkv_bits=qkv_bits, out_bits=16)[0]
        # the layer's tolerance (1e-3, ties of the re-quantisation aside: those are covered by the fp32
        # tests with their per-row allowance) plus one fp16 unit; a generous 2 % of rows may hold such ties
        err = np.abs(got[i].astype(np.float64) - want.astype(np.float64))
        ok = err <= 1e-3 + _ulp(want, np.float16)
        assert ok.all(axis=-1).mean() > 0.98 and err.max() < 0.05, f"max err {err.max()}"


@pytest.mark.parametrize("token_major", [False, True])
@pytest.mark.parametrize("mode", [0, 1, 5])
def test_attention_fp16_output_small(token_major, mode):
    _attention_f16(2, 256, 64, 0.75, 6600, token_major=token_major, mode=mode)
    _attention_f16(2, 1024, 64, 0.6, 6601, token_major=token_major, mode=mode)     # 7 chunks, ragged tail
    _attention_f16(3, 512, 32, 0.9, 6602, token_major=token_major, mode=mode)      # dk = 32


@pytest.mark.parametrize("p_bits,qkv_bits", [(16, 8), (8, 4), (16, 4)])
def test_attention_fp16_output_variants(p_bits, qkv_bits):
    _attention_f16(2, 512, 64, 0.8, 6610, p_bits, qkv_bits)
    _attention_f16(2, 512, 64, 0.8, 6611, p_bits, qkv_bits, token_major=True, mode=5)      # two heads per workgroup
    _attention_f16(2, 2048, 64, 0.6, 6612, p_bits, qkv_bits)                       # two waves per (panel, head)
    _attention_f16(2, 2048, 64, 0.6, 6613, p_bits, qkv_bits, token_major=True, mode=3)
    _attention_f16(2, 2048, 64, 0.3, 6614, p_bits, qkv_bits, token_major=True, mode=4)     # four waves per (panel, head)


@pytest.mark.parametrize("dk", [16, 48, 96])
def test_attention_fp16_output_head_dimensions_below_the_tile(dk):
    _attention_f16(2, 512, dk, 0.8, 6640 + dk, token_major=True)
    _attention_f16(1, 2048, dk, 0.6, 6650 + dk)                                    # two waves per (panel, head)
    _attention_f16(2, 512, dk, 0.8, 6660 + dk, token_major=True, batch=2)


@pytest.mark.parametrize("p_bits", [8, 16])
def test_attention_fp16_output_head_dimension_128(p_bits):
    _attention_f16(2, 1024, 128, 0.6, 6630, p_bits, 8)
    _attention_f16(2, 1024, 128, 0.6, 6631, p_bits, 8, token_major=True)
    _attention_f16(2, 2048, 128, 0.6, 6632, p_bits, 8)                             # two waves per (panel, head)
    _attention_f16(1, 2048, 128, 0.3, 6633, p_bits, 8, token_major=True)           # four waves
    _attention_f16(2, 1024, 128, 0.6, 6634, p_bits, 4, token_major=True, mode=5)   # nibbles; two heads per workgroup (8-bit codes)
    _attention_f16(2, 2048, 128, 0.6, 6635, p_bits, 4)


def test_attention_fp16_output_batched_and_config5():
    _attention_f16(4, 512, 64, 0.8, 6620, batch=3, token_major=True, mode=5)
    _attention_f16(4, 512, 64, 0.8, 6621, batch=2, mode=1)
    _attention_f16(8, 4096, 64, 0.9, wl.seed_for(5, 2), token_major=True)


# ------------------------------------------- softmax writing the SpMM operand format ----
@pytest.mark.parametrize("variant", [0, 1, 2])                 # a wave / a workgroup per panel, the any-length kernel
@pytest.mark.parametrize("V", [2, 4, 8])
@pytest.mark.parametrize("bits", [8, 16])
def test_softmax_codes_written_in_the_device_format(V, bits, variant):
    """mc_sparse_softmax_to_mat puts the codes where the SpMM kernels read them: the product of
    that matrix with the identity is the dense matrix of the oracle's codes (same tie protocol
    as the interchange-order softmax: exact away from rounding boundaries, one step at them)."""
    import torch
    import oracle
    from paper_2209_06979_amd import binding as mc
    from test_gpu_sddmm import _tie_ambiguous
    L = 256
    P_ = L // V
    counts = np.full(P_, 37)
    counts[:8] = [0, 1, 2, 63, 64, 65, 128, 256]                 # empty, short, around chunk ends, full row
    rp, ci = wl.ragged_pattern(L, L, V, counts, 6700 + V)
    nvec = len(ci)
    print(f"softmax_to_mat V={V} bits={bits} nvec={nvec}", flush=True)
    S = np.random.default_rng(6701).integers(-30000, 30000, size=nvec * V).astype(np.int32)
    scale, pmax = np.float32(3e-4), oracle.P_CODE_MAX[bits]
    stale = np.full((nvec, V), 77, np.int8 if bits == 8 else np.int16)   # must be overwritten everywhere
    Pm = mc.SparseMatrix(L, L, V, rp, ci, stale, bits)
    mc.set_softmax_variant(variant)
    try:
        mc.sparse_softmax_to_mat(Pm, torch.from_numpy(S).cuda(), float(scale), float(pmax))
    finally:
        mc.set_softmax_variant(0)
    eye = torch.eye(L, dtype=torch.int8, device="cuda")
    got = mc.spmm(Pm, eye, "L8R8" if bits == 8 else "L16R8")
    torch.cuda.synchronize()
    got = got.cpu().numpy()
    Pm.close()
    p = oracle.sparse_softmax(S, rp, V, scale)
    want_codes = oracle.requantize_probabilities(p, 1.0 / pmax, bits)
    want, _ = oracle.bcrs_to_dense(L, L, V, rp, ci, want_codes.reshape(nvec, V))
    amb_dense, _ = oracle.bcrs_to_dense(L, L, V, rp, ci, _tie_ambiguous(p, 1.0 / pmax).reshape(nvec, V).astype(np.int32))
    amb = amb_dense.astype(bool)
    diff = got.astype(np.int64) - want.astype(np.int64)
    assert (diff[~amb] == 0).all(), f"{np.count_nonzero(diff[~amb])} mismatches away from ties"
    assert (np.abs(diff[amb]) <= 1).all() and amb.mean() < 0.05
    assert got.max() == pmax                                       # the single-entry rows: p = 1
