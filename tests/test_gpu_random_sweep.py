"""Seeded random sweep over valid problems, against the CPU oracle: shapes, sparsities, precisions,
operand signedness, tile variants, chunks in flight, attention modes / layouts / widths / output
types drawn at random (the combinations no hand-written case names).  Integer results must be
bit-exact; the attention output obeys the layer's tolerance with the tie protocol of the other
attention tests."""
import numpy as np
import pytest

from paper_2209_06979_amd import workloads as wl
import input_prep as prep
from gpu_util import run_spmm_gpu, run_spmm_oracle, run_sddmm_gpu, run_sddmm_oracle

pytestmark = pytest.mark.gpu

SPMM_PRECS = ["L8R8", "L8R4", "L4R4", "L16R8", "L16R16", "L16R4", "L12R4"]
SPARSITIES = [0.0, 0.3, 0.5, 0.8, 0.95, 0.99]


@pytest.mark.parametrize("seed", [1, 2, 3])
def test_random_spmm(seed):
    from paper_2209_06979_amd import binding as mc
    rng = np.random.default_rng(9000 + seed)
    for n in range(120):
        V = int(rng.choice([2, 4, 8]))
        prec = str(rng.choice(SPMM_PRECS))
        big = rng.random() < 0.1
        M = V * int(rng.integers(1, 400 if big else 80))
        K = 16 * int(rng.integers(1, 200 if big else 40))
        N = {8: 16, 4: 32, 16: 8}[mc.RHS_BITS[prec]] * int(rng.integers(1, 24))
        s = float(rng.choice(SPARSITIES))
        case = wl.spmm_case(M, K, N, V, max(s, 0.5) if big else s, prec, int(rng.integers(1 << 30)))
        if prec in ("L8R8", "L8R4", "L4R4") and rng.random() < 0.3:
            case["lhs_unsigned"], case["rhs_unsigned"] = bool(rng.integers(2)), bool(rng.integers(2))
        splitting = True
        if rng.random() < 0.3:      # panels of very unequal length, with and without work items
            cnt = np.clip(np.rint(rng.lognormal(0, float(rng.choice([0.5, 1.0, 2.0])), M // V) * max(1, (1 - s) * K)), 0, K)
            rp, ci = wl.ragged_pattern(M, K, V, cnt.astype(np.int64), int(rng.integers(1 << 30)))
            vb = case["values"]
            vals = rng.integers(-7, 8, size=(len(ci), vb.shape[1])).astype(vb.dtype)
            case.update(row_ptr=rp, col_idx=ci, values=vals)
            splitting = bool(rng.integers(2))
        variant = (int(rng.choice([0, 64, 128, 256])), int(rng.choice([0, 1, 2, 4, 8])))
        stages = int(rng.choice([1, 2]))
        merge = int(rng.choice([0, 1, 1, -1]))
        print(f"#{n} spmm {prec} M={M} K={K} N={N} V={V} s={s} variant={variant} stages={stages} merge={merge} "
              f"unsigned={case.get('lhs_unsigned', False)},{case.get('rhs_unsigned', False)}", flush=True)
        mc.set_spmm_stages(stages)
        mc.set_spmm_splitting(splitting)
        try:
            got = run_spmm_gpu(case, variant, merge)
        finally:
            mc.set_spmm_stages(2)
            mc.set_spmm_splitting(True)
        assert np.array_equal(got, run_spmm_oracle(case))


@pytest.mark.parametrize("seed", [1, 2, 3])
def test_random_sddmm(seed):
    from paper_2209_06979_amd import binding as mc
    rng = np.random.default_rng(9100 + seed)
    for n in range(120):
        V = int(rng.choice([2, 4, 8]))
        prec = str(rng.choice(["L8R8", "L4R4", "L16R16"]))
        big = rng.random() < 0.1
        M = V * int(rng.integers(1, 400 if big else 80))
        Nc = 8 * int(rng.integers(1, 400 if big else 60))
        Kd = (128 // mc.LHS_BITS[prec]) * int(rng.integers(1, 20))
        s = float(rng.choice(SPARSITIES))
        case = wl.sddmm_case(M, Nc, Kd, V, max(s, 0.5) if big else s, prec, int(rng.integers(1 << 30)))
        if prec != "L16R16" and rng.random() < 0.3:
            case["lhs_unsigned"], case["rhs_unsigned"] = bool(rng.integers(2)), bool(rng.integers(2))
        splitting = True
        if rng.random() < 0.3:
            cnt = np.clip(np.rint(rng.lognormal(0, float(rng.choice([0.5, 1.0, 2.0])), M // V) * max(1, (1 - s) * Nc)), 0, Nc)
            rp, ci = wl.ragged_pattern(M, Nc, V, cnt.astype(np.int64), int(rng.integers(1 << 30)))
            case.update(row_ptr=rp, col_idx=ci)
            splitting = bool(rng.integers(2))
        waves = int(rng.choice([-1, 0, 1, 2, 4, 8]))
        print(f"#{n} sddmm {prec} M={M} Nc={Nc} Kd={Kd} V={V} s={s} waves={waves} "
              f"unsigned={case.get('lhs_unsigned', False)},{case.get('rhs_unsigned', False)}", flush=True)
        mc.set_spmm_splitting(splitting)
        try:
            got = run_sddmm_gpu(case, waves)
        finally:
            mc.set_spmm_splitting(True)
        assert np.array_equal(got, run_sddmm_oracle(case))


@pytest.mark.parametrize("seed", [1, 2])
def test_random_attention(seed):
    import torch
    import oracle
    from paper_2209_06979_amd import binding as mc
    from test_gpu_sddmm import _tie_ambiguous, _layout
    rng = np.random.default_rng(9200 + seed)
    for n in range(40):
        heads = int(rng.integers(1, 5))
        L = 8 * int(rng.integers(12, 120))
        dk = int(rng.choice([32, 64, 64, 64, 128]))
        s = float(rng.choice([0.3, 0.6, 0.9]))
        p_bits, qkv_bits = int(rng.choice([8, 16])), int(rng.choice([8, 4]))
        mode, tmaj, f16 = int(rng.choice([0, 1, 2, 3, 4, 5])), bool(rng.integers(2)), bool(rng.integers(2))
        c = wl.attention_case(heads, L, dk, 8, s, int(rng.integers(1 << 30)))
        quant = prep.quantize_inputs_int4 if qkv_bits == 4 else prep.quantize_inputs_int8
        (q, s_q), (k, s_k), (v, s_v) = (quant(c[nm]) for nm in "qkv")
        s_p = np.float32(1.0 / oracle.P_CODE_MAX[p_bits] / float(rng.choice([1, 1, 3])))
        print(f"#{n} attention heads={heads} L={L} dk={dk} s={s} {p_bits}b-{qkv_bits}b mode={mode} token_major={tmaj} "
              f"fp16={f16} s_p={s_p}", flush=True)
        mask = mc.SparseMatrix(L, L, 8, c["row_ptr"], c["col_idx"])
        mc.set_attention_mode(mode)
        try:
            O = mc.sparse_attention(_layout(q, tmaj), _layout(k, tmaj), _layout(v, tmaj), mask, s_q, s_k, s_v, s_p,
                                    p_bits=p_bits, qkv_bits=qkv_bits, out_dtype=torch.float16 if f16 else torch.float32)
            torch.cuda.synchronize()
        finally:
            mc.set_attention_mode(0)
            mask.close()
        want, _, probs, _ = oracle.attention(q, k, v, c["row_ptr"], c["col_idx"], 8, s_q, s_k, s_v, s_p,
                                             p_bits=p_bits, qkv_bits=qkv_bits)
        err = np.abs(O.float().cpu().numpy().astype(np.float64) - want)
        amb = _tie_ambiguous(probs, s_p).reshape(heads, -1, 8)
        rp = c["row_ptr"]
        namb = np.zeros((heads, L), np.int64)
        for p in range(L // 8):
            namb[:, p * 8:(p + 1) * 8] = amb[:, rp[p]:rp[p + 1], :].sum(axis=1)
        vmax = 7 if qkv_bits == 4 else 127
        # 1e-3, one code step per entry within fp32 accuracy of a rounding boundary, one fp16 step for fp16 outputs
        tol = 1e-3 + namb[:, :, None] * float(s_p) * float(s_v) * vmax + (np.abs(want) * 2.0 ** -10 if f16 else 0)
        assert (err <= tol).all(), f"max err {err.max()}"
