"""GPU parity of SDDMM, sparse softmax and the attention layer against the CPU oracle."""
import numpy as np
import pytest

from paper_2209_06979_amd import workloads as wl
import input_prep as prep
from gpu_util import run_sddmm_gpu, run_sddmm_oracle, torch_dev

pytestmark = pytest.mark.gpu


def _check(case, variants=(-1,)):
    want = run_sddmm_oracle(case)
    for waves in variants:
        print(f"sddmm case M={case['M']} Nc={case['Nc']} Kd={case['Kd']} V={case['V']} {case['prec']} waves={waves}",
              flush=True)
        got = run_sddmm_gpu(case, waves)
        assert got.shape == want.shape
        bad = np.flatnonzero(got != want)
        assert bad.size == 0, f"{len(bad)} mismatches, first at {bad[0]}: got {got[bad[0]]} want {want[bad[0]]}"


@pytest.mark.parametrize("prec", ["L8R8", "L4R4"])
@pytest.mark.parametrize("V", [2, 4, 8])
@pytest.mark.parametrize("Kd", [64, 128, 256])
def test_small(prec, V, Kd):
    _check(wl.sddmm_case(16 * V, 300, Kd, V, 0.7, prec, 1000 + V + Kd), variants=(-1, 0, 1, 2, 4, 8))


@pytest.mark.parametrize("prec,Kd", [("L8R8", 512), ("L4R4", 1024), ("L8R8", 1024), ("L4R4", 2048), ("L16R16", 256),
                                     ("L16R16", 512)])
@pytest.mark.parametrize("V", [2, 8])
def test_rows_of_512_and_1024_bytes(prec, Kd, V):
    """Rows longer than the 256-byte stage go through it in two or four passes."""
    _check(wl.sddmm_case(8 * V, 300, Kd, V, 0.5, prec, 1150 + Kd + V), variants=(-1, 0, 1, 2, 4, 8))


@pytest.mark.parametrize("prec,Kd", [("L8R8", 16), ("L8R8", 48), ("L8R8", 320), ("L8R8", 1024), ("L4R4", 32),
                                     ("L4R4", 96), ("L4R4", 1056)])
def test_odd_reduction_lengths(prec, Kd):
    _check(wl.sddmm_case(64, 200, Kd, 8, 0.5, prec, 1100 + Kd))


@pytest.mark.parametrize("prec", ["L8R8", "L4R4"])
def test_ragged_and_empty_panels(prec):
    V, Nc, Kd = 8, 500, 128
    counts = [0, 1, 15, 16, 17, 63, 64, 65, 0, 129, 500, 3]
    M = V * len(counts)
    rp, ci = wl.ragged_pattern(M, Nc, V, counts, 81)
    if prec == "L4R4":
        Q, Km = wl.uniform_packed_int4((M, Kd // 2), 82), wl.uniform_packed_int4((Nc, Kd // 2), 83)
    else:
        Q, Km = wl.uniform_int8((M, Kd), 82), wl.uniform_int8((Nc, Kd), 83)
    _check(dict(M=M, Nc=Nc, Kd=Kd, V=V, prec=prec, row_ptr=rp, col_idx=ci, Q=Q, Kmat=Km), variants=(-1, 0, 2, 8))


@pytest.mark.parametrize("prec,Kd,s", [("L8R8", 64, 0.9), ("L8R8", 256, 0.7), ("L4R4", 128, 0.95), ("L4R4", 64, 0.9)])
def test_full_size_4096(prec, Kd, s):
    """BASELINE config 3 at full size, whole output compared."""
    _check(wl.sddmm_case(4096, 4096, Kd, 8, s, prec, wl.seed_for(3, Kd + int(100 * s))))


def test_unsupported_precisions():
    import torch
    from paper_2209_06979_amd import binding as mc
    c = wl.sddmm_case(16, 64, 64, 8, 0.5, "L8R8", 5)
    mask = mc.SparseMatrix(c["M"], c["Nc"], c["V"], c["row_ptr"], c["col_idx"])
    for prec in ("L8R4", "L16R8"):
        with pytest.raises(mc.MagicubeError) as e:
            mc.sddmm(torch_dev(c["Q"]), torch_dev(c["Kmat"]), mask, prec)
        assert e.value.status == mc.MC_EUNSUPPORTED
    mask.close()


# ------------------------------------------------------------------ softmax ----
def _tie_ambiguous(probs, s_p):
    """Entries whose code may legitimately differ by one step between fp32 and fp64.

    x = p / s_p lies within the fp32 error of a rounding boundary.  The fp32 path makes a
    relative error of a few 1e-6 on p (two roundings of |x| <= ~30 in the exponent, expf,
    the sum and the division), i.e. up to ~1e-5 * x absolute on x, plus 1e-4 of slack.
    """
    x = probs / np.float64(s_p)
    return np.abs((x - np.floor(x)) - 0.5) < 1e-4 + 1e-5 * x


def test_sparse_softmax_codes():
    import torch
    import oracle
    from paper_2209_06979_amd import binding as mc
    V, L = 8, 512
    rp, ci = wl.ragged_pattern(L, L, V, np.r_[[1, 2, 0, 64, 300], np.full(L // V - 5, 51)], 91)
    nnz = len(ci) * V
    rng = np.random.default_rng(92)
    S = rng.integers(-60000, 60000, size=(3, nnz)).astype(np.int32)
    scale = np.float32(2.5e-4)
    mask = mc.SparseMatrix(L, L, V, rp, ci)
    codes = mc.sparse_softmax(mask, torch_dev(S), float(scale), 127.0)
    torch.cuda.synchronize()
    codes = codes.cpu().numpy()
    for b in range(3):
        p = oracle.sparse_softmax(S[b], rp, V, scale)
        want = oracle.requantize_probabilities(p, 1 / 127)
        amb = _tie_ambiguous(p, 1 / 127)
        diff = codes[b].astype(np.int32) - want.astype(np.int32)
        assert (diff[~amb] == 0).all(), f"{np.count_nonzero(diff[~amb])} code mismatches away from ties"
        assert (np.abs(diff[amb]) <= 1).all()
    mask.close()


# ---------------------------------------------------------------- attention ----
def _layout(t, token_major):
    """(heads, L, dk) device tensor; token_major: a view of a contiguous (L, heads, dk) buffer."""
    import torch
    x = torch.from_numpy(np.ascontiguousarray(t)).cuda()
    return x.permute(1, 0, 2).contiguous().permute(1, 0, 2) if token_major else x


def _attention_check(heads, L, dk, sparsity, seed, mode=0, token_major=False, counts=None):
    """counts: vectors per panel of a mask with panels of unequal length (sparsity is then ignored)."""
    import torch
    import oracle
    from paper_2209_06979_amd import binding as mc
    V = 8
    if counts is None:
        c = wl.attention_case(heads, L, dk, V, sparsity, seed)
    else:
        rp, ci = wl.ragged_pattern(L, L, V, counts, seed)
        c = dict(row_ptr=rp, col_idx=ci, **{n: wl.normal_fp32((heads, L, dk), seed + 1 + i) for i, n in enumerate("qkv")})
    q8, s_q = prep.quantize_inputs_int8(c["q"]); k8, s_k = prep.quantize_inputs_int8(c["k"])
    v8, s_v = prep.quantize_inputs_int8(c["v"])
    s_p = np.float32(1.0 / 127.0)
    print(f"attention heads={heads} L={L} dk={dk} s={sparsity} mode={mode} token_major={token_major}", flush=True)
    mask = mc.SparseMatrix(L, L, V, c["row_ptr"], c["col_idx"])
    mc.set_attention_mode(mode)
    try:
        out = _layout(np.full((heads, L, dk), np.nan, np.float32), token_major)
        O = mc.sparse_attention(_layout(q8, token_major), _layout(k8, token_major), _layout(v8, token_major), mask,
                                s_q, s_k, s_v, s_p, out=out)
        torch.cuda.synchronize()
    finally:
        mc.set_attention_mode(0)
    O = O.cpu().numpy().astype(np.float64)
    mask.close()
    want, scores, probs, codes = oracle.attention(q8, k8, v8, c["row_ptr"], c["col_idx"], V, s_q, s_k, s_v, s_p)
    # rows that contain a rounding tie of the re-quantisation may differ by one code step
    # per tied entry: allow s_p * s_v * 127 for each of them, 1e-3 everywhere else
    amb = _tie_ambiguous(probs, s_p).reshape(heads, -1, V)
    rp = c["row_ptr"]
    n_amb_rows = np.zeros((heads, L), np.int64)
    for p in range(L // V):
        n_amb_rows[:, p * V:(p + 1) * V] = amb[:, rp[p]:rp[p + 1], :].sum(axis=1)
    tol = 1e-3 + n_amb_rows[:, :, None] * float(s_p) * float(s_v) * 127.0
    err = np.abs(O - want)
    assert (err <= tol).all(), f"max err {err.max()} (ambiguous entries: {int(amb.sum())})"
    clean = n_amb_rows == 0
    assert clean.mean() > (0.9 if counts is None else 0.5)      # (rows of thousands of entries hold more near-ties)
    print(f"  max abs err {err.max():.3e}; clean rows max err {err[clean].max():.3e}; ambiguous {int(amb.sum())}",
          flush=True)


@pytest.mark.parametrize("token_major", [False, True])
@pytest.mark.parametrize("mode", [0, 1, 5])   # 5: two heads per workgroup on token-major tensors also in small launches
def test_attention_small(mode, token_major):
    _attention_check(2, 256, 64, 0.75, 1200, mode, token_major)   # one chunk per panel
    _attention_check(3, 512, 32, 0.9, 1201, mode, token_major)    # dk = 32: half of every row of the fused kernel's tile is padding
    _attention_check(2, 1024, 64, 0.6, 1202, mode, token_major)   # 410 vectors per panel: 7 chunks, ragged tail
    _attention_check(3, 1024, 64, 0.8, 1205, mode, token_major)   # odd head count: one head per workgroup
    _attention_check(2, 2048, 64, 0.75, 1203, mode, token_major)  # 512 vectors: the longest panel the fused kernel takes
    _attention_check(1, 2048, 64, 0.7, 1204, mode, token_major)   # 614 vectors: two waves share a (panel, head)


@pytest.mark.parametrize("token_major", [False, True])
@pytest.mark.parametrize("mode", [1, 6])   # 1: scores and softmax in one kernel, then the SpMM; 6: three kernels
def test_attention_pipeline_head_dimensions_and_long_panels(mode, token_major):
    """Head dimensions the single fused kernel does not take (16, 32, 96, 160, 256) and panels beyond its 2048
    vectors, through both forms of the kernel pipeline."""
    _attention_check(2, 256, 16, 0.5, 1260, mode, token_major)     # rows of 16 bytes: one copy segment real, three repeated
    _attention_check(3, 512, 32, 0.9, 1261, mode, token_major)
    _attention_check(2, 512, 96, 0.8, 1262, mode, token_major)     # 96 bytes in a 128-byte stage
    _attention_check(1, 512, 160, 0.75, 1263, mode, token_major)   # 160 bytes in a 256-byte stage
    _attention_check(2, 256, 256, 0.5, 1264, mode, token_major)    # the longest rows the one-kernel form takes
    _attention_check(1, 4096, 64, 0.45, 1265, mode, token_major)   # 2253 vectors per panel
    _attention_check(1, 4096, 32, 0.0, 1266, mode, token_major)    # 4096 vectors: 131 KB of scores per panel in LDS, two waves
    _attention_check(1, 2048, 320, 0.8, 1267, mode, token_major)   # rows of 320 bytes: three kernels in either mode
    _attention_check(2, 512, 64, 0.95, 1268, mode, token_major)    # 26 vectors per panel: a single ragged chunk


@pytest.mark.parametrize("token_major", [False, True])
@pytest.mark.parametrize("mode", [0, 3, 4])   # automatic; two / four waves per (panel, head)
def test_attention_fused_kernel_head_dimensions_below_its_tile(mode, token_major):
    """Head dimensions 16 .. 112 run in the fused kernel's tile of 64 or 128 with the missing pieces of every row
    read as zeros (no workspace needed)."""
    from paper_2209_06979_amd import binding as mc
    c = wl.attention_case(1, 256, 16, 8, 0.5, 1)
    m = mc.SparseMatrix(256, 256, 8, c["row_ptr"], c["col_idx"])
    for dk in (16, 32, 48, 80, 96, 112):
        assert mc.attention_workspace_needed(2, dk, m, 8, mc.Options(attention_mode=mode)) == 0
    m.close()
    _attention_check(2, 256, 16, 0.5, 1270, mode, token_major)     # one piece of four
    _attention_check(3, 512, 32, 0.9, 1271, mode, token_major)
    _attention_check(2, 1024, 48, 0.6, 1272, mode, token_major)    # 7 chunks, ragged tail
    _attention_check(2, 512, 80, 0.8, 1273, mode, token_major)     # five pieces of eight
    _attention_check(3, 1024, 96, 0.6, 1274, mode, token_major)
    _attention_check(1, 512, 112, 0.75, 1275, mode, token_major)
    _attention_check(1, 2048, 32, 0.4, 1276, mode, token_major)    # 1229 vectors: four waves in every mode
    _attention_check(2, 2048, 96, 0.6, 1277, mode, token_major)    # 819 vectors: at least two waves


def _lognormal_counts(P, mean, sigma, cap, seed):
    rng = np.random.default_rng(seed)
    c = rng.lognormal(0.0, sigma, P)
    return np.clip(np.rint(c / c.mean() * mean), 0, cap).astype(np.int64)


@pytest.mark.parametrize("token_major", [False, True])
@pytest.mark.parametrize("dk", [64, 96, 128])
def test_attention_panels_of_very_different_lengths_run_class_by_class(dk, token_major):
    """Masks whose panels span all four length classes (up to 8, 16, 32 and 64 chunks): one launch of the fused
    kernel per class, with 1, 2, 4 and 8 waves per (panel, head)."""
    L = 4096
    counts = _lognormal_counts(L // 8, 300, 1.0, L, 1280)
    counts[:6] = [4096, 0, 2049, 2048, 513, 1]
    assert (counts > 2048).sum() >= 2 and ((counts > 1024) & (counts <= 2048)).any() and ((counts > 512) & (counts <= 1024)).any()
    _attention_check(2, L, dk, None, 1281 + dk, 0, token_major, counts=counts)
    # two classes only, the long one with a single panel
    counts = np.full(L // 8, 100)
    counts[77] = 3000
    _attention_check(3, L, dk, None, 1290 + dk, 0, token_major, counts=counts)


@pytest.mark.parametrize("token_major", [False, True])
def test_attention_eight_waves_per_panel(token_major):
    _attention_check(1, 4096, 64, 0.45, 1295, 0, token_major)      # 2253 vectors in every panel: 36 chunks, eight waves
    _attention_check(2, 4096, 32, 0.0, 1296, 0, token_major)       # full panels of 4096 vectors, rows of half a tile
    _attention_check(1, 4096, 128, 0.3, 1297, 4, token_major)      # mode 4 asks for four waves: eight where needed


def test_attention_panels_beyond_on_chip_memory_fall_back_to_three_kernels():
    _attention_check(1, 8192, 32, 0.3, 1269, 1, False)             # 5734 vectors per panel: the scores do not fit LDS


@pytest.mark.parametrize("token_major", [False, True])
@pytest.mark.parametrize("mode", [2, 3, 4])
def test_attention_forced_fused_variants(mode, token_major):
    """One head per workgroup (2) and two / four waves per (panel, head) (3, 4) on short and long panels."""
    _attention_check(2, 256, 64, 0.75, 1210, mode, token_major)   # one chunk: most waves of a panel have nothing to do
    _attention_check(3, 1024, 64, 0.6, 1211, mode, token_major)   # 7 chunks, ragged tail
    _attention_check(2, 2048, 64, 0.75, 1212, mode, token_major)  # 8 chunks


@pytest.mark.parametrize("token_major", [False, True])
def test_attention_long_panels(token_major):
    _attention_check(2, 2048, 64, 0.6, 1220, 0, token_major)      # 819 vectors (13 chunks): two waves per (panel, head)
    _attention_check(1, 2048, 64, 0.4, 1221, 0, token_major)      # 1229 vectors (20 chunks): four waves
    _attention_check(1, 2048, 64, 0.0, 1222, 0, token_major)      # 2048 vectors (32 chunks): the longest fused panel
    _attention_check(1, 4096, 64, 0.45, 1223, 0, token_major)     # 2253 vectors: the kernel pipeline
    _attention_check(4, 2048, 64, 0.4, 1224, 0, token_major)      # 20 chunks, an even number of heads
    _attention_check(2, 2048, 64, 0.0, 1225, 0, token_major)      # 32 chunks, an even number of heads


@pytest.mark.parametrize("token_major", [False, True])
@pytest.mark.parametrize("mode", [0, 1, 3, 4])
def test_attention_head_dimension_128(mode, token_major):
    """Rows of 128 bytes: two MFMA steps per score tile and eight column tiles of output in the fused kernel."""
    _attention_check(2, 256, 128, 0.75, 1230, mode, token_major)   # one chunk per panel
    _attention_check(3, 1024, 128, 0.6, 1231, mode, token_major)   # 7 chunks, ragged tail
    _attention_check(2, 2048, 128, 0.75, 1232, mode, token_major)  # 8 chunks


@pytest.mark.parametrize("token_major", [False, True])
def test_attention_head_dimension_128_long_panels(token_major):
    _attention_check(2, 2048, 128, 0.6, 1233, 0, token_major)      # 13 chunks: two waves per (panel, head)
    _attention_check(1, 2048, 128, 0.0, 1234, 0, token_major)      # 32 chunks: four waves
    _attention_check(4, 4096, 128, 0.9, 1235, 0, token_major)      # the bench layer's pattern at head dimension 128


def test_attention_long_sequences():
    """Sequences of 16384 and 32768 tokens (2048 and 4096 panels per head)."""
    _attention_check(2, 16384, 64, 0.97, 1240, 0, True)      # 492 vectors per panel
    _attention_check(2, 16384, 128, 0.95, 1241, 0, False)    # 819 vectors: two waves per (panel, head), 128-byte rows
    _attention_check(1, 32768, 64, 0.98, 1242, 0, False)     # 655 vectors
    _attention_check(2, 16384, 64, 0.9, 1243, 0, True)       # 1638 vectors: four waves


@pytest.mark.parametrize("token_major", [False, True])
@pytest.mark.parametrize("mode", [0, 1, 6])
def test_attention_config5_full(mode, token_major):
    """BASELINE config 5: 8 heads, L=4096, dk=64, 90 % vector sparsity, diagonal kept."""
    _attention_check(8, 4096, 64, 0.9, wl.seed_for(5), mode, token_major)


def test_attention_ragged_rows():
    """Panels of very different lengths, including empty ones (their output rows are zero)."""
    import torch
    import oracle
    from paper_2209_06979_amd import binding as mc
    V, L, dk, heads = 8, 512, 64, 2
    counts = np.r_[[0, 1, 2, 15, 16, 17, 63, 64, 65, 127, 128, 129, 300, 511, 512, 0], np.full(L // V - 16, 40)]
    rp, ci = wl.ragged_pattern(L, L, V, counts, 1300)
    q8, s_q = prep.quantize_inputs_int8(wl.normal_fp32((heads, L, dk), 1301))
    k8, s_k = prep.quantize_inputs_int8(wl.normal_fp32((heads, L, dk), 1302))
    v8, s_v = prep.quantize_inputs_int8(wl.normal_fp32((heads, L, dk), 1303))
    s_p = np.float32(1 / 127)
    want, _, probs, _ = oracle.attention(q8, k8, v8, rp, ci, V, s_q, s_k, s_v, s_p)
    amb = _tie_ambiguous(probs, s_p).reshape(heads, -1, V)
    mask = mc.SparseMatrix(L, L, V, rp, ci)
    for mode, token_major in ((0, False), (0, True), (1, False), (1, True), (5, True), (3, True)):
        mc.set_attention_mode(mode)
        out = _layout(np.full((heads, L, dk), np.nan, np.float32), token_major)
        O = mc.sparse_attention(_layout(q8, token_major), _layout(k8, token_major), _layout(v8, token_major), mask,
                                s_q, s_k, s_v, s_p, out=out)
        torch.cuda.synchronize()
        mc.set_attention_mode(0)
        O = O.cpu().numpy().astype(np.float64)
        tol = np.full((heads, L), 1e-3)
        for p in range(L // V):
            tol[:, p * V:(p + 1) * V] += amb[:, rp[p]:rp[p + 1], :].sum(axis=1) * float(s_p) * float(s_v) * 127
        assert (np.abs(O - want) <= tol[:, :, None]).all(), mode
        assert not O[:, :8].any() and not O[:, 15 * 8:16 * 8].any()
    mask.close()


@pytest.mark.parametrize("p_bits,out_dtype", [(8, "float32"), (16, "float32"), (8, "float16")])
@pytest.mark.parametrize("dk", [64, 96])
def test_attention_pipeline_shares_very_long_panels(dk, p_bits, out_dtype):
    """A mask with a few panels many times longer than the rest: in the kernel pipeline the last SpMM cuts them into
    work items whose exact int32 tiles meet in workspace rows before they are scaled and rounded, so the output is
    the same, bit for bit, as with whole panels; and it matches the oracle."""
    import torch
    import oracle
    from paper_2209_06979_amd import binding as mc
    V, L, heads = 8, 2048, 2
    counts = np.r_[[2048, 1500, 0, 1], np.full(L // V - 4, 30)]
    rp, ci = wl.ragged_pattern(L, L, V, counts, 1400)
    (q8, s_q), (k8, s_k), (v8, s_v) = (prep.quantize_inputs_int8(wl.normal_fp32((heads, L, dk), 1401 + i)) for i in range(3))
    s_p = np.float32(1.0 / oracle.P_CODE_MAX[p_bits])
    dt = getattr(torch, out_dtype)
    mask = mc.SparseMatrix(L, L, V, rp, ci)
    results = {}
    for mode in (1, 6):
        for split in (1, 0, -1):
            o = mc.Options(attention_mode=mode, spmm_splitting=split)
            need = mc.attention_workspace_needed(heads, dk, mask, p_bits, o)
            for ws_bytes in ((need, need - 256) if split == 1 else (need,)):   # too small for the shared rows: whole panels
                ws = torch.empty(ws_bytes, dtype=torch.uint8, device="cuda")
                out = torch.full((heads, L, dk), float("nan"), dtype=dt, device="cuda")
                mc.sparse_attention(torch.from_numpy(q8).cuda(), torch.from_numpy(k8).cuda(), torch.from_numpy(v8).cuda(), mask,
                                    s_q, s_k, s_v, s_p, out=out, workspace=ws, p_bits=p_bits, out_dtype=dt, options=o)
                torch.cuda.synchronize()
                results[(mode, split, ws_bytes == need)] = out.cpu().numpy()
        assert (mc.attention_workspace_needed(heads, dk, mask, p_bits, mc.Options(attention_mode=mode, spmm_splitting=-1))
                == mc.attention_workspace_needed(heads, dk, mask, p_bits, mc.Options(attention_mode=mode))
                < mc.attention_workspace_needed(heads, dk, mask, p_bits, mc.Options(attention_mode=mode, spmm_splitting=1)))
    ref = results[(1, -1, True)]
    assert np.isfinite(ref).all()
    for key, O in results.items():
        assert np.array_equal(O, ref), key
    want, _, probs, _ = oracle.attention(q8, k8, v8, rp, ci, V, s_q, s_k, s_v, s_p, p_bits=p_bits)
    amb = _tie_ambiguous(probs, s_p).reshape(heads, -1, V)
    tol = np.full((heads, L), 1e-3 if out_dtype == "float32" else 3e-3)
    for p in range(L // V):
        tol[:, p * V:(p + 1) * V] += amb[:, rp[p]:rp[p + 1], :].sum(axis=1) * float(s_p) * float(s_v) * 127
    assert (np.abs(ref.astype(np.float64) - want) <= tol[:, :, None]).all()
    mask.close()


@pytest.mark.parametrize("prec,Kd,s,V", [("L8R8", 128, 0.9, 8), ("L8R8", 64, 0.7, 4), ("L4R4", 256, 0.7, 8),
                                          ("L8R8", 256, 0.95, 2), ("L4R4", 64, 0.95, 4)])
def test_config3_more_points_full_size(prec, Kd, s, V):
    _check(wl.sddmm_case(4096, 4096, Kd, V, s, prec, wl.seed_for(3, 500 + Kd + int(100 * s) + V)))


@pytest.mark.parametrize("prec", ["L8R8", "L4R4", "L16R16"])
def test_very_unequal_panels_use_work_items(prec):
    """A few panels many times longer than the rest are cut into several work items (one workgroup each)."""
    from paper_2209_06979_amd import binding as mc
    V, Nc, Kd = 8, 2048, 128
    counts = [30] * 40 + [2048, 1500, 0, 1] + [50] * 20
    M = V * len(counts)
    rp, ci = wl.ragged_pattern(M, Nc, V, counts, 191)
    if prec == "L4R4":
        Q, Km = wl.uniform_packed_int4((M, Kd // 2), 192), wl.uniform_packed_int4((Nc, Kd // 2), 193)
    elif prec == "L16R16":
        Q, Km = wl.uniform_int16((M, Kd), 192), wl.uniform_int16((Nc, Kd), 193)
    else:
        Q, Km = wl.uniform_int8((M, Kd), 192), wl.uniform_int8((Nc, Kd), 193)
    case = dict(M=M, Nc=Nc, Kd=Kd, V=V, prec=prec, row_ptr=rp, col_idx=ci, Q=Q, Kmat=Km)
    _check(case, variants=(-1, 0, 1, 4))
    mc.set_spmm_splitting(False)
    try:
        _check(case)
    finally:
        mc.set_spmm_splitting(True)
    if prec != "L16R16":
        case["lhs_unsigned"] = case["rhs_unsigned"] = True
        _check(case)


@pytest.mark.parametrize("prec", ["L8R8", "L4R4", "L16R16"])
@pytest.mark.parametrize("M,Nc,s", [(128, 4096, 0.5), (256, 2304, 0.7), (1024, 4096, 0.7), (8, 4096, 0.0)])
def test_few_long_panels_are_cut_into_work_items(prec, M, Nc, s):
    """Masks with fewer than 256 panels: the panels are cut into pieces of 8 chunks and more so that the
    launch has a workgroup for (about) every compute unit; with the cutting switched off: whole panels."""
    from paper_2209_06979_amd import binding as mc
    case = wl.sddmm_case(M, Nc, 128, 8, s, prec, 7000 + M)
    _check(case, variants=(-1, 0, 2, 8))
    mc.set_spmm_splitting(False)
    try:
        _check(case)
    finally:
        mc.set_spmm_splitting(True)


@pytest.mark.parametrize("waves", [-1, 0])
@pytest.mark.parametrize("prec", ["L8R8", "L4R4"])
def test_kmat_spanning_more_than_4_gib(prec, waves):
    """Rows of Kmat a mebibyte apart: the last rows start beyond 2^32 bytes (64-bit row offsets)."""
    import torch
    from paper_2209_06979_amd import binding as mc
    Nc, ld = 4128, (1 << 20) + 16
    c = wl.sddmm_case(256, Nc, 128, 8, 0.9, prec, 7500)
    want = run_sddmm_oracle(c)
    Kh = torch.from_numpy(c["Kmat"])
    big = torch.empty((Nc, ld), dtype=Kh.dtype, device="cuda")
    assert big.element_size() == 1 and (Nc - 32) * ld > 1 << 32
    Kv = big[:, :Kh.shape[1]]
    Kv.copy_(Kh.cuda())
    mask = mc.SparseMatrix(256, Nc, 8, c["row_ptr"], c["col_idx"])
    print(f"sddmm {prec} waves={waves} with Kmat rows {ld} bytes apart", flush=True)
    mc.set_sddmm_variant(waves)
    try:
        got = mc.sddmm(torch.from_numpy(c["Q"]).cuda(), Kv, mask, prec)
        torch.cuda.synchronize()
    finally:
        mc.set_sddmm_variant(-1)
        mask.close()
    assert np.array_equal(got.cpu().numpy(), want)
    del big


@pytest.mark.parametrize("prec", ["L8R8", "L4R4", "L16R16"])
def test_large_masks(prec):
    """Masks of 16384 x 16384 (98 % sparse) and 8192 x 32768 (V = 4, 99 % sparse)."""
    _check(wl.sddmm_case(16384, 16384, 64, 8, 0.98, prec, 7300))
    _check(wl.sddmm_case(8192, 32768, 128, 4, 0.99, prec, 7301))


def test_config3_whole_grid_full_size():
    """Every point of BASELINE config 3: Kd in {64,128,256} x sparsity in {0.7,0.9,0.95} x {L8-R8, L4-R4} at
    4096 x 4096, V = 8, whole outputs compared (18 points)."""
    for prec in ("L8R8", "L4R4"):
        for s in (0.7, 0.9, 0.95):
            for Kd in (64, 128, 256):
                _check(wl.sddmm_case(4096, 4096, Kd, 8, s, prec, wl.seed_for(3, 3000 + Kd + int(100 * s))))


def test_mask_without_any_stored_vector():
    """A mask that stores nothing is valid: SDDMM and the softmax have empty outputs and succeed."""
    import torch
    from paper_2209_06979_amd import binding as mc
    M, Nc, Kd, V = 32, 64, 64, 8
    rp, ci = wl.ragged_pattern(M, Nc, V, np.zeros(M // V, np.int64), 95)
    mask = mc.SparseMatrix(M, Nc, V, rp, ci)
    Q, Km = torch_dev(wl.uniform_int8((M, Kd), 96)), torch_dev(wl.uniform_int8((Nc, Kd), 97))
    S = mc.sddmm(Q, Km, mask, "L8R8")
    assert S.numel() == 0
    assert mc.sddmm_dequant(Q, Km, mask, "L8R8", 0.5, torch.float16).numel() == 0
    assert mc.sparse_softmax(mask, S.reshape(1, 0), 1.0, 127.0).numel() == 0
    torch.cuda.synchronize()
    mask.close()
