"""SDDMM whose epilogue re-quantises the scores and writes the device format of the following SpMM's sparse
operand (Section 4.3), through the C ABI: the chained SpMM must equal the oracle's SpMM of the oracle's codes,
bit for bit (the codes are decided in binary32 on both sides)."""
import numpy as np
import pytest

from paper_2209_06979_amd import workloads as wl
from gpu_util import torch_dev

pytestmark = pytest.mark.gpu


def _chain(M, Nc, Kd, V, pattern, prec, p_bits, scale, N, seed, variant=-1, spmm_prec=None):
    import torch
    import oracle
    from paper_2209_06979_amd import binding as mc
    rp, ci = pattern
    c = wl.sddmm_case(M, Nc, Kd, V, 0.5, prec, seed)
    nvec = len(ci)
    print(f"sddmm_to_mat {prec} -> {p_bits}-bit codes M={M} Nc={Nc} Kd={Kd} V={V} nvec={nvec} variant={variant}", flush=True)
    S = oracle.sddmm(M, Nc, V, rp, ci, c["Q"], c["Kmat"], prec)
    codes = oracle.requantize_scores(S, scale, p_bits).reshape(nvec, V)
    assert np.abs(codes).max(initial=0) > 3                       # the scale leaves something to compare
    spmm_prec = spmm_prec or ("L8R8" if p_bits == 8 else "L16R8")
    B = wl.uniform_int8((Nc, N), seed + 7)
    want = oracle.spmm(M, Nc, V, rp, ci, codes, B, spmm_prec)
    # P starts with poison values so that slots the kernel does not write show up
    poison = np.full((nvec, V), 77, np.int8 if p_bits == 8 else np.int16)
    P = mc.SparseMatrix(M, Nc, V, rp, ci, poison, p_bits)
    mc.set_sddmm_variant(variant)
    try:
        mc.sddmm_to_mat(torch_dev(c["Q"]), torch_dev(c["Kmat"]), P, prec, scale)
    finally:
        mc.set_sddmm_variant(-1)
    out = torch.full((M, N), -7777777, dtype=torch.int32, device="cuda")
    mc.spmm(P, torch_dev(B), spmm_prec, out=out)
    torch.cuda.synchronize()
    P.close()
    got = out.cpu().numpy()
    bad = np.argwhere(got != want)
    assert len(bad) == 0, f"{len(bad)} mismatches, first at {bad[:5].tolist()}"


def _uniform(M, Nc, V, s, seed):
    return wl.vector_sparse_pattern(M, Nc, V, s, seed)


@pytest.mark.parametrize("V", [2, 4, 8])
@pytest.mark.parametrize("prec,p_bits,Kd,scale", [("L8R8", 8, 64, 2e-3), ("L8R8", 16, 128, 0.4), ("L4R4", 8, 64, 0.15),
                                                  ("L4R4", 16, 256, 7.0), ("L16R16", 8, 64, 3e-7), ("L16R16", 16, 128, 6e-5)])
def test_chain_into_spmm_equals_the_oracle(V, prec, p_bits, Kd, scale):
    _chain(32 * V, 512, Kd, V, _uniform(32 * V, 512, V, 0.7, 9000 + V), prec, p_bits, scale, 64, 9001 + V + Kd)


@pytest.mark.parametrize("variant", [0, 1, 2, 4, 8])
def test_every_kernel_variant_and_ragged_panels(variant):
    """Ragged and empty panels (the padded slots of every last chunk must come out as zeros), the kernel that
    loads operands straight from memory (0) and the LDS-staged one with 1 .. 8 waves."""
    V, Nc = 8, 700
    counts = [0, 1, 63, 64, 65, 130, 0, 17, 300, 700, 2, 0]
    pattern = wl.ragged_pattern(V * len(counts), Nc, V, counts, 9100)
    _chain(V * len(counts), Nc, 128, V, pattern, "L8R8", 8, 1.5e-3, 48, 9101, variant)
    _chain(V * len(counts), Nc, 64, V, pattern, "L4R4", 16, 3.0, 48, 9102, variant)
    _chain(V * len(counts), Nc, 80, V, pattern, "L8R8", 8, 2e-3, 48, 9103, variant)      # 80-byte rows: direct kernel whatever the variant


def test_saturation_and_exact_ties():
    """Scale 0.5 makes every odd score an exact tie (rounded to even); a large scale saturates at +-127 / +-32639."""
    V = 8
    pattern = _uniform(64, 256, V, 0.5, 9200)
    _chain(64, 256, 64, V, pattern, "L4R4", 8, 0.5, 32, 9201)
    _chain(64, 256, 64, V, pattern, "L4R4", 16, 0.5, 32, 9202)
    _chain(64, 256, 64, V, pattern, "L8R8", 8, 1.0, 32, 9203)
    _chain(64, 256, 64, V, pattern, "L8R8", 16, 1.0, 32, 9204)


def test_skewed_mask_with_work_items():
    """One panel many times longer than the others: the mask is cut into work items, every item writes its own chunks."""
    V, Nc = 8, 4096
    counts = [40] * 63 + [4000]
    pattern = wl.ragged_pattern(V * len(counts), Nc, V, counts, 9300)
    _chain(V * len(counts), Nc, 64, V, pattern, "L8R8", 8, 2e-3, 64, 9301)


def test_full_size_attention_like_shape():
    """4096 x 4096 mask at 90 % sparsity, Kd = 64: the score matrix of one attention head fed back as an SpMM operand."""
    _chain(4096, 4096, 64, 8, wl.vector_sparse_pattern(4096, 4096, 8, 0.9, 9400, keep_diagonal=True), "L8R8", 8, 2e-3, 64, 9401)


def test_argument_checks():
    import torch
    from paper_2209_06979_amd import binding as mc
    rp, ci = _uniform(64, 256, 8, 0.5, 9500)
    Q = torch.zeros((64, 64), dtype=torch.int8, device="cuda")
    K = torch.zeros((256, 64), dtype=torch.int8, device="cuda")
    mask = mc.SparseMatrix(64, 256, 8, rp, ci)
    with pytest.raises(mc.MagicubeError) as e:
        mc.sddmm_to_mat(Q, K, mask, "L8R8", 1.0)
    assert e.value.status == mc.MC_EINVAL
    P4 = mc.SparseMatrix(64, 256, 8, rp, ci, np.zeros((len(ci), 4), np.uint8), 4)
    with pytest.raises(mc.MagicubeError) as e:
        mc.sddmm_to_mat(Q, K, P4, "L8R8", 1.0)
    assert e.value.status == mc.MC_EUNSUPPORTED
    P = mc.SparseMatrix(64, 256, 8, rp, ci, np.zeros((len(ci), 8), np.int8), 8)
    for bad in (float("nan"), float("inf")):
        with pytest.raises(mc.MagicubeError):
            mc.sddmm_to_mat(Q, K, P, "L8R8", bad)
    with pytest.raises(mc.MagicubeError) as e:
        mc.sddmm_to_mat(Q, K, P, "L8R4", 1.0)
    assert e.value.status == mc.MC_EUNSUPPORTED
    for m in (mask, P4, P):
        m.close()
