"""GPU parity of the sparse softmax with fused re-quantisation (Section 5.3) against the CPU oracle:
every vector length and code width, both kernels (scores kept in registers / any panel length),
both output orders.  Codes are integers decided by fp32 arithmetic on the GPU and fp64 in the oracle:
they must agree except where p / s_p lies within fp32 accuracy of a rounding boundary, where one
code step is allowed (the entries are identified from the oracle's probabilities)."""
import numpy as np
import pytest

from paper_2209_06979_amd import workloads as wl
from gpu_util import torch_dev
from test_gpu_sddmm import _tie_ambiguous

pytestmark = pytest.mark.gpu


def _check(V, L, counts, seed, bits, variant=0, batch=2, score_range=60000, scale=2.5e-4):
    import torch
    import oracle
    from paper_2209_06979_amd import binding as mc
    rp, ci = wl.ragged_pattern(L, L, V, counts, seed)
    nnz = len(ci) * V
    print(f"softmax V={V} L={L} nvec={len(ci)} longest={int(np.max(counts))} bits={bits} variant={variant}", flush=True)
    S = np.random.default_rng(seed + 1).integers(-score_range, score_range, size=(batch, nnz)).astype(np.int32)
    pmax = oracle.P_CODE_MAX[bits]
    mask = mc.SparseMatrix(L, L, V, rp, ci)
    mc.set_softmax_variant(variant)
    try:
        out = torch.full((batch, nnz), -3, dtype=torch.int8 if bits == 8 else torch.int16, device="cuda")
        codes = mc.sparse_softmax(mask, torch_dev(S), float(np.float32(scale)), float(pmax), out=out, code_bits=bits)
        torch.cuda.synchronize()
    finally:
        mc.set_softmax_variant(0)
        mask.close()
    codes = codes.cpu().numpy()
    for b in range(batch):
        p = oracle.sparse_softmax(S[b], rp, V, np.float32(scale))
        want = oracle.requantize_probabilities(p, 1.0 / pmax, bits)
        amb = _tie_ambiguous(p, 1.0 / pmax)
        diff = codes[b].astype(np.int32) - want.astype(np.int32)
        assert (diff[~amb] == 0).all(), f"{np.count_nonzero(diff[~amb])} code mismatches away from ties"
        assert (np.abs(diff[amb]) <= 1).all()
        # the allowance must stay an exception: few entries near a boundary (8-bit codes; a 16-bit code of
        # some thousands is within fp32 accuracy of a boundary more often) and most codes equal anyway
        assert (amb.mean() < 0.05 or bits == 16) and (diff == 0).mean() > 0.97


def _counts(P, head, fill):
    c = np.full(P, fill)
    c[:len(head)] = head
    return c


@pytest.mark.parametrize("variant", [0, 1, 2])     # a wave per panel / a workgroup per panel / the any-length kernel
@pytest.mark.parametrize("bits", [8, 16])
@pytest.mark.parametrize("V", [2, 4, 8])
def test_softmax_ragged_panels(V, bits, variant):
    # empty, one vector, odd counts (for V = 2 the following panels start at 2-byte / 4-byte offsets
    # that are no multiple of a whole piece), around the 64-vector chunk and the full row
    L = 512
    _check(V, L, _counts(L // V, [1, 0, 3, 63, 64, 65, 129, 512], 51), 7000 + V, bits, variant)


@pytest.mark.parametrize("bits", [8, 16])
@pytest.mark.parametrize("V", [2, 4, 8])
def test_softmax_panel_lengths_around_the_register_limits(V, bits):
    """4096 and 16384 scores per panel (padding included) are the limits of the kernels that keep a
    panel in the registers of a wave / of a workgroup; the panels here sit just below, at and above them."""
    L = 4096
    per = lambda scores: scores // V            # vectors for a number of scores
    head = [per(4096) - 1, per(4096), per(4096) + 1]
    _check(V, L, _counts(L // V, head, 5), 7100 + V, bits)                     # longest > 4096 scores: a workgroup per panel
    _check(V, L, _counts(L // V, [per(4096)], 5), 7110 + V, bits)              # exactly 4096: a wave per panel
    if per(16384) <= L:
        _check(V, L, _counts(L // V, [per(16384)], 5), 7120 + V, bits)         # exactly 16384
    if per(16384) + 1 <= L:
        _check(V, L, _counts(L // V, [per(16384) + 1, 7], 5), 7130 + V, bits)  # beyond: the any-length kernel


def test_softmax_extreme_scores_and_single_entries():
    # scores over the whole int32 range; |x| up to 215: exp underflows to 0 for all but the largest entries
    # (beyond that the fp32 product S * scale itself is too coarse for the comparison); single-entry rows: p = 1
    _check(8, 256, _counts(32, [1, 1, 2], 40), 7200, 8, score_range=2 ** 31 - 1, scale=1e-7)
    _check(8, 256, _counts(32, [1, 1, 2], 40), 7201, 16, score_range=2 ** 31 - 1, scale=1e-8)
    _check(4, 256, _counts(64, [1], 9), 7202, 8, score_range=3, scale=1e-3)    # nearly uniform rows


@pytest.mark.parametrize("variant", [0, 1, 2])
def test_softmax_config5_shape(variant):
    c = wl.attention_case(1, 4096, 64, 8, 0.9, wl.seed_for(5, 3))
    counts = np.diff(c["row_ptr"])
    _check(8, 4096, counts, 7300, 8, variant, batch=2)     # 1024 (panel, score set) units: two waves per panel
    _check(8, 4096, counts, 7301, 16, variant, batch=3)    # 1536 units: one wave per panel
