"""Host logic of the merged copy of an SpMM operand (no GPU): `group` consecutive panels as one panel of V * group
rows at the union of their columns.  Pinned against the oracle's dense matrix: merging must not change it."""
import numpy as np
import pytest

import oracle
from paper_2209_06979_amd import binding as mc
from paper_2209_06979_amd import workloads as wl


def _case(V, bits, counts, K=300, seed=1):
    M = V * len(counts)
    rp, ci = wl.ragged_pattern(M, K, V, counts, seed)
    nvec = len(ci)
    if bits == 8:
        vals = wl.uniform_int8((nvec, V), seed + 1)
    elif bits in (12, 16):
        vals = wl.uniform_int16((nvec, V), seed + 1, -2048, 2047)
    else:
        vals = wl.uniform_packed_int4((nvec, V // 2), seed + 1)
    return M, K, rp, ci, vals


GROUPS = [(V, bits, g) for V in (2, 4, 8) for bits in (4, 8, 16) for g in (2, 4, 8)
          if V * g == 8 or (V * g == 16 and bits in (4, 8))]


@pytest.mark.parametrize("V,bits,group", GROUPS)
def test_merged_operand_is_the_same_matrix(V, bits, group):
    counts = [0, 1, 63, 64, 65, 130, 0, 17, 0, 0, 5, 299, 300, 2, 2, 2, 2, 9, 31]   # 19 panels: the last group is ragged
    M, K, rp, ci, vals = _case(V, bits, counts, seed=100 * V + bits + group)
    m_rp, m_ci, m_vals, m_src = mc.merge_host(M, K, V, bits, rp, ci, vals, group)
    Vm, Pm = V * group, (len(counts) + group - 1) // group
    assert len(m_rp) == Pm + 1 and m_rp[0] == 0 and m_rp[-1] == len(m_ci)
    dense, _ = oracle.bcrs_to_dense(M, K, V, rp, ci, oracle.vector_values_as_int(vals, len(ci), V, bits))
    dense_m, flags_m = oracle.bcrs_to_dense(Pm * Vm, K, Vm, m_rp, m_ci, oracle.vector_values_as_int(m_values_view(m_vals, bits), len(m_ci), Vm, bits))
    assert np.array_equal(dense_m[:M], dense)
    assert not dense_m[M:].any()                     # rows past the matrix: zeros only
    # the merged pattern is exactly the union of its panels' patterns, ascending
    flags = oracle.stored_flags(M, K, V, rp, ci)
    for sp in range(Pm):
        union = np.flatnonzero(flags[sp * group:(sp + 1) * group].any(axis=0))
        assert np.array_equal(m_ci[m_rp[sp]:m_rp[sp + 1]], union)
    # every vector of the operand fills exactly one share, in its own panel's rows, at its own column
    src = m_src.reshape(-1, group)
    used = src[src >= 0]
    assert np.array_equal(np.sort(used), np.arange(len(ci)))
    panel_of = np.repeat(np.arange(len(counts)), np.diff(rp))
    for i in range(0, len(m_ci), 7):
        sp = int(np.searchsorted(m_rp, i, side="right") - 1)
        for g in range(group):
            v = src[i, g]
            if v >= 0:
                assert panel_of[v] == sp * group + g and ci[v] == m_ci[i]
    vb = V * (16 if bits == 16 else bits) // 8
    shares = m_vals.reshape(-1, vb)
    raw = np.ascontiguousarray(vals).view(np.uint8).reshape(-1, vb)
    assert np.array_equal(shares[src.reshape(-1) >= 0], raw[used])
    assert not shares[src.reshape(-1) < 0].any()


def m_values_view(m_vals, bits):
    return m_vals.view(np.int16) if bits == 16 else m_vals


def test_merged_query_rejects_what_it_cannot_build():
    M, K, rp, ci, vals = _case(4, 8, [3, 0, 5, 7])
    ml = mc.MergedLayout()
    q = lambda V, bits, group: mc.lib.mc_merged_query(M, K, V, bits, mc._p32(mc._i32(rp)), mc._p32(mc._i32(ci)), group, None if group == 99 else ml)
    assert q(4, 8, 2) == mc.MC_OK and ml.group == 2 and ml.P == 2
    assert q(4, 8, 4) == mc.MC_OK and ml.P == 1
    assert q(4, 16, 4) == mc.MC_EINVAL          # 16 rows of two-plane values do not fit the matrix unit
    assert q(4, 8, 3) == mc.MC_EINVAL and q(4, 8, 1) == mc.MC_EINVAL and q(4, 8, 8) == mc.MC_EINVAL
    assert q(4, 8, 99) == mc.MC_EINVAL          # no output structure
    bad = np.array(ci); bad[1], bad[0] = bad[0], bad[1]
    assert mc.lib.mc_merged_query(M, K, 4, 8, mc._p32(mc._i32(rp)), mc._p32(mc._i32(bad)), 2, ml) == mc.MC_EINVAL
    # the public builders keep to the interchange format's vector lengths
    lay = mc.Layout()
    assert mc.lib.mc_layout_query(32, K, 16, 8, mc._p32(mc._i32(np.array([0, 1, 2]))), lay) == mc.MC_EINVAL


def test_pattern_only_and_empty_operands():
    counts = [0, 0, 0, 0, 0]
    M, K, rp, ci, vals = _case(2, 8, counts)
    m_rp, m_ci, m_vals, m_src = mc.merge_host(M, K, 2, 8, rp, ci, vals, 4)
    assert list(m_rp) == [0, 0, 0] and len(m_ci) == 0 and len(m_src) == 0 and len(m_vals) == 0
    M, K, rp, ci, vals = _case(4, 8, [5, 0, 9])
    m_rp, m_ci, m_vals, m_src = mc.merge_host(M, K, 4, 0, rp, ci, None, 2)      # a pattern without values
    assert m_vals is None
    flags = oracle.stored_flags(M, K, 4, rp, ci)
    assert np.array_equal(m_ci[m_rp[0]:m_rp[1]], np.flatnonzero(flags[0] | flags[1]))
    assert np.array_equal(m_ci[m_rp[1]:m_rp[2]], np.flatnonzero(flags[2]))
    assert (m_src.reshape(-1, 2)[m_rp[1]:, 1] == -1).all()                       # the ragged group's missing panel
