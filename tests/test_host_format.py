"""Host logic of the library (no GPU): format builder round trips, padding, argument
checks, and that the shared library exports every symbol the header declares."""
import ctypes
import os
import re

import numpy as np
import pytest

from paper_2209_06979_amd import binding as mc
from paper_2209_06979_amd import workloads as wl

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _case(V, bits, counts, K=300, seed=1):
    M = V * len(counts)
    rp, ci = wl.ragged_pattern(M, K, V, counts, seed)
    nvec = len(ci)
    if bits == 8:
        vals = wl.uniform_int8((nvec, V), seed + 1)
    elif bits == 16:
        vals = wl.uniform_int16((nvec, V), seed + 1, -32768, 32639)
    else:
        vals = wl.uniform_packed_int4((nvec, V // 2), seed + 1)
    return M, K, rp, ci, vals


def test_header_symbols_are_exported():
    text = open(os.path.join(ROOT, "include", "magicube.h")).read()
    names = set(re.findall(r"\b(mc_[a-z0-9_]+)\s*\(", text))
    assert {"mc_spmm", "mc_sddmm", "mc_sparse_attention", "mc_mat_create", "mc_pack_host"} <= names
    lib = ctypes.CDLL(mc.LIB_PATH)
    for n in sorted(names):
        assert hasattr(lib, n), f"{n} declared in magicube.h but not exported"
    assert mc.lib.mc_version().decode().endswith("gfx950")
    assert mc.lib.mc_strerror(mc.MC_EALIGN).decode().startswith("pointer")


@pytest.mark.parametrize("V", [2, 4, 8])
@pytest.mark.parametrize("bits", [4, 8, 16])
def test_round_trip_and_padding(V, bits):
    counts = [0, 1, 63, 64, 65, 130, 0, 17]
    M, K, rp, ci, vals = _case(V, bits, counts, seed=10 * V + bits)
    pp, si, sv = mc.pack_host(M, K, V, bits, rp, ci, vals)
    lay = mc.layout_query(M, K, V, bits, rp)
    assert lay.P == len(counts) and lay.nvec == sum(counts)
    assert lay.nslots == sum((c + 63) // 64 * 64 for c in counts)
    assert lay.vals_bytes == lay.nslots * V * bits // 8
    for p, c in enumerate(counts):
        assert pp[2 * p] % 64 == 0 and pp[2 * p + 1] - pp[2 * p] == c      # aligned start, real end
    rp2, ci2, vals2 = mc.unpack_host(M, K, V, bits, pp, si, sv)
    assert np.array_equal(rp2, rp) and np.array_equal(ci2, ci)
    assert np.array_equal(vals2, np.ascontiguousarray(vals).view(np.uint8).reshape(-1))
    # padded slots: a valid column and all-zero values
    assert si.min() >= 0 and si.max() < K
    cb = 64 * V * bits // 8
    chunks = sv.reshape(-1, cb)
    for p, c in enumerate(counts):
        for s in range(pp[2 * p + 1], pp[2 * p] + (c + 63) // 64 * 64):
            ch, g, b = chunks[s // 64], (s % 64) // 16, s % 16
            if bits == 8:
                assert not ch.reshape(4, V, 16)[g, :, b].any()
            elif bits == 16:
                assert not ch.reshape(4, 2, V, 16)[g, :, :, b].any()
            else:
                byte = ch.reshape(4, V, 8)[g, :, b % 8]
                assert not ((byte >> (4 * (b // 8))) & 15).any()
            assert si[s] == ci[rp[p + 1] - 1]


def test_device_layout_int8_and_int16_planes():
    """Slot s of a panel sits at [chunk s/64][sub-stride (s%64)/16][row v][s%16]."""
    V = 8
    M, K, rp, ci, vals = _case(V, 8, [70], seed=3)
    pp, si, sv = mc.pack_host(M, K, V, 8, rp, ci, vals)
    arr = sv.view(np.int8).reshape(2, 4, V, 16)
    for s in range(70):
        assert np.array_equal(arr[s // 64, (s % 64) // 16, :, s % 16], vals[s])
    M, K, rp, ci, v16 = _case(V, 16, [70], seed=4)
    pp, si, sv = mc.pack_host(M, K, V, 16, rp, ci, v16)
    arr = sv.view(np.int8).reshape(2, 4, 2, V, 16).astype(np.int32)
    for s in range(70):
        hi, lo = arr[s // 64, (s % 64) // 16, 0, :, s % 16], arr[s // 64, (s % 64) // 16, 1, :, s % 16]
        assert np.array_equal(hi * 256 + lo, v16[s].astype(np.int32))       # both planes signed int8


def test_int16_range_and_bad_arguments():
    V, K = 8, 16
    rp = np.array([0, 1], np.int32); ci = np.array([3], np.int32)
    ok = np.full((1, V), 32639, np.int16)
    mc.pack_host(V, K, V, 16, rp, ci, ok)
    bad = np.full((1, V), 32640, np.int16)
    with pytest.raises(mc.MagicubeError) as e:
        mc.pack_host(V, K, V, 16, rp, ci, bad)
    assert e.value.status == mc.MC_ERANGE
    vals = np.zeros((1, V), np.int8)
    for kw in (dict(V=3), dict(M=7), dict(bits=5), dict(K=0)):
        a = dict(M=V, K=K, V=V, bits=8); a.update(kw)
        with pytest.raises(mc.MagicubeError) as e:
            mc.pack_host(a["M"], a["K"], a["V"], a["bits"], rp, ci, vals)
        assert e.value.status == mc.MC_EINVAL
    for bad_ci in ([16], [-1]):
        with pytest.raises(mc.MagicubeError) as e:
            mc.pack_host(V, K, V, 8, rp, np.array(bad_ci, np.int32), vals)
        assert e.value.status == mc.MC_EINVAL
    rp2 = np.array([0, 2], np.int32)
    for bad_ci in ([5, 5], [6, 2]):                                        # duplicates / descending
        with pytest.raises(mc.MagicubeError) as e:
            mc.pack_host(V, K, V, 8, rp2, np.array(bad_ci, np.int32), np.zeros((2, V), np.int8))
        assert e.value.status == mc.MC_EINVAL
    with pytest.raises(mc.MagicubeError):
        mc.pack_host(V, K, V, 8, np.array([1, 2], np.int32), ci, vals)      # row_ptr[0] != 0
    with pytest.raises(mc.MagicubeError):
        mc.pack_host(2 * V, K, V, 8, np.array([0, 2, 1], np.int32), np.array([1, 2], np.int32),
                     np.zeros((2, V), np.int8))                             # decreasing row_ptr


def test_compute_entry_points_reject_null_handles_without_a_gpu():
    assert mc.lib.mc_spmm(None, None, 16, 16, 0, None, 16, None) == mc.MC_EINVAL
    assert mc.lib.mc_sddmm(None, 16, None, 16, 16, None, 0, None, None) == mc.MC_EINVAL
    assert mc.lib.mc_sparse_softmax(None, 1, None, 1.0, 127.0, None, None) == mc.MC_EINVAL
    assert mc.lib.mc_sparse_attention(None, None, None, 1, 8, 16, None, 1, 1, 1, 1, None, None, 0, None) == mc.MC_EINVAL
    assert mc.lib.mc_attention_workspace_bytes(1, None) == 0
    assert mc.lib.mc_mat_info(None, None, None, None, None, None, None) == mc.MC_EINVAL
    assert mc.lib.mc_set_spmm_variant(96, 0) == mc.MC_EINVAL and mc.lib.mc_set_spmm_variant(0, 3) == mc.MC_EINVAL
    assert mc.lib.mc_set_spmm_variant(0, 0) == mc.MC_OK
    mc.lib.mc_mat_destroy(None)


def test_12_bit_values_are_stored_like_16_and_range_checked():
    counts = [3, 0, 70]
    M, K, rp, ci, _ = _case(8, 16, counts, seed=99)
    vals = wl.uniform_int16((len(ci), 8), 100, -2048, 2047)
    pp, si, sv = mc.pack_host(M, K, 8, 12, rp, ci, vals)
    pp16, si16, sv16 = mc.pack_host(M, K, 8, 16, rp, ci, vals)
    assert np.array_equal(sv, sv16) and np.array_equal(si, si16)
    rp2, ci2, v2 = mc.unpack_host(M, K, 8, 12, pp, si, sv)
    assert np.array_equal(v2.view(np.int16).reshape(-1, 8), vals)
    bad = vals.copy()
    bad[1, 2] = 2048
    with pytest.raises(mc.MagicubeError) as e:
        mc.pack_host(M, K, 8, 12, rp, ci, bad)
    assert e.value.status == mc.MC_ERANGE


def test_entry_points_reject_bad_arguments_before_touching_the_gpu():
    """Null handles / pointers and unknown knob values come back as status codes (no GPU needed)."""
    L = mc.lib
    assert L.mc_spmm(None, None, 16, 16, 0, None, 16, None) == mc.MC_EINVAL
    assert L.mc_spmm_flags(None, None, 16, 16, 0, 0, None, 16, None) == mc.MC_EINVAL
    assert L.mc_sddmm(None, 64, None, 64, 64, None, 0, None, None) == mc.MC_EINVAL
    assert L.mc_sddmm_flags(None, 64, None, 64, 64, None, 0, 3, None, None) == mc.MC_EINVAL
    assert L.mc_sparse_softmax_bits(None, 1, None, 1.0, 1.0, 8, None, None) == mc.MC_EINVAL
    assert L.mc_sparse_attention_batched(None, None, None, 1, 1, 8, 64, 0, 512, 64, None, 8, 8, 1.0, 1.0, 1.0, 1.0,
                                         None, None, 0, None) == mc.MC_EINVAL
    assert L.mc_sparse_attention_out(None, None, None, 1, 1, 8, 64, 0, 512, 64, None, 8, 8, 1.0, 1.0, 1.0, 1.0, 1,
                                     None, None, 0, None) == mc.MC_EINVAL
    assert L.mc_sparse_attention_out(None, None, None, 1, 1, 8, 64, 0, 512, 64, None, 8, 8, 1.0, 1.0, 1.0, 1.0, 2,
                                     None, None, 0, None) == mc.MC_EUNSUPPORTED     # unknown output type
    assert L.mc_spmm_dequant(None, None, 16, 16, 0, 0, 1.0, 0, None, 16, None) == mc.MC_EINVAL
    assert L.mc_spmm_dequant(None, None, 16, 16, 0, 0, 1.0, 7, None, 16, None) == mc.MC_EUNSUPPORTED
    assert L.mc_sddmm_dequant(None, 64, None, 64, 64, None, 0, 0, 1.0, 1, None, None) == mc.MC_EINVAL
    assert L.mc_sddmm_dequant(None, 64, None, 64, 64, None, 0, 0, 1.0, -1, None, None) == mc.MC_EUNSUPPORTED
    assert L.mc_sparse_softmax_to_mat(None, None, 1.0, 1.0, None) == mc.MC_EINVAL
    assert L.mc_absmax(None, 4, None, None) == mc.MC_EINVAL
    assert L.mc_quantize(None, 4, 1.0, 8, None, None) == mc.MC_EINVAL
    assert L.mc_probe_gather(None, None, 16, 16, 0, None, None) == mc.MC_EINVAL
    assert L.mc_mat_info(None, None, None, None, None, None, None) == mc.MC_EINVAL
    assert L.mc_mat_set_values_device(None, None, None) == mc.MC_EINVAL
    assert L.mc_set_attention_mode(9) == mc.MC_EINVAL and L.mc_set_attention_mode(7) == mc.MC_EINVAL
    assert L.mc_set_attention_mode(-1) == mc.MC_EINVAL
    assert L.mc_set_attention_mode(5) == mc.MC_OK and L.mc_set_attention_mode(0) == mc.MC_OK
    assert L.mc_set_spmm_variant(100, 1) == mc.MC_EINVAL and L.mc_set_spmm_variant(0, 0) == mc.MC_OK
    assert L.mc_set_sddmm_variant(3) == mc.MC_EINVAL and L.mc_set_sddmm_variant(-1) == mc.MC_OK
    assert L.mc_attention_workspace_bytes_bits(4, None, 8) == 0
    assert L.mc_probe_gather_sink_len(None, 16, 0) == 0
    assert L.mc_probe_spmm_phases_len(None, 16) == 0
    assert L.mc_probe_spmm_phases(None, None, 16, 16, None, 16, None, None) == mc.MC_EINVAL
    assert L.mc_mat_merged_info(None, None, None) == mc.MC_EINVAL


# ---- K-blocked variant of the format --------------------------------------------------------
@pytest.mark.parametrize("V", [2, 4, 8])
@pytest.mark.parametrize("bits", [4, 8, 16])
def test_blocked_format_holds_the_same_matrix(V, bits):
    """Every stored vector appears exactly once, in the list of the K-block its column falls in, with its own
    values; every list is padded to whole chunks with zero values and a row of the same block."""
    K = 2500                                               # three blocks of 1024 columns, the last one partial
    counts = [0, 1, 63, 64, 65, 700, 0, 17, 2500]
    M, K, rp, ci, vals = _case(V, bits, counts, K=K, seed=20 * V + bits)
    nblk, bp, rows, bv, src = mc.pack_blocked_host(M, K, V, bits, rp, ci, vals)
    assert nblk == 3 and bp[0] == 0 and len(bp) == len(counts) * nblk + 1 and (np.diff(bp) >= 0).all()
    assert len(rows) == bp[-1] * 64 == len(src)
    # the ordinary device format of the same data, as the reference for the value layout of a chunk
    vbytes = 64 * V * bits // 8
    seen = np.zeros(len(ci), np.int64)
    for p in range(len(counts)):
        for b in range(nblk):
            c0, c1 = bp[p * nblk + b], bp[p * nblk + b + 1]
            want = [i for i in range(rp[p], rp[p + 1]) if b * 1024 <= ci[i] < (b + 1) * 1024]
            assert c1 - c0 == (len(want) + 63) // 64
            s = src[c0 * 64:c1 * 64]
            assert s[:len(want)].tolist() == want and (s[len(want):] == -1).all()
            pos = np.array([(t // 16) * 16 + (t % 8) * 2 + (t % 16) // 8 for t in range(64)])   # slot -> place in its chunk
            r = rows[c0 * 64:c1 * 64].astype(np.int64).reshape(-1, 64)[:, pos].reshape(-1)
            assert np.array_equal(r[:len(want)] + b * 1024, ci[want])
            assert (r[len(want):] == (r[len(want) - 1] if want else 0)).all()
            seen[want] += 1
            # values: pack the same vectors as one panel of an ordinary matrix and compare chunk by chunk
            if want:
                sub_rp = np.array([0, len(want)], np.int32)
                sub_vals = np.ascontiguousarray(vals)[want]
                _, _, ref = mc.pack_host(V, K, V, bits, sub_rp, ci[want], sub_vals)
                assert np.array_equal(bv[c0 * vbytes:c1 * vbytes], ref)
    assert (seen == 1).all()


def test_blocked_format_argument_checks():
    V, K = 8, 3000
    rp, ci = wl.ragged_pattern(16, K, V, [5, 9], 3)
    vals = wl.uniform_int8((len(ci), V), 4)
    bad = ci.copy(); bad[1] = bad[0]                         # not ascending
    with pytest.raises(mc.MagicubeError):
        mc.pack_blocked_host(16, K, V, 8, rp, bad, vals)
    bad = ci.copy(); bad[-1] = K                             # column out of range
    with pytest.raises(mc.MagicubeError):
        mc.pack_blocked_host(16, K, V, 8, rp, bad, vals)
    v16 = wl.uniform_int16((len(ci), V), 5, 32640, 32767)    # cannot be split into two signed bytes
    with pytest.raises(mc.MagicubeError) as e:
        mc.pack_blocked_host(16, K, V, 16, rp, ci, v16)
    assert e.value.status == mc.MC_ERANGE
    nblk, bp, rows, bv, src = mc.pack_blocked_host(16, K, V, 0, rp, ci, None)   # pattern only
    assert nblk == 3 and len(bv) == 0 and bp[-1] * 64 == len(rows)
