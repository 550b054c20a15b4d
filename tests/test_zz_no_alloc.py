"""The entry point that allocates nothing (mc_sparse_attention_static) against the entry point that takes a
caller's workspace (mc_sparse_attention_ex), through the C ABI: two calls in a row, the second on a smaller
input, so that what the first call left in the library's own array is there when the second one runs."""
import numpy as np
import pytest

from paper_2209_06979_amd import workloads as wl
import input_prep as prep

pytestmark = pytest.mark.gpu


def _inputs(heads, L, dk, sparsity, seed, qkv_bits):
    import torch
    c = wl.attention_case(heads, L, dk, 8, sparsity, seed)
    quant = prep.quantize_inputs_int4 if qkv_bits == 4 else prep.quantize_inputs_int8
    (q, s_q), (k, s_k), (v, s_v) = (quant(c[n]) for n in "qkv")
    dev = [torch.from_numpy(np.ascontiguousarray(t)).cuda() for t in (q, k, v)]
    return c, dev, (s_q, s_k, s_v)


def _both(mc, heads, L, dk, sparsity, seed, p_bits=8, qkv_bits=8, options=None, out_dtype=None):
    """Returns (result of the no-allocation entry point, result of the entry point with a workspace), as numpy."""
    import torch
    out_dtype = out_dtype or torch.float32
    c, (q, k, v), (s_q, s_k, s_v) = _inputs(heads, L, dk, sparsity, seed, qkv_bits)
    s_p = np.float32(1.0 / (32639.0 if p_bits == 16 else 127.0))
    mask = mc.SparseMatrix(L, L, 8, c["row_ptr"], c["col_idx"])
    opts = options if options is not None else mc.Options()
    want = mc.sparse_attention(q, k, v, mask, s_q, s_k, s_v, s_p, p_bits=p_bits, qkv_bits=qkv_bits, out_dtype=out_dtype,
                               options=opts)
    got = torch.full((heads, L, dk), float("nan"), dtype=out_dtype, device="cuda")
    torch.cuda.synchronize()
    before = torch.cuda.memory_allocated()
    mc.sparse_attention_static(q, k, v, mask, s_q, s_k, s_v, s_p, got, p_bits=p_bits, qkv_bits=qkv_bits, options=opts)
    torch.cuda.synchronize()
    assert torch.cuda.memory_allocated() == before          # the wrapper took no device memory from torch either
    mask.close()
    return got.cpu().numpy(), want.cpu().numpy(), c, (q, k, v, s_q, s_k, s_v, s_p)


def test_two_calls_second_smaller_equal_the_workspace_entry_point():
    """dk = 160 always runs as the kernel pipeline, whose codes (and scores) live in the library's array.  Both entry
    points launch the same kernels on the same inputs, so the outputs must be identical bit for bit."""
    from paper_2209_06979_amd import binding as mc
    print("no-alloc: 3 heads x 512 x 160, then 2 heads x 256 x 160", flush=True)
    got, want, _, _ = _both(mc, 3, 512, 160, 0.8, 7001)
    assert not np.isnan(got).any() and np.array_equal(got, want)
    got, want, _, _ = _both(mc, 2, 256, 160, 0.75, 7002)       # smaller: the array still holds the first call's data
    assert not np.isnan(got).any() and np.array_equal(got, want)


def test_against_the_oracle_after_a_larger_call():
    """The second, smaller call also agrees with the CPU oracle (so stale contents of the shared array are not read)."""
    import oracle
    from paper_2209_06979_amd import binding as mc
    _both(mc, 4, 1024, 160, 0.8, 7003)
    got, want, c, (q, k, v, s_q, s_k, s_v, s_p) = _both(mc, 2, 256, 160, 0.75, 7004)
    ref, _, probs, _ = oracle.attention(q.cpu().numpy(), k.cpu().numpy(), v.cpu().numpy(), c["row_ptr"], c["col_idx"], 8,
                                        s_q, s_k, s_v, s_p)
    x = probs / np.float64(s_p)
    amb = (np.abs((x - np.floor(x)) - 0.5) < 1e-4 + 1e-5 * x).reshape(2, -1, 8)
    rp = c["row_ptr"]
    n_amb = np.zeros((2, 256), np.int64)
    for p in range(256 // 8):
        n_amb[:, p * 8:(p + 1) * 8] = amb[:, rp[p]:rp[p + 1], :].sum(axis=1)
    tol = 1e-3 + n_amb[:, :, None] * float(s_p) * float(s_v) * 127.0
    assert (np.abs(got.astype(np.float64) - ref) <= tol).all()


@pytest.mark.parametrize("p_bits,qkv_bits", [(16, 8), (8, 4)])
def test_other_widths_and_fp16_output(p_bits, qkv_bits):
    import torch
    from paper_2209_06979_amd import binding as mc
    pipeline = mc.Options()
    pipeline.attention_mode = 1                                  # dk = 64 through the kernel pipeline
    got, want, _, _ = _both(mc, 2, 512, 64, 0.8, 7010 + p_bits, p_bits, qkv_bits, pipeline, torch.float16)
    assert np.array_equal(got.view(np.uint16), want.view(np.uint16))
    got, want, _, _ = _both(mc, 2, 256, 64, 0.75, 7020 + p_bits, p_bits, qkv_bits, pipeline)
    assert np.array_equal(got, want)


def test_fused_path_needs_no_scratch_and_sizes_beyond_the_array_are_refused():
    import torch
    from paper_2209_06979_amd import binding as mc
    got, want, _, _ = _both(mc, 2, 512, 64, 0.8, 7030)           # automatic: the fused kernel, nothing staged
    assert np.array_equal(got, want)
    # 8 heads x L = 4096 at 90 % with 16-bit codes: 29 MB of codes alone, the array holds 16 MiB
    c, (q, k, v), (s_q, s_k, s_v) = _inputs(8, 4096, 160, 0.9, 7031, 8)
    mask = mc.SparseMatrix(4096, 4096, 8, c["row_ptr"], c["col_idx"])
    assert mc.attention_workspace_needed(8, 160, mask, 16) > mc.STATIC_SCRATCH_BYTES
    out = torch.full((8, 4096, 160), 5.0, dtype=torch.float32, device="cuda")
    with pytest.raises(mc.MagicubeError) as e:
        mc.sparse_attention_static(q, k, v, mask, s_q, s_k, s_v, np.float32(1 / 32639), out, p_bits=16)
    assert e.value.status == mc.MC_ENOMEM
    torch.cuda.synchronize()
    assert bool((out == 5.0).all())                               # refused before any launch
    # the same layer with 8-bit codes fits since its scores never leave the chip (14.7 MB of codes)
    assert mc.attention_workspace_needed(8, 160, mask, 8) <= mc.STATIC_SCRATCH_BYTES
    want = mc.sparse_attention(q, k, v, mask, s_q, s_k, s_v, np.float32(1 / 127))
    mc.sparse_attention_static(q, k, v, mask, s_q, s_k, s_v, np.float32(1 / 127), out)
    torch.cuda.synchronize()
    assert torch.equal(out, want)
    mask.close()
