"""The benchmark replays its step as a HIP graph: every replay must equal the eager result."""
import numpy as np
import pytest

from paper_2209_06979_amd import workloads as wl
import input_prep as prep

pytestmark = pytest.mark.gpu


def test_graph_replays_match_eager():
    import torch
    from paper_2209_06979_amd import binding as mc
    dev = torch.device("cuda:0")
    c = wl.spmm_case(512, 512, 128, 8, 0.8, "L8R8", 11)
    A = mc.SparseMatrix(512, 512, 8, c["row_ptr"], c["col_idx"], c["values"], 8)
    B = torch.from_numpy(c["B"]).to(dev)
    s = wl.sddmm_case(512, 512, 64, 8, 0.8, "L8R8", 12)
    mask = mc.SparseMatrix(512, 512, 8, s["row_ptr"], s["col_idx"])
    Q, Km = torch.from_numpy(s["Q"]).to(dev), torch.from_numpy(s["Kmat"]).to(dev)
    a = wl.attention_case(2, 512, 64, 8, 0.8, 13)
    q8, s_q = prep.quantize_inputs_int8(a["q"]); k8, s_k = prep.quantize_inputs_int8(a["k"])
    v8, s_v = prep.quantize_inputs_int8(a["v"])
    amask = mc.SparseMatrix(512, 512, 8, a["row_ptr"], a["col_idx"])
    q8, k8, v8 = (torch.from_numpy(t).to(dev) for t in (q8, k8, v8))
    C = torch.empty((512, 128), dtype=torch.int32, device=dev)
    S = torch.empty(mask.nvec * 8, dtype=torch.int32, device=dev)
    O = torch.empty((2, 512, 64), dtype=torch.float32, device=dev)
    ws = torch.empty(mc.attention_workspace_bytes(2, amask), dtype=torch.uint8, device=dev)

    def step():
        mc.spmm(A, B, "L8R8", out=C)
        mc.sddmm(Q, Km, mask, "L8R8", out=S)
        mc.sparse_attention(q8, k8, v8, amask, s_q, s_k, s_v, np.float32(1 / 127), out=O, workspace=ws)

    for mode in (0, 1):
        mc.set_attention_mode(mode)
        step()
        torch.cuda.synchronize()
        want = [t.clone() for t in (C, S, O)]
        stream = torch.cuda.Stream()
        with torch.cuda.stream(stream):
            g = torch.cuda.CUDAGraph()
            with torch.cuda.graph(g, stream=stream):
                step()
            for _ in range(4):
                for t in (C, S, O):
                    t.zero_()                       # eager work between the replays
                torch.cuda.synchronize()
                g.replay()
                torch.cuda.synchronize()
                for got, ref in zip((C, S, O), want):
                    assert torch.equal(got, ref)
        mc.set_attention_mode(0)
    for h in (A, mask, amask):
        h.close()


def test_graph_replays_of_the_other_entry_points():
    """Captured once, replayed with eager work in between: the SpMM over work items (a row-clearing
    kernel plus atomics), the dequantising SpMM / SDDMM, the softmax writing a matrix's values, and
    absmax (its result cell is reset by a kernel, not by a memset) / quantize."""
    import torch
    from paper_2209_06979_amd import binding as mc
    dev = torch.device("cuda:0")
    V, K, N = 8, 2048, 128
    counts = np.r_[[2048, 1500, 0, 1], np.full(60, 30)]
    M = V * len(counts)
    rp, ci = wl.ragged_pattern(M, K, V, counts, 21)
    A = mc.SparseMatrix(M, K, V, rp, ci, wl.uniform_int8((len(ci), V), 22), 8)      # long panels: work items
    B = torch.from_numpy(wl.uniform_int8((K, N), 23)).to(dev)
    Q = torch.from_numpy(wl.uniform_int8((M, 64), 24)).to(dev)
    Km = torch.from_numpy(wl.uniform_int8((K, 64), 25)).to(dev)
    P = mc.SparseMatrix(M, K, V, rp, ci, np.zeros((len(ci), V), np.int8), 8)
    x = torch.from_numpy(wl.normal_fp32((1 << 16,), 26)).to(dev)
    C = torch.empty((M, N), dtype=torch.int32, device=dev)
    Ch = torch.empty((M, N), dtype=torch.float16, device=dev)
    Sf = torch.empty(A.nvec * V, dtype=torch.float32, device=dev)
    Si = torch.empty(A.nvec * V, dtype=torch.int32, device=dev)
    Cp = torch.empty((M, N), dtype=torch.int32, device=dev)
    mx = torch.empty(1, dtype=torch.float32, device=dev)
    xq = torch.empty(x.numel(), dtype=torch.int8, device=dev)
    outs = (C, Ch, Sf, Si, Cp, mx, xq)

    def step():
        mc.spmm(A, B, "L8R8", out=C)
        mc.spmm_dequant(A, B, "L8R8", 1e-3, torch.float16, out=Ch)
        mc.sddmm_dequant(Q, Km, A, "L8R8", 1e-3, torch.float32, out=Sf)
        mc.sddmm(Q, Km, A, "L8R8", out=Si)
        mc.sparse_softmax_to_mat(P, Si, 1e-3, 127.0)
        mc.spmm(P, B, "L8R8", out=Cp)
        mc.absmax(x, out=mx)
        mc.quantize(x, 0.03, 8, out=xq)

    step()
    torch.cuda.synchronize()
    want = [t.clone() for t in outs]
    stream = torch.cuda.Stream()
    with torch.cuda.stream(stream):
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g, stream=stream):
            step()
        for _ in range(4):
            for t in outs:
                t.fill_(3)                          # eager work between the replays; C is NOT left cleared
            torch.cuda.synchronize()
            g.replay()
            torch.cuda.synchronize()
            for got, ref in zip(outs, want):
                assert torch.equal(got, ref)
    A.close()
    P.close()
