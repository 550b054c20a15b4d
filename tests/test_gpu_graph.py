"""The benchmark replays its step as a HIP graph: every replay must equal the eager result."""
import numpy as np
import pytest

from paper_2209_06979_amd import workloads as wl

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
    q8, s_q = wl.quantize_inputs_int8(a["q"]); k8, s_k = wl.quantize_inputs_int8(a["k"])
    v8, s_v = wl.quantize_inputs_int8(a["v"])
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
