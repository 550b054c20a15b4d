"""Helpers for the GPU parity tests: run one problem through the C ABI (via the thin
binding) and through the CPU oracle on the same seeded inputs."""
import numpy as np


def torch_dev(a: np.ndarray):
    import torch
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def run_spmm_gpu(case, variant=(0, 0), merge=0):
    """merge: the operand's merged copy forced (1: built and used wherever the call allows it), forbidden (-1) or
    left to the library (0)."""
    import torch
    from paper_2209_06979_amd import binding as mc
    bits = mc.LHS_BITS[case["prec"]]
    o = mc.get_thread_options()
    o.spmm_merge = merge
    mc.set_thread_options(o)
    A = mc.SparseMatrix(case["M"], case["K"], case["V"], case["row_ptr"], case["col_idx"], case["values"], bits)
    mc.set_spmm_variant(*variant)
    try:
        B = torch_dev(case["B"])
        # poison the output so that unwritten elements are caught
        out = torch.full((case["M"], case["N"]), -7777777, dtype=torch.int32, device="cuda")
        C = mc.spmm(A, B, case["prec"], out=out, lhs_unsigned=case.get("lhs_unsigned", False),
                    rhs_unsigned=case.get("rhs_unsigned", False))
        torch.cuda.synchronize()
        return C.cpu().numpy()
    finally:
        mc.set_spmm_variant(0, 0)
        o = mc.get_thread_options()
        o.spmm_merge = 0
        mc.set_thread_options(o)
        A.close()


def run_spmm_oracle(case):
    import oracle
    return oracle.spmm(case["M"], case["K"], case["V"], case["row_ptr"], case["col_idx"], case["values"],
                       case["B"], case["prec"], lhs_unsigned=case.get("lhs_unsigned", False),
                       rhs_unsigned=case.get("rhs_unsigned", False))


def run_sddmm_gpu(case, waves=-1):
    import torch
    from paper_2209_06979_amd import binding as mc
    mask = mc.SparseMatrix(case["M"], case["Nc"], case["V"], case["row_ptr"], case["col_idx"])
    mc.set_sddmm_variant(waves)
    try:
        out = torch.full((mask.nvec * mask.V,), -7777777, dtype=torch.int32, device="cuda")
        S = mc.sddmm(torch_dev(case["Q"]), torch_dev(case["Kmat"]), mask, case["prec"], out=out,
                     lhs_unsigned=case.get("lhs_unsigned", False), rhs_unsigned=case.get("rhs_unsigned", False))
        torch.cuda.synchronize()
        return S.cpu().numpy()
    finally:
        mc.set_sddmm_variant(-1)
        mask.close()


def run_sddmm_oracle(case):
    import oracle
    return oracle.sddmm(case["M"], case["Nc"], case["V"], case["row_ptr"], case["col_idx"], case["Q"],
                        case["Kmat"], case["prec"], lhs_unsigned=case.get("lhs_unsigned", False),
                        rhs_unsigned=case.get("rhs_unsigned", False))
