"""Helpers for the GPU parity tests: upload a problem, call the C ABI through the binding."""
import numpy as np


def device_problem(p, device="cuda:0"):
    import torch
    import paper_2602_01027_amd as S

    L, s2, s3, s4, index = S.sfmp_pack(p.codes, p.bitmap)
    S.sfmp_layout_set_quant(L, p.group, p.scale_format)
    dp = S.upload_packed(L, s2, s3, s4, index, p.scales, p.zeros, p.bitmap, device)
    cp = torch.from_numpy(p.col_perm).to(device) if p.col_perm is not None else None
    rp = torch.from_numpy(p.row_perm).to(device) if p.row_perm is not None else None
    return dp, cp, rp


def make_workspace(layout, M, device="cuda:0"):
    import torch
    import paper_2602_01027_amd as S

    nbytes = S.sfmp_gemm_workspace(layout, M)
    ws = torch.empty(nbytes, dtype=torch.uint8, device=device)
    S.sfmp_workspace_init(ws)
    return ws


def run_gemm(p, dp=None, cp=None, rp=None, ws=None, X=None, device="cuda:0"):
    """Y (numpy fp16 [M, N]) of the HIP path for problem p."""
    import torch
    import paper_2602_01027_amd as S

    if dp is None:
        dp, cp, rp = device_problem(p, device)
    Xh = p.X if X is None else X
    M = Xh.shape[0]
    Xd = torch.from_numpy(np.ascontiguousarray(Xh)).to(device)
    if ws is None:
        ws = make_workspace(dp.layout, M, device)
    Y = torch.full((M, p.N), float("nan"), dtype=torch.float16, device=device)
    S.sfmp_gemm(Xd, cp, dp.layout, dp.s2, dp.s3, dp.s4, dp.index, dp.scales, dp.zeros, dp.bitmap, rp, Y, ws)
    torch.cuda.synchronize()
    return Y.cpu().numpy()
