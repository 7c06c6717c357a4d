"""Host <-> device plumbing for the GPU parity tests (no arithmetic of the method)."""
import numpy as np
import torch

from paper_1910_00932_amd import binding as B

TDT = {"f32": torch.float32, "bf16": torch.bfloat16}
CDT = {"f32": B.TSM_F32, "bf16": B.TSM_BF16}
CLAY = {"ntchw": B.TSM_NTCHW, "nthwc": B.TSM_NTHWC}
TOL = {"f32": 1e-4, "bf16": 2e-2}   # relative L2 against the fp64 oracle (spec tolerances)


def to_dev(a, dtype, layout="ntchw"):
    """numpy [N,T,C,H,W] -> contiguous CUDA tensor in the requested memory order."""
    t = torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32))
    if layout == "nthwc":
        t = t.permute(0, 1, 3, 4, 2).contiguous()
    return t.to(TDT[dtype]).cuda()


def from_dev(t, layout="ntchw"):
    """CUDA tensor written in `layout` (viewed as [N,T,C,H,W] or [N,T,H,W,C]) -> float64 numpy [N,T,C,H,W]."""
    a = t.float().cpu().numpy().astype(np.float64)
    if layout == "nthwc":
        a = np.transpose(a, (0, 1, 4, 2, 3))
    return np.ascontiguousarray(a)


def empty_act(shape_ntchw, dtype, layout):
    N, T, C, H, W = shape_ntchw
    shp = (N, T, C, H, W) if layout == "ntchw" else (N, T, H, W, C)
    return torch.empty(shp, dtype=TDT[dtype], device="cuda")


def dev_vec(a, dtype="f32"):
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).to(TDT[dtype]).cuda()


def workspace(nbytes):
    return torch.empty(max(int(nbytes), 16), dtype=torch.uint8, device="cuda")
