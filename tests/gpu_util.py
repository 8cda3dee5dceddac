"""Helpers for the GPU tests: torch supplies device memory, nothing else."""
import numpy as np
import torch

from paper_2203_12533_amd import binding as pwb
from paper_2203_12533_amd import inputs as I
from parity import assert_close, rel_l2  # noqa: F401  (the criterion lives in parity.py, numpy only)


def dev_f32(a):
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).cuda()


def dev_i32(a):
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.int32)).cuda()


def dev_act(a, bf16: bool):
    """Activation tensor in the path's element type; returns (tensor, values-as-float64 the kernel will see)."""
    a32 = np.ascontiguousarray(a, dtype=np.float32)
    if bf16:
        a32 = I.round_to_bf16(a32)
        return torch.from_numpy(a32).cuda().to(torch.bfloat16).contiguous(), a32.astype(np.float64)
    return torch.from_numpy(a32).cuda(), a32.astype(np.float64)


def empty_act(shape, bf16: bool):
    return torch.empty(shape, dtype=torch.bfloat16 if bf16 else torch.float32, device="cuda")


def host(t):
    return t.detach().float().cpu().numpy().astype(np.float64)


def ptr(t):
    """Device address of a torch tensor.  torch fills tensors on its own stream and the library runs on the
    context's executor stream, so wait for torch first."""
    torch.cuda.synchronize()
    return 0 if t is None else t.data_ptr()


DT = {False: pwb.PW_F32, True: pwb.PW_BF16}
# parity bars of this build: fp32 path 1e-4, bf16 path 2e-2 (relative L2 per tensor and, at the same bar, every
# element - parity.assert_close; |d|/|ref| for the loss)
TOL = {False: 1e-4, True: 2e-2}
