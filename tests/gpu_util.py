"""Helpers shared by the GPU parity tests (device plumbing only)."""
import numpy as np


def torch_dtype(dtype: str):
    import torch
    return torch.float16 if dtype == "f16" else torch.bfloat16


def to_dev(bits_u16: np.ndarray, dtype: str):
    """uint16 bit patterns -> CUDA tensor of the 16-bit float dtype (bit-preserving)."""
    import torch
    t = torch.from_numpy(np.ascontiguousarray(bits_u16).view(np.int16).copy())
    return t.view(torch_dtype(dtype)).cuda()


def to_bits(t) -> np.ndarray:
    """CUDA 16-bit float tensor -> uint16 bit patterns on the host."""
    import torch
    return t.detach().contiguous().view(torch.int16).cpu().numpy().view(np.uint16)


class DeviceCase:
    """A synthetic case uploaded to the GPU, packed with the library's own packer."""

    def __init__(self, lutq, case):
        import torch
        self.case = case
        self.packed_host = lutq.lutq_pack(case.Q, case.bits, case.group_size)
        self.packed = torch.from_numpy(self.packed_host.copy()).cuda()
        self.X = to_dev(case.X, case.dtype)
        self.S = to_dev(case.S, case.dtype)
        self.T = to_dev(case.T, case.dtype)
        self.ws = lutq.new_workspace(case.N, case.K, case.bits, case.group_size)

    def matmul(self, lutq, plan=None, X=None):
        import torch
        X = self.X if X is None else X
        Y = torch.full((X.shape[0], self.case.N), float("nan"), dtype=X.dtype, device="cuda")
        lutq.lutq_matmul(X, self.packed, self.S, self.T, self.case.bits, self.case.group_size, Y, self.ws, plan=plan)
        torch.cuda.synchronize()
        return Y


def ulp16(x: np.ndarray, dtype: str) -> np.ndarray:
    """Spacing of the 16-bit format at |x| (float64)."""
    mbits, emin = (10, -14) if dtype == "f16" else (7, -126)
    ax = np.abs(x)
    e = np.floor(np.log2(np.maximum(ax, 2.0 ** emin)))
    return 2.0 ** (np.maximum(e, emin) - mbits)
