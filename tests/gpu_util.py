"""Helpers for the GPU parity tests: run the HIP library through its C ABI on torch device buffers."""
from __future__ import annotations

import numpy as np

import paper_2411_06360_amd as R


class DeviceIndex:
    """Context manager around rsr_preprocess / rsr_destroy."""

    def __init__(self, A: np.ndarray, k: int):
        self.handle = R.rsr_preprocess(A, k)
        self.info = R.rsr_info(self.handle)

    def __enter__(self):
        return self

    def __exit__(self, *a):
        import torch

        torch.cuda.synchronize()
        R.rsr_destroy(self.handle)
        self.handle = None

    def matvec(self, v: np.ndarray) -> np.ndarray:
        """v: [batch][rows] (or [rows]) float32 or int8 host array -> host result (float32 / int32)."""
        import torch

        squeeze = v.ndim == 1
        v2 = np.ascontiguousarray(v[None, :] if squeeze else v)
        batch = v2.shape[0]
        dv = torch.from_numpy(v2).cuda()
        stream = torch.cuda.current_stream().cuda_stream
        if v2.dtype == np.float32:
            out = torch.full((batch, self.info.cols), float("nan"), dtype=torch.float32, device="cuda")
            R.rsr_matvec(self.handle, dv, out, batch, stream)
        elif v2.dtype == np.int8:
            out = torch.full((batch, self.info.cols), -(2**31), dtype=torch.int32, device="cuda")
            R.rsr_matvec_i8(self.handle, dv, out, batch, stream)
        else:
            raise TypeError(v2.dtype)
        torch.cuda.synchronize()
        res = out.cpu().numpy()
        return res[0] if squeeze else res


def assert_f32_close(got: np.ndarray, exact64: np.ndarray, v: np.ndarray, rel: float = 1e-5) -> float:
    """The stated bound: |gpu - oracle| <= rel * sum_i |v_i| for every output of every batch lane."""
    v2 = v[None, :] if v.ndim == 1 else v
    g2 = got[None, :] if got.ndim == 1 else got
    e2 = exact64[None, :] if exact64.ndim == 1 else exact64
    assert g2.shape == e2.shape
    assert np.isfinite(g2).all(), "non-finite output (an output was not written?)"
    bound = rel * np.abs(v2.astype(np.float64)).sum(axis=1, keepdims=True)
    err = np.abs(g2.astype(np.float64) - e2)
    worst = float((err / bound).max())
    assert worst <= 1.0, f"max error is {worst:.3g} x the allowed 1e-5*sum|v|"
    return worst
