"""Helpers for the GPU parity tests: host<->device marshalling and tolerances.

torch is used for device memory only (allocation, copies, layout permutes on
the host side of the test); every operator under test runs in libsgprs.
"""
from __future__ import annotations

import numpy as np
import torch

import paper_2406_09425_amd as S

# max|gpu - ref| <= TOL * max|ref| per compared tensor
TOL = {S.SGPRS_F32: 1e-4, S.SGPRS_BF16: 2e-2}
TORCH_DT = {S.SGPRS_F32: torch.float32, S.SGPRS_BF16: torch.bfloat16}


def dev_nhwc(x_nchw: np.ndarray, dtype: int) -> torch.Tensor:
    """Logical NCHW fp32 host array -> contiguous NHWC device tensor in dtype."""
    t = torch.from_numpy(np.ascontiguousarray(np.transpose(x_nchw, (0, 2, 3, 1)), dtype=np.float32))
    return t.to(TORCH_DT[dtype]).cuda().contiguous()


def dev_f32(a: np.ndarray) -> torch.Tensor:
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).cuda()


def dev_bytes(a: np.ndarray) -> torch.Tensor:
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.uint8)).cuda()


def dev_empty(shape, dtype: int) -> torch.Tensor:
    # filled with a sentinel so that unwritten elements are caught
    return torch.full(tuple(shape), float("nan"), dtype=TORCH_DT[dtype], device="cuda")


def host_nchw(t_nhwc: torch.Tensor) -> np.ndarray:
    return np.transpose(t_nhwc.float().cpu().numpy().astype(np.float64), (0, 3, 1, 2))


def rel_err(gpu: np.ndarray, ref: np.ndarray) -> float:
    assert gpu.shape == ref.shape, (gpu.shape, ref.shape)
    assert np.all(np.isfinite(gpu)), "non-finite (or unwritten) GPU output"
    scale = float(np.max(np.abs(ref)))
    return float(np.max(np.abs(gpu - ref))) / (scale if scale > 0 else 1.0)


def assert_close(gpu: np.ndarray, ref: np.ndarray, dtype: int, what: str = "") -> float:
    e = rel_err(gpu, ref)
    assert e <= TOL[dtype], f"{what}: max|err|/max|ref| = {e:.3e} > {TOL[dtype]:.0e}"
    return e


class DevConv:
    """Device-side operands of one convolution: packed weight, scale, shift."""

    def __init__(self, desc: S.ConvDesc, w_oihw, gamma, beta, mean, var, eps):
        self.desc = desc
        self.w = dev_bytes(S.sgprs_pack_conv_weights(desc, w_oihw))
        sc, sh = S.sgprs_fold_bn(gamma, beta, mean, var, eps)
        self.scale, self.shift = dev_f32(sc), dev_f32(sh)

    def run(self, x: torch.Tensor, y: torch.Tensor, residual, pool, partition: int, cus: int):
        ws_bytes = S.sgprs_conv2d_workspace(self.desc, cus)
        ws = torch.empty(max(ws_bytes, 16), dtype=torch.uint8, device="cuda")
        S.sgprs_conv2d(self.desc, x.data_ptr(), self.w.data_ptr(), self.scale.data_ptr(), self.shift.data_ptr(),
                       residual.data_ptr() if residual is not None else None, y.data_ptr(), ws.data_ptr(),
                       ws_bytes, pool, partition)
        return ws  # keep alive until synced
