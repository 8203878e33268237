"""The entry point that allocates nothing: sgprs_avgpool_fc_static keeps the pooled
vectors in an array of the library's device image instead of a caller's workspace.

Two calls in a row through the C ABI, the second with a smaller input (the array
keeps the first call's contents), each compared bit for bit with sgprs_avgpool_fc
on the same operands and, to the parity bar, with the fp64 oracle.  Sizes beyond
the array are rejected before anything is enqueued.
"""
import numpy as np
import pytest
import torch

import oracle
import paper_2406_09425_amd as S
from workloads import make_conv_weight, make_input

from gpu_util import assert_close, dev_f32, dev_nhwc

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("dtype", [S.SGPRS_F32, S.SGPRS_BF16], ids=["f32", "bf16"])
def test_static_scratch_entry_matches_workspace_entry(dtype):
    bf = dtype == S.SGPRS_BF16
    info = S.Pool(1, 8)
    total = info.info()["total_cus"]
    info.destroy()
    pool = S.Pool(1, total)
    try:
        for n in (33, 12):  # both beyond the fused one-launch path, so the scratch is written and read
            x = make_input(95, n, (n, 512, 7, 7), bf16=bf)
            w = make_conv_weight(95, n, 1, 1000, 512, 1, bf16=bf)[:, :, 0, 0]
            bias = (make_input(95, n, (1000,), tensor_id=2) * 0.1).astype(np.float32)
            ref = oracle.fc(oracle.global_avgpool(x), w, bias)
            xd = dev_nhwc(x, dtype)
            wd = torch.from_numpy(np.ascontiguousarray(w)).to(xd.dtype).cuda()
            bd = dev_f32(bias)
            ws = torch.empty(n * 512, dtype=torch.float32, device="cuda")
            want = torch.full((n, 1000), float("nan"), dtype=torch.float32, device="cuda")
            got = torch.full((n, 1000), float("nan"), dtype=torch.float32, device="cuda")
            S.sgprs_avgpool_fc(dtype, n, 49, 512, 1000, xd.data_ptr(), wd.data_ptr(), bd.data_ptr(), want.data_ptr(),
                               ws.data_ptr(), pool, 0)
            S.sgprs_avgpool_fc_static(dtype, n, 49, 512, 1000, xd.data_ptr(), wd.data_ptr(), bd.data_ptr(),
                                      got.data_ptr(), pool, 0)
            pool.sync()
            assert torch.isfinite(got).all()
            assert torch.equal(got, want), f"n={n}: static-scratch logits differ from the workspace entry point's"
            assert_close(got.cpu().numpy().astype(np.float64), ref, dtype, f"avgpool_fc_static n={n}")
        # beyond the array: rejected, nothing enqueued
        with pytest.raises(S.SgprsError) as e:
            S.sgprs_avgpool_fc_static(dtype, 65, 49, 2048, 1000, xd.data_ptr(), wd.data_ptr(), None, got.data_ptr(), pool, 0)
        assert e.value.status == -5
    finally:
        pool.destroy()
