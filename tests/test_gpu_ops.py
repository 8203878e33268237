"""GPU parity of the per-operator entry points against the fp64 oracle.

Every case calls libsgprs through its C ABI (via the ctypes binding) on seeded
inputs and compares element by element with the oracle:
max|gpu - ref| <= 1e-4 * max|ref| for fp32 and <= 2e-2 * max|ref| for
bf16-storage / fp32-accumulate (the oracle is fed the bf16-rounded values).
"""
import numpy as np
import pytest
import torch

import oracle
import paper_2406_09425_amd as S
from workloads import BN_EPS, make_bn, make_conv_weight, make_input, round_to_bf16

from gpu_util import (DevConv, assert_close, dev_empty, dev_f32, dev_nhwc, host_nchw, rel_err)

pytestmark = pytest.mark.gpu
DTYPES = [S.SGPRS_F32, S.SGPRS_BF16]
DT_ID = {S.SGPRS_F32: "f32", S.SGPRS_BF16: "bf16"}
PART_SIZES = (8, 64, "full")   # keys of the `pools` fixture


@pytest.fixture(scope="module")
def pools():
    info = S.Pool(1, 8)
    total = info.info()["total_cus"]
    info.destroy()
    ps = {c: S.Pool(1, c) for c in (8, 64, total)}
    ps["full"] = ps[total]
    yield ps
    for p in set(ps.values()):
        p.destroy()


def conv_case(dtype, n, h, w, cin, cout, k, stride, pad, relu, with_res, seed, pool, cus, absx=False):
    bf = dtype == S.SGPRS_BF16
    x = make_input(90, seed, (n, cin, h, w), "absnormal" if absx else "normal", bf16=bf)
    wt = make_conv_weight(90, seed, 1, cout, cin, k, bf16=bf)
    g, b, m, v = make_bn(90, seed, 2, cout)
    ref = oracle.bn(oracle.conv2d(x, wt, stride, pad), g, b, m, v, BN_EPS)
    res = None
    if with_res:
        res = make_input(90, seed, ref.shape, bf16=bf, tensor_id=7)
        ref = oracle.add(ref, res)
    if relu:
        ref = oracle.relu(ref)
    d = S.ConvDesc(n, h, w, cin, cout, k, k, stride, pad, dtype, int(relu))
    dc = DevConv(d, wt, g, b, m, v, BN_EPS)
    xd = dev_nhwc(x, dtype)
    rd = dev_nhwc(res, dtype) if with_res else None
    yd = dev_empty((n, ref.shape[2], ref.shape[3], cout), dtype)
    keep = dc.run(xd, yd, rd, pool, 0, cus)
    pool.sync()
    del keep
    return host_nchw(yd), ref


IGEMM_SHAPES = [
    # n, h, w, cin, cout, k, stride, pad   (ResNet18 shapes at batch 1 + ragged ones)
    (1, 56, 56, 64, 64, 3, 1, 1),
    (1, 56, 56, 64, 128, 3, 2, 1),
    (1, 56, 56, 64, 128, 1, 2, 0),
    (1, 28, 28, 128, 128, 3, 1, 1),
    (1, 14, 14, 256, 256, 3, 1, 1),
    (1, 14, 14, 256, 512, 3, 2, 1),
    (1, 7, 7, 512, 512, 3, 1, 1),
    (1, 14, 14, 256, 512, 1, 2, 0),
    (3, 9, 13, 64, 64, 3, 1, 1),     # ragged M = 351
    (2, 11, 7, 128, 192, 3, 2, 1),   # odd sizes, cout 192 = 3 x 64
    (5, 5, 5, 64, 64, 1, 1, 0),      # 1x1 stride 1
]


@pytest.mark.parametrize("dtype", DTYPES, ids=DT_ID.get)
@pytest.mark.parametrize("shape", IGEMM_SHAPES, ids=lambda s: "x".join(map(str, s)))
def test_conv_igemm_parity(pools, dtype, shape):
    for i, cus in enumerate((8, "full")):
        pool = pools[cus]
        ncus = pool.partition_cus(0)
        got, ref = conv_case(dtype, *shape, relu=True, with_res=True, seed=11 + i, pool=pool, cus=ncus)
        e = assert_close(got, ref, dtype, f"conv {shape} on {ncus} CUs")
        if dtype == S.SGPRS_F32:
            assert e < 2e-5, e  # fp32 accumulation error should sit far inside the tolerance


@pytest.mark.parametrize("dtype", DTYPES, ids=DT_ID.get)
def test_conv_flags_no_relu_no_residual(pools, dtype):
    pool = pools["full"]
    got, ref = conv_case(dtype, 2, 14, 14, 128, 128, 3, 1, 1, relu=False, with_res=False, seed=21, pool=pool,
                         cus=pool.partition_cus(0))
    assert_close(got, ref, dtype, "conv without relu/residual")
    assert np.min(ref) < 0 and np.min(got) < 0


@pytest.mark.parametrize("dtype", DTYPES, ids=DT_ID.get)
@pytest.mark.parametrize("shape", [(1, 224, 224), (2, 50, 70), (1, 30, 33)], ids=str)
def test_conv_stem_parity(pools, dtype, shape):
    n, h, w = shape
    for cus in (8, "full"):
        pool = pools[cus]
        got, ref = conv_case(dtype, n, h, w, 3, 64, 7, 2, 3, relu=True, with_res=False, seed=31, pool=pool,
                             cus=pool.partition_cus(0))
        assert_close(got, ref, dtype, f"stem {shape}")


@pytest.mark.parametrize("dtype", DTYPES, ids=DT_ID.get)
def test_conv_is_deterministic_and_mask_independent(pools, dtype):
    shape = (1, 14, 14, 256, 256, 3, 1, 1)
    outs = {}
    for cus in (8, 64, "full"):
        pool = pools[cus]
        a, ref = conv_case(dtype, *shape, relu=True, with_res=True, seed=41, pool=pool, cus=pool.partition_cus(0))
        b, _ = conv_case(dtype, *shape, relu=True, with_res=True, seed=41, pool=pool, cus=pool.partition_cus(0))
        assert np.array_equal(a, b), "two runs of the same launch differ"
        assert_close(a, ref, dtype)
        outs[cus] = a
    # masks change the split-K factor at most: results agree to rounding
    assert rel_err(outs[8], outs["full"]) <= (1e-5 if dtype == S.SGPRS_F32 else 1e-2)


def test_pack_unpack_roundtrip_on_device_copy():
    d = S.ConvDesc(1, 8, 8, 64, 64, 3, 3, 1, 1, S.SGPRS_BF16, 0)
    w = make_conv_weight(90, 0, 3, 64, 64, 3, bf16=True)
    assert np.array_equal(S.sgprs_unpack_conv_weights(d, S.sgprs_pack_conv_weights(d, w)), w)


@pytest.mark.parametrize("dtype", DTYPES, ids=DT_ID.get)
@pytest.mark.parametrize("shape", [(1, 64, 112, 112), (2, 16, 9, 11), (3, 64, 7, 8)], ids=str)
def test_maxpool_parity_exact(pools, dtype, shape):
    n, c, h, w = shape
    x = make_input(91, 0, shape, bf16=dtype == S.SGPRS_BF16)  # has negatives: padding must not win
    ref = oracle.maxpool2d(x)
    xd = dev_nhwc(x, dtype)
    for cus in PART_SIZES:   # the partition sizes the per-operator sweep times
        yd = dev_empty((n, ref.shape[2], ref.shape[3], c), dtype)
        S.sgprs_maxpool2d(dtype, n, h, w, c, xd.data_ptr(), yd.data_ptr(), pools[cus], 0)
        pools[cus].sync()
        assert np.array_equal(host_nchw(yd), ref), cus  # selection only: bit exact


@pytest.mark.parametrize("dtype", DTYPES, ids=DT_ID.get)
def test_bn_relu_parity(pools, dtype):
    shape = (1, 128, 28, 28)
    x = make_input(92, 0, shape, bf16=dtype == S.SGPRS_BF16)
    g, b, m, v = make_bn(92, 0, 1, 128)
    ref = oracle.relu(oracle.bn(x, g, b, m, v, BN_EPS))
    sc, sh = S.sgprs_fold_bn(g, b, m, v, BN_EPS)
    xd, scd, shd = dev_nhwc(x, dtype), dev_f32(sc), dev_f32(sh)
    for cus in PART_SIZES:
        yd = dev_empty((1, 28, 28, 128), dtype)
        S.sgprs_bn_relu(dtype, 28 * 28, 128, xd.data_ptr(), scd.data_ptr(), shd.data_ptr(), yd.data_ptr(),
                        pools[cus], 0)
        pools[cus].sync()
        assert_close(host_nchw(yd), ref, dtype, f"bn_relu on {cus} CUs")


@pytest.mark.parametrize("dtype", DTYPES, ids=DT_ID.get)
@pytest.mark.parametrize("relu", [False, True])
def test_add_parity(pools, dtype, relu):
    shape = (1, 512, 7, 7)
    bf = dtype == S.SGPRS_BF16
    a, b = make_input(93, 0, shape, bf16=bf), make_input(93, 1, shape, bf16=bf)
    ref = oracle.add(a, b)
    if relu:
        ref = oracle.relu(ref)
    ad, bd = dev_nhwc(a, dtype), dev_nhwc(b, dtype)
    for cus in PART_SIZES:
        yd = dev_empty((1, 7, 7, 512), dtype)
        S.sgprs_add_relu(dtype, a.size, ad.data_ptr(), bd.data_ptr(), yd.data_ptr(), relu, pools[cus], 0)
        pools[cus].sync()
        assert_close(host_nchw(yd), ref, dtype, f"add on {cus} CUs")
        if not relu:
            assert np.min(host_nchw(yd)) < 0


@pytest.mark.parametrize("dtype", DTYPES, ids=DT_ID.get)
@pytest.mark.parametrize("n", [1, 5, 33, 515])
def test_avgpool_fc_parity(pools, dtype, n):
    """1 and 5 images: one launch; 33: two launches, in bf16 the FC on the matrix cores; 515 (ragged
    against the 4 images per workgroup of the streaming avg-pool and the 32 of the FC tiles): the
    many-image avg-pool kernel."""
    bf = dtype == S.SGPRS_BF16
    x = make_input(94, n, (n, 512, 7, 7), bf16=bf)
    w = make_conv_weight(94, n, 1, 1000, 512, 1, bf16=bf)[:, :, 0, 0]
    bias = (make_input(94, n, (1000,), tensor_id=2) * 0.1).astype(np.float32)
    ref = oracle.fc(oracle.global_avgpool(x), w, bias)
    xd = dev_nhwc(x, dtype)
    wd = torch.from_numpy(np.ascontiguousarray(w)).to(xd.dtype).cuda()
    bd = dev_f32(bias)
    ws = torch.empty(n * 512, dtype=torch.float32, device="cuda")
    for cus in PART_SIZES:
        yd = torch.full((n, 1000), float("nan"), dtype=torch.float32, device="cuda")
        S.sgprs_avgpool_fc(dtype, n, 49, 512, 1000, xd.data_ptr(), wd.data_ptr(), bd.data_ptr(), yd.data_ptr(),
                           ws.data_ptr(), pools[cus], 0)
        pools[cus].sync()
        got = yd.cpu().numpy().astype(np.float64)
        assert_close(got, ref, dtype, f"avgpool_fc on {cus} CUs")
    # the average pool alone: against the oracle, and the same bits as the two-kernel path's workspace
    pd = torch.full((n, 512), float("nan"), dtype=torch.float32, device="cuda")
    S.sgprs_global_avgpool(dtype, n, 49, 512, xd.data_ptr(), pd.data_ptr(), pools["full"], 0)
    pools["full"].sync()
    assert rel_err(pd.cpu().numpy().astype(np.float64), oracle.global_avgpool(x).reshape(n, 512)) < (1e-6 if not bf else 1e-6)
    if n > 8:
        assert torch.equal(pd.flatten(), ws)
    # without bias
    S.sgprs_avgpool_fc(dtype, n, 49, 512, 1000, xd.data_ptr(), wd.data_ptr(), None, yd.data_ptr(),
                       ws.data_ptr(), pools["full"], 0)
    pools["full"].sync()
    assert_close(yd.cpu().numpy().astype(np.float64), ref - bias, dtype, "avgpool_fc no bias")


@pytest.mark.parametrize("dtype", DTYPES, ids=DT_ID.get)
@pytest.mark.parametrize("cin,hw", [(512, 49), (1024, 21), (512, 3)])
def test_avgpool_fc_one_launch_equals_two(pools, dtype, cin, hw):
    """Up to 8 images take the single fused launch, more take avg-pool then FC: the same bits."""
    bf = dtype == S.SGPRS_BF16
    x = make_input(96, cin + hw, (9, cin, hw, 1), bf16=bf)
    w = make_conv_weight(96, cin + hw, 1, 1000, cin, 1, bf16=bf)[:, :, 0, 0]
    bias = make_input(96, cin + hw, (1000,), tensor_id=2).astype(np.float32)
    xd = dev_nhwc(x, dtype).reshape(9, hw, cin)
    wd = torch.from_numpy(np.ascontiguousarray(w)).to(xd.dtype).cuda()
    bd = dev_f32(bias)
    ws = torch.empty(9 * cin, dtype=torch.float32, device="cuda")
    two = torch.full((9, 1000), float("nan"), dtype=torch.float32, device="cuda")
    one = torch.full((8, 1000), float("nan"), dtype=torch.float32, device="cuda")
    S.sgprs_avgpool_fc(dtype, 9, hw, cin, 1000, xd.data_ptr(), wd.data_ptr(), bd.data_ptr(), two.data_ptr(),
                       ws.data_ptr(), pools["full"], 0)
    S.sgprs_avgpool_fc(dtype, 8, hw, cin, 1000, xd.data_ptr(), wd.data_ptr(), bd.data_ptr(), one.data_ptr(),
                       ws.data_ptr(), pools["full"], 0)
    pools["full"].sync()
    assert torch.isfinite(one).all()
    assert torch.equal(one, two[:8])
    ref = oracle.fc(oracle.global_avgpool(x), w, bias)
    assert_close(two.cpu().numpy().astype(np.float64), ref, dtype, "two launches")
    assert_close(one.cpu().numpy().astype(np.float64), ref[:8], dtype, "one launch")


def test_error_paths_enqueue_nothing(pools):
    pool = pools["full"]
    x = torch.zeros(64, device="cuda")
    with pytest.raises(S.SgprsError) as e:
        S.sgprs_maxpool2d(S.SGPRS_F32, 1, 4, 4, 4, x.data_ptr(), x.data_ptr(), pool, 0)  # aliasing
    assert e.value.status == -1
    with pytest.raises(S.SgprsError):
        S.sgprs_maxpool2d(S.SGPRS_F32, 1, 4, 4, 4, x.data_ptr(), x.data_ptr() + 256, pool, 3)  # bad partition
    with pytest.raises(S.SgprsError) as e:
        S.sgprs_conv2d_workspace(S.ConvDesc(1, 8, 8, 48, 64, 3, 3, 1, 1, 0, 0), 256)  # cin % 32
    assert e.value.status == -5
    with pytest.raises(S.SgprsError):
        S.sgprs_add_relu(S.SGPRS_F32, 12, x.data_ptr(), x.data_ptr(), x.data_ptr(), False, pool, 0)


# ---- the LDS-patch 3x3 kernel, every tile variant forced in turn ----------------
PATCH_SHAPES = [
    # n, h, w, cin, cout: tiles straddle image boundaries, ragged last tile, several channel blocks/chunks
    (5, 14, 14, 64, 64),
    (3, 28, 28, 64, 128),
    (9, 7, 7, 128, 64),
    (2, 56, 56, 64, 64),
    (7, 9, 11, 128, 128),
]


@pytest.mark.parametrize("variant", range(5))
@pytest.mark.parametrize("shape", PATCH_SHAPES, ids=lambda s: "x".join(map(str, s)))
def test_conv3x3_patch_variants_parity(pools, variant, shape):
    n, h, w, cin, cout = shape
    pool = pools["full"]
    dtype = S.SGPRS_BF16
    try:
        for splits in (1, 2):
            S.sgprs_conv_tuning_override(1, variant, splits)
            for with_res in (True, False):
                got, ref = conv_case(dtype, n, h, w, cin, cout, 3, 1, 1, relu=with_res, with_res=with_res,
                                     seed=50 + variant, pool=pool, cus=pool.partition_cus(0))
                assert_close(got, ref, dtype, f"patch variant {variant} splits {splits} {shape}")
    finally:
        S.sgprs_conv_tuning_override(-1, 0, 1)


S2_SHAPES = [
    # n, h, w, cin, cout: several row tiles and image borders inside a tile, ragged last tile, 2-8 channel blocks
    (9, 14, 14, 64, 128),
    (3, 28, 28, 64, 128),
    (2, 56, 56, 64, 128),
    (20, 14, 14, 256, 512),
    (5, 10, 6, 128, 192),
    (7, 8, 12, 192, 64),
]


@pytest.mark.parametrize("variant", range(2))
@pytest.mark.parametrize("shape", S2_SHAPES, ids=lambda s: "x".join(map(str, s)))
def test_conv3x3s2_patch_variants_parity(pools, variant, shape):
    """The stride-2 patch kernel alone (no shortcut), both tile shapes, forced; shapes it
    declines fall back to the implicit GEMM and must match just the same."""
    n, h, w, cin, cout = shape
    pool = pools["full"]
    try:
        S.sgprs_conv_tuning_override(3, variant, 1)
        for relu in (True, False):
            got, ref = conv_case(S.SGPRS_BF16, n, h, w, cin, cout, 3, 2, 1, relu=relu, with_res=False, seed=80 + variant,
                                 pool=pool, cus=pool.partition_cus(0))
            assert_close(got, ref, S.SGPRS_BF16, f"stride-2 patch variant {variant} relu {relu} {shape}")
        # with a residual the planner must leave this kernel out (it has no residual input)
        got, ref = conv_case(S.SGPRS_BF16, n, h, w, cin, cout, 3, 2, 1, relu=True, with_res=True, seed=83, pool=pool,
                             cus=pool.partition_cus(0))
        assert_close(got, ref, S.SGPRS_BF16, f"stride-2 with residual {shape}")
    finally:
        S.sgprs_conv_tuning_override(-1, 0, 1)


# ---- the row-streaming 3x3 kernel of the 64 -> 64 layers -----------------------------
ROWS_CASES = [
    # batch, image height, partition, rows per stream and job the planner picks: one job per CU, jobs that cross
    # the middle of an image (7, 14) or cover whole images (28), several jobs per workgroup (batch 16 on 8 CUs),
    # and a 28-row image (two jobs of 2 x 7 rows)
    (2, 56, 8, 7), (4, 56, 8, 14), (8, 56, 8, 28), (16, 56, 64, 7), (16, 56, 8, 28), (4, 28, 8, 7),
]


@pytest.mark.parametrize("case", ROWS_CASES, ids=lambda c: "n%d-h%d-%dcu-S%d" % c)
def test_conv3x3_rows_parity(pools, case):
    """56-pixel rows, 64 -> 64 channels in bf16 on partitions where every CU gets whole jobs: the planner
    picks the row-streaming kernel; element by element against the oracle with and without residual
    and ReLU, and against the LDS-patch kernel (tuning override 5) on the same inputs."""
    n, h, cus, rows = case
    pool = pools[cus]
    dtype = S.SGPRS_BF16
    d = S.ConvDesc(n, h, 56, 64, 64, 3, 3, 1, 1, dtype, 1)
    assert S.sgprs_conv2d_plan(d, cus, True) == (3, rows)
    assert S.sgprs_conv2d_plan(d, cus, False) == (3, rows)
    for with_res, relu in ((True, True), (False, True), (False, False), (True, False)):
        got, ref = conv_case(dtype, n, h, 56, 64, 64, 3, 1, 1, relu=relu, with_res=with_res, seed=70 + n, pool=pool, cus=cus)
        assert_close(got, ref, dtype, f"rows kernel {case} res {with_res} relu {relu}")
        try:
            S.sgprs_conv_tuning_override(5, 0, 1)
            assert S.sgprs_conv2d_plan(d, cus, with_res)[0] == 1
            other, _ = conv_case(dtype, n, h, 56, 64, 64, 3, 1, 1, relu=relu, with_res=with_res, seed=70 + n, pool=pool, cus=cus)
        finally:
            S.sgprs_conv_tuning_override(-1, 0, 1)
        # the same bf16 inputs, fp32 sums in another order: at most a bf16 step apart
        assert np.all(np.abs(got - other) <= np.maximum(np.abs(other), 1e-2) * 2.0 ** -7)


def test_masks_that_leave_a_die_empty_are_rejected_and_odd_masks_work():
    """Mask bit i selects a CU of die i % 8.  A mask without a CU on some die is refused with a
    clear error; a mask of 9 CUs (two on die 0) is fine, and the forced patch kernels on it (a grid
    of 8 workgroups walking the padded, die-keyed work-item space) match the oracle."""
    n_xcd = S.Pool(1, 8).info()["n_xcd"]
    for bits in ((1 << 1) - 1, (1 << 4) - 1, (1 << 7) - 1):
        mask = np.zeros((1, 8), dtype=np.uint32)
        mask[0, 0] = bits
        if n_xcd > 1:
            with pytest.raises(S.SgprsError) as e:
                S.Pool(1, 0, masks=mask)
            assert e.value.status == -1 and "die" in str(e.value)
    mask = np.zeros((1, 8), dtype=np.uint32)
    mask[0, 0] = (1 << 9) - 1
    pool = S.Pool(1, 0, masks=mask)
    assert pool.partition_cus(0) == 9
    dtype = S.SGPRS_BF16
    try:
        for variant, shape in ((0, (1, 28, 28, 128, 128)), (1, (3, 14, 14, 64, 256)), (3, (2, 14, 14, 64, 512)),
                               (4, (2, 28, 28, 64, 128))):
            S.sgprs_conv_tuning_override(1, variant, 1)
            n, h, w, cin, cout = shape
            got, ref = conv_case(dtype, n, h, w, cin, cout, 3, 1, 1, relu=True, with_res=True, seed=120,
                                 pool=pool, cus=9)
            assert_close(got, ref, dtype, f"patch variant {variant} {shape} on 9 CUs")
        for variant, shape in ((0, (3, 28, 28, 64, 128)), (1, (9, 14, 14, 64, 512))):
            S.sgprs_conv_tuning_override(3, variant, 1)
            n, h, w, cin, cout = shape
            got, ref = conv_case(dtype, n, h, w, cin, cout, 3, 2, 1, relu=True, with_res=False, seed=130,
                                 pool=pool, cus=9)
            assert_close(got, ref, dtype, f"stride-2 patch variant {variant} {shape} on 9 CUs")
    finally:
        S.sgprs_conv_tuning_override(-1, 0, 1)
        pool.destroy()


def test_conv_planner_choices_agree(pools):
    """Automatic choice, implicit GEMM only and a forced patch variant give the
    same result to bf16 rounding on a batch large enough for the patch kernel."""
    pool = pools["full"]
    shape = (64, 14, 14, 64, 64, 3, 1, 1)
    outs = []
    try:
        for kind in (-1, 0, 1):
            S.sgprs_conv_tuning_override(kind, 3, 1)
            got, ref = conv_case(S.SGPRS_BF16, *shape, relu=True, with_res=True, seed=61, pool=pool,
                                 cus=pool.partition_cus(0))
            assert_close(got, ref, S.SGPRS_BF16, f"kind {kind}")
            outs.append(got)
    finally:
        S.sgprs_conv_tuning_override(-1, 0, 1)
    assert rel_err(outs[0], outs[1]) < 1e-2 and rel_err(outs[2], outs[1]) < 1e-2


@pytest.mark.parametrize("dtype", [S.SGPRS_F32, S.SGPRS_BF16], ids=["f32", "bf16"])
def test_igemm_forced_tiles_and_splits_parity(pools, dtype):
    """Every implicit-GEMM tile shape, with the planner's split factor and with
    forced ones, on a stride-2 3x3 and a 1x1 layer (ragged last row tile)."""
    pool = pools["full"]
    shapes = [(3, 14, 14, 64, 128, 3, 2, 1), (3, 14, 14, 64, 128, 1, 2, 0)]
    try:
        for variant in range(4):
            for splits in (0, 1, 2):
                for shape in shapes:
                    S.sgprs_conv_tuning_override(2, variant, splits)
                    got, ref = conv_case(dtype, *shape, relu=True, with_res=True, seed=70 + variant, pool=pool,
                                         cus=pool.partition_cus(0))
                    assert_close(got, ref, dtype, f"igemm variant {variant} splits {splits} {shape}")
    finally:
        S.sgprs_conv_tuning_override(-1, 0, 1)
