"""GPU parity of the stage/task entry points against the fp64 oracle on the
benchmark configurations: the single layer1 block (fp32), the full ResNet18 at
batch 1 (fp32, six stages), eight concurrent bf16 instances on an 8 x 32-CU
pool, and the batch-64 bf16 forward."""
import numpy as np
import pytest
import torch

import oracle
import paper_2406_09425_amd as S
from workloads import BN_EPS, STAGE_IO, make_bn, make_conv_weight, make_input, make_resnet18_params

from gpu_util import DevConv, TOL, assert_close, dev_empty, dev_nhwc, host_nchw, rel_err

pytestmark = pytest.mark.gpu
DT_ID = {S.SGPRS_F32: "f32", S.SGPRS_BF16: "bf16"}


@pytest.fixture(scope="module")
def full_pool():
    total = S.Pool(1, 8).info()["total_cus"]
    p = S.Pool(1, total)
    yield p
    p.destroy()


def stage_shape(j, n, out=True):
    c, h, w = STAGE_IO[j][1 if out else 0]
    return (n, h, w, c)


def run_stages_chained(task, pool, part, x_dev, n):
    """Each stage through sgprs_stage_run, chained on one partition."""
    outs, cur = [], x_dev
    for j in range(6):
        if j == 5:
            o = torch.full((n, 1000), float("nan"), dtype=torch.float32, device="cuda")
        else:
            o = dev_empty(stage_shape(j, n), task.dtype)
        task.stage_run(j, n, cur.data_ptr(), o.data_ptr(), pool, part)
        outs.append(o)
        cur = o
    pool.sync(part)
    return outs


def host_stage(t, j):
    return t.cpu().numpy().astype(np.float64) if j == 5 else host_nchw(t)


def check_argmax(logits_gpu, logits_ref, err, what):
    """Top-1 must agree; a disagreement is reported with the oracle's margin."""
    for i in range(logits_ref.shape[0]):
        a, b = int(np.argmax(logits_gpu[i])), int(np.argmax(logits_ref[i]))
        if a != b:
            top2 = np.sort(logits_ref[i])[-2:]
            margin = (top2[1] - top2[0]) / np.max(np.abs(logits_ref[i]))
            pytest.fail(f"{what}: argmax differs for image {i}: gpu {a} oracle {b}; oracle top-2 margin "
                        f"{margin:.3e} of max|ref|, measured error {err:.3e}")


# ------------------------------------------------------------- config 0
def test_config0_layer1_basic_block_fp32(full_pool):
    dtype = S.SGPRS_F32
    x = make_input(0, 0, (1, 64, 56, 56), "absnormal")
    convs = []
    for i in range(2):
        w = make_conv_weight(0, 0, 1 + 5 * i, 64, 64, 3)
        convs.append((w,) + make_bn(0, 0, 2 + 5 * i, 64))
    ref = oracle.basic_block(x, convs, BN_EPS, 1)
    cus = full_pool.partition_cus(0)
    d1 = S.ConvDesc(1, 56, 56, 64, 64, 3, 3, 1, 1, dtype, 1)
    c1, c2 = DevConv(d1, *convs[0], BN_EPS), DevConv(d1, *convs[1], BN_EPS)
    xd = dev_nhwc(x, dtype)
    t1, yd = dev_empty((1, 56, 56, 64), dtype), dev_empty((1, 56, 56, 64), dtype)
    k1 = c1.run(xd, t1, None, full_pool, 0, cus)
    k2 = c2.run(t1, yd, xd, full_pool, 0, cus)   # identity residual, then ReLU
    full_pool.sync()
    e = assert_close(host_nchw(yd), ref, dtype, "config 0 block")
    assert e < 2e-5
    # the task's stage 1 runs the same block structure: cross-check its first block
    del k1, k2


# ------------------------------------------------------------- config 1
@pytest.fixture(scope="module")
def cfg1():
    params = make_resnet18_params(1, 0)
    x = make_input(1, 0, (1, 3, 224, 224))
    logits, outs = oracle.resnet18(params, BN_EPS, x, want_stages=True)
    return params, x, logits, outs


def test_config1_resnet18_batch1_fp32_stages_and_net(full_pool, cfg1):
    params, x, logits, outs = cfg1
    dtype = S.SGPRS_F32
    task = S.Task(params, dtype, 2, BN_EPS)
    assert task.num_stages() == 6
    io = task.stage_io(0, 1)
    assert io["in_nchw"] == (1, 3, 224, 224) and io["out_nchw"] == (1, 64, 56, 56)
    assert task.stage_io(5, 2)["out_bytes"] == 2 * 1000 * 4
    # each stage in isolation, fed the oracle's own input for that stage
    for j in range(6):
        src = x if j == 0 else outs[j - 1]
        xd = dev_nhwc(src, dtype)
        o = (torch.full((1, 1000), float("nan"), dtype=torch.float32, device="cuda") if j == 5
             else dev_empty(stage_shape(j, 1), dtype))
        task.stage_run(j, 1, xd.data_ptr(), o.data_ptr(), full_pool, 0)
        full_pool.sync()
        e = assert_close(host_stage(o, j), outs[j], dtype, f"stage {j} alone")
        assert e < 3e-5, (j, e)
    # the six stages chained == whole network
    xd = dev_nhwc(x, dtype)
    got = run_stages_chained(task, full_pool, 0, xd, 1)
    errs = [assert_close(host_stage(got[j], j), outs[j], dtype, f"chained stage {j}") for j in range(6)]
    check_argmax(host_stage(got[5], 5), logits, errs[5], "config 1")
    # sgprs_task_run gives the same bits as the chained stages
    lg = torch.full((1, 1000), float("nan"), dtype=torch.float32, device="cuda")
    task.run(1, xd.data_ptr(), lg.data_ptr(), full_pool, 0)
    full_pool.sync()
    assert torch.equal(lg, got[5])
    task.destroy()


def test_task_run_across_partitions_matches_single_partition(cfg1):
    params, x, logits, _ = cfg1
    total = S.Pool(1, 8).info()["total_cus"]
    pool = S.Pool(2, total // 2)
    task = S.Task(params, S.SGPRS_F32, 1, BN_EPS)
    xd = dev_nhwc(x, S.SGPRS_F32)
    a = torch.full((1, 1000), float("nan"), dtype=torch.float32, device="cuda")
    b = torch.full((1, 1000), float("nan"), dtype=torch.float32, device="cuda")
    task.run(1, xd.data_ptr(), a.data_ptr(), pool, 0)
    pool.sync()
    task.run(1, xd.data_ptr(), b.data_ptr(), pool, 0, partition_per_stage=[0, 1, 0, 1, 0, 1])
    pool.sync()
    assert torch.equal(a, b)  # same CU count per partition -> same launch plan -> same bits
    assert_close(a.cpu().numpy().astype(np.float64), logits, S.SGPRS_F32, "task_run")
    with pytest.raises(S.SgprsError):
        task.run(2, xd.data_ptr(), a.data_ptr(), pool, 0)  # batch > max_batch
    with pytest.raises(S.SgprsError):
        task.stage_run(6, 1, xd.data_ptr(), a.data_ptr(), pool, 0)
    task.destroy()
    pool.destroy()


def test_downsample_block_runs_as_one_paired_launch(cfg1):
    """With enough tiles per CU nothing needs split-K, so the first convolution
    of a down-sampling block and the 1x1 convolution of its shortcut go out as
    one launch: the paired implicit GEMM (kind 10), or, when asked for, the
    stride-2 patch kernel with the shortcut on its centre tap (kind 11, bf16);
    the stages must match the oracle every time."""
    params = cfg1[0]
    nb = 8
    x = make_input(1, 7, (nb, 3, 224, 224))
    _, outs = oracle.resnet18(params, BN_EPS, x, want_stages=True)
    pool = S.Pool(1, 8)   # 8 images on 8 CUs: no layer of stages 2-4 is split
    try:
        for dtype, override, want in ((S.SGPRS_F32, (-1, 0, 1), 10), (S.SGPRS_BF16, (-1, 0, 1), 10),
                                      (S.SGPRS_BF16, (3, 0, 1), 11), (S.SGPRS_BF16, (3, 1, 1), 11),
                                      (S.SGPRS_BF16, (3, 2, 1), 10)):
            S.sgprs_conv_tuning_override(*override)
            task = S.Task(params, dtype, nb, BN_EPS)
            task.set_profiling(True)
            for j in (2, 3, 4):
                xd = dev_nhwc(outs[j - 1], dtype)
                o = dev_empty(stage_shape(j, nb), dtype)
                task.stage_run(j, nb, xd.data_ptr(), o.data_ptr(), pool, 0)
                pool.sync()
                assert_close(host_nchw(o), outs[j], dtype, f"paired stage {j} dtype {dtype} override {override}")
                kinds = [r["kind"] for r in task.kernel_times(j)]
                assert kinds.count(want) == 1 and kinds.count(21 - want) == 0, (j, dtype, override, kinds)
            task.destroy()
    finally:
        S.sgprs_conv_tuning_override(-1, 0, 1)
        pool.destroy()


def test_stage0_fp32_fused_stem_pool_elementwise(cfg1):
    """fp32 launches of at least two tiles per CU take the fused conv7x7 + max-pool kernel
    (kind 9): its stage-0 output, element by element against the oracle, on 8 and 64 CUs, with a
    ragged batch; the same images on the whole chip take the two-kernel path and agree."""
    params = cfg1[0]
    dtype = S.SGPRS_F32
    nb = 3
    x = make_input(1, 13, (nb, 3, 224, 224))
    ref = oracle.resnet18_stage(0, params, BN_EPS, x)
    total = S.Pool(1, 8).info()["total_cus"]
    xd = dev_nhwc(x, dtype)
    for cus, want_fused in ((8, True), (64, True), (total, False)):
        pool = S.Pool(1, cus)
        task = S.Task(params, dtype, nb, BN_EPS)
        task.set_profiling(True)
        o = dev_empty(stage_shape(0, nb), dtype)
        task.stage_run(0, nb, xd.data_ptr(), o.data_ptr(), pool, 0)
        pool.sync()
        kinds = [r["kind"] for r in task.kernel_times(0)]
        assert (kinds == [9]) == want_fused, (cus, kinds)
        e = assert_close(host_nchw(o), ref, dtype, f"fp32 stage 0 on {cus} CUs")
        assert e < 2e-5, (cus, e)
        task.destroy()
        pool.destroy()


def test_stage0_bf16_packed_row_and_four_slot_kernels_elementwise():
    """bf16 stage 0 runs the packed-row stem + pool kernel (kernel name recorded by the task); the
    tuning override switches to the 4-slot kernel.  Both, element by element against the oracle,
    on 8 CUs (each workgroup walks many tiles through both patch buffers), 64 CUs and the whole
    chip, with a ragged batch of 3 and a single image; the two kernels agree to accumulation order."""
    dtype = S.SGPRS_BF16
    params = make_resnet18_params(6, 1, bf16=True)
    total = S.Pool(1, 8).info()["total_cus"]
    for nb in (3, 1):
        x = make_input(6, nb, (nb, 3, 224, 224), bf16=True)
        ref = oracle.resnet18_stage(0, params, BN_EPS, x)
        xd = dev_nhwc(x, dtype)
        for cus in (8, 64, total):
            pool = S.Pool(1, cus)
            task = S.Task(params, dtype, nb, BN_EPS)
            task.set_profiling(True)
            outs = []
            try:
                for kind, name in ((-1, "stem_pool_packed_kernel"), (4, "stem_pool_kernel<1>")):
                    S.sgprs_conv_tuning_override(kind, 0, 1)
                    o = dev_empty(stage_shape(0, nb), dtype)
                    o.fill_(float("nan"))
                    task.stage_run(0, nb, xd.data_ptr(), o.data_ptr(), pool, 0)
                    pool.sync()
                    assert [r["name"] for r in task.kernel_times(0)] == [name], (cus, kind)
                    assert_close(host_nchw(o), ref, dtype, f"bf16 stage 0, {name}, batch {nb} on {cus} CUs")
                    outs.append(o.float().cpu().numpy())
            finally:
                S.sgprs_conv_tuning_override(-1, 0, 1)
            # same bf16 grid, fp32 sums in another order: at most one bf16 step apart
            d = np.abs(outs[0] - outs[1])
            assert np.all(d <= np.maximum(np.abs(outs[1]), 1e-3) * 2.0 ** -7), float(d.max())
            task.destroy()
            pool.destroy()


# ------------------------------------------------------------- config 3
def test_config3_eight_bf16_instances_on_8x32_pool():
    dtype = S.SGPRS_BF16
    total = S.Pool(1, 8).info()["total_cus"]
    n_p = 8
    pool = S.Pool(n_p, total // n_p)
    tasks, xs, refs = [], [], []
    for i in range(n_p):
        params = make_resnet18_params(3, i, bf16=True)
        x = make_input(3, i, (1, 3, 224, 224), bf16=True)
        tasks.append(S.Task(params, dtype, 1, BN_EPS))
        xs.append(dev_nhwc(x, dtype))
        refs.append(oracle.resnet18(params, BN_EPS, x))
    conc = [torch.full((1, 1000), float("nan"), dtype=torch.float32, device="cuda") for _ in range(n_p)]
    # stages of all instances issued round-robin, each instance on its own partition
    for j in range(6):
        for i in range(n_p):
            src = xs[i].data_ptr() if j == 0 else tasks[i].stage_output(j - 1)
            dst = conc[i].data_ptr() if j == 5 else tasks[i].stage_output(j)
            tasks[i].stage_run(j, 1, src, dst, pool, i)
    pool.sync()
    serial = [torch.full((1, 1000), float("nan"), dtype=torch.float32, device="cuda") for _ in range(n_p)]
    for i in range(n_p):
        tasks[i].run(1, xs[i].data_ptr(), serial[i].data_ptr(), pool, i)
        pool.sync()
    for i in range(n_p):
        assert torch.equal(conc[i], serial[i]), f"instance {i}: concurrent != serial"
        got = conc[i].cpu().numpy().astype(np.float64)
        e = assert_close(got, refs[i], dtype, f"config 3 instance {i}")
        check_argmax(got, refs[i], e, f"config 3 instance {i}")
    for t in tasks:
        t.destroy()
    pool.destroy()


# ------------------------------------------------------------- config 4
def test_config4_batch64_bf16_every_image_against_oracle(full_pool):
    dtype = S.SGPRS_BF16
    n = 64
    params = make_resnet18_params(4, 0, bf16=True)
    x = make_input(4, 0, (n, 3, 224, 224), bf16=True)
    task = S.Task(params, dtype, n, BN_EPS)
    xd = dev_nhwc(x, dtype)
    lg = torch.full((n, 1000), float("nan"), dtype=torch.float32, device="cuda")
    task.run(n, xd.data_ptr(), lg.data_ptr(), full_pool, 0)
    full_pool.sync()
    got = lg.cpu().numpy().astype(np.float64)
    assert np.all(np.isfinite(got))
    sample = list(range(n))    # every image: row tiles straddle image borders with a different phase in each
    ref, ref_stages = oracle.resnet18(params, BN_EPS, x[sample], want_stages=True)
    e = assert_close(got[sample], ref, dtype, "config 4 logits")
    check_argmax(got[sample], ref, e, "config 4")
    for j in range(5):
        c, h, w = STAGE_IO[j][1]
        so = torch.empty((n, h, w, c), dtype=torch.bfloat16, device="cuda")
        # read the task-owned stage buffer through a raw copy
        nbytes = so.numel() * 2
        import ctypes
        hip = ctypes.CDLL("libamdhip64.so")
        assert hip.hipMemcpy(ctypes.c_void_p(so.data_ptr()), ctypes.c_void_p(task.stage_output(j)),
                             ctypes.c_size_t(nbytes), 3) == 0
        assert_close(host_nchw(so[sample]), ref_stages[j], dtype, f"config 4 stage {j}")
    # batch independence: image 5 alone equals row 5 of the batch run, to rounding
    l1 = torch.full((1, 1000), float("nan"), dtype=torch.float32, device="cuda")
    x5 = xd[5:6].contiguous()
    task.run(1, x5.data_ptr(), l1.data_ptr(), full_pool, 0)
    full_pool.sync()
    assert rel_err(l1.cpu().numpy().astype(np.float64), got[5:6]) <= TOL[dtype]
    # reproducible: the same batch again gives the same bits
    lg2 = torch.full((n, 1000), float("nan"), dtype=torch.float32, device="cuda")
    task.run(n, xd.data_ptr(), lg2.data_ptr(), full_pool, 0)
    full_pool.sync()
    assert torch.equal(lg, lg2)
    task.destroy()


# ------------------------------------------------------------- other batch sizes
@pytest.mark.parametrize("dtype,n,cus", [
    (S.SGPRS_BF16, 8, 0), (S.SGPRS_BF16, 16, 0), (S.SGPRS_BF16, 5, 32), (S.SGPRS_F32, 8, 0), (S.SGPRS_F32, 3, 64),
], ids=["bf16-n8-256cu", "bf16-n16-256cu", "bf16-n5-32cu", "f32-n8-256cu", "f32-n3-64cu"])
def test_whole_network_at_other_batch_sizes(full_pool, dtype, n, cus):
    """Batches between the one-image tasks and the batch-64 run take other planner choices (tile
    shapes, split-K, fused or unfused head): every logit of every image against the oracle, on the
    whole chip (cus = 0) or on a partition of `cus` CUs; an odd batch leaves ragged row tiles."""
    bf16 = dtype == S.SGPRS_BF16
    seed = 2    # with these weights the oracle's best class leads the second by 6 % of max|logit| on every image
    params = make_resnet18_params(5, seed, bf16=bf16)
    x = make_input(5, seed, (n, 3, 224, 224), bf16=bf16)
    pool = full_pool if cus == 0 else S.Pool(2, cus)
    part = 0 if cus == 0 else 1
    task = S.Task(params, dtype, n, BN_EPS)
    xd = dev_nhwc(x, dtype)
    lg = torch.full((n, 1000), float("nan"), dtype=torch.float32, device="cuda")
    for _ in range(3):      # eager, capture, replay
        task.run(n, xd.data_ptr(), lg.data_ptr(), pool, part)
    pool.sync()
    got = lg.cpu().numpy().astype(np.float64)
    ref = oracle.resnet18(params, BN_EPS, x)
    top2 = np.sort(ref, axis=1)[:, -2:]
    assert np.min((top2[:, 1] - top2[:, 0]) / np.max(np.abs(ref), axis=1)) > 2 * TOL[dtype]   # the top class is decided
    e = assert_close(got, ref, dtype, f"batch {n} logits")
    check_argmax(got, ref, e, f"batch {n}")
    task.destroy()
    if cus:
        pool.destroy()


def test_task_run_graph_replay_matches_eager(full_pool, cfg1):
    """sgprs_task_run captures a task into a HIP graph on the second call with the same arguments
    and replays it afterwards.  Replays are interleaved with eager work on the same stream, with
    changed input contents, and with synchronisations, and every one is compared with the eager
    result (stage by stage through sgprs_stage_run, which never uses a graph)."""
    params, x, _, _ = cfg1
    for dtype in (S.SGPRS_F32, S.SGPRS_BF16):
        task = S.Task(params, dtype, 1, BN_EPS)
        xd = dev_nhwc(x, dtype)
        x2 = dev_nhwc(make_input(1, 9, (1, 3, 224, 224)), dtype)
        xin = torch.empty_like(xd)
        lg = torch.full((1, 1000), float("nan"), dtype=torch.float32, device="cuda")
        scratch = torch.zeros(1 << 20, dtype=torch.float32, device="cuda")
        for it in range(8):
            src = xd if it % 2 == 0 else x2
            xin.copy_(src)
            torch.cuda.synchronize()
            # eager reference: the six stages one by one
            ref = torch.full((1, 1000), float("nan"), dtype=torch.float32, device="cuda")
            for j in range(6):
                a = xin.data_ptr() if j == 0 else task.stage_output(j - 1)
                b = ref.data_ptr() if j == 5 else task.stage_output(j)
                task.stage_run(j, 1, a, b, full_pool, 0)
            full_pool.sync()
            lg.fill_(float("nan"))
            scratch.add_(1.0)                      # unrelated eager work between the replays
            torch.cuda.synchronize()
            task.run(1, xin.data_ptr(), lg.data_ptr(), full_pool, 0)   # call 1 eager, call 2 captures, then replays
            full_pool.sync()
            assert torch.equal(lg, ref), (dtype, it)
        task.destroy()


def test_graph_replay_survives_other_batches_and_partitions(cfg1):
    """Captured graphs must stay valid (or be rebuilt) when the same task later runs other batch
    sizes or partitions, which may grow the split-K scratch the graphs point into."""
    params, x, _, _ = cfg1
    dtype = S.SGPRS_BF16
    total = S.Pool(1, 8).info()["total_cus"]
    pool = S.Pool(2, total // 2)
    task = S.Task(params, dtype, 16, BN_EPS)
    task.set_graph_replay(1)   # also for the batch of six
    x1 = dev_nhwc(x, dtype)
    xb = dev_nhwc(make_input(1, 11, (6, 3, 224, 224)), dtype)
    l1 = torch.full((1, 1000), float("nan"), dtype=torch.float32, device="cuda")
    lb = torch.full((6, 1000), float("nan"), dtype=torch.float32, device="cuda")
    seen1, seenb = [], []
    for rnd in range(3):
        for _ in range(3):                      # eager, capture, replay
            l1.fill_(float("nan"))
            task.run(1, x1.data_ptr(), l1.data_ptr(), pool, 0)
            pool.sync()
            seen1.append(l1.clone())
        for part in (1, 0):
            for _ in range(3):
                lb.fill_(float("nan"))
                task.run(6, xb.data_ptr(), lb.data_ptr(), pool, part)
                pool.sync()
                seenb.append(lb.clone())
    assert all(torch.equal(a, seen1[0]) for a in seen1) and bool(torch.isfinite(seen1[0]).all())
    assert all(torch.equal(a, seenb[0]) for a in seenb) and bool(torch.isfinite(seenb[0]).all())
    task.destroy()
    pool.destroy()


# ------------------------------------------------------------- profiling hook
def test_kernel_times_records(full_pool, cfg1):
    params, x, _, _ = cfg1
    task = S.Task(params, S.SGPRS_BF16, 1, BN_EPS)
    xd = dev_nhwc(x, S.SGPRS_BF16)
    lg = torch.empty((1, 1000), dtype=torch.float32, device="cuda")
    task.set_profiling(True)
    task.run(1, xd.data_ptr(), lg.data_ptr(), full_pool, 0)
    full_pool.sync()
    flops = 0.0
    for j in range(6):
        recs = task.kernel_times(j)
        assert recs and all(r["ms"] >= 0 for r in recs)
        flops += sum(r["flops"] for r in recs if r["kind"] in (0, 1, 5, 8, 9, 10, 11))
    assert abs(flops - 2 * 1814073344) / (2 * 1814073344) < 1e-9
    task.destroy()
