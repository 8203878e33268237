"""The periodic-release run (sgprs_sched_run_periodic) on the GPU: scheduler decisions from the
C++ core, stages from the HIP kernels, on a pool of two contexts with two lanes each (lanes of a
context share a CU mask).  Checked: the logits every task ends up with are the oracle's for its
input, the counters add up, a light load misses nothing, an impossible load terminates with
misses or drops instead of hanging."""
import numpy as np
import pytest
import torch

import oracle
import paper_2406_09425_amd as S
from workloads import BN_EPS, make_input, make_resnet18_params

from gpu_util import TOL, dev_nhwc, rel_err

pytestmark = pytest.mark.gpu
N_CTX, LANES = 2, 2


@pytest.fixture(scope="module")
def rig():
    total = S.Pool(1, 8).info()["total_cus"]
    half = S.Pool(2, total // 2)
    masks = np.stack([half.mask(c) for c in range(N_CTX) for _ in range(LANES)])
    half.destroy()
    pool = S.Pool(N_CTX * LANES, 0, masks=masks)
    n_tasks = 4
    params = [make_resnet18_params(3, i, bf16=True) for i in range(n_tasks)]
    xs_host = [make_input(3, i, (1, 3, 224, 224), bf16=True) for i in range(n_tasks)]
    tasks = [S.Task(p, S.SGPRS_BF16, 1, BN_EPS) for p in params]
    xs = [dev_nhwc(x, S.SGPRS_BF16) for x in xs_host]
    yield dict(pool=pool, tasks=tasks, xs=xs, xs_host=xs_host, params=params, cus=total // 2)
    for t in tasks:
        t.destroy()
    pool.destroy()


def test_lanes_of_a_context_share_its_mask(rig):
    pool = rig["pool"]
    assert np.array_equal(pool.mask(0), pool.mask(1)) and np.array_equal(pool.mask(2), pool.mask(3))
    assert not np.array_equal(pool.mask(0), pool.mask(2))
    assert pool.partition_cus(0) == rig["cus"] == pool.partition_cus(3)


def test_light_load_meets_every_deadline_and_computes_the_oracles_logits(rig):
    n = len(rig["tasks"])
    sch = S.Sched(N_CTX, LANES)
    for _ in range(n):
        sch.add_task([100e-6] * 6, 2.0 ** -7, 2.0 ** -7)   # 128 fps tasks (a period that is exact in binary), generous WCETs
    lgs = [torch.full((1, 1000), float("nan"), dtype=torch.float32, device="cuda") for _ in range(n)]
    for t, x, l in zip(rig["tasks"], rig["xs"], lgs):   # first use of a task allocates its scratch: not part of the run
        t.run(1, x.data_ptr(), l.data_ptr(), rig["pool"], 0)
    rig["pool"].sync()
    for l in lgs:
        l.fill_(float("nan"))
    rep = sch.run_periodic(rig["pool"], rig["tasks"], [x.data_ptr() for x in rig["xs"]], [l.data_ptr() for l in lgs], 1,
                           duration_s=10 * 2.0 ** -7, offsets=[i * 2.0 ** -10 for i in range(n)])
    rig["pool"].sync()
    assert rep["releases"] == 10 * n and rep["dropped"] == 0
    assert rep["jobs_released"] == rep["jobs_completed"] == 10 * n and rep["stages_completed"] == 60 * n
    # every job meets its 7.8 ms deadline with a wide margin; a virtual stage deadline (1.3 ms) may be
    # overrun once or twice by a first launch on a fresh launcher thread, which only changes a level
    assert rep["jobs_missed"] == 0 and rep["dmr"] == 0.0 and rep["stages_missed"] <= 6
    assert abs(rep["fps"] - 10 * n / rep["elapsed_s"]) < 1e-9 and 10 * 2.0 ** -7 <= rep["elapsed_s"] < 0.2
    assert 0 < rep["mean_response_s"] <= rep["max_response_s"] < 2.0 ** -7
    for i in (0, n - 1):
        ref = oracle.resnet18(rig["params"][i], BN_EPS, rig["xs_host"][i])
        got = lgs[i].cpu().numpy().astype(np.float64)
        assert rel_err(got, ref) <= TOL[S.SGPRS_BF16]
        assert int(np.argmax(got)) == int(np.argmax(ref))
    assert sch.stats()["jobs_completed"] == 10 * n
    sch.destroy()


def test_impossible_load_ends_with_misses_not_with_a_hang(rig):
    n = len(rig["tasks"])
    sch = S.Sched(N_CTX, LANES)
    for _ in range(n):
        sch.add_task([20e-6] * 6, 2.0 ** -14, 2.0 ** -14)  # 16 384 fps per task: far beyond the GPU
    lgs = [torch.empty((1, 1000), dtype=torch.float32, device="cuda") for _ in range(n)]
    rep = sch.run_periodic(rig["pool"], rig["tasks"], [x.data_ptr() for x in rig["xs"]], [l.data_ptr() for l in lgs], 1,
                           duration_s=2.0 ** -6)
    rig["pool"].sync()
    assert rep["releases"] == 256 * n
    assert rep["jobs_released"] + rep["dropped"] == rep["releases"]
    assert rep["jobs_completed"] == rep["jobs_released"] and rep["stages_completed"] == 6 * rep["jobs_completed"]
    assert rep["dropped"] > 0 and rep["jobs_missed"] > 0 and 0.5 < rep["dmr"] <= 1.0
    assert all(torch.isfinite(l).all() for l in lgs)
    sch.destroy()


def test_run_rejects_mismatched_arguments(rig):
    sch = S.Sched(N_CTX, LANES)
    sch.add_task([1e-4] * 6, 1e-2, 1e-2)
    lg = torch.empty((1, 1000), dtype=torch.float32, device="cuda")
    x = rig["xs"][0]
    with pytest.raises(S.SgprsError):     # two tasks given, one known
        sch.run_periodic(rig["pool"], rig["tasks"][:2], [x.data_ptr()] * 2, [lg.data_ptr()] * 2, 1, 0.01)
    with pytest.raises(S.SgprsError):     # duration out of range
        sch.run_periodic(rig["pool"], rig["tasks"][:1], [x.data_ptr()], [lg.data_ptr()], 1, 0.0)
    big = S.Sched(3, 2)                   # needs six partitions, the pool has four
    big.add_task([1e-4] * 6, 1e-2, 1e-2)
    with pytest.raises(S.SgprsError):
        big.run_periodic(rig["pool"], rig["tasks"][:1], [x.data_ptr()], [lg.data_ptr()], 1, 0.01)
    wrong = S.Sched(N_CTX, LANES)         # a five-stage task against the six-stage network
    wrong.add_task([1e-4] * 5, 1e-2, 1e-2)
    with pytest.raises(S.SgprsError):
        wrong.run_periodic(rig["pool"], rig["tasks"][:1], [x.data_ptr()], [lg.data_ptr()], 1, 0.01)
    for s in (sch, big, wrong):
        s.destroy()


def test_two_contexts_of_four_lanes_the_papers_shape():
    """"Stage Queuing": a context carries two high- and two low-priority streams, at most four stages in
    flight.  Eight lanes = eight CU-masked streams; the run loop keeps at most four of them busy at once
    (more collapse on this GPU), so the eight tasks still all finish, meet a generous deadline, and end
    with the oracle's logits.  A second run right after a failed one starts from a clean scheduler."""
    n_ctx, lanes, n_tasks = 2, 4, 8
    total = S.Pool(1, 8).info()["total_cus"]
    half = S.Pool(2, total // 2)
    masks = np.stack([half.mask(c) for c in range(n_ctx) for _ in range(lanes)])
    half.destroy()
    pool = S.Pool(n_ctx * lanes, 0, masks=masks)
    params = [make_resnet18_params(3, i, bf16=True) for i in range(n_tasks)]
    xs_host = [make_input(3, i, (1, 3, 224, 224), bf16=True) for i in range(n_tasks)]
    tasks = [S.Task(p, S.SGPRS_BF16, 1, BN_EPS) for p in params]
    xs = [dev_nhwc(x, S.SGPRS_BF16) for x in xs_host]
    lgs = [torch.full((1, 1000), float("nan"), dtype=torch.float32, device="cuda") for _ in range(n_tasks)]
    try:
        for t, x, l in zip(tasks, xs, lgs):
            t.run(1, x.data_ptr(), l.data_ptr(), pool, 0)
        pool.sync()
        for l in lgs:
            l.fill_(float("nan"))
        sch = S.Sched(n_ctx, lanes)
        for _ in range(n_tasks):
            sch.add_task([100e-6] * 6, 2.0 ** -7, 2.0 ** -7)
        # a failing run (one input pointer missing) must leave nothing behind
        with pytest.raises(S.SgprsError):
            sch.run_periodic(pool, tasks, [x.data_ptr() for x in xs[:-1]] + [None], [l.data_ptr() for l in lgs], 1, 0.01)
        rep = sch.run_periodic(pool, tasks, [x.data_ptr() for x in xs], [l.data_ptr() for l in lgs], 1,
                               duration_s=10 * 2.0 ** -7, offsets=[i * 2.0 ** -11 for i in range(n_tasks)])
        pool.sync()
        assert rep["releases"] == 10 * n_tasks and rep["dropped"] == 0
        assert rep["jobs_completed"] == 10 * n_tasks and rep["stages_completed"] == 60 * n_tasks
        assert rep["jobs_missed"] == 0 and rep["max_response_s"] < 2.0 ** -7
        for i in range(n_tasks):
            ref = oracle.resnet18(params[i], BN_EPS, xs_host[i])
            got = lgs[i].cpu().numpy().astype(np.float64)
            assert rel_err(got, ref) <= TOL[S.SGPRS_BF16], i
            assert int(np.argmax(got)) == int(np.argmax(ref)), i
        # without the gate the same run still completes (slower): the gate changes speed, not results
        sch.set_max_busy(0)
        rep2 = sch.run_periodic(pool, tasks, [x.data_ptr() for x in xs], [l.data_ptr() for l in lgs], 1,
                                duration_s=4 * 2.0 ** -7)
        assert rep2["jobs_completed"] == rep2["jobs_released"] == 4 * n_tasks
        with pytest.raises(S.SgprsError):
            sch.set_max_busy(-1)
        sch.destroy()
    finally:
        for t in tasks:
            t.destroy()
        pool.destroy()


def test_static_execution_on_eight_partitions_with_the_gate():
    """sgprs_pool_run_static: eight tasks, each on its own 32-CU partition, at most four partitions busy
    at once; every task's logits are the oracle's, with and without the gate, and bad arguments are
    refused before anything runs."""
    n = 8
    total = S.Pool(1, 8).info()["total_cus"]
    pool = S.Pool(n, total // n)
    params = [make_resnet18_params(3, i, bf16=True) for i in range(n)]
    xs_host = [make_input(3, i, (1, 3, 224, 224), bf16=True) for i in range(n)]
    tasks = [S.Task(p, S.SGPRS_BF16, 1, BN_EPS) for p in params]
    xs = [dev_nhwc(x, S.SGPRS_BF16) for x in xs_host]
    refs = [oracle.resnet18(params[i], BN_EPS, xs_host[i]) for i in range(n)]
    try:
        for gate in (4, 0):
            lgs = [torch.full((1, 1000), float("nan"), dtype=torch.float32, device="cuda") for _ in range(n)]
            el = pool.run_static(tasks, [x.data_ptr() for x in xs], [l.data_ptr() for l in lgs], 1, list(range(n)), rounds=5,
                                 max_busy=gate)
            assert 0 < el < 5.0
            for i in range(n):
                got = lgs[i].cpu().numpy().astype(np.float64)
                assert rel_err(got, refs[i]) <= TOL[S.SGPRS_BF16], (gate, i)
                assert int(np.argmax(got)) == int(np.argmax(refs[i])), (gate, i)
        lg = torch.empty((1, 1000), dtype=torch.float32, device="cuda")
        with pytest.raises(S.SgprsError):
            pool.run_static(tasks[:1], [xs[0].data_ptr()], [lg.data_ptr()], 1, [n], rounds=1)       # partition outside the pool
        with pytest.raises(S.SgprsError):
            pool.run_static(tasks[:1], [xs[0].data_ptr()], [lg.data_ptr()], 1, [0], rounds=0)       # no rounds
    finally:
        for t in tasks:
            t.destroy()
        pool.destroy()
