"""Context pool on the GPU: CU-masked streams, placement evidence, error paths."""
import json
import os

import numpy as np
import pytest
import torch

import paper_2406_09425_amd as S

pytestmark = pytest.mark.gpu


def probe(pool, p, n_blocks=4096, spin=20000):
    out = torch.zeros(2 * n_blocks, dtype=torch.int32, device="cuda")
    pool.probe(p, n_blocks, spin, out.data_ptr())
    pool.sync(p)
    a = out.cpu().numpy().astype(np.uint32).reshape(n_blocks, 2)
    xcc = a[:, 0] & 0xF
    hw = a[:, 1]
    cu, sh, se = (hw >> 8) & 0xF, (hw >> 12) & 0x1, (hw >> 13) & 0x7
    return xcc, se, sh, cu


def test_pool_info_and_masks():
    pool = S.Pool(2, 64)
    info = pool.info()
    assert info["n_p"] == 2 and info["cus_per_partition"] == 64
    total, nx = info["total_cus"], info["n_xcd"]
    assert total % nx == 0
    m0, m1 = pool.mask(0), pool.mask(1)
    assert sum(bin(int(w)).count("1") for w in m0) == 64 == pool.partition_cus(1)
    assert not np.any(m0 & m1)  # disjoint partitions
    assert np.array_equal(m0[: (total + 31) // 32], S.sgprs_build_cu_mask(total, nx, 64, 0))
    assert pool.stream(0) != pool.stream(1)
    with pytest.raises(S.SgprsError):
        pool.stream(2)
    pool.destroy()


def test_oversubscription_needs_flag():
    total = S.Pool(1, 8).info()["total_cus"]
    with pytest.raises(S.SgprsError) as e:
        S.Pool(3, total // 2)
    assert e.value.status == -6
    pool = S.Pool(3, total // 2, S.SGPRS_POOL_OVERSUBSCRIBE)
    assert np.any(pool.mask(0) & pool.mask(2))  # wrapped around: overlaps partition 0
    pool.destroy()
    with pytest.raises(S.SgprsError):
        S.Pool(1, 12)  # not a multiple of the die count


def test_partition_placement_matches_mask():
    """Workgroups of a partition land on as many distinct CUs as its mask has
    bits, evenly over the dies; disjoint partitions use disjoint CUs."""
    pool = S.Pool(1, 8)
    info = pool.info()
    total, nx = info["total_cus"], info["n_xcd"]
    pool.destroy()
    report = {}
    for cus in (8, 32, total // 2):
        pool = S.Pool(2, cus)
        seen = []
        for p in range(2):
            xcc, se, sh, cu = probe(pool, p)
            ids = set(zip(xcc.tolist(), se.tolist(), sh.tolist(), cu.tolist()))
            per_die = {int(x): len({i for i in ids if i[0] == x}) for x in set(xcc.tolist())}
            report[f"{cus}cus_p{p}"] = dict(distinct_cus=len(ids), per_die=per_die)
            assert len(ids) == cus, (cus, p, len(ids), per_die)
            assert len(per_die) == nx and set(per_die.values()) == {cus // nx}, per_die
            seen.append(ids)
        assert not (seen[0] & seen[1]), "disjoint masks share a CU"
        pool.destroy()
    os.makedirs("gpurun_out", exist_ok=True)
    with open("gpurun_out/placement_probe.json", "w") as f:
        json.dump(report, f, indent=1)
    print(json.dumps(report))


def test_explicit_masks_pool():
    total = S.Pool(1, 8).info()["total_cus"]
    words = (total + 31) // 32
    masks = np.zeros((2, words), dtype=np.uint32)
    masks[0, 0] = 0xFF
    masks[1, 0] = 0xFF00
    pool = S.Pool(2, 0, masks=masks)
    assert pool.partition_cus(0) == 8 and pool.partition_cus(1) == 8
    xcc, se, sh, cu = probe(pool, 0, 512, 5000)
    assert len(set(zip(xcc.tolist(), se.tolist(), sh.tolist(), cu.tolist()))) == 8
    pool.destroy()
    with pytest.raises(S.SgprsError):
        S.Pool(1, 0, masks=np.zeros((1, words), dtype=np.uint32))


def test_mfma_probe_checksum_and_errors():
    """The sustained-rate probe really runs its MFMAs: with constant operands (1.0) every
    accumulator element ends at 16 * 18 * steps, and workgroup 0 reports the sum of its 64."""
    total = S.Pool(1, 8).info()["total_cus"]
    pool = S.Pool(1, total)
    out = torch.zeros(3, dtype=torch.int64, device="cuda")
    steps = 10
    pool.mfma_probe(0, False, steps, out.data_ptr())
    pool.sync()
    ticks, clocks, bits = (int(v) for v in out.cpu().tolist())
    assert ticks > 0 and clocks > 0
    assert np.array([bits], dtype=np.uint32).view(np.float32)[0] == 64.0 * 16 * 18 * steps
    pool.mfma_probe(0, True, steps, out.data_ptr())
    pool.sync()
    assert np.isfinite(np.array([int(out[2])], dtype=np.uint32).view(np.float32)[0])
    with pytest.raises(S.SgprsError):
        pool.mfma_probe(0, False, 0, out.data_ptr())
    with pytest.raises(S.SgprsError):
        pool.mfma_probe(0, False, 10, 0)
    pool.destroy()


def test_load_probe_checksum_and_errors():
    """The load probe really moves its data: the buffer holds ones, so every workgroup finds
    16384 of them in LDS after its last iteration, whatever the region size."""
    pool = S.Pool(2, 32)
    cus = pool.partition_cus(1)
    buf = torch.ones(4 << 20, dtype=torch.int32, device="cuda")  # 16 MiB
    for region in (16 << 10, 64 << 10, 1 << 20):
        out = torch.zeros(cus, dtype=torch.int32, device="cuda")
        pool.load_probe(1, buf.data_ptr(), buf.numel() * 4, region, 5, out.data_ptr())
        pool.sync()
        assert out.cpu().tolist() == [16384] * cus
    out = torch.zeros(cus, dtype=torch.int32, device="cuda")
    for bad in (dict(region=48 << 10), dict(region=8 << 10), dict(nbytes=(64 << 10) + 16), dict(iters=0), dict(buf=0),
                dict(buf=buf.data_ptr() + 4), dict(out=0)):
        kw = dict(buf=buf.data_ptr(), nbytes=1 << 20, region=64 << 10, iters=1, out=out.data_ptr())
        kw.update(bad)
        with pytest.raises(S.SgprsError):
            pool.load_probe(1, kw["buf"], kw["nbytes"], kw["region"], kw["iters"], kw["out"])
    pool.sync()
    pool.destroy()


def test_graph_launch_keeps_to_the_partition():
    """A kernel recorded by stream capture and launched as a HIP graph on a partition's stream
    runs on that partition's CUs only (sgprs_task_run replays captured tasks this way)."""
    total = S.Pool(1, 8).info()["total_cus"]
    pool = S.Pool(8, total // 8)
    n_blocks = 4096
    for p in (0, 3, 7):
        sets = []
        for graph in (False, True):
            out = torch.zeros(2 * n_blocks, dtype=torch.int32, device="cuda")
            (pool.probe_graph if graph else pool.probe)(p, n_blocks, 20000, out.data_ptr())
            pool.sync(p)
            a = out.cpu().numpy().astype(np.uint32).reshape(n_blocks, 2)
            sets.append(set(zip((a[:, 0] & 0xF).tolist(), ((a[:, 1] >> 8) & 0x7F).tolist())))
        assert sets[1] == sets[0] and len(sets[0]) == total // 8, (p, len(sets[0]), len(sets[1]))
    pool.destroy()
