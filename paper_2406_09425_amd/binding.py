"""ctypes binding of libsgprs.so (see include/sgprs.h for the contract).

Argument marshalling only.  Functions keep the C names; `Pool` and `Task` are
small owners of the opaque handles.  Device tensors are passed as integer
addresses (for instance ``torch.Tensor.data_ptr()``).
"""
from __future__ import annotations

import ctypes
import os
from ctypes import (POINTER, c_char_p, c_double, c_float, c_int, c_size_t, c_uint, c_uint32,
                    c_void_p)

import numpy as np

__all__ = [
    "SgprsError", "SGPRS_F32", "SGPRS_BF16", "SGPRS_POOL_OVERSUBSCRIBE", "SGPRS_POOL_BLOCKED_LAYOUT",
    "ConvDesc", "lib", "lib_path", "Pool", "Task", "Sched", "Dispatch", "SchedStats", "RunReport",
    "sgprs_version", "sgprs_status_string", "sgprs_last_error", "sgprs_build_cu_mask",
    "sgprs_fold_bn", "sgprs_conv_packed_weight_bytes", "sgprs_pack_conv_weights",
    "sgprs_unpack_conv_weights", "sgprs_conv2d_workspace", "sgprs_conv2d", "sgprs_maxpool2d",
    "sgprs_conv_tuning_override", "sgprs_conv2d_plan", "sgprs_bn_relu", "sgprs_add_relu", "sgprs_avgpool_fc", "sgprs_global_avgpool", "sgprs_avgpool_fc_static",
    "sgprs_kernel_name",
]

SGPRS_F32, SGPRS_BF16 = 0, 1
SGPRS_POOL_OVERSUBSCRIBE, SGPRS_POOL_BLOCKED_LAYOUT = 1, 2
ERR_NAMES = {-1: "INVALID_ARG", -2: "NO_DEVICE", -3: "HIP", -4: "OOM", -5: "UNSUPPORTED", -6: "OVERSUBSCRIBED"}

_PKG = os.path.dirname(os.path.abspath(__file__))


class SgprsError(RuntimeError):
    def __init__(self, status: int, detail: str):
        super().__init__(f"SGPRS_ERR_{ERR_NAMES.get(status, status)}: {detail}")
        self.status = status


class ConvDesc(ctypes.Structure):
    _fields_ = [(n, c_int) for n in ("n", "h", "w", "cin", "cout", "r", "s", "stride", "pad", "dtype", "relu")]


class _Params(ctypes.Structure):
    _fields_ = [("conv_w", POINTER(c_float) * 20), ("bn_gamma", POINTER(c_float) * 20),
                ("bn_beta", POINTER(c_float) * 20), ("bn_mean", POINTER(c_float) * 20),
                ("bn_var", POINTER(c_float) * 20), ("fc_w", POINTER(c_float)), ("fc_b", POINTER(c_float)),
                ("bn_eps", c_float)]


def lib_path() -> str:
    return os.path.join(_PKG, "libsgprs.so")


_lib = None


class Dispatch(ctypes.Structure):
    _fields_ = [("task", c_int), ("job", c_int), ("stage", c_int), ("context", c_int), ("lane", c_int),
                ("level", c_int), ("deadline", c_double), ("wcet", c_double)]


class SchedStats(ctypes.Structure):
    _fields_ = [(n, ctypes.c_longlong) for n in ("jobs_released", "jobs_completed", "jobs_missed",
                                                 "stages_completed", "stages_missed")]


class RunReport(ctypes.Structure):
    _fields_ = [("elapsed_s", c_double), ("releases", ctypes.c_longlong), ("dropped", ctypes.c_longlong),
                ("sched", SchedStats), ("fps", c_double), ("dmr", c_double), ("mean_response_s", c_double),
                ("max_response_s", c_double)]


def lib():
    """Loads libsgprs.so; raises if it has not been built (no fallback)."""
    global _lib
    if _lib is not None:
        return _lib
    path = lib_path()
    if not os.path.exists(path):
        raise ImportError(f"{path} is missing: build it with `python -m paper_2406_09425_amd.build` "
                          "(there is no CPU fallback)")
    L = ctypes.CDLL(path)
    vp, ip, fp = c_void_p, POINTER(c_int), POINTER(c_float)
    sig = {
        "sgprs_status_string": (c_char_p, [c_int]),
        "sgprs_last_error": (c_char_p, []),
        "sgprs_version": (c_int, []),
        "sgprs_build_cu_mask": (c_int, [c_int, c_int, c_int, c_int, c_int, POINTER(c_uint32), c_int]),
        "sgprs_pool_create": (c_int, [c_int, c_int, c_int, c_uint, POINTER(vp)]),
        "sgprs_pool_create_masks": (c_int, [c_int, c_int, POINTER(c_uint32), c_int, POINTER(vp)]),
        "sgprs_pool_destroy": (c_int, [vp]),
        "sgprs_pool_info": (c_int, [vp, ip, ip, ip, ip]),
        "sgprs_pool_partition_cus": (c_int, [vp, c_int, ip]),
        "sgprs_pool_get_mask": (c_int, [vp, c_int, POINTER(c_uint32), c_int]),
        "sgprs_pool_stream": (vp, [vp, c_int]),
        "sgprs_partition_sync": (c_int, [vp, c_int]),
        "sgprs_pool_sync": (c_int, [vp]),
        "sgprs_partition_probe": (c_int, [vp, c_int, c_int, c_int, vp]),
        "sgprs_mfma_probe": (c_int, [vp, c_int, c_int, c_int, vp]),
        "sgprs_load_probe": (c_int, [vp, c_int, vp, c_size_t, c_size_t, c_int, vp]),
        "sgprs_partition_probe_graph": (c_int, [vp, c_int, c_int, c_int, vp]),
        "sgprs_fold_bn": (c_int, [fp, fp, fp, fp, c_float, c_int, fp, fp]),
        "sgprs_conv_packed_weight_bytes": (c_int, [POINTER(ConvDesc), POINTER(c_size_t)]),
        "sgprs_pack_conv_weights": (c_int, [POINTER(ConvDesc), fp, vp, c_size_t]),
        "sgprs_unpack_conv_weights": (c_int, [POINTER(ConvDesc), vp, c_size_t, fp]),
        "sgprs_conv2d_workspace": (c_int, [POINTER(ConvDesc), c_int, POINTER(c_size_t)]),
        "sgprs_conv2d": (c_int, [POINTER(ConvDesc), vp, vp, vp, vp, vp, vp, vp, c_size_t, vp, c_int]),
        "sgprs_conv_tuning_override": (c_int, [c_int, c_int, c_int]),
        "sgprs_conv2d_plan": (c_int, [POINTER(ConvDesc), c_int, c_int, POINTER(c_int), POINTER(c_int)]),
        "sgprs_maxpool2d": (c_int, [c_int, c_int, c_int, c_int, c_int, vp, vp, vp, c_int]),
        "sgprs_bn_relu": (c_int, [c_int, c_size_t, c_int, vp, vp, vp, vp, vp, c_int]),
        "sgprs_add_relu": (c_int, [c_int, c_size_t, vp, vp, vp, c_int, vp, c_int]),
        "sgprs_avgpool_fc": (c_int, [c_int, c_int, c_int, c_int, c_int, vp, vp, vp, vp, vp, vp, c_int]),
        "sgprs_avgpool_fc_static": (c_int, [c_int, c_int, c_int, c_int, c_int, vp, vp, vp, vp, vp, c_int]),
        "sgprs_global_avgpool": (c_int, [c_int, c_int, c_int, c_int, vp, vp, vp, c_int]),
        "sgprs_task_create_resnet18": (c_int, [c_int, c_int, c_int, POINTER(_Params), POINTER(vp)]),
        "sgprs_task_destroy": (c_int, [vp]),
        "sgprs_task_num_stages": (c_int, [vp]),
        "sgprs_task_stage_io": (c_int, [vp, c_int, c_int, POINTER(c_size_t), POINTER(c_size_t), ip, ip]),
        "sgprs_stage_run": (c_int, [vp, c_int, c_int, vp, vp, vp, c_int]),
        "sgprs_task_run": (c_int, [vp, c_int, vp, vp, vp, c_int, ip]),
        "sgprs_task_stage_output": (vp, [vp, c_int]),
        "sgprs_task_set_profiling": (c_int, [vp, c_int]),
        "sgprs_task_set_graph_replay": (c_int, [vp, c_int]),
        "sgprs_task_kernel_times": (c_int, [vp, c_int, ip, ip, ip, fp, POINTER(c_double), POINTER(c_double)]),
        "sgprs_kernel_name": (c_char_p, [c_int, c_int]),
        "sgprs_sched_create": (c_int, [c_int, c_int, POINTER(vp)]),
        "sgprs_sched_destroy": (None, [vp]),
        "sgprs_sched_add_task": (c_int, [vp, c_int, POINTER(c_double), c_double, c_double, ip]),
        "sgprs_sched_virtual_deadlines": (c_int, [vp, c_int, c_int, POINTER(c_double)]),
        "sgprs_sched_release": (c_int, [vp, c_int, c_double, ip]),
        "sgprs_sched_next": (c_int, [vp, c_double, POINTER(Dispatch)]),
        "sgprs_sched_complete": (c_int, [vp, c_int, c_int, c_int, c_double, ip]),
        "sgprs_sched_get_stats": (c_int, [vp, POINTER(SchedStats)]),
        "sgprs_sched_set_max_busy": (c_int, [vp, c_int]),
        "sgprs_pool_run_static": (c_int, [vp, POINTER(vp), c_int, POINTER(vp), POINTER(vp), c_int, ip, c_int, c_int, POINTER(c_double)]),
        "sgprs_sched_run_periodic": (c_int, [vp, vp, POINTER(vp), c_int, POINTER(vp), POINTER(vp), c_int, POINTER(c_double), c_double,
                                             POINTER(RunReport)]),
    }
    for name, (res, args) in sig.items():
        f = getattr(L, name)
        f.restype, f.argtypes = res, args
    _lib = L
    return L


def _check(rc: int) -> int:
    if rc < 0:
        raise SgprsError(rc, lib().sgprs_last_error().decode())
    return rc


def _f32(a) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.float32)


def _fp(a: np.ndarray):
    return a.ctypes.data_as(POINTER(c_float))


def sgprs_version() -> int:
    return lib().sgprs_version()


def sgprs_status_string(status: int) -> str:
    return lib().sgprs_status_string(status).decode()


def sgprs_last_error() -> str:
    return lib().sgprs_last_error().decode()


def sgprs_kernel_name(kind: int, variant: int) -> str:
    return lib().sgprs_kernel_name(kind, variant).decode()


def sgprs_build_cu_mask(total_cus: int, n_xcd: int, cus: int, partition: int, blocked_layout: bool = False,
                        n_words: int | None = None) -> np.ndarray:
    n_words = (total_cus + 31) // 32 if n_words is None else n_words
    words = np.zeros(max(n_words, 1), dtype=np.uint32)
    _check(lib().sgprs_build_cu_mask(total_cus, n_xcd, cus, partition, int(blocked_layout),
                                     words.ctypes.data_as(POINTER(c_uint32)), n_words))
    return words


def sgprs_fold_bn(gamma, beta, mean, var, eps: float):
    g, b, m, v = _f32(gamma), _f32(beta), _f32(mean), _f32(var)
    c = g.shape[0]
    scale, shift = np.empty(c, np.float32), np.empty(c, np.float32)
    _check(lib().sgprs_fold_bn(_fp(g), _fp(b), _fp(m), _fp(v), eps, c, _fp(scale), _fp(shift)))
    return scale, shift


def sgprs_conv_packed_weight_bytes(desc: ConvDesc) -> int:
    n = c_size_t(0)
    _check(lib().sgprs_conv_packed_weight_bytes(ctypes.byref(desc), ctypes.byref(n)))
    return n.value


def sgprs_pack_conv_weights(desc: ConvDesc, w_oihw) -> np.ndarray:
    """Packed weights as a uint8 host array (copy it to the device as is)."""
    w = _f32(w_oihw)
    assert w.shape == (desc.cout, desc.cin, desc.r, desc.s), (w.shape, desc.cout, desc.cin, desc.r, desc.s)
    n = sgprs_conv_packed_weight_bytes(desc)
    out = np.zeros(n, dtype=np.uint8)
    _check(lib().sgprs_pack_conv_weights(ctypes.byref(desc), _fp(w), out.ctypes.data, n))
    return out


def sgprs_unpack_conv_weights(desc: ConvDesc, packed: np.ndarray) -> np.ndarray:
    packed = np.ascontiguousarray(packed, dtype=np.uint8)
    w = np.empty((desc.cout, desc.cin, desc.r, desc.s), dtype=np.float32)
    _check(lib().sgprs_unpack_conv_weights(ctypes.byref(desc), packed.ctypes.data, packed.size, _fp(w)))
    return w


def sgprs_conv2d_workspace(desc: ConvDesc, partition_cus: int) -> int:
    n = c_size_t(0)
    _check(lib().sgprs_conv2d_workspace(ctypes.byref(desc), partition_cus, ctypes.byref(n)))
    return n.value


def sgprs_conv2d_plan(desc: ConvDesc, partition_cus: int, has_residual: bool = False):
    """(family, detail) of the kernel sgprs_conv2d would launch."""
    fam, det = c_int(-1), c_int(-1)
    _check(lib().sgprs_conv2d_plan(ctypes.byref(desc), partition_cus, int(has_residual), ctypes.byref(fam), ctypes.byref(det)))
    return fam.value, det.value


class Pool:
    """Context pool CP: n_p partitions of `cus` compute units each."""

    def __init__(self, n_p: int, cus_per_partition: int, flags: int = 0, device: int = 0, masks=None):
        h = c_void_p()
        if masks is not None:
            m = np.ascontiguousarray(masks, dtype=np.uint32)
            assert m.ndim == 2 and m.shape[0] == n_p
            _check(lib().sgprs_pool_create_masks(device, n_p, m.ctypes.data_as(POINTER(c_uint32)), m.shape[1],
                                                 ctypes.byref(h)))
        else:
            _check(lib().sgprs_pool_create(device, n_p, cus_per_partition, flags, ctypes.byref(h)))
        self.handle = h

    def info(self):
        a, b, c, d = c_int(), c_int(), c_int(), c_int()
        _check(lib().sgprs_pool_info(self.handle, ctypes.byref(a), ctypes.byref(b), ctypes.byref(c), ctypes.byref(d)))
        return dict(n_p=a.value, cus_per_partition=b.value, total_cus=c.value, n_xcd=d.value)

    def partition_cus(self, p: int) -> int:
        c = c_int()
        _check(lib().sgprs_pool_partition_cus(self.handle, p, ctypes.byref(c)))
        return c.value

    def mask(self, p: int) -> np.ndarray:
        w = np.zeros(16, dtype=np.uint32)
        _check(lib().sgprs_pool_get_mask(self.handle, p, w.ctypes.data_as(POINTER(c_uint32)), 16))
        return w

    def stream(self, p: int) -> int:
        s = lib().sgprs_pool_stream(self.handle, p)
        if not s:
            raise SgprsError(-1, sgprs_last_error())
        return s

    def sync(self, p: int | None = None) -> None:
        _check(lib().sgprs_pool_sync(self.handle) if p is None else lib().sgprs_partition_sync(self.handle, p))

    def probe(self, p: int, n_blocks: int, spin_cycles: int, out_ptr: int) -> None:
        _check(lib().sgprs_partition_probe(self.handle, p, n_blocks, spin_cycles, out_ptr))

    def probe_graph(self, p: int, n_blocks: int, spin_cycles: int, out_ptr: int) -> None:
        _check(lib().sgprs_partition_probe_graph(self.handle, p, n_blocks, spin_cycles, out_ptr))

    def mfma_probe(self, p: int, random_data: bool, steps: int, out_ptr: int) -> None:
        _check(lib().sgprs_mfma_probe(self.handle, p, int(bool(random_data)), steps, out_ptr))

    def load_probe(self, p: int, buf_ptr: int, buf_bytes: int, region_bytes: int, iters: int, out_ptr: int) -> None:
        _check(lib().sgprs_load_probe(self.handle, p, buf_ptr, buf_bytes, region_bytes, iters, out_ptr))

    def run_static(self, tasks, input_ptrs, logits_ptrs, batch: int, partition_of_task, rounds: int, max_busy: int = 4) -> float:
        """sgprs_pool_run_static: seconds from the first launch to the last completion."""
        n = len(tasks)
        th = (c_void_p * n)(*[getattr(t.handle, "value", t.handle) for t in tasks])
        ins = (c_void_p * n)(*input_ptrs)
        outs = (c_void_p * n)(*logits_ptrs)
        parts = (c_int * n)(*[int(p) for p in partition_of_task])
        el = c_double()
        _check(lib().sgprs_pool_run_static(self.handle, th, n, ins, outs, batch, parts, rounds, max_busy, ctypes.byref(el)))
        return el.value

    def destroy(self) -> None:
        if self.handle:
            h, self.handle = self.handle, None
            _check(lib().sgprs_pool_destroy(h))

    def __del__(self):
        try:
            self.destroy()
        except Exception:
            pass


def _h(pool):
    return pool.handle if isinstance(pool, Pool) else pool


def sgprs_conv2d(desc: ConvDesc, x: int, w_packed: int, scale: int, shift: int, residual: int | None, y: int,
                 workspace: int | None, workspace_bytes: int, pool, partition: int) -> None:
    _check(lib().sgprs_conv2d(ctypes.byref(desc), x, w_packed, scale, shift, residual, y, workspace,
                              workspace_bytes, _h(pool), partition))


def sgprs_conv_tuning_override(kind: int, variant: int = 0, splits: int = 1) -> None:
    _check(lib().sgprs_conv_tuning_override(kind, variant, splits))


def sgprs_maxpool2d(dtype: int, n: int, h: int, w: int, c: int, x: int, y: int, pool, partition: int) -> None:
    _check(lib().sgprs_maxpool2d(dtype, n, h, w, c, x, y, _h(pool), partition))


def sgprs_bn_relu(dtype: int, pixels: int, c: int, x: int, scale: int, shift: int, y: int, pool,
                  partition: int) -> None:
    _check(lib().sgprs_bn_relu(dtype, pixels, c, x, scale, shift, y, _h(pool), partition))


def sgprs_add_relu(dtype: int, count: int, a: int, b: int, y: int, relu: bool, pool, partition: int) -> None:
    _check(lib().sgprs_add_relu(dtype, count, a, b, y, int(relu), _h(pool), partition))


def sgprs_avgpool_fc(dtype: int, n: int, hw: int, cin: int, cout: int, x: int, w: int, bias: int | None,
                     logits: int, workspace: int, pool, partition: int) -> None:
    _check(lib().sgprs_avgpool_fc(dtype, n, hw, cin, cout, x, w, bias, logits, workspace, _h(pool), partition))


def sgprs_global_avgpool(dtype: int, n: int, hw: int, c: int, x: int, pooled: int, pool, partition: int) -> None:
    _check(lib().sgprs_global_avgpool(dtype, n, hw, c, x, pooled, _h(pool), partition))


def sgprs_avgpool_fc_static(dtype: int, n: int, hw: int, cin: int, cout: int, x: int, w: int, bias: int | None,
                            logits: int, pool, partition: int) -> None:
    _check(lib().sgprs_avgpool_fc_static(dtype, n, hw, cin, cout, x, w, bias, logits, _h(pool), partition))


class Task:
    """Task tau_i: one ResNet18 instance with its six stages."""

    def __init__(self, params: dict, dtype: int, max_batch: int, eps: float, device: int = 0):
        keep = []
        P = _Params()

        def put(arr_field, i, a):
            a = _f32(a)
            keep.append(a)
            arr_field[i] = _fp(a)

        for i in range(20):
            put(P.conv_w, i, params["conv_w"][i])
            put(P.bn_gamma, i, params["gamma"][i])
            put(P.bn_beta, i, params["beta"][i])
            put(P.bn_mean, i, params["mean"][i])
            put(P.bn_var, i, params["var"][i])
        fw = _f32(params["fc_w"]); keep.append(fw); P.fc_w = _fp(fw)
        if params.get("fc_b") is not None:
            fb = _f32(params["fc_b"]); keep.append(fb); P.fc_b = _fp(fb)
        P.bn_eps = eps
        h = c_void_p()
        _check(lib().sgprs_task_create_resnet18(device, dtype, max_batch, ctypes.byref(P), ctypes.byref(h)))
        self.handle, self.dtype, self.max_batch = h, dtype, max_batch

    def num_stages(self) -> int:
        return _check(lib().sgprs_task_num_stages(self.handle))

    def stage_io(self, stage: int, batch: int):
        a, b = c_size_t(), c_size_t()
        i4, o4 = (c_int * 4)(), (c_int * 4)()
        _check(lib().sgprs_task_stage_io(self.handle, stage, batch, ctypes.byref(a), ctypes.byref(b), i4, o4))
        return dict(in_bytes=a.value, out_bytes=b.value, in_nchw=tuple(i4), out_nchw=tuple(o4))

    def stage_run(self, stage: int, batch: int, inp: int, out: int, pool, partition: int) -> None:
        _check(lib().sgprs_stage_run(self.handle, stage, batch, inp, out, _h(pool), partition))

    def run(self, batch: int, inp: int, logits: int, pool, partition: int, partition_per_stage=None) -> None:
        pps = (c_int * 6)(*partition_per_stage) if partition_per_stage is not None else None
        _check(lib().sgprs_task_run(self.handle, batch, inp, logits, _h(pool), partition, pps))

    def stage_output(self, stage: int) -> int:
        p = lib().sgprs_task_stage_output(self.handle, stage)
        if not p:
            raise SgprsError(-1, sgprs_last_error())
        return p

    def set_graph_replay(self, mode: int) -> None:
        """1 always, 0 never, -1 automatic (small batches)."""
        _check(lib().sgprs_task_set_graph_replay(self.handle, int(mode)))

    def set_profiling(self, on: bool) -> None:
        _check(lib().sgprs_task_set_profiling(self.handle, int(on)))

    def kernel_times(self, stage: int):
        cap = 64
        n = c_int(cap)
        kind, var = (c_int * cap)(), (c_int * cap)()
        ms = (c_float * cap)()
        fl, by = (c_double * cap)(), (c_double * cap)()
        _check(lib().sgprs_task_kernel_times(self.handle, stage, ctypes.byref(n), kind, var, ms, fl, by))
        return [dict(kind=kind[i], variant=var[i], ms=ms[i], flops=fl[i], bytes=by[i],
                     name=sgprs_kernel_name(kind[i], var[i])) for i in range(n.value)]

    def destroy(self) -> None:
        if self.handle:
            h, self.handle = self.handle, None
            _check(lib().sgprs_task_destroy(h))

    def __del__(self):
        try:
            self.destroy()
        except Exception:
            pass


class Sched:
    """sgprs_sched_*: the scheduler core (host logic; the caller supplies the clock)."""

    def __init__(self, n_contexts: int, lanes_per_context: int):
        h = c_void_p()
        _check(lib().sgprs_sched_create(n_contexts, lanes_per_context, ctypes.byref(h)))
        self.handle = h

    def add_task(self, wcet, period: float, rel_deadline: float) -> int:
        w = (c_double * len(wcet))(*[float(v) for v in wcet])
        tid = c_int()
        _check(lib().sgprs_sched_add_task(self.handle, len(wcet), w, period, rel_deadline, ctypes.byref(tid)))
        return tid.value

    def virtual_deadlines(self, task: int, n_stages: int):
        out = (c_double * n_stages)()
        _check(lib().sgprs_sched_virtual_deadlines(self.handle, task, n_stages, out))
        return list(out)

    def release(self, task: int, now: float) -> int:
        job = c_int()
        _check(lib().sgprs_sched_release(self.handle, task, now, ctypes.byref(job)))
        return job.value

    def next(self, now: float):
        d = Dispatch()
        return d if _check(lib().sgprs_sched_next(self.handle, now, ctypes.byref(d))) == 1 else None

    def complete(self, task: int, job: int, stage: int, now: float) -> bool:
        m = c_int()
        _check(lib().sgprs_sched_complete(self.handle, task, job, stage, now, ctypes.byref(m)))
        return bool(m.value)

    def run_periodic(self, pool, tasks, input_ptrs, logits_ptrs, batch: int, duration_s: float, offsets=None) -> dict:
        n = len(tasks)
        th = (c_void_p * n)(*[getattr(t.handle, "value", t.handle) for t in tasks])
        ins = (c_void_p * n)(*input_ptrs)
        outs = (c_void_p * n)(*logits_ptrs)
        off = (c_double * n)(*[float(v) for v in offsets]) if offsets is not None else None
        rep = RunReport()
        _check(lib().sgprs_sched_run_periodic(self.handle, _h(pool), th, n, ins, outs, batch, off, duration_s, ctypes.byref(rep)))
        out = {k: getattr(rep, k) for k in ("elapsed_s", "releases", "dropped", "fps", "dmr", "mean_response_s", "max_response_s")}
        out.update({k: int(getattr(rep.sched, k)) for k, _ in SchedStats._fields_})
        return out

    def set_max_busy(self, max_busy: int) -> None:
        _check(lib().sgprs_sched_set_max_busy(self.handle, max_busy))

    def stats(self) -> dict:
        st = SchedStats()
        _check(lib().sgprs_sched_get_stats(self.handle, ctypes.byref(st)))
        return {n: int(getattr(st, n)) for n, _ in SchedStats._fields_}

    def destroy(self) -> None:
        if self.handle:
            h, self.handle = self.handle, None
            lib().sgprs_sched_destroy(h)

    def __del__(self):
        try:
            self.destroy()
        except Exception:
            pass
