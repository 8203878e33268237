"""Seeded synthetic tensors with the shapes of the ResNet18 benchmark task.

The paper's benchmark task is a ResNet18 forward pass on a 224x224 input
(section "Simulation Results"), split into six stages; it ships no weights and
no data set, so seeded synthetic tensors are the workload.  Recipe:

* generator: numpy ``Generator(PCG64(SeedSequence(ENTROPY, spawn_key=(config,
  instance, tensor_id))))``, drawn in fp64, stored as fp32;
* inputs: N(0,1) (``|N(0,1)|`` for the single-block configuration);
* conv / FC weights: He-normal, std = sqrt(2 / fan_in), fan_in = Cin*R*S;
* BN: gamma ~ U[0.5,1.5], beta ~ N(0,0.1), mean ~ N(0,0.1), var ~ U[0.5,1.5]
  (0.1 is a standard deviation), eps = 1e-5;
* FC bias ~ N(0,0.1).

tensor_id 0 is the input; conv i (forward order) owns ids 1+5i .. 5+5i for
weight, gamma, beta, mean, var; the FC weight and bias are 101 and 102.

For the bf16 configurations the fp32 draws are rounded to the nearest bf16
(ties to even) here, so that the oracle and the HIP path are handed the very
same values.
"""
from __future__ import annotations

import numpy as np

ENTROPY = 240609425
BN_EPS = 1e-5
NUM_CLASSES = 1000
FC_IN = 512

# (name, cin, cout, kernel, stride, pad, hin) in forward order; square maps.
CONV_SPECS = [
    ("stem", 3, 64, 7, 2, 3, 224),
    ("layer1.0.conv1", 64, 64, 3, 1, 1, 56),
    ("layer1.0.conv2", 64, 64, 3, 1, 1, 56),
    ("layer1.1.conv1", 64, 64, 3, 1, 1, 56),
    ("layer1.1.conv2", 64, 64, 3, 1, 1, 56),
    ("layer2.0.conv1", 64, 128, 3, 2, 1, 56),
    ("layer2.0.conv2", 128, 128, 3, 1, 1, 28),
    ("layer2.0.down", 64, 128, 1, 2, 0, 56),
    ("layer2.1.conv1", 128, 128, 3, 1, 1, 28),
    ("layer2.1.conv2", 128, 128, 3, 1, 1, 28),
    ("layer3.0.conv1", 128, 256, 3, 2, 1, 28),
    ("layer3.0.conv2", 256, 256, 3, 1, 1, 14),
    ("layer3.0.down", 128, 256, 1, 2, 0, 28),
    ("layer3.1.conv1", 256, 256, 3, 1, 1, 14),
    ("layer3.1.conv2", 256, 256, 3, 1, 1, 14),
    ("layer4.0.conv1", 256, 512, 3, 2, 1, 14),
    ("layer4.0.conv2", 512, 512, 3, 1, 1, 7),
    ("layer4.0.down", 256, 512, 1, 2, 0, 14),
    ("layer4.1.conv1", 512, 512, 3, 1, 1, 7),
    ("layer4.1.conv2", 512, 512, 3, 1, 1, 7),
]

# per-image (C, H, W) at the input and output of each of the six stages
STAGE_IO = [
    ((3, 224, 224), (64, 56, 56)),
    ((64, 56, 56), (64, 56, 56)),
    ((64, 56, 56), (128, 28, 28)),
    ((128, 28, 28), (256, 14, 14)),
    ((256, 14, 14), (512, 7, 7)),
    ((512, 7, 7), (NUM_CLASSES, 1, 1)),
]

# the six isolated operators of the CU-scaling sweep (batch 1)
SWEEP_OPS = {
    "conv3x3_256": dict(cin=256, cout=256, k=3, stride=1, pad=1, h=14),
    "conv7x7_stem": dict(cin=3, cout=64, k=7, stride=2, pad=3, h=224),
    "maxpool": dict(c=64, h=112),
    "bn_relu": dict(c=128, h=28),
    "add": dict(c=512, h=7),
    "avgpool_fc": dict(c=512, h=7, out=1000),
}


def conv_out_hw(h: int, k: int, stride: int, pad: int) -> int:
    return (h + 2 * pad - k) // stride + 1


def rng_for(config: int, instance: int, tensor_id: int) -> np.random.Generator:
    ss = np.random.SeedSequence(entropy=ENTROPY, spawn_key=(config, instance, tensor_id))
    return np.random.Generator(np.random.PCG64(ss))


def bf16_bits(a: np.ndarray) -> np.ndarray:
    """fp32 -> bf16 bit patterns (uint16), round to nearest, ties to even."""
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32).astype(np.uint64)
    lsb = (u >> 16) & 1
    r = (u + 0x7FFF + lsb) >> 16
    return r.astype(np.uint16)


def bf16_from_bits(b: np.ndarray) -> np.ndarray:
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << 16).view(np.float32)


def round_to_bf16(a: np.ndarray) -> np.ndarray:
    """fp32 array whose values are all exactly representable in bf16."""
    return bf16_from_bits(bf16_bits(a)).reshape(np.shape(a))


def _finish(a64: np.ndarray, bf16: bool) -> np.ndarray:
    a = a64.astype(np.float32)
    return round_to_bf16(a) if bf16 else a


def make_input(config: int, instance: int, shape, dist: str = "normal", bf16: bool = False,
               tensor_id: int = 0) -> np.ndarray:
    """Input tensor in logical NCHW order, fp32."""
    g = rng_for(config, instance, tensor_id)
    a = g.standard_normal(size=tuple(shape))
    if dist == "absnormal":
        a = np.abs(a)
    elif dist != "normal":
        raise ValueError(dist)
    return _finish(a, bf16)


def make_conv_weight(config: int, instance: int, tensor_id: int, cout: int, cin: int, k: int,
                     bf16: bool = False) -> np.ndarray:
    """He-normal OIHW weight, std = sqrt(2 / (cin*k*k))."""
    g = rng_for(config, instance, tensor_id)
    std = np.sqrt(2.0 / (cin * k * k))
    return _finish(g.standard_normal(size=(cout, cin, k, k)) * std, bf16)


def make_bn(config: int, instance: int, first_tensor_id: int, c: int):
    """(gamma, beta, mean, var) fp32 vectors; ids first_tensor_id .. +3."""
    gamma = rng_for(config, instance, first_tensor_id).uniform(0.5, 1.5, size=c)
    beta = rng_for(config, instance, first_tensor_id + 1).standard_normal(size=c) * 0.1
    mean = rng_for(config, instance, first_tensor_id + 2).standard_normal(size=c) * 0.1
    var = rng_for(config, instance, first_tensor_id + 3).uniform(0.5, 1.5, size=c)
    return tuple(v.astype(np.float32) for v in (gamma, beta, mean, var))


def make_resnet18_params(config: int, instance: int, bf16: bool = False) -> dict:
    """All parameters of one ResNet18 instance as fp32 numpy arrays.

    keys: conv_w[20] (OIHW), gamma/beta/mean/var[20], fc_w (1000x512), fc_b.
    With bf16=True the conv and FC weights are bf16-representable; BN
    statistics and the FC bias stay fp32 (they are applied in fp32).
    """
    p = dict(conv_w=[], gamma=[], beta=[], mean=[], var=[])
    for i, (_, cin, cout, k, _, _, _) in enumerate(CONV_SPECS):
        base = 1 + 5 * i
        p["conv_w"].append(make_conv_weight(config, instance, base, cout, cin, k, bf16))
        g, b, m, v = make_bn(config, instance, base + 1, cout)
        p["gamma"].append(g); p["beta"].append(b); p["mean"].append(m); p["var"].append(v)
    gw = rng_for(config, instance, 101)
    p["fc_w"] = _finish(gw.standard_normal(size=(NUM_CLASSES, FC_IN)) * np.sqrt(2.0 / FC_IN), bf16)
    gb = rng_for(config, instance, 102)
    p["fc_b"] = (gb.standard_normal(size=NUM_CLASSES) * 0.1).astype(np.float32)
    return p
