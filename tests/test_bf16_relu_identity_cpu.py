"""The conv epilogues apply the ReLU after the conversion to bf16, as a signed 16-bit maximum of
the bit pattern against 0 (and against the smallest 16-bit integer when there is no ReLU).  This
checks, on the CPU and for every bf16 neighbourhood that matters, the identity that makes it
legal: rounding to nearest even keeps the sign, so clamp-then-round equals round-then-clamp."""
import numpy as np


def bf16_rne_bits(x):
    u = np.asarray(x, dtype=np.float32).view(np.uint32).astype(np.uint64)
    r = (u + 0x7FFF + ((u >> 16) & 1)) >> 16
    return r.astype(np.uint16)


def test_relu_after_rounding_equals_relu_before_rounding():
    rng = np.random.default_rng(5)
    # every finite bf16 value, its two neighbours' midpoints and a little beyond them, plus noise
    pats = np.arange(0x10000, dtype=np.uint32)
    pats = pats[((pats >> 7) & 0xFF) != 0xFF]
    base = (pats << 16).astype(np.uint32)
    cand = np.concatenate([base, base + 0x7FFF, base + 0x8000, base + 0x8001, base + 1,
                           rng.integers(0, 1 << 32, 1 << 20, dtype=np.uint64).astype(np.uint32)])
    x = cand.view(np.float32)
    x = x[np.isfinite(x)]
    before = bf16_rne_bits(np.maximum(x, np.float32(0.0)))
    after = np.maximum(bf16_rne_bits(x).view(np.int16), np.int16(0)).view(np.uint16)
    # max(-0.0, 0.0) may keep either zero in numpy: compare with the sign of zero cleared
    before = np.where(before == 0x8000, 0, before)
    assert np.array_equal(before, after)
    # without a ReLU the floor is the smallest int16: every pattern passes unchanged
    plain = bf16_rne_bits(x)
    assert np.array_equal(np.maximum(plain.view(np.int16), np.int16(-32768)).view(np.uint16), plain)
