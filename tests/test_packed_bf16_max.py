"""The premise of the library's packed pooling (csrc/bf16_common.h, bf16x2_max): of two bf16 bit patterns that are
finite numbers in both formats, the one that is larger read as fp16 is the one that is larger read as bf16, so an
fp16 maximum on the raw bits returns the bf16 maximum bit for bit.  Checked here on the CPU over every pair of a
grid of patterns that spans signs, zeros, half-denormal patterns and the largest admissible magnitudes."""
import numpy as np


def bf16_value(bits):
    return (bits.astype(np.uint32) << 16).view(np.float32).astype(np.float64)


def test_fp16_order_equals_bf16_order_on_shared_finite_patterns():
    rng = np.random.default_rng(7)
    mags = np.unique(np.concatenate([np.arange(0, 0x0500), rng.integers(0, 0x7C00, 3000), np.arange(0x7B00, 0x7C00)])).astype(np.uint16)
    pats = np.concatenate([mags, mags | np.uint16(0x8000)])               # finite as fp16: magnitude bits below 0x7C00
    a, b = np.meshgrid(pats[::7], pats, indexing="ij")
    a, b = a.ravel(), b.ravel()
    with np.errstate(all="ignore"):
        m16 = np.maximum(a.view(np.float16), b.view(np.float16)).view(np.uint16)
    va, vb = bf16_value(a), bf16_value(b)
    want = np.where(va >= vb, a, b)
    same_value = bf16_value(m16) == bf16_value(want)                      # +0 / -0 may come back either way
    assert same_value.all()
    differ = m16 != want
    assert (bf16_value(m16[differ]) == 0).all()                           # only the two zeros are interchangeable


def test_padding_pattern_is_below_every_activation_and_finite_as_fp16():
    low = np.array([0xFBFF], np.uint16)
    assert np.isfinite(low.view(np.float16)[0]) and low.view(np.float16)[0] == -65504.0
    assert bf16_value(low)[0] < -2.6e36
