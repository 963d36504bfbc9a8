"""Pins for the oracle's own binary16 / bfloat16 decoders: every one of the 65536 patterns
against an independent conversion (numpy's float16, torch's bfloat16)."""
import numpy as np
import torch

import oracle


def _all_bits():
    return np.arange(65536, dtype=np.uint32).astype(np.uint16)


def test_f16_decoder_all_patterns_vs_numpy():
    b = _all_bits()
    got = oracle.decode(b, oracle.F16)
    want = b.view(np.float16).astype(np.float64)
    nan = np.isnan(want)
    assert np.array_equal(np.isnan(got), nan)
    assert np.array_equal(got[~nan], want[~nan])
    assert np.array_equal(np.signbit(got[~nan]), np.signbit(want[~nan]))   # -0.0 keeps its sign


def test_bf16_decoder_all_patterns_vs_torch():
    b = _all_bits()
    got = oracle.decode(b, oracle.BF16)
    want = torch.from_numpy(b.view(np.int16)).view(torch.bfloat16).to(torch.float64).numpy()
    nan = np.isnan(want)
    assert np.array_equal(np.isnan(got), nan)
    assert np.array_equal(got[~nan], want[~nan])
    assert np.array_equal(np.signbit(got[~nan]), np.signbit(want[~nan]))


def test_bf16_is_top_half_of_fp32():
    # closed form: a bfloat16 pattern is the upper 16 bits of the fp32 with the same value
    b = _all_bits()
    with np.errstate(invalid="ignore"):
        f32 = (b.astype(np.uint32) << 16).view(np.float32).astype(np.float64)
    got = oracle.decode(b, oracle.BF16)
    ok = ~np.isnan(f32)
    assert np.array_equal(got[ok], f32[ok])


def test_known_values():
    # textbook constants of the two formats
    f = lambda h: float(oracle.decode(np.array([h], dtype=np.uint16), oracle.F16)[0])
    g = lambda h: float(oracle.decode(np.array([h], dtype=np.uint16), oracle.BF16)[0])
    assert f(0x3C00) == 1.0 and f(0xC000) == -2.0 and f(0x7BFF) == 65504.0
    assert f(0x0001) == 2.0 ** -24 and f(0x0400) == 2.0 ** -14 and f(0x7C00) == float("inf")
    assert g(0x3F80) == 1.0 and g(0xC000) == -2.0 and g(0x0080) == 2.0 ** -126
    assert g(0x0001) == 2.0 ** -133 and g(0x7F80) == float("inf")
