"""Pins for the 16-bit storage oracle: torch's own conversions (an independent library routine),
hand-picked ties, and the properties of a correct rounding."""
import numpy as np
import pytest
import torch

from oracle import storage as st
from paper_2302_13053_amd import workloads as wl


def specials():
    f = np.float32
    vals = [0.0, -0.0, 1.0, -1.0, 65504.0, 65520.0, 65536.0, 1e-8, 6e-8, 5.96e-8, 2.98e-8, 2.99e-8, 1e-40, 3.4e38, 3.39e38,
            np.inf, -np.inf, 1 + 2.0 ** -8, 1 + 3 * 2.0 ** -8, 1 + 2.0 ** -9, 1 + 2.0 ** -11, 1 + 3 * 2.0 ** -11,
            1 + 2.0 ** -8 + 2.0 ** -20, 0.1, -0.3, 2.0 ** -126, 2.0 ** -133, 2.0 ** -24, 2.0 ** -25, 1.5 * 2.0 ** -25]
    return np.array(vals, f)


@pytest.mark.parametrize("fmt,tt", [("bf16", torch.bfloat16), ("fp16", torch.float16)])
def test_store_matches_torch_conversion(fmt, tt):
    x = np.concatenate([specials(), wl.random_matrix(200, 50, 3).ravel() * np.float32(3.0),
                        (wl.random_matrix(50, 50, 4).ravel() * np.float32(1e-6)),
                        (wl.random_matrix(50, 50, 5).ravel() * np.float32(1e5))])
    got = st.store(x, fmt)
    ref = torch.from_numpy(x).to(tt).view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(got, ref)
    back = st.load(got, fmt)
    assert np.array_equal(back, torch.from_numpy(x).to(tt).to(torch.float32).numpy())


def test_ties_go_to_even_and_nan_stays_nan():
    f = np.float32
    # bf16 keeps 8 significant bits: 1 + 2^-8 lies halfway between 1 and 1 + 2^-7 -> even (1.0);
    # 1 + 3*2^-8 halfway between 1 + 2^-7 and 1 + 2^-6 -> even (1 + 2^-6)
    assert st.load(st.store(f(1 + 2.0 ** -8), "bf16"), "bf16") == f(1.0)
    assert st.load(st.store(f(1 + 3 * 2.0 ** -8), "bf16"), "bf16") == f(1 + 2.0 ** -6)
    assert st.load(st.store(f(1 + 2.0 ** -8 + 2.0 ** -20), "bf16"), "bf16") == f(1 + 2.0 ** -7)
    # fp16 keeps 11 significant bits
    assert st.load(st.store(f(1 + 2.0 ** -11), "fp16"), "fp16") == f(1.0)
    assert st.load(st.store(f(1 + 3 * 2.0 ** -11), "fp16"), "fp16") == f(1 + 2.0 ** -9)
    assert st.load(st.store(f(65520.0), "fp16"), "fp16") == np.inf          # halfway to 2^16 rounds up to infinity
    assert st.load(st.store(f(3.4e38), "bf16"), "bf16") == np.inf
    for fmt in ("bf16", "fp16"):
        assert np.isnan(st.load(st.store(f(np.nan), fmt), fmt))
        assert st.store(f(-0.0), fmt) == 0x8000


@pytest.mark.parametrize("fmt,bits", [("bf16", 8), ("fp16", 11)])
def test_rounding_is_nearest_and_idempotent(fmt, bits):
    x = wl.random_matrix(300, 40, 9).ravel()
    y = st.load(st.store(x, fmt), fmt)
    assert np.all(np.abs(y - x) <= np.abs(x) * 2.0 ** -bits)               # half an ulp of the target format
    assert np.array_equal(st.store(y, fmt), st.store(x, fmt))              # stored values are fixed points
    # monotone
    xs = np.sort(x)
    assert np.all(np.diff(st.load(st.store(xs, fmt), fmt)) >= 0)
