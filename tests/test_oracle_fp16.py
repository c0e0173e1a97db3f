"""Pins for the oracle's own fp16 <-> fp32 conversions (it cannot use _Float16 with this gcc)."""
import os

import numpy as np

from oracle import reference as R


def test_f16_to_f32_exhaustive():
    h = np.arange(65536, dtype=np.uint16)
    got = R.f16_to_f32(h)
    want = h.view(np.float16).astype(np.float32)
    nan = np.isnan(want)
    assert np.array_equal(got.view(np.uint32)[~nan], want.view(np.uint32)[~nan])
    assert np.isnan(got[nan]).all()


def test_f32_to_f16_hand_cases(golden_dir):
    rows = [ln.split() for ln in open(os.path.join(golden_dir, "fp16_rounding.txt")) if ln.strip() and ln[0] != "#"]
    f = np.array([int(r[0], 16) for r in rows], dtype=np.uint32).view(np.float32)
    want = np.array([int(r[1], 16) for r in rows], dtype=np.uint16)
    got = R.f32_to_f16(f).view(np.uint16)
    assert np.array_equal(got, want), [(rows[i], hex(got[i])) for i in np.nonzero(got != want)[0]]


def test_f32_to_f16_against_numpy():
    rng = np.random.default_rng(5)
    parts = [rng.standard_normal(200000).astype(np.float32) * s for s in (1e-8, 1e-5, 1e-3, 1.0, 30.0, 3e4, 1e6)]
    # every representable half, its neighbours' midpoints, and values a hair to either side
    h = np.arange(0x7C00, dtype=np.uint16).view(np.float16).astype(np.float64)
    mid = (h[:-1] + h[1:]) / 2
    parts += [h.astype(np.float32), mid.astype(np.float32),
              np.nextafter(mid.astype(np.float32), np.float32(np.inf)),
              np.nextafter(mid.astype(np.float32), np.float32(-np.inf))]
    f = np.concatenate(parts)
    f = np.concatenate([f, -f])
    with np.errstate(over="ignore"):
        want = f.astype(np.float16).view(np.uint16)
    got = R.f32_to_f16(f).view(np.uint16)
    assert np.array_equal(got, want)


def test_roundtrip_all_halves():
    h = np.arange(65536, dtype=np.uint16)
    f = R.f16_to_f32(h)
    back = R.f32_to_f16(f).view(np.uint16)
    finite_or_inf = ~np.isnan(f)
    assert np.array_equal(back[finite_or_inf], h[finite_or_inf])
