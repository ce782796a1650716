"""Pins for the oracle's Philox4x32-10 + Box-Muller sketch (Algorithm 1 step 1)."""
import os

import numpy as np
import pytest
from scipy import stats

from oracle import philox


def _kat(golden_dir):
    rows = []
    for line in open(os.path.join(golden_dir, "philox4x32_10_kat.txt")):
        if line.startswith("#") or not line.strip():
            continue
        rows.append([int(x, 16) for x in line.split()])
    return rows


def test_known_answer_vectors(golden_dir):
    rows = _kat(golden_dir)
    assert len(rows) == 3
    for w in rows:
        out = philox.philox4x32_10(np.array([w[:4]], dtype=np.uint64), w[4:6])[0]
        assert [int(x) for x in out] == w[6:]


def test_counter_and_key_layout():
    # group g of stream s under seed: counter (g lo, g hi, s, 0), key (seed lo, seed hi)
    seed, g, s = 0x0123456789ABCDEF, (5 << 32) | 77, 3
    a = philox.philox_groups(seed, g, 1, stream=s)[0]
    b = philox.philox4x32_10(np.array([[77, 5, 3, 0]], dtype=np.uint64), (0x89ABCDEF, 0x01234567))[0]
    assert (a == b).all()
    # the all-zero known-answer vector is group 0, stream 0, seed 0
    z = philox.philox_groups(0, 0, 1)[0]
    assert [int(x) for x in z] == [0x6627E8D5, 0xE169C58D, 0xBC57AC4C, 0x9B00DBD8]


def test_uniforms_open_interval_and_exact():
    x = np.array([[0, 0xFFFFFFFF, 0x80000000, 0x000000FF]], dtype=np.uint32)
    u32 = philox.uniforms(x, np.float32)[0]
    assert u32[0] == 2.0 ** -25 and u32[1] == 1.0 - 2.0 ** -25 and u32[3] == 2.0 ** -25
    u64 = philox.uniforms(x, np.float64)[0]
    assert u64[0] == ((0xFFFFFFFF >> 12) + 0.5) * 2.0 ** -52
    big = np.array([[0xFFFFFFFF] * 4, [0] * 4], dtype=np.uint32)
    for dt in (np.float32, np.float64):
        u = philox.uniforms(big, dt)
        assert (u > 0).all() and (u < 1).all()


@pytest.mark.parametrize("dtype", [np.float32, np.float64])
def test_element_order_and_box_muller_closed_form(dtype):
    n, l, seed = 37, 12, 9
    Om = philox.philox_normal(seed, n, l, dtype)
    assert Om.shape == (n, l) and Om.dtype == dtype
    per = 4 if dtype == np.float32 else 2
    flat = Om.reshape(-1).astype(np.float64)
    # element e = i*l + j lives in group e // per, lane e % per
    for e in (0, 1, 5, 130, n * l - 1):
        g, lane = divmod(e, per)
        u = philox.uniforms(philox.philox_groups(seed, g, 1), dtype)[0]
        pair = lane // 2
        r2 = -2.0 * np.log(u[2 * pair])
        ang = 2.0 * np.pi * u[2 * pair + 1]
        want = np.sqrt(r2) * (np.cos(ang) if lane % 2 == 0 else np.sin(ang))
        assert flat[e] == pytest.approx(want, rel=4 * np.finfo(dtype).eps, abs=1e-300)
    # closed form: z0^2 + z1^2 = -2 ln u0 for every Box-Muller pair
    ngr = (n * l) // per
    u = philox.uniforms(philox.philox_groups(seed, 0, ngr), dtype)
    z = flat[:ngr * per].reshape(ngr, per)
    tol = 16 * np.finfo(dtype).eps
    np.testing.assert_allclose(z[:, 0] ** 2 + z[:, 1] ** 2, -2 * np.log(u[:, 0]), rtol=tol, atol=tol)
    if per == 4:
        np.testing.assert_allclose(z[:, 2] ** 2 + z[:, 3] ** 2, -2 * np.log(u[:, 2]), rtol=tol, atol=tol)


@pytest.mark.parametrize("dtype", [np.float32, np.float64])
def test_gaussian_statistics(dtype):
    n, l = 4000, 100
    z = philox.philox_normal(1, n, l, dtype).astype(np.float64)
    N = z.size
    assert abs(z.mean()) < 5 / np.sqrt(N)
    assert abs(z.var() - 1) < 5 * np.sqrt(2 / N)
    assert abs(stats.kurtosis(z.ravel(), fisher=False) - 3) < 5 * np.sqrt(24 / N)
    assert abs(stats.skew(z.ravel())) < 5 * np.sqrt(6 / N)
    assert stats.kstest(z.ravel()[:200000], "norm").pvalue > 1e-3
    f = z.ravel()
    assert abs(np.corrcoef(f[:-1], f[1:])[0, 1]) < 5 / np.sqrt(N)        # lag-1
    assert abs(np.corrcoef(z[:, 0], z[:, 1])[0, 1]) < 5 / np.sqrt(n)     # across columns
    assert abs(np.corrcoef(z[0::2, 3], z[1::2, 3])[0, 1]) < 5 / np.sqrt(n / 2)


def test_seed_and_stream_separate_the_streams():
    a = philox.philox_normal(0, 16, 8, np.float64)
    b = philox.philox_normal(1, 16, 8, np.float64)
    c = philox.philox_normal(0, 16, 8, np.float64, stream=1)
    assert not np.allclose(a, b) and not np.allclose(a, c)
    assert (a == philox.philox_normal(0, 16, 8, np.float64)).all()
    # chunked generation is seamless
    big = philox.philox_normal(5, 300, 7, np.float32, chunk=64)
    assert (big == philox.philox_normal(5, 300, 7, np.float32)).all()
