"""Pins for the oracle's scale-word codec (SwExMy) against its definition and known formats."""
import numpy as np
import pytest

from oracle import pairsearch as ps

FORMATS = [(0, 4, 4), (1, 4, 3), (0, 4, 6), (1, 4, 5), (1, 5, 5), (0, 4, 3), (0, 8, 0)]


def test_ue4m4_landmarks():
    f = ps.make_fmt(0, 4, 4)
    assert f.bias == 7 and f.max_code == 255
    assert ps.scale_value(f, 0) == 0.0
    assert ps.scale_value(f, 1) == 2.0 ** -10            # smallest subnormal
    assert ps.scale_value(f, 16) == 2.0 ** -6            # smallest normal
    assert ps.scale_value(f, 255) == 496.0               # 1.9375 * 2^8
    f = ps.make_fmt(1, 4, 3)
    assert f.max_code == 127 and ps.scale_value(f, 127) == 480.0


def test_matches_ieee_half_and_bfloat():
    # E5M10 with bias 15 is IEEE binary16; E8M7 with bias 127 is bfloat16: the value rule must
    # reproduce numpy's decoding of the same bit patterns (finite codes only)
    f = ps.make_fmt(1, 5, 10)
    q = np.arange(0, 31 << 10)
    assert all(ps.scale_value(f, int(v)) == float(np.uint16(v).view(np.float16)) for v in q[::37])
    f = ps.make_fmt(1, 8, 7)
    for v in list(range(0, 255 << 7, 301)):
        assert ps.scale_value(f, v) == float((np.uint32(v) << np.uint32(16)).view(np.float32))


@pytest.mark.parametrize("w,x,y", FORMATS)
def test_monotone_and_round_trip(w, x, y):
    f = ps.make_fmt(w, x, y)
    v = np.array([ps.scale_value(f, q) for q in range(f.max_code + 1)])
    assert np.all(np.diff(v) > 0)
    step = max(1, (f.max_code + 1) // 512)
    for q in range(0, f.max_code + 1, step):
        assert ps.scale_encode(f, v[q]) == q == ps.scale_encode(f, v[q], exhaustive=True)


@pytest.mark.parametrize("w,x,y", FORMATS)
def test_midpoints_round_down_and_saturation(w, x, y):
    f = ps.make_fmt(w, x, y)
    v = np.array([ps.scale_value(f, q) for q in range(f.max_code + 1)])
    step = max(1, (f.max_code + 1) // 256)
    for q in range(0, f.max_code, step):
        mid = np.float32(0.5 * (v[q] + v[q + 1]))
        if float(mid) != 0.5 * (v[q] + v[q + 1]):
            continue                                   # midpoint not a binary32 number
        assert ps.scale_encode(f, mid) == q
        assert ps.scale_encode(f, np.nextafter(mid, np.float32(np.inf))) == q + 1
        assert ps.scale_encode(f, np.nextafter(mid, np.float32(-np.inf))) == q
    assert ps.scale_encode(f, np.float32(v[-1] * 4)) == f.max_code
    assert ps.scale_encode(f, np.float32(np.inf)) == f.max_code
    assert ps.scale_encode(f, np.float32(0.0)) == 0


@pytest.mark.parametrize("w,x,y", FORMATS)
def test_bisection_equals_exhaustive_scan(w, x, y):
    f = ps.make_fmt(w, x, y)
    rng = np.random.default_rng(5)
    lo, hi = ps.scale_value(f, 1), ps.scale_value(f, f.max_code)
    xs = np.exp(rng.uniform(np.log(lo / 8), np.log(min(hi * 8, 1e38)), 600)).astype(np.float32)
    for s in xs:
        assert ps.scale_encode(f, s) == ps.scale_encode(f, s, exhaustive=True)


def test_max_code_restriction():
    f = ps.make_fmt(1, 4, 3, max_code=0x7E)
    assert ps.scale_encode(f, np.float32(1e9)) == 0x7E
    assert ps.scale_value(f, 0x7E) == 448.0              # 1.75 * 2^8
