"""Pins for the oracle's number formats and quantizers (CPU only).

Each check compares the oracle with something other than itself: numpy / torch
conversions (library routines), closed forms of the formats, brute force over the
whole code space, hand-worked rows, and the error bounds the definitions imply.
"""
import numpy as np
import pytest

import oracle


def _all_f16():
    return np.arange(65536, dtype=np.uint16)


def test_f16_decode_matches_numpy_on_all_codes():
    bits = _all_f16()
    ref = bits.view(np.float16).astype(np.float32)
    got = np.array([oracle.f16_to_f32(int(b)) for b in bits], dtype=np.float32)
    nan = np.isnan(ref)
    assert np.array_equal(np.isnan(got), nan)
    assert np.array_equal(got[~nan].view(np.uint32), ref[~nan].view(np.uint32))


def test_f16_encode_matches_numpy():
    bits = _all_f16()
    vals = bits.view(np.float16).astype(np.float32)
    finite = np.isfinite(vals)
    # exact values, midpoints between neighbours (ties), and points just off the midpoints
    pos = np.sort(vals[finite & (vals >= 0)])
    mids = ((pos[:-1].astype(np.float64) + pos[1:].astype(np.float64)) / 2).astype(np.float32)
    rng = np.random.default_rng(7)
    rnd = (rng.standard_normal(20000) * np.exp(rng.uniform(-20, 12, 20000))).astype(np.float32)
    extra = np.array([65504.0, 65519.99, 65520.0, 70000.0, 1e-8, 2.9802322e-08, 2.98e-8, 5.9604645e-08, 6.1e-5,
                      6.1035156e-05, 6.0975552e-05, 0.0, -0.0], dtype=np.float32)
    xs = np.concatenate([vals[finite], mids, np.nextafter(mids, np.float32(0)), np.nextafter(mids, np.float32(1e9)),
                         -mids, rnd, extra])
    with np.errstate(over="ignore"):
        ref = xs.astype(np.float16).view(np.uint16)
    got = np.array([oracle.f32_to_f16(float(x)) for x in xs], dtype=np.uint16)
    assert np.array_equal(got, ref)


def _e4m3_closed_form():
    t = np.empty(256, np.float64)
    for b in range(256):
        s, e, m = b >> 7, (b >> 3) & 15, b & 7
        if e == 15 and m == 7:
            v = np.nan
        elif e == 0:
            v = 2.0 ** -6 * m / 8
        else:
            v = 2.0 ** (e - 7) * (1 + m / 8)
        t[b] = -v if s else v
    return t


def test_e4m3_decode_closed_form_and_torch():
    torch = pytest.importorskip("torch")
    t = _e4m3_closed_form()
    got = np.array([oracle.e4m3_decode(b) for b in range(256)], dtype=np.float64)
    assert np.array_equal(np.isnan(got), np.isnan(t))
    ok = ~np.isnan(t)
    assert np.array_equal(got[ok], t[ok])
    assert got[0x7E] == 448.0 and got[0x01] == 2.0 ** -9 and got[0x08] == 2.0 ** -6
    tt = torch.arange(256, dtype=torch.uint8).view(torch.float8_e4m3fn).to(torch.float32).numpy().astype(np.float64)
    assert np.array_equal(got[ok], tt[ok])


def _brute_force_e4m3(y):
    """Nearest finite E4M3 code by exhaustive search; ties to the even code; saturating."""
    t = _e4m3_closed_form()
    mags = t[:0x7F]  # codes 0..0x7E, non-negative, increasing
    a = abs(float(y))
    if a >= 448.0:
        code = 0x7E
    else:
        d = np.abs(mags - a)
        best = np.flatnonzero(d == d.min())
        code = int(best[0]) if len(best) == 1 else int([c for c in best if c % 2 == 0][0])
    return code | (0x80 if np.signbit(y) else 0)


def test_e4m3_encode_all_fp16_inputs_and_midpoints():
    bits = _all_f16()
    vals = bits.view(np.float16).astype(np.float32)
    vals = vals[np.isfinite(vals)]
    t = _e4m3_closed_form()
    mags = t[:0x7F]
    mids = (mags[:-1] + mags[1:]) / 2  # exactly representable in fp32
    xs = np.concatenate([vals, mids.astype(np.float32), -mids.astype(np.float32),
                         np.nextafter(mids.astype(np.float32), np.float32(0)),
                         np.nextafter(mids.astype(np.float32), np.float32(1e9)),
                         np.array([448.0, 449.0, 463.9, 464.0, 1e6, -1e6, 0.0, -0.0, 1e-12, -1e-12], np.float32)])
    # brute force is slow in python: vectorise it here independently of the oracle's search
    a = np.abs(xs.astype(np.float64))
    d = np.abs(a[:, None] - mags[None, :])
    dmin = d.min(axis=1, keepdims=True)
    is_min = d == dmin
    first = is_min.argmax(axis=1)
    two = is_min.sum(axis=1) == 2
    code = np.where(two & (first % 2 == 1), first + 1, first)
    code = np.where(a >= 448.0, 0x7E, code)
    ref = (code | np.where(np.signbit(xs), 0x80, 0)).astype(np.uint8)
    got = np.array([oracle.e4m3_encode(float(x)) for x in xs], dtype=np.uint8)
    assert np.array_equal(got, ref)
    # spot-check the vectorised reference against the scalar brute force
    for x in [0.3, -0.3, 17.0, 447.0, 0.001, 2.0 ** -10, 3 * 2.0 ** -10]:
        assert _brute_force_e4m3(np.float32(x)) == oracle.e4m3_encode(float(np.float32(x)))
    # known ties: 2^-10 is halfway between 0 and 2^-9 -> even code 0; 3*2^-10 -> code 2
    assert oracle.e4m3_encode(2.0 ** -10) == 0 and oracle.e4m3_encode(3 * 2.0 ** -10) == 2
    assert oracle.e4m3_encode(-0.0) == 0x80 and oracle.e4m3_encode(-1e-12) == 0x80


def test_e4m3_encode_matches_torch_cast_in_range():
    torch = pytest.importorskip("torch")
    rng = np.random.default_rng(3)
    xs = np.concatenate([rng.standard_normal(20000) * np.exp(rng.uniform(-8, 5, 20000)),
                         rng.uniform(-448, 448, 5000)]).astype(np.float32)
    xs = xs[np.abs(xs) <= 448]
    ref = torch.from_numpy(xs).to(torch.float8_e4m3fn).view(torch.uint8).numpy()
    got = np.array([oracle.e4m3_encode(float(x)) for x in xs], dtype=np.uint8)
    assert np.array_equal(got, ref)


def _f16(bits):
    return float(np.uint16(bits).view(np.float16))


def test_int8_hand_worked_rows():
    # amax 127 -> scale exactly 1: codes are the half-even roundings of the inputs
    q, s = oracle.quant_row_int8([127.0, -64.0, 0.4, 0.5, 1.5, 2.5, -2.5, -127.0])
    assert _f16(s) == 1.0 and q.tolist() == [127, -64, 0, 0, 2, 2, -2, -127]
    # amax 254 -> scale 2
    q, s = oracle.quant_row_int8([254.0, 3.0, -5.0, 1.0])
    assert _f16(s) == 2.0 and q.tolist() == [127, 2, -2, 0]  # 1.5->2, -2.5->-2, 0.5->0
    # all-zero row: scale falls back to 1, codes 0
    q, s = oracle.quant_row_int8(np.zeros(16))
    assert _f16(s) == 1.0 and not q.any()
    # scale underflowing fp16 to zero also falls back to 1
    q, s = oracle.quant_row_int8(np.full(8, 1e-9))
    assert _f16(s) == 1.0 and not q.any()
    # constant row: every code is +-127
    q, s = oracle.quant_row_int8(np.full(8, -3.0))
    assert set(q.tolist()) == {-127}


def test_int8_error_bound_and_idempotence():
    rng = np.random.default_rng(11)
    for _ in range(300):
        D = int(rng.choice([8, 64, 128]))
        x = (rng.standard_normal(D) * np.exp(rng.uniform(-6, 6))).astype(np.float32)
        q, s = oracle.quant_row_int8(x)
        sf = _f16(s)
        xh = q.astype(np.float64) * sf
        amax = np.abs(x).max()
        assert abs(sf - amax / 127) <= amax / 127 * 2.0 ** -10  # fp16 rounding of the scale
        assert np.all(np.abs(x - xh) <= sf * (0.5 + 127 * 2.0 ** -10) + 1e-30)
        assert np.abs(q).max() == 127
        q2, s2 = oracle.quant_row_int8(xh.astype(np.float32))
        assert s2 == s and np.array_equal(q2, q)


def test_int4_hand_worked_rows():
    # range [0, 15] -> scale 1, zero-point 0
    q, s, z = oracle.quant_row_int4([0.0, 15.0, 7.5, 2.5, 3.5, 14.6])
    assert _f16(s) == 1.0 and _f16(z) == 0.0
    codes = [(int(b) >> sh) & 15 for b in q for sh in (0, 4)]
    assert codes == [0, 15, 8, 2, 4, 15]
    # range [-5, 10] -> scale 1, zero-point 5, codes x+5
    q, s, z = oracle.quant_row_int4([-5.0, 10.0, 0.0, -1.0, 3.0, 9.0])
    assert _f16(s) == 1.0 and _f16(z) == 5.0
    assert [(int(b) >> sh) & 15 for b in q for sh in (0, 4)] == [0, 15, 5, 4, 8, 14]
    # packing: element 2j in the low nibble
    assert q[0] == (0 | (15 << 4))
    # all-positive row: the range is widened to include 0, zero-point 0
    q, s, z = oracle.quant_row_int4([30.0, 15.0])
    assert _f16(s) == 2.0 and _f16(z) == 0.0 and q[0] == (15 | (8 << 4))  # 7.5 -> 8 (half-even)
    # all-negative row: zero-point 15
    q, s, z = oracle.quant_row_int4([-30.0, -16.0])
    assert _f16(s) == 2.0 and _f16(z) == 15.0 and q[0] == (0 | (7 << 4))
    # all-zero row
    q, s, z = oracle.quant_row_int4(np.zeros(8))
    assert _f16(s) == 1.0 and _f16(z) == 0.0 and not q.any()


def test_int4_error_bound_and_idempotence():
    rng = np.random.default_rng(13)
    for _ in range(300):
        D = int(rng.choice([8, 64, 128]))
        x = (rng.standard_normal(D) * np.exp(rng.uniform(-6, 6)) + rng.uniform(-1, 1)).astype(np.float32)
        q, s, z = oracle.quant_row_int4(x)
        sf, zf = _f16(s), _f16(z)
        assert zf == int(zf) and 0 <= zf <= 15
        codes = np.array([(int(b) >> sh) & 15 for b in q for sh in (0, 4)], dtype=np.float64)
        xh = (codes - zf) * sf
        # the zero-point is rounded, so the clipped end of the range can be off by up to one step
        assert np.all(np.abs(x - xh) <= sf * 1.02 + 1e-30)
        inner = (x > (0 - zf + 0.5) * sf) & (x < (15 - zf - 0.5) * sf)
        assert np.all(np.abs(x - xh)[inner] <= sf * 0.5 * (1 + 2.0 ** -9) + 1e-30)
        q2, s2, z2 = oracle.quant_row_int4(xh.astype(np.float32))
        assert (s2, z2) == (s, z) and np.array_equal(q2, q)
