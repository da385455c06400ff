"""Pins of the FP8 E4M3 reference (oracle/fp8_e4m3.py) against things it does not compute itself:
values the OCP 8-bit floating point specification fixes, PyTorch's own float8_e4m3fn conversions, and
brute force over all codes.  CPU only."""
import numpy as np
import pytest
import torch

from oracle import fp8_e4m3 as F8


def test_decode_values_fixed_by_the_format():
    t = F8.decode_table()
    # bias 7, 3 mantissa bits, subnormals m * 2^-9, largest finite 448, NaN only at S.1111.111
    fixed = {0x00: 0.0, 0x01: 2.0 ** -9, 0x07: 7 * 2.0 ** -9, 0x08: 2.0 ** -6, 0x09: 1.125 * 2.0 ** -6, 0x38: 1.0, 0x3C: 1.5,
             0x40: 2.0, 0x77: 1.875 * 128, 0x78: 256.0, 0x7E: 448.0, 0xB8: -1.0, 0xFE: -448.0, 0x81: -(2.0 ** -9)}
    for code, val in fixed.items():
        assert t[code] == val, hex(code)
    assert np.isnan(t[0x7F]) and np.isnan(t[0xFF]) and np.isfinite(np.delete(t, [0x7F, 0xFF])).all()
    assert t[0x80] == 0.0 and np.signbit(t[0x80])
    assert np.all(np.diff(t[:127]) > 0)  # codes of one sign are ordered like their values


def test_decode_equals_pytorch_float8_e4m3fn():
    codes = torch.arange(256, dtype=torch.int32).to(torch.uint8)
    ref = codes.view(torch.float8_e4m3fn).to(torch.float32).numpy().astype(np.float64)
    got = F8.decode(codes.numpy())
    assert np.array_equal(np.isnan(ref), np.isnan(got))
    ok = ~np.isnan(ref)
    assert np.array_equal(ref[ok], got[ok]) and np.array_equal(np.signbit(ref[ok]), np.signbit(got[ok]))


def probe_values():
    t = F8.decode_table()[:127]
    mids = 0.5 * (t[1:] + t[:-1])
    rng = np.random.default_rng(7)
    rnd = rng.uniform(-1, 1, 20000) * 2.0 ** rng.integers(-12, 9, 20000)
    x = np.concatenate([t, mids, mids * (1 + 2.0 ** -20), mids * (1 - 2.0 ** -20), rnd, [2.0 ** -10, 2.0 ** -10 * 1.001, 2.0 ** -11]])
    x = np.concatenate([x, -x]).astype(np.float32).astype(np.float64)
    return x[np.abs(x) <= 448.0]


def test_encode_equals_pytorch_round_to_nearest_even():
    x = probe_values()
    ref = torch.from_numpy(x.astype(np.float32)).to(torch.float8_e4m3fn).view(torch.uint8).numpy()
    got = F8.encode(x)
    nz = x != 0  # the sign of a zero result is compared through the value
    assert np.array_equal(F8.decode(got), F8.decode(ref))
    assert np.array_equal(got[nz] & 0x80, ref[nz] & 0x80)


def test_encode_is_the_nearest_code_with_ties_to_even_by_brute_force():
    x = probe_values()[::7]
    t = F8.decode_table()
    finite = np.array([c for c in range(256) if not np.isnan(t[c])])
    got = F8.encode(x)
    dist = np.abs(x[:, None] - t[finite][None, :])
    best = dist.min(axis=1)
    assert np.array_equal(np.abs(x - t[got]), best)          # a nearest one
    tie = (dist == best[:, None]).sum(axis=1) > 1
    tie &= x != 0
    assert tie.any() and np.all((got[tie] & 1) == 0)         # of two nearest, the even mantissa
    assert np.array_equal(F8.encode(t[finite]), np.where(finite == 0x80, 0x80, finite))  # codes are fixed points


def test_encode_saturates():
    assert list(F8.encode(np.array([449.0, 464.0, 480.0, 1e6, -1e6, -500.0]))) == [0x7E, 0x7E, 0x7E, 0x7E, 0xFE, 0xFE]


def test_scale_exponent_is_the_smallest_that_fits():
    rng = np.random.default_rng(3)
    pw = 2.0 ** np.arange(-60, 61)
    amax = np.concatenate([pw, 448 * pw, np.nextafter(448 * pw, np.inf), np.nextafter(448 * pw, 0), rng.uniform(0.1, 1, 500) * 2.0 ** rng.integers(-40, 40, 500)])
    e = F8.scale_exponent(amax)
    assert np.all(np.ldexp(amax, -e) <= 448.0) and np.all(np.ldexp(amax, -(e - 1)) > 448.0)
    assert F8.scale_exponent(np.array([0.0]))[0] == 0
    assert F8.scale_exponent(np.array([448.0]))[0] == 0 and F8.scale_exponent(np.array([449.0]))[0] == 1
    assert F8.scale_exponent(np.array([1.0]))[0] == -8          # 256 fits, 512 does not
    assert F8.scale_exponent(np.array([2.0 ** -140]))[0] == -100  # kept within fp32's exponent range


def test_scale_granularity_and_error_bound():
    rng = np.random.default_rng(11)
    T, Hq, Hkv, D = 37, 4, 2, 64
    q = rng.standard_normal((T, Hq, D)) * 0.5
    k = rng.standard_normal((T, Hkv, D)) * 0.5
    v = rng.standard_normal((T, Hkv, D)) * 0.5
    f = F8.q_factor(0.0, D)
    assert f == np.float32(np.float32(1.0 / np.sqrt(64.0)) * np.float32(1.4426950408889634))
    q = q.astype(np.float32).astype(np.float64)  # the reference takes float32-representable values
    z = F8.quantise_qkv(q, k, v, f)
    assert z["q_exp"].shape == (T, Hq) and z["k_exp"].shape == (Hkv,) and z["v_exp"].shape == (Hkv,)
    # the largest element of every scaled slice lands in [224, 448]
    assert np.all(np.abs(F8.decode(z["q_codes"])).max(axis=2) >= 224)
    assert np.all(np.abs(F8.decode(z["k_codes"])).max(axis=(0, 2)) >= 224)
    # one large value in K: its head changes scale for every token, the other head and Q do not
    k2 = k.copy()
    k2[5, 1, 3] = 1000.0
    z2 = F8.quantise_qkv(q, k2, v, f)
    assert z2["k_exp"][1] > z["k_exp"][1] and z2["k_exp"][0] == z["k_exp"][0]
    assert np.array_equal(z2["k_codes"][:, 0], z["k_codes"][:, 0]) and not np.array_equal(z2["k_codes"][:, 1], z["k_codes"][:, 1])
    assert np.array_equal(z2["q_codes"], z["q_codes"])
    # one large value in a Q row: only that (token, head) changes
    q2 = q.copy()
    q2[9, 2, 0] = 77.0
    z3 = F8.quantise_qkv(q2, k, v, f)
    same = np.ones((T, Hq), bool)
    same[9, 2] = False
    assert np.array_equal(z3["q_codes"][same], z["q_codes"][same]) and z3["q_exp"][9, 2] > z["q_exp"][9, 2]
    # normal-range elements keep a relative error of at most 2^-4 (half a unit of a 3-bit mantissa)
    qd, kd, vd = F8.dequantised_qkv(q, k, v, f)
    qs = (q.astype(np.float32) * f).astype(np.float64)  # what is quantised of Q
    for x, xd, e in ((qs, qd * np.float64(f), z["q_exp"][:, :, None]), (k, kd, z["k_exp"][None, :, None]), (v, vd, z["v_exp"][None, :, None])):
        normal = np.abs(x) >= np.ldexp(1.0, e - 6)
        assert np.all(np.abs(xd - x)[normal] <= 2.0 ** -4 * np.abs(x)[normal])
        assert np.all(np.abs(xd - x)[~normal] <= np.broadcast_to(np.ldexp(1.0, e - 10), x.shape)[~normal])
