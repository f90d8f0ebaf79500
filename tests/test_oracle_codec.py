"""Pins for the oracle's two codecs (Sec. 3.2 of arXiv 1811.03619: truncation
keeps 16 bits, scalar quantization keeps 8 bits with the range set by the
largest magnitude; compression ratios 2x and 4x, Sec. 4 "Timing Breakdown").

Every expected value here comes from IEEE-754 facts, from hand arithmetic
written out in the comments, or from a property that holds for any correct
implementation -- never from the oracle itself.
"""
import numpy as np
import pytest

from paper_1811_03619_amd import workloads as W


def bits(x):
    return np.asarray(x, dtype=np.float32).view(np.uint32)


# ------------------------------------------------------------ truncation --

def test_trunc16_known_patterns(orc):
    # IEEE-754 binary32 layouts: 1.0 = 0x3F800000, -2.0 = 0xC0000000,
    # pi ~ 0x40490FDB, 1+2^-7 = 0x3F810000, 1+2^-8 = 0x3F808000.
    x = np.array([1.0, -2.0, np.float32(np.pi), 1 + 2.0 ** -7, 1 + 2.0 ** -8, 0.0, -0.0,
                  np.inf, -np.inf], dtype=np.float32)
    pay, sc = orc.compress(orc.TRUNC16, x)
    assert sc is None and pay.dtype == np.uint16
    assert pay.tolist() == [0x3F80, 0xC000, 0x4049, 0x3F81, 0x3F80, 0x0000, 0x8000, 0x7F80, 0xFF80]
    back = orc.decompress(orc.TRUNC16, pay)
    # 0x40490000 = 3.140625 ; the 2^-8 term is dropped, the 2^-7 term survives
    assert back.tolist()[:5] == [1.0, -2.0, 3.140625, 1.0078125, 1.0]
    assert bits(back).tolist()[5:] == [0x00000000, 0x80000000, 0x7F800000, 0xFF800000]


def test_trunc16_exhaustive_payloads_roundtrip(orc):
    u = np.arange(1 << 16, dtype=np.uint32).astype(np.uint16)
    x = orc.decompress(orc.TRUNC16, u)
    assert np.array_equal(bits(x), u.astype(np.uint32) << 16)
    again, _ = orc.compress(orc.TRUNC16, x)
    assert np.array_equal(again, u)


def test_trunc16_properties_over_bit_patterns(orc):
    rng = np.random.Generator(np.random.Philox(key=11))
    u = rng.integers(0, 1 << 32, size=1 << 20, dtype=np.uint64).astype(np.uint32)
    edge = np.array([0x00000001, 0x0000FFFF, 0x00010000, 0x007FFFFF, 0x00800000, 0x7F7FFFFF,
                     0x3F7FFFFF, 0x3F80FFFF, 0x80000001, 0xFF7FFFFF], dtype=np.uint32)
    u = np.concatenate([u, edge])
    x = u.view(np.float32)
    pay, _ = orc.compress(orc.TRUNC16, x)
    y = orc.decompress(orc.TRUNC16, pay)
    yb = bits(y)
    assert np.all((yb & 0xFFFF) == 0)                       # 16 bits dropped
    assert np.array_equal(yb >> 23, u >> 23)                # sign and exponent kept
    fin = np.isfinite(x)
    assert np.all(np.abs(y[fin].astype(np.float64)) <= np.abs(x[fin].astype(np.float64)))  # toward zero
    normal = fin & (np.abs(x) >= np.finfo(np.float32).tiny)
    xd, yd = x[normal].astype(np.float64), y[normal].astype(np.float64)
    assert np.all(np.abs(xd - yd) < 2.0 ** -7 * np.abs(xd))  # 7 mantissa bits kept
    pay2, _ = orc.compress(orc.TRUNC16, y)
    assert np.array_equal(pay2, pay)                        # idempotent
    assert pay.nbytes * 2 == x.nbytes                       # the 2x ratio


def test_trunc16_denormals_are_truncated_not_flushed(orc):
    # 0x00018000 is a denormal whose top half 0x0001 survives: 2^-133 exactly.
    x = np.array([0x00018000, 0x00007FFF], dtype=np.uint32).view(np.float32)
    pay, _ = orc.compress(orc.TRUNC16, x)
    assert pay.tolist() == [0x0001, 0x0000]
    y = orc.decompress(orc.TRUNC16, pay)
    assert bits(y).tolist() == [0x00010000, 0]


# ---------------------------------------------------------- quantization --

def test_quant8_identity_grid(orc):
    # scale = 127 -> inv = 1, step = 1: integers in [-127,127] are their own code.
    x = np.arange(-127, 128, dtype=np.float32)
    q, sc = orc.compress(orc.QUANT8, x)
    assert q.dtype == np.int8 and sc.tolist() == [127.0]
    assert q.tolist() == list(range(-127, 128))
    assert np.array_equal(orc.decompress(orc.QUANT8, q, sc), x)
    # scale = 63.5 -> inv = 2, step = 0.5: half-integers k/2 get code k.
    x2 = np.arange(-127, 128, dtype=np.float32) / 2
    q2, sc2 = orc.compress(orc.QUANT8, x2)
    assert sc2.tolist() == [63.5] and q2.tolist() == list(range(-127, 128))
    assert np.array_equal(orc.decompress(orc.QUANT8, q2, sc2), x2)


def test_quant8_ties_round_to_even(orc):
    # with scale 127 the scaled value equals x, so x = k + 0.5 is an exact tie
    x = np.array([127.0, 0.5, 1.5, 2.5, 3.5, -0.5, -1.5, -2.5, 125.5, 126.5, -126.5], dtype=np.float32)
    q, _ = orc.compress(orc.QUANT8, x)
    assert q.tolist() == [127, 0, 2, 2, 4, 0, -2, -2, 126, 126, -126]


def test_quant8_extreme_element_and_error_bound(orc):
    for seed, n in [(1, 4096), (2, 4096 * 3 + 17), (3, 1), (4, 5)]:
        x = W.gaussian(n, 0.02, seed)
        q, sc = orc.compress(orc.QUANT8, x)
        y = orc.decompress(orc.QUANT8, q, sc)
        assert q.size == n and sc.size == -(-n // 4096)
        assert q.min() >= -127                                # -128 never produced
        for b in range(sc.size):
            xs, qs, ys = x[b * 4096:(b + 1) * 4096], q[b * 4096:(b + 1) * 4096], y[b * 4096:(b + 1) * 4096]
            k = int(np.argmax(np.abs(xs)))
            assert sc[b] == np.abs(xs[k])                      # range = largest magnitude, exactly
            assert qs[k] == (127 if xs[k] > 0 else -127)
            assert abs(float(ys[k]) - float(xs[k])) <= 2 * np.spacing(np.float32(abs(xs[k])))
            half_step = float(sc[b]) / 254.0
            assert np.max(np.abs(xs.astype(np.float64) - ys.astype(np.float64))) <= half_step * (1 + 1e-4)


def test_quant8_blocks_are_independent_4096_runs(orc):
    x = np.zeros(4096 * 2 + 1, dtype=np.float32)
    x[0:4096] = 1.0
    x[100] = 127.0
    x[4096:8192] = 0.25
    x[8192] = -3.0                       # ragged third block of one element
    q, sc = orc.compress(orc.QUANT8, x)
    assert sc.tolist() == [127.0, 0.25, 3.0]
    assert q[0] == 1 and q[100] == 127 and q[4096] == 127 and q[8191] == 127 and q[8192] == -127
    y = orc.decompress(orc.QUANT8, q, sc)
    assert y[8192] == -3.0 and y[4096] == 0.25 and y[0] == 1.0


def test_quant8_operation_order_against_the_workload_formula(orc):
    # The workload list writes the code as round(x / scale * 127); the reading taken here is
    # rint(x * (127 / scale)) -- one division per block instead of one per element.  In binary32 the two
    # differ only where x/scale*127 falls within an ulp or so of a rounding tie: about one element in a
    # million on Gaussian blocks, and then by exactly one code.  The oracle must follow the reading taken
    # (bit for bit, against numpy's correctly rounded float32 operations), and the literal formula must
    # stay that close to it -- which is all that can be pinned: no text fixes the order of operations.
    x = W.gaussian(4096 * 1500, 1e-4, 71)
    pay, sc = orc.compress(orc.QUANT8, x)
    xb = x.reshape(-1, 4096)
    s = np.abs(xb).max(axis=1, keepdims=True).astype(np.float32)
    assert np.array_equal(sc, s.ravel())
    taken = np.clip(np.rint(xb * (np.float32(127.0) / s)), -127, 127).astype(np.int8)
    literal = np.clip(np.rint((xb / s) * np.float32(127.0)), -127, 127).astype(np.int8)
    assert np.array_equal(pay.reshape(-1, 4096), taken)
    differ = taken != literal
    assert differ.mean() < 1e-5
    assert np.abs(taken.astype(np.int16) - literal.astype(np.int16)).max() <= 1


def test_quant8_zero_block(orc):
    x = np.zeros(4096 + 7, dtype=np.float32)
    x[4096 + 3] = 1e-3
    q, sc = orc.compress(orc.QUANT8, x)
    assert sc[0] == 0.0 and not q[:4096].any()
    y = orc.decompress(orc.QUANT8, q, sc)
    assert not y[:4096].any() and bits(y[:4096]).max() == 0   # +0, not -0 or NaN
    assert q[4096 + 3] == 127


def test_quant8_tiny_scale_saturates_inverse(orc):
    # 127/scale overflows binary32 for scale < 127/FLT_MAX ~ 3.7e-37.  Reading:
    # the inverse saturates at FLT_MAX, so codes shrink toward zero instead of
    # turning into inf/NaN; zeros stay zero.
    x = np.array([1e-40, 0.0, -5e-41, 1e-38], dtype=np.float32)
    q, sc = orc.compress(orc.QUANT8, x)
    assert sc[0] == np.float32(1e-38)
    # 1e-38 * FLT_MAX ~ 3.40 -> 3 ; 1e-40 * FLT_MAX ~ 0.034 -> 0
    assert q.tolist() == [0, 0, 0, 3]
    y = orc.decompress(orc.QUANT8, q, sc)
    assert np.all(np.isfinite(y))


def test_quant8_payload_size_is_quarter(orc):
    n = 4096 * 250 + 1
    assert orc.payload_bytes(orc.QUANT8, n) == n + 4 * 251       # int8 + one fp32 scale per block
    assert orc.payload_bytes(orc.TRUNC16, n) == 2 * n
    assert orc.payload_bytes(orc.NONE, n) == 4 * n
    assert 4 * n / orc.payload_bytes(orc.QUANT8, n) > 3.99        # the 4x ratio


def test_none_codec_is_identity(orc):
    x = W.gaussian(1000, 1.0, 5)
    pay, sc = orc.compress(orc.NONE, x)
    assert sc is None and np.array_equal(bits(pay), bits(x))
    assert np.array_equal(bits(orc.decompress(orc.NONE, pay)), bits(x))


@pytest.mark.parametrize("mode", [0, 1, 2])
def test_empty_input(orc, mode):
    pay, sc = orc.compress(mode, np.empty(0, np.float32))
    assert pay.size == 0
    assert orc.decompress(mode, pay, sc).size == 0
