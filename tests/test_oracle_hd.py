"""Pins for the oracle's third AllReduce schedule, recursive halving and doubling
(arXiv 1811.03619, Sec. 3.1 closing remark names it among the AllReduce
algorithms the analysis covers; the algorithm itself is Thakur, Rabenseifner
and Gropp's reduce-scatter by halving + all-gather by doubling).  The result is
still the element-wise sum, delivered to every worker; what is specific to the
schedule -- the pairing tree, which operand goes through the codec, the round
and volume counts -- is pinned by hand arithmetic and by the already pinned
ring on the one case where the two coincide (p = 2).
"""
import numpy as np
import pytest

from paper_1811_03619_amd import workloads as W

F = np.float32
CE = 4096


def role_inputs(values, p=4, ce=CE, n=None):
    """values[d] is what worker c XOR d holds in block c, for every block c."""
    n = p * ce if n is None else n
    g = [np.zeros(n, dtype=F) for _ in range(p)]
    for c in range(p):
        for d in range(p):
            g[c ^ d][c * ce:(c + 1) * ce] = values[d]
    return g


@pytest.mark.parametrize("mode", [0, 1, 2])
@pytest.mark.parametrize("p,n", [(2, 10007), (4, CE * 8 + 9), (4, 5), (8, 30000 * 8 + 11), (8, CE * 3), (1, 5000),
                                 (4, 1), (16, CE * 16 * 2 + 77)])
def test_hd_equals_plain_sum_on_exact_inputs(orc, mode, p, n):
    # integers in [-7, 7]: sums of up to 16 stay below 128 (exact after truncation to 16 bits).  For
    # the quantiser every block of every worker also carries one 127 where the others hold 0, so that
    # every message and every partial sum is quantised with scale 127 (step 1).
    g = [W.small_integers(n, -7, 7, 71, (p, r, 0, 0)) for r in range(p)]
    if mode == 2:
        for blk in range(0, n, CE):
            if min(n, blk + CE) - blk < p:
                for q in range(p):
                    g[q][blk:blk + CE] = 0.0          # too short for the markers: an all-zero block
                continue
            for r in range(p):
                for q in range(p):
                    g[q][blk + r] = 127.0 if q == r else 0.0
    want = np.sum(np.stack(g).astype(np.float64), axis=0).astype(F)
    res = orc.allreduce_hd(mode, g)
    assert len(res) == p
    for pay, sc in res:
        assert np.array_equal(orc.decompress(mode, pay, sc), want)
    for r in range(1, p):
        assert np.array_equal(res[r][0], res[0][0])
        if mode == 2:
            assert np.array_equal(res[r][1], res[0][1])


def test_hd_pairing_tree(orc):
    # block c: (g_c + g_{c^2}) + (g_{c^1} + g_{c^3}) in fp32 with (2^24, 1, -2^24, 3) in the roles
    # (c, c^2, c^1, c^3): (2^24 + 1 -> 2^24) + (-2^24 + 3) = 3.  Pairing c with c^1 first gives 4,
    # c with c^3 first gives 5, left to right gives 3 only by accident of a different input.
    g = role_inputs({0: 2.0 ** 24, 2: 1.0, 1: -2.0 ** 24, 3: 3.0})
    for pay, _ in orc.allreduce_hd(orc.NONE, g):
        assert np.all(pay == F(3.0))
    # and with the roles of c^1 and c^2 exchanged the same tree gives (2^24 - 2^24) + (1 + 3) = 4
    g = role_inputs({0: 2.0 ** 24, 1: 1.0, 2: -2.0 ** 24, 3: 3.0})
    for pay, _ in orc.allreduce_hd(orc.NONE, g):
        assert np.all(pay == F(4.0))


def test_hd_own_operand_stays_in_full_precision(orc):
    # block c: own 1 + 2^-8 (not representable in 16 bits), the three others 2^-8 each:
    # (1 + 2^-8 + 2^-8) + D(C(2^-8 + 2^-8)) = 1 + 2^-6 = 0x3F82.  A receiver that truncated its own
    # operand would end at 0x3F81; the ring, which truncates the running sum on every hop, gives 0x3F80.
    g = role_inputs({0: 1 + 2.0 ** -8, 1: 2.0 ** -8, 2: 2.0 ** -8, 3: 2.0 ** -8})
    for pay, _ in orc.allreduce_hd(orc.TRUNC16, g):
        assert np.all(pay == 0x3F82)
    for pay, _ in orc.allreduce(orc.TRUNC16, g):
        assert np.all(pay == 0x3F80)


def test_hd_partial_sums_are_compressed_when_sent(orc):
    # block c: worker c^1's partial sum after the first round is (1 + 2^-7) + 2^-8, which travels as
    # 1 + 2^-7; worker c holds 1 + 2^-8:  (1 + 2^-8) + (1 + 2^-7) = 2 + 2^-7 + 2^-8 -> cut to 2.0 = 0x4000.
    # Sent uncompressed it would give 2 + 2^-6 = 0x4001.
    g = role_inputs({0: 1 + 2.0 ** -8, 2: 0.0, 1: 1 + 2.0 ** -7, 3: 2.0 ** -8})
    for pay, _ in orc.allreduce_hd(orc.TRUNC16, g):
        assert np.all(pay == 0x4000)


def test_hd_quantised_hand_case(orc):
    # every worker has a 127 of its own in every block (position = its rank), so all scales are 127
    # and the quantiser is rint().  Data position 8 of block c holds, in the roles (c, c^2, c^1, c^3),
    # (10.3, 20.4, 5.3, 7.4):   10.3 + rint(20.4) = 30.3;   5.3 + rint(7.4) = 12.3 -> travels as 12;
    # 30.3 + 12 = 42.3 -> code 42.  (Uncompressed partial: 42.6 -> 43; uncompressed first message: 42.7 -> 43.)
    p = 4
    g = [np.zeros(p * CE, dtype=F) for _ in range(p)]
    vals = {0: 10.3, 2: 20.4, 1: 5.3, 3: 7.4}
    for c in range(p):
        for r in range(p):
            g[r][c * CE + r] = 127.0
        for d, x in vals.items():
            g[c ^ d][c * CE + 8] = x
    for q, sc in orc.allreduce_hd(orc.QUANT8, g):
        assert sc.tolist() == [127.0] * p
        for c in range(p):
            assert q[c * CE + 8] == 42
            assert q[c * CE:c * CE + p].tolist() == [127] * p


@pytest.mark.parametrize("mode", [0, 1, 2])
def test_hd_with_two_workers_is_the_ring_with_the_workers_exchanged(orc, mode):
    # p = 2, block c: halving-doubling gives g_c + D(C(g_{c^1})) on worker c; the ring gives
    # D(C(g_c)) + g_{c+1} on worker c+1.  Swapping the two inputs maps one onto the other.
    n = CE * 5 + 123
    g = [W.gaussian(n, 0.03, 73, (mode, r, 0, 0)) for r in range(2)]
    a = orc.allreduce_hd(mode, g)
    b = orc.allreduce(mode, [g[1], g[0]])
    for r in range(2):
        assert np.array_equal(a[r][0].view(np.uint8), b[r][0].view(np.uint8))
        if mode == 2:
            assert np.array_equal(a[r][1], b[r][1])


@pytest.mark.parametrize("mode", [1, 2])
def test_hd_error_bound_follows_the_tree_depth(orc, mode):
    p, n = 8, CE * 8 + 1001
    g = [W.gaussian(n, 1e-3, 75, (mode, r, 0, 0)) for r in range(p)]
    exact = np.sum(np.stack(g).astype(np.float64), axis=0)
    res = orc.allreduce_hd(mode, g)
    out = orc.decompress(mode, *res[0]).astype(np.float64)
    if mode == 1:
        # a value passes through at most log2(p) + 1 = 4 truncations, each losing < 2^-7 of a partial
        # sum whose magnitude is at most the sum of magnitudes
        sabs = np.sum(np.abs(np.stack(g).astype(np.float64)), axis=0)
        assert np.all(np.abs(out - exact) <= 4 * 2.0 ** -7 * sabs * (1 + 1e-6))
        ring = orc.decompress(mode, *orc.allreduce(mode, g)[0]).astype(np.float64)
        # the ring's chain is p - 1 = 7 deep: larger error on average
        assert np.mean(np.abs(out - exact)) < np.mean(np.abs(ring - exact))
    else:
        for b in range(-(-n // CE)):
            sl = slice(b * CE, min(n, (b + 1) * CE))
            smax = sum(float(np.max(np.abs(x[sl]))) for x in g)
            # every message and the result lose at most half a step of a scale that is at most smax:
            # log2(p) levels of messages plus the final compression
            assert np.max(np.abs(out[sl] - exact[sl])) <= 4 * smax / 254.0 * 1.05
    for r in range(1, p):
        assert np.array_equal(res[r][0], res[0][0])


@pytest.mark.parametrize("p", [2, 4, 8])
def test_hd_round_and_volume_counts(orc, p):
    # 2 log2(p) rounds (against the ring's 2(p-1)); the volume is the ring's: per worker
    # n/2 + n/4 + ... = (p-1)/p n sent while halving, the same again while doubling, (p-1)/p n reduced
    n = p * CE * 3
    g = [W.gaussian(n, 0.01, 77, (0, r, 0, 0)) for r in range(p)]
    c = np.zeros(3, dtype=np.uint64)
    orc.allreduce_hd(orc.TRUNC16, g, c)
    assert c.tolist() == [2 * (p.bit_length() - 1), 2 * (p - 1) * n // p, (p - 1) * n // p]


def test_hd_needs_a_power_of_two(orc):
    g = [np.zeros(100, dtype=F) for _ in range(3)]
    with pytest.raises(ValueError):
        orc.allreduce_hd(orc.NONE, g)


def test_hd_gaussian_uncompressed_is_the_sum_to_rounding(orc):
    p, n = 4, CE * 4 + 55
    g = [W.gaussian(n, 0.03, 79, (0, r, 0, 0)) for r in range(p)]
    exact = np.sum(np.stack(g).astype(np.float64), axis=0)
    sabs = np.sum(np.abs(np.stack(g).astype(np.float64)), axis=0)
    for pay, _ in orc.allreduce_hd(orc.NONE, g):
        assert np.all(np.abs(pay.astype(np.float64) - exact) <= (p - 1) * 2.0 ** -24 * sabs)
