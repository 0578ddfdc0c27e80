"""Pins for the oracle's primitives: Philox, fixlog2, the key (Alg. 2, key step)."""
import os
import random
from decimal import Decimal, getcontext
from fractions import Fraction

import pytest

import oracle

GOLD = os.path.join(os.path.dirname(__file__), "golden")
getcontext().prec = 60
LN2 = Decimal(2).ln()


def _rows(name):
    with open(os.path.join(GOLD, name)) as f:
        return [ln.split() for ln in f if ln.strip() and not ln.startswith("#")]


def test_philox_published_known_answers():
    rows = _rows("philox4x32_10_kat.txt")
    assert len(rows) == 3
    for r in rows:
        v = [int(t, 16) for t in r]
        assert oracle.philox4x32_10(v[0:4], v[4:6]) == v[6:10]


def _philox_py(ctr, key):
    """Second, separately written Philox4x32-10 (Python integers)."""
    c = list(ctr)
    k0, k1 = key
    for r in range(10):
        p0 = 0xD2511F53 * c[0]
        p1 = 0xCD9E8D57 * c[2]
        c = [(p1 >> 32) ^ c[1] ^ k0, p1 & 0xFFFFFFFF, (p0 >> 32) ^ c[3] ^ k1, p0 & 0xFFFFFFFF]
        k0 = (k0 + 0x9E3779B9) & 0xFFFFFFFF
        k1 = (k1 + 0xBB67AE85) & 0xFFFFFFFF
    return c


def test_philox_matches_second_implementation_and_draw_layout():
    rnd = random.Random(1)
    for _ in range(300):
        ctr = [rnd.getrandbits(32) for _ in range(4)]
        key = [rnd.getrandbits(32) for _ in range(2)]
        assert oracle.philox4x32_10(ctr, key) == _philox_py(ctr, key)
    # counter layout of a draw: (slot >> 2, node lo, node hi, hop), key = (seed lo, seed hi), word slot & 3
    for _ in range(200):
        seed, node = rnd.getrandbits(64), rnd.getrandbits(40)
        hop, slot = rnd.randrange(8), rnd.randrange(1 << 20)
        blk = _philox_py([slot >> 2, node & 0xFFFFFFFF, node >> 32, hop], [seed & 0xFFFFFFFF, seed >> 32])
        assert oracle.draw(seed, hop, node, slot) == blk[slot & 3]


def _log2_exact_q32(U):
    return (Decimal(U).ln() / LN2) * Decimal(1 << 32)


def test_fixlog2_powers_of_two_exact():
    for e in range(33):
        assert oracle.fixlog2_q32(1 << e) == e << 32


def test_fixlog2_within_error_bound_of_true_log2():
    rnd = random.Random(2)
    samples = [3, 5, 7, 0xC0000000, 0xFFFFFFFF, 0x12345678, 0xFFFF0000, (1 << 32) - 2]
    samples += [rnd.randrange(1, 1 << 32) for _ in range(3000)]
    samples += [rnd.randrange(1, 1 << 12) for _ in range(500)]
    worst = Decimal(0)
    for U in samples:
        got = Decimal(oracle.fixlog2_q32(U))
        err = _log2_exact_q32(U) - got
        # truncation only: never above the true value, and within 2^-29 (8 units of Q32)
        assert err >= 0, U
        worst = max(worst, err)
    assert worst < 8, worst


def test_fixlog2_monotone():
    rnd = random.Random(3)
    pts = sorted(set(rnd.randrange(1, 1 << 32) for _ in range(5000)))
    prev = -1
    for U in pts:
        cur = oracle.fixlog2_q32(U)
        assert cur >= prev
        prev = cur
    # adjacent arguments, dense near the top where mantissa steps are smallest
    for base in [1, 1000, 1 << 16, (1 << 31) - 300, (1 << 32) - 600]:
        prev = -1
        for U in range(base, base + 600):
            if U > (1 << 32):
                break
            cur = oracle.fixlog2_q32(U)
            assert cur >= prev
            prev = cur


def test_key_is_minus_log2_u_over_w_in_q32():
    """Alg. 2, key step: k = u^(1/w); the oracle's K is -log2(k) in Q32, u = (x+1)/2^32."""
    rnd = random.Random(4)
    for _ in range(1500):
        x = rnd.getrandbits(32)
        w_q16 = rnd.choice([65536, 2 * 65536, 4 * 65536, 8 * 65536, rnd.randrange(65536, 1 << 32)])
        K = oracle.key(x, w_q16)
        true_L = Decimal(32 << 32) - _log2_exact_q32(x + 1)
        true_K = true_L * Decimal(65536) / Decimal(w_q16)
        # L is over-estimated by < 8 units (fixlog2 truncates), then divided by w >= 1 and floored
        assert true_K - 1 <= K <= true_K + 8
    assert oracle.key(0xFFFFFFFF, 65536) == 0            # u = 1: the best possible key
    assert oracle.key(0, 65536) == 32 << 32              # u = 2^-32
    assert oracle.key(0, 4 * 65536) == 8 << 32


def test_key_monotone_in_x_within_a_weight_class():
    rnd = random.Random(5)
    for w in [65536, 3 * 65536 + 17, 1 << 31]:
        xs = sorted(rnd.getrandbits(32) for _ in range(2000))
        ks = [oracle.key(x, w) for x in xs]
        assert all(a >= b for a, b in zip(ks, ks[1:]))


def test_worked_example_fixture():
    rows = _rows("worked_example_node5.txt")
    weights = []
    for slot, cached, xh, K in rows:
        s = int(slot)
        x = oracle.draw(0, 0, 5, s)
        assert x == int(xh, 16)
        w = 262144 if cached == "1" else 65536
        assert oracle.key(x, w) == int(K)
        weights.append(w)
    assert oracle.select(0, 0, 5, 8, 3, weights) == [0, 5, 7]
    assert oracle.select(0, 0, 5, 8, 3, None) == [5, 6, 7]
    assert oracle.select(0, 0, 5, 8, 3, [262144] * 8) == [5, 6, 7]
