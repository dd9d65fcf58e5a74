"""The arithmetic claims behind the server-side transform kernels (csrc/rlwe_kernels.hpp), checked
on Python integers: ranges of the two products by a table constant, of the fold, of the
conditional subtraction by sign, and the bounds that let the kernels for moduli below 2^58 and
2^59 run without conditional subtractions.  Nothing here runs GPU code: the parity tests do;
these tests say why the ranges those kernels rely on hold (Appendix B.1's Enc / Dec multiply
polynomials through a number-theoretic transform; the paper gives no arithmetic for it)."""
import random

M64 = (1 << 64) - 1


def _moduli(rng, lo_bits, hi_bits, count):
    out = []
    for _ in range(count):
        b = rng.randrange(lo_bits, hi_bits + 1)
        out.append(rng.randrange(1 << (b - 1), 1 << b) | 1)
    return out + [(1 << (lo_bits - 1)) + 1, (1 << hi_bits) - 1]


def _xs(rng, q):
    return [0, 1, q - 1, q, 2 * q, 4 * q - 1, M64, M64 - 1, 1 << 63, (1 << 32) - 1, 1 << 32] + \
           [rng.getrandbits(64) for _ in range(200)]


def test_exact_product_lies_below_two_q_for_every_word():
    """x w - floor(x w' / 2^64) q with w' = floor(w 2^64 / q): in [0, 2q), congruent to x w"""
    rng = random.Random(1)
    for q in _moduli(rng, 20, 62, 40):
        for _ in range(5):
            w = rng.randrange(q)
            ws = (w << 64) // q
            for x in _xs(rng, q):
                h = (x * ws) >> 64
                r = x * w - h * q
                assert 0 <= r < 2 * q and r % q == x * w % q
                # as the kernel computes it: a sum with 2^64 - q, modulo 2^64
                assert (x * w + h * ((1 << 64) - q)) & M64 == r


def test_product_with_the_estimate_from_three_partial_products_lies_below_four_q():
    """h' = x1 w1' + floor(x0 w1' / 2^32) + floor(x1 w0' / 2^32) is at most 2 short of the exact
    quotient estimate, so the result grows by at most 2q"""
    rng = random.Random(2)
    for q in _moduli(rng, 35, 58, 40):
        for _ in range(5):
            w = rng.randrange(q)
            ws = (w << 64) // q
            w0, w1 = ws & 0xFFFFFFFF, ws >> 32
            for x in _xs(rng, q):
                x0, x1 = x & 0xFFFFFFFF, x >> 32
                h = x1 * w1 + ((x0 * w1) >> 32) + ((x1 * w0) >> 32)
                exact = (x * ws) >> 64
                assert 0 <= exact - h <= 2
                r = x * w - h * q
                assert 0 <= r < 4 * q and r % q == x * w % q
                assert (x * w + h * ((1 << 64) - q)) & M64 == r


def test_fold_brings_every_word_below_two_q():
    """h = floor(floor(x / 2^32) m / 2^(32+k)), m = floor(2^(64+k) / q), k = bitlen(q) - 33"""
    rng = random.Random(3)
    for q in _moduli(rng, 35, 59, 60):
        k = q.bit_length() - 33
        m = (1 << (64 + k)) // q
        assert k >= 1 and m < (1 << 32)
        for x in _xs(rng, q):
            h = (((x >> 32) * m) >> 32) >> k
            r = x - h * q
            assert 0 <= r < 2 * q and r % q == x % q
            assert (x + h * ((1 << 64) - q)) & M64 == r


def test_conditional_subtraction_by_the_sign_of_the_sum():
    """u >= m ? u - m : u decided by bit 63 of u + (2^64 - m), for m <= 2^63 and u < m + 2^63"""
    rng = random.Random(4)
    for q in _moduli(rng, 20, 62, 40):
        for m in (q, 2 * q):
            for u in [0, m - 1, m, m + 1, 2 * m - 1, 4 * q - 1] + [rng.randrange(4 * q) for _ in range(100)]:
                if u >= m + (1 << 63):
                    continue
                d = (u + (1 << 64) - m) & M64
                got = u if d >> 63 else d
                assert got == (u - m if u >= m else u)


# ---- the bounds of the kernels without conditional subtractions, in multiples of q ----
def _round_stages(stages, maxs):
    rounds = -(-stages // maxs)
    return -(-stages // rounds)


def _rounds(log_n, pre, maxs):
    p, out = pre, []
    while p < log_n:
        s = _round_stages(log_n - p, maxs)
        out.append(s)
        p += s
    return out


def _inverse_round(S, bin_, tout, prod):
    """bounds of the 2^S registers after the S inverse stages of a round; returns (largest bound
    seen in a sum or difference, bounds after the fold)"""
    R = 1 << S
    b = [bin_] * R
    most = 0
    for st in range(S - 1, -1, -1):
        half = R >> (st + 1)
        for r in range(R):
            if r & half:
                continue
            most = max(most, b[r] + b[r + half])      # u + v, and u + bound(v) q - v
            b[r] += b[r + half]
            b[r + half] = prod
    return most, [2 if v > tout else v for v in b]


def test_no_word_overflows_without_conditional_subtractions():
    """forward: inputs below q (3q behind the stage done on the way in), every stage adds the
    product's bound; inverse: sums of bounds, folds at the end of a round; all below 2^64 / q"""
    for units, prod, q_bits in ((64, 4, 58), (32, 2, 59)):
        assert units << q_bits <= 1 << 64                 # `units` multiples of q < 2^q_bits fit a word
        for log_n in range(5, 16):
            pre = 1 if log_n == 15 else 0
            for maxs in ((4,) if pre else (2, 3, 4)):
                stages = _rounds(log_n, pre, maxs)
                assert sum(stages) == log_n - pre and max(stages) <= 4
                # forward
                assert (3 if pre else 1) + prod * (log_n - pre) <= units
                # inverse: the round in the middle starts from products, the others from what
                # the round before left
                bin_ = prod
                order = stages[::-1]                      # inverse rounds run from the last forward round back
                for i, S in enumerate(order):
                    tout = units >> order[i + 1] if i + 1 < len(order) else 2
                    most, after = _inverse_round(S, bin_, tout, prod)
                    assert most <= units, (log_n, maxs, i)
                    bin_ = max(after)
                assert bin_ <= 2                          # what the last round leaves: below 2q
