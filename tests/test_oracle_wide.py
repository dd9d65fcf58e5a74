"""Pins for the oracle's COP with shares of up to 64 bits (the paper's own setting l = 64,
Section 5.1): Python big-int recomputation including the largest share; agreement with the
32-bit definition where both apply; the special cases of the narrow version; and phase
linearity per limb.  (No decryption pin: with t = 2^64 and q ~ 2^114 the scaled noise k t e
exceeds Delta/2, so the toy scheme cannot decrypt such a product; the paper does not say how
its parameters cope, and the hot path does not depend on it.)
"""
import numpy as np

import cop_inputs as ci

MODULI = ci.limb_primes(59, 14, 1) + ci.limb_primes(55, 14, 1)      # 1 mod 2N for N = 8192


def _inputs(seed, m, k, N, x_bits):
    X = ci.gen_X(seed, m, k, x_bits)
    ctW = ci.gen_ctW_uniform(seed, k, 1, MODULI, N)
    mask = ci.gen_mask_uniform(seed, m, 1, MODULI, N)
    return X, ctW, mask


def test_wide_against_python_big_ints(oracle):
    m, k, N = 5, 9, 16
    X, ctW, mask = _inputs(1, m, k, N, 64)
    X[0, 0] = (1 << 64) - 1
    X[1, :] = (1 << 64) - 1
    for l, q in enumerate(MODULI):
        ctW[:, 0, :, l, :2] = q - 1
        mask[1, 0, :, l, :2] = q - 1
    got, _ = oracle.cop_ref(X, ctW, MODULI, N, N, mask, wide=True)
    for j in range(m):
        for p in range(2):
            for l, q in enumerate(MODULI):
                for c in range(N):
                    v = sum(int(X[j, i]) * int(ctW[i, 0, p, l, c]) for i in range(k)) + int(mask[j, 0, p, l, c])
                    assert int(got[j, 0, p, l, c]) == v % q


def test_wide_equals_narrow_on_32_bit_shares(oracle):
    X, ctW, mask = _inputs(2, 7, 33, 32, 32)
    a, _ = oracle.cop_ref(X, ctW, MODULI, 32, 32, mask)
    b, _ = oracle.cop_ref(X, ctW, MODULI, 32, 32, mask, wide=True)
    assert np.array_equal(a, b)


def test_wide_special_cases(oracle):
    k, N = 6, 32
    _, ctW, mask = _inputs(3, k, k, N, 64)
    zero = np.zeros((k, k), dtype=np.uint64)
    out, _ = oracle.cop_ref(zero, ctW, MODULI, N, N, mask, wide=True)
    assert np.array_equal(out, mask)                               # X = 0: only the mask
    eye = np.eye(k, dtype=np.uint64)
    out, _ = oracle.cop_ref(eye, ctW, MODULI, N, N, None, wide=True)
    assert np.array_equal(out, ctW)                                # X = I: a copy
    # a share that is a multiple of q_0 annihilates limb 0 and not limb 1
    X = np.zeros((1, k), dtype=np.uint64)
    X[0, 2] = np.uint64(MODULI[0] * 3)
    out, _ = oracle.cop_ref(X, ctW, MODULI, N, N, None, wide=True)
    assert (out[0, 0, :, 0] == 0).all() and (out[0, 0, :, 1] != 0).any()


def test_wide_is_high_half_times_2_32_plus_low_half(oracle):
    """x = x_lo + 2^32 x_hi: the identity the two-pass GPU path rests on, with big ints"""
    X, ctW, mask = _inputs(4, 4, 10, 16, 64)
    full, _ = oracle.cop_ref(X, ctW, MODULI, 16, 16, mask, wide=True)
    lo, _ = oracle.cop_ref(X & np.uint64(0xffffffff), ctW, MODULI, 16, 16, mask)
    hi, _ = oracle.cop_ref(X >> np.uint64(32), ctW, MODULI, 16, 16, None)
    for l, q in enumerate(MODULI):
        want = (hi[:, :, :, l].astype(object) * (1 << 32) + lo[:, :, :, l].astype(object)) % q
        assert np.array_equal(full[:, :, :, l], want.astype(np.uint64))


def test_wide_phase_linearity(oracle):
    """phi(out_j) = sum_i X[j,i] phi(ct_i) + phi(mask_j) (mod q_l) for arbitrary ciphertexts"""
    m, k, N = 3, 8, 32
    X, ctW, mask = _inputs(5, m, k, N, 64)
    s = ci.gen_secret(6, N)
    out, _ = oracle.cop_ref(X, ctW, MODULI, N, N, mask, wide=True)
    phi_w = [oracle.phase(ctW[i, 0], s, MODULI) for i in range(k)]
    for j in range(m):
        phi_out = oracle.phase(out[j, 0], s, MODULI)
        phi_m = oracle.phase(mask[j, 0], s, MODULI)
        for l, q in enumerate(MODULI):
            acc = phi_m[l].astype(object)
            for i in range(k):
                acc = acc + int(X[j, i]) * phi_w[i][l].astype(object)
            assert np.array_equal((acc % q).astype(np.uint64), phi_out[l])
