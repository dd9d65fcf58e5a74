"""Pins for the oracle's scheme functions for up to four limbs (256-bit integers written out in
C): agreement with the 128-bit functions where both apply, and Python integers elsewhere.
None of the expected values comes from the functions under test."""
import numpy as np
import pytest

import cop_inputs as ci


def _params(seed, rows, N, L, t_bits, q_bits):
    moduli = ci.limb_primes(q_bits, t_bits, L)
    s = ci.gen_secret(seed, N)
    a, e = ci.gen_enc_randomness(seed, rows, 1, moduli, N)
    return moduli, s, a[:, 0], e[:, 0]


def _Q(moduli):
    Q = 1
    for q in moduli:
        Q *= int(q)
    return Q


@pytest.mark.parametrize("L,t_bits,q_bits", [(1, 16, 50), (2, 20, 54), (2, 32, 62), (1, 7, 30)])
def test_agrees_with_the_128_bit_functions(oracle, L, t_bits, q_bits):
    N, rows = 64, 6
    moduli, s, a, e = _params(21, rows, N, L, t_bits, q_bits)
    w_hat = ci.uniform_below(21, 4, (rows, N), 1 << t_bits)
    ct = oracle.encrypt(w_hat, s, a, e, moduli, t_bits)
    assert np.array_equal(oracle.encrypt_rns(w_hat, s, a, e, moduli, t_bits), ct)
    uni = ci.uniform_residues(22, 5, (rows, 2), moduli, N)
    for r in range(rows):
        assert np.array_equal(oracle.decrypt_rns(ct[r], s, moduli, t_bits),
                              oracle.decrypt(ct[r], s, moduli, t_bits))
        assert np.array_equal(oracle.decrypt_rns(uni[r], s, moduli, t_bits),
                              oracle.decrypt(uni[r], s, moduli, t_bits))
    R = ci.uniform_below(23, 6, (N,), 1 << t_bits)
    assert np.array_equal(oracle.share_mask_rns(R, moduli, t_bits),
                          oracle.share_mask(R, moduli, t_bits))


@pytest.mark.parametrize("L,t_bits,q_bits", [(3, 24, 55), (4, 20, 54), (3, 32, 62), (4, 1, 40),
                                             (2, 20, 54), (1, 16, 50)])
def test_decoding_of_chosen_phases_against_python_integers(oracle, L, t_bits, q_bits):
    """ciphertexts with c1 = 0 and c0 = the residues of a chosen integer v: the phase is v, so
    the expected plaintext is ((v + Delta // 2) // Delta) % t straight from v.  v runs over
    the rounding boundaries, both ends of [0, Q) and random values."""
    N = 64
    moduli = ci.limb_primes(q_bits, t_bits, L)
    Q = _Q(moduli)
    t = 1 << t_bits
    delta = Q >> t_bits
    values = [0, 1, Q - 1, Q - 2, delta // 2, delta // 2 - 1, delta // 2 + 1, delta - 1, delta]
    for mm in (1, 2, t // 2, t - 2, t - 1):
        for d in (-2, -1, 0, 1, 2):
            for v in (delta * mm + delta // 2 + d, delta * mm + d):
                if 0 <= v < Q:
                    values.append(v)
    values += [min(Q - 1, delta * t + delta // 2), min(Q - 1, delta * t + delta // 2 - 1)]
    rng = np.random.default_rng(7)
    while len(values) % N:
        values.append(int.from_bytes(rng.bytes(40), "little") % Q)
    s = ci.gen_secret(3, N)
    for blk in range(len(values) // N):
        vs = values[blk * N:(blk + 1) * N]
        ct = np.zeros((2, L, N), dtype=np.uint64)
        for c, v in enumerate(vs):
            for l, q in enumerate(moduli):
                ct[0, l, c] = v % int(q)
        got = oracle.decrypt_rns(ct, s, moduli, t_bits)
        want = [((v + delta // 2) // delta) % t for v in vs]
        assert [int(x) for x in got] == want


@pytest.mark.parametrize("L,t_bits,q_bits", [(3, 24, 55), (4, 20, 54), (3, 16, 50)])
def test_round_trip_and_phase_structure(oracle, L, t_bits, q_bits):
    """Dec(Enc(w)) = w, c1 = a, and per limb  phase = (Delta mod q_l) w + e  with Delta from
    Python integers"""
    N, rows = 64, 5
    moduli, s, a, e = _params(31, rows, N, L, t_bits, q_bits)
    w_hat = ci.uniform_below(31, 4, (rows, N), 1 << t_bits)
    w_hat[0, :4] = [(1 << t_bits) - 1, 0, 1, (1 << t_bits) - 1]
    ct = oracle.encrypt_rns(w_hat, s, a, e, moduli, t_bits)
    delta = _Q(moduli) >> t_bits
    for r in range(rows):
        assert np.array_equal(ct[r, 1], a[r])
        assert np.array_equal(oracle.decrypt_rns(ct[r], s, moduli, t_bits), w_hat[r])
        phi = oracle.phase(ct[r], s, moduli)
        for l, q in enumerate(moduli):
            want = [(delta % int(q) * int(w) + int(ee)) % int(q) for w, ee in zip(w_hat[r], e[r])]
            assert [int(x) for x in phi[l]] == want


def test_share_mask_and_protocol_invariant_three_limbs(oracle):
    """config-5-like parameters (three limbs of 55 bits, t = 2^24) on a small shape: the mask
    is (Q - Delta R) limb by limb (Python integers), and after the COP accumulation on really
    encrypted weights  Dec(out_j) + R_j = (X W)_j mod t  (Theorem 1) by brute force"""
    m, k, n, N, L, t_bits, q_bits = 4, 24, 48, 64, 3, 24, 55
    t = 1 << t_bits
    moduli, s, a, e = _params(41, k, N, L, t_bits, q_bits)
    Q = _Q(moduli)
    delta = Q >> t_bits
    W = ci.gen_W(41, k, n, t_bits)
    X = ci.gen_X(41, m, k, t_bits)
    R = ci.gen_R(41, m, N, t_bits)
    mask = np.stack([oracle.share_mask_rns(R[j], moduli, t_bits) for j in range(m)])
    for j in range(m):
        for l, q in enumerate(moduli):
            want = [((Q - delta * int(r)) % Q) % int(q) for r in R[j]]
            assert [int(x) for x in mask[j, 0, l]] == want
        assert not mask[j, 1].any()
    ct = oracle.encrypt_rns(oracle.encode_rows(W, N)[:, 0], s, a, e, moduli, t_bits)
    out, _ = oracle.cop_ref(X, ct[:, None], moduli, n, N, mask[:, None])
    Y = (X.astype(object) @ W.astype(object)) % t
    for j in range(m):
        dec = oracle.decrypt_rns(out[j, 0], s, moduli, t_bits)
        total = (dec.astype(object) + R[j].astype(object)) % t
        assert np.array_equal(total[:n], Y[j])
        assert not total[n:].any()
