"""Pins for the toy RLWE scheme of the oracle and for cop_ref against the paper's
correctness statement (Algorithm 1, Output line; step 5): after the protocol,
client share + server share = X W mod t.  Restated for the hot path:
Dec(out_j) + R_j = (X W)_j mod t, with the right-hand side by brute force.
"""
import numpy as np
import pytest

import cop_inputs as ci


def dense_negacyclic(a, s, q):
    """O(N^2) product in Z_q[X]/(X^N+1) with Python ints: reduce X^(N+d) to -X^d"""
    N = len(a)
    out = [0] * N
    for i in range(N):
        for j in range(N):
            d = i + j
            term = int(a[i]) * int(s[j])
            if d >= N:
                out[d - N] -= term
            else:
                out[d] += term
    return np.array([v % q for v in out], dtype=np.uint64)


def test_negacyclic_against_dense_schoolbook(oracle):
    N = 16
    q = ci.limb_primes(54, 20, 1)[0]
    a = ci.uniform_below(1, 1, (N,), q)
    s = ci.gen_secret(2, N)
    assert np.array_equal(oracle.negacyclic_mul_small(a, s, q), dense_negacyclic(a, s, q))


def test_multiplying_by_X_N_times_negates(oracle):
    """X^N = -1 in the ring: N successive multiplications by X negate the polynomial"""
    N = 32
    q = ci.limb_primes(50, 16, 1)[0]
    a0 = ci.uniform_below(3, 1, (N,), q)
    xpoly = np.zeros(N, np.int8)
    xpoly[1] = 1
    a = a0.copy()
    for step in range(N):
        a = oracle.negacyclic_mul_small(a, xpoly, q)
        if step == 0:   # one multiplication by X is a right shift with the top wrapping negated
            assert a[0] == (q - int(a0[N - 1])) % q and np.array_equal(a[1:], a0[:-1])
    assert np.array_equal(a, (np.uint64(q) - a0) % np.uint64(q))


def _toy(seed, rows, N, L, t_bits, q_bits):
    moduli = ci.limb_primes(q_bits, t_bits, L)
    s = ci.gen_secret(seed, N)
    a, e = ci.gen_enc_randomness(seed, rows, 1, moduli, N)
    return moduli, s, a[:, 0], e[:, 0]


@pytest.mark.parametrize("L,t_bits,q_bits", [(1, 16, 50), (2, 20, 54)])
def test_encrypt_decrypt_round_trip(oracle, L, t_bits, q_bits):
    N, rows = 64, 5
    moduli, s, a, e = _toy(11, rows, N, L, t_bits, q_bits)
    w_hat = ci.uniform_below(11, 4, (rows, N), 1 << t_bits)
    w_hat[0, :4] = [(1 << t_bits) - 1, 0, 1, (1 << t_bits) - 1]
    ct = oracle.encrypt(w_hat, s, a, e, moduli, t_bits)
    for r in range(rows):
        assert np.array_equal(ct[r, 1], a[r])           # c1 is the uniform polynomial
        got, noise = oracle.decrypt(ct[r], s, moduli, t_bits, with_noise=True)
        assert np.array_equal(got, w_hat[r])
        assert np.array_equal(noise, e[r].astype(np.int64))   # fresh noise is exactly e


def test_phase_is_delta_m_plus_e(oracle):
    """c0 + c1 s = Delta m + e  (mod Q), checked per limb with Python ints"""
    N, L, t_bits = 32, 2, 20
    moduli, s, a, e = _toy(5, 1, N, L, t_bits, 54)
    w_hat = ci.uniform_below(5, 4, (1, N), 1 << t_bits)
    ct = oracle.encrypt(w_hat, s, a, e, moduli, t_bits)
    phi = oracle.phase(ct[0], s, moduli)
    Q = moduli[0] * moduli[1]
    Delta = Q // (1 << t_bits)
    for l, q in enumerate(moduli):
        want = [(Delta * int(w) + int(err)) % q for w, err in zip(w_hat[0], e[0])]
        assert phi[l].tolist() == want


def test_additive_and_scalar_homomorphism(oracle):
    """Appendix B.1: (+) decrypts to m0 + m1, c (x) ct decrypts to c * m  (mod t)"""
    N, L, t_bits = 64, 2, 20
    t = 1 << t_bits
    moduli, s, a, e = _toy(21, 2, N, L, t_bits, 54)
    w_hat = ci.uniform_below(21, 4, (2, N), t)
    ct = oracle.encrypt(w_hat, s, a, e, moduli, t_bits)
    qv = np.array(moduli, dtype=object).reshape(1, L, 1)
    added = ((ct[0].astype(object) + ct[1].astype(object)) % qv).astype(np.uint64)
    assert np.array_equal(oracle.decrypt(added, s, moduli, t_bits), (w_hat[0] + w_hat[1]) % t)
    c = 123457
    scaled = ((ct[0].astype(object) * c) % qv).astype(np.uint64)
    assert np.array_equal(oracle.decrypt(scaled, s, moduli, t_bits), (w_hat[0] * c) % t)
    # the same two facts through cop_ref: X = [[1, 1]] and X = [[c, 0]]
    ctW = ct.reshape(2, 1, 2, L, N)
    out, _ = oracle.cop_ref(np.array([[1, 1], [c, 0]], np.uint64), ctW, moduli, N, N, None)
    assert np.array_equal(out[0, 0], added) and np.array_equal(out[1, 0], scaled)


def test_encode_rows_eq2_and_chunking(oracle):
    k, n, N = 3, 21, 8
    W = np.arange(k * n, dtype=np.uint64).reshape(k, n) + 1
    w_hat = oracle.encode_rows(W, N)
    assert w_hat.shape == (k, 3, N)
    for i in range(k):
        flat = w_hat[i].reshape(-1)
        assert np.array_equal(flat[:n], W[i])       # w_hat_i[j] = W[i][j]
        assert (flat[n:] == 0).all()                # the last N - n coefficients are zero
    w_hat = oracle.encode_rows(W[:, :5], N)         # n < N: one chunk, zero tail
    assert w_hat.shape == (k, 1, N) and np.array_equal(w_hat[:, 0, :5], W[:, :5])
    assert (w_hat[:, 0, 5:] == 0).all()


def _protocol_case(oracle, seed, m, k, n, N, L, t_bits, q_bits, rows_to_check):
    """encrypt W for real, run cop_ref with the share mask, decrypt, compare with brute force"""
    t = 1 << t_bits
    moduli = ci.limb_primes(q_bits, t_bits, L)
    Ch = -(-n // N)
    X = ci.gen_X(seed, m, k, t_bits)
    W = ci.gen_W(seed, k, n, t_bits)
    s = ci.gen_secret(seed, N)
    a, e = ci.gen_enc_randomness(seed, k, Ch, moduli, N)
    R = ci.gen_R(seed, m, Ch * N, t_bits)
    w_hat = oracle.encode_rows(W, N)                                  # [k][Ch][N]
    ct = oracle.encrypt(w_hat.reshape(k * Ch, N), s, a.reshape(k * Ch, L, N),
                        e.reshape(k * Ch, N), moduli, t_bits)
    ctW = ct.reshape(k, Ch, 2, L, N)
    mask = np.stack([np.stack([oracle.share_mask(R[j, ch * N:(ch + 1) * N], moduli, t_bits)
                               for ch in range(Ch)]) for j in range(m)])
    out, _ = oracle.cop_ref(X, ctW, moduli, n, N, mask)
    XW = X.astype(object) @ W.astype(object)                          # brute force, exact
    noise_max = 0
    for j in rows_to_check:
        for ch in range(Ch):
            dec, noise = oracle.decrypt(out[j, ch], s, moduli, t_bits, with_noise=True)
            got = (dec + R[j, ch * N:(ch + 1) * N]) % np.uint64(t)
            want = np.zeros(N, dtype=np.uint64)
            lo, hi = ch * N, min(n, (ch + 1) * N)
            want[:hi - lo] = (XW[j, lo:hi] % t).astype(np.uint64)
            assert np.array_equal(got, want), (j, ch)
            noise_max = max(noise_max, int(np.abs(noise).max()))
    # noise after the accumulation: k shares times (|e| <= 19) plus the k*t wrap term
    assert noise_max <= k * t * 19 + k * t
    return noise_max


def test_protocol_invariant_config1_full(oracle):
    cfg = ci.CONFIGS[1]
    _protocol_case(oracle, ci.config_seed(1), cfg.m, cfg.k, cfg.n, cfg.N, cfg.L,
                   cfg.t_bits, cfg.q_bits, range(cfg.m))


def test_protocol_invariant_two_limbs_and_chunks(oracle):
    # n > N: three chunks, the last one partial; two limbs
    _protocol_case(oracle, 77, 5, 24, 150, 64, 2, 20, 54, range(5))


def test_phase_linearity_for_uniform_ciphertexts(oracle):
    """phi(out_j) = sum_i X[j,i] phi(ct_i) + phi(mask_j) mod q_l also for random 'ciphertexts':
    catches polynomial / limb / chunk index mix-ups without any real encryption"""
    m, k, n, N, L, t_bits = 3, 6, 40, 16, 3, 24
    moduli = ci.limb_primes(55, t_bits, L)
    Ch = -(-n // N)
    X = ci.gen_X(8, m, k, t_bits)
    ctW = ci.gen_ctW_uniform(8, k, Ch, moduli, N)
    mask = ci.gen_mask_uniform(8, m, Ch, moduli, N)
    s = ci.gen_secret(8, N)
    out, _ = oracle.cop_ref(X, ctW, moduli, n, N, mask)
    qv = np.array(moduli, dtype=object).reshape(L, 1)
    for j in range(m):
        for ch in range(Ch):
            acc = oracle.phase(mask[j, ch], s, moduli).astype(object)
            for i in range(k):
                acc = acc + int(X[j, i]) * oracle.phase(ctW[i, ch], s, moduli).astype(object)
            assert np.array_equal(oracle.phase(out[j, ch], s, moduli), (acc % qv).astype(np.uint64))


def test_primes_are_one_mod_t_and_distinct():
    for cfg in ci.CONFIGS.values():
        qs = cfg.moduli
        assert len(set(qs)) == cfg.L
        for q in qs:
            assert ci.is_prime(q) and q % cfg.t == 1 and q % (2 * cfg.N) == 1
            assert (1 << (cfg.q_bits - 1)) < q < (1 << cfg.q_bits)
