"""GPU parity of the server side (key tables, encryption of the weight rows, phase, decoding)
against the CPU oracle's schoolbook definitions, bit for bit.

The oracle multiplies by the secret with the O(N^2) negacyclic schoolbook sum; the GPU uses a
number-theoretic transform.  Both are exact, so every output word must be equal.
"""
import sys

import numpy as np
import pytest

import cop_inputs as ci

pytestmark = pytest.mark.gpu


def _say(msg):
    print(msg, flush=True)
    sys.stdout.flush()


def _primes(q_bits, t_bits, N, L):
    # q = 1 modulo 2N (the transform needs a 2N-th root of unity) and modulo t
    return ci.limb_primes(q_bits, max(t_bits, N.bit_length()), L)


def _tables(N, moduli, s):
    import torch
    import paper_2411_15707_amd as nc
    L = len(moduli)
    tables = torch.empty(nc.nimbus_rlwe_tables_bytes(N, L), dtype=torch.uint8, device="cuda")
    nc.nimbus_rlwe_setup(N, L, moduli, torch.from_numpy(s).cuda(), tables)
    return tables


def _gpu_phase(ct, moduli, tables):
    import torch
    import gpu_util as gu
    import paper_2411_15707_amd as nc
    T, _, L, N = ct.shape
    phi = torch.empty((T, L, N), dtype=torch.int64, device="cuda")
    nc.nimbus_rlwe_phase(gu.dev(ct), T, N, L, moduli, tables, phi)
    torch.cuda.synchronize()
    return gu.host(phi)


def _gpu_decrypt(ct, moduli, t_bits, tables):
    import torch
    import gpu_util as gu
    import paper_2411_15707_amd as nc
    T, _, L, N = ct.shape
    phi = torch.empty((T, L, N), dtype=torch.int64, device="cuda")
    m_hat = torch.empty((T, N), dtype=torch.int64, device="cuda")
    nc.nimbus_rlwe_decrypt(gu.dev(ct), T, N, L, moduli, t_bits, tables, phi, m_hat)
    torch.cuda.synchronize()
    return gu.host(m_hat), gu.host(phi)


# N, L, q_bits, T
PHASE_SHAPES = [
    (32, 1, 50, 3),          # smallest ring: 2 + 2 + 1 stages, most threads idle
    (64, 2, 54, 5),          # 2 + 2 + 2 stages
    (128, 3, 55, 2),         # three limbs
    (256, 1, 30, 3),         # small modulus
    (512, 4, 40, 2),         # four limbs, 2 + 2 + 2 + 2 + 1
    (1024, 1, 50, 8),        # config 1 ring
    (2048, 2, 62, 3),        # widest moduli
    (4096, 2, 54, 7),        # BERT-base ring: six rounds of 2 stages, 1024 threads
    (8192, 3, 55, 3),        # config 5 ring: 3 + 3 + 3 + 2 + 2
    (16384, 1, 61, 2),       # largest ring: 136 KiB of LDS, 4 + 4 + 3 + 3
    # the stages per round follow the ring degree and the batch size: batches of 1024
    # polynomials and more take min(4, log N - 8) stages per round (256 threads each), smaller
    # ones (all shapes above) min(4, log N - 10) but at least 2 (up to 1024 threads each)
    (256, 2, 54, 600),       # 1200 polynomials, 2 stages per round
    (2048, 1, 50, 1100),     # 3 stages per round: 3 + 3 + 3 + 2
    (4096, 2, 54, 512),      # BERT-base ring, 1024 polynomials: 4 + 4 + 4
    (8192, 3, 55, 350),      # config 5 ring, 1050 polynomials: 4 + 3 + 3 + 3
    (16384, 2, 61, 520),     # largest ring, 4 + 4 + 3 + 3, two groups per thread and round
    (1024, 1, 50, 1100),     # config 1 ring in a large batch: 2 stages per round
    (32768, 2, 54, 2),       # ring that does not fit the LDS: two halves and a joining pass
    (32768, 1, 62, 3),
    # moduli from 2^34 to 2^58 take the kernels without conditional subtractions: both ends of
    # that range, and the first moduli outside it on either side, at the longest transforms
    (1024, 1, 35, 8),        # smallest moduli of the range
    (1024, 1, 34, 8),        # just below it
    (2048, 2, 59, 3),        # 58 to 59 bits: the same without the cheaper quotient estimate
    (16384, 2, 59, 520),     # ... at 14 stages, two groups per thread and round
    (32768, 1, 59, 2),       # ... a stage on the way in and 14 in the LDS: 31 q in a word
    (2048, 1, 60, 3),        # just above: conditional subtractions
    (4096, 2, 58, 512),      # largest moduli of the range: least room, 4 + 4 + 4
    (8192, 2, 58, 3),        # 3 + 3 + 3 + 2 + 2
    (16384, 1, 58, 2),       # 14 stages
    (16384, 2, 58, 520),     # two groups per thread and round
    (32768, 1, 58, 2),       # a stage on the way in, 14 in the LDS
]


@pytest.mark.parametrize("N,L,q_bits,T", PHASE_SHAPES)
def test_phase_of_uniform_ciphertexts_matches_schoolbook(oracle, N, L, q_bits, T):
    """phi = c0 + c1 s per limb on uniform random ciphertexts (every value of c1 is a valid
    input), ternary secret"""
    seed = 7000 + N + L
    moduli = _primes(q_bits, 16, N, L)
    s = ci.gen_secret(seed, N)
    ct = ci.uniform_residues(seed, 41, (T, 2), moduli, N)
    _say(f"[rlwe] phase N={N} L={L} q_bits={q_bits} T={T}")
    got = _gpu_phase(ct, moduli, _tables(N, moduli, s))
    # (the schoolbook product costs N^2: large batches are checked on a sample of rows)
    rows = range(T) if T <= 16 else sorted({0, 1, T // 3, T // 2, T - 2, T - 1})
    for r in rows:
        want = oracle.phase(ct[r], s, moduli)
        assert np.array_equal(got[r], want), f"ciphertext {r}"


@pytest.mark.parametrize("kind", ["zero", "plus", "minus", "wide"])
def test_phase_with_degenerate_secrets(oracle, kind):
    """s = 0 (phase = c0), all +1, all -1, and coefficients up to +-127 (the table holds the
    transform of any small signed polynomial)"""
    N, L = 256, 2
    moduli = _primes(54, 16, N, L)
    if kind == "zero":
        s = np.zeros(N, dtype=np.int8)
    elif kind == "plus":
        s = np.ones(N, dtype=np.int8)
    elif kind == "minus":
        s = -np.ones(N, dtype=np.int8)
    else:
        s = (np.arange(N) % 255 - 127).astype(np.int8)
    ct = ci.uniform_residues(99, 42, (3, 2), moduli, N)
    _say(f"[rlwe] phase with secret kind {kind}")
    got = _gpu_phase(ct, moduli, _tables(N, moduli, s))
    for r in range(3):
        assert np.array_equal(got[r], oracle.phase(ct[r], s, moduli))
    if kind == "zero":
        assert np.array_equal(got, ct[:, 0])


@pytest.mark.parametrize("N,q_bits", [(1024, 62), (1024, 58), (16384, 58), (32768, 58), (32768, 59)])
def test_phase_with_extreme_residues(oracle, N, q_bits):
    """c1 = q - 1 everywhere and c1 = 0 everywhere: the lazy ranges of the transform at their
    ends, for the widest moduli of either kind of kernel"""
    L = 2
    moduli = _primes(q_bits, 16, N, L)
    s = ci.gen_secret(5, N)
    ct = np.zeros((2, 2, L, N), dtype=np.uint64)
    for l, q in enumerate(moduli):
        ct[0, 1, l] = q - 1
        ct[0, 0, l] = q - 1
    got = _gpu_phase(ct, moduli, _tables(N, moduli, s))
    for r in range(2):
        assert np.array_equal(got[r], oracle.phase(ct[r], s, moduli))


def test_phase_with_the_moduli_of_the_64_bit_setting(oracle):
    """N = 8192 with one 59-bit and one 55-bit limb (Section 5, experimental setup): the limbs of
    one call take the same kernel, the one the wider modulus allows; small and large batch"""
    N = 8192
    moduli = (ci.limb_primes(59, 14, 1)[0], ci.limb_primes(55, 14, 1)[0])
    assert [q.bit_length() for q in moduli] == [59, 55]
    s = ci.gen_secret(64, N)
    tables = _tables(N, moduli, s)
    for T in (3, 520):
        ct = ci.uniform_residues(6400 + T, 43, (T, 2), moduli, N)
        _say(f"[rlwe] phase N={N} moduli of 59 and 55 bits T={T}")
        got = _gpu_phase(ct, moduli, tables)
        for r in sorted({0, T // 2, T - 1}):
            assert np.array_equal(got[r], oracle.phase(ct[r], s, moduli)), f"ciphertext {r}"


# N, L, q_bits, t_bits, T
DECRYPT_SHAPES = [
    (1024, 1, 50, 16, 8),        # config 1 parameters
    (4096, 2, 54, 20, 5),        # BERT-base parameters
    (8192, 2, 55, 24, 2),        # config 5 ring and share width (two limbs: Q < 2^128)
    (64, 1, 30, 7, 3),
    (2048, 2, 62, 32, 3),        # widest plaintext modulus and moduli: Q just below 2^124
    (128, 2, 40, 1, 2),          # t = 2
    (8192, 3, 55, 24, 2),        # config 5 parameters: three limbs, Q ~ 2^165
    (256, 4, 54, 20, 3),         # four limbs
    (512, 4, 62, 32, 2),         # four limbs of 62 bits: Q just below 2^248
    (64, 3, 30, 7, 3),           # three small limbs
    (32768, 2, 55, 24, 2),       # largest ring
    (4096, 2, 58, 20, 5),        # widest moduli of the kernels with the cheaper quotient estimate
    (2048, 2, 59, 20, 3),        # 59 bits: no conditional subtractions, exact quotient
    (1024, 1, 35, 7, 4),         # smallest moduli without conditional subtractions
]


@pytest.mark.parametrize("N,L,q_bits,t_bits,T", DECRYPT_SHAPES)
def test_decrypt_of_uniform_ciphertexts_matches_oracle(oracle, N, L, q_bits, t_bits, T):
    """Dec on uniform random ciphertexts: the phase is uniform in [0, Q), so the rounding
    division sees every region of its input range"""
    seed = 8000 + N + t_bits
    moduli = _primes(q_bits, t_bits, N, L)
    s = ci.gen_secret(seed, N)
    ct = ci.uniform_residues(seed, 43, (T, 2), moduli, N)
    _say(f"[rlwe] decrypt N={N} L={L} q_bits={q_bits} t_bits={t_bits} T={T}")
    got, phi = _gpu_decrypt(ct, moduli, t_bits, _tables(N, moduli, s))
    for r in range(T):
        assert np.array_equal(phi[r], oracle.phase(ct[r], s, moduli)), f"phase of {r}"
        want = oracle.decrypt(ct[r], s, moduli, t_bits) if L <= 2 else \
            oracle.decrypt_rns(ct[r], s, moduli, t_bits)
        assert np.array_equal(got[r], want), f"ciphertext {r}"


@pytest.mark.parametrize("L,q_bits,t_bits", [(1, 50, 16), (2, 54, 20), (2, 62, 32), (1, 20, 3),
                                             (3, 55, 24), (4, 62, 32), (4, 40, 1), (3, 54, 20)])
def test_decode_at_the_rounding_boundaries(oracle, L, q_bits, t_bits):
    """phases placed on and next to the rounding boundaries Delta m + Delta/2, at 0, at Q - 1
    and at the largest m: c1 = 0, so the phase is c0 itself"""
    N = 64
    moduli = _primes(q_bits, t_bits, N, L)
    Q = 1
    for q in moduli:
        Q *= int(q)
    t = 1 << t_bits
    delta = Q >> t_bits
    values = [0, 1, Q - 1, Q - 2, delta // 2, delta // 2 - 1, delta // 2 + 1, delta - 1, delta,
              delta + 1]
    for mm in (1, 2, t // 2, t - 2, t - 1):
        for d in (-2, -1, 0, 1, 2):
            v = delta * mm + delta // 2 + d
            if 0 <= v < Q:
                values.append(v)
            v = delta * mm + d
            if 0 <= v < Q:
                values.append(v)
    values.append(min(Q - 1, delta * t + delta // 2))     # rounds up to t, which wraps to 0
    values.append(min(Q - 1, delta * t + delta // 2 - 1))
    rng = np.random.default_rng(5)
    while len(values) % N:
        values.append(int.from_bytes(rng.bytes(40), "little") % Q)
    T = len(values) // N
    ct = np.zeros((T, 2, L, N), dtype=np.uint64)
    for i, v in enumerate(values):
        for l, q in enumerate(moduli):
            ct[i // N, 0, l, i % N] = v % int(q)
    s = ci.gen_secret(1, N)
    got, _ = _gpu_decrypt(ct, moduli, t_bits, _tables(N, moduli, s))
    for r in range(T):
        want = oracle.decrypt_rns(ct[r], s, moduli, t_bits)
        assert np.array_equal(got[r], want), f"row {r}"
    # and against the plain formula on Python integers
    flat = got.reshape(-1)
    for i, v in enumerate(values):
        assert int(flat[i]) == ((v + delta // 2) // delta) % t, (i, v)


# k, n, N, L, q_bits, t_bits
ENCRYPT_SHAPES = [
    (64, 64, 1024, 1, 50, 16),       # config 1: one chunk, payload far shorter than the ring
    (5, 2500, 1024, 2, 54, 20),      # n > N: three chunks, the last partial
    (7, 32, 32, 1, 30, 7),           # payload fills the ring exactly
    (3, 3072, 4096, 2, 54, 20),      # BERT-base FFN row
    (2, 4096, 8192, 2, 55, 24),      # config 5 row
    (4, 100, 64, 2, 62, 32),         # 32-bit plaintexts, widest moduli, ragged chunks
    (3, 4096, 8192, 3, 55, 24),      # config 5 row with its three limbs
    (5, 200, 128, 4, 54, 20),        # four limbs, two chunks
    (2, 40000, 32768, 2, 55, 24),    # largest ring, two chunks: the joining pass assembles c0
    (3, 5000, 4096, 2, 58, 20),      # moduli at the upper edges of the two kernels without conditional
    (3, 5000, 4096, 2, 59, 20),      # subtractions, two chunks
    (600, 100, 256, 2, 59, 20),      # 1200 polynomials: the large-batch kernel at 59 bits
]


@pytest.mark.parametrize("k,n,N,L,q_bits,t_bits", ENCRYPT_SHAPES)
def test_encrypt_matches_oracle(oracle, k, n, N, L, q_bits, t_bits):
    """row-wise encoding + encryption with the same randomness (a, e) on both sides"""
    import torch
    import gpu_util as gu
    import paper_2411_15707_amd as nc
    seed = 9000 + k + n
    moduli = _primes(q_bits, t_bits, N, L)
    Ch = -(-n // N)
    s = ci.gen_secret(seed, N)
    W = ci.gen_W(seed, k, n, t_bits)
    a, e = ci.gen_enc_randomness(seed, k, Ch, moduli, N)
    _say(f"[rlwe] encrypt k={k} n={n} N={N} L={L} q_bits={q_bits} t_bits={t_bits}")
    w_hat = oracle.encode_rows(W, N)                       # [k][Ch][N]
    enc = oracle.encrypt if L <= 2 else oracle.encrypt_rns
    want = enc(w_hat.reshape(k * Ch, N), s, a.reshape(k * Ch, L, N),
               e.reshape(k * Ch, N), moduli, t_bits).reshape(k, Ch, 2, L, N)
    tables = _tables(N, moduli, s)
    ctW = torch.empty((k, Ch, 2, L, N), dtype=torch.int64, device="cuda")
    nc.nimbus_rlwe_encrypt(gu.dev(W), k, n, t_bits, N, L, moduli, tables, gu.dev(a),
                           torch.from_numpy(e).cuda(), ctW)
    torch.cuda.synchronize()
    got = gu.host(ctW)
    assert np.array_equal(got[:, :, 1], a), "c1 must be the uniform polynomial"
    assert np.array_equal(got, want), gu.first_mismatch(got, want)
    # Dec(Enc(w)) = w-hat on the GPU as well
    m_hat, _ = _gpu_decrypt(got.reshape(k * Ch, 2, L, N), moduli, t_bits, tables)
    assert np.array_equal(m_hat.reshape(k, Ch, N), w_hat)


def test_whole_layer_on_the_gpu_config1(oracle):
    """Algorithm 1 end to end with every step on the GPU: the server encrypts W, the client
    runs the COP accumulation, packs the rows and masks them with its output share, the
    server decrypts; share_client + share_server = X W mod t (Theorem 1)."""
    import torch
    import gpu_util as gu
    import paper_2411_15707_amd as nc
    cfg = ci.CONFIGS[1]
    seed = ci.config_seed(1)
    m, k, n, N, L, t_bits = cfg.m, cfg.k, cfg.n, cfg.N, cfg.L, cfg.t_bits
    moduli = cfg.moduli
    t = 1 << t_bits
    s = ci.gen_secret(seed, N)
    W = ci.gen_W(seed, k, n, t_bits)
    X = ci.gen_X(seed, m, k, t_bits)
    a, e = ci.gen_enc_randomness(seed, k, 1, moduli, N)
    tables = _tables(N, moduli, s)
    # server, setup phase
    ctW = torch.empty((k, 1, 2, L, N), dtype=torch.int64, device="cuda")
    nc.nimbus_rlwe_encrypt(gu.dev(W), k, n, t_bits, N, L, moduli, tables, gu.dev(a),
                           torch.from_numpy(e).cuda(), ctW)
    # client, online phase: accumulate, pack, mask with -R
    P = N // n
    Tn = nc.nimbus_cop_packed_count(m, n, N)
    R = ci.gen_R(seed, Tn, N, t_bits)
    pmask = np.stack([oracle.share_mask(R[th], moduli, t_bits) for th in range(Tn)])
    rows = gu.run_mfma(X, gu.host(ctW), moduli, n, N, t_bits, None)          # [m][1][2][L][N]
    packed = torch.empty((Tn, 2, L, N), dtype=torch.int64, device="cuda")
    nc.nimbus_cop_pack(gu.dev(rows[:, 0]), m, n, N, L, moduli, gu.dev(pmask), packed)
    # server, online phase: decrypt
    phi = torch.empty((Tn, L, N), dtype=torch.int64, device="cuda")
    m_hat = torch.empty((Tn, N), dtype=torch.int64, device="cuda")
    nc.nimbus_rlwe_decrypt(packed, Tn, N, L, moduli, t_bits, tables, phi, m_hat)
    torch.cuda.synchronize()
    share_server = gu.host(m_hat)
    Y = (X.astype(object) @ W.astype(object)) % t
    for th in range(Tn):
        total = (share_server[th].astype(object) + R[th].astype(object)) % t
        for u in range(P):
            j = th * P + u
            want = Y[j] if j < m else np.zeros(n, dtype=object)
            assert np.array_equal(total[u * n:(u + 1) * n], want), (th, u)
    # the GPU decryption equals the oracle's on the same ciphertexts
    pk = gu.host(packed)
    for th in range(Tn):
        assert np.array_equal(share_server[th], oracle.decrypt(pk[th], s, moduli, t_bits))


def test_whole_layer_on_the_gpu_three_limbs(oracle):
    """the same end to end with config 5's parameters (three 55-bit limbs, t = 2^24) on a small
    shape with three rows per packed ciphertext"""
    import torch
    import gpu_util as gu
    import paper_2411_15707_amd as nc
    m, k, n, N, L, t_bits, q_bits = 8, 48, 40, 128, 3, 24, 55
    moduli = _primes(q_bits, t_bits, N, L)
    seed = 5150
    t = 1 << t_bits
    s = ci.gen_secret(seed, N)
    W = ci.gen_W(seed, k, n, t_bits)
    X = ci.gen_X(seed, m, k, t_bits)
    a, e = ci.gen_enc_randomness(seed, k, 1, moduli, N)
    tables = _tables(N, moduli, s)
    ctW = torch.empty((k, 1, 2, L, N), dtype=torch.int64, device="cuda")
    nc.nimbus_rlwe_encrypt(gu.dev(W), k, n, t_bits, N, L, moduli, tables, gu.dev(a),
                           torch.from_numpy(e).cuda(), ctW)
    P = N // n
    Tn = nc.nimbus_cop_packed_count(m, n, N)
    R = ci.gen_R(seed, Tn, N, t_bits)
    pmask = np.stack([oracle.share_mask_rns(R[th], moduli, t_bits) for th in range(Tn)])
    rows = gu.run_mfma(X, gu.host(ctW), moduli, n, N, t_bits, None)
    packed = torch.empty((Tn, 2, L, N), dtype=torch.int64, device="cuda")
    nc.nimbus_cop_pack(gu.dev(rows[:, 0]), m, n, N, L, moduli, gu.dev(pmask), packed)
    phi = torch.empty((Tn, L, N), dtype=torch.int64, device="cuda")
    m_hat = torch.empty((Tn, N), dtype=torch.int64, device="cuda")
    nc.nimbus_rlwe_decrypt(packed, Tn, N, L, moduli, t_bits, tables, phi, m_hat)
    torch.cuda.synchronize()
    share_server = gu.host(m_hat)
    Y = (X.astype(object) @ W.astype(object)) % t
    for th in range(Tn):
        total = (share_server[th].astype(object) + R[th].astype(object)) % t
        for u in range(P):
            j = th * P + u
            want = Y[j] if j < m else np.zeros(n, dtype=object)
            assert np.array_equal(total[u * n:(u + 1) * n], want), (th, u)
        assert np.array_equal(share_server[th],
                              oracle.decrypt_rns(gu.host(packed)[th], s, moduli, t_bits))


def test_random_parameter_sweep_server_side(oracle):
    """sixty seeded random parameter sets (ring degree 32..1024, one to four limbs of different
    sizes, plaintext widths 1..32 bits, one or two chunks): decryption of uniform ciphertexts
    and encryption of random rows against the oracle"""
    import torch
    import gpu_util as gu
    import paper_2411_15707_amd as nc
    rng = np.random.default_rng(241115707)
    for case in range(60):
        N = int(rng.choice([32, 64, 128, 256, 512, 1024]))
        L = int(rng.integers(1, 5))
        t_bits = int(rng.integers(1, 33))
        need = max(t_bits, N.bit_length())
        moduli = []
        while len(moduli) < L:
            b = int(rng.integers(max(need + 6, 20), 63))
            try:
                q = ci.limb_primes(b, need, 1)[0]
            except ValueError:
                continue
            if q not in moduli:
                moduli.append(q)
        moduli = tuple(moduli)
        T = int(rng.integers(1, 6))
        k, n = int(rng.integers(1, 4)), int(rng.integers(1, 2 * N + 1))
        Ch = -(-n // N)
        label = (f"sweep {case}: N={N} L={L} t_bits={t_bits} "
                 f"q_bits={[q.bit_length() for q in moduli]} T={T} k={k} n={n}")
        _say("[rlwe] " + label)
        s = ci.gen_secret(50000 + case, N)
        ct = ci.uniform_residues(50000 + case, 3, (T, 2), moduli, N)
        tables = _tables(N, moduli, s)
        m_hat, phi = _gpu_decrypt(ct, moduli, t_bits, tables)
        for r in range(T):
            assert np.array_equal(phi[r], oracle.phase(ct[r], s, moduli)), label
            assert np.array_equal(m_hat[r], oracle.decrypt_rns(ct[r], s, moduli, t_bits)), label
        W = ci.gen_W(50000 + case, k, n, t_bits)
        a, e = ci.gen_enc_randomness(50000 + case, k, Ch, moduli, N)
        ctW = torch.empty((k, Ch, 2, L, N), dtype=torch.int64, device="cuda")
        nc.nimbus_rlwe_encrypt(gu.dev(W), k, n, t_bits, N, L, moduli, tables, gu.dev(a),
                               torch.from_numpy(e).cuda(), ctW)
        torch.cuda.synchronize()
        want = oracle.encrypt_rns(oracle.encode_rows(W, N).reshape(k * Ch, N), s,
                                  a.reshape(k * Ch, L, N), e.reshape(k * Ch, N), moduli, t_bits)
        assert np.array_equal(gu.host(ctW).reshape(want.shape), want), label
