"""Pins for the definition oracle cop_ref (Algorithm 1 steps 2 and 4, Appendix B.1 (x)/(+)).

Nothing here re-calls the oracle to check itself: the expected values come from
Python's unbounded integers, from closed forms, or from numpy's object matmul.
"""
import os

import numpy as np
import pytest

import cop_inputs as ci

HERE = os.path.dirname(os.path.abspath(__file__))


def bigint_cop(X, ctW, moduli, N, mask):
    """third implementation: Python ints, one output element at a time"""
    m, k = X.shape
    _, Ch, P, L, _ = ctW.shape
    out = np.empty((m, Ch, P, L, N), dtype=np.uint64)
    Xl = X.tolist()
    for ch in range(Ch):
        for p in range(P):
            for l in range(L):
                q = int(moduli[l])
                cols = ctW[:, ch, p, l, :].T.tolist()      # [N][k]
                for c in range(N):
                    col = cols[c]
                    for j in range(m):
                        acc = 0
                        row = Xl[j]
                        for i in range(k):
                            acc += row[i] * col[i]
                        if mask is not None:
                            acc += int(mask[j, ch, p, l, c])
                        out[j, ch, p, l, c] = acc % q
    return out


def test_config1_full_against_python_ints(oracle):
    cfg = ci.CONFIGS[1]
    seed = ci.config_seed(1)
    X = ci.gen_X(seed, cfg.m, cfg.k, cfg.t_bits)
    ctW = ci.gen_ctW_uniform(seed, cfg.k, cfg.Ch, cfg.moduli, cfg.N)
    mask = ci.gen_mask_uniform(seed, cfg.m, cfg.Ch, cfg.moduli, cfg.N)
    got, _ = oracle.cop_ref(X, ctW, cfg.moduli, cfg.n, cfg.N, mask)
    want = bigint_cop(X, ctW, cfg.moduli, cfg.N, mask)
    assert np.array_equal(got, want)


@pytest.mark.parametrize("m,k,n,N,L,t_bits,q_bits", [
    (3, 5, 10, 16, 3, 24, 55),      # three limbs
    (2, 7, 40, 16, 2, 20, 54),      # n > N: three chunks, last partial
    (4, 9, 16, 16, 1, 32, 62),      # widest share and widest modulus allowed
    (1, 1, 5, 8, 2, 16, 50),
])
def test_small_shapes_against_python_ints(oracle, m, k, n, N, L, t_bits, q_bits):
    moduli = ci.limb_primes(q_bits, t_bits, L)
    Ch = -(-n // N)
    seed = 99 + m * 7 + k
    X = ci.gen_X(seed, m, k, t_bits)
    # push the extremes in: largest share, largest residues
    X[0, 0] = (1 << t_bits) - 1
    ctW = ci.gen_ctW_uniform(seed, k, Ch, moduli, N)
    for l, q in enumerate(moduli):
        ctW[0, 0, 0, l, 0] = q - 1
        ctW[:, 0, 1, l, 1] = q - 1
    mask = ci.gen_mask_uniform(seed, m, Ch, moduli, N)
    mask[0, 0, 0, :, 0] = np.array(moduli, dtype=np.uint64) - np.uint64(1)
    got, _ = oracle.cop_ref(X, ctW, moduli, n, N, mask)
    assert np.array_equal(got, bigint_cop(X, ctW, moduli, N, mask))
    got_nomask, _ = oracle.cop_ref(X, ctW, moduli, n, N, None)
    assert np.array_equal(got_nomask, bigint_cop(X, ctW, moduli, N, None))


def test_numpy_object_matmul(oracle):
    """the path is a textbook integer matmul followed by a column-wise mod"""
    m, k, n, N, L = 6, 33, 64, 64, 2
    moduli = ci.limb_primes(54, 20, L)
    X = ci.gen_X(5, m, k, 20)
    ctW = ci.gen_ctW_uniform(5, k, 1, moduli, N)
    mask = ci.gen_mask_uniform(5, m, 1, moduli, N)
    got, _ = oracle.cop_ref(X, ctW, moduli, n, N, mask)
    C = 2 * L * N
    prod = X.astype(object) @ ctW.reshape(k, C).astype(object) + mask.reshape(m, C).astype(object)
    qcol = np.array([moduli[(c // N) % L] for c in range(C)], dtype=object)
    want = (prod % qcol).astype(np.uint64).reshape(got.shape)
    assert np.array_equal(got, want)


def test_special_cases(oracle):
    m = k = 12
    N, L, n = 32, 2, 20
    moduli = ci.limb_primes(54, 20, L)
    ctW = ci.gen_ctW_uniform(3, k, 1, moduli, N)
    mask = ci.gen_mask_uniform(3, m, 1, moduli, N)
    qv = np.array(moduli, dtype=np.uint64).reshape(1, 1, 1, L, 1)

    # X = 0: the output is the mask
    out, _ = oracle.cop_ref(np.zeros((m, k), np.uint64), ctW, moduli, n, N, mask)
    assert np.array_equal(out, mask)

    # X = identity: a vector add mod q
    out, _ = oracle.cop_ref(np.eye(m, dtype=np.uint64), ctW, moduli, n, N, mask)
    s = ctW + mask                      # < 2^55, no wrap
    want = np.where(s >= qv, s - qv, s)
    assert np.array_equal(out, want)

    # k = 1, X = [1], no mask: a copy
    out, _ = oracle.cop_ref(np.ones((1, 1), np.uint64), ctW[:1], moduli, n, N, None)
    assert np.array_equal(out[0], ctW[0])

    # all-ones row: column sums
    out, _ = oracle.cop_ref(np.ones((1, k), np.uint64), ctW, moduli, n, N, None)
    want = (ctW.astype(object).sum(axis=0) % qv[0].astype(object)).astype(np.uint64)
    assert np.array_equal(out[0], want)

    # a permutation matrix picks rows: out_j = ct_{perm[j]}
    perm = np.random.default_rng(0).permutation(k)
    P = np.zeros((m, k), np.uint64)
    P[np.arange(m), perm] = 1
    out, _ = oracle.cop_ref(P, ctW, moduli, n, N, None)
    assert np.array_equal(out, ctW[perm])


def test_limb_of_a_column_is_its_own_modulus(oracle):
    """two limbs with very different primes: a limb/polynomial index mix-up shows"""
    N, n, k, m = 8, 8, 3, 2
    moduli = (ci.limb_primes(50, 16, 1)[0], ci.limb_primes(30, 16, 1)[0])
    ctW = ci.gen_ctW_uniform(1, k, 1, moduli, N)
    X = ci.gen_X(1, m, k, 16)
    out, _ = oracle.cop_ref(X, ctW, moduli, n, N, None)
    assert np.array_equal(out, bigint_cop(X, ctW, moduli, N, None))
    assert (out[:, :, :, 1, :] < moduli[1]).all()


def test_thread_count_does_not_change_the_result(oracle):
    cfg = ci.CONFIGS[1]
    X = ci.gen_X(1, cfg.m, cfg.k, cfg.t_bits)
    ctW = ci.gen_ctW_uniform(1, cfg.k, cfg.Ch, cfg.moduli, cfg.N)
    a, used1 = oracle.cop_ref(X, ctW, cfg.moduli, cfg.n, cfg.N, None, threads=1)
    b, used4 = oracle.cop_ref(X, ctW, cfg.moduli, cfg.n, cfg.N, None, threads=4)
    assert used1 == 1 and 1 <= used4 <= 4
    assert np.array_equal(a, b)


def test_full_size_samples_against_python_ints(oracle):
    """config 3 shape (the headline workload) on two rows, sampled columns by big ints"""
    cfg = ci.CONFIGS[3]
    seed = ci.config_seed(3)
    X = ci.gen_X(seed, cfg.m, cfg.k, cfg.t_bits)[[0, cfg.m - 1]]
    ctW = ci.gen_ctW_uniform(seed, cfg.k, cfg.Ch, cfg.moduli, cfg.N)
    mask = ci.gen_mask_uniform(seed, cfg.m, cfg.Ch, cfg.moduli, cfg.N)[[0, cfg.m - 1]]
    out, _ = oracle.cop_ref(X, ctW, cfg.moduli, cfg.n, cfg.N, mask)
    flat_ct = ctW.reshape(cfg.k, cfg.C)
    rng = np.random.default_rng(7)
    cols = rng.choice(cfg.C, size=160, replace=False)
    for col in cols.tolist():
        q = cfg.moduli[(col // cfg.N) % cfg.L]
        column = flat_ct[:, col].tolist()
        for jj in range(2):
            acc = sum(int(x) * c for x, c in zip(X[jj].tolist(), column))
            acc += int(mask.reshape(2, cfg.C)[jj, col])
            assert int(out.reshape(2, cfg.C)[jj, col]) == acc % q


def test_table5_sizes_pin_one_dense_ciphertext_per_weight_row():
    """Table 5: bytes = weight rows x 2 polynomials x N x log2(q)/8 with N = 8192, log2 q = 114.

    This fixes the shape of the ciphertext operand: one ciphertext per weight row,
    both polynomials dense in all N coefficients (so the kernel processes all N).
    """
    rows = {}
    with open(os.path.join(HERE, "golden", "table5_encrypted_weight_mb.txt")) as f:
        for line in f:
            if line.startswith("#") or not line.strip():
                continue
            h, qkv, o, h1, h2 = (int(v) for v in line.split())
            rows[h] = (qkv, o, h1, h2)
    N, logq = 8192, 114
    for hidden, (qkv, o, h1, h2) in rows.items():
        per_row = 2 * N * logq / 8
        # qkv, o and h1 have `hidden` weight rows, h2 has 4*hidden
        for printed, nrows in ((qkv, hidden), (o, hidden), (h1, hidden), (h2, 4 * hidden)):
            assert abs(nrows * per_row / 1e6 - printed) / printed < 0.01


def test_table1_client_cost_count():
    """Table 1: client work is tokens x inner x N scalar-coefficient products per polynomial
    limb; the config table's MAC count is that times 2 polynomials x L limbs x chunks."""
    for cfg in ci.CONFIGS.values():
        assert cfg.mod_macs == cfg.m * cfg.k * cfg.N * 2 * cfg.L * cfg.Ch
    assert ci.CONFIGS[3].mod_macs == 1_610_612_736
    assert ci.CONFIGS[3].alg_bytes == 135_004_160
