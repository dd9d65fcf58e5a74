"""Seeded synthetic inputs for the COP ciphertext x share matmul.

This module only draws random numbers and picks parameters.  It holds none of
the method's arithmetic (no modular accumulation, no encryption, no digit
splitting): both the CPU oracle and the HIP path receive the arrays produced
here as plain inputs.

Workload shapes follow BERT-base linear layers (hidden 768, FFN 3072, fused QKV
2304, 128 tokens; Section 5 "Experimental setup" and Table 5 of the paper) and
the value distributions the protocol fixes: additive shares are uniform over
Z_t (Section 2.3), RLWE ciphertext polynomials are (pseudo-)uniform over Z_q,
masks are uniform (Algorithm 1 step 4).

Dimension names: m = tokens (rows of X), k = inner dimension (rows of W = number
of weight ciphertexts), n = output features, N = ring degree, L = RNS limbs.
The paper calls the first two k and m.
"""
from __future__ import annotations

from dataclasses import dataclass
from functools import lru_cache

import numpy as np

BASE_SEED = 241115707

# tensor tags: one independent Philox stream per (seed, tag)
TAG_X, TAG_CTW, TAG_MASK, TAG_W, TAG_S, TAG_A, TAG_E, TAG_R = 1, 2, 3, 4, 5, 6, 7, 8


@dataclass(frozen=True)
class CopConfig:
    name: str
    m: int          # tokens
    k: int          # inner / reduction dimension
    n: int          # output features
    N: int          # ring degree
    L: int          # RNS limbs
    t_bits: int     # plaintext / share modulus t = 2**t_bits
    q_bits: int     # every limb prime is the largest primes below 2**q_bits with q = 1 mod t
    calls: int = 1  # back-to-back calls with distinct seeds (layer stack)

    @property
    def t(self) -> int:
        return 1 << self.t_bits

    @property
    def Ch(self) -> int:
        return -(-self.n // self.N)

    @property
    def C(self) -> int:
        """independent coefficient columns: chunks x 2 polynomials x limbs x N"""
        return self.Ch * 2 * self.L * self.N

    @property
    def moduli(self) -> tuple:
        return limb_primes(self.q_bits, self.t_bits, self.L)

    @property
    def mod_macs(self) -> int:
        return self.m * self.k * self.C

    @property
    def alg_bytes(self) -> int:
        """ctW read once + mask read + out write + X read, 8 bytes per residue"""
        return 8 * (self.k * self.C + 2 * self.m * self.C + self.m * self.k)


CONFIGS = {
    1: CopConfig("toy", 8, 64, 64, 1024, 1, 16, 50),
    2: CopConfig("bert_base_qkv", 128, 768, 2304, 4096, 2, 20, 54),
    3: CopConfig("bert_base_ffn_up", 128, 768, 3072, 4096, 2, 20, 54),
    4: CopConfig("bert_base_ffn_down", 128, 3072, 768, 4096, 2, 20, 54),
    5: CopConfig("long_seq_large", 512, 1024, 4096, 8192, 3, 24, 55, calls=12),
}


def config_seed(cfg_id: int, call: int = 0) -> int:
    return BASE_SEED + cfg_id + 1000 * call


# ---------------------------------------------------------------------------
# parameter choice: primes q = 1 (mod t).  Since t >= 2N in every configuration
# this also makes them NTT friendly (q = 1 mod 2N).
# ---------------------------------------------------------------------------
def is_prime(n: int) -> bool:
    """deterministic Miller-Rabin, valid for n < 3.3e24"""
    if n < 2:
        return False
    small = (2, 3, 5, 7, 11, 13, 17, 19, 23, 29, 31, 37, 41)
    for p in small:
        if n % p == 0:
            return n == p
    d, r = n - 1, 0
    while d % 2 == 0:
        d //= 2
        r += 1
    for a in small:
        x = pow(a, d, n)
        if x in (1, n - 1):
            continue
        for _ in range(r - 1):
            x = x * x % n
            if x == n - 1:
                break
        else:
            return False
    return True


@lru_cache(maxsize=None)
def limb_primes(q_bits: int, t_bits: int, L: int) -> tuple:
    """the L largest primes below 2**q_bits that are 1 modulo 2**t_bits"""
    t = 1 << t_bits
    out = []
    q = (1 << q_bits) - t + 1
    while len(out) < L:
        if q <= t:
            raise ValueError("no prime found")
        if is_prime(q):
            out.append(q)
        q -= t
    return tuple(out)


# ---------------------------------------------------------------------------
# seeded draws
# ---------------------------------------------------------------------------
def _rng(seed: int, tag: int) -> np.random.Generator:
    return np.random.Generator(np.random.Philox(key=[seed, tag]))


def uniform_below(seed: int, tag: int, shape, bound: int) -> np.ndarray:
    """uint64 array, exactly uniform in [0, bound)"""
    return _rng(seed, tag).integers(0, bound, size=shape, dtype=np.uint64)


def uniform_residues(seed: int, tag: int, lead_shape, moduli, N: int) -> np.ndarray:
    """uint64 array [*lead_shape, L, N]; limb l uniform in [0, moduli[l])"""
    L = len(moduli)
    rng = _rng(seed, tag)
    out = np.empty(tuple(lead_shape) + (L, N), dtype=np.uint64)
    for l, q in enumerate(moduli):
        out[..., l, :] = rng.integers(0, q, size=tuple(lead_shape) + (N,), dtype=np.uint64)
    return out


def gen_X(seed: int, m: int, k: int, t_bits: int) -> np.ndarray:
    """client share matrix, [m][k], uniform in [0, t)"""
    return uniform_below(seed, TAG_X, (m, k), 1 << t_bits)


def gen_ctW_uniform(seed: int, k: int, Ch: int, moduli, N: int) -> np.ndarray:
    """weight ciphertexts as uniform residues, canonical layout [k][Ch][2][L][N]"""
    return uniform_residues(seed, TAG_CTW, (k, Ch, 2), moduli, N)


def gen_mask_uniform(seed: int, m: int, Ch: int, moduli, N: int) -> np.ndarray:
    """mask polynomials, canonical layout [m][Ch][2][L][N]"""
    return uniform_residues(seed, TAG_MASK, (m, Ch, 2), moduli, N)


def gen_W(seed: int, k: int, n: int, t_bits: int) -> np.ndarray:
    """plaintext weights [k][n], uniform in [0, t)"""
    return uniform_below(seed, TAG_W, (k, n), 1 << t_bits)


def gen_R(seed: int, m: int, n_padded: int, t_bits: int) -> np.ndarray:
    """client output share R, [m][n_padded], uniform in [0, t)"""
    return uniform_below(seed, TAG_R, (m, n_padded), 1 << t_bits)


def gen_secret(seed: int, N: int) -> np.ndarray:
    """ternary secret, int8 in {-1, 0, 1}, uniform"""
    return (_rng(seed, TAG_S).integers(0, 3, size=N, dtype=np.int64) - 1).astype(np.int8)


def gen_enc_randomness(seed: int, rows: int, Ch: int, moduli, N: int, sigma: float = 3.2):
    """per-ciphertext encryption randomness.

    Returns (a, e): a uint64 [rows][Ch][L][N] uniform per limb (the same ring
    element is NOT enforced across limbs: every limb of `a` is drawn on its own,
    which is a valid uniform element of R_Q by the CRT), e int8 [rows][Ch][N]
    rounded Gaussian of standard deviation sigma clipped at 6 sigma.
    """
    a = uniform_residues(seed, TAG_A, (rows, Ch), moduli, N)
    bound = int(6 * sigma)
    e = np.rint(_rng(seed, TAG_E).normal(0.0, sigma, size=(rows, Ch, N)))
    e = np.clip(e, -bound, bound).astype(np.int8)
    return a, e
