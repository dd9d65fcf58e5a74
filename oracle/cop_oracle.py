"""ctypes front end of the CPU oracle (oracle/nimbus_oracle.c).

TEST INFRASTRUCTURE ONLY.  Imported by tests/, by the smoke check and by the
benchmark's cpu_baseline leg; the product package never imports it.  All the
arithmetic lives in the C file; this module only marshals numpy arrays.
"""
from __future__ import annotations

import ctypes
import os

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libnimbus_oracle.so")
_lib = None

_u64p = ctypes.POINTER(ctypes.c_uint64)
_i64p = ctypes.POINTER(ctypes.c_int64)
_i8p = ctypes.POINTER(ctypes.c_int8)


def _load():
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        from . import build as _b
        _b.build(force=True)
    lib = ctypes.CDLL(_LIB_PATH)
    lib.oracle_max_threads.restype = ctypes.c_int
    lib.oracle_cop_ref.restype = ctypes.c_int
    lib.oracle_cop_ref.argtypes = [_u64p, ctypes.c_int, ctypes.c_int, _u64p, ctypes.c_int,
                                   ctypes.c_int, ctypes.c_int, _u64p, _u64p, _u64p, ctypes.c_int]
    lib.oracle_encode_rows.restype = None
    lib.oracle_encode_rows.argtypes = [_u64p, ctypes.c_int, ctypes.c_int, ctypes.c_int, _u64p]
    lib.oracle_negacyclic_mul_small.restype = None
    lib.oracle_negacyclic_mul_small.argtypes = [_u64p, _i8p, ctypes.c_int, ctypes.c_uint64, _u64p]
    lib.oracle_encrypt.restype = ctypes.c_int
    lib.oracle_encrypt.argtypes = [_u64p, ctypes.c_int, _i8p, _u64p, _i8p, ctypes.c_int,
                                   ctypes.c_int, _u64p, ctypes.c_int, _u64p, ctypes.c_int]
    lib.oracle_phase.restype = None
    lib.oracle_phase.argtypes = [_u64p, _i8p, ctypes.c_int, ctypes.c_int, _u64p, _u64p]
    lib.oracle_decrypt.restype = ctypes.c_int
    lib.oracle_decrypt.argtypes = [_u64p, _i8p, ctypes.c_int, ctypes.c_int, _u64p, ctypes.c_int,
                                   _u64p, _i64p]
    lib.oracle_share_mask.restype = ctypes.c_int
    lib.oracle_share_mask.argtypes = [_u64p, ctypes.c_int, ctypes.c_int, _u64p, ctypes.c_int, _u64p]
    lib.oracle_encrypt_rns.restype = ctypes.c_int
    lib.oracle_encrypt_rns.argtypes = lib.oracle_encrypt.argtypes
    lib.oracle_decrypt_rns.restype = ctypes.c_int
    lib.oracle_decrypt_rns.argtypes = [_u64p, _i8p, ctypes.c_int, ctypes.c_int, _u64p, ctypes.c_int,
                                       _u64p]
    lib.oracle_share_mask_rns.restype = ctypes.c_int
    lib.oracle_share_mask_rns.argtypes = lib.oracle_share_mask.argtypes
    lib.oracle_rshift.restype = None
    lib.oracle_rshift.argtypes = [_u64p, ctypes.c_int, ctypes.c_int, ctypes.c_int, _u64p, _u64p]
    lib.oracle_pack_ref.restype = ctypes.c_int
    lib.oracle_pack_ref.argtypes = [_u64p, ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_int,
                                    _u64p, _u64p, _u64p]
    _lib = lib
    return lib


def _u64(a, shape=None):
    a = np.ascontiguousarray(a, dtype=np.uint64)
    if shape is not None:
        assert a.shape == tuple(shape), (a.shape, shape)
    return a


def _p(a, typ=_u64p):
    return a.ctypes.data_as(typ)


def max_threads() -> int:
    return int(_load().oracle_max_threads())


def cop_ref(X, ctW, moduli, n, N, mask=None, threads=None, wide=False):
    """out[m][Ch][2][L][N] = (X @ ctW + mask) mod q_l, the definition.

    X [m][k]; ctW [k][Ch][2][L][N]; mask like out or None.  wide=True: shares of up to 64
    bits (every product reduced before it is added); otherwise shares of at most 32 bits.
    Returns (out, threads_used).
    """
    lib = _load()
    X = _u64(X)
    m, k = X.shape
    L = len(moduli)
    Ch = -(-n // N)
    ctW = _u64(ctW, (k, Ch, 2, L, N))
    mod = np.asarray(moduli, dtype=np.uint64)
    out = np.empty((m, Ch, 2, L, N), dtype=np.uint64)
    mp = None
    if mask is not None:
        mask = _u64(mask, out.shape)
        mp = _p(mask)
    if threads is None:
        threads = max_threads()
    fn = lib.oracle_cop_ref_wide if wide else lib.oracle_cop_ref
    used = fn(_p(X), m, k, _p(ctW), n, N, L, _p(mod), mp, _p(out), int(threads))
    return out, int(used)


def encode_rows(W, N):
    """Eq. (2) row-wise encoding (+ chunking for n > N): W [k][n] -> [k][Ch][N]"""
    lib = _load()
    W = _u64(W)
    k, n = W.shape
    Ch = -(-n // N)
    w_hat = np.empty((k, Ch, N), dtype=np.uint64)
    lib.oracle_encode_rows(_p(W), k, n, N, _p(w_hat))
    return w_hat


def negacyclic_mul_small(a, s, q):
    lib = _load()
    a = _u64(a)
    s = np.ascontiguousarray(s, dtype=np.int8)
    N = a.shape[0]
    assert s.shape == (N,)
    out = np.empty(N, dtype=np.uint64)
    lib.oracle_negacyclic_mul_small(_p(a), _p(s, _i8p), N, ctypes.c_uint64(int(q)), _p(out))
    return out


def encrypt(w_hat, s, a, e, moduli, t_bits, threads=None):
    """w_hat [rows][N], s [N] int8, a [rows][L][N], e [rows][N] int8 -> ct [rows][2][L][N]"""
    lib = _load()
    w_hat = _u64(w_hat)
    rows, N = w_hat.shape
    L = len(moduli)
    s = np.ascontiguousarray(s, dtype=np.int8)
    a = _u64(a, (rows, L, N))
    e = np.ascontiguousarray(e, dtype=np.int8)
    assert s.shape == (N,) and e.shape == (rows, N)
    mod = np.asarray(moduli, dtype=np.uint64)
    ct = np.empty((rows, 2, L, N), dtype=np.uint64)
    if threads is None:
        threads = max_threads()
    rc = lib.oracle_encrypt(_p(w_hat), rows, _p(s, _i8p), _p(a), _p(e, _i8p), N, L, _p(mod),
                            int(t_bits), _p(ct), int(threads))
    if rc != 0:
        raise ValueError("oracle_encrypt: L > 2 is not supported")
    return ct


def phase(ct, s, moduli):
    """ct [2][L][N] -> phi [L][N] = c0 + c1*s mod q_l"""
    lib = _load()
    ct = _u64(ct)
    _, L, N = ct.shape
    assert ct.shape[0] == 2 and L == len(moduli)
    s = np.ascontiguousarray(s, dtype=np.int8)
    mod = np.asarray(moduli, dtype=np.uint64)
    phi = np.empty((L, N), dtype=np.uint64)
    lib.oracle_phase(_p(ct), _p(s, _i8p), N, L, _p(mod), _p(phi))
    return phi


def decrypt(ct, s, moduli, t_bits, with_noise=False):
    """ct [2][L][N] -> m_hat [N] (and the centred noise, int64)"""
    lib = _load()
    ct = _u64(ct)
    _, L, N = ct.shape
    assert ct.shape[0] == 2 and L == len(moduli)
    s = np.ascontiguousarray(s, dtype=np.int8)
    mod = np.asarray(moduli, dtype=np.uint64)
    m_hat = np.empty(N, dtype=np.uint64)
    noise = np.empty(N, dtype=np.int64)
    rc = lib.oracle_decrypt(_p(ct), _p(s, _i8p), N, L, _p(mod), int(t_bits), _p(m_hat),
                            _p(noise, _i64p))
    if rc != 0:
        raise ValueError("oracle_decrypt: L > 2 is not supported")
    return (m_hat, noise) if with_noise else m_hat


def share_mask(R_row, moduli, t_bits):
    """R_row [N] (< t) -> mask [2][L][N] that subtracts Delta*R_row from c0"""
    lib = _load()
    R_row = _u64(R_row)
    N = R_row.shape[0]
    L = len(moduli)
    mod = np.asarray(moduli, dtype=np.uint64)
    mask = np.empty((2, L, N), dtype=np.uint64)
    rc = lib.oracle_share_mask(_p(R_row), N, L, _p(mod), int(t_bits), _p(mask))
    if rc != 0:
        raise ValueError("oracle_share_mask: L > 2 is not supported")
    return mask


def encrypt_rns(w_hat, s, a, e, moduli, t_bits, threads=None):
    """encrypt() for one to four limbs (256-bit integers instead of 128-bit ones)"""
    lib = _load()
    w_hat = _u64(w_hat)
    rows, N = w_hat.shape
    L = len(moduli)
    s = np.ascontiguousarray(s, dtype=np.int8)
    a = _u64(a, (rows, L, N))
    e = np.ascontiguousarray(e, dtype=np.int8)
    assert s.shape == (N,) and e.shape == (rows, N)
    mod = np.asarray(moduli, dtype=np.uint64)
    ct = np.empty((rows, 2, L, N), dtype=np.uint64)
    if threads is None:
        threads = max_threads()
    rc = lib.oracle_encrypt_rns(_p(w_hat), rows, _p(s, _i8p), _p(a), _p(e, _i8p), N, L, _p(mod),
                                int(t_bits), _p(ct), int(threads))
    if rc != 0:
        raise ValueError("oracle_encrypt_rns: L out of range")
    return ct


def decrypt_rns(ct, s, moduli, t_bits):
    """decrypt() for one to four limbs: ct [2][L][N] -> m_hat [N]"""
    lib = _load()
    ct = _u64(ct)
    _, L, N = ct.shape
    assert ct.shape[0] == 2 and L == len(moduli)
    s = np.ascontiguousarray(s, dtype=np.int8)
    mod = np.asarray(moduli, dtype=np.uint64)
    m_hat = np.empty(N, dtype=np.uint64)
    rc = lib.oracle_decrypt_rns(_p(ct), _p(s, _i8p), N, L, _p(mod), int(t_bits), _p(m_hat))
    if rc != 0:
        raise ValueError("oracle_decrypt_rns: L out of range")
    return m_hat


def share_mask_rns(R_row, moduli, t_bits):
    """share_mask() for one to four limbs"""
    lib = _load()
    R_row = _u64(R_row)
    N = R_row.shape[0]
    L = len(moduli)
    mod = np.asarray(moduli, dtype=np.uint64)
    mask = np.empty((2, L, N), dtype=np.uint64)
    rc = lib.oracle_share_mask_rns(_p(R_row), N, L, _p(mod), int(t_bits), _p(mask))
    if rc != 0:
        raise ValueError("oracle_share_mask_rns: L out of range")
    return mask


def rshift(ct, s, moduli):
    """ct [2][L][N] -> RShift(ct, s): both polynomials times X^s, negacyclic"""
    lib = _load()
    ct = _u64(ct)
    _, L, N = ct.shape
    assert L == len(moduli) and 0 <= s < N
    mod = np.asarray(moduli, dtype=np.uint64)
    out = np.empty_like(ct)
    lib.oracle_rshift(_p(ct), int(s), N, L, _p(mod), _p(out))
    return out


def packed_count(m, n, N):
    """number of packed ciphertexts for m rows of n payload slots in degree N"""
    return -(-m // (N // n))


def pack_ref(rows, n, moduli, mask=None):
    """rows [m][2][L][N] (one ring chunk), mask [ceil(m/P)][2][L][N] or None
    -> packed [ceil(m/P)][2][L][N], P = N // n  (Algorithm 1 step 3, then the mask)"""
    lib = _load()
    rows = _u64(rows)
    m, two, L, N = rows.shape
    assert two == 2 and L == len(moduli) and 0 < n <= N
    T = packed_count(m, n, N)
    mod = np.asarray(moduli, dtype=np.uint64)
    if mask is not None:
        mask = _u64(mask, (T, 2, L, N))
    out = np.empty((T, 2, L, N), dtype=np.uint64)
    rc = lib.oracle_pack_ref(_p(rows), m, int(n), N, L, _p(mod),
                             _p(mask) if mask is not None else None, _p(out))
    if rc != T:
        raise ValueError(f"oracle_pack_ref returned {rc}")
    return out
