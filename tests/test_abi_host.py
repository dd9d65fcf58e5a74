"""CPU-side checks of the C ABI: the library loads, exports every declared symbol,
and rejects bad arguments before anything reaches a GPU."""
import ctypes
import os
import re

import pytest

import cop_inputs as ci
import paper_2411_15707_amd as nc

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_functions():
    text = open(os.path.join(ROOT, "include", "nimbus_cop.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(nimbus_cop_\w+)\s*\(", text)))


def test_header_and_binding_agree():
    assert declared_functions() == sorted(nc.EXPORTED_SYMBOLS)


def test_library_exports_every_declared_symbol():
    lib = ctypes.CDLL(nc.lib_path())
    for name in declared_functions():
        assert hasattr(lib, name), name
    # the calibration header of the benchmark
    text = open(os.path.join(ROOT, "include", "nimbus_calib.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    calib = sorted(set(re.findall(r"\b(nimbus_calib_\w+)\s*\(", text)))
    assert calib == sorted(nc.CALIBRATION_SYMBOLS)
    for name in calib:
        assert hasattr(lib, name), name


def test_version_and_strerror():
    assert nc.nimbus_cop_version() >= 100
    assert nc.nimbus_cop_strerror(0) == "ok"
    for code in (-1, -2, -3, -4, -99):
        assert nc.nimbus_cop_strerror(code)


def test_size_queries():
    cfg = ci.CONFIGS[3]
    # 7 signed byte planes per residue (k padded to 32) + one column sum per column
    want = (cfg.C // 32) * (cfg.k // 32) * 7 * 1024 + cfg.C * 8
    assert nc.nimbus_cop_prepared_bytes(cfg.k, cfg.n, cfg.N, cfg.L, cfg.moduli) == want
    assert nc.nimbus_cop_workspace_bytes(cfg.m, cfg.k, cfg.t_bits) == 4 * 24 * 3 * 1024
    # ragged m and k round up to whole 32 x 32 tiles
    assert nc.nimbus_cop_workspace_bytes(33, 65, 16) == 2 * 3 * 2 * 1024
    assert nc.nimbus_cop_prepared_bytes(0, 8, 32, 1, (97,)) == 0
    assert nc.nimbus_cop_workspace_bytes(0, 8, 16) == 0
    # sizes whose rounding up would leave the range of an int are refused, not wrapped
    assert nc.nimbus_cop_workspace_bytes(2**31 - 1, 64, 20) == 0
    assert nc.nimbus_cop_workspace_bytes(1 << 30, 64, 20) == (1 << 25) * 2 * 3 * 1024
    assert nc.nimbus_cop_prepared_bytes(4, 2**31 - 1, 65536, 1, (cfg.moduli[0],)) == 0
    assert nc.nimbus_cop_packed_count(2**31 - 1, 4, 32) == 0


def _raw():
    lib = nc.load_library()
    return lib


@pytest.mark.parametrize("kw", [
    dict(m=0), dict(k=0), dict(n=0), dict(N=48), dict(N=16), dict(N=1 << 17), dict(L=0), dict(L=5),
    dict(x_bits=0), dict(x_bits=65), dict(moduli=(1 << 54,)), dict(moduli=((1 << 62) + 1,)),
    dict(moduli=(65537,), x_bits=20), dict(X=None), dict(ctW=None), dict(out=None),
    dict(moduli=None), dict(m=(1 << 30) + 1), dict(m=2**31 - 1), dict(n=2**31 - 1),
    dict(n=2**31 - 1, N=65536),
])
def test_invalid_arguments_are_rejected_on_the_host(kw):
    """every bad call returns INVALID_ARG without touching the (dummy, never dereferenced) pointers"""
    lib = _raw()
    a = dict(X=0x1000, m=4, k=8, x_bits=16, ctW=0x2000, n=32, N=32, L=1,
             moduli=ci.limb_primes(50, 16, 1), mask=None, out=0x3000)
    a.update(kw)
    mod = None
    if a["moduli"] is not None:
        mod = (ctypes.c_uint64 * len(a["moduli"]))(*a["moduli"])
    rc = lib.nimbus_cop_matmul(a["X"], a["m"], a["k"], a["x_bits"], a["ctW"], a["n"], a["N"],
                               a["L"], mod, a["mask"], a["out"], None)
    assert rc == -1
    rc = lib.nimbus_cop_matmul_prepared(a["X"], a["m"], a["k"], a["x_bits"], a["ctW"], a["n"],
                                        a["N"], a["L"], mod, a["mask"], a["out"], 0x4000, 1 << 30,
                                        None)
    assert rc == -1
    rc = lib.nimbus_cop_matmul_prepared_static(a["X"], a["m"], a["k"], a["x_bits"], a["ctW"],
                                               a["n"], a["N"], a["L"], mod, a["mask"], a["out"],
                                               None)
    assert rc == -1


def test_static_workspace_limit_is_checked_on_the_host():
    """the entry point without allocation refuses shares beyond its built-in 8 MiB buffer
    before it asks the runtime for anything"""
    lib = _raw()
    mod = (ctypes.c_uint64 * 1)(*ci.limb_primes(54, 20, 1))
    m = 32 * 2731 + 1                  # 2732 row tiles x 1 k-block x 3 planes x 1 KiB > 8 MiB
    assert nc.nimbus_cop_workspace_bytes(m, 32, 20) == 2732 * 3 * 1024
    rc = lib.nimbus_cop_matmul_prepared_static(0x1000, m, 32, 20, 0x2000, 32, 32, 1, mod, None,
                                               0x1000000, None)
    assert rc == -5
    assert "built-in" in nc.nimbus_cop_strerror(-5)
    # unsupported parameters are reported as such, not as a size problem
    rc = lib.nimbus_cop_matmul_prepared_static(0x1000, 4, 50000, 20, 0x2000, 32, 32, 1, mod, None,
                                               0x3000, None)
    assert rc == -2


def test_batch_entry_points_check_their_arguments_on_the_host():
    """the entry points that take several problems in one launch: count, the pointer arrays, a
    mask for every problem or for none, no output on top of another buffer of the batch"""
    lib = _raw()
    mod = (ctypes.c_uint64 * 1)(*ci.limb_primes(54, 20, 1))
    vp = ctypes.c_void_p
    m, k, n, N, L, xb = 4, 64, 32, 32, 1, 20
    out_bytes = m * 2 * L * N * 8

    def arr(*v):
        return (vp * len(v))(*v)
    good = dict(staged=arr(0x100000, 0x200000), prep=arr(0x300000, 0x400000),
                masks=arr(0x500000, 0x600000), outs=arr(0x700000, 0x800000))

    def call(count=2, **kw):
        a = dict(good, **kw)
        return lib.nimbus_cop_matmul_staged_batch(count, a["staged"], m, k, xb, a["prep"], n, N, L, mod,
                                                  a["masks"], a["outs"], None)
    assert call(count=0) == -1
    assert call(count=17) == -1
    assert call(staged=None) == -1
    assert call(outs=arr(0x700000, None)) == -1
    assert call(prep=arr(0x300000, 0x400008)) == -1                      # misaligned
    assert call(masks=arr(0x500000, None)) == -1                         # a mask for one problem only
    assert call(outs=arr(0x700000, 0x700000 + out_bytes // 2)) == -1     # outputs on top of each other
    assert call(outs=arr(0x700000, 0x500000)) == -1                      # output on another problem's mask
    assert call(outs=arr(0x700000, 0x300000)) == -1                      # output on prepared weights
    assert lib.nimbus_cop_matmul_staged_batch(2, good["staged"], m, k, 40, good["prep"], n, N, L, mod,
                                              None, good["outs"], None) == -2      # wide shares
    assert lib.nimbus_cop_matmul_staged_batch(2, good["staged"], m, 50000, xb, good["prep"], n, N, L, mod,
                                              None, good["outs"], None) == -2      # k beyond the bound
    # staging
    ws = nc.nimbus_cop_workspace_bytes(m, k, xb)
    X = arr(0x100000, 0x200000)
    W = arr(0x300000, 0x400000)
    assert lib.nimbus_cop_stage_shares_batch(0, X, m, k, xb, W, ws, None) == -1
    assert lib.nimbus_cop_stage_shares_batch(17, X, m, k, xb, W, ws, None) == -1
    assert lib.nimbus_cop_stage_shares_batch(2, X, m, k, xb, W, ws - 1, None) == -4
    assert lib.nimbus_cop_stage_shares_batch(2, X, m, k, 40, W, ws, None) == -2
    assert lib.nimbus_cop_stage_shares_batch(2, X, m, k, xb, arr(0x300000, 0x300008), ws, None) == -1
    assert lib.nimbus_cop_stage_shares_batch(2, X, m, k, xb, arr(0x300000, 0x300000 + 16), ws, None) == -1
    assert lib.nimbus_cop_stage_shares_batch(2, X, m, k, xb, arr(0x300000, 0x100000), ws, None) == -1


def test_prepared_path_limits_and_buffer_sizes():
    lib = _raw()
    mod = (ctypes.c_uint64 * 1)(*ci.limb_primes(54, 20, 1))
    # k beyond the int32 accumulator bound of the matrix-core kernel
    rc = lib.nimbus_cop_matmul_prepared(0x1000, 4, 50000, 20, 0x2000, 32, 32, 1, mod, None, 0x3000,
                                        0x4000, 1 << 40, None)
    assert rc == -2
    # workspace too small
    rc = lib.nimbus_cop_matmul_prepared(0x1000, 4, 64, 20, 0x2000, 32, 32, 1, mod, None, 0x3000,
                                        0x4000, 16, None)
    assert rc == -4
    # misaligned buffers
    rc = lib.nimbus_cop_matmul_prepared(0x1000, 4, 64, 20, 0x2008, 32, 32, 1, mod, None, 0x3000,
                                        0x4000, 1 << 30, None)
    assert rc == -1
    rc = lib.nimbus_cop_prepare(0x1000, 64, 32, 32, 1, mod, 0x2000, 16, None)
    assert rc == -4
    rc = lib.nimbus_cop_prepare(None, 64, 32, 32, 1, mod, 0x2000, 1 << 30, None)
    assert rc == -1


def test_missing_library_fails_loudly(monkeypatch, tmp_path):
    from paper_2411_15707_amd import binding
    monkeypatch.setattr(binding, "_lib", None)
    monkeypatch.setattr(binding, "_HERE", str(tmp_path))
    with pytest.raises(FileNotFoundError):
        binding.load_library()


def test_packed_count_and_pack_argument_checks():
    lib = _raw()
    assert nc.nimbus_cop_packed_count(128, 768, 4096) == 26        # P = 5
    assert nc.nimbus_cop_packed_count(8, 64, 1024) == 1            # P = 16
    assert nc.nimbus_cop_packed_count(512, 4096, 8192) == 256      # P = 2
    assert nc.nimbus_cop_packed_count(7, 40, 64) == 7              # P = 1
    assert nc.nimbus_cop_packed_count(7, 65, 64) == 0              # n > N
    assert nc.nimbus_cop_packed_count(0, 8, 64) == 0
    mod = (ctypes.c_uint64 * 1)(*ci.limb_primes(50, 16, 1))
    ok = dict(rows=0x1000, m=4, n=16, N=64, L=1, mask=None, packed=0x2000)
    for kw, want in [(dict(rows=None), -1), (dict(packed=None), -1), (dict(packed=0x1000), -1),
                     (dict(m=0), -1), (dict(n=0), -1), (dict(N=48), -1), (dict(L=0), -1),
                     (dict(n=65), -2)]:
        a = dict(ok)
        a.update(kw)
        rc = lib.nimbus_cop_pack(a["rows"], a["m"], a["n"], a["N"], a["L"], mod, a["mask"],
                                 a["packed"], None)
        assert rc == want, (kw, rc)


def test_wide_shares_only_on_the_prepared_path():
    """33..64-bit shares: the canonical-layout entry point answers UNSUPPORTED; the size
    query counts the byte planes of both halves"""
    lib = _raw()
    mod = (ctypes.c_uint64 * 1)(*ci.limb_primes(59, 14, 1))
    rc = lib.nimbus_cop_matmul(0x1000, 4, 8, 64, 0x2000, 32, 32, 1, mod, None, 0x3000, None)
    assert rc == -2
    # 33 rows x 65 k -> 2 x 3 tiles; 4 planes for the lower half + 4 (64 bits) or 2 (40 bits)
    assert nc.nimbus_cop_workspace_bytes(33, 65, 64) == 2 * 3 * (4 + 4) * 1024
    assert nc.nimbus_cop_workspace_bytes(33, 65, 40) == 2 * 3 * (4 + 2) * 1024
    assert nc.nimbus_cop_workspace_bytes(33, 65, 65) == 0


def test_rlwe_header_binding_and_exports_agree():
    text = open(os.path.join(ROOT, "include", "nimbus_rlwe.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    declared = sorted(set(re.findall(r"\b(nimbus_rlwe_\w+)\s*\(", text)))
    assert declared == sorted(nc.RLWE_SYMBOLS)
    lib = ctypes.CDLL(nc.lib_path())
    for name in declared:
        assert hasattr(lib, name), name


def test_rlwe_argument_checks_on_the_host():
    """bad calls of the server-side entry points return before anything is enqueued; the
    pointers are dummies that are never dereferenced"""
    lib = _raw()
    N, L = 64, 2
    good = ci.limb_primes(54, 20, L)                      # = 1 mod 2^20, so also mod 2N
    mod = (ctypes.c_uint64 * L)(*good)
    # per limb three sets (natural order, large batches, small batches) of three tables of N
    # entries of 16 bytes
    assert nc.nimbus_rlwe_tables_bytes(N, L) == L * 3 * 3 * N * 16
    assert nc.nimbus_rlwe_tables_bytes(48, 1) == 0
    assert nc.nimbus_rlwe_tables_bytes(16, 1) == 0
    assert nc.nimbus_rlwe_tables_bytes(32768, 1) == 3 * 3 * 32768 * 16
    assert nc.nimbus_rlwe_tables_bytes(65536, 1) == 0
    assert nc.nimbus_rlwe_tables_bytes(64, 5) == 0
    big = nc.nimbus_rlwe_tables_bytes(N, L)
    # setup
    assert lib.nimbus_rlwe_setup(N, L, mod, None, 0x1000, big, None) == -1
    assert lib.nimbus_rlwe_setup(N, L, mod, 0x2000, None, big, None) == -1
    assert lib.nimbus_rlwe_setup(N, L, None, 0x2000, 0x1000, big, None) == -1
    assert lib.nimbus_rlwe_setup(48, L, mod, 0x2000, 0x1000, big, None) == -1
    assert lib.nimbus_rlwe_setup(N, L, mod, 0x2000, 0x1008, big, None) == -1       # alignment
    assert lib.nimbus_rlwe_setup(N, L, mod, 0x2000, 0x1000, big - 1, None) == -4
    assert lib.nimbus_rlwe_setup(65536, L, mod, 0x2000, 0x1000, 1 << 30, None) == -2
    # a modulus that is not 1 modulo 2N has no 2N-th root of unity
    bad = (ctypes.c_uint64 * 1)(97)                         # 96 is not a multiple of 128
    assert lib.nimbus_rlwe_setup(N, 1, bad, 0x2000, 0x1000, big, None) == -1
    even = (ctypes.c_uint64 * 1)(1 << 20)
    assert lib.nimbus_rlwe_setup(N, 1, even, 0x2000, 0x1000, big, None) == -1
    twice = (ctypes.c_uint64 * 2)(good[0], good[0])         # limbs must be distinct
    assert lib.nimbus_rlwe_setup(N, 2, twice, 0x2000, 0x1000, big, None) == -1
    # phase
    assert lib.nimbus_rlwe_phase(None, 1, N, L, mod, 0x1000, 0x3000, None) == -1
    assert lib.nimbus_rlwe_phase(0x4000, -1, N, L, mod, 0x1000, 0x3000, None) == -1
    assert lib.nimbus_rlwe_phase(0x4000, 0, N, L, mod, 0x1000, 0x3000, None) == 0   # nothing to do
    assert lib.nimbus_rlwe_phase(0x4000, 1, N, L, bad, 0x1000, 0x3000, None) == -1
    # decode / decrypt / encrypt: 1 <= t_bits <= 32, t < q
    five = (ctypes.c_uint64 * 5)(*ci.limb_primes(54, 20, 5))
    assert lib.nimbus_rlwe_decode(0x3000, 1, N, 5, five, 20, 0x5000, None) == -1
    assert lib.nimbus_rlwe_decode(0x3000, 1, N, L, mod, 0, 0x5000, None) == -1
    assert lib.nimbus_rlwe_decode(0x3000, 1, N, L, mod, 33, 0x5000, None) == -1
    assert lib.nimbus_rlwe_decode(0x3000, 0, N, L, mod, 20, 0x5000, None) == 0
    small = (ctypes.c_uint64 * 1)(ci.limb_primes(20, 7, 1)[0])
    assert lib.nimbus_rlwe_decode(0x3000, 1, N, 1, small, 20, 0x5000, None) == -1   # t >= q
    assert lib.nimbus_rlwe_decrypt(0x4000, 1, N, 5, five, 20, 0x1000, 0x3000, 0x5000, None) == -1
    assert lib.nimbus_rlwe_decrypt(0x4000, 1, N, L, mod, 20, 0x1000, None, 0x5000, None) == -1
    assert lib.nimbus_rlwe_encrypt(0x6000, 0, 8, 20, N, L, mod, 0x1000, 0x7000, 0x8000, 0x9000,
                                   None) == -1
    assert lib.nimbus_rlwe_encrypt(0x6000, 4, 8, 33, N, L, mod, 0x1000, 0x7000, 0x8000, 0x9000,
                                   None) == -1
    assert lib.nimbus_rlwe_encrypt(0x6000, 4, 8, 20, N, L, mod, 0x1000, None, 0x8000, 0x9000,
                                   None) == -1


def test_loader_header_binding_and_argument_checks():
    text = open(os.path.join(ROOT, "include", "nimbus_loader.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    declared = sorted(set(re.findall(r"\b(nimbus_loader_\w+)\s*\(", text)))
    assert declared == sorted(nc.LOADER_SYMBOLS)
    lib = _raw()
    for name in declared:
        assert hasattr(lib, name), name
    handle = ctypes.c_void_p()
    assert lib.nimbus_loader_create(0, ctypes.byref(handle)) == -1
    assert lib.nimbus_loader_create(65, ctypes.byref(handle)) == -1
    assert lib.nimbus_loader_create(2, None) == -1
    assert lib.nimbus_loader_destroy(None) == 0
    assert lib.nimbus_loader_load(None, 0, 0x1000, 0x2000, 16, None) == -1
    assert lib.nimbus_loader_acquire(None, 0, None) == -1
    assert lib.nimbus_loader_release(None, 0, None) == -1


def test_check_inputs_argument_checks():
    lib = _raw()
    mod = (ctypes.c_uint64 * 1)(*ci.limb_primes(50, 16, 1))
    assert lib.nimbus_cop_check_inputs(0x1000, 4, 8, 16, 0x2000, 32, 32, 1, mod, None, None, None) == -1
    assert lib.nimbus_cop_check_inputs(None, 4, 8, 16, 0x2000, 32, 32, 1, mod, None, 0x3000, None) == -1
    assert lib.nimbus_cop_check_inputs(0x1000, 4, 8, 16, None, 32, 32, 1, mod, None, 0x3000, None) == -1
    assert lib.nimbus_cop_check_inputs(0x1000, 0, 8, 16, 0x2000, 32, 32, 1, mod, None, 0x3000, None) == -1
    assert lib.nimbus_cop_check_inputs(0x1000, 4, 8, 16, 0x2000, 32, 48, 1, mod, None, 0x3000, None) == -1


def test_overlapping_buffers_are_rejected_on_the_host():
    """a written buffer that shares a byte with a buffer that is read: INVALID_ARG, nothing enqueued
    (dummy addresses, never dereferenced: every call returns before a launch)"""
    lib = _raw()
    mod = (ctypes.c_uint64 * 1)(*ci.limb_primes(54, 20, 1))
    m, k, n, N, L = 4, 64, 32, 32, 1                     # X: 2 KiB, ctW: 32 KiB, out / mask: 2 KiB
    X, W, MK, OUT = 0x100000, 0x200000, 0x300000, 0x400000
    assert lib.nimbus_cop_matmul(X, m, k, 20, W, n, N, L, mod, MK, X + 0x7f8, None) == -1      # last word of X
    assert lib.nimbus_cop_matmul(X, m, k, 20, W, n, N, L, mod, MK, W + 0x7000, None) == -1     # inside ctW
    assert lib.nimbus_cop_matmul(X, m, k, 20, W, n, N, L, mod, MK, MK, None) == -1             # out = mask
    prep = nc.nimbus_cop_prepared_bytes(k, n, N, L, tuple(mod))
    wsb = nc.nimbus_cop_workspace_bytes(m, k, 20)
    PREP, WS = 0x500000, 0x600000
    args = lambda out, ws, prepared=PREP, mask=MK: (X, m, k, 20, prepared, n, N, L, mod, mask, out, ws, wsb, None)
    assert lib.nimbus_cop_matmul_prepared(*args(PREP + prep - 16, WS)) == -1                  # out in prepared
    assert lib.nimbus_cop_matmul_prepared(*args(OUT, OUT + 0x400)) == -1                      # workspace in out
    assert lib.nimbus_cop_matmul_prepared(*args(OUT, X)) == -1                                # workspace = X
    assert lib.nimbus_cop_matmul_staged(WS, m, k, 20, PREP, n, N, L, mod, MK, WS, None) == -1  # out = staged shares
    assert lib.nimbus_cop_prepare(W, k, n, N, L, mod, W + 0x1000, prep, None) == -1
    assert lib.nimbus_cop_stage_shares(X, m, k, 20, X + 0x400, wsb, None) == -1
    # packing: 4 rows of n = 16 columns into one ciphertext of N = 64 (1 KiB each)
    assert lib.nimbus_cop_pack(X, 4, 16, 64, 1, mod, None, X + 0xc00, None) == -1              # packed = last row
    assert lib.nimbus_cop_pack(X, 4, 16, 64, 1, mod, MK, MK + 8, None) == -1                   # packed in mask
    # server side
    N2, L2 = 64, 2
    mod2 = (ctypes.c_uint64 * L2)(*ci.limb_primes(54, 20, L2))
    TAB, CT, PHI, MH = 0x700000, 0x800000, 0x900000, 0xa00000     # ct: 2 KiB per ciphertext, phi 1 KiB
    assert lib.nimbus_rlwe_phase(CT, 2, N2, L2, mod2, TAB, CT + 0x800, None) == -1             # phi = second ciphertext
    assert lib.nimbus_rlwe_decode(PHI, 2, N2, L2, mod2, 20, PHI + 0x400, None) == -1
    assert lib.nimbus_rlwe_decrypt(CT, 2, N2, L2, mod2, 20, TAB, PHI, CT, None) == -1          # m_hat = ct
    assert lib.nimbus_rlwe_decrypt(CT, 2, N2, L2, mod2, 20, TAB, PHI, PHI + 8, None) == -1     # m_hat in phi
    Wp, A, E, CW = 0xb00000, 0xc00000, 0xd00000, 0xe00000
    assert lib.nimbus_rlwe_encrypt(Wp, 4, 8, 20, N2, L2, mod2, TAB, A, E, A + 0x800, None) == -1   # ctW in a
    assert lib.nimbus_rlwe_encrypt(Wp, 4, 8, 20, N2, L2, mod2, TAB, A, E, Wp, None) == -1          # ctW = W
    assert lib.nimbus_rlwe_encrypt(Wp, 4, 8, 20, N2, L2, mod2, TAB, A, E, E, None) == -1           # ctW = e
