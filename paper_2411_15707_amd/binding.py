"""ctypes binding of libnimbus_cop.so.  Same names as the C entry points.

Tensors are torch tensors on the GPU holding raw 64-bit words (dtype int64 or
uint64; the library reads them as uint64_t).  There is no CPU fallback: if the
shared library is missing, loading raises.
"""
from __future__ import annotations

import ctypes
import os

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_NAME = "libnimbus_cop.so"
_lib = None
NIMBUS_INVALID = -1

EXPORTED_SYMBOLS = (
    "nimbus_cop_matmul",
    "nimbus_cop_matmul_valu",
    "nimbus_cop_prepared_bytes",
    "nimbus_cop_prepare",
    "nimbus_cop_workspace_bytes",
    "nimbus_cop_stage_shares",
    "nimbus_cop_matmul_staged",
    "nimbus_cop_stage_shares_batch",
    "nimbus_cop_matmul_staged_batch",
    "nimbus_cop_matmul_prepared",
    "nimbus_cop_matmul_prepared_static",
    "nimbus_cop_packed_count",
    "nimbus_cop_pack",
    "nimbus_cop_check_inputs",
    "nimbus_cop_strerror",
    "nimbus_cop_version",
)


CALIBRATION_SYMBOLS = ("nimbus_calib_mfma_i8", "nimbus_calib_stream_read",
                       "nimbus_calib_butterflies")

LOADER_SYMBOLS = (
    "nimbus_loader_create",
    "nimbus_loader_destroy",
    "nimbus_loader_load",
    "nimbus_loader_acquire",
    "nimbus_loader_release",
)

RLWE_SYMBOLS = (
    "nimbus_rlwe_tables_bytes",
    "nimbus_rlwe_setup",
    "nimbus_rlwe_phase",
    "nimbus_rlwe_decode",
    "nimbus_rlwe_decrypt",
    "nimbus_rlwe_encrypt",
)


class NimbusCopError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {nimbus_cop_strerror(status)} (status {status})")


def lib_path() -> str:
    return os.path.join(_HERE, _LIB_NAME)


def load_library():
    """dlopen the HIP library; raises if it has not been built"""
    global _lib
    if _lib is not None:
        return _lib
    path = lib_path()
    if not os.path.exists(path):
        raise FileNotFoundError(
            f"{path} is missing: build it with `python -m paper_2411_15707_amd.build` "
            "(there is no CPU fallback)")
    # The library launches on PyTorch's streams and pointers, so both must use one and the
    # same HIP runtime: PyTorch ships its own copy and loads it by path, and whichever copy
    # is mapped first serves every later request for that soname.  Import torch first.
    import torch  # noqa: F401
    lib = ctypes.CDLL(path)
    vp, ci, sz = ctypes.c_void_p, ctypes.c_int, ctypes.c_size_t
    lib.nimbus_cop_matmul.restype = ci
    lib.nimbus_cop_matmul.argtypes = [vp, ci, ci, ci, vp, ci, ci, ci, vp, vp, vp, vp]
    lib.nimbus_cop_matmul_valu.restype = ci
    lib.nimbus_cop_matmul_valu.argtypes = [vp, ci, ci, ci, vp, ci, ci, ci, vp, vp, vp, vp]
    lib.nimbus_cop_prepared_bytes.restype = sz
    lib.nimbus_cop_prepared_bytes.argtypes = [ci, ci, ci, ci, vp]
    lib.nimbus_cop_prepare.restype = ci
    lib.nimbus_cop_prepare.argtypes = [vp, ci, ci, ci, ci, vp, vp, sz, vp]
    lib.nimbus_cop_workspace_bytes.restype = sz
    lib.nimbus_cop_workspace_bytes.argtypes = [ci, ci, ci]
    lib.nimbus_cop_stage_shares.restype = ci
    lib.nimbus_cop_stage_shares.argtypes = [vp, ci, ci, ci, vp, sz, vp]
    lib.nimbus_cop_matmul_staged.restype = ci
    lib.nimbus_cop_matmul_staged.argtypes = [vp, ci, ci, ci, vp, ci, ci, ci, vp, vp, vp, vp]
    lib.nimbus_cop_stage_shares_batch.restype = ci
    lib.nimbus_cop_stage_shares_batch.argtypes = [ci, vp, ci, ci, ci, vp, sz, vp]
    lib.nimbus_cop_matmul_staged_batch.restype = ci
    lib.nimbus_cop_matmul_staged_batch.argtypes = [ci, vp, ci, ci, ci, vp, ci, ci, ci, vp, vp, vp, vp]
    lib.nimbus_cop_matmul_prepared.restype = ci
    lib.nimbus_cop_matmul_prepared.argtypes = [vp, ci, ci, ci, vp, ci, ci, ci, vp, vp, vp, vp, sz, vp]
    lib.nimbus_cop_matmul_prepared_static.restype = ci
    lib.nimbus_cop_matmul_prepared_static.argtypes = [vp, ci, ci, ci, vp, ci, ci, ci, vp, vp, vp, vp]
    lib.nimbus_cop_packed_count.restype = ci
    lib.nimbus_cop_packed_count.argtypes = [ci, ci, ci]
    lib.nimbus_cop_pack.restype = ci
    lib.nimbus_cop_pack.argtypes = [vp, ci, ci, ci, ci, vp, vp, vp, vp]
    lib.nimbus_cop_check_inputs.restype = ci
    lib.nimbus_cop_check_inputs.argtypes = [vp, ci, ci, ci, vp, ci, ci, ci, vp, vp, vp, vp]
    lib.nimbus_calib_mfma_i8.restype = ctypes.c_longlong
    lib.nimbus_calib_mfma_i8.argtypes = [ci, ci, ci, vp, sz, vp]
    lib.nimbus_calib_stream_read.restype = ctypes.c_longlong
    lib.nimbus_calib_stream_read.argtypes = [vp, sz, vp, vp]
    lib.nimbus_calib_butterflies.restype = ctypes.c_longlong
    lib.nimbus_calib_butterflies.argtypes = [ci, ci, ctypes.c_ulonglong, vp, sz, vp]
    lib.nimbus_rlwe_tables_bytes.restype = sz
    lib.nimbus_rlwe_tables_bytes.argtypes = [ci, ci]
    lib.nimbus_rlwe_setup.restype = ci
    lib.nimbus_rlwe_setup.argtypes = [ci, ci, vp, vp, vp, sz, vp]
    lib.nimbus_rlwe_phase.restype = ci
    lib.nimbus_rlwe_phase.argtypes = [vp, ci, ci, ci, vp, vp, vp, vp]
    lib.nimbus_rlwe_decode.restype = ci
    lib.nimbus_rlwe_decode.argtypes = [vp, ci, ci, ci, vp, ci, vp, vp]
    lib.nimbus_rlwe_decrypt.restype = ci
    lib.nimbus_rlwe_decrypt.argtypes = [vp, ci, ci, ci, vp, ci, vp, vp, vp, vp]
    lib.nimbus_rlwe_encrypt.restype = ci
    lib.nimbus_rlwe_encrypt.argtypes = [vp, ci, ci, ci, ci, ci, vp, vp, vp, vp, vp, vp]
    lib.nimbus_loader_create.restype = ci
    lib.nimbus_loader_create.argtypes = [ci, ctypes.POINTER(vp)]
    lib.nimbus_loader_destroy.restype = ci
    lib.nimbus_loader_destroy.argtypes = [vp]
    lib.nimbus_loader_load.restype = ci
    lib.nimbus_loader_load.argtypes = [vp, ci, vp, vp, sz, vp]
    lib.nimbus_loader_acquire.restype = ci
    lib.nimbus_loader_acquire.argtypes = [vp, ci, vp]
    lib.nimbus_loader_release.restype = ci
    lib.nimbus_loader_release.argtypes = [vp, ci, vp]
    lib.nimbus_cop_strerror.restype = ctypes.c_char_p
    lib.nimbus_cop_strerror.argtypes = [ci]
    lib.nimbus_cop_version.restype = ci
    lib.nimbus_cop_version.argtypes = []
    _lib = lib
    return lib


def _moduli(moduli):
    arr = (ctypes.c_uint64 * len(moduli))(*[int(q) for q in moduli])
    return arr


def _dev_ptr(t, name, allow_none=False):
    if t is None:
        if allow_none:
            return None
        raise ValueError(f"{name} is None")
    if not t.is_cuda:
        raise ValueError(f"{name} must live on the GPU")
    if not t.is_contiguous():
        raise ValueError(f"{name} must be contiguous")
    return ctypes.c_void_p(t.data_ptr())


def _words(t, name, count):
    if t.element_size() != 8:
        raise ValueError(f"{name} must hold 64-bit words")
    if t.numel() != count:
        raise ValueError(f"{name} has {t.numel()} words, expected {count}")


def _stream(stream):
    if stream is None:
        import torch
        return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)
    if isinstance(stream, int):
        return ctypes.c_void_p(stream)
    return ctypes.c_void_p(stream.cuda_stream)


def _columns(n, N, L):
    return (-(-n // N)) * 2 * L * N


def nimbus_cop_strerror(status: int) -> str:
    return load_library().nimbus_cop_strerror(int(status)).decode()


def nimbus_cop_version() -> int:
    return int(load_library().nimbus_cop_version())


def _canonical(entry, X, m, k, x_bits, ctW, n, N, L, moduli, mask, out, stream):
    lib = load_library()
    C = _columns(n, N, L)
    _words(X, "X", m * k)
    _words(ctW, "ctW", k * C)
    _words(out, "out", m * C)
    if mask is not None:
        _words(mask, "mask", m * C)
    rc = getattr(lib, entry)(_dev_ptr(X, "X"), m, k, x_bits, _dev_ptr(ctW, "ctW"), n, N, L,
                             _moduli(moduli), _dev_ptr(mask, "mask", True),
                             _dev_ptr(out, "out"), _stream(stream))
    if rc != 0:
        raise NimbusCopError(rc, entry)


def nimbus_cop_matmul(X, m, k, x_bits, ctW, n, N, L, moduli, mask, out, stream=None):
    _canonical("nimbus_cop_matmul", X, m, k, x_bits, ctW, n, N, L, moduli, mask, out, stream)


def nimbus_cop_matmul_valu(X, m, k, x_bits, ctW, n, N, L, moduli, mask, out, stream=None):
    _canonical("nimbus_cop_matmul_valu", X, m, k, x_bits, ctW, n, N, L, moduli, mask, out, stream)


def nimbus_cop_prepared_bytes(k, n, N, L, moduli) -> int:
    return int(load_library().nimbus_cop_prepared_bytes(k, n, N, L, _moduli(moduli)))


def nimbus_cop_prepare(ctW, k, n, N, L, moduli, prepared, stream=None):
    lib = load_library()
    _words(ctW, "ctW", k * _columns(n, N, L))
    nbytes = prepared.numel() * prepared.element_size()
    rc = lib.nimbus_cop_prepare(_dev_ptr(ctW, "ctW"), k, n, N, L, _moduli(moduli),
                                _dev_ptr(prepared, "prepared"), nbytes, _stream(stream))
    if rc != 0:
        raise NimbusCopError(rc, "nimbus_cop_prepare")


def nimbus_cop_workspace_bytes(m, k, x_bits) -> int:
    return int(load_library().nimbus_cop_workspace_bytes(m, k, x_bits))


def nimbus_cop_stage_shares(X, m, k, x_bits, workspace, stream=None):
    lib = load_library()
    _words(X, "X", m * k)
    ws_bytes = workspace.numel() * workspace.element_size()
    rc = lib.nimbus_cop_stage_shares(_dev_ptr(X, "X"), m, k, x_bits,
                                     _dev_ptr(workspace, "workspace"), ws_bytes, _stream(stream))
    if rc != 0:
        raise NimbusCopError(rc, "nimbus_cop_stage_shares")


def nimbus_cop_matmul_staged(staged, m, k, x_bits, prepared, n, N, L, moduli, mask, out,
                             stream=None):
    lib = load_library()
    C = _columns(n, N, L)
    _words(out, "out", m * C)
    if mask is not None:
        _words(mask, "mask", m * C)
    if staged.numel() * staged.element_size() < nimbus_cop_workspace_bytes(m, k, x_bits):
        raise ValueError("staged shares buffer is smaller than nimbus_cop_workspace_bytes")
    rc = lib.nimbus_cop_matmul_staged(
        _dev_ptr(staged, "staged"), m, k, x_bits, _dev_ptr(prepared, "prepared"), n, N, L,
        _moduli(moduli), _dev_ptr(mask, "mask", True), _dev_ptr(out, "out"), _stream(stream))
    if rc != 0:
        raise NimbusCopError(rc, "nimbus_cop_matmul_staged")


def nimbus_cop_stage_shares_batch(Xs, m, k, x_bits, workspaces, stream=None):
    """nimbus_cop_stage_shares for several share matrices of one shape in one launch"""
    lib = load_library()
    count = len(Xs)
    if len(workspaces) != count:
        raise ValueError("one workspace per share matrix")
    for X in Xs:
        _words(X, "X", m * k)
    size = min(w.numel() * w.element_size() for w in workspaces)
    ptrs = ctypes.c_void_p * count
    rc = lib.nimbus_cop_stage_shares_batch(count, ptrs(*[_dev_ptr(X, "X") for X in Xs]), m, k, x_bits,
                                           ptrs(*[_dev_ptr(w, "workspace") for w in workspaces]),
                                           size, _stream(stream))
    if rc != 0:
        raise NimbusCopError(rc, "nimbus_cop_stage_shares_batch")


def nimbus_cop_matmul_staged_batch(staged, m, k, x_bits, prepared, n, N, L, moduli, masks, outs,
                                   stream=None):
    """`len(outs)` calls of nimbus_cop_matmul_staged in one launch; staged, prepared, masks (or
    None) and outs are sequences of tensors, one per problem"""
    lib = load_library()
    count = len(outs)
    if len(staged) != count or len(prepared) != count or (masks is not None and len(masks) != count):
        raise ValueError("one staged buffer, one prepared buffer and one mask (or none) per output")
    C = _columns(n, N, L)
    need = nimbus_cop_workspace_bytes(m, k, x_bits)
    for i in range(count):
        _words(outs[i], "out", m * C)
        if masks is not None and masks[i] is not None:
            _words(masks[i], "mask", m * C)
        if staged[i].numel() * staged[i].element_size() < need:
            raise ValueError("staged shares buffer is smaller than nimbus_cop_workspace_bytes")
    ptrs = ctypes.c_void_p * count
    a_staged = ptrs(*[_dev_ptr(t, "staged") for t in staged])
    a_prep = ptrs(*[_dev_ptr(t, "prepared") for t in prepared])
    a_out = ptrs(*[_dev_ptr(t, "out") for t in outs])
    a_mask = None if masks is None else ptrs(*[_dev_ptr(t, "mask", True) for t in masks])
    rc = lib.nimbus_cop_matmul_staged_batch(count, a_staged, m, k, x_bits, a_prep, n, N, L,
                                            _moduli(moduli), a_mask, a_out, _stream(stream))
    if rc != 0:
        raise NimbusCopError(rc, "nimbus_cop_matmul_staged_batch")


def nimbus_cop_matmul_prepared(X, m, k, x_bits, prepared, n, N, L, moduli, mask, out,
                               workspace, stream=None):
    lib = load_library()
    C = _columns(n, N, L)
    _words(X, "X", m * k)
    _words(out, "out", m * C)
    if mask is not None:
        _words(mask, "mask", m * C)
    ws_bytes = workspace.numel() * workspace.element_size()
    rc = lib.nimbus_cop_matmul_prepared(
        _dev_ptr(X, "X"), m, k, x_bits, _dev_ptr(prepared, "prepared"), n, N, L,
        _moduli(moduli), _dev_ptr(mask, "mask", True), _dev_ptr(out, "out"),
        _dev_ptr(workspace, "workspace"), ws_bytes, _stream(stream))
    if rc != 0:
        raise NimbusCopError(rc, "nimbus_cop_matmul_prepared")


def nimbus_cop_matmul_prepared_static(X, m, k, x_bits, prepared, n, N, L, moduli, mask, out,
                                      stream=None):
    """nimbus_cop_matmul_prepared on the library's built-in share workspace (no allocation)"""
    lib = load_library()
    C = _columns(n, N, L)
    _words(X, "X", m * k)
    _words(out, "out", m * C)
    if mask is not None:
        _words(mask, "mask", m * C)
    rc = lib.nimbus_cop_matmul_prepared_static(
        _dev_ptr(X, "X"), m, k, x_bits, _dev_ptr(prepared, "prepared"), n, N, L,
        _moduli(moduli), _dev_ptr(mask, "mask", True), _dev_ptr(out, "out"), _stream(stream))
    if rc != 0:
        raise NimbusCopError(rc, "nimbus_cop_matmul_prepared_static")


def nimbus_cop_packed_count(m, n, N) -> int:
    return int(load_library().nimbus_cop_packed_count(m, n, N))


def nimbus_cop_pack(rows, m, n, N, L, moduli, mask, packed, stream=None):
    lib = load_library()
    T = nimbus_cop_packed_count(m, n, N)
    _words(rows, "rows", m * 2 * L * N)
    if T > 0:
        _words(packed, "packed", T * 2 * L * N)
        if mask is not None:
            _words(mask, "mask", T * 2 * L * N)
    rc = lib.nimbus_cop_pack(_dev_ptr(rows, "rows"), m, n, N, L, _moduli(moduli),
                             _dev_ptr(mask, "mask", True), _dev_ptr(packed, "packed"),
                             _stream(stream))
    if rc != 0:
        raise NimbusCopError(rc, "nimbus_cop_pack")


def nimbus_cop_check_inputs(X, m, k, x_bits, ctW, n, N, L, moduli, mask, violations, stream=None):
    """violations: device tensor of 3 64-bit words (shares, ciphertext residues, mask residues)"""
    lib = load_library()
    C = _columns(n, N, L)
    _words(X, "X", m * k)
    _words(ctW, "ctW", k * C)
    if mask is not None:
        _words(mask, "mask", m * C)
    _words(violations, "violations", 3)
    rc = lib.nimbus_cop_check_inputs(_dev_ptr(X, "X"), m, k, x_bits, _dev_ptr(ctW, "ctW"), n, N, L,
                                     _moduli(moduli), _dev_ptr(mask, "mask", True),
                                     _dev_ptr(violations, "violations"), _stream(stream))
    if rc != 0:
        raise NimbusCopError(rc, "nimbus_cop_check_inputs")


def nimbus_calib_mfma_i8(workgroups, iters, random_operands, sink, stream=None) -> int:
    """enqueue the register-only int8 matrix-core loop; returns the int8 operations enqueued"""
    ops = load_library().nimbus_calib_mfma_i8(workgroups, iters, int(bool(random_operands)),
                                              _dev_ptr(sink, "sink"),
                                              sink.numel() * sink.element_size(), _stream(stream))
    if ops < 0:
        raise NimbusCopError(NIMBUS_INVALID, "nimbus_calib_mfma_i8")
    return int(ops)


def nimbus_calib_butterflies(workgroups, iters, q, sink, stream=None) -> int:
    """enqueue the register-only transform-butterfly loop; returns the butterflies enqueued"""
    n = load_library().nimbus_calib_butterflies(workgroups, iters, int(q), _dev_ptr(sink, "sink"),
                                                sink.numel() * sink.element_size(), _stream(stream))
    if n < 0:
        raise NimbusCopError(NIMBUS_INVALID, "nimbus_calib_butterflies")
    return int(n)


def nimbus_calib_stream_read(src, sink, stream=None) -> int:
    """enqueue a streaming read of the whole tensor `src`; returns the bytes read"""
    n = load_library().nimbus_calib_stream_read(_dev_ptr(src, "src"),
                                                src.numel() * src.element_size(),
                                                _dev_ptr(sink, "sink"), _stream(stream))
    if n < 0:
        raise NimbusCopError(NIMBUS_INVALID, "nimbus_calib_stream_read")
    return int(n)


# ---------------------------------------------------------------------------
# server side: key tables, encryption of the weight rows, decryption
# ---------------------------------------------------------------------------
def _bytes_of(t, name, count):
    if t.element_size() != 1:
        raise ValueError(f"{name} must hold bytes")
    if t.numel() != count:
        raise ValueError(f"{name} has {t.numel()} bytes, expected {count}")


def nimbus_rlwe_tables_bytes(N, L) -> int:
    return int(load_library().nimbus_rlwe_tables_bytes(N, L))


def nimbus_rlwe_setup(N, L, moduli, s, tables, stream=None):
    lib = load_library()
    _bytes_of(s, "s", N)
    rc = lib.nimbus_rlwe_setup(N, L, _moduli(moduli), _dev_ptr(s, "s"), _dev_ptr(tables, "tables"),
                               tables.numel() * tables.element_size(), _stream(stream))
    if rc != 0:
        raise NimbusCopError(rc, "nimbus_rlwe_setup")


def nimbus_rlwe_phase(ct, T, N, L, moduli, tables, phi, stream=None):
    lib = load_library()
    _words(ct, "ct", T * 2 * L * N)
    _words(phi, "phi", T * L * N)
    rc = lib.nimbus_rlwe_phase(_dev_ptr(ct, "ct"), T, N, L, _moduli(moduli),
                               _dev_ptr(tables, "tables"), _dev_ptr(phi, "phi"), _stream(stream))
    if rc != 0:
        raise NimbusCopError(rc, "nimbus_rlwe_phase")


def nimbus_rlwe_decode(phi, T, N, L, moduli, t_bits, m_hat, stream=None):
    lib = load_library()
    _words(phi, "phi", T * L * N)
    _words(m_hat, "m_hat", T * N)
    rc = lib.nimbus_rlwe_decode(_dev_ptr(phi, "phi"), T, N, L, _moduli(moduli), t_bits,
                                _dev_ptr(m_hat, "m_hat"), _stream(stream))
    if rc != 0:
        raise NimbusCopError(rc, "nimbus_rlwe_decode")


def nimbus_rlwe_decrypt(ct, T, N, L, moduli, t_bits, tables, phi, m_hat, stream=None):
    lib = load_library()
    _words(ct, "ct", T * 2 * L * N)
    _words(phi, "phi", T * L * N)
    _words(m_hat, "m_hat", T * N)
    rc = lib.nimbus_rlwe_decrypt(_dev_ptr(ct, "ct"), T, N, L, _moduli(moduli), t_bits,
                                 _dev_ptr(tables, "tables"), _dev_ptr(phi, "phi"),
                                 _dev_ptr(m_hat, "m_hat"), _stream(stream))
    if rc != 0:
        raise NimbusCopError(rc, "nimbus_rlwe_decrypt")


def nimbus_rlwe_encrypt(W, k, n, t_bits, N, L, moduli, tables, a, e, ctW, stream=None):
    lib = load_library()
    Ch = -(-n // N)
    _words(W, "W", k * n)
    _words(a, "a", k * Ch * L * N)
    _bytes_of(e, "e", k * Ch * N)
    _words(ctW, "ctW", k * Ch * 2 * L * N)
    rc = lib.nimbus_rlwe_encrypt(_dev_ptr(W, "W"), k, n, t_bits, N, L, _moduli(moduli),
                                 _dev_ptr(tables, "tables"), _dev_ptr(a, "a"), _dev_ptr(e, "e"),
                                 _dev_ptr(ctW, "ctW"), _stream(stream))
    if rc != 0:
        raise NimbusCopError(rc, "nimbus_rlwe_encrypt")


# ---------------------------------------------------------------------------
# asynchronous weight loading (pinned host memory -> device slot on a copy stream)
# ---------------------------------------------------------------------------
def nimbus_loader_create(slots: int):
    """returns the opaque loader handle"""
    handle = ctypes.c_void_p()
    rc = load_library().nimbus_loader_create(slots, ctypes.byref(handle))
    if rc != 0:
        raise NimbusCopError(rc, "nimbus_loader_create")
    return handle


def nimbus_loader_destroy(loader):
    rc = load_library().nimbus_loader_destroy(loader)
    if rc != 0:
        raise NimbusCopError(rc, "nimbus_loader_destroy")


def nimbus_loader_load(loader, slot, dst, src_host, copy_stream):
    """dst: device tensor; src_host: pinned host tensor of the same byte size"""
    if src_host.is_cuda or not src_host.is_pinned():
        raise ValueError("src_host must be a pinned host tensor")
    nbytes = src_host.numel() * src_host.element_size()
    if dst.numel() * dst.element_size() < nbytes:
        raise ValueError("dst is smaller than src_host")
    if not src_host.is_contiguous():
        raise ValueError("src_host must be contiguous")
    rc = load_library().nimbus_loader_load(loader, slot, _dev_ptr(dst, "dst"),
                                           ctypes.c_void_p(src_host.data_ptr()), nbytes,
                                           _stream(copy_stream))
    if rc != 0:
        raise NimbusCopError(rc, "nimbus_loader_load")


def nimbus_loader_acquire(loader, slot, compute_stream=None):
    rc = load_library().nimbus_loader_acquire(loader, slot, _stream(compute_stream))
    if rc != 0:
        raise NimbusCopError(rc, "nimbus_loader_acquire")


def nimbus_loader_release(loader, slot, compute_stream=None):
    rc = load_library().nimbus_loader_release(loader, slot, _stream(compute_stream))
    if rc != 0:
        raise NimbusCopError(rc, "nimbus_loader_release")
