"""Helpers for the GPU parity tests: upload, call the C ABI through the binding, download."""
import numpy as np
import torch

import paper_2411_15707_amd as nc


def dev(a: np.ndarray) -> torch.Tensor:
    """uint64 numpy -> int64 cuda tensor holding the same 64-bit words"""
    return torch.from_numpy(np.ascontiguousarray(a).view(np.int64)).cuda()


def host(t: torch.Tensor) -> np.ndarray:
    return t.cpu().numpy().view(np.uint64)


def _run_canonical(entry, X, ctW, moduli, n, N, x_bits, mask=None):
    m, k = X.shape
    L = len(moduli)
    Ch = -(-n // N)
    dX, dW = dev(X), dev(ctW)
    dM = dev(mask) if mask is not None else None
    out = torch.full((m, Ch, 2, L, N), -1, dtype=torch.int64, device="cuda")
    entry(dX, m, k, x_bits, dW, n, N, L, moduli, dM, out)
    torch.cuda.synchronize()
    return host(out)


def run_valu(X, ctW, moduli, n, N, x_bits, mask=None):
    """the vector-ALU kernel on the canonical layout"""
    return _run_canonical(nc.nimbus_cop_matmul_valu, X, ctW, moduli, n, N, x_bits, mask)


def run_canon(X, ctW, moduli, n, N, x_bits, mask=None):
    """nimbus_cop_matmul: the matrix-core kernel on the canonical layout where its limits
    allow, the vector-ALU kernel otherwise"""
    return _run_canonical(nc.nimbus_cop_matmul, X, ctW, moduli, n, N, x_bits, mask)


def prepare(ctW, moduli, n, N):
    k = ctW.shape[0]
    L = len(moduli)
    nbytes = nc.nimbus_cop_prepared_bytes(k, n, N, L, moduli)
    assert nbytes > 0
    prepared = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
    nc.nimbus_cop_prepare(dev(ctW), k, n, N, L, moduli, prepared)
    torch.cuda.synchronize()
    return prepared


def run_mfma(X, ctW, moduli, n, N, x_bits, mask=None, prepared=None):
    m, k = X.shape
    L = len(moduli)
    Ch = -(-n // N)
    if prepared is None:
        prepared = prepare(ctW, moduli, n, N)
    ws = torch.empty(nc.nimbus_cop_workspace_bytes(m, k, x_bits), dtype=torch.uint8, device="cuda")
    dX = dev(X)
    dM = dev(mask) if mask is not None else None
    out = torch.full((m, Ch, 2, L, N), -1, dtype=torch.int64, device="cuda")
    nc.nimbus_cop_matmul_prepared(dX, m, k, x_bits, prepared, n, N, L, moduli, dM, out, ws)
    torch.cuda.synchronize()
    return host(out)


def first_mismatch(got, want):
    bad = np.argwhere(got != want)
    if len(bad) == 0:
        return None
    idx = tuple(bad[0])
    return f"{len(bad)} mismatches, first at {idx}: got {got[idx]} want {want[idx]}"
