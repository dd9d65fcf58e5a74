"""The entry point that allocates nothing, nimbus_cop_matmul_prepared_static, against
nimbus_cop_matmul_prepared (and the oracle): two calls in a row on the library's built-in
share workspace, the second with a smaller input, every output word equal."""
import sys

import numpy as np
import pytest

import cop_inputs as ci

pytestmark = pytest.mark.gpu


def _say(msg):
    print(msg, flush=True)
    sys.stdout.flush()


# m, k, n, N, L, t_bits, q_bits: a large call, then smaller ones that reuse the same buffer
CALLS = [
    (130, 300, 128, 128, 2, 20, 54),    # two row blocks (one ragged), ten k-blocks with a tail
    (33, 100, 64, 64, 2, 20, 54),       # smaller in both dimensions: stale planes lie behind it
    (20, 70, 64, 64, 1, 40, 54),        # shares of 40 bits: both halves' planes in the buffer
]


def test_static_workspace_entry_point_matches_the_allocating_one(oracle):
    import torch
    import gpu_util as gu
    import paper_2411_15707_amd as nc
    for call, (m, k, n, N, L, t_bits, q_bits) in enumerate(CALLS):
        moduli = ci.limb_primes(q_bits, min(t_bits, 32), L)
        seed = 9000 + call
        Ch = -(-n // N)
        X = ci.gen_X(seed, m, k, t_bits)
        ctW = ci.gen_ctW_uniform(seed, k, Ch, moduli, N)
        mask = ci.gen_mask_uniform(seed, m, Ch, moduli, N)
        _say(f"[no-alloc] call {call}: m={m} k={k} n={n} N={N} L={L} x_bits={t_bits}")
        prepared = gu.prepare(ctW, moduli, n, N)
        dX, dM = gu.dev(X), gu.dev(mask)
        ws = torch.empty(nc.nimbus_cop_workspace_bytes(m, k, t_bits), dtype=torch.uint8, device="cuda")
        ref = torch.full((m, Ch, 2, L, N), -1, dtype=torch.int64, device="cuda")
        got = torch.full((m, Ch, 2, L, N), -2, dtype=torch.int64, device="cuda")
        nc.nimbus_cop_matmul_prepared(dX, m, k, t_bits, prepared, n, N, L, moduli, dM, ref, ws)
        torch.cuda.synchronize()
        before = torch.cuda.memory_allocated()
        nc.nimbus_cop_matmul_prepared_static(dX, m, k, t_bits, prepared, n, N, L, moduli, dM, got)
        torch.cuda.synchronize()
        assert torch.cuda.memory_allocated() == before
        g, r = gu.host(got), gu.host(ref)
        assert np.array_equal(g, r), f"call {call}: " + gu.first_mismatch(g, r)
        want, _ = oracle.cop_ref(X, ctW, moduli, n, N, mask, wide=t_bits > 32)
        assert np.array_equal(g, want), f"call {call} vs oracle: " + gu.first_mismatch(g, want)


def test_static_workspace_limit_is_an_error():
    import torch
    import paper_2411_15707_amd as nc
    moduli = ci.limb_primes(54, 20, 1)
    # 8193 row tiles x 1 k-block x 3 planes of 1 KiB: one tile more than the 8 MiB built in
    m, k = 32 * 2731 + 1, 32
    assert nc.nimbus_cop_workspace_bytes(m, k, 20) > (8 << 20)
    X = torch.zeros((m, k), dtype=torch.int64, device="cuda")
    prepared = torch.zeros(nc.nimbus_cop_prepared_bytes(k, 32, 32, 1, moduli), dtype=torch.uint8,
                           device="cuda")
    out = torch.full((m, 1, 2, 1, 32), 7, dtype=torch.int64, device="cuda")
    with pytest.raises(nc.NimbusCopError) as ei:
        nc.nimbus_cop_matmul_prepared_static(X, m, k, 20, prepared, 32, 32, 1, moduli, None, out)
    assert ei.value.status == -5
    torch.cuda.synchronize()
    assert (out == 7).all()
