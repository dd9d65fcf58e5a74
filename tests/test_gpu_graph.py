"""The entry points allocate nothing and never wait for the GPU, so a caller can record them into
a HIP graph.  A graph holding the whole layer (client step, packing, server decryption) is
replayed several times with new shares written into the same buffers between the replays;
every replay must equal the oracle (and so the eager calls)."""
import sys

import numpy as np
import pytest

import cop_inputs as ci

pytestmark = pytest.mark.gpu


def _say(msg):
    print(msg, flush=True)
    sys.stdout.flush()


# m, k, n, N, L, t_bits, q_bits
@pytest.mark.parametrize("m,k,n,N,L,t_bits,q_bits,static", [
    (33, 100, 40, 128, 2, 20, 54, False),     # ragged rows and k, three rows per packed ciphertext
    (8, 64, 64, 1024, 1, 16, 50, False),      # config 1
    (128, 256, 3072, 4096, 2, 20, 54, False), # BERT-base FFN width, shortened inner dimension
    # the entry point for callers that cannot allocate: share planes in the library's own buffer
    (40, 96, 64, 128, 2, 20, 54, True),
])
def test_layer_recorded_in_a_graph_replays_exactly(oracle, m, k, n, N, L, t_bits, q_bits, static):
    import torch
    import gpu_util as gu
    import paper_2411_15707_amd as nc
    moduli = ci.limb_primes(q_bits, max(t_bits, N.bit_length()), L)
    seed = 31337 + m
    C = 2 * L * N
    ctW = ci.gen_ctW_uniform(seed, k, 1, moduli, N)
    mask = ci.gen_mask_uniform(seed, m, 1, moduli, N)
    s = ci.gen_secret(seed, N)
    T = nc.nimbus_cop_packed_count(m, n, N)
    pmask = ci.gen_mask_uniform(seed + 1, T, 1, moduli, N)[:, 0]
    prepared = gu.prepare(ctW, moduli, n, N)
    tables = torch.empty(nc.nimbus_rlwe_tables_bytes(N, L), dtype=torch.uint8, device="cuda")
    nc.nimbus_rlwe_setup(N, L, moduli, torch.from_numpy(s).cuda(), tables)
    dX = torch.zeros((m, k), dtype=torch.int64, device="cuda")
    dmask, dpmask = gu.dev(mask), gu.dev(pmask)
    ws = torch.empty(nc.nimbus_cop_workspace_bytes(m, k, t_bits), dtype=torch.uint8, device="cuda")
    out = torch.zeros((m, C), dtype=torch.int64, device="cuda")
    packed = torch.zeros((T, 2, L, N), dtype=torch.int64, device="cuda")
    phi = torch.zeros((T, L, N), dtype=torch.int64, device="cuda")
    m_hat = torch.zeros((T, N), dtype=torch.int64, device="cuda")
    with_decrypt = L <= 2

    def layer():
        if static:
            nc.nimbus_cop_matmul_prepared_static(dX, m, k, t_bits, prepared, n, N, L, moduli, dmask, out)
        else:
            nc.nimbus_cop_matmul_prepared(dX, m, k, t_bits, prepared, n, N, L, moduli, dmask, out, ws)
        nc.nimbus_cop_pack(out, m, n, N, L, moduli, dpmask, packed)
        if with_decrypt:
            nc.nimbus_rlwe_decrypt(packed, T, N, L, moduli, t_bits, tables, phi, m_hat)

    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        layer()                                    # warm-up on the capture stream
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        layer()
    torch.cuda.synchronize()
    for rep in range(4):
        X = ci.gen_X(seed + 100 * rep, m, k, t_bits)
        _say(f"[graph] m={m} k={k} N={N}: replay {rep}")
        # the program's own eager work between the replays: new inputs, cleared outputs
        dX.copy_(gu.dev(X))
        out.zero_(); packed.zero_(); m_hat.zero_()
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        want_rows = oracle.cop_ref(X, ctW, moduli, n, N, mask)[0]
        assert np.array_equal(gu.host(out).reshape(want_rows.shape), want_rows), f"replay {rep}: rows"
        want_packed = oracle.pack_ref(want_rows[:, 0], n, moduli, pmask)
        assert np.array_equal(gu.host(packed), want_packed), f"replay {rep}: packed"
        if with_decrypt:
            got = gu.host(m_hat)
            for th in sorted({0, T // 2, T - 1}):
                assert np.array_equal(got[th], oracle.decrypt(want_packed[th], s, moduli, t_bits)), \
                    f"replay {rep}: decryption of {th}"
