"""Asynchronous weight loading on the GPU: a stack of layers whose prepared weights live in
pinned host memory is streamed through two device slots while the previous layer computes;
every layer's output must equal the oracle's, whichever of copy and kernel is the slower."""
import sys

import numpy as np
import pytest

import cop_inputs as ci

pytestmark = pytest.mark.gpu


def _say(msg):
    print(msg, flush=True)
    sys.stdout.flush()


# layers, m, k, n, N, L, t_bits, q_bits
STACKS = [
    (6, 16, 96, 64, 64, 2, 20, 54),          # tiny: launch-bound on both streams
    (8, 512, 2048, 64, 64, 1, 16, 50),       # kernel (64 k-blocks, 8 workgroups) slower than its 1.8 MB copy
    (4, 64, 256, 3072, 4096, 2, 20, 54),     # 29 MB per layer: the copy is far slower than the kernel
]


@pytest.mark.parametrize("layers,m,k,n,N,L,t_bits,q_bits", STACKS)
def test_layer_stack_streamed_through_two_slots(oracle, layers, m, k, n, N, L, t_bits, q_bits):
    import torch
    import gpu_util as gu
    import paper_2411_15707_amd as nc
    moduli = ci.limb_primes(q_bits, t_bits, L)
    Ch = -(-n // N)
    C = Ch * 2 * L * N
    pbytes = nc.nimbus_cop_prepared_bytes(k, n, N, L, moduli)
    _say(f"[loader] {layers} layers m={m} k={k} n={n} N={N} L={L}: {pbytes} bytes per layer")
    host_w, Xs, masks, wants = [], [], [], []
    tmp = torch.empty(pbytes, dtype=torch.uint8, device="cuda")
    for i in range(layers):
        seed = 4242 + 17 * i
        X = ci.gen_X(seed, m, k, t_bits)
        ctW = ci.gen_ctW_uniform(seed, k, Ch, moduli, N)
        mask = ci.gen_mask_uniform(seed, m, Ch, moduli, N)
        nc.nimbus_cop_prepare(gu.dev(ctW), k, n, N, L, moduli, tmp)       # setup phase
        torch.cuda.synchronize()
        hw = torch.empty(pbytes, dtype=torch.uint8, pin_memory=True)       # "disk": pinned host memory
        hw.copy_(tmp)
        host_w.append(hw)
        Xs.append(gu.dev(X))
        masks.append(gu.dev(mask))
        wants.append(oracle.cop_ref(X, ctW, moduli, n, N, mask)[0])
    del tmp
    slots = [torch.zeros(pbytes, dtype=torch.uint8, device="cuda") for _ in range(2)]
    outs = [torch.empty((m, C), dtype=torch.int64, device="cuda") for _ in range(layers)]
    ws = torch.empty(nc.nimbus_cop_workspace_bytes(m, k, t_bits), dtype=torch.uint8, device="cuda")
    copy_stream = torch.cuda.Stream()
    compute = torch.cuda.current_stream()
    torch.cuda.synchronize()
    ld = nc.nimbus_loader_create(2)
    try:
        for rep in range(2):                       # the second pass reuses slots that were released
            nc.nimbus_loader_load(ld, 0, slots[0], host_w[0], copy_stream)
            for i in range(layers):
                if i + 1 < layers:
                    nc.nimbus_loader_load(ld, (i + 1) % 2, slots[(i + 1) % 2], host_w[i + 1], copy_stream)
                nc.nimbus_loader_acquire(ld, i % 2, compute)
                nc.nimbus_cop_matmul_prepared(Xs[i], m, k, t_bits, slots[i % 2], n, N, L, moduli,
                                              masks[i], outs[i], ws)
                nc.nimbus_loader_release(ld, i % 2, compute)
            torch.cuda.synchronize()
            for i in range(layers):
                got = gu.host(outs[i]).reshape(wants[i].shape)
                assert np.array_equal(got, wants[i]), f"pass {rep} layer {i}: " + gu.first_mismatch(got, wants[i])
                outs[i].zero_()
            torch.cuda.synchronize()
    finally:
        nc.nimbus_loader_destroy(ld)


def test_loader_slot_checks_on_a_live_handle():
    import torch
    import paper_2411_15707_amd as nc
    lib = nc.load_library()
    ld = nc.nimbus_loader_create(2)
    try:
        assert lib.nimbus_loader_acquire(ld, 2, None) == -1
        assert lib.nimbus_loader_release(ld, -1, None) == -1
        assert lib.nimbus_loader_load(ld, 0, None, 0x1000, 16, None) == -1
        assert lib.nimbus_loader_load(ld, 0, 0x1000, 0x2000, 0, None) == -1
        # acquiring a slot that was never loaded waits for nothing
        nc.nimbus_loader_acquire(ld, 1)
        nc.nimbus_loader_release(ld, 1)
        torch.cuda.synchronize()
    finally:
        nc.nimbus_loader_destroy(ld)
