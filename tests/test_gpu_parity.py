"""GPU parity: both C-ABI entry points against the CPU oracle, bit for bit.

Integer work, so the bar is exact equality of every output word.
"""
import sys

import numpy as np
import pytest

import cop_inputs as ci

pytestmark = pytest.mark.gpu


def _say(msg):
    print(msg, flush=True)
    sys.stdout.flush()


def _inputs(seed, m, k, n, N, moduli, t_bits, with_mask=True):
    Ch = -(-n // N)
    X = ci.gen_X(seed, m, k, t_bits)
    ctW = ci.gen_ctW_uniform(seed, k, Ch, moduli, N)
    mask = ci.gen_mask_uniform(seed, m, Ch, moduli, N) if with_mask else None
    return X, ctW, mask


def _check_both(oracle, X, ctW, moduli, n, N, x_bits, mask, label):
    import gpu_util as gu
    want, _ = oracle.cop_ref(X, ctW, moduli, n, N, mask)
    _say(f"[parity] {label}: valu kernel")
    got = gu.run_valu(X, ctW, moduli, n, N, x_bits, mask)
    assert got.shape == want.shape
    assert np.array_equal(got, want), "valu: " + gu.first_mismatch(got, want)
    _say(f"[parity] {label}: matrix-core kernel")
    got = gu.run_mfma(X, ctW, moduli, n, N, x_bits, mask)
    assert np.array_equal(got, want), "mfma: " + gu.first_mismatch(got, want)
    _say(f"[parity] {label}: canonical-layout entry point")
    got = gu.run_canon(X, ctW, moduli, n, N, x_bits, mask)
    assert np.array_equal(got, want), "canonical: " + gu.first_mismatch(got, want)
    return want


# m, k, n, N, L, t_bits, q_bits
SMALL = [
    (8, 64, 64, 1024, 1, 16, 50),       # config 1 shape
    (5, 7, 32, 32, 1, 16, 50),          # k and m far below one tile
    (33, 100, 40, 64, 2, 20, 54),       # ragged m and k (33 rows, 100 = 3*32 + 4)
    (130, 131, 64, 64, 2, 20, 54),      # two row blocks, ragged k, several k stages + tail
    (64, 300, 2500, 1024, 1, 20, 54),   # n > N: three ring chunks, last partial
    (40, 96, 128, 128, 3, 24, 55),      # three limbs, 24-bit shares
    (17, 70, 64, 64, 1, 32, 62),        # widest shares and modulus: 4 x 8 byte planes
    (17, 70, 64, 64, 1, 32, 54),        # 32-bit shares: 4 x 7 byte planes
    (19, 65, 64, 64, 2, 24, 62),        # 62-bit moduli: 3 x 8 byte planes
    (20, 257, 64, 64, 2, 9, 40),        # small modulus, odd share width
    (1, 1, 32, 32, 1, 16, 50),          # k = 1, m = 1
    (16, 160, 64, 64, 1, 12, 50),       # 12-bit shares: the upper share plane holds unshifted digits
    (7, 33, 64, 64, 1, 7, 30),          # 7-bit shares (no shifted plane at all), 30-bit modulus
    (9, 128, 64, 64, 2, 20, 62),        # 3 x 8 planes (operands read after the barrier), four k-blocks
    (12, 192, 64, 64, 1, 32, 62),       # 4 x 8 planes, six k-blocks
    (100, 1024, 64, 64, 1, 16, 50),     # 2 x 7 planes, 32 k-blocks
    (6, 50, 32, 32, 3, 20, 54),         # smallest ring with several limbs: a 64-column tile spans two limbs
    # m a multiple of 128: the builds of the kernel without row tests, one per plane count
    (128, 64, 64, 64, 1, 16, 50),       # 2 x 7
    (128, 96, 64, 64, 2, 20, 54),       # 3 x 7, two limbs
    (128, 70, 64, 64, 1, 32, 54),       # 4 x 7
    (128, 64, 64, 64, 1, 16, 62),       # 2 x 8
    (128, 65, 64, 64, 2, 24, 62),       # 3 x 8
    (128, 64, 32, 32, 1, 32, 62),       # 4 x 8, smallest ring
    (256, 100, 64, 64, 2, 20, 54),      # two full row blocks
    # the mask tile through LDS (m a multiple of 128, at least 13 k-blocks) for the plane counts
    # the BERT-shaped configs do not reach, alone and with several row blocks per column tile
    (128, 512, 64, 64, 1, 16, 50),      # 2 x 7
    (128, 448, 64, 64, 1, 16, 62),      # 2 x 8
    (256, 480, 64, 64, 1, 16, 50),      # 2 x 7, two row blocks
    (256, 417, 64, 64, 1, 16, 62),      # 2 x 8, two row blocks, ragged k
    (384, 512, 128, 128, 2, 20, 54),    # 3 x 7, three row blocks
    # row blocks dealt to the XCDs: 8 and 12 column-tile pairs (a whole round, a round and a tail)
    (256, 100, 256, 256, 1, 20, 54),
    (384, 70, 128, 128, 3, 20, 54),
    (200, 500, 256, 256, 1, 16, 50),    # ragged m with two row blocks, 16 k-blocks
    # more output tiles than compute units: a workgroup walks several tiles, the first stages of
    # the next one in flight under the epilogue of the one before
    (128, 512, 8192, 8192, 3, 20, 54),  # 768 tiles, mask tile through LDS
    (70, 100, 8192, 8192, 3, 20, 54),   # 768 tiles, a wave without rows in every tile
    (200, 70, 4096, 4096, 2, 20, 54),   # 512 tiles in two row blocks, the second ragged
    (128, 96, 16384, 16384, 1, 32, 62), # 512 tiles, 4 x 8 planes (operands read after the barrier)
    # the ends of the accepted ranges
    (6, 50, 64, 64, 4, 20, 54),         # four limbs
    (3, 33, 32768, 32768, 2, 20, 54),   # the paper's largest ring degree
    (4, 40, 65536, 65536, 1, 20, 54),   # the largest ring degree the client side accepts
    (2, 34, 70000, 65536, 1, 16, 50),   # two chunks of the largest ring, the second nearly empty
]


@pytest.mark.parametrize("m,k,n,N,L,t_bits,q_bits", SMALL)
def test_small_and_ragged_shapes(oracle, m, k, n, N, L, t_bits, q_bits):
    moduli = ci.limb_primes(q_bits, t_bits, L)
    X, ctW, mask = _inputs(1000 + m + k, m, k, n, N, moduli, t_bits)
    # extremes: largest share, largest residues in a few places
    X[0, 0] = (1 << t_bits) - 1
    X[-1, -1] = (1 << t_bits) - 1
    for l, q in enumerate(moduli):
        ctW[:, 0, :, l, :4] = q - 1
        mask[0, 0, :, l, :4] = q - 1
    _check_both(oracle, X, ctW, moduli, n, N, t_bits, mask, f"small m={m} k={k} n={n} N={N} L={L}")
    _check_both(oracle, X, ctW, moduli, n, N, t_bits, None, f"small/no-mask m={m} k={k}")


@pytest.mark.parametrize("k", [20, 40, 80])
@pytest.mark.parametrize("t_bits,q_bits", [(16, 50), (20, 54), (32, 54), (16, 62), (24, 62), (32, 62)])
def test_one_to_three_k_blocks_per_plane_count(oracle, t_bits, q_bits, k):
    """every plane count with one, two and three k-blocks: the loop's prologue is all there is,
    its first wait covers the load of the column sums, and with shares of t-1 the term
    OFFX * S that needs them is as large as it gets"""
    m, n, N, L = 8, 32, 32, 1
    moduli = ci.limb_primes(q_bits, t_bits, L)
    X, ctW, mask = _inputs(2000 + k + t_bits + q_bits, m, k, n, N, moduli, t_bits)
    X[0, :] = (1 << t_bits) - 1
    X[1, :] = 0
    _check_both(oracle, X, ctW, moduli, n, N, t_bits, mask, f"k={k} t={t_bits} q={q_bits}")


def test_all_maximal_operands(oracle):
    """every share t-1 and every residue q-1: the largest sums the accumulators can see"""
    m, k, n, N, L, t_bits = 32, 512, 64, 64, 2, 24
    moduli = ci.limb_primes(55, t_bits, L)
    qv = np.array(moduli, dtype=np.uint64).reshape(1, 1, 1, L, 1)
    X = np.full((m, k), (1 << t_bits) - 1, dtype=np.uint64)
    ctW = np.broadcast_to(qv - np.uint64(1), (k, 1, 2, L, N)).copy()
    mask = np.broadcast_to(qv - np.uint64(1), (m, 1, 2, L, N)).copy()
    _check_both(oracle, X, ctW, moduli, n, N, t_bits, mask, "maximal")
    # residues just above and below q/2 exercise both branches of the centring
    half = (qv - np.uint64(1)) // np.uint64(2)
    ctW[::2] = half
    ctW[1::2] = half + np.uint64(1)
    _check_both(oracle, X, ctW, moduli, n, N, t_bits, mask, "half-modulus")
    X[:] = 0
    _check_both(oracle, X, ctW, moduli, n, N, t_bits, mask, "zero shares")


@pytest.mark.parametrize("q_bits,t_bits", [(54, 24), (62, 16), (50, 20)])
def test_all_maximal_operands_uncentred_digits(oracle, q_bits, t_bits):
    """the same extremes for moduli whose residues the canonical-layout kernel splits into
    digits without centring them first: sums twice as large as with centred digits"""
    m, k, n, N, L = 32, 512, 64, 64, 2
    moduli = ci.limb_primes(q_bits, t_bits, L)
    qv = np.array(moduli, dtype=np.uint64).reshape(1, 1, 1, L, 1)
    X = np.full((m, k), (1 << t_bits) - 1, dtype=np.uint64)
    ctW = np.broadcast_to(qv - np.uint64(1), (k, 1, 2, L, N)).copy()
    mask = np.broadcast_to(qv - np.uint64(1), (m, 1, 2, L, N)).copy()
    _check_both(oracle, X, ctW, moduli, n, N, t_bits, mask, f"maximal {q_bits}")
    X[::2] = 0
    ctW[1::2] = 0
    _check_both(oracle, X, ctW, moduli, n, N, t_bits, None, f"maximal and zero {q_bits}")


@pytest.mark.parametrize("q", [0x7F7F7F7F7F7F7F, 0x7F7F7F7F7F7F81, 0x7F7F7F7F7F7F7D])
def test_moduli_at_the_edge_of_seven_signed_digits(oracle, q):
    """Seven signed base-256 digits express the values up to 0x7F7F7F7F7F7F7F.  A modulus whose
    residues stay below that is split into digits as it is, one above is centred first; the
    residues next to the edge are the ones whose top digit is 127 after the carries.  (The
    client side only needs odd moduli above 2^x_bits.)"""
    m, k, n, N, L, t_bits = 16, 96, 32, 32, 1, 20
    moduli = (q,)
    X, ctW, mask = _inputs(4242, m, k, n, N, moduli, t_bits)
    edge = np.array([q - 1, q - 2, 0x7F7F7F7F7F7F7E, 0x7F7F7F7F7F7F00, 0x7F7F7F7F7F0080, 0x7F80, 0x80, 0x7F, 0],
                    dtype=np.uint64) % np.uint64(q)
    ctW.reshape(k, -1)[:, :edge.size] = edge
    ctW.reshape(k, -1)[::3, edge.size:2 * edge.size] = edge[::-1]
    X[0, :] = (1 << t_bits) - 1
    _check_both(oracle, X, ctW, moduli, n, N, t_bits, mask, f"edge modulus {q:#x}")


def test_special_cases_on_gpu(oracle):
    import gpu_util as gu
    m = k = 48
    n = N = 64
    L, t_bits = 2, 20
    moduli = ci.limb_primes(54, t_bits, L)
    _, ctW, mask = _inputs(5, m, k, n, N, moduli, t_bits)
    qv = np.array(moduli, dtype=np.uint64).reshape(1, 1, 1, L, 1)
    for run in (gu.run_valu, gu.run_mfma, gu.run_canon):
        out = run(np.zeros((m, k), np.uint64), ctW, moduli, n, N, t_bits, mask)
        assert np.array_equal(out, mask)                         # X = 0: the mask
        out = run(np.eye(m, dtype=np.uint64), ctW, moduli, n, N, t_bits, mask)
        s = ctW + mask
        assert np.array_equal(out, np.where(s >= qv, s - qv, s))   # X = I: vector add mod q
        out = run(np.eye(m, dtype=np.uint64), ctW, moduli, n, N, t_bits, None)
        assert np.array_equal(out, ctW)                          # X = I, no mask: a copy


def test_config1_real_encryption_and_decrypt_invariant(oracle):
    """config 1 in full: weights encrypted for real, GPU output decrypted, Dec(out_j) + R_j
    must equal (X W)_j mod t (Algorithm 1, output condition)"""
    import gpu_util as gu
    cfg = ci.CONFIGS[1]
    seed = ci.config_seed(1)
    t = cfg.t
    X = ci.gen_X(seed, cfg.m, cfg.k, cfg.t_bits)
    W = ci.gen_W(seed, cfg.k, cfg.n, cfg.t_bits)
    s = ci.gen_secret(seed, cfg.N)
    a, e = ci.gen_enc_randomness(seed, cfg.k, 1, cfg.moduli, cfg.N)
    R = ci.gen_R(seed, cfg.m, cfg.N, cfg.t_bits)
    w_hat = oracle.encode_rows(W, cfg.N)
    ct = oracle.encrypt(w_hat[:, 0], s, a[:, 0], e[:, 0], cfg.moduli, cfg.t_bits)
    ctW = ct.reshape(cfg.k, 1, 2, cfg.L, cfg.N)
    mask = np.stack([oracle.share_mask(R[j], cfg.moduli, cfg.t_bits)[None] for j in range(cfg.m)])
    want, _ = oracle.cop_ref(X, ctW, cfg.moduli, cfg.n, cfg.N, mask)
    XW = X.astype(object) @ W.astype(object)
    for run in (gu.run_valu, gu.run_mfma, gu.run_canon):
        out = run(X, ctW, cfg.moduli, cfg.n, cfg.N, cfg.t_bits, mask)
        assert np.array_equal(out, want)
        for j in range(cfg.m):
            dec = oracle.decrypt(out[j, 0], s, cfg.moduli, cfg.t_bits)
            got = (dec + R[j]) % np.uint64(t)
            assert np.array_equal(got[:cfg.n], (XW[j] % t).astype(np.uint64))
            assert (got[cfg.n:] == 0).all()


@pytest.mark.parametrize("cfg_id", [2, 3, 4])
def test_bert_base_configs_full(oracle, cfg_id):
    """configs 2-4 at full size, every output word compared"""
    cfg = ci.CONFIGS[cfg_id]
    seed = ci.config_seed(cfg_id)
    _say(f"[parity] config {cfg_id}: generating inputs")
    X, ctW, mask = _inputs(seed, cfg.m, cfg.k, cfg.n, cfg.N, cfg.moduli, cfg.t_bits)
    _check_both(oracle, X, ctW, cfg.moduli, cfg.n, cfg.N, cfg.t_bits, mask, f"config {cfg_id}")


@pytest.mark.parametrize("cfg_id", [2, 3, 4])
def test_bert_base_real_encryption_spot_check(oracle, cfg_id):
    """configs 2-4 with every weight row encrypted for real; four output rows of the GPU
    result are decrypted and compared with the brute-force X W mod t (Theorem 1's invariant
    restated for the hot path: Dec(out_j) + R_j = (X W)_j mod t, zero beyond column n)"""
    import gpu_util as gu
    cfg = ci.CONFIGS[cfg_id]
    seed = ci.config_seed(cfg_id) + 500
    t = cfg.t
    rows = [0, 1, cfg.m // 2, cfg.m - 1]
    X = ci.gen_X(seed, cfg.m, cfg.k, cfg.t_bits)
    W = ci.gen_W(seed, cfg.k, cfg.n, cfg.t_bits)
    s = ci.gen_secret(seed, cfg.N)
    a, e = ci.gen_enc_randomness(seed, cfg.k, 1, cfg.moduli, cfg.N)
    R = ci.gen_R(seed, cfg.m, cfg.N, cfg.t_bits)
    _say(f"[parity] config {cfg_id} real encryption: encrypting {cfg.k} rows on the CPU")
    ct = oracle.encrypt(oracle.encode_rows(W, cfg.N)[:, 0], s, a[:, 0], e[:, 0], cfg.moduli,
                        cfg.t_bits)
    ctW = ct.reshape(cfg.k, 1, 2, cfg.L, cfg.N)
    mask = ci.gen_mask_uniform(seed, cfg.m, 1, cfg.moduli, cfg.N)
    for j in rows:
        mask[j, 0] = oracle.share_mask(R[j], cfg.moduli, cfg.t_bits)
    _say(f"[parity] config {cfg_id} real encryption: matrix-core kernel")
    out = gu.run_mfma(X, ctW, cfg.moduli, cfg.n, cfg.N, cfg.t_bits, mask)
    XW = X[rows].astype(object) @ W.astype(object)
    for r, j in enumerate(rows):
        dec, noise = oracle.decrypt(out[j, 0], s, cfg.moduli, cfg.t_bits, with_noise=True)
        got = (dec + R[j]) % np.uint64(t)
        assert np.array_equal(got[:cfg.n], (XW[r] % t).astype(np.uint64))
        assert (got[cfg.n:] == 0).all()
        assert np.abs(noise).max() <= cfg.k * t * 20
    # the server side at this config's full size: the GPU encrypts the same rows with the
    # same randomness (all k ciphertexts must equal the oracle's) and decrypts the output
    # rows (the four sampled rows must equal the oracle's decryption)
    import torch
    import paper_2411_15707_amd as nc
    _say(f"[parity] config {cfg_id} real encryption: server side on the GPU")
    tables = torch.empty(nc.nimbus_rlwe_tables_bytes(cfg.N, cfg.L), dtype=torch.uint8, device="cuda")
    nc.nimbus_rlwe_setup(cfg.N, cfg.L, cfg.moduli, torch.from_numpy(s).cuda(), tables)
    ct_gpu = torch.empty((cfg.k, 1, 2, cfg.L, cfg.N), dtype=torch.int64, device="cuda")
    nc.nimbus_rlwe_encrypt(gu.dev(W), cfg.k, cfg.n, cfg.t_bits, cfg.N, cfg.L, cfg.moduli, tables,
                           gu.dev(a), torch.from_numpy(e).cuda(), ct_gpu)
    torch.cuda.synchronize()
    assert np.array_equal(gu.host(ct_gpu), ctW), "GPU encryption differs from the oracle's"
    phi = torch.empty((cfg.m, cfg.L, cfg.N), dtype=torch.int64, device="cuda")
    m_hat = torch.empty((cfg.m, cfg.N), dtype=torch.int64, device="cuda")
    nc.nimbus_rlwe_decrypt(gu.dev(out[:, 0]), cfg.m, cfg.N, cfg.L, cfg.moduli, cfg.t_bits, tables,
                           phi, m_hat)
    torch.cuda.synchronize()
    got_all = gu.host(m_hat)
    for j in rows:
        assert np.array_equal(got_all[j], oracle.decrypt(out[j, 0], s, cfg.moduli, cfg.t_bits))


def test_config5_layer_stack_on_one_stream(oracle):
    """config 5: 12 back-to-back calls with distinct inputs on one stream, no host
    synchronisation in between; every word of every call compared (all 512 rows x 49,152
    columns), and every word of the canonical-layout kernel's output for the last call"""
    import torch
    import paper_2411_15707_amd as nc
    import gpu_util as gu
    cfg = ci.CONFIGS[5]
    stream = torch.cuda.Stream()
    ws = torch.empty(nc.nimbus_cop_workspace_bytes(cfg.m, cfg.k, cfg.t_bits), dtype=torch.uint8,
                     device="cuda")
    held = []
    for call in range(cfg.calls):
        seed = ci.config_seed(5, call)
        _say(f"[parity] config 5 call {call}: inputs + oracle (all rows)")
        X, ctW, mask = _inputs(seed, cfg.m, cfg.k, cfg.n, cfg.N, cfg.moduli, cfg.t_bits)
        want, _ = oracle.cop_ref(X, ctW, cfg.moduli, cfg.n, cfg.N, mask)
        prepared = gu.prepare(ctW, cfg.moduli, cfg.n, cfg.N)
        dX, dM = gu.dev(X), gu.dev(mask)
        out = torch.full((cfg.m, cfg.Ch, 2, cfg.L, cfg.N), -1, dtype=torch.int64, device="cuda")
        held.append((dX, prepared, dM, out, want))
        if call + 1 < cfg.calls:
            del ctW, mask
    torch.cuda.synchronize()
    _say("[parity] config 5: launching 12 calls back to back")
    with torch.cuda.stream(stream):
        for dX, prepared, dM, out, _ in held:
            nc.nimbus_cop_matmul_prepared(dX, cfg.m, cfg.k, cfg.t_bits, prepared, cfg.n, cfg.N,
                                          cfg.L, cfg.moduli, dM, out, ws, stream)
    stream.synchronize()
    for call, (_, _, _, out, want) in enumerate(held):
        got = gu.host(out)
        assert got.shape == want.shape
        assert np.array_equal(got, want), f"call {call}: " + gu.first_mismatch(got, want)
    # the canonical-layout entry point on the last call's inputs, every word
    want_last = held[-1][4]
    del held
    _say("[parity] config 5: canonical-layout entry point, last call")
    got = gu.run_canon(X, ctW, cfg.moduli, cfg.n, cfg.N, cfg.t_bits, mask)
    assert np.array_equal(got, want_last), "canonical: " + gu.first_mismatch(got, want_last)
    _say("[parity] config 5: vector-ALU kernel, last call")
    got = gu.run_valu(X, ctW, cfg.moduli, cfg.n, cfg.N, cfg.t_bits, mask)
    assert np.array_equal(got, want_last), "valu: " + gu.first_mismatch(got, want_last)


def test_repeat_runs_are_identical(oracle):
    """integer sums are order independent: two runs that differ point at a race"""
    import gpu_util as gu
    cfg = ci.CONFIGS[2]
    X, ctW, mask = _inputs(42, cfg.m, 256, cfg.n, cfg.N, cfg.moduli, cfg.t_bits)
    prepared = gu.prepare(ctW, cfg.moduli, cfg.n, cfg.N)
    a = gu.run_mfma(X, ctW, cfg.moduli, cfg.n, cfg.N, cfg.t_bits, mask, prepared)
    b = gu.run_mfma(X, ctW, cfg.moduli, cfg.n, cfg.N, cfg.t_bits, mask, prepared)
    assert np.array_equal(a, b)


def test_errors_leave_out_untouched():
    import torch
    import paper_2411_15707_amd as nc
    moduli = ci.limb_primes(50, 16, 1)
    X = torch.zeros((4, 8), dtype=torch.int64, device="cuda")
    ctW = torch.zeros((8, 1, 2, 1, 32), dtype=torch.int64, device="cuda")
    out = torch.full((4, 1, 2, 1, 32), 7, dtype=torch.int64, device="cuda")
    with pytest.raises(nc.NimbusCopError) as ei:
        nc.nimbus_cop_matmul(X, 4, 8, 16, ctW, 32, 32, 1, (moduli[0] + 1,), None, out)
    assert ei.value.status == -1
    torch.cuda.synchronize()
    assert (out == 7).all()


def test_two_step_entry_points_match_the_fused_call(oracle):
    """nimbus_cop_stage_shares + nimbus_cop_matmul_staged == nimbus_cop_matmul_prepared == oracle"""
    import torch
    import paper_2411_15707_amd as nc
    import gpu_util as gu
    m, k, n, N, L, t_bits = 70, 200, 128, 128, 2, 20
    moduli = ci.limb_primes(54, t_bits, L)
    X, ctW, mask = _inputs(77, m, k, n, N, moduli, t_bits)
    want, _ = oracle.cop_ref(X, ctW, moduli, n, N, mask)
    prepared = gu.prepare(ctW, moduli, n, N)
    ws = torch.empty(nc.nimbus_cop_workspace_bytes(m, k, t_bits), dtype=torch.uint8, device="cuda")
    out = torch.full((m, 1, 2, L, N), -1, dtype=torch.int64, device="cuda")
    nc.nimbus_cop_stage_shares(gu.dev(X), m, k, t_bits, ws)
    nc.nimbus_cop_matmul_staged(ws, m, k, t_bits, prepared, n, N, L, moduli, gu.dev(mask), out)
    torch.cuda.synchronize()
    assert np.array_equal(gu.host(out), want)
    assert np.array_equal(gu.run_mfma(X, ctW, moduli, n, N, t_bits, mask, prepared), want)


# m, n, N, L, t_bits, q_bits
PACK_SHAPES = [
    (8, 64, 1024, 1, 16, 50),       # config 1: 16 rows per ciphertext, half-filled
    (7, 10, 32, 2, 20, 54),         # ragged: three per ciphertext, the last holds one row
    (5, 40, 64, 2, 20, 54),         # one row per ciphertext: only the mask is added
    (33, 64, 64, 3, 24, 55),        # n = N
    (128, 768, 4096, 2, 20, 54),    # config 4: five per ciphertext, 26 ciphertexts
    (512, 4096, 8192, 3, 24, 55),   # config 5: two per ciphertext
    (9, 7, 32, 2, 20, 54),          # odd n: odd shifts, one word per thread
    (20, 333, 1024, 1, 16, 50),     # odd n, three per ciphertext
]


@pytest.mark.parametrize("m,n,N,L,t_bits,q_bits", PACK_SHAPES)
def test_pack_matches_the_oracle(oracle, m, n, N, L, t_bits, q_bits):
    import gpu_util as gu
    import paper_2411_15707_amd as nc
    moduli = ci.limb_primes(q_bits, t_bits, L)
    T = oracle.packed_count(m, n, N)
    rows = ci.gen_mask_uniform(4000 + m, m, 1, moduli, N)[:, 0]
    mask = ci.gen_mask_uniform(5000 + m, T, 1, moduli, N)[:, 0]
    for l, q in enumerate(moduli):                      # extremes: largest residues, zeros
        rows[0, :, l, :3] = q - 1
        rows[-1, :, l, -3:] = q - 1
        rows[0, :, l, 3:5] = 0
        mask[0, :, l, :3] = q - 1
    _say(f"[parity] pack m={m} n={n} N={N} L={L}")
    for msk in (mask, None):
        d_rows, d_out = gu.dev(rows), gu.dev(np.zeros((T, 2, L, N), dtype=np.uint64))
        nc.nimbus_cop_pack(d_rows, m, n, N, L, moduli, gu.dev(msk) if msk is not None else None, d_out)
        got = gu.host(d_out)
        want = oracle.pack_ref(rows, n, moduli, msk)
        assert np.array_equal(got, want), gu.first_mismatch(got, want)
    # the same call on buffers that start 8 bytes off a 16-byte boundary (one word per thread)
    import torch
    def off8(a):
        big = torch.empty(a.size + 1, dtype=torch.int64, device="cuda")
        view = big[1:].view(a.shape)
        view.copy_(gu.dev(a))
        return view
    d_rows, d_mask, d_out = off8(rows), off8(mask), off8(np.zeros((T, 2, L, N), dtype=np.uint64))
    assert d_rows.data_ptr() % 16 == 8
    nc.nimbus_cop_pack(d_rows, m, n, N, L, moduli, d_mask, d_out)
    got = gu.host(d_out)
    want = oracle.pack_ref(rows, n, moduli, mask)
    assert np.array_equal(got, want), gu.first_mismatch(got, want)


def test_config1_matmul_then_pack_decrypts_to_side_by_side_payloads(oracle):
    """whole client step on the GPU: COP on really encrypted weights without mask, packing
    with a share mask, then Dec(packed)[u n + c] + R[u n + c] = (X W)[u][c] mod t"""
    import gpu_util as gu
    import paper_2411_15707_amd as nc
    cfg = ci.CONFIGS[1]
    seed = ci.config_seed(1) + 900
    t, n, N, L, m = cfg.t, cfg.n, cfg.N, cfg.L, cfg.m
    P, T = N // n, oracle.packed_count(m, n, N)
    X = ci.gen_X(seed, m, cfg.k, cfg.t_bits)
    W = ci.gen_W(seed, cfg.k, n, cfg.t_bits)
    s = ci.gen_secret(seed, N)
    a, e = ci.gen_enc_randomness(seed, cfg.k, 1, cfg.moduli, N)
    ct = oracle.encrypt(oracle.encode_rows(W, N)[:, 0], s, a[:, 0], e[:, 0], cfg.moduli, cfg.t_bits)
    rows = gu.run_mfma(X, ct.reshape(cfg.k, 1, 2, L, N), cfg.moduli, n, N, cfg.t_bits, None)
    R = ci.gen_R(seed, T, N, cfg.t_bits)
    mask = np.stack([oracle.share_mask(R[th], cfg.moduli, cfg.t_bits) for th in range(T)])
    d_out = gu.dev(np.zeros((T, 2, L, N), dtype=np.uint64))
    nc.nimbus_cop_pack(gu.dev(rows[:, 0]), m, n, N, L, cfg.moduli, gu.dev(mask), d_out)
    packed = gu.host(d_out)
    assert np.array_equal(packed, oracle.pack_ref(rows[:, 0], n, cfg.moduli, mask))
    XW = X.astype(object) @ W.astype(object)
    for th in range(T):
        got = (oracle.decrypt(packed[th], s, cfg.moduli, cfg.t_bits) + R[th]) % np.uint64(t)
        want = np.zeros(N, dtype=object)
        for u in range(P):
            if th * P + u < m:
                want[u * n:(u + 1) * n] = XW[th * P + u] % t
        assert np.array_equal(got, want.astype(np.uint64))


# m, k, n, N, L, x_bits, q_bits (per limb)
WIDE = [
    (5, 40, 32, 32, 2, 64, (59, 55)),        # the paper's limb sizes, full 64-bit shares
    (33, 100, 64, 64, 1, 64, (54,)),         # 4 + 4 share planes x 7 ciphertext planes
    (17, 70, 64, 64, 2, 48, (62, 55)),       # 48-bit shares: upper half has two planes
    (9, 33, 32, 32, 1, 33, (50,)),           # one bit above 32
    (32, 128, 8192, 8192, 2, 64, (59, 55)),  # the paper's ring degree and moduli, one chunk
    (128, 64, 64, 64, 2, 64, (59, 55)),      # full row block: both passes in the build without row tests
    (128, 40, 32, 32, 1, 40, (54,)),         # the same with a one-plane upper half
]


@pytest.mark.parametrize("m,k,n,N,L,x_bits,q_bits", WIDE)
def test_wide_shares_two_pass_path(oracle, m, k, n, N, L, x_bits, q_bits):
    """shares of more than 32 bits (Section 5.1: l = 64) through the prepared path against the
    per-term-reduced oracle, with and without mask, extremes included"""
    import gpu_util as gu
    moduli = tuple(ci.limb_primes(b, 14, 1)[0] for b in q_bits)
    X = ci.gen_X(7000 + m, m, k, x_bits)
    X[0, 0] = (1 << x_bits) - 1
    X[-1, :] = (1 << x_bits) - 1
    X[0, 1] = 0
    ctW = ci.gen_ctW_uniform(7000 + m, k, 1, moduli, N)
    mask = ci.gen_mask_uniform(7000 + m, m, 1, moduli, N)
    for l, q in enumerate(moduli):
        ctW[:, 0, :, l, :4] = q - 1
        mask[0, 0, :, l, :4] = q - 1
    _say(f"[parity] wide shares m={m} k={k} N={N} L={L} x_bits={x_bits}")
    prepared = gu.prepare(ctW, moduli, n, N)
    for msk in (mask, None):
        want, _ = oracle.cop_ref(X, ctW, moduli, n, N, msk, wide=True)
        got = gu.run_mfma(X, ctW, moduli, n, N, x_bits, msk, prepared=prepared)
        assert np.array_equal(got, want), gu.first_mismatch(got, want)


# m, k, n, N, L, t_bits, q_bits, problems, with masks
BATCHES = [
    (128, 416, 64, 64, 2, 20, 54, 5, True),       # mask tile through LDS, 13 k-blocks
    (33, 100, 40, 64, 2, 20, 54, 3, True),        # ragged rows and k
    (256, 100, 256, 256, 1, 20, 54, 3, True),     # two row blocks per column tile
    (128, 96, 8192, 8192, 3, 20, 54, 2, False),   # 768 tiles each: more tiles than compute units
    (64, 70, 64, 64, 1, 32, 62, 4, True),         # 4 x 8 planes (operands read after the barrier)
    (8, 64, 64, 1024, 1, 16, 50, 16, True),       # the largest batch, config 1's shape
    (40, 96, 128, 128, 3, 24, 55, 1, True),       # a batch of one
]


@pytest.mark.parametrize("m,k,n,N,L,t_bits,q_bits,count,with_mask", BATCHES)
def test_several_problems_in_one_launch(oracle, m, k, n, N, L, t_bits, q_bits, count, with_mask):
    """nimbus_cop_stage_shares_batch + nimbus_cop_matmul_staged_batch: independent share
    matrices, weights, masks and outputs of one shape in one launch each, every output equal
    to the oracle's (and so to separate calls)"""
    import torch
    import gpu_util as gu
    import paper_2411_15707_amd as nc
    moduli = ci.limb_primes(q_bits, t_bits, L)
    Ch = -(-n // N)
    probs = [_inputs(9000 + 17 * i + m, m, k, n, N, moduli, t_bits, with_mask) for i in range(count)]
    probs[0][0][0, :] = (1 << t_bits) - 1
    _say(f"[parity] batch of {count}: m={m} k={k} n={n} N={N} L={L}")
    dXs = [gu.dev(X) for X, _, _ in probs]
    preps = [gu.prepare(ctW, moduli, n, N) for _, ctW, _ in probs]
    masks = [gu.dev(mk) for _, _, mk in probs] if with_mask else None
    wss = [torch.empty(nc.nimbus_cop_workspace_bytes(m, k, t_bits), dtype=torch.uint8, device="cuda")
           for _ in range(count)]
    outs = [torch.full((m, Ch, 2, L, N), -1, dtype=torch.int64, device="cuda") for _ in range(count)]
    nc.nimbus_cop_stage_shares_batch(dXs, m, k, t_bits, wss)
    nc.nimbus_cop_matmul_staged_batch(wss, m, k, t_bits, preps, n, N, L, moduli, masks, outs)
    torch.cuda.synchronize()
    for i, (X, ctW, mk) in enumerate(probs):
        want, _ = oracle.cop_ref(X, ctW, moduli, n, N, mk)
        got = gu.host(outs[i])
        assert np.array_equal(got, want), f"problem {i}: " + gu.first_mismatch(got, want)


def test_calibration_launches_run():
    """the benchmark's calibration kernels enqueue and report the work they were asked for"""
    import torch
    import paper_2411_15707_amd as nc
    sink = torch.zeros(8 * 256, dtype=torch.int32, device="cuda")
    assert nc.nimbus_calib_mfma_i8(8, 3, 1, sink) == 8 * 4 * 3 * 21 * 65536
    assert nc.nimbus_calib_mfma_i8(8, 3, 0, sink) == 8 * 4 * 3 * 21 * 65536
    torch.cuda.synchronize()
    assert int(sink.abs().max()) == 0                      # zero operands leave zero accumulators
    src = torch.ones(1 << 20, dtype=torch.int32, device="cuda")
    assert nc.nimbus_calib_stream_read(src, sink) == 4 << 20
    torch.cuda.synchronize()
    with pytest.raises(nc.NimbusCopError):
        nc.nimbus_calib_mfma_i8(8, 3, 1, sink[:16])        # sink too small: refused on the host
    bsink = torch.zeros(8 * 256, dtype=torch.int64, device="cuda")
    assert nc.nimbus_calib_butterflies(8, 5, (1 << 54) - 33, bsink) == 8 * 256 * 5 * 12
    torch.cuda.synchronize()
    assert int((bsink != 0).sum()) > 8 * 256 // 2          # the loop ran and wrote its values
    with pytest.raises(nc.NimbusCopError):
        nc.nimbus_calib_butterflies(8, 5, 1 << 54, bsink)  # even modulus: refused on the host


@pytest.mark.parametrize("t_bits,q_bits", [(32, 62), (20, 54), (16, 50)])
def test_longest_inner_dimension_with_extreme_digits(oracle, t_bits, q_bits):
    """k = 16383, the largest the matrix-core path accepts: 512 k-blocks, int32 accumulators
    closest to their bound.  Shares 0 and t-1 give share digits -128 and 127 in every shifted
    plane; residues around q/2 give ciphertext digits of the largest magnitude the centred
    recoding can produce."""
    import gpu_util as gu
    m, k, n, N, L = 3, 16383, 32, 32, 1
    moduli = ci.limb_primes(q_bits, t_bits, L)
    q = moduli[0]
    X = ci.gen_X(31, m, k, t_bits)
    X[0, :] = 0
    X[1, :] = (1 << t_bits) - 1
    ctW = ci.gen_ctW_uniform(31, k, 1, moduli, N)
    ctW[:, 0, :, 0, 0] = (q - 1) // 2          # centred: the most positive value
    ctW[:, 0, :, 0, 1] = (q - 1) // 2 + 1      # the most negative
    ctW[:, 0, :, 0, 2] = q - 1
    ctW[:, 0, :, 0, 3] = 0
    mask = ci.gen_mask_uniform(31, m, 1, moduli, N)
    _say(f"[parity] k=16383 t_bits={t_bits} q_bits={q_bits}")
    want, _ = oracle.cop_ref(X, ctW, moduli, n, N, mask)
    got = gu.run_mfma(X, ctW, moduli, n, N, t_bits, mask)
    assert np.array_equal(got, want), gu.first_mismatch(got, want)


def test_random_parameter_sweep(oracle):
    """forty seeded random parameter sets (ring degree, limbs of different sizes, share widths
    1..64 bits, ragged m and k, one to three ring chunks), both kernels where they apply"""
    import gpu_util as gu
    rng = np.random.default_rng(20241115707)
    for case in range(40):
        N = int(rng.choice([32, 64, 128]))
        L = int(rng.integers(1, 4))
        n = int(rng.integers(1, 3 * N + 1))
        m = int(rng.integers(1, 141))
        k = int(rng.integers(1, 401))
        x_bits = int(rng.integers(1, 65)) if case % 4 == 3 else int(rng.integers(1, 33))
        lo = max(min(x_bits, 32) + 2, 20)
        moduli = []
        while len(moduli) < L:                       # limbs of different sizes, all distinct
            b = int(rng.integers(lo, 63))
            q = ci.limb_primes(b, 5, 1)[0]
            if q not in moduli:
                moduli.append(q)
        moduli = tuple(moduli)
        Ch = -(-n // N)
        X = ci.gen_X(9000 + case, m, k, x_bits)
        ctW = ci.gen_ctW_uniform(9000 + case, k, Ch, moduli, N)
        mask = ci.gen_mask_uniform(9000 + case, m, Ch, moduli, N) if case % 3 else None
        label = f"sweep {case}: m={m} k={k} n={n} N={N} L={L} x_bits={x_bits} q_bits={[q.bit_length() for q in moduli]}"
        _say("[parity] " + label)
        want, _ = oracle.cop_ref(X, ctW, moduli, n, N, mask, wide=x_bits > 32)
        got = gu.run_mfma(X, ctW, moduli, n, N, x_bits, mask)
        assert np.array_equal(got, want), label + " mfma: " + gu.first_mismatch(got, want)
        if x_bits <= 32:
            got = gu.run_valu(X, ctW, moduli, n, N, x_bits, mask)
            assert np.array_equal(got, want), label + " valu: " + gu.first_mismatch(got, want)


def test_check_inputs_counts_planted_violations():
    """the debugging aid counts exactly the words that break the value-range preconditions:
    shares >= 2^x_bits, residues >= the modulus of their own limb (a word between the two
    moduli counts only in the columns of the smaller one)"""
    import torch
    import gpu_util as gu
    import paper_2411_15707_amd as nc
    m, k, n, N, L, t_bits = 20, 37, 100, 64, 2, 20
    moduli = (ci.limb_primes(54, t_bits, 1)[0], ci.limb_primes(50, t_bits, 1)[0])
    Ch = -(-n // N)
    X, ctW, mask = _inputs(77, m, k, n, N, moduli, t_bits)
    v = torch.full((3,), 123, dtype=torch.int64, device="cuda")
    nc.nimbus_cop_check_inputs(gu.dev(X), m, k, t_bits, gu.dev(ctW), n, N, L, moduli, gu.dev(mask), v)
    torch.cuda.synchronize()
    assert v.tolist() == [0, 0, 0]
    X = X.copy(); ctW = ctW.copy(); mask = mask.copy()
    X[3, 5] = 1 << t_bits                       # one too many bits
    X[19, 36] = (1 << 64) - 1
    between = np.uint64(moduli[1] + 5)          # >= q_1, < q_0
    ctW[0, 0, 0, 1, 0] = between                # limb 1: counts
    ctW[7, 1, 1, 0, 63] = between               # limb 0: a valid residue
    ctW[36, 1, 1, 0, 63] = np.uint64(moduli[0]) # exactly q_0: counts
    ctW[2, 0, 1, 1, 17] = np.uint64((1 << 64) - 1)
    mask[19, Ch - 1, 1, 1, 63] = np.uint64(moduli[1])
    nc.nimbus_cop_check_inputs(gu.dev(X), m, k, t_bits, gu.dev(ctW), n, N, L, moduli, gu.dev(mask), v)
    torch.cuda.synchronize()
    assert v.tolist() == [2, 3, 1]
    nc.nimbus_cop_check_inputs(gu.dev(X), m, k, t_bits, gu.dev(ctW), n, N, L, moduli, None, v)
    torch.cuda.synchronize()
    assert v.tolist() == [2, 3, 0]
    # 64-bit shares: nothing can be out of range
    nc.nimbus_cop_check_inputs(gu.dev(X), m, k, 64, gu.dev(ctW), n, N, L, moduli, None, v)
    torch.cuda.synchronize()
    assert v.tolist() == [0, 3, 0]


def test_concurrent_calls_on_two_streams(oracle):
    """the library keeps no state between calls: two layers enqueued alternately on two
    streams (own workspaces and outputs, the same prepared weights) both come out right"""
    import torch
    import gpu_util as gu
    import paper_2411_15707_amd as nc
    m, k, n, N, L, t_bits = 128, 192, 256, 256, 2, 20
    moduli = ci.limb_primes(54, t_bits, L)
    C = 2 * L * N
    ctW = ci.gen_ctW_uniform(606, k, 1, moduli, N)
    prepared = gu.prepare(ctW, moduli, n, N)
    streams = [torch.cuda.Stream(), torch.cuda.Stream()]
    Xs = [ci.gen_X(607 + i, m, k, t_bits) for i in range(2)]
    masks = [ci.gen_mask_uniform(609 + i, m, 1, moduli, N) for i in range(2)]
    dX = [gu.dev(x) for x in Xs]
    dM = [gu.dev(x) for x in masks]
    ws = [torch.empty(nc.nimbus_cop_workspace_bytes(m, k, t_bits), dtype=torch.uint8, device="cuda")
          for _ in range(2)]
    outs = [torch.zeros((m, C), dtype=torch.int64, device="cuda") for _ in range(2)]
    torch.cuda.synchronize()
    for rep in range(20):
        for i in range(2):
            nc.nimbus_cop_matmul_prepared(dX[i], m, k, t_bits, prepared, n, N, L, moduli, dM[i],
                                          outs[i], ws[i], stream=streams[i])
    torch.cuda.synchronize()
    for i in range(2):
        want = oracle.cop_ref(Xs[i], ctW, moduli, n, N, masks[i])[0]
        assert np.array_equal(gu.host(outs[i]).reshape(want.shape), want), f"stream {i}"
