#!/usr/bin/env python3
"""Benchmark of the COP ciphertext x share matmul on one MI355X.

A step = one pass of the whole hot path over one batch: stage the client's shares
X, stream the prepared weight ciphertexts, accumulate, reduce, add the mask, store
(nimbus_cop_matmul_prepared).  The workload is config 3 of the benchmark spec (BERT-base
FFN up-projection: m=128, k=768, n=3072, N=4096, L=2, t=2^20).  Inputs are seeded
and synthetic, resident in HBM before the timed region; the step rotates over
enough distinct weight / mask / output buffers that the 256 MB last-level cache
cannot serve them.  The one-time weight re-layout (nimbus_cop_prepare) is the
protocol's setup phase and is not timed.

Prints ONE JSON line.  `roofline` is for the matrix-core kernel alone, timed with
events on the launch stream; `cpu_baseline` is the CPU oracle on the host cores.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0          # MI355X HBM3E
INT8_PEAK_TOPS = 5000.0         # MI355X dense int8 MFMA, tera-ops/s (2 ops per MAC)
# 32-bit integer vector operations: 256 compute units x 4 SIMDs x 16 lanes x 2.4 GHz
INT32_PEAK_TOPS = 256 * 4 * 16 * 2.4e9 / 1e12
METRIC = "modular MACs/sec (Z_q) + HBM GB/s, COP ct×share matmul, BERT-base FFN shape"


def read_traffic(workload_key):
    """HBM bytes per launch measured with rocprofv3 --pmc (profiles/*_traffic.txt), or None"""
    path = os.path.join(ROOT, "profiles", f"cop_mfma_kernel_{workload_key}_traffic.txt")
    if not os.path.exists(path):
        return None
    for line in open(path):
        if line.startswith("traffic_bytes_per_launch"):
            return float(line.split()[1])
    return None


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=2000)
    ap.add_argument("--warmup", type=int, default=500)
    ap.add_argument("--config", type=int, default=3, help="BASELINE.json config number (1-5)")
    ap.add_argument("--buffers", type=int, default=0, help="distinct weight buffers (0 = auto)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-prefetch", action="store_true", help="skip the weight-loading stack")
    ap.add_argument("--no-graph", action="store_true", help="skip the HIP-graph replay of the steps")
    ap.add_argument("--no-paper-setting", action="store_true",
                    help="skip the run at the paper's own parameters (64-bit shares, N = 8192)")
    ap.add_argument("--no-batched", action="store_true",
                    help="skip the run with several steps per launch")
    ap.add_argument("--no-two-streams", action="store_true",
                    help="skip the run with two batches in flight on two streams")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU; the path shards over coefficient columns "
              "with no exchange, but no multi-GPU run exists. Use --gpus 1.", file=sys.stderr)
        return 2

    import numpy as np
    import torch

    import cop_inputs as ci
    import paper_2411_15707_amd as nc

    nc.load_library()                      # fails loudly if the HIP library is missing
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 2
    torch.cuda.set_device(0)
    cfg = ci.CONFIGS[args.config]
    m, k, n, N, L, xb, moduli = cfg.m, cfg.k, cfg.n, cfg.N, cfg.L, cfg.t_bits, cfg.moduli
    C = cfg.C

    def dev(a):
        return torch.from_numpy(np.ascontiguousarray(a).view(np.int64)).cuda()

    prep_bytes = nc.nimbus_cop_prepared_bytes(k, n, N, L, moduli)
    R = args.buffers or max(2, -(-(1 << 30) // prep_bytes))
    ws = torch.empty(nc.nimbus_cop_workspace_bytes(m, k, xb), dtype=torch.uint8, device="cuda")
    Xs, preps, masks, outs = [], [], [], []
    first = None
    for r in range(R):
        seed = ci.config_seed(args.config, call=100 + r)
        X = ci.gen_X(seed, m, k, xb)
        ctW = ci.gen_ctW_uniform(seed, k, cfg.Ch, moduli, N)
        mask = ci.gen_mask_uniform(seed, m, cfg.Ch, moduli, N)
        if r == 0:
            first = (X, ctW, mask)
        dW = dev(ctW)
        prepared = torch.empty(prep_bytes, dtype=torch.uint8, device="cuda")
        nc.nimbus_cop_prepare(dW, k, n, N, L, moduli, prepared)      # setup phase, untimed
        torch.cuda.synchronize()
        del dW
        Xs.append(dev(X))
        preps.append(prepared)
        masks.append(dev(mask))
        outs.append(torch.empty((m, C), dtype=torch.int64, device="cuda"))

    def step(r):
        nc.nimbus_cop_matmul_prepared(Xs[r], m, k, xb, preps[r], n, N, L, moduli, masks[r],
                                      outs[r], ws)

    # A chip that has been idle, even for ten milliseconds of host work, takes some 25 ms of
    # load (700 launches of this kernel) to settle its clocks, and runs up to a quarter slower
    # meanwhile.  Every timed region below therefore follows directly on about 50 ms of untimed
    # launches of the same work, whatever W and K are.
    def settle(fn, seconds=0.05):
        """untimed calls fn(0), fn(1), ... for `seconds` of wall-clock, never far ahead of the GPU"""
        c0, i = time.perf_counter(), 0
        while time.perf_counter() - c0 < seconds:
            fn(i)
            i += 1
            if i % 64 == 0:
                torch.cuda.synchronize()

    def event_timed(fn, count, record_on=None):
        """ms per call of fn(i), i < count: settle, then one event pair around all the calls, on the
        stream they are launched on"""
        st = record_on if record_on is not None else torch.cuda.current_stream()
        settle(fn)
        a_, b_ = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        a_.record(st)
        for i in range(count):
            fn(i)
        b_.record(st)
        torch.cuda.synchronize()
        return a_.elapsed_time(b_) / count
    # launches of the event-timed side regions: K, but never so few that one clock step decides
    side_launches = max(args.steps, 500)

    # ---- whole-path timing: W warm-up steps, then exactly K steps ----
    settle(lambda i: step(i % R))
    for s in range(args.warmup):
        step(s % R)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for s in range(args.steps):
        step(s % R)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_per_step = (t1 - t0) * 1e3 / args.steps
    value = cfg.mod_macs / (ms_per_step * 1e-3)

    # ---- two batches in flight: the same steps dealt alternately to two streams (each with its
    # own share workspace; every weight / mask / output buffer stays with one stream).  Launches
    # on one stream are serialised by the queue, with a few microseconds between the end of one
    # kernel and the start of the next; a second stream fills them, and the staging kernel of
    # one batch runs under the main kernel of the other.  What a client serving two queries
    # gets; reported beside the one-stream figures, which stay the headline. ----
    two_streams = None
    if not args.no_two_streams and R >= 2:
        S = 2
        Rs = R - R % S
        streams = [torch.cuda.Stream() for _ in range(S)]          # default priority
        wss = [ws] + [torch.empty_like(ws) for _ in range(S - 1)]
        want = [outs[r].clone() for r in range(S)]                  # results of the one-stream run

        def run(count):
            for s in range(count):
                r = s % Rs
                nc.nimbus_cop_matmul_prepared(Xs[r], m, k, xb, preps[r], n, N, L, moduli, masks[r],
                                              outs[r], wss[r % S], stream=streams[r % S])

        def timed_two_streams(fn, count):
            """ms per call of fn(count): events on both streams, the later end minus the earlier start"""
            ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True))
                  for _ in range(S)]
            torch.cuda.synchronize()
            for i, st in enumerate(streams):
                ev[i][0].record(st)
            fn(count)
            for i, st in enumerate(streams):
                ev[i][1].record(st)
            torch.cuda.synchronize()
            # both start events are recorded on idle streams within microseconds of each other:
            # the span is the longest of (start of either -> end of either)
            return max(ev[i][0].elapsed_time(ev[j][1]) for i in range(S) for j in range(S)) / count

        for r in range(S):
            outs[r].zero_()
        torch.cuda.synchronize()
        settle(lambda i: run(Rs))
        torch.cuda.synchronize()
        steps2 = max(Rs, args.steps, 1000)          # enough launches whatever --steps is
        steps2 -= steps2 % Rs
        ms2 = timed_two_streams(run, steps2)
        two_streams = {
            "streams": S,
            "steps": steps2,
            "ms_per_step": round(ms2, 5),
            "value": round(cfg.mod_macs / (ms2 * 1e-3), 1),
            "hbm_gbps_whole_step": round(cfg.alg_bytes / (ms2 * 1e-3) / 1e9, 1),
            "frac_of_hbm_peak": round(cfg.alg_bytes / (ms2 * 1e-3) / 1e9 / HBM_PEAK_GBPS, 4),
            "outputs_equal_one_stream": all(bool(torch.equal(outs[r], want[r])) for r in range(S)),
        }
        del want

    # ---- the same steps recorded once in a HIP graph (one step per weight buffer) and replayed:
    # what a caller who records its layer loop pays per step ----
    graph_ms_per_step = None
    if not args.no_graph:
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            step(0)
        torch.cuda.current_stream().wait_stream(side)
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=side):
            for r in range(R):
                step(r)
        replays = max(1, side_launches // R)
        settle(lambda i: graph.replay())
        for _ in range(max(1, args.warmup // R)):
            graph.replay()
        torch.cuda.synchronize()
        g0 = time.perf_counter()
        for _ in range(replays):
            graph.replay()
        torch.cuda.synchronize()
        graph_ms_per_step = (time.perf_counter() - g0) * 1e3 / (replays * R)
        del graph

    # ---- dominant kernel alone (shares already staged), events on the launch stream ----
    staged = []
    for r in range(R):
        w = torch.empty_like(ws)
        nc.nimbus_cop_stage_shares(Xs[r], m, k, xb, w)
        staged.append(w)
    torch.cuda.synchronize()
    # One pair of events around all the launches of the timed region, on the stream they are
    # launched on: average duration per launch = elapsed / launches (launch gaps included).  An
    # event pair around every single launch would add several microseconds of queue
    # draining to each.
    stream = torch.cuda.current_stream()
    kernel_launches = side_launches
    kernel_ms_avg = event_timed(
        lambda i: nc.nimbus_cop_matmul_staged(staged[i % R], m, k, xb, preps[i % R], n, N, L, moduli,
                                              masks[i % R], outs[i % R]), kernel_launches, stream)
    alg_bytes = cfg.alg_bytes              # 8 B/residue: ctW once + mask + out + X
    achieved_gbps = alg_bytes / (kernel_ms_avg * 1e-3) / 1e9
    # byte-digit MACs the kernel issues: DX x DQ int8 MACs per modular MAC (k padded to 32)
    DX = max(2, -(-xb // 8))
    DQ = max(7, -(-(max(q.bit_length() for q in moduli) + 1) // 8))
    i8_ops = 2.0 * DX * DQ * m * (-(-k // 32) * 32) * C
    workload_key = f"config{args.config}"
    i8_tops = i8_ops / (kernel_ms_avg * 1e-3) / 1e12
    # the roofline that binds: the one whose time at the published peak is longer (HBM for
    # configs 1-4, slightly before the matrix cores; the matrix cores for config 5, m = 512)
    t_hbm = alg_bytes / (HBM_PEAK_GBPS * 1e9)
    t_mfma = i8_ops / (INT8_PEAK_TOPS * 1e12)
    # the instance the library launches for this shape (share planes, ciphertext planes, m a
    # multiple of 128, mask tile through LDS, several row blocks per column tile)
    full = m % 128 == 0
    pipelined = (DX + DQ - 1) * 16 + 2 * (DX + DQ) * 4 + 12 <= 256
    mask_lds = full and pipelined and -(-k // 32) - 3 >= 10 and C * 8 * 128 < (1 << 32)
    flags = ",".join("true" if f else "false" for f in (full, mask_lds, m > 128))
    roofline = {"kernel": f"cop_mfma_kernel<{DX},{DQ},{flags}>"}
    if t_hbm >= t_mfma:
        roofline.update({"bound": "hbm", "achieved": round(achieved_gbps, 1), "peak": HBM_PEAK_GBPS,
                         "unit": "GB/s", "frac": round(achieved_gbps / HBM_PEAK_GBPS, 4)})
    else:
        roofline.update({"bound": "mfma", "achieved": round(i8_tops, 1),
                         "peak": INT8_PEAK_TOPS, "unit": "TOP/s",
                         "frac": round(i8_tops / INT8_PEAK_TOPS, 4)})
    roofline.update({
        "traffic": read_traffic(workload_key),
        "algorithmic_bytes_per_launch": alg_bytes,
        "hbm_gbps_achieved": round(achieved_gbps, 1),
        "hbm_frac_of_peak": round(achieved_gbps / HBM_PEAK_GBPS, 4),
        "kernel_ms_avg": round(kernel_ms_avg, 5),
        "launches_timed": kernel_launches,
        "mfma_int8_tops_achieved": round(i8_tops, 1),
        "mfma_int8_frac_of_peak": round(i8_tops / INT8_PEAK_TOPS, 4),
    })

    # the kernel alone with its launches dealt alternately to the two streams
    if two_streams is not None:
        S = two_streams["streams"]
        Rs = R - R % S

        def run_kernel(count):
            for s in range(count):
                r = s % Rs
                nc.nimbus_cop_matmul_staged(staged[r], m, k, xb, preps[r], n, N, L, moduli, masks[r],
                                            outs[r], stream=streams[r % S])

        settle(lambda i: run_kernel(Rs))
        torch.cuda.synchronize()
        launches2 = max(Rs, args.steps, 1000)
        launches2 -= launches2 % Rs
        k2 = timed_two_streams(run_kernel, launches2)
        two_streams["kernel_only_ms_per_launch"] = round(k2, 5)
        two_streams["kernel_only_hbm_gbps"] = round(alg_bytes / (k2 * 1e-3) / 1e9, 1)
        two_streams["kernel_only_frac_of_hbm_peak"] = round(alg_bytes / (k2 * 1e-3) / 1e9 / HBM_PEAK_GBPS, 4)

    # ---- several steps in one launch (nimbus_cop_stage_shares_batch + nimbus_cop_matmul_staged_batch):
    # what a caller pays per step who has the shares of several layers or requests at hand.
    # Same problems, same buffers, same outputs as the timed steps above. ----
    batched = None
    if not args.no_batched and R >= 2 and xb <= 32:
        Bn = min(12, R)
        bws = [torch.empty_like(ws) for _ in range(Bn)]
        want = []
        for r in range(Bn):
            step(r)
        torch.cuda.synchronize()
        want = [outs[r].clone() for r in range(Bn)]
        for r in range(Bn):
            outs[r].zero_()

        def batch_step():
            nc.nimbus_cop_stage_shares_batch(Xs[:Bn], m, k, xb, bws)
            nc.nimbus_cop_matmul_staged_batch(bws, m, k, xb, preps[:Bn], n, N, L, moduli, masks[:Bn], outs[:Bn])

        def batch_kernel():
            nc.nimbus_cop_matmul_staged_batch(bws, m, k, xb, preps[:Bn], n, N, L, moduli, masks[:Bn], outs[:Bn])
        batch_step()
        torch.cuda.synchronize()
        same = all(bool(torch.equal(outs[r], want[r])) for r in range(Bn))
        del want
        reps_b = max(10, min(side_launches, 2000) // Bn)

        def timed_b(fn):
            return event_timed(lambda i: fn(), reps_b, stream) / Bn
        bstep_ms, bkern_ms = timed_b(batch_step), timed_b(batch_kernel)
        batched = {
            "problems_per_launch": Bn,
            "launches_timed": reps_b,
            "ms_per_step": round(bstep_ms, 5),
            "value": round(cfg.mod_macs / (bstep_ms * 1e-3), 1),
            "kernel_ms_per_problem": round(bkern_ms, 5),
            "kernel_hbm_gbps": round(alg_bytes / (bkern_ms * 1e-3) / 1e9, 1),
            "kernel_frac_of_hbm_peak": round(alg_bytes / (bkern_ms * 1e-3) / 1e9 / HBM_PEAK_GBPS, 4),
            "outputs_equal_separate_calls": same,
            "note": "one staging launch and one matmul launch for all the problems; per problem",
        }
        del bws

    # ---- the canonical-layout entry points on the same workload (no setup pass, 8 B residues):
    # nimbus_cop_matmul (matrix-core kernel that splits the words into byte planes itself) and
    # nimbus_cop_matmul_valu (vector-ALU kernel, any parameters) ----
    # (weights rotated over enough canonical buffers of uniform residues to defeat the 256 MB
    # last-level cache, as for the prepared path; the output check of buffer 0 is further down)
    canon_bytes = k * C * 8
    Rc = max(2, -(-(1 << 30) // canon_bytes))
    dWs = [dev(first[1])] + [torch.randint(0, min(moduli), (k, C), dtype=torch.int64, device="cuda")
                             for _ in range(Rc - 1)]

    def timed_entry(fn, reps):
        return event_timed(lambda i: fn(Xs[0], m, k, xb, dWs[i % Rc], n, N, L, moduli, masks[0], outs[0]),
                           reps, stream)
    canon_ms = timed_entry(nc.nimbus_cop_matmul, min(side_launches, 1000))
    valu_ms = timed_entry(nc.nimbus_cop_matmul_valu, 10)
    # digits of the centred residue only where seven or eight signed digits cannot express q - 1
    centre = any(q - 1 > int("7f" * DQ, 16) for q in moduli)
    canonical = {
        "entry_point": "nimbus_cop_matmul",
        "kernel": "cop_canon_kernel<%d,%d,%s>" % (DX, DQ, ",".join(
            "true" if f else "false" for f in (m % 128 == 0, m > 128, centre))),
        "kernel_ms_avg": round(canon_ms, 5),
        "value": round(cfg.mod_macs / (canon_ms * 1e-3), 1),
        "algorithmic_bytes_per_launch": alg_bytes,
        "hbm_gbps_achieved": round(alg_bytes / (canon_ms * 1e-3) / 1e9, 1),
        "hbm_frac_of_peak": round(alg_bytes / (canon_ms * 1e-3) / 1e9 / HBM_PEAK_GBPS, 4),
        "weight_buffers_rotated": Rc,
        "vector_alu_kernel_ms": round(valu_ms, 4),
    }
    del dWs

    # ---- the paper's own parameter set (Section 5, experimental setup): shares in Z_{2^64},
    # N = 8192, one limb of 59 and one of 55 bits, a BERT-base projection (128 tokens, k = 768) onto
    # one ciphertext's worth of columns.  Shares wider than 32 bits take two passes over the same
    # prepared weights; (4 + 4) x 8 byte products per modular MAC instead of 21. ----
    paper_setting = None
    if not args.no_paper_setting and args.config == 3:
        pm, pk, pn, pN, pL, pxb = 128, 768, 8192, 8192, 2, 64
        pmoduli = (ci.limb_primes(59, 14, 1)[0], ci.limb_primes(55, 14, 1)[0])
        pC = 2 * pL * pN
        pbytes = nc.nimbus_cop_prepared_bytes(pk, pn, pN, pL, pmoduli)
        pR = max(2, -(-(1 << 30) // pbytes))
        pX, pprep, pmask, pout = [], [], [], []
        for r in range(pR):
            W = torch.empty((pk, pC), dtype=torch.int64, device="cuda")
            Mk = torch.empty((pm, pC), dtype=torch.int64, device="cuda")
            for l, q in enumerate(pmoduli):          # columns of limb l: blocks of N, every other one
                for p_ in range(2):
                    c0 = (p_ * pL + l) * pN
                    W[:, c0:c0 + pN].random_(0, q)
                    Mk[:, c0:c0 + pN].random_(0, q)
            pr = torch.empty(pbytes, dtype=torch.uint8, device="cuda")
            nc.nimbus_cop_prepare(W, pk, pn, pN, pL, pmoduli, pr)
            torch.cuda.synchronize()
            del W
            # 64-bit shares: two 32-bit halves (randint's upper bound is 2^63)
            Xw = (torch.randint(0, 1 << 32, (pm, pk), dtype=torch.int64, device="cuda") << 32) | \
                torch.randint(0, 1 << 32, (pm, pk), dtype=torch.int64, device="cuda")
            pX.append(Xw); pprep.append(pr); pmask.append(Mk)
            pout.append(torch.empty((pm, pC), dtype=torch.int64, device="cuda"))
        pws = torch.empty(nc.nimbus_cop_workspace_bytes(pm, pk, pxb), dtype=torch.uint8, device="cuda")
        p_ms = event_timed(
            lambda i: nc.nimbus_cop_matmul_prepared(pX[i % pR], pm, pk, pxb, pprep[i % pR], pn, pN, pL, pmoduli,
                                                    pmask[i % pR], pout[i % pR], pws),
            min(side_launches, 300), stream)
        p_macs = pm * pk * pC
        p_i8 = 2.0 * 64 * p_macs
        paper_setting = {
            "workload": "m=128 k=768 n=8192 N=8192 L=2 (59 + 55 bits) x_bits=64",
            "entry_point": "nimbus_cop_matmul_prepared (two passes: upper and lower halves of the shares)",
            "ms_per_step": round(p_ms, 5),
            "value": round(p_macs / (p_ms * 1e-3), 1),
            "byte_products_per_mod_mac": 64,
            "mfma_int8_frac_of_peak": round(p_i8 / (p_ms * 1e-3) / 1e12 / INT8_PEAK_TOPS, 4),
            "weight_buffers_rotated": pR,
        }
        del pX, pprep, pmask, pout, pws

    # ---- output packing by right shifts (Algorithm 1 step 3) on this config's output ----
    # rows: the unmasked outputs of the step above; P = floor(N/n) rows per packed ciphertext
    pack = None
    if cfg.n <= N and N // cfg.n == 1:
        pack = {
            "rows_per_ciphertext": 1,
            "kernel": None,
            "note": "n > N/2: every output row fills a ciphertext of its own, there is nothing to merge; "
                    "the mask of step 4 goes through the matmul's epilogue (the timed step above) and "
                    "no packing pass runs",
        }
    elif cfg.n <= N:
        P = N // cfg.n
        T = nc.nimbus_cop_packed_count(m, cfg.n, N)
        packed = [torch.empty((T, 2, L, N), dtype=torch.int64, device="cuda") for _ in range(R)]
        pmask = [masks[r].reshape(-1)[:T * 2 * L * N] for r in range(R)]     # T <= m rows of residues
        def pack_call(i):
            nc.nimbus_cop_pack(outs[i % R], m, cfg.n, N, L, moduli, pmask[i % R], packed[i % R])
        pack_ms = event_timed(pack_call, side_launches, stream)
        torch.cuda.synchronize()
        h0 = time.perf_counter()
        for s in range(200):
            pack_call(s)
        pack_host_us = (time.perf_counter() - h0) * 1e6 / 200
        torch.cuda.synchronize()
        pack_bytes = 8 * 2 * L * N * (m + 2 * T)       # rows read, mask read, packed written

        # Algorithm 1 steps 2-4 as a caller who packs runs them: matmul without mask, then the
        # packing pass with the mask, enqueued back to back on one stream (no host round trip)
        def layer(r):
            nc.nimbus_cop_matmul_prepared(Xs[r], m, k, xb, preps[r], n, N, L, moduli, None, outs[r], ws)
            nc.nimbus_cop_pack(outs[r], m, cfg.n, N, L, moduli, pmask[r], packed[r])
        layer_ms = event_timed(lambda i: layer(i % R), side_launches, stream)
        # the matmul kernel of that sequence alone: no mask to read (Algorithm 1 masks after the
        # packing), so 8 bytes per output less than the masked call of the roofline object
        nomask_ms = event_timed(
            lambda i: nc.nimbus_cop_matmul_staged(staged[i % R], m, k, xb, preps[i % R], n, N, L, moduli,
                                                  None, outs[i % R]), side_launches, stream)
        nomask_bytes = alg_bytes - 8 * m * C
        pack = {
            "kernel": "cop_pack_kernel<%d,%d>" % (2 if cfg.n % 2 == 0 else 1, 2 if P <= 2 else 4),
            "rows_per_ciphertext": P,
            "packed_ciphertexts": T,
            "kernel_ms_avg": round(pack_ms, 5),
            "host_enqueue_us_per_call": round(pack_host_us, 2),
            "algorithmic_bytes_per_launch": pack_bytes,
            "achieved_gbps": round(pack_bytes / (pack_ms * 1e-3) / 1e9, 1),
            "frac_of_hbm_peak": round(pack_bytes / (pack_ms * 1e-3) / 1e9 / HBM_PEAK_GBPS, 4),
            "matmul_without_mask_kernel_ms": round(nomask_ms, 5),
            "matmul_without_mask_frac_of_hbm_peak": round(nomask_bytes / (nomask_ms * 1e-3) / 1e9 / HBM_PEAK_GBPS, 4),
            "matmul_without_mask_frac_of_int8_peak": round(i8_ops / (nomask_ms * 1e-3) / 1e12 / INT8_PEAK_TOPS, 4),
            "matmul_then_pack_ms_per_step": round(layer_ms, 5),
            "matmul_then_pack_note": "stage + matmul (mask = NULL) + pack (with the mask) per step, "
                                     "back to back on one stream",
        }

    # ---- server side of this layer (Algorithm 1 steps 1 and 5): encryption of the k weight
    # rows and decryption of the m returned rows, plus the rate of the transform kernel on a
    # batch large enough to fill the chip several times ----
    server = None
    if N <= 16384:
        logN = N.bit_length() - 1
        seed = ci.config_seed(args.config, call=100)
        s_dev = torch.from_numpy(ci.gen_secret(seed, N)).cuda()
        tables = torch.empty(nc.nimbus_rlwe_tables_bytes(N, L), dtype=torch.uint8, device="cuda")
        nc.nimbus_rlwe_setup(N, L, moduli, s_dev, tables)
        Wp = dev(ci.gen_W(seed, k, n, xb))
        a_np, e_np = ci.gen_enc_randomness(seed, k, cfg.Ch, moduli, N)
        a_dev, e_dev = dev(a_np), torch.from_numpy(e_np).cuda()
        ct_enc = torch.empty((k, cfg.Ch, 2, L, N), dtype=torch.int64, device="cuda")
        rows = m * cfg.Ch
        phi = torch.empty((rows, L, N), dtype=torch.int64, device="cuda")
        m_hat = torch.empty((rows, N), dtype=torch.int64, device="cuda")
        Tb = max(rows, (256 << 20) // (2 * L * N * 8))          # about 256 MiB of ciphertexts
        ct_big = torch.empty((Tb, 2, L, N), dtype=torch.int64, device="cuda")
        for l, q in enumerate(moduli):
            ct_big[:, :, l].random_(0, q)
        phi_big = torch.empty((Tb, L, N), dtype=torch.int64, device="cuda")

        def timed_ms(launch, reps):
            return event_timed(lambda i: launch(), reps, stream)
        enc_ms = timed_ms(lambda: nc.nimbus_rlwe_encrypt(Wp, k, n, xb, N, L, moduli, tables, a_dev,
                                                         e_dev, ct_enc), 20)
        dec_ms = timed_ms(lambda: nc.nimbus_rlwe_decrypt(outs[0].view(rows, 2, L, N), rows, N, L,
                                                         moduli, xb, tables, phi, m_hat), 50)
        big_ms = timed_ms(lambda: nc.nimbus_rlwe_phase(ct_big, Tb, N, L, moduli, tables, phi_big), 10)
        # 32-bit integer operations of one product by the secret: two transforms of (N/2) log N
        # butterflies and N pointwise products, counted as the butterfly the kernels run for
        # these moduli: 16 and 13 where every modulus lies in [2^34, 2^58) (no conditional
        # subtractions, quotient estimate from three partial products), else 24 and 16
        loose = all((1 << 34) <= q < (1 << 58) for q in moduli)
        ops_bf, ops_pw = (16, 13) if loose else (24, 16)
        int_ops = (N * logN * ops_bf + N * ops_pw) * Tb * L
        server = {
            "kernel": f"rlwe_poly_kernel<{logN}>",
            "encrypt_weight_rows_ms": round(enc_ms, 4),
            "encrypt_polynomials": k * cfg.Ch * L,
            "decrypt_output_rows_ms": round(dec_ms, 4),
            "decrypt_ciphertexts": rows,
            "batch_ciphertexts": Tb,
            "batch_phase_ms": round(big_ms, 4),
            "products_by_secret_per_s": round(Tb * L / (big_ms * 1e-3), 1),
            "bound": "alu",
            "operations_per_butterfly": ops_bf,
            "operations_per_pointwise_product": ops_pw,
            "achieved": round(int_ops / (big_ms * 1e-3) / 1e12, 2),
            "peak": INT32_PEAK_TOPS,
            "unit": "Tint32op/s",
            "frac": round(int_ops / (big_ms * 1e-3) / 1e12 / INT32_PEAK_TOPS, 4),
            "hbm_gbps": round(Tb * L * N * 8 * 3 / (big_ms * 1e-3) / 1e9, 1),
        }
        del ct_big, phi_big, ct_enc, a_dev, e_dev

    # ---- asynchronous weight loading (Section 3.2): a stack of layers whose prepared weights
    # sit in pinned host memory, streamed through two device slots while the previous layer
    # computes; against the same copies and kernels in one stream ----
    prefetch = None
    if not args.no_prefetch:
        layers = 12
        host_w = []
        for i in range(layers):
            hw = torch.empty(prep_bytes, dtype=torch.uint8, pin_memory=True)
            hw.copy_(preps[i % R])
            host_w.append(hw)
        slots = [torch.empty(prep_bytes, dtype=torch.uint8, device="cuda") for _ in range(2)]
        copy_stream = torch.cuda.Stream()
        ld = nc.nimbus_loader_create(2)

        def stack_overlapped():
            nc.nimbus_loader_load(ld, 0, slots[0], host_w[0], copy_stream)
            for i in range(layers):
                if i + 1 < layers:
                    nc.nimbus_loader_load(ld, (i + 1) % 2, slots[(i + 1) % 2], host_w[i + 1],
                                          copy_stream)
                nc.nimbus_loader_acquire(ld, i % 2, stream)
                nc.nimbus_cop_matmul_prepared(Xs[i % R], m, k, xb, slots[i % 2], n, N, L, moduli,
                                              masks[i % R], outs[i % R], ws)
                nc.nimbus_loader_release(ld, i % 2, stream)

        def stack_serial():
            for i in range(layers):
                slots[0].copy_(host_w[i], non_blocking=True)
                nc.nimbus_cop_matmul_prepared(Xs[i % R], m, k, xb, slots[0], n, N, L, moduli,
                                              masks[i % R], outs[i % R], ws)

        def copies_only():
            for i in range(layers):
                slots[i % 2].copy_(host_w[i], non_blocking=True)

        def wall_ms(fn, reps=3):
            fn()
            torch.cuda.synchronize()
            c0 = time.perf_counter()
            for _ in range(reps):
                fn()
            torch.cuda.synchronize()
            return (time.perf_counter() - c0) * 1e3 / reps
        over_ms, serial_ms, copy_ms = wall_ms(stack_overlapped), wall_ms(stack_serial), wall_ms(copies_only)
        nc.nimbus_loader_destroy(ld)
        prefetch = {
            "layers": layers,
            "bytes_per_layer": prep_bytes,
            "stack_ms_overlapped": round(over_ms, 3),
            "stack_ms_one_stream": round(serial_ms, 3),
            "stack_ms_copies_only": round(copy_ms, 3),
            "stack_ms_compute_only": round(layers * ms_per_step, 3),
            "host_to_device_gbps": round(layers * prep_bytes / (copy_ms * 1e-3) / 1e9, 1),
        }
        del host_w, slots

    # ---- calibration: what this chip sustains on the two resources that bound the kernel ----
    # (register-only int8 matrix-core loop with zero and with random operand bytes; streaming
    # read of one prepared weight buffer per launch, rotating over all of them)
    def timed(launch, reps):
        settle(launch)
        a_, b_ = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        a_.record(stream)
        work = 0
        for i in range(reps):
            work += launch(i)
        b_.record(stream)
        torch.cuda.synchronize()
        return work / (a_.elapsed_time(b_) * 1e-3)
    sink = torch.empty(512 * 256, dtype=torch.int32, device="cuda")
    mfma_zero = timed(lambda i: nc.nimbus_calib_mfma_i8(512, 2000, 0, sink), 4) / 1e12
    mfma_rand = timed(lambda i: nc.nimbus_calib_mfma_i8(512, 2000, 1, sink), 4) / 1e12
    read_gbps = timed(lambda i: nc.nimbus_calib_stream_read(preps[i % R], sink), 3 * R) / 1e9
    t_hbm_us = alg_bytes / (read_gbps * 1e9) * 1e6
    t_mfma_us = i8_ops / (mfma_rand * 1e12) * 1e6
    calibration = {
        "int8_mfma_tops_zero_operands": round(mfma_zero, 1),
        "int8_mfma_tops_random_operands": round(mfma_rand, 1),
        "hbm_stream_read_gbps": round(read_gbps, 1),
        "t_hbm_us_at_measured_rate": round(t_hbm_us, 2),
        "t_mfma_us_at_measured_rate": round(t_mfma_us, 2),
        "kernel_frac_of_measured_bound": round(max(t_hbm_us, t_mfma_us) / (kernel_ms_avg * 1e3), 4),
    }

    # the server side's transform kernel against a measured ceiling: the rate of its butterfly
    # in a register-only loop (no LDS, no memory), in the same unit as its derived peak
    if server is not None:
        bsink = torch.empty(2048 * 256, dtype=torch.int64, device="cuda")
        bf_per_s = timed(lambda i: nc.nimbus_calib_butterflies(2048, 1000, moduli[0], bsink), 4)
        ceiling = bf_per_s * ops_bf / 1e12          # same count per butterfly as `achieved`
        server["measured_ceiling"] = round(ceiling, 2)
        server["measured_ceiling_note"] = ("register-only loop of the butterfly the kernel runs for these "
                                           f"moduli, {bf_per_s / 1e12:.3f} T butterflies/s x {ops_bf} operations")
        server["frac_of_measured_ceiling"] = round(server["achieved"] / ceiling, 4)
        del bsink

    # ---- a plain device-to-device copy of known size: reference point for HBM byte counters ----
    # (an elementwise add kernel: reads 256 MiB, writes 256 MiB)
    ca = torch.zeros(64 << 20, dtype=torch.int32, device="cuda")
    cb = torch.empty_like(ca)
    torch.add(ca, 1, out=cb)
    torch.cuda.synchronize()
    del ca, cb

    # ---- oracle: output check of buffer 0 and the CPU baseline (full parity lives in tests/) ----
    cpu_baseline = None
    verified = None
    if not args.no_cpu_baseline:
        from oracle import cop_oracle
        X0, ctW0, mask0 = first
        step(0)
        torch.cuda.synchronize()
        got = outs[0].cpu().numpy().view(np.uint64).reshape(m, cfg.Ch, 2, L, N)
        threads = cop_oracle.max_threads()
        want, used = cop_oracle.cop_ref(X0, ctW0, moduli, n, N, mask0, threads)  # also warms up
        verified = bool(np.array_equal(got, want))
        # bounded sample: whole calls of this workload until about 1.5 s of wall time
        reps, c0 = 0, time.perf_counter()
        while True:
            cop_oracle.cop_ref(X0, ctW0, moduli, n, N, mask0, threads)
            reps += 1
            c1 = time.perf_counter()
            if c1 - c0 >= 1.5 or reps >= 50:
                break
        # one thread, on a slice of the same call (rows 0 .. 7: an eighth of a second or so)
        rows1 = min(m, 8)
        cop_oracle.cop_ref(X0[:rows1], ctW0, moduli, n, N, mask0[:rows1], 1)
        d0 = time.perf_counter()
        cop_oracle.cop_ref(X0[:rows1], ctW0, moduli, n, N, mask0[:rows1], 1)
        d1 = time.perf_counter()
        one_thread = rows1 * k * C / (d1 - d0)
        cpu_baseline = {
            "value": round(reps * cfg.mod_macs / (c1 - c0), 1),
            "unit": "modMAC/s",
            "cores": used,
            "kind": "oracle",
            "sample": f"{reps} full calls of config {args.config} ({cfg.mod_macs} modular MACs "
                      f"each), {c1 - c0:.2f} s wall = {(c1 - c0) * used:.0f} core-seconds on "
                      f"{used} threads",
            "one_thread_value": round(one_thread, 1),
            "one_thread_sample": f"{rows1} rows of the same call ({rows1 * k * C} modular MACs), "
                                 f"{d1 - d0:.2f} s on one thread",
            "build": "gcc -O3 -march=x86-64-v2 -fopenmp (the baseline instruction set every box of "
                     "the pool runs; the oracle is built before the GPU box is known)",
        }

    line = {
        "metric": METRIC,
        "value": round(value, 1),
        "unit": "modMAC/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 5),
        "higher_is_better": True,
        "scaling": "weak",          # one GPU: no scaling run exists (see --gpus)
        "vs_baseline": None,
        "dtype": "u64 residues mod q_l, exact (int8 matrix-core digit products, int32 sums, one reduction per output)",
        "data": "synthetic",
        "config": {
            "workload": f"config {args.config}: {cfg.name} m={m} k={k} n={n} N={N} L={L} "
                        f"t=2^{xb} q~2^{cfg.q_bits}",
            "entry_point": "nimbus_cop_matmul_prepared",
            "weight_buffers_rotated": R,
            "mod_macs_per_step": cfg.mod_macs,
        },
        "ms_per_step_hip_graph": None if graph_ms_per_step is None else round(graph_ms_per_step, 5),
        "two_streams": two_streams,
        "batched": batched,
        "hbm_gbps_whole_step": round(alg_bytes / (ms_per_step * 1e-3) / 1e9, 1),
        "canonical_layout": canonical,
        "paper_setting": paper_setting,
        "roofline": roofline,
        "pack": pack,
        "server": server,
        "prefetch": prefetch,
        "calibration": calibration,
        "cpu_baseline": cpu_baseline,
        "output_matches_oracle": verified,
    }
    print(json.dumps(line))
    return 0


if __name__ == "__main__":
    sys.exit(main())
