#!/usr/bin/env python3
"""Benchmark of one rank's attention under MM-SP on one MI355X.

A "step" is one pass of the whole hot path for one virtual rank of the zigzag ring:
layout/plan (host), N forward ring steps with the LSE merge fused into the kernel epilogue,
the cast of the final O, the delta pre-pass and N backward ring steps -- on synthetic,
seeded inputs already resident in HBM.  Default workload: the 256K-token shard
(28/4 heads, d 128, bf16, N 32, C 4096, T 262144), rank 0.

Prints ONE JSON line: causal-adjusted TFLOP/s (4d flops per visible pair forward, 10d
backward, pairs counted exactly; paper_2408_10188_amd/accounting.py), the roofline entry of
the dominant kernel (timed with HIP events in an instrumented pass), and the fp64 oracle
timed on the host cores on a bounded sample of the same workload.  `value` and `ms_per_step`
come from the wall clock around exactly --steps passes; `pass_ms` gives the median and the
minimum of the same passes, each bracketed by HIP events.
"""
import argparse
import json
import math
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

BF16_DENSE_PEAK_TFLOPS = 2500.0      # MI355X published dense bf16 MFMA peak
HBM_PEAK_GBS = 8000.0


def sample_clock_and_power(seconds, out):
    """Samples rocm-smi (shader clock in MHz, socket power in W) for about `seconds` in a side
    thread while passes run; appends (sclk_mhz, watts) tuples to out.  Best effort: leaves out
    empty if the tool is missing or prints something else."""
    import re
    import subprocess
    end = time.time() + seconds
    while time.time() < end:
        try:
            txt = subprocess.run(["rocm-smi", "--showclocks", "--showpower"], capture_output=True, text=True, timeout=5).stdout
        except Exception:
            return
        m = re.search(r"sclk clock level[^(]*\((\d+)Mhz\)", txt)
        w = re.search(r"Power \(W\):\s*([0-9.]+)", txt)
        if m:
            out.append((int(m.group(1)), float(w.group(1)) if w else None))


def time_passes(one_pass, warmup, steps, torch):
    """`warmup` untimed passes, then exactly `steps` passes between two synchronisations.  Returns
    (wall-clock ms per pass, {"median", "min", "all"} of the per-pass HIP-event times).  The events
    are recorded on the current stream, which every pass joins its side stream back into."""
    for _ in range(warmup):
        one_pass()
    torch.cuda.synchronize()
    ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(steps)]
    t0 = time.perf_counter()
    for e0, e1 in ev:
        e0.record()
        one_pass()
        e1.record()
    torch.cuda.synchronize()
    wall_ms = (time.perf_counter() - t0) / steps * 1e3
    ms = sorted(e0.elapsed_time(e1) for e0, e1 in ev)
    mid = ms[len(ms) // 2] if len(ms) % 2 else 0.5 * (ms[len(ms) // 2 - 1] + ms[len(ms) // 2])
    return wall_ms, {"median": mid, "min": ms[0], "all": ms}


def measured_traffic(config, kernel):
    """HBM bytes per launch of `kernel` from the counters summary under profiles/, or None when
    nothing was measured for this very workload."""
    path = os.path.join(ROOT, "profiles", "hbm_traffic_per_launch.txt")
    try:
        for line in open(path):
            f = line.split()
            if len(f) == 3 and not line.startswith("#") and f[0] == config and f[1] == kernel:
                return int(f[2])
    except Exception:
        pass
    return None


def bench_ulysses(args, cfg, torch, np, B, ring, synth, acc):
    """Head-shard mode: one GPU's 7/1 heads over the whole packed sequence, document-causal mask
    from cu_seqlens, one forward and one backward step."""
    T, Hq, Hkv, d = 2 * cfg["C"], cfg["Hq"], cfg["Hkv"], cfg["d"]
    dev = "cuda:0"
    torch.cuda.set_device(0)
    Cg = 8192

    def gen(name, H, sig):
        out = torch.empty(T, H, d, dtype=torch.bfloat16, device=dev)
        for c in range(T // Cg):
            x = synth.chunk(name, c, Cg, H, d, sig, cfg["seed"])
            out[c * Cg:(c + 1) * Cg] = torch.from_numpy(synth.bf16_bits(x).view(np.int16)).view(torch.bfloat16).to(dev)
        return out

    q, k, v, d_o = gen("q", Hq, cfg["sigma"]), gen("k", Hkv, cfg["sigma"]), gen("v", Hkv, cfg["sigma"]), gen("do", Hq, 1.0)
    cu = synth.packed_cu_seqlens(T, cfg["seed"])
    cud = torch.from_numpy(cu).to(dev)
    n_docs = len(cu) - 1
    shape = ring.shape_for(q, k, B.MMSP_BF16, T, 1.0 / math.sqrt(d))
    o_acc = torch.empty(T, Hq, d, dtype=torch.float32, device=dev)
    lse = torch.empty(Hq, T, dtype=torch.float32, device=dev)
    o_final, delta, dq = torch.empty_like(q), torch.empty_like(lse), torch.zeros_like(o_acc)
    dk = torch.zeros(T, Hkv, d, dtype=torch.float32, device=dev)
    dv = torch.zeros_like(dk)
    ws_bytes = ring.workspace_bytes(shape, T, T)
    ws = torch.empty(ws_bytes, dtype=torch.uint8, device=dev)

    side = None
    if not args.one_stream:      # dQ and dK/dV kernels on two streams (the side lane's accumulators are not used here)
        side = ring.SideLane(torch.cuda.Stream(), None, None, torch.empty_like(ws), ws_bytes)

    def fwd():
        ring.ulysses_forward(shape, T, q, k, v, cud, n_docs, o_acc, lse, o_final, ws=ws, ws_bytes=ws_bytes)

    def bwd():
        dq.zero_()
        ring.ulysses_backward(shape, T, q, k, v, cud, n_docs, o_final, d_o, lse, delta, dq, dk, dv, ws=ws, ws_bytes=ws_bytes,
                              side=side, cu_host=cu, q_block=args.query_block or None)

    def one_pass():
        fwd(); bwd()

    ms_per_step, pass_ms = time_passes(one_pass, args.warmup, args.steps, torch)
    lens = np.diff(cu).astype(np.int64)
    pairs = acc.packed_pairs(lens)
    flops = acc.attention_flops(pairs, d, Hq)
    e = [torch.cuda.Event(enable_timing=True) for _ in range(3)]
    e[0].record(); fwd(); e[1].record(); bwd(); e[2].record()
    torch.cuda.synchronize()
    value = flops / (ms_per_step * 1e-3) / 1e12
    return {
        "metric": "causal attention TFLOP/s fwd+bwd per rank shard; % of MI355X bf16 MFMA peak",
        "value": value, "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step, "pass_ms": pass_ms, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic", "frac_of_bf16_dense_peak": value / BF16_DENSE_PEAK_TFLOPS,
        "config": {"workload": "ulysses: head shard %d/%d heads, d=%d, bf16, T=%d packed from %d documents (%d..%d tokens), "
                               "document-causal mask, fwd+bwd in one step" % (Hq, Hkv, d, T, n_docs, lens.min(), lens.max()),
                   "pairs_per_head": pairs, "tflop_fwd": acc.attention_flops(pairs, d, Hq, True, False) / 1e12,
                   "tflop_bwd": acc.attention_flops(pairs, d, Hq, False, True) / 1e12},
        "roofline": {"kernel": "fwd+bwd (all kernels of the step)", "bound": "mfma", "achieved": value,
                     "peak": BF16_DENSE_PEAK_TFLOPS, "unit": "TFLOP/s", "frac": value / BF16_DENSE_PEAK_TFLOPS,
                     "traffic": measured_traffic("ulysses", "fwd+bwd")},
        "cpu_baseline": None,
        "breakdown": {"fwd_ms": e[0].elapsed_time(e[1]), "bwd_ms": e[1].elapsed_time(e[2])},
    }


def bench_data_movement(args, torch, B):
    """Row permutations around the attention path, bf16, T = 262144, 28 heads, d = 128."""
    T, N, H, d, U = 262144, 32, 28, 128, 4
    dev = "cuda:0"
    x = torch.randn(T, H, d, device=dev).bfloat16()
    shards = torch.empty(N, T // N, H, d, dtype=torch.bfloat16, device=dev)
    back = torch.empty_like(x)
    n_tok = T // U                                     # tokens per GPU of the all-to-all group
    xs = x[:n_tok]
    packed = torch.empty(U, n_tok, H // U, d, dtype=torch.bfloat16, device=dev)
    unp = torch.empty_like(xs)
    row_bytes, slice_bytes = H * d * 2, (H // U) * d * 2
    ops = {"zigzag_gather": (lambda: B.mmsp_zigzag_gather(T, N, row_bytes, x, shards), 2 * x.numel() * 2),
           "zigzag_scatter": (lambda: B.mmsp_zigzag_scatter(T, N, row_bytes, shards, back), 2 * x.numel() * 2),
           "a2a_pack_heads": (lambda: B.mmsp_a2a_pack_heads(n_tok, U, slice_bytes, xs, packed), 2 * xs.numel() * 2),
           "a2a_unpack_heads": (lambda: B.mmsp_a2a_unpack_heads(n_tok, U, slice_bytes, packed, unp), 2 * xs.numel() * 2)}
    out = {}
    for name, (fn, nbytes) in ops.items():
        for _ in range(3):
            fn()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(10):
            fn()
        e1.record(); torch.cuda.synchronize()
        ms = e0.elapsed_time(e1) / 10
        out[name] = {"ms": ms, "alg_bytes": nbytes, "gbs": nbytes / (ms * 1e-3) / 1e9, "frac_of_hbm_peak": nbytes / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS}
    assert torch.equal(back, x) and torch.equal(unp, xs)
    worst = min(out, key=lambda k: out[k]["gbs"])
    return {"metric": "HBM GB/s of the sharding kernels (read + written bytes / time)", "value": out[worst]["gbs"], "unit": "GB/s",
            "n_gpus": 1, "higher_is_better": True, "dtype": "bf16", "data": "synthetic",
            "config": {"workload": "T=262144 x 28 heads x d=128 bf16: zigzag gather/scatter over N=32; head packing for U=4 on T/4 tokens"},
            "roofline": {"kernel": worst, "bound": "hbm", "achieved": out[worst]["gbs"], "peak": HBM_PEAK_GBS, "unit": "GB/s",
                         "frac": out[worst]["gbs"] / HBM_PEAK_GBS, "traffic": None},
            "ops": out}


def bench_packed(args, cfg, torch, np, B, ring, synth, env):
    """One zigzag rank over a packed sequence: document-causal mask on global positions."""
    N, C, Hq, Hkv, d, T, rank = (env[k] for k in ("N", "C", "Hq", "Hkv", "d", "T", "rank"))
    q, d_o, k_zz, v_zz, shape, ws, ws_bytes = (env[k] for k in ("q", "d_o", "k_zz", "v_zz", "shape", "ws", "ws_bytes"))
    o_acc, lse, o_final, delta, dq, dk_zz, dv_zz = (env[k] for k in ("o_acc", "lse", "o_final", "delta", "dq", "dk_zz", "dv_zz"))
    cu = synth.packed_cu_seqlens(T, cfg["seed"])
    cud = torch.from_numpy(cu).to("cuda:0")
    n_docs = len(cu) - 1

    def one_pass():
        ring.rank_forward_packed(shape, T, N, rank, q, k_zz, v_zz, cud, n_docs, o_acc, lse, o_final, ws=ws, ws_bytes=ws_bytes,
                                 cu_host=cu)
        dq.zero_()
        ring.rank_backward_packed(shape, T, N, rank, q, k_zz, v_zz, cud, n_docs, o_final, d_o, lse, delta, dq, dk_zz, dv_zz,
                                  ws=ws, ws_bytes=ws_bytes, cu_host=cu)

    ms_per_step, pass_ms = time_passes(one_pass, args.warmup, args.steps, torch)
    # visible pairs of this rank's rows: position - start of its document + 1
    pos = np.concatenate([np.arange(c * C, (c + 1) * C, dtype=np.int64) for c in (rank, 2 * N - 1 - rank)])
    start = cu[np.searchsorted(cu, pos, side="right") - 1].astype(np.int64)
    pairs = int((pos - start + 1).sum())
    all_pos = np.arange(T, dtype=np.int64)
    total = int((all_pos - cu[np.searchsorted(cu, all_pos, side="right") - 1] + 1).sum())
    value = env["acc"].attention_flops(pairs, d, Hq) / (ms_per_step * 1e-3) / 1e12
    return {
        "metric": "causal attention TFLOP/s fwd+bwd per rank shard; % of MI355X bf16 MFMA peak",
        "value": value, "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step, "pass_ms": pass_ms, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic", "frac_of_bf16_dense_peak": value / BF16_DENSE_PEAK_TFLOPS,
        "config": {"workload": "%s packed: zigzag rank %d of N=%d, C=%d (T=%d) over %d packed documents, %d/%d heads, d=%d, "
                               "bf16, fwd+bwd, document-causal mask" % (args.config, rank, N, C, T, n_docs, Hq, Hkv, d),
                   "streams": 1, "pairs_per_head": pairs, "share_of_all_pairs": pairs / total, "balanced_share": 1.0 / N},
        "roofline": {"kernel": "fwd+bwd (all kernels of the pass)", "bound": "mfma", "achieved": value,
                     "peak": BF16_DENSE_PEAK_TFLOPS, "unit": "TFLOP/s", "frac": value / BF16_DENSE_PEAK_TFLOPS, "traffic": None},
        "cpu_baseline": None,
    }


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=5)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--config", default="long", choices=["cfg2", "cfg3", "long", "ulysses", "2d"],
                    help="long (default, the headline workload) and cfg3: one zigzag rank, fwd+bwd; cfg2: N=4, C=2048, all "
                         "four ranks one after the other, forward only (the case that is sensitive to launch overhead); "
                         "ulysses: head-shard mode, 7/1 heads over the whole packed 256K sequence, fwd+bwd in one step; "
                         "2d: one GPU of a 2D-attention mesh (head degree 4 x ring degree 8): 7/1 heads, zigzag "
                         "N=8 with 16384-token chunks of the same 256K sequence")
    ap.add_argument("--rank", type=int, default=0)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-clock-sample", action="store_true", help="skip the 2 s of extra passes during which rocm-smi is polled")
    ap.add_argument("--layout", default="zigzag", choices=["zigzag", "contiguous"],
                    help="zigzag workloads: contiguous = the plain ring layout (rank r holds tokens [r T/N, (r+1) T/N)), whose "
                         "work grows with the rank, for comparison with the balanced both-ends layout")
    ap.add_argument("--fwd-only", action="store_true",
                    help="zigzag workloads: time the forward ring steps only (the long-prefill compute of the inference mode)")
    ap.add_argument("--packed", action="store_true",
                    help="zigzag workloads: the sequence is packed from documents (synth.packed_cu_seqlens) and the ring "
                         "steps run the sub-blocks of mmsp_zigzag_plan_packed under the document-causal mask, one stream")
    ap.add_argument("--one-stream", action="store_true", help="all launches on one stream (no overlap of ring steps)")
    ap.add_argument("--graph", action="store_true",
                    help="forward-only zigzag workloads: capture one pass in a HIP graph and time its replays (the launches "
                         "of a short pass then cost one submission); every replay is checked against the eager result")
    ap.add_argument("--query-block", type=int, default=0,
                    help="ulysses: cut the backward into launches over query blocks of this many rows (default 0: one launch "
                         "per kernel over the whole sequence, whose workgroups drift apart and re-read Q / dO from HBM)")
    ap.add_argument("--cpu-rows", type=int, default=32, help="query rows per chunk in the oracle sample")
    ap.add_argument("--data-movement", action="store_true",
                    help="only time the HBM-bound sharding kernels at the 256K-token shapes (zigzag gather / scatter of Q, "
                         "head packing around the all-to-all) and print one JSON line with their GB/s")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py measures one GPU's share of the ring (one rank); this build has no multi-GPU path: "
              "run with --gpus 1", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    from paper_2408_10188_amd import accounting as acc
    from paper_2408_10188_amd import binding as B
    from paper_2408_10188_amd import ring, synth

    if args.data_movement:
        print(json.dumps(bench_data_movement(args, torch, B)))
        return

    cfg = synth.CONFIGS[args.config]
    if args.config == "ulysses":
        print(json.dumps(bench_ulysses(args, cfg, torch, np, B, ring, synth, acc)))
        return
    N, C, Hq, Hkv, d = cfg["N"], cfg["C"], cfg["Hq"], cfg["Hkv"], cfg["d"]
    T, n = 2 * N * C, 2 * C
    all_ranks = args.config == "cfg2"
    if all_ranks:
        args.fwd_only = True
    if args.graph and not args.fwd_only:
        sys.exit("--graph is for forward-only passes (--fwd-only, or --config cfg2)")
    ranks = list(range(N)) if all_ranks else [args.rank]
    rank = ranks[0]
    dev = "cuda:0"
    torch.cuda.set_device(0)

    def upload(x):
        return torch.from_numpy(synth.bf16_bits(x).view(np.int16)).view(torch.bfloat16).to(dev)

    # ---- synthetic inputs, chunk by chunk (the full K/V never sit on the host in fp32 at once)
    k_zz = torch.empty(N, n, Hkv, d, dtype=torch.bfloat16, device=dev)
    v_zz = torch.empty_like(k_zz)
    contiguous = args.layout == "contiguous"
    chunks_of = (lambda r: (2 * r, 2 * r + 1)) if contiguous else (lambda r: (r, 2 * N - 1 - r))
    plan = B.mmsp_contiguous_plan if contiguous else B.mmsp_zigzag_plan
    for r in range(N):
        for half, c in enumerate(chunks_of(r)):
            k_zz[r, half * C:(half + 1) * C] = upload(synth.chunk("k", c, C, Hkv, d, cfg["sigma"], cfg["seed"]))
            v_zz[r, half * C:(half + 1) * C] = upload(synth.chunk("v", c, C, Hkv, d, cfg["sigma"], cfg["seed"]))
    q_host, do_host, qs, d_os, o_accs, lses, o_finals = {}, {}, {}, {}, {}, {}, {}
    for r in ranks:
        q_host[r] = np.concatenate([synth.chunk("q", c, C, Hq, d, cfg["sigma"], cfg["seed"]) for c in chunks_of(r)])
        qs[r] = upload(q_host[r])
        o_accs[r] = torch.empty(n, Hq, d, dtype=torch.float32, device=dev)
        lses[r] = torch.empty(Hq, n, dtype=torch.float32, device=dev)
        o_finals[r] = torch.empty_like(qs[r])
        if not args.fwd_only:
            do_host[r] = np.concatenate([synth.chunk("do", c, C, Hq, d, 1.0, cfg["seed"]) for c in chunks_of(r)])
            d_os[r] = upload(do_host[r])
    q, o_acc, lse, o_final = qs[rank], o_accs[rank], lses[rank], o_finals[rank]
    d_o = d_os.get(rank)

    shape = ring.shape_for(q, k_zz, B.MMSP_BF16, n, 1.0 / math.sqrt(d))
    delta = torch.empty_like(lse)
    dq = torch.zeros_like(o_acc)
    dk_zz = torch.zeros(N, n, Hkv, d, dtype=torch.float32, device=dev)   # rows this rank never reaches stay 0
    dv_zz = torch.zeros_like(dk_zz)

    ws_bytes = ring.workspace_bytes(shape, n, n)
    ws = torch.empty(max(ws_bytes, 16), dtype=torch.uint8, device=dev)

    # second launch lane (HIP stream, (O, LSE) accumulator, workspace): consecutive ring steps
    # overlap so that the partly filled last round of one launch does not leave CUs idle
    side = None
    if not args.one_stream:
        side = ring.SideLane(torch.cuda.Stream(), torch.empty_like(o_acc), torch.empty_like(lse),
                             torch.empty_like(ws), ws_bytes)

    def eager_pass():
        for r in ranks:
            ring.rank_forward(shape, T, N, r, qs[r], k_zz, v_zz, o_accs[r], lses[r], o_finals[r], ws=ws, ws_bytes=ws_bytes,
                              side=side, plan=plan, stream=torch.cuda.current_stream().cuda_stream)
        if args.fwd_only:
            return
        dq.zero_()
        ring.rank_backward(shape, T, N, rank, q, k_zz, v_zz, o_final, d_o, lse, delta, dq, dk_zz, dv_zz, ws=ws,
                           ws_bytes=ws_bytes, side=side, plan=plan)

    if args.packed:
        acc_mod = acc
        env = dict(locals(), acc=acc_mod)
        print(json.dumps(bench_packed(args, cfg, torch, np, B, ring, synth, env)))
        return

    one_pass = eager_pass
    graph_note = None
    if args.graph:
        eager_pass()
        torch.cuda.synchronize()
        want = [o_finals[r].clone() for r in ranks]
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            eager_pass()
        for i in range(3):                      # replays with eager work in between, each checked
            for r in ranks:
                o_finals[r].zero_()
            graph.replay()
            torch.cuda.synchronize()
            if not all(torch.equal(o_finals[r], w) for r, w in zip(ranks, want)):
                sys.exit("replay %d of the captured pass differs from the eager result" % i)
            eager_pass()
        one_pass = graph.replay
        graph_note = "one HIP graph per pass; 3 replays checked bit for bit against the eager pass"

    ms_per_step, pass_ms = time_passes(one_pass, args.warmup, args.steps, torch)

    # shader clock and socket power under this load: a couple of seconds of extra passes with rocm-smi polled beside them
    clock_samples = []
    if not args.no_clock_sample:
        import threading
        th = threading.Thread(target=sample_clock_and_power, args=(2.0, clock_samples))
        th.start()
        t_end = time.time() + 2.2
        while time.time() < t_end:
            one_pass()
            torch.cuda.synchronize()
        th.join()

    pairs = sum(acc.contiguous_pairs_of_rank(N, C, r) if contiguous else acc.zigzag_pairs_of_rank(N, C) for r in ranks)
    flops_fwd = acc.attention_flops(pairs, d, Hq, True, False)
    flops_bwd = 0 if args.fwd_only else acc.attention_flops(pairs, d, Hq, False, True)
    value = (flops_fwd + flops_bwd) / (ms_per_step * 1e-3) / 1e12
    # launches of one pass: per rank the N step kernels, the final merge + cast and, with two lanes, the
    # fill of the side accumulator; the backward adds delta and per step the statistics, dK/dV (+ the
    # reduction of cut key tiles) and dQ kernels
    launches = len(ranks) * (N + 1 + (1 if side is not None and N > 1 else 0))

    # ---- instrumented pass: HIP events around each kind of call (same stream the kernels run on)
    def timed(fn):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record(); fn(); e1.record()
        return e0, e1

    plans = [plan(T, N, rank, s) for s in range(N)]
    kinds = {"fwd_step": [], "merge_cast": []}
    if not args.fwd_only:
        kinds.update({"delta": [], "bwd_dq": [], "bwd_dkdv": []})
    torch.cuda.synchronize()
    for _ in range(2):
        for s, (src, blk) in enumerate(plans):
            kinds["fwd_step"].append((timed(lambda: B.mmsp_attn_step_fwd(shape, blk, q, k_zz[src], v_zz[src], o_acc, lse, s > 0, ws, ws_bytes)), blk))
        kinds["merge_cast"].append((timed(lambda: B.mmsp_attn_merge(shape, 0, n, o_acc, lse, None, None, o_final)), None))
        if args.fwd_only:
            continue
        kinds["delta"].append((timed(lambda: B.mmsp_attn_delta(shape, 0, n, o_final, d_o, delta)), None))
        dq.zero_()
        for src, blk in plans:
            kinds["bwd_dq"].append((timed(lambda: B.mmsp_attn_step_bwd(shape, blk, q, k_zz[src], v_zz[src], None, d_o, lse, delta, 0, dq, None, None, 0, ws, ws_bytes)), blk))
            kinds["bwd_dkdv"].append((timed(lambda: B.mmsp_attn_step_bwd(shape, blk, q, k_zz[src], v_zz[src], None, d_o, lse, delta, 0, None, dk_zz[src], dv_zz[src], 0, ws, ws_bytes)), blk))
    torch.cuda.synchronize()

    def blk_pairs(blk):
        if blk.mask == B.MMSP_MASK_NONE:
            return 0
        if blk.mask == B.MMSP_MASK_CAUSAL_DIAG:
            return blk.n_q * (blk.n_q + 1) // 2
        return blk.n_q * blk.n_k

    # algorithmic flops per visible pair and head of each kernel: forward S and PV (4d); the dK/dV
    # kernel owns S, dP, dV, dK (8d); the dQ kernel owns dQ (2d) -- its S/dP recompute earns nothing
    per_pair = {"fwd_step": 4 * d, "bwd_dq": 2 * d, "bwd_dkdv": 8 * d}
    breakdown = {}
    for name, lst in kinds.items():
        ms = [e0.elapsed_time(e1) for (e0, e1), _ in lst]
        entry = {"calls_per_pass": len(lst) // 2, "avg_ms": sum(ms) / len(ms), "total_ms_per_pass": sum(ms) / 2}
        if name in per_pair:
            fl = sum(per_pair[name] * Hq * blk_pairs(b) for _, b in lst) / len(lst)
            entry["alg_tflops_per_launch"] = fl / 1e12
            entry["tflops"] = fl / (entry["avg_ms"] * 1e-3) / 1e12
        else:
            elt = 2  # bf16 O / dO
            byts = n * Hq * (d * (4 + elt) + 4) if name == "merge_cast" else n * Hq * (2 * d * elt + 4)
            entry["alg_bytes_per_launch"] = byts
            entry["gbs"] = byts / (entry["avg_ms"] * 1e-3) / 1e9
        breakdown[name] = entry
    dominant = max((k for k in per_pair if k in breakdown), key=lambda k: breakdown[k]["total_ms_per_pass"])
    plain = args.layout == "zigzag" and rank == 0          # the workload the counters under profiles/ were taken on
    roofline = {"kernel": dominant, "bound": "mfma", "achieved": breakdown[dominant]["tflops"],
                "peak": BF16_DENSE_PEAK_TFLOPS, "unit": "TFLOP/s",
                "frac": breakdown[dominant]["tflops"] / BF16_DENSE_PEAK_TFLOPS,
                "traffic": measured_traffic(args.config, dominant) if plain else None,
                "avg_launch_ms": breakdown[dominant]["avg_ms"],
                "whole_pass_frac": value / BF16_DENSE_PEAK_TFLOPS}

    # ---- the oracle on the host cores, on a bounded sample of the same workload (first rank of the pass)
    cpu = None
    if not args.no_cpu_baseline:
        from oracle import mmsp_oracle as orc
        rows = np.concatenate([np.linspace(0, C - 1, args.cpu_rows).astype(np.int64),
                               C + np.linspace(0, C - 1, args.cpu_rows).astype(np.int64)])
        l2g = np.arange(rank * n, (rank + 1) * n, dtype=np.int64) if contiguous else orc.zigzag_layout(T, N, rank)[1]
        K = np.empty((T, Hkv, d)); V = np.empty((T, Hkv, d))
        for c in range(2 * N):
            K[c * C:(c + 1) * C] = synth.chunk("k", c, C, Hkv, d, cfg["sigma"], cfg["seed"])
            V[c * C:(c + 1) * C] = synth.chunk("v", c, C, Hkv, d, cfg["sigma"], cfg["seed"])
        tc = time.perf_counter()
        ref = orc.causal_attention(q_host[rank][rows].astype(np.float64), K, V, 1.0 / math.sqrt(d), q_pos=l2g[rows],
                                   dO=None if args.fwd_only else do_host[rank][rows].astype(np.float64))
        cpu_s = time.perf_counter() - tc
        sample_pairs = int((l2g[rows] + 1).sum())
        cpu_flops = acc.attention_flops(sample_pairs, d, Hq, True, not args.fwd_only)
        idx = torch.from_numpy(rows).to(dev)
        errs = {"o": np.abs(o_acc[idx].double().cpu().numpy() - ref[0])}
        if not args.fwd_only:
            errs["dq"] = np.abs(dq[idx].double().cpu().numpy() - ref[2])
        errs = {k: (float(v.max()) if np.isfinite(v).all() else float("inf")) for k, v in errs.items()}
        if max(errs.values()) > 2e-2:             # a NaN or an infinity counts as a miss
            sys.exit("the timed buffers disagree with the oracle on the sampled rows: %r" % errs)
        cpu = {"value": cpu_flops / cpu_s / 1e12, "unit": "TFLOP/s", "cores": len(os.sched_getaffinity(0)),
               "kind": "oracle", "seconds": cpu_s,
               "sample": "%d query rows (%d per chunk, evenly spaced) of rank %d x all %d heads, %s, fp64 numpy; "
                         "%.3e of the pass's pairs"
                         % (len(rows), args.cpu_rows, rank, Hq,
                            "forward" if args.fwd_only else "fwd+bwd (dQ rows; dK/dV contribution of those rows)",
                            sample_pairs / pairs),
               "gpu_vs_oracle_max_abs": errs}

    who = "ranks 0..%d one after the other" % (N - 1) if all_ranks else "rank %d" % rank
    out = {
        "metric": "causal attention TFLOP/s fwd+bwd per rank shard; % of MI355X bf16 MFMA peak",
        "value": value, "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step, "pass_ms": pass_ms, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "frac_of_bf16_dense_peak": value / BF16_DENSE_PEAK_TFLOPS,
        "config": {"workload": "%s: %s %s of N=%d, C=%d (T=%d), %d/%d heads, d=%d, bf16, %s over all %d "
                               "ring steps" % (args.config, args.layout, who, N, C, T, Hq, Hkv, d,
                                               "forward only" if args.fwd_only else "fwd+bwd", N),
                   "streams": 1 if side is None else 2, "graph": graph_note,
                   "pairs_per_head": pairs, "tflop_fwd": flops_fwd / 1e12, "tflop_bwd": flops_bwd / 1e12},
        "roofline": roofline, "cpu_baseline": cpu, "breakdown": breakdown,
        "clock_under_load": None if not clock_samples else {
            "sclk_mhz_min_mean_max": [min(c for c, _ in clock_samples), sum(c for c, _ in clock_samples) / len(clock_samples),
                                      max(c for c, _ in clock_samples)],
            "socket_power_w_mean": (sum(w for _, w in clock_samples if w) / max(1, sum(1 for _, w in clock_samples if w))) or None,
            "samples": len(clock_samples),
            "note": "rocm-smi polled while extra passes of the same workload run after the timed region"},
    }
    if args.fwd_only:
        out["launches_per_pass"] = launches
        out["us_per_launch"] = pass_ms["median"] * 1e3 / launches
    print(json.dumps(out))


if __name__ == "__main__":
    main()
