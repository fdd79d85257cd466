#!/usr/bin/env python3
"""Benchmark of the CaliDrop hot path on one MI355X.

One step = one pass of the whole hot path over one batch of synthetic input: calidrop_compress
of a 32-layer Llama-3-8B-shaped stack at 32k context (budget 512, window 32, pooling 7; the
layers are independent tensors passed as batch entries), followed by T = 256 calibrated decode
steps (one calidrop_decode call per step over the whole stack).  Inputs are resident in HBM
before the timed region.  Prints ONE JSON line.

  value                    decode attention GB/s: algorithmic bytes of one decode call divided by
                           its mean duration (HIP events on the launch stream), with the decode
                           calls cycling over `--rotate` copies of the compressed cache so that the
                           working set exceeds the 256 MB Infinity Cache (HBM-honest).
  compress_us_per_layer    mean calidrop_compress time / layers.
  roofline                 the dominant kernel (the decode streaming-attention kernel).
  cpu_baseline             the fp64 numpy oracle timed on a bounded sample of the same workload.
"""
from __future__ import annotations

import argparse
import json
import os
import statistics
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0          # MI355X HBM3E, published
# HBM bytes per decode launch measured with rocprofv3 counters on the default workload
# (profiles/bench_cfg3_B512_pmc_hbm_bytes.md): FETCH_SIZE 33597.4 KiB x 2.0 + WRITE_SIZE 272 KiB x 1.0
DECODE_TRAFFIC_BYTES_PMC = 69085933


def decode_bytes(wl, cache_len: int) -> int:
    """Algorithmic bytes of one decode call: K_c and V_c rows once, plus query, calibration
    state and output."""
    E = 2 if wl.dtype == "bf16" else 4
    kv = 2 * wl.batch * wl.n_kv_heads * cache_len * wl.head_dim * E
    small = wl.batch * wl.n_q_heads * (wl.head_dim * E + (2 * wl.head_dim + 1) * 4 + wl.head_dim * E)
    return kv + small


def compress_bytes(wl) -> int:
    """Lower bound for compress: K and V read once."""
    E = 2 if wl.dtype == "bf16" else 4
    return 2 * sum(wl.seq_lens) * wl.n_kv_heads * wl.head_dim * E


def cpu_baseline(wl, x, layers: int, decode_steps: int):
    """Time the oracle (as it stands) on the first `layers` layers of the stack: compress of
    each, then `decode_steps` decode steps over all of them.  Scaled to the metric's units."""
    import numpy as np
    import torch
    from oracle import calidrop_ref as ref
    from paper_2507_19906_amd import synth
    to64 = lambda t: t.detach().to("cpu").to(torch.float64).numpy()
    layers = min(layers, wl.batch)
    t_comp = 0.0
    state = []
    for b in range(layers):
        K = to64(synth.seq_view(x["k"], wl, b))
        V = to64(synth.seq_view(x["v"], wl, b))
        qw = to64(x["q_win"][b])
        t0 = time.perf_counter()
        r = ref.compress(qw, K, V, wl.window, wl.budget, wl.pool_kernel)
        t_comp += time.perf_counter() - t0
        state.append({k: r[k] for k in ("K_c", "V_c", "c_q", "c_out", "c_lse")})
        del K, V, r
    qd = to64(x["q_dec"][:decode_steps, :layers])
    t0 = time.perf_counter()
    for t in range(decode_steps):
        for b in range(layers):
            st = state[b]
            ref.decode(qd[t, b], st["K_c"], st["V_c"], wl.budget, st["c_q"], st["c_out"], st["c_lse"], wl.theta1, wl.theta2)
    t_dec = (time.perf_counter() - t0) / decode_steps
    E = 2
    dec_bytes = 2 * layers * wl.n_kv_heads * wl.budget * wl.head_dim * E      # same accounting as the GPU side
    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
    except Exception:
        cores = os.cpu_count() or 1
    return {
        "value": dec_bytes / t_dec / 1e9, "unit": "GB/s", "cores": int(cores), "kind": "oracle",
        "sample": f"the first {layers} of {wl.batch} layers: compress of each ({t_comp:.2f} s in total) and "
                  f"{decode_steps} decode steps over those layers ({t_dec * 1e3:.3f} ms per step); fp64 numpy; "
                  f"{t_comp + t_dec * decode_steps:.1f} s of oracle time",
        "compress_us_per_layer": t_comp * 1e6 / layers,
    }


def machine_probes(dev, stream):
    """What a plain streaming read and a dense bf16 matrix-core loop reach on this GPU (the probes of
    libcalidrop_probes.so), for reading the roofline fractions against measured ceilings."""
    import ctypes
    import torch
    import paper_2507_19906_amd
    path = os.path.join(os.path.dirname(os.path.abspath(paper_2507_19906_amd.__file__)), "libcalidrop_probes.so")
    L = ctypes.CDLL(path)
    L.calidrop_probe_stream_read.argtypes = [ctypes.c_void_p, ctypes.c_uint64, ctypes.c_int32, ctypes.c_void_p, ctypes.c_void_p]
    L.calidrop_probe_stream_read_nt.argtypes = L.calidrop_probe_stream_read.argtypes
    L.calidrop_probe_mfma_loop.argtypes = [ctypes.c_void_p, ctypes.c_int32, ctypes.c_int32, ctypes.c_void_p]
    st = stream.cuda_stream or None
    buf = torch.ones(2 << 30, dtype=torch.uint8, device=dev)
    out = torch.zeros(1 << 21, dtype=torch.float32, device=dev)
    ev = lambda: torch.cuda.Event(enable_timing=True)
    res = {}
    for label, nbytes, blocks, reps in (("64MiB", 64 << 20, 2048, 32), ("256MiB", 256 << 20, 8192, 16), ("2GiB", 2 << 30, 32768, 6)):
        nrot = (2 << 30) // nbytes                 # rotate through the buffer: never re-read cached data
        for kind, fn in (("", L.calidrop_probe_stream_read), ("_nontemporal", L.calidrop_probe_stream_read_nt)):
            def launch(r):
                rc = fn(buf.data_ptr() + (r % nrot) * nbytes, nbytes, blocks, out.data_ptr(), st)
                assert rc == 0
            for r in range(3):
                launch(r)
            e0, e1 = ev(), ev()
            e0.record(stream)
            for r in range(reps):
                launch(r + 3)
            e1.record(stream)
            torch.cuda.synchronize()
            us = e0.elapsed_time(e1) * 1e3 / reps
            res["stream_read" + kind + "_" + label] = {"us_per_launch": us, "GBps": nbytes / us / 1e3}
    blocks, iters = 2048, 20000
    for _ in range(2):
        assert L.calidrop_probe_mfma_loop(out.data_ptr(), blocks, 2000, st) == 0
    e0, e1 = ev(), ev()
    e0.record(stream)
    assert L.calidrop_probe_mfma_loop(out.data_ptr(), blocks, iters, st) == 0
    e1.record(stream)
    torch.cuda.synchronize()
    flop = blocks * 4 * iters * 8 * 16384.0
    ms = e0.elapsed_time(e1)
    res["mfma_bf16_loop"] = {"ms": ms, "TFLOPps": flop / ms / 1e9, "pct_published_peak": 100.0 * flop / ms / 1e9 / 2500.0}
    del buf, out
    return res


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--layers", type=int, default=32)
    ap.add_argument("--budget", type=int, default=512)
    ap.add_argument("--decode-steps", type=int, default=256)
    ap.add_argument("--rotate", type=int, default=0, help="cache copies cycled by decode (0 = enough for 512 MiB)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--offset-array", action="store_true",
                    help="pass cache_offsets to calidrop_decode (default: NULL = uniform capacity)")
    ap.add_argument("--no-extra", action="store_true", help="skip the additional budget-2048 decode measurement")
    ap.add_argument("--copy-probe", action="store_true",
                    help="also run a plain 1 GiB device copy 4 times (calibrates the profiler's HBM byte counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only; --gpus must be 1 (no multi-GPU path exists)",
              file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2507_19906_amd import binding as cd
    from paper_2507_19906_amd import synth

    from paper_2507_19906_amd import build as _build
    if not (os.path.exists(cd.LIB_PATH) and os.path.exists(_build.PROBES_PATH)):
        _build.build()
    assert torch.cuda.is_available(), "bench.py needs the GPU (there is no CPU path)"
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)

    if args.copy_probe:     # known traffic: 1 GiB read + 1 GiB written per launch
        src = torch.empty(1 << 30, dtype=torch.uint8, device=dev).random_(0, 255)
        dst = torch.empty_like(src)
        for _ in range(4):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    wl = synth.config(3, layers=args.layers, budget=args.budget, decode_steps=args.decode_steps)
    x = synth.make_inputs(wl, device=dev)
    p = cd.make_params(dtype=wl.dtype, batch=wl.batch, n_q_heads=wl.n_q_heads, n_kv_heads=wl.n_kv_heads,
                       head_dim=wl.head_dim, window=wl.window, budget=wl.budget, pool_kernel=wl.pool_kernel,
                       theta1=wl.theta1, theta2=wl.theta2)
    bufs = cd.CompressBuffers(p, wl.seq_lens, dev)
    dbytes = decode_bytes(wl, wl.budget)
    rotate = args.rotate or max(1, -(-(512 << 20) // dbytes))
    # extra copies of the compressed cache (same contents, different addresses)
    k_copies = [bufs.k_c] + [torch.empty_like(bufs.k_c) for _ in range(rotate - 1)]
    v_copies = [bufs.v_c] + [torch.empty_like(bufs.v_c) for _ in range(rotate - 1)]
    T = wl.decode_steps
    stream = torch.cuda.current_stream()

    # the compressed cache here has one capacity for every layer: cache_offsets is left out unless
    # --offset-array asks for the general (variable-capacity) form of the call
    offs = bufs.cache_offsets if args.offset_array else None

    def decode_call(t, kc, vc):
        cd.calidrop_decode(p, x["q_dec"][t], kc, vc, offs, bufs.cache_lens, bufs.max_cache_len,
                           bufs.c_q, bufs.c_out, bufs.c_lse, bufs.out, bufs.a_lse, bufs.flags, bufs.ws_decode,
                           stream)

    ev = lambda: torch.cuda.Event(enable_timing=True)
    comp_ms, dec_ms = [], []

    def one_step(record: bool):
        e0, e1, e2 = ev(), ev(), ev()
        e0.record(stream)
        bufs.compress(x["q_win"], x["k"], x["v"], x["seq_offsets"], stream=stream)
        e1.record(stream)
        for t in range(T):
            decode_call(t, k_copies[t % rotate], v_copies[t % rotate])
        e2.record(stream)
        if record:
            return (e0, e1, e2)

    for _ in range(args.warmup):
        one_step(False)
        for i in range(1, rotate):                    # fill the copies once compress has run
            k_copies[i].copy_(bufs.k_c); v_copies[i].copy_(bufs.v_c)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    evs = [one_step(True) for _ in range(args.steps)]
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    for e0, e1, e2 in evs:
        comp_ms.append(e0.elapsed_time(e1))
        dec_ms.append(e1.elapsed_time(e2) / T)
    comp = sum(comp_ms) / len(comp_ms)
    dec = sum(dec_ms) / len(dec_ms)

    # cache-resident variant (single copy: 64 MiB per call stays in the Infinity Cache)
    e0, e1 = ev(), ev()
    e0.record(stream)
    for t in range(T):
        decode_call(t, bufs.k_c, bufs.v_c)
    e1.record(stream)
    torch.cuda.synchronize()
    dec_res = e0.elapsed_time(e1) / T

    # config 3's other budgets, each a run of its own: compress of the stack, then decode calls that
    # cycle over enough address-distinct copies of the compressed cache to exceed the Infinity Cache
    # (budget 128: 16 MiB per call, the launch is mostly fixed latency; budget 2048: 256 MiB per call,
    # enough bytes for the fixed in-kernel latency to stop dominating)
    other = {}
    if args.budget == 512 and args.layers == 32 and not args.no_extra:
        for bud in (128, 2048):
            wl2 = synth.config(3, layers=args.layers, budget=bud, decode_steps=1)
            p2 = cd.make_params(dtype=wl2.dtype, batch=wl2.batch, n_q_heads=wl2.n_q_heads, n_kv_heads=wl2.n_kv_heads,
                                head_dim=wl2.head_dim, window=wl2.window, budget=wl2.budget, pool_kernel=wl2.pool_kernel,
                                theta1=wl2.theta1, theta2=wl2.theta2)
            b2 = cd.CompressBuffers(p2, wl2.seq_lens, dev)
            cms = []
            for it in range(5):
                e0, e1 = ev(), ev()
                e0.record(stream)
                b2.compress(x["q_win"], x["k"], x["v"], x["seq_offsets"], stream=stream)
                e1.record(stream)
                torch.cuda.synchronize()
                if it >= 2:
                    cms.append(e0.elapsed_time(e1))
            nbytes = decode_bytes(wl2, bud)
            ncopy = max(3, -(-(512 << 20) // nbytes))
            kc2 = [b2.k_c] + [b2.k_c.clone() for _ in range(ncopy - 1)]
            vc2 = [b2.v_c] + [b2.v_c.clone() for _ in range(ncopy - 1)]
            offs2 = b2.cache_offsets if args.offset_array else None

            def call2(t):
                cd.calidrop_decode(p2, x["q_dec"][t % T], kc2[t % ncopy], vc2[t % ncopy], offs2, b2.cache_lens,
                                   b2.max_cache_len, b2.c_q, b2.c_out, b2.c_lse, b2.out, b2.a_lse, b2.flags,
                                   b2.ws_decode, stream)
            ncall = 2 * ncopy if bud == 128 else 60
            for t in range(6):
                call2(t)
            e0, e1 = ev(), ev()
            e0.record(stream)
            for t in range(ncall):
                call2(t)
            e1.record(stream)
            torch.cuda.synchronize()
            us2 = e0.elapsed_time(e1) * 1e3 / ncall
            other[bud] = {"budget": bud, "bytes_per_call": nbytes, "us_per_call": us2,
                          "GBps": nbytes / us2 / 1e3, "pct_hbm_peak": 100.0 * nbytes / us2 / 1e3 / HBM_PEAK_GBPS,
                          "cache_copies_rotated": ncopy,
                          "compress_us_per_layer": sum(cms) / len(cms) * 1e3 / wl2.batch}
            del b2, kc2, vc2

    # the same T decode calls captured once in a HIP graph and replayed (no per-call host work)
    graph_us = None
    if not args.no_extra:
        side = torch.cuda.Stream()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.stream(side):
            decode_call_on = lambda t, st: cd.calidrop_decode(
                p, x["q_dec"][t], k_copies[t % rotate], v_copies[t % rotate], offs, bufs.cache_lens,
                bufs.max_cache_len, bufs.c_q, bufs.c_out, bufs.c_lse, bufs.out, bufs.a_lse, bufs.flags,
                bufs.ws_decode, st)
            decode_call_on(0, side)
            side.synchronize()
            with torch.cuda.graph(graph, stream=side):
                for t in range(T):
                    decode_call_on(t, torch.cuda.current_stream())
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        e0, e1 = ev(), ev()
        e0.record(stream)
        for _ in range(3):
            graph.replay()
        e1.record(stream)
        torch.cuda.synchronize()
        graph_us = e0.elapsed_time(e1) * 1e3 / (3 * T)

    # compress with the window rows' log-sum-exp handed over by the caller (the by-product of the
    # prefill attention that precedes Alg. 1 step 3): pass 1 over K is skipped.  The values are
    # taken from the library's own row table of the last compress call (log2 units, rows of a KV
    # head = head-in-group x window index), which is what such a caller would have.
    comp_lse_us = None
    if not args.no_extra and wl.n_q_heads // wl.n_kv_heads * wl.window <= 128:
        G_ = wl.n_q_heads // wl.n_kv_heads
        tab = bufs.region(cd.REGION_ROW_LSE).view(wl.batch, wl.n_kv_heads, 128)[:, :, :G_ * wl.window]
        win_lse = (tab.reshape(wl.batch, wl.n_q_heads, wl.window) * 0.6931471805599453).contiguous()
        times = []
        for it in range(5):
            e0, e1 = ev(), ev()
            e0.record(stream)
            bufs.compress(x["q_win"], x["k"], x["v"], x["seq_offsets"], stream=stream, win_lse=win_lse)
            e1.record(stream)
            torch.cuda.synchronize()
            times.append(e0.elapsed_time(e1) * 1e3)
        comp_lse_us = sorted(times[1:])[len(times[1:]) // 2]

    # recomputation branch (Alg. 2 steps 3-8), worst case: every head of every layer flagged
    recal_us = None
    if not args.no_extra:
        bufs.decode(x["q_dec"][0], stream=stream)
        times = []
        for _ in range(5):
            bufs.flags.fill_(cd.FLAG_RECOMPUTE)
            e0, e1 = ev(), ev()
            e0.record(stream)
            bufs.recalibrate(x["q_dec"][0], x["k"], x["v"], x["seq_offsets"], stream=stream)
            e1.record(stream)
            torch.cuda.synchronize()
            times.append(e0.elapsed_time(e1) * 1e3)
        recal_us = sorted(times)[len(times) // 2]

    # the same branch reading KV_evict from its packed (offloadable) form: device-resident, then
    # page-locked host memory pulled over the host link by the kernel itself (2 layers' worth)
    packed = None
    if not args.no_extra:
        L2 = min(2, wl.batch)
        wl3 = synth.config(3, layers=L2, budget=args.budget, decode_steps=1)
        p3 = cd.make_params(dtype=wl3.dtype, batch=wl3.batch, n_q_heads=wl3.n_q_heads, n_kv_heads=wl3.n_kv_heads,
                            head_dim=wl3.head_dim, window=wl3.window, budget=wl3.budget, pool_kernel=wl3.pool_kernel,
                            theta1=wl3.theta1, theta2=wl3.theta2)
        b3 = cd.CompressBuffers(p3, wl3.seq_lens, dev)
        nel = L2 * wl.seq_lens[0] * wl.n_kv_heads * wl.head_dim
        k3, v3, so3 = x["k"][:nel], x["v"][:nel], x["seq_offsets"][:L2 + 1].clone()
        q3 = x["q_dec"][0][:L2].contiguous()
        b3.compress(x["q_win"][:L2].contiguous(), k3, v3, so3, stream=stream)
        packed = {}
        for where in ("device", "host"):
            store = cd.EvictedStore(b3, wl3.seq_lens, host=(where == "host"))
            store.pack(k3, v3, so3, stream=stream)
            b3.decode(q3, stream=stream)
            times = []
            for _ in range(4):
                b3.flags.fill_(cd.FLAG_RECOMPUTE)
                e0, e1 = ev(), ev()
                e0.record(stream)
                store.recalibrate(q3, stream=stream)
                e1.record(stream)
                torch.cuda.synchronize()
                times.append(e0.elapsed_time(e1) * 1e3)
            us = sorted(times)[len(times) // 2]
            nbytes = 2 * store.k_e.numel() * store.k_e.element_size()
            packed[where] = {"us_per_layer": us / L2, "GBps": nbytes / us / 1e3, "bytes_per_layer": nbytes // L2}
            del store
        del b3

    # H2O as the eviction strategy (accumulated attention of every prompt query: two dense causal
    # passes on the matrix cores) for one layer of the same shape
    h2o = None
    if not args.no_extra:
        wl4 = synth.config(3, layers=1, budget=args.budget, decode_steps=1)
        p4 = cd.make_params(dtype=wl4.dtype, batch=1, n_q_heads=wl4.n_q_heads, n_kv_heads=wl4.n_kv_heads,
                            head_dim=wl4.head_dim, window=wl4.window, budget=wl4.budget, pool_kernel=1,
                            theta1=wl4.theta1, theta2=wl4.theta2)
        n4 = wl4.seq_lens[0]
        x4 = {"q_win": x["q_win"][:1].contiguous()}
        qf = synth.full_queries(wl4, x4, synth.BASE_SEED, dev)
        nel = n4 * wl.n_kv_heads * wl.head_dim
        b4 = cd.CompressBuffers(p4, wl4.seq_lens, dev)
        so4 = x["seq_offsets"][:2].clone()
        times = []
        for _ in range(3):
            e0, e1 = ev(), ev()
            e0.record(stream)
            b4.compress_h2o(qf, x["k"][:nel], x["v"][:nel], so4, stream=stream)
            e1.record(stream)
            torch.cuda.synchronize()
            times.append(e0.elapsed_time(e1))
        ms = min(times)
        flop = 2 * 2.0 * wl4.n_q_heads * (n4 * (n4 + 1) / 2) * wl4.head_dim       # two causal QK^T passes
        h2o = {"ms_per_layer": ms, "causal_TFLOP": flop / 1e12, "TFLOPps": flop / ms / 1e9,
               "pct_bf16_mfma_peak": 100.0 * flop / ms / 1e9 / 2500.0}
        del b4, qf

    probes = machine_probes(dev, stream) if not args.no_extra else None

    gbps = dbytes / (dec * 1e-3) / 1e9
    # window scoring (the two MFMA passes of compress): 2*Hq*w*n*D flop per layer and pass
    score_flop = 2.0 * wl.n_q_heads * wl.window * wl.seq_lens[0] * wl.head_dim * wl.batch
    default_cfg = args.budget == 512 and args.layers == 32
    out = {
        "metric": "decode attn GB/s (% HBM peak) + compress us/layer at 32k ctx, budget 512",
        "value": gbps, "unit": "GB/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": wall * 1e3 / args.steps, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": wl.name, "layers": wl.batch, "context": wl.seq_lens[0], "budget": wl.budget,
                   "window": wl.window, "pool_kernel": wl.pool_kernel, "q_heads": wl.n_q_heads,
                   "kv_heads": wl.n_kv_heads, "head_dim": wl.head_dim, "decode_steps_per_step": T,
                   "cache_copies_rotated": rotate},
        "pct_hbm_peak": 100.0 * gbps / HBM_PEAK_GBPS,
        "decode_us_per_call": dec * 1e3,
        "decode_bytes_per_call": dbytes,
        "decode_GBps_cache_resident": dbytes / (dec_res * 1e-3) / 1e9,
        "decode_us_per_call_hip_graph": graph_us,
        "decode_us_per_call_median_min": [statistics.median(dec_ms) * 1e3, min(dec_ms) * 1e3],
        "compress_us_per_layer_median_min": [statistics.median(comp_ms) * 1e3 / wl.batch, min(comp_ms) * 1e3 / wl.batch],
        "budget_128": other.get(128),
        "budget_2048": other.get(2048),
        "compress_us_per_layer": comp * 1e3 / wl.batch,
        "compress_GBps_vs_read_kv_once": compress_bytes(wl) / (comp * 1e-3) / 1e9,
        "compress_pct_of_16.8us_bound": 100.0 * (compress_bytes(wl) / wl.batch / (HBM_PEAK_GBPS * 1e3)) / (comp * 1e3 / wl.batch),
        "compress_us_per_layer_with_supplied_window_lse": None if comp_lse_us is None else comp_lse_us / wl.batch,
        "scoring_algorithmic_TFLOP": score_flop / 1e12,
        "recalibrate_all_heads_us_per_layer": None if recal_us is None else recal_us / wl.batch,
        "recalibrate_all_heads_GBps": None if recal_us is None else compress_bytes(wl) / recal_us / 1e3,
        "recalibrate_all_heads_from_packed_evicted": packed,
        "compress_h2o_strategy": h2o,
        "machine_probes": probes,
        "roofline": {"bound": "hbm", "kernel": "decode_fused_kernel<bf16,128,8>",
                     "achieved": gbps, "peak": HBM_PEAK_GBPS, "unit": "GB/s", "frac": gbps / HBM_PEAK_GBPS,
                     # rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE per launch of this kernel on this workload,
                     # scaled by the counters' readings for a plain 1 GiB copy (x2.0 / x1.0)
                     "traffic": DECODE_TRAFFIC_BYTES_PMC if default_cfg else None,
                     "duration_us": dec * 1e3,
                     "note": "duration = HIP-event time over all decode calls of the timed region / calls; "
                             "one kernel per call"},
    }
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(wl, x, layers=24, decode_steps=128)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
