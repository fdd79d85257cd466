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
MFMA_BF16_PEAK_TFLOPS = 2500.0  # MI355X dense bf16 matrix cores, published
HBM_PROFILE = os.path.join(ROOT, "profiles", "bench_cfg3_B512_pmc_hbm_bytes.md")


def decode_traffic_from_profile(kernel: str):
    """HBM bytes per launch of `kernel` as the committed rocprofv3 counter summary states them
    (FETCH_SIZE and WRITE_SIZE in KiB per launch, scaled by the factors the same file derives from a
    plain 1 GiB copy).  None when the file is missing or lists the decode kernel under another name
    (a summary that belongs to another build of the kernel must not be quoted for this one)."""
    import re
    try:
        text = open(HBM_PROFILE).read()
    except OSError:
        return None, f"{os.path.relpath(HBM_PROFILE, ROOT)} not found"
    m = re.search(r"scale factors are x([0-9.]+) \(fetch\) and x([0-9.]+) \(write\)", text)
    row = [l for l in text.splitlines() if l.startswith("| `decode_fused_kernel")]
    if not m or not row:
        return None, "no decode kernel row / scale factors in the profile summary"
    cells = [c.strip() for c in row[0].strip("|").split("|")]
    name = cells[0].strip("`")
    if name.replace(" ", "") != kernel.replace(" ", ""):
        return None, f"profile summary lists {name}, this run timed {kernel}"
    fetch_kib, write_kib = float(cells[2]), float(cells[3])
    return int(round((fetch_kib * float(m.group(1)) + write_kib * float(m.group(2))) * 1024)), os.path.relpath(HBM_PROFILE, ROOT)


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
    # "64MiB_256wg": the launch shape of the headline decode call (one workgroup of 256 threads per compute unit)
    for label, nbytes, blocks, reps in (("64MiB", 64 << 20, 2048, 32), ("64MiB_256wg", 64 << 20, 256, 32),
                                        ("256MiB", 256 << 20, 8192, 16), ("2GiB", 2 << 30, 32768, 6)):
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
    # a 2 GiB streaming read alone and with 32 / 160 MiB of full-line stores mixed in (what the votes and the
    # exported logits of scoring pass 2 are to its K stream)
    L.calidrop_probe_stream_read_store.argtypes = [ctypes.c_void_p, ctypes.c_void_p] + [ctypes.c_int32] * 3 + [ctypes.c_void_p] * 2
    dst = torch.empty(5 * 4096 * 32 * 64, dtype=torch.float32, device=dev)
    mix = {}
    for rows in (0, 1, 5, 0):
        for it in range(3):
            e0, e1 = ev(), ev()
            e0.record(stream)
            assert L.calidrop_probe_stream_read_store(buf.data_ptr(), dst.data_ptr(), 4096, 32, rows, out.data_ptr(), st) == 0
            e1.record(stream)
            torch.cuda.synchronize()
        mix[f"{rows * 32}MiB_of_stores"] = e0.elapsed_time(e1) * 1e3
    res["stream_read_2GiB_with_stores_us"] = mix
    del dst
    # matrix and vector instructions on the same SIMDs: alone and together (4 waves per SIMD)
    L.calidrop_probe_mfma_valu.argtypes = [ctypes.c_void_p] + [ctypes.c_int32] * 5 + [ctypes.c_void_p]
    def coissue(matrix, nv, use_exp, iters=4000):
        for n in (200, iters):
            e0, e1 = ev(), ev()
            e0.record(stream)
            assert L.calidrop_probe_mfma_valu(out.data_ptr(), 1024, n, matrix, nv, use_exp, st) == 0
            e1.record(stream)
            torch.cuda.synchronize()
        return e0.elapsed_time(e1) * 1e6 / (iters * 8 * 4)      # ns per pair of matrix instructions and SIMD
    t_m = coissue(1, 0, 0)
    co = {"ns_per_pair_of_matrix_instructions": t_m}
    for kind, use_exp in (("fma", 0), ("exp2", 1)):
        t_v, t_b = coissue(0, 8, use_exp), coissue(1, 8, use_exp)
        co["8_" + kind] = {"vector_only_ns": t_v, "both_ns": t_b, "hidden_share_of_vector_time": (t_m + t_v - t_b) / t_v}
    res["matrix_and_vector_together_4_waves_per_simd"] = co
    del buf, out
    return res


def pinned_read_probe(host_tensor, stream):
    """GB/s of the streaming-read probe kernels over a page-locked host tensor (the ceiling for any kernel
    that pulls its operands over the host link itself): requested as whole rows, and as the 64-byte
    pieces of a matrix-operand fragment load."""
    import ctypes
    import torch
    import paper_2507_19906_amd
    path = os.path.join(os.path.dirname(os.path.abspath(paper_2507_19906_amd.__file__)), "libcalidrop_probes.so")
    L = ctypes.CDLL(path)
    L.calidrop_probe_stream_read_nt.argtypes = [ctypes.c_void_p, ctypes.c_uint64, ctypes.c_int32, ctypes.c_void_p, ctypes.c_void_p]
    L.calidrop_probe_stream_read_pieces.argtypes = L.calidrop_probe_stream_read_nt.argtypes
    blocks = 1024
    nbytes = (host_tensor.numel() * host_tensor.element_size()) // (32768 * blocks) * (32768 * blocks)
    out = torch.zeros(blocks, dtype=torch.int32, device="cuda")
    st = stream.cuda_stream or None
    best = {}
    for name, fn in (("whole_rows", L.calidrop_probe_stream_read_nt), ("64_byte_pieces", L.calidrop_probe_stream_read_pieces)):
        best[name] = 0.0
        for it in range(3):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record(stream)
            assert fn(host_tensor.data_ptr(), nbytes, blocks, out.data_ptr(), st) == 0
            e1.record(stream)
            torch.cuda.synchronize()
            best[name] = max(best[name], nbytes / (e0.elapsed_time(e1) * 1e3) / 1e3)
    return best


def timed(fn, stream, n, warm=2):
    """Mean microseconds per call of fn(i), HIP events on `stream` around n calls after `warm` calls."""
    import torch
    for i in range(warm):
        fn(i)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record(stream)
    for i in range(n):
        fn(warm + i)
    e1.record(stream)
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) * 1e3 / n


def other_configs(dev, stream, which=(2, 4, 5)):
    """The other workloads of the brief, each through the same two entry points: the single 8k-context
    layer (config 2), the batch of 64 variable-length sequences with the compressed caches packed behind an
    offsets array (config 4) and the 131k-context layer (config 5).  Compress time per call, decode time per
    call with the calls cycling over address-distinct copies of the compressed cache (more than the 256 MB
    Infinity Cache in total whenever one call moves at least 16 MiB), and for the window scoring the time of
    its first pass, taken as the difference between compress and compress with the window rows' log-sum-exp
    supplied (which skips exactly that pass)."""
    import numpy as np
    import torch
    from paper_2507_19906_amd import binding as cd
    from paper_2507_19906_amd import synth
    res = {}
    for idx in which:
        wl = synth.config(idx, decode_steps=8)
        x = synth.make_inputs(wl, device=dev)
        p = cd.make_params(dtype=wl.dtype, batch=wl.batch, n_q_heads=wl.n_q_heads, n_kv_heads=wl.n_kv_heads,
                           head_dim=wl.head_dim, window=wl.window, budget=wl.budget, pool_kernel=wl.pool_kernel,
                           theta1=wl.theta1, theta2=wl.theta2)
        caps = None
        if idx == 4:        # variable capacities: budget + 0..40 rows per sequence, packed back to back
            rng = np.random.default_rng(4)
            caps = [min(wl.budget, n) + int(e) for n, e in zip(wl.seq_lens, rng.integers(0, 41, wl.batch))]
        bufs = cd.CompressBuffers(p, wl.seq_lens, dev, capacities=caps)
        comp_us = timed(lambda i: bufs.compress(x["q_win"], x["k"], x["v"], x["seq_offsets"], stream=stream), stream, 5)
        G, w = wl.group, wl.window
        tab = bufs.region(cd.REGION_ROW_LSE).view(wl.batch, wl.n_kv_heads, -1)[:, :, :G * w]
        win_lse = (tab.reshape(wl.batch, wl.n_q_heads, w) * 0.6931471805599453).contiguous()
        comp_lse_us = timed(lambda i: bufs.compress(x["q_win"], x["k"], x["v"], x["seq_offsets"], stream=stream,
                                                    win_lse=win_lse), stream, 5)
        bufs.compress(x["q_win"], x["k"], x["v"], x["seq_offsets"], stream=stream)
        torch.cuda.synchronize()
        E = 2
        tokens = sum(wl.seq_lens)
        k_bytes = tokens * wl.n_kv_heads * wl.head_dim * E
        flop = 2.0 * wl.n_q_heads * w * tokens * wl.head_dim                  # one Q_win K^T pass
        pass1_us = comp_us - comp_lse_us
        # decode: bytes of the live rows actually streamed
        live = bufs.cache_lens.cpu().numpy().astype(np.int64)
        dbytes = int(2 * wl.n_kv_heads * wl.head_dim * E * live.sum()
                     + wl.batch * wl.n_q_heads * (wl.head_dim * E + (2 * wl.head_dim + 1) * 4 + wl.head_dim * E))
        ncopy = max(2, -(-(512 << 20) // dbytes)) if dbytes >= (16 << 20) else 1
        kc = [bufs.k_c] + [bufs.k_c.clone() for _ in range(ncopy - 1)]
        vc = [bufs.v_c] + [bufs.v_c.clone() for _ in range(ncopy - 1)]
        offs = None if bufs.uniform else bufs.cache_offsets
        T = x["q_dec"].shape[0]

        def dec(i):
            cd.calidrop_decode(p, x["q_dec"][i % T], kc[i % ncopy], vc[i % ncopy], offs, bufs.cache_lens, bufs.max_cache_len,
                               bufs.c_q, bufs.c_out, bufs.c_lse, bufs.out, bufs.a_lse, bufs.flags, bufs.ws_decode, stream)
        dec_us = timed(dec, stream, 64 if ncopy > 1 else 200, warm=8)
        r = {"workload": wl.name, "tokens": tokens, "compress_us_per_call": comp_us,
             "compress_us_per_call_with_supplied_window_lse": comp_lse_us,
             "compress_GBps_vs_read_kv_once": 2 * k_bytes / comp_us / 1e3,
             "scoring_pass1_us_by_difference": pass1_us,
             "scoring_pass1_TFLOPps": flop / pass1_us / 1e6 if pass1_us > 0 else None,
             "scoring_pass1_pct_bf16_mfma_peak": 100.0 * flop / pass1_us / 1e6 / MFMA_BF16_PEAK_TFLOPS if pass1_us > 0 else None,
             "scoring_pass1_K_GBps": k_bytes / pass1_us / 1e3 if pass1_us > 0 else None,
             "scoring_flop_per_K_byte": w * G,
             "decode_us_per_call": dec_us, "decode_bytes_per_call": dbytes, "cache_copies_rotated": ncopy,
             "cache_offsets_array": offs is not None}
        if ncopy > 1:
            r["decode_GBps"] = dbytes / dec_us / 1e3
            r["decode_pct_hbm_peak"] = 100.0 * dbytes / dec_us / 1e3 / HBM_PEAK_GBPS
        else:
            r["decode_note"] = "under 16 MiB per call: bound by launch and memory latency, no bandwidth figure"
        res[f"config{idx}"] = r
        del bufs, kc, vc, x
        torch.cuda.empty_cache()
    return res


def alg2_loop(cd, bufs, x, T, stream):
    """The complete decode step of Alg. 2 with the state carried on the GPU: calidrop_decode, then
    calidrop_recalibrate for the heads it flagged (rho < theta1).  The headline figure times the
    decode calls alone; this says what the recomputation branch adds on these synthetic queries and
    how many heads take it."""
    import torch
    steps = min(T, 64)
    bufs.compress(x["q_win"], x["k"], x["v"], x["seq_offsets"], stream=stream)
    seen = torch.zeros((steps,) + tuple(bufs.flags.shape), dtype=torch.uint8, device=bufs.flags.device)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record(stream)
    for t in range(steps):
        bufs.decode(x["q_dec"][t], stream=stream)
        seen[t].copy_(bufs.flags)                    # a 1 KiB device copy, no host round trip: the flags as decode left them
        bufs.recalibrate(x["q_dec"][t], x["k"], x["v"], x["seq_offsets"], stream=stream)
    e1.record(stream)
    torch.cuda.synchronize()
    h = [int((seen == v).sum().item()) for v in range(3)]
    G = bufs.p.n_q_heads // bufs.p.n_kv_heads
    groups = (seen == 2).view(steps, bufs.p.batch, bufs.p.n_kv_heads, G).any(dim=3)
    return {"steps": steps, "us_per_step_decode_plus_recalibrate": e0.elapsed_time(e1) * 1e3 / steps,
            "flags_after_decode_none_calibrated_recompute": h,
            "fraction_of_heads_recomputed_per_step": h[2] / max(1, sum(h)),
            "fraction_of_kv_groups_whose_evicted_rows_are_read_per_step": float(groups.float().mean().item()),
            "note": "includes a 1 KiB device copy of the flags per step"}


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
    ap.add_argument("--profile-config", type=int, choices=(2, 4, 5), default=0,
                    help="run only this other configuration (compress and decode calls, no headline workload) and print "
                         "its figures: the command the rocprofv3 summaries of configs 2, 4 and 5 are made with")
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

    if args.profile_config:
        print(json.dumps(other_configs(dev, torch.cuda.current_stream(), which=(args.profile_config,))))
        return

    wl = synth.config(3, layers=args.layers, budget=args.budget, decode_steps=args.decode_steps)
    default_cfg_early = args.budget == 512 and args.layers == 32
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
    if not args.no_extra:
        G_ = wl.n_q_heads // wl.n_kv_heads
        tab = bufs.region(cd.REGION_ROW_LSE).view(wl.batch, wl.n_kv_heads, -1)[:, :, :G_ * wl.window]
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
        store = None
        for where in ("device", "host", "host_staged"):
            if where == "host_staged":        # the same page-locked buffers as "host" (their placement decides the link rate)
                store.staged = True
            else:
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
            if where == "host":
                # the plain copy rate of the host link for the same bytes, and what a kernel that only
                # reads the page-locked rows reaches (the probe's streaming read)
                kd, vd = torch.empty_like(store.k_dev), torch.empty_like(store.v_dev)
                for it in range(3):
                    e0, e1 = ev(), ev()
                    e0.record(stream)
                    kd.copy_(store.k_e, non_blocking=True)
                    vd.copy_(store.v_e, non_blocking=True)
                    e1.record(stream)
                    torch.cuda.synchronize()
                packed["host_link_plain_copy_GBps"] = nbytes / (e0.elapsed_time(e1) * 1e3) / 1e3
                packed["host_link_kernel_read_GBps"] = pinned_read_probe(store.k_e, stream)
                del kd, vd
        del store, b3

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
    loop = alg2_loop(cd, bufs, x, T, stream) if not args.no_extra else None
    flags_last = torch.bincount(bufs.flags.flatten().long(), minlength=4)[:3].cpu().tolist()
    others = None
    if not args.no_extra and default_cfg_early:
        del k_copies, v_copies
        torch.cuda.empty_cache()
        others = other_configs(dev, stream)

    gbps = dbytes / (dec * 1e-3) / 1e9
    # window scoring (the two MFMA passes of compress): 2*Hq*w*n*D flop per layer and pass
    score_flop = 2.0 * wl.n_q_heads * wl.window * wl.seq_lens[0] * wl.head_dim * wl.batch
    default_cfg = default_cfg_early
    # the kernel calidrop_decode launches for this shape (4 waves per workgroup when the pairs fill the chip)
    decode_kernel = "decode_fused_kernel<bf16_t, 128, %d>" % (4 if wl.batch * wl.n_kv_heads >= 192 or wl.budget <= 128 else 8)
    traffic, traffic_src = decode_traffic_from_profile(decode_kernel) if default_cfg else (None, "not the profiled workload")
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
        "alg2_loop_with_recomputation": loop,
        "flags_of_last_decode_call_none_calibrated_recompute": flags_last,
        "timed_step_note": "one step = compress + T decode calls; heads that a decode call flags for recomputation "
                           "(rho < theta1) are not recomputed inside the timed step - see alg2_loop_with_recomputation",
        "other_configs": others,
        "roofline": {"bound": "hbm", "kernel": decode_kernel,
                     "achieved": gbps, "peak": HBM_PEAK_GBPS, "unit": "GB/s", "frac": gbps / HBM_PEAK_GBPS,
                     # rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE per launch of this kernel on this workload, read
                     # from the committed counter summary (null when that summary is of another kernel build)
                     "traffic": traffic, "traffic_source": traffic_src,
                     "duration_us": dec * 1e3,
                     "note": "duration = HIP-event time over all decode calls of the timed region / calls; "
                             "one kernel per call"},
    }
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(wl, x, layers=24, decode_steps=128)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
