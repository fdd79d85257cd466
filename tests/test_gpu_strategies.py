"""Retained sets that do not come from the scored selection (Sec. 4.1.3: StreamingLLM; or any
list a caller computed): index arithmetic, gather and calibration state on the GPU vs the
oracle, then Alg. 2 (decode and the recomputation branch) on that state.  Needs an MI355X."""
import numpy as np
import pytest
import torch

from oracle import calidrop_ref as ref
from paper_2507_19906_amd import binding as cd
from paper_2507_19906_amd import synth
from tests import helpers as H

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def to_dev(x):
    return {k: v.to(DEV) for k, v in x.items()}


def small(dtype, Hq, Hkv, D, lens, w, B, k, T=4, name="small"):
    return synth.Workload(name, len(lens), Hq, Hkv, D, list(lens), w, B, k, dtype, T)


def check_given(wl, x, bufs, q_cal, lists, rep):
    """Everything calidrop_compress_given wrote vs the oracle, for the retained `lists`
    [batch][Hkv] (None for sequences within the budget)."""
    B, G = wl.budget, wl.group
    for b in range(wl.batch):
        n = wl.seq_lens[b]
        K = H.to64(synth.seq_view(x["k"], wl, b))
        V = H.to64(synth.seq_view(x["v"], wl, b))
        orc = ref.compress_given(H.to64(q_cal[b]), K, V, B, lists[b])
        length = min(n, B)
        assert int(bufs.cache_lens[b].item()) == length
        gi = bufs.indices[b].cpu().numpy()
        assert np.array_equal(gi[:, :length], orc["idx"]) and np.all(gi[:, length:] == -1)
        assert np.array_equal(H.to64(bufs.cache_view("k", b))[:, :length], orc["K_c"])
        assert np.array_equal(H.to64(bufs.cache_view("v", b))[:, :length], orc["V_c"])
        assert np.array_equal(H.to64(bufs.c_q[b]), orc["c_q"])
        c_out, c_lse = H.to64(bufs.c_out[b]), H.to64(bufs.c_lse[b])
        if n <= B:
            assert np.all(c_lse == -np.inf) and np.all(c_out == 0)
            continue
        e_o, e_l = np.abs(c_out - orc["c_out"]).max(), np.abs(c_lse - orc["c_lse"]).max()
        rep["c_out_err"] = max(rep.get("c_out_err", 0), e_o)
        rep["c_lse_err"] = max(rep.get("c_lse_err", 0), e_l)
        assert e_o <= H.TOL_OUT[wl.dtype] and e_l <= H.TOL_LSE[wl.dtype], (e_o, e_l)


def decode_and_recalibrate(wl, x, bufs, rep, steps):
    for t in range(steps):
        q_t = x["q_dec"][t]
        bufs.decode(q_t)
        torch.cuda.synchronize()
        for b in range(wl.batch):
            H.check_decode_step(wl, bufs, q_t, b, report=rep)
        before = H.snapshot_state(bufs)
        bufs.recalibrate(q_t, x["k"], x["v"], x["seq_offsets"])
        torch.cuda.synchronize()
        for b in range(wl.batch):
            H.check_recalibrate(wl, x, bufs, q_t, b, before, report=rep)


@pytest.mark.parametrize("wl,n_sink", [
    (small("bf16", 8, 2, 128, [900, 40, 2100], 16, 128, 5, T=6, name="slm_varlen_bf16"), 32),
    (small("fp32", 8, 2, 64, [1031], 16, 96, 3, T=4, name="slm_fp32_d64"), 32),
    (small("bf16", 32, 8, 128, [4096, 513], 32, 512, 7, T=3, name="slm_llama_shape"), 32),
    (small("fp32", 4, 2, 64, [300], 8, 64, 1, T=3, name="slm_window_only"), 0),
    (small("fp32", 4, 2, 64, [300], 8, 64, 1, T=3, name="slm_sinks_only"), 64),
    # a prompt whose skip bitmap (one bit per position) no longer fits the 48 KiB of LDS the recomputation
    # builds it in: the bitmap is then built in global memory
    (small("bf16", 2, 1, 64, [400000, 3000], 16, 256, 1, T=3, name="slm_400k_bitmap_in_global_memory"), 32),
], ids=lambda v: v.name if hasattr(v, "name") else str(v))
def test_streaming_llm_strategy(wl, n_sink):
    x = to_dev(synth.make_inputs(wl, 77))
    p = H.params_for(wl)
    bufs = cd.CompressBuffers(p, wl.seq_lens, DEV)
    bufs.indices.fill_(-7)
    bufs.streaming_indices(n_sink, x["seq_offsets"])
    torch.cuda.synchronize()
    lists = []
    for b, n in enumerate(wl.seq_lens):
        want = ref.streaming_llm_retained(n, wl.budget, n_sink)
        got = bufs.indices[b].cpu().numpy()
        for g in range(wl.n_kv_heads):
            assert np.array_equal(got[g, :len(want)], want) and np.all(got[g, len(want):] == -1)
        lists.append([want] * wl.n_kv_heads if n > wl.budget else None)
    q_cal = x["q_win"][:, :, -1].contiguous()                    # Q_{-1}
    bufs.compress_given(q_cal, x["k"], x["v"], x["seq_offsets"])
    torch.cuda.synchronize()
    rep = {}
    check_given(wl, x, bufs, q_cal, lists, rep)
    decode_and_recalibrate(wl, x, bufs, rep, wl.decode_steps)
    flags = np.bincount(rep.pop("flags"), minlength=4)
    print(wl.name, rep, flags.tolist(), flush=True)


def test_caller_supplied_lists_differ_per_head_and_need_not_hold_the_window():
    # any f: random distinct positions per (sequence, KV head), window not necessarily retained
    wl = small("bf16", 8, 4, 128, [1500, 700, 90], 16, 100, 5, T=4, name="given_random")
    x = to_dev(synth.make_inputs(wl, 5))
    rng = np.random.default_rng(99)
    p = H.params_for(wl)
    bufs = cd.CompressBuffers(p, wl.seq_lens, DEV)
    host = np.full((wl.batch, wl.n_kv_heads, wl.budget), -1, np.int32)
    lists = []
    for b, n in enumerate(wl.seq_lens):
        if n <= wl.budget:
            lists.append(None)
            host[b] = 123456                                    # ignored and overwritten by the library
            continue
        per = [np.sort(rng.choice(n, wl.budget, replace=False)) for _ in range(wl.n_kv_heads)]
        lists.append(per)
        host[b] = np.stack(per)
    bufs.indices.copy_(torch.from_numpy(host))
    q_cal = x["q_win"][:, :, -1].contiguous()
    bufs.compress_given(q_cal, x["k"], x["v"], x["seq_offsets"])
    torch.cuda.synchronize()
    rep = {}
    check_given(wl, x, bufs, q_cal, lists, rep)
    decode_and_recalibrate(wl, x, bufs, rep, wl.decode_steps)
    rep.pop("flags")
    print(wl.name, rep, flush=True)


def test_given_path_with_the_scored_lists_reproduces_compress():
    # feeding calidrop_compress's own retained lists back gives the same cache and state
    wl = small("fp32", 8, 2, 64, [1200, 333], 16, 80, 5, T=1, name="given_equals_scored")
    x = to_dev(synth.make_inputs(wl, 3))
    a = H.gpu_compress(wl, x)
    p = H.params_for(wl)
    b2 = cd.CompressBuffers(p, wl.seq_lens, DEV)
    b2.indices.copy_(a.indices)
    b2.compress_given(x["q_win"][:, :, -1].contiguous(), x["k"], x["v"], x["seq_offsets"])
    torch.cuda.synchronize()
    assert torch.equal(a.k_c, b2.k_c) and torch.equal(a.v_c, b2.v_c) and torch.equal(a.cache_lens, b2.cache_lens)
    assert torch.equal(a.c_q, b2.c_q)
    assert (a.c_out - b2.c_out).abs().max().item() < 1e-4
    assert (a.c_lse - b2.c_lse).abs().max().item() < 1e-4


def test_out_of_range_entries_are_memory_safe():
    # a broken list must not make the kernels read or write outside the buffers: entries outside
    # [0, n) are clamped by the gather and mark nothing as retained
    wl = small("fp32", 4, 2, 64, [400], 8, 32, 1, T=1, name="given_bad_entries")
    x = to_dev(synth.make_inputs(wl, 4))
    p = H.params_for(wl)
    bufs = cd.CompressBuffers(p, wl.seq_lens, DEV)
    host = np.tile(np.arange(32, dtype=np.int32) * 3, (1, 2, 1))
    host[0, 0, 5] = -9
    host[0, 1, 7] = 1 << 30
    bufs.indices.copy_(torch.from_numpy(host))
    guard_k, guard_v = x["k"].clone(), x["v"].clone()
    bufs.compress_given(x["q_win"][:, :, -1].contiguous(), x["k"], x["v"], x["seq_offsets"])
    torch.cuda.synchronize()
    assert torch.equal(guard_k, x["k"]) and torch.equal(guard_v, x["v"])
    assert torch.isfinite(bufs.c_out).all()
    K = H.to64(synth.seq_view(x["k"], wl, 0))
    Kc = H.to64(bufs.cache_view("k", 0))
    assert np.array_equal(Kc[0, 5], K[0, 0]) and np.array_equal(Kc[1, 7], K[1, 399])     # clamped rows
    assert np.array_equal(Kc[0, 6], K[0, 18])


# ---- offloading KV_evict: packed rows, and the recomputation branch reading them -------------------
def check_packed(wl, x, bufs, store, orc_evicted):
    """Packed lists and rows vs the oracle's evicted / calibration sets (bit-exact)."""
    for b, n in enumerate(wl.seq_lens):
        rows = store.rows[b]
        assert int(store.evict_lens[b].item()) == rows
        if rows == 0:
            continue
        K = H.to64(synth.seq_view(x["k"], wl, b))
        V = H.to64(synth.seq_view(x["v"], wl, b))
        gi = store.view("idx", b).cpu().numpy()[:, :rows]
        ke = H.to64(store.view("k", b))[:, :rows]
        ve = H.to64(store.view("v", b))[:, :rows]
        for g in range(wl.n_kv_heads):
            want = orc_evicted[b][g]
            assert np.array_equal(gi[g], want), (b, g)
            assert np.array_equal(ke[g], K[g][want]) and np.array_equal(ve[g], V[g][want])


@pytest.mark.parametrize("wl,m,host", [
    (small("bf16", 8, 2, 128, [900, 40, 2100], 16, 128, 5, T=6, name="pack_varlen_bf16"), 0, False),
    (small("bf16", 8, 2, 128, [900, 40, 2100], 16, 128, 5, T=6, name="pack_varlen_bf16_host"), 0, True),
    (small("fp32", 8, 2, 64, [1031, 97], 16, 96, 3, T=4, name="pack_fp32_calib"), 50, False),
    (small("fp32", 8, 2, 64, [1031, 97], 16, 96, 3, T=4, name="pack_fp32_calib_host"), 50, True),
    (small("bf16", 32, 8, 128, [4099], 32, 512, 7, T=3, name="pack_llama_shape"), 0, True),
    (small("fp32", 8, 2, 128, [777, 1290], 16, 96, 3, T=4, name="pack_fp32_d128_host"), 0, True),
    (small("bf16", 8, 4, 64, [1100, 333], 8, 64, 5, T=4, name="pack_bf16_d64_host"), 0, True),
    # brought back by plain copies through two staging buffers, one sequence ahead of the recomputation
    (small("bf16", 8, 2, 128, [900, 40, 2100, 700, 1300], 16, 128, 5, T=6, name="pack_varlen_bf16_staged"), 0, "staged"),
    (small("fp32", 8, 2, 64, [1031, 97, 400], 16, 96, 3, T=4, name="pack_fp32_calib_staged"), 50, "staged"),
], ids=lambda v: v.name if hasattr(v, "name") else str(v))
def test_packed_evicted_rows_and_recomputation_from_them(wl, m, host):
    x = to_dev(synth.make_inputs(wl, 21))
    bufs = H.gpu_compress(wl, x, calib_size=m)
    rep = {}
    orc_evicted = []
    for b in range(wl.batch):
        orc, _ = H.check_compress(wl, x, bufs, b, report=rep)
        orc_evicted.append(orc["evicted"])
    assert rep.get("tie_band_heads", 0) == 0 and rep.get("tie_band_cal_heads", 0) == 0
    store = cd.EvictedStore(bufs, wl.seq_lens, host=bool(host), staged=(host == "staged"))
    store.pack(x["k"], x["v"], x["seq_offsets"])
    torch.cuda.synchronize()
    check_packed(wl, x, bufs, store, orc_evicted)
    # a twin that recomputes from the prompt tensors must agree bit for bit at every step
    twin = H.gpu_compress(wl, x, calib_size=m)
    for t in range(wl.decode_steps):
        q_t = x["q_dec"][t]
        bufs.decode(q_t)
        twin.decode(q_t)
        torch.cuda.synchronize()
        before = H.snapshot_state(bufs)
        store.recalibrate(q_t)
        twin.recalibrate(q_t, x["k"], x["v"], x["seq_offsets"])
        torch.cuda.synchronize()
        for b in range(wl.batch):
            H.check_recalibrate(wl, x, bufs, q_t, b, before, report=rep)
        for name in ("out", "flags", "c_q", "c_out", "c_lse"):
            a, c = getattr(bufs, name), getattr(twin, name)
            if name in ("c_out", "c_lse", "out"):      # different split points: rounding-level differences only
                fin = torch.isfinite(c.float())
                assert torch.equal(torch.isfinite(a.float()), fin)
                assert (a.float() - c.float())[fin].abs().max().item() <= (2e-2 if wl.dtype == "bf16" else 1e-5), name
            else:
                assert torch.equal(a, c), name
    print(wl.name, {k: v for k, v in rep.items() if k != "flags"}, flush=True)
    assert wl.decode_steps < 4 or rep["recal_heads"] > 0


def test_packing_a_streaming_llm_cache():
    wl = small("bf16", 8, 2, 128, [1500, 60], 16, 128, 5, T=3, name="pack_slm")
    x = to_dev(synth.make_inputs(wl, 8))
    p = H.params_for(wl)
    bufs = cd.CompressBuffers(p, wl.seq_lens, DEV)
    bufs.streaming_indices(32, x["seq_offsets"])
    q_cal = x["q_win"][:, :, -1].contiguous()
    bufs.compress_given(q_cal, x["k"], x["v"], x["seq_offsets"])
    store = cd.EvictedStore(bufs, wl.seq_lens, host=True)
    store.pack(x["k"], x["v"], x["seq_offsets"])
    torch.cuda.synchronize()
    ev = [[np.arange(32, 1500 - 96)] * 2, None]
    check_packed(wl, x, bufs, store, ev)
    rep = {}
    for t in range(wl.decode_steps):
        q_t = x["q_dec"][t]
        bufs.decode(q_t)
        torch.cuda.synchronize()
        before = H.snapshot_state(bufs)
        store.recalibrate(q_t)
        torch.cuda.synchronize()
        for b in range(wl.batch):
            H.check_recalibrate(wl, x, bufs, q_t, b, before, report=rep)
    print(wl.name, rep, flush=True)


def test_random_sweep_over_strategies_shapes_and_offload():
    # seeded sweep: strategy (StreamingLLM / caller's lists / H2O), dtype, head shape, lengths,
    # budget, then packing (device or page-locked host) and two decode + recomputation steps,
    # every value against the oracle
    from tests.test_gpu_h2o import check_h2o
    rng = np.random.default_rng(20250719)
    counts = {"slm": 0, "given": 0, "h2o": 0}
    for case in range(14):
        dtype = ["bf16", "fp32"][int(rng.integers(2))]
        D = [64, 128][int(rng.integers(2))]
        Hkv = int(rng.integers(1, 4))
        G = [1, 2, 4, 8][int(rng.integers(4))]
        w = [4, 8, 16][int(rng.integers(3))]
        B = int(rng.integers(w + 6, 260))
        lens = [int(rng.integers(40, 1300)) for _ in range(int(rng.integers(1, 4)))]
        strat = ["slm", "given", "h2o"][case % 3]
        wl = small(dtype, Hkv * G, Hkv, D, lens, w, B, 1, T=2, name=f"sweep{case}_{strat}_{dtype}_D{D}_G{G}")
        print(wl.name, lens, "B", B, flush=True)
        x = to_dev(synth.make_inputs(wl, 1000 + case))
        p = H.params_for(wl)
        bufs = cd.CompressBuffers(p, wl.seq_lens, DEV)
        q_cal = x["q_win"][:, :, -1].contiguous()
        rep = {}
        if strat == "slm":
            n_sink = int(rng.integers(0, B + 1))
            bufs.streaming_indices(n_sink, x["seq_offsets"])
            bufs.compress_given(q_cal, x["k"], x["v"], x["seq_offsets"])
            torch.cuda.synchronize()
            lists = [[ref.streaming_llm_retained(n, B, n_sink)] * Hkv if n > B else None for n in lens]
            check_given(wl, x, bufs, q_cal, lists, rep)
        elif strat == "given":
            host = np.full((len(lens), Hkv, B), -1, np.int32)
            lists = []
            for b, n in enumerate(lens):
                if n <= B:
                    lists.append(None)
                    continue
                per = [np.sort(rng.choice(n, B, replace=False)) for _ in range(Hkv)]
                lists.append(per)
                host[b] = np.stack(per)
            bufs.indices.copy_(torch.from_numpy(host))
            bufs.compress_given(q_cal, x["k"], x["v"], x["seq_offsets"])
            torch.cuda.synchronize()
            check_given(wl, x, bufs, q_cal, lists, rep)
        else:
            n_local = int(rng.integers(1, B))
            q_full = synth.full_queries(wl, x, 1000 + case, DEV)
            bufs.compress_h2o(q_full, x["k"], x["v"], x["seq_offsets"], n_local=n_local)
            torch.cuda.synchronize()
            check_h2o(wl, x, q_full, bufs, n_local, rep)
        counts[strat] += 1
        store = cd.EvictedStore(bufs, wl.seq_lens, host=bool(rng.integers(2)))
        store.pack(x["k"], x["v"], x["seq_offsets"])
        torch.cuda.synchronize()
        idx = bufs.indices.cpu().numpy()
        ev = []
        for b, n in enumerate(lens):
            ev.append([np.setdiff1d(np.arange(n), idx[b, g][idx[b, g] >= 0]) for g in range(Hkv)] if n > B else None)
        check_packed(wl, x, bufs, store, ev)
        for t in range(wl.decode_steps):
            q_t = x["q_dec"][t]
            bufs.decode(q_t)
            torch.cuda.synchronize()
            for b in range(wl.batch):
                H.check_decode_step(wl, bufs, q_t, b, report=rep)
            before = H.snapshot_state(bufs)
            bufs.flags.fill_(cd.FLAG_RECOMPUTE)                  # exercise the branch on every head
            before["flags"][:] = cd.FLAG_RECOMPUTE
            store.recalibrate(q_t)
            torch.cuda.synchronize()
            for b in range(wl.batch):
                H.check_recalibrate(wl, x, bufs, q_t, b, before, report=rep)
    assert min(counts.values()) >= 4


def test_pack_with_too_little_capacity_writes_nothing_for_that_sequence():
    wl = small("fp32", 4, 2, 64, [400, 300], 8, 32, 1, T=1, name="pack_small_capacity")
    x = to_dev(synth.make_inputs(wl, 9))
    bufs = H.gpu_compress(wl, x)
    p = bufs.p
    rows = [cd.calidrop_packed_rows(p, n) for n in wl.seq_lens]            # 368, 268
    caps = [rows[0] - 1, rows[1]]                                          # sequence 0 one row short
    offs = torch.tensor([0, caps[0], caps[0] + caps[1]], dtype=torch.int32, device=DEV)
    tot = (caps[0] + caps[1]) * 2
    k_e = torch.full((tot * 64,), 5.0, device=DEV); v_e = torch.full((tot * 64,), 5.0, device=DEV)
    lens = torch.full((2,), -3, dtype=torch.int32, device=DEV)
    ev_idx = torch.full((tot,), -9, dtype=torch.int32, device=DEV)
    ws = torch.empty(cd.calidrop_pack_evicted_workspace_bytes(p, bufs.max_seq_len), dtype=torch.uint8, device=DEV)
    cd.calidrop_pack_evicted(p, x["k"], x["v"], x["seq_offsets"], bufs.total_tokens, bufs.max_seq_len, bufs.indices,
                             None, k_e, v_e, offs, lens, ev_idx, ws)
    torch.cuda.synchronize()
    assert lens.tolist() == [0, rows[1]]
    n0 = caps[0] * 2
    assert torch.all(k_e[:n0 * 64] == 5.0) and torch.all(ev_idx[:n0] == -9)           # untouched
    K1 = synth.seq_view(x["k"], wl, 1)
    idx1 = bufs.indices[1].cpu().numpy()
    for g in range(2):
        want = np.setdiff1d(np.arange(300), idx1[g])
        got = ev_idx[n0 + g * caps[1]: n0 + (g + 1) * caps[1]].cpu().numpy()
        assert np.array_equal(got, want)
        rows_g = k_e[(n0 + g * caps[1]) * 64:(n0 + (g + 1) * caps[1]) * 64].view(caps[1], 64)
        assert torch.equal(rows_g, K1[g][torch.from_numpy(want).to(DEV)])
