"""Compressed caches of different capacities packed back to back behind cache_offsets (the layout of
the batched workload: variable-length retained caches laid out contiguously, with an offsets array),
through every entry point that takes the offsets: compress, append, decode (one-workgroup and split
forms), recalibrate, and the packed evicted rows.  HIP path vs fp64 oracle.  Needs an MI355X."""
import numpy as np
import pytest
import torch

from paper_2507_19906_amd import binding as cd
from paper_2507_19906_amd import synth
from tests import helpers as H
from tests.test_gpu_strategies import check_packed

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
SENTINEL = 7.0


def to_dev(x):
    return {k: v.to(DEV) for k, v in x.items()}


def capacities(lens, B, extras):
    return [min(B, n) + int(e) for n, e in zip(lens, extras)]


def poisoned_buffers(wl, caps, **over):
    bufs = cd.CompressBuffers(H.params_for(wl, **over), wl.seq_lens, DEV, capacities=caps)
    assert not bufs.uniform
    bufs.k_c.fill_(SENTINEL); bufs.v_c.fill_(SENTINEL)
    return bufs


def rows_beyond_are_untouched(bufs, b, length):
    for which in ("k", "v"):
        assert torch.all(bufs.cache_view(which, b)[:, length:] == SENTINEL), (which, b)


def run_varcap(wl, extras, seed, m=0, seqs=None, append=True, pack=True):
    lens, B = wl.seq_lens, wl.budget
    caps = capacities(lens, B, extras)
    x = to_dev(synth.make_inputs(wl, seed))
    bufs = poisoned_buffers(wl, caps, calib_size=m)
    bufs.compress(x["q_win"], x["k"], x["v"], x["seq_offsets"])
    torch.cuda.synchronize()
    seqs = list(range(wl.batch)) if seqs is None else seqs
    rep, evicted = {}, {}
    for b in seqs:
        orc, _ = H.check_compress(wl, x, bufs, b, report=rep)
        evicted[b] = orc["evicted"]
    for b in range(wl.batch):                       # nothing written past the live rows of any sequence
        rows_beyond_are_untouched(bufs, b, min(B, lens[b]))
    lens0 = bufs.cache_lens.cpu().numpy().copy()
    assert np.array_equal(lens0, np.minimum(B, lens))
    dt = bufs.k_c.dtype
    g = torch.Generator(device=DEV).manual_seed(seed)
    news = []
    for t in range(wl.decode_steps):
        q_t = x["q_dec"][t]
        if append:
            news.append(tuple(torch.randn((wl.batch, wl.n_kv_heads, wl.head_dim), generator=g, device=DEV).to(dt)
                              for _ in range(2)))
            bufs.append(*news[t])
        bufs.decode(q_t)                            # non-uniform capacities: the offsets are passed
        torch.cuda.synchronize()
        for b in range(wl.batch):
            grown = min(len(news), caps[b] - int(lens0[b]))      # a full cache is left unchanged
            assert int(bufs.cache_lens[b]) == int(lens0[b]) + grown, (t, b)
        for b in seqs:
            L0 = int(lens0[b])
            for j in range(min(len(news), caps[b] - L0)):
                assert torch.equal(bufs.cache_view("k", b)[:, L0 + j], news[j][0][b])
                assert torch.equal(bufs.cache_view("v", b)[:, L0 + j], news[j][1][b])
            rows_beyond_are_untouched(bufs, b, int(bufs.cache_lens[b]))
            H.check_decode_step(wl, bufs, q_t, b, report=rep)
        before = H.snapshot_state(bufs)
        bufs.recalibrate(q_t, x["k"], x["v"], x["seq_offsets"])
        torch.cuda.synchronize()
        for b in seqs:
            H.check_recalibrate(wl, x, bufs, q_t, b, before, report=rep)
    if pack and len(seqs) == wl.batch and rep.get("tie_band_heads", 0) == 0 and rep.get("tie_band_cal_heads", 0) == 0:
        # the offloadable form of KV_evict, with slack behind every sequence's rows, and the
        # recomputation branch reading it (every head flagged)
        store = cd.EvictedStore(bufs, lens, extra_rows=[(3 * b + 1) % 11 for b in range(wl.batch)])
        store.pack(x["k"], x["v"], x["seq_offsets"])
        torch.cuda.synchronize()
        check_packed(wl, x, bufs, store, [evicted[b] for b in range(wl.batch)])
        q_t = x["q_dec"][0]
        bufs.decode(q_t)
        bufs.flags.fill_(cd.FLAG_RECOMPUTE)
        torch.cuda.synchronize()
        before = H.snapshot_state(bufs)
        store.recalibrate(q_t)
        torch.cuda.synchronize()
        for b in seqs:
            H.check_recalibrate(wl, x, bufs, q_t, b, before, report=rep)
    flags = np.bincount(rep.pop("flags"), minlength=4).tolist()
    print(wl.name, "capacities", caps if len(caps) <= 8 else f"{min(caps)}..{max(caps)}", rep,
          "flags", flags, "tie-band heads", rep.get("tie_band_heads", 0), flush=True)
    return rep


def small(dtype, Hq, Hkv, D, lens, w, B, k, T, name):
    return synth.Workload(name, len(lens), Hq, Hkv, D, list(lens), w, B, k, dtype, T)


@pytest.mark.parametrize("dtype,D", [("bf16", 128), ("fp32", 64), ("bf16", 64), ("fp32", 128)])
def test_packed_caches_one_workgroup_decode(dtype, D):
    # few pairs, short caches: the one-workgroup form of the decode step; sequences shorter than the
    # budget (capacity n_b + e_b), a full cache from the start (e_b = 0) and capacities 0..40 rows
    # above the retained length
    lens = [700, 60, 900, 300, 96, 97, 2000]
    extras = [0, 3, 40, 17, 0, 1, 29]
    wl = small(dtype, 8, 2, D, lens, 16, 96, 5, 6, f"varcap_fused_{dtype}_{D}")
    rep = run_varcap(wl, extras, seed=51)
    assert rep["recal_heads"] > 0


@pytest.mark.parametrize("dtype,D", [("bf16", 64), ("fp32", 64), ("bf16", 128)])
def test_packed_caches_split_decode(dtype, D):
    # few pairs and caches above 2048 rows: the decode step splits the rows over workgroups (two launches)
    lens = [2600, 1000, 3100, 2101]
    extras = [5, 12, 0, 40]
    wl = small(dtype, 4, 2, D, lens, 16, 2100, 5, 3, f"varcap_split_{dtype}_{D}")
    run_varcap(wl, extras, seed=52)


@pytest.mark.parametrize("dtype,budget", [("bf16", 64), ("bf16", 600), ("fp32", 200)])
def test_packed_caches_many_sequences(dtype, budget):
    # >= 192 (sequence, KV head) pairs: one workgroup per pair with 4 or 8 waves; 100 different capacities
    rng = np.random.default_rng(budget)
    lens = rng.integers(budget // 2, 3 * budget, 100).tolist()
    extras = rng.integers(0, 41, 100).tolist()
    extras[0], extras[1] = 0, 40
    wl = small(dtype, 8, 2, 128, lens, 16, budget, 5, 3, f"varcap_many_{dtype}_{budget}")
    run_varcap(wl, extras, seed=53, seqs=[0, 1, 37, 99, int(np.argmin(lens)), int(np.argmax(lens))])


def test_packed_caches_with_calibration_size_and_llama_shape():
    lens = [2100, 513, 4099]
    extras = [7, 0, 33]
    wl = small("bf16", 32, 8, 128, lens, 32, 512, 7, 3, "varcap_llama_calib")
    run_varcap(wl, extras, seed=54, m=300)


def test_capacity_below_the_retained_length_writes_nothing():
    # a capacity smaller than min(B, n_b) breaks the contract: that sequence's rows are not written
    # (nothing may spill into the neighbour), the others are unaffected
    lens = [700, 900, 500]
    wl = small("bf16", 8, 2, 128, lens, 16, 96, 5, 1, "varcap_short_capacity")
    x = to_dev(synth.make_inputs(wl, 55))
    good = poisoned_buffers(wl, [96, 100, 99])
    good.compress(x["q_win"], x["k"], x["v"], x["seq_offsets"])
    bad = poisoned_buffers(wl, [96, 95, 99])
    bad.compress(x["q_win"], x["k"], x["v"], x["seq_offsets"])
    torch.cuda.synchronize()
    assert torch.all(bad.cache_view("k", 1) == SENTINEL) and torch.all(bad.cache_view("v", 1) == SENTINEL)
    for b in (0, 2):
        assert torch.equal(bad.cache_view("k", b)[:, :96], good.cache_view("k", b)[:, :96])
        assert torch.equal(bad.cache_view("v", b)[:, :96], good.cache_view("v", b)[:, :96])
    assert torch.equal(bad.indices, good.indices)
    # decode treats the sequence whose live length exceeds its capacity as empty
    bad.decode(x["q_dec"][0])
    torch.cuda.synchronize()
    assert torch.all(torch.isinf(bad.a_lse[1])) and torch.isfinite(bad.out.float()).all()
