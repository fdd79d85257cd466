"""Full-size workloads in the launch configuration the benchmark times, checked on sampled
(sequence, KV head) pairs that the oracle can afford.  Needs an MI355X."""
import numpy as np
import pytest
import torch

from paper_2507_19906_amd import binding as cd
from paper_2507_19906_amd import synth
from tests import helpers as H

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def sampled(wl, samples, decode_steps=2, seed=synth.BASE_SEED, capacities=None, recalibrate=False):
    """samples: (sequence, KV head) pairs checked against the oracle; everything else gets the
    properties that hold for every pair.  `capacities`: per-sequence cache capacities (packed caches
    behind an offsets array) instead of one capacity for all."""
    x = synth.make_inputs(wl, seed, device=DEV)
    bufs = cd.CompressBuffers(H.params_for(wl), wl.seq_lens, DEV, capacities=capacities)
    bufs.compress(x["q_win"], x["k"], x["v"], x["seq_offsets"])
    torch.cuda.synchronize()
    by_seq = {}
    for b, g in samples:
        by_seq.setdefault(b, []).append(g)
    rep = {}
    for b, heads in by_seq.items():
        H.check_compress(wl, x, bufs, b, heads=heads, report=rep)
    for t in range(decode_steps):
        q_t = x["q_dec"][t]
        bufs.decode(q_t)
        torch.cuda.synchronize()
        for b, heads in by_seq.items():
            H.check_decode_step(wl, bufs, q_t, b, heads=heads, report=rep)
        if recalibrate:                      # Alg. 2 complete: the state is carried on the GPU from step to step
            before = H.snapshot_state(bufs)
            bufs.recalibrate(q_t, x["k"], x["v"], x["seq_offsets"])
            torch.cuda.synchronize()
            for b, heads in by_seq.items():
                H.check_recalibrate(wl, x, bufs, q_t, b, before, heads=heads, report=rep)
            assert not torch.any(bufs.flags == cd.FLAG_RECOMPUTE)
    # properties that hold for every (sequence, head), checked on all of them
    idx = bufs.indices.cpu().numpy()
    lens_gpu = bufs.cache_lens.cpu().numpy()
    for b, n in enumerate(wl.seq_lens):
        L = min(wl.budget, n)
        assert int(lens_gpu[b]) == L
        assert np.all(np.diff(idx[b, :, :L], axis=1) > 0)
        if n > wl.budget:
            assert np.array_equal(idx[b, :, L - wl.window:L],
                                  np.tile(np.arange(n - wl.window, n), (wl.n_kv_heads, 1)))
            assert np.all(idx[b, :, 0] >= 0) and np.all(idx[b, :, L - 1] == n - 1)
    assert torch.isfinite(bufs.c_out).all() and torch.isfinite(bufs.out.float()).all()
    flags = np.bincount(rep.pop("flags"), minlength=4).tolist()
    print(wl.name, f"{len(samples)} (sequence, KV head) pairs x {decode_steps} decode steps;",
          "tie-band heads:", rep.get("tie_band_heads", 0), "| flags [none, calibrated, recompute, recomputed]:", flags,
          "|", {k: float(v) for k, v in rep.items()}, flush=True)
    return rep


def spread(n_seq, n_heads, count):
    """`count` sequences spread over the batch, each with a different KV head: every head is covered
    when count >= n_heads."""
    seqs = sorted({int(round(i * (n_seq - 1) / max(count - 1, 1))) for i in range(count)})
    return [(b, (3 * i + 1) % n_heads) for i, b in enumerate(seqs)]


def test_config3_stack_32_layers_budget_512():
    # 16 layers with all their 8 KV heads (128 of the 256 pairs), and more layers with one head each
    wl = synth.config(3, layers=32, budget=512, decode_steps=8)
    full_layers = list(range(0, 32, 2))
    samples = [(b, g) for b in full_layers for g in range(8)] + [(b, g) for b, g in spread(32, 8, 12) if b not in full_layers]
    sampled(wl, samples, decode_steps=8)


@pytest.mark.parametrize("budget", [128, 2048])
def test_config3_other_budgets(budget):
    # the stack bench.py times these budgets on: 4 layers with all their KV heads, 10 more with one each
    wl = synth.config(3, layers=32, budget=budget, decode_steps=4)
    full = [(b, g) for b in (1, 12, 20, 30) for g in range(8)]
    sampled(wl, full + [s for s in spread(32, 8, 10) if s[0] not in (1, 12, 20, 30)], decode_steps=4)


def test_config3_decode_and_recomputation_loop():
    # the stateful loop of Alg. 2 at full size: 16 steps of decode + recomputation branch over the whole
    # 32-layer stack, the state of the sampled heads checked against the oracle at every step
    wl = synth.config(3, layers=32, budget=512, decode_steps=16)
    rep = sampled(wl, spread(32, 8, 8), decode_steps=16, recalibrate=True)
    assert rep["recal_heads"] > 0


def test_config2_decode_and_recomputation_loop_all_heads():
    # one 8k-context layer, all 8 KV heads, 24 steps of Alg. 2 with the state carried on the GPU
    wl = synth.config(2, decode_steps=24)
    rep = sampled(wl, [(0, g) for g in range(8)], decode_steps=24, recalibrate=True)
    assert rep["recal_heads"] > 0


def test_config4_batch64_varlen():
    # the batched workload as stated: variable-length retained caches laid out contiguously behind an
    # offsets array (capacity = budget + 0..40 rows per sequence); shortest, longest and 14 other
    # sequences, all 8 KV heads of each
    wl = synth.config(4, decode_steps=4)
    lens = wl.seq_lens
    rng = np.random.default_rng(4)
    caps = [min(wl.budget, n) + int(e) for n, e in zip(lens, rng.integers(0, 41, len(lens)))]
    b_short, b_long = int(np.argmin(lens)), int(np.argmax(lens))
    seqs = sorted({b_short, b_long} | set(range(0, 64, 9)) | {5, 17, 26, 33, 41, 50, 58})
    sampled(wl, [(b, g) for b in seqs for g in range(8)], decode_steps=4, capacities=caps)


def test_config4_uniform_capacity_without_offsets():
    # the same workload with one capacity for all: decode takes the form without the offsets array
    wl = synth.config(4, decode_steps=2)
    sampled(wl, spread(64, 8, 8), decode_steps=2)


def test_config5_long_context_131k():
    # all 8 KV heads; the selection runs as the multi-workgroup chain (prefix > 32768)
    wl = synth.config(5, decode_steps=6)
    sampled(wl, [(0, g) for g in range(8)], decode_steps=6, recalibrate=True)


def test_h2o_one_layer_32k_properties_and_samples():
    # H2O strategy at the benchmark's shape (one 32k-context layer).  The oracle cannot follow a
    # dense 32k x 32k pass, so: sampled rows of pass 1 and the last columns of pass 2 against the
    # oracle, conservation of probability mass over all columns, and the selection checked
    # against a brute-force ranking of the scores the GPU itself reports.
    from oracle import calidrop_ref as ref
    wl = synth.config(3, layers=1, budget=512, decode_steps=1)
    n, G, D, B = wl.seq_lens[0], wl.group, wl.head_dim, wl.budget
    loc = B // 2
    x = synth.make_inputs(wl, synth.BASE_SEED, device=DEV)
    q_full = synth.full_queries(wl, x, synth.BASE_SEED, DEV)
    bufs = cd.CompressBuffers(H.params_for(wl), wl.seq_lens, DEV)
    bufs.compress_h2o(q_full, x["k"], x["v"], x["seq_offsets"])
    torch.cuda.synchronize()
    lse = bufs.h2o_region(cd.REGION_ROW_LSE).view(wl.n_q_heads, -1).cpu().numpy().astype(np.float64)
    planes = bufs.h2o_region(cd.REGION_VOTE_PLANES).view(G, wl.n_kv_heads, n).cpu().numpy().astype(np.float64)
    score = bufs.h2o_region(cd.REGION_SCORE).view(wl.n_kv_heads, n).cpu().numpy()
    scale = D ** -0.5
    Q = synth.seq_view_q(q_full, wl, 0)
    K = synth.seq_view(x["k"], wl, 0)
    rng = np.random.default_rng(7)
    # pass 1: row log-sum-exp (log2 units) of sampled rows
    for h in (0, 13, 31):
        Kg = H.to64(K[h // G])
        for i in [0, 1, 127, 128, 4095, 20000, n - 1] + rng.integers(0, n, 5).tolist():
            z = ref.logits(H.to64(Q[h, i]), Kg[:i + 1], scale)
            want = (z.max() + np.log(np.exp(z - z.max()).sum())) * np.log2(np.e)
            assert abs(lse[h, i] - want) < 2e-3, (h, i, lse[h, i], want)
    # pass 2: the last 48 columns of one KV head (only the rows at or after them contribute)
    g = 5
    Kg = H.to64(K[g])
    want = np.zeros(48)
    for hh in range(G):
        Qh = H.to64(Q[g * G + hh, n - 48:])
        for r in range(48):
            i = n - 48 + r
            z = ref.logits(Qh[r], Kg[:i + 1], scale)
            p = np.exp(z - z.max()); p /= p.sum()
            want[:r + 1] += p[n - 48:i + 1]
    got = planes[:, g, n - 48:].sum(axis=0)
    assert np.abs(got - want).max() / want.max() < 5e-4
    # conservation: every query row hands out probability 1
    tot = planes.sum(axis=2)                                       # [G][Hkv]
    assert np.abs(tot / n - 1.0).max() < 1e-4, tot / n
    # the reported scores are the plane sums, and the retained set is their exact top-k
    idx = bufs.indices[0].cpu().numpy()
    for g in range(wl.n_kv_heads):
        s = score[g, :n - loc]
        ps = planes[0, g].astype(np.float32)
        for hh in range(1, G):
            ps = ps + planes[hh, g].astype(np.float32)
        assert np.array_equal(s, ps[:n - loc])
        order = np.lexsort((np.arange(n - loc), -s.astype(np.float64)))[:B - loc]
        assert np.array_equal(idx[g, :B - loc], np.sort(order))
        assert np.array_equal(idx[g, B - loc:], np.arange(n - loc, n))
    assert torch.isfinite(bufs.c_out).all() and torch.isfinite(bufs.c_lse).all()
