"""H2O as the eviction strategy (Sec. 4.1.3): the two dense scoring passes, selection, gather and
calibration state on the GPU vs the oracle, then Alg. 2 on that state.  Needs an MI355X."""
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


def check_h2o(wl, x, q_full, bufs, n_local, rep, calib=0):
    B, G = wl.budget, wl.group
    loc = n_local or B // 2
    vote_gpu = bufs.h2o_region(cd.REGION_SCORE, n_local).cpu().numpy().astype(np.float64)
    lse_gpu = bufs.h2o_region(cd.REGION_ROW_LSE, n_local).cpu().numpy().astype(np.float64)
    lse_gpu = lse_gpu.reshape(wl.batch, wl.n_q_heads, -1)
    for b, n in enumerate(wl.seq_lens):
        K = H.to64(synth.seq_view(x["k"], wl, b))
        V = H.to64(synth.seq_view(x["v"], wl, b))
        Q = H.to64(synth.seq_view_q(q_full, wl, b))
        orc = ref.compress_h2o(Q, K, V, B, loc)
        length = min(n, B)
        assert int(bufs.cache_lens[b].item()) == length
        gi = bufs.indices[b].cpu().numpy()
        assert np.all(gi[:, length:] == -1)
        if n > B:
            # scores first: they explain any index difference
            off = int(sum(wl.seq_lens[:b])) * wl.n_kv_heads
            for g in range(wl.n_kv_heads):
                s_gpu = vote_gpu[off + g * n: off + g * n + (n - loc)]      # scores of the candidates
                s_ref = orc["vote"][g][:n - loc]
                rel = np.abs(s_gpu - s_ref) / (np.abs(s_ref) + 1e-30)
                big = s_ref > 1e-9 * s_ref.max()
                rep["vote_rel_err"] = max(rep.get("vote_rel_err", 0), rel[big].max())
                assert rel[big].max() < 5e-4, f"vote relative error {rel[big].max()}"
            # row log-sum-exp of every query (log2 units) vs a dense fp64 computation
            scale = wl.head_dim ** -0.5
            for h in range(wl.n_q_heads):
                S = (Q[h] @ K[h // G].T) * scale
                S[np.triu_indices(n, 1)] = -np.inf
                want = np.log2(np.exp(S - S.max(axis=1, keepdims=True)).sum(axis=1)) + S.max(axis=1) * np.log2(np.e)
                err = np.abs(lse_gpu[b, h, :n] - want).max()
                rep["row_lse_err"] = max(rep.get("row_lse_err", 0), err)
                assert err < 2e-3 and np.all(np.isposinf(lse_gpu[b, h, n:((n + 127) // 128) * 128]))
            # retained set: bit-exact except rounding-order swaps inside the tie band
            fake = dict(idx=orc["idx"], score=[v[:n - loc] for v in orc["vote"]], margin=orc["margin"])
            override = H.check_indices(gi, fake, wl.dtype, B - loc, rep)
            if override is not None:
                full = [np.concatenate([override[g], np.arange(n - loc, n)]) for g in range(wl.n_kv_heads)]
                orc = ref.compress_h2o(Q, K, V, B, loc, retained_override=full)
        else:
            assert np.array_equal(gi[:, :length], orc["idx"])
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


@pytest.mark.parametrize("wl,n_local", [
    (small("fp32", 4, 2, 64, [700], 8, 64, 1, T=4, name="h2o_fp32_d64"), 0),
    (small("bf16", 8, 2, 128, [1100, 50, 333], 16, 128, 1, T=4, name="h2o_bf16_varlen"), 0),
    (small("bf16", 4, 4, 64, [513], 16, 100, 1, T=2, name="h2o_bf16_d64_g1"), 30),
    (small("fp32", 16, 2, 128, [400], 16, 60, 1, T=2, name="h2o_fp32_g8"), 59),
    (small("bf16", 32, 8, 128, [2050], 32, 512, 1, T=2, name="h2o_llama_shape"), 0),
    (small("bf16", 14, 2, 128, [900, 130], 16, 128, 1, T=2, name="h2o_g7"), 0),
    (small("fp32", 6, 2, 64, [611], 16, 90, 1, T=2, name="h2o_g3_fp32"), 17),
], ids=lambda v: v.name if hasattr(v, "name") else str(v))
def test_h2o_strategy(wl, n_local):
    x = to_dev(synth.make_inputs(wl, 61))
    q_full = synth.full_queries(wl, x, 61, DEV)
    p = H.params_for(wl)
    bufs = cd.CompressBuffers(p, wl.seq_lens, DEV)
    bufs.compress_h2o(q_full, x["k"], x["v"], x["seq_offsets"], n_local=n_local)
    torch.cuda.synchronize()
    rep = {}
    check_h2o(wl, x, q_full, bufs, n_local, rep)
    for t in range(wl.decode_steps):
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
    rep.pop("flags", None)
    print(wl.name, rep, flush=True)


def test_h2o_is_deterministic():
    wl = small("bf16", 8, 2, 128, [1500], 16, 128, 1, T=1, name="h2o_det")
    x = to_dev(synth.make_inputs(wl, 62))
    q_full = synth.full_queries(wl, x, 62, DEV)
    outs = []
    for _ in range(2):
        bufs = cd.CompressBuffers(H.params_for(wl), wl.seq_lens, DEV)
        bufs.compress_h2o(q_full, x["k"], x["v"], x["seq_offsets"])
        torch.cuda.synchronize()
        score = bufs.h2o_region(cd.REGION_SCORE).view(wl.n_kv_heads, 1500)[:, :1500 - 64]   # candidates only
        outs.append((bufs.indices.clone(), bufs.c_out.clone(), bufs.c_lse.clone(), score.clone()))
    for a, c in zip(*outs):
        assert torch.equal(a, c)


@pytest.fixture
def wide_selection():
    old = H.TEST_FLAGS
    H.TEST_FLAGS = old | cd.OPT_WIDE_SELECTION
    yield
    H.TEST_FLAGS = old


def test_h2o_with_multi_workgroup_selection(wide_selection):
    # the same strategy through the selection variant long prompts take (several workgroups per
    # head, per-head vote planes added by the pooling kernel), at a size the oracle can follow
    wl = small("bf16", 8, 2, 128, [9000, 300], 16, 256, 1, T=2, name="h2o_wide")
    x = to_dev(synth.make_inputs(wl, 63))
    q_full = synth.full_queries(wl, x, 63, DEV)
    bufs = cd.CompressBuffers(H.params_for(wl, calib_size=700), wl.seq_lens, DEV)
    bufs.compress_h2o(q_full, x["k"], x["v"], x["seq_offsets"])
    torch.cuda.synchronize()
    # same lists as the single-workgroup variant
    twin = cd.CompressBuffers(H.params_for(wl, calib_size=700, flags=cd.OPT_WRITE_SCORES), wl.seq_lens, DEV)
    twin.compress_h2o(q_full, x["k"], x["v"], x["seq_offsets"])
    torch.cuda.synchronize()
    assert torch.equal(bufs.indices, twin.indices) and torch.equal(bufs.cal_indices, twin.cal_indices)
    assert torch.equal(bufs.k_c, twin.k_c) and torch.equal(bufs.c_out, twin.c_out)
    # and the oracle on the retained set (calibration state is over the 700 best evicted tokens)
    n, B = 9000, 256
    K = H.to64(synth.seq_view(x["k"], wl, 0)); V = H.to64(synth.seq_view(x["v"], wl, 0))
    Q = H.to64(synth.seq_view_q(q_full, wl, 0))
    orc = ref.compress_h2o(Q, K, V, B, B // 2)
    rep = {}
    fake = dict(idx=orc["idx"], score=[v[:n - B // 2] for v in orc["vote"]], margin=orc["margin"])
    assert H.check_indices(bufs.indices[0].cpu().numpy(), fake, wl.dtype, B - B // 2, rep) is None
    cal = bufs.cal_indices[0].cpu().numpy()
    for g in range(2):
        ev = orc["evicted"][g]
        ev = ev[ev < n - B // 2]
        order = np.argsort(-orc["vote"][g][ev], kind="stable")[:700]
        assert np.array_equal(cal[g], np.sort(ev[order]))


@pytest.mark.parametrize("dtype", ["fp32", "bf16"])
def test_h2o_rows_whose_logits_outgrow_the_reference(dtype):
    # pass 1 sums exp2(s - m) against the logit of key 0 and only falls back to the true row maximum
    # when a sum outgrows 2^64: a tiny key 0 and a few huge later keys force that fallback (and
    # fp32 overflow of the first attempt) on many rows
    wl = small(dtype, 4, 2, 128, [900], 16, 64, 1, T=1, name=f"h2o_huge_logits_{dtype}")
    x = synth.make_inputs(wl, 64)
    K = synth.seq_view(x["k"], wl, 0)
    K[:, 0] *= 0.01
    K[:, 300] *= 10.0
    K[:, 640] *= 25.0
    x = to_dev(x)
    q_full = synth.full_queries(wl, x, 64, DEV)
    bufs = cd.CompressBuffers(H.params_for(wl), wl.seq_lens, DEV)
    bufs.compress_h2o(q_full, x["k"], x["v"], x["seq_offsets"])
    torch.cuda.synchronize()
    rep = {}
    check_h2o(wl, x, q_full, bufs, 0, rep)
    lse = bufs.h2o_region(cd.REGION_ROW_LSE).view(wl.n_q_heads, -1)[:, :900]
    assert torch.isfinite(lse).all() and float(lse.max()) > 150.0       # log2 units: far beyond 64 above key 0
    print(wl.name, rep, float(lse.max()), flush=True)
