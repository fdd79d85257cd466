"""Shared test plumbing: run the HIP path through the C ABI, run the oracle on the same arrays,
compare with the stated tolerances and the tie-band protocol for retained indices."""
from __future__ import annotations

import numpy as np
import torch

from oracle import calidrop_ref as ref
from paper_2507_19906_amd import binding as cd
from paper_2507_19906_amd import synth

# tolerances (max-abs): outputs per dtype as the targets state; log-sum-exp values are fp32
# reductions of exact products, far tighter than the outputs
TOL_OUT = {"bf16": 2e-2, "fp32": 1e-4}
TOL_LSE = {"bf16": 2e-3, "fp32": 1e-4}
# relative boundary margin below which a retained-set difference is a rounding-order swap
TIE_BAND = {"bf16": 1e-4, "fp32": 1e-5}


# per-call options every test's params carry unless it says otherwise: the parity checks read the
# pooled scores; the `wide_selection` fixtures add OPT_WIDE_SELECTION for the duration of a test
TEST_FLAGS = cd.OPT_WRITE_SCORES


def params_for(wl: synth.Workload, **over) -> cd.Params:
    kw = dict(flags=TEST_FLAGS, dtype=wl.dtype, batch=wl.batch, n_q_heads=wl.n_q_heads, n_kv_heads=wl.n_kv_heads,
              head_dim=wl.head_dim, window=wl.window, budget=wl.budget, pool_kernel=wl.pool_kernel,
              theta1=wl.theta1, theta2=wl.theta2)
    kw.update(over)
    return cd.make_params(**kw)


def to64(t: torch.Tensor) -> np.ndarray:
    return t.detach().to("cpu").to(torch.float64).numpy()


def gpu_compress(wl, x, q_cal=None, extra_capacity=0, win_lse=None, **over):
    """x: dict from synth.make_inputs already on the GPU.  Returns CompressBuffers."""
    p = params_for(wl, **over)
    dev = x["k"].device
    bufs = cd.CompressBuffers(p, wl.seq_lens, dev, extra_capacity=extra_capacity)
    bufs.compress(x["q_win"], x["k"], x["v"], x["seq_offsets"], q_cal=q_cal, win_lse=win_lse)
    torch.cuda.synchronize()
    return bufs


def oracle_compress(wl, x, b, heads=None, q_cal=None, override=None, budget=None, pool_kernel=None,
                    calib_size=0, win_lse=None):
    """Oracle compress of sequence b (optionally only the KV heads in `heads`)."""
    G = wl.group
    heads = list(range(wl.n_kv_heads)) if heads is None else list(heads)
    K = to64(synth.seq_view(x["k"], wl, b)[heads])          # only the sampled heads leave the device
    V = to64(synth.seq_view(x["v"], wl, b)[heads])
    qh = [g * G + j for g in heads for j in range(G)]
    q_win = to64(x["q_win"][b][qh])
    qc = None if q_cal is None else to64(q_cal[b])[qh]
    lse = None if win_lse is None else to64(win_lse[b])[qh]
    return ref.compress(q_win, K, V, wl.window, budget or wl.budget, pool_kernel or wl.pool_kernel,
                        q_cal=qc, retained_override=override, calib_size=calib_size, win_lse=lse)


def check_indices(gpu_idx: np.ndarray, orc: dict, dtype: str, k_sel: int, report: dict):
    """Bit-exact retained indices, except for rounding-order swaps inside the tie band, which
    are counted in `report` and must involve only positions whose oracle score lies within the
    band of the boundary value.  Returns per-head override lists when a swap happened."""
    tau = TIE_BAND[dtype]
    override = None
    for g in range(gpu_idx.shape[0]):
        want = orc["idx"][g]
        got = gpu_idx[g][:len(want)]
        if np.array_equal(got, want):
            continue
        assert orc["score"][g] is not None, "index mismatch without eviction"
        assert np.all(np.diff(got) > 0), f"head {g}: indices not ascending"
        assert np.array_equal(got[k_sel:], want[k_sel:]), f"head {g}: window positions differ"
        score = orc["score"][g]
        srt = np.sort(score)[::-1]
        boundary = srt[k_sel - 1]
        diff = np.setxor1d(got[:k_sel], want[:k_sel])
        assert orc["margin"][g] < tau, (
            f"head {g}: retained set differs ({len(diff)} positions) although the boundary margin "
            f"{orc['margin'][g]:.3e} is above the tie band {tau}")
        assert np.all(np.abs(score[diff] - boundary) <= tau * boundary), (
            f"head {g}: swapped positions are not within the tie band of the boundary")
        report["tie_band_heads"] = report.get("tie_band_heads", 0) + 1
        if override is None:
            override = [orc["idx"][gg][:k_sel] for gg in range(gpu_idx.shape[0])]
        override[g] = got[:k_sel]
    return override


def check_calibration_set(gpu_cal, orc, dtype, k_sel, m, report):
    """The calibration set (Sec. 5.3 calibration size) per head: exact, except rounding-order
    swaps at its own rank boundary (same tie-band rule as the retained set).  Returns the lists
    to evaluate the calibration state with (the GPU's when a swap happened)."""
    tau = TIE_BAND[dtype]
    lists = []
    for g in range(gpu_cal.shape[0]):
        want = orc["evicted"][g]
        got = gpu_cal[g]
        assert np.all(got[len(want):] == -1), f"head {g}: calibration list not padded with -1"
        got = got[:len(want)]
        if not np.array_equal(got, want):
            assert np.all(np.diff(got) > 0) and len(set(got) & set(orc["idx"][g])) == 0
            score = orc["score"][g]
            cand = np.sort(np.delete(score, orc["idx"][g][:k_sel]))[::-1]      # evicted tokens' scores
            boundary, nxt = cand[m - 1], cand[m]
            assert (boundary - nxt) / boundary < tau, f"head {g}: calibration set differs outside the tie band"
            diff = np.setxor1d(got, want)
            assert np.all(np.abs(score[diff] - boundary) <= tau * boundary)
            report["tie_band_cal_heads"] = report.get("tie_band_cal_heads", 0) + 1
        lists.append(got)
    return lists


def check_compress(wl, x, bufs, b, heads=None, q_cal=None, report=None, check_scores=True, win_lse=None):
    """Compare everything calidrop_compress wrote for sequence b against the oracle."""
    report = {} if report is None else report
    dt = wl.dtype
    G, B, w = wl.group, wl.budget, wl.window
    n = wl.seq_lens[b]
    heads = list(range(wl.n_kv_heads)) if heads is None else list(heads)
    m = int(bufs.p.calib_size)
    orc = oracle_compress(wl, x, b, heads, q_cal, calib_size=m, win_lse=win_lse)
    length = min(B, n)
    assert int(bufs.cache_lens[b].item()) == length
    gpu_idx = bufs.indices[b].cpu().numpy()[heads]
    if n < B:
        assert np.all(gpu_idx[:, n:] == -1)
    override = check_indices(gpu_idx, orc, dt, B - w, report)
    if override is not None:        # evaluate downstream values for the GPU's retained set
        orc = oracle_compress(wl, x, b, heads, q_cal, override=override, calib_size=m, win_lse=win_lse)
    if m > 0:
        gpu_cal = bufs.cal_indices[b].cpu().numpy()[heads]
        if n <= B:
            assert np.all(gpu_cal == -1)
        else:
            lists = check_calibration_set(gpu_cal, orc, dt, B - w, m, report)
            if any(not np.array_equal(lists[j], orc["evicted"][j]) for j in range(len(heads))):
                Kh = to64(synth.seq_view(x["k"], wl, b)[heads])
                Vh = to64(synth.seq_view(x["v"], wl, b)[heads])
                _, orc["c_out"], orc["c_lse"] = ref.calibration_state(orc["c_q"], Kh, Vh, lists, G, wl.head_dim ** -0.5)
    # gathered rows are copies: bit-exact
    Kc = to64(bufs.cache_view("k", b)[heads][:, :length])
    Vc = to64(bufs.cache_view("v", b)[heads][:, :length])
    assert np.array_equal(Kc, orc["K_c"]) and np.array_equal(Vc, orc["V_c"])
    qh = [g * G + j for g in heads for j in range(G)]
    c_q, c_out, c_lse = (to64(bufs.c_q[b])[qh], to64(bufs.c_out[b])[qh], to64(bufs.c_lse[b])[qh])
    assert np.array_equal(c_q, orc["c_q"])
    if n <= B:
        assert np.all(c_lse == -np.inf) and np.all(c_out == 0)
    else:
        err_o = np.abs(c_out - orc["c_out"]).max()
        err_l = np.abs(c_lse - orc["c_lse"]).max()
        report["c_out_err"] = max(report.get("c_out_err", 0), err_o)
        report["c_lse_err"] = max(report.get("c_lse_err", 0), err_l)
        assert err_o <= TOL_OUT[dt], f"c_out max-abs error {err_o}"
        assert err_l <= TOL_LSE[dt], f"c_lse max-abs error {err_l}"
        if check_scores and (bufs.p.flags & cd.OPT_WRITE_SCORES):
            score = bufs.region(cd.REGION_SCORE)
            off = int(sum(wl.seq_lens[:b])) * wl.n_kv_heads
            for j, g in enumerate(heads):
                # only the prefix positions are written: slice before leaving the device
                s_gpu = score[off + g * n: off + g * n + (n - w)].cpu().numpy().astype(np.float64)
                s_ref = orc["score"][j]
                rel = np.abs(s_gpu - s_ref) / (np.abs(s_ref) + 1e-30)
                big = s_ref > 1e-12 * s_ref.max()
                report["score_rel_err"] = max(report.get("score_rel_err", 0), rel[big].max())
                assert rel[big].max() < 5e-4, f"pooled score relative error {rel[big].max()}"
    return orc, report


def oracle_state_from_gpu(wl, bufs, b, heads=None):
    """Compressed cache and calibration state as the GPU produced them, widened to fp64, so
    that decode parity is judged on identical inputs."""
    G = wl.group
    heads = list(range(wl.n_kv_heads)) if heads is None else list(heads)
    qh = [g * G + j for g in heads for j in range(G)]
    return dict(K_c=to64(bufs.cache_view("k", b)[heads]), V_c=to64(bufs.cache_view("v", b)[heads]),
                c_q=to64(bufs.c_q[b])[qh], c_out=to64(bufs.c_out[b])[qh],
                c_lse=to64(bufs.c_lse[b])[qh], qh=qh)


def check_decode_step(wl, bufs, q_t, b, heads=None, theta=None, report=None, length=None,
                      rho_guard=1e-5):
    """One decode step already executed on the GPU (bufs.out/a_lse/flags) vs the oracle run on
    the same cache and calibration state."""
    report = {} if report is None else report
    dt = wl.dtype
    st = oracle_state_from_gpu(wl, bufs, b, heads)
    th = theta if theta is not None else (wl.theta1, wl.theta2)
    length = int(bufs.cache_lens[b].item()) if length is None else length
    q = to64(q_t[b])[st["qh"]]
    out, a_lse, flags, rho = ref.decode(q, st["K_c"], st["V_c"], length, st["c_q"], st["c_out"],
                                        st["c_lse"], th[0], th[1])
    g_out = to64(bufs.out[b])[st["qh"]]
    g_lse = to64(bufs.a_lse[b])[st["qh"]]
    g_flags = bufs.flags[b].cpu().numpy()[st["qh"]]
    # the gate is decided in fp32 on both sides; only compare flags where rho is not within
    # rounding distance of a threshold
    near = np.zeros_like(rho, bool)
    for t in th:
        if np.isfinite(t):
            near |= np.abs(rho - t) < rho_guard
    assert np.array_equal(g_flags[~near], flags[~near]), (g_flags, flags, rho)
    same = g_flags == flags
    err = np.abs(g_out - out)[same].max() if same.any() else 0.0
    fin = np.isfinite(a_lse)
    err_l = np.abs(g_lse - a_lse)[fin].max() if fin.any() else 0.0
    assert np.array_equal(np.isfinite(g_lse), fin)
    report["out_err"] = max(report.get("out_err", 0), err)
    report["a_lse_err"] = max(report.get("a_lse_err", 0), err_l)
    report.setdefault("flags", []).extend(g_flags.tolist())
    assert err <= TOL_OUT[dt], f"decode out max-abs error {err}"
    assert err_l <= TOL_LSE[dt], f"a_lse max-abs error {err_l}"
    return report


def check_recalibrate(wl, x, bufs, q_t, b, before, heads=None, report=None):
    """The recomputation branch just executed on the GPU (bufs updated in place) vs the oracle's
    Alg. 2 steps 3-8 applied to the state `before` = dict(out, a_lse, flags, c_q, c_out, c_lse)
    that the GPU held after decode (all widened to fp64)."""
    report = {} if report is None else report
    dt = wl.dtype
    G = wl.group
    heads = list(range(wl.n_kv_heads)) if heads is None else list(heads)
    qh = [g * G + j for g in heads for j in range(G)]
    K = to64(synth.seq_view(x["k"], wl, b)[heads])
    V = to64(synth.seq_view(x["v"], wl, b)[heads])
    idx = bufs.indices[b].cpu().numpy()[heads]
    cal_idx = bufs.cal_indices[b].cpu().numpy()[heads] if bufs.p.calib_size > 0 else None
    out, flags, c_q, c_out, c_lse = ref.recalibrate(
        to64(q_t[b])[qh], K, V, idx, before["flags"][b][qh], before["a_lse"][b][qh], before["out"][b][qh],
        before["c_q"][b][qh], before["c_out"][b][qh], before["c_lse"][b][qh], cal_idx=cal_idx)
    g_flags = bufs.flags[b].cpu().numpy()[qh]
    assert np.array_equal(g_flags, flags), (g_flags, flags)
    g_out, g_cq = to64(bufs.out[b])[qh], to64(bufs.c_q[b])[qh]
    g_co, g_cl = to64(bufs.c_out[b])[qh], to64(bufs.c_lse[b])[qh]
    assert np.array_equal(g_cq, c_q)
    fin = np.isfinite(c_lse)
    assert np.array_equal(np.isfinite(g_cl), fin)
    e_out, e_co = np.abs(g_out - out).max(), np.abs(g_co - c_out).max()
    e_cl = np.abs(g_cl - c_lse)[fin].max() if fin.any() else 0.0
    report["recal_out_err"] = max(report.get("recal_out_err", 0), e_out)
    report["recal_c_out_err"] = max(report.get("recal_c_out_err", 0), e_co)
    report["recal_c_lse_err"] = max(report.get("recal_c_lse_err", 0), e_cl)
    report["recal_heads"] = report.get("recal_heads", 0) + int((flags == ref.FLAG_RECOMPUTED).sum())
    assert e_out <= TOL_OUT[dt] and e_co <= TOL_OUT[dt] and e_cl <= TOL_LSE[dt], (e_out, e_co, e_cl)
    return report


def snapshot_state(bufs):
    """fp64 host copies of everything calidrop_recalibrate reads or updates."""
    return dict(out=to64(bufs.out), a_lse=to64(bufs.a_lse), flags=bufs.flags.cpu().numpy().copy(),
                c_q=to64(bufs.c_q), c_out=to64(bufs.c_out), c_lse=to64(bufs.c_lse))
