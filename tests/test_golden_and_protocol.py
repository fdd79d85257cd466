"""Regression fixture of the oracle, and the tie-band protocol of the index comparison
(host logic, CPU only)."""
import json
import os

import numpy as np
import pytest

from oracle import calidrop_ref as ref
from tests import helpers as H

HERE = os.path.dirname(os.path.abspath(__file__))


def test_oracle_reproduces_golden_fixture():
    g = json.load(open(os.path.join(HERE, "golden", "tiny_case.json")))
    s = g["shapes"]
    r = ref.compress(np.array(g["q_win"]), np.array(g["K"]), np.array(g["V"]), s["w"], s["B"], s["k"])
    assert r["idx"].tolist() == g["idx"]
    np.testing.assert_allclose(np.array(r["score"]), np.array(g["score"]), rtol=1e-13)
    np.testing.assert_allclose(r["c_out"], np.array(g["c_out"]), atol=1e-13)
    np.testing.assert_allclose(r["c_lse"], np.array(g["c_lse"]), atol=1e-13)
    out, a_lse, flags, rho = ref.decode(np.array(g["q_t"]), r["K_c"], r["V_c"], s["B"], r["c_q"], r["c_out"],
                                        r["c_lse"], s["theta1"], s["theta2"])
    np.testing.assert_allclose(out, np.array(g["out"]), atol=1e-13)
    assert flags.tolist() == g["flags"]


def test_oracle_reproduces_strategy_fixture():
    g = json.load(open(os.path.join(HERE, "golden", "tiny_strategies.json")))
    s = g["shapes"]
    qf, K, V, q_t = (np.array(g[k]) for k in ("q_full", "K", "V", "q_t"))
    slm = ref.streaming_llm_retained(s["n"], s["B"], s["n_sink"])
    assert slm.tolist() == g["slm_idx"]
    rs = ref.compress_given(qf[:, -1], K, V, s["B"], [slm, slm])
    np.testing.assert_allclose(rs["c_out"], np.array(g["slm_c_out"]), atol=1e-13)
    np.testing.assert_allclose(rs["c_lse"], np.array(g["slm_c_lse"]), atol=1e-13)
    rh = ref.compress_h2o(qf, K, V, s["B"], s["n_local"])
    np.testing.assert_allclose(np.array(rh["vote"]), np.array(g["h2o_vote"]), rtol=1e-13)
    assert rh["idx"].tolist() == g["h2o_idx"]
    np.testing.assert_allclose(rh["c_out"], np.array(g["h2o_c_out"]), atol=1e-13)
    np.testing.assert_allclose(rh["c_lse"], np.array(g["h2o_c_lse"]), atol=1e-13)
    out, a_lse, flags, _ = ref.decode(q_t, rh["K_c"], rh["V_c"], s["B"], rh["c_q"], rh["c_out"], rh["c_lse"], 0.7, 0.85)
    assert flags.tolist() == g["flags"] and set(g["flags"]) == {ref.FLAG_RECOMPUTE}
    out2, flags2, _, c_out2, c_lse2 = ref.recalibrate(q_t, K, V, rh["idx"], flags, a_lse, out, rh["c_q"], rh["c_out"],
                                                      rh["c_lse"])
    np.testing.assert_allclose(out2, np.array(g["recal_out"]), atol=1e-13)
    np.testing.assert_allclose(c_out2, np.array(g["recal_c_out"]), atol=1e-13)
    np.testing.assert_allclose(c_lse2, np.array(g["recal_c_lse"]), atol=1e-13)
    assert flags2.tolist() == g["recal_flags"]


def fake_oracle(score, k_sel, w):
    P = len(score)
    sel, margin = ref.select_top(score, k_sel)
    idx = np.concatenate([sel, np.arange(P, P + w)])
    return dict(idx=idx[None], score=[np.asarray(score, float)], margin=np.array([margin]))


def test_tie_band_protocol_accepts_only_sub_rounding_swaps():
    w, k_sel = 2, 3
    # boundary between rank 3 (1.0) and rank 4 (1.0 - 2e-5): inside the bf16 band, outside the fp32 band
    score = np.array([5.0, 1.0 - 2e-5, 3.0, 1.0, 0.1, 0.2])
    orc = fake_oracle(score, k_sel, w)
    assert orc["idx"][0].tolist() == [0, 2, 3, 6, 7]
    swapped = np.array([[0, 1, 2, 6, 7]])
    rep = {}
    override = H.check_indices(swapped, orc, "bf16", k_sel, rep)
    assert rep["tie_band_heads"] == 1 and override[0].tolist() == [0, 1, 2]
    with pytest.raises(AssertionError, match="above the tie band"):
        H.check_indices(swapped, orc, "fp32", k_sel, {})
    # a swap with a position far from the boundary is never accepted, even inside the band
    wrong = np.array([[0, 2, 4, 6, 7]])
    with pytest.raises(AssertionError, match="not within the tie band"):
        H.check_indices(wrong, orc, "bf16", k_sel, {})
    # identical sets pass silently; wrong window positions or unsorted output fail
    assert H.check_indices(orc["idx"].copy(), orc, "fp32", k_sel, {}) is None
    with pytest.raises(AssertionError, match="window"):
        H.check_indices(np.array([[0, 1, 2, 6, 8]]), orc, "bf16", k_sel, {})
    with pytest.raises(AssertionError, match="ascending"):
        H.check_indices(np.array([[2, 1, 0, 6, 7]]), orc, "bf16", k_sel, {})
