"""Writes tests/golden/tiny_case.json and tiny_strategies.json: tiny seeded cases evaluated by the
oracle alone (no HIP code is involved).  The paper prints no worked numeric example for this
path, so this fixture is a regression guard for the oracle, not a value from the paper; the
oracle itself is pinned by tests/test_oracle_pins.py.  Run: python tests/golden/make_golden.py"""
import json
import os
import sys

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)
from oracle import calidrop_ref as ref  # noqa: E402


def build():
    rng = np.random.default_rng(20250719)
    Hq, Hkv, D, n, w, B, k = 4, 2, 8, 24, 4, 10, 3
    # values on a coarse grid so that the JSON text reproduces them exactly
    q_win = np.round(rng.standard_normal((Hq, w, D)) * 4) / 4
    K = np.round(rng.standard_normal((Hkv, n, D)) * 4) / 4
    V = np.round(rng.standard_normal((Hkv, n, D)) * 4) / 4
    K[:, 0] *= 3
    q_t = np.round((q_win[:, -1] * 0.9 + 0.3 * rng.standard_normal((Hq, D))) * 4) / 4
    r = ref.compress(q_win, K, V, w, B, k)
    out, a_lse, flags, rho = ref.decode(q_t, r["K_c"], r["V_c"], B, r["c_q"], r["c_out"], r["c_lse"], 0.7, 0.85)
    return dict(
        shapes=dict(Hq=Hq, Hkv=Hkv, D=D, n=n, w=w, B=B, k=k, theta1=0.7, theta2=0.85),
        q_win=q_win.tolist(), K=K.tolist(), V=V.tolist(), q_t=q_t.tolist(),
        idx=r["idx"].tolist(), score=[s.tolist() for s in r["score"]],
        c_out=r["c_out"].tolist(), c_lse=r["c_lse"].tolist(),
        out=out.tolist(), a_lse=a_lse.tolist(), flags=flags.tolist(), rho=rho.tolist())


def build_strategies():
    """The same tiny tensors through the other strategies: StreamingLLM list, H2O votes and
    retained set, Alg. 1 on top of both, and one recomputation step (Alg. 2 steps 3-8)."""
    rng = np.random.default_rng(20250720)
    Hq, Hkv, D, n, B = 4, 2, 8, 24, 10
    q_full = np.round(rng.standard_normal((Hq, n, D)) * 4) / 4
    K = np.round(rng.standard_normal((Hkv, n, D)) * 4) / 4
    V = np.round(rng.standard_normal((Hkv, n, D)) * 4) / 4
    K[:, 0] *= 3
    q_t = np.round(-q_full[:, -1] * 4) / 4                       # rho = -1: every head recomputes
    slm = ref.streaming_llm_retained(n, B, 3)
    rs = ref.compress_given(q_full[:, -1], K, V, B, [slm, slm])
    rh = ref.compress_h2o(q_full, K, V, B, B // 2)
    out, a_lse, flags, _ = ref.decode(q_t, rh["K_c"], rh["V_c"], B, rh["c_q"], rh["c_out"], rh["c_lse"], 0.7, 0.85)
    out2, flags2, c_q2, c_out2, c_lse2 = ref.recalibrate(q_t, K, V, rh["idx"], flags, a_lse, out, rh["c_q"],
                                                         rh["c_out"], rh["c_lse"])
    return dict(
        shapes=dict(Hq=Hq, Hkv=Hkv, D=D, n=n, B=B, n_sink=3, n_local=B // 2),
        q_full=q_full.tolist(), K=K.tolist(), V=V.tolist(), q_t=q_t.tolist(),
        slm_idx=slm.tolist(), slm_c_out=rs["c_out"].tolist(), slm_c_lse=rs["c_lse"].tolist(),
        h2o_vote=[v.tolist() for v in rh["vote"]], h2o_idx=rh["idx"].tolist(),
        h2o_c_out=rh["c_out"].tolist(), h2o_c_lse=rh["c_lse"].tolist(),
        flags=flags.tolist(), recal_out=out2.tolist(), recal_flags=flags2.tolist(),
        recal_c_out=c_out2.tolist(), recal_c_lse=c_lse2.tolist())


if __name__ == "__main__":
    here = os.path.dirname(os.path.abspath(__file__))
    for name, fn in (("tiny_case.json", build), ("tiny_strategies.json", build_strategies)):
        path = os.path.join(here, name)
        with open(path, "w") as f:
            json.dump(fn(), f, indent=1)
        print("wrote", path)
