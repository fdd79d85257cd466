"""Writes tests/golden/tiny_case.json: a tiny seeded compress + decode case evaluated by the
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


if __name__ == "__main__":
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "tiny_case.json")
    with open(path, "w") as f:
        json.dump(build(), f, indent=1)
    print("wrote", path)
