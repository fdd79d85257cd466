"""Pins for the fp64 oracle: closed forms, invariants the paper states, library routines and
brute force.  None of these retype the oracle's own formulas; each is chosen so that a
plausible mistake in the oracle (dropped term, wrong sign / index, transposed operand, wrong
mask or pad rule) makes at least one of them fail.  CPU only."""
import itertools

import numpy as np
import pytest
import torch
from scipy.special import logsumexp

from oracle import calidrop_ref as ref

RNG = np.random.default_rng(12345)


def rand_case(Hq=4, Hkv=2, D=8, n=40, w=4, heavy=True, rng=RNG):
    q_win = rng.standard_normal((Hq, w, D))
    K = rng.standard_normal((Hkv, n, D))
    V = rng.standard_normal((Hkv, n, D))
    if heavy:
        K[:, 0] *= 3.0
        K[:, 5] *= 2.5
    return q_win, K, V


def sdpa64(q, K, V, scale):
    """Library attention (torch scaled_dot_product_attention, float64, CPU) for one query."""
    qt = torch.from_numpy(np.asarray(q, np.float64)).view(1, 1, 1, -1)
    Kt = torch.from_numpy(np.asarray(K, np.float64)).unsqueeze(0).unsqueeze(0)
    Vt = torch.from_numpy(np.asarray(V, np.float64)).unsqueeze(0).unsqueeze(0)
    o = torch.nn.functional.scaled_dot_product_attention(qt, Kt, Vt, scale=float(scale))
    return o.view(-1).numpy()


# ---- attention + Eq. 1-2 -------------------------------------------------------------------
def test_attention_matches_library_sdpa():
    q = RNG.standard_normal(16)
    K = RNG.standard_normal((33, 16))
    V = RNG.standard_normal((33, 16))
    out, lse = ref.attention(q, K, V, 0.25)
    np.testing.assert_allclose(out, sdpa64(q, K, V, 0.25), rtol=0, atol=1e-13)
    np.testing.assert_allclose(lse, logsumexp(0.25 * K @ q), rtol=0, atol=1e-13)


def test_attention_two_keys_closed_form():
    # two keys: the weight of key 0 is the logistic function of the logit difference
    q = np.array([1.0, 2.0])
    K = np.array([[0.5, -1.0], [2.0, 0.25]])
    V = np.array([[1.0, 0.0], [0.0, 1.0]])
    s = 0.7
    z0, z1 = s * (0.5 - 2.0), s * (2.0 + 0.5)
    w0 = 1.0 / (1.0 + np.exp(z1 - z0))
    out, lse = ref.attention(q, K, V, s)
    np.testing.assert_allclose(out, [w0, 1.0 - w0], atol=1e-15)
    np.testing.assert_allclose(lse, np.log(np.exp(z0) + np.exp(z1)), atol=1e-14)


def test_attention_empty_set():
    out, lse = ref.attention(np.ones(4), np.zeros((0, 4)), np.zeros((0, 4)), 0.5)
    assert lse == -np.inf and np.all(out == 0)


def test_eq1_merge_of_any_partition_is_full_attention():
    # Eq. 1 with proof (Sec. 3.1.2): exact for any disjoint partition
    q = RNG.standard_normal(16)
    K = RNG.standard_normal((50, 16)) * 2
    V = RNG.standard_normal((50, 16))
    full = sdpa64(q, K, V, 0.25)
    for trial in range(5):
        mask = RNG.random(50) < 0.3
        oi, li = ref.attention(q, K[mask], V[mask], 0.25)
        oj, lj = ref.attention(q, K[~mask], V[~mask], 0.25)
        out, lse = ref.merge(oi, li, oj, lj)
        np.testing.assert_allclose(out, full, atol=1e-13)
        np.testing.assert_allclose(lse, logsumexp(0.25 * K @ q), atol=1e-13)
        ai, aj = ref.merge_weights(li, lj)
        assert abs(ai + aj - 1.0) < 1e-15 and 0 <= aj <= 1          # alpha_i + alpha_j = 1
        # Eq. 2 literally: ratio of exponential sums
        z = 0.25 * K @ q
        np.testing.assert_allclose(ai, np.exp(z[mask]).sum() / np.exp(z).sum(), rtol=1e-12)


def test_merge_three_way_split_equals_one_pass():
    # splitting the evicted set and merging halves by Eq. 1 == one pass
    q = RNG.standard_normal(8)
    K = RNG.standard_normal((30, 8))
    V = RNG.standard_normal((30, 8))
    o1, l1 = ref.attention(q, K[:7], V[:7], 0.3)
    o2, l2 = ref.attention(q, K[7:19], V[7:19], 0.3)
    o3, l3 = ref.attention(q, K[19:], V[19:], 0.3)
    o12, l12 = ref.merge(o1, l1, o2, l2)
    o, l = ref.merge(o12, l12, o3, l3)
    of, lf = ref.attention(q, K, V, 0.3)
    np.testing.assert_allclose(o, of, atol=1e-14)
    np.testing.assert_allclose(l, lf, atol=1e-14)


def test_merge_with_empty_side():
    o, l = ref.merge(np.array([1.0, 2.0]), 0.3, np.zeros(2), -np.inf)
    np.testing.assert_array_equal(o, [1.0, 2.0])
    assert l == 0.3


# ---- SnapKV-style scoring: closed forms and library cross-checks ---------------------------
def test_votes_uniform_keys_closed_form():
    # all keys equal => every row's softmax is uniform over its causal span of P+i+1 columns
    G, w, D, n = 3, 5, 4, 37
    P = n - w
    q = RNG.standard_normal((G, w, D))
    K = np.tile(RNG.standard_normal(D), (n, 1))
    vote = ref.window_votes(q, K, w, 0.5)
    expect = G * sum(1.0 / (P + i + 1) for i in range(w))
    np.testing.assert_allclose(vote, np.full(P, expect), rtol=1e-13)


def test_votes_match_dense_masked_softmax_library():
    # independent formulation: dense [w x n] logits, additive causal mask, torch.softmax
    G, w, D, n = 2, 6, 8, 45
    P = n - w
    q = RNG.standard_normal((G, w, D))
    K = RNG.standard_normal((n, D)) * 1.5
    vote = ref.window_votes(q, K, w, 0.35)
    S = torch.from_numpy(q) @ torch.from_numpy(K).T * 0.35                # [G][w][n]
    col = torch.arange(n).view(1, 1, n)
    row = torch.arange(w).view(1, w, 1)
    S = S.masked_fill(col > P + row, float("-inf"))
    Pm = torch.softmax(S, dim=-1)
    np.testing.assert_allclose(vote, Pm[..., :P].sum(dim=(0, 1)).numpy(), atol=1e-13)
    # mass conservation: prefix votes + window-column mass = G*w (every row sums to 1)
    np.testing.assert_allclose(vote.sum() + Pm[..., P:].sum().item(), G * w, atol=1e-12)


def test_votes_last_window_row_sees_all_first_row_sees_P_plus_1():
    # a key only visible to later window rows: make window column P+2 dominant; rows i<2 must
    # not see it (their prefix mass stays ~1), rows i>=2 lose almost all prefix mass to it.
    G, w, D, n = 1, 4, 4, 20
    P = n - w
    q = np.ones((G, w, D))
    K = np.zeros((n, D))
    K[P + 2] = 50.0
    vote = ref.window_votes(q, K, w, 1.0)
    # rows 0,1: uniform over P+1 / P+2 columns; rows 2,3: ~0 on the prefix
    expect = 1.0 / (P + 1) + 1.0 / (P + 2)
    np.testing.assert_allclose(vote, np.full(P, expect), rtol=1e-9)


def test_votes_with_supplied_row_lse():
    # the rows' log-sum-exp from an independent routine (torch.logsumexp over the causal span)
    # reproduces the self-normalised votes; an lse that is off by log 2 on one head halves that
    # head's contribution and nothing else; uniform keys give the closed form exp(-delta)/(P+i+1)
    G, w, D, n = 2, 6, 8, 45
    P = n - w
    q = RNG.standard_normal((G, w, D))
    K = RNG.standard_normal((n, D)) * 1.5
    S = torch.from_numpy(q) @ torch.from_numpy(K).T * 0.35
    col = torch.arange(n).view(1, 1, n)
    row = torch.arange(w).view(1, w, 1)
    lse = torch.logsumexp(S.masked_fill(col > P + row, float("-inf")), dim=-1).numpy()      # [G][w]
    base = ref.window_votes(q, K, w, 0.35)
    np.testing.assert_allclose(ref.window_votes(q, K, w, 0.35, win_lse=lse), base, rtol=1e-12)
    off = lse.copy()
    off[1] += np.log(2.0)
    head0 = ref.window_votes(q[:1], K, w, 0.35)
    head1 = ref.window_votes(q[1:], K, w, 0.35)
    np.testing.assert_allclose(ref.window_votes(q, K, w, 0.35, win_lse=off), head0 + 0.5 * head1, rtol=1e-12)
    Ku = np.tile(RNG.standard_normal(D), (n, 1))
    zu = 0.35 * q @ Ku[0]                                                                       # [G][w] the common logit
    delta = RNG.standard_normal((G, w))
    true_lse = zu + np.log(P + np.arange(w) + 1.0)
    got = ref.window_votes(q, Ku, w, 0.35, win_lse=true_lse + delta)
    expect = sum(np.exp(-delta[h, i]) / (P + i + 1) for h in range(G) for i in range(w))
    np.testing.assert_allclose(got, np.full(P, expect), rtol=1e-12)
    # compress passes it through: same retained set and calibration state as without it
    V = RNG.standard_normal((1, n, D))
    r0 = ref.compress(q, K[None], V, w, 16, 3, scale=0.35)
    r1 = ref.compress(q, K[None], V, w, 16, 3, scale=0.35, win_lse=lse)
    np.testing.assert_array_equal(r0["idx"], r1["idx"])
    np.testing.assert_allclose(r0["c_out"], r1["c_out"], atol=1e-13)


@pytest.mark.parametrize("k", [1, 3, 5, 7])
@pytest.mark.parametrize("P", [1, 2, 5, 33])
def test_avg_pool_matches_library(k, P):
    vote = RNG.random(P)
    got = ref.avg_pool(vote, k)
    lib = torch.nn.functional.avg_pool1d(torch.from_numpy(vote).view(1, 1, -1), kernel_size=k,
                                         stride=1, padding=k // 2, count_include_pad=True)
    np.testing.assert_allclose(got, lib.view(-1).numpy(), atol=1e-15)
    if k == 1:
        np.testing.assert_array_equal(got, vote)


def test_avg_pool_edges_closed_form():
    got = ref.avg_pool(np.ones(10), 5)
    np.testing.assert_allclose(got, [3 / 5, 4 / 5, 1, 1, 1, 1, 1, 1, 4 / 5, 3 / 5], atol=1e-15)


def brute_force_top(score, k_sel):
    """Repeated arg-max with removal; among equal maxima take the lowest index."""
    score = list(score)
    alive = set(range(len(score)))
    chosen = []
    for _ in range(k_sel):
        best = None
        for j in sorted(alive):
            if best is None or score[j] > score[best]:
                best = j
        chosen.append(best)
        alive.remove(best)
    return sorted(chosen)


def test_select_matches_brute_force_with_ties():
    for trial in range(50):
        P = int(RNG.integers(1, 40))
        score = RNG.integers(0, 6, size=P).astype(float)          # many exact ties
        k_sel = int(RNG.integers(0, P + 1))
        keep, _ = ref.select_top(score, k_sel)
        assert list(keep) == brute_force_top(score, k_sel)


def test_select_enumeration_tiny():
    # exhaustive: the chosen set maximises (sum of scores, then lexicographically lowest)
    score = np.array([0.3, 0.9, 0.3, 0.1, 0.9, 0.3])
    for k_sel in range(0, 7):
        keep, _ = ref.select_top(score, k_sel)
        best = None
        for comb in itertools.combinations(range(6), k_sel):
            key = (-sum(score[list(comb)]), comb)
            if best is None or key < best[0]:
                best = (key, comb)
        assert tuple(keep) == best[1]


def test_select_margin():
    keep, margin = ref.select_top(np.array([4.0, 1.0, 2.0, 3.0]), 2)
    assert list(keep) == [0, 3] and margin == pytest.approx((3.0 - 2.0) / 3.0)


# ---- Alg. 1 ---------------------------------------------------------------------------------
def test_compress_structure_and_gather():
    q_win, K, V = rand_case()
    w, B, k = 4, 12, 3
    r = ref.compress(q_win, K, V, w, B, k)
    n = K.shape[1]
    P = n - w
    for g in range(K.shape[0]):
        idx = r["idx"][g]
        assert idx.shape == (B,) and np.all(np.diff(idx) > 0)
        assert list(idx[-w:]) == list(range(P, n))                       # window always kept
        np.testing.assert_array_equal(r["K_c"][g], K[g][idx])
        np.testing.assert_array_equal(r["V_c"][g], V[g][idx])
        ev = r["evicted"][g]
        assert len(ev) == n - B and set(ev).isdisjoint(idx) and set(ev) | set(idx) == set(range(n))
        # selected prefix tokens are exactly the top (B-w) of the pooled score
        assert list(idx[:B - w]) == brute_force_top(r["score"][g], B - w)
    np.testing.assert_array_equal(r["c_q"], q_win[:, -1])


def test_compress_group_sum_before_pool_equals_pool_then_sum():
    # GQA reading: votes of the G heads are summed before pooling; pooling is linear
    q_win, K, V = rand_case(Hq=6, Hkv=2)
    w, k = 4, 5
    G = 3
    g = 1
    total = ref.window_votes(q_win[g * G:(g + 1) * G], K[g], w, 0.3)
    parts = [ref.window_votes(q_win[h:h + 1], K[g], w, 0.3) for h in range(g * G, (g + 1) * G)]
    np.testing.assert_allclose(ref.avg_pool(total, k), sum(ref.avg_pool(p, k) for p in parts),
                               atol=1e-14)


def test_full_budget_means_full_attention():
    # budget >= n: nothing evicted, c_lse = -inf, decode == exact attention for any theta
    q_win, K, V = rand_case(n=20)
    r = ref.compress(q_win, K, V, 4, 32, 5)
    assert np.all(r["c_lse"] == -np.inf) and np.all(r["c_out"] == 0)
    assert r["idx"].shape == (2, 20)
    q_t = RNG.standard_normal((4, 8))
    for th in [(0.7, 0.85), (-np.inf, -np.inf), (2.0, 3.0)]:
        out, a_lse, flags, _ = ref.decode(q_t, r["K_c"], r["V_c"], 20, r["c_q"], r["c_out"],
                                          r["c_lse"], *th)
        for h in range(4):
            np.testing.assert_allclose(out[h], sdpa64(q_t[h], K[h // 2], V[h // 2], 8 ** -0.5),
                                       atol=1e-13)
        assert not np.any(flags == ref.FLAG_CALIBRATED)


def test_identical_query_calibration_is_exact():
    # the zero-loss case of Sec. 3.1.3 (calibration query identical to the current query):
    # q_cal == q_t  =>  calibrated output == full attention
    q_win, K, V = rand_case(n=64, w=8, D=16)
    q_t = RNG.standard_normal((4, 16)) * 1.7
    r = ref.compress(q_win, K, V, 8, 20, 5, q_cal=q_t)
    out, a_lse, flags, rho = ref.decode(q_t, r["K_c"], r["V_c"], 20, r["c_q"], r["c_out"],
                                        r["c_lse"], 0.7, 0.85)
    assert np.all(flags == ref.FLAG_CALIBRATED)
    np.testing.assert_allclose(rho, 1.0, atol=1e-15)
    for h in range(4):
        np.testing.assert_allclose(out[h], sdpa64(q_t[h], K[h // 2], V[h // 2], 0.25),
                                   atol=1e-13)
    # and without calibration the compressed attention is NOT exact (the test has teeth)
    out0, *_ = ref.decode(q_t, r["K_c"], r["V_c"], 20, r["c_q"], r["c_out"], r["c_lse"],
                          0.7, np.inf)
    assert np.abs(out0 - out).max() > 1e-3


def test_denominators_add_up():
    # Eq. 2: denominator over evicted + denominator over retained = denominator over all
    q_win, K, V = rand_case(n=48, w=4)
    r = ref.compress(q_win, K, V, 4, 16, 3)
    for h in range(4):
        g = h // 2
        q = q_win[h, -1]
        lse_all = logsumexp(K[g] @ q * 8 ** -0.5)
        lse_ret = logsumexp(r["K_c"][g] @ q * 8 ** -0.5)
        np.testing.assert_allclose(np.logaddexp(r["c_lse"][h], lse_ret), lse_all, atol=1e-13)


def test_calibration_state_is_attention_over_evicted_only():
    q_win, K, V = rand_case(n=48, w=4)
    r = ref.compress(q_win, K, V, 4, 16, 3)
    for h in range(4):
        g = h // 2
        ev = np.array(sorted(set(range(48)) - set(r["idx"][g])))
        np.testing.assert_allclose(r["c_out"][h], sdpa64(q_win[h, -1], K[g][ev], V[g][ev],
                                                         8 ** -0.5), atol=1e-13)


def test_permutation_equivariance_k1():
    # k = 1 (no pooling): permuting prefix tokens permutes the selected set
    q_win, K, V = rand_case(n=40, w=4)
    perm = RNG.permutation(36)
    full = np.concatenate([perm, np.arange(36, 40)])
    r0 = ref.compress(q_win, K, V, 4, 14, 1)
    r1 = ref.compress(q_win, K[:, full], V[:, full], 4, 14, 1)
    for g in range(2):
        assert set(full[r1["idx"][g]]) == set(r0["idx"][g])
    np.testing.assert_allclose(r0["c_out"], r1["c_out"], atol=1e-13)
    np.testing.assert_allclose(r0["c_lse"], r1["c_lse"], atol=1e-13)


def test_scale_sanity():
    q_win, K, V = rand_case()
    r0 = ref.compress(q_win, K, V, 4, 12, 3, scale=0.3)
    r1 = ref.compress(q_win, K * 4.0, V, 4, 12, 3, scale=0.3 / 4.0)
    np.testing.assert_array_equal(r0["idx"], r1["idx"])
    np.testing.assert_allclose(r0["c_out"], r1["c_out"], atol=1e-13)
    np.testing.assert_allclose(r0["c_lse"], r1["c_lse"], atol=1e-12)


# ---- Alg. 2 ---------------------------------------------------------------------------------
def test_decode_uncalibrated_is_library_attention():
    q_win, K, V = rand_case(n=48, w=4)
    r = ref.compress(q_win, K, V, 4, 16, 3)
    q_t = RNG.standard_normal((4, 8))
    out, a_lse, flags, _ = ref.decode(q_t, r["K_c"], r["V_c"], 16, r["c_q"], r["c_out"],
                                      r["c_lse"], -np.inf, np.inf)
    assert np.all(flags == 0)
    for h in range(4):
        np.testing.assert_allclose(out[h], sdpa64(q_t[h], r["K_c"][h // 2], r["V_c"][h // 2],
                                                  8 ** -0.5), atol=1e-13)
        np.testing.assert_allclose(a_lse[h], logsumexp(r["K_c"][h // 2] @ q_t[h] * 8 ** -0.5),
                                   atol=1e-13)
    # row order of the cache does not matter; rows past `length` are ignored
    p = RNG.permutation(16)
    Kp = np.concatenate([r["K_c"][:, p], 99 * np.ones((2, 3, 8))], axis=1)
    Vp = np.concatenate([r["V_c"][:, p], 99 * np.ones((2, 3, 8))], axis=1)
    out2, *_ = ref.decode(q_t, Kp, Vp, 16, r["c_q"], r["c_out"], r["c_lse"], -np.inf, np.inf)
    np.testing.assert_allclose(out2, out, atol=1e-13)


def test_gate_three_branches_and_equalities():
    # c_q = e1, q_t = (a, b, 0..): rho = a / sqrt(a^2+b^2); 3-4-5 triangles give exact values
    D = 8
    c_q = np.zeros((1, D)); c_q[0, 0] = 1.0
    K_c = RNG.standard_normal((1, 6, D)); V_c = RNG.standard_normal((1, 6, D))
    c_out = RNG.standard_normal((1, D)); c_lse = np.array([0.2])

    def run(a, b, t1, t2):
        q = np.zeros((1, D)); q[0, 0] = a; q[0, 1] = b
        return ref.decode(q, K_c, V_c, 6, c_q, c_out, c_lse, t1, t2)

    t06, t08 = np.float32(0.6), np.float32(0.8)
    assert run(3, 4, 0.7, 0.85)[2][0] == ref.FLAG_RECOMPUTE          # rho 0.6 < 0.7
    assert run(4, 3, 0.7, 0.85)[2][0] == ref.FLAG_NONE               # 0.7 <= 0.8 <= 0.85
    assert run(12, 5, 0.7, 0.85)[2][0] == ref.FLAG_CALIBRATED        # 12/13 > 0.85
    assert run(3, 4, t06, 0.85)[2][0] == ref.FLAG_NONE               # rho == theta1: strict <
    assert run(4, 3, 0.7, t08)[2][0] == ref.FLAG_NONE                # rho == theta2: strict >
    assert run(0, 0, 0.7, 0.85)[2][0] == ref.FLAG_RECOMPUTE          # zero query: rho := 0
    # flagged-recompute and in-between outputs are the plain compressed attention
    for a, b in [(3, 4), (4, 3)]:
        q = np.zeros(D); q[0] = a; q[1] = b
        np.testing.assert_allclose(run(a, b, 0.7, 0.85)[0][0], sdpa64(q, K_c[0], V_c[0], D ** -0.5),
                                   atol=1e-13)
    # calibrated output is the Eq. 1 blend with alpha_j = sigmoid(c_lse - a_lse)
    out, a_lse, _, _ = run(12, 5, 0.7, 0.85)
    q = np.zeros(D); q[0] = 12; q[1] = 5
    aj = 1.0 / (1.0 + np.exp(a_lse[0] - 0.2))
    np.testing.assert_allclose(out[0], (1 - aj) * sdpa64(q, K_c[0], V_c[0], D ** -0.5) + aj * c_out[0],
                               atol=1e-13)


def test_always_calibrate_thresholds():
    q_win, K, V = rand_case(n=48, w=4)
    r = ref.compress(q_win, K, V, 4, 16, 3)
    q_t = -q_win[:, -1]                                               # rho = -1
    _, _, flags, _ = ref.decode(q_t, r["K_c"], r["V_c"], 16, r["c_q"], r["c_out"], r["c_lse"],
                                -np.inf, -np.inf)
    assert np.all(flags == ref.FLAG_CALIBRATED)


def test_recompute_branch_gives_exact_attention_and_refreshes_state():
    # Alg. 2 steps 3-8: after recomputation with the current query the calibrated output is the
    # exact attention over all prompt tokens (Eq. 1 with the true query on both sides)
    q_win, K, V = rand_case(n=60, w=6, D=16)
    r = ref.compress(q_win, K, V, 6, 18, 3)
    q_t = -q_win[:, -1] + 0.1 * RNG.standard_normal((4, 16))          # rho ~ -1 < theta1
    out, a_lse, flags, rho = ref.decode(q_t, r["K_c"], r["V_c"], 18, r["c_q"], r["c_out"], r["c_lse"], 0.7, 0.85)
    assert np.all(flags == ref.FLAG_RECOMPUTE)
    out2, flags2, c_q, c_out, c_lse = ref.recalibrate(q_t, K, V, r["idx"], flags, a_lse, out, r["c_q"], r["c_out"],
                                                      r["c_lse"])
    assert np.all(flags2 == ref.FLAG_RECOMPUTED)
    np.testing.assert_array_equal(c_q, q_t)
    for h in range(4):
        g = h // 2
        np.testing.assert_allclose(out2[h], sdpa64(q_t[h], K[g], V[g], 0.25), atol=1e-13)
        ev = np.array(sorted(set(range(54)) - set(r["idx"][g])))
        np.testing.assert_allclose(c_out[h], sdpa64(q_t[h], K[g][ev], V[g][ev], 0.25), atol=1e-13)
        np.testing.assert_allclose(c_lse[h], logsumexp(0.25 * K[g][ev] @ q_t[h]), atol=1e-13)
    # the refreshed state calibrates the same query exactly on the next step (rho = 1)
    out3, _, flags3, rho3 = ref.decode(q_t, r["K_c"], r["V_c"], 18, c_q, c_out, c_lse, 0.7, 0.85)
    assert np.all(flags3 == ref.FLAG_CALIBRATED)
    np.testing.assert_allclose(out3, out2, atol=1e-13)
    # heads that were not flagged are left alone
    flags_mixed = flags.copy(); flags_mixed[1] = ref.FLAG_NONE
    o4, f4, cq4, co4, cl4 = ref.recalibrate(q_t, K, V, r["idx"], flags_mixed, a_lse, out, r["c_q"], r["c_out"],
                                            r["c_lse"])
    np.testing.assert_array_equal(o4[1], out[1]); np.testing.assert_array_equal(cq4[1], r["c_q"][1])
    assert f4[1] == ref.FLAG_NONE and f4[0] == ref.FLAG_RECOMPUTED


def test_recompute_with_nothing_evicted_is_a_noop_on_the_output():
    q_win, K, V = rand_case(n=20)
    r = ref.compress(q_win, K, V, 4, 32, 5)
    q_t = -q_win[:, -1]
    out, a_lse, flags, _ = ref.decode(q_t, r["K_c"], r["V_c"], 20, r["c_q"], r["c_out"], r["c_lse"], 0.7, 0.85)
    out2, flags2, c_q, c_out, c_lse = ref.recalibrate(q_t, K, V, r["idx"], flags, a_lse, out, r["c_q"], r["c_out"],
                                                      r["c_lse"])
    np.testing.assert_array_equal(out2, out)
    assert np.all(c_lse == -np.inf) and np.all(flags2 == ref.FLAG_RECOMPUTED)
    np.testing.assert_array_equal(c_q, q_t)


def test_calibration_size_keeps_the_most_important_evicted_tokens():
    # Sec. 5.3: only the m evicted tokens of highest importance are offloaded / calibrated
    q_win, K, V = rand_case(n=60, w=6, D=16)
    full = ref.compress(q_win, K, V, 6, 18, 3)
    for m in [1, 5, 17]:
        r = ref.compress(q_win, K, V, 6, 18, 3, calib_size=m)
        np.testing.assert_array_equal(r["idx"], full["idx"])                 # selection itself is unchanged
        for g in range(2):
            ev_all = full["evicted"][g]
            # brute force: repeated arg-max with removal over the evicted tokens' scores
            want = [int(ev_all[i]) for i in brute_force_top(full["score"][g][ev_all], m)]
            assert r["evicted"][g].tolist() == sorted(want)
        for h in range(4):
            g = h // 2
            ev = r["evicted"][g]
            np.testing.assert_allclose(r["c_out"][h], sdpa64(q_win[h, -1], K[g][ev], V[g][ev], 0.25), atol=1e-13)
            np.testing.assert_allclose(r["c_lse"][h], logsumexp(0.25 * K[g][ev] @ q_win[h, -1]), atol=1e-13)
    # m >= number of evicted tokens, and m = 0, both mean "all of them"
    for m in [0, 42, 1000]:
        r = ref.compress(q_win, K, V, 6, 18, 3, calib_size=m)
        np.testing.assert_array_equal(r["c_out"], full["c_out"])
        np.testing.assert_array_equal(r["c_lse"], full["c_lse"])
    # the recomputation branch then only sees the offloaded subset
    r = ref.compress(q_win, K, V, 6, 18, 3, calib_size=5)
    q_t = -q_win[:, -1]
    out, a_lse, flags, _ = ref.decode(q_t, r["K_c"], r["V_c"], 18, r["c_q"], r["c_out"], r["c_lse"], 0.7, 0.85)
    cal_idx = np.stack(r["evicted"])
    out2, _, _, c_out, c_lse = ref.recalibrate(q_t, K, V, r["idx"], flags, a_lse, out, r["c_q"], r["c_out"], r["c_lse"],
                                               cal_idx=cal_idx)
    for h in range(4):
        g = h // 2
        keep = np.concatenate([r["idx"][g], r["evicted"][g]])
        np.testing.assert_allclose(out2[h], sdpa64(q_t[h], K[g][keep], V[g][keep], 0.25), atol=1e-13)


# ---- other strategies: StreamingLLM list, Alg. 1 for a known retained set ---------------------
def test_streaming_llm_list_by_hand_and_by_properties():
    # n = 12, B = 6, 2 sinks: positions 0,1 and the 4 most recent
    np.testing.assert_array_equal(ref.streaming_llm_retained(12, 6, 2), [0, 1, 8, 9, 10, 11])
    np.testing.assert_array_equal(ref.streaming_llm_retained(5, 6, 2), [0, 1, 2, 3, 4])      # fits: keep all
    np.testing.assert_array_equal(ref.streaming_llm_retained(9, 4, 0), [5, 6, 7, 8])         # pure sliding window
    np.testing.assert_array_equal(ref.streaming_llm_retained(9, 4, 4), [0, 1, 2, 3])         # sinks only
    for n, B, s in [(100, 40, 32), (41, 40, 32), (4096, 512, 32)]:
        r = ref.streaming_llm_retained(n, B, s)
        assert len(r) == B and len(set(r.tolist())) == B and np.all(np.diff(r) > 0)
        assert set(range(s)) <= set(r.tolist())
        assert set(range(n - (B - s), n)) <= set(r.tolist())
    # the same set as a top-B selection of "sinks first, then the newer the better"
    n, B, s = 57, 20, 6
    pref = np.where(np.arange(n) < s, 1e9, np.arange(n).astype(float))
    top, _ = ref.select_top(pref, B)
    np.testing.assert_array_equal(ref.streaming_llm_retained(n, B, s), top)


def test_compress_given_merges_to_full_attention_and_gathers_the_list():
    q_win, K, V = rand_case(n=50, w=4, D=8)
    q_cal = RNG.standard_normal((4, 8))
    kept = [np.array([0, 3, 7, 20, 21, 40, 48, 49]), np.array([1, 2, 30, 31, 32, 33, 46, 49])]
    r = ref.compress_given(q_cal, K, V, 8, kept)
    for g in range(2):
        np.testing.assert_array_equal(r["idx"][g], kept[g])
        np.testing.assert_array_equal(r["K_c"][g], K[g][kept[g]])
        np.testing.assert_array_equal(r["V_c"][g], V[g][kept[g]])
        assert set(r["evicted"][g].tolist()) == set(range(50)) - set(kept[g].tolist())
    for h in range(4):
        g = h // 2
        ev = np.array(sorted(set(range(50)) - set(kept[g].tolist())))
        np.testing.assert_allclose(r["c_out"][h], sdpa64(q_cal[h], K[g][ev], V[g][ev], 8 ** -0.5), atol=1e-13)
        np.testing.assert_allclose(r["c_lse"][h], logsumexp(K[g][ev] @ q_cal[h] * 8 ** -0.5), atol=1e-13)
        # Eq. 1: retained part + calibration state = attention over the whole prompt
        o_a, l_a = ref.attention(q_cal[h], r["K_c"][g], r["V_c"][g], 8 ** -0.5)
        full, _ = ref.merge(o_a, l_a, r["c_out"][h], r["c_lse"][h])
        np.testing.assert_allclose(full, sdpa64(q_cal[h], K[g], V[g], 8 ** -0.5), atol=1e-13)
    np.testing.assert_array_equal(r["c_q"], q_cal)
    # prompt within the budget: nothing evicted, list ignored
    r2 = ref.compress_given(q_cal, K, V, 64, None)
    assert np.all(r2["c_lse"] == -np.inf) and np.all(r2["c_out"] == 0)
    np.testing.assert_array_equal(r2["idx"][0], np.arange(50))


def test_compress_given_with_the_scored_list_equals_compress():
    q_win, K, V = rand_case(n=64, w=8, D=16)
    r = ref.compress(q_win, K, V, 8, 24, 5)
    r2 = ref.compress_given(q_win[:, -1], K, V, 24, [r["idx"][0], r["idx"][1]])
    for key in ("K_c", "V_c", "c_q", "c_out", "c_lse"):
        np.testing.assert_allclose(r2[key], r[key], atol=1e-14)


# ---- H2O: accumulated attention over all prompt queries -------------------------------------------
def test_h2o_votes_match_dense_causal_softmax_and_conserve_mass():
    rng = np.random.default_rng(5)
    G, n, D = 3, 37, 8
    q = rng.standard_normal((G, n, D)); K = rng.standard_normal((n, D))
    vote = ref.h2o_votes(q, K, 0.3)
    S = torch.from_numpy(q) @ torch.from_numpy(K).T * 0.3                     # [G][n][n]
    mask = torch.tril(torch.ones(n, n, dtype=torch.bool))
    Pm = torch.softmax(S.masked_fill(~mask, float("-inf")), dim=-1)
    np.testing.assert_allclose(vote, Pm.sum(dim=(0, 1)).numpy(), atol=1e-12)
    np.testing.assert_allclose(vote.sum(), G * n, atol=1e-10)                 # every row distributes mass 1
    # a transposed or anti-causal mask would give the first position the least mass, not the most
    assert vote[0] > vote[-1]


def test_h2o_votes_uniform_keys_closed_form():
    # identical keys: row i spreads 1/(i+1) over columns 0..i  =>  vote[j] = G * (H_n - H_j)
    G, n, D = 2, 25, 4
    q = RNG.standard_normal((G, n, D)); K = np.tile(RNG.standard_normal(D), (n, 1))
    vote = ref.h2o_votes(q, K, 0.5)
    Hn = np.cumsum(1.0 / np.arange(1, n + 1))
    want = G * (Hn[-1] - np.concatenate([[0.0], Hn[:-1]]))
    np.testing.assert_allclose(vote, want, atol=1e-12)


def test_h2o_votes_reduce_to_the_window_votes_on_the_last_rows():
    # rows below P only see keys below P, so: votes(all rows) - votes(rows < P) on the prefix
    # columns = the observation-window votes of the last w rows
    G, n, D, w = 2, 40, 8, 6
    P = n - w
    q = RNG.standard_normal((G, n, D)); K = RNG.standard_normal((n, D))
    full = ref.h2o_votes(q, K, 0.35)
    head = ref.h2o_votes(q[:, :P], K[:P], 0.35)
    np.testing.assert_allclose(full[:P] - head, ref.window_votes(q[:, P:], K, w, 0.35), atol=1e-12)


def test_h2o_retained_set_and_compress():
    vote = np.array([5.0, 0.1, 3.0, 3.0, 0.2, 9.0, 0.3, 0.4, 7.0, 0.5])
    keep, margin = ref.h2o_retained(vote, 10, 6, 3)
    # local = positions 7, 8, 9; heavy hitters among 0..6: 5 (9.0), 0 (5.0), then the tie 2/3 -> 2
    np.testing.assert_array_equal(keep, [0, 2, 5, 7, 8, 9])
    assert margin == 0.0
    np.testing.assert_array_equal(ref.h2o_retained(vote, 10, 12, 6)[0], np.arange(10))
    # brute force on random scores
    for _ in range(20):
        n, B, loc = 30, 12, int(RNG.integers(1, 11))
        v = np.round(RNG.random(n), 1)                                         # many ties
        keep, _ = ref.h2o_retained(v, n, B, loc)
        cand = sorted(range(n - loc), key=lambda j: (-v[j], j))[:B - loc]
        np.testing.assert_array_equal(keep, sorted(cand) + list(range(n - loc, n)))
    # end to end: retained + calibration state merge to the full attention of Q_{-1} (Eq. 1)
    Hq, Hkv, n, D = 4, 2, 45, 8
    qf = RNG.standard_normal((Hq, n, D)); K = RNG.standard_normal((Hkv, n, D)); V = RNG.standard_normal((Hkv, n, D))
    r = ref.compress_h2o(qf, K, V, 14, 7)
    assert r["idx"].shape == (2, 14) and np.all(r["idx"][:, 7:] == np.arange(38, 45))
    for h in range(Hq):
        g = h // 2
        o_a, l_a = ref.attention(qf[h, -1], r["K_c"][g], r["V_c"][g], 8 ** -0.5)
        full, _ = ref.merge(o_a, l_a, r["c_out"][h], r["c_lse"][h])
        np.testing.assert_allclose(full, sdpa64(qf[h, -1], K[g], V[g], 8 ** -0.5), atol=1e-13)
    np.testing.assert_array_equal(r["c_q"], qf[:, -1])
