"""CaliDrop reference ("oracle"): plain, slow, float64 numpy.  TEST INFRASTRUCTURE ONLY.

This file is the yardstick the HIP path is compared against.  It shares no code with the HIP
path and must never be imported by the product (only by tests/, the smoke check and the
benchmark's CPU-baseline leg).  Every function follows the paper step by step, in the paper's
order and notation; nothing is blocked, fused or reordered.

What the paper fixes and what it leaves open
--------------------------------------------
* Eq. 1-2 (attention decomposition) and Alg. 1 / Alg. 2 are followed literally, with the logit
  scale 1/sqrt(d_k) of Eq. 2 (Alg. 1/2 print d_k; Eq. 1 only holds with a single scale).
* C_weight of Alg. 1 is kept as its logarithm ``c_lse`` (same information, no overflow).
* The eviction strategy f of Alg. 1 step 3 is "SnapKV-style" (Sec. 4.1.3: observation window,
  average pooling).  The paper does not spell out its internals; the reading implemented here
  is: softmax of the window queries over all keys with a causal mask inside the window,
  summed over the window and over the query heads of a KV group, 1-D average pooling (stride
  1, zero padding, divisor k), top-(B - w) prefix positions, ties to the lower index, window
  always kept.  PARITY UNPINNED for these internal choices: no value in the paper checks them;
  closed forms and brute force pin the arithmetic of the chosen reading.
* H2O (Sec. 4.1.3: accumulated attention, budget split evenly into important and local tokens)
  is read as: causal softmax of every prompt query, column sums over all queries and over the
  query heads of a KV group, no pooling, the most recent half of the budget always kept.  PARITY
  UNPINNED for the group sum and the prefill-only accumulation, like the SnapKV-style internals.
* The gate rho is compared with the thresholds in float32 (the precision the kernels decide
  in); everything else is float64.
"""
from __future__ import annotations

import numpy as np

F = np.float64


# --------------------------------------------------------------------------------------------
# Attention and its decomposition (Sec. 3.1.2, Eq. 1-2)
# --------------------------------------------------------------------------------------------
def logits(q, K, scale):
    """z_t = scale * q . K_t for one query vector q [D] and keys K [n][D]."""
    return scale * (np.asarray(K, F) @ np.asarray(q, F))


def attention(q, K, V, scale):
    """Att(q, K, V) = softmax(q K^T * scale) V for one query; also returns log sum exp.

    Returns (out [D], lse).  For an empty key set: (zeros, -inf)."""
    K = np.asarray(K, F)
    V = np.asarray(V, F)
    if K.shape[0] == 0:
        return np.zeros(V.shape[1], F), -np.inf
    z = logits(q, K, scale)
    m = z.max()
    e = np.exp(z - m)
    denom = e.sum()
    return (e @ V) / denom, m + np.log(denom)


def merge_weights(lse_i, lse_j):
    """alpha_i, alpha_j of Eq. 2 from the two subsets' log-denominators."""
    if lse_j == -np.inf:
        return 1.0, 0.0
    if lse_i == -np.inf:
        return 0.0, 1.0
    m = max(lse_i, lse_j)
    wi, wj = np.exp(lse_i - m), np.exp(lse_j - m)
    return wi / (wi + wj), wj / (wi + wj)


def merge(out_i, lse_i, out_j, lse_j):
    """Eq. 1: Att over S_i u S_j from the two partial attentions.  Returns (out, lse)."""
    ai, aj = merge_weights(lse_i, lse_j)
    out = ai * np.asarray(out_i, F) + aj * np.asarray(out_j, F)
    return out, np.logaddexp(lse_i, lse_j)


# --------------------------------------------------------------------------------------------
# Eviction strategy f (Alg. 1 step 3), SnapKV-style (Sec. 4.1.3)
# --------------------------------------------------------------------------------------------
def window_votes(q_win_group, K_g, w, scale, win_lse=None):
    """Accumulated attention of the observation window onto the prefix, for one KV head.

    q_win_group [G][w][D]: the window queries of the G query heads that share this KV head;
    query i of the window sits at position P + i (P = n - w) and may attend positions
    0..P+i.  Returns vote [P]: sum over heads and window rows of the softmax probability that
    lands on each prefix column.  Window columns take part in the softmax but get no vote.

    win_lse [G][w] (optional): the rows' log-sum-exp as handed over by whoever ran the prompt's
    attention (Alg. 1 steps 1-2); the probabilities are then exp(z - win_lse) with the values as
    given, instead of being normalised here."""
    q = np.asarray(q_win_group, F)
    K = np.asarray(K_g, F)
    n = K.shape[0]
    P = n - w
    vote = np.zeros(P, F)
    for h in range(q.shape[0]):
        for i in range(w):
            z = logits(q[h, i], K[:P + i + 1], scale)       # causal: columns 0..P+i
            if win_lse is None:
                e = np.exp(z - z.max())
                p = e / e.sum()
            else:
                p = np.exp(z - F(win_lse[h][i]))
            vote += p[:P]
    return vote


def avg_pool(vote, k):
    """1-D average pooling, stride 1, zero padding floor(k/2) each side, divisor always k."""
    vote = np.asarray(vote, F)
    P = vote.shape[0]
    half = k // 2
    score = np.zeros(P, F)
    for d in range(-half, half + 1):            # same operation order at every position
        shifted = np.zeros(P, F)                # shifted[j] = vote[j + d], 0 outside [0, P)
        lo, hi = max(0, -d), min(P, P - d)
        if hi > lo:
            shifted[lo:hi] = vote[lo + d:hi + d]
        score = score + shifted
    return score / k


def select_top(score, k_sel):
    """Positions of the k_sel largest scores, ties to the lower index, returned ascending.

    Also returns the relative boundary margin (s_(k_sel) - s_(k_sel+1)) / s_(k_sel) of the
    sorted scores (inf when nothing is left out)."""
    score = np.asarray(score, F)
    order = np.argsort(-score, kind="stable")   # stable: equal scores keep index order
    keep = np.sort(order[:k_sel])
    if k_sel >= score.shape[0] or k_sel == 0:
        return keep, np.inf
    a, b = score[order[k_sel - 1]], score[order[k_sel]]
    margin = (a - b) / a if a > 0 else 0.0
    return keep, margin


# --------------------------------------------------------------------------------------------
# Alg. 1 (prefill side): compression + calibration state, one sequence
# --------------------------------------------------------------------------------------------
def calibration_state(q_cal, K, V, evicted, G, scale):
    """Alg. 1 steps 5-8 for every query head: attention of the calibration query over the
    evicted tokens of its KV head.  evicted: list over KV heads of position arrays."""
    q_cal = np.asarray(q_cal, F)
    Hq, D = q_cal.shape
    c_out = np.zeros((Hq, D), F)
    c_lse = np.full(Hq, -np.inf, F)
    for h in range(Hq):
        g = h // G
        ev = evicted[g]
        c_out[h], c_lse[h] = attention(q_cal[h], np.asarray(K[g], F)[ev],
                                       np.asarray(V[g], F)[ev], scale)
    return q_cal.copy(), c_out, c_lse


def compress(q_win, K, V, w, B, k, q_cal=None, scale=None, retained_override=None, calib_size=0, win_lse=None):
    """Alg. 1 steps 3-8 for one sequence.

    calib_size = m > 0 keeps only the m evicted tokens of highest importance (pooled score, ties
    to the lower position) for calibration and offloading - the "calibration size" of Sec. 5.3;
    every other evicted token is dropped for good.  m = 0 keeps every evicted token.

    q_win [Hq][w][D] last w prompt queries; K, V [Hkv][n][D]; B = KV budget (window included);
    k = pooling kernel; q_cal [Hq][D] calibration query (default Q_{-1} = q_win[:, -1]).
    retained_override: optional list over KV heads of ascending position arrays to use instead
    of the selection (lets a test evaluate downstream values for a given retained set).
    win_lse [Hq][w]: optional log-sum-exp of the window rows, taken as given (see window_votes).

    Returns dict: idx [Hkv][min(B,n)] ascending retained positions, K_c, V_c [Hkv][len][D],
    c_q, c_out [Hq][D], c_lse [Hq], vote/score (lists per KV head, None if n <= B),
    margin [Hkv]."""
    q_win = np.asarray(q_win, F)
    K = np.asarray(K, F)
    V = np.asarray(V, F)
    Hq, _, D = q_win.shape
    Hkv, n, _ = K.shape
    G = Hq // Hkv
    if scale is None:
        scale = 1.0 / np.sqrt(D)
    if q_cal is None:
        q_cal = q_win[:, w - 1]
    P = n - w
    idx, votes, scores, margins, evicted = [], [], [], [], []
    for g in range(Hkv):
        if n <= B:                                   # nothing to evict (upper bound: FullKV)
            keep_all = np.arange(n)
            idx.append(keep_all)
            votes.append(None)
            scores.append(None)
            margins.append(np.inf)
            evicted.append(np.zeros(0, np.int64))
            continue
        vote = window_votes(q_win[g * G:(g + 1) * G], K[g], w, scale,
                            None if win_lse is None else np.asarray(win_lse, F)[g * G:(g + 1) * G])
        score = avg_pool(vote, k)
        if retained_override is not None:
            sel = np.asarray(retained_override[g])[:B - w]
            margin = np.inf
        else:
            sel, margin = select_top(score, B - w)
        idx_g = np.concatenate([sel, np.arange(P, n)])
        mask = np.ones(P, bool)
        mask[sel] = False
        ev = np.nonzero(mask)[0]                     # KV_evict = KV_full minus KV_compress
        if calib_size > 0 and calib_size < len(ev):  # Sec. 5.3: rank the evicted tokens by importance
            order = np.argsort(-score[ev], kind="stable")
            ev = np.sort(ev[order[:calib_size]])
        idx.append(idx_g)
        votes.append(vote)
        scores.append(score)
        margins.append(margin)
        evicted.append(ev)
    idx = np.stack(idx)
    K_c = np.stack([K[g][idx[g]] for g in range(Hkv)])
    V_c = np.stack([V[g][idx[g]] for g in range(Hkv)])
    c_q, c_out, c_lse = calibration_state(q_cal, K, V, evicted, G, scale)
    return dict(idx=idx, K_c=K_c, V_c=V_c, c_q=c_q, c_out=c_out, c_lse=c_lse,
                vote=votes, score=scores, margin=np.asarray(margins), evicted=evicted)


# --------------------------------------------------------------------------------------------
# Other eviction strategies f (Sec. 4.1.3) and Alg. 1 for a retained set that is already known
# --------------------------------------------------------------------------------------------
def streaming_llm_retained(n, B, n_sink):
    """StreamingLLM as configured in Sec. 4.1.3: n_sink attention-sink positions at the start of
    the prompt, the rest of the budget on the most recent positions.  Ascending positions."""
    if n <= B:
        return np.arange(n)
    keep = [j for j in range(n) if j < n_sink or j >= n - (B - n_sink)]
    return np.asarray(keep, np.int64)


def compress_given(q_cal, K, V, B, retained, scale=None):
    """Alg. 1 steps 4-8 for one sequence when step 3 (the choice of KV_compress) was made elsewhere.

    retained: list over KV heads of position arrays (ascending); ignored when n <= B (nothing is
    evicted).  KV_evict = every position of the prompt that is not retained.  q_cal [Hq][D] is
    Q_{-1}.  Returns dict idx, K_c, V_c, c_q, c_out, c_lse, evicted."""
    q_cal = np.asarray(q_cal, F)
    K = np.asarray(K, F)
    V = np.asarray(V, F)
    Hq, D = q_cal.shape
    Hkv, n, _ = K.shape
    G = Hq // Hkv
    if scale is None:
        scale = 1.0 / np.sqrt(D)
    idx, evicted = [], []
    for g in range(Hkv):
        keep = np.arange(n) if n <= B else np.asarray(retained[g], np.int64)
        ev = np.asarray([j for j in range(n) if j not in set(keep.tolist())], np.int64)
        idx.append(keep)
        evicted.append(ev)
    idx = np.stack(idx)
    K_c = np.stack([K[g][idx[g]] for g in range(Hkv)])
    V_c = np.stack([V[g][idx[g]] for g in range(Hkv)])
    c_q, c_out, c_lse = calibration_state(q_cal, K, V, evicted, G, scale)
    return dict(idx=idx, K_c=K_c, V_c=V_c, c_q=c_q, c_out=c_out, c_lse=c_lse, evicted=evicted)


def h2o_votes(q_group, K_g, scale):
    """Accumulated attention score of H2O (Sec. 4.1.3) for one KV head.

    q_group [G][n][D]: every prompt query of the G query heads that share this KV head; the query
    at position i attends positions 0..i (causal).  Returns vote [n]: for each position the
    attention probability it received, summed over all queries and over the G heads."""
    q = np.asarray(q_group, F)
    K = np.asarray(K_g, F)
    n = K.shape[0]
    vote = np.zeros(n, F)
    for h in range(q.shape[0]):
        for i in range(n):
            z = logits(q[h, i], K[:i + 1], scale)
            e = np.exp(z - z.max())
            vote[:i + 1] += e / e.sum()
    return vote


def h2o_retained(vote, n, B, n_local):
    """H2O's retained set: the n_local most recent positions plus the B - n_local positions of
    highest accumulated score among the others (ties to the lower position).  Sec. 4.1.3 splits
    the budget evenly (n_local = B / 2).  Ascending positions; also the boundary margin."""
    if n <= B:
        return np.arange(n), np.inf
    sel, margin = select_top(np.asarray(vote, F)[:n - n_local], B - n_local)
    return np.concatenate([sel, np.arange(n - n_local, n)]), margin


def compress_h2o(q_full, K, V, B, n_local, scale=None, retained_override=None):
    """Alg. 1 steps 3-8 with H2O as the eviction strategy f, one sequence.

    q_full [Hq][n][D] all prompt queries; K, V [Hkv][n][D].  The calibration query is Q_{-1}.
    Returns the dict of compress_given plus vote (list per KV head) and margin [Hkv]."""
    q_full = np.asarray(q_full, F)
    K = np.asarray(K, F)
    Hq, n, D = q_full.shape
    Hkv = K.shape[0]
    G = Hq // Hkv
    if scale is None:
        scale = 1.0 / np.sqrt(D)
    votes, kept, margins = [], [], []
    for g in range(Hkv):
        if n <= B:
            votes.append(None); kept.append(np.arange(n)); margins.append(np.inf)
            continue
        vote = h2o_votes(q_full[g * G:(g + 1) * G], K[g], scale)
        keep, margin = h2o_retained(vote, n, B, n_local)
        if retained_override is not None:
            keep, margin = np.asarray(retained_override[g]), np.inf
        votes.append(vote); kept.append(keep); margins.append(margin)
    r = compress_given(q_full[:, n - 1], K, V, B, kept, scale)
    r["vote"], r["margin"] = votes, np.asarray(margins)
    r["score"] = votes
    return r


# --------------------------------------------------------------------------------------------
# Alg. 2 (decode side), one sequence, one step
# --------------------------------------------------------------------------------------------
FLAG_NONE, FLAG_CALIBRATED, FLAG_RECOMPUTE, FLAG_RECOMPUTED = 0, 1, 2, 3


def cosine(a, b):
    """rho = cos(a, b); 0 when either vector has zero norm."""
    a = np.asarray(a, F)
    b = np.asarray(b, F)
    na, nb = np.sqrt(a @ a), np.sqrt(b @ b)
    if na == 0.0 or nb == 0.0:
        return 0.0
    return (a @ b) / (na * nb)


def decode(q_t, K_c, V_c, length, c_q, c_out, c_lse, theta1, theta2, scale=None):
    """Alg. 2 for one sequence: attention over the compressed cache, cosine gate, Eq. 1 merge.

    q_t [Hq][D]; K_c, V_c [Hkv][cap][D] of which the first `length` rows are live.
    The recompute branch (rho < theta1) is only flagged: the output there is the uncalibrated
    attention (recomputation needs the evicted K/V, which this entry point does not take).
    Returns (out [Hq][D], a_lse [Hq], flags [Hq] uint8, rho [Hq])."""
    q_t = np.asarray(q_t, F)
    Hq, D = q_t.shape
    Hkv = np.asarray(K_c).shape[0]
    G = Hq // Hkv
    if scale is None:
        scale = 1.0 / np.sqrt(D)
    out = np.zeros((Hq, D), F)
    a_lse = np.zeros(Hq, F)
    flags = np.zeros(Hq, np.uint8)
    rhos = np.zeros(Hq, F)
    t1, t2 = np.float32(theta1), np.float32(theta2)
    for h in range(Hq):
        g = h // G
        o_a, lse_a = attention(q_t[h], np.asarray(K_c[g], F)[:length],
                               np.asarray(V_c[g], F)[:length], scale)      # Alg. 2 step 1
        rho = cosine(q_t[h], c_q[h])                                       # Alg. 2 step 2
        rho32 = np.float32(rho)                                            # decision precision
        rhos[h] = rho
        a_lse[h] = lse_a
        if rho32 < t1:                                                     # recompute branch
            flags[h] = FLAG_RECOMPUTE
            out[h] = o_a
        elif rho32 > t2 and c_lse[h] > -np.inf:                            # calibrate (Eq. 1)
            flags[h] = FLAG_CALIBRATED
            out[h], _ = merge(o_a, lse_a, c_out[h], c_lse[h])
        else:
            out[h] = o_a
    return out, a_lse, flags, rhos


def recalibrate(q_t, K, V, idx, flags, a_lse, out, c_q, c_out, c_lse, scale=None, cal_idx=None):
    """Alg. 2 steps 3-8 (the rho < theta1 branch) for the heads that `decode` flagged.

    The evicted K/V are the rows of the prompt tensors K, V [Hkv][n][D] that are not in
    idx [Hkv][B] (Alg. 1 step 4: KV_evict = KV_full minus KV_compress, frozen at prefill).  For every head with
    flag FLAG_RECOMPUTE: C_weight and C_out are recomputed with the CURRENT query (the prose of
    Sec. 3.2; the listing prints Q_{-1} but then sets C_q = Q_t), C_q = Q_t, and the output is
    calibrated by Eq. 1: out = alpha_i * out + alpha_j * C_out.  `out`, `a_lse` are what decode
    returned for this step.  With a calibration size (Sec. 5.3) only the offloaded subset exists:
    cal_idx [Hkv][m] lists its positions (-1 padded) and replaces "every evicted token".
    Returns new (out, flags, c_q, c_out, c_lse); inputs are not modified."""
    q_t = np.asarray(q_t, F)
    K = np.asarray(K, F)
    V = np.asarray(V, F)
    Hq, D = q_t.shape
    Hkv, n, _ = K.shape
    G = Hq // Hkv
    if scale is None:
        scale = 1.0 / np.sqrt(D)
    out = np.array(out, F)
    flags = np.array(flags, np.uint8)
    c_q, c_out, c_lse = np.array(c_q, F), np.array(c_out, F), np.array(c_lse, F)
    for h in range(Hq):
        if flags[h] != FLAG_RECOMPUTE:
            continue
        g = h // G
        keep = np.asarray(idx[g])
        mask = np.ones(n, bool)
        mask[keep[(keep >= 0) & (keep < n)]] = False
        ev = np.nonzero(mask)[0]
        if cal_idx is not None:
            ci = np.asarray(cal_idx[g])
            ev = ci[ci >= 0]
        c_out[h], c_lse[h] = attention(q_t[h], K[g][ev], V[g][ev], scale)     # steps 5-6
        c_q[h] = q_t[h]                                                       # step 7
        out[h], _ = merge(out[h], a_lse[h], c_out[h], c_lse[h])               # step 8 (Eq. 1)
        flags[h] = FLAG_RECOMPUTED
    return out, flags, c_q, c_out, c_lse
