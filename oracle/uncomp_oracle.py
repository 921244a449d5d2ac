"""Float64 CPU oracle for UNComp's prefill-time KV compression pass.

TEST INFRASTRUCTURE ONLY.  This module is the slow, plain statement of what the
hot path computes, written from the paper.  It shares no code with the HIP
library and must never be imported by the product package: only tests, the
smoke check and the bench's cpu_baseline leg may call it.

Everything is numpy float64.  Library primitives used as single steps:
``numpy.linalg.eigvalsh`` (eigenvalues of a symmetric matrix), ``@`` (matmul),
``numpy.argsort`` (stable sort).  No blocking, fusion or reordering beyond what
the definitions state.

Parity status of each function (what pins it lives in tests/test_oracle_*.py):

* head_entropy      pinned: closed-form spectra, isotropic / rank-1 closed
                    forms, 2x2 analytic eigenvalues, Lemma-4 bounds, invariances.
* assign_budgets    head budgets pinned by the paper's printed budget vectors
                    (Sec. 4.2 "Main Results"; App. "Number of Head Groups" table).
                    layer_group / layer_tokens: PARITY UNPINNED (the paper prints
                    no worked example for Eq. 8-10; only the arithmetic of the
                    reading below is checked, by a hand-worked case).
* window_score      pinned: uniform-attention closed form (causal harmonic sums),
                    single-row reduction to a library softmax, probability-mass
                    conservation, spike -> plateau behaviour of the max-pool.
* window_lse        pinned: zero queries give ln(P+i+1), a library logsumexp per causal
                    row, and exp(logit - lse) summed over the window reproduces window_score
                    with pool 1.
* select_gather     pinned: exhaustive subset search on tiny inputs, structural
                    invariants, byte compare of gathered rows.
* decode_init /     pinned: without eviction the cumulative scores of T decode steps
  decode_step       equal the unpooled window score of the same T queries (the prefill
                    function above, itself pinned); equal keys give the uniform closed
                    form (each entry gains G/n, the output is the mean value row);
                    probability mass G per step; a dominant key takes the whole step;
                    the evicted entry checked by exhaustive search on tiny caches;
                    occupancy and recent-window invariants over long runs.
* hidden_evict      pinned: the score equals the head sum of the pinned window score with
                    a one-token window and no pooling; zero queries give the uniform 1/N
                    closed form (ties then keep the lowest positions); total mass = number
                    of query heads; a dominant key is always kept; exhaustive subset
                    search on tiny inputs; rows copied bit for bit.
* prepare_* /       pinned: hand-worked two-sample example (mean and vote labellings that
  budgets_from_     differ), one sample reproduces assign_budgets' groups, sample order
  labels            does not matter, vote ties go to the lower label, budgets from labels
                    equal the paper's printed budget vector.
"""
from __future__ import annotations

import numpy as np

# Flag bits (same numeric values as the C header so tests can pass one integer
# to both sides; the values are interface, not arithmetic).
FLAG_CENTER = 1          # Eq. 1 centred covariance (otherwise X^T X, as in the proof of Lemma 3)
FLAG_TRUNC_RENORM = 2    # renormalise the top-k eigenvalues to sum to one
FLAG_LAYER_DELTA_INCREASE = 4  # Alg. 2 sign for the layer partition instead of Eq. 8
DEFAULT_FLAGS = FLAG_CENTER | FLAG_TRUNC_RENORM


# --------------------------------------------------------------------------
# O1  truncated matrix entropy  (Sec. 3.1 Eq. 1, Lemma 2; Sec. 3.2 Eq. 5-6;
#     trace-one normalisation from the proof of Lemma 4)
# --------------------------------------------------------------------------
def covariance(X: np.ndarray, center: bool = True) -> np.ndarray:
    """Sec. 3.1 Eq. 1: Sigma = 1/(N-1) sum_i (x_i - xbar)(x_i - xbar)^T for the
    token matrix X (N rows = tokens, D columns).  With ``center=False`` the
    uncentred form X^T X/(N-1) used in the proof of Lemma 3.  N < 2 gives the
    zero matrix (no spread can be measured from one token)."""
    X = np.asarray(X, dtype=np.float64)
    N, D = X.shape
    if N < 2:
        return np.zeros((D, D))
    if center:
        xbar = X.mean(axis=0)
        Xc = X - xbar
    else:
        Xc = X
    return (Xc.T @ Xc) / (N - 1)


def spectrum(Sigma: np.ndarray) -> np.ndarray:
    """Eigenvalues of Sigma scaled to unit trace (proof of Lemma 4: Tr Sigma = 1),
    sorted descending; rounding negatives are clamped to zero.  A zero matrix
    returns all zeros."""
    lam = np.linalg.eigvalsh(np.asarray(Sigma, dtype=np.float64))[::-1].copy()
    lam[lam < 0.0] = 0.0
    tr = lam.sum()
    if tr <= 0.0:
        return np.zeros_like(lam)
    return lam / tr


def truncated_entropy(p: np.ndarray, k: int, renorm: bool = True) -> float:
    """Sec. 3.2 Eq. 5: H_k = - sum_{i<=k} s_i log s_i over the k largest
    eigenvalues (natural log; 0 log 0 = 0).  ``p`` is the unit-trace spectrum,
    descending.  renorm=True: s_i = p_i / sum_{j<=k} p_j (the top-k block treated
    as a density of its own, so the bound H_k <= log k of Lemma 4 is attained by
    an isotropic matrix); renorm=False: s_i = p_i, Eq. 5 symbol for symbol."""
    k = int(min(k, p.shape[0]))
    s = np.asarray(p[:k], dtype=np.float64)
    if renorm:
        tot = s.sum()
        if tot <= 0.0:
            return 0.0
        s = s / tot
    s = s[s > 0.0]
    return float(-(s * np.log(s)).sum())


def head_entropy(X: np.ndarray, k_trunc: int = 32, flags: int = DEFAULT_FLAGS):
    """Truncated matrix entropy of each token matrix in X [n_mat, N, D].
    Returns (H [n_mat] float64, eig [n_mat, D] unit-trace spectrum descending).
    erank_k = exp(H) (Eq. 6)."""
    X = np.asarray(X, dtype=np.float64)
    n_mat, N, D = X.shape
    H = np.zeros(n_mat)
    eig = np.zeros((n_mat, D))
    for m in range(n_mat):
        p = spectrum(covariance(X[m], center=bool(flags & FLAG_CENTER)))
        eig[m] = p
        H[m] = truncated_entropy(p, k_trunc, renorm=bool(flags & FLAG_TRUNC_RENORM))
    return H, eig


# --------------------------------------------------------------------------
# O2  budgets  (Sec. 3.3.3 "Design", Eq. 11; Sec. 3.3.2 Eq. 8-10)
# --------------------------------------------------------------------------
def assign_budgets(entropy, M: int, n_max: int, step: int, N: int, w: int,
                   eps: float, delta_n: int, flags: int = DEFAULT_FLAGS):
    """entropy [L, B, H] (the float32 values the entropy stage emitted; they are
    widened to float64 here, so both sides rank the same numbers).

    Head budgets, per (layer, batch): heads are ranked by truncated entropy,
    largest first (ties: lower head index first), cut into M groups of H/M heads
    in rank order, and group g (0-based) gets N_{i,1} - g*step tokens (Eq. 11:
    an arithmetic progression starting from n_max for the highest-entropy
    group), clamped to [min(w, N), N].

    Layer stages: e_l = mean over (b, h) of erank_k = exp(H); walking the layers,
    a new compression stage starts after layer l when e_l - e_{l+1} > eps
    (Eq. 8-9; with FLAG_LAYER_DELTA_INCREASE the sign of Alg. 2's prefill test,
    e_{l+1} - e_l > eps).  layer_group[l] = number of boundaries before l;
    layer_tokens[l] = max(N - layer_group[l]*delta_n, w): the first stage keeps
    all tokens, each later stage delta_n fewer (Eq. 10 read so that it
    compresses).  Returns int32 arrays head_budget [L,B,H], head_group [L,B,H],
    layer_group [L], layer_tokens [L]."""
    e = np.asarray(entropy, dtype=np.float32).astype(np.float64)
    L, B, H = e.shape
    assert H % M == 0
    per = H // M
    head_budget = np.zeros((L, B, H), dtype=np.int32)
    head_group = np.zeros((L, B, H), dtype=np.int32)
    lo = min(w, N)
    for l in range(L):
        for b in range(B):
            order = sorted(range(H), key=lambda h: (-e[l, b, h], h))
            for rank, h in enumerate(order):
                g = rank // per
                head_group[l, b, h] = g
                head_budget[l, b, h] = min(max(n_max - g * step, lo), N)
    erank = np.exp(e)
    layer_mean = np.array([erank[l].sum() / (B * H) for l in range(L)])
    layer_group = np.zeros(L, dtype=np.int32)
    layer_tokens = np.zeros(L, dtype=np.int32)
    c = 0
    for l in range(L):
        if l > 0:
            d = layer_mean[l - 1] - layer_mean[l]
            if flags & FLAG_LAYER_DELTA_INCREASE:
                d = -d
            if d > eps:
                c += 1
        layer_group[l] = c
        layer_tokens[l] = max(N - c * delta_n, w)
    return head_budget, head_group, layer_group, layer_tokens


# --------------------------------------------------------------------------
# O3  observation-window score  (Sec. 3.3.3 "Dynamic KV Cache Eviction":
#     sum of the attention of the last l tokens; pooling and GQA group sum are
#     the benchmark's statement of the scoring step)
# --------------------------------------------------------------------------
def window_score(Qwin: np.ndarray, K: np.ndarray, G: int, pool: int) -> np.ndarray:
    """Qwin [B, Hq, w, D] are the queries of the last w positions, K [B, H, N, D]
    all keys (Hq = G*H, query head q reads KV head q // G).  For window row i at
    position P+i (P = N-w) the attention row is softmax_j(q_i . k_j / sqrt(D))
    over the causal range j <= P+i.  vote_q[j] = sum_i p_ij for prefix tokens
    j < P; pooled_q[j] = max of vote_q over the |j'-j| <= pool//2 neighbours that
    lie inside the prefix; score[b,h,j] = sum of pooled_q over the G query heads
    of KV head h.  Returns [B, H, P] float64."""
    Qwin = np.asarray(Qwin, dtype=np.float64)
    K = np.asarray(K, dtype=np.float64)
    B, Hq, w, D = Qwin.shape
    _, H, N, _ = K.shape
    assert Hq == G * H and pool % 2 == 1 and 0 < w < N
    P = N - w
    half = pool // 2
    score = np.zeros((B, H, P))
    for b in range(B):
        for q in range(Hq):
            h = q // G
            logits = (Qwin[b, q] @ K[b, h].T) / np.sqrt(D)      # [w, N]
            vote = np.zeros(P)
            for i in range(w):
                row = logits[i, : P + i + 1]
                ex = np.exp(row - row.max())
                prob = ex / ex.sum()
                vote += prob[:P]
            pooled = np.empty(P)
            for j in range(P):
                pooled[j] = vote[max(0, j - half): min(P, j + half + 1)].max()
            score[b, h] += pooled
    return score


def window_lse(Qwin: np.ndarray, K: np.ndarray, G: int) -> np.ndarray:
    """Natural-log normaliser of every window row of window_score: for row i of
    query head q at position P+i, ln sum_{j <= P+i} exp(q_i . k_j / sqrt(D)).  It is
    what an attention kernel keeps per row beside its output; the library accepts
    it in place of its own statistics pass.  Returns [B, Hq, w] float64."""
    Qwin = np.asarray(Qwin, dtype=np.float64)
    K = np.asarray(K, dtype=np.float64)
    B, Hq, w, D = Qwin.shape
    _, H, N, _ = K.shape
    assert Hq == G * H and 0 < w < N
    P = N - w
    out = np.empty((B, Hq, w))
    for b in range(B):
        for q in range(Hq):
            logits = (Qwin[b, q] @ K[b, q // G].T) / np.sqrt(D)      # [w, N]
            for i in range(w):
                row = logits[i, : P + i + 1]
                m = row.max()
                out[b, q, i] = m + np.log(np.exp(row - m).sum())
    return out


# --------------------------------------------------------------------------
# O4  per-head top-k and compaction  (Sec. 3.3.3: keep the N_{i,g} tokens with
#     the highest scores; Alg. 2 prefill: compress each head by its group)
# --------------------------------------------------------------------------
def select_indices(score_row: np.ndarray, budget: int, N: int, w: int) -> np.ndarray:
    """Kept positions of one head, ascending.  The w window positions are always
    kept and count towards the budget; the remaining budget-w slots go to the
    prefix tokens of largest score, equal scores resolved towards the lower
    position.  budget is clamped to [min(w,N), N]; if it is below w only the last
    ``budget`` positions survive."""
    P = N - w
    budget = int(min(max(int(budget), min(w, N)), N))
    keep_prefix = min(max(budget - w, 0), P)
    order = np.argsort(-np.asarray(score_row, dtype=np.float64), kind="stable")
    chosen = np.sort(order[:keep_prefix])
    n_win = min(budget, w)
    window = np.arange(N - n_win, N)
    return np.concatenate([chosen, window]).astype(np.int32)


def select_gather(score, budget, K, V, w: int, cap: int):
    """score [B,H,P], budget [B,H] int, K/V [B,H,N,D] (any dtype; rows are copied
    verbatim).  Returns K_out, V_out [B,H,cap,D] (rows >= len zero), idx
    [B,H,cap] int32 (entries >= len are -1), length [B,H] int32."""
    B, H, N, D = K.shape
    K_out = np.zeros((B, H, cap, D), dtype=K.dtype)
    V_out = np.zeros((B, H, cap, D), dtype=V.dtype)
    idx = np.full((B, H, cap), -1, dtype=np.int32)
    length = np.zeros((B, H), dtype=np.int32)
    for b in range(B):
        for h in range(H):
            sel = select_indices(score[b, h], budget[b, h], N, w)
            n = sel.shape[0]
            assert n <= cap
            length[b, h] = n
            idx[b, h, :n] = sel
            for r in range(n):
                K_out[b, h, r] = K[b, h, sel[r]]
                V_out[b, h, r] = V[b, h, sel[r]]
    return K_out, V_out, idx, length


# --------------------------------------------------------------------------
# O5  decode-time eviction  (Sec. 3.3.3 "Dynamic KV Cache Eviction", last
#     sentence; Alg. 2 "Decoding": the new token joins the head's cache, the
#     query attends to the joined cache, then the cache is updated)
# --------------------------------------------------------------------------
def decode_init(score_row: np.ndarray, idx: np.ndarray, N: int, w: int) -> np.ndarray:
    """Cumulative scores a head's compacted cache starts decoding with: the
    prefill score of every kept prefix position (position < N-w).  The w window
    positions carry no prefill score (they were kept unconditionally) and start
    at zero, like every token that joins later."""
    P = N - w
    score_row = np.asarray(score_row, dtype=np.float64)
    return np.array([score_row[j] if j < P else 0.0 for j in np.asarray(idx)], dtype=np.float64)


def decode_step(Kc: np.ndarray, Vc: np.ndarray, idx: np.ndarray, cum: np.ndarray,
                q: np.ndarray, k_new: np.ndarray, v_new: np.ndarray, pos: int,
                budget: int, w: int, decide_dtype=np.float32):
    """One generated token for one KV head.

    Kc, Vc [n, D] are the head's cached rows, idx [n] their original positions
    (distinct, all < pos), cum [n] their cumulative scores; q [G, D] the new
    token's G query heads, k_new / v_new [D] its key and value, pos its position.

    1. the new token joins the cache with cumulative score 0;
    2. every query head attends to the n+1 entries:
       p_g = softmax_j(q_g . k_j / sqrt(D)), out_g = sum_j p_gj v_j;
    3. every entry's cumulative score grows by sum_g p_gj;
    4. if the cache now holds more than ``budget`` entries (a budget below w counts
       as w, as at prefill), the entry of lowest cumulative score leaves.  The most recent w positions (pos-w+1 .. pos) are
       exempt, as the observation window is at prefill; equal scores resolve
       towards the older position.  The comparison is made on scores rounded to
       ``decide_dtype`` (the precision the compared path keeps them in).

    Returns (Kc, Vc, idx, cum, out [G, D], evicted position or -1), entries in
    ascending position order."""
    Kc = np.asarray(Kc, dtype=np.float64)
    Vc = np.asarray(Vc, dtype=np.float64)
    q = np.asarray(q, dtype=np.float64)
    n, D = Kc.shape
    assert w >= 1
    budget = max(int(budget), w)
    keys = np.concatenate([Kc, np.asarray(k_new, dtype=np.float64)[None, :]], axis=0)
    vals = np.concatenate([Vc, np.asarray(v_new, dtype=np.float64)[None, :]], axis=0)
    where = np.concatenate([np.asarray(idx, dtype=np.int64), [pos]])
    total = np.concatenate([np.asarray(cum, dtype=np.float64), [0.0]])
    G = q.shape[0]
    out = np.zeros((G, D))
    for g in range(G):
        logits = keys @ q[g] / np.sqrt(D)
        ex = np.exp(logits - logits.max())
        prob = ex / ex.sum()
        out[g] = prob @ vals
        total = total + prob
    evicted = -1
    if n + 1 > budget:
        seen = total.astype(decide_dtype)
        best = -1
        for j in range(n + 1):
            if where[j] > pos - w:
                continue
            if best < 0 or seen[j] < seen[best] or (seen[j] == seen[best] and where[j] < where[best]):
                best = j
        assert best >= 0
        evicted = int(where[best])
        keep = np.arange(n + 1) != best
        keys, vals, where, total = keys[keep], vals[keep], where[keep], total[keep]
    return keys, vals, where.astype(np.int32), total, out, evicted


# --------------------------------------------------------------------------
# O6  stage-1 hidden-state eviction  (Sec. 3.3.2 "Hidden State Eviction": the
#     tokens entering layer i+1 are the N_{i+1} that receive the most attention
#     from the last token in layer i; N_{i+1} from Eq. 10)
# --------------------------------------------------------------------------
def last_token_score(q_last: np.ndarray, K: np.ndarray, G: int) -> np.ndarray:
    """q_last [Hq, D] the last position's queries, K [H, N, D] the layer's keys
    (query head q reads KV head q // G).  score[j] = sum over the Hq query heads
    of softmax_j(q . k_j / sqrt(D)), the last token attending to all N positions."""
    q_last = np.asarray(q_last, dtype=np.float64)
    K = np.asarray(K, dtype=np.float64)
    Hq, D = q_last.shape
    N = K.shape[1]
    score = np.zeros(N)
    for q in range(Hq):
        logits = K[q // G] @ q_last[q] / np.sqrt(D)
        ex = np.exp(logits - logits.max())
        score += ex / ex.sum()
    return score


def hidden_evict(q_last, K, Hs, n_keep: int, w: int, G: int):
    """q_last [B, Hq, D], K [B, H, N, D], Hs [B, N, Dm] (any dtype; rows are copied
    verbatim).  Per batch entry the n_keep positions that survive are the last w
    (kept unconditionally: the last token carries the next prediction) plus the
    n_keep - w earlier positions of largest last-token score, equal scores
    towards the lower position; n_keep is clamped to [min(w, N), N].  Returns
    (rows [B, n, Dm], idx [B, n] int32 ascending, score [B, N] float64)."""
    B, N = Hs.shape[0], Hs.shape[1]
    rows, idx, scores = [], [], []
    for b in range(B):
        sc = last_token_score(q_last[b], K[b], G)
        sel = select_indices(sc[: N - w], n_keep, N, w)
        rows.append(np.stack([Hs[b, j] for j in sel]) if len(sel) else Hs[b, :0])
        idx.append(sel)
        scores.append(sc)
    return np.stack(rows), np.stack(idx), np.stack(scores)


# --------------------------------------------------------------------------
# O7  offline preparation  (Sec. 3.3.1 "Preparation Stage", Eq. 7: the grouping
#     metric of a head is its erank averaged over the d sampled prompts;
#     App. "A Comprehensive Walk-Through", Alg. 1: per sample every head gets one
#     of M labels from its entropy, the final label is the majority's)
# --------------------------------------------------------------------------
def _rank_groups(values: np.ndarray, M: int) -> np.ndarray:
    """Group index of each of the H entries: rank by value, largest first, equal
    values by lower index; rank r falls in group r // (H/M)."""
    H = values.shape[0]
    order = np.argsort(-np.asarray(values, dtype=np.float64), kind="stable")
    group = np.empty(H, dtype=np.int32)
    group[order] = np.arange(H) // (H // M)
    return group


def prepare_new(L: int, H: int, M: int) -> dict:
    return {"erank_sum": np.zeros((L, H)), "votes": np.zeros((L, H, M), dtype=np.int64), "count": 0}


def prepare_accumulate(state: dict, entropy: np.ndarray, M: int) -> None:
    """Adds the B samples of entropy [L, B, H] to the running statistics: the sum of
    erank = exp(entropy) per (layer, head) for Eq. 7, and one vote per sample for the
    label the head gets inside its layer in that sample (Alg. 1; the labels are the
    M equal-size rank groups of Sec. 3.3.3, the paper names no other clustering)."""
    entropy = np.asarray(entropy)
    L, B, H = entropy.shape
    for b in range(B):
        for l in range(L):
            e = entropy[l, b].astype(np.float64)
            state["erank_sum"][l] += np.exp(e)
            g = _rank_groups(e, M)
            for h in range(H):
                state["votes"][l, h, g[h]] += 1
        state["count"] += 1


def prepare_finish(state: dict, M: int):
    """Returns (labels_mean [L, H], labels_vote [L, H], mean_erank [L, H]).
    labels_mean: heads of a layer ranked by their mean erank (Eq. 7) into M groups,
    group 0 = largest.  labels_vote: the label most samples gave the head, equal
    counts towards the lower label."""
    mean = state["erank_sum"] / max(state["count"], 1)
    L, H = mean.shape
    labels_mean = np.stack([_rank_groups(mean[l], M) for l in range(L)])
    labels_vote = np.zeros((L, H), dtype=np.int32)
    for l in range(L):
        for h in range(H):
            best = 0
            for g in range(1, M):
                if state["votes"][l, h, g] > state["votes"][l, h, best]:
                    best = g
            labels_vote[l, h] = best
    return labels_mean, labels_vote, mean


def budgets_from_labels(labels: np.ndarray, B: int, n_max: int, step: int, N: int, w: int) -> np.ndarray:
    """Eq. 11 from stored labels: head_budget[l, b, h] = clamp(n_max - label*step,
    min(w, N), N), the same for every batch entry."""
    labels = np.asarray(labels)
    bud = np.clip(n_max - labels.astype(np.int64) * step, min(w, N), N).astype(np.int32)
    return np.repeat(bud[:, None, :], B, axis=1)
