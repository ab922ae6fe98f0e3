"""CPU oracle for head-aware KV-cache compression in next-scale generation.

TEST INFRASTRUCTURE ONLY.  Nothing in the product path may import this file;
only tests/, the smoke check and the benchmark's cpu_baseline leg use it.  It
shares no code with the HIP library and never calls it.

Everything is float64 numpy, written in the order and notation of the paper
(arXiv 2504.09261).  The method is a heuristic (it changes the attention
result), so the oracle is the algorithm taken step by step; only with a budget
that covers the whole cache does it reduce to plain full-cache attention.

Notation (paper, Preliminaries and Sec. 4):
  N_k   tokens of the current scale            T_k  uncompressed cache length
  Q_k   queries of the current scale [N_k, D_h]
  K, V  one head's cache (rows = tokens)       B_C, B_S  per-class budgets
  N_obs observation queries (32)               N_init tokens of the first two scales

Readings taken where the paper is silent:
  * softmax scale is an explicit argument (the equations print none);
  * "uniformly sample" = the evenly strided rows floor(i*N_k/n_obs);
  * n_obs = min(N_obs, N_k);
  * TOPK ties go to the lowest index; kept rows stay in ascending index order;
  * the structural TOPK ranks only the intermediate segment;
  * a structural budget too small for init + recent keeps the init rows and
    the highest-scoring recent rows (parity unpinned: no passage fixes this);
  * the ranking is decided on importance rounded to float32, the precision in
    which the device stores it, so that both sides decide on the same numbers;
  * the attention variance of the head classification is the population
    variance; alpha * L * H is rounded to the nearest integer;
  * the final-step merge of contextual heads (the paper names the operation and
    defers its definition to another work: parity unpinned against that work):
    similarity = cosine similarity between key rows; an evicted row's nearest
    retained counterpart = the kept row of highest similarity (ties to the lower
    index, decided on similarities rounded to float32, the device's precision);
    the kept row becomes the weighted average of itself (weight 1) and the rows
    merged into it (weight = their similarity, negative ones count as 0), keys
    and values with the same weights.

Pinned by tests/test_oracle_pins.py (brute force in pure Python on tiny
inputs, closed forms, invariants, the full-budget reduction to plain attention
and the complexity closed form of the supplementary analysis); the pins
themselves are checked by tests/test_oracle_mutations.py, which plants
mistakes into this file's functions and requires a pin to fail.
"""
from __future__ import annotations

import numpy as np

CONTEXTUAL = 0
STRUCTURAL = 1


# ---------------------------------------------------------------------------
# Sec. 4.4, "Importance Estimation via Efficient Subset Attention"
# ---------------------------------------------------------------------------
def observation_rows(N_k: int, N_obs: int = 32) -> np.ndarray:
    """Row ids of the uniformly sampled query subset (evenly strided)."""
    n_obs = min(N_obs, N_k)
    i = np.arange(n_obs, dtype=np.int64)
    return (i * N_k) // n_obs


def softmax_rows(S: np.ndarray) -> np.ndarray:
    """Row-wise softmax of a float64 matrix (max-shifted)."""
    S = S - S.max(axis=1, keepdims=True)
    E = np.exp(S)
    return E / E.sum(axis=1, keepdims=True)


def subset_attention(Q_obs: np.ndarray, K: np.ndarray, scale: float) -> np.ndarray:
    """A~ = Softmax(scale * Q~ K^T)  (subset-attention equation, Sec. 4.4).
    K is the uncompressed key matrix of this step: retained cache rows followed
    by the current scale's rows (supplementary complexity analysis)."""
    return softmax_rows(scale * (Q_obs @ K.T))


def importance(Q_obs: np.ndarray, K: np.ndarray, scale: float) -> np.ndarray:
    """Cumulative attention score of every key: sum_i A~[i, :] (f_C / f_S equations)."""
    return subset_attention(Q_obs, K, scale).sum(axis=0)


# ---------------------------------------------------------------------------
# Sec. 4.2, "Offline Head Classification via Attention Variance"
# ---------------------------------------------------------------------------
def head_variance(Q: np.ndarray, K: np.ndarray, scale: float) -> float:
    """sigma = sum_j Var(A[:, j]) with A = Softmax(scale * Q K^T) the attention
    matrix of the final step over the full (uncompressed) cache: the sum of the
    column-wise variances across queries (variance equation of Sec. 4.2).
    Reading: population variance (divide by the number of queries); the sample
    variance differs by the constant factor N/(N-1), which no ranking sees."""
    A = softmax_rows(scale * (Q @ K.T))
    mean = A.sum(axis=0) / A.shape[0]
    return float((((A - mean) ** 2).sum(axis=0) / A.shape[0]).sum())


def classify_heads(sigma: np.ndarray, alpha: float) -> np.ndarray:
    """Global ranking of all (layer, head) variance scores: the round(alpha * L * H)
    heads of lowest variance are contextual (0), the others structural (1).
    Ties go to the lower flat index.  sigma has shape [L, H] (or [H])."""
    sigma = np.asarray(sigma, dtype=np.float64)
    flat = sigma.reshape(-1)
    n_ctx = int(round(float(alpha) * flat.shape[0]))
    order = np.argsort(flat, kind="stable")
    types = np.full(flat.shape[0], STRUCTURAL, dtype=np.uint8)
    types[order[:n_ctx]] = CONTEXTUAL
    return types.reshape(sigma.shape)


# ---------------------------------------------------------------------------
# Sec. 4.4, selection policies
# ---------------------------------------------------------------------------
def decision_values(imp: np.ndarray) -> np.ndarray:
    """Importance in the precision the ranking is decided in (float32)."""
    return np.asarray(imp, dtype=np.float64).astype(np.float32)


def topk_indices(values: np.ndarray, k: int) -> np.ndarray:
    """Indices of the k largest values; equal values go to the lower index.
    Returned in ascending index order."""
    k = int(k)
    if k <= 0:
        return np.zeros(0, np.int64)
    n = values.shape[0]
    if k >= n:
        return np.arange(n, dtype=np.int64)
    order = np.argsort(-values, kind="stable")      # stable: lower index first among equals
    return np.sort(order[:k]).astype(np.int64)


def select_contextual(imp: np.ndarray, B_C: int) -> np.ndarray:
    """f_C: I = TOPK(importance, B_C) over the whole cache."""
    return topk_indices(decision_values(imp), min(int(B_C), imp.shape[0]))


def select_structural(imp: np.ndarray, B_S: int, N_init: int, N_k: int) -> np.ndarray:
    """f_S: first N_init rows + TOPK(importance, M) among the intermediate rows
    + last N_k rows, with M = B_S - N_init - N_k."""
    T = imp.shape[0]
    B_S = min(int(B_S), T)
    vals = decision_values(imp)
    n_rec = min(int(N_k), T)
    n0 = min(int(N_init), T - n_rec)
    M = B_S - n0 - n_rec
    if M >= 0:
        init = np.arange(n0, dtype=np.int64)
        mid = n0 + topk_indices(vals[n0:T - n_rec], M)
        rec = np.arange(T - n_rec, T, dtype=np.int64)
        return np.concatenate([init, mid, rec])
    # Budget smaller than init + recent (the paper is silent; this reading is unpinned):
    # the init rows first, then the best of the recent scale, nothing from the middle.
    n_keep0 = min(n0, B_S)
    init = np.arange(n_keep0, dtype=np.int64)
    rec = (T - n_rec) + topk_indices(vals[T - n_rec:], B_S - n_keep0)
    return np.concatenate([init, rec])


def select(imp: np.ndarray, head_type: int, budget: int, N_init: int, N_k: int) -> np.ndarray:
    if head_type == CONTEXTUAL:
        return select_contextual(imp, budget)
    return select_structural(imp, budget, N_init, N_k)


# ---------------------------------------------------------------------------
# gather and attention
# ---------------------------------------------------------------------------
def compact(K: np.ndarray, V: np.ndarray, I: np.ndarray):
    """K^ = K[I, :], V^ = V[I, :]."""
    return K[I], V[I]


def attention(Q: np.ndarray, K: np.ndarray, V: np.ndarray, scale: float) -> np.ndarray:
    """O = Softmax(scale * Q K^T) V over the whole (compressed) cache; no mask
    inside a scale step (Preliminaries, attention equation)."""
    return softmax_rows(scale * (Q @ K.T)) @ V


# ---------------------------------------------------------------------------
# Sec. 4.4, paragraph after the f_C equation: merge at the final generation step
# ---------------------------------------------------------------------------
def key_similarity(K_a: np.ndarray, K_b: np.ndarray) -> np.ndarray:
    """Cosine similarity between every row of K_a and every row of K_b (a row of
    zero norm is similar to nothing: 0)."""
    na = np.sqrt((K_a * K_a).sum(axis=1))
    nb = np.sqrt((K_b * K_b).sum(axis=1))
    S = K_a @ K_b.T
    den = na[:, None] * nb[None, :]
    return np.divide(S, den, out=np.zeros_like(S), where=den > 0)


def merge_final(K: np.ndarray, V: np.ndarray, I: np.ndarray):
    """Discarded rows are folded into their nearest retained counterparts by
    similarity-weighted averaging.  K, V [T, d]: the uncompressed cache of the step;
    I: ascending kept indices.  Returns (K^, V^, nearest, weight): the merged kept
    rows, and for every evicted row (ascending) the position in I of the row it
    was merged into and the weight it entered with."""
    T = K.shape[0]
    I = np.asarray(I, dtype=np.int64)
    evicted = np.setdiff1d(np.arange(T, dtype=np.int64), I)
    K_hat, V_hat = K[I].copy(), V[I].copy()
    if evicted.size == 0:
        return K_hat, V_hat, np.zeros(0, np.int64), np.zeros(0)
    S = key_similarity(K[evicted], K[I])
    nearest = np.argmax(S.astype(np.float32), axis=1)           # first maximum = lowest kept index
    weight = np.maximum(S[np.arange(evicted.size), nearest], 0.0)
    total = np.ones(I.size)                                      # the kept row itself enters with weight 1
    np.add.at(K_hat, nearest, weight[:, None] * K[evicted])
    np.add.at(V_hat, nearest, weight[:, None] * V[evicted])
    np.add.at(total, nearest, weight)
    return K_hat / total[:, None], V_hat / total[:, None], nearest.astype(np.int64), weight


# ---------------------------------------------------------------------------
# one unit = one (batch, head) pair
# ---------------------------------------------------------------------------
def unit_step(Kc, Vc, Pc, Qk, Kk, Vk, pos0, head_type, budget, N_init, scale,
              N_obs=32, q_rows=None, final_merge=False):
    """One scale step of one unit.

    Kc, Vc [L, d]: cache before the step;  Pc [L]: global token ids of its rows
    Qk, Kk, Vk [N_k, d]: this scale;       pos0: global id of this scale's first token
    final_merge: this is the last generation step; a contextual head that compresses
    merges what it discards into what it keeps (supplementary, Compression Setting:
    only f_C, only the final step).
    Returns dict(K, V, pos, O, imp, I, compressed).
    """
    N_k = Qk.shape[0]
    K_in = np.concatenate([Kc, Kk], axis=0)                 # cache update (Concat)
    V_in = np.concatenate([Vc, Vk], axis=0)
    P_in = np.concatenate([Pc, pos0 + np.arange(N_k, dtype=np.int64)])
    T_in = K_in.shape[0]
    imp = None
    I = None
    compressed = budget < T_in                              # "cache length exceeds its budget"
    if compressed:                                          # compress *before* attention
        rows = observation_rows(N_k, N_obs) if q_rows is None else np.asarray(q_rows)
        imp = importance(Qk[rows], K_in, scale)
        I = select(imp, head_type, budget, N_init, N_k)
        if final_merge and head_type == CONTEXTUAL:
            K_in, V_in, _, _ = merge_final(K_in, V_in, I)
        else:
            K_in, V_in = compact(K_in, V_in, I)
        P_in = P_in[I]
    O = attention(Qk, K_in, V_in, scale)
    return dict(K=K_in, V=V_in, pos=P_in, O=O, imp=imp, I=I, compressed=compressed)


def run_schedule(steps, head_types, budgets_per_step, N_init, scale, N_obs=32,
                 units=None, keep_outputs=True, final_merge=False):
    """Whole scale schedule of one layer.

    steps: list of (Q, K, V) float arrays [B, H, N_k, d], one per scale
    head_types: [H]; budgets_per_step: list of int arrays [B*H]
    final_merge: contextual heads merge at the last step of `steps` (see unit_step)
    Returns per step a list of per-unit dicts (see unit_step); evicted rows never
    come back (supplementary, Compression Setting).
    """
    B, H = steps[0][0].shape[:2]
    d = steps[0][0].shape[3]
    unit_ids = list(range(B * H)) if units is None else list(units)
    state = {u: (np.zeros((0, d)), np.zeros((0, d)), np.zeros(0, np.int64)) for u in unit_ids}
    pos0 = 0
    trace = []
    for k, (Q, K, V) in enumerate(steps):
        N_k = Q.shape[2]
        res = {}
        for u in unit_ids:
            b, h = divmod(u, H)
            Kc, Vc, Pc = state[u]
            r = unit_step(Kc, Vc, Pc,
                          np.asarray(Q[b, h], np.float64), np.asarray(K[b, h], np.float64),
                          np.asarray(V[b, h], np.float64), pos0, int(head_types[h]),
                          int(budgets_per_step[k][u]), N_init, scale, N_obs,
                          final_merge=final_merge and k == len(steps) - 1)
            state[u] = (r["K"], r["V"], r["pos"])
            if not keep_outputs:
                r = dict(pos=r["pos"], I=r["I"], compressed=r["compressed"], len=r["K"].shape[0])
            res[u] = r
        trace.append(res)
        pos0 += N_k
    return trace


# ---------------------------------------------------------------------------
# complexity model (Sec. 4.5 and the supplementary derivation)
# ---------------------------------------------------------------------------
def attention_cost_full(N):
    """sum_k N_k * T_k for a schedule given by its per-scale token counts."""
    T = np.cumsum(np.asarray(N, dtype=np.int64))
    return int((np.asarray(N, dtype=np.int64) * T).sum())


def attention_cost_budgeted(N, B):
    """sum_k N_k * min(T_k, B)."""
    N = np.asarray(N, dtype=np.int64)
    T = np.cumsum(N)
    return int((N * np.minimum(T, B)).sum())


def subset_attention_cost(N, B, k_s, N_obs=32):
    """sum_{k >= k_s} N_obs * (B + N_k), k_s 1-based."""
    N = np.asarray(N, dtype=np.int64)
    return int((N_obs * (B + N[k_s - 1:])).sum())
