"""CPU oracle for WindowKV's prefill-time window selection — TEST INFRASTRUCTURE ONLY.

A plain, slow, float64 statement of what the hot path computes, written from the paper
(WindowKV, arXiv 2503.17922, Section 2.2).  It shares no code with the HIP library and never
imports it.  Only the tests, the smoke check and the benchmark's ``cpu_baseline`` leg may
call it; the product path never does.

Every function takes plain numpy float64 arrays (callers widen bf16 / fp32 inputs exactly
before calling) and follows the paper's steps in the paper's order; nothing is blocked,
fused or reordered.  Notation: n = prefix length (``L``), alpha = observation window
(``w_obs``), omega = review-window size (``win``), p = top-p inside a window, gamma = layers
per group.

Readings taken where the paper is silent or ambiguous (each is listed in the design notes):
  * Eq. 2 prints closed index ranges; they are read half-open: rows n-alpha .. n-1 (exactly
    alpha observation queries), columns 0 .. n-alpha-1 (the review context).
  * Eq. 1 is "standard LLM" attention, so the softmax is causal over the whole prefix: the
    observation query at position q sees keys 0 .. q.  Only the last alpha columns are ever
    masked; they take part in the normaliser but receive no score t_j.
  * The paper shows one head; with grouped-query attention the scores of the query heads that
    share a KV head are summed, giving one score row and one index set per KV head.
  * Eq. 4 on a partial last window keeps the divisor min(p, omega) and takes the
    min(p, |W|) largest of the tokens that exist.
  * Equal window scores: the lower window index wins.  Kept rows are in ascending position.

Parity pins (tests/test_oracle_pins.py): rows of A sum to 1; a hand-built rational example
(tests/golden); torch's scaled_dot_product_attention with an identity V; closed forms for
zero queries (harmonic numbers) and two-level keys (pins the 1/sqrt(d) scale); mass
conservation; library pooling routines (mean / max_pool1d / topk); exhaustive search over all
window subsets; a scalar pure-Python re-derivation on tiny inputs; index_select for the
gather; scipy's logsumexp and ln(position+1) for the hand-over form of the normaliser;
torch's scaled_dot_product_attention, the mean of V for zero queries and a one-hot limit for
the decode step.
The absolute values of t and s on random data have no printed example in the paper:
beyond those pins they are "parity unpinned".  The value of p in aggregation mode, the
partial-window rule and the budget rounding are conventions of this repository (the paper
gives none) and are likewise "parity unpinned".
"""
from __future__ import annotations

import math
from typing import List, Sequence, Tuple

import numpy as np


# --------------------------------------------------------------------------------------
# Eq. 1 — attention probabilities of the observation queries
# --------------------------------------------------------------------------------------
def attention_probs(q_obs: np.ndarray, keys: np.ndarray, scale: float | None = None) -> np.ndarray:
    """Eq. 1 for one query head, restricted to the rows Eq. 2 uses.

    q_obs: [alpha, d]  the last alpha query vectors (positions n-alpha .. n-1)
    keys:  [n, d]      all key vectors of the prefix
    returns A: [alpha, n], A[i, j] = softmax_j( q_i . k_j / sqrt(d) ) over the keys the query
    at position n-alpha+i may see (j <= n-alpha+i); masked entries are 0.
    """
    q_obs = np.asarray(q_obs, dtype=np.float64)
    keys = np.asarray(keys, dtype=np.float64)
    alpha, d = q_obs.shape
    n = keys.shape[0]
    if scale is None:
        scale = 1.0 / math.sqrt(d)
    logits = (q_obs @ keys.T) * scale                       # Q . K^T / sqrt(d_k)
    pos_q = n - alpha + np.arange(alpha)[:, None]           # absolute position of each query
    visible = np.arange(n)[None, :] <= pos_q                # causal mask of a standard LLM
    logits = np.where(visible, logits, -np.inf)
    logits = logits - logits.max(axis=1, keepdims=True)
    e = np.exp(logits)
    return e / e.sum(axis=1, keepdims=True)


def softmax_lse(q_obs: np.ndarray, keys: np.ndarray, scale: float | None = None) -> np.ndarray:
    """The normaliser of Eq. 1 in the form an attention kernel hands it on: for each observation
    query i, lse_i = ln sum_{j <= n-alpha+i} exp(q_i . k_j / sqrt(d)), so A_ij = exp(logit_ij - lse_i).

    q_obs: [alpha, d], keys: [n, d]; returns [alpha].
    """
    q_obs = np.asarray(q_obs, dtype=np.float64)
    keys = np.asarray(keys, dtype=np.float64)
    alpha, d = q_obs.shape
    n = keys.shape[0]
    if scale is None:
        scale = 1.0 / math.sqrt(d)
    out = np.empty(alpha, dtype=np.float64)
    for i in range(alpha):
        logits = (keys[: n - alpha + i + 1] @ q_obs[i]) * scale    # the keys this query may see
        m = logits.max()
        out[i] = m + math.log(np.exp(logits - m).sum())
    return out


# --------------------------------------------------------------------------------------
# Eq. 2 — token scores from the observation window (summed over the GQA heads)
# --------------------------------------------------------------------------------------
def token_scores(q_obs_heads: np.ndarray, keys: np.ndarray, scale: float | None = None) -> np.ndarray:
    """Eq. 2 for one KV head.

    q_obs_heads: [G, alpha, d]  observation queries of the G query heads sharing the KV head
    keys:        [n, d]
    returns t: [n - alpha],  t_j = sum_g sum_{i in observation window} A^g_{ij}
    """
    q_obs_heads = np.asarray(q_obs_heads, dtype=np.float64)
    G, alpha, _ = q_obs_heads.shape
    n = keys.shape[0]
    t = np.zeros(n - alpha, dtype=np.float64)
    for g in range(G):
        A = attention_probs(q_obs_heads[g], keys, scale)
        t += A[:, : n - alpha].sum(axis=0)
    return t


# --------------------------------------------------------------------------------------
# Eq. 3-4 — review windows and their task-adaptive scores
# --------------------------------------------------------------------------------------
def window_scores(t: np.ndarray, omega: int, p: int) -> np.ndarray:
    """Eq. 3-4: s_k = sum(Top-p(W_k)) / min(p, omega) for the ceil(len(t)/omega) windows of
    omega consecutive token scores (the last one may be shorter)."""
    t = np.asarray(t, dtype=np.float64)
    n_win = -(-len(t) // omega)
    s = np.zeros(n_win, dtype=np.float64)
    for k in range(n_win):
        W = t[k * omega: (k + 1) * omega]
        top = np.sort(W)[::-1][: min(p, len(W))]            # the p highest scores in the window
        s[k] = top.sum() / min(p, omega)
    return s


# --------------------------------------------------------------------------------------
# window selection under the budget, and the retained indices
# --------------------------------------------------------------------------------------
def select_windows(s: np.ndarray, k: int) -> np.ndarray:
    """The k highest-scoring windows (equal scores: lower index first), ascending."""
    s = np.asarray(s, dtype=np.float64)
    order = np.argsort(-s, kind="stable")                   # stable: ties keep index order
    return np.sort(order[:k]).astype(np.int64)


def token_indices(selected: Sequence[int], omega: int, n: int, alpha: int) -> np.ndarray:
    """Retained positions: every token of each selected window, then the observation window."""
    idx: List[int] = []
    for w in selected:
        idx.extend(range(w * omega, min((w + 1) * omega, n - alpha)))
    idx.extend(range(n - alpha, n))
    return np.asarray(idx, dtype=np.int64)


def select_indices(q_obs_heads: np.ndarray, keys: np.ndarray, omega: int, p: int, k: int,
                   scale: float | None = None):
    """Section 2.2.1 end to end for one (sequence, KV head) of a group's first layer.
    Returns (t, s, selected windows, retained token indices)."""
    alpha = q_obs_heads.shape[1]
    n = keys.shape[0]
    t = token_scores(q_obs_heads, keys, scale)
    s = window_scores(t, omega, p)
    sel = select_windows(s, k)
    return t, s, sel, token_indices(sel, omega, n, alpha)


# --------------------------------------------------------------------------------------
# Section 2.2.2 — the group's layers share the first layer's indices
# --------------------------------------------------------------------------------------
def gather_rows(states: np.ndarray, tok_idx: np.ndarray) -> np.ndarray:
    """Retained K or V states of one layer, one KV head: rows of ``states [n, d]`` at the
    shared indices."""
    return np.asarray(states)[np.asarray(tok_idx, dtype=np.int64)]


def compress_group(q_obs_heads, keys_per_layer, values_per_layer, omega, p, k, scale=None):
    """One (sequence, KV head) of one layer group.

    Selection runs on the first layer only (``keys_per_layer[0]`` and its queries); every layer
    of the group, the first included, keeps the rows at those indices.
    Returns (t, s, selected windows, token indices, [K_out per layer], [V_out per layer]).
    """
    t, s, sel, idx = select_indices(q_obs_heads, keys_per_layer[0], omega, p, k, scale)
    k_out = [gather_rows(K, idx) for K in keys_per_layer]
    v_out = [gather_rows(V, idx) for V in values_per_layer]
    return t, s, sel, idx, k_out, v_out


# --------------------------------------------------------------------------------------
# Section 2.2.3, Eq. 5-7 — arithmetic-sequence budgets per group
# --------------------------------------------------------------------------------------
def group_budgets(b_total: float, n_groups: int, lam: float) -> np.ndarray:
    """Eq. 5-7: b^{H-1} = b_total/(lambda*H), b^0 = 2*b_total/H - b^{H-1}, linear in between
    (real-valued; rounding to whole windows is the caller's convention)."""
    H = n_groups
    b_top = b_total / (lam * H)
    b_bottom = 2.0 * b_total / H - b_top
    if H == 1:
        return np.asarray([b_total], dtype=np.float64)
    h = np.arange(H, dtype=np.float64)
    return b_bottom - (b_bottom - b_top) / (H - 1) * h


# --------------------------------------------------------------------------------------
# Generation over the compressed cache (Section 3.5 measures it end to end): one decode step
# --------------------------------------------------------------------------------------
def decode_step(q_new: np.ndarray, k_kept: np.ndarray, v_kept: np.ndarray, k_new: np.ndarray, v_new: np.ndarray,
                scale: float | None = None):
    """One generated token on one KV head of one layer: the new token's key and value are
    appended to the retained cache and its G query heads attend to all of it, new token
    included (Eq. 1 with a single query row; nothing is masked).

    q_new: [G, d]; k_kept, v_kept: [n, d] retained rows; k_new, v_new: [d].
    Returns (out [G, d], K' [n+1, d], V' [n+1, d]).
    """
    q_new = np.asarray(q_new, dtype=np.float64)
    K = np.concatenate([np.asarray(k_kept, dtype=np.float64), np.asarray(k_new, dtype=np.float64)[None, :]], axis=0)
    V = np.concatenate([np.asarray(v_kept, dtype=np.float64), np.asarray(v_new, dtype=np.float64)[None, :]], axis=0)
    d = q_new.shape[1]
    if scale is None:
        scale = 1.0 / math.sqrt(d)
    out = np.empty_like(q_new)
    for g in range(q_new.shape[0]):
        logits = (K @ q_new[g]) * scale
        e = np.exp(logits - logits.max())
        out[g] = (e / e.sum()) @ V
    return out, K, V


# --------------------------------------------------------------------------------------
# Section 3.2 — how alike the retained positions of two layers are
# --------------------------------------------------------------------------------------
def jaccard(idx_a: Sequence[int], idx_b: Sequence[int]) -> float:
    """Jaccard similarity |A n B| / |A u B| of two sets of retained token positions (1.0 when
    both are empty)."""
    a, b = set(int(x) for x in idx_a), set(int(x) for x in idx_b)
    union = len(a | b)
    return 1.0 if union == 0 else len(a & b) / union
