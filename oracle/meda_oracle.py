"""Plain fp64 CPU oracle for MEDA's prefill-time KV-cache compression pass.

TEST INFRASTRUCTURE ONLY.  This file is the slow, obviously-correct statement of what the
compression pass computes, written from the paper (MEDA, arXiv 2502.17599, Sections 3.2 and
3.3, Section 4.3, Appendix A.3).  It shares no code with the HIP path and imports nothing
from it; only the tests, the smoke check and the benchmark's CPU-baseline leg may call it.
It is never tuned for speed.

All arithmetic is numpy float64.  Library primitives used as steps: ``@`` (matrix product)
for the two contractions, ``np.exp`` / ``np.log``, ``np.lexsort`` / ``np.argmax``.

Steps, in the paper's order (one layer unless stated):

  window_logits        s = Q K^T / sqrt(d)                        Sec. 3.2 eq. for A_TV/A_VT, Sec. 3.3 A_p
  window_softmax       causal softmax over all visible keys       Sec. 3.3, A_p
  column_scores        A_s = sum of attention rows                Sec. 3.3, cumulative attention score
  cross_modal_entropy  E_CM = -(E_TV + E_VT)                      Sec. 3.2, cross-modal attention entropy
  allocate_budgets     S_l from softmax over layers of E_CM       Sec. 3.2 allocation eq., App. A.3, Sec. 4.3
  select_tokens        text boost, recent window, Top-N           Sec. 3.3, selection eqs.
  nn_assign            cosine similarity, row argmax              Sec. 3.3, similarity matrix U
  average_merge        k_j <- (k_j + sum k_i)/(|N_j|+1), same V   Sec. 3.3, average merging
  meda_compress        all layers, ragged output                  the whole pass

Readings taken where the paper is silent or ambiguous are stated at each function.
Pins (tests/test_oracle_*.py): closed forms (uniform rows, one-hot rows), library routines
(scipy softmax / entropy), brute-force loops on tiny inputs, invariants (mass conservation,
budgets summing to the total), special cases (budget = 100 % is the identity).  Not pinned by
anything the paper prints (it prints no intermediate value): the causal mask, the GQA head
mapping, the re-normalisation of the cross-modal sub-block, the clamp / rounding rule of the
allocation and the M:N = 3:1 split -- these are "parity unpinned" with respect to the paper
and pinned only to the readings written here.
"""
from __future__ import annotations

import numpy as np

F64 = np.float64


# --------------------------------------------------------------------------------------
# Step 1: attention of the observation window
# --------------------------------------------------------------------------------------

def window_logits(q_win: np.ndarray, k: np.ndarray, scale: float | None = None) -> np.ndarray:
    """Logits of the window queries against every cached key of one layer.

    q_win [Hq, W, d], k [Hkv, T, d] -> s [Hq, W, T] with s[h] = q_win[h] @ k[h // G].T * scale.
    Section 3.2 / 3.3 write Q K^T / sqrt(D); attention is per head, so the scale is
    1/sqrt(head_dim).  The paper drops head indices; a query head h reads the kv head
    h // G (grouped-query attention, G = Hq / Hkv).
    """
    q_win = np.asarray(q_win, dtype=F64)
    k = np.asarray(k, dtype=F64)
    Hq, W, d = q_win.shape
    Hkv = k.shape[0]
    assert Hq % Hkv == 0
    G = Hq // Hkv
    if scale is None or scale == 0.0:
        scale = 1.0 / np.sqrt(F64(d))
    s = np.empty((Hq, W, k.shape[1]), dtype=F64)
    for h in range(Hq):
        s[h] = (q_win[h] @ k[h // G].T) * F64(scale)
    return s


def causal_allowed(T: int, W: int) -> np.ndarray:
    """allowed[i, j]: window row i sits at position T-W+i and sees keys j <= T-W+i.

    The attention weights of prompt encoding (Section 3.3, A_p) are those of a causal
    decoder, so the mask is causal; it only bites inside the last W columns.
    """
    pos = T - W + np.arange(W)
    return np.arange(T)[None, :] <= pos[:, None]


def masked_softmax(s: np.ndarray, allowed: np.ndarray) -> np.ndarray:
    """Row softmax of s over the columns where ``allowed`` is true; 0 elsewhere.

    s [..., W, T], allowed [W, T] (broadcast over leading axes).  A row with no allowed
    column is all zero.
    """
    s = np.asarray(s, dtype=F64)
    neg = np.where(allowed, s, -np.inf)
    m = np.max(neg, axis=-1, keepdims=True)
    m = np.where(np.isfinite(m), m, 0.0)
    e = np.where(allowed, np.exp(np.where(allowed, s, 0.0) - m), 0.0)
    z = np.sum(e, axis=-1, keepdims=True)
    return np.divide(e, z, out=np.zeros_like(e), where=z > 0)


def column_scores(p_all: np.ndarray, n_kv_heads: int) -> np.ndarray:
    """Cumulative attention score per key (Section 3.3, A_s = sum_i A_p[i, :]).

    p_all [Hq, W, T] -> A_s [Hkv, T].  Rows are the window rows; the scores of the G query
    heads that share a kv head are added (a sum, not a mean: the ranking is the same).
    """
    Hq, W, T = p_all.shape
    G = Hq // n_kv_heads
    return p_all.reshape(n_kv_heads, G * W, T).sum(axis=1)


# --------------------------------------------------------------------------------------
# Step 2: cross-modal attention entropy
# --------------------------------------------------------------------------------------

def cross_modal_probs(s: np.ndarray, mask: np.ndarray) -> np.ndarray:
    """Head-averaged cross-modal attention of the window rows.

    s [Hq, W, T] logits, mask [T] (0 text, 1 vision).  Row i (position T-W+i, modality
    mask[T-W+i]) attends, in the cross-modal matrix, only to the visible keys of the *other*
    modality, and the softmax is taken over that sub-block (Section 3.2: A_TV is the softmax
    of Q_T K_V^T, A_VT the softmax of Q_V K_T^T).  The per-head matrices are averaged over
    the heads before the entropy (Section 3.2, definition of E(A): the matrix whose entropy is
    taken is the head average).
    Returns pbar [W, T]; entries outside a row's cross-modal set are 0.
    """
    Hq, W, T = s.shape
    mask = np.asarray(mask)
    allowed = causal_allowed(T, W)
    row_mod = mask[T - W:]
    cross = allowed & (mask[None, :] != row_mod[:, None])
    return masked_softmax(s, cross).mean(axis=0)


def row_entropy(p: np.ndarray) -> np.ndarray:
    """Shannon entropy in nats of each row, -sum p log p with 0 log 0 = 0 (Section 3.2, E(A_i))."""
    p = np.asarray(p, dtype=F64)
    plogp = np.zeros_like(p)
    np.multiply(p, np.log(p, out=np.zeros_like(p), where=p > 0), out=plogp, where=p > 0)
    return -plogp.sum(axis=-1)


def cross_modal_entropy(s: np.ndarray, mask: np.ndarray):
    """(H_TV, H_VT, E_CM) of one layer (Section 3.2).

    E_TV = (1/|T|) sum_i sum_j A_TV log A_TV over text rows, E_VT likewise over vision rows
    (the printed limits of E_VT repeat E_TV's; rows are vision queries and columns text keys),
    E_CM = -(E_TV + E_VT) = H_TV + H_VT.  |T| and |V| count the window rows of each modality;
    a direction without rows contributes 0, and a row whose cross-modal set is empty has
    entropy 0 but still counts in its denominator.
    """
    Hq, W, T = s.shape
    mask = np.asarray(mask)
    ent = row_entropy(cross_modal_probs(s, mask))
    row_mod = mask[T - W:]
    text_rows = row_mod == 0
    vis_rows = ~text_rows
    h_tv = ent[text_rows].sum() / text_rows.sum() if text_rows.any() else F64(0.0)
    h_vt = ent[vis_rows].sum() / vis_rows.sum() if vis_rows.any() else F64(0.0)
    return F64(h_tv), F64(h_vt), F64(h_tv + h_vt)


# --------------------------------------------------------------------------------------
# Step 3: layer budgets
# --------------------------------------------------------------------------------------

def allocation_reals(entropy: np.ndarray, total_budget: int, lo: int, hi: int) -> np.ndarray:
    """Real-valued layer budgets x_l = clamp(lambda * exp(E_l), lo, hi) with sum x_l = B.

    Section 3.2 / Appendix A.3: S_l = softmax_l(E_CM) * L * rho * S with S the context length,
    so sum_l S_l = L*rho*T =: B and S_l is proportional to exp(E_l) (higher entropy, larger
    share).  The paper does not say what happens when a share exceeds the context length or
    falls below the recent window; here shares are clamped to [lo, hi] and the remainder is
    redistributed proportionally (water-filling): lambda is the solution of
    sum_l clamp(lambda w_l, lo, hi) = B, w_l = exp(E_l - max E).  Without active clamps this
    is exactly the paper's formula.
    """
    e = np.asarray(entropy, dtype=F64)
    L = e.size
    B = F64(total_budget)
    assert L * lo <= total_budget <= L * hi, "budget outside [L*lo, L*hi]"
    w = np.exp(e - e.max())

    def filled(lam: float) -> float:
        return float(np.clip(lam * w, lo, hi).sum())

    if total_budget == L * hi:
        return np.full(L, F64(hi))
    if total_budget == L * lo:
        return np.full(L, F64(lo))
    # sum_l clamp(lam*w_l) is piecewise linear and non-decreasing in lam; its kinks are
    # lo/w_l and hi/w_l.  Find the first kink at which the sum reaches B, then solve the
    # linear piece that ends there.
    kinks = np.sort(np.concatenate([lo / w, hi / w]))
    upper = None
    lower = 0.0
    for b in kinks:
        if filled(b) >= B:
            upper = b
            break
        lower = b
    assert upper is not None
    mid = 0.5 * (lower + upper)
    at_lo = mid * w <= lo
    at_hi = mid * w >= hi
    free = ~(at_lo | at_hi)
    wsum = w[free].sum()
    if wsum > 0:
        lam = (B - lo * at_lo.sum() - hi * at_hi.sum()) / wsum
    else:
        lam = upper
    return np.clip(lam * w, lo, hi)


def allocate_budgets(entropy: np.ndarray, total_budget: int, seq_len: int, window: int,
                     recent_num: int = 3, recent_den: int = 4):
    """Integer layer budgets S_l, recent counts M_l, Top-N counts N_l and offsets.

    Rounding (paper silent): largest remainder -- S_l = floor(x_l), then +1 to the
    B - sum floor(x_l) layers with the largest fractional parts, ties to the lower layer
    index; a layer already at the cap is skipped.  So sum_l S_l = B exactly.
    Split (Section 4.3: recent M : important N = 3 : 1): M_l = max(min(W, S_l),
    floor(S_l * num/den)), N_l = S_l - M_l; the observation window is always inside the
    recent part.
    Returns (S, M, N, off) as int64 arrays, off of length L+1 with off[L] = B.
    """
    L = len(entropy)
    lo = min(window, seq_len)
    hi = seq_len
    x = allocation_reals(entropy, total_budget, lo, hi)
    S = np.floor(x).astype(np.int64)
    S = np.clip(S, lo, hi)
    frac = x - np.floor(x)
    rest = int(total_budget - S.sum())
    # decreasing fractional part, ties -> lower index (lexsort: last key is primary)
    order = np.lexsort((np.arange(L), -frac))
    guard = 0
    while rest > 0:
        for l in order:
            if rest == 0:
                break
            if S[l] < hi:
                S[l] += 1
                rest -= 1
        guard += 1
        assert guard <= 2, "allocation rounding did not converge"
    while rest < 0:          # only reachable through floating-point fuzz
        for l in order[::-1]:
            if rest == 0:
                break
            if S[l] > lo:
                S[l] -= 1
                rest += 1
    M = np.maximum(np.minimum(window, S), (S * recent_num) // recent_den)
    N = S - M
    off = np.concatenate([[0], np.cumsum(S)]).astype(np.int64)
    return S, M.astype(np.int64), N.astype(np.int64), off


# --------------------------------------------------------------------------------------
# Step 4: token selection
# --------------------------------------------------------------------------------------

def select_tokens(a_s: np.ndarray, mask: np.ndarray, n_top: int, n_recent: int):
    """Conserved and less-important positions of one (layer, kv head) (Section 3.3).

    a_s [T] cumulative scores, mask [T].  Text positions get max(A_s) added (the max is over
    all T positions, before the boost).  The last ``n_recent`` positions are always kept;
    I = the ``n_top`` highest boosted scores among positions [0, T - n_recent), equal scores
    resolved towards the smaller position.  The conserved set is returned in ascending
    position (attention over a KV set does not depend on its order), as is the rest.
    Returns (idx_c int64 [n_top + n_recent], idx_less int64 [T - n_top - n_recent]).
    """
    a = np.asarray(a_s, dtype=F64)
    T = a.size
    boosted = a + np.where(np.asarray(mask) == 0, a.max(), 0.0)
    n_cand = T - n_recent
    assert 0 <= n_top <= n_cand
    cand = np.arange(n_cand)
    order = np.lexsort((cand, -boosted[:n_cand]))      # score descending, then position ascending
    top = np.sort(order[:n_top])
    idx_c = np.concatenate([top, np.arange(n_cand, T)]).astype(np.int64)
    keep = np.zeros(T, dtype=bool)
    keep[idx_c] = True
    idx_less = np.flatnonzero(~keep).astype(np.int64)
    return idx_c, idx_less


def boosted_scores(a_s: np.ndarray, mask: np.ndarray) -> np.ndarray:
    """A_s with max(A_s) added on the text positions (Section 3.3, text prior)."""
    a = np.asarray(a_s, dtype=F64)
    return a + np.where(np.asarray(mask) == 0, a.max(), 0.0)


# --------------------------------------------------------------------------------------
# Step 5: nearest conserved key
# --------------------------------------------------------------------------------------

TIE_EPS = 1e-12   # float64 rounding noise of a 128-term cosine is ~1e-16; real gaps are >> 1e-12


def cosine_matrix(k_less: np.ndarray, k_c: np.ndarray) -> np.ndarray:
    """u[i, j] = k_i . k_j / (|k_i| |k_j|) (Section 3.3); a zero key has its norm guarded."""
    a = np.asarray(k_less, dtype=F64)
    b = np.asarray(k_c, dtype=F64)
    an = a / np.maximum(np.linalg.norm(a, axis=1, keepdims=True), 1e-30)
    bn = b / np.maximum(np.linalg.norm(b, axis=1, keepdims=True), 1e-30)
    return an @ bn.T


def nn_assign(k: np.ndarray, idx_c: np.ndarray, idx_less: np.ndarray, chunk: int = 4096,
              return_margin: bool = False):
    """For every less-important key the conserved slot with the highest cosine similarity.

    k [T, d] keys of one (layer, kv head) -- the original, un-merged keys: one similarity
    matrix is formed and all merges happen at once.  Targets are all conserved slots (Top-N
    and recent).  Equal similarities resolve to the lower slot; "equal" means equal as real
    numbers, so similarities within ``TIE_EPS`` of the row maximum (the rounding noise of a
    float64 matrix product, which can differ between two identical conserved keys) count as
    equal.  Returns assign int64
    [len(idx_less)] of slot numbers in [0, len(idx_c)); with ``return_margin`` also the best
    similarity and the gap to the runner-up slot (inf when there is one slot).
    """
    k = np.asarray(k, dtype=F64)
    k_c = k[idx_c]
    n = len(idx_less)
    assign = np.empty(n, dtype=np.int64)
    best = np.empty(n, dtype=F64)
    gap = np.full(n, np.inf, dtype=F64)
    for a in range(0, n, chunk):
        u = cosine_matrix(k[idx_less[a:a + chunk]], k_c)
        j = np.argmax(u >= u.max(axis=1, keepdims=True) - TIE_EPS, axis=1)   # first maximum = lowest slot
        assign[a:a + chunk] = j
        if return_margin:
            rows = np.arange(u.shape[0])
            top = u[rows, j]
            best[a:a + chunk] = top
            if u.shape[1] > 1:
                u[rows, j] = -np.inf
                gap[a:a + chunk] = np.maximum(top - u.max(axis=1), 0.0)
    if return_margin:
        return assign, best, gap
    return assign


# --------------------------------------------------------------------------------------
# Step 6: average merging and the ragged output
# --------------------------------------------------------------------------------------

def average_merge(k: np.ndarray, v: np.ndarray, idx_c: np.ndarray, idx_less: np.ndarray,
                  assign: np.ndarray):
    """Merged conserved keys and values (Section 3.3, average merging).

    k_j <- (k_j + sum_{i in N_j} k_i) / (|N_j| + 1), and the same assignment and average for
    the values.  Returns (k_m [S, d], v_m [S, d], members [S]) in float64, before rounding to
    the storage type.
    """
    k = np.asarray(k, dtype=F64)
    v = np.asarray(v, dtype=F64)
    S = len(idx_c)
    k_sum = k[idx_c].copy()
    v_sum = v[idx_c].copy()
    members = np.zeros(S, dtype=np.int64)
    if len(idx_less):
        np.add.at(k_sum, assign, k[idx_less])
        np.add.at(v_sum, assign, v[idx_less])
        np.add.at(members, assign, 1)
    denom = (members + 1).astype(F64)[:, None]
    return k_sum / denom, v_sum / denom, members


def round_to_storage(x: np.ndarray, dtype: str) -> np.ndarray:
    """Round float64 values once, to nearest-even, to the storage type; result widened to float64.

    "f32": IEEE binary32.  "bf16": the 16-bit format made of binary32's upper half (8-bit
    exponent, 8 significant bits); rounded directly from float64 (no intermediate binary32
    rounding) by scaling to an integer significand.
    """
    x = np.asarray(x, dtype=F64)
    if dtype == "f32":
        return x.astype(np.float32).astype(F64)
    assert dtype == "bf16"
    out = np.zeros_like(x)
    nz = (x != 0) & np.isfinite(x)
    m, e = np.frexp(x[nz])                 # x = m * 2^e, 0.5 <= |m| < 1
    # 8 significant bits: significand integer = round_half_even(m * 2^8); the values of the
    # workloads are far from bf16's subnormal range, which is not handled here
    sig = np.rint(m * 256.0)               # np.rint rounds half to even
    out[nz] = np.ldexp(sig, e - 8)
    out[~np.isfinite(x)] = x[~np.isfinite(x)]
    return out


# --------------------------------------------------------------------------------------
# The whole pass
# --------------------------------------------------------------------------------------

def layer_scores_and_entropy(q_win_l, k_l, mask, scale=None):
    """Column scores A_s [Hkv, T] and (H_TV, H_VT, E_CM) of one layer."""
    Hkv, T, _ = k_l.shape
    W = q_win_l.shape[1]
    s = window_logits(q_win_l, k_l, scale)
    p_all = masked_softmax(s, causal_allowed(T, W))
    a_s = column_scores(p_all, Hkv)
    return a_s, cross_modal_entropy(s, mask)


def compress_layer_head(k_g, v_g, a_s_g, mask, n_top, n_recent, dtype):
    """Selection, matching, merging of one (layer, kv head); outputs rounded to ``dtype``."""
    idx_c, idx_less = select_tokens(a_s_g, mask, n_top, n_recent)
    assign = nn_assign(k_g, idx_c, idx_less) if len(idx_less) else np.empty(0, dtype=np.int64)
    k_m, v_m, members = average_merge(k_g, v_g, idx_c, idx_less, assign)
    return {
        "idx_c": idx_c, "idx_less": idx_less, "assign": assign, "members": members,
        "k_exact": k_m, "v_exact": v_m,
        "k_out": round_to_storage(k_m, dtype), "v_out": round_to_storage(v_m, dtype),
    }


def meda_compress(q_win, k, v, mask, total_budget, window, dtype="f32", scale=None,
                  recent_num=3, recent_den=4):
    """The whole compression pass on float64 copies of the stored inputs.

    q_win [L, Hq, R, d], k, v [L, Hkv, T, d], mask [T].  The R query rows are the last R positions:
    R = window is the observation-window variant (only the last W positions score the keys), R = T is
    the scoring as the paper writes it (Section 3.3 sums A_p over all prompt rows, Section 3.2 builds
    A_TV / A_VT from all text / vision queries); ``window`` stays the lower bound of the recent part and
    of every layer budget either way.  Returns a dict with, per layer,
    entropies (h_tv, h_vt, e_cm), budgets (S, M, N, off), the column scores and, per
    (layer, kv head), index sets, assignments and merged rows; plus the ragged outputs
    ``k_out`` / ``v_out`` as lists over layers of [Hkv, S_l, d] arrays.
    """
    q_win = np.asarray(q_win, dtype=F64)
    k = np.asarray(k, dtype=F64)
    v = np.asarray(v, dtype=F64)
    mask = np.asarray(mask)
    L, Hkv, T, d = k.shape
    assert q_win.shape[2] in (window, T), "query rows: the observation window or every prompt position"
    a_s = []
    ent = np.zeros((L, 3), dtype=F64)
    for l in range(L):
        a_l, e_l = layer_scores_and_entropy(q_win[l], k[l], mask, scale)
        a_s.append(a_l)
        ent[l] = e_l
    S, M, N, off = allocate_budgets(ent[:, 2], total_budget, T, window, recent_num, recent_den)
    heads = []
    k_out, v_out = [], []
    for l in range(L):
        per_head = [compress_layer_head(k[l, g], v[l, g], a_s[l][g], mask, int(N[l]), int(M[l]), dtype)
                    for g in range(Hkv)]
        heads.append(per_head)
        k_out.append(np.stack([h["k_out"] for h in per_head]))
        v_out.append(np.stack([h["v_out"] for h in per_head]))
    return {"entropy": ent[:, 2].copy(), "h_tv": ent[:, 0].copy(), "h_vt": ent[:, 1].copy(),
            "S": S, "M": M, "N": N, "off": off, "a_s": a_s, "heads": heads,
            "k_out": k_out, "v_out": v_out}


def meda_compress_batch(q_win, k, v, masks, total_budget, window, dtype="f32", scale=None,
                        recent_num=3, recent_den=4):
    """A batch of sequences (the paper's throughput figures are taken on batches, Table 6): the sequences are
    independent, each is compressed on its own with the budget ``total_budget``.  Arrays carry a leading
    dimension N (masks [N, T]); returns the list of the N results of ``meda_compress``."""
    return [meda_compress(q_win[n], k[n], v[n], masks[n], total_budget, window, dtype, scale, recent_num, recent_den)
            for n in range(len(masks))]


def kv_cache_bytes(tokens: int, n_layers: int, n_heads: int, head_dim: int, elt_bytes: int) -> int:
    """Bytes of a K+V cache holding ``tokens`` positions per layer (Appendix A.2 memory formula)."""
    return tokens * 2 * n_layers * n_heads * head_dim * elt_bytes
