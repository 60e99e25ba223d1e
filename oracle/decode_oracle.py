"""Plain fp64 CPU oracle for one decoding step over a (compressed, ragged) multimodal KV cache.

TEST INFRASTRUCTURE ONLY.  Written from the paper (MEDA, arXiv 2502.17599, Section 3.1, "Decoding with
Multimodal KV Cache": the cache update K = [K, x_t W_K], V = [V, x_t W_V] and the output
x_out = Softmax(q_t K^T / sqrt(D)) V).  It shares no code with the HIP path and imports nothing from it;
only the tests, the smoke check and the benchmark's CPU-baseline leg may call it.  Never tuned for speed.

The result is the plain definition of single-query attention, written out: numpy float64, ``@`` for the
two contractions.

Readings where the paper is silent:
  * attention is per head and the scale is 1/sqrt(head_dim) (the paper writes sqrt(D) and drops head
    indices); a query head h reads kv head h // G (grouped-query attention);
  * the cache of layer l holds S_l rows per kv head (the compression pass gives every layer its own
    budget, Section 3.2), followed by the rows appended since (the update equation); a decoding query
    sees all of them (it is the newest position, so the causal mask removes nothing);
  * the order of the cached rows does not matter (a softmax-weighted sum is symmetric in its terms).

Pins (tests/test_oracle_decode.py): scipy softmax, closed forms (equal logits -> mean of V, one dominant
key -> its value, two-key logistic form), invariance under a permutation of the cached rows and under a
shift of all logits, the head mapping, append == concatenate, and "a cache compressed at budget 100 % is
the full cache" together with the compression oracle.
"""
from __future__ import annotations

import numpy as np

F64 = np.float64


def attend(q: np.ndarray, k: np.ndarray, v: np.ndarray, scale: float | None = None) -> np.ndarray:
    """One query against n cached (key, value) pairs: softmax(q K^T * scale) V.  q [d], k, v [n, d]."""
    q = np.asarray(q, dtype=F64)
    k = np.asarray(k, dtype=F64)
    v = np.asarray(v, dtype=F64)
    if scale is None or scale == 0.0:
        scale = 1.0 / np.sqrt(F64(q.shape[-1]))
    s = (k @ q) * scale
    p = np.exp(s - s.max())
    p /= p.sum()
    return p @ v


def append_rows(cache: np.ndarray, new: np.ndarray | None) -> np.ndarray:
    """K = [K, k_t]: the rows computed since the cache was built follow the cached rows (Section 3.1)."""
    if new is None or len(new) == 0:
        return np.asarray(cache, dtype=F64)
    return np.concatenate([np.asarray(cache, dtype=F64), np.asarray(new, dtype=F64)], axis=0)


def decode_layer(q_l: np.ndarray, k_l: np.ndarray, v_l: np.ndarray, k_new_l=None, v_new_l=None,
                 scale: float | None = None) -> np.ndarray:
    """All query heads of one layer.  q_l [Hq, d]; k_l, v_l [Hkv, S_l, d]; k_new_l, v_new_l [Hkv, n_new, d]
    or None -> out [Hq, d].  Query head h reads kv head h // G."""
    Hq, d = q_l.shape
    Hkv = k_l.shape[0]
    assert Hq % Hkv == 0
    G = Hq // Hkv
    out = np.empty((Hq, d), dtype=F64)
    for h in range(Hq):
        g = h // G
        kk = append_rows(k_l[g], None if k_new_l is None else k_new_l[g])
        vv = append_rows(v_l[g], None if v_new_l is None else v_new_l[g])
        out[h] = attend(q_l[h], kk, vv, scale)
    return out


def decode_step(q: np.ndarray, k_cache: np.ndarray, v_cache: np.ndarray, layer_len, layer_off, n_kv_heads: int,
                k_new=None, v_new=None, scale: float | None = None) -> np.ndarray:
    """One decoding step over a ragged cache in the layout the compression pass writes.

    q [L, Hq, d]; k_cache, v_cache [B * Hkv, d] where layer l occupies the rows
    [off[l] * Hkv, (off[l] + S_l) * Hkv) as [Hkv][S_l][d]; k_new, v_new [L, Hkv, n_new, d] or None.
    Returns out [L, Hq, d]."""
    L, Hq, d = q.shape
    out = np.empty((L, Hq, d), dtype=F64)
    for l in range(L):
        S = int(layer_len[l])
        a = int(layer_off[l]) * n_kv_heads
        k_l = np.asarray(k_cache[a:a + n_kv_heads * S], dtype=F64).reshape(n_kv_heads, S, d)
        v_l = np.asarray(v_cache[a:a + n_kv_heads * S], dtype=F64).reshape(n_kv_heads, S, d)
        out[l] = decode_layer(np.asarray(q[l], dtype=F64), k_l, v_l,
                              None if k_new is None else k_new[l], None if v_new is None else v_new[l], scale)
    return out
