"""Seeded generator for window queries, keys, values and the modality mask.

Recipe (every random draw comes from a Philox stream keyed by (seed, layer, tensor id),
so any single layer can be generated on its own and the result does not depend on
how many threads are used):

* values and text keys: iid N(0, 1);
* vision keys: for every (layer, kv-head, image/frame) ``n_centres`` centres c ~ N(0, I);
  every vision token picks one centre of its image uniformly and its key is
  c + cluster_sigma * N(0, I); with ``drift_sigma`` > 0 the centres of frame f are the
  centres of frame f-1 plus N(0, drift_sigma^2 I) (video);
* window queries: tau_l * N(0, I) with one temperature tau_l ~ U[tau_lo, tau_hi] per layer;
* heavy hitters: floor(heavy_frac * T) positions per layer (same for all heads) whose key
  is replaced by 3 * sqrt(d) * (mean window query of the kv-head's group, normalised);
  all heavy keys of a (layer, kv-head) are identical, which makes exact score ties and
  exact duplicate keys part of every workload;
* everything is rounded (nearest-even) to the workload's storage type before anyone
  sees it, so the oracle and the GPU path read the same bytes.
"""
from __future__ import annotations

from concurrent.futures import ThreadPoolExecutor
from typing import Dict, Iterable, Optional

import numpy as np
import torch

from .configs import Workload

_T_TAU, _T_Q, _T_K, _T_V, _T_CENTRE, _T_CHOICE, _T_HEAVY, _T_DRIFT = range(8)


def _rng(seed: int, layer: int, tensor_id: int) -> np.random.Generator:
    return np.random.Generator(np.random.Philox(key=[seed, ((layer + 1) << 8) | tensor_id]))


def modality_mask(wl: Workload) -> np.ndarray:
    """uint8[T]: 0 = text position, 1 = vision position."""
    parts = [np.full(n, 1 if kind == "v" else 0, dtype=np.uint8) for kind, n, _ in wl.layout]
    return np.concatenate(parts)


def _group_ids(wl: Workload) -> np.ndarray:
    parts = [np.full(n, grp, dtype=np.int64) for _, n, grp in wl.layout]
    return np.concatenate(parts)


def layer_taus(wl: Workload) -> np.ndarray:
    """Per-layer query temperature, from a stream that does not depend on the layer."""
    return _rng(wl.seed, -1, _T_TAU).uniform(wl.tau_lo, wl.tau_hi, size=wl.n_layers)


def generate_layer(wl: Workload, layer: int):
    """float32 arrays (q [Hq,R,d], k [Hkv,T,d], v [Hkv,T,d]) of one layer, before the storage cast; R query
    rows = the last R positions (the observation window, or all T positions)."""
    T, W, d, R = wl.seq_len, wl.window, wl.head_dim, wl.n_score_rows
    Hq, Hkv, G = wl.n_q_heads, wl.n_kv_heads, wl.group_size
    tau = np.float32(layer_taus(wl)[layer])

    q = _rng(wl.seed, layer, _T_Q).standard_normal((Hq, R, d), dtype=np.float32) * tau
    k = _rng(wl.seed, layer, _T_K).standard_normal((Hkv, T, d), dtype=np.float32)
    v = _rng(wl.seed, layer, _T_V).standard_normal((Hkv, T, d), dtype=np.float32)

    mask = modality_mask(wl)
    vis = np.flatnonzero(mask == 1)
    if vis.size:
        grp = _group_ids(wl)[vis]
        n_groups = wl.n_groups
        centres = _rng(wl.seed, layer, _T_CENTRE).standard_normal(
            (Hkv, n_groups, wl.n_centres, d), dtype=np.float32)
        if wl.drift_sigma > 0.0:
            steps = _rng(wl.seed, layer, _T_DRIFT).standard_normal(
                (Hkv, n_groups, wl.n_centres, d), dtype=np.float32) * np.float32(wl.drift_sigma)
            steps[:, 0] = centres[:, 0]
            centres = np.cumsum(steps, axis=1, dtype=np.float32)
        choice = _rng(wl.seed, layer, _T_CHOICE).integers(0, wl.n_centres, size=(Hkv, vis.size))
        sig = np.float32(wl.cluster_sigma)
        for g in range(Hkv):
            k[g, vis] = centres[g][grp, choice[g]] + sig * k[g, vis]

    n_heavy = int(wl.heavy_frac * T)
    if n_heavy > 0:
        heavy = np.sort(_rng(wl.seed, layer, _T_HEAVY).choice(T, size=n_heavy, replace=False))
        for g in range(Hkv):
            qbar = q[g * G:(g + 1) * G, R - W:].reshape(-1, d).mean(axis=0)   # mean query of the last W positions
            direction = qbar / max(float(np.linalg.norm(qbar)), 1e-20)
            k[g, heavy] = (3.0 * np.sqrt(np.float32(d))) * direction.astype(np.float32)
    return q, k, v


def storage_dtype(wl: Workload) -> torch.dtype:
    return {"f32": torch.float32, "bf16": torch.bfloat16}[wl.dtype]


def generate(wl: Workload, layers: Optional[Iterable[int]] = None, threads: int = 8
             ) -> Dict[str, object]:
    """Inputs of ``wl`` as CPU torch tensors in the workload's storage type.

    Returns ``{"q": [L,Hq,R,d] (R = W, or T when the workload scores with every prompt row), "k": [L,Hkv,T,d], "v": [L,Hkv,T,d], "mask": uint8 [T]}``.
    ``layers`` restricts generation to a subset (the tensors then hold only those layers,
    in the given order).
    """
    layer_list = list(range(wl.n_layers)) if layers is None else list(layers)
    n = len(layer_list)
    dt = storage_dtype(wl)
    T, d = wl.seq_len, wl.head_dim
    q = torch.empty((n, wl.n_q_heads, wl.n_score_rows, d), dtype=dt)
    k = torch.empty((n, wl.n_kv_heads, T, d), dtype=dt)
    v = torch.empty((n, wl.n_kv_heads, T, d), dtype=dt)

    def work(i: int) -> None:
        ql, kl, vl = generate_layer(wl, layer_list[i])
        q[i].copy_(torch.from_numpy(ql))   # copy_ rounds to nearest-even when narrowing to bf16
        k[i].copy_(torch.from_numpy(kl))
        v[i].copy_(torch.from_numpy(vl))

    if threads > 1 and n > 1:
        with ThreadPoolExecutor(max_workers=min(threads, n)) as pool:
            list(pool.map(work, range(n)))
    else:
        for i in range(n):
            work(i)
    return {"q": q, "k": k, "v": v, "mask": torch.from_numpy(modality_mask(wl))}


def generate_batch(wls, threads: int = 8) -> Dict[str, object]:
    """Inputs of several workloads of one shape (they may differ in seed and in layout, not in any size),
    stacked along a new leading dimension: ``q`` [N,L,Hq,R,d], ``k``, ``v`` [N,L,Hkv,T,d], ``mask`` [N,T]."""
    parts = [generate(w, threads=threads) for w in wls]
    return {key: torch.stack([p[key] for p in parts]).contiguous() for key in ("q", "k", "v", "mask")}


def to_float64(t: torch.Tensor) -> np.ndarray:
    """Exact widening of a stored tensor (f32 or bf16) to a float64 numpy array."""
    return t.to(torch.float64).numpy()
