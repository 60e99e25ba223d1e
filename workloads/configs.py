"""The named synthetic workloads (shapes, layouts, budgets) and small variants of them.

A layout is a tuple of segments ``(kind, length, group)``: kind 't' is text, 'v' is
vision; ``group`` numbers the image / video frame a vision segment belongs to
(-1 for text).  Vision keys of one group share a set of cluster centres.
"""
from __future__ import annotations

from dataclasses import dataclass, replace
from typing import Tuple

Segment = Tuple[str, int, int]


@dataclass(frozen=True)
class Workload:
    name: str
    n_layers: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    dtype: str                     # "f32" or "bf16": storage type of q/k/v and of the outputs
    layout: Tuple[Segment, ...]
    window: int                    # W: observation window = last W positions
    total_budget: int              # B: token slots per kv-head summed over layers
    seed: int = 0
    tau_lo: float = 0.5            # per-layer query temperature ~ U[tau_lo, tau_hi]
    tau_hi: float = 3.0
    heavy_frac: float = 0.02       # fraction of positions made heavy hitters
    n_centres: int = 16            # cluster centres per image / frame
    cluster_sigma: float = 0.3
    drift_sigma: float = 0.0       # >0: group g's centres = group g-1's + N(0, drift_sigma^2)
    recent_num: int = 3            # recent : important = 3 : 1 (Section 4.3)
    recent_den: int = 4
    score_rows: int = 0            # query rows that score the keys: 0 = the observation window (last W
                                   # positions); seq_len = every prompt position, as the paper writes it

    @property
    def seq_len(self) -> int:
        return sum(s[1] for s in self.layout)

    @property
    def n_score_rows(self) -> int:
        return self.score_rows if self.score_rows > 0 else self.window

    @property
    def n_text(self) -> int:
        return sum(s[1] for s in self.layout if s[0] == "t")

    @property
    def n_vision(self) -> int:
        return sum(s[1] for s in self.layout if s[0] == "v")

    @property
    def n_groups(self) -> int:
        return 1 + max([s[2] for s in self.layout if s[0] == "v"], default=-1)

    @property
    def group_size(self) -> int:
        return self.n_q_heads // self.n_kv_heads


def _interleaved(n_img: int, img_len: int, n_text: int) -> Tuple[Segment, ...]:
    """Before each image a short text segment, then the image; the rest of the text trails."""
    gap = n_text // (2 * n_img)
    segs = []
    for i in range(n_img):
        segs.append(("t", gap, -1))
        segs.append(("v", img_len, i))
    segs.append(("t", n_text - gap * n_img, -1))
    return tuple(segs)


def _video(n_frames: int, frame_len: int, head_text: int, tail_text: int) -> Tuple[Segment, ...]:
    segs = [("t", head_text, -1)]
    segs += [("v", frame_len, f) for f in range(n_frames)]
    segs.append(("t", tail_text, -1))
    return tuple(segs)


def _pct(pct: int, n_layers: int, seq_len: int) -> int:
    return (pct * n_layers * seq_len) // 100


_tiny_layout = (("t", 64, -1), ("v", 256, 0), ("v", 256, 1), ("v", 256, 2), ("t", 192, -1))
_c2_layout = _interleaved(6, 576, 640)
_c3_layout = _interleaved(24, 576, 2560)
_c4_layout = _video(256, 144, 64, 448)
_c5_layout = _interleaved(220, 576, 4352)

WORKLOADS = {
    "tiny": Workload("tiny", 2, 4, 4, 64, "f32", _tiny_layout, 32, _pct(25, 2, 1024)),
    "llava7b_multi_image": Workload("llava7b_multi_image", 32, 32, 32, 128, "bf16", _c2_layout, 32,
                                    512 * 32),
    "long_multi_image": Workload("long_multi_image", 32, 32, 8, 128, "bf16", _c3_layout, 64,
                                 _pct(20, 32, 16384)),
    "long_video": Workload("long_video", 28, 28, 4, 128, "bf16", _c4_layout, 64,
                           _pct(15, 28, 37376), drift_sigma=0.05),
    "extreme": Workload("extreme", 32, 32, 8, 128, "bf16", _c5_layout, 64,
                        _pct(10, 32, 131072), tau_lo=0.3, tau_hi=4.0),
}

# order in which the configurations are usually listed
ORDER = ("tiny", "llava7b_multi_image", "long_multi_image", "long_video", "extreme")


def get_workload(name: str) -> Workload:
    return WORKLOADS[name]


def variant(base: Workload, **changes) -> Workload:
    """A copy of ``base`` with fields replaced (layout, budget, seed, ...)."""
    return replace(base, **changes)
