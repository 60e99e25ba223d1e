"""Seeded synthetic multimodal KV-cache workloads.

This module only produces inputs: token layouts (which positions are text and
which are vision), window queries, keys and values.  It holds none of the
compression method's arithmetic and is the one module that both the CPU oracle's
tests and the GPU path's tests/bench import.

The layouts stand in for the paper's interleaved text/multi-image prompts and its
long-video prompts (Section 3.1: an interleaved sequence of text and image
embeddings, or text followed by many video-frame embeddings).  Only shapes and
structure are taken; no benchmark data is reproduced.
"""
from .configs import Workload, WORKLOADS, get_workload, variant
from .gen import generate, generate_batch, generate_layer, modality_mask

__all__ = ["Workload", "WORKLOADS", "get_workload", "variant",
           "generate", "generate_batch", "generate_layer", "modality_mask"]
