"""ctypes binding of libmeda.so: argument marshalling only, every step runs in the HIP kernels."""
from __future__ import annotations

import ctypes
import os
from dataclasses import dataclass
from typing import Optional

import torch

_PKG_DIR = os.path.dirname(os.path.abspath(__file__))
_LIB_NAME = "libmeda.so"

EXPORTED_SYMBOLS = ("meda_workspace_bytes", "meda_compress", "meda_workspace_region",
                    "meda_profile_enable", "meda_profile_read", "meda_phase_name", "meda_status_string",
                    "meda_decode_workspace_bytes", "meda_decode_attention",
                    "meda_quantize_fp8", "meda_dequantize_fp8", "meda_decode_attention_fp8",
                    "meda_decode_attention_noalloc", "meda_peak_stream_read", "meda_peak_mfma_bf16", "meda_peak_mfma_valu")
DECODE_NOALLOC_MAX_BYTES = 40 << 20
REGIONS = {"col_scores": 0, "inv_norm": 1, "row_stats": 2, "alloc": 3, "less_idx": 4, "less_slot": 5}
N_PHASES = 8
FLAG_UNIFORM_BUDGET = 1
FLAG_NO_MERGE = 2
FLAG_FULL_PROMPT = 4
_DTYPES = {torch.float32: 0, torch.bfloat16: 1}


class MedaError(RuntimeError):
    def __init__(self, status: int, message: str):
        super().__init__(f"libmeda: {message} (status {status})")
        self.status = status


class MedaParams(ctypes.Structure):
    _fields_ = [("n_layers", ctypes.c_int32), ("n_q_heads", ctypes.c_int32), ("n_kv_heads", ctypes.c_int32),
                ("head_dim", ctypes.c_int32), ("seq_len", ctypes.c_int32), ("window", ctypes.c_int32),
                ("total_budget", ctypes.c_int64), ("recent_num", ctypes.c_int32), ("recent_den", ctypes.c_int32),
                ("dtype", ctypes.c_int32), ("softmax_scale", ctypes.c_float), ("flags", ctypes.c_int32),
                ("n_seqs", ctypes.c_int32)]


class MedaDecodeParams(ctypes.Structure):
    _fields_ = [("n_layers", ctypes.c_int32), ("n_q_heads", ctypes.c_int32), ("n_kv_heads", ctypes.c_int32),
                ("head_dim", ctypes.c_int32), ("n_new", ctypes.c_int32), ("dtype", ctypes.c_int32),
                ("total_budget", ctypes.c_int64), ("softmax_scale", ctypes.c_float)]


def library_path() -> str:
    """The built library next to this file, or the file named by the MEDA_LIBRARY environment variable."""
    return os.environ.get("MEDA_LIBRARY") or os.path.join(_PKG_DIR, _LIB_NAME)


_lib = None


def load_library() -> ctypes.CDLL:
    """Load libmeda.so from the package directory; raises if it has not been built."""
    global _lib
    if _lib is not None:
        return _lib
    path = library_path()
    if not os.path.exists(path):
        raise MedaError(-1, f"{path} is missing: build it with `python -m paper_2502_17599_amd.build` "
                            "(there is no fallback path)")
    lib = ctypes.CDLL(path)
    vp, pp = ctypes.c_void_p, ctypes.POINTER(MedaParams)
    lib.meda_workspace_bytes.restype = ctypes.c_size_t
    lib.meda_workspace_bytes.argtypes = [pp]
    lib.meda_compress.restype = ctypes.c_int
    lib.meda_compress.argtypes = [pp, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, ctypes.c_size_t, vp]
    lib.meda_workspace_region.restype = ctypes.c_int
    lib.meda_workspace_region.argtypes = [pp, ctypes.c_int, ctypes.POINTER(ctypes.c_size_t),
                                          ctypes.POINTER(ctypes.c_size_t)]
    lib.meda_profile_enable.restype = ctypes.c_int
    lib.meda_profile_enable.argtypes = [ctypes.c_int]
    lib.meda_profile_read.restype = ctypes.c_int
    lib.meda_profile_read.argtypes = [ctypes.POINTER(ctypes.c_double), ctypes.POINTER(ctypes.c_int32), ctypes.c_int]
    lib.meda_phase_name.restype = ctypes.c_char_p
    lib.meda_phase_name.argtypes = [ctypes.c_int]
    lib.meda_status_string.restype = ctypes.c_char_p
    lib.meda_status_string.argtypes = [ctypes.c_int]
    dp = ctypes.POINTER(MedaDecodeParams)
    lib.meda_decode_workspace_bytes.restype = ctypes.c_size_t
    lib.meda_decode_workspace_bytes.argtypes = [dp]
    lib.meda_decode_attention.restype = ctypes.c_int
    lib.meda_decode_attention.argtypes = [dp, vp, vp, vp, vp, vp, vp, vp, vp, vp, ctypes.c_size_t, vp]
    lib.meda_decode_attention_noalloc.restype = ctypes.c_int
    lib.meda_decode_attention_noalloc.argtypes = [dp, vp, vp, vp, vp, vp, vp, vp, vp, vp]
    lib.meda_peak_stream_read.restype = ctypes.c_int
    lib.meda_peak_stream_read.argtypes = [vp, ctypes.c_size_t, vp, vp]
    lib.meda_peak_mfma_bf16.restype = ctypes.c_int
    lib.meda_peak_mfma_bf16.argtypes = [ctypes.c_int64, ctypes.c_int32, ctypes.POINTER(ctypes.c_int64), vp, vp]
    lib.meda_peak_mfma_valu.restype = ctypes.c_int
    lib.meda_peak_mfma_valu.argtypes = [ctypes.c_int64, ctypes.c_int32, ctypes.c_int32, ctypes.c_int32, vp, vp]
    lib.meda_quantize_fp8.restype = ctypes.c_int
    lib.meda_quantize_fp8.argtypes = [vp, ctypes.c_int32, ctypes.c_int64, ctypes.c_int32, vp, vp, vp]
    lib.meda_dequantize_fp8.restype = ctypes.c_int
    lib.meda_dequantize_fp8.argtypes = [vp, vp, ctypes.c_int32, ctypes.c_int64, ctypes.c_int32, vp, vp]
    lib.meda_decode_attention_fp8.restype = ctypes.c_int
    lib.meda_decode_attention_fp8.argtypes = [dp, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, ctypes.c_size_t, vp]
    _lib = lib
    return lib


def meda_status_string(status: int) -> str:
    return load_library().meda_status_string(status).decode()


def meda_phase_name(phase: int) -> str:
    return load_library().meda_phase_name(phase).decode()


def _check(status: int) -> None:
    if status != 0:
        raise MedaError(status, meda_status_string(status))


def make_params(n_layers, n_q_heads, n_kv_heads, head_dim, seq_len, window, total_budget, dtype,
                recent_num=3, recent_den=4, softmax_scale=0.0, flags=0, n_seqs=0) -> MedaParams:
    """``n_seqs`` = 0: one sequence, arrays without a batch dimension; N >= 1: a batch, every array has a
    leading dimension N (``total_budget`` is the budget of each sequence)."""
    code = _DTYPES.get(dtype, dtype if isinstance(dtype, int) else -1)
    return MedaParams(n_layers, n_q_heads, n_kv_heads, head_dim, seq_len, window, total_budget,
                      recent_num, recent_den, code, softmax_scale, flags, n_seqs)


def meda_workspace_bytes(params: MedaParams) -> int:
    return int(load_library().meda_workspace_bytes(ctypes.byref(params)))


def meda_workspace_region(params: MedaParams, region) -> tuple:
    """(byte offset, byte size) of an intermediate result inside the workspace."""
    rid = REGIONS[region] if isinstance(region, str) else int(region)
    off, size = ctypes.c_size_t(0), ctypes.c_size_t(0)
    _check(load_library().meda_workspace_region(ctypes.byref(params), rid, ctypes.byref(off), ctypes.byref(size)))
    return off.value, size.value


def meda_profile_enable(enable, phase: Optional[int] = None) -> None:
    """Off (False), every kernel (True), or only the kernel of ``phase`` (True with a phase index)."""
    mode = 0 if not enable else (1 if phase is None else 2 + int(phase))
    _check(load_library().meda_profile_enable(mode))


def meda_profile_read(reset: bool = True):
    """(list of per-phase summed milliseconds, number of calls) since the last reset."""
    ms = (ctypes.c_double * N_PHASES)()
    n = ctypes.c_int32(0)
    _check(load_library().meda_profile_read(ms, ctypes.byref(n), 1 if reset else 0))
    return [float(x) for x in ms], int(n.value)


def _ptr(t: Optional[torch.Tensor]):
    return None if t is None else ctypes.c_void_p(t.data_ptr())


@dataclass
class CompressedCache:
    """Outputs of one call (device tensors; reading lengths on the host synchronises)."""
    k_out: torch.Tensor           # [B*Hkv, d]
    v_out: torch.Tensor
    layer_len: torch.Tensor       # int32 [L]
    layer_off: torch.Tensor       # int64 [L+1]
    entropy: Optional[torch.Tensor]
    sel_idx: Optional[torch.Tensor]
    merge_assign: Optional[torch.Tensor]
    n_kv_heads: int

    def sequence(self, n: int) -> "CompressedCache":
        """Sequence n of a batched call: the same ragged buffers with that sequence's lengths and (absolute)
        offsets, so ``layer`` and ``meda_decode_attention`` work on it as on the result of a single call."""
        if self.layer_len.dim() != 2:
            raise ValueError("not a batched result")
        return CompressedCache(self.k_out, self.v_out, self.layer_len[n], self.layer_off[n],
                               None if self.entropy is None else self.entropy[n], self.sel_idx,
                               None if self.merge_assign is None else self.merge_assign[n], self.n_kv_heads)

    def layer(self, l: int):
        """(K, V[, positions]) of layer l as [Hkv, S_l, d] views."""
        off = int(self.layer_off[l]); s = int(self.layer_len[l]); h = self.n_kv_heads
        sl = slice(off * h, (off + s) * h)
        d = self.k_out.shape[-1]
        out = [self.k_out[sl].view(h, s, d), self.v_out[sl].view(h, s, d)]
        if self.sel_idx is not None:
            out.append(self.sel_idx[sl].view(h, s))
        return tuple(out)


class Compressor:
    """Holds the parameters, the workspace and the output buffers for repeated calls of one shape."""

    def __init__(self, params: MedaParams, device="cuda:0", want_entropy=True, want_sel_idx=True,
                 want_merge_assign=False):
        self.lib = load_library()
        self.params = params
        self.device = torch.device(device)
        nbytes = meda_workspace_bytes(params)
        if nbytes == 0:
            # let the library say what is wrong with the parameters
            off, size = ctypes.c_size_t(0), ctypes.c_size_t(0)
            _check(self.lib.meda_workspace_region(ctypes.byref(params), 0, ctypes.byref(off), ctypes.byref(size)))
            raise MedaError(1, "invalid parameters")
        p = params
        dt = {0: torch.float32, 1: torch.bfloat16}[p.dtype]
        dev = self.device
        self.workspace = torch.empty(nbytes, dtype=torch.uint8, device=dev)
        self.batch = (p.n_seqs,) if p.n_seqs >= 1 else ()   # leading dimension of every array
        rows = max(1, p.n_seqs) * p.total_budget * p.n_kv_heads
        self.k_out = torch.empty((rows, p.head_dim), dtype=dt, device=dev)
        self.v_out = torch.empty((rows, p.head_dim), dtype=dt, device=dev)
        self.layer_len = torch.empty(self.batch + (p.n_layers,), dtype=torch.int32, device=dev)
        self.layer_off = torch.empty(self.batch + (p.n_layers + 1,), dtype=torch.int64, device=dev)
        self.entropy = (torch.empty(self.batch + (p.n_layers,), dtype=torch.float64, device=dev)
                        if want_entropy else None)
        self.sel_idx = torch.empty(rows, dtype=torch.int32, device=dev) if want_sel_idx else None
        self.merge_assign = (torch.empty(self.batch + (p.n_layers, p.n_kv_heads, p.seq_len), dtype=torch.int32,
                                         device=dev) if want_merge_assign else None)

    def region(self, name: str, dtype: torch.dtype) -> torch.Tensor:
        off, size = meda_workspace_region(self.params, name)
        return self.workspace[off:off + size].view(dtype)

    def __call__(self, q_win: torch.Tensor, k: torch.Tensor, v: torch.Tensor, modality: torch.Tensor,
                 stream: Optional[torch.cuda.Stream] = None) -> CompressedCache:
        p = self.params
        dt = {0: torch.float32, 1: torch.bfloat16}[p.dtype]
        q_rows = p.seq_len if (p.flags & FLAG_FULL_PROMPT) else p.window
        nb = self.batch
        for name, t, shape in (("q_win", q_win, nb + (p.n_layers, p.n_q_heads, q_rows, p.head_dim)),
                               ("k", k, nb + (p.n_layers, p.n_kv_heads, p.seq_len, p.head_dim)),
                               ("v", v, nb + (p.n_layers, p.n_kv_heads, p.seq_len, p.head_dim))):
            if tuple(t.shape) != shape or t.dtype != dt or not t.is_contiguous() or t.device != self.device:
                raise ValueError(f"{name}: expected contiguous {dt} tensor of shape {shape} on {self.device}")
        if (tuple(modality.shape) != nb + (p.seq_len,) or modality.dtype != torch.uint8
                or modality.device != self.device or not modality.is_contiguous()):
            raise ValueError(f"modality: expected contiguous uint8 tensor of shape {nb + (p.seq_len,)} on the same device")
        s = stream if stream is not None else torch.cuda.current_stream(self.device)
        st = self.lib.meda_compress(ctypes.byref(p), _ptr(q_win), _ptr(k), _ptr(v), _ptr(modality),
                                    _ptr(self.k_out), _ptr(self.v_out), _ptr(self.layer_len), _ptr(self.layer_off),
                                    _ptr(self.entropy), _ptr(self.sel_idx), _ptr(self.merge_assign),
                                    _ptr(self.workspace), self.workspace.numel(), ctypes.c_void_p(s.cuda_stream))
        _check(st)
        return CompressedCache(self.k_out, self.v_out, self.layer_len, self.layer_off, self.entropy,
                               self.sel_idx, self.merge_assign, p.n_kv_heads)


def meda_compress(q_win, k, v, modality, total_budget, recent_num=3, recent_den=4, softmax_scale=0.0,
                  flags=0, want_merge_assign=False, stream=None) -> CompressedCache:
    """One-shot call: allocates workspace and outputs with torch, then runs the pass on the GPU.  Arrays with a
    leading batch dimension (q_win of rank 5) are compressed as a batch of sequences, each with ``total_budget``."""
    n_seqs = q_win.shape[0] if q_win.dim() == 5 else 0
    L, Hq, W, d = q_win.shape[-4:]
    Hkv, T = k.shape[-3], k.shape[-2]
    if flags & FLAG_FULL_PROMPT:
        raise ValueError("with FLAG_FULL_PROMPT the window cannot be read off q_win: use make_params and Compressor")
    params = make_params(L, Hq, Hkv, d, T, W, int(total_budget), q_win.dtype, recent_num, recent_den,
                         softmax_scale, flags, n_seqs)
    comp = Compressor(params, q_win.device, want_merge_assign=want_merge_assign)
    return comp(q_win, k, v, modality, stream)


def make_decode_params(n_layers, n_q_heads, n_kv_heads, head_dim, total_budget, dtype, n_new=0,
                       softmax_scale=0.0) -> MedaDecodeParams:
    code = _DTYPES.get(dtype, dtype if isinstance(dtype, int) else -1)
    return MedaDecodeParams(n_layers, n_q_heads, n_kv_heads, head_dim, n_new, code, total_budget, softmax_scale)


def meda_decode_workspace_bytes(params: MedaDecodeParams) -> int:
    return int(load_library().meda_decode_workspace_bytes(ctypes.byref(params)))


def _check_decode_tensors(p: MedaDecodeParams, q, k_rows, v_rows, row_dtype, layer_len, layer_off, k_new, v_new,
                          out=None) -> None:
    """Shapes, types and placement of the tensors of one decoding step (the library sees only pointers)."""
    dt = torch.bfloat16 if p.dtype == 1 else torch.float32
    dev = q.device
    def want(name, t, shape, dtype, exact=True):
        ok = (t is not None and t.dtype == dtype and t.device == dev and t.is_contiguous() and t.dim() == len(shape)
              and tuple(t.shape[1:]) == tuple(shape[1:])
              and (t.shape[0] == shape[0] if exact else t.shape[0] >= shape[0]))
        if not ok:
            raise ValueError(f"{name}: expected a contiguous {dtype} tensor of shape {tuple(shape)}"
                             f"{'' if exact else ' (or more rows)'} on {dev}")
    if not q.is_cuda:
        raise ValueError("q: expected a tensor on the GPU")
    want("q", q, (p.n_layers, p.n_q_heads, p.head_dim), dt)
    rows = p.total_budget * p.n_kv_heads
    want("k cache", k_rows, (rows, p.head_dim), row_dtype, exact=False)
    want("v cache", v_rows, (rows, p.head_dim), row_dtype, exact=False)
    want("layer_len", layer_len, (p.n_layers,), torch.int32)
    want("layer_off", layer_off, (p.n_layers + 1,), torch.int64)
    if p.n_new > 0:
        want("k_new", k_new, (p.n_layers, p.n_kv_heads, p.n_new, p.head_dim), dt)
        want("v_new", v_new, (p.n_layers, p.n_kv_heads, p.n_new, p.head_dim), dt)
    if out is not None:
        want("out", out, (p.n_layers, p.n_q_heads, p.head_dim), dt)


class Decoder:
    """Holds the workspace and the output row for meda_decode_attention calls with fixed parameters."""

    def __init__(self, params: MedaDecodeParams, device="cuda:0"):
        self.params = params
        self.device = torch.device(device)
        need = meda_decode_workspace_bytes(params)
        if need == 0:
            raise MedaError(1, "invalid or unsupported decode parameters")
        self.workspace = torch.empty(need, dtype=torch.uint8, device=self.device)
        dt = torch.bfloat16 if params.dtype == 1 else torch.float32
        self.out = torch.empty(params.n_layers, params.n_q_heads, params.head_dim, dtype=dt, device=self.device)

    def fp8(self, q, k_codes, v_codes, k_scales, v_scales, layer_len, layer_off, k_new=None, v_new=None, stream=None):
        """The step over a cache stored with meda_quantize_fp8 (bf16 queries only)."""
        _check_decode_tensors(self.params, q, k_codes, v_codes, torch.uint8, layer_len, layer_off, k_new, v_new)
        for name, t in (("k_scales", k_scales), ("v_scales", v_scales)):
            if (t.dtype != torch.float32 or t.device != q.device or not t.is_contiguous() or t.dim() != 1
                    or t.shape[0] < self.params.total_budget * self.params.n_kv_heads):
                raise ValueError(f"{name}: expected a contiguous float32 vector with one entry per cache row on {q.device}")
        stream = stream if stream is not None else torch.cuda.current_stream(self.device)
        _check(load_library().meda_decode_attention_fp8(
            ctypes.byref(self.params), _ptr(q), _ptr(k_codes), _ptr(v_codes), _ptr(k_scales), _ptr(v_scales),
            _ptr(layer_len), _ptr(layer_off), _ptr(k_new), _ptr(v_new), _ptr(self.out), _ptr(self.workspace),
            self.workspace.numel(), ctypes.c_void_p(stream.cuda_stream)))
        return self.out

    def __call__(self, q, k_cache, v_cache, layer_len, layer_off, k_new=None, v_new=None, stream=None):
        _check_decode_tensors(self.params, q, k_cache, v_cache, q.dtype, layer_len, layer_off, k_new, v_new)
        stream = stream if stream is not None else torch.cuda.current_stream(self.device)
        _check(load_library().meda_decode_attention(
            ctypes.byref(self.params), _ptr(q), _ptr(k_cache), _ptr(v_cache), _ptr(layer_len), _ptr(layer_off),
            _ptr(k_new), _ptr(v_new), _ptr(self.out), _ptr(self.workspace), self.workspace.numel(),
            ctypes.c_void_p(stream.cuda_stream)))
        return self.out


def meda_decode_attention_noalloc(params: MedaDecodeParams, q, k_cache, v_cache, layer_len, layer_off, out,
                                  k_new=None, v_new=None, stream=None):
    """meda_decode_attention without a workspace: the library's built-in device array holds the chunk partials.
    ``out`` [L][Hq][d] is written in place (the call itself allocates nothing)."""
    _check_decode_tensors(params, q, k_cache, v_cache, q.dtype, layer_len, layer_off, k_new, v_new, out)
    stream = stream if stream is not None else torch.cuda.current_stream(q.device)
    _check(load_library().meda_decode_attention_noalloc(
        ctypes.byref(params), _ptr(q), _ptr(k_cache), _ptr(v_cache), _ptr(layer_len), _ptr(layer_off),
        _ptr(k_new), _ptr(v_new), _ptr(out), ctypes.c_void_p(stream.cuda_stream)))
    return out


def meda_peak_stream_read(buf: torch.Tensor, sink: torch.Tensor, stream=None) -> None:
    """Enqueue one streaming read of ``buf`` (measurement aid; ``sink`` is a 4-byte device word)."""
    stream = stream if stream is not None else torch.cuda.current_stream(buf.device)
    _check(load_library().meda_peak_stream_read(_ptr(buf), buf.numel() * buf.element_size(), _ptr(sink),
                                                ctypes.c_void_p(stream.cuda_stream)))


def meda_peak_mfma_bf16(mfma_per_wave: int, sink: torch.Tensor, random_operands: bool = False, stream=None) -> int:
    """Enqueue the matrix-instruction micro-kernel (measurement aid); returns the instructions issued chip-wide."""
    stream = stream if stream is not None else torch.cuda.current_stream(sink.device)
    total = ctypes.c_int64(0)
    _check(load_library().meda_peak_mfma_bf16(int(mfma_per_wave), 1 if random_operands else 0, ctypes.byref(total), _ptr(sink),
                                              ctypes.c_void_p(stream.cuda_stream)))
    return int(total.value)


def meda_peak_mfma_valu(rounds: int, valu_per_mfma: int, interleaved: bool, waves_per_simd: int, sink: torch.Tensor,
                        stream=None) -> None:
    """Enqueue the matrix-plus-vector micro-kernel (measurement aid): 16 matrix instructions and 16 * valu_per_mfma
    multiply-adds per round and wave."""
    stream = stream if stream is not None else torch.cuda.current_stream(sink.device)
    _check(load_library().meda_peak_mfma_valu(int(rounds), int(valu_per_mfma), 1 if interleaved else 0, int(waves_per_simd),
                                              _ptr(sink), ctypes.c_void_p(stream.cuda_stream)))


def meda_quantize_fp8(rows: torch.Tensor, stream=None):
    """Row-wise 8-bit (E4M3) storage of ``rows`` [n, d]: returns (codes uint8 [n, d], scales float32 [n])."""
    if rows.dim() != 2 or not rows.is_contiguous() or rows.dtype not in _DTYPES or not rows.is_cuda:
        raise ValueError("rows: expected a contiguous 2-d float32 or bfloat16 tensor on the GPU")
    n, d = rows.shape
    codes = torch.empty((n, d), dtype=torch.uint8, device=rows.device)
    scales = torch.empty(n, dtype=torch.float32, device=rows.device)
    stream = stream if stream is not None else torch.cuda.current_stream(rows.device)
    _check(load_library().meda_quantize_fp8(_ptr(rows), _DTYPES[rows.dtype], n, d, _ptr(codes), _ptr(scales),
                                            ctypes.c_void_p(stream.cuda_stream)))
    return codes, scales


def meda_dequantize_fp8(codes: torch.Tensor, scales: torch.Tensor, dtype=torch.bfloat16, stream=None):
    """The rows a quantised cache stands for, in ``dtype``."""
    if codes.dim() != 2 or codes.dtype != torch.uint8 or not codes.is_contiguous() or not codes.is_cuda:
        raise ValueError("codes: expected a contiguous 2-d uint8 tensor on the GPU")
    n, d = codes.shape
    if tuple(scales.shape) != (n,) or scales.dtype != torch.float32 or scales.device != codes.device:
        raise ValueError("scales: expected float32 [n] on the same device")
    rows = torch.empty((n, d), dtype=dtype, device=codes.device)
    stream = stream if stream is not None else torch.cuda.current_stream(codes.device)
    _check(load_library().meda_dequantize_fp8(_ptr(codes), _ptr(scales), _DTYPES[dtype], n, d, _ptr(rows),
                                              ctypes.c_void_p(stream.cuda_stream)))
    return rows


def meda_decode_attention(q, cache: "CompressedCache", k_new=None, v_new=None, softmax_scale=0.0, stream=None):
    """One decoding step over a cache returned by meda_compress (plus rows appended since)."""
    L, Hq, d = q.shape
    Hkv = cache.n_kv_heads
    n_new = 0 if k_new is None else k_new.shape[2]
    params = make_decode_params(L, Hq, Hkv, d, int(cache.k_out.shape[0]) // Hkv, q.dtype, n_new, softmax_scale)
    return Decoder(params, q.device)(q, cache.k_out, cache.v_out, cache.layer_len, cache.layer_off, k_new, v_new,
                                     stream)
