"""The C-ABI library loads, exports every symbol include/meda.h declares, and rejects bad arguments on
the host before anything is launched (no GPU needed)."""
import ctypes
import os
import re

import pytest
import torch

import paper_2502_17599_amd as pkg

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(pkg.library_path()):
        from paper_2502_17599_amd.build import build_library
        build_library()
    return pkg.load_library()


def test_every_declared_symbol_is_exported(lib):
    header = open(os.path.join(ROOT, "include", "meda.h")).read()
    declared = set(re.findall(r"\b(meda_[a-z0-9_]+)\s*\(", header))
    assert declared == set(pkg.EXPORTED_SYMBOLS)
    for name in declared:
        assert getattr(lib, name) is not None


def test_params_struct_matches_header_layout():
    assert ctypes.sizeof(pkg.MedaParams) == 56
    assert pkg.MedaParams.total_budget.offset == 24 and pkg.MedaParams.flags.offset == 48
    assert pkg.MedaParams.n_seqs.offset == 52


def _params(**kw):
    base = dict(n_layers=4, n_q_heads=8, n_kv_heads=2, head_dim=128, seq_len=1000, window=32,
                total_budget=4 * 250, dtype=torch.bfloat16)
    base.update(kw)
    return pkg.make_params(**base)


def test_workspace_bytes_valid_and_invalid(lib):
    assert pkg.meda_workspace_bytes(_params()) > 0
    assert pkg.meda_workspace_bytes(_params()) % 256 == 0
    for bad in (dict(n_layers=0), dict(n_q_heads=7), dict(head_dim=96), dict(window=0), dict(window=2000),
                dict(total_budget=4 * 31), dict(total_budget=4 * 1000 + 1), dict(recent_den=0),
                dict(recent_num=5, recent_den=4), dict(dtype=7), dict(n_q_heads=66, n_kv_heads=2),
                dict(n_layers=300, total_budget=300 * 250), dict(n_seqs=-1), dict(n_seqs=65)):
        assert pkg.meda_workspace_bytes(_params(**bad)) == 0, bad
    # observation windows of more than 128 rows take the row-block mode of the scoring kernels
    assert pkg.meda_workspace_bytes(_params(window=129, seq_len=4096, total_budget=4 * 500)) > 0
    assert pkg.meda_workspace_bytes(_params(window=1000, total_budget=4 * 1000)) > 0
    # sizes whose 32-bit offsets would wrap are refused: a row of one (layer, head) must start below 2 GiB, and the
    # row statistics of all (layer, head, scoring row) triples are counted with 32 bits
    big = dict(n_layers=1, n_q_heads=1, n_kv_heads=1, window=32)
    assert pkg.meda_workspace_bytes(_params(seq_len=(1 << 23) - 1, total_budget=1 << 22, **big)) > 0
    assert pkg.meda_workspace_bytes(_params(seq_len=1 << 23, total_budget=1 << 22, **big)) == 0
    assert pkg.meda_workspace_bytes(_params(seq_len=1 << 22, total_budget=1 << 21, dtype=torch.float32, **big)) == 0
    wide = dict(n_layers=32, n_q_heads=64, n_kv_heads=2, seq_len=1 << 20, total_budget=32 << 19, flags=4)
    assert pkg.meda_workspace_bytes(_params(**wide)) == 0                       # 32 * 64 * 2^20 rows of statistics
    assert pkg.meda_workspace_bytes(_params(**dict(wide, flags=0))) > 0         # 128 rows per head without the flag
    # a batch: the workspace grows with the number of sequences (64 x 4 layers is the largest batch of this shape)
    one, four = pkg.meda_workspace_bytes(_params()), pkg.meda_workspace_bytes(_params(n_seqs=4))
    assert pkg.meda_workspace_bytes(_params(n_seqs=1)) == one and 3 * one < four <= 4 * one + 4096
    assert pkg.meda_workspace_bytes(_params(n_seqs=64)) > 0


def _status(lib, params, ptrs, ws_bytes):
    args = [ctypes.byref(params)] + [ctypes.c_void_p(p) for p in ptrs[:12]] + [ctypes.c_size_t(ws_bytes), None]
    return lib.meda_compress(*args)


def test_compress_rejects_bad_arguments_before_launching(lib):
    p = _params()
    need = pkg.meda_workspace_bytes(p)
    fake = 0x10000  # never dereferenced: every case below fails validation on the host
    good = [fake] * 8 + [0, 0, 0] + [fake]          # entropy, sel_idx, merge_assign may be null
    assert _status(lib, _params(total_budget=1), good, need) == 2          # MEDA_ERR_BUDGET
    assert _status(lib, _params(head_dim=80), good, need) == 3             # MEDA_ERR_UNSUPPORTED
    assert _status(lib, _params(n_q_heads=3), good, need) == 1             # MEDA_ERR_INVALID_ARG
    for i in range(8):                                                      # required pointers
        ptrs = list(good); ptrs[i] = 0
        assert _status(lib, p, ptrs, need) == 1, i
    ptrs = list(good); ptrs[11] = 0
    assert _status(lib, p, ptrs, need) == 4                                 # MEDA_ERR_WORKSPACE: null
    assert _status(lib, p, good, need - 1) == 4                             # too small
    ptrs = list(good); ptrs[11] = fake + 8
    assert _status(lib, p, ptrs, need) == 4                                 # misaligned
    ptrs = list(good); ptrs[1] = fake + 4
    assert _status(lib, p, ptrs, need) == 1                                 # k not 16-byte aligned


def test_status_strings_and_regions(lib):
    assert pkg.meda_status_string(0) == "ok"
    assert "budget" in pkg.meda_status_string(2)
    p = _params()
    total = pkg.meda_workspace_bytes(p)
    seen = []
    for name in pkg.REGIONS:
        off, size = pkg.meda_workspace_region(p, name)
        assert off % 256 == 0 and off + size <= total
        seen.append((off, off + size))
    seen.sort()
    assert all(a[1] <= b[0] for a, b in zip(seen, seen[1:]))
    with pytest.raises(pkg.MedaError):
        pkg.meda_workspace_region(p, 99)
    assert [pkg.meda_phase_name(i) for i in range(pkg.N_PHASES)][0] == "score_stats"


def test_binding_refuses_without_library(monkeypatch, tmp_path):
    import paper_2502_17599_amd._lib as L
    monkeypatch.setattr(L, "_lib", None)
    monkeypatch.setattr(L, "_PKG_DIR", str(tmp_path))
    with pytest.raises(pkg.MedaError):
        L.load_library()


def test_profile_mode_range(lib):
    # 0 off, 1 every phase, 2 + p only phase p; nothing is launched, nothing was recorded
    for mode in (1, 2, 1 + pkg.N_PHASES, 0):
        assert lib.meda_profile_enable(mode) == 0
    assert lib.meda_profile_enable(-1) == 1 and lib.meda_profile_enable(2 + pkg.N_PHASES) == 1
    ms, calls = pkg.meda_profile_read(reset=True)
    assert calls == 0 and all(m == 0.0 for m in ms)


def test_decode_workspace_and_argument_checks(lib):
    p = pkg.make_decode_params(4, 8, 2, 128, 4 * 250, torch.bfloat16, n_new=3)
    need = pkg.meda_decode_workspace_bytes(p)
    assert need > 0 and need % 256 == 0
    assert ctypes.sizeof(pkg.MedaDecodeParams) == 40 and pkg.MedaDecodeParams.total_budget.offset == 24
    for bad in (dict(n_layers=0), dict(n_q_heads=7), dict(head_dim=96), dict(n_new=-1), dict(total_budget=3),
                dict(n_q_heads=18, n_kv_heads=2), dict(dtype=5), dict(softmax_scale=float("inf")),
                dict(n_layers=60000, n_q_heads=512, n_kv_heads=64, total_budget=60000)):
        kw = dict(n_layers=4, n_q_heads=8, n_kv_heads=2, head_dim=128, total_budget=1000, dtype=torch.bfloat16)
        kw.update(bad)
        assert pkg.meda_decode_workspace_bytes(pkg.make_decode_params(**kw)) == 0, bad
    fake = 0x10000   # never dereferenced: every case below fails validation on the host
    def call(params, ptrs, ws_bytes):
        args = [ctypes.byref(params)] + [ctypes.c_void_p(x) for x in ptrs] + [ctypes.c_size_t(ws_bytes), None]
        return lib.meda_decode_attention(*args)
    good = [fake] * 9                                  # q, k, v, len, off, k_new, v_new, out, workspace
    for i in (0, 1, 2, 3, 4, 5, 6, 7):
        ptrs = list(good); ptrs[i] = 0
        assert call(p, ptrs, need) == 1, i             # required pointers (appended rows: n_new > 0)
    ptrs = list(good); ptrs[8] = 0
    assert call(p, ptrs, need) == 4 and call(p, good, need - 1) == 4
    ptrs = list(good); ptrs[1] = fake + 8
    assert call(p, ptrs, need) == 1                    # cache not 16-byte aligned
    p0 = pkg.make_decode_params(4, 8, 2, 128, 1000, torch.bfloat16, n_new=0)
    ptrs = list(good); ptrs[5] = 0; ptrs[6] = 0
    assert call(p0, ptrs, 0) == 4                      # passes the pointer checks, stops at the workspace size


def test_fp8_entry_points_validate_on_the_host(lib):
    q = lib.meda_quantize_fp8
    assert q(None, 1, 0, 128, None, None, None) == 0                 # nothing to do
    assert q(None, 1, -1, 128, None, None, None) == 1
    assert q(None, 1, 8, 128, None, None, None) == 1                 # null pointers
    assert q(None, 1, 8, 96, None, None, None) == 3 and q(None, 5, 8, 128, None, None, None) == 3
    assert q(ctypes.c_void_p(4096 + 8), 1, 8, 128, ctypes.c_void_p(4096), ctypes.c_void_p(4096), None) == 1   # misaligned
    dq = lib.meda_dequantize_fp8
    assert dq(None, None, 1, 0, 64, None, None) == 0 and dq(None, None, 1, 3, 64, None, None) == 1
    assert dq(None, None, 1, 3, 100, None, None) == 3
    # the 8-bit decoding step: bf16 queries only, scales required
    p16 = pkg.make_decode_params(2, 4, 4, 128, 64, torch.bfloat16)
    p32 = pkg.make_decode_params(2, 4, 4, 128, 64, torch.float32)
    a = ctypes.c_void_p(4096)
    f = lib.meda_decode_attention_fp8
    assert f(ctypes.byref(p32), a, a, a, a, a, a, a, None, None, a, a, 1 << 30, None) == 3
    assert f(ctypes.byref(p16), a, a, a, None, a, a, a, None, None, a, a, 1 << 30, None) == 1
    assert f(ctypes.byref(p16), a, a, a, a, a, a, a, None, None, a, a, 16, None) == 4            # workspace too small


def test_decode_binding_checks_tensors_before_the_library_sees_pointers():
    # shapes, types and placement are checked in the binding (the C entry points take plain pointers); without a GPU
    # the first check, placement, is the one that can be exercised
    from paper_2502_17599_amd import _lib
    p = pkg.make_decode_params(2, 4, 2, 64, 2 * 10, torch.float32)
    q = torch.zeros(2, 4, 64)
    rows = torch.zeros(2 * 10 * 2, 64)
    lens = torch.full((2,), 10, dtype=torch.int32)
    offs = torch.tensor([0, 10, 20], dtype=torch.int64)
    with pytest.raises(ValueError, match="on the GPU"):
        _lib._check_decode_tensors(p, q, rows, rows, torch.float32, lens, offs, None, None)


def test_peak_probe_validates_its_arguments_on_the_host(lib):
    fake = ctypes.c_void_p(0x10000)  # never dereferenced: every call below fails validation
    for rounds, v, inter, waves, sink in ((0, 4, 1, 1, fake), (1 << 23, 4, 1, 1, fake), (100, 5, 1, 1, fake),
                                          (100, 4, 1, 3, fake), (100, 4, 0, 0, fake), (100, 4, 1, 1, None),
                                          (100, 4, 1, 1, ctypes.c_void_p(0x10002))):
        assert lib.meda_peak_mfma_valu(rounds, v, inter, waves, sink, None) == 1, (rounds, v, inter, waves)
