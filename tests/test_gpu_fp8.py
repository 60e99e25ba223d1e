"""8-bit (E4M3) storage of the compressed cache: the quantiser must give the oracle's codes and scales bit for
bit (both take the decision in float32), the inverse map must reproduce the format's table for all 256 codes,
and the decoding step over a quantised cache must match the oracle's attention over the values the codes stand
for.  Inputs are seeded synthetic rows; nothing here comes from the HIP path except what is being checked."""
import numpy as np
import pytest
import torch

from oracle import decode_oracle, fp8_oracle
from workloads import generate, get_workload, variant
from workloads.gen import to_float64

from parity import decode_error

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _rows(n, d, dtype, seed):
    g = torch.Generator().manual_seed(seed)
    x = torch.randn(n, d, generator=g) * torch.exp(2.0 * torch.randn(n, 1, generator=g))   # rows of very different size
    x[::7] *= 1e-3
    if n > 3:
        x[3] = 0.0                                   # an all-zero row
        x[2, :] = 0.0
        x[2, 5] = -1.25                              # a single non-zero element
    return x.to(dtype)


@pytest.mark.parametrize("dtype,d,n", [(torch.bfloat16, 128, 1000), (torch.bfloat16, 64, 517), (torch.float32, 128, 301),
                                       (torch.float32, 64, 64), (torch.bfloat16, 128, 1), (torch.bfloat16, 128, 70001)])
def test_quantiser_codes_and_scales_bit_exact(dtype, d, n):
    import paper_2502_17599_amd as pkg
    x = _rows(n, d, dtype, seed=n + d)
    codes, scales = pkg.meda_quantize_fp8(x.to(DEV))
    torch.cuda.synchronize()
    ref_codes, ref_scales = fp8_oracle.quantize_rows(to_float64(x))
    assert np.array_equal(scales.cpu().numpy().view(np.uint32), ref_scales.view(np.uint32))
    assert np.array_equal(codes.cpu().numpy(), ref_codes)


def test_quantiser_ties_and_subnormals():
    """Rows built so that x / scale hits every tie and every subnormal of the format (scale is exactly 1)."""
    import paper_2502_17599_amd as pkg
    t = fp8_oracle.e4m3_decode_table()[:0x7F]
    mids = (t[:-1] + t[1:]) / 2
    vals = np.concatenate([t, mids, -t, -mids, [448.0]])
    vals = vals[np.abs(vals) <= 448.0]
    n = (len(vals) + 126) // 127
    x = np.zeros((n, 128), dtype=np.float32)
    x[:, 0] = 448.0                                   # scale = 1 in every row
    flat = np.zeros(n * 127, dtype=np.float32)
    flat[:len(vals)] = vals                           # all exactly representable in float32
    x[:, 1:] = flat.reshape(n, 127)
    codes, scales = pkg.meda_quantize_fp8(torch.from_numpy(x).to(DEV))
    torch.cuda.synchronize()
    assert (scales.cpu().numpy() == 1.0).all()
    ref_codes, _ = fp8_oracle.quantize_rows(x.astype(np.float64))
    assert np.array_equal(codes.cpu().numpy(), ref_codes)


@pytest.mark.parametrize("dtype", [torch.bfloat16, torch.float32])
def test_inverse_map_reproduces_the_table(dtype):
    import paper_2502_17599_amd as pkg
    finite = np.array([c for c in range(256) if c not in (0x7F, 0xFF)], dtype=np.uint8)
    codes = np.zeros((4, 128), dtype=np.uint8)
    codes.reshape(-1)[:len(finite)] = finite
    scales = np.array([1.0, 1.0, 0.375, 3.0], dtype=np.float32)
    codes[2] = codes[0]
    codes[3] = codes[1]
    out = pkg.meda_dequantize_fp8(torch.from_numpy(codes).to(DEV), torch.from_numpy(scales).to(DEV), dtype)
    torch.cuda.synchronize()
    ref = fp8_oracle.dequantize_rows(codes, scales)
    # value * scale is exact in float32 here (3-bit mantissa times 0.375 or 3) and in bf16 for scale 1
    got = out.double().cpu().numpy()
    assert np.array_equal(got[:2], ref[:2])
    if dtype == torch.float32:
        assert np.array_equal(got, ref)
    else:
        assert np.abs(got - ref).max() <= 2.0 ** -8 * np.abs(ref).max()


def test_round_trip_error_bound():
    import paper_2502_17599_amd as pkg
    x = _rows(4096, 128, torch.bfloat16, seed=9)
    codes, scales = pkg.meda_quantize_fp8(x.to(DEV))
    back = pkg.meda_dequantize_fp8(codes, scales, torch.float32).double().cpu().numpy()
    xd = to_float64(x)
    s = scales.double().cpu().numpy()[:, None]
    assert (np.abs(back - xd) <= np.maximum(np.abs(xd) * 2.0 ** -4, s * 2.0 ** -10) * (1 + 1e-6)).all()


def _decode_case(wl, n_new, seed):
    """Compress with the HIP pass, quantise with the HIP quantiser, decode over the codes; the oracle attends over
    the values the SAME codes stand for (its own table and its own arithmetic)."""
    import paper_2502_17599_amd as pkg
    data = generate(wl)
    dev = torch.device(DEV)
    out = pkg.meda_compress(data["q"].to(dev), data["k"].to(dev), data["v"].to(dev), data["mask"].to(dev),
                            wl.total_budget, wl.recent_num, wl.recent_den)
    kc, ks = pkg.meda_quantize_fp8(out.k_out)
    vc, vs = pkg.meda_quantize_fp8(out.v_out)
    g = torch.Generator().manual_seed(seed)
    L, Hq, Hkv, d = wl.n_layers, wl.n_q_heads, wl.n_kv_heads, wl.head_dim
    q = torch.randn(L, Hq, d, generator=g).to(torch.bfloat16)
    k_new = v_new = None
    if n_new:
        k_new = torch.randn(L, Hkv, n_new, d, generator=g).to(torch.bfloat16)
        v_new = torch.randn(L, Hkv, n_new, d, generator=g).to(torch.bfloat16)
    params = pkg.make_decode_params(L, Hq, Hkv, d, wl.total_budget, torch.bfloat16, n_new)
    dec = pkg.Decoder(params, dev)
    att = dec.fp8(q.to(dev), kc, vc, ks, vs, out.layer_len, out.layer_off,
                  None if k_new is None else k_new.to(dev), None if v_new is None else v_new.to(dev))
    torch.cuda.synchronize()
    k_deq = fp8_oracle.dequantize_rows(kc.cpu().numpy(), ks.cpu().numpy())
    v_deq = fp8_oracle.dequantize_rows(vc.cpu().numpy(), vs.cpu().numpy())
    ref = decode_oracle.decode_step(to_float64(q), k_deq, v_deq, out.layer_len.cpu().numpy(),
                                    out.layer_off.cpu().numpy(), Hkv,
                                    None if k_new is None else to_float64(k_new),
                                    None if v_new is None else to_float64(v_new))
    vmax = max(np.abs(v_deq).max(), 0.0 if v_new is None else float(v_new.abs().max()))
    # fp32 arithmetic on exact inputs, one rounding of the output to bf16
    err = decode_error(att.double().cpu().numpy(), ref, vmax, True)
    print(f"  fp8 decode {wl.name} n_new={n_new}: max error / max|v| = {err:.3e}")
    # and against the bf16 cache: the quantisation error itself (3-bit mantissas) stays small on the output
    att16 = pkg.Decoder(params, dev)(q.to(dev), out.k_out, out.v_out, out.layer_len, out.layer_off,
                                     None if k_new is None else k_new.to(dev), None if v_new is None else v_new.to(dev))
    torch.cuda.synchronize()
    rel = (att.double() - att16.double()).abs().max().item() / vmax
    assert rel <= 0.1, rel


def test_decode_over_quantised_cache_one_head_per_kv_head():
    wl = variant(get_workload("tiny"), name="fp8_mha", n_layers=3, n_q_heads=4, n_kv_heads=4, head_dim=128, dtype="bf16",
                 window=32, total_budget=3 * 300, layout=(("t", 50, -1), ("v", 900, 0), ("t", 74, -1)))
    _decode_case(wl, n_new=0, seed=1)


def test_decode_over_quantised_cache_grouped_heads_with_appended_rows():
    wl = variant(get_workload("tiny"), name="fp8_gqa", n_layers=2, n_q_heads=14, n_kv_heads=2, head_dim=128, dtype="bf16",
                 window=64, total_budget=2 * 333, layout=(("t", 30, -1), ("v", 1500, 0), ("t", 133, -1)))
    _decode_case(wl, n_new=5, seed=2)


def test_decode_over_quantised_cache_head_dim_64():
    wl = variant(get_workload("tiny"), name="fp8_d64", n_layers=2, n_q_heads=8, n_kv_heads=4, head_dim=64, dtype="bf16",
                 window=32, total_budget=2 * 257, layout=(("v", 700, 0), ("t", 199, -1)))
    _decode_case(wl, n_new=200, seed=3)


def test_fp8_decode_needs_bf16_queries():
    import paper_2502_17599_amd as pkg
    params = pkg.make_decode_params(2, 4, 4, 128, 64, torch.float32)
    dec = pkg.Decoder(params, torch.device(DEV))
    q = torch.zeros(2, 4, 128, device=DEV)
    codes = torch.zeros(64 * 4, 128, dtype=torch.uint8, device=DEV)
    scales = torch.ones(64 * 4, device=DEV)
    lens = torch.full((2,), 32, dtype=torch.int32, device=DEV)
    offs = torch.tensor([0, 32, 64], dtype=torch.int64, device=DEV)
    with pytest.raises(pkg.MedaError) as ei:
        dec.fp8(q, codes, codes, scales, scales, lens, offs)
    assert ei.value.status == 3
    # the binding checks shapes, types and placement before the library sees the pointers
    with pytest.raises(ValueError):
        dec(q, codes, codes, lens, offs)                      # cache rows of another type than q
    with pytest.raises(ValueError):
        dec(q, q.new_zeros(100, 128), q.new_zeros(100, 128), lens, offs)   # fewer rows than the budget
    with pytest.raises(ValueError):
        dec(q, q.new_zeros(256, 128), q.new_zeros(256, 128), lens.long(), offs)
