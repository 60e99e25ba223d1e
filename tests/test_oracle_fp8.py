"""Pins of the fp8 storage oracle (oracle/fp8_oracle.py): the E4M3 code table against the format's definition,
the encoder against brute-force search and against torch's own float8_e4m3fn conversion, the row scheme against
its stated properties.  The paper fixes no quantisation scheme (it names quantisation as combinable future work),
so none of these values is the paper's."""
import numpy as np
import torch

from oracle import fp8_oracle as F


def test_table_named_values_and_structure():
    t = F.e4m3_decode_table()
    assert t[0x00] == 0.0 and t[0x01] == 2.0 ** -9 and t[0x07] == 7 * 2.0 ** -9     # subnormals m * 2^-9
    assert t[0x08] == 2.0 ** -6                                                      # smallest normal
    assert t[0x38] == 1.0 and t[0x3C] == 1.5 and t[0x40] == 2.0
    assert t[0x7E] == 448.0 and t[0x77] == 240.0
    assert np.isnan(t[0x7F]) and np.isnan(t[0xFF])                                   # the only NaNs, no infinities
    assert np.isfinite(np.delete(t, [0x7F, 0xFF])).all()
    pos = t[:0x7F]
    assert (np.diff(pos) > 0).all()                                                  # codes order like values
    assert np.array_equal(t[0x80:0xFF], -pos)                                        # sign bit only flips the sign
    # spacing of the grid: 2^-9 through the subnormals and the first normal binade, then doubling every 8 codes
    i = np.arange(0x7E)
    assert np.array_equal(np.diff(pos), 2.0 ** (np.maximum(i >> 3, 1) - 10))


def _brute_force_encode(x):
    """Nearest table value; of two equally near ones the code with even mantissa; |x| > 448 saturates."""
    t = F.e4m3_decode_table()[:0x7F]
    out = np.empty(x.shape, dtype=np.uint8)
    for i, v in enumerate(x):
        a = min(abs(v), 448.0)
        d = np.abs(t - a)
        best = np.flatnonzero(d == d.min())
        c = best[0] if len(best) == 1 else [b for b in best if b % 2 == 0][0]
        out[i] = c | (0x80 if np.signbit(v) else 0)
    return out


def test_encoder_is_nearest_with_ties_to_even():
    rng = np.random.default_rng(0)
    t = F.e4m3_decode_table()[:0x7F]
    mids = (t[:-1] + t[1:]) / 2                               # every tie of the format
    near = np.concatenate([mids * (1 - 2.0 ** -20), mids * (1 + 2.0 ** -20)])
    rand = np.concatenate([rng.uniform(-460, 460, 4000), rng.normal(0, 1, 4000), rng.normal(0, 0.01, 2000),
                           rng.uniform(-2.0 ** -6, 2.0 ** -6, 2000)])
    x = np.concatenate([t, -t, mids, -mids, near, rand, [1e9, -1e9, 448.0, 449.0, 464.0]])
    assert np.array_equal(F.e4m3_encode(x), _brute_force_encode(x))


def test_round_trip_and_saturation():
    t = F.e4m3_decode_table()
    finite = np.array([c for c in range(256) if c not in (0x7F, 0xFF)], dtype=np.uint8)
    assert np.array_equal(F.e4m3_encode(t[finite]), finite)   # includes -0 -> 0x80
    assert F.e4m3_encode(np.array([1e30]))[0] == 0x7E and F.e4m3_encode(np.array([-1e30]))[0] == 0xFE
    assert F.e4m3_encode(np.array([2.0 ** -10]))[0] == 0x00   # tie between 0 and the smallest subnormal -> even
    assert F.e4m3_encode(np.array([1.5 * 2.0 ** -9]))[0] == 0x02
    assert F.e4m3_encode(np.array([17.0]))[0] == 0x58 and F.e4m3_encode(np.array([19.0]))[0] == 0x5A


def test_encoder_matches_torch_conversion():
    """An independent implementation of the same format (inside its range: torch maps larger magnitudes to NaN)."""
    rng = np.random.default_rng(1)
    x = np.concatenate([rng.uniform(-448, 448, 20000), rng.normal(0, 1, 20000), rng.normal(0, 2.0 ** -7, 5000)])
    x = x.astype(np.float32)
    ref = torch.from_numpy(x).to(torch.float8_e4m3fn).view(torch.uint8).numpy()
    assert np.array_equal(F.e4m3_encode(x.astype(np.float64)), ref)


def test_rows_scale_extremes_and_error_bound():
    rng = np.random.default_rng(2)
    x = torch.from_numpy(rng.normal(0, 3, (300, 128)).astype(np.float32)).to(torch.bfloat16).double().numpy()
    x[5] = 0.0                                                # an all-zero row
    x[6, :] = 0.0
    x[6, 17] = -2.5                                           # a row with a single non-zero element
    codes, scales = F.quantize_rows(x)
    assert codes.dtype == np.uint8 and scales.dtype == np.float32 and codes.shape == x.shape
    t = F.e4m3_decode_table()
    assert not np.isnan(t[codes]).any()                       # never a NaN code
    amax = np.abs(x).max(axis=1)
    # the largest element of every non-zero row lands on +-448
    j = np.abs(x).argmax(axis=1)
    top = codes[np.arange(len(x)), j] & 0x7F
    assert (top[amax > 0] == 0x7E).all()
    assert scales[5] == 1.0 and (codes[5] == 0).all()
    assert codes[6, 17] == 0xFE and (np.delete(codes[6], 17) == 0).all()
    assert np.array_equal(scales[amax > 0], (amax[amax > 0].astype(np.float32) / np.float32(448.0)))
    # error per element: half a step of the grid, i.e. 2^-4 relative for normal results, scale * 2^-10 below
    deq = F.dequantize_rows(codes, scales)
    err = np.abs(deq - x)
    bound = np.maximum(np.abs(x) * 2.0 ** -4, scales[:, None].astype(np.float64) * 2.0 ** -10) * (1 + 1e-6)
    assert (err <= bound).all()
    # scaling a row by a power of two scales the scale and leaves the codes alone
    codes2, scales2 = F.quantize_rows(x * 4.0)
    assert np.array_equal(codes2, codes) and np.array_equal(scales2[amax > 0], scales[amax > 0] * 4)
