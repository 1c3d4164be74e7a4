"""Pins of the oracle's 16-bit element handling against numpy's and torch's own conversions (independent
implementations): every binary16 pattern widens to numpy's value; fp32 -> binary16 and fp32 -> bf16 round
like numpy / torch on edge cases and on random values; a forward pass on float16 inputs equals the fp32
forward pass on the widened inputs (the 16-bit types are storage formats only)."""
import numpy as np
import torch

import oracle
from paper_2403_07221_amd import synth


def test_every_half_pattern_widens_to_numpys_value():
    bits = np.arange(65536, dtype=np.uint16)
    got = oracle.half_to_float(bits)
    want = bits.view(np.float16).astype(np.float32)
    nan = np.isnan(want)
    assert np.array_equal(np.isnan(got), nan)
    assert np.array_equal(got[~nan].view(np.uint32), want[~nan].view(np.uint32))     # signed zeros included


def edge_values():
    rng = np.random.default_rng(5)
    halves = np.arange(65536, dtype=np.uint16).view(np.float16).astype(np.float32)
    halves = halves[np.isfinite(halves)]
    mid = (halves[:-1].astype(np.float64) + halves[1:].astype(np.float64)) / 2          # exact ties where representable
    vals = [halves, mid.astype(np.float32), np.nextafter(mid.astype(np.float32), np.float32(np.inf)),
            np.nextafter(mid.astype(np.float32), np.float32(-np.inf)),
            np.array([0.0, -0.0, 65504.0, 65519.99, 65520.0, 65536.0, 1e10, -1e10, np.inf, -np.inf, 2.0 ** -24,
                      2.0 ** -25, 2.0 ** -25 * 1.0000001, 2.0 ** -26, 1e-30, -1e-30], dtype=np.float32),
            rng.standard_normal(200000).astype(np.float32) * np.float32(3.0),
            (rng.standard_normal(100000) * 10.0 ** rng.uniform(-10, 6, 100000)).astype(np.float32),
            rng.integers(0, 2 ** 32, 200000, dtype=np.uint64).astype(np.uint32).view(np.float32)]
    v = np.concatenate(vals)
    return v[~np.isnan(v)]


def test_float_to_half_rounds_like_numpy():
    v = edge_values()
    with np.errstate(over="ignore"):
        want = v.astype(np.float16).view(np.uint16)
    assert np.array_equal(oracle.float_to_half(v), want)
    assert oracle.float_to_half(np.array([np.nan], dtype=np.float32))[0] & 0x7C00 == 0x7C00


def test_float_to_bf16_rounds_like_torch_and_like_the_input_recipe():
    v = edge_values()
    want = torch.from_numpy(v).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    got = oracle.float_to_bf16(v)
    assert np.array_equal(got, want)
    fin = np.isfinite(v) & (np.abs(v) < 3e38)
    assert np.array_equal(got[fin], synth.to_bf16_bits(v[fin]))


def test_half_inputs_are_storage_only():
    """float16 x and tables give the bits of the fp32 pass on their widened values, in every variant."""
    rng = np.random.default_rng(11)
    n, d, k, tau, d_out, R = 19, 100, 20, 5, 24, 3
    x16 = rng.standard_normal((n, d)).astype(np.float16)
    t16 = (rng.standard_normal((k, 1 << tau, d_out)) * 0.02).astype(np.float16)
    signs = synth.make_signs(3, 1, R, 128)
    x32, t32 = x16.astype(np.float32), t16.astype(np.float32)
    assert np.array_equal(oracle.hash_codes(x16, signs, k, tau), oracle.hash_codes(x32, signs, k, tau))
    for acc64 in (False, True):
        assert np.array_equal(oracle.forward(x16, signs, t16, acc64=acc64), oracle.forward(x32, signs, t32, acc64=acc64))
    assert np.array_equal(oracle.forward_weighted(x16, signs, t16), oracle.forward_weighted(x32, signs, t32))
    assert np.array_equal(oracle.forward_probes(x16, signs, t16), oracle.forward_probes(x32, signs, t32))
    bm = synth.make_bmats(4, 1, 4, 128, 16)
    assert np.array_equal(oracle.bh_forward(x16, bm, t16), oracle.bh_forward(x32, bm, t32))
