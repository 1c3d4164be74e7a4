"""GPU parity of the d_pad = 1024 hash kernel that keeps four tokens per wavefront (Sec. 3.2, eq. hadamard;
Sec. 3.1 codes): codes bit-exact against the oracle, and the one-token-per-wavefront kernel (hash_path = 2)
on the same inputs, over the shapes that select each of its forms."""
import numpy as np
import pytest
import torch

import oracle
from paper_2403_07221_amd import binding as B
from paper_2403_07221_amd import synth

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module", autouse=True)
def _gpu():
    assert torch.cuda.is_available(), "these tests need the MI355X"
    B.lib()
    yield
    B.lookupffn_set_option("hash_path", 0)
    B.lookupffn_set_option("hash_blocks", 0)


def gpu_hash(x, signs, k, tau):
    codes = B.lookupffn_hash(B.to_device(x), B.to_device(signs), k, tau)
    torch.cuda.synchronize()
    return B.codes_to_numpy(codes)


X4_SHAPES = [
    # n, d, k, tau, R, x dtype          (d a multiple of 16 in (512, 1024], up to four rounds)
    (1, 768, 96, 8, 3, "f32"),          # one token: three rows of the wave read the same row again
    (2, 768, 96, 8, 3, "f32"),
    (3, 768, 96, 8, 3, "bf16"),
    (5, 1024, 96, 8, 3, "f32"),         # one full group and one token
    (4099, 768, 96, 8, 3, "f32"),       # ragged last group
    (4099, 768, 96, 8, 3, "f16"),
    (20011, 768, 96, 8, 3, "f32"),      # more groups than waves: several per wave, rows in flight
    (9001, 1024, 128, 10, 3, "bf16"),   # two projections, several groups per wave
    (1500, 768, 170, 9, 3, "f32"),      # the paper's RoBERTa-base shape: a code straddles the projections
    (700, 1024, 192, 16, 3, "f32"),     # three projections, widest code
    (333, 528, 64, 8, 3, "f32"),        # other row lengths: run-time bounds (33 registers in range)
    (333, 1008, 101, 10, 3, "f16"),     # 63 registers in range, odd k
    (333, 784, 50, 13, 1, "f32"),       # one round
    (333, 768, 96, 8, 2, "bf16"),       # two rounds
    (333, 1024, 250, 4, 4, "f32"),      # four rounds
    (333, 768, 7, 1, 3, "f32"),         # tau = 1
]


@pytest.mark.parametrize("n,d,k,tau,R,xdt", X4_SHAPES)
def test_hash_four_tokens_per_wave_bit_exact(n, d, k, tau, R, xdt):
    print(f"hash (four tokens per wave) n={n} d={d} k={k} tau={tau} R={R} {xdt}", flush=True)
    w = synth.Workload("t", 7, n, d, R, k, tau, 8, x_dtype=xdt)
    signs = synth.make_signs(1000 * d + k + R, w.n_proj, R, w.d_pad)
    x = synth.make_x(n + d + 1, n, d, xdt)
    want = oracle.hash_codes(x, signs, k, tau)
    got = gpu_hash(x, signs, k, tau)
    assert np.array_equal(got, want), f"{np.count_nonzero(got != want)} codes differ"
    B.lookupffn_set_option("hash_path", 2)      # the one-token-per-wave kernel on the same inputs
    try:
        assert np.array_equal(gpu_hash(x, signs, k, tau), want)
    finally:
        B.lookupffn_set_option("hash_path", 0)


@pytest.mark.parametrize("blocks", [1, 3, 64])
def test_hash_four_tokens_per_wave_small_grids(blocks):
    print(f"hash (four tokens per wave) with a grid of {blocks} workgroups: many groups per wave", flush=True)
    n, d, k, tau, R = 2050, 768, 96, 8, 3
    signs = synth.make_signs(77, 1, R, 1024)
    x = synth.make_x(78, n, d, "f32")
    B.lookupffn_set_option("hash_blocks", blocks)
    try:
        got = gpu_hash(x, signs, k, tau)
    finally:
        B.lookupffn_set_option("hash_blocks", 0)
    assert np.array_equal(got, oracle.hash_codes(x, signs, k, tau))


def test_hash_four_tokens_per_wave_special_values():
    print("hash (four tokens per wave): zeros, signed zeros, subnormals, large values, all-equal diagonals", flush=True)
    d, k, tau, R = 1024, 128, 8, 3
    x = np.zeros((9, d), np.float32)
    x[1, 0] = 1
    x[2, 0] = -1
    x[3, :] = 1                       # z = sqrt(n) e_0 and exact zeros elsewhere
    x[4, :] = 1e-41                   # subnormal inputs must not be flushed
    x[5, ::2] = 3e-39
    x[5, 1::2] = -2e-39
    x[6, 5] = 3e38
    x[7, :] = -0.0                    # negative zeros
    x[8, 1023] = -7.5                 # the last coordinate only
    for s in (1, -1, 0):
        signs = (np.full((1, R, d), s, np.int8) if s else synth.make_signs(5, 1, R, d))
        got = gpu_hash(x, signs, k, tau)
        assert np.array_equal(got, oracle.hash_codes(x, signs, k, tau)), f"diagonal {s}"
    # rows shorter than 1024: the padding registers' first-round work is left out
    x768 = np.ascontiguousarray(x[:, :768])
    x768[8, 767] = -7.5
    for s in (1, -1, 0):
        signs = (np.full((1, R, d), s, np.int8) if s else synth.make_signs(6, 1, R, d))
        got = gpu_hash(x768, signs, 96, tau)
        assert np.array_equal(got, oracle.hash_codes(x768, signs, 96, tau)), f"diagonal {s}, d = 768"
