"""GPU parity of the hash kernel that keeps a token per row of lanes (d_pad = 1024: four tokens per wavefront,
d_pad = 512: eight; Sec. 3.2, eq. hadamard; Sec. 3.1 codes): codes bit-exact against the oracle, and the
one-token-per-wavefront kernels (hash_path = 2) on the same inputs, over the shapes that select each of its forms."""
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
    B.lookupffn_set_option("hash_path", 3)      # the lane-row kernel at every batch size (by default: large batches only)
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
    # d_pad = 512: eight tokens per wavefront, eight lanes per token
    (1, 512, 64, 8, 3, "f32"),
    (7, 512, 64, 8, 3, "bf16"),         # one group, one row short
    (9, 512, 64, 8, 3, "f32"),          # one full group and one token
    (4099, 512, 64, 8, 3, "f32"),
    (40003, 512, 128, 8, 3, "f32"),     # the paper's small-model shape: two projections, several groups per wave
    (9001, 512, 20, 13, 3, "f16"),      # the paper's tau = 13 ablation shape
    (333, 272, 30, 9, 3, "f32"),        # run-time bounds: 34 registers in range
    (333, 496, 61, 8, 1, "f32"),        # one round
    (333, 512, 64, 8, 2, "f32"),
    (333, 384, 100, 16, 4, "bf16"),     # four rounds, four projections
]


@pytest.mark.parametrize("n,d,k,tau,R,xdt", X4_SHAPES)
def test_hash_four_tokens_per_wave_bit_exact(n, d, k, tau, R, xdt):
    print(f"hash (four tokens per wave) n={n} d={d} k={k} tau={tau} R={R} {xdt}", flush=True)
    w = synth.Workload("t", 7, n, d, R, k, tau, 8, x_dtype=xdt)
    signs = synth.make_signs(1000 * d + k + R, w.n_proj, R, w.d_pad)
    x = synth.make_x(n + d + 1, n, d, xdt)
    want = oracle.hash_codes(x, signs, k, tau)
    got = gpu_hash(x, signs, k, tau)
    assert B.lookupffn_last_hash_kernel() == "hash_row_kernel"
    assert np.array_equal(got, want), f"{np.count_nonzero(got != want)} codes differ"
    B.lookupffn_set_option("hash_path", 2)      # the one-token-per-wave kernel on the same inputs
    try:
        assert np.array_equal(gpu_hash(x, signs, k, tau), want)
        assert B.lookupffn_last_hash_kernel() == ("hash1024_kernel" if d > 512 else "hash_kernel")
    finally:
        B.lookupffn_set_option("hash_path", 3)


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


TOL_W = 2e-5   # relative, per weight: fp32 sum and product of at most 16 terms, exp2 and the fast quotient


X4_WEIGHTED_SHAPES = [
    # n, d, k, tau, R, x dtype      (weights come from this kernel when tau divides 16)
    (1003, 768, 96, 8, 3, "f32"),       # the benchmark's layer: two tables per register
    (4099, 768, 96, 8, 3, "bf16"),
    (20011, 768, 96, 8, 3, "f32"),      # several groups per wave
    (777, 1024, 64, 16, 3, "f32"),      # a table per register
    (777, 1024, 190, 16, 3, "f16"),     # three projections (3040 bits), the last one partly used
    (777, 768, 250, 4, 3, "f32"),       # four tables per register
    (333, 1024, 500, 2, 2, "f32"),      # tau = 2
    (333, 768, 700, 1, 3, "f32"),       # tau = 1: the sigmoid unit
    (333, 528, 37, 8, 4, "f32"),        # run-time bounds, an odd number of tables
    (5, 768, 96, 8, 3, "f32"),
    # d_pad = 512: tau divides 8
    (4099, 512, 64, 8, 3, "f32"),       # a table per register
    (20011, 512, 128, 8, 3, "bf16"),    # two projections
    (777, 512, 200, 4, 3, "f32"),       # two tables per register
    (333, 496, 300, 2, 2, "f32"),
    (333, 272, 400, 1, 4, "f16"),
]


@pytest.mark.parametrize("n,d,k,tau,R,xdt", X4_WEIGHTED_SHAPES)
def test_hash_weighted_four_tokens_per_wave(n, d, k, tau, R, xdt):
    print(f"weighted hash (four tokens per wave) n={n} d={d} k={k} tau={tau} R={R} {xdt}", flush=True)
    w = synth.Workload("t", 7, n, d, R, k, tau, 8, x_dtype=xdt)
    signs = synth.make_signs(1000 * d + k + R, w.n_proj, R, w.d_pad)
    x = synth.make_x(n + d + 2, n, d, xdt)
    want_codes = oracle.hash_codes(x, signs, k, tau)
    want_w = oracle.weights(x, signs, k, tau)
    out = {}
    try:
        for path in (3, 2):                    # 2: the one-token-per-wave kernel on the same inputs
            B.lookupffn_set_option("hash_path", path)
            codes, wts = B.lookupffn_hash_weighted(B.to_device(x), B.to_device(signs), k, tau)
            torch.cuda.synchronize()
            assert B.lookupffn_last_hash_kernel() == ("hash_row_kernel" if path == 3 else "hash1024_kernel" if d > 512 else "hash_kernel")
            out[path] = (B.codes_to_numpy(codes), wts.cpu().numpy())
    finally:
        B.lookupffn_set_option("hash_path", 3)
    for path, (codes, wts) in out.items():
        assert np.array_equal(codes, want_codes), f"hash_path {path}"
        err = np.abs(wts.astype(np.float64) - want_w) / np.maximum(np.abs(want_w), 1e-30)
        assert err.max() <= TOL_W, f"hash_path {path}: weights off by {err.max():.2e}"


def test_forward_weighted_with_the_four_token_hash():
    print("weighted forward, 16384 tokens: hash writes packed codes and table-major weights for the staged gather", flush=True)
    w = synth.C2
    x, signs, tables = synth.make_layer(w)
    xd, sd, td = B.to_device(x), B.to_device(signs), B.to_device(tables)
    ys = {}
    try:
        for path in (3, 2):
            B.lookupffn_set_option("hash_path", path)
            ys[path] = B.lookupffn_forward_weighted(xd, sd, td).cpu().numpy()
            assert B.lookupffn_last_gather_kernel() == "gather_lds_kernel"
    finally:
        B.lookupffn_set_option("hash_path", 3)
    rms = np.sqrt(np.mean(ys[2].astype(np.float64) ** 2))
    assert np.max(np.abs(ys[3].astype(np.float64) - ys[2])) / rms <= 1e-5   # weights differ in the last bits only
    idx = np.r_[0:64, 8000:8064, 16320:16384]
    ref = oracle.forward_weighted(x[idx], signs, tables)
    assert np.max(np.abs(ys[3][idx].astype(np.float64) - ref)) / np.sqrt(np.mean(ref.astype(np.float64) ** 2)) <= 1e-4


def test_hash_kernel_choice_by_batch_size_and_shape():
    print("hash: which kernel the library picks by default", flush=True)
    B.lookupffn_set_option("hash_path", 0)
    try:
        def kernel(n, d, k, tau, weighted=False, R=3):
            w = synth.Workload("t", 7, n, d, R, k, tau, 8)
            signs = B.to_device(synth.make_signs(3, w.n_proj, R, w.d_pad))
            x = B.to_device(synth.make_x(4, n, d))
            (B.lookupffn_hash_weighted if weighted else B.lookupffn_hash)(x, signs, k, tau)
            torch.cuda.synchronize()
            return B.lookupffn_last_hash_kernel()
        assert kernel(2048, 768, 96, 8) == "hash_row_kernel"
        assert kernel(2047, 768, 96, 8) == "hash1024_kernel"          # small batches: one group's latency decides
        assert kernel(4096, 768, 96, 8, weighted=True) == "hash_row_kernel"
        assert kernel(4095, 768, 96, 8, weighted=True) == "hash1024_kernel"
        assert kernel(4096, 768, 80, 10, weighted=True) == "hash_row_kernel"   # tau does not divide 16: z window
        assert kernel(4096, 1000, 96, 8) == "hash1024_kernel"         # d not a multiple of 16
        assert kernel(4096, 768, 96, 8, R=5) == "hash_kernel"         # five rounds
        assert kernel(6144, 512, 64, 8) == "hash_row_kernel"          # d_pad = 512: eight tokens per wavefront
        assert kernel(6143, 512, 64, 8) == "hash_kernel"
        assert kernel(12288, 512, 64, 8, weighted=True) == "hash_row_kernel"
        assert kernel(12287, 512, 64, 8, weighted=True) == "hash_kernel"
        assert kernel(12288, 512, 32, 16, weighted=True) == "hash_row_kernel"  # tau = 16 spans two registers there: z window
        assert kernel(4096, 256, 32, 8) == "hash_kernel"              # d_pad = 256
        assert kernel(4096, 1024, 200, 16) == "hash1024_kernel"       # four projections: the constants outgrow 64 KB of LDS
    finally:
        B.lookupffn_set_option("hash_path", 3)


X_WINDOW_SHAPES = [
    # n, d, k, tau, R, x dtype      (weights of a tau that does not divide the lanes of a token: z window in LDS)
    (4099, 768, 170, 9, 3, "f32"),      # the paper's RoBERTa-base shape: table 113 straddles the two projections
    (20011, 1024, 128, 10, 3, "f32"),   # the benchmark's tau = 10 layer: table 102 straddles
    (777, 1024, 78, 13, 3, "bf16"),     # one projection, last table ends at bit 1014
    (777, 768, 130, 15, 3, "f32"),      # two projections, table 68 straddles them
    (777, 768, 300, 3, 2, "f16"),       # tau = 3
    (5, 768, 170, 9, 3, "f32"),
    (4099, 512, 100, 9, 3, "f32"),      # d_pad = 512: eight tokens per wave, two projections
    (777, 512, 30, 16, 3, "f32"),       # tau = 16 spans two registers of the 8-lane form
    (777, 384, 61, 7, 4, "bf16"),
]


@pytest.mark.parametrize("n,d,k,tau,R,xdt", X_WINDOW_SHAPES)
def test_hash_weighted_lane_rows_any_tau(n, d, k, tau, R, xdt):
    print(f"weighted hash (token per lane row, z window) n={n} d={d} k={k} tau={tau} R={R} {xdt}", flush=True)
    w = synth.Workload("t", 7, n, d, R, k, tau, 8, x_dtype=xdt)
    signs = synth.make_signs(1000 * d + k + R + 1, w.n_proj, R, w.d_pad)
    x = synth.make_x(n + d + 3, n, d, xdt)
    want_codes = oracle.hash_codes(x, signs, k, tau)
    want_w = oracle.weights(x, signs, k, tau)
    codes, wts = B.lookupffn_hash_weighted(B.to_device(x), B.to_device(signs), k, tau)
    torch.cuda.synchronize()
    assert B.lookupffn_last_hash_kernel() == "hash_row_kernel"
    assert np.array_equal(B.codes_to_numpy(codes), want_codes)
    err = np.abs(wts.cpu().numpy().astype(np.float64) - want_w) / np.maximum(np.abs(want_w), 1e-30)
    assert err.max() <= TOL_W, f"weights off by {err.max():.2e}"
