"""Pins for the hash half of the CPU oracle (no GPU).

Each test checks the oracle against something that is not the oracle: the
explicit Sylvester matrix from scipy, an fp64 dense evaluation of
R = D1 H D2 H ... (Sec. 3.2, eq. "hadamard"), closed forms, invariances, and
the arg-max form of the hash (Sec. 3.1, f_k(x) = argmax_i <z_k, S_i>) by brute
force over all 2^tau sign rows.
"""
import numpy as np
import pytest
from scipy.linalg import hadamard

import oracle
from paper_2403_07221_amd import synth


def dense_soft_codes(x, signs, d_pad):
    """fp64 dense evaluation: per projection, v <- ((v * D_r) @ H) / sqrt(d_pad), r = 1..R."""
    H = hadamard(d_pad).astype(np.float64) / np.sqrt(d_pad)
    n, d = x.shape
    P, R, _ = signs.shape
    out = np.zeros((n, P * d_pad))
    xp = np.zeros((n, d_pad))
    xp[:, :d] = x
    for p in range(P):
        v = xp.copy()
        for r in range(R):
            v = (v * signs[p, r].astype(np.float64)[None, :]) @ H
        out[:, p * d_pad:(p + 1) * d_pad] = v
    return out


def brute_codes(z, k, tau):
    """decimal(sign(z_j)) spelled out: coordinate b of table j's slice is bit b."""
    n = z.shape[0]
    codes = np.zeros((n, k), dtype=np.int64)
    for t in range(n):
        for j in range(k):
            s = "".join("1" if z[t, j * tau + b] >= 0 else "0" for b in range(tau))
            codes[t, j] = int(s[::-1], 2)
    return codes


def rand_signs(seed, P, R, d_pad):
    return synth.make_signs(seed, P, R, d_pad)


# ---------------------------------------------------------------- FWHT

@pytest.mark.parametrize("n", [1, 2, 4, 8, 16, 64, 256, 1024])
def test_fwht_matches_dense_sylvester_matrix(n):
    rng = np.random.default_rng(n)
    v = rng.standard_normal(n).astype(np.float32)
    got = oracle.fwht(v).astype(np.float64)
    want = hadamard(n).astype(np.float64) @ v.astype(np.float64) if n > 1 else v.astype(np.float64)
    # log2(n) fp32 additions per output, each <= 2^-24 relative to the running magnitude
    tol = max(1, int(np.log2(n))) * 2.0 ** -23 * np.abs(v).sum()
    assert np.max(np.abs(got - want)) <= tol


@pytest.mark.parametrize("n", [2, 8, 64, 512])
def test_fwht_exact_on_small_integers(n):
    # integers this small stay exact in fp32, so any index or sign slip shows as != 0
    rng = np.random.default_rng(100 + n)
    v = rng.integers(-8, 9, size=n).astype(np.float32)
    want = hadamard(n).astype(np.int64) @ v.astype(np.int64)
    assert np.array_equal(oracle.fwht(v).astype(np.int64), want)


def test_fwht_closed_forms_and_involution():
    n = 128
    e0 = np.zeros(n, np.float32)
    e0[0] = 1
    assert np.array_equal(oracle.fwht(e0), np.ones(n, np.float32))
    ones = np.ones(n, np.float32)
    out = oracle.fwht(ones)
    assert out[0] == n and not out[1:].any()
    v = np.random.default_rng(3).integers(-100, 100, size=n).astype(np.float32)
    assert np.array_equal(oracle.fwht(oracle.fwht(v)) / n, v)


def test_fwht_is_not_symmetric_in_a_wrong_way():
    # H e_j must be column j of the Sylvester matrix (catches a permuted / sequency ordering)
    n = 32
    H = hadamard(n)
    for j in (1, 2, 5, 17, 31):
        e = np.zeros(n, np.float32)
        e[j] = 1
        assert np.array_equal(oracle.fwht(e), H[:, j].astype(np.float32))


# ---------------------------------------------------------------- projection z = x R

@pytest.mark.parametrize("d,k,tau,R", [
    (64, 8, 8, 2),      # tiny benchmark shape
    (48, 6, 8, 3),      # zero-padded 48 -> 64, k*tau < d_pad
    (16, 3, 10, 3),     # 30 of 32 bits from P = 2 projections, a code straddles them
    (8, 5, 4, 1),       # P = 3
    (32, 4, 8, 4),
    (100, 20, 5, 3),    # d_pad = 128: the scale 128^-1/2 is not a power of two
])
def test_soft_codes_match_fp64_dense_projection(d, k, tau, R):
    d_pad, P = oracle.d_pad(d), oracle.n_proj(d, k, tau)
    assert d_pad == 1 << int(np.ceil(np.log2(d))) and P == -(-k * tau // d_pad)
    signs = rand_signs(11 * d + k, P, R, d_pad)
    x = np.random.default_rng(d + tau).standard_normal((33, d)).astype(np.float32)
    z = oracle.soft_codes(x, signs, k, tau)
    assert z.shape == (33, P * d_pad)
    zd = dense_soft_codes(x.astype(np.float64), signs, d_pad)
    scale = np.linalg.norm(x, axis=1, keepdims=True)
    assert np.max(np.abs(z - zd) / scale) < 2e-6
    # independent projections must really differ (own sign diagonals each)
    if P > 1:
        assert np.max(np.abs(z[:, :d_pad] - z[:, d_pad:2 * d_pad])) > 0.1


def test_projection_is_orthonormal_per_round_count():
    d, k, tau = 64, 8, 8
    x = np.random.default_rng(5).standard_normal((50, d)).astype(np.float32)
    for R in (1, 2, 3, 5):
        signs = rand_signs(R, 1, R, 64)
        z = oracle.soft_codes(x, signs, k, tau)
        np.testing.assert_allclose(np.linalg.norm(z, axis=1), np.linalg.norm(x, axis=1), rtol=1e-6)


def test_order_is_sign_flip_then_transform():
    # with one round, x = e_0 and D = diag(s): (x D) H = s_0 * (row 0 of H) = s_0 / sqrt(n) everywhere;
    # the other order (x H) D would give s_i / sqrt(n) instead.
    n = 16
    signs = rand_signs(77, 1, 1, n)
    signs[0, 0, 0] = -1
    signs[0, 0, 1] = 1
    x = np.zeros((1, n), np.float32)
    x[0, 0] = 1
    z = oracle.soft_codes(x, signs, 2, 8)
    assert np.array_equal(z[0], np.full(n, -0.25, np.float32))


# ---------------------------------------------------------------- sign + pack

def test_codes_closed_forms():
    d, k, tau = 64, 8, 8
    plus = np.ones((1, 3, d), np.int8)
    e0 = np.zeros((1, d), np.float32)
    e0[0, 0] = 1
    assert (oracle.hash_codes(e0, plus, k, tau) == 255).all()       # every z = +8^-3 > 0
    assert (oracle.hash_codes(-e0, plus, k, tau) == 0).all()        # every z < 0
    ones = np.ones((1, d), np.float32)
    z = oracle.soft_codes(ones, plus, k, tau)
    assert z[0, 0] == 8.0 and not z[0, 1:].any()                     # odd #rounds: sqrt(n) e_0
    assert (oracle.hash_codes(ones, plus, k, tau) == 255).all()     # z == 0 counts as bit 1


def test_negative_zero_counts_as_nonnegative():
    # x = 0 with an all -1 diagonal makes v = -0 everywhere; (-0)+(-0) = -0 survives at index 0
    d, k, tau = 8, 2, 4
    minus = -np.ones((1, 1, d), np.int8)
    x = np.zeros((1, d), np.float32)
    z = oracle.soft_codes(x, minus, k, tau)
    assert z[0, 0] == 0 and np.signbit(z[0, 0])
    assert (oracle.hash_codes(x, minus, k, tau) == 15).all()


def test_codes_complement_under_negation_and_scale_invariance():
    d, k, tau, R = 64, 8, 8, 3
    signs = rand_signs(9, 1, R, 64)
    x = np.random.default_rng(6).standard_normal((200, d)).astype(np.float32)
    z = oracle.soft_codes(x, signs, k, tau)
    assert (z != 0).all()
    c = oracle.hash_codes(x, signs, k, tau)
    assert np.array_equal(oracle.hash_codes(-x, signs, k, tau), 255 - c)   # eq. "min_max"
    assert np.array_equal(oracle.hash_codes(x * np.float32(2.0 ** -7), signs, k, tau), c)
    assert np.array_equal(oracle.hash_codes(x * np.float32(2.0 ** 9), signs, k, tau), c)


@pytest.mark.parametrize("d,k,tau,R", [(64, 8, 8, 2), (48, 6, 8, 3), (16, 3, 10, 3), (8, 5, 4, 1),
                                        (64, 5, 11, 3), (128, 9, 13, 2), (32, 7, 9, 3), (100, 20, 5, 3)])
def test_codes_match_fp64_recount(d, k, tau, R):
    d_pad, P = oracle.d_pad(d), oracle.n_proj(d, k, tau)
    signs = rand_signs(1000 + d + tau, P, R, d_pad)
    x = np.random.default_rng(7 + tau).standard_normal((257, d)).astype(np.float32)
    codes = oracle.hash_codes(x, signs, k, tau).astype(np.int64)
    assert codes.shape == (257, k) and codes.max() < (1 << tau)
    zd = dense_soft_codes(x.astype(np.float64), signs, d_pad)
    want = brute_codes(zd, k, tau)
    # a bit may differ only where the fp64 value sits inside the fp32 rounding margin of zero
    margin = 1e-5 * np.linalg.norm(x, axis=1) / np.sqrt(d_pad)
    diff = codes ^ want
    for t, j in zip(*np.nonzero(diff)):
        for b in range(tau):
            if (diff[t, j] >> b) & 1:
                assert abs(zd[t, j * tau + b]) <= margin[t], (t, j, b)
    assert np.count_nonzero(diff) <= 2       # such near-zero coordinates are rare
    # and the packing itself, from the oracle's own fp32 z, is exact
    z32 = oracle.soft_codes(x, signs, k, tau)
    assert np.array_equal(brute_codes(z32, k, tau), codes)


@pytest.mark.parametrize("tau", [1, 3, 8])
def test_hash_is_argmax_over_sign_rows(tau):
    # Sec. 3.1: f_k(x) = argmax_i <z_k, S_i>, S_i = the +-1 binary representation of i
    d, k, R = 64, 64 // tau if tau > 1 else 64, 3
    k = min(k, 8)
    signs = rand_signs(tau, 1, R, 64)
    x = np.random.default_rng(tau).standard_normal((64, d)).astype(np.float32)
    z = oracle.soft_codes(x, signs, k, tau).astype(np.float64)
    codes = oracle.hash_codes(x, signs, k, tau)
    i = np.arange(1 << tau)
    S = np.where((i[:, None] >> np.arange(tau)[None, :]) & 1, 1.0, -1.0)     # [2^tau, tau]
    for j in range(k):
        zj = z[:, j * tau:(j + 1) * tau]
        assert np.array_equal(np.argmax(zj @ S.T, axis=1), codes[:, j])
        assert np.array_equal(np.argmin(zj @ S.T, axis=1), (1 << tau) - 1 - codes[:, j])


def test_trailing_coordinates_are_ignored_and_tables_are_contiguous_slices():
    # k*tau = 40 of 64 coordinates used; dropping tables from the end must not change earlier codes
    d, tau, R = 64, 8, 2
    signs = rand_signs(21, 1, R, 64)
    x = np.random.default_rng(8).standard_normal((40, d)).astype(np.float32)
    c8 = oracle.hash_codes(x, signs, 8, tau)
    c5 = oracle.hash_codes(x, signs, 5, tau)
    assert np.array_equal(c8[:, :5], c5)


def test_bf16_input_is_widened_exactly():
    import torch
    d, k, tau, R = 48, 6, 8, 3
    signs = rand_signs(31, 1, R, 64)
    xb = synth.make_x(5, 64, d, "bf16")
    xf = torch.from_numpy(xb.view(np.int16)).view(torch.bfloat16).float().numpy()
    assert np.array_equal(oracle.soft_codes(xb, signs, k, tau), oracle.soft_codes(xf, signs, k, tau))
    assert np.array_equal(oracle.hash_codes(xb, signs, k, tau), oracle.hash_codes(xf, signs, k, tau))


def test_thread_count_does_not_change_results():
    w = synth.C1
    x, signs, _ = synth.make_layer(w)
    oracle.set_threads(1)
    a = oracle.hash_codes(x, signs, w.k, w.tau)
    oracle.set_threads(4)
    b = oracle.hash_codes(x, signs, w.k, w.tau)
    assert np.array_equal(a, b)


def test_bad_arguments_are_rejected():
    x = np.zeros((2, 8), np.float32)
    with pytest.raises(ValueError):      # tau above 16 does not fit a uint16 code
        oracle.hash_codes(x, np.ones((3, 1, 8), np.int8), 1, 17)
    with pytest.raises(ValueError):      # an index outside the table
        oracle.gather(np.full((1, 1), 4, np.uint16), np.zeros((1, 4, 4), np.float32))
