"""Pins for the oracle's BH4 hash (Sec. 3.2, eq. "block_acdc": R = prod_i B_i H; no GPU).

The oracle's loop (fused multiply-add chain per output coordinate, in-place transform, scale) is checked
against explicit dense matrices in fp64 (scipy block_diag and hadamard), against the sign-diagonal hash
it must reduce to when every block is a signed identity, and against single-entry matrices that fix the
index convention (row vector times matrix: (v B)_j = sum_c v_c B[c][j]).
"""
import numpy as np
import pytest
from scipy.linalg import block_diag, hadamard

import oracle
from paper_2403_07221_amd import cost, synth


def dense_R(bm_p, d_pad):
    """R = prod_i blockdiag(B_i) H / sqrt(d_pad) in fp64 for one projection; bm_p [m][nb][b][b]."""
    H = hadamard(d_pad).astype(np.float64) / np.sqrt(d_pad) if d_pad > 1 else np.ones((1, 1))
    R = np.eye(d_pad)
    for f in range(bm_p.shape[0]):
        R = R @ block_diag(*[bm_p[f, i].astype(np.float64) for i in range(bm_p.shape[1])]) @ H
    return R


SHAPES = [
    # n, d, k, tau, block, factors
    (20, 64, 8, 8, 16, 4),
    (20, 48, 6, 8, 16, 4),       # padded 48 -> 64
    (12, 128, 40, 8, 32, 4),     # three projections, the last partly used
    (12, 256, 20, 13, 64, 4),    # two projections, a table straddles them
    (9, 64, 8, 8, 64, 1),        # one dense factor
    (9, 32, 4, 8, 4, 2),
    (9, 16, 3, 5, 1, 3),         # block 1: a diagonal scaling
]


@pytest.mark.parametrize("n,d,k,tau,b,m", SHAPES)
def test_bh_matches_dense_fp64_matrices(n, d, k, tau, b, m):
    w = synth.Workload("t", 9, n, d, m, k, tau, 8)
    bm = synth.make_bmats(7 + d + b, w.n_proj, m, w.d_pad, b)
    x = synth.make_x(3, n, d)
    z = oracle.bh_soft_codes(x, bm, k, tau)
    xp = np.zeros((n, w.d_pad))
    xp[:, :d] = x
    z64 = np.concatenate([xp @ dense_R(bm[p], w.d_pad) for p in range(w.n_proj)], axis=1)
    scale = np.abs(z64).max()
    assert np.max(np.abs(z - z64)) <= 2e-6 * scale * (m + 1)
    # every bit the fp64 value decides with a margin must agree
    codes = oracle.bh_hash_codes(x, bm, k, tau)
    zz = z64[:, :k * tau].reshape(n, k, tau)
    sure = (np.abs(zz) > 1e-5 * scale).all(axis=2)
    want = ((zz >= 0).astype(np.int64) << np.arange(tau)).sum(axis=2)
    assert sure.mean() > 0.9 and np.array_equal(codes[sure], want[sure])
    # and the codes are the bits of the oracle's own z
    own = ((z[:, :k * tau].reshape(n, k, tau) >= 0).astype(np.int64) << np.arange(tau)).sum(axis=2)
    assert np.array_equal(codes, own)


@pytest.mark.parametrize("d,k,tau,R,b", [(64, 8, 8, 2, 16), (768, 96, 8, 3, 64), (100, 30, 7, 4, 32)])
def test_signed_identity_blocks_reduce_to_the_sign_diagonal_hash(d, k, tau, R, b):
    w = synth.Workload("t", 9, 40, d, R, k, tau, 8)
    signs = synth.make_signs(11, w.n_proj, R, w.d_pad)
    bm = np.zeros((w.n_proj, R, w.d_pad // b, b, b), np.float32)
    idx = np.arange(b)
    bm[:, :, :, idx, idx] = signs.reshape(w.n_proj, R, w.d_pad // b, b).astype(np.float32)
    x = synth.make_x(5, 40, d)
    assert np.array_equal(oracle.bh_hash_codes(x, bm, k, tau), oracle.hash_codes(x, signs, k, tau))
    assert np.array_equal(oracle.bh_soft_codes(x, bm, k, tau), oracle.soft_codes(x, signs, k, tau))


def test_index_convention_row_vector_times_matrix():
    # one factor, one block; B has the single entry B[c][j] = 1: e_c B = e_j, so z = row j of H / sqrt(N)
    N, c, j = 16, 3, 10
    bm = np.zeros((1, 1, 1, N, N), np.float32)
    bm[0, 0, 0, c, j] = 1.0
    x = np.zeros((2, N), np.float32)
    x[0, c] = 1.0
    x[1, j] = 1.0                      # would respond if the matrix were applied transposed
    z = oracle.bh_soft_codes(x, bm, 2, 8)
    np.testing.assert_array_equal(z[0], hadamard(N)[j].astype(np.float32) / 4.0)
    assert not z[1].any()
    # block index: the same entry in the second block of a block-8 matrix acts on coordinates 8 + c', 8 + j'
    bm8 = np.zeros((1, 1, 2, 8, 8), np.float32)
    bm8[0, 0, 1, 2, 5] = 1.0
    x2 = np.zeros((1, N), np.float32)
    x2[0, 8 + 2] = 1.0
    np.testing.assert_array_equal(oracle.bh_soft_codes(x2, bm8, 2, 8)[0], hadamard(N)[8 + 5].astype(np.float32) / 4.0)


def test_factor_order_first_factor_acts_first():
    # B_1 = 2 I then B_2 = projector on coordinate 0: x B_1 H B_2 H differs from x B_2 H B_1 H
    N = 8
    bm = np.zeros((1, 2, 1, N, N), np.float32)
    bm[0, 0, 0] = 2 * np.eye(N)
    bm[0, 1, 0, 0, 0] = 1.0
    x = np.arange(1, N + 1, dtype=np.float32)[None, :]
    z = oracle.bh_soft_codes(x, bm, 1, 8)
    H = hadamard(N) / np.sqrt(N)
    want = ((2 * x.astype(np.float64)) @ H * np.eye(N)[0]) @ H          # keeps only coordinate 0 after the first round
    np.testing.assert_allclose(z, want, rtol=1e-6)
    swapped = bm[:, ::-1].copy()
    assert not np.allclose(oracle.bh_soft_codes(x, swapped, 1, 8), want)


def test_accumulation_is_a_fused_chain_in_ascending_order():
    # three terms whose fp32 sum depends on order and on fusing: 2^24, 1, -2^24 (ascending chain gives 0 + ... )
    N = 4
    bm = np.zeros((1, 1, 1, N, N), np.float32)
    bm[0, 0, 0, :, 0] = [1.0, 1.0, 1.0, 0.0]
    x = np.array([[2.0 ** 24, 1.0, -2.0 ** 24, 0.0]], np.float32)
    # ascending fp32 chain: (2^24 + 1) rounds to 2^24, minus 2^24 -> 0; any other order gives 1
    u0 = 0.0
    z = oracle.bh_soft_codes(x, bm, 1, 4)
    assert z[0, 0] == u0 * 0.5 and (z[0] == 0).all()
    # fused: x0*b0 + acc with x0*b0 inexact in fp32 but exact inside the fused operation
    a, b_ = np.float32(1 + 2.0 ** -12), np.float32(1 + 2.0 ** -12)       # product 1 + 2^-11 + 2^-24
    bm2 = np.zeros((1, 1, 1, 2, 2), np.float32)
    bm2[0, 0, 0, :, 0] = [b_, 1.0]
    x2 = np.array([[a, -(1 + 2.0 ** -11)]], np.float32)
    z2 = oracle.bh_soft_codes(x2, bm2, 1, 2)
    # chain: acc = fl(a*b) = 1 + 2^-11 (2^-24 lost, fused with +0 rounds once); then fma(x1, 1, acc) = 0
    assert z2[0, 0] == 0.0
    bm3 = bm2.copy()
    bm3[0, 0, 0, :, 0] = [1.0, b_]
    x3 = np.array([[-(1 + 2.0 ** -11), a]], np.float32)
    # other order: acc = -(1 + 2^-11); fma(a, b, acc) keeps the 2^-24 exactly
    assert oracle.bh_soft_codes(x3, bm3, 1, 2)[0, 0] == np.float32(2.0 ** -24 / np.sqrt(2.0))


def test_bf16_inputs_are_widened_exactly_and_forward_chains_hash_and_gather():
    w = synth.Workload("t", 9, 30, 64, 4, 8, 8, 32)
    bm = synth.make_bmats(2, 1, 4, 64, 16)
    xb = synth.make_x(4, 30, 64, "bf16")
    assert np.array_equal(oracle.bh_hash_codes(xb, bm, 8, 8), oracle.bh_hash_codes(synth.bf16_bits_to_f32(xb), bm, 8, 8))
    tables = synth.make_tables(6, 8, 256, 32)
    x = synth.make_x(4, 30, 64)
    y, codes = oracle.bh_forward(x, bm, tables, return_codes=True)
    assert np.array_equal(codes, oracle.bh_hash_codes(x, bm, 8, 8))
    assert np.array_equal(y, oracle.gather(codes, tables))


def test_flop_model_matches_the_loop_counts():
    # per token and projection: m * (2 * d_pad * b multiply-adds + d_pad log2 d_pad butterflies)
    for d, h, tau, b in [(512, 128, 8, 64), (512, 128, 8, 16), (768, 96, 8, 32)]:
        dp = 1 << (d - 1).bit_length()
        P = -(-h * tau // dp)
        assert cost.hash_flops(d, h, tau, "bh4", b) == P * 4 * (2 * dp * b + dp * int(np.log2(dp)))


def test_bh_weighted_forward_from_dense_matrices_and_explicit_softmax():
    """BH hash + weighted gather (Sec. 3.2 + Sec. 4) rebuilt from dense fp64 matrices, the sign matrix S
    and the explicit soft-max over all 2^tau rows: y = sum_j (top * softmax_top) T_j[argmax]."""
    n, d, k, tau, b, m, d_out = 25, 64, 8, 8, 16, 4, 12
    w = synth.Workload("t", 9, n, d, m, k, tau, d_out)
    bm = synth.make_bmats(21, w.n_proj, m, w.d_pad, b)
    x = synth.make_x(4, n, d)
    tables = synth.make_tables(5, k, 1 << tau, d_out)
    y, codes, wts = oracle.bh_forward_weighted(x, bm, tables, return_all=True)
    z64 = x.astype(np.float64) @ dense_R(bm[0], w.d_pad)
    i = np.arange(1 << tau)
    S = np.where((i[:, None] >> np.arange(tau)[None, :]) & 1, 1.0, -1.0)
    want = np.zeros((n, d_out))
    for j in range(k):
        scores = z64[:, j * tau:(j + 1) * tau] @ S.T
        g = np.argmax(scores, axis=1)
        top = scores[np.arange(n), g]
        wj = top * np.exp(top) / np.exp(scores).sum(axis=1)
        sure = np.abs(z64[:, j * tau:(j + 1) * tau]).min(axis=1) > 1e-5
        assert np.array_equal(codes[sure, j], g[sure])
        np.testing.assert_allclose(wts[:, j], wj, rtol=2e-5)
        want += wj[:, None] * tables[j, codes[:, j]].astype(np.float64)
    assert np.max(np.abs(y - want)) <= 2e-5 * np.sqrt(np.mean(want ** 2))
    # the weights do not move the codes
    assert np.array_equal(codes, oracle.bh_hash_codes(x, bm, k, tau))
