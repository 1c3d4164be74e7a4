"""Pins for the oracle's multi-probe lookup (Sec. 3.1, eq. "partial_softmax" with the rows within one
sign flip of sign(z_k); no GPU).

The oracle enumerates g and its tau one-bit neighbours directly; here the neighbourhood is rebuilt from
its definition (all 2^tau rows filtered by l0 distance to sign(z)), the weights from the explicit soft-max
over all rows, and the sum from torch's embedding_bag.
"""
import numpy as np
import pytest
import torch

import oracle
from paper_2403_07221_amd import synth


def sign_rows(tau):
    i = np.arange(1 << tau)
    return np.where((i[:, None] >> np.arange(tau)[None, :]) & 1, 1.0, -1.0)


def brute_probes(z, k, tau):
    """dense weight matrix W[n, k, 2^tau]: soft-max share of the rows with l0 distance <= 1 to sign(z), else 0."""
    S = sign_rows(tau)
    n = z.shape[0]
    W = np.zeros((n, k, 1 << tau))
    for j in range(k):
        zz = z[:, j * tau:(j + 1) * tau].astype(np.float64)
        scores = zz @ S.T
        soft = np.exp(scores) / np.exp(scores).sum(axis=1, keepdims=True)
        sgn = np.where(zz >= 0, 1.0, -1.0)
        l0 = (S[None, :, :] != sgn[:, None, :]).sum(axis=2)
        W[:, j, :] = np.where(l0 <= 1, soft, 0.0)
    return W


@pytest.mark.parametrize("tau,k", [(1, 5), (2, 4), (3, 4), (8, 6), (10, 2)])
def test_probe_weights_match_the_filtered_full_softmax(tau, k):
    rng = np.random.default_rng(tau)
    z = (rng.standard_normal((40, k * tau + 2)) * rng.uniform(0.05, 2.0, size=(40, 1))).astype(np.float32)
    codes, p = oracle.probe_weights_from_z(z, k, tau)
    W = brute_probes(z, k, tau)
    dense = np.zeros_like(W)
    n = z.shape[0]
    for probe in range(tau + 1):
        rows = codes.astype(np.int64) if probe == 0 else codes.astype(np.int64) ^ (1 << (probe - 1))
        np.add.at(dense, (np.arange(n)[:, None], np.arange(k)[None, :], rows), p[:, :, probe])
    np.testing.assert_allclose(dense, W, rtol=1e-12, atol=1e-300)
    assert (W > 0).sum(axis=2).max() == tau + 1            # exactly 1 + tau probes
    # codes are the top-1 hash codes (arg-max row)
    S = sign_rows(tau)
    for j in range(k):
        assert np.array_equal(np.argmax(z[:, j * tau:(j + 1) * tau].astype(np.float64) @ S.T, axis=1), codes[:, j])


def test_probe_weight_structure():
    tau, k = 8, 3
    rng = np.random.default_rng(0)
    z = rng.standard_normal((25, k * tau)).astype(np.float32)
    _, p = oracle.probe_weights_from_z(z, k, tau)
    assert (p > 0).all() and (p.sum(axis=2) < 1).all()
    a = np.abs(z.astype(np.float64)).reshape(25, k, tau)
    # share of g is prod sigmoid(2|z|); a flip at bit b costs a factor exp(-2|z_b|)
    np.testing.assert_allclose(p[:, :, 0], torch.sigmoid(torch.from_numpy(2 * a)).numpy().prod(-1), rtol=1e-12)
    np.testing.assert_allclose(p[:, :, 1:], p[:, :, :1] * np.exp(-2 * a), rtol=1e-12)
    # tau = 1: both rows are probed, the soft-max is complete
    z1 = rng.standard_normal((25, 4)).astype(np.float32)
    _, p1 = oracle.probe_weights_from_z(z1, 4, 1)
    np.testing.assert_allclose(p1.sum(axis=2), 1.0, rtol=1e-14)
    # far from every hyperplane the best row takes everything: the lookup degenerates to the plain sum
    _, pb = oracle.probe_weights_from_z(np.full((1, 16), 12.0, np.float32), 2, 8)
    np.testing.assert_allclose(pb[:, :, 0], 1.0, rtol=1e-9)
    assert pb[:, :, 1:].max() < 1e-10


def test_gather_probes_is_an_embedding_bag_over_the_probed_rows():
    n, k, tau, d_out = 33, 5, 4, 12
    rng = np.random.default_rng(2)
    tables = synth.make_tables(8, k, 1 << tau, d_out)
    codes = rng.integers(0, 1 << tau, size=(n, k)).astype(np.uint16)
    p = rng.uniform(0, 1, size=(n, k, tau + 1))
    flips = np.concatenate([[0], 1 << np.arange(tau)])
    rows = codes.astype(np.int64)[:, :, None] ^ flips[None, None, :]
    idx = (rows + (np.arange(k) << tau)[None, :, None]).reshape(n, -1)
    flat = torch.from_numpy(tables.astype(np.float64).reshape(k << tau, d_out))
    want = torch.nn.functional.embedding_bag(torch.from_numpy(idx), flat, mode="sum",
                                             per_sample_weights=torch.from_numpy(p.reshape(n, -1))).numpy()
    got = oracle.gather_probes(codes, p, tables)
    assert np.max(np.abs(got - want)) <= 2e-7 * np.max(np.abs(want))
    # weight 1 on the first probe and 0 elsewhere is the plain gather
    p0 = np.zeros_like(p)
    p0[:, :, 0] = 1.0
    assert np.array_equal(oracle.gather_probes(codes, p0, tables), oracle.gather(codes, tables))
    tb = synth.make_tables(9, k, 1 << tau, d_out, "bf16")
    assert np.array_equal(oracle.gather_probes(codes, p, tb), oracle.gather_probes(codes, p, synth.bf16_bits_to_f32(tb)))


@pytest.mark.parametrize("wl", [synth.C1, synth.Workload("straddle", 9, 24, 16, 3, 3, 10, 12),
                                synth.Workload("tau1", 9, 24, 32, 2, 20, 1, 8)])
def test_forward_probes_from_dense_matrices(wl):
    x, signs, tables = synth.make_layer(wl)
    y, codes, p = oracle.forward_probes(x, signs, tables, return_all=True)
    assert np.array_equal(codes, oracle.hash_codes(x, signs, wl.k, wl.tau))
    z = oracle.soft_codes(x, signs, wl.k, wl.tau)
    W = brute_probes(z, wl.k, wl.tau)                                    # [n, k, rows]
    want = np.einsum("nkr,krc->nc", W, tables.astype(np.float64))
    assert np.max(np.abs(y - want)) <= 3e-7 * np.max(np.abs(want))
    if wl.tau == 1:   # complete soft-max: eq. "full_softmax"
        S = sign_rows(1)
        sc = z[:, :wl.k, None].astype(np.float64) * S[None, None, :, 0]
        full = np.exp(sc) / np.exp(sc).sum(axis=2, keepdims=True)
        np.testing.assert_allclose(np.einsum("nkr,krc->nc", full, tables.astype(np.float64)), want, rtol=1e-10)
