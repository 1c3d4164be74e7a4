"""GPU parity of the BH4 hash with the weighted gather (Sec. 3.2 hash, Sec. 4 forward pass) through the
C ABI against the CPU oracle: the configuration of the paper's experiments.

Bars: codes bit-exact; weights within 1e-5 relative of the oracle's fp64 value computed from the same
fp32 z; y within max|dy| / rms(y) <= 1e-4 (fp32 tables) or 1e-2 (bf16 tables) of the fp64 reference.
"""
import numpy as np
import pytest
import torch

import oracle
from paper_2403_07221_amd import binding as B
from paper_2403_07221_amd import synth
from sampling import sample_tokens

pytestmark = pytest.mark.gpu

TOL_W = 1e-5
TOL_F32 = 1e-4
TOL_BF16 = 1e-2


@pytest.fixture(scope="module", autouse=True)
def _gpu():
    assert torch.cuda.is_available(), "these tests need the MI355X"
    B.lib()
    yield
    B.lookupffn_set_option("gather_path", 0)


def rel_err(y, ref):
    ref64 = ref.astype(np.float64)
    return float(np.max(np.abs(y.astype(np.float64) - ref64)) / np.sqrt(np.mean(ref64 ** 2)))


def bmats_for(w, b, m=4):
    return synth.make_bmats(synth.seed_for(w.seed_index or w.index, 0, 3) + b, w.n_proj, m, w.d_pad, b)


SHAPES = [
    # n, d, k, tau, block, factors, x dtype
    (64, 64, 8, 8, 16, 4, "f32"),
    (1, 64, 8, 8, 16, 4, "f32"),         # a single token: 15 idle token lanes
    (77, 64, 16, 4, 64, 4, "f32"),       # tau = 4: four tables per tile
    (77, 64, 4, 16, 32, 4, "f32"),       # tau = 16: one table per tile
    (200, 100, 13, 8, 32, 4, "f32"),     # 100 -> 128; k*tau below the width: the last tiles carry no table
    (300, 512, 128, 8, 16, 4, "f32"),    # the paper's small model: two projections
    (300, 512, 256, 4, 64, 4, "f32"),
    (517, 768, 96, 8, 64, 4, "f32"),     # RoBERTa-base width, padded to 1024
    (517, 768, 96, 8, 16, 4, "bf16"),
    (50, 1000, 60, 16, 32, 1, "f32"),    # BH1
    (50, 600, 100, 8, 16, 6, "bf16"),    # six factors
    (2100, 768, 96, 8, 32, 4, "f32"),    # several token groups per wave
    (515, 130, 75, 4, 16, 4, "f32"),     # odd width: rows read one coordinate at a time; two projections
    # tau other than 4, 8, 16: tables straddle the kernel's 16-coordinate tiles, the weights are formed from z
    (300, 768, 170, 9, 64, 4, "f32"),    # the paper's RoBERTa-base row: two projections, a table straddles them
    (129, 768, 100, 9, 16, 4, "bf16"),
    (77, 64, 20, 3, 16, 4, "f32"),
    (200, 512, 40, 13, 32, 4, "f32"),    # tau = 13 (the paper's ablation), two projections
    (50, 1000, 1000, 1, 64, 2, "f32"),   # tau = 1
]


@pytest.mark.parametrize("n,d,k,tau,b,m,xdt", SHAPES)
def test_bh_weighted_codes_exact_weights_close(n, d, k, tau, b, m, xdt):
    print(f"bh weighted hash n={n} d={d} k={k} tau={tau} block={b} m={m} {xdt}", flush=True)
    w = synth.Workload("t", 7, n, d, m, k, tau, 8, x_dtype=xdt)
    bm = synth.make_bmats(100 * d + b, w.n_proj, m, w.d_pad, b)
    x = synth.make_x(n + d, n, d, xdt)
    codes, wts = B.lookupffn_hash_bh_weighted(B.to_device(x), torch.from_numpy(bm).cuda(), k, tau)
    torch.cuda.synchronize()
    assert np.array_equal(B.codes_to_numpy(codes), oracle.bh_hash_codes(x, bm, k, tau))
    want = oracle.weights_from_z(oracle.bh_soft_codes(x, bm, k, tau), k, tau)
    err = np.abs(wts.cpu().numpy().astype(np.float64) - want) / np.maximum(np.abs(want), 1e-30)
    print(f"  weights: max relative error {float(err.max()):.2e}", flush=True)
    assert float(err.max()) <= TOL_W


def test_bh_weighted_hash_leaves_plain_codes_unchanged():
    print("bh weighted hash: same codes as the plain BH hash", flush=True)
    n, d, k, tau, b = 333, 768, 96, 8, 32
    bm = synth.make_bmats(5, 1, 4, 1024, b)
    x = synth.make_x(6, n, d)
    xd, bd = B.to_device(x), torch.from_numpy(bm).cuda()
    codes, _ = B.lookupffn_hash_bh_weighted(xd, bd, k, tau)
    plain = B.lookupffn_hash_bh(xd, bd, k, tau)
    torch.cuda.synchronize()
    assert torch.equal(codes, plain)
    codes9, _ = B.lookupffn_hash_bh_weighted(xd, bd, 100, 9)      # weights through z in scratch memory
    assert torch.equal(codes9, B.lookupffn_hash_bh(xd, bd, 100, 9))


def check_forward(w, b, sample=None, m=4):
    x, _, tables = synth.make_layer(w)
    bm = bmats_for(w, b, m)
    y = B.lookupffn_forward_bh_weighted(B.to_device(x), torch.from_numpy(bm).cuda(), B.to_device(tables))
    torch.cuda.synchronize()
    y = y.cpu().numpy()
    idx = np.arange(x.shape[0]) if sample is None else sample
    err = rel_err(y[idx], oracle.bh_forward_weighted(x[idx], bm, tables))
    print(f"  {w.name} block {b}: weighted max|dy|/rms = {err:.3e} on {len(idx)} tokens "
          f"({B.lookupffn_last_gather_kernel()})", flush=True)
    assert err <= (TOL_BF16 if w.table_dtype == "bf16" else TOL_F32)
    return x, bm, tables, y


def test_forward_bh_weighted_config1_paths_and_workspace():
    print("bh weighted forward C1: direct and staged gather, caller workspace", flush=True)
    w = synth.C1
    ys = {}
    try:
        for path in (1, 2):
            B.lookupffn_set_option("gather_path", path)
            x, bm, tables, ys[path] = check_forward(w, 16)
    finally:
        B.lookupffn_set_option("gather_path", 0)
    assert np.array_equal(ys[1], ys[2])
    xd, bd, td = B.to_device(x), torch.from_numpy(bm).cuda(), B.to_device(tables)
    ws = torch.empty(B.lookupffn_workspace_bytes_bh_weighted(w.n_tokens, w.d, w.k, w.tau, 16, 4), dtype=torch.uint8,
                     device="cuda")
    y2 = B.lookupffn_forward_bh_weighted(xd, bd, td, workspace=ws)
    torch.cuda.synchronize()
    assert np.array_equal(y2.cpu().numpy(), ys[1])
    with pytest.raises(B.LookupFFNError) as e:
        B.lookupffn_forward_bh_weighted(xd, bd, td, workspace=torch.empty(256, dtype=torch.uint8, device="cuda"))
    assert e.value.status == -7
    empty = B.lookupffn_forward_bh_weighted(torch.empty((0, w.d), device="cuda"), bd, td)
    assert tuple(empty.shape) == (0, w.d_out)


def test_forward_bh_weighted_equals_hash_then_gather():
    print("bh weighted forward equals its two halves chained by the caller", flush=True)
    w = synth.C2.with_tokens(3000)
    x, _, tables = synth.make_layer(w)
    bm = bmats_for(w, 64)
    xd, bd, td = B.to_device(x), torch.from_numpy(bm).cuda(), B.to_device(tables)
    codes, wts = B.lookupffn_hash_bh_weighted(xd, bd, w.k, w.tau)
    y_parts = B.lookupffn_gather_weighted(codes, wts, td)
    y = B.lookupffn_forward_bh_weighted(xd, bd, td)
    torch.cuda.synchronize()
    assert torch.equal(y, y_parts)


@pytest.mark.parametrize("w,b,step", [(synth.C2, 64, 5), (synth.C2, 16, 7), (synth.C3, 32, 17), (synth.P7, 32, 13),
                                      (synth.P8, 64, 21)],     # P8: the paper's RoBERTa-base row, tau = 9
                         ids=lambda v: getattr(v, "name", str(v)))
def test_forward_bh_weighted_full_size(w, b, step):
    print(f"bh weighted forward {w.name} block {b} ({w.n_tokens} tokens)", flush=True)
    check_forward(w, b, sample=sample_tokens(w.n_tokens, step))
