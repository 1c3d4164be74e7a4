"""GPU parity of the multi-probe lookup (Sec. 3.1, eq. "partial_softmax", rows within one sign flip)
through the C ABI against the CPU oracle.

Bars: codes bit-exact; shares within 1e-5 relative of the fp64 value (fp32 product of tau factors with
the hardware exp2, one reciprocal); y within max|dy| / rms(y) <= 1e-4 (fp32 tables) / 1e-2 (bf16 tables).
"""
import numpy as np
import pytest
import torch

import oracle
from paper_2403_07221_amd import binding as B
from paper_2403_07221_amd import synth
from sampling import sample_tokens

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module", autouse=True)
def _gpu():
    assert torch.cuda.is_available(), "these tests need the MI355X"
    B.lib()
    yield
    B.lookupffn_set_option("hash_path", 0)
    B.lookupffn_set_option("lanes_per_token", 0)
    B.lookupffn_set_option("gather_path", 0)


def rel_err(y, ref):
    ref64 = ref.astype(np.float64)
    return float(np.max(np.abs(y.astype(np.float64) - ref64)) / np.sqrt(np.mean(ref64 ** 2)))


SHAPES = [
    # n, d, k, tau, R, x dtype
    (64, 64, 8, 8, 2, "f32"),
    (1003, 768, 96, 8, 3, "f32"),    # two-layout kernel
    (300, 1024, 128, 10, 3, "f32"),  # a table straddles two projections
    (77, 768, 170, 9, 3, "bf16"),
    (41, 768, 96, 8, 5, "f32"),      # generic kernel at width 1024
    (200, 100, 20, 5, 3, "f32"),
    (50, 2048, 100, 16, 2, "f32"),   # 17 probes per table
    (40, 2000, 7, 1, 3, "bf16"),     # tau = 1: the soft-max is complete
    (65, 8, 3, 12, 2, "f32"),        # a table spans three projections
    (3000, 512, 256, 8, 3, "f32"),
]


@pytest.mark.parametrize("n,d,k,tau,R,xdt", SHAPES)
def test_hash_probes_codes_exact_shares_close(n, d, k, tau, R, xdt):
    print(f"probe hash n={n} d={d} k={k} tau={tau} R={R} {xdt}", flush=True)
    w = synth.Workload("t", 7, n, d, R, k, tau, 8, x_dtype=xdt)
    signs = synth.make_signs(1000 * d + k, w.n_proj, R, w.d_pad)
    x = synth.make_x(n + d, n, d, xdt)
    codes, shares = B.lookupffn_hash_probes(B.to_device(x), B.to_device(signs), k, tau)
    torch.cuda.synchronize()
    z = oracle.soft_codes(x, signs, k, tau)
    want_codes, want = oracle.probe_weights_from_z(z, k, tau)
    assert np.array_equal(B.codes_to_numpy(codes), want_codes)
    got = shares.cpu().numpy().astype(np.float64)
    err = np.abs(got - want) / np.maximum(want, 1e-30)
    worst = float(err[want > 1e-30].max())
    print(f"  shares: max relative error {worst:.2e}", flush=True)
    assert worst <= 1e-5
    if tau == 1:
        np.testing.assert_allclose(got.sum(axis=2), 1.0, rtol=1e-6)


GATHER_SHAPES = [
    (1003, 96, 8, 768, "f32"),
    (515, 96, 8, 768, "bf16"),
    (130, 128, 10, 1024, "f32"),
    (77, 7, 5, 20, "f32"),
    (77, 13, 3, 40, "bf16"),
    (5, 1, 1, 4, "f32"),
    (60, 4, 16, 64, "f32"),          # 17 probes, 65536-row tables
]


@pytest.mark.parametrize("n,k,tau,d_out,tdt", GATHER_SHAPES)
def test_gather_probes_matches_oracle(n, k, tau, d_out, tdt):
    print(f"probe gather n={n} k={k} tau={tau} d_out={d_out} {tdt}", flush=True)
    rng = np.random.default_rng(n)
    tables = synth.make_tables(n + k, k, 1 << tau, d_out, tdt)
    codes = rng.integers(0, 1 << tau, size=(n, k)).astype(np.uint16)
    p = rng.uniform(0.0, 1.0, size=(n, k, tau + 1)).astype(np.float32)
    y = B.lookupffn_gather_probes(torch.from_numpy(codes.view(np.int16)).cuda(), torch.from_numpy(p).cuda(),
                                  B.to_device(tables))
    torch.cuda.synchronize()
    want = oracle.gather_probes(codes, p.astype(np.float64), tables)
    assert rel_err(y.cpu().numpy(), want) <= (1e-2 if tdt == "bf16" else 1e-4)


@pytest.mark.parametrize("lpt", [1, 8, 64])
def test_gather_probes_first_probe_only_equals_the_plain_gather(lpt):
    print(f"probe gather, share 1 on the selected row, lanes per token {lpt}", flush=True)
    n, k, tau, d_out = 300, 12, 6, 136
    tables = synth.make_tables(3, k, 1 << tau, d_out)
    codes = np.random.default_rng(4).integers(0, 1 << tau, size=(n, k)).astype(np.uint16)
    p = np.zeros((n, k, tau + 1), np.float32)
    p[:, :, 0] = 1.0
    B.lookupffn_set_option("lanes_per_token", lpt)
    try:
        y = B.lookupffn_gather_probes(torch.from_numpy(codes.view(np.int16)).cuda(), torch.from_numpy(p).cuda(),
                                      B.to_device(tables))
        torch.cuda.synchronize()
    finally:
        B.lookupffn_set_option("lanes_per_token", 0)
    assert np.array_equal(y.cpu().numpy(), oracle.gather(codes, tables, acc64=False))


LDS_SHAPES = [
    # n, k, tau, d_out      (gather_path = 2 forces the LDS-staged kernel: fp32 tables, tau 7 .. 10; odd k has a file of its own)
    (1003, 96, 8, 768),      # 128-byte slices, two tables per stage
    (16384, 8, 8, 768),      # 13 token slots per lane
    (5000, 24, 7, 200),      # 128-row tables, ragged last slice
    (777, 2, 8, 64),         # a single stage
    (700, 6, 8, 64),         # an odd number of stages
    (3000, 20, 9, 768),      # 64-byte slices, two 512-row tables per stage
    (40000, 4, 9, 72),       # 16 token slots per lane, ragged slice
    (5000, 6, 10, 256),      # one 1024-row table per stage: code-word halves alternate
    (2500, 2, 10, 16),
]


@pytest.mark.parametrize("n,k,tau,d_out", LDS_SHAPES)
def test_gather_probes_lds_staged_kernel(n, k, tau, d_out):
    print(f"probe gather (LDS-staged) n={n} k={k} tau={tau} d_out={d_out}", flush=True)
    rng = np.random.default_rng(n)
    tables = synth.make_tables(n + k, k, 1 << tau, d_out)
    codes = rng.integers(0, 1 << tau, size=(n, k)).astype(np.uint16)
    p = rng.uniform(0.0, 1.0, size=(n, k, tau + 1)).astype(np.float32)
    cd, pd, td = torch.from_numpy(codes.view(np.int16)).cuda(), torch.from_numpy(p).cuda(), B.to_device(tables)
    B.lookupffn_set_option("gather_path", 2)
    try:
        y_lds = B.lookupffn_gather_probes(cd, pd, td)
        torch.cuda.synchronize()
        assert B.lookupffn_last_gather_kernel() == "gather_lds_kernel"
        B.lookupffn_set_option("gather_path", 1)
        y_direct = B.lookupffn_gather_probes(cd, pd, td)
        torch.cuda.synchronize()
        assert B.lookupffn_last_gather_kernel() == "gather_kernel"
    finally:
        B.lookupffn_set_option("gather_path", 0)
    want = oracle.gather_probes(codes, p.astype(np.float64), tables)
    # the two kernels add the same terms in different orders (probe-major per stage against table-major)
    assert rel_err(y_lds.cpu().numpy(), want) <= 1e-4
    assert rel_err(y_direct.cpu().numpy(), want) <= 1e-4


def check_forward_probes(w, x, signs, tables, sample=None):
    y = B.lookupffn_forward_probes(B.to_device(x), B.to_device(signs), B.to_device(tables))
    torch.cuda.synchronize()
    y = y.cpu().numpy()
    idx = np.arange(x.shape[0]) if sample is None else sample
    err = rel_err(y[idx], oracle.forward_probes(x[idx], signs, tables))
    print(f"  {w.name}: multi-probe max|dy|/rms = {err:.3e} on {len(idx)} tokens", flush=True)
    assert err <= (1e-2 if w.table_dtype == "bf16" else 1e-4)
    return y


def test_forward_probes_config1_and_workspace():
    print("multi-probe forward C1", flush=True)
    w = synth.C1
    x, signs, tables = synth.make_layer(w)
    y = check_forward_probes(w, x, signs, tables)
    ws = torch.empty(B.lookupffn_workspace_bytes_probes(w.n_tokens, w.k, w.tau), dtype=torch.uint8, device="cuda")
    y2 = B.lookupffn_forward_probes(B.to_device(x), B.to_device(signs), B.to_device(tables), workspace=ws)
    torch.cuda.synchronize()
    assert np.array_equal(y2.cpu().numpy(), y)
    with pytest.raises(B.LookupFFNError) as e:
        B.lookupffn_forward_probes(B.to_device(x), B.to_device(signs), B.to_device(tables),
                                   workspace=torch.empty(256, dtype=torch.uint8, device="cuda"))
    assert e.value.status == -7
    empty = B.lookupffn_forward_probes(torch.empty((0, w.d), device="cuda"), B.to_device(signs), B.to_device(tables))
    assert tuple(empty.shape) == (0, w.d_out)


@pytest.mark.parametrize("w,step", [(synth.C2, 7), (synth.C3, 61), (synth.P7, 29), (synth.P8, 61)],
                         ids=lambda v: getattr(v, "name", str(v)))
def test_forward_probes_full_size(w, step):
    print(f"multi-probe forward {w.name} ({w.n_tokens} tokens)", flush=True)
    x, signs, tables = synth.make_layer(w)
    check_forward_probes(w, x, signs, tables, sample=sample_tokens(w.n_tokens, step))
