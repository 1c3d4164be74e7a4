"""GPU parity of the weighted variant (Sec. 4 of the paper) through the C ABI against the CPU oracle.

Bars: codes bit-exact; weights within 1e-5 relative of the oracle's fp64 value (the kernel evaluates
|z|_1 / prod(1 + exp(-2|z|)) in fp32 with the hardware exp2: a few ulp per factor, tau <= 16 factors);
y within max|dy| / rms(y) <= 1e-4 (fp32 tables) or 1e-2 (bf16 tables) of the fp64 reference.
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
    B.lookupffn_set_option("hash_path", 0)
    B.lookupffn_set_option("lanes_per_token", 0)
    B.lookupffn_set_option("gather_path", 0)


def rel_err(y, ref):
    ref64 = ref.astype(np.float64)
    return float(np.max(np.abs(y.astype(np.float64) - ref64)) / np.sqrt(np.mean(ref64 ** 2)))


def check_weights(got, want):
    assert got.shape == want.shape
    err = np.abs(got.astype(np.float64) - want) / np.maximum(np.abs(want), 1e-30)
    worst = float(err.max()) if err.size else 0.0
    print(f"  weights: max relative error {worst:.2e}", flush=True)
    assert worst <= TOL_W


def gpu_hash_weighted(x, signs, k, tau):
    codes, w = B.lookupffn_hash_weighted(B.to_device(x), B.to_device(signs), k, tau)
    torch.cuda.synchronize()
    return B.codes_to_numpy(codes), w.cpu().numpy()


WEIGHT_SHAPES = [
    # n, d, k, tau, R, x dtype
    (64, 64, 8, 8, 2, "f32"),
    (1, 64, 8, 8, 2, "f32"),
    (1003, 768, 96, 8, 3, "f32"),    # two-layout kernel, one projection
    (517, 768, 96, 8, 3, "bf16"),
    (300, 1024, 128, 10, 3, "f32"),  # two projections, table 102 straddles them
    (77, 768, 170, 9, 3, "f32"),     # the paper's RoBERTa-base shape: table 113 straddles
    (37, 1024, 250, 4, 4, "f32"),
    (37, 520, 64, 16, 3, "bf16"),    # widest code
    (41, 768, 96, 8, 5, "f32"),      # five rounds: generic kernel
    (129, 48, 6, 8, 3, "f32"),
    (200, 100, 20, 5, 3, "f32"),
    (77, 512, 20, 13, 3, "f32"),
    (50, 2048, 100, 16, 2, "f32"),
    (40, 2000, 7, 1, 3, "bf16"),     # tau = 1: the sigmoid unit
    (65, 16, 3, 10, 3, "f32"),       # sub-wavefront width: a table spans the projection boundary
    (65, 8, 5, 4, 1, "f32"),
    (65, 8, 3, 12, 2, "f32"),        # a table spans three 8-wide projections
    (9, 1, 2, 3, 2, "f32"),          # width 1: every coordinate is its own projection
    (70, 5, 3, 5, 4, "f32"),
    (3000, 512, 256, 8, 3, "f32"),   # four projections, several tokens per wave
]


@pytest.mark.parametrize("n,d,k,tau,R,xdt", WEIGHT_SHAPES)
def test_hash_weighted_codes_exact_weights_close(n, d, k, tau, R, xdt):
    print(f"weighted hash n={n} d={d} k={k} tau={tau} R={R} {xdt}", flush=True)
    w = synth.Workload("t", 7, n, d, R, k, tau, 8, x_dtype=xdt)
    signs = synth.make_signs(1000 * d + k, w.n_proj, R, w.d_pad)
    x = synth.make_x(n + d, n, d, xdt)
    codes, wts = gpu_hash_weighted(x, signs, k, tau)
    assert np.array_equal(codes, oracle.hash_codes(x, signs, k, tau))
    check_weights(wts, oracle.weights(x, signs, k, tau))


def test_hash_weighted_generic_kernel_at_width_1024():
    print("weighted hash, generic kernel, d_pad 1024", flush=True)
    B.lookupffn_set_option("hash_path", 1)
    try:
        for (n, d, k, tau) in [(200, 768, 170, 9), (200, 1024, 128, 10)]:
            w = synth.Workload("t", 7, n, d, 3, k, tau, 8)
            signs = synth.make_signs(5, w.n_proj, 3, w.d_pad)
            x = synth.make_x(6, n, d)
            codes, wts = gpu_hash_weighted(x, signs, k, tau)
            assert np.array_equal(codes, oracle.hash_codes(x, signs, k, tau))
            check_weights(wts, oracle.weights(x, signs, k, tau))
    finally:
        B.lookupffn_set_option("hash_path", 0)


def test_hash_weighted_scale_extremes():
    print("weighted hash, tiny / huge / zero inputs", flush=True)
    d, k, tau, R = 64, 8, 8, 3
    signs = synth.make_signs(5, 1, R, d)
    x = synth.make_x(9, 8, d)
    x[0] *= 1e-6          # weights ~ |z|_1 / 2^tau
    x[1] *= 30.0          # every sigmoid saturates: weight ~ |z|_1
    x[2] = 0.0            # weight 0
    x[3] *= 1e-30
    x[4] *= 1e4           # exp(-2|z|) underflows: still finite
    codes, wts = gpu_hash_weighted(x, signs, k, tau)
    assert np.isfinite(wts).all() and (wts[2] == 0).all()
    assert np.array_equal(codes, oracle.hash_codes(x, signs, k, tau))
    want = oracle.weights(x, signs, k, tau)
    err = np.abs(wts - want) / np.maximum(np.abs(want), 1e-300)
    assert err[want > 1e-36].max() <= TOL_W      # below that the fp32 quotient is subnormal


GATHER_SHAPES = [
    (1003, 96, 8, 768, "f32"),
    (1003, 96, 8, 768, "bf16"),
    (130, 128, 10, 1024, "f32"),
    (77, 7, 5, 20, "f32"),           # k not a multiple of 8: scalar code / weight reads
    (77, 13, 3, 40, "bf16"),
    (5, 1, 1, 4, "f32"),
    (300, 170, 9, 768, "bf16"),
]


@pytest.mark.parametrize("n,k,tau,d_out,tdt", GATHER_SHAPES)
def test_gather_weighted_matches_oracle(n, k, tau, d_out, tdt):
    print(f"weighted gather n={n} k={k} tau={tau} d_out={d_out} {tdt}", flush=True)
    rng = np.random.default_rng(n)
    tables = synth.make_tables(n + k, k, 1 << tau, d_out, tdt)
    codes = rng.integers(0, 1 << tau, size=(n, k)).astype(np.uint16)
    wts = rng.uniform(0.0, 4.0, size=(n, k)).astype(np.float32)
    y = B.lookupffn_gather_weighted(torch.from_numpy(codes.view(np.int16)).cuda(), torch.from_numpy(wts).cuda(),
                                    B.to_device(tables))
    torch.cuda.synchronize()
    want = oracle.gather_weighted(codes, wts.astype(np.float64), tables)
    assert rel_err(y.cpu().numpy(), want) <= (TOL_BF16 if tdt == "bf16" else TOL_F32)


@pytest.mark.parametrize("lpt", [1, 4, 8, 64])
def test_gather_weighted_unit_weights_equal_the_plain_gather(lpt):
    print(f"weighted gather, unit weights, lanes per token {lpt}", flush=True)
    n, k, tau, d_out = 515, 24, 6, 136
    tables = synth.make_tables(3, k, 1 << tau, d_out)
    codes = np.random.default_rng(4).integers(0, 1 << tau, size=(n, k)).astype(np.uint16)
    cd, td = torch.from_numpy(codes.view(np.int16)).cuda(), B.to_device(tables)
    B.lookupffn_set_option("lanes_per_token", lpt)
    try:
        yw = B.lookupffn_gather_weighted(cd, torch.ones((n, k), device="cuda"), td)
        torch.cuda.synchronize()
    finally:
        B.lookupffn_set_option("lanes_per_token", 0)
    assert np.array_equal(yw.cpu().numpy(), oracle.gather(codes, tables, acc64=False))


LDS_SHAPES = [
    # n, k, tau, d_out      (gather_path = 2 forces the LDS-staged kernel: fp32 tables, tau 7 .. 10; odd k has a file of its own)
    (1003, 96, 8, 768),      # three slices per XCD, ragged chunks
    (16384, 32, 8, 768),     # the benchmark's split, two chunks of 6 tokens per lane
    (5000, 24, 7, 200),      # ragged last slice, 128-row tables
    (130, 2, 7, 4),          # a single 16-byte piece per row
    (120000, 4, 7, 128),     # several chunks per workgroup, 12 tokens per lane
    (300, 2, 7, 8192),       # as many slice-units as workgroups
    (1, 6, 8, 64),           # one token
    (777, 2, 8, 64),         # a single stage
    (700, 6, 8, 64),         # an odd number of stages, 6 tokens per lane
    (3000, 170, 9, 768),     # tau = 9: one table per stage
    (1500, 2, 9, 64),        # tau = 9, a single code word
    (9000, 6, 9, 200),       # tau = 9, three code words, ragged last slice
    (5000, 128, 10, 1024),   # tau = 10: 64-byte column slices
    (9000, 6, 10, 200),
]


@pytest.mark.parametrize("n,k,tau,d_out", LDS_SHAPES)
def test_gather_weighted_lds_staged_kernel(n, k, tau, d_out):
    print(f"weighted gather (LDS-staged) n={n} k={k} tau={tau} d_out={d_out}", flush=True)
    rng = np.random.default_rng(n)
    tables = synth.make_tables(n + k, k, 1 << tau, d_out)
    codes = rng.integers(0, 1 << tau, size=(n, k)).astype(np.uint16)
    wts = rng.uniform(0.0, 4.0, size=(n, k)).astype(np.float32)
    cd, wd, td = torch.from_numpy(codes.view(np.int16)).cuda(), torch.from_numpy(wts).cuda(), B.to_device(tables)
    B.lookupffn_set_option("gather_path", 2)
    try:
        y_lds = B.lookupffn_gather_weighted(cd, wd, td)
        torch.cuda.synchronize()
        assert B.lookupffn_last_gather_kernel() == "gather_lds_kernel"
        B.lookupffn_set_option("gather_path", 1)
        y_direct = B.lookupffn_gather_weighted(cd, wd, td)
        torch.cuda.synchronize()
        assert B.lookupffn_last_gather_kernel() == "gather_kernel"
    finally:
        B.lookupffn_set_option("gather_path", 0)
    # both kernels do the same fused multiply-adds in the same order
    assert np.array_equal(y_lds.cpu().numpy(), y_direct.cpu().numpy())
    assert rel_err(y_lds.cpu().numpy(), oracle.gather_weighted(codes, wts.astype(np.float64), tables)) <= TOL_F32


def test_forward_weighted_both_gather_paths_agree():
    print("weighted forward, staged against direct gather", flush=True)
    w = synth.C2.with_tokens(3000)
    x, signs, tables = synth.make_layer(w)
    xd, sd, td = B.to_device(x), B.to_device(signs), B.to_device(tables)
    ys = {}
    try:
        for path in (2, 1):
            B.lookupffn_set_option("gather_path", path)
            ys[path] = B.lookupffn_forward_weighted(xd, sd, td)
            torch.cuda.synchronize()
            assert B.lookupffn_last_gather_kernel() == ("gather_lds_kernel" if path == 2 else "gather_kernel")
    finally:
        B.lookupffn_set_option("gather_path", 0)
    assert np.array_equal(ys[1].cpu().numpy(), ys[2].cpu().numpy())
    assert rel_err(ys[2].cpu().numpy(), oracle.forward_weighted(x, signs, tables)) <= TOL_F32


def check_forward_weighted(w, x, signs, tables, sample=None):
    tol = TOL_BF16 if w.table_dtype == "bf16" else TOL_F32
    y = B.lookupffn_forward_weighted(B.to_device(x), B.to_device(signs), B.to_device(tables))
    torch.cuda.synchronize()
    y = y.cpu().numpy()
    idx = np.arange(x.shape[0]) if sample is None else sample
    err = rel_err(y[idx], oracle.forward_weighted(x[idx], signs, tables))
    print(f"  {w.name}: weighted max|dy|/rms = {err:.3e} on {len(idx)} tokens", flush=True)
    assert err <= tol
    return y


def test_forward_weighted_config1_and_workspace():
    print("weighted forward C1", flush=True)
    w = synth.C1
    x, signs, tables = synth.make_layer(w)
    y = check_forward_weighted(w, x, signs, tables)
    ws = torch.empty(B.lookupffn_workspace_bytes_weighted(w.n_tokens, w.k), dtype=torch.uint8, device="cuda")
    y2 = B.lookupffn_forward_weighted(B.to_device(x), B.to_device(signs), B.to_device(tables), workspace=ws)
    torch.cuda.synchronize()
    assert np.array_equal(y2.cpu().numpy(), y)
    small = torch.empty(256, dtype=torch.uint8, device="cuda")
    with pytest.raises(B.LookupFFNError) as e:
        B.lookupffn_forward_weighted(B.to_device(x), B.to_device(signs), B.to_device(tables), workspace=small)
    assert e.value.status == -7
    empty = B.lookupffn_forward_weighted(torch.empty((0, w.d), device="cuda"), B.to_device(signs), B.to_device(tables))
    assert tuple(empty.shape) == (0, w.d_out)


@pytest.mark.parametrize("w,step", [(synth.C2, 1), (synth.C3, 17), (synth.C4, 7), (synth.P6, 17), (synth.P8, 13)],
                         ids=lambda v: getattr(v, "name", str(v)))
def test_forward_weighted_full_size(w, step):
    print(f"weighted forward {w.name} ({w.n_tokens} tokens)", flush=True)
    x, signs, tables = synth.make_layer(w)
    check_forward_weighted(w, x, signs, tables, sample=sample_tokens(w.n_tokens, step))
