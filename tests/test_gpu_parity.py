"""GPU parity: the HIP path (through the C ABI) against the CPU oracle on identical seeded inputs.

Bars: codes bit-exact; y within max|dy| / rms(y) <= 1e-4 (fp32 tables) or 1e-2 (bf16 tables) of the
oracle's fp64-accumulated reference.  The kernels add in table order in fp32, so y is additionally
required to equal the oracle's fp32 sequential mode bit for bit.
"""
import numpy as np
import pytest
import torch

import oracle
from paper_2403_07221_amd import binding as B
from paper_2403_07221_amd import synth
from sampling import sample_tokens

pytestmark = pytest.mark.gpu

TOL_F32 = 1e-4
TOL_BF16 = 1e-2


@pytest.fixture(scope="module", autouse=True)
def _gpu():
    assert torch.cuda.is_available(), "these tests need the MI355X"
    B.lib()                      # fail loudly if the HIP library is not built
    yield
    B.lookupffn_set_option("lanes_per_token", 0)
    B.lookupffn_set_option("xcd_order", 0)
    B.lookupffn_set_option("gather_path", 0)
    B.lookupffn_set_option("hash_path", 0)
    B.lookupffn_set_option("hash_blocks", 0)
    B.lookupffn_set_option("slice_lanes", 0)


def rel_err(y, ref):
    ref64 = ref.astype(np.float64)
    rms = np.sqrt(np.mean(ref64 ** 2))
    return float(np.max(np.abs(y.astype(np.float64) - ref64)) / rms)


def gpu_hash(x, signs, k, tau):
    codes = B.lookupffn_hash(B.to_device(x), B.to_device(signs), k, tau)
    torch.cuda.synchronize()
    return B.codes_to_numpy(codes)


def gpu_gather(codes, tables):
    y = B.lookupffn_gather(torch.from_numpy(codes.view(np.int16)).cuda(), B.to_device(tables))
    torch.cuda.synchronize()
    return y.cpu().numpy()


def gpu_forward(x, signs, tables, **kw):
    y = B.lookupffn_forward(B.to_device(x), B.to_device(signs), B.to_device(tables), **kw)
    torch.cuda.synchronize()
    return y.cpu().numpy()


def assert_codes_equal(got, want):
    if not np.array_equal(got, want):
        t, j = np.argwhere(got != want)[0]
        raise AssertionError(f"{np.count_nonzero(got != want)} codes differ; first at token {t}, table {j}: "
                             f"gpu {got[t, j]} oracle {want[t, j]}")


# ------------------------------------------------------------------ hash

HASH_SHAPES = [
    # n, d, k, tau, R, x dtype
    (64, 64, 8, 8, 2, "f32"),        # tiny benchmark shape
    (1, 64, 8, 8, 2, "f32"),         # a single token
    (1003, 768, 96, 8, 3, "f32"),    # 768 -> 1024 padding, ragged token count
    (517, 768, 96, 8, 3, "bf16"),
    (300, 1024, 128, 10, 3, "f32"),  # two projections, a code straddles them
    (129, 48, 6, 8, 3, "f32"),       # 48 -> 64, trailing coordinates unused
    (200, 100, 20, 5, 3, "f32"),     # d_pad = 128: scale is not a power of two
    (77, 512, 20, 13, 3, "f32"),     # the paper's tau = 13 ablation shape
    (77, 768, 170, 9, 3, "f32"),     # the paper's RoBERTa-base shape: two projections
    (50, 2048, 100, 16, 2, "f32"),   # widest code
    (33, 4096, 300, 11, 1, "f32"),   # largest supported width
    (40, 2000, 7, 1, 3, "bf16"),     # tau = 1
    (65, 16, 3, 10, 3, "f32"),       # sub-wavefront width, two projections
    (65, 32, 9, 7, 2, "f32"),
    (65, 8, 5, 4, 1, "f32"),         # three 8-wide projections
    (9, 1, 2, 1, 2, "f32"),          # degenerate width 1
    (70, 5, 3, 5, 4, "f32"),
    # d_pad = 1024 takes the two-layout kernel: every round count, scalar and vector row loads
    (37, 1001, 60, 8, 1, "f32"),     # d not a multiple of 4: scalar loads
    (37, 600, 128, 8, 2, "f32"),
    (37, 1024, 250, 4, 4, "f32"),
    (37, 520, 64, 16, 3, "bf16"),
    (37, 999, 30, 7, 3, "bf16"),
    (41, 768, 96, 8, 5, "f32"),      # five rounds: back to the generic kernel
    (5000, 768, 96, 8, 3, "f32"),    # several tokens per wave
]


@pytest.mark.parametrize("n,d,k,tau,R,xdt", HASH_SHAPES)
def test_hash_codes_bit_exact(n, d, k, tau, R, xdt):
    print(f"hash n={n} d={d} k={k} tau={tau} R={R} {xdt}", flush=True)
    w = synth.Workload("t", 7, n, d, R, k, tau, 8, x_dtype=xdt)
    signs = synth.make_signs(1000 * d + k, w.n_proj, R, w.d_pad)
    x = synth.make_x(n + d, n, d, xdt)
    assert_codes_equal(gpu_hash(x, signs, k, tau), oracle.hash_codes(x, signs, k, tau))


def test_hash_special_inputs():
    print("hash special inputs", flush=True)
    d, k, tau, R = 64, 8, 8, 3
    x = np.zeros((6, d), np.float32)
    x[1, 0] = 1                       # e_0
    x[2, 0] = -1                      # -e_0
    x[3, :] = 1                       # ones: z = sqrt(n) e_0, exact zeros elsewhere
    x[4, :] = 1e-41                   # subnormal inputs must not be flushed
    x[5, ::2] = 3e-39
    x[5, 1::2] = -2e-39
    for s in (1, -1, 0):
        signs = (np.full((1, R, d), s, np.int8) if s else synth.make_signs(5, 1, R, d))
        assert_codes_equal(gpu_hash(x, signs, k, tau), oracle.hash_codes(x, signs, k, tau))
    # zero input with an all -1 diagonal yields -0 at coordinate 0: must still count as bit 1
    got = gpu_hash(x[:1], np.full((1, 1, d), -1, np.int8), k, tau)
    assert (got == 255).all()


def test_hash_special_inputs_wide():
    print("hash special inputs, d_pad = 1024", flush=True)
    d, k, tau, R = 768, 96, 8, 3
    x = np.zeros((7, d), np.float32)
    x[1, 0] = 1
    x[2, 0] = -1
    x[3, :] = 1
    x[4, :] = 1e-41                   # subnormal inputs must not be flushed
    x[5, ::2] = 3e-39
    x[5, 1::2] = -2e-39
    x[6, 5] = 3e38                    # large values: the scale keeps intermediate sums finite
    for s in (1, -1, 0):
        signs = (np.full((1, R, 1024), s, np.int8) if s else synth.make_signs(5, 1, R, 1024))
        assert_codes_equal(gpu_hash(x, signs, k, tau), oracle.hash_codes(x, signs, k, tau))
    B.lookupffn_set_option("hash_path", 1)      # and the generic kernel on the same inputs
    try:
        signs = synth.make_signs(6, 1, R, 1024)
        assert_codes_equal(gpu_hash(x, signs, k, tau), oracle.hash_codes(x, signs, k, tau))
    finally:
        B.lookupffn_set_option("hash_path", 0)


def test_hash_large_dynamic_range_inputs():
    print("hash dynamic range", flush=True)
    n, d, k, tau, R = 256, 768, 96, 8, 3
    rng = np.random.default_rng(12)
    x = (rng.standard_normal((n, d)) * np.exp(rng.uniform(-30, 30, size=(n, 1)))).astype(np.float32)
    x[rng.random((n, d)) < 0.3] = 0
    signs = synth.make_signs(3, 1, R, 1024)
    assert_codes_equal(gpu_hash(x, signs, k, tau), oracle.hash_codes(x, signs, k, tau))


# ------------------------------------------------------------------ gather

GATHER_SHAPES = [
    # n, k, tau, d_out, table dtype
    (64, 8, 8, 64, "f32"),
    (1003, 96, 8, 768, "f32"),      # several token blocks, ragged tail
    (1003, 96, 8, 768, "bf16"),
    (130, 128, 10, 1024, "f32"),
    (77, 7, 5, 20, "f32"),          # k not a multiple of 8, ragged last slice
    (77, 13, 3, 40, "bf16"),
    (5, 1, 1, 4, "f32"),
    (2048, 20, 13, 512, "f32"),
    (300, 170, 9, 768, "bf16"),
]


@pytest.mark.parametrize("n,k,tau,d_out,tdt", GATHER_SHAPES)
def test_gather_matches_oracle(n, k, tau, d_out, tdt):
    print(f"gather n={n} k={k} tau={tau} d_out={d_out} {tdt}", flush=True)
    tables = synth.make_tables(n + k, k, 1 << tau, d_out, tdt)
    codes = np.random.default_rng(n).integers(0, 1 << tau, size=(n, k)).astype(np.uint16)
    y = gpu_gather(codes, tables)
    assert rel_err(y, oracle.gather(codes, tables, acc64=True)) <= (TOL_BF16 if tdt == "bf16" else TOL_F32)
    assert np.array_equal(y, oracle.gather(codes, tables, acc64=False))


@pytest.mark.parametrize("lpt", [1, 2, 4, 8, 16, 32, 64])
@pytest.mark.parametrize("xcd", [1, -1])
def test_gather_every_launch_shape(lpt, xcd):
    print(f"gather launch shape lpt={lpt} xcd={xcd}", flush=True)
    B.lookupffn_set_option("lanes_per_token", lpt)
    B.lookupffn_set_option("xcd_order", xcd)
    try:
        for tdt, d_out, n in (("f32", 200, 333), ("bf16", 776, 259)):
            k, tau = 24, 6
            tables = synth.make_tables(lpt, k, 1 << tau, d_out, tdt)
            codes = np.random.default_rng(lpt).integers(0, 1 << tau, size=(n, k)).astype(np.uint16)
            assert np.array_equal(gpu_gather(codes, tables), oracle.gather(codes, tables, acc64=False))
    finally:
        B.lookupffn_set_option("lanes_per_token", 0)
        B.lookupffn_set_option("xcd_order", 0)


LDS_SHAPES = [
    # n, k, tau, d_out, table dtype     (gather_path = 2 forces the LDS-staged kernel: tau 7 .. 10; odd k has a file of its own)
    (1003, 96, 8, 768, "f32"),       # three slices per XCD, ragged chunks
    (1003, 96, 8, 768, "bf16"),
    (16384, 32, 8, 768, "f32"),      # the benchmark's split: 11/11/10 workgroups per slice, 13 tokens per lane
    (5000, 24, 7, 200, "f32"),       # ragged last slice (50 pieces), 128-row tables
    (3000, 10, 8, 520, "bf16"),      # ragged last slice with bf16 rows
    (130, 2, 7, 4, "f32"),           # a single 16-byte piece per row
    (120000, 4, 7, 128, "f32"),      # several chunks per workgroup
    (300, 2, 7, 8192, "f32"),        # as many slice-units as workgroups
    (200, 2, 8, 16384, "bf16"),      # more slice-units than workgroups
    (1, 6, 8, 64, "f32"),            # one token
    (777, 2, 8, 64, "f32"),          # a single stage
    (777, 6, 8, 64, "bf16"),         # an odd number of stages
    (500, 10, 6, 64, "f32"),         # tau outside the staged kernel's range: falls back to the direct kernel
    (3000, 170, 9, 768, "f32"),      # tau = 9: one 512-row table per stage, 85 code words
    (1500, 2, 9, 64, "f32"),         # tau = 9, a single code word
    (1500, 4, 9, 64, "bf16"),        # tau = 9, two code words
    (9000, 6, 9, 200, "f32"),        # tau = 9, three code words, ragged last slice, several chunks
    (600, 12, 9, 72, "bf16"),
    (5000, 128, 10, 1024, "f32"),    # tau = 10: 64-byte column slices, one 1024-row table per stage
    (2500, 2, 10, 16, "f32"),        # tau = 10, a single code word, one piece per row
    (9000, 6, 10, 200, "f32"),       # tau = 10, ragged last slice (50 pieces in slices of 4)
]


@pytest.mark.parametrize("n,k,tau,d_out", [(1003, 96, 8, 768), (16384, 32, 8, 768), (3000, 170, 9, 768),
                                           (9000, 6, 9, 200), (777, 2, 8, 64), (40000, 4, 8, 72),
                                           (65536, 6, 9, 200),      # 16 token slots per lane
                                           (16384, 8, 10, 1024)])   # tau = 10 at the benchmark's split: 16 slots
def test_gather_lds_staged_kernel_64_byte_slices(n, k, tau, d_out):
    print(f"gather (LDS-staged, 4 lanes per token) n={n} k={k} tau={tau} d_out={d_out}", flush=True)
    tables = synth.make_tables(n + k, k, 1 << tau, d_out)
    codes = np.random.default_rng(n).integers(0, 1 << tau, size=(n, k)).astype(np.uint16)
    B.lookupffn_set_option("gather_path", 2)
    B.lookupffn_set_option("slice_lanes", 4)
    try:
        y = gpu_gather(codes, tables)
        assert B.lookupffn_last_gather_kernel() == "gather_lds_kernel"
    finally:
        B.lookupffn_set_option("gather_path", 0)
        B.lookupffn_set_option("slice_lanes", 0)
    assert np.array_equal(y, oracle.gather(codes, tables, acc64=False))


@pytest.mark.parametrize("n,k,tau,d_out,tdt", [(3000, 170, 9, 768, "f32"), (9000, 6, 9, 200, "f32"), (1500, 2, 9, 64, "f32")])
def test_gather_lds_staged_kernel_128_byte_slices_at_tau_9(n, k, tau, d_out, tdt):
    print(f"gather (LDS-staged, 8 lanes per token on request) n={n} k={k} tau={tau} d_out={d_out}", flush=True)
    tables = synth.make_tables(n + k, k, 1 << tau, d_out, tdt)
    codes = np.random.default_rng(n).integers(0, 1 << tau, size=(n, k)).astype(np.uint16)
    B.lookupffn_set_option("gather_path", 2)
    B.lookupffn_set_option("slice_lanes", 8)
    try:
        y = gpu_gather(codes, tables)
        assert B.lookupffn_last_gather_kernel() == "gather_lds_kernel"
    finally:
        B.lookupffn_set_option("gather_path", 0)
        B.lookupffn_set_option("slice_lanes", 0)
    assert np.array_equal(y, oracle.gather(codes, tables, acc64=False))


def test_forward_64_byte_slices_on_request():
    print("forward with the 64-byte-slice staged gather (codes re-packed from the ABI layout)", flush=True)
    w = synth.C2.with_tokens(5000)
    x, signs, tables = synth.make_layer(w)
    B.lookupffn_set_option("gather_path", 2)
    B.lookupffn_set_option("slice_lanes", 4)
    try:
        y = gpu_forward(x, signs, tables)
        assert B.lookupffn_last_gather_kernel() == "gather_lds_kernel"
    finally:
        B.lookupffn_set_option("gather_path", 0)
        B.lookupffn_set_option("slice_lanes", 0)
    assert np.array_equal(y, oracle.forward(x, signs, tables, acc64=False))


@pytest.mark.parametrize("n,k,tau,d_out,tdt", LDS_SHAPES)
def test_gather_lds_staged_kernel(n, k, tau, d_out, tdt):
    print(f"gather (LDS-staged) n={n} k={k} tau={tau} d_out={d_out} {tdt}", flush=True)
    tables = synth.make_tables(n + k, k, 1 << tau, d_out, tdt)
    codes = np.random.default_rng(n).integers(0, 1 << tau, size=(n, k)).astype(np.uint16)
    want = oracle.gather(codes, tables, acc64=False)
    B.lookupffn_set_option("gather_path", 2)
    try:
        y_lds = gpu_gather(codes, tables)
        B.lookupffn_set_option("gather_path", 1)
        y_direct = gpu_gather(codes, tables)
    finally:
        B.lookupffn_set_option("gather_path", 0)
    assert np.array_equal(y_lds, want)
    assert np.array_equal(y_direct, want)
    assert rel_err(y_lds, oracle.gather(codes, tables, acc64=True)) <= (TOL_BF16 if tdt == "bf16" else TOL_F32)


def test_gather_reduces_codes_modulo_table_size():
    print("gather out-of-range codes", flush=True)
    n, k, tau, d_out = 40, 8, 7, 16
    tables = synth.make_tables(1, k, 128, d_out)
    codes = np.random.default_rng(0).integers(0, 65536, size=(n, k)).astype(np.uint16)
    for path in (1, 2):
        B.lookupffn_set_option("gather_path", path)
        try:
            assert np.array_equal(gpu_gather(codes, tables), oracle.gather(codes & 127, tables, acc64=False))
        finally:
            B.lookupffn_set_option("gather_path", 0)


def test_gather_unaligned_code_rows_take_the_scalar_path():
    print("gather codes not 16-byte aligned", flush=True)
    n, k, tau, d_out = 100, 16, 5, 64
    tables = synth.make_tables(2, k, 32, d_out)
    codes = np.random.default_rng(1).integers(0, 32, size=(n, k)).astype(np.uint16)
    buf = torch.zeros(n * k + 1, dtype=torch.int16, device="cuda")
    view = buf[1:].view(n, k)
    view.copy_(torch.from_numpy(codes.view(np.int16)))
    y = B.lookupffn_gather(view, B.to_device(tables))
    torch.cuda.synchronize()
    assert np.array_equal(y.cpu().numpy(), oracle.gather(codes, tables, acc64=False))


# ------------------------------------------------------------------ whole forward pass

def check_forward(w, x, signs, tables, sample=None):
    tol = TOL_BF16 if w.table_dtype == "bf16" else TOL_F32
    xd, sd, td = B.to_device(x), B.to_device(signs), B.to_device(tables)
    codes = B.lookupffn_hash(xd, sd, w.k, w.tau)
    y = B.lookupffn_forward(xd, sd, td)
    torch.cuda.synchronize()
    codes, y = B.codes_to_numpy(codes), y.cpu().numpy()
    assert_codes_equal(codes, oracle.hash_codes(x, signs, w.k, w.tau))
    idx = np.arange(x.shape[0]) if sample is None else sample
    ref64, ref_codes = oracle.forward(x[idx], signs, tables, acc64=True, return_codes=True)
    assert_codes_equal(codes[idx], ref_codes)
    err = rel_err(y[idx], ref64)
    print(f"  {w.name}: max|dy|/rms = {err:.3e} on {len(idx)} tokens", flush=True)
    assert err <= tol
    assert np.array_equal(y[idx], oracle.forward(x[idx], signs, tables, acc64=False))
    return y


def test_forward_config1_tiny():
    print("forward C1", flush=True)
    w = synth.C1
    x, signs, tables = synth.make_layer(w)
    y = check_forward(w, x, signs, tables)
    # a caller-provided workspace gives the same result as the library-owned one, run to run
    ws = torch.empty(B.lookupffn_workspace_bytes(w.n_tokens, w.k), dtype=torch.uint8, device="cuda")
    assert np.array_equal(gpu_forward(x, signs, tables, workspace=ws), y)
    assert np.array_equal(gpu_forward(x, signs, tables), y)


def test_forward_config2_full_size():
    print("forward C2 (16384 tokens, fp32)", flush=True)
    w = synth.C2
    x, signs, tables = synth.make_layer(w)
    check_forward(w, x, signs, tables)


def test_forward_config3_full_size_bf16():
    print("forward C3 (65536 tokens, bf16)", flush=True)
    w = synth.C3
    x, signs, tables = synth.make_layer(w)
    check_forward(w, x, signs, tables, sample=sample_tokens(w.n_tokens, 7))


def test_forward_bf16_tables_prepared_once_take_the_staged_gather():
    """bf16 tables: the staged gather reads fp32 rows, so it runs on the copy lookupffn_prepare_tables makes
    once; the raw bf16 tables take the direct gather.  Same bits either way."""
    print("forward bf16 tables, 16384 tokens: raw tables (direct gather) and prepared tables (staged gather)", flush=True)
    w = synth.C3.with_tokens(16384)
    x, signs, tables = synth.make_layer(w)
    xd, sd, td = B.to_device(x), B.to_device(signs), B.to_device(tables)
    prep = B.lookupffn_prepare_tables(td)
    assert prep.buf.numel() == w.k * w.rows * w.d_out * 4 == B.lookupffn_prepared_tables_bytes(w.k, w.tau, w.d_out, "bf16")
    sel = sample_tokens(w.n_tokens, 17)
    want = oracle.forward(x[sel], signs, tables, acc64=False)
    ws = torch.empty(B.lookupffn_workspace_bytes(w.n_tokens, w.k), dtype=torch.uint8, device="cuda")
    for tab, work, kernel in ((prep, ws, "gather_lds_kernel"), (td, ws, "gather_kernel"), (prep, None, "gather_lds_kernel")):
        y = B.lookupffn_forward(xd, sd, tab, workspace=work)
        torch.cuda.synchronize()
        assert B.lookupffn_last_gather_kernel() == kernel
        assert np.array_equal(y.cpu().numpy()[sel], want)
    yw = B.lookupffn_forward_weighted(xd, sd, prep)
    torch.cuda.synchronize()
    assert B.lookupffn_last_gather_kernel() == "gather_lds_kernel"
    ref = oracle.forward_weighted(x[sel], signs, tables)
    assert rel_err(yw.cpu().numpy()[sel], ref) <= TOL_BF16
    # a small batch does not repay staging: direct gather, reading the prepared copy
    small = B.lookupffn_forward(xd[:2000], sd, prep)
    torch.cuda.synchronize()
    assert B.lookupffn_last_gather_kernel() == "gather_kernel"
    sel_small = sel[sel < 2000]
    assert np.array_equal(small.cpu().numpy()[sel_small], want[:len(sel_small)])


PREPARED_SHAPES = [
    # n, k, tau, d_out, table dtype
    (3000, 96, 8, 768, "f32"),       # 128-byte pieces, no padding
    (3000, 10, 8, 520, "bf16"),      # ragged last piece (2080-byte fp32 rows: 16.25 pieces)
    (5000, 24, 7, 200, "f32"),       # tau = 7, ragged
    (130, 2, 7, 4, "f32"),           # one 16-byte piece per row in a 128-byte piece
    (9000, 6, 9, 200, "f32"),        # tau = 9: 64-byte pieces, ragged
    (3000, 170, 9, 768, "bf16"),
    (5000, 128, 10, 1024, "f32"),    # tau = 10
    (2500, 2, 10, 16, "f32"),
    (500, 10, 6, 64, "f32"),         # tau outside the staged kernel's range: the direct kernel reads the copy
    (300, 7, 11, 72, "bf16"),        # odd k, tau = 11, 64-byte pieces
    (40, 3, 1, 8, "bf16"),           # two-row tables
]


@pytest.mark.parametrize("n,k,tau,d_out,tdt", PREPARED_SHAPES)
def test_gather_prepared_tables_equal_row_major_tables(n, k, tau, d_out, tdt):
    print(f"gather with prepared tables n={n} k={k} tau={tau} d_out={d_out} {tdt}", flush=True)
    tables = synth.make_tables(n + k + 1, k, 1 << tau, d_out, tdt)
    codes = np.random.default_rng(n + 1).integers(0, 1 << tau, size=(n, k)).astype(np.uint16)
    want = oracle.gather(codes, tables, acc64=False)
    td = B.to_device(tables)
    prep = B.lookupffn_prepare_tables(td)
    assert prep.buf.numel() == B.lookupffn_prepared_tables_bytes(k, tau, d_out, tdt)
    cd = torch.from_numpy(codes.view(np.int16)).cuda()
    ws = torch.empty(max(B.lookupffn_workspace_bytes_gather(n, k), 256), dtype=torch.uint8, device="cuda")
    try:
        for path in (2, 4, 1):
            B.lookupffn_set_option("gather_path", path)
            for lanes in ((0, 4, 8) if path == 2 else (0,)):
                B.lookupffn_set_option("slice_lanes", lanes)
                y = B.lookupffn_gather(cd, prep, workspace=ws)
                torch.cuda.synchronize()
                assert np.array_equal(y.cpu().numpy(), want), f"path {path}, slice_lanes {lanes}"
        for lpt in (1, 2, 4, 8, 16):           # the direct kernel's lane widths, clamped to the prepared piece
            B.lookupffn_set_option("gather_path", 1)
            B.lookupffn_set_option("lanes_per_token", lpt)
            y = B.lookupffn_gather(cd, prep)
            torch.cuda.synchronize()
            assert np.array_equal(y.cpu().numpy(), want), f"direct, lanes_per_token {lpt}"
    finally:
        B.lookupffn_set_option("gather_path", 0)
        B.lookupffn_set_option("slice_lanes", 0)
        B.lookupffn_set_option("lanes_per_token", 0)


RING_SHAPES = [
    # n, k, tau, d_out, table dtype   (prepared tables, plain sum, tau 7 or 8: the lagged, bank-interleaved staged gather)
    (16384, 96, 8, 768, "f32"),      # the benchmark's shape: 12 token slots, one chunk per workgroup
    (6144, 96, 8, 768, "bf16"),
    (1003, 96, 8, 768, "f32"),       # ragged token count, 4 slots
    (1, 6, 8, 64, "f32"),            # one token
    (777, 2, 8, 64, "f32"),          # fewer tables than the pipeline is deep
    (777, 1, 8, 64, "f32"),
    (777, 3, 8, 64, "bf16"),         # odd k
    (2000, 5, 8, 72, "f32"),         # odd k, ragged last slice (18 pieces in slices of 4)
    (3000, 13, 8, 520, "bf16"),
    (5000, 24, 7, 200, "f32"),       # tau = 7: half-filled ring slices
    (130, 2, 7, 4, "f32"),           # a single 16-byte piece per row
    (120000, 4, 8, 128, "f32"),      # several chunks per workgroup
    (300, 2, 8, 8192, "f32"),        # more slice-units than workgroups
    (40000, 17, 8, 72, "f32"),       # 16 slots, odd k
    (32768, 128, 8, 512, "f32"),     # the paper's small-model shape
    (9000, 200, 8, 64, "f32"),       # many tables
]


@pytest.mark.parametrize("n,k,tau,d_out,tdt", RING_SHAPES)
def test_gather_ring_kernel(n, k, tau, d_out, tdt):
    print(f"gather (lagged ring) n={n} k={k} tau={tau} d_out={d_out} {tdt}", flush=True)
    tables = synth.make_tables(n + 3 * k, k, 1 << tau, d_out, tdt)
    codes = np.random.default_rng(n + k).integers(0, 1 << tau, size=(n, k)).astype(np.uint16)
    want = oracle.gather(codes, tables, acc64=False)
    prep = B.lookupffn_prepare_tables(B.to_device(tables))
    cd = torch.from_numpy(codes.view(np.int16)).cuda()
    try:
        for slots, threads in ((0, 0), (4, 1024), (8, 0), (13, 1024), (14, 1024), (16, 512), (32, 512)):
            B.lookupffn_set_option("gather_path", 4)
            B.lookupffn_set_option("token_slots", slots)
            B.lookupffn_set_option("ring_threads", threads)
            y = torch.full((n, d_out), float("nan"), dtype=torch.float32, device="cuda")
            B.lookupffn_gather(cd, prep, y=y)
            torch.cuda.synchronize()
            assert B.lookupffn_last_gather_kernel() == "gather_ring_kernel"
            assert np.array_equal(y.cpu().numpy(), want), f"token_slots {slots}, ring_threads {threads}"
    finally:
        B.lookupffn_set_option("gather_path", 0)
        B.lookupffn_set_option("token_slots", 0)
        B.lookupffn_set_option("ring_threads", 0)
    assert rel_err(want, oracle.gather(codes, tables, acc64=True)) <= (TOL_BF16 if tdt == "bf16" else TOL_F32)


def test_prepared_tables_in_every_variant():
    print("prepared tables: plain / weighted / multi-probe / BH forward equal the row-major results", flush=True)
    w = synth.C2.with_tokens(3000)
    x, signs, tables = synth.make_layer(w)
    xd, sd, td = B.to_device(x), B.to_device(signs), B.to_device(tables)
    prep = B.lookupffn_prepare_tables(td)
    bm = synth.make_bmats(9, w.n_proj, 4, w.d_pad, 32)
    bd = torch.from_numpy(bm).cuda()
    pbh = B.lookupffn_prepare_bh(bd, w.d, w.k, w.tau)
    for name, fwd, par, ppar in (("plain", B.lookupffn_forward, sd, sd), ("weighted", B.lookupffn_forward_weighted, sd, sd),
                                 ("probes", B.lookupffn_forward_probes, sd, sd), ("bh", B.lookupffn_forward_bh, bd, pbh),
                                 ("bh weighted", B.lookupffn_forward_bh_weighted, bd, pbh)):
        for path in (2, 1):
            B.lookupffn_set_option("gather_path", path)
            try:
                a = fwd(xd, par, td)
                b = fwd(xd, ppar, prep)
                torch.cuda.synchronize()
            finally:
                B.lookupffn_set_option("gather_path", 0)
            assert torch.equal(a, b), f"{name}, gather_path {path}"
    # the stand-alone BH hashes with prepared factors
    assert torch.equal(B.lookupffn_hash_bh(xd, bd, w.k, w.tau), B.lookupffn_hash_bh(xd, pbh, w.k, w.tau))
    c1, w1 = B.lookupffn_hash_bh_weighted(xd, bd, w.k, w.tau)
    c2, w2 = B.lookupffn_hash_bh_weighted(xd, pbh, w.k, w.tau)
    assert torch.equal(c1, c2) and torch.equal(w1, w2)
    assert np.array_equal(B.codes_to_numpy(c1), oracle.bh_hash_codes(x, bm, w.k, w.tau))


def test_forward_config4_full_size():
    print("forward C4 (16384 tokens, tau=10, 512 MB of tables)", flush=True)
    w = synth.C4
    x, signs, tables = synth.make_layer(w)
    check_forward(w, x, signs, tables, sample=sample_tokens(w.n_tokens, 5))


@pytest.mark.parametrize("w", [synth.P6, synth.P7, synth.P8], ids=lambda w: w.name)
def test_forward_paper_shapes_full_size(w):
    print(f"forward {w.name} ({w.n_tokens} tokens, d={w.d}, h={w.k}, tau={w.tau})", flush=True)
    x, signs, tables = synth.make_layer(w)
    check_forward(w, x, signs, tables, sample=sample_tokens(w.n_tokens, 7))


def test_forward_config5_stacked_layers():
    print("forward C5 (8 tokens x 12 layers)", flush=True)
    w = synth.C5
    layers = [synth.make_layer(w, layer=l, with_x=(l == 0)) for l in range(w.n_layers)]
    x0 = layers[0][0]
    dev = [(B.to_device(s), B.to_device(t)) for _, s, t in layers]
    # teacher-forced: every GPU layer is fed the oracle's input of that layer
    h = x0
    for l, (_, signs, tables) in enumerate(layers):
        y_ref, c_ref = oracle.forward(h, signs, tables, acc64=True, return_codes=True)
        hd = B.to_device(h)
        codes = B.codes_to_numpy(B.lookupffn_hash(hd, dev[l][0], w.k, w.tau))
        y = B.lookupffn_forward(hd, dev[l][0], dev[l][1]).cpu().numpy()
        assert_codes_equal(codes, c_ref)
        assert rel_err(y, y_ref) <= TOL_F32
        h = oracle.forward(h, signs, tables, acc64=False)
    # free-running chain on the GPU against the oracle's fp32-sequential chain: identical bits
    g = B.to_device(x0)
    for l in range(w.n_layers):
        g = B.lookupffn_forward(g, dev[l][0], dev[l][1])
    torch.cuda.synchronize()
    assert np.array_equal(g.cpu().numpy(), h)


def test_forward_with_more_than_4_gib_of_activations():
    """1.5 M tokens: x and y are 4.8 GB each, so token offsets pass 2^32 bytes in every kernel.  The batch
    is a 65536-token block repeated 24 times on the device: every repetition of y must equal the first,
    and sampled rows (the last ones included) must match the oracle."""
    w = synth.C2
    reps, block = 24, 65536
    n = reps * block
    print(f"forward with {n} tokens ({n * w.d_out * 4 / 2**30:.2f} GiB of y)", flush=True)
    x, signs, tables = synth.make_layer(w, n_tokens=block)
    xd = B.to_device(x).repeat(reps, 1)
    sd, td = B.to_device(signs), B.to_device(tables)
    assert xd.shape == (n, w.d) and xd.numel() * 4 > 2**32
    idx = np.unique(np.concatenate([np.arange(0, n, 9973), np.arange(n - 300, n)]))
    want = oracle.forward(x[idx % block], signs, tables, acc64=False)
    bm = synth.make_bmats(77, w.n_proj, 4, w.d_pad, 16)
    bd = torch.from_numpy(bm).cuda()
    results = {}
    try:
        for name, path, fwd, par in (("staged", 2, B.lookupffn_forward, sd), ("direct", 1, B.lookupffn_forward, sd),
                                     ("weighted staged", 2, B.lookupffn_forward_weighted, sd),
                                     ("multi-probe staged", 2, B.lookupffn_forward_probes, sd),
                                     ("bh staged", 2, B.lookupffn_forward_bh, bd),
                                     ("bh weighted direct", 1, B.lookupffn_forward_bh_weighted, bd)):
            print(f"  {name}", flush=True)
            B.lookupffn_set_option("gather_path", path)
            y = torch.full((n, w.d_out), float("nan"), dtype=torch.float32, device="cuda")
            fwd(xd, par, td, y=y)
            torch.cuda.synchronize()
            yb = y.view(reps, block, w.d_out)
            assert bool((yb == yb[0]).all()), f"{name}: a repetition of the block differs from the first"
            results[name] = y[torch.from_numpy(idx).cuda()].cpu().numpy()
            del y, yb
    finally:
        B.lookupffn_set_option("gather_path", 0)
    assert np.array_equal(results["staged"], want) and np.array_equal(results["direct"], want)
    xs = x[idx % block]
    assert rel_err(results["weighted staged"], oracle.forward_weighted(xs, signs, tables)) <= TOL_F32
    assert rel_err(results["multi-probe staged"], oracle.forward_probes(xs, signs, tables)) <= TOL_F32
    assert np.array_equal(results["bh staged"], oracle.bh_forward(xs, bm, tables, acc64=False))
    assert rel_err(results["bh weighted direct"], oracle.bh_forward_weighted(xs, bm, tables)) <= TOL_F32


def test_forward_is_deterministic_and_stream_ordered():
    print("forward determinism / side stream", flush=True)
    w = synth.C2.with_tokens(2000)
    x, signs, tables = synth.make_layer(w, n_tokens=2000)
    xd, sd, td = B.to_device(x), B.to_device(signs), B.to_device(tables)
    a = B.lookupffn_forward(xd, sd, td)
    s = torch.cuda.Stream()
    s.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(s):
        b = B.lookupffn_forward(xd, sd, td)
    s.synchronize()
    torch.cuda.synchronize()
    assert torch.equal(a, b)


def test_empty_batch_and_timing_counters():
    print("empty batch / timing", flush=True)
    w = synth.C1
    x, signs, tables = synth.make_layer(w)
    xd, sd, td = B.to_device(x), B.to_device(signs), B.to_device(tables)
    y = B.lookupffn_forward(xd[:0], sd, td)
    assert y.shape == (0, w.d_out)
    B.lookupffn_timing_reset()
    B.lookupffn_timing_enable(True)
    try:
        for _ in range(3):
            B.lookupffn_forward(xd, sd, td)
        (h_ms, h_n), (g_ms, g_n) = B.lookupffn_timing_read(0), B.lookupffn_timing_read(1)
    finally:
        B.lookupffn_timing_enable(0)
        B.lookupffn_timing_reset()
    assert h_n == 3 and g_n == 3 and h_ms > 0 and g_ms > 0
