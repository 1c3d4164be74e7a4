"""GPU parity with IEEE half (float16) inputs and tables, every entry point: the 16-bit types are storage
formats only, so the bars are those of the fp32 path -- codes bit-exact, plain sums equal to the oracle's fp32
sequential sum bit for bit and within 1e-2 (the 16-bit row of the tolerance) of its fp64 sum."""
import numpy as np
import pytest
import torch

import oracle
from paper_2403_07221_amd import binding as B
from paper_2403_07221_amd import synth

pytestmark = pytest.mark.gpu
TOL_16 = 1e-2


@pytest.fixture(scope="module", autouse=True)
def _gpu():
    assert torch.cuda.is_available(), "these tests need the MI355X"
    B.lib()
    yield
    B.lookupffn_set_option("gather_path", 0)
    B.lookupffn_set_option("small_tokens", 0)


def rel_err(y, ref):
    ref64 = ref.astype(np.float64)
    return float(np.max(np.abs(y.astype(np.float64) - ref64)) / np.sqrt(np.mean(ref64 ** 2)))


def make(seed, n, d, k, tau, R, d_out, xdt="f16", tdt="f16"):
    w = synth.Workload("t", 7, n, d, R, k, tau, d_out, x_dtype=xdt, table_dtype=tdt)
    x = synth.make_x(seed, n, d, xdt)
    signs = synth.make_signs(seed + 1, w.n_proj, R, w.d_pad)
    tables = synth.make_tables(seed + 2, k, 1 << tau, d_out, tdt)
    return w, x, signs, tables


HASH_SHAPES = [
    (517, 768, 96, 8, 3),      # the two-layout kernel, vector row loads
    (37, 999, 30, 7, 3),       # d % 4 != 0: element-wise row loads
    (129, 48, 6, 8, 3),        # the generic kernel, padded width
    (77, 768, 170, 9, 3),      # two projections
    (33, 4096, 300, 11, 1),    # the widest transform
]


@pytest.mark.parametrize("n,d,k,tau,R", HASH_SHAPES)
def test_hash_of_half_input_is_bit_exact(n, d, k, tau, R):
    print(f"hash f16 n={n} d={d} k={k} tau={tau} R={R}", flush=True)
    w, x, signs, _ = make(n + d, n, d, k, tau, R, 8)
    assert x.dtype == np.float16
    codes = B.codes_to_numpy(B.lookupffn_hash(B.to_device(x), B.to_device(signs), k, tau))
    assert np.array_equal(codes, oracle.hash_codes(x, signs, k, tau))


GATHER_SHAPES = [
    # n, k, tau, d_out
    (1003, 96, 8, 768),
    (77, 13, 3, 40),           # narrow rows, odd k
    (300, 170, 9, 768),
    (259, 6, 8, 776),          # ragged last slice
]


@pytest.mark.parametrize("n,k,tau,d_out", GATHER_SHAPES)
def test_gather_of_half_tables_direct_and_prepared(n, k, tau, d_out):
    print(f"gather f16 n={n} k={k} tau={tau} d_out={d_out}", flush=True)
    tables = synth.make_tables(n + k, k, 1 << tau, d_out, "f16")
    codes = np.random.default_rng(n).integers(0, 1 << tau, size=(n, k), dtype=np.uint16)
    cd, td = torch.from_numpy(codes.view(np.int16)).cuda(), B.to_device(tables)
    assert td.dtype == torch.float16
    want = oracle.gather(codes, tables, acc64=False)
    prep = B.lookupffn_prepare_tables(td)
    assert prep.buf.numel() == B.lookupffn_prepared_tables_bytes(k, tau, d_out, "f16")
    try:
        for path, tabs, kernel in ((1, td, "gather_kernel"), (1, prep, "gather_kernel"), (2, prep, None)):
            B.lookupffn_set_option("gather_path", path)
            y = B.lookupffn_gather(cd, tabs).cpu().numpy()
            if kernel:
                assert B.lookupffn_last_gather_kernel() == kernel
            assert np.array_equal(y, want), (path, type(tabs).__name__)
    finally:
        B.lookupffn_set_option("gather_path", 0)
    assert rel_err(want, oracle.gather(codes, tables, acc64=True)) <= TOL_16


def test_forward_variants_with_half_input_and_tables():
    print("forward f16: plain, weighted, multi-probe, BH4, BH4 weighted", flush=True)
    w, x, signs, tables = make(91, 3000, 768, 96, 8, 3, 768)
    xd, sd, td = B.to_device(x), B.to_device(signs), B.to_device(tables)
    prep = B.lookupffn_prepare_tables(td)
    want = oracle.forward(x, signs, tables, acc64=False)
    for tabs in (td, prep):
        y = B.lookupffn_forward(xd, sd, tabs).cpu().numpy()
        assert np.array_equal(y, want)
    try:
        B.lookupffn_set_option("gather_path", 2)                        # prepared tables: the staged kernel
        y = B.lookupffn_forward(xd, sd, prep).cpu().numpy()
        assert B.lookupffn_last_gather_kernel() == "gather_lds_kernel" and np.array_equal(y, want)
    finally:
        B.lookupffn_set_option("gather_path", 0)
    assert rel_err(want, oracle.forward(x, signs, tables, acc64=True)) <= TOL_16
    for tabs in (td, prep):
        yw = B.lookupffn_forward_weighted(xd, sd, tabs).cpu().numpy()
        assert rel_err(yw, oracle.forward_weighted(x, signs, tables)) <= 1e-4
        yp = B.lookupffn_forward_probes(xd, sd, tabs).cpu().numpy()
        assert rel_err(yp, oracle.forward_probes(x, signs, tables)) <= 1e-4
    bm = synth.make_bmats(77, w.n_proj, 4, w.d_pad, 16)
    bd = torch.from_numpy(bm).cuda()
    yb = B.lookupffn_forward_bh(xd, bd, prep).cpu().numpy()
    assert np.array_equal(yb, oracle.bh_forward(x, bm, tables, acc64=False))
    ybw = B.lookupffn_forward_bh_weighted(xd, bd, td).cpu().numpy()
    assert rel_err(ybw, oracle.bh_forward_weighted(x, bm, tables)) <= 1e-4


def test_mixed_storage_types():
    """x and the tables need not share a storage type."""
    for xdt, tdt in (("f16", "bf16"), ("bf16", "f16"), ("f32", "f16"), ("f16", "f32")):
        print(f"forward x={xdt} tables={tdt}", flush=True)
        w, x, signs, tables = make(17, 200, 600, 40, 9, 2, 600, xdt, tdt)
        y = B.lookupffn_forward(B.to_device(x), B.to_device(signs), B.to_device(tables)).cpu().numpy()
        assert np.array_equal(y, oracle.forward(x, signs, tables, acc64=False))


def test_single_launch_path_with_half_storage():
    print("stack f16", flush=True)
    n, d, k, tau, R, layers = 9, 768, 96, 8, 3, 3
    x = synth.make_x(5, n, d, "f16")
    signs = [synth.make_signs(10 + l, 1, R, 1024) for l in range(layers)]
    tables = [synth.make_tables(20 + l, k, 1 << tau, d, "f16", sigma=1.0 / np.sqrt(k)) for l in range(layers)]
    h = x
    for s, t in zip(signs, tables):
        h = oracle.forward(h, s, t, acc64=False)
    y = B.lookupffn_forward_stack(B.to_device(x), [B.to_device(s) for s in signs], [B.to_device(t) for t in tables])
    assert B.lookupffn_last_gather_kernel() == "forward_stack_kernel"
    assert np.array_equal(y.cpu().numpy(), h)
    y1 = B.lookupffn_forward(B.to_device(x), B.to_device(signs[0]), B.to_device(tables[0]))   # 9 tokens: the same kernel
    assert B.lookupffn_last_gather_kernel() == "forward_stack_kernel"
    assert np.array_equal(y1.cpu().numpy(), oracle.forward(x, signs[0], tables[0], acc64=False))


# ------------------------------------------------------------------ outputs stored in 16 bits

def y16_bits(y: torch.Tensor) -> np.ndarray:
    return y.view(torch.int16).cpu().numpy().view(np.uint16)


def close16(y: torch.Tensor, ref: np.ndarray, tol32: float) -> bool:
    """y (16-bit storage) against a reference: the fp32 tolerance (relative to the rms) plus one rounding to
    y's type per element (half an ulp: 2^-9 relative for bf16, 2^-12 for half; twice that is allowed)."""
    rel = 2.0 ** -8 if y.dtype == torch.bfloat16 else 2.0 ** -11
    got = y.float().cpu().numpy().astype(np.float64)
    r = ref.astype(np.float64)
    return bool(np.all(np.abs(got - r) <= rel * np.abs(r) + tol32 * np.sqrt(np.mean(r ** 2))))


def expect16(y32: np.ndarray, dtype) -> np.ndarray:
    return oracle.float_to_bf16(y32) if dtype == torch.bfloat16 else oracle.float_to_half(y32)


@pytest.mark.parametrize("ydt", [torch.bfloat16, torch.float16])
def test_outputs_stored_in_16_bits_are_the_rounded_fp32_sums(ydt):
    """Every gather kernel and entry point: y in bf16 / half holds exactly the oracle's fp32 sequential sums
    rounded once to nearest even; against the fp64 sums that is the fp32 tolerance plus one rounding to y's type."""
    print(f"y stored as {ydt}", flush=True)
    w = synth.C2.with_tokens(3000)
    x, signs, tables = synth.make_layer(w)
    xd, sd, td = B.to_device(x), B.to_device(signs), B.to_device(tables)
    prep = B.lookupffn_prepare_tables(td)
    y32, codes = oracle.forward(x, signs, tables, acc64=False, return_codes=True)
    want = expect16(y32, ydt)
    cd = torch.from_numpy(codes.view(np.int16)).cuda()
    try:
        for path, tabs, kernel in ((1, td, "gather_kernel"), (2, prep, "gather_lds_kernel"), (4, prep, "gather_ring_kernel")):
            B.lookupffn_set_option("gather_path", path)
            y = torch.empty((w.n_tokens, w.d_out), dtype=ydt, device="cuda")
            B.lookupffn_gather(cd, tabs, y=y)
            assert B.lookupffn_last_gather_kernel() == kernel
            assert np.array_equal(y16_bits(y), want), kernel
            y.zero_()
            B.lookupffn_forward(xd, sd, tabs, y=y)
            assert np.array_equal(y16_bits(y), want), ("forward", kernel)
    finally:
        B.lookupffn_set_option("gather_path", 0)
    ref64 = oracle.forward(x, signs, tables, acc64=True)
    assert close16(y, ref64, 1e-4)
    # weighted and multi-probe: within tolerance of the fp64 oracle (their fp32 values are not pinned bit for bit)
    yw = torch.empty((w.n_tokens, w.d_out), dtype=ydt, device="cuda")
    B.lookupffn_forward_weighted(xd, sd, prep, y=yw)
    assert close16(yw, oracle.forward_weighted(x, signs, tables), 1e-4)
    B.lookupffn_forward_probes(xd, sd, prep, y=yw)
    assert close16(yw, oracle.forward_probes(x, signs, tables), 1e-4)
    # bf16 rows in, 16-bit rows out, through the direct kernel's 8-element pieces
    t16 = synth.make_tables(5, w.k, w.rows, w.d_out, "bf16")
    y = torch.empty((200, w.d_out), dtype=ydt, device="cuda")
    B.lookupffn_gather(cd[:200].contiguous(), B.to_device(t16), y=y)
    assert np.array_equal(y16_bits(y), expect16(oracle.gather(codes[:200], t16, acc64=False), ydt))
    # the single launch: a few tokens, and a chain (only the last layer's output is rounded)
    y8 = torch.empty((8, w.d_out), dtype=ydt, device="cuda")
    B.lookupffn_forward(xd[:8].contiguous(), sd, td, y=y8)
    assert B.lookupffn_last_gather_kernel() == "forward_stack_kernel"
    assert np.array_equal(y16_bits(y8), want[:8])
    chain = [synth.make_layer(synth.C5, layer=l, with_x=False) for l in range(3)]
    h = x[:8]
    for _, s_, t_ in chain:
        h = oracle.forward(h, s_, t_, acc64=False)
    B.lookupffn_forward_stack(xd[:8].contiguous(), [B.to_device(s_) for _, s_, _ in chain],
                              [B.to_device(t_) for _, _, t_ in chain], y=y8)
    assert np.array_equal(y16_bits(y8), expect16(h, ydt))
