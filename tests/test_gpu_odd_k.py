"""GPU parity for an odd number of tables on the LDS-staged gather.

The staged kernel takes its tables in pairs (two codes per packed word).  With an odd k it sums the first
k - 1 tables and the direct kernel adds the last one onto those fp32 sums, so the order of the additions
is still the table order: the plain sum must equal the oracle's fp32 sequential mode bit for bit, the
weighted sum must equal the direct kernel's, and the multi-probe sum meets its tolerance (Sec. 3,
eq. lookup; Sec. 4's weighted form; eq. partial_softmax).
"""
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
    B.lookupffn_set_option("gather_path", 0)
    B.lookupffn_set_option("slice_lanes", 0)


def rel_err(y, ref):
    ref64 = ref.astype(np.float64)
    return float(np.max(np.abs(y.astype(np.float64) - ref64)) / np.sqrt(np.mean(ref64 ** 2)))


ODD_SHAPES = [
    # n, k, tau, d_out, table dtype
    (1003, 97, 8, 768, "f32"),       # the benchmark's layer with one more table
    (16384, 33, 8, 768, "f32"),      # 13 token slots per lane
    (5000, 25, 7, 200, "f32"),       # ragged last slice, 128-row tables
    (777, 3, 8, 64, "f32"),          # a single stage and the added table
    (3000, 171, 9, 768, "f32"),      # tau = 9: 64-byte slices (codes re-packed with the other scale)
    (9000, 7, 10, 200, "f32"),       # tau = 10, ragged last slice
    (3000, 11, 8, 520, "bf16"),      # 16-bit rows: staged once prepared
    (1, 5, 8, 64, "f32"),            # one token
]


@pytest.mark.parametrize("n,k,tau,d_out,tdt", ODD_SHAPES)
def test_gather_odd_k_staged_plus_last_table(n, k, tau, d_out, tdt):
    print(f"gather, odd k, staged + last table: n={n} k={k} tau={tau} d_out={d_out} {tdt}", flush=True)
    tables = synth.make_tables(n + k, k, 1 << tau, d_out, tdt)
    codes = np.random.default_rng(n + 7 * k).integers(0, 1 << tau, size=(n, k)).astype(np.uint16)
    want = oracle.gather(codes, tables, acc64=False)
    cd, td = torch.from_numpy(codes.view(np.int16)).cuda(), B.to_device(tables)
    prep = B.lookupffn_prepare_tables(td)
    B.lookupffn_set_option("gather_path", 2)
    try:
        for name, tb in (("row-major", td), ("prepared", prep)):
            if name == "row-major" and tdt != "f32":
                continue                      # 16-bit row-major tables take the direct kernel
            y = B.lookupffn_gather(cd, tb)
            torch.cuda.synchronize()
            assert B.lookupffn_last_gather_kernel() == "gather_lds_kernel", name
            assert np.array_equal(y.cpu().numpy(), want), name
    finally:
        B.lookupffn_set_option("gather_path", 0)


def test_gather_odd_k_code_rows_at_odd_halfword_offsets():
    print("gather, odd k: code rows start at 2-byte offsets that are not multiples of 4", flush=True)
    n, k, tau, d_out = 2000, 9, 8, 136
    tables = synth.make_tables(5, k, 1 << tau, d_out)
    codes = np.random.default_rng(3).integers(0, 65536, size=(n, k)).astype(np.uint16)   # also out of range
    want = oracle.gather(codes & 255, tables, acc64=False)
    B.lookupffn_set_option("gather_path", 2)
    try:
        y = B.lookupffn_gather(torch.from_numpy(codes.view(np.int16)).cuda(), B.to_device(tables))
        torch.cuda.synchronize()
        assert B.lookupffn_last_gather_kernel() == "gather_lds_kernel"
    finally:
        B.lookupffn_set_option("gather_path", 0)
    assert np.array_equal(y.cpu().numpy(), want)


@pytest.mark.parametrize("n,k,tau,d_out", [(1003, 97, 8, 768), (5000, 25, 7, 200), (3000, 21, 9, 768), (5000, 7, 10, 256)])
def test_gather_weighted_and_probes_odd_k(n, k, tau, d_out):
    print(f"weighted and multi-probe gather, odd k: n={n} k={k} tau={tau} d_out={d_out}", flush=True)
    rng = np.random.default_rng(n + k)
    tables = synth.make_tables(n + k, k, 1 << tau, d_out)
    codes = rng.integers(0, 1 << tau, size=(n, k)).astype(np.uint16)
    wts = rng.uniform(0.0, 4.0, size=(n, k)).astype(np.float32)
    p = rng.uniform(0.0, 1.0, size=(n, k, tau + 1)).astype(np.float32)
    cd, td = torch.from_numpy(codes.view(np.int16)).cuda(), B.to_device(tables)
    wd, pd = torch.from_numpy(wts).cuda(), torch.from_numpy(p).cuda()
    out = {}
    try:
        for path in (2, 1):
            B.lookupffn_set_option("gather_path", path)
            kernel = "gather_lds_kernel" if path == 2 else "gather_kernel"
            out["w", path] = B.lookupffn_gather_weighted(cd, wd, td)
            torch.cuda.synchronize()
            assert B.lookupffn_last_gather_kernel() == kernel
            out["p", path] = B.lookupffn_gather_probes(cd, pd, td)
            torch.cuda.synchronize()
            assert B.lookupffn_last_gather_kernel() == kernel
    finally:
        B.lookupffn_set_option("gather_path", 0)
    out = {key: v.cpu().numpy() for key, v in out.items()}
    assert np.array_equal(out["w", 2], out["w", 1])       # the same fused multiply-adds in the same order
    assert rel_err(out["w", 2], oracle.gather_weighted(codes, wts.astype(np.float64), tables)) <= 1e-4
    want = oracle.gather_probes(codes, p.astype(np.float64), tables)
    assert rel_err(out["p", 2], want) <= 1e-4
    assert rel_err(out["p", 1], want) <= 1e-4


def test_forward_odd_k_every_variant():
    print("forward, odd k (k = 95): plain, weighted, multi-probe; 16-bit outputs stay on the direct kernel", flush=True)
    w = synth.Workload("odd", 7, 6000, 768, 3, 95, 8, 768)
    x, signs, tables = synth.make_layer(w)
    xd, sd, td = B.to_device(x), B.to_device(signs), B.to_device(tables)
    prep = B.lookupffn_prepare_tables(td)
    try:
        B.lookupffn_set_option("gather_path", 2)
        for tb in (td, prep):
            y = B.lookupffn_forward(xd, sd, tb)
            torch.cuda.synchronize()
            assert B.lookupffn_last_gather_kernel() == "gather_lds_kernel"
            assert np.array_equal(y.cpu().numpy(), oracle.forward(x, signs, tables, acc64=False))
        yw = B.lookupffn_forward_weighted(xd, sd, prep)
        torch.cuda.synchronize()
        assert B.lookupffn_last_gather_kernel() == "gather_lds_kernel"
        assert rel_err(yw.cpu().numpy(), oracle.forward_weighted(x, signs, tables)) <= 1e-4
        yp = B.lookupffn_forward_probes(xd, sd, prep)
        torch.cuda.synchronize()
        assert B.lookupffn_last_gather_kernel() == "gather_lds_kernel"
        assert rel_err(yp.cpu().numpy(), oracle.forward_probes(x, signs, tables)) <= 1e-4
        # a 16-bit y is rounded once from the complete sum: no second pass over it
        y16 = torch.empty(w.n_tokens, w.d_out, dtype=torch.bfloat16, device="cuda")
        B.lookupffn_forward(xd, sd, prep, y=y16)
        torch.cuda.synchronize()
        assert B.lookupffn_last_gather_kernel() == "gather_kernel"
        ref = oracle.forward(x, signs, tables, acc64=False)
        assert np.array_equal(y16.view(torch.int16).cpu().numpy().view(np.uint16), oracle.float_to_bf16(ref))
    finally:
        B.lookupffn_set_option("gather_path", 0)
