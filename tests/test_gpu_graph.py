"""The forward pass under HIP graph capture: with a caller workspace and a caller y the entry points only
launch kernels on the given stream (no allocation, no synchronisation, no memset), so a chain of layers
can be captured once and replayed.  Every replay is checked against the eager result, with eager work and
synchronisations between the replays and with new input contents in the captured buffers."""
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
    B.lookupffn_timing_enable(0)
    yield


def test_captured_chain_of_layers_replays_like_eager():
    print("graph capture: C5 chain (8 tokens x 12 layers)", flush=True)
    w = synth.C5
    layers = [synth.make_layer(w, layer=l, with_x=(l == 0)) for l in range(w.n_layers)]
    dev = [(B.to_device(s), B.to_device(t)) for _, s, t in layers]
    ws = torch.empty(B.lookupffn_workspace_bytes(w.n_tokens, w.k), dtype=torch.uint8, device="cuda")
    x_in = B.to_device(layers[0][0]).clone()
    ys = [torch.empty((w.n_tokens, w.d_out), dtype=torch.float32, device="cuda") for _ in range(2)]

    def chain():
        h = x_in
        for l in range(w.n_layers):
            h = B.lookupffn_forward(h, dev[l][0], dev[l][1], y=ys[l & 1], workspace=ws)
        return h

    chain()                                   # eager warm-up: code objects loaded, attributes set
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        out = chain()
    torch.cuda.synchronize()
    for rep in range(4):
        x_new = synth.make_x(100 + rep, w.n_tokens, w.d)
        x_in.copy_(torch.from_numpy(x_new).cuda())
        graph.replay()
        torch.cuda.synchronize()
        got = out.clone().cpu().numpy()
        want = chain().clone().cpu().numpy()  # eager, same buffers, between the replays
        assert np.array_equal(got, want), f"replay {rep} differs from the eager chain"
        h = x_new
        for _, signs, tables in layers:       # and the oracle's fp32-sequential chain: identical bits
            h = oracle.forward(h, signs, tables, acc64=False)
        assert np.array_equal(got, h), f"replay {rep} differs from the oracle"
        print(f"  replay {rep} ok", flush=True)


@pytest.mark.parametrize("variant", ["plain", "weighted", "bh-weighted"])
def test_captured_single_layer_replays_like_eager(variant):
    print(f"graph capture: C2 with 3000 tokens, {variant}", flush=True)
    w = synth.C2.with_tokens(3000)
    x, signs, tables = synth.make_layer(w)
    td = B.to_device(tables)
    if variant == "bh-weighted":
        bm = synth.make_bmats(5, w.n_proj, 4, w.d_pad, 32)
        par, fwd = torch.from_numpy(bm).cuda(), B.lookupffn_forward_bh_weighted
        nbytes = B.lookupffn_workspace_bytes_bh_weighted(w.n_tokens, w.d, w.k, w.tau, 32, 4)
        ref = lambda xs: oracle.bh_forward_weighted(xs, bm, tables)
    elif variant == "weighted":
        par, fwd = B.to_device(signs), B.lookupffn_forward_weighted
        nbytes = B.lookupffn_workspace_bytes_weighted(w.n_tokens, w.k)
        ref = lambda xs: oracle.forward_weighted(xs, signs, tables)
    else:
        par, fwd = B.to_device(signs), B.lookupffn_forward
        nbytes = B.lookupffn_workspace_bytes(w.n_tokens, w.k)
        ref = lambda xs: oracle.forward(xs, signs, tables)
    ws = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
    x_in = B.to_device(x).clone()
    y = torch.empty((w.n_tokens, w.d_out), dtype=torch.float32, device="cuda")
    fwd(x_in, par, td, y=y, workspace=ws)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        fwd(x_in, par, td, y=y, workspace=ws)
    torch.cuda.synchronize()
    for rep in range(3):
        x_new = synth.make_x(200 + rep, w.n_tokens, w.d)
        x_in.copy_(torch.from_numpy(x_new).cuda())
        y.fill_(float("nan"))
        graph.replay()
        torch.cuda.synchronize()
        got = y.clone().cpu().numpy()
        eager = fwd(x_in, par, td, y=y, workspace=ws).clone().cpu().numpy()
        assert np.array_equal(got, eager), f"replay {rep} differs from the eager call"
        r = ref(x_new).astype(np.float64)
        assert np.max(np.abs(got - r)) / np.sqrt(np.mean(r ** 2)) <= 1e-4


@pytest.mark.parametrize("variant", ["plain", "weighted", "probes"])
def test_captured_stand_alone_gather_replays_like_eager(variant):
    """lookupffn_gather* with a caller workspace after lookupffn_init(): kernel launches only, so the call
    (re-pack kernels + the LDS-staged gather) can be captured without an eager warm-up of its own."""
    print(f"graph capture: stand-alone gather, {variant}, 3000 tokens of the C2 shape", flush=True)
    B.lookupffn_init()
    n, k, tau, d_out = 3000, 96, 8, 768
    tables = synth.make_tables(31, k, 1 << tau, d_out)
    prep = B.lookupffn_prepare_tables(B.to_device(tables))
    rng = np.random.default_rng(17)
    codes_in = torch.zeros((n, k), dtype=torch.int16, device="cuda")
    if variant == "plain":
        wts_in, call = None, lambda y: B.lookupffn_gather(codes_in, prep, y=y, workspace=ws)
        nbytes = B.lookupffn_workspace_bytes_gather(n, k)
    elif variant == "weighted":
        wts_in = torch.zeros((n, k), dtype=torch.float32, device="cuda")
        call = lambda y: B.lookupffn_gather_weighted(codes_in, wts_in, prep, y=y, workspace=ws)
        nbytes = B.lookupffn_workspace_bytes_gather_weighted(n, k)
    else:
        wts_in = torch.zeros((n, k, tau + 1), dtype=torch.float32, device="cuda")
        call = lambda y: B.lookupffn_gather_probes(codes_in, wts_in, prep, y=y, workspace=ws)
        nbytes = B.lookupffn_workspace_bytes_gather_probes(n, k, tau)
    ws = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
    y = torch.empty((n, d_out), dtype=torch.float32, device="cuda")
    B.lookupffn_set_option("gather_path", 2)
    try:
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            call(y)
        assert B.lookupffn_last_gather_kernel() == "gather_lds_kernel"
        torch.cuda.synchronize()
        for rep in range(3):
            codes = rng.integers(0, 1 << tau, size=(n, k)).astype(np.uint16)
            codes_in.copy_(torch.from_numpy(codes.view(np.int16)))
            if wts_in is not None:
                wts = rng.random(tuple(wts_in.shape), dtype=np.float32)
                wts_in.copy_(torch.from_numpy(wts))
            y.fill_(float("nan"))
            graph.replay()
            torch.cuda.synchronize()
            got = y.clone().cpu().numpy()
            eager = call(y).clone().cpu().numpy()       # eager, same buffers, between the replays
            assert np.array_equal(got, eager), f"replay {rep} differs from the eager call"
            if variant == "plain":
                assert np.array_equal(got, oracle.gather(codes, tables, acc64=False))
            elif variant == "weighted":
                r = oracle.gather_weighted(codes, wts.astype(np.float64), tables).astype(np.float64)
                assert np.max(np.abs(got - r)) / np.sqrt(np.mean(r ** 2)) <= 1e-4
            else:
                r = oracle.gather_probes(codes, wts.astype(np.float64), tables).astype(np.float64)
                assert np.max(np.abs(got - r)) / np.sqrt(np.mean(r ** 2)) <= 1e-4
    finally:
        B.lookupffn_set_option("gather_path", 0)
