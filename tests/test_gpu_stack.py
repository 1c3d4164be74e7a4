"""GPU parity of the single-launch small-batch path (lookupffn_forward_stack, and lookupffn_forward's use of
it for a few tokens) against the CPU oracle and against the two-kernel path.

Bars: y of every layer chain equals the oracle's fp32 sequential chain bit for bit (the kernel adds in table
order, as the large-batch kernels do), is within 1e-4 (fp32 tables) / 1e-2 (bf16 tables) of the oracle's
fp64-accumulated result for a single layer, and equals a loop of lookupffn_forward calls bit for bit.
"""
import numpy as np
import pytest
import torch

import oracle
from paper_2403_07221_amd import binding as B
from paper_2403_07221_amd import synth

pytestmark = pytest.mark.gpu

TOL_F32 = 1e-4
TOL_BF16 = 1e-2


@pytest.fixture(scope="module", autouse=True)
def _gpu():
    assert torch.cuda.is_available(), "these tests need the MI355X"
    B.lib()
    yield
    B.lookupffn_set_option("small_tokens", 0)
    B.lookupffn_set_option("gather_path", 0)


def rel_err(y, ref):
    ref64 = ref.astype(np.float64)
    rms = np.sqrt(np.mean(ref64 ** 2))
    return float(np.max(np.abs(y.astype(np.float64) - ref64)) / rms)


def make_stack(seed, n, d, k, tau, n_rounds, n_layers, xdt, tdt, d_out=None):
    d_out = d if d_out is None else d_out
    P = (k * tau + 1023) // 1024
    x = synth.make_x(seed, n, d, xdt)
    signs = [synth.make_signs(seed + 10 * l + 1, P, n_rounds, 1024) for l in range(n_layers)]
    # sigma chosen so that the chain neither dies out nor blows up: |y| stays near 1 per coordinate
    tables = [synth.make_tables(seed + 10 * l + 2, k, 1 << tau, d_out, tdt, sigma=1.0 / np.sqrt(k))
              for l in range(n_layers)]
    return x, signs, tables


def oracle_chain(x, signs, tables):
    """The oracle's fp32 sequential chain: (final y, final layer's fp64-accumulated y on the same input)."""
    h = x
    for s, t in zip(signs, tables):
        y64 = oracle.forward(h, s, t, acc64=True)
        h = oracle.forward(h, s, t, acc64=False)
    return h, y64


def dev_tables(t, prepared):
    td = B.to_device(t)
    return B.lookupffn_prepare_tables(td) if prepared else td


STACK_SHAPES = [
    # n, d, k, tau, R, layers, x dtype, table dtype, prepared, d_out
    (8, 768, 96, 8, 3, 12, "f32", "f32", False, None),     # the latency configuration's shape
    (1, 768, 96, 8, 3, 1, "f32", "f32", False, None),      # one token, one layer
    (9, 768, 96, 8, 3, 3, "bf16", "bf16", False, None),    # bf16 input and rows; later layers read fp32
    (8, 768, 96, 8, 3, 2, "f32", "f32", True, None),       # prepared tables, 128-byte pieces
    (5, 768, 33, 8, 2, 2, "f32", "bf16", True, None),      # prepared from bf16 rows; k not a multiple of the chunk
    (3, 600, 40, 9, 2, 2, "f32", "f32", True, None),       # prepared tables, 64-byte pieces, ragged last piece
    (5, 520, 103, 10, 3, 2, "f32", "f32", False, None),    # two projections (1030 bits), 9 waves
    (7, 1024, 37, 7, 4, 3, "f32", "f32", False, None),     # no padding, four rounds, odd k
    (4, 1000, 1, 5, 1, 2, "f32", "f32", False, None),      # a single table
    (6, 999, 50, 7, 3, 1, "f32", "f32", False, 4100),      # d % 4 != 0 (scalar row loads); rows wider than a workgroup
    (6, 998, 50, 7, 3, 1, "bf16", "bf16", False, 2056),    # bf16 rows wider than a workgroup
    (300, 768, 64, 8, 3, 2, "f32", "f32", False, None),    # more tokens than compute units
]


@pytest.mark.parametrize("n,d,k,tau,R,layers,xdt,tdt,prepared,d_out", STACK_SHAPES)
def test_forward_stack_matches_the_oracle_chain(n, d, k, tau, R, layers, xdt, tdt, prepared, d_out):
    print(f"stack n={n} d={d} k={k} tau={tau} R={R} layers={layers} x={xdt} tables={tdt} "
          f"prepared={prepared} d_out={d_out}", flush=True)
    x, signs, tables = make_stack(4100 + n + d + k, n, d, k, tau, R, layers, xdt, tdt, d_out)
    want, want64 = oracle_chain(x, signs, tables)
    sd = [B.to_device(s) for s in signs]
    td = [dev_tables(t, prepared) for t in tables]
    y = B.lookupffn_forward_stack(B.to_device(x), sd, td)
    torch.cuda.synchronize()
    assert B.lookupffn_last_gather_kernel() == "forward_stack_kernel"
    y = y.cpu().numpy()
    assert np.array_equal(y, want)
    assert rel_err(y, want64) <= (TOL_BF16 if tdt == "bf16" else TOL_F32)


@pytest.mark.parametrize("prepared", [False, True])
def test_forward_stack_equals_the_layer_loop(prepared):
    """C5: one launch for 12 layers == 12 x (hash kernel, gather kernel) == 12 single-layer launches."""
    w = synth.C5
    print(f"stack C5 against the loops, prepared={prepared}", flush=True)
    layers = [synth.make_layer(w, layer=l, with_x=(l == 0)) for l in range(w.n_layers)]
    xd = B.to_device(layers[0][0])
    sd = [B.to_device(s) for _, s, _ in layers]
    td = [dev_tables(t, prepared) for _, _, t in layers]
    y = B.lookupffn_forward_stack(xd, sd, td).cpu().numpy()
    results = {}
    try:
        for name, small in (("two kernels", -1), ("one launch per layer", 0)):
            B.lookupffn_set_option("small_tokens", small)
            g = xd
            for l in range(w.n_layers):
                g = B.lookupffn_forward(g, sd[l], td[l])
                assert (B.lookupffn_last_gather_kernel() == "forward_stack_kernel") == (small == 0)
            results[name] = g.cpu().numpy()
    finally:
        B.lookupffn_set_option("small_tokens", 0)
    for name, g in results.items():
        assert np.array_equal(y, g), name


def test_forward_takes_the_single_launch_up_to_its_token_limit():
    w = synth.C2
    x, signs, tables = synth.make_layer(w, n_tokens=600)
    sd, td = B.to_device(signs), B.to_device(tables)
    want = oracle.forward(x, signs, tables, acc64=False)
    try:
        for n, limit, single in ((512, 0, True), (513, 0, False), (600, 600, True), (3, -1, False),
                                 (3, 2, False), (2, 2, True)):
            print(f"forward n={n} small_tokens={limit}", flush=True)
            B.lookupffn_set_option("small_tokens", limit)
            y = B.lookupffn_forward(B.to_device(x[:n]), sd, td)
            torch.cuda.synchronize()
            assert (B.lookupffn_last_gather_kernel() == "forward_stack_kernel") == single
            assert np.array_equal(y.cpu().numpy(), want[:n])
        # a forced gather path keeps the two-kernel route whatever the batch size
        B.lookupffn_set_option("small_tokens", 0)
        B.lookupffn_set_option("gather_path", 1)
        y = B.lookupffn_forward(B.to_device(x[:8]), sd, td)
        assert B.lookupffn_last_gather_kernel() == "gather_kernel"
        assert np.array_equal(y.cpu().numpy(), want[:8])
    finally:
        B.lookupffn_set_option("small_tokens", 0)
        B.lookupffn_set_option("gather_path", 0)


def test_forward_stack_refuses_what_its_kernel_does_not_take():
    x = torch.zeros((4, 64), dtype=torch.float32, device="cuda")
    signs = torch.ones((1, 2, 64), dtype=torch.int8, device="cuda")
    tables = torch.zeros((8, 256, 64), dtype=torch.float32, device="cuda")
    with pytest.raises(B.LookupFFNError) as e:
        B.lookupffn_forward_stack(x, [signs], [tables])          # d_pad = 64
    assert e.value.status == -6
    x = torch.zeros((4, 768), dtype=torch.float32, device="cuda")
    signs = torch.ones((1, 3, 1024), dtype=torch.int8, device="cuda")
    tables = torch.zeros((16, 256, 512), dtype=torch.float32, device="cuda")
    with pytest.raises(B.LookupFFNError) as e:
        B.lookupffn_forward_stack(x, [signs, signs], [tables, tables])   # chained layers need d_out == d
    assert e.value.status == -2
    with pytest.raises(B.LookupFFNError) as e:
        B.lookupffn_forward_stack(x, [signs] * 33, [tables] * 33)
    assert e.value.status == -2
    y = B.lookupffn_forward_stack(x[:0], [signs], [tables])      # an empty batch is a successful no-op
    assert tuple(y.shape) == (0, 512)


def test_forward_stack_replays_in_a_hip_graph():
    """The call allocates nothing and never synchronises: it is captured as it stands; every replay, with
    eager work in between, gives the eager bits."""
    w = synth.C5
    layers = [synth.make_layer(w, layer=l, with_x=(l == 0)) for l in range(4)]
    xd = B.to_device(layers[0][0])
    sd = [B.to_device(s) for _, s, _ in layers]
    td = [B.to_device(t) for _, _, t in layers]
    B.lookupffn_init()
    eager = B.lookupffn_forward_stack(xd, sd, td).clone()
    torch.cuda.synchronize()
    y = torch.empty_like(eager)
    g = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    with torch.cuda.stream(side):
        with torch.cuda.graph(g, stream=side):
            B.lookupffn_forward_stack(xd, sd, td, y=y)
    x2 = B.to_device(synth.make_x(991, w.n_tokens, w.d))
    eager2 = B.lookupffn_forward_stack(x2, sd, td).clone()
    torch.cuda.synchronize()
    for rep in range(3):
        y.fill_(float("nan"))
        xd.copy_(B.to_device(layers[0][0]) if rep != 1 else x2)
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        assert torch.equal(y, eager if rep != 1 else eager2), f"replay {rep}"
        _ = B.lookupffn_forward(x2, sd[0], td[0])                # eager work between the replays
        torch.cuda.synchronize()
