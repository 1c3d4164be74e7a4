"""lookupffn_forward_static: the forward pass for callers that cannot allocate.  Through the C ABI it must
give lookupffn_forward's y bit for bit (and the oracle's), on two calls in a row that share the static
device array, the second with a smaller input; sizes beyond the array are refused."""
import numpy as np
import pytest
import torch

import oracle
from paper_2403_07221_amd import binding as B
from paper_2403_07221_amd import synth

pytestmark = pytest.mark.gpu


def test_forward_static_matches_forward_on_two_calls_in_a_row():
    assert torch.cuda.is_available(), "this test needs the MI355X"
    B.lib()
    w = synth.C2
    assert B.lookupffn_workspace_bytes(w.n_tokens, w.k) <= B.lookupffn_static_scratch_bytes() == 16 << 20
    x, signs, tables = synth.make_layer(w)
    sd, td = B.to_device(signs), B.to_device(tables)
    prep = B.lookupffn_prepare_tables(td)
    ws = torch.empty(B.lookupffn_workspace_bytes(w.n_tokens, w.k), dtype=torch.uint8, device="cuda")
    # first the full batch (LDS-staged gather, packed codes in the array), then a smaller one (direct gather,
    # codes in the ABI layout at the same addresses), then a mid-sized one with prepared tables
    for n, tab, kernel in ((w.n_tokens, td, "gather_lds_kernel"), (1000, td, "gather_kernel"),
                           (7000, prep, "gather_lds_kernel")):
        print(f"forward_static with {n} tokens", flush=True)
        xd = B.to_device(x[:n])
        want = B.lookupffn_forward(xd, sd, tab, workspace=ws)
        y = torch.full((n, w.d_out), float("nan"), dtype=torch.float32, device="cuda")
        B.lookupffn_forward_static(xd, sd, tab, y)
        torch.cuda.synchronize()
        assert B.lookupffn_last_gather_kernel() == kernel
        assert torch.equal(y, want), f"{n} tokens: differs from lookupffn_forward"
        sel = np.unique(np.concatenate([np.arange(0, n, 37), np.arange(n - 50, n)]))
        assert np.array_equal(y.cpu().numpy()[sel], oracle.forward(x[sel], signs, tables, acc64=False))
    # a batch whose intermediates exceed the static array is refused, not truncated
    big = 45000
    assert B.lookupffn_workspace_bytes(big, w.k) > B.lookupffn_static_scratch_bytes()
    xb = torch.zeros((big, w.d), dtype=torch.float32, device="cuda")
    yb = torch.empty((big, w.d_out), dtype=torch.float32, device="cuda")
    with pytest.raises(B.LookupFFNError) as e:
        B.lookupffn_forward_static(xb, sd, td, yb)
    assert e.value.status == -7
