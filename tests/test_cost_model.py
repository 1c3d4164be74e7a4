"""The analytic cost model against every MFLOP value the paper prints (tests/golden/paper_mflop.csv)."""
import csv
from pathlib import Path

import pytest

import oracle
from paper_2403_07221_amd import cost, synth

GOLDEN = Path(__file__).parent / "golden" / "paper_mflop.csv"


def rows():
    with open(GOLDEN) as f:
        for r in csv.reader(l for l in f if not l.startswith("#")):
            src, d, h, tau, proj, block, part, mflop = r
            yield pytest.param(int(d), int(h), int(tau), proj, int(block), part, float(mflop), id=src)


@pytest.mark.parametrize("d,h,tau,proj,block,part,printed", list(rows()))
def test_printed_mflop_values(d, h, tau, proj, block, part, printed):
    assert round(cost.paper_mflop(d, h, tau, proj, block, part) + 1e-9, 2) == pytest.approx(printed, abs=1e-9)


def test_padding_rule_is_the_one_the_flop_tables_imply():
    # RoBERTa-base row: d = 768 pads to 1024 and h*tau = 1530 needs two projections; with one
    # projection, or with d_pad = 768, the printed 1.39 MFLOP cannot be reached.
    assert cost.d_pad(768) == 1024 and cost.n_proj(768, 170, 9) == 2
    one_proj = (4 * (2 * 1024 * 64 + 1024 * 10) + 2 * 170 * 768) / 1e6
    assert round(one_proj, 2) != 1.39
    # the oracle and the workload descriptions use the same rule
    for d, h, tau in [(768, 170, 9), (512, 256, 8), (512, 20, 13), (768, 96, 8), (1024, 128, 10), (64, 8, 8)]:
        assert oracle.d_pad(d) == cost.d_pad(d)
        assert oracle.n_proj(d, h, tau) == cost.n_proj(d, h, tau)
    assert (synth.P6.n_proj, synth.P7.n_proj, synth.P8.n_proj) == (4, 2, 2)
    for w in synth.CONFIGS.values():
        assert (w.d_pad, w.n_proj) == (cost.d_pad(w.d), cost.n_proj(w.d, w.k, w.tau))


def test_algorithmic_bytes_of_the_benchmark_configurations():
    c2, c3, c4 = synth.C2, synth.C3, synth.C4
    assert cost.bytes_per_token(c2.d, c2.k, c2.d_out) == 301056
    assert cost.bytes_per_token(c3.d, c3.k, c3.d_out, x_bytes=2, table_bytes=2) == 152064
    assert cost.bytes_per_token(c4.d, c4.k, c4.d_out) == 532480
    assert cost.flops_per_token(c2.d, c2.k, c2.tau, c2.d_out, c2.n_rounds) == 33792 + 73728
    assert cost.flops_per_token(c4.d, c4.k, c4.tau, c4.d_out, c4.n_rounds) == 67584 + 131072
