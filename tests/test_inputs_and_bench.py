"""Host-side checks of the seeded input recipes and of bench.py's command line (no GPU needed)."""
import subprocess
import sys
from pathlib import Path

import numpy as np

from paper_2403_07221_amd import synth

ROOT = Path(__file__).resolve().parent.parent


def test_inputs_are_seeded_and_shaped_as_stated():
    w = synth.C2.with_tokens(100)
    x, signs, tables = synth.make_layer(w)
    x2, signs2, tables2 = synth.make_layer(w)
    assert np.array_equal(x, x2) and np.array_equal(signs, signs2) and np.array_equal(tables, tables2)
    assert x.shape == (100, 768) and x.dtype == np.float32
    assert signs.shape == (1, 3, 1024) and signs.dtype == np.int8 and set(np.unique(signs)) == {-1, 1}
    assert tables.shape == (96, 256, 768) and abs(float(tables.std()) - 0.02) < 2e-4
    assert abs(float(x.std()) - 1.0) < 0.02
    # the prefix of a longer batch is the shorter batch (row-major draws)
    xl, _, _ = synth.make_layer(synth.C2.with_tokens(300), with_tables=False)
    assert np.array_equal(xl[:100], x)


def test_bf16_rounding_is_nearest_even():
    a = np.array([1.0, 1.00390625, 1.01171875, -2.5, 3.0e-39], dtype=np.float32)   # ties at 2^-8 and 3*2^-8
    bits = synth.to_bf16_bits(a)
    back = (bits.astype(np.uint32) << 16).view(np.float32)
    assert back[0] == 1.0 and back[1] == 1.0 and back[2] == 1.015625 and back[3] == -2.5
    assert abs(back[4] - 3.0e-39) <= 2.0 ** -133


def test_zipf_codes_are_in_range_skewed_and_differently_ranked_per_table():
    codes = synth.make_zipf_codes(5, 20000, 4, 8, s=1.0)
    assert codes.shape == (20000, 4) and codes.dtype == np.uint16 and int(codes.max()) < 256
    for j in range(4):
        counts = np.bincount(codes[:, j], minlength=256)
        top = np.sort(counts)[::-1]
        assert top[0] > 20 * np.median(counts) and 0.12 < top[0] / 20000 < 0.21     # 1/H_256 = 0.163
    assert len({int(np.argmax(np.bincount(codes[:, j], minlength=256))) for j in range(4)}) > 1
    assert np.array_equal(codes, synth.make_zipf_codes(5, 20000, 4, 8, s=1.0))


def test_bench_refuses_more_than_one_gpu_with_a_message():
    r = subprocess.run([sys.executable, str(ROOT / "bench.py"), "--gpus", "2"], capture_output=True, text=True,
                       timeout=120)
    assert r.returncode == 2 and "one GPU" in r.stderr and r.stdout.strip() == ""
