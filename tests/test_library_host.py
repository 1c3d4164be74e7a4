"""Host-side checks of the C-ABI library that need no GPU: it loads, exports every symbol the
header declares, and rejects bad arguments before touching HIP."""
import ctypes
import re
from pathlib import Path

import pytest

from paper_2403_07221_amd import binding

ROOT = Path(__file__).resolve().parent.parent
HEADER = (ROOT / "include" / "lookupffn.h").read_text()
FAKE = 1 << 20          # a non-NULL, 16-byte aligned stand-in for a device pointer (never dereferenced)


@pytest.fixture(scope="module")
def L():
    return binding.lib()


def declared_functions():
    body = re.sub(r"/\*.*?\*/", "", HEADER, flags=re.S)
    return sorted(set(re.findall(r"\b(lookupffn_\w+)\s*\(", body)))


def test_every_declared_symbol_is_exported(L):
    names = declared_functions()
    assert len(names) >= 12 and sorted(binding.EXPORTS) == names
    for n in names:
        assert getattr(L, n) is not None


def test_version_and_strerror(L):
    assert L.lookupffn_version() >= 100
    assert L.lookupffn_strerror(0).decode() == "success"
    for s in range(-8, 0):
        assert L.lookupffn_strerror(s).decode() not in ("", "unknown status")
    assert L.lookupffn_strerror(-99).decode() == "unknown status"


def hash_call(L, x=FAKE, signs=FAKE, codes=FAKE, n=0, d=768, k=96, tau=8, rounds=3, dt=0):
    return L.lookupffn_hash(x, signs, codes, n, d, k, tau, rounds, dt, None)


def gather_call(L, codes=FAKE, tables=FAKE, y=FAKE, n=0, k=96, tau=8, d_out=768, dt=0, ws=None, wsb=0):
    return L.lookupffn_gather(codes, tables, y, n, k, tau, d_out, dt, ws, wsb, None)


def forward_call(L, x=FAKE, signs=FAKE, tables=FAKE, y=FAKE, n=0, d=768, k=96, tau=8, d_out=768, rounds=3,
                 xdt=0, tdt=0, ws=None, wsb=0):
    return L.lookupffn_forward(x, signs, tables, y, n, d, k, tau, d_out, rounds, xdt, tdt, ws, wsb, None)


def test_empty_batch_is_a_successful_noop(L):
    assert hash_call(L) == 0 and gather_call(L) == 0 and forward_call(L) == 0


def test_hash_argument_errors(L):
    assert hash_call(L, x=None) == -1 and hash_call(L, signs=None) == -1 and hash_call(L, codes=None) == -1
    assert hash_call(L, n=-1) == -2 and hash_call(L, d=0) == -2 and hash_call(L, k=0) == -2
    assert hash_call(L, rounds=0) == -2
    assert hash_call(L, tau=0) == -3 and hash_call(L, tau=17) == -3
    assert hash_call(L, dt=2) == 0 and hash_call(L, dt=3) == -4                # 2 = IEEE half
    assert hash_call(L, x=FAKE + 2) == -5 and hash_call(L, x=FAKE + 2, dt=1) == 0
    assert hash_call(L, codes=FAKE + 1) == -5
    assert hash_call(L, d=4097) == -6 and hash_call(L, d=4096, k=512) == 0


def test_gather_argument_errors(L):
    assert gather_call(L, codes=None) == -1 and gather_call(L, tables=None) == -1 and gather_call(L, y=None) == -1
    assert gather_call(L, n=-5) == -2 and gather_call(L, k=0) == -2 and gather_call(L, d_out=0) == -2
    assert gather_call(L, tau=0) == -3 and gather_call(L, tau=17) == -3
    assert gather_call(L, dt=7) == -4
    assert gather_call(L, d_out=770) == -5                    # fp32 rows must be whole 16-byte pieces
    assert gather_call(L, d_out=772) == 0 and gather_call(L, d_out=772, dt=1) == -5
    assert gather_call(L, tables=FAKE + 4) == -5 and gather_call(L, y=FAKE + 8) == -5
    # prepared tables: the flag with either source dtype; the buffer is 256-byte aligned
    assert gather_call(L, dt=0x100) == 0 and gather_call(L, dt=0x101) == 0 and gather_call(L, dt=0x102) == 0 and gather_call(L, dt=0x103) == -4
    assert gather_call(L, dt=0x800) == -4 and gather_call(L, tables=FAKE + 16, dt=0x100) == -5
    # 16-bit outputs: one of the two flags, y then 8-byte aligned
    assert gather_call(L, dt=0x200) == 0 and gather_call(L, dt=0x401) == 0 and gather_call(L, dt=0x600) == -4
    assert gather_call(L, y=FAKE + 8, dt=0x200) == 0 and gather_call(L, y=FAKE + 4, dt=0x200) == -5
    assert gather_call(L, d_out=772, dt=0x101) == -5          # the source rows were bf16: whole 16-byte pieces of those
    # scratch of the stand-alone gather: too small or misaligned is refused before any launch
    need = L.lookupffn_workspace_bytes_gather(1000, 96)
    assert need >= 48 * 1000 * 4 and need % 256 == 0 and L.lookupffn_workspace_bytes_gather(0, 96) == 0
    assert gather_call(L, n=1000, ws=FAKE, wsb=need - 1) == -7 and gather_call(L, n=1000, ws=FAKE + 16, wsb=need) == -5


def test_forward_argument_errors(L):
    assert forward_call(L, x=None) == -1 and forward_call(L, tables=None) == -1 and forward_call(L, y=None) == -1
    assert forward_call(L, tau=0) == -3 and forward_call(L, xdt=3) == -4 and forward_call(L, tdt=-1) == -4
    need = L.lookupffn_workspace_bytes(1000, 96)
    assert need >= 1000 * 96 * 2 and need % 256 == 0
    assert L.lookupffn_workspace_bytes(0, 96) == 0
    # a caller workspace that is too small or misaligned is refused before any launch
    assert forward_call(L, n=1000, ws=FAKE, wsb=need - 1) == -7
    assert forward_call(L, n=1000, ws=FAKE + 16, wsb=need) == -5


def test_forward_static_argument_errors(L):
    def fs(x=FAKE, signs=FAKE, tables=FAKE, y=FAKE, n=0, d=768, k=96, tau=8, d_out=768, xdt=0, tdt=0):
        return L.lookupffn_forward_static(x, signs, tables, y, n, d, k, tau, d_out, 3, xdt, tdt, None)

    assert L.lookupffn_static_scratch_bytes() == 16 << 20
    assert fs() == 0                                                   # empty batch
    assert fs(x=None) == -1 and fs(y=None) == -1 and fs(tau=0) == -3 and fs(tdt=9) == -4 and fs(d=5000) == -6
    assert fs(n=5, x=None) == -1                                       # argument errors need no GPU
    # the static array bounds the batch: refused before any HIP call
    assert L.lookupffn_workspace_bytes(39000, 96) <= 16 << 20 < L.lookupffn_workspace_bytes(45000, 96)
    assert fs(n=45000) == -7 and fs(n=1 << 30) == -7


def test_forward_stack_argument_errors(L):
    vp = ctypes.c_void_p

    def st(x=FAKE, signs=(FAKE,), tables=(FAKE,), y=FAKE, n=0, d=768, k=96, tau=8, d_out=768, rounds=3, xdt=0, tdt=0):
        sp = (vp * len(signs))(*signs) if signs is not None else None
        tp = (vp * len(tables))(*tables) if tables is not None else None
        return L.lookupffn_forward_stack(x, sp, tp, y, n, d, k, tau, d_out, rounds, len(signs or ()), xdt, tdt, None)

    assert st() == 0 and st(signs=(FAKE,) * 12, tables=(FAKE,) * 12) == 0          # empty batch
    assert st(signs=None) == -1 and st(x=None) == -1 and st(y=None) == -1
    assert st(signs=(FAKE, None), tables=(FAKE, FAKE)) == -1 and st(signs=(FAKE, FAKE), tables=(FAKE, None)) == -1
    assert st(signs=(FAKE,) * 33, tables=(FAKE,) * 33) == -2                       # at most 32 layers
    assert st(tau=0) == -3 and st(tdt=7) == -4 and st(d_out=770) == -5
    assert st(signs=(FAKE,) * 2, tables=(FAKE,) * 2, d_out=512) == -2              # chained layers: d_out == d
    assert st(d_out=512) == 0                                                     # a single layer may differ
    # shapes the single-launch kernel does not take: other transform widths, more than four rounds,
    # a table set of 2 GiB or more, signs off the 16-byte grid
    assert st(d=64) == -6 and st(d=512) == -6 and st(d=2048) == -6 and st(rounds=5) == -6
    assert st(k=128, tau=12, d_out=1024) == -6 and st(k=128, tau=11, d_out=1024) == 0
    assert st(signs=(FAKE + 4,)) == -6


def test_weighted_argument_errors(L):
    def hw(x=FAKE, signs=FAKE, codes=FAKE, w=FAKE, n=0, d=768, k=96, tau=8, rounds=3, dt=0):
        return L.lookupffn_hash_weighted(x, signs, codes, w, n, d, k, tau, rounds, dt, None)

    def gw(codes=FAKE, w=FAKE, tables=FAKE, y=FAKE, n=0, k=96, tau=8, d_out=768, dt=0, ws=None, wsb=0):
        return L.lookupffn_gather_weighted(codes, w, tables, y, n, k, tau, d_out, dt, ws, wsb, None)

    def fw(x=FAKE, tables=FAKE, y=FAKE, n=0, d=768, tau=8, ws=None, wsb=0):
        return L.lookupffn_forward_weighted(x, FAKE, tables, y, n, d, 96, tau, 768, 3, 0, 0, ws, wsb, None)

    assert hw() == 0 and gw() == 0 and fw() == 0                      # empty batch: successful no-op
    assert hw(w=None) == -1 and hw(x=None) == -1 and hw(w=FAKE + 2) == -5 and hw(tau=17) == -3
    assert hw(d=4096, k=512) == -6 and hw(d=2048, k=256) == 0         # working set of the widest transform
    assert gw(w=None) == -1 and gw(codes=None) == -1 and gw(w=FAKE + 1) == -5 and gw(d_out=770) == -5
    assert fw(x=None) == -1 and fw(tau=0) == -3 and fw(d=4096) == -6
    need = L.lookupffn_workspace_bytes_weighted(1000, 96)
    assert need >= 1000 * 96 * 6 and need % 256 == 0 and L.lookupffn_workspace_bytes_weighted(0, 96) == 0
    assert fw(n=1000, ws=FAKE, wsb=need - 1) == -7 and fw(n=1000, ws=FAKE + 16, wsb=need) == -5
    gneed = L.lookupffn_workspace_bytes_gather_weighted(1000, 96)
    assert L.lookupffn_workspace_bytes_gather(1000, 96) + 1000 * 96 * 4 <= gneed < need
    assert gw(n=1000, ws=FAKE, wsb=gneed - 1) == -7 and gw(n=1000, ws=FAKE + 16, wsb=gneed) == -5


def test_prepare_tables_sizes_and_argument_errors(L):
    def prep(tables=FAKE, k=96, tau=8, d_out=768, dt=0, out=FAKE, nbytes=None):
        nbytes = L.lookupffn_prepared_tables_bytes(k, tau, d_out, dt) if nbytes is None else nbytes
        return L.lookupffn_prepare_tables(tables, k, tau, d_out, dt, out, nbytes, None)

    # fp32 copy, slice-major: whole 128-byte (tau <= 8) or 64-byte (tau >= 9) pieces per row
    assert L.lookupffn_prepared_tables_bytes(96, 8, 768, 0) == 96 * 256 * 768 * 4
    assert L.lookupffn_prepared_tables_bytes(96, 8, 768, 1) == 96 * 256 * 768 * 4       # bf16 rows are widened
    assert L.lookupffn_prepared_tables_bytes(2, 7, 8, 0) == 2 * 128 * 128                # 32-byte rows padded to a piece
    assert L.lookupffn_prepared_tables_bytes(6, 9, 200, 0) == 6 * 512 * 13 * 64          # 800-byte rows: 13 pieces of 64
    assert L.lookupffn_prepared_tables_bytes(3, 10, 72, 1) % 256 == 0
    for bad in ((0, 8, 768, 0), (96, 17, 768, 0), (96, 0, 768, 0), (96, 8, 770, 0), (96, 8, 772, 1), (96, 8, 772, 2), (96, 8, 768, 3)):
        assert L.lookupffn_prepared_tables_bytes(*bad) == 0
    assert prep(tables=None) == -1 and prep(out=None) == -1
    assert prep(k=0) == -2 and prep(tau=0) == -3 and prep(tau=17) == -3 and prep(dt=3) == -4 and prep(dt=0x100) == -4
    assert prep(d_out=770) == -5 and prep(d_out=772, dt=1) == -5
    assert prep(tables=FAKE + 8) == -5 and prep(out=FAKE + 16) == -5
    assert prep(nbytes=96 * 256 * 768 * 4 - 1) == -7


def test_prepare_bh_sizes_and_argument_errors(L):
    def prep(bm=FAKE, d=768, k=96, tau=8, block=64, m=4, out=FAKE, nbytes=None):
        nbytes = L.lookupffn_prepared_bh_bytes(d, k, tau, block, m) if nbytes is None else nbytes
        return L.lookupffn_prepare_bh(bm, d, k, tau, block, m, out, nbytes, None)

    assert L.lookupffn_prepared_bh_bytes(768, 96, 8, 64, 4) == 4 * 1024 * 64 * 4         # P * m * d_pad * block floats
    assert L.lookupffn_prepared_bh_bytes(512, 256, 8, 16, 4) == 4 * 4 * 512 * 16 * 4
    assert L.lookupffn_prepared_bh_bytes(768, 96, 8, 48, 4) == 0 and L.lookupffn_prepared_bh_bytes(2000, 96, 8, 64, 4) == 0
    assert prep(bm=None) == -1 and prep(out=None) == -1 and prep(block=8) == -6 and prep(d=20, k=4) == -6
    assert prep(tau=0) == -3 and prep(m=0) == -2 and prep(out=FAKE + 16) == -5 and prep(bm=FAKE + 2) == -5
    assert prep(nbytes=1024) == -7
    # a workspace for the prepared form need not hold the re-ordered factors
    full = L.lookupffn_workspace_bytes_bh(1000, 768, 96, 8, 64, 4)
    assert L.lookupffn_workspace_bytes_bh(1000, 768, 96, 8, 0x100 | 64, 4) == full - 4 * 1024 * 64 * 4
    assert L.lookupffn_hash_bh(FAKE, FAKE, FAKE, 0, 768, 96, 8, 0x100 | 64, 4, 0, None, 0, None) == 0
    assert L.lookupffn_hash_bh(FAKE, FAKE + 16, FAKE, 0, 768, 96, 8, 0x100 | 64, 4, 0, None, 0, None) == -5
    assert L.lookupffn_hash_bh(FAKE, FAKE, FAKE, 0, 768, 96, 8, 0x100 | 48, 4, 0, None, 0, None) == -6


def test_timing_read_argument_errors(L):
    cnt = ctypes.c_int64(0)
    ms = ctypes.c_double(0)
    assert L.lookupffn_timing_read(2, ctypes.byref(ms), ctypes.byref(cnt)) == -2
    assert L.lookupffn_timing_read(0, None, ctypes.byref(cnt)) == -1
    assert L.lookupffn_timing_read_each(0, None, 0, ctypes.byref(cnt)) == 0 and cnt.value == 0
    assert L.lookupffn_timing_read_each(0, None, 4, ctypes.byref(cnt)) == -1
    assert L.lookupffn_timing_read_each(3, None, 0, ctypes.byref(cnt)) == -2
    assert L.lookupffn_timing_read_each(0, None, -1, ctypes.byref(cnt)) == -2
    assert L.lookupffn_timing_read_each(0, None, 0, None) == -1


def test_bh_argument_errors(L):
    def hb(x=FAKE, bm=FAKE, codes=FAKE, n=0, d=768, k=96, tau=8, block=64, m=4, dt=0, ws=None, wsb=0):
        return L.lookupffn_hash_bh(x, bm, codes, n, d, k, tau, block, m, dt, ws, wsb, None)

    def fb(x=FAKE, tables=FAKE, y=FAKE, n=0, d=768, tau=8, block=64, ws=None, wsb=0):
        return L.lookupffn_forward_bh(x, FAKE, tables, y, n, d, 96, tau, 768, block, 4, 0, 0, ws, wsb, None)

    assert hb() == 0 and fb() == 0
    assert hb(x=None) == -1 and hb(bm=None) == -1 and hb(codes=None) == -1 and hb(tau=0) == -3 and hb(dt=5) == -4
    assert hb(block=8) == -6 and hb(block=128) == -6 and hb(d=2000) == -6 and hb(d=20, k=4) == -6
    assert hb(d=64, k=8, block=64) == 0 and hb(d=60, k=8, block=64) == 0 and hb(m=0) == -2
    assert fb(tables=None) == -1 and fb(block=48) == -6 and fb(tau=17) == -3
    need = L.lookupffn_workspace_bytes_bh(1000, 768, 96, 8, 64, 4)
    assert need >= 4 * 1024 * 64 * 4 + 1000 * 96 * 2 and need % 256 == 0
    assert hb(n=1000, ws=FAKE, wsb=1024) == -7 and fb(n=1000, ws=FAKE, wsb=need - 1) == -7
    assert fb(n=1000, ws=FAKE + 16, wsb=need) == -5


def test_bh_weighted_argument_errors(L):
    def hb(x=FAKE, bm=FAKE, codes=FAKE, w=FAKE, n=0, d=768, k=96, tau=8, block=64, m=4, dt=0, ws=None, wsb=0):
        return L.lookupffn_hash_bh_weighted(x, bm, codes, w, n, d, k, tau, block, m, dt, ws, wsb, None)

    def fb(x=FAKE, tables=FAKE, y=FAKE, n=0, d=768, tau=8, block=64, ws=None, wsb=0):
        return L.lookupffn_forward_bh_weighted(x, FAKE, tables, y, n, d, 96, tau, 768, block, 4, 0, 0, ws, wsb, None)

    assert hb() == 0 and fb() == 0 and hb(tau=4) == 0 and hb(tau=16, k=60) == 0
    assert hb(w=None) == -1 and hb(codes=None) == -1 and hb(w=FAKE + 2) == -5 and hb(x=None) == -1
    assert hb(tau=9) == 0 and hb(tau=2) == 0 and fb(tau=10) == 0 and hb(tau=17) == -3        # any tau up to 16
    # tau other than 4, 8, 16: the weights come from z inside the kernel, no scratch of their own
    assert L.lookupffn_workspace_bytes_bh_weighted(1000, 768, 170, 9, 64, 4) == L.lookupffn_workspace_bytes_bh_weighted(1000, 768, 170, 8, 64, 4)
    assert hb(tau=9, k=600) == 0 and hb(tau=9, k=700) == -6    # seven projections and the z window do not fit the LDS
    assert hb(block=8) == -6 and hb(d=2000) == -6 and fb(tables=None) == -1
    need = L.lookupffn_workspace_bytes_bh_weighted(1000, 768, 96, 8, 64, 4)
    plain = L.lookupffn_workspace_bytes_bh(1000, 768, 96, 8, 64, 4)
    assert need > plain + 1000 * 96 * 4 and need % 256 == 0
    assert fb(n=1000, ws=FAKE, wsb=need - 1) == -7 and fb(n=1000, ws=FAKE + 16, wsb=need) == -5
    assert hb(n=1000, ws=FAKE, wsb=1024) == -7


def test_probe_argument_errors(L):
    def hp(x=FAKE, signs=FAKE, codes=FAKE, sh=FAKE, n=0, d=768, k=96, tau=8):
        return L.lookupffn_hash_probes(x, signs, codes, sh, n, d, k, tau, 3, 0, None)

    def gp(codes=FAKE, sh=FAKE, tables=FAKE, y=FAKE, n=0, tau=8, d_out=768, ws=None, wsb=0):
        return L.lookupffn_gather_probes(codes, sh, tables, y, n, 96, tau, d_out, 0, ws, wsb, None)

    def fp(x=FAKE, y=FAKE, n=0, tau=8, ws=None, wsb=0):
        return L.lookupffn_forward_probes(x, FAKE, FAKE, y, n, 768, 96, tau, 768, 3, 0, 0, ws, wsb, None)

    assert hp() == 0 and gp() == 0 and fp() == 0
    assert hp(sh=None) == -1 and hp(sh=FAKE + 2) == -5 and hp(tau=0) == -3 and hp(d=4096, k=512) == -6
    assert gp(sh=None) == -1 and gp(tables=None) == -1 and gp(d_out=770) == -5 and gp(tau=17) == -3
    assert fp(x=None) == -1 and fp(y=None) == -1
    need = L.lookupffn_workspace_bytes_probes(1000, 96, 8)
    assert need >= 1000 * 96 * (2 + 9 * 4) and need % 256 == 0 and L.lookupffn_workspace_bytes_probes(0, 96, 8) == 0
    assert fp(n=1000, ws=FAKE, wsb=need - 1) == -7 and fp(n=1000, ws=FAKE + 16, wsb=need) == -5
    gneed = L.lookupffn_workspace_bytes_gather_probes(1000, 96, 8)
    assert 1000 * 96 * 9 * 4 <= gneed < need and L.lookupffn_workspace_bytes_gather_probes(1000, 96, 17) == 0
    assert gp(n=1000, ws=FAKE, wsb=gneed - 1) == -7 and gp(n=1000, ws=FAKE + 16, wsb=gneed) == -5


def test_options(L):
    assert L.lookupffn_set_option(b"lanes_per_token", 16) == 0
    assert L.lookupffn_set_option(b"lanes_per_token", 3) == -2
    assert L.lookupffn_set_option(b"lanes_per_token", 128) == -2
    assert L.lookupffn_set_option(b"lanes_per_token", 0) == 0
    assert L.lookupffn_set_option(b"xcd_order", 2) == -2 and L.lookupffn_set_option(b"xcd_order", 0) == 0
    assert L.lookupffn_set_option(b"gather_path", 5) == -2 and L.lookupffn_set_option(b"gather_path", 4) == 0
    assert L.lookupffn_set_option(b"gather_path", 0) == 0
    assert L.lookupffn_set_option(b"hash_path", 4) == -2 and L.lookupffn_set_option(b"hash_path", 0) == 0
    assert L.lookupffn_set_option(b"hash_blocks", -1) == -2 and L.lookupffn_set_option(b"hash_blocks", 0) == 0
    assert L.lookupffn_set_option(b"slice_lanes", 4) == 0 and L.lookupffn_set_option(b"slice_lanes", 3) == -2
    assert L.lookupffn_set_option(b"slice_lanes", 0) == 0
    assert L.lookupffn_set_option(b"token_slots", 8) == 0 and L.lookupffn_set_option(b"token_slots", 33) == -2
    assert L.lookupffn_set_option(b"ring_threads", 512) == 0 and L.lookupffn_set_option(b"ring_threads", 256) == -2
    assert L.lookupffn_set_option(b"ring_threads", 0) == 0
    assert L.lookupffn_set_option(b"token_slots", 0) == 0
    assert L.lookupffn_set_option(b"small_tokens", -1) == 0 and L.lookupffn_set_option(b"small_tokens", -2) == -2
    assert L.lookupffn_set_option(b"small_tokens", 256) == 0 and L.lookupffn_set_option(b"small_tokens", 0) == 0
    assert L.lookupffn_set_option(b"no_such_key", 1) == -2
    assert L.lookupffn_set_option(None, 1) == -1


def test_binding_refuses_cpu_tensors():
    import torch
    x = torch.zeros(4, 64)
    signs = torch.ones(1, 2, 64, dtype=torch.int8)
    with pytest.raises(ValueError):
        binding.lookupffn_hash(x, signs, 8, 8, codes=torch.zeros(4, 8, dtype=torch.int16))


def test_kernel_argument_structs_are_value_initialised():
    """Every kernel-argument struct the host code fills starts zeroed: a field that one call path forgets
    is then 0 / NULL in the kernel, never stack garbage (a run-time mode flag left unset once sent a
    weighted gather down the multi-probe branch, which reads 1 + tau floats per table from a one-float
    buffer)."""
    src = (ROOT / "paper_2403_07221_amd" / "csrc" / "lookupffn.hip").read_text()
    names = set(re.findall(r"\bstruct (\w+Args)\b", "".join(
        (ROOT / "paper_2403_07221_amd" / "csrc" / f).read_text()
        for f in ("hash_kernel.hpp", "bh_hash_kernel.hpp", "gather_kernel.hpp", "gather_lds_kernel.hpp",
                  "gather_ring_kernel.hpp", "forward_stack_kernel.hpp"))))
    assert {"HashArgs", "BhArgs", "GatherArgs", "GatherLdsArgs", "GatherRingArgs", "StackArgs"} <= names
    decl = re.compile(r"^\s*(?:%s)\s+\w+\s*;" % "|".join(sorted(names)), re.M)
    assert decl.findall(src) == []
    assert len(re.findall(r"^\s*(?:%s)\s+\w+\{\};" % "|".join(sorted(names)), src, re.M)) >= 8
