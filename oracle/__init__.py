"""CPU oracle for the LookupFFN forward pass -- TEST INFRASTRUCTURE ONLY.

Thin ctypes loader around ``lookupffn_oracle.c`` (plain C, fp32 hash as the
paper's precision, fp64 reference accumulation for the gather).  Only tests,
the smoke check and the bench's ``cpu_baseline`` leg may import this package;
the GPU library never does and shares no code with it.

numpy conventions: fp32 data are ``float32`` arrays; bf16 data are ``uint16``
arrays holding the raw bf16 bit patterns; IEEE half data are ``float16`` arrays.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from pathlib import Path

import numpy as np

_HERE = Path(__file__).resolve().parent
_SRC = _HERE / "lookupffn_oracle.c"
_LIB = _HERE / "liblookupffn_oracle.so"
CFLAGS = ["-O2", "-std=c11", "-ffp-contract=off", "-fno-fast-math", "-fopenmp",
          "-shared", "-fPIC", "-Wall", "-Wextra"]
# fmaf() is exact either way; with the FMA instruction set it is one instruction instead of a
# software routine (explicit fmaf calls only: -ffp-contract=off still keeps a*b+c unfused)
try:
    if " fma " in open("/proc/cpuinfo").read():
        CFLAGS.append("-mfma")
except OSError:
    pass

F32, BF16, F16 = 0, 1, 2
_lib = None


def build(force: bool = False) -> Path:
    """Compile the oracle with gcc (no GPU toolchain involved)."""
    if force or not _LIB.exists() or _LIB.stat().st_mtime < _SRC.stat().st_mtime:
        tmp = _LIB.with_suffix(f".so.tmp{os.getpid()}")
        subprocess.run(["gcc", *CFLAGS, "-o", str(tmp), str(_SRC), "-lm"], check=True)
        os.replace(tmp, _LIB)
    return _LIB


def lib() -> ctypes.CDLL:
    global _lib
    if _lib is None:
        build()
        L = ctypes.CDLL(str(_LIB))
        vp, i64, ci = ctypes.c_void_p, ctypes.c_int64, ctypes.c_int
        L.oracle_d_pad.argtypes = [ci]
        L.oracle_n_proj.argtypes = [ci, ci, ci]
        L.oracle_fwht.argtypes = [vp, ci]
        L.oracle_fwht.restype = None
        L.oracle_set_threads.argtypes = [ci]
        L.oracle_set_threads.restype = None
        L.oracle_soft_codes.argtypes = [vp, ci, vp, vp, i64, ci, ci, ci, ci]
        L.oracle_hash.argtypes = [vp, ci, vp, vp, i64, ci, ci, ci, ci]
        L.oracle_gather.argtypes = [vp, vp, ci, vp, i64, ci, ci, ci, ci]
        L.oracle_forward.argtypes = [vp, ci, vp, vp, ci, vp, vp, i64, ci, ci, ci, ci, ci, ci]
        L.oracle_bh_hash.argtypes = [vp, ci, vp, vp, vp, i64, ci, ci, ci, ci, ci]
        L.oracle_bh_forward.argtypes = [vp, ci, vp, vp, ci, vp, vp, i64, ci, ci, ci, ci, ci, ci, ci]
        L.oracle_probe_weights_from_z.argtypes = [vp, i64, vp, vp, i64, ci, ci]
        L.oracle_gather_probes.argtypes = [vp, vp, vp, ci, vp, i64, ci, ci, ci]
        L.oracle_forward_probes.argtypes = [vp, ci, vp, vp, ci, vp, vp, vp, i64, ci, ci, ci, ci, ci]
        L.oracle_weights_from_z.argtypes = [vp, i64, vp, i64, ci, ci]
        L.oracle_weights.argtypes = [vp, ci, vp, vp, i64, ci, ci, ci, ci]
        L.oracle_gather_weighted.argtypes = [vp, vp, vp, ci, vp, i64, ci, ci, ci]
        L.oracle_forward_weighted.argtypes = [vp, ci, vp, vp, ci, vp, vp, vp, i64, ci, ci, ci, ci, ci]
        for name in ("oracle_half_to_float", "oracle_float_to_bf16", "oracle_float_to_half"):
            getattr(L, name).argtypes = [vp, vp, i64]
            getattr(L, name).restype = None
        _lib = L
    return _lib


def _dtype_code(a: np.ndarray) -> int:
    if a.dtype == np.float32:
        return F32
    if a.dtype == np.uint16:
        return BF16
    if a.dtype == np.float16:
        return F16
    raise TypeError(f"oracle takes float32, uint16 (raw bf16) or float16 arrays, got {a.dtype}")


def _ptr(a: np.ndarray):
    assert a.flags["C_CONTIGUOUS"]
    return a.ctypes.data_as(ctypes.c_void_p)


def _check(rc: int, what: str):
    if rc != 0:
        raise ValueError(f"oracle {what} failed with code {rc}")


def d_pad(d: int) -> int:
    return lib().oracle_d_pad(d)


def n_proj(d: int, k: int, tau: int) -> int:
    return lib().oracle_n_proj(d, k, tau)


def max_threads() -> int:
    return lib().oracle_max_threads()


def set_threads(n: int) -> None:
    lib().oracle_set_threads(n)


def half_to_float(bits: np.ndarray) -> np.ndarray:
    """Values of IEEE binary16 bit patterns (uint16), as float32."""
    bits = np.ascontiguousarray(bits, dtype=np.uint16)
    out = np.empty(bits.shape, dtype=np.float32)
    lib().oracle_half_to_float(_ptr(bits), _ptr(out), bits.size)
    return out


def float_to_bf16(f: np.ndarray) -> np.ndarray:
    """fp32 -> raw bf16 bit patterns (uint16), round to nearest even."""
    f = np.ascontiguousarray(f, dtype=np.float32)
    out = np.empty(f.shape, dtype=np.uint16)
    lib().oracle_float_to_bf16(_ptr(f), _ptr(out), f.size)
    return out


def float_to_half(f: np.ndarray) -> np.ndarray:
    """fp32 -> IEEE binary16 bit patterns (uint16), round to nearest even."""
    f = np.ascontiguousarray(f, dtype=np.float32)
    out = np.empty(f.shape, dtype=np.uint16)
    lib().oracle_float_to_half(_ptr(f), _ptr(out), f.size)
    return out


def fwht(v: np.ndarray) -> np.ndarray:
    """Unnormalised Sylvester-order Walsh-Hadamard transform of a 1-D float32 vector."""
    out = np.ascontiguousarray(v, dtype=np.float32).copy()
    n = out.shape[0]
    assert out.ndim == 1 and n >= 1 and n & (n - 1) == 0
    lib().oracle_fwht(_ptr(out), n)
    return out


def _check_signs(signs: np.ndarray, d: int, k: int, tau: int, n_rounds: int):
    assert signs.dtype == np.int8
    assert signs.shape == (n_proj(d, k, tau), n_rounds, d_pad(d)), signs.shape


def soft_codes(x: np.ndarray, signs: np.ndarray, k: int, tau: int) -> np.ndarray:
    """z = x R, shape [n, P*d_pad] float32."""
    n, d = x.shape
    n_rounds = signs.shape[1]
    _check_signs(signs, d, k, tau, n_rounds)
    x = np.ascontiguousarray(x)
    signs = np.ascontiguousarray(signs)
    z = np.empty((n, signs.shape[0] * signs.shape[2]), dtype=np.float32)
    _check(lib().oracle_soft_codes(_ptr(x), _dtype_code(x), _ptr(signs), _ptr(z),
                                   n, d, k, tau, n_rounds), "soft_codes")
    return z


def hash_codes(x: np.ndarray, signs: np.ndarray, k: int, tau: int) -> np.ndarray:
    """codes[n, k] uint16."""
    n, d = x.shape
    n_rounds = signs.shape[1]
    _check_signs(signs, d, k, tau, n_rounds)
    x = np.ascontiguousarray(x)
    signs = np.ascontiguousarray(signs)
    codes = np.empty((n, k), dtype=np.uint16)
    _check(lib().oracle_hash(_ptr(x), _dtype_code(x), _ptr(signs), _ptr(codes),
                             n, d, k, tau, n_rounds), "hash")
    return codes


def gather(codes: np.ndarray, tables: np.ndarray, acc64: bool = True) -> np.ndarray:
    """y[n, d_out] float32 = sum_j tables[j, codes[:, j], :]."""
    n, k = codes.shape
    k2, rows, d_out = tables.shape
    tau = rows.bit_length() - 1
    assert k2 == k and 1 << tau == rows and codes.dtype == np.uint16
    codes = np.ascontiguousarray(codes)
    tables = np.ascontiguousarray(tables)
    y = np.empty((n, d_out), dtype=np.float32)
    _check(lib().oracle_gather(_ptr(codes), _ptr(tables), _dtype_code(tables), _ptr(y),
                               n, k, tau, d_out, int(acc64)), "gather")
    return y


def forward(x: np.ndarray, signs: np.ndarray, tables: np.ndarray, acc64: bool = True,
            return_codes: bool = False):
    """Whole forward pass; y[n, d_out] float32 (and codes[n, k] uint16 on request)."""
    n, d = x.shape
    k, rows, d_out = tables.shape
    tau = rows.bit_length() - 1
    assert 1 << tau == rows
    n_rounds = signs.shape[1]
    _check_signs(signs, d, k, tau, n_rounds)
    x = np.ascontiguousarray(x)
    signs = np.ascontiguousarray(signs)
    tables = np.ascontiguousarray(tables)
    y = np.empty((n, d_out), dtype=np.float32)
    codes = np.empty((n, k), dtype=np.uint16)
    _check(lib().oracle_forward(_ptr(x), _dtype_code(x), _ptr(signs), _ptr(tables),
                                _dtype_code(tables), _ptr(y), _ptr(codes), n, d, k, tau,
                                d_out, n_rounds, int(acc64)), "forward")
    return (y, codes) if return_codes else y


# ---- weighted variant (Sec. 4 of the paper) ---------------------------------------------------

def weights_from_z(z: np.ndarray, k: int, tau: int) -> np.ndarray:
    """w[n, k] float64 from soft codes z[n, >= k*tau] float32."""
    z = np.ascontiguousarray(z, dtype=np.float32)
    n, zs = z.shape
    w = np.empty((n, k), dtype=np.float64)
    _check(lib().oracle_weights_from_z(_ptr(z), zs, _ptr(w), n, k, tau), "weights_from_z")
    return w


def weights(x: np.ndarray, signs: np.ndarray, k: int, tau: int) -> np.ndarray:
    """w[n, k] float64 for tokens x[n, d]."""
    n, d = x.shape
    n_rounds = signs.shape[1]
    _check_signs(signs, d, k, tau, n_rounds)
    x = np.ascontiguousarray(x)
    signs = np.ascontiguousarray(signs)
    w = np.empty((n, k), dtype=np.float64)
    _check(lib().oracle_weights(_ptr(x), _dtype_code(x), _ptr(signs), _ptr(w), n, d, k, tau, n_rounds), "weights")
    return w


def gather_weighted(codes: np.ndarray, w: np.ndarray, tables: np.ndarray) -> np.ndarray:
    """y[n, d_out] float32 = sum_j w[:, j] * tables[j, codes[:, j], :] (fp64 accumulation)."""
    n, k = codes.shape
    k2, rows, d_out = tables.shape
    tau = rows.bit_length() - 1
    assert k2 == k and 1 << tau == rows and codes.dtype == np.uint16 and w.shape == (n, k)
    codes = np.ascontiguousarray(codes)
    w = np.ascontiguousarray(w, dtype=np.float64)
    tables = np.ascontiguousarray(tables)
    y = np.empty((n, d_out), dtype=np.float32)
    _check(lib().oracle_gather_weighted(_ptr(codes), _ptr(w), _ptr(tables), _dtype_code(tables), _ptr(y),
                                        n, k, tau, d_out), "gather_weighted")
    return y


def forward_weighted(x: np.ndarray, signs: np.ndarray, tables: np.ndarray, return_all: bool = False):
    """Whole weighted forward pass; y[n, d_out] float32 (and codes, weights on request)."""
    n, d = x.shape
    k, rows, d_out = tables.shape
    tau = rows.bit_length() - 1
    assert 1 << tau == rows
    n_rounds = signs.shape[1]
    _check_signs(signs, d, k, tau, n_rounds)
    x = np.ascontiguousarray(x)
    signs = np.ascontiguousarray(signs)
    tables = np.ascontiguousarray(tables)
    y = np.empty((n, d_out), dtype=np.float32)
    codes = np.empty((n, k), dtype=np.uint16)
    w = np.empty((n, k), dtype=np.float64)
    _check(lib().oracle_forward_weighted(_ptr(x), _dtype_code(x), _ptr(signs), _ptr(tables), _dtype_code(tables),
                                         _ptr(y), _ptr(codes), _ptr(w), n, d, k, tau, d_out, n_rounds),
           "forward_weighted")
    return (y, codes, w) if return_all else y


# ---- BH4 hash (Sec. 3.2, eq. "block_acdc") -----------------------------------------------------

def _check_bmats(bmats: np.ndarray, d: int, k: int, tau: int):
    assert bmats.dtype == np.float32 and bmats.ndim == 5, "bmats must be float32 [P][m][d_pad/b][b][b]"
    P, m, nb, b, b2 = bmats.shape
    assert b == b2 and nb * b == d_pad(d) and P == n_proj(d, k, tau), bmats.shape
    return b, m


def bh_soft_codes(x: np.ndarray, bmats: np.ndarray, k: int, tau: int) -> np.ndarray:
    """z = x R with R = prod_i B_i H per projection; z[n, P*d_pad] float32."""
    n, d = x.shape
    b, m = _check_bmats(bmats, d, k, tau)
    x, bmats = np.ascontiguousarray(x), np.ascontiguousarray(bmats)
    z = np.empty((n, bmats.shape[0] * d_pad(d)), dtype=np.float32)
    _check(lib().oracle_bh_hash(_ptr(x), _dtype_code(x), _ptr(bmats), _ptr(z), None, n, d, k, tau, b, m), "bh_soft_codes")
    return z


def bh_hash_codes(x: np.ndarray, bmats: np.ndarray, k: int, tau: int) -> np.ndarray:
    """codes[n, k] uint16 of the BH hash."""
    n, d = x.shape
    b, m = _check_bmats(bmats, d, k, tau)
    x, bmats = np.ascontiguousarray(x), np.ascontiguousarray(bmats)
    codes = np.empty((n, k), dtype=np.uint16)
    _check(lib().oracle_bh_hash(_ptr(x), _dtype_code(x), _ptr(bmats), None, _ptr(codes), n, d, k, tau, b, m), "bh_hash")
    return codes


def bh_forward(x: np.ndarray, bmats: np.ndarray, tables: np.ndarray, acc64: bool = True, return_codes: bool = False):
    """Whole forward pass with the BH hash; y[n, d_out] float32."""
    n, d = x.shape
    k, rows, d_out = tables.shape
    tau = rows.bit_length() - 1
    assert 1 << tau == rows
    b, m = _check_bmats(bmats, d, k, tau)
    x, bmats, tables = np.ascontiguousarray(x), np.ascontiguousarray(bmats), np.ascontiguousarray(tables)
    y = np.empty((n, d_out), dtype=np.float32)
    codes = np.empty((n, k), dtype=np.uint16)
    _check(lib().oracle_bh_forward(_ptr(x), _dtype_code(x), _ptr(bmats), _ptr(tables), _dtype_code(tables), _ptr(y),
                                   _ptr(codes), n, d, k, tau, d_out, b, m, int(acc64)), "bh_forward")
    return (y, codes) if return_codes else y


def bh_forward_weighted(x: np.ndarray, bmats: np.ndarray, tables: np.ndarray, return_all: bool = False):
    """BH hash (Sec. 3.2) followed by the weighted gather (Sec. 4): the weights come from the z of the BH
    hash.  A chain of bh_soft_codes / bh_hash_codes, weights_from_z and gather_weighted, nothing more."""
    k, rows, d_out = tables.shape
    tau = rows.bit_length() - 1
    assert 1 << tau == rows
    z = bh_soft_codes(x, bmats, k, tau)
    codes = bh_hash_codes(x, bmats, k, tau)
    w = weights_from_z(z, k, tau)
    y = gather_weighted(codes, w, tables)
    return (y, codes, w) if return_all else y


# ---- multi-probe lookup (Sec. 3.1, eq. "partial_softmax", neighbourhood of l0 radius 1) ---------

def probe_weights_from_z(z: np.ndarray, k: int, tau: int):
    """(codes[n, k] uint16, p[n, k, 1+tau] float64) from soft codes z[n, >= k*tau] float32."""
    z = np.ascontiguousarray(z, dtype=np.float32)
    n, zs = z.shape
    codes = np.empty((n, k), dtype=np.uint16)
    p = np.empty((n, k, tau + 1), dtype=np.float64)
    _check(lib().oracle_probe_weights_from_z(_ptr(z), zs, _ptr(codes), _ptr(p), n, k, tau), "probe_weights_from_z")
    return codes, p


def gather_probes(codes: np.ndarray, p: np.ndarray, tables: np.ndarray) -> np.ndarray:
    """y[n, d_out] = sum_j sum_probe p[:, j, probe] * tables[j, row(probe), :]."""
    n, k = codes.shape
    k2, rows, d_out = tables.shape
    tau = rows.bit_length() - 1
    assert k2 == k and 1 << tau == rows and codes.dtype == np.uint16 and p.shape == (n, k, tau + 1)
    codes, tables = np.ascontiguousarray(codes), np.ascontiguousarray(tables)
    p = np.ascontiguousarray(p, dtype=np.float64)
    y = np.empty((n, d_out), dtype=np.float32)
    _check(lib().oracle_gather_probes(_ptr(codes), _ptr(p), _ptr(tables), _dtype_code(tables), _ptr(y), n, k, tau,
                                      d_out), "gather_probes")
    return y


def forward_probes(x: np.ndarray, signs: np.ndarray, tables: np.ndarray, return_all: bool = False):
    """Whole multi-probe forward pass; y[n, d_out] float32 (and codes, probe weights on request)."""
    n, d = x.shape
    k, rows, d_out = tables.shape
    tau = rows.bit_length() - 1
    assert 1 << tau == rows
    n_rounds = signs.shape[1]
    _check_signs(signs, d, k, tau, n_rounds)
    x, signs, tables = np.ascontiguousarray(x), np.ascontiguousarray(signs), np.ascontiguousarray(tables)
    y = np.empty((n, d_out), dtype=np.float32)
    codes = np.empty((n, k), dtype=np.uint16)
    p = np.empty((n, k, tau + 1), dtype=np.float64)
    _check(lib().oracle_forward_probes(_ptr(x), _dtype_code(x), _ptr(signs), _ptr(tables), _dtype_code(tables),
                                       _ptr(y), _ptr(codes), _ptr(p), n, d, k, tau, d_out, n_rounds), "forward_probes")
    return (y, codes, p) if return_all else y
