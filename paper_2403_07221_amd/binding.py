"""ctypes binding of the C-ABI library declared in include/lookupffn.h.

Argument marshalling only: every function takes torch CUDA tensors (used for
device memory and streams), checks dtypes/contiguity, and passes raw device
pointers to the entry point of the same name.  There is no fallback: if the
shared library has not been built the first call raises.
"""
from __future__ import annotations

import ctypes
from pathlib import Path

import torch

_LIB_PATH = Path(__file__).resolve().parent / "liblookupffn.so"
_lib = None

F32, BF16, F16 = 0, 1, 2
Y_BF16, Y_F16 = 0x200, 0x400   # OR-ed into table_dtype: y is stored in 16 bits
PREPARED = 0x100   # OR-ed into table_dtype / block: the buffer is a prepared copy (see include/lookupffn.h)
EXPORTS = (
    "lookupffn_init",
    "lookupffn_hash", "lookupffn_gather", "lookupffn_forward", "lookupffn_workspace_bytes",
    "lookupffn_forward_static", "lookupffn_static_scratch_bytes", "lookupffn_forward_stack",
    "lookupffn_workspace_bytes_gather", "lookupffn_prepared_tables_bytes", "lookupffn_prepare_tables",
    "lookupffn_release_workspace", "lookupffn_timing_enable", "lookupffn_timing_reset",
    "lookupffn_timing_read", "lookupffn_timing_read_each", "lookupffn_set_option", "lookupffn_strerror",
    "lookupffn_last_hip_error", "lookupffn_last_gather_kernel", "lookupffn_last_hash_kernel", "lookupffn_version",
    "lookupffn_hash_weighted", "lookupffn_gather_weighted", "lookupffn_forward_weighted",
    "lookupffn_workspace_bytes_weighted", "lookupffn_workspace_bytes_gather_weighted",
    "lookupffn_prepared_bh_bytes", "lookupffn_prepare_bh",
    "lookupffn_hash_bh", "lookupffn_forward_bh", "lookupffn_workspace_bytes_bh",
    "lookupffn_hash_bh_weighted", "lookupffn_forward_bh_weighted", "lookupffn_workspace_bytes_bh_weighted",
    "lookupffn_hash_probes", "lookupffn_gather_probes", "lookupffn_forward_probes",
    "lookupffn_workspace_bytes_probes", "lookupffn_workspace_bytes_gather_probes",
)


class LookupFFNError(RuntimeError):
    def __init__(self, status: int, text: str):
        super().__init__(f"lookupffn status {status}: {text}")
        self.status = status


def lib() -> ctypes.CDLL:
    """Load liblookupffn.so (built by paper_2403_07221_amd.build); raises if it is missing."""
    global _lib
    if _lib is None:
        if not _LIB_PATH.exists():
            raise FileNotFoundError(
                f"{_LIB_PATH} not found: build it with `python -m paper_2403_07221_amd.build` "
                "(there is no CPU fallback)")
        L = ctypes.CDLL(str(_LIB_PATH))
        vp, i64, ci = ctypes.c_void_p, ctypes.c_int64, ctypes.c_int
        L.lookupffn_hash.argtypes = [vp, vp, vp, i64, ci, ci, ci, ci, ci, vp]
        L.lookupffn_gather.argtypes = [vp, vp, vp, i64, ci, ci, ci, ci, vp, i64, vp]
        L.lookupffn_forward.argtypes = [vp, vp, vp, vp, i64, ci, ci, ci, ci, ci, ci, ci, vp, i64, vp]
        L.lookupffn_forward_static.argtypes = [vp, vp, vp, vp, i64, ci, ci, ci, ci, ci, ci, ci, vp]
        L.lookupffn_static_scratch_bytes.restype = i64
        L.lookupffn_forward_stack.argtypes = [vp, ctypes.POINTER(vp), ctypes.POINTER(vp), vp, i64,
                                              ci, ci, ci, ci, ci, ci, ci, ci, vp]
        L.lookupffn_hash_weighted.argtypes = [vp, vp, vp, vp, i64, ci, ci, ci, ci, ci, vp]
        L.lookupffn_gather_weighted.argtypes = [vp, vp, vp, vp, i64, ci, ci, ci, ci, vp, i64, vp]
        L.lookupffn_forward_weighted.argtypes = L.lookupffn_forward.argtypes
        L.lookupffn_hash_probes.argtypes = L.lookupffn_hash_weighted.argtypes
        L.lookupffn_gather_probes.argtypes = L.lookupffn_gather_weighted.argtypes
        L.lookupffn_forward_probes.argtypes = L.lookupffn_forward.argtypes
        for name, args in (("lookupffn_workspace_bytes", [i64, ci]), ("lookupffn_workspace_bytes_gather", [i64, ci]),
                           ("lookupffn_workspace_bytes_weighted", [i64, ci]),
                           ("lookupffn_workspace_bytes_gather_weighted", [i64, ci]),
                           ("lookupffn_workspace_bytes_probes", [i64, ci, ci]),
                           ("lookupffn_workspace_bytes_gather_probes", [i64, ci, ci]),
                           ("lookupffn_workspace_bytes_bh", [i64, ci, ci, ci, ci, ci]),
                           ("lookupffn_workspace_bytes_bh_weighted", [i64, ci, ci, ci, ci, ci]),
                           ("lookupffn_prepared_tables_bytes", [ci, ci, ci, ci]),
                           ("lookupffn_prepared_bh_bytes", [ci, ci, ci, ci, ci])):
            getattr(L, name).argtypes = args
            getattr(L, name).restype = i64
        L.lookupffn_prepare_tables.argtypes = [vp, ci, ci, ci, ci, vp, i64, vp]
        L.lookupffn_prepare_bh.argtypes = [vp, ci, ci, ci, ci, ci, vp, i64, vp]
        L.lookupffn_hash_bh.argtypes = [vp, vp, vp, i64, ci, ci, ci, ci, ci, ci, vp, i64, vp]
        L.lookupffn_forward_bh.argtypes = [vp, vp, vp, vp, i64, ci, ci, ci, ci, ci, ci, ci, ci, vp, i64, vp]
        L.lookupffn_hash_bh_weighted.argtypes = [vp, vp, vp, vp, i64, ci, ci, ci, ci, ci, ci, vp, i64, vp]
        L.lookupffn_forward_bh_weighted.argtypes = L.lookupffn_forward_bh.argtypes
        L.lookupffn_timing_enable.argtypes = [ci]
        L.lookupffn_timing_read.argtypes = [ci, ctypes.POINTER(ctypes.c_double), ctypes.POINTER(i64)]
        L.lookupffn_timing_read_each.argtypes = [ci, ctypes.POINTER(ctypes.c_double), i64, ctypes.POINTER(i64)]
        L.lookupffn_set_option.argtypes = [ctypes.c_char_p, ci]
        L.lookupffn_strerror.argtypes = [ci]
        L.lookupffn_strerror.restype = ctypes.c_char_p
        L.lookupffn_last_hip_error.restype = ctypes.c_char_p
        L.lookupffn_last_gather_kernel.restype = ctypes.c_char_p
        L.lookupffn_last_hash_kernel.restype = ctypes.c_char_p
        _lib = L
    return _lib


def _check(status: int):
    if status != 0:
        L = lib()
        text = L.lookupffn_strerror(status).decode()
        if status == -8:
            text += " (" + L.lookupffn_last_hip_error().decode() + ")"
        raise LookupFFNError(status, text)


def _dtype_code(t: torch.Tensor) -> int:
    if t.dtype == torch.float32:
        return F32
    if t.dtype == torch.bfloat16:
        return BF16
    if t.dtype == torch.float16:
        return F16
    raise TypeError(f"expected float32, bfloat16 or float16, got {t.dtype}")


def _y_flag(y: torch.Tensor) -> int:
    """table_dtype flag for the storage type of an output tensor."""
    if y.dtype == torch.float32:
        return 0
    if y.dtype == torch.bfloat16:
        return Y_BF16
    if y.dtype == torch.float16:
        return Y_F16
    raise TypeError(f"y must be float32, bfloat16 or float16, got {y.dtype}")


def _dev(t: torch.Tensor, name: str) -> int:
    if not t.is_cuda:
        raise ValueError(f"{name} must live on the GPU")
    if not t.is_contiguous():
        raise ValueError(f"{name} must be contiguous")
    return t.data_ptr()


def _stream(t: torch.Tensor) -> int:
    return torch.cuda.current_stream(t.device).cuda_stream


def _pad(d: int) -> int:
    p = 1
    while p < d:
        p <<= 1
    return p


def _check_signs(signs: torch.Tensor, d: int, k: int, tau: int):
    if signs.dtype != torch.int8 or signs.dim() != 3:
        raise TypeError("signs must be int8 [P][n_rounds][d_pad]")
    n_pad = _pad(d)
    P = -(-k * tau // n_pad)
    if signs.shape[0] != P or signs.shape[2] != n_pad:
        raise ValueError(f"signs has shape {tuple(signs.shape)}, expected ({P}, n_rounds, {n_pad})")


def _ws(workspace):
    if workspace is None:
        return None, 0
    return _dev(workspace, "workspace"), workspace.numel() * workspace.element_size()


class PreparedTables:
    """The learned tables in the layout lookupffn_prepare_tables wrote (an opaque device buffer plus the
    shape it was made from); accepted wherever a `tables` tensor is."""

    def __init__(self, buf: torch.Tensor, k: int, tau: int, d_out: int, src_dtype: int):
        self.buf, self.k, self.tau, self.d_out, self.src_dtype = buf, k, tau, d_out, src_dtype
        self.device = buf.device

    @property
    def shape(self):
        return (self.k, 1 << self.tau, self.d_out)


def _tables(tables):
    """(device pointer, k, tau, d_out, table_dtype code, device) of a tables tensor or a PreparedTables."""
    if isinstance(tables, PreparedTables):
        return _dev(tables.buf, "prepared tables"), tables.k, tables.tau, tables.d_out, PREPARED | tables.src_dtype, tables.device
    k, rows, d_out = tables.shape
    tau = rows.bit_length() - 1
    if (1 << tau) != rows:
        raise ValueError("tables must be [k, 2^tau, d_out]")
    return _dev(tables, "tables"), k, tau, d_out, _dtype_code(tables), tables.device


def lookupffn_init() -> None:
    """Registers the kernels' LDS needs with the runtime on the current device (before graph capture)."""
    _check(lib().lookupffn_init())


def lookupffn_prepared_tables_bytes(k: int, tau: int, d_out: int, table_dtype) -> int:
    code = table_dtype if isinstance(table_dtype, int) else (
        BF16 if table_dtype in ("bf16", torch.bfloat16) else F16 if table_dtype in ("f16", torch.float16) else F32)
    return lib().lookupffn_prepared_tables_bytes(k, tau, d_out, code)


def lookupffn_prepare_tables(tables: torch.Tensor, out: torch.Tensor | None = None) -> PreparedTables:
    """One-time re-layout of tables[k, 2^tau, d_out] for the gather kernels (see include/lookupffn.h)."""
    ptr, k, tau, d_out, code, dev = _tables(tables)
    need = lib().lookupffn_prepared_tables_bytes(k, tau, d_out, code)
    if out is None:
        out = torch.empty(need, dtype=torch.uint8, device=dev)
    with torch.cuda.device(dev):
        _check(lib().lookupffn_prepare_tables(ptr, k, tau, d_out, code, _dev(out, "prepared"),
                                              out.numel() * out.element_size(), _stream(tables)))
    return PreparedTables(out, k, tau, d_out, code)


def lookupffn_hash(x: torch.Tensor, signs: torch.Tensor, k: int, tau: int,
                   codes: torch.Tensor | None = None) -> torch.Tensor:
    """codes[n, k] (int16 storage of the uint16 codes) for x[n, d]."""
    n, d = x.shape
    _check_signs(signs, d, k, tau)
    if codes is None:
        codes = torch.empty((n, k), dtype=torch.int16, device=x.device)
    assert codes.dtype == torch.int16 and tuple(codes.shape) == (n, k)
    if n == 0:
        return codes            # torch gives empty tensors a NULL data pointer; nothing to launch
    with torch.cuda.device(x.device):
        _check(lib().lookupffn_hash(_dev(x, "x"), _dev(signs, "signs"), _dev(codes, "codes"), n, d, k, tau,
                                    signs.shape[1], _dtype_code(x), _stream(x)))
    return codes


def _gather(entry: str, codes, weights, tables, y, workspace, wshape):
    n, k = codes.shape
    tptr, k2, tau, d_out, tcode, dev = _tables(tables)
    if k2 != k:
        raise ValueError("tables must be [k, 2^tau, d_out] with k matching codes")
    assert codes.dtype == torch.int16
    if weights is not None:
        assert weights.dtype == torch.float32 and tuple(weights.shape) == wshape(n, k, tau)
    if y is None:
        y = torch.empty((n, d_out), dtype=torch.float32, device=dev)
    assert tuple(y.shape) == (n, d_out)
    tcode |= _y_flag(y)      # a bfloat16 / float16 y is stored in that type
    if n == 0:
        return y
    ws_ptr, ws_bytes = _ws(workspace)
    args = [_dev(codes, "codes")] + ([_dev(weights, "weights")] if weights is not None else [])
    with torch.cuda.device(dev):
        _check(getattr(lib(), entry)(*args, tptr, _dev(y, "y"), n, k, tau, d_out, tcode, ws_ptr, ws_bytes,
                                     _stream(codes)))
    return y


def lookupffn_gather(codes: torch.Tensor, tables, y: torch.Tensor | None = None,
                     workspace: torch.Tensor | None = None) -> torch.Tensor:
    """y[n, d_out] = sum_j tables[j, codes[:, j], :]; tables[k, 2^tau, d_out] float32 / bfloat16 or PreparedTables."""
    return _gather("lookupffn_gather", codes, None, tables, y, workspace, None)


def lookupffn_workspace_bytes_gather(n_tokens: int, k: int) -> int:
    return lib().lookupffn_workspace_bytes_gather(n_tokens, k)


def lookupffn_workspace_bytes_gather_weighted(n_tokens: int, k: int) -> int:
    return lib().lookupffn_workspace_bytes_gather_weighted(n_tokens, k)


def lookupffn_workspace_bytes_gather_probes(n_tokens: int, k: int, tau: int) -> int:
    return lib().lookupffn_workspace_bytes_gather_probes(n_tokens, k, tau)


def lookupffn_hash_weighted(x: torch.Tensor, signs: torch.Tensor, k: int, tau: int,
                            codes: torch.Tensor | None = None, weights: torch.Tensor | None = None):
    """(codes[n, k] int16 storage, weights[n, k] float32) of the weighted variant for x[n, d]."""
    n, d = x.shape
    _check_signs(signs, d, k, tau)
    if codes is None:
        codes = torch.empty((n, k), dtype=torch.int16, device=x.device)
    if weights is None:
        weights = torch.empty((n, k), dtype=torch.float32, device=x.device)
    assert codes.dtype == torch.int16 and tuple(codes.shape) == (n, k)
    assert weights.dtype == torch.float32 and tuple(weights.shape) == (n, k)
    if n == 0:
        return codes, weights
    with torch.cuda.device(x.device):
        _check(lib().lookupffn_hash_weighted(_dev(x, "x"), _dev(signs, "signs"), _dev(codes, "codes"),
                                             _dev(weights, "weights"), n, d, k, tau, signs.shape[1],
                                             _dtype_code(x), _stream(x)))
    return codes, weights


def lookupffn_gather_weighted(codes: torch.Tensor, weights: torch.Tensor, tables, y: torch.Tensor | None = None,
                              workspace: torch.Tensor | None = None) -> torch.Tensor:
    """y[n, d_out] = sum_j weights[:, j] * tables[j, codes[:, j], :]."""
    return _gather("lookupffn_gather_weighted", codes, weights, tables, y, workspace, lambda n, k, tau: (n, k))


def lookupffn_hash_probes(x: torch.Tensor, signs: torch.Tensor, k: int, tau: int):
    """(codes[n, k] int16 storage, shares[n, k, 1+tau] float32) of the multi-probe lookup."""
    n, d = x.shape
    _check_signs(signs, d, k, tau)
    codes = torch.empty((n, k), dtype=torch.int16, device=x.device)
    shares = torch.empty((n, k, tau + 1), dtype=torch.float32, device=x.device)
    if n == 0:
        return codes, shares
    with torch.cuda.device(x.device):
        _check(lib().lookupffn_hash_probes(_dev(x, "x"), _dev(signs, "signs"), _dev(codes, "codes"),
                                           _dev(shares, "shares"), n, d, k, tau, signs.shape[1], _dtype_code(x),
                                           _stream(x)))
    return codes, shares


def lookupffn_gather_probes(codes: torch.Tensor, shares: torch.Tensor, tables, y: torch.Tensor | None = None,
                            workspace: torch.Tensor | None = None) -> torch.Tensor:
    """y[n, d_out] = sum_j sum_probe shares[:, j, probe] * tables[j, codes[:, j] ^ flip(probe), :]."""
    return _gather("lookupffn_gather_probes", codes, shares, tables, y, workspace,
                   lambda n, k, tau: (n, k, tau + 1))


def lookupffn_workspace_bytes_probes(n_tokens: int, k: int, tau: int) -> int:
    return lib().lookupffn_workspace_bytes_probes(n_tokens, k, tau)


def lookupffn_forward_probes(x: torch.Tensor, signs: torch.Tensor, tables: torch.Tensor,
                             y: torch.Tensor | None = None, workspace: torch.Tensor | None = None) -> torch.Tensor:
    """Whole multi-probe forward pass y[n, d_out] (Sec. 3.1, eq. "partial_softmax")."""
    return lookupffn_forward(x, signs, tables, y, workspace, _entry="lookupffn_forward_probes")


def lookupffn_workspace_bytes(n_tokens: int, k: int) -> int:
    return lib().lookupffn_workspace_bytes(n_tokens, k)


def lookupffn_workspace_bytes_weighted(n_tokens: int, k: int) -> int:
    return lib().lookupffn_workspace_bytes_weighted(n_tokens, k)


def lookupffn_forward_weighted(x: torch.Tensor, signs: torch.Tensor, tables: torch.Tensor,
                               y: torch.Tensor | None = None, workspace: torch.Tensor | None = None) -> torch.Tensor:
    """Whole weighted forward pass y[n, d_out] (Sec. 4 of the paper)."""
    return lookupffn_forward(x, signs, tables, y, workspace, _entry="lookupffn_forward_weighted")


def lookupffn_forward(x: torch.Tensor, signs: torch.Tensor, tables,
                      y: torch.Tensor | None = None, workspace: torch.Tensor | None = None,
                      _entry: str = "lookupffn_forward") -> torch.Tensor:
    """Whole forward pass y[n, d_out]; `tables` a [k, 2^tau, d_out] tensor or a PreparedTables; `workspace`
    an optional uint8 CUDA tensor of lookupffn_workspace_bytes*() bytes for the intermediates."""
    n, d = x.shape
    tptr, k, tau, d_out, tcode, _ = _tables(tables)
    _check_signs(signs, d, k, tau)
    if y is None:
        y = torch.empty((n, d_out), dtype=torch.float32, device=x.device)
    assert tuple(y.shape) == (n, d_out)
    tcode |= _y_flag(y)      # a bfloat16 / float16 y is stored in that type
    if n == 0:
        return y
    ws_ptr, ws_bytes = _ws(workspace)
    with torch.cuda.device(x.device):
        _check(getattr(lib(), _entry)(_dev(x, "x"), _dev(signs, "signs"), tptr, _dev(y, "y"),
                                      n, d, k, tau, d_out, signs.shape[1], _dtype_code(x), tcode,
                                      ws_ptr, ws_bytes, _stream(x)))
    return y


def lookupffn_forward_stack(x: torch.Tensor, signs, tables, y: torch.Tensor | None = None) -> torch.Tensor:
    """Chained layers in one launch: `signs` and `tables` are sequences with one entry per layer (tables all
    tensors or all PreparedTables, same shape and dtype); returns the last layer's y[n, d_out]."""
    n, d = x.shape
    n_layers = len(signs)
    if n_layers != len(tables) or n_layers < 1:
        raise ValueError("signs and tables need one entry per layer")
    refs = [_tables(t) for t in tables]
    tptr0, k, tau, d_out, tcode, _ = refs[0]
    for (_, k_, tau_, d_out_, tcode_, _), sg in zip(refs, signs):
        if (k_, tau_, d_out_, tcode_) != (k, tau, d_out, tcode) or tuple(sg.shape) != tuple(signs[0].shape):
            raise ValueError("all layers must share one shape, dtype and layout")
        _check_signs(sg, d, k, tau)
    if y is None:
        y = torch.empty((n, d_out), dtype=torch.float32, device=x.device)
    assert tuple(y.shape) == (n, d_out)
    tcode |= _y_flag(y)      # a bfloat16 / float16 y is stored in that type
    if n == 0:
        return y
    vp = ctypes.c_void_p
    sp = (vp * n_layers)(*[_dev(sg, "signs") for sg in signs])
    tp = (vp * n_layers)(*[r[0] for r in refs])
    with torch.cuda.device(x.device):
        _check(lib().lookupffn_forward_stack(_dev(x, "x"), sp, tp, _dev(y, "y"), n, d, k, tau, d_out,
                                             signs[0].shape[1], n_layers, _dtype_code(x), tcode, _stream(x)))
    return y


def lookupffn_static_scratch_bytes() -> int:
    return lib().lookupffn_static_scratch_bytes()


def lookupffn_forward_static(x: torch.Tensor, signs: torch.Tensor, tables, y: torch.Tensor) -> torch.Tensor:
    """lookupffn_forward with the intermediates in the library's static device array: no allocation at all
    (y is the caller's).  Raises LookupFFNError(-7) when the batch needs more than that array holds."""
    n, d = x.shape
    tptr, k, tau, d_out, tcode, _ = _tables(tables)
    _check_signs(signs, d, k, tau)
    assert tuple(y.shape) == (n, d_out)
    tcode |= _y_flag(y)      # a bfloat16 / float16 y is stored in that type
    if n == 0:
        return y
    with torch.cuda.device(x.device):
        _check(lib().lookupffn_forward_static(_dev(x, "x"), _dev(signs, "signs"), tptr, _dev(y, "y"), n, d, k, tau,
                                              d_out, signs.shape[1], _dtype_code(x), tcode, _stream(x)))
    return y


class PreparedBh:
    """The block-diagonal factors in the order lookupffn_prepare_bh wrote; accepted wherever `bmats` is."""

    def __init__(self, buf: torch.Tensor, block: int, n_factors: int):
        self.buf, self.block, self.n_factors = buf, block, n_factors


def lookupffn_prepare_bh(bmats: torch.Tensor, d: int, k: int, tau: int) -> PreparedBh:
    """One-time re-ordering of the BH factors into matrix-core operand order."""
    block, m = _check_bmats(bmats, d, k, tau)
    need = lib().lookupffn_prepared_bh_bytes(d, k, tau, block, m)
    out = torch.empty(max(need, 256), dtype=torch.uint8, device=bmats.device)
    with torch.cuda.device(bmats.device):
        _check(lib().lookupffn_prepare_bh(_dev(bmats, "bmats"), d, k, tau, block, m, _dev(out, "prepared"),
                                          out.numel(), _stream(bmats)))
    return PreparedBh(out, block, m)


def _bh(bmats, d: int, k: int, tau: int):
    """(device pointer, block argument, n_factors) of a bmats tensor or a PreparedBh."""
    if isinstance(bmats, PreparedBh):
        return _dev(bmats.buf, "prepared bmats"), PREPARED | bmats.block, bmats.n_factors
    block, m = _check_bmats(bmats, d, k, tau)
    return _dev(bmats, "bmats"), block, m


def _check_bmats(bmats: torch.Tensor, d: int, k: int, tau: int):
    if bmats.dtype != torch.float32 or bmats.dim() != 5 or bmats.shape[3] != bmats.shape[4]:
        raise TypeError("bmats must be float32 [P][n_factors][d_pad/block][block][block]")
    n_pad = _pad(d)
    P = -(-k * tau // n_pad)
    block = bmats.shape[3]
    if bmats.shape[0] != P or bmats.shape[2] * block != n_pad:
        raise ValueError(f"bmats has shape {tuple(bmats.shape)}, expected ({P}, m, {n_pad}//block, block, block)")
    return block, bmats.shape[1]


def lookupffn_workspace_bytes_bh(n_tokens: int, d: int, k: int, tau: int, block: int, n_factors: int) -> int:
    return lib().lookupffn_workspace_bytes_bh(n_tokens, d, k, tau, block, n_factors)


def lookupffn_hash_bh(x: torch.Tensor, bmats, k: int, tau: int, codes: torch.Tensor | None = None,
                      workspace: torch.Tensor | None = None) -> torch.Tensor:
    """codes[n, k] of the BH hash (Sec. 3.2 of the paper); bmats[P, m, d_pad/b, b, b] float32 or a PreparedBh."""
    n, d = x.shape
    bptr, block, m = _bh(bmats, d, k, tau)
    if codes is None:
        codes = torch.empty((n, k), dtype=torch.int16, device=x.device)
    assert codes.dtype == torch.int16 and tuple(codes.shape) == (n, k)
    if n == 0:
        return codes
    ws_ptr, ws_bytes = _ws(workspace)
    with torch.cuda.device(x.device):
        _check(lib().lookupffn_hash_bh(_dev(x, "x"), bptr, _dev(codes, "codes"), n, d, k, tau, block,
                                       m, _dtype_code(x), ws_ptr, ws_bytes, _stream(x)))
    return codes


def lookupffn_forward_bh(x: torch.Tensor, bmats, tables, y: torch.Tensor | None = None,
                         workspace: torch.Tensor | None = None, _entry: str = "lookupffn_forward_bh") -> torch.Tensor:
    """Whole forward pass with the BH hash: y[n, d_out]."""
    n, d = x.shape
    tptr, k, tau, d_out, tcode, _ = _tables(tables)
    bptr, block, m = _bh(bmats, d, k, tau)
    if y is None:
        y = torch.empty((n, d_out), dtype=torch.float32, device=x.device)
    assert tuple(y.shape) == (n, d_out)
    tcode |= _y_flag(y)      # a bfloat16 / float16 y is stored in that type
    if n == 0:
        return y
    ws_ptr, ws_bytes = _ws(workspace)
    with torch.cuda.device(x.device):
        _check(getattr(lib(), _entry)(_dev(x, "x"), bptr, tptr, _dev(y, "y"),
                                      n, d, k, tau, d_out, block, m, _dtype_code(x), tcode,
                                      ws_ptr, ws_bytes, _stream(x)))
    return y


def lookupffn_workspace_bytes_bh_weighted(n_tokens: int, d: int, k: int, tau: int, block: int,
                                          n_factors: int) -> int:
    return lib().lookupffn_workspace_bytes_bh_weighted(n_tokens, d, k, tau, block, n_factors)


def lookupffn_hash_bh_weighted(x: torch.Tensor, bmats, k: int, tau: int,
                               codes: torch.Tensor | None = None, weights: torch.Tensor | None = None,
                               workspace: torch.Tensor | None = None):
    """(codes[n, k], weights[n, k]) of the BH hash with the gather weights of Sec. 4 of the paper."""
    n, d = x.shape
    bptr, block, m = _bh(bmats, d, k, tau)
    if codes is None:
        codes = torch.empty((n, k), dtype=torch.int16, device=x.device)
    if weights is None:
        weights = torch.empty((n, k), dtype=torch.float32, device=x.device)
    assert codes.dtype == torch.int16 and tuple(codes.shape) == (n, k)
    assert weights.dtype == torch.float32 and tuple(weights.shape) == (n, k)
    if n == 0:
        return codes, weights
    ws_ptr, ws_bytes = _ws(workspace)
    with torch.cuda.device(x.device):
        _check(lib().lookupffn_hash_bh_weighted(_dev(x, "x"), bptr, _dev(codes, "codes"),
                                                _dev(weights, "weights"), n, d, k, tau, block, m, _dtype_code(x),
                                                ws_ptr, ws_bytes, _stream(x)))
    return codes, weights


def lookupffn_forward_bh_weighted(x: torch.Tensor, bmats: torch.Tensor, tables: torch.Tensor,
                                  y: torch.Tensor | None = None, workspace: torch.Tensor | None = None) -> torch.Tensor:
    """Whole forward pass with the BH hash and the weighted gather: y[n, d_out]."""
    return lookupffn_forward_bh(x, bmats, tables, y, workspace, _entry="lookupffn_forward_bh_weighted")


def lookupffn_release_workspace() -> None:
    _check(lib().lookupffn_release_workspace())


def lookupffn_timing_enable(mask) -> None:
    """mask: bit 0 = time hash launches, bit 1 = time gather launches; True = both, False = off."""
    if mask is True:
        mask = 3
    _check(lib().lookupffn_timing_enable(int(mask)))


def lookupffn_timing_reset() -> None:
    _check(lib().lookupffn_timing_reset())


def lookupffn_timing_read_each(which: int) -> list[float]:
    """Milliseconds of every bracketed launch of kernel `which` since the last reset, in launch order."""
    _, cnt = lookupffn_timing_read(which)
    buf = (ctypes.c_double * max(cnt, 1))()
    got = ctypes.c_int64(0)
    _check(lib().lookupffn_timing_read_each(which, buf, cnt, ctypes.byref(got)))
    return list(buf[:min(cnt, got.value)])


def lookupffn_timing_read(which: int) -> tuple[float, int]:
    """(total milliseconds, launches) of kernel `which` (0 = hash, 1 = gather) since the last reset."""
    ms, cnt = ctypes.c_double(0), ctypes.c_int64(0)
    _check(lib().lookupffn_timing_read(which, ctypes.byref(ms), ctypes.byref(cnt)))
    return ms.value, cnt.value


def lookupffn_set_option(key: str, value: int) -> None:
    _check(lib().lookupffn_set_option(key.encode(), value))


def lookupffn_last_gather_kernel() -> str:
    return lib().lookupffn_last_gather_kernel().decode()


def lookupffn_last_hash_kernel() -> str:
    return lib().lookupffn_last_hash_kernel().decode()


def lookupffn_version() -> int:
    return lib().lookupffn_version()


# ---- helpers for moving the synthetic numpy inputs to the GPU (no arithmetic) -------------

def to_device(a, device="cuda:0") -> torch.Tensor:
    """numpy array -> CUDA tensor; uint16 arrays are raw bf16 bit patterns -> bfloat16 tensor."""
    import numpy as np
    if a.dtype == np.uint16:
        return torch.from_numpy(a.view(np.int16)).to(device).view(torch.bfloat16)
    return torch.from_numpy(a).to(device)


def codes_to_numpy(codes: torch.Tensor):
    import numpy as np
    return codes.cpu().numpy().view(np.uint16)
