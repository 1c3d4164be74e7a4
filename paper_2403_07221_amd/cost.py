"""Analytic per-token cost model: the paper's FLOP accounting and this path's bytes.

The FLOP side follows how the paper counts operations of one token (Sec. 4,
"FLOPs are estimated as the number of floating operations of processing a
single instance") and reproduces every MFLOP value its tables print; that is
also the only evidence in the paper for how widths that are not a power of two
are handled: pad d to the next power of two and take ceil(h*tau/d_pad)
independent projections.

The byte side is what one launch of the forward pass must move at minimum:
each token's x once, its k selected table rows once, its y once.
"""
from __future__ import annotations

from math import log2


def d_pad(d: int) -> int:
    p = 1
    while p < d:
        p <<= 1
    return p


def n_proj(d: int, h: int, tau: int) -> int:
    return -(-h * tau // d_pad(d))


def vanilla_ffn_flops(d: int, hidden: int | None = None) -> int:
    """Two GEMVs d x hidden and hidden x d, multiply + add each (Sec. 2.1, eq. "ffn")."""
    hidden = 4 * d if hidden is None else hidden
    return 2 * 2 * d * hidden


def hash_flops(d: int, h: int, tau: int, projection: str, block: int = 64, factors: int = 4,
               n_rounds: int = 3) -> int:
    """FLOP of the Hash step for one token.

    dense : x R with R a d x (h*tau) matrix (Sec. 3.2, "The problem")
    bh4   : `factors` block-diagonal x Hadamard factors per projection (Sec. 3.2, eq. "block_acdc")
    hd    : `n_rounds` sign-diagonal x Hadamard rounds per projection (Sec. 3.2, eq. "hadamard"),
            the hash this library computes
    """
    dp, P = d_pad(d), n_proj(d, h, tau)
    if projection == "dense":
        return 2 * h * tau * d
    if projection == "bh4":
        return P * factors * (2 * dp * block + dp * int(log2(dp)))
    if projection == "hd":
        return P * n_rounds * (dp + dp * int(log2(dp)))
    raise ValueError(projection)


def gather_flops(d_out: int, h: int, weighted: bool = True) -> int:
    """One row per table: a multiply-add per element when weighted (Sec. 4), an add otherwise."""
    return (2 if weighted else 1) * h * d_out


def paper_mflop(d: int, h: int, tau: int, projection: str, block: int, part: str) -> float:
    """The quantity the paper's tables print, in MFLOP."""
    if projection == "vanilla":
        return vanilla_ffn_flops(d) / 1e6
    hs = hash_flops(d, h, tau, projection, block)
    g = gather_flops(d, h, weighted=True)
    return {"hash": hs, "gather": g, "total": hs + g}[part] / 1e6


def bytes_per_token(d: int, k: int, d_out: int, x_bytes: int = 4, table_bytes: int = 4,
                    y_bytes: int = 4) -> int:
    """Algorithmic bytes one token moves: x row + k table rows + y row."""
    return d * x_bytes + k * d_out * table_bytes + d_out * y_bytes


def flops_per_token(d: int, k: int, tau: int, d_out: int, n_rounds: int) -> int:
    """Algorithmic FLOP of this library's path for one token (sign-diagonal hash, plain sum)."""
    return hash_flops(d, k, tau, "hd", n_rounds=n_rounds) + gather_flops(d_out, k, weighted=False)
