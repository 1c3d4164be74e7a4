"""Which tokens a full-size parity test compares with the oracle."""
import numpy as np


def sample_tokens(n: int, step: int, edge: int = 300) -> np.ndarray:
    """Every `step`-th token plus the first and last `edge` tokens.

    `step` must be odd: the kernels map tokens to lanes, token slots and workgroups in
    power-of-two strides (4, 8, 128, 512, 1024 ...), so a power-of-two sample would only ever
    visit some of the lanes and slots; an odd step visits all of them.  The edges cover the
    first and the ragged last chunk of every workgroup split.
    """
    assert step % 2 == 1, "use an odd step: power-of-two steps alias with the kernels' token maps"
    idx = np.concatenate([np.arange(0, n, step), np.arange(0, min(edge, n)), np.arange(max(0, n - edge), n)])
    return np.unique(idx)
