"""Per-head influence metric of the plan search -- TEST INFRASTRUCTURE, not the product.

Sec. 3.4.1, Eq. 1 of DiTFastAttnV2, as Alg. 1 uses it (Influence[h, m] = RSE(O[h], O'[h])): for one
head, the squared error of the method's attention output y_m against the original output y_o,
relative to the spread of y_o about its own mean,

    I = sum (y_m - y_o)^2 / sum (y_o - mean(y_o))^2,

all three sums over every element the head owns (batch entries, tokens, features).  The printed
equation has mean(y_o) in the numerator too; with that reading a perfect method (y_m = y_o) would
score 1 instead of 0, so the numerator is read as the error against y_o.

Plain numpy in fp64, two passes (mean first), no blocking.  Nothing in the product path may import
this module.
"""
import numpy as np


def head_rse(y_m, y_o):
    """y_m, y_o: arrays [B, H, N, D] (any float dtype, or torch CPU tensors).  Returns float64 [H]."""
    ym = _to_f64(y_m)
    yo = _to_f64(y_o)
    assert ym.shape == yo.shape and ym.ndim == 4
    H = ym.shape[1]
    out = np.empty(H, dtype=np.float64)
    for h in range(H):
        a = ym[:, h].reshape(-1)
        b = yo[:, h].reshape(-1)
        mean = b.sum() / b.size
        num = ((a - b) ** 2).sum()
        den = ((b - mean) ** 2).sum()
        out[h] = num / den
    return out


def _to_f64(x):
    if hasattr(x, "detach"):            # torch tensor (bf16 has no numpy dtype: widen first)
        return x.detach().double().cpu().numpy()
    return np.asarray(x, dtype=np.float64)
