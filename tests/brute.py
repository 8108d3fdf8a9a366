"""Float64 numpy brute-force definitions used to pin the oracle.  None of them is tiled or online:
they work on the full N x N score matrix, so they share no structure with the oracle's recurrences."""
import numpy as np


def widen(bits):
    """uint16 bf16 bit patterns -> float64."""
    return (bits.astype(np.uint32) << 16).view(np.float32).astype(np.float64)


def scores(q, k):
    """S = Q K^T / sqrt(d) (paper eq. 1) for [N,d] float64 operands."""
    return q @ k.T / np.sqrt(q.shape[1])


def dense_attention(q, k, v, col_live=None):
    """softmax(S) V (paper eqs. 1-3); `col_live` [N,N] bool removes entries from numerator and denominator."""
    s = scores(q, k)
    if col_live is not None:
        s = np.where(col_live, s, -np.inf)
    with np.errstate(invalid="ignore"):                                  # a row with no live column (mutants only)
        s = s - s.max(axis=1, keepdims=True)
    p = np.exp(s)
    return (p / p.sum(axis=1, keepdims=True)) @ v


def expand_tiles(live, tq, tk, n):
    """[Tq,Tk] bool per tile -> [N,N] bool per element."""
    return np.repeat(np.repeat(live, tq, axis=0), tk, axis=1)[:n, :n]


def predicate_values(q, k, entry_mask, tq, tk, visit=None):
    """g_ij of eq. (sparge_cond) for every tile live on entry, from the dense S: R[r,j] = max of S over
    the columns of tile j; the cumulative max m_ij is the max of R over live tiles up to j; g_ij is the
    max over the tile's rows of R[r,j] - m_ij[r].  NaN for tiles skipped on entry."""
    n = q.shape[0]
    s = scores(q, k)
    Tq, Tk = -(-n // tq), -(-n // tk)
    R = np.full((n, Tk), -np.inf)
    for j in range(Tk):
        R[:, j] = s[:, j * tk:(j + 1) * tk].max(axis=1)
    g = np.full((Tq, Tk), np.nan)
    for i in range(Tq):
        rows = slice(i * tq, min(n, (i + 1) * tq))
        order = np.arange(Tk) if visit is None else np.asarray(visit[i])  # the cumulative max follows the visiting order
        Ri = np.where(entry_mask[i][None, :] != 0, -np.inf, R[rows])[:, order]   # skipped tiles are never seen
        cum = np.maximum.accumulate(Ri, axis=1)
        with np.errstate(invalid="ignore"):                              # -inf - -inf on skipped tiles
            diff = (Ri - cum).max(axis=0)
        g[i, order] = np.where(entry_mask[i][order] != 0, np.nan, diff)
    return g
