"""Which rows of a full-size batch a parity test compares with the oracle.

Tokens are independent in an MoE layer, so any subset of rows can be checked exactly.  A random subset
hits the interior of the grouped GEMMs' tiles and hardly ever their borders, so the rows are picked by
PERMUTED position instead: for every expert the first and the last row of each of its m-tiles (an expert
with m rows is cut into ceil(m / BM) tiles of equal numbers of 32-row blocks, the last one ragged), then
random rows up to the requested count.  Every (expert, m-tile) of the launch then holds a compared row.
"""
import numpy as np


def m_tile_edges(m: int, bm: int):
    """Positions (inside an expert's m rows) of the first and last row of each m-tile of at most bm rows."""
    if m <= 0:
        return []
    tiles = -(-m // bm)
    blocks = -(-m // 32)
    per = -(-blocks // tiles) * 32
    out = []
    for t in range(tiles):
        lo, hi = t * per, min((t + 1) * per, m)
        if lo < hi:
            out += [lo, hi - 1]
    return out


def stratified_tokens(offsets: np.ndarray, perm: np.ndarray, K: int, T: int, bm: int, n_min: int, seed: int):
    """Sorted unique token ids: tile-edge rows of every expert for tiles of bm rows, plus random tokens up to
    n_min, plus the first and the last token of the batch."""
    pos = []
    for e in range(len(offsets) - 1):
        lo, hi = int(offsets[e]), int(offsets[e + 1])
        pos += [lo + p for p in m_tile_edges(hi - lo, bm)]
    tok = set((perm[np.asarray(pos, dtype=np.int64)] // K).tolist()) if pos else set()
    tok |= {0, T - 1}
    if len(tok) < n_min:
        rng = np.random.default_rng(seed)
        rest = np.setdiff1d(np.arange(T), np.fromiter(tok, dtype=np.int64))
        tok |= set(rng.choice(rest, size=min(n_min - len(tok), len(rest)), replace=False).tolist())
    return np.array(sorted(tok), dtype=np.int64)
