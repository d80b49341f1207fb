"""Integer side of the oracle (test infrastructure): what the packed layout implies.

Section 5.2: documents l_1..l_k with sum N; attention cost is proportional to the number
of (query, key) pairs inside the block-diagonal causal mask, sum_b l_b (l_b + 1) / 2.
Plain Python integers throughout (exact).
"""
from __future__ import annotations

from typing import List, Tuple


def doc_of_token(cu) -> List[int]:
    cu = [int(x) for x in cu]
    out = []
    for b in range(len(cu) - 1):
        out.extend([b] * (cu[b + 1] - cu[b]))
    return out


def pairs(cu) -> int:
    cu = [int(x) for x in cu]
    return sum((cu[b + 1] - cu[b]) * (cu[b + 1] - cu[b] + 1) // 2 for b in range(len(cu) - 1))


def flops_fwd_bwd(cu, n_q_heads: int, head_dim: int) -> int:
    """Two contractions forward and five backward, 2*d flop per pair each."""
    return 14 * head_dim * n_q_heads * pairs(cu)


def row_tiles(cu, block_rows: int) -> List[Tuple[int, int, int, int]]:
    """Per-document tiling of the token axis: every non-empty document is cut into tiles of
    ``block_rows`` rows starting at its first token.  Returns (doc, tile index inside the
    document, first row, number of valid rows), in document order."""
    cu = [int(x) for x in cu]
    out = []
    for b in range(len(cu) - 1):
        l = cu[b + 1] - cu[b]
        for i in range((l + block_rows - 1) // block_rows):
            r0 = cu[b] + i * block_rows
            out.append((b, i, r0, min(block_rows, cu[b + 1] - r0)))
    return out


def causal_tile_pairs(cu, block_q: int, block_k: int) -> int:
    """Number of (q tile, kv tile) pairs that contain at least one allowed (t, j)."""
    cu = [int(x) for x in cu]
    total = 0
    for b in range(len(cu) - 1):
        l = cu[b + 1] - cu[b]
        for i in range((l + block_q - 1) // block_q):
            last_row = min(l, (i + 1) * block_q) - 1          # inside the document
            total += last_row // block_k + 1
    return total


def row_chain_steps(cu, tile_rows: int, step_rows: int):
    """Forward / dQ direction.  For every tile (doc, i, row0, rows) the number of key steps
    of `step_rows` rows, counted from the first token of the document, that hold at least
    one key some query of the tile may see."""
    cu = [int(x) for x in cu]
    out = {}
    for b, i, r0, rows in row_tiles(cu, tile_rows):
        last = r0 + rows - 1
        out[(r0, cu[b], cu[b + 1])] = (last - cu[b]) // step_rows + 1
    return out


def col_chain_steps(cu, tile_rows: int, step_rows: int):
    """dK / dV direction.  For every tile the number of query steps of `step_rows` rows,
    counted from the first row of the tile, up to the end of the document."""
    cu = [int(x) for x in cu]
    out = {}
    for b, i, r0, rows in row_tiles(cu, tile_rows):
        out[(r0, cu[b], cu[b + 1])] = -(-(cu[b + 1] - r0) // step_rows)
    return out
