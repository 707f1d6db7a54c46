"""Host emulation of the paper's BSpMM.BBB procedure (Algorithm 1 and steps 1-6
of Section 3.3.2), used as a structurally different formulation to pin the
plain-definition oracle.

It follows the paper's data layout: the adjacency is stored as CSR over 4x4
bit tiles (RowPtr, ColInd, BitTiles: four 4-bit nibbles per tile), a tile row
(4 nodes) is processed in tile sets of TS = 32/4 = 8 tiles, the nibbles of a
tile set are concatenated into one 32-bit vector per node, the 32 gathered
activation words are bit-transposed, and the trinary dot product is
popc(a & b) - popc(a & ~b) (method 2).  The accumulator is summed across tile
sets, and the output bit is (c >= 0).  Activations are 32-bit words, one bit
per channel.

Pure Python integers; only for small graphs.  Shares no code with the oracle
or the library.
"""
from __future__ import annotations

from typing import Dict, List, Tuple

TILE = 4
SIMD_UNIT = 32
TS = SIMD_UNIT // TILE          # tiles per tile set


def build_frdc(n: int, rowptr, col) -> Tuple[List[int], List[int], List[List[int]]]:
    """CSR adjacency -> (RowPtr, ColInd, BitTiles) over 4x4 tiles.  BitTiles[t]
    holds 4 nibbles, nibble r = row r of the tile, bit q (value 1 << q) set when
    the tile's column q is a neighbour."""
    n_tr = (n + TILE - 1) // TILE
    tile_rowptr = [0]
    colind: List[int] = []
    tiles: List[List[int]] = []
    for tr in range(n_tr):
        found: Dict[int, List[int]] = {}
        for r in range(TILE):
            i = tr * TILE + r
            if i >= n:
                continue
            for e in range(int(rowptr[i]), int(rowptr[i + 1])):
                j = int(col[e])
                t = found.setdefault(j // TILE, [0, 0, 0, 0])
                t[r] |= 1 << (j % TILE)
        for tc in sorted(found):
            colind.append(tc)
            tiles.append(found[tc])
        tile_rowptr.append(len(colind))
    return tile_rowptr, colind, tiles


def n_tile_sets(nt: int) -> int:
    return (nt + TS - 1) // TS


def bspmm_bbb(n: int, frdc, words: List[List[int]], n_words: int) -> List[List[int]]:
    """words[j][w] is the 32-bit activation word w of node j (bit c = channel
    32*w + c, 1 = +1).  Returns the same layout for the output, bit = (c >= 0)."""
    tile_rowptr, colind, tiles = frdc
    n_tr = len(tile_rowptr) - 1
    out = [[0] * n_words for _ in range(n)]
    mask32 = (1 << 32) - 1
    for tr in range(n_tr):
        lo, hi = tile_rowptr[tr], tile_rowptr[tr + 1]
        nt = hi - lo
        for w in range(n_words):
            acc = [[0] * 32 for _ in range(TILE)]      # c[n] per lane (channel)
            for s in range(n_tile_sets(nt)):
                # step 2: load TS tiles (zero padded) and the activation rows
                # of the 4 nodes of every tile: 32 words B[p], p = 4*slot + q
                a_tiles = []
                b_rows = []
                for slot in range(TS):
                    t = lo + s * TS + slot
                    if t < hi:
                        a_tiles.append(tiles[t])
                        base = colind[t] * TILE
                    else:
                        a_tiles.append([0, 0, 0, 0])
                        base = 0
                    for q in range(TILE):
                        j = base + q
                        b_rows.append(words[j][w] if j < n else 0)
                # step 3: concatenate the nibbles of node r into a 32-bit vector;
                # bit p of a[r] <-> neighbour p = 4*slot + q
                a = [0] * TILE
                for r in range(TILE):
                    for slot in range(TS):
                        a[r] |= a_tiles[slot][r] << (TILE * slot)
                # step 4: 32x32 bit transpose: bt[c] bit p = bit c of B[p]
                bt = [0] * 32
                for c in range(32):
                    x = 0
                    for p in range(32):
                        x |= ((b_rows[p] >> c) & 1) << p
                    bt[c] = x
                # step 5: trinary dot product, method 2, summed over tile sets
                for r in range(TILE):
                    for c in range(32):
                        pos = bin(a[r] & bt[c]).count("1")
                        neg = bin(a[r] & (~bt[c] & mask32)).count("1")
                        acc[r][c] += pos - neg
            # step 6: binarize (c >= 0) and pack
            for r in range(TILE):
                i = tr * TILE + r
                if i >= n:
                    continue
                word = 0
                for c in range(32):
                    if acc[r][c] >= 0:
                        word |= 1 << c
                out[i][w] = word
    return out
