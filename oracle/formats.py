"""Format oracle -- TEST INFRASTRUCTURE ONLY.

Plain numpy constructions of the two sparse mask formats from ONE dense boolean
mask M (S x S, nonzero = attend):

* per-row column-index format (CSR): the paper leaves the row-wise kernel's
  storage undefined (Sec. 4.1); this build uses row_ptr / col_idx, columns
  ascending inside a row.
* two-level block format (Sec. 4.2.1, Fig. 6): block-compressed sparse rows over
  bs x bs outer tiles plus one bitmap per partially filled tile.
  Reading taken for "full": every one of the bs*bs entries is unmasked (a tile
  with holes must be masked in the kernel, so it cannot be "full"); "part":
  between 1 and bs*bs-1 entries set; otherwise empty and absent.  Entries beyond
  S (ragged last tile) count as masked, so a ragged tile is never "full".
  Canonical bitmap layout of a part tile: bs words of 64 bits, word r = tile row
  r, bit c (LSB = 0) = tile column c.
  The paper's own layout (64 words, one per 8x8 inner tile, inner tiles in
  column-major order) is produced by bitmap_inner_tiles(); inside an inner tile
  bit 8*r + c is entry (r, c) (bit order is not stated in the paper).
"""
from __future__ import annotations

import numpy as np


def csr(M: np.ndarray):
    """(row_ptr int32[S+1], col_idx int32[nnz])"""
    S = M.shape[0]
    row_ptr = np.zeros(S + 1, dtype=np.int32)
    cols = []
    for i in range(S):
        c = np.nonzero(M[i])[0]
        cols.append(c)
        row_ptr[i + 1] = row_ptr[i] + len(c)
    col_idx = np.concatenate(cols).astype(np.int32) if cols else np.zeros(0, np.int32)
    return row_ptr, col_idx


def bsr(M: np.ndarray, bs: int):
    """Dictionary with load/full/part row_ptr + col_idx (int32), flags (uint8 per
    load entry: 1 = full, 0 = part) and bitmap (uint64 [npart][bs])."""
    assert bs in (16, 32, 64)
    Sq, Sk = M.shape                      # tile rows cover queries, tile columns keys
    nb, nbc = -(-Sq // bs), -(-Sk // bs)
    P = np.zeros((nb * bs, nbc * bs), dtype=np.uint8)
    P[:Sq, :Sk] = (M != 0)
    cnt = P.reshape(nb, bs, nbc, bs).sum(axis=(1, 3))
    load_row_ptr = np.zeros(nb + 1, np.int32)
    full_row_ptr = np.zeros(nb + 1, np.int32)
    part_row_ptr = np.zeros(nb + 1, np.int32)
    load_col, full_col, part_col, flags, bitmaps = [], [], [], [], []
    weights = (np.uint64(1) << np.arange(bs, dtype=np.uint64))
    for br in range(nb):
        for bc in range(nbc):
            c = int(cnt[br, bc])
            if c == 0:
                continue
            load_col.append(bc)
            if c == bs * bs:
                full_col.append(bc)
                flags.append(1)
            else:
                part_col.append(bc)
                flags.append(0)
                tile = P[br * bs:(br + 1) * bs, bc * bs:(bc + 1) * bs].astype(np.uint64)
                bitmaps.append((tile * weights[None, :]).sum(axis=1, dtype=np.uint64))
        load_row_ptr[br + 1] = len(load_col)
        full_row_ptr[br + 1] = len(full_col)
        part_row_ptr[br + 1] = len(part_col)
    i32 = lambda x: np.asarray(x, dtype=np.int32)
    return {
        "load_row_ptr": load_row_ptr, "load_col_idx": i32(load_col),
        "full_row_ptr": full_row_ptr, "full_col_idx": i32(full_col),
        "part_row_ptr": part_row_ptr, "part_col_idx": i32(part_col),
        "flags": np.asarray(flags, dtype=np.uint8),
        "bitmap": (np.stack(bitmaps) if bitmaps else np.zeros((0, bs), np.uint64)),
        "nnz": int(P.sum()),
    }


def bitmap_inner_tiles(bitmap_rows: np.ndarray) -> np.ndarray:
    """Canonical bitmaps [npart][64] of 64x64 tiles -> the paper's layout
    [npart][64]: word (ic*8 + ir) describes the 8x8 inner tile at inner row ir,
    inner column ic; bit 8*r + c is entry (r, c) of that inner tile."""
    npart = bitmap_rows.shape[0]
    out = np.zeros((npart, 64), dtype=np.uint64)
    for p in range(npart):
        for ir in range(8):
            for ic in range(8):
                w = 0
                for r in range(8):
                    byte = (int(bitmap_rows[p, ir * 8 + r]) >> (8 * ic)) & 0xFF
                    w |= byte << (8 * r)
                out[p, ic * 8 + ir] = w
    return out


def dense_from_csr(row_ptr, col_idx, S: int, Sk: int | None = None) -> np.ndarray:
    M = np.zeros((S, S if Sk is None else Sk), dtype=np.uint8)
    for i in range(S):
        M[i, col_idx[row_ptr[i]:row_ptr[i + 1]]] = 1
    return M


def dense_from_bsr(f: dict, S: int, bs: int, Sk: int | None = None) -> np.ndarray:
    Sk = S if Sk is None else Sk
    nb = -(-S // bs)
    P = np.zeros((nb * bs, -(-Sk // bs) * bs), dtype=np.uint8)
    part = 0
    for br in range(nb):
        for e in range(f["load_row_ptr"][br], f["load_row_ptr"][br + 1]):
            bc = int(f["load_col_idx"][e])
            if f["flags"][e]:
                P[br * bs:(br + 1) * bs, bc * bs:(bc + 1) * bs] = 1
            else:
                words = f["bitmap"][part]
                part += 1
                for r in range(bs):
                    w = int(words[r])
                    for c in range(bs):
                        P[br * bs + r, bc * bs + c] = (w >> c) & 1
    return P[:S, :Sk]
