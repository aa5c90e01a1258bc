"""Independent reader of the RS-Tile plan arrays (paper, Section 3.2) --
TEST INFRASTRUCTURE ONLY.

Given the raw arrays a plan exposes (the bytes the device kernels read), rebuild
the list of stored entries (row, column, binary16 bits, path) with plain Python /
numpy, following only the layout documented in the public header:

* a window has W = 16 * NW rows; window w owns fragments win_tile_off[w] ..
  win_tile_off[w+1]; fragment t has K (16 or 32) column ids and NW sub-fragments (rows
  16 s .. 16 s + 15 of the window); with Q = K / 4, sub-fragment (t, s) has a 16 x K bit
  map (Q 64-bit words at index (t * NW + s) * Q; cell (row r, column k) is bit
  (k // Q) * 16 + r of word k % Q) and a run of values that starts at
  tile_val_off[t * NW + s] and is ordered by ((k // Q) * 16 + r, k % Q);
* an irregular wave (start, count, dst, info) is, by info & 3: kind 0 -- count rows
  of exactly L = (info >> 8) & 255 entries each, back to back from start, whose row
  ids are irr_row[dst .. dst+count); kind 1 -- count consecutive entries of one row,
  the row being dst itself or, when info has bit 2 set, the row whose combine entry
  (row, first slot, parts, stride) covers scratch slot dst; kind 2 -- no entries.

Panel form (window_rows == 128 or 256): a window is G = 4 or 8 row groups of 32 rows, a fragment is 32
condensed columns = two K steps of 16; the entries of (row group g, fragment t, K step h) of window w
are the words panel_ent[panel_off[u] .. panel_off[u+1]) with u = 2 * G * t0 + (g * nt + (t - t0)) * 2 + h
(t0 = win_tile_off[w], nt = the window's fragment count); a word is value bits | address << 16 with
address = ((r + 32 * (k // 8)) * 8 + k % 8) * 2 for row r of the group and column k of the K step;
units start at multiples of four words and are padded with words whose address is >= 1024.
"""
from __future__ import annotations

import numpy as np


def panel_entries(win_row, win_tile_off, tile_colid, panel_off, panel_ent, window_rows=128):
    """(rows, cols, value bits) of the dense-fragment part of a plan in the panel form."""
    rows, cols, vals = [], [], []
    G = window_rows // 32
    n_win = len(win_row) // window_rows
    for w in range(n_win):
        t0, t1 = int(win_tile_off[w]), int(win_tile_off[w + 1])
        nt = t1 - t0
        for g in range(G):
            for t in range(nt):
                for h in range(2):
                    u = 2 * G * t0 + (g * nt + t) * 2 + h
                    for q in range(int(panel_off[u]), int(panel_off[u + 1])):
                        word = int(panel_ent[q])
                        addr = word >> 16
                        if addr >= 1024:              # padding of the unit to four words
                            continue
                        assert addr % 2 == 0
                        lane, j = addr // 16, (addr % 16) // 2
                        r, k = lane % 32, 16 * h + 8 * (lane // 32) + j
                        row = int(win_row[window_rows * w + 32 * g + r])
                        assert row >= 0, "an entry in an absent window row"
                        rows.append(row)
                        cols.append(int(tile_colid[32 * (t0 + t) + k]))
                        vals.append(word & 0xFFFF)
    return rows, cols, vals


def entries_from_arrays(win_row, win_tile_off, tile_colid, tile_mask, tile_val_off, tile_val,
                        irr_col, irr_val, irr_wave, irr_row, combine, n_scratch_slots, window_rows=16, tile_k=16):
    rows, cols, vals, paths = [], [], [], []
    if window_rows >= 128:          # panel form: the caller passes (panel_off, panel_ent) in place of the bitmap arrays
        rows, cols, vals = panel_entries(win_row, win_tile_off, tile_colid, tile_mask, tile_val, window_rows)
        paths = [0] * len(rows)
        win_row = []
    W, NW = window_rows, window_rows // 16
    K, Q = tile_k, tile_k // 4
    n_win = len(win_row) // W
    for w in range(n_win):
        for t in range(int(win_tile_off[w]), int(win_tile_off[w + 1])):
            for s in range(NW):
                cells = []
                for k in range(K):
                    word = int(tile_mask[Q * (t * NW + s) + (k % Q)])
                    for r in range(16):
                        if (word >> ((k // Q) * 16 + r)) & 1:
                            cells.append(((k // Q) * 16 + r, k % Q, r, k))
                cells.sort()
                for pos, (_, _, r, k) in enumerate(cells):
                    row = int(win_row[W * w + 16 * s + r])
                    assert row >= 0, "a set bit in an absent window row"
                    rows.append(row)
                    cols.append(int(tile_colid[K * t + k]))
                    vals.append(int(tile_val[int(tile_val_off[t * NW + s]) + pos]))
                    paths.append(0)
    slot_row = {}
    for e in range(len(combine) // 4):
        row, first, parts, stride = (int(x) for x in combine[4 * e:4 * e + 4])
        for p in range(parts):
            slot = first + p * stride
            assert slot not in slot_row and slot < n_scratch_slots
            slot_row[slot] = row
    for s in range(len(irr_wave) // 4):
        start, count, dst, info = (int(x) for x in irr_wave[4 * s:4 * s + 4])
        kind = info & 3
        if kind == 0:
            L = (info >> 8) & 255
            for q in range(count):
                for j in range(L):
                    rows.append(int(irr_row[dst + q]))
                    cols.append(int(irr_col[start + q * L + j]))
                    vals.append(int(irr_val[start + q * L + j]))
                    paths.append(1)
        elif kind == 1:
            row = slot_row[dst] if (info & 4) else dst
            for q in range(count):
                rows.append(row)
                cols.append(int(irr_col[start + q]))
                vals.append(int(irr_val[start + q]))
                paths.append(1)
    return (np.array(rows, dtype=np.int64), np.array(cols, dtype=np.int64),
            np.array(vals, dtype=np.uint16), np.array(paths, dtype=np.uint8))


def csr_from_entries(rows, cols, vals, paths, n_rows, n_cols):
    """Sort entries into CSR; raises if an entry is covered twice."""
    keys = rows * n_cols + cols
    order = np.argsort(keys, kind="stable")
    keys = keys[order]
    if keys.size > 1 and np.any(keys[1:] == keys[:-1]):
        raise AssertionError("a stored entry appears more than once in the plan")
    row_ptr = np.zeros(n_rows + 1, dtype=np.int64)
    np.cumsum(np.bincount(rows, minlength=n_rows), out=row_ptr[1:])
    return row_ptr, cols[order].astype(np.int32), vals[order], paths[order]
