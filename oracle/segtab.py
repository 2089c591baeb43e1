"""TEST INFRASTRUCTURE -- the oracle's own chunk-alignment table builder (pure Python).

Follows the paper's two alignment steps (section 3.5, "Reinventing Packing with
Chunk-Based Alignment"): (1) each task's sequences are packed, task by task, inside that
task's own batch; (2) every pack is cut into equal-size chunks, a pack longer than one
chunk occupying consecutive chunks, and a pack whose length is not a multiple of the
chunk size leaving zero padding at the end of its last chunk (section 5.4,
"Effectiveness of Data Alignment": chunk 128 with 64-token sequences).

It shares nothing with the library's builder; tests compare the two serialised images
byte for byte.  Written as loops over tokens' containers, not as index algebra, so it
can be checked by eye.
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import List, Sequence

import numpy as np

MAGIC = 0x5458554D          # "MUXT", little endian
VERSION = 1
FLAG_DENSE = 1              # tasks back to back; only the tail of the whole batch is padded

HEADER_INTS = 16
TASK_INTS = 8
PACK_INTS = 6
CHUNK_INTS = 4
SEG_INTS = 6
SEQ_INTS = 4


@dataclass
class SegTab:
    image: np.ndarray          # canonical int32 image
    T: int
    chunk: int
    n_chunks: int
    valid_total: int
    row_task: np.ndarray       # int32[T], -1 on padding rows
    task_rows: List[np.ndarray]  # per task: indices of its valid rows, ascending


def choose_chunk_size(lens: Sequence[int], floor: int = 64) -> int:
    """Greatest power of two dividing every sequence length, not below `floor`
    (section 3.5: chunk size = greatest power-of-2 divisor of all lengths, with a
    minimum threshold, typically 64)."""
    lens = [int(l) for l in lens if int(l) > 0]
    if not lens:
        return int(floor)
    p = 1
    while all(l % (2 * p) == 0 for l in lens):
        p *= 2
    return max(p, int(floor))


def _packs_of(seq_lens: Sequence[int], max_pack_len: int) -> List[List[int]]:
    """Step 1: greedy in-order packing of one task's sequences."""
    packs: List[List[int]] = []
    cur: List[int] = []
    for l in seq_lens:
        if max_pack_len > 0 and cur and sum(cur) + l > max_pack_len:
            packs.append(cur)
            cur = []
        cur.append(int(l))
    if cur:
        packs.append(cur)
    return packs


def build(task_seq_lens: Sequence[Sequence[int]], chunk: int, max_pack_len: int = 0,
          flags: int = 0) -> SegTab:
    c = int(chunk)
    if c < 1 or (c & (c - 1)) != 0:
        raise ValueError("chunk must be a power of two")
    for lens in task_seq_lens:
        for l in lens:
            if int(l) < 1:
                raise ValueError("sequence lengths must be >= 1")
    dense = bool(flags & FLAG_DENSE)
    M = len(task_seq_lens)

    # Lay the tokens out row by row.  `rows` lists, for every row of the aligned batch,
    # (task, pack, seq) or None for padding.
    rows: List[object] = []
    packs = []      # dicts
    seqs = []       # [task, pack, first_row, len]
    tasks = []      # dicts
    for t, lens in enumerate(task_seq_lens):
        task_first_row = len(rows)
        task_pack_begin = len(packs)
        task_seq_begin = len(seqs)
        for pk in _packs_of(lens, max_pack_len):
            p = len(packs)
            first = len(rows)
            for l in pk:
                seqs.append([t, p, len(rows), l])
                rows.extend([(t, p)] * l)
            packs.append({"task": t, "row_begin": first, "valid": len(rows) - first})
            if not dense:
                while len(rows) % c != 0:       # zero padding up to the chunk boundary
                    rows.append(None)
        tasks.append({"row_begin": task_first_row, "row_count": len(rows) - task_first_row,
                      "valid": sum(int(l) for l in lens), "pack_begin": task_pack_begin,
                      "pack_count": len(packs) - task_pack_begin, "seq_begin": task_seq_begin})
    while len(rows) % c != 0:
        rows.append(None)
    T = len(rows)
    n_chunks = T // c

    # Segments = maximal runs of one pack inside one chunk, in row order.
    segs = []       # [task, pack, chunk, row_begin, n_rows, index_in_pack]
    chunks = []     # [valid, seg_begin, seg_count, first_task]
    pieces_seen = [0] * len(packs)
    for ch in range(n_chunks):
        seg_begin = len(segs)
        valid = 0
        i = ch * c
        while i < (ch + 1) * c:
            if rows[i] is None:
                i += 1
                continue
            t, p = rows[i]
            j = i
            while j < (ch + 1) * c and rows[j] == (t, p):
                j += 1
            segs.append([t, p, ch, i, j - i, pieces_seen[p]])
            pieces_seen[p] += 1
            valid += j - i
            i = j
        first_task = segs[seg_begin][0] if len(segs) > seg_begin else -1
        chunks.append([valid, seg_begin, len(segs) - seg_begin, first_task])

    valid_total = sum(1 for r in rows if r is not None)

    img: List[int] = [MAGIC, VERSION, int(flags), M, c, int(max_pack_len), n_chunks, T,
                      valid_total, len(packs), len(segs), len(seqs), 0, 0, 0, 0]
    for t in range(M):
        tk = tasks[t]
        touched = sorted({s[2] for s in segs if s[0] == t})
        chunk_begin = touched[0] if touched else tk["row_begin"] // c
        img += [tk["row_begin"], tk["row_count"], tk["valid"], chunk_begin, len(touched),
                tk["pack_begin"], tk["pack_count"], tk["seq_begin"]]
    for p, pk in enumerate(packs):
        mine = [k for k, s in enumerate(segs) if s[1] == p]
        img += [pk["task"], pk["row_begin"], pk["valid"], segs[mine[0]][2], len(mine), mine[0]]
    for chv in chunks:
        img += chv
    for s in segs:
        img += s
    for s in seqs:
        img += s

    row_task = np.full(T, -1, dtype=np.int32)
    for i, r in enumerate(rows):
        if r is not None:
            row_task[i] = r[0]
    task_rows = [np.nonzero(row_task == t)[0].astype(np.int64) for t in range(M)]
    return SegTab(image=np.asarray(img, dtype="<i4"), T=T, chunk=c, n_chunks=n_chunks,
                  valid_total=valid_total, row_task=row_task, task_rows=task_rows)


def sequences(st: SegTab) -> List[List[int]]:
    """The sequences of the aligned batch as [task, pack, first_row, len], read back from the canonical image."""
    img = [int(v) for v in st.image]
    M, n_chunks, n_packs, n_segs, n_seqs = img[3], img[6], img[9], img[10], img[11]
    off = HEADER_INTS + M * TASK_INTS + n_packs * PACK_INTS + n_chunks * CHUNK_INTS + n_segs * SEG_INTS
    return [img[off + SEQ_INTS * i: off + SEQ_INTS * (i + 1)] for i in range(n_seqs)]
