"""Reference planner (test infrastructure only): the workload-distribution and
load-balancing steps of the paper in plain Python, one window at a time.

It follows, in the paper's order and notation:

* Section 2.2 - rows are cut into windows of height m (here ``W``); in a window
  every column with at least one nonzero is an m x 1 nonzero column vector;
  vectors are condensed, k (here ``KB``) at a time, into TC blocks.
* Section 4.2, Eq. 6 and the worked rule of Fig. 6 - SpMM: a vector goes to the
  matrix unit iff NNZ_vector / m >= eta_thr, i.e. NNZ_vector >= tau_spmm; free
  slots of a window's last block may be filled with vectors that would
  otherwise go to the scalar path.  SDDMM: vectors are sorted by descending
  NNZ_vector, condensed into m x n blocks, and a block goes to the matrix unit
  iff NNZ_block >= tau_sddmm.  A whole-matrix form of the same utilisation
  argument sits on top (a reading of this build, an option): in the hybrid mode
  the SDDMM sub-plan keeps its dense blocks only if together they hold at least
  `sddmm_min_dense_pct` percent of the nonzeros; otherwise every nonzero takes
  the scalar path.
* Section 4.3 - the dense part of a window is decomposed into groups of Ts
  blocks only if it holds more than Ts; a residual row with fewer than
  Short_len nonzeros is short, otherwise long, and a long row is decomposed
  into groups of Cs nonzeros only if it holds more than Cs; every segment of a
  decomposed piece of work is flagged atomic.

Readings taken where the paper is silent (the product planner takes the same):
ties in the SDDMM sort break by ascending column; SpMM blocks hold their dense
vectors in ascending column order and promoted filler vectors after them, in
(NNZ descending, column ascending) order; bit (r, s) of a block's bitmap is
bit r*KB+s, packed values follow bit order; the atomic flag is kept per row:
a row is atomic iff more than one task writes it.

Slow by design: dict-of-windows, Python loops.  Use on small inputs only.
"""
from __future__ import annotations

from dataclasses import dataclass, field

import numpy as np

HYBRID, DENSE_ONLY, SCALAR_ONLY = 0, 1, 2
TASK_WINDOW, TASK_CHUNK = 0, 1


@dataclass
class Opts:
    mode: int = HYBRID
    W: int = 16
    KB: int = 16
    tau_spmm: int = 3
    tau_sddmm: int = 64
    Ts: int = 16
    Cs: int = 128
    short_len: int = 3
    fill_padding: bool = True
    sddmm_Cs: int = 128
    sddmm_Ts: int = 4
    sddmm_min_dense_pct: int = 0      # 0: the rule is off


@dataclass
class Block:
    window: int
    cols: list            # KB entries, -1 = padding
    bitmap: list          # ceil(W*KB/64) python ints (uint64)
    perm: list            # CSR positions in bit order
    nnz: int


@dataclass
class SubPlan:
    label: np.ndarray                 # int8 per CSR nonzero: 1 dense path, 0 scalar path
    blocks: list = field(default_factory=list)
    win_blkptr: list = field(default_factory=list)
    res_perm: list = field(default_factory=list)      # residual nonzeros (CSR position of each)
    res_row: list = field(default_factory=list)       # row of each residual nonzero
    win_resptr: list = field(default_factory=lambda: [0])   # SpMM only: first residual nonzero of each window
    # (kind, id, blk_begin, blk_end, res_begin, res_end, scalar_mask, atomic_mask, store_mask)
    tasks: list = field(default_factory=list)
    zero_rows: list = field(default_factory=list)     # SpMM only
    n_short_rows: int = 0
    n_long_rows: int = 0
    n_split_rows: int = 0
    stats: dict = field(default_factory=dict)


def _census(rowptr, col, w, W, M):
    """column -> list of (row_in_window, csr_pos) for window w."""
    vec = {}
    for i in range(w * W, min(M, (w + 1) * W)):
        for p in range(int(rowptr[i]), int(rowptr[i + 1])):
            vec.setdefault(int(col[p]), []).append((i - w * W, p))
    return vec


def _make_block(w, cols, vec, W, KB):
    nwords = (W * KB + 63) // 64
    bits = [0] * nwords
    entries = []
    for s, c in enumerate(cols):
        for (r, p) in vec[c]:
            b = r * KB + s
            bits[b // 64] |= 1 << (b % 64)
            entries.append((b, p))
    entries.sort()
    padded = list(cols) + [-1] * (KB - len(cols))
    return Block(w, padded, bits, [p for _b, p in entries], len(entries))


def plan_spmm(M, rowptr, col, o: Opts) -> SubPlan:
    nnz = int(rowptr[M])
    W, KB = o.W, o.KB
    nwin = (M + W - 1) // W
    sp = SubPlan(label=np.zeros(nnz, dtype=np.int8))
    sp.win_blkptr = [0]
    n_vec = n_vec1 = n_dense_vec = n_pad = 0
    res_by_row = [[] for _ in range(M)]
    for w in range(nwin):
        vec = _census(rowptr, col, w, W, M)
        n_vec += len(vec)
        n_vec1 += sum(1 for v in vec.values() if len(v) == 1)
        if o.mode == SCALAR_ONLY:
            dense = []
        elif o.mode == DENSE_ONLY:
            dense = sorted(vec)
        else:
            dense = sorted(c for c, v in vec.items() if len(v) >= o.tau_spmm)
        # fill the free slots of the last block (Section 4.2, Fig. 6 text)
        if dense and o.fill_padding and o.mode == HYBRID and len(dense) % KB:
            free = KB - len(dense) % KB
            rest = sorted((c for c in vec if len(vec[c]) < o.tau_spmm), key=lambda c: (-len(vec[c]), c))
            dense = dense + rest[:free]
        n_dense_vec += len(dense)
        blocks = [_make_block(w, dense[s:s + KB], vec, W, KB) for s in range(0, len(dense), KB)]
        n_pad += sum(b.cols.count(-1) for b in blocks)
        for b in blocks:
            sp.label[b.perm] = 1
        sp.blocks.extend(blocks)
        sp.win_blkptr.append(len(sp.blocks))
        dense_set = set(dense)
        for c, lst in vec.items():
            if c not in dense_set:
                for (r, p) in lst:
                    res_by_row[w * W + r].append(p)
    # ---- hybrid load balancing (Section 4.3) and the residual array ----
    # Residual nonzeros are stored window by window: first the rows that are not
    # decomposed (row order, CSR order inside a row), then the decomposed rows.
    zero = set()
    for w in range(nwin):
        b0, b1 = sp.win_blkptr[w], sp.win_blkptr[w + 1]
        nb = b1 - b0
        rows = range(w * W, min(M, (w + 1) * W))
        rlen = {i: len(res_by_row[i]) for i in rows}
        split_rows = set()
        for i in rows:
            r = rlen[i]
            if r == 0:
                continue
            if r < o.short_len:
                sp.n_short_rows += 1
            else:
                sp.n_long_rows += 1
                if r > o.Cs:
                    split_rows.add(i)
        sp.n_split_rows += len(split_rows)

        def touched(bl0, bl1):
            m = 0
            for b in sp.blocks[bl0:bl1]:
                for wd, word in enumerate(b.bitmap):
                    for bit in range(64):
                        if word >> bit & 1:
                            m |= 1 << ((wd * 64 + bit) // KB)
            return m

        q0 = len(sp.res_perm)
        for i in rows:
            if i not in split_rows:
                sp.res_perm.extend(sorted(res_by_row[i]))
                sp.res_row.extend([i] * rlen[i])
        q1 = len(sp.res_perm)
        valid = sum(1 << (i - w * W) for i in rows)
        split_mask = sum(1 << (i - w * W) for i in split_rows)
        scalar_mask = sum(1 << (i - w * W) for i in rows if rlen[i] > 0 and i not in split_rows)
        if nb > o.Ts:
            # decomposed dense part: every segment of the window is atomic
            for g0 in range(b0, b1, o.Ts):
                g1 = min(b1, g0 + o.Ts)
                sp.tasks.append((TASK_WINDOW, w, g0, g1, q0, q0, 0, touched(g0, g1), 0))
            if scalar_mask:
                sp.tasks.append((TASK_WINDOW, w, b1, b1, q0, q1, scalar_mask, scalar_mask, 0))
            zero.update(rows)
        else:
            atomic_mask = split_mask & touched(b0, b1)
            sp.tasks.append((TASK_WINDOW, w, b0, b1, q0, q1, scalar_mask, atomic_mask, valid & ~split_mask))
            zero.update(split_rows)
        for i in sorted(split_rows):
            s = len(sp.res_perm)
            sp.res_perm.extend(sorted(res_by_row[i]))
            sp.res_row.extend([i] * rlen[i])
            e = len(sp.res_perm)
            for c0 in range(s, e, o.Cs):
                sp.tasks.append((TASK_CHUNK, i, 0, 0, c0, min(e, c0 + o.Cs), 0, 0, 0))
        sp.win_resptr.append(len(sp.res_perm))
    sp.zero_rows = sorted(zero)
    dense_nnz = int(sp.label.sum())
    sp.stats = dict(n_windows=nwin, n_vectors=n_vec, n_vectors_nnz1=n_vec1, n_dense_vectors=n_dense_vec,
                    n_blocks=len(sp.blocks), n_pad_slots=n_pad, dense_nnz=dense_nnz,
                    scalar_nnz=nnz - dense_nnz)
    return sp


def plan_sddmm(M, rowptr, col, o: Opts) -> SubPlan:
    nnz = int(rowptr[M])
    W, KB = o.W, o.KB
    nwin = (M + W - 1) // W
    sp = SubPlan(label=np.zeros(nnz, dtype=np.int8))
    sp.win_blkptr = [0]
    n_vec = n_vec1 = n_dense_vec = n_pad = 0
    for w in range(nwin):
        vec = _census(rowptr, col, w, W, M)
        n_vec += len(vec)
        n_vec1 += sum(1 for v in vec.values() if len(v) == 1)
        order = sorted(vec, key=lambda c: (-len(vec[c]), c))
        for s in range(0, len(order), KB):
            cols = order[s:s + KB]
            blk_nnz = sum(len(vec[c]) for c in cols)
            if o.mode == SCALAR_ONLY:
                take = False
            elif o.mode == DENSE_ONLY:
                take = True
            else:
                take = blk_nnz >= o.tau_sddmm
            if not take:
                break                       # block sums never increase: dense blocks are a prefix
            b = _make_block(w, cols, vec, W, KB)
            sp.blocks.append(b)
            sp.label[b.perm] = 1
            n_dense_vec += len(cols)
            n_pad += KB - len(cols)
        sp.win_blkptr.append(len(sp.blocks))
    if o.mode == HYBRID and o.sddmm_min_dense_pct > 0 and 100 * int(sp.label.sum()) < o.sddmm_min_dense_pct * nnz:
        # too small a share for the matrix units to pay: the whole sub-plan goes to the scalar path
        from dataclasses import replace
        return plan_sddmm(M, rowptr, col, replace(o, mode=SCALAR_ONLY))
    sp.res_perm = [int(p) for p in np.flatnonzero(sp.label == 0)]
    rows_of = np.repeat(np.arange(M), np.diff(np.asarray(rowptr[:M + 1], dtype=np.int64)))
    sp.res_row = [int(rows_of[p]) for p in sp.res_perm]
    # load balancing: groups of sddmm_Ts blocks per window (Ts of Section 4.3 for this sub-plan: its tasks write disjoint
    # outputs, so the limit is its own); residual list in groups of sddmm_Cs nonzeros
    for w in range(nwin):
        b0, b1 = sp.win_blkptr[w], sp.win_blkptr[w + 1]
        for g0 in range(b0, b1, o.sddmm_Ts):
            sp.tasks.append((TASK_WINDOW, w, g0, min(b1, g0 + o.sddmm_Ts), 0, 0, 0, 0, 0))
    for c0 in range(0, len(sp.res_perm), o.sddmm_Cs):
        sp.tasks.append((TASK_CHUNK, 0, 0, 0, c0, min(len(sp.res_perm), c0 + o.sddmm_Cs), 0, 0, 0))
    dense_nnz = int(sp.label.sum())
    sp.stats = dict(n_windows=nwin, n_vectors=n_vec, n_vectors_nnz1=n_vec1, n_dense_vectors=n_dense_vec,
                    n_blocks=len(sp.blocks), n_pad_slots=n_pad, dense_nnz=dense_nnz,
                    scalar_nnz=nnz - dense_nnz)
    return sp


# ---------------------------------------------------------------------------
# Cost model of Section 4.2 (Eq. 2-6), for a single block / vector
# ---------------------------------------------------------------------------
def r_spmm(nnz_block: int, k: int) -> float:
    """Eq. 2: scalar-path operand traffic NNZ*n over matrix-unit traffic k*n."""
    return nnz_block / k


def r_sddmm(nnz_block: int, m: int, n: int) -> float:
    """Eq. 4: 2*NNZ*k over (m+n)*k."""
    return 2.0 * nnz_block / (m + n)


def eta_spmm(nnz_vector: int, m: int) -> float:
    return nnz_vector / m


def eta_sddmm(nnz_block: int, m: int, n: int) -> float:
    return nnz_block / (m * n)
