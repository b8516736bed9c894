"""Pins for the reference planner (oracle/planner_ref.py): hand-built windows
that follow the paper's worked rules, the values the paper prints for its
thresholds, closed forms of its cost model and structural invariants.
CPU only."""
import os

import numpy as np
import pytest

from oracle import planner_ref as pr
from paper_2506_22714_amd import workloads as wl


def popcount(x: int) -> int:
    return bin(x).count("1")


def window_from_counts(counts, W):
    """A one-window matrix whose column c has counts[c] nonzeros in rows 0..counts[c]-1."""
    A = np.zeros((W, len(counts)))
    for c, n in enumerate(counts):
        A[:n, c] = 1.0
    return wl.from_dense(A)


# --------------------------------------------------------- printed thresholds
def test_threshold_values_printed_in_the_paper(golden_dir):
    rows = []
    with open(os.path.join(golden_dir, "paper_thresholds.txt")) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            name, m, n, eta_thr, min_nnz = [t.strip() for t in line.split("|")]
            rows.append((name, int(m), int(n), float(eta_thr), int(min_nnz)))
    assert len(rows) == 5
    for name, m, n, eta_thr, min_nnz in rows:
        eta = (lambda z: pr.eta_spmm(z, m)) if n == 1 else (lambda z: pr.eta_sddmm(z, m, n))
        assert eta(min_nnz) >= eta_thr, name
        if min_nnz > 1:
            assert eta(min_nnz - 1) < eta_thr, name
        # the integer rule the planners use: tau = ceil(eta_thr * m * n)
        assert int(np.ceil(eta_thr * m * n - 1e-12)) == min_nnz, name


def test_cost_model_closed_forms():
    # Eq. 2/3: R_spmm = NNZ/k = m*rho
    m, k = 16, 16
    for nnz_blk in (16, 40, 256):
        rho = nnz_blk / (m * k)
        assert pr.r_spmm(nnz_blk, k) == pytest.approx(m * rho)
    assert pr.r_spmm(256, 16) == 16 and pr.eta_spmm(16, 16) == 1.0
    # a block made of k vectors has NNZ >= k, so R_spmm >= 1 (Section 4.2.1)
    assert pr.r_spmm(k, k) == 1.0
    # Eq. 4/5: R_sddmm = 2 NNZ/(m+n); with NNZ >= n and m < n it exceeds 1
    assert pr.r_sddmm(16, 8, 16) == pytest.approx(2 * 16 / 24)
    assert pr.r_sddmm(16, 8, 16) > 1.0
    assert pr.eta_sddmm(24, 8, 16) == 0.1875


# ------------------------------------------------------------ Fig. 6 style rule
def test_spmm_rule_4x4_example():
    # W=4, tau=2 (eta_thr = 0.5): vectors with >= 2 nonzeros go to the matrix unit
    A = window_from_counts([3, 1, 2, 1], W=4)
    o = pr.Opts(W=4, KB=4, tau_spmm=2, fill_padding=False, Ts=4, Cs=5, short_len=2)
    sp = pr.plan_spmm(A.M, A.rowptr, A.col, o)
    assert len(sp.blocks) == 1 and sp.blocks[0].cols == [0, 2, -1, -1]
    dense_cols = set(A.col[sp.label == 1])
    assert dense_cols == {0, 2} and int(sp.label.sum()) == 5
    # bit (r, s) = r*KB + s: column 0 (slot 0) rows 0..2, column 2 (slot 1) rows 0..1
    assert sp.blocks[0].bitmap == [0b0001_0011_0011]
    # with padding fill the two single-nonzero vectors take the free slots, lower column first
    o.fill_padding = True
    sp = pr.plan_spmm(A.M, A.rowptr, A.col, o)
    assert sp.blocks[0].cols == [0, 2, 1, 3] and int(sp.label.sum()) == A.nnz


def test_filler_vectors_are_promoted_by_nnz_descending_then_column():
    # W=4, KB=4, tau=3: only column 0 qualifies; the three free slots of its block go to the scalar-bound vectors in
    # (NNZ descending, column ascending) order: columns 1 and 3 (two nonzeros each), then column 2 (one; column 4 is left)
    A = window_from_counts([3, 2, 1, 2, 1], W=4)
    o = pr.Opts(W=4, KB=4, tau_spmm=3, fill_padding=True, Ts=4, Cs=5, short_len=2)
    sp = pr.plan_spmm(A.M, A.rowptr, A.col, o)
    assert len(sp.blocks) == 1 and sp.blocks[0].cols == [0, 1, 3, 2]       # by column alone it would be [0, 1, 2, 3]
    assert set(A.col[sp.label == 0]) == {4}
    # the same through the product's host planner
    from paper_2506_22714_amd import binding as lb
    p = lb.Plan.from_csr(A, window_rows=4, block_cols=4, spmm_min_vec_nnz=3, ts=4, cs=5, short_len=2)
    assert p.export(0)["blk_cols"].tolist() == [[0, 1, 3, 2]]
    p.close()


def test_sddmm_rule_4x4_example():
    # W=4, KB=4, tau=4 (eta_thr = 0.25): vectors sorted by NNZ desc, blocks with NNZ >= 4 are dense
    counts = [1, 3, 1, 2, 1, 1, 1, 1, 1]          # sorted: c1(3) c3(2) c0 c2 | c4 c5 c6 c7 | c8
    A = window_from_counts(counts, W=4)
    o = pr.Opts(W=4, KB=4, tau_sddmm=4, Ts=4)
    sp = pr.plan_sddmm(A.M, A.rowptr, A.col, o)
    assert [b.cols for b in sp.blocks] == [[1, 3, 0, 2], [4, 5, 6, 7]]
    assert [b.nnz for b in sp.blocks] == [7, 4]
    assert set(A.col[sp.label == 0]) == {8}
    o.tau_sddmm = 5
    sp = pr.plan_sddmm(A.M, A.rowptr, A.col, o)
    assert [b.cols for b in sp.blocks] == [[1, 3, 0, 2]]


def test_modes_are_the_extremes():
    A = wl.random_pattern(70, 90, 0.08, seed=1, empty_rows=0.1)
    for plan in (pr.plan_spmm, pr.plan_sddmm):
        assert plan(A.M, A.rowptr, A.col, pr.Opts(mode=pr.DENSE_ONLY)).label.all()
        assert not plan(A.M, A.rowptr, A.col, pr.Opts(mode=pr.SCALAR_ONLY)).label.any()
    # tau above the window height: nothing can qualify
    assert not pr.plan_spmm(A.M, A.rowptr, A.col, pr.Opts(tau_spmm=17)).label.any()
    assert not pr.plan_sddmm(A.M, A.rowptr, A.col, pr.Opts(tau_sddmm=257)).label.any()
    # tau = 1 is the matrix-unit-only mode
    assert pr.plan_spmm(A.M, A.rowptr, A.col, pr.Opts(tau_spmm=1)).label.all()


# ------------------------------------------------------------------ invariants
@pytest.mark.parametrize("seed,W,KB,tau,fill", [(1, 16, 16, 2, True), (2, 16, 16, 3, False), (3, 8, 4, 2, True), (4, 4, 8, 2, True)])
def test_spmm_plan_invariants(seed, W, KB, tau, fill):
    A = wl.random_pattern(101, 77, 0.12, seed=seed, empty_rows=0.15)
    o = pr.Opts(W=W, KB=KB, tau_spmm=tau, fill_padding=fill, Ts=2, Cs=6)
    sp = pr.plan_spmm(A.M, A.rowptr, A.col, o)
    # every nonzero exactly once, on exactly one path
    allp = [p for b in sp.blocks for p in b.perm] + sp.res_perm
    assert sorted(allp) == list(range(A.nnz))
    rows = np.repeat(np.arange(A.M), np.diff(A.rowptr))
    for b in sp.blocks:
        assert sum(popcount(x) for x in b.bitmap) == b.nnz == len(b.perm)
        real = [c for c in b.cols if c >= 0]
        assert len(set(real)) == len(real)
        # each bit points at the nonzero (row, column) it encodes
        bits = [i for wd, x in enumerate(b.bitmap) for i in range(wd * 64, wd * 64 + 64) if x >> (i % 64) & 1]
        for bit, p in zip(bits, b.perm):
            assert rows[p] == b.window * W + bit // KB and A.col[p] == b.cols[bit % KB]
    # a dense vector has >= tau nonzeros unless it was promoted into a free slot
    for w in range(sp.stats["n_windows"]):
        blks = sp.blocks[sp.win_blkptr[w]:sp.win_blkptr[w + 1]]
        cols = [c for b in blks for c in b.cols if c >= 0]
        cnt = {c: int(((rows // W == w) & (A.col == c)).sum()) for c in cols}
        below = [c for c in cols if cnt[c] < tau]
        if not fill:
            assert not below
        else:
            assert len(below) < KB and all(c in blks[-1].cols for c in below)
    # the residual array is the scalar-labelled nonzeros, each with its row, grouped by window
    assert sorted(sp.res_perm) == list(np.flatnonzero(sp.label == 0))
    assert [int(rows[p]) for p in sp.res_perm] == sp.res_row
    assert sp.win_resptr[-1] == len(sp.res_perm)
    for w in range(sp.stats["n_windows"]):
        assert all(r // W == w for r in sp.res_row[sp.win_resptr[w]:sp.win_resptr[w + 1]])
    # load balancing: sizes respect Ts / Cs, residual ranges tile the residual array exactly once
    covered = np.zeros(len(sp.res_perm), dtype=int)
    for (kind, ident, a, b_, q0, q1, smask, amask, stmask) in sp.tasks:
        covered[q0:q1] += 1
        if kind == pr.TASK_WINDOW:
            assert 0 <= b_ - a <= o.Ts
            assert sp.win_blkptr[ident] <= a and b_ <= sp.win_blkptr[ident + 1]
            assert {r - ident * W for r in sp.res_row[q0:q1]} == {r for r in range(W) if smask >> r & 1}
            assert all(q1 - q0 == 0 or sp.res_row[q0:q1].count(ident * W + r) <= o.Cs for r in range(W))
        else:
            assert 0 < q1 - q0 <= o.Cs and set(sp.res_row[q0:q1]) == {ident}
    assert np.all(covered == 1)
    # writers per row: >1 writer => every writer atomic and the row is zero-initialised
    writers = np.zeros(A.M, dtype=int)
    plain = np.zeros(A.M, dtype=int)
    for (kind, ident, a, b_, q0, q1, smask, amask, stmask) in sp.tasks:
        if kind == pr.TASK_WINDOW:
            assert amask & stmask == 0
            for r in range(W):
                if (amask | stmask) >> r & 1:
                    writers[ident * W + r] += 1
                if stmask >> r & 1:
                    plain[ident * W + r] += 1
        else:
            writers[ident] += 1
    assert np.all(plain <= 1)
    for i in range(A.M):
        if plain[i]:
            assert writers[i] == 1 and i not in sp.zero_rows
        else:
            assert i in sp.zero_rows
    # every row is defined: written by a task, or cleared by the zero-init list
    assert all(writers[i] >= 1 or i in sp.zero_rows for i in range(A.M))


@pytest.mark.parametrize("seed,W,KB,tau", [(1, 16, 16, 24), (2, 8, 16, 24), (3, 4, 4, 4)])
def test_sddmm_plan_invariants(seed, W, KB, tau):
    A = wl.random_pattern(90, 120, 0.1, seed=seed, empty_rows=0.1)
    o = pr.Opts(W=W, KB=KB, tau_sddmm=tau, Ts=7, sddmm_Ts=2, sddmm_Cs=50)
    sp = pr.plan_sddmm(A.M, A.rowptr, A.col, o)
    allp = [p for b in sp.blocks for p in b.perm] + sp.res_perm
    assert sorted(allp) == list(range(A.nnz))
    # the window tasks tile each window's blocks in groups of at most sddmm_Ts (the SpMM limit Ts plays no part here)
    wt = [(i, a, b) for (k, i, a, b, *_r) in sp.tasks if k == pr.TASK_WINDOW]
    assert all(0 < b - a <= 2 for _i, a, b in wt) and any(b - a == 2 for _i, a, b in wt)
    for w in range(sp.stats["n_windows"]):
        mine = sorted((a, b) for i, a, b in wt if i == w)
        assert [a for a, _b in mine] == list(range(sp.win_blkptr[w], sp.win_blkptr[w + 1], 2))
        assert not mine or mine[-1][1] == sp.win_blkptr[w + 1]
    for w in range(sp.stats["n_windows"]):
        blks = sp.blocks[sp.win_blkptr[w]:sp.win_blkptr[w + 1]]
        nn = [b.nnz for b in blks]
        assert nn == sorted(nn, reverse=True)                   # densest first: dense blocks are a prefix
        assert all(n >= tau for n in nn)
        for b in blks:
            if -1 not in b.cols:
                assert b.nnz >= KB                              # a full block holds >= n nonzeros (Section 4.2.1)
    sizes = [q1 - q0 for (k, _i, _a, _b, q0, q1, *_r) in sp.tasks if k == pr.TASK_CHUNK]
    assert sum(sizes) == len(sp.res_perm) and all(0 < s <= 50 for s in sizes)


def test_sddmm_dense_share_rule():
    """The whole-matrix form of the utilisation rule: in the hybrid mode the SDDMM sub-plan keeps its dense blocks only if they
    hold at least the given percentage of the nonzeros; below it the plan is the scalar-only plan.  Off (0), and in the
    two single-path modes, nothing changes."""
    A = wl.community(n_blocks=6, seed=2)
    base = pr.plan_sddmm(A.M, A.rowptr, A.col, pr.Opts(tau_sddmm=40))
    share = 100.0 * base.stats["dense_nnz"] / A.nnz
    assert 5 < share < 95
    scalar = pr.plan_sddmm(A.M, A.rowptr, A.col, pr.Opts(mode=pr.SCALAR_ONLY))
    just_below, just_above = int(np.floor(share)), int(np.floor(share)) + 1        # share is not a whole number here
    assert just_below < share < just_above
    kept = pr.plan_sddmm(A.M, A.rowptr, A.col, pr.Opts(tau_sddmm=40, sddmm_min_dense_pct=just_below))
    dropped = pr.plan_sddmm(A.M, A.rowptr, A.col, pr.Opts(tau_sddmm=40, sddmm_min_dense_pct=just_above))
    assert kept.stats == base.stats and kept.res_perm == base.res_perm and kept.tasks == base.tasks
    assert dropped.stats["dense_nnz"] == 0 and not dropped.blocks
    assert dropped.res_perm == scalar.res_perm == list(range(A.nnz)) and dropped.tasks == scalar.tasks
    dense_only = pr.plan_sddmm(A.M, A.rowptr, A.col, pr.Opts(mode=pr.DENSE_ONLY, sddmm_min_dense_pct=100))
    assert dense_only.stats["dense_nnz"] == A.nnz                                  # the rule belongs to the hybrid mode


# ------------------------------------------------- three decomposition cases
def test_three_decomposition_cases():
    """Section 4.3: (0) dense part and a long row both decomposed -> every
    segment atomic; (1) only a long row decomposed -> the dense part's
    contribution to that row is atomic too; (2,3) single kind of work, not
    decomposed -> no atomics."""
    W, KB, Ts, Cs = 4, 2, 2, 5
    ncol = 64
    A = np.zeros((16, ncol))
    # window 0: 6 dense vectors (3 blocks > Ts) and row 1 with 7 single-nonzero columns (> Cs)
    for c in range(6):
        A[0:2, c] = 1
    A[1, 10:17] = 1
    # window 1: 2 dense vectors (1 block) and row 5 with 6 single-nonzero columns (> Cs)
    A[4:6, 20] = 1
    A[4:6, 21] = 1
    A[5, 30:36] = 1
    # window 2: dense only, 2 blocks (= Ts, not decomposed); window 3: scalar only, short rows
    for c in range(4):
        A[8:11, 40 + c] = 1
    A[12, 50] = 1
    A[13, 51] = 1
    csr = wl.from_dense(A)
    o = pr.Opts(W=W, KB=KB, tau_spmm=2, fill_padding=False, Ts=Ts, Cs=Cs, short_len=3)
    sp = pr.plan_spmm(csr.M, csr.rowptr, csr.col, o)
    by_win = {w: [t for t in sp.tasks if (t[0] == pr.TASK_WINDOW and t[1] == w) or (t[0] == pr.TASK_CHUNK and t[1] // W == w)] for w in range(4)}
    # window 0: 2 dense groups (2+1 blocks), 2 chunks of row 1 (5+2); all atomic, nothing plain-stored
    k0 = by_win[0]
    assert sorted(t[3] - t[2] for t in k0 if t[0] == pr.TASK_WINDOW) == [1, 2]
    assert sorted(t[5] - t[4] for t in k0 if t[0] == pr.TASK_CHUNK) == [2, 5]
    assert all(t[8] == 0 for t in k0 if t[0] == pr.TASK_WINDOW)
    assert all(t[7] == 0b0011 for t in k0 if t[0] == pr.TASK_WINDOW)
    assert {0, 1, 2, 3} <= set(sp.zero_rows)
    # window 1: one window task; row 5 (bit 1) is atomic because its chunks write it too, row 4 is plain
    k1 = by_win[1]
    wt = [t for t in k1 if t[0] == pr.TASK_WINDOW]
    assert len(wt) == 1 and wt[0][7] == 0b0010 and wt[0][8] == 0b1101
    assert sorted(t[5] - t[4] for t in k1 if t[0] == pr.TASK_CHUNK) == [1, 5]
    assert 5 in sp.zero_rows and 4 not in sp.zero_rows
    # windows 2 and 3: single task each, no atomics, all rows plain
    for w in (2, 3):
        assert len(by_win[w]) == 1 and by_win[w][0][7] == 0 and by_win[w][0][8] == 0b1111
    assert not ({8, 9, 10, 11, 12, 13, 14, 15} & set(sp.zero_rows))
    assert sp.n_split_rows == 2 and sp.n_short_rows == 2 and sp.n_long_rows == 2


def test_community_config_expected_vector_density():
    # in-block vectors of a 16-row window: Binomial(16, 0.3) conditioned on >= 1  (config 3 recipe)
    A = wl.community(n_blocks=8, seed=3)
    sp = pr.plan_spmm(A.M, A.rowptr, A.col, pr.Opts())
    st = sp.stats
    in_block_vectors = 8 * 4 * 64 * (1 - 0.7 ** 16)
    expect_mean = 16 * 0.3 / (1 - 0.7 ** 16)
    dense_mean = st["dense_nnz"] / st["n_dense_vectors"]
    assert abs(st["n_vectors"] - st["n_vectors_nnz1"] - in_block_vectors) / in_block_vectors < 0.08
    assert abs(dense_mean - expect_mean) / expect_mean < 0.1
