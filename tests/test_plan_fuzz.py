"""Randomised cross-check of the product planner against the reference planner: random small matrices with
random shapes, densities, long rows and options must give bit-identical plans.  CPU only."""
from hypothesis import HealthCheck, given, settings
from hypothesis import strategies as st

from oracle import planner_ref as pr
from paper_2506_22714_amd import binding as lb
from paper_2506_22714_amd import workloads as wl
from test_plan_host import check_subplan, ref_opts


@settings(max_examples=60, deadline=None, suppress_health_check=[HealthCheck.too_slow])
@given(M=st.integers(1, 90), Kc=st.integers(1, 120), density=st.floats(0.0, 0.5), seed=st.integers(0, 10_000),
       W=st.sampled_from([1, 4, 8, 16, 32]), KB=st.sampled_from([1, 4, 16, 64]),
       tau=st.integers(1, 6), tau_blk=st.integers(1, 64), ts=st.integers(1, 5), cs=st.integers(1, 20),
       short_len=st.integers(1, 4), sddmm_cs=st.integers(1, 50), mode=st.integers(0, 2), flags=st.sampled_from([0, 1, 8, 9, 16, 17, 32, 33, 64, 128, 256, 257, 288]),
       threads=st.integers(1, 5), share=st.sampled_from([0, 0, 25, 60, 100]))
def test_random_plans_match_reference(M, Kc, density, seed, W, KB, tau, tau_blk, ts, cs, short_len, sddmm_cs, mode, flags, threads, share):
    A = wl.random_pattern(M, Kc, density, seed=seed, empty_rows=0.2)
    if M > 3 and Kc > 30:
        A = wl.with_long_rows(A, [M // 2], min(Kc, 40), seed=seed + 1)
    kw = dict(mode=mode, window_rows=W, block_cols=KB, spmm_min_vec_nnz=tau, sddmm_min_blk_nnz=tau_blk, ts=ts, cs=cs,
              short_len=short_len, sddmm_cs=sddmm_cs, flags=flags, sddmm_min_dense_pct=share)
    p = lb.Plan.from_csr(A, threads=threads, **kw)
    o = ref_opts(kw)
    check_subplan(A, p.export(0), pr.plan_spmm(A.M, A.rowptr, A.col, o), spmm=True)
    check_subplan(A, p.export(1), pr.plan_sddmm(A.M, A.rowptr, A.col, o), spmm=False)
    p.close()
