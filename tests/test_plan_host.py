"""Host logic of the per-graph plan (no GPU): ftc_plan_graph on the statistics of the benchmark
graphs must pick what the measurements picked (relabelling paid on the skewed graphs whose feature
matrix exceeds one L2, and nowhere else), and reject inconsistent arguments."""
import numpy as np
import pytest
import torch

import synth
from paper_2412_12218_amd import binding as B

F32, F16, BF16 = torch.float32, torch.float16, torch.bfloat16


def stats_of(g, oracle):
    deg = np.diff(g.row_ptr).astype(np.int64)
    sum_uniq = int(oracle.build_windows(g.row_ptr, g.col_idx)["summary"][0])
    return int((deg * deg).sum()), sum_uniq


NONE, CLASSES, COMM = B.FTC_ORDER_NONE, B.FTC_ORDER_DEGREE_CLASSES, B.FTC_ORDER_COMMUNITIES


@pytest.mark.parametrize("cfg,scale,D,dtype,reorder", [
    (1, 1.0, 16, F32, NONE),       # Erdos-Renyi: skew 1.1, 128 KB of features
    (2, 1.0, 32, F16, CLASSES),    # Chung-Lu, skew 9.3, 6.4 MB of features
    (3, 1.0, 32, F16, CLASSES),    # Chung-Lu, skew 7.8
    (4, 0.1, 64, BF16, COMM),      # SBM: flat degrees, 12.8 MB of features: only communities can help
    (4, 0.02, 64, BF16, NONE),     # ... but not while everything fits one L2
    (5, 0.25, 32, F16, CLASSES),   # R-MAT at a quarter of the benchmark size: 16 MB of features
    (5, 1 / 64, 32, F16, NONE),    # the same skew, but 1 MB of features: everything stays in L2
])
def test_plan_reorders_where_the_measurements_say_it_pays(oracle, cfg, scale, D, dtype, reorder):
    g = synth.config_graph(cfg, scale)
    sq, su = stats_of(g, oracle)
    plan = B.ftc_plan_graph(g.n, g.nnz, sq, su, D, dtype)
    deg = np.diff(g.row_ptr).astype(np.float64)
    assert plan["skew"] == pytest.approx(g.n * (deg * deg).sum() / g.nnz ** 2, rel=1e-12)
    assert plan["reuse"] == pytest.approx(g.nnz / su, rel=1e-12)
    assert plan["reorder"] == reorder


def test_plan_reports_what_the_kernels_cover():
    base = dict(n=1 << 20, nnz=1 << 25, sum_deg_sq=(1 << 25) * 40, sum_uniq=1 << 24)
    p = B.ftc_plan_graph(D=32, dtype=F16, **base)
    assert p["agnn_single_pass"] == 1 and p["agnn_backward_single_pass"] == 1
    assert p["spmm_mfma_windows"] == 0 and p["sddmm_mfma_windows"] == 0 and p["mfma_min_reuse"] < 0
    p = B.ftc_plan_graph(D=256, dtype=F16, **base)
    assert p["sddmm_mfma_windows"] == 1 and p["mfma_min_reuse"] == pytest.approx(2.6)
    assert p["spmm_mfma_windows"] == 0                       # the vector path won at every density measured
    assert p["agnn_single_pass"] == 1 and p["agnn_backward_single_pass"] == 0
    p = B.ftc_plan_graph(D=256, dtype=F32, **base)
    assert p["sddmm_mfma_windows"] == 0                       # the matrix-core path is 16-bit only


def test_plan_rejects_inconsistent_statistics():
    with pytest.raises(B.FtcError):
        B.ftc_plan_graph(100, 1000, 20000, 1001, 32, F16)     # more distinct columns than entries
    with pytest.raises(B.FtcError):
        B.ftc_plan_graph(100, 1000, -1, 900, 32, F16)
    with pytest.raises(B.FtcError):
        B.ftc_plan_graph(100, 1000, 20000, 900, 0, F16)
    empty = B.ftc_plan_graph(0, 0, 0, 0, 32, F16)
    assert empty["skew"] == 0 and empty["reuse"] == 0 and empty["reorder"] == B.FTC_ORDER_NONE
