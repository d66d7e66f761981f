"""GPU parity of the locality reordering: permutation, relabelled CSR and row maps, called through
the C ABI, bit-exact against the reordering oracle; then the permutation-in / permutation-out
contract end to end (a layer on the relabelled graph, mapped back, against the forward oracle on
the original graph)."""
import numpy as np
import pytest
import torch

import synth
from oracle import ftc_oracle_reorder as OR
from parity import TOL, dev_graph, norm_err, quantise
from paper_2412_12218_amd import binding as B

pytestmark = pytest.mark.gpu

F32, F16, BF16 = torch.float32, torch.float16, torch.bfloat16


def say(msg):
    print(msg, flush=True)


def skewed_graph():
    """Degrees from 0 to 70 000 (a row longer than many sorting tiles), duplicates, unsorted
    columns, n not a multiple of anything convenient."""
    rng = np.random.default_rng(17)
    n = 9973
    deg = rng.integers(0, 40, size=n)
    deg[::7] = 0
    deg[100] = 70_000
    deg[101] = 4096
    deg[n - 1] = 2049
    row_ptr = np.zeros(n + 1, dtype=np.int32)
    row_ptr[1:] = np.cumsum(deg)
    col = rng.integers(0, n, size=int(row_ptr[-1])).astype(np.int32)
    return synth.Graph(n, row_ptr, col, "skewed")


@pytest.fixture(scope="module")
def graphs():
    return {
        "cfg1": synth.config_graph(1),
        "cfg2s": synth.config_graph(2, 0.2),
        "cfg5s": synth.config_graph(5, 1 / 32),
        "skewed": skewed_graph(),
        "one": synth.Graph(1, np.array([0, 1], dtype=np.int32), np.array([0], dtype=np.int32), "one"),
        "no_edges": synth.Graph(50, np.zeros(51, dtype=np.int32), np.zeros(0, dtype=np.int32), "no_edges"),
    }


@pytest.mark.parametrize("name", ["cfg1", "cfg2s", "cfg5s", "skewed", "one", "no_edges"])
@pytest.mark.parametrize("mode", [B.FTC_ORDER_DEGREE, B.FTC_ORDER_DEGREE_CLASSES])
def test_degree_order_and_permute_graph(graphs, name, mode):
    g = graphs[name]
    say(f"reorder {name} n={g.n} nnz={g.nnz} mode={mode}")
    perm_ref, inv_ref = OR.degree_order(g.row_ptr, mode)
    dg = dev_graph(g)
    perm, inv = B.ftc_degree_order(dg, mode)
    assert np.array_equal(perm.cpu().numpy().astype(np.int64), perm_ref)
    assert np.array_equal(inv.cpu().numpy().astype(np.int64), inv_ref)
    rp_ref, ci_ref = OR.permute_graph(g.row_ptr, g.col_idx, perm_ref, inv_ref)
    pg, flag = B.ftc_permute_graph(dg, perm, inv)
    assert int(flag.item()) == 0
    assert np.array_equal(pg.row_ptr.cpu().numpy().astype(np.int64), rp_ref)
    assert np.array_equal(pg.col_idx.cpu().numpy().astype(np.int64), ci_ref)
    pg2, _ = B.ftc_permute_graph(dg, perm, inv)                 # same answer again
    assert torch.equal(pg.col_idx, pg2.col_idx) and torch.equal(pg.row_ptr, pg2.row_ptr)


def test_permute_graph_with_a_callers_permutation(graphs):
    """Any permutation is accepted, not only the library's own orderings."""
    g = graphs["cfg2s"]
    rng = np.random.default_rng(4)
    perm_ref = rng.permutation(g.n)
    inv_ref = np.empty(g.n, dtype=np.int64)
    inv_ref[perm_ref] = np.arange(g.n)
    rp_ref, ci_ref = OR.permute_graph(g.row_ptr, g.col_idx, perm_ref, inv_ref)
    perm = torch.from_numpy(perm_ref.astype(np.int32)).cuda()
    inv = torch.from_numpy(inv_ref.astype(np.int32)).cuda()
    pg, flag = B.ftc_permute_graph(dev_graph(g), perm, inv)
    assert int(flag.item()) == 0
    assert np.array_equal(pg.row_ptr.cpu().numpy().astype(np.int64), rp_ref)
    assert np.array_equal(pg.col_idx.cpu().numpy().astype(np.int64), ci_ref)


def test_permute_graph_flags_what_is_not_a_permutation(graphs):
    g = graphs["cfg1"]
    dg = dev_graph(g)
    perm, inv = B.ftc_degree_order(dg)
    bad = perm.clone()
    bad[5] = bad[6]                                   # a repeated id
    _, flag = B.ftc_permute_graph(dg, bad, inv)
    assert int(flag.item()) == 1
    bad = perm.clone()
    bad[0] = g.n + 3                                  # out of range: must not be followed
    _, flag = B.ftc_permute_graph(dg, bad, inv)
    assert int(flag.item()) == 1
    bad_inv = inv.clone()
    bad_inv[9] = -1
    _, flag = B.ftc_permute_graph(dg, perm, bad_inv)
    assert int(flag.item()) == 1
    _, flag = B.ftc_permute_graph(dg, perm, inv)      # and the valid pair is still accepted
    assert int(flag.item()) == 0


@pytest.mark.parametrize("dtype,D,ld", [(F16, 32, 32), (F32, 16, 16), (BF16, 24, 24), (F16, 5, 5), (F32, 7, 12),
                                        (F16, 8, 24)])
def test_permute_rows(dtype, D, ld):
    n = 4099
    rng = np.random.default_rng(1)
    perm = rng.permutation(n)
    inv = np.empty(n, dtype=np.int64)
    inv[perm] = np.arange(n)
    full = torch.from_numpy(synth.normal_features(n, ld, seed=2)).to(dtype).cuda()
    X = full[:, :D]
    pd, idd = torch.from_numpy(perm.astype(np.int32)).cuda(), torch.from_numpy(inv.astype(np.int32)).cuda()
    Xp = B.ftc_permute_rows(X, pd)
    assert torch.equal(Xp.cpu(), X.cpu()[torch.from_numpy(perm)])
    back = B.ftc_permute_rows(Xp, idd)
    assert torch.equal(back, X.contiguous())
    bad = pd.clone()
    bad[3] = -7
    Xz = B.ftc_permute_rows(X, bad)
    assert torch.all(Xz[3] == 0) and torch.equal(Xz[4], Xp[4])


@pytest.mark.parametrize("name", ["cfg2s", "cfg5s", "skewed"])
def test_layers_on_the_relabelled_graph_match_the_original(oracle, graphs, name):
    """Permutation in, permutation out: GCN and AGNN layers computed on the relabelled graph and
    mapped back equal the oracle's layers on the original graph."""
    g = graphs[name]
    dg = dev_graph(g)
    perm, inv = B.ftc_degree_order(dg)
    pg, _ = B.ftc_permute_graph(dg, perm, inv)
    win = B.ftc_build_windows(pg)
    _, dinv = B.ftc_gcn_norm(pg, win, want_vals=False)
    Xd, X64 = quantise(synth.uniform_features(g.n, 64, seed=9), F16)
    Wd, W64 = quantise(synth.glorot_uniform(64, 16, seed=10), F16)
    out_p = B.ftc_gcn_layer(pg, win, None, B.ftc_permute_rows(Xd, perm), Wd, relu=True, dinv=dinv)
    out = B.ftc_permute_rows(out_p, inv)
    _, dinv64 = oracle.gcn_norm(g.row_ptr, g.col_idx)
    d32 = np.nan_to_num(dinv64, posinf=0.0).astype(np.float32).astype(np.float64)
    rows = np.repeat(np.arange(g.n), np.diff(g.row_ptr))
    ref, ab = oracle.gcn_layer(g.row_ptr, g.col_idx, d32[rows] * d32[g.col_idx], X64, W64, relu=True)
    err = norm_err(out, ref, ab)
    say(f"gcn layer through the reordering, {name}: err {err:.3e}")
    assert err < TOL[F16]
    Hd, H64 = quantise(synth.normal_features(g.n, 32, seed=11), F16)
    ref, ab, _ = oracle.agnn_layer(g.row_ptr, g.col_idx, H64, 1.0)
    out = B.ftc_permute_rows(B.ftc_agnn_layer(pg, win, B.ftc_permute_rows(Hd, perm)), inv)
    err = norm_err(out, ref, ab)
    say(f"agnn layer through the reordering, {name}: err {err:.3e}")
    assert err < TOL[F16]


@pytest.mark.parametrize("name", ["cfg1", "cfg5s", "skewed", "no_edges"])
def test_degree_stats_and_plan_from_device_numbers(graphs, name):
    """Sum of squared row lengths and longest row, exact; then the plan from the numbers the device
    produced (statistics + the window build's summary)."""
    g = graphs[name]
    deg = np.diff(g.row_ptr).astype(np.int64)
    dg = dev_graph(g)
    stats = B.ftc_degree_stats(dg).cpu().numpy()
    assert int(stats[0]) == int((deg * deg).sum()) and int(stats[1]) == int(deg.max())
    win = B.ftc_build_windows(dg)
    plan = B.ftc_plan_graph(g.n, g.nnz, int(stats[0]), int(win.summary[0].item()), 32, F16)
    say(f"plan {name}: {plan}")
    expect = name in ("cfg5s",) and g.n * 64 > 4 << 20
    assert (plan["reorder"] != B.FTC_ORDER_NONE) == expect
    if g.nnz:
        assert plan["reuse"] >= 1.0 and plan["skew"] >= 1.0 - 1e-9


# ------------------------------------------------------------------ the plan carried out
@pytest.mark.parametrize("which", ["rmat", "sbm", "small"])
def test_planned_graph_applies_the_plan_and_keeps_the_original_numbering(oracle, which):
    """PlannedGraph: statistics -> plan -> relabelled graph.  The skewed R-MAT graph is relabelled by degree
    class, the permuted block model gets the community trial and keeps it (its windows then share columns),
    a graph whose features fit one L2 is left alone; in every case a GCN layer and an AGNN layer run through
    enter() / leave() equal the oracle on the graph as given."""
    from paper_2412_12218_amd.models import PlannedGraph
    if which == "rmat":
        g, dtype, D, expect = synth.config_graph(5, 1 / 16), F16, 64, "degree classes"
    elif which == "sbm":
        g, dtype, D, expect = synth.config_graph(4, 0.05), BF16, 64, "communities"
    else:
        g, dtype, D, expect = synth.config_graph(1), F16, 32, "none"
    dg = dev_graph(g)
    pl = PlannedGraph(dg, D, dtype)
    say(f"planned {which}: n={g.n} nnz={g.nnz} plan={pl.plan} applied={pl.applied} sum_uniq {pl.sum_uniq_given} -> {pl.sum_uniq}")
    assert pl.applied == expect
    if which == "sbm":
        assert pl.sum_uniq < 0.98 * pl.sum_uniq_given
    _, dinv = B.ftc_gcn_norm(pl.g, pl.win, want_vals=False)
    Xd, X64 = quantise(synth.uniform_features(g.n, D, seed=9), dtype)
    Wd, W64 = quantise(synth.glorot_uniform(D, 16, seed=10), dtype)
    out = pl.leave(B.ftc_gcn_layer(pl.g, pl.win, None, pl.enter(Xd), Wd, relu=True, dinv=dinv))
    _, dinv64 = oracle.gcn_norm(g.row_ptr, g.col_idx)
    d32 = dinv64.astype(np.float32).astype(np.float64)
    rows = np.repeat(np.arange(g.n), np.diff(g.row_ptr))
    ref, ab = oracle.gcn_layer(g.row_ptr, g.col_idx, d32[rows] * d32[g.col_idx], X64, W64, relu=True)
    err = norm_err(out, ref, ab)
    say(f"  gcn layer on the planned graph: err {err:.3e}")
    assert err < TOL[dtype]
    Hd, H64 = quantise(synth.normal_features(g.n, D, seed=11), dtype)
    ref, ab, _ = oracle.agnn_layer(g.row_ptr, g.col_idx, H64, 1.0)
    out = pl.leave(B.ftc_agnn_layer(pl.g, pl.win, pl.enter(Hd)))
    err = norm_err(out, ref, ab)
    say(f"  agnn layer on the planned graph: err {err:.3e}")
    assert err < TOL[dtype]


def test_planned_graph_drops_a_community_trial_that_does_not_help():
    """The block model once more, this time already in community order (the graph the first plan produced):
    the plan proposes the trial again (the statistics cannot see the order), the relabelled windows share no
    more columns than before, and the graph stays as it is."""
    from paper_2412_12218_amd.models import PlannedGraph
    g = synth.config_graph(4, 0.05)
    first = PlannedGraph(dev_graph(g), 64, BF16)
    assert first.applied == "communities"
    pl = PlannedGraph(first.g, 64, BF16)
    say(f"planned twice: plan={pl.plan} applied={pl.applied} trial={getattr(pl, 'trial', None)}")
    assert pl.plan["reorder"] == B.FTC_ORDER_COMMUNITIES
    assert pl.applied == "none" and pl.trial["kept"] is False and pl.perm is None and pl.g is first.g


# ------------------------------------------------------------------ community ordering
def sbm_small():
    return synth.sbm(12, 200, 14 * 12 * 200, 2 * 12 * 200, seed=5)


@pytest.mark.parametrize("name", ["cfg1", "sbm", "skewed", "one", "no_edges"])
@pytest.mark.parametrize("rounds", [0, 1, 4])
def test_label_propagation(graphs, name, rounds):
    g = sbm_small() if name == "sbm" else graphs[name]
    say(f"label propagation {name} n={g.n} nnz={g.nnz} rounds={rounds}")
    ref = OR.label_propagation(g.row_ptr, g.col_idx, rounds)
    lab = B.ftc_label_propagation(dev_graph(g), rounds)
    assert np.array_equal(lab.cpu().numpy().astype(np.int64), ref)


def test_community_order_recovers_the_blocks_and_concentrates_the_columns(oracle):
    """Ten rounds on the permuted block model, then the ordering by label: bit-exact against the
    oracle, and the relabelled graph's windows hold far fewer distinct columns."""
    g = sbm_small()
    dg = dev_graph(g)
    lab = B.ftc_label_propagation(dg, 10)
    ref = OR.label_propagation(g.row_ptr, g.col_idx, 10)
    assert np.array_equal(lab.cpu().numpy().astype(np.int64), ref)
    perm, inv, flag = B.ftc_order_by_key(lab)
    perm_ref, inv_ref = OR.order_by_key(ref)
    assert int(flag.item()) == 0
    assert np.array_equal(perm.cpu().numpy().astype(np.int64), perm_ref)
    assert np.array_equal(inv.cpu().numpy().astype(np.int64), inv_ref)
    pg, pflag = B.ftc_permute_graph(dg, perm, inv)
    assert int(pflag.item()) == 0
    before = int(B.ftc_build_windows(dg).summary[0].item())
    after = int(B.ftc_build_windows(pg).summary[0].item())
    say(f"distinct window columns {before} -> {after} of {g.nnz} entries")
    assert after < 0.75 * before


def test_order_by_key_random_keys_and_negative_flag():
    rng = np.random.default_rng(3)
    n = 70_001
    keys = rng.integers(0, 50, size=n).astype(np.int32)
    keys[::1000] = rng.integers(1 << 20, (1 << 31) - 1, size=keys[::1000].size)     # all four digit passes matter
    perm_ref, inv_ref = OR.order_by_key(keys)
    perm, inv, flag = B.ftc_order_by_key(torch.from_numpy(keys).cuda())
    assert int(flag.item()) == 0
    assert np.array_equal(perm.cpu().numpy().astype(np.int64), perm_ref)
    assert np.array_equal(inv.cpu().numpy().astype(np.int64), inv_ref)
    keys[5] = -3
    _, _, flag = B.ftc_order_by_key(torch.from_numpy(keys).cuda())
    assert int(flag.item()) == 1
