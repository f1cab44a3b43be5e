"""The oracle run end to end on workload 0 (tiny power-law graph): the invariants the
method must satisfy, checked with set/array library routines."""
import numpy as np
import pytest
import torch

from paper_2310_00837_amd import workload as W


@pytest.fixture(scope="module")
def w0():
    sp = W.spec(0)
    g = W.make_graph(sp, 1234, "cpu")
    feats = W.feature_rows(1234, torch.arange(g.n_nodes), sp.dim, sp.dtype).numpy().view(np.uint8)
    return sp, g, feats


@pytest.mark.parametrize("batch", [0, 1, 2])
def test_pipeline_invariants(oracle, w0, batch):
    sp, g, feats = w0
    off, idx, order = g.offsets.numpy(), g.indices.numpy(), g.order.numpy()
    seeds = W.seed_batch(sp, g, batch).numpy()
    hops = oracle.sample(off, idx, seeds, sp.fanouts, W.batch_rng_seed(1234, batch))
    for h, (fr, ip, fl) in enumerate(hops):
        deg = off[fr + 1] - off[fr]
        assert (np.diff(ip) == np.minimum(deg, sp.fanouts[h])).all()
        for i in range(0, fr.size, 7):
            row = idx[off[fr[i]]:off[fr[i] + 1]]
            mine = fl[ip[i]:ip[i + 1]]
            assert np.isin(mine, row).all() and np.unique(mine).size == mine.size
    cat = np.concatenate([seeds] + [fl for _, _, fl in hops])
    uniq, inv = oracle.dedup(g.n_nodes, cat)
    assert set(uniq.tolist()) == set(cat.tolist()) and np.unique(uniq).size == uniq.size    # I4
    assert (uniq[:seeds.size] == seeds).all()                                               # distinct seeds stay a prefix
    assert (uniq[inv] == cat).all()
    n_hbm, n_host, n_rest = sp.tier_rows(g.n_nodes)
    rank = oracle.rank_build(order)
    by_rank = feats[order]
    out = np.full((uniq.size, sp.row_bytes), 0xA5, np.uint8)
    mp, mi, ms, stats = oracle.gather(uniq, rank, n_hbm, n_host, np.ascontiguousarray(by_rank[:n_hbm]),
                                      np.ascontiguousarray(by_rank[n_hbm:n_hbm + n_host]), out)
    assert stats[1] + stats[2] + stats[3] == uniq.size == stats[0]                          # I7
    r = rank[uniq]
    assert stats[1] == (r < n_hbm).sum() and stats[3] == (r >= n_hbm + n_host).sum()
    oracle.gather_miss(mp, ms, np.ascontiguousarray(by_rank[n_hbm + n_host:]), out)
    assert (out == feats[uniq]).all()                                                       # I6
    # skew: the raw sampled IDs hit the top-10 % tier far more often than 10 % (cf. Sec. 3.2.1)
    raw = np.concatenate([fl for _, _, fl in hops])
    assert (rank[raw] < n_hbm).mean() > 0.35
