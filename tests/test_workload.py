"""Properties of the seeded input generators (CPU, small scales)."""
import hashlib

import numpy as np
import pytest
import torch

from paper_2310_00837_amd import workload as W


@pytest.fixture(scope="module")
def g0():
    return W.make_graph(W.spec(0), 1234, "cpu")


def test_graph_shape_and_rows(g0):
    sp = W.spec(0)
    assert g0.n_nodes == sp.n_nodes and 0.9 * sp.n_edges < g0.n_edges <= 1.02 * sp.n_edges
    off, idx = g0.offsets.numpy(), g0.indices.numpy()
    assert off[0] == 0 and off[-1] == idx.size and (np.diff(off) >= 0).all()
    assert idx.min() >= 0 and idx.max() < g0.n_nodes
    for v in range(0, g0.n_nodes, 37):
        row = idx[off[v]:off[v + 1]]
        assert (np.diff(row) > 0).all()          # sorted, duplicate-free
        assert v not in row                      # no self loop
    deg = np.diff(off)
    assert deg.max() > 20 * np.median(deg)       # heavy tail


def test_generation_is_deterministic(g0):
    again = W.make_graph(W.spec(0), 1234, "cpu")
    assert torch.equal(again.offsets, g0.offsets) and torch.equal(again.indices, g0.indices)
    assert torch.equal(again.order, g0.order)
    other = W.make_graph(W.spec(0), 1235, "cpu")
    assert not torch.equal(other.indices[:1000], g0.indices[:1000])


def test_hotness_order_is_in_degree_descending_with_id_ties(g0):
    n = g0.n_nodes
    indeg = np.bincount(g0.indices.numpy(), minlength=n)
    order = g0.order.numpy()
    assert sorted(order.tolist()) == list(range(n))
    want = sorted(range(n), key=lambda v: (-indeg[v], v))
    assert order.tolist() == want


def test_tier_rows_closed_forms():
    assert W.spec(0).tier_rows() == (1000, 2000, 7000)
    assert W.spec(1).tier_rows() == (100_000, 300_000, 600_000)
    assert W.spec(2).tier_rows() == (39_062_500, 58_593_750, 13_343_750)
    assert W.spec(3).tier_rows() == (31_250_000, 11_718_750, 7_031_250)
    assert W.spec(4, 0.0).tier_rows() == (0, 55_500_000, 55_500_000)
    assert W.spec(4, 0.25).tier_rows() == (27_750_000, 41_625_000, 41_625_000)
    assert W.spec(4, 1.0).tier_rows() == (111_000_000, 0, 0)
    assert W.spec(2).row_bytes == 512 and W.spec(3).row_bytes == 2048 and W.spec(0).row_bytes == 256


def test_features_exact_and_in_range():
    ids = torch.tensor([0, 1, 5, 99_999_999])
    f32 = W.feature_rows(7, ids, 128, torch.float32)
    f16 = W.feature_rows(7, ids, 1024, torch.float16)
    assert f32.dtype == torch.float32 and f16.dtype == torch.float16
    assert float(f32.min()) >= -1 and float(f32.max()) < 1 and float(f16.min()) >= -1 and float(f16.max()) < 1
    assert torch.equal((f32.double() + 1) * 2 ** 23, torch.round((f32.double() + 1) * 2 ** 23))
    assert torch.equal((f16.double() + 1) * 2 ** 10, torch.round((f16.double() + 1) * 2 ** 10))
    # a row depends on (seed, id) only, not on the batch it is generated in
    assert torch.equal(W.feature_rows(7, ids[2:3], 128, torch.float32)[0], f32[2])
    assert not torch.equal(W.feature_rows(8, ids, 128, torch.float32), f32)
    assert abs(float(f16.float().mean())) < 0.05
    dst = torch.empty(4, 128)
    W.fill_rows(dst, 7, ids, chunk_elems=256)
    assert torch.equal(dst, f32)


def test_seed_batches(g0):
    sp = W.spec(0)
    n_train = int(0.10 * g0.n_nodes)
    train = set(g0.perm_seed[:n_train].tolist())
    b0, b1 = W.seed_batch(sp, g0, 0), W.seed_batch(sp, g0, 1)
    assert b0.dtype == torch.int32 and b0.numel() == 128
    assert len(set(b0.tolist())) == 128 and set(b0.tolist()) <= train
    assert not (set(b0.tolist()) & set(b1.tolist()))       # consecutive batches of one epoch are disjoint
    assert torch.equal(W.seed_batch(sp, g0, 0), b0)
    z = W.spec(4)
    z.batch = 4096
    zs = W.seed_batch(z, g0, 0)
    top = g0.perm_seed[:10].tolist()
    share = sum(1 for v in zs.tolist() if v in top) / 4096
    want = np.log(11) / np.log(g0.n_nodes + 1)               # P(k <= 10) for the s = 1 law
    assert abs(share - want) < 0.04
    assert W.batch_rng_seed(1, 0) != W.batch_rng_seed(1, 1) != W.batch_rng_seed(2, 1)
    assert 0 <= W.batch_rng_seed(1, 5) < 2 ** 64


def test_golden_hash_of_config0_inputs(g0):
    # guards the generator against silent change; written by tests/golden/make_workload_hash.py
    import os
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden", "workload_cfg0_seed1234.sha256")
    h = hashlib.sha256()
    for t in (g0.offsets, g0.indices, g0.order, W.seed_batch(W.spec(0), g0, 0)):
        h.update(t.numpy().tobytes())
    h.update(W.feature_rows(1234, torch.arange(16), 64, torch.float32).numpy().tobytes())
    assert h.hexdigest() == open(path).read().split()[0]
