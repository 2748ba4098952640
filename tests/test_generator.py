"""Structure checks for the seeded synthetic-input generator."""
import numpy as np
import pytest

import sdt_gen as gen


def _check_csr(indptr, indices, n):
    assert indptr[0] == 0 and indptr[-1] == len(indices) and len(indptr) == n + 1
    assert indices.min() >= 0 and indices.max() < n
    rows = np.repeat(np.arange(n), np.diff(indptr))
    assert not np.any(rows == indices)                                   # no self-loops
    key = rows.astype(np.int64) * n + indices
    assert np.all(np.diff(key) > 0)                                      # sorted rows, no duplicates
    rkey = np.sort(indices.astype(np.int64) * n + rows)
    assert np.array_equal(key, rkey)                                     # (u,v) present <=> (v,u) present


def test_rmat_structure_and_degree():
    wl = gen.WORKLOADS["tiny"]
    indptr, indices = gen.make_graph(wl)
    _check_csr(indptr, indices, wl.n_nodes)
    avg = len(indices) / wl.n_nodes
    assert 0.8 * wl.avg_deg <= avg <= wl.avg_deg                          # duplicates only lower it
    deg = np.diff(indptr)
    assert deg.max() > 20 * avg                                           # heavy tail
    ip2, ix2 = gen.make_graph(wl)
    assert np.array_equal(indptr, ip2) and np.array_equal(indices, ix2)   # deterministic


def test_chunglu_structure_and_tail():
    n = 1 << 12
    ip, ix = gen.chunglu_csr(n, n * 40 // 2, 40.0, 2.1, seed=2)
    _check_csr(ip, ix, n)
    deg = np.sort(np.diff(ip))[::-1].astype(np.float64)
    assert 0.6 * 40 <= deg.mean() <= 40
    # power-law tail: log-log CCDF slope about -(gamma-1) = -1.1 between the 1 % and 20 % quantiles
    ranks = np.arange(1, n + 1) / n
    sel = (ranks > 0.01) & (ranks < 0.2)
    slope = np.polyfit(np.log(deg[sel]), np.log(ranks[sel]), 1)[0]
    assert -1.6 < slope < -0.7, slope


def test_features_labels_weights_batches():
    X = gen.normal_features(4096, 64, seed=0)
    assert abs(X.mean()) < 0.01 and abs(X.std() - 1) < 0.01
    Xb = gen.normal_features(4096, 64, seed=0, bf16=True)
    hi = (X.view(np.uint32) >> 16).astype(np.int64)
    assert np.all(np.abs(Xb.astype(np.int64) - hi) <= 1)                  # rounding of the same draws
    y = gen.labels(100000, 47, seed=1)
    cnt = np.bincount(y, minlength=47)
    assert y.min() >= 0 and y.max() == 46 and cnt.min() > 1800 and cnt.max() < 2500
    W, b = gen.glorot_sage_weights([100, 256, 47], seed=1)
    assert W[0].shape == (200, 256) and W[1].shape == (512, 47) and not b[0].any()
    lim = np.sqrt(6.0 / (100 + 256))
    assert np.abs(W[0]).max() <= lim and np.abs(W[0]).max() > 0.99 * lim and abs(W[0].mean()) < 0.01 * lim * 3
    s0, s1 = gen.seed_batch(256, 0, 8192, 0, 0), gen.seed_batch(256, 0, 8192, 0, 1)
    assert len(np.unique(s0)) == 256 and s0.min() >= 0 and s0.max() < 8192 and not np.array_equal(s0, s1)
    assert sorted(gen.seed_batch(16, 5, 21, 0, 0)) == list(range(5, 21))  # range == batch: a permutation
    with pytest.raises(ValueError):
        gen.seed_batch(10, 0, 5, 0, 0)


def test_workload_table_matches_the_configs():
    w = gen.WORKLOADS
    assert w["tiny"].dims == [64, 64, 8] and w["tiny"].fanouts == [10, 5] and w["tiny"].batch == 256
    assert w["products"].dims == [100, 256, 47] and w["products"].log2n == 21
    assert w["dense"].dims == [602, 256, 41] and w["dense"].fanouts == [25, 10]
    assert w["sparse_bf16"].dims == [128, 256, 256, 172] and w["sparse_bf16"].bf16
    assert w["fullgraph"].dims == [256, 256] and w["fullgraph"].log2n == 22


def test_partition_instance_recipe():
    """A partition with replicas: owned nodes of all partitions tile the graph, features and labels are
    the global nodes', seeds are owned nodes, the local graph of an owned node is its global one."""
    wl = gen.Workload("part", "rmat", 11, 10, 16, 5, 16, 2, [4, 3], 32, 9, 1)
    ip, ix = gen.drop_isolated(*gen.make_graph(wl))
    n = len(ip) - 1
    assert np.all(np.diff(ip) > 0) and ix.max() == n - 1
    X = gen.normal_features(n, wl.feat, wl.seed)
    y = gen.labels(n, wl.classes, wl.seed)
    seen = np.zeros(n, dtype=np.int64)
    for k in range(3):
        inst = gen.make_partition_instance(wl, p=3, which=k)
        gid = inst.global_id
        seen[gid[:inst.n_owned]] += 1
        assert inst.n_nodes == len(gid) and inst.info["n_global"] == n
        assert np.array_equal(inst.X, X[gid]) and np.array_equal(inst.y, y[gid])
        b = inst.batch(0)
        assert b.min() >= 0 and b.max() < inst.n_owned and len(set(b.tolist())) == wl.batch
        for i in (0, inst.n_owned // 2, inst.n_owned - 1):          # owned rows: the global neighbour list
            loc = inst.indices[inst.indptr[i]:inst.indptr[i + 1]]
            assert sorted(gid[loc].tolist()) == ix[ip[gid[i]]:ip[gid[i] + 1]].tolist()
        for i in range(inst.n_owned, inst.n_nodes):                 # replica rows: owned neighbours only
            loc = inst.indices[inst.indptr[i]:inst.indptr[i + 1]]
            assert len(loc) > 0 and loc.max() < inst.n_owned
    assert np.all(seen == 1)
