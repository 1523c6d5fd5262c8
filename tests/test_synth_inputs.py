"""The seeded input generators: shape, determinism and the stated structure."""
import numpy as np

import synth


def test_rmat_structure_and_thread_independence():
    n, e = 5000, 60000
    ip1, ix1 = synth.rmat_csr(n, e, seed=7, threads=1)
    ip4, ix4 = synth.rmat_csr(n, e, seed=7, threads=4)
    assert np.array_equal(ip1, ip4) and np.array_equal(ix1, ix4)
    assert ip1[0] == 0 and ip1[-1] == e and (np.diff(ip1) >= 0).all()
    assert ix1.min() >= 0 and ix1.max() < n
    for v in np.random.default_rng(0).integers(0, n, 200):
        lst = ix1[ip1[v]:ip1[v + 1]]
        assert (np.diff(lst) >= 0).all()
    deg = np.diff(ip1)
    assert deg.max() > 20 * deg.mean()          # heavy tail
    ip2, ix2 = synth.rmat_csr(n, e, seed=8)
    assert not np.array_equal(ix1, ix2)


def test_seeds_distinct_and_features_normal():
    s = synth.seeds(16384, 2048, 3)
    assert len(np.unique(s)) == 2048 and s.min() >= 0 and s.max() < 16384
    assert np.array_equal(s, synth.seeds(16384, 2048, 3))
    f = synth.features(4000, 63, 2)              # odd total exercises the pair tail
    assert f.shape == (4000, 63) and abs(f.mean()) < 0.01 and abs(f.std() - 1.0) < 0.01
    assert np.array_equal(f, synth.features(4000, 63, 2, threads=3))


def test_workload_table():
    w = synth.WORKLOADS["tiny"]
    assert w.adj_bytes == 1_441_800 and w.feat_bytes == 4_194_304 and w.budget_bytes == 1_127_220
    assert w.dims == (64, 64, 16) and w.num_batches == 8
    m = synth.WORKLOADS["medium"]
    assert m.dims == (602, 256, 256, 41) and m.cap_nodes() == [1024, 6144, 67584, 232965]
    assert m.cap_edges() == [5120, 61440, 1013760]
    ws, wn, b = synth.sage_weights(w.dims, w.weight_seed)
    assert [x.shape for x in ws] == [(64, 64), (64, 16)] and not np.array_equal(ws[0], wn[0])
    assert abs(ws[0]).max() <= np.sqrt(6 / 128) + 1e-7
