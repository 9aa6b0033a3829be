"""Pins for the CPU oracle: everything here checks ``oracle/`` against something that is not the
oracle - a hand-worked example, closed forms, scipy routines, exhaustive enumeration on tiny
inputs, and the invariants a minimum spanning tree and a linkage must satisfy."""
import itertools

import numpy as np
import pytest
import scipy.cluster.hierarchy as sch
import scipy.sparse as sp
import scipy.sparse.csgraph as csg
from scipy.spatial.distance import cdist

import oracle
import slhc_inputs as gen


# ----------------------------------------------------------------------------- helpers
def all_pairs_f64(X):
    """Every squared distance by explicit differences in float64 (numpy, no oracle code)."""
    Xd = X.astype(np.float64)
    diff = Xd[:, None, :] - Xd[None, :, :]
    return np.einsum("ijt,ijt->ij", diff, diff)


def exhaustive_knn(X, k):
    D = all_pairs_f64(X)
    N = X.shape[0]
    idx = np.empty((N, k), dtype=np.int64)
    dist = np.empty((N, k))
    for i in range(N):
        cand = [(D[i, j], j) for j in range(N) if j != i]
        cand.sort()
        idx[i] = [c[1] for c in cand[:k]]
        dist[i] = [c[0] for c in cand[:k]]
    return idx, dist


def kruskal_all_pairs(X):
    """Second MST algorithm: sort all N(N-1)/2 pairs by (w, lo, hi), union-find."""
    D = all_pairs_f64(X)
    N = X.shape[0]
    iu, ju = np.triu_indices(N, 1)
    w = D[iu, ju]
    order = np.lexsort((ju, iu, w))
    parent = list(range(N))

    def find(a):
        while parent[a] != a:
            parent[a] = parent[parent[a]]
            a = parent[a]
        return a

    edges = []
    for e in order:
        a, b = find(int(iu[e])), find(int(ju[e]))
        if a != b:
            parent[a] = b
            edges.append((int(iu[e]), int(ju[e]), float(w[e])))
            if len(edges) == N - 1:
                break
    return edges


def as_edge_set(src, dst):
    return {(min(int(a), int(b)), max(int(a), int(b))) for a, b in zip(src, dst)}


def check_spanning_tree(src, dst, N):
    assert len(src) == N - 1
    parent = list(range(N))

    def find(a):
        while parent[a] != a:
            parent[a] = parent[parent[a]]
            a = parent[a]
        return a

    for a, b in zip(src, dst):
        ra, rb = find(int(a)), find(int(b))
        assert ra != rb, "cycle"
        parent[ra] = rb
    assert len({find(v) for v in range(N)}) == 1


# ----------------------------------------------------------------------------- golden
def test_five_points_knn(golden_five_points):
    g = golden_five_points
    X = np.array(g["points"], dtype=np.float32)
    idx, dist = oracle.knn_graph(X, 2)
    exp = np.array(g["knn2"])
    assert idx.tolist() == exp[:, [0, 2]].astype(int).tolist()
    assert dist.tolist() == exp[:, [1, 3]].tolist()


def test_five_points_mst_and_dendrogram(golden_five_points):
    g = golden_five_points
    X = np.array(g["points"], dtype=np.float32)
    out = oracle.slhc(X)
    exp_mst = np.array(g["mst"])
    assert out["src"].tolist() == exp_mst[:, 0].astype(int).tolist()
    assert out["dst"].tolist() == exp_mst[:, 1].astype(int).tolist()
    assert out["w"].tolist() == exp_mst[:, 2].tolist()
    assert out["total_weight"] == 109.0
    exp_d = np.array(g["dendrogram"])
    assert out["children"].tolist() == exp_d[:, :2].astype(int).tolist()
    assert out["heights"].tolist() == exp_d[:, 2].tolist()
    assert out["sizes"].tolist() == exp_d[:, 3].astype(int).tolist()


# ----------------------------------------------------------------------------- kNN
@pytest.mark.parametrize("N,d,k", [(5, 1, 4), (17, 3, 5), (64, 16, 16), (33, 7, 32)])
def test_knn_exhaustive_small(N, d, k):
    X = np.random.default_rng(N * 100 + d).standard_normal((N, d)).astype(np.float32)
    idx, dist = oracle.knn_graph(X, k)
    eidx, edist = exhaustive_knn(X, k)
    assert np.array_equal(idx, eidx)
    np.testing.assert_allclose(dist, edist, rtol=1e-14, atol=0)


def test_knn_vs_scipy_cdist():
    X, _, k = gen.make("c1", n=1500)
    idx, dist = oracle.knn_graph(X, k)
    D = cdist(X.astype(np.float64), X.astype(np.float64), "sqeuclidean")
    np.fill_diagonal(D, np.inf)
    order = np.argsort(D, axis=1, kind="stable")[:, :k]
    assert np.array_equal(idx, order)
    np.testing.assert_allclose(dist, np.take_along_axis(D, order, 1), rtol=1e-12)


def test_knn_sampled_rows_match_full():
    X, _, k = gen.make("c2", n=3000)
    rows = np.array([0, 7, 2999, 1234, 7], dtype=np.int64)
    fi, fd = oracle.knn_graph(X, k)
    si, sd = oracle.knn_rows(X, rows, k)
    assert np.array_equal(si, fi[rows]) and np.array_equal(sd, fd[rows])


def test_knn_lattice_closed_form():
    # 5x5x5 integer lattice: all squared distances are exact small integers; ties everywhere.
    X = gen.integer_lattice(5, 3, seed=3)
    N, k = X.shape[0], 10
    idx, dist = oracle.knn_graph(X, k)
    Xi = X.astype(np.int64)
    for i in range(N):
        D = ((Xi - Xi[i]) ** 2).sum(1)
        cand = sorted((int(D[j]), j) for j in range(N) if j != i)[:k]
        assert idx[i].tolist() == [c[1] for c in cand]
        assert dist[i].tolist() == [float(c[0]) for c in cand]
    centre = int(np.where((Xi == 2).all(1))[0][0])
    assert dist[centre, :6].tolist() == [1.0] * 6 and dist[centre, 6:].tolist() == [2.0] * 4


def test_knn_invariants_and_duplicates():
    X, _, k = gen.make("c5", n=3000)
    N = X.shape[0]
    idx, dist = oracle.knn_graph(X, k)
    assert idx.min() >= 0 and idx.max() < N
    assert not (idx == np.arange(N)[:, None]).any(), "self listed"
    assert all(len(set(r)) == k for r in idx.tolist()), "repeat"
    assert (np.diff(dist, axis=1) >= 0).all()
    D = all_pairs_f64(X[:400])                       # selection bound on a corner of the matrix
    full = cdist(X[:50].astype(np.float64), X.astype(np.float64), "sqeuclidean")
    for i in range(50):
        unlisted = np.setdiff1d(np.arange(N), np.append(idx[i], i))
        assert full[i, unlisted].min() >= dist[i, -1]
    # exact duplicates exist in this workload: they sit at distance exactly 0 and are listed
    dup_rows = np.where(dist[:, 0] == 0.0)[0]
    assert dup_rows.size > 0
    for i in dup_rows[:20]:
        assert np.array_equal(X[i], X[idx[i, 0]]) and idx[i, 0] != i
    assert D.shape == (400, 400)


def test_knn_bad_arguments():
    X = np.zeros((4, 2), dtype=np.float32)
    with pytest.raises(ValueError):
        oracle.knn_graph(X, 4)          # k > N-1
    with pytest.raises(ValueError):
        oracle.knn_graph(X, 0)


# ----------------------------------------------------------------------------- cross-colour 1-NN
def test_cross_1nn_vs_numpy():
    X, labels, _ = gen.make("c1", n=600)
    colour = (labels % 3).astype(np.int32)
    rows = np.arange(0, 600, 7, dtype=np.int64)
    idx, dist = oracle.cross_1nn(X, colour, rows)
    D = all_pairs_f64(X)
    for q, i in enumerate(rows):
        Dm = np.where(colour != colour[i], D[i], np.inf)
        j = int(np.argmin(Dm))
        assert idx[q] == j and dist[q] == pytest.approx(Dm[j], rel=1e-14)
    one = np.zeros(600, dtype=np.int32)
    idx, dist = oracle.cross_1nn(X, one, rows)
    assert (idx == -1).all() and np.isinf(dist).all()


# ----------------------------------------------------------------------------- MST
@pytest.mark.parametrize("name,n", [("c1", 300), ("c2", 257), ("c4", 120)])
def test_mst_vs_kruskal(name, n):
    X, _, _ = gen.make(name, n=n)
    src, dst, w = oracle.mst_prim(X)
    check_spanning_tree(src, dst, n)
    kr = kruskal_all_pairs(X)
    assert as_edge_set(src, dst) == {(a, b) for a, b, _ in kr}
    assert np.sum(np.sort(w)) == pytest.approx(sum(sorted(e[2] for e in kr)), rel=1e-13)
    D = all_pairs_f64(X)
    np.testing.assert_allclose(w, D[src, dst], rtol=1e-14)


def test_mst_vs_scipy_csgraph():
    X, _, _ = gen.make("c1", n=1200)       # tie-free and zero-free, so csgraph is usable
    src, dst, w = oracle.mst_prim(X)
    D = cdist(X.astype(np.float64), X.astype(np.float64), "sqeuclidean")
    T = csg.minimum_spanning_tree(D).tocoo()
    assert as_edge_set(src, dst) == as_edge_set(T.row, T.col)
    assert np.sum(np.sort(w)) == pytest.approx(np.sum(np.sort(T.data)), rel=1e-12)


@pytest.mark.parametrize("N", [4, 7, 10])
def test_mst_cut_property_all_cuts(N):
    X = np.random.default_rng(N).standard_normal((N, 3)).astype(np.float32)
    src, dst, _ = oracle.mst_prim(X)
    tree = as_edge_set(src, dst)
    D = all_pairs_f64(X)
    for r in range(1, N):
        for rest in itertools.combinations(range(1, N), r - 1):
            S = {0, *rest}
            if len(S) == N:
                continue
            T = [v for v in range(N) if v not in S]
            best = min(((D[a, b], min(a, b), max(a, b)) for a in S for b in T))
            assert (best[1], best[2]) in tree


def test_mst_increasing_gaps_closed_form():
    N = 200
    X, pos = gen.increasing_gaps_line(N, 3, seed=5)
    src, dst, w = oracle.mst_prim(X)
    order = np.argsort(pos)
    expected = {(min(int(order[i]), int(order[i + 1])), max(int(order[i]), int(order[i + 1])))
                for i in range(N - 1)}
    assert as_edge_set(src, dst) == expected
    assert sorted(w.tolist()) == [float((i + 1) ** 2) for i in range(N - 1)]


def test_mst_unit_lattice_all_ties():
    X = gen.integer_lattice(6, 2, seed=9)
    src, dst, w = oracle.mst_prim(X)
    check_spanning_tree(src, dst, 36)
    assert (w == 1.0).all()


def test_mst_knn_graph_is_not_enough_example():
    # Seven points whose 2-NN graph is connected but does not contain the minimum spanning tree:
    # two vertical triples half a unit apart and one far point that lists one point of each.
    X = np.array([[0, 0], [0, -.1], [0, -.2], [.5, 0], [.5, -.1], [.5, -.2], [.2, 10]],
                 dtype=np.float32)
    out = oracle.slhc(X)
    assert out["total_weight"] == pytest.approx(0.04 + 0.25 + 100.04, rel=1e-6)
    assert (0, 3) in as_edge_set(out["src"], out["dst"])
    idx, _ = oracle.knn_graph(X, 2)
    listed = {(min(i, int(j)), max(i, int(j))) for i in range(7) for j in idx[i]}
    assert (0, 3) not in listed


def test_mst_two_far_blobs_last_edge():
    rng = np.random.default_rng(11)
    A = rng.standard_normal((150, 5))
    B = rng.standard_normal((130, 5)) + 40.0
    X = np.concatenate([A, B]).astype(np.float32)
    out = oracle.slhc(X)
    D = all_pairs_f64(X)
    assert out["heights"][-1] == pytest.approx(D[:150, 150:].min(), rel=1e-14)
    assert out["sizes"][-1] == 280


# ----------------------------------------------------------------------------- dendrogram
@pytest.mark.parametrize("name,n", [("c1", 800), ("c2", 500), ("c3", 700)])
def test_dendrogram_vs_scipy_linkage(name, n):
    X, _, _ = gen.make(name, n=n)
    out = oracle.slhc(X)
    Z = sch.linkage(X.astype(np.float64), method="single", metric="sqeuclidean")
    np.testing.assert_allclose(out["heights"], Z[:, 2], rtol=1e-12)
    assert np.array_equal(out["sizes"], Z[:, 3].astype(np.int32))
    zc = np.sort(Z[:, :2].astype(np.int32), axis=1)
    assert np.array_equal(out["children"], zc)


def test_dendrogram_invariants_with_ties():
    X, _, _ = gen.make("c5", n=2500)
    N = X.shape[0]
    out = oracle.slhc(X)
    ch, h, sz = out["children"], out["heights"], out["sizes"]
    assert (np.diff(h) >= 0).all()
    assert sz[-1] == N
    assert sorted(ch.ravel().tolist()) == list(range(2 * N - 2))     # every node is a child once
    assert (ch[:, 0] < ch[:, 1]).all()
    assert (ch < (N + np.arange(N - 1))[:, None]).all()
    Z = sch.linkage(X.astype(np.float64), method="single", metric="sqeuclidean")
    np.testing.assert_allclose(h, Z[:, 2], rtol=1e-12, atol=0)        # heights are unique as a multiset
    assert h[0] == 0.0                                                  # duplicates merge first


def test_dendrogram_rejects_cycle():
    with pytest.raises(ValueError):
        oracle.dendrogram([0, 1, 0], [1, 2, 2], [1.0, 2.0, 3.0], 4)


def test_oracle_reports_threads():
    assert oracle.num_threads() >= 1


# ----------------------------------------------------------------------------- flat clusters
def test_five_points_flat_clusters(golden_five_points):
    g = golden_five_points
    children = np.array(g["dendrogram"])[:, :2].astype(int)
    assert oracle.flat_clusters(children, 2).tolist() == [int(v) for v in g["flat2"][0]]
    assert oracle.flat_clusters(children, 3).tolist() == [int(v) for v in g["flat3"][0]]


def _same_partition(a, b):
    pairs = set(zip(a.tolist(), b.tolist()))
    return len(pairs) == len(set(a.tolist())) == len(set(b.tolist()))


@pytest.mark.parametrize("name,n", [("c1", 1500), ("c2", 900), ("c3", 700)])
def test_flat_clusters_vs_scipy_fcluster(name, n):
    X, _, _ = gen.make(name, n=n)
    out = oracle.slhc(X)
    Z = sch.linkage(X.astype(np.float64), method="single", metric="sqeuclidean")
    for nc in (1, 2, 3, 7, 50, n // 2, n):
        mine = oracle.flat_clusters(out["children"], nc)
        ref = sch.fcluster(Z, nc, criterion="maxclust")
        assert len(set(mine.tolist())) == nc
        assert _same_partition(mine, ref), nc


def test_flat_clusters_are_components_of_the_trimmed_tree():
    # second definition: drop the n_clusters - 1 heaviest tree edges; the connected components of
    # what is left are the clusters (tie-free data)
    X, _, _ = gen.make("c1", n=800)
    out = oracle.slhc(X)
    N = X.shape[0]
    for nc in (2, 5, 31):
        keep = N - nc
        graph = sp.coo_matrix((np.ones(keep), (out["src"][:keep], out["dst"][:keep])), shape=(N, N))
        ncomp, comp = csg.connected_components(graph, directed=False)
        assert ncomp == nc
        assert _same_partition(oracle.flat_clusters(out["children"], nc), comp)


def test_flat_clusters_numbering_and_extremes():
    X, _, _ = gen.make("c2", n=300)
    out = oracle.slhc(X)
    N = X.shape[0]
    ch = out["children"]
    assert oracle.flat_clusters(ch, 1).tolist() == [0] * N
    assert oracle.flat_clusters(ch, N).tolist() == list(range(N))          # every row its own root
    # labels are the ranks of the root ids: rebuild the roots independently from the sizes array
    nc = 9
    lab = oracle.flat_clusters(ch, nc)
    kept = N - nc
    used = set(ch[:kept].ravel().tolist())
    roots = sorted(set(range(N + kept)) - used)
    assert len(roots) == nc
    members = {r: set() for r in roots}
    def leaves(node):
        stack, acc = [node], []
        while stack:
            x = stack.pop()
            if x < N:
                acc.append(x)
            else:
                stack.extend(ch[x - N].tolist())
        return acc
    for rank, r in enumerate(roots):
        assert {int(lab[v]) for v in leaves(r)} == {rank}
    with pytest.raises(ValueError):
        oracle.flat_clusters(ch, 0)
    with pytest.raises(ValueError):
        oracle.flat_clusters(ch, N + 1)


# ----------------------------------------------------------------------------- CSR spanning forest
def _dense_to_csr(D):
    V = D.shape[0]
    src, dst = np.nonzero(~np.eye(V, dtype=bool))
    offsets = np.arange(V + 1, dtype=np.int32) * (V - 1)
    return offsets, dst.astype(np.int32), D[src, dst].astype(np.float32)


def test_csr_msf_equals_dense_prim_on_points():
    # the complete squared-L2 graph of tie-free points: Kruskal on its CSR must give Prim's tree
    X, _, _ = gen.make("c1", n=300)
    D = cdist(X.astype(np.float64), X.astype(np.float64), "sqeuclidean")
    lo, hi, w, comp = oracle.csr_msf(*_dense_to_csr(D))
    out = oracle.slhc(X)
    assert lo.tolist() == out["src"].tolist() and hi.tolist() == out["dst"].tolist()
    assert np.allclose(w, out["w"], rtol=1e-6)
    assert (comp == 0).all()


@pytest.mark.parametrize("V", [4, 5, 6])
def test_csr_msf_brute_force_all_spanning_trees(V):
    rng = np.random.default_rng(V)
    D = rng.permutation(V * V).reshape(V, V).astype(np.float64) + 1.0      # distinct weights
    D = np.minimum(D, D.T)
    lo, hi, w, _ = oracle.csr_msf(*_dense_to_csr(D))
    pairs = list(itertools.combinations(range(V), 2))
    best = None
    for tree in itertools.combinations(pairs, V - 1):
        up = list(range(V))
        def find(a):
            while up[a] != a:
                a = up[a]
            return a
        ok = True
        for a, b in tree:
            ra, rb = find(a), find(b)
            if ra == rb:
                ok = False
                break
            up[ra] = rb
        if ok:
            tot = sum(D[a, b] for a, b in tree)
            if best is None or tot < best[0]:
                best = (tot, sorted(tree))
    assert sorted(zip(lo.tolist(), hi.tolist())) == best[1]
    assert float(w.sum()) == best[0]


def test_csr_msf_forest_cycle_and_ties():
    # two disjoint cycles: the forest drops exactly the heaviest edge of each; ties go by (lo, hi)
    offsets = np.array([0, 2, 4, 6, 8, 10, 12, 14], dtype=np.int32)
    und = [(0, 1, 1.0), (1, 2, 2.0), (0, 2, 3.0), (3, 4, 5.0), (4, 5, 5.0), (5, 6, 5.0), (3, 6, 5.0)]
    rows = {v: [] for v in range(7)}
    for a, b, w in und:
        rows[a].append((b, w))
        rows[b].append((a, w))
    indices = np.array([u for v in range(7) for u, _ in sorted(rows[v])], dtype=np.int32)
    weights = np.array([w for v in range(7) for _, w in sorted(rows[v])], dtype=np.float32)
    lo, hi, w, comp = oracle.csr_msf(offsets, indices, weights)
    assert list(zip(lo.tolist(), hi.tolist(), w.tolist())) == [(0, 1, 1.0), (1, 2, 2.0), (3, 4, 5.0), (3, 6, 5.0),
                                                                 (4, 5, 5.0)]
    assert comp.tolist() == [0, 0, 0, 3, 3, 3, 3]


@pytest.mark.parametrize("integer_weights", [False, True])
def test_csr_msf_road_graph_vs_scipy(integer_weights):
    offsets, indices, weights = gen.road_graph(60, seed=3, integer_weights=integer_weights)
    V = offsets.shape[0] - 1
    lo, hi, w, comp = oracle.csr_msf(offsets, indices, weights)
    G = sp.csr_matrix((weights.astype(np.float64), indices, offsets), shape=(V, V))
    ncomp, ref_comp = csg.connected_components(G, directed=False)
    assert lo.shape[0] == V - ncomp
    assert _same_partition(comp, ref_comp)
    T = csg.minimum_spanning_tree(G)                  # weights are >= 1: no zero-means-absent trap
    assert abs(float(T.sum()) - float(w.astype(np.float64).sum())) < 1e-6 * float(T.sum())
    assert (np.diff(w) >= 0).all() and (lo < hi).all()
    deg = np.diff(offsets)
    assert 2.2 < deg.mean() < 2.8

