"""Pins for the oracle's level interpreter (Table 2): the paper's printed
fragments, closed forms and brute force. CPU only."""
import os

import numpy as np

import oracle
import workloads as wl
from workloads import LevelSpec, TensorSpec

GOLD = os.path.join(os.path.dirname(__file__), "golden", "paper_level_fragments.txt")


def _golden():
    g = {}
    for line in open(GOLD):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        k, v = line.split("=")
        g[k.strip()] = [int(t) for t in v.split()]
    return g


# An own 4x6 matrix that satisfies every fragment the paper's text states about
# its running example (it is NOT claimed to be the figure's matrix).
ROWS = np.array([0, 0, 1, 1, 2, 3, 3, 3])
COLS = np.array([0, 1, 0, 1, 2, 1, 3, 4])
VALS = np.array([5., 1., 7., 3., 8., 4., 2., 9.])


def test_compressed_level_matches_paper_fragment():
    g = _golden()
    csr = wl.csr_from_sorted_coo(4, 6, ROWS, COLS, VALS)
    lv = csr.levels[1]
    assert lv.pos[1] == g["compressed.pos1"][0] and lv.pos[2] == g["compressed.pos2"][0]
    ci, cp = oracle.level_children(lv, p_parent=1)
    assert list(ci) == g["compressed.parent1.children"]
    assert list(cp) == [2, 3]
    coords, vals = oracle.to_coo(csr)
    assert coords[0, -1] == g["last.row"][0] and coords[1, -1] == g["last.col"][0]
    assert vals[-1] == g["last.val"][0]
    # last three stored components share row 3 (Section 2, CSR paragraph)
    assert list(coords[0, -3:]) == [3, 3, 3]


def test_range_and_offset_levels_match_paper_fragment():
    g = _golden()
    N, M = g["range.N"][0], g["range.M"][0]
    # offset[1] is fixed by the fragment: max(0,-o)=1 and min(4,6-o)=4 -> o=-1
    offsets = np.array([-2, -1, 0, 1], np.int32)
    rng_lv = LevelSpec(wl.RANGE, 0, N, M=M, offset=offsets)
    ci, cp = oracle.level_children(rng_lv, p_parent=1, i_parent=g["range.parent"][0])
    assert ci[0] == g["range.lo"][0] and ci[-1] + 1 == g["range.hi"][0]
    assert list(cp) == [1 * N + i for i in ci]          # p = p_parent*N + i
    off_lv = LevelSpec(wl.OFFSET, 1, M, offset=offsets)
    ci, cp = oracle.level_children(off_lv, p_parent=7, i_parent=g["offset.parent"][0],
                                   i_grand=g["offset.index"][0])
    assert list(ci) == g["offset.coord"] and list(cp) == [7]


def test_range_bounds_closed_form_all_offsets():
    N, M = 5, 8
    for o in range(-6, 10):
        lv = LevelSpec(wl.RANGE, 0, N, M=M, offset=np.array([o], np.int32))
        ci, _ = oracle.level_children(lv, 0, 0)
        want = [i for i in range(N) if 0 <= i + o < M]   # the diagonal's in-matrix rows
        assert list(ci) == want


def test_dense_and_singleton_levels():
    ci, cp = oracle.level_children(LevelSpec(wl.DENSE, 0, 5), p_parent=3)
    assert list(ci) == [0, 1, 2, 3, 4] and list(cp) == [15, 16, 17, 18, 19]
    s = LevelSpec(wl.SINGLETON, 1, 9, crd=np.array([4, -1, 8], np.int32))
    assert [list(a) for a in oracle.level_children(s, 0)] == [[4], [0]]
    assert [list(a) for a in oracle.level_children(s, 1)] == [[], []]   # padding
    assert [list(a) for a in oracle.level_children(s, 2)] == [[8], [2]]


def _hash_insert(table, W, parent, key):
    """Insert with the probing rule of Table 2 (start at key % W, step +1 with
    wrap inside the parent's segment); written independently for the test."""
    for s in range(W):
        p = parent * W + (key % W + s) % W
        if table[p] in (-1, key):
            table[p] = key
            return p
    raise RuntimeError("full")


def test_hashed_level_iteration_and_locate_brute_force():
    rng = np.random.default_rng(7)
    W, parents = 11, 3
    table = np.full(W * parents, -1, np.int32)
    where = {}
    for parent in range(parents):
        for key in rng.choice(200, size=7 + parent, replace=False):   # last segment nearly full
            where[(parent, int(key))] = _hash_insert(table, W, parent, int(key))
    lv = LevelSpec(wl.HASHED, 0, 200, M=W, crd=table, ordered=False)
    for parent in range(parents):
        ci, cp = oracle.level_children(lv, parent)
        want = sorted(k for (q, k) in where if q == parent)
        assert sorted(ci) == want
        assert all(table[p] == i for i, p in zip(ci, cp))
        for key in range(200):
            p, found = oracle.hashed_locate(lv, parent, key)
            assert found == ((parent, key) in where)
            if found:
                assert p == where[(parent, key)]
    # completely full segment: absent key must terminate and report not found
    full = np.arange(W, dtype=np.int32) * 3
    t2 = np.full(W, -1, np.int32)
    for k in full:
        _hash_insert(t2, W, 0, int(k))
    lv2 = LevelSpec(wl.HASHED, 0, 200, M=W, crd=t2, ordered=False)
    assert oracle.hashed_locate(lv2, 0, 1)[1] is False


def test_hashed_vector_walk():
    W = 7
    table = np.full(W, -1, np.int32)
    vals = np.zeros(W)
    for key, v in [(3, 1.5), (10, -2.0), (6, 4.0)]:
        vals[_hash_insert(table, W, 0, key)] = v
    spec = TensorSpec((20,), [LevelSpec(wl.HASHED, 0, 20, M=W, crd=table, ordered=False)], vals)
    coords, v = oracle.to_coo(spec)
    assert sorted(zip(coords[0], v)) == [(3, 1.5), (6, 4.0), (10, -2.0)]


def _entries(spec):
    c, v = oracle.to_coo(spec)
    o = np.lexsort(tuple(c[::-1]))
    return c[:, o], v[o]


def test_formats_of_one_matrix_encode_the_same_entries():
    """COO / CSR / DIA / ELL walks vs the entry list they were laid out from."""
    # DIA and CSR of config 2 (scaled) -- poison cells must never be visited
    c2 = wl.config2(N=50, seed=3, poison=True)
    cd, vd = _entries(c2["dia"])
    cc, vc = _entries(c2["csr"])
    assert np.array_equal(cd, cc) and np.array_equal(vd, vc)
    assert not np.isnan(vd).any()
    assert len(vd) == sum(50 - abs(o) for o in wl.config2_offsets(50))
    # closed form of the DIA walk: cell (d,i) <-> (i, i+off[d])
    off = wl.config2_offsets(50)
    dv = c2["dia"].vals.reshape(len(off), 50)
    for d, o in enumerate(off):
        for i in range(max(0, -o), min(50, 50 - o)):
            k = np.flatnonzero((cd[0] == i) & (cd[1] == i + o))
            assert len(k) == 1 and vd[k[0]] == dv[d, i]
    # ELL and CSR of config 3 (scaled)
    c3 = wl.config3(N=40, lo=0, hi=6, seed=5)
    ce, ve = _entries(c3["ell"])
    cc, vc = _entries(c3["csr"])
    assert np.array_equal(ce, cc) and np.array_equal(ve, vc)
    assert len(ve) == c3["nnz"]
    # COO and CSR of config 1 (scaled)
    c1 = wl.config1(N=30, nnz=100, seed=9)
    co, vo = _entries(c1["coo"])
    cc, vc = _entries(c1["csr"])
    r, c, v = c1["entries"]
    assert np.array_equal(co, cc) and np.array_equal(vo, vc)
    assert np.array_equal(co, np.stack([r, c]).astype(np.int64)) and np.array_equal(vo, v)


def test_csf_walk_matches_sorted_coo():
    ci, cj, ck, v = wl.random_coo3_entries((6, 5, 4), 60, seed=2, dtype=np.float64, skew=1.5)
    coo = wl.coo3_spec((6, 5, 4), ci, cj, ck, v)
    csf = wl.csf3_from_sorted_coo((6, 5, 4), ci, cj, ck, v)
    c1, v1 = oracle.to_coo(coo)
    c2, v2 = oracle.to_coo(csf)
    assert np.array_equal(c1, c2) and np.array_equal(v1, v2)
    assert np.array_equal(c1, np.stack([ci, cj, ck]).astype(np.int64))
    # CSF invariants: pos monotone, ends at the child count, crd strictly ascending per segment
    for k, lv in enumerate(csf.levels):
        assert lv.pos[0] == 0 and np.all(np.diff(lv.pos) >= 0)
        assert lv.pos[-1] == len(lv.crd)
        for a, b in zip(lv.pos[:-1], lv.pos[1:]):
            assert np.all(np.diff(lv.crd[a:b]) > 0)
    assert len(csf.levels[1].crd) == len(np.unique(ci.astype(np.int64) * 5 + cj))


def test_empty_tensors_walk_to_nothing():
    z = np.zeros(0, np.int32)
    coo = wl.coo_spec(4, 5, z, z, np.zeros(0))
    csr = wl.csr_from_sorted_coo(4, 5, z, z, np.zeros(0))
    assert oracle.to_coo(coo)[1].size == 0 and oracle.to_coo(csr)[1].size == 0


# ---------------------------------------------------------------- other compositions
# DCSR, CSC, a dense matrix, hashed rows and a (dense, compressed, compressed) tensor have no
# kernel of their own: the oracle's level walk is their reference, pinned here against scipy /
# the entry list they were built from.

def test_other_matrix_compositions_walk_to_the_same_entries_and_products():
    import scipy.sparse as sp
    N, M = 23, 31
    r, c, v = wl.random_coo_entries(N, M, 120, seed=91, dtype=np.float64)
    r[r == 5] = 6                                   # leave rows empty so DCSR really compresses rows
    order = np.lexsort((c, r))
    key, first = np.unique(r[order].astype(np.int64) * M + c[order], return_index=True)
    r, c, v = r[order][first], c[order][first], v[order][first]
    S = sp.coo_matrix((v, (r, c)), shape=(N, M))
    x = wl.dense_vector(M, 92, np.float64)
    want = S @ x
    specs = {
        "dcsr": wl.dcsr_from_sorted_coo(N, M, r, c, v),
        "csc": wl.csc_from_coo(N, M, r, c, v),
        "dense": wl.dense_matrix_spec(S.toarray()),
        "dhash": wl.hashed_rows_from_coo(N, M, r, c, v, W=16),
        "sdia": wl.sparse_dia_from_coo(N, M, r, c, v),     # (dense, compressed, offset), Section 3.1
    }
    assert len(specs["dcsr"].levels[0].crd) < N
    for name, spec in specs.items():
        co, w = oracle.to_coo(spec)
        if name == "dense":                          # every cell is a leaf; the zeros are stored too
            assert co.shape[1] == N * M
            keep = w != 0
            co, w = co[:, keep], w[keep]
        o = np.lexsort((co[1], co[0]))
        assert np.array_equal(co[0][o], r) and np.array_equal(co[1][o], c), name
        assert np.array_equal(w[o], v), name
        y, _ = oracle.spmv(spec, x)
        np.testing.assert_allclose(y, want, rtol=0, atol=1e-13, err_msg=name)
    # CSC is stored column-major: its storage order is by (col, row)
    co, _ = oracle.to_coo(specs["csc"])
    assert np.all(np.diff(co[1] * N + co[0]) > 0)


def test_dense_compressed_compressed_tensor_walk():
    dims = (6, 5, 7)
    ci, cj, ck, v = wl.random_coo3_entries(dims, 90, seed=93, dtype=np.float64, skew=1.5)
    spec = wl.dcc3_from_sorted_coo(dims, ci, cj, ck, v)
    co, w = oracle.to_coo(spec)
    assert np.array_equal(co[0], ci) and np.array_equal(co[1], cj) and np.array_equal(co[2], ck)
    assert np.array_equal(w, v)


def test_aos_coo_walks_like_soa_coo():
    """Array-of-structs COO (Section 5.2): one interleaved coordinate array, each level reading it
    with a stride. The walk, SpMV and the 3rd-order kernels see the same tensor as through SoA."""
    import scipy.sparse as sp
    N, M = 23, 31
    r, c, v = wl.random_coo_entries(N, M, 200, seed=301, dtype=np.float64)
    aos = wl.coo_aos_spec((N, M), (r, c), v)
    inter = aos.levels[0].crd
    assert np.array_equal(inter[0::2], r) and np.array_equal(inter[1::2], c)      # (i, j) (i, j) ...
    assert np.shares_memory(aos.levels[0].crd, aos.levels[1].crd)                 # one array, two views
    assert aos.levels[1].crd[0] == c[0] and aos.levels[0].crd_stride == 2
    coords, vals = oracle.to_coo(aos)
    assert np.array_equal(coords[0], r) and np.array_equal(coords[1], c) and np.array_equal(vals, v)
    x = wl.dense_vector(M, 302)
    y, mag = oracle.spmv(aos, x)
    np.testing.assert_allclose(y, sp.coo_matrix((v, (r, c)), shape=(N, M)).tocsr() @ x, rtol=0,
                               atol=1e-13 * max(mag.max(), 1))
    dims = (7, 6, 5)
    ci, cj, ck, w = wl.random_coo3_entries(dims, 90, 303, dtype=np.float64)
    aos3 = wl.coo_aos_spec(dims, (ci, cj, ck), w)
    assert np.array_equal(aos3.levels[2].crd[0::3], ck)
    cvec = wl.dense_vector(dims[2], 304)
    a = oracle.ttv(aos3, cvec)
    b = oracle.ttv(wl.coo3_spec(dims, ci, cj, ck, w), cvec)
    assert all(np.array_equal(p, q) for p, q in zip(a, b))
