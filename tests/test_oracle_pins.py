"""Pins for the CPU oracle: every check compares it with something other than itself --
brute force (Eq. 1), closed forms, hand-computed fixtures, library routines, invariants."""
import os

import numpy as np
import pytest
from scipy.spatial.distance import cdist

from oracle import pqt_build as B
from oracle import pqt_index_io as IO
from oracle import pqt_query as Q

GOLD = os.path.join(os.path.dirname(__file__), "golden")


# ---- P1: exhaustive visit + exact re-ranking reproduces brute force (Eq. 1) ----------------
def test_exhaustive_exact_rerank_equals_brute_force(tiny):
    cfg, X, Y, ix = tiny
    for q in range(8):
        tr = Q.query(ix, Y[q], k=10, w=cfg.k1, T=ix.K, C=cfg.N, X=X, exact_rerank=True)
        # textbook routine, not the oracle's own brute force
        d = cdist(Y[q:q + 1].astype(np.float64), X.astype(np.float64), "sqeuclidean")[0]
        want = np.lexsort((np.arange(cfg.N), d))[:10]
        assert np.array_equal(tr.out_ids, want)
        np.testing.assert_allclose(tr.out_dists, d[want], rtol=1e-12)
        ids, dd = Q.brute_force(Y[q], X, 10)
        assert np.array_equal(ids, want)
        np.testing.assert_allclose(dd, d[want], rtol=1e-12)


# ---- P2: bins are a partition of the database; every id sits in slot m(x) -------------------
def test_bins_partition_the_database(tiny):
    cfg, X, Y, ix = tiny
    tr = Q.query(ix, Y[3], k=10, w=cfg.k1, T=ix.K, C=cfg.N)
    assert np.array_equal(np.sort(tr.cand_ids), np.arange(cfg.N))
    off = ix.offsets.astype(np.int64)
    assert off[0] == 0 and off[-1] == cfg.N and np.all(np.diff(off) >= 0)
    slot_of_pos = np.repeat(np.arange(ix.H), np.diff(off))
    hist = np.bincount(slot_of_pos, minlength=ix.H)
    assert np.array_equal(np.cumsum(hist), off[1:])          # pointer array = prefix sum (Sec. 4)
    for t in range(0, cfg.N, 97):
        assert slot_of_pos[t] == B.bin_slot(X[ix.ids[t]], ix.C1, ix.C2, ix.H)
    for s in np.nonzero(hist > 1)[0][:50]:
        run = ix.ids[off[s]:off[s + 1]]
        assert np.all(np.diff(run.astype(np.int64)) > 0)     # ids ascending inside a slot


def test_leaf_is_nearest_child_of_nearest_cell(tiny):
    """m(x) by a library routine: per part, argmin over level-1 then over that cell's children."""
    cfg, X, Y, ix = tiny
    dp = cfg.D // cfg.P
    for n in range(0, 200, 7):
        leaf = B.leaf_of(X[n], ix.C1, ix.C2)
        for p in range(cfg.P):
            xp = X[n:n + 1, p * dp:(p + 1) * dp].astype(np.float64)
            i = int(np.argmin(cdist(xp, ix.C1[p].astype(np.float64), "sqeuclidean")[0]))
            j = int(np.argmin(cdist(xp, ix.C2[p, i].astype(np.float64), "sqeuclidean")[0]))
            assert leaf[p] == i * cfg.k2 + j


# ---- P3: Eq. 9 is the exact distance to the reconstructed (line-quantised) vector -----------
def test_adc_score_equals_distance_to_reconstruction(tiny):
    cfg, X, Y, ix = tiny
    cc64 = B.pair_table(ix.C1, ix.M)
    for q in range(5):
        a = Q.level1_subpart_distances(Y[q], ix.C1, ix.M)
        lut = Q.build_lut(a, ix.tbl_i, ix.tbl_j, ix.tbl_lam, cc64)
        pos = np.arange(q, cfg.N, 211)
        s = Q.score_codes(lut, ix.codes[pos])
        for t, ps in enumerate(pos):
            xr = Q.reconstruct(ix, ix.codes[ps])
            want = float(np.sum((Y[q].astype(np.float64) - xr) ** 2))
            assert abs(s[t] - want) <= 1e-9 * max(want, 1e-30)


def test_codes_are_nearest_code_points(tiny):
    cfg, X, Y, ix = tiny
    ds = cfg.D // cfg.M
    for t in range(0, cfg.N, 503):
        x = X[ix.ids[t]].astype(np.float64)
        assert np.array_equal(ix.codes[t], B.encode_vector(X[ix.ids[t]], ix.C1, ix.M, ix.tbl_i, ix.tbl_j, ix.tbl_lam))
        for m in range(cfg.M):
            # brute force over explicit reconstructions of all 256 code points
            best, bestc = np.inf, -1
            for c in range(256):
                code = ix.codes[t].copy()
                code[m] = c
                xr = Q.reconstruct(ix, code)[m * ds:(m + 1) * ds]
                e = float(np.sum((x[m * ds:(m + 1) * ds] - xr) ** 2))
                if e < best:
                    best, bestc = e, c
            assert bestc == ix.codes[t, m]


# ---- P4: Eq. 9 special cases and hand-computed triangle -------------------------------------
def test_eq9_hand_computed_triangle():
    rows = np.loadtxt(os.path.join(GOLD, "eq9_triangle.txt"))
    for lam, b2, a2, c2, h2 in rows:
        a = np.array([[b2, a2]])
        cc = np.array([[[0.0, c2], [c2, 0.0]]])
        lut = Q.build_lut(a, np.array([[0]], np.uint8), np.array([[1]], np.uint8),
                          np.array([[lam]], np.float32), cc)
        assert lut[0, 0] == pytest.approx(h2, rel=1e-12)


def test_eq9_closed_forms(rng):
    for _ in range(20):
        ci, cj, y = rng.normal(size=(3, 6))
        b2, a2, c2 = np.sum((y - ci) ** 2), np.sum((y - cj) ** 2), np.sum((ci - cj) ** 2)
        a = np.array([[b2, a2]])
        cc = np.array([[[0.0, c2], [c2, 0.0]]])
        ti, tj = np.zeros((1, 3), np.uint8), np.ones((1, 3), np.uint8)
        lut = Q.build_lut(a, ti, tj, np.array([[0.0, 1.0, 0.5]], np.float32), cc)
        assert lut[0, 0] == pytest.approx(b2, rel=1e-12)                      # lambda = 0: the c_i end
        assert lut[0, 1] == pytest.approx(a2, rel=1e-12)                      # lambda = 1: the c_j end
        assert lut[0, 2] == pytest.approx((a2 + b2) / 2 - c2 / 4, rel=1e-12)  # median of a triangle
        # swapping the roles of i and j must NOT give the same value for lambda != 1/2
        lam = np.float32(0.3)
        l_ij = Q.build_lut(a, ti[:, :1], tj[:, :1], np.array([[lam]], np.float32), cc)[0, 0]
        want = np.sum((y - ((1 - float(lam)) * ci + float(lam) * cj)) ** 2)
        assert l_ij == pytest.approx(want, rel=1e-10)


def test_line_projection_is_orthogonal(rng):
    for _ in range(10):
        ci, cj, x = rng.normal(size=(3, 5))
        lam, err = B.line_projection(x, ci, cj)
        proj = (1 - lam) * ci + lam * cj
        assert abs(np.dot(x - proj, cj - ci)) < 1e-12
        assert err == pytest.approx(np.sum((x - proj) ** 2))
        # Pythagoras on the right triangle (x, proj, ci)
        assert err == pytest.approx(np.sum((x - ci) ** 2) - lam ** 2 * np.sum((cj - ci) ** 2), abs=1e-10)


# ---- P5: bin order ---------------------------------------------------------------------------
def _sorted_lists(rng, P, R, integer):
    if integer:
        return [np.sort(rng.integers(0, 12, size=R)).astype(np.float32) for _ in range(P)]
    return [np.sort(rng.random(R)).astype(np.float32) for _ in range(P)]


@pytest.mark.parametrize("integer", [False, True])
def test_bin_order_fullsort_equals_priority_queue(rng, integer):
    for R in (1, 5, 16):
        L = _sorted_lists(rng, 2, R, integer)
        for T in (1, 7, R * R, R * R + 5):
            t1, k1_ = Q.bin_order(L, T, "fullsort")
            t2, k2_ = Q.bin_order(L, T, "pq")
            assert np.array_equal(t1, t2) and np.array_equal(k1_, k2_)
            assert t1.shape[0] == min(T, R * R)
            assert tuple(t1[0]) == (0, 0)
            assert np.all(np.diff(k1_) >= 0)
            # brute-force definition: python sort of (fl32 sum, r1, r2)
            ref = sorted((np.float32(L[0][a] + L[1][b]), a, b) for a in range(R) for b in range(R))[:T]
            assert [tuple(x) for x in t1] == [(a, b) for _, a, b in ref]


@pytest.mark.parametrize("integer", [False, True])
def test_bin_order_four_parts_truncation_is_exact(rng, integer):
    L = _sorted_lists(rng, 4, 6, integer)
    for T in (1, 10, 100, 6 ** 4):
        full, kf = Q.bin_order(L, T, "fullsort", truncate_pairs=False)
        trunc, kt = Q.bin_order(L, T, "fullsort", truncate_pairs=True)
        pq, kp = Q.bin_order(L, T, "pq", truncate_pairs=True)
        assert np.array_equal(full, trunc) and np.array_equal(full, pq)
        assert np.array_equal(kf, kt) and np.array_equal(kf, kp)
        assert tuple(full[0]) == (0, 0, 0, 0) and np.all(np.diff(kf) >= 0)


def test_bin_order_on_tiny_lists(tiny):
    cfg, X, Y, ix = tiny
    for q in range(10):
        tr = Q.query(ix, Y[q], cfg.k, cfg.w, order_method="pq")
        tr2 = Q.query(ix, Y[q], cfg.k, cfg.w, order_method="fullsort")
        assert np.array_equal(tr.tuples, tr2.tuples) and np.array_equal(tr.out_ids, tr2.out_ids)
        # the first proposed bin is the combination of the per-part best leaves (Sec. 3.2)
        assert [tr.Lid[p][0] for p in range(cfg.P)] == [tr.Lid[p][tr.tuples[0, p]] for p in range(cfg.P)]


# ---- P6: counts printed in the paper ----------------------------------------------------------
def test_distance_evaluation_counts_and_bin_count():
    rows = np.loadtxt(os.path.join(GOLD, "paper_counts.txt"), dtype=np.int64)
    for k1, k2, w, P, evals, bins in rows:
        if k1 > 64:      # closed form only (building an 8192-centroid tree is not needed)
            assert k1 + w * k2 == evals and (k1 * k2) ** P == bins
            continue
        rng = np.random.default_rng(1)
        dp = 3
        C1 = rng.normal(size=(P, k1, dp)).astype(np.float32)
        C2 = rng.normal(size=(P, k1, k2, dp)).astype(np.float32)
        y = rng.normal(size=P * dp)
        a = Q.level1_subpart_distances(y, C1, P)
        sel = Q.select_clusters(Q.part_distances(a, P), w)
        d2, ids2 = Q.level2_distances(y, C2, sel)
        assert a.shape[1] + d2.shape[1] == evals          # per part: k1 + w*k2
        ix = Q.PQTIndex(D=P * dp, P=P, k1=k1, k2=k2, M=P, N=0, H=1, T=1, C=1, C1=C1, C2=C2,
                        tbl_i=None, tbl_j=None, tbl_lam=None, cc=None, offsets=None, ids=None, codes=None)
        assert ix.K == bins
        assert len(set(ids2[0].tolist())) == w * k2 and ids2.max() < k1 * k2


# ---- P7: elementary steps against library routines ---------------------------------------------
def test_level1_distances_match_cdist(tiny):
    cfg, X, Y, ix = tiny
    ds, dp = cfg.D // cfg.M, cfg.D // cfg.P
    a = Q.level1_subpart_distances(Y[0], ix.C1, cfg.M)
    for m in range(cfg.M):
        p = (m * ds) // dp
        lo = m * ds - p * dp
        want = cdist(Y[0:1, m * ds:(m + 1) * ds].astype(np.float64),
                     ix.C1[p, :, lo:lo + ds].astype(np.float64), "sqeuclidean")[0]
        np.testing.assert_allclose(a[m], want, rtol=1e-12)
    d1 = Q.part_distances(a, cfg.P)
    for p in range(cfg.P):
        want = cdist(Y[0:1, p * dp:(p + 1) * dp].astype(np.float64), ix.C1[p].astype(np.float64), "sqeuclidean")[0]
        np.testing.assert_allclose(d1[p], want, rtol=1e-12)


def test_level2_distances_match_cdist(tiny):
    cfg, X, Y, ix = tiny
    dp = cfg.D // cfg.P
    sel = np.array([[3, 0, 5], [7, 2, 1]])
    d2, ids2 = Q.level2_distances(Y[1], ix.C2, sel)
    for p in range(cfg.P):
        for s, i in enumerate(sel[p]):
            want = cdist(Y[1:2, p * dp:(p + 1) * dp].astype(np.float64), ix.C2[p, i].astype(np.float64), "sqeuclidean")[0]
            np.testing.assert_allclose(d2[p, s * cfg.k2:(s + 1) * cfg.k2], want, rtol=1e-12)
            assert ids2[p, s * cfg.k2:(s + 1) * cfg.k2].tolist() == [i * cfg.k2 + j for j in range(cfg.k2)]


def test_sorts_match_python_sorted(rng):
    v = rng.integers(0, 5, size=40).astype(np.float64)      # many ties
    ids = rng.permutation(40)
    o = Q.order_by_value_then_id(v, ids)
    assert [(v[t], ids[t]) for t in o] == sorted(zip(v.tolist(), ids.tolist()))
    sel = Q.select_clusters(v[None, :16], 5)[0]
    assert sel.tolist() == [i for _, i in sorted(zip(v[:16].tolist(), range(16)))[:5]]
    Ld, Lid = Q.sort_level2(v[None], ids[None])
    assert list(zip(Ld[0].tolist(), Lid[0].tolist())) == sorted(zip(v.tolist(), ids.tolist()))
    oi, od = Q.top_k(v, ids, 45)
    ref = sorted(zip(v.tolist(), ids.tolist()))
    assert oi[:40].tolist() == [i for _, i in ref] and np.all(oi[40:] == -1) and np.all(np.isinf(od[40:]))


def test_score_is_sum_of_table_entries(rng):
    lut = rng.random((4, 256))
    codes = rng.integers(0, 256, size=(50, 4)).astype(np.uint8)
    s = Q.score_codes(lut, codes)
    for n in range(50):
        assert s[n] == pytest.approx(sum(lut[m, codes[n, m]] for m in range(4)), rel=1e-14)


# ---- P8: P=1, k2=1 degenerates to a plain inverted file over k1 Voronoi cells -----------------
def test_single_part_single_child_is_inverted_file(rng):
    X = rng.normal(size=(600, 8)).astype(np.float32)
    ix = B.build_index(X, P=1, k1=8, k2=1, M=1, T=8, C=600, iters=5)
    y = rng.normal(size=8)
    d = cdist(y[None], ix.C1[0].astype(np.float64), "sqeuclidean")[0]
    cells = np.argsort(d, kind="stable")
    lab = np.argmin(cdist(X.astype(np.float64), ix.C1[0].astype(np.float64), "sqeuclidean"), axis=1)
    for w in (1, 3, 8):
        tr = Q.query(ix, y, k=5, w=w)
        want = np.concatenate([np.nonzero(lab == c)[0] for c in cells[:w]])
        assert np.array_equal(tr.cand_ids, want)


# ---- P10: recall bookkeeping --------------------------------------------------------------------
def test_exact_rerank_finds_nn_iff_its_bin_was_visited(tiny):
    cfg, X, Y, ix = tiny
    for q in range(20):
        gt = int(np.argmin(cdist(Y[q:q + 1].astype(np.float64), X.astype(np.float64), "sqeuclidean")[0]))
        tr = Q.query(ix, Y[q], cfg.k, cfg.w, X=X, exact_rerank=True)
        assert (gt in tr.cand_ids) == (tr.out_ids[0] == gt)
        assert len(tr.cand_ids) <= cfg.C and len(set(tr.cand_ids.tolist())) == len(tr.cand_ids)


# ---- hashing: colliding bins share one list, a slot is proposed once ---------------------------
def test_modulo_hash_dedupes_slots(tiny):
    cfg, X, Y, _ = tiny
    ixh = B.build_index(X[:2000], cfg.P, cfg.k1, cfg.k2, cfg.M, H=97, T=1024, C=2000, iters=5)
    tr = Q.query(ixh, Y[0], k=10, w=cfg.k1, T=ixh.K, C=2000)
    assert len(set(tr.slots.tolist())) == len(tr.slots)
    assert np.array_equal(np.sort(tr.cand_ids), np.arange(2000))   # still a partition
    for t in range(0, 2000, 131):
        slot = int(np.searchsorted(ixh.offsets, t, side="right")) - 1
        assert slot == B.bin_slot(X[ixh.ids[t]], ixh.C1, ixh.C2, 97)


# ---- index file round trip -----------------------------------------------------------------------
def test_index_file_roundtrip(tiny, tmp_path):
    cfg, X, Y, ix = tiny
    path = str(tmp_path / "tiny.pqt")
    IO.write_index(path, ix)
    ix2 = IO.read_index(path)
    for name in ("C1", "C2", "tbl_i", "tbl_j", "tbl_lam", "cc", "offsets", "ids", "codes"):
        assert np.array_equal(getattr(ix, name), getattr(ix2, name))
    assert (ix2.D, ix2.P, ix2.k1, ix2.k2, ix2.M, ix2.N, ix2.H, ix2.T, ix2.C) == \
        (ix.D, ix.P, ix.k1, ix.k2, ix.M, ix.N, ix.H, ix.T, ix.C)
    with open(path, "r+b") as f:
        f.truncate(os.path.getsize(path) - 10)
    with pytest.raises(ValueError):
        IO.read_index(path)


# ---- input generators: the torch port of the SIFT-shaped stream is bit-identical ----------------
def test_sift_like_numpy_and_torch_agree():
    from workloads import sift_like, sift_like_torch
    a = sift_like(987654, 3000, seed=1)
    b = sift_like_torch(987654, 3000, seed=1).numpy()
    assert np.array_equal(a, b)
    assert a.min() >= 0 and a.max() <= 255 and np.array_equal(a, np.round(a))
    assert np.array_equal(sift_like(987654 + 100, 50, seed=1), a[100:150])     # counter based: any chunk


def test_exact_short_list_rerank_is_brute_force_on_the_list(tiny, rng):
    """Re-ranking a short list by exact distance = brute force (cdist + sort) restricted to the list;
    with the whole database as the list it is Eq. 1."""
    from scipy.spatial.distance import cdist
    cfg, X, Y, ix = tiny
    y = Y[3]
    short = rng.choice(cfg.N, size=200, replace=False)
    short[10] = -1
    ids, d = Q.exact_rerank_short_list(y, X, short, 20)
    keep = short[short >= 0]
    dd = cdist(y[None].astype(np.float64), X[keep].astype(np.float64), "sqeuclidean")[0]
    want = sorted(zip(dd.tolist(), keep.tolist()))[:20]
    assert ids.tolist() == [i for _, i in want]
    assert np.allclose(d, [v for v, _ in want], rtol=1e-12)
    ids_all, d_all = Q.exact_rerank_short_list(y, X, np.arange(cfg.N), 10)
    bf_ids, bf_d = Q.brute_force(y, X, 10)
    assert np.array_equal(ids_all, bf_ids) and np.array_equal(d_all, bf_d)


# ---- the fixed anisotropic traversal order (Sec. 3.2 "Bin Proposal Heuristic") -------------------
def test_static_order_slopes_are_the_papers():
    s = Q.slopes()
    assert s.shape == (10,) and s[5] == 1.0                        # ten slopes 1.08^k, k = -5 .. 4
    assert np.allclose(s, [1.08 ** k for k in range(-5, 5)], rtol=1e-14, atol=0)
    thr = Q.slope_thresholds(np.float64)
    assert thr.shape == (9,) and np.all(s[:-1] < thr) and np.all(thr < s[1:])
    assert np.allclose(thr * thr, s[:-1] * s[1:], rtol=1e-14, atol=0)       # geometric midpoints


def test_static_order_is_a_valid_traversal(rng):
    """No duplicates; a pair never comes before a pair that is smaller in both ranks; slope 1 is the
    isotropic order by the Euclidean norm of the 1-based rank vector; slopes s and 1/s mirror each other."""
    import math
    for R, T in ((4, 16), (7, 30), (16, 100), (32, 1024)):
        for i, s in enumerate(Q.slopes()):
            tup = Q.static_order(R, T, s)
            assert tup.shape == (min(T, R * R), 2)
            seen = set()
            for a, b in tup.tolist():
                assert (a, b) not in seen
                assert (a == 0 or (a - 1, b) in seen) and (b == 0 or (a, b - 1) in seen)
                seen.add((a, b))
        iso = sorted(((a, b) for a in range(R) for b in range(R)), key=lambda v: (math.hypot(v[0] + 1, v[1] + 1), v))
        got = [tuple(v) for v in Q.static_order(R, T, 1.0).tolist()]
        # hypot rounds; integer squared norms decide exactly
        assert [(a + 1) ** 2 + (b + 1) ** 2 for a, b in got] == [(a + 1) ** 2 + (b + 1) ** 2 for a, b in iso[:len(got)]]
        lo, hi = Q.slopes()[2], Q.slopes()[8]                       # 1.08^-3 and 1.08^3
        A = Q.static_order(R, R * R, lo)
        Bm = Q.static_order(R, R * R, hi)
        ka = (A[:, 0] + 1.0) ** 2 + (lo * (A[:, 1] + 1.0)) ** 2
        n = min(T, R * R)
        if n < R * R and ka[n - 1] < ka[n] * (1 - 1e-9):            # no tie at the cut: the sets mirror
            assert {(a, b) for a, b in A[:n].tolist()} == {(b, a) for a, b in Bm[:n].tolist()}
    few = Q.static_order(32, 200, Q.slopes()[0])
    many = Q.static_order(32, 200, Q.slopes()[9])
    assert few[:, 1].max() > few[:, 0].max() and many[:, 0].max() > many[:, 1].max()   # smaller slope: deeper into part 2


def test_static_order_slope_choice():
    base = np.arange(20, dtype=np.float32) ** 1.5
    assert Q.choose_slope(base, base) == 5                           # same rise: slope 1
    assert Q.choose_slope(3.0 * base + 7.0, 3.0 * base + 1.0) == 5   # offsets and a common scale do not matter
    assert Q.choose_slope(base, 0.0 * base) == 0                     # list 2 flat: go deep into part 2
    assert Q.choose_slope(0.0 * base, base) == 9
    for k in range(-5, 5):
        assert Q.choose_slope(base, np.float32(1.08 ** k) * base) == k + 5
        assert Q.choose_slope(base.astype(np.float64), (1.08 ** k) * base.astype(np.float64)) == k + 5
    assert Q.choose_slope(base[:1], base[:1]) == 0                   # a single entry: nothing rises


def test_static_order_costs_at_least_the_summed_distance_order(tiny):
    """The order by summed distance takes the T smallest sums; any other order's first T sums add up to
    at least as much, and for T = R^2 both visit everything."""
    cfg, X, Y, ix = tiny
    for q in range(10):
        tr = Q.query(ix, Y[q], cfg.k, cfg.w, with_margins=False)
        for T in (1, 10, 100):
            _, ke = Q.bin_order([tr.Ld[0], tr.Ld[1]], T)
            ts, ks = Q.bin_order_static([tr.Ld[0], tr.Ld[1]], T)
            assert ks.shape == ke.shape and ks.sum() >= ke.sum() * (1 - 1e-12)
            assert np.allclose(ks, tr.Ld[0][ts[:, 0]] + tr.Ld[1][ts[:, 1]])
        R = tr.Ld[0].shape[0]
        te, _ = Q.bin_order([tr.Ld[0], tr.Ld[1]], R * R)
        ts, _ = Q.bin_order_static([tr.Ld[0], tr.Ld[1]], R * R)
        assert {tuple(t) for t in te.tolist()} == {tuple(t) for t in ts.tolist()}
        assert tuple(ts[0]) == (0, 0)                                # the best bin first (Sec. 3.2)


# ---- codes stored as (centroid pair, lambda level): Eq. 7 directly -----------------------------
def test_pair_lambda_score_equals_distance_to_reconstruction(tiny_pair):
    cfg, X, Y, ix = tiny_pair
    cc64 = B.pair_table(ix.C1, ix.M)
    assert ix.codes.shape == (cfg.N, 2 * cfg.M)
    for q in range(5):
        a = Q.level1_subpart_distances(Y[q], ix.C1, ix.M)
        pos = np.arange(q, cfg.N, 211)
        s = Q.score_pair_lambda(a, cc64, ix.codes[pos])
        for t, ps in enumerate(pos):
            xr = Q.reconstruct(ix, ix.codes[ps])
            want = float(np.sum((Y[q].astype(np.float64) - xr) ** 2))
            assert abs(s[t] - want) <= 1e-9 * max(want, 1e-30)


def test_pair_lambda_codes_are_nearest_code_points(tiny_pair):
    """Brute force over every (pair, level): explicit reconstruction of all k1(k1-1)/2 x 256 points."""
    cfg, X, Y, ix = tiny_pair
    ds = cfg.D // cfg.M
    pairs = Q.centroid_pairs(cfg.k1)
    lam = Q.lambda_of_level(np.arange(256))[:, None]
    for t in range(0, cfg.N, 487):
        x = X[ix.ids[t]].astype(np.float64)
        for m in range(cfg.M):
            cen = B.subpart_centroids(ix.C1, ix.M, m)
            xs = x[m * ds:(m + 1) * ds]
            best, best_code = np.inf, None
            for pi, (i, j) in enumerate(pairs):
                pts = (1.0 - lam) * cen[i][None] + lam * cen[j][None]          # 256 points of this line
                e = np.sum((pts - xs[None]) ** 2, axis=1)
                lv = int(np.argmin(e))
                if e[lv] < best:
                    best, best_code = float(e[lv]), (pi, lv)
            got = (int(ix.codes[t, 2 * m]), int(ix.codes[t, 2 * m + 1]))
            if got != best_code:                                               # only an exact tie may differ
                i, j = pairs[got[0]]
                p = (1.0 - lam[got[1], 0]) * cen[i] + lam[got[1], 0] * cen[j]
                assert abs(float(np.sum((p - xs) ** 2)) - best) <= 1e-12 * max(best, 1e-30), (t, m, got, best_code)


def test_pair_lambda_beats_nearest_centroid_and_table_of_same_lines(tiny_pair, tiny):
    """Every centroid is a code point (lambda = 0 or 1 of a line through it), so the error can never
    exceed the distance to the nearest level-1 centroid of the sub-part."""
    cfg, X, Y, ix = tiny_pair
    ds = cfg.D // cfg.M
    for t in range(0, cfg.N, 97):
        x = X[ix.ids[t]].astype(np.float64)
        xr = Q.reconstruct(ix, ix.codes[t])
        for m in range(cfg.M):
            cen = B.subpart_centroids(ix.C1, ix.M, m)
            xs = x[m * ds:(m + 1) * ds]
            nearest = float(np.min(np.sum((cen - xs[None]) ** 2, axis=1)))
            assert float(np.sum((xr[m * ds:(m + 1) * ds] - xs) ** 2)) <= nearest * (1 + 1e-12) + 1e-12


def test_pair_lambda_grid_and_pair_numbering():
    assert Q.lambda_of_level(96) == 0.0 and Q.lambda_of_level(112) == 1.0
    assert Q.lambda_of_level(0) == -6.0 and Q.lambda_of_level(255) == 159.0 / 16
    assert list(Q.level_of_lambda([-10.0, 10.0, 0.0, 1.0, 0.5 / 16, 0.49 / 16, -0.51 / 16])) == [0, 255, 96, 112, 97, 96, 95]
    for k1 in (2, 5, 16, 23):
        pairs = Q.centroid_pairs(k1)
        assert len(pairs) == k1 * (k1 - 1) // 2
        for pi, (i, j) in enumerate(pairs):
            assert i < j and pi == i * (2 * k1 - i - 1) // 2 + (j - i - 1)


def test_pair_lambda_point_on_a_segment_is_reproduced(rng):
    """A vector whose sub-vectors sit on a centroid segment at a grid lambda costs nothing."""
    P, k1, D, M = 2, 6, 8, 4
    C1 = rng.normal(size=(P, k1, D // P)).astype(np.float32)
    ds = D // M
    x = np.zeros(D)
    want = []
    for m, (i, j, level) in enumerate([(0, 3, 100), (1, 2, 96 + 16), (4, 5, 99), (2, 5, 10)]):
        cen = B.subpart_centroids(C1, M, m)
        lam = (level - 96) / 16
        x[m * ds:(m + 1) * ds] = (1 - lam) * cen[i] + lam * cen[j]
        want += [Q.centroid_pairs(k1).index((i, j)), level]
    code = B.encode_pair_lambda(x[None], C1, M)[0]
    # lambda = 1 on (1, 2) is the point c_2 itself, which lies on every line through c_2: the first such pair wins
    assert list(code[:2]) == want[:2] and list(code[4:]) == want[4:]
    ix = Q.PQTIndex(D=D, P=P, k1=k1, k2=1, M=M, N=1, H=1, T=1, C=1, C1=C1, C2=None, tbl_i=None, tbl_j=None,
                    tbl_lam=None, cc=None, offsets=None, ids=None, codes=code[None], code_format=1)
    assert np.allclose(Q.reconstruct(ix, code), x, rtol=0, atol=1e-12)


def test_pair_lambda_index_file_roundtrip(tiny_pair, tmp_path):
    cfg, X, Y, ix = tiny_pair
    path = str(tmp_path / "pair.pqt")
    IO.write_index(path, ix)
    back = IO.read_index(path)
    assert back.code_format == 1 and np.array_equal(back.codes, ix.codes) and np.array_equal(back.ids, ix.ids)
    tr0, tr1 = Q.query(ix, Y[0], cfg.k, cfg.w), Q.query(back, Y[0], cfg.k, cfg.w)
    assert np.array_equal(tr0.out_ids, tr1.out_ids)


# ---- bin order for four tree parts against its definition written out (Sec. 2.3, Sec. 3.2) ---------
def _four_part_order_by_definition(L, T):
    """All R^4 rank tuples ordered by the recursive definition: parts (1,2) and (3,4) are ranked as
    two-part orders (fl32 sum, r, r'); a tuple's key is (fl32(s12 + s34), pos12, pos34) with pos the
    position of its pair in those orders.  Plain Python, no call into the oracle."""
    R = [len(l) for l in L]
    o12 = sorted((np.float32(L[0][a] + L[1][b]), a, b) for a in range(R[0]) for b in range(R[1]))
    o34 = sorted((np.float32(L[2][c] + L[3][d]), c, d) for c in range(R[2]) for d in range(R[3]))
    pos12 = {(a, b): n for n, (_, a, b) in enumerate(o12)}
    pos34 = {(c, d): n for n, (_, c, d) in enumerate(o34)}
    items = []
    for a in range(R[0]):
        for b in range(R[1]):
            for c in range(R[2]):
                for d in range(R[3]):
                    s = np.float32(o12[pos12[(a, b)]][0] + o34[pos34[(c, d)]][0])
                    items.append((s, pos12[(a, b)], pos34[(c, d)], (a, b, c, d)))
    items.sort(key=lambda it: it[:3])
    return [it[3] for it in items[:T]], np.array([it[0] for it in items[:T]], dtype=np.float32)


@pytest.mark.parametrize("integer", [False, True])
def test_bin_order_four_parts_equals_definition(rng, integer):
    """The four lists differ in length and scale, so exchanging any two parts (or the positions
    in the two pair lists) changes the order."""
    for lens in ((3, 4, 5, 2), (6, 6, 6, 6), (1, 7, 2, 3)):
        if integer:
            L = [np.sort(rng.integers(0, 6 + 3 * p, size=n)).astype(np.float32) for p, n in enumerate(lens)]
        else:
            L = [np.sort(rng.random(n) * (1.0 + p)).astype(np.float32) for p, n in enumerate(lens)]
        total = int(np.prod(lens))
        for T in (1, 5, total // 2, total, total + 3):
            want_t, want_k = _four_part_order_by_definition(L, T)
            for method in ("fullsort", "pq"):
                for trunc in (False, True):
                    got_t, got_k = Q.bin_order(L, T, method, truncate_pairs=trunc)
                    assert [tuple(t) for t in got_t.tolist()] == want_t, (lens, T, method, trunc)
                    assert np.array_equal(got_k.astype(np.float32), want_k)


def test_linear_bin_is_row_major_part_one_most_significant():
    """Eq. 5: the multi-index (id_1, .., id_P) as one number, part 1 most significant."""
    assert Q.linear_bin([1, 2], 10) == 12
    assert Q.linear_bin([2, 1], 10) == 21
    assert Q.linear_bin([3, 0, 1], 7) == (3 * 7 + 0) * 7 + 1
    assert Q.linear_bin([5], 9) == 5
    assert Q.linear_bin([255, 255, 255, 255], 256) == 2 ** 32 - 1        # (16*16)^4 bins fit 32 bits (Sec. 3.2)
    assert Q.linear_bin([1023, 1023, 1023, 1023], 1024) == 2 ** 40 - 1   # beyond 32 bits: plain integers


def test_propose_bins_uses_part_one_as_the_high_digit():
    """A hand-made pointer array in which only bin (leaf 1, leaf 2) = 1 * k1k2 + 2 holds vectors."""
    k1k2 = 10
    offsets = np.zeros(101, dtype=np.int64)
    offsets[13:] = 4                                   # slot 12 holds four vectors
    Lid = [np.array([1, 2]), np.array([2, 1])]
    tuples = np.array([[0, 0], [1, 1], [0, 1], [1, 0]])     # leaves (1,2), (2,1), (1,1), (2,2)
    assert Q.propose_bins(tuples, Lid, k1k2, 100, offsets).tolist() == [12]
    # hashed to 7 slots: 12 % 7 = 5, 21 % 7 = 0, 11 % 7 = 4, 22 % 7 = 1
    off7 = np.array([0, 1, 1, 1, 1, 3, 6, 6])          # slots 0, 4, 5 hold vectors
    assert Q.propose_bins(tuples, Lid, k1k2, 7, off7).tolist() == [5, 0, 4]
    # a slot is proposed once: 12 and 19 collide modulo 7
    Lid2 = [np.array([1, 1]), np.array([2, 9])]
    assert Q.propose_bins(np.array([[0, 0], [1, 1]]), Lid2, k1k2, 7, off7).tolist() == [5]


def test_decision_margins_on_a_hand_made_trace():
    """Every gap computed by hand: relative gap = (hi - lo) / max(|lo|, |hi|)."""
    ix = Q.PQTIndex(D=4, P=2, k1=3, k2=2, M=2, N=9, H=36, T=3, C=5, C1=None, C2=None, tbl_i=None, tbl_j=None,
                    tbl_lam=None, cc=None, offsets=None, ids=None, codes=None)
    off = np.zeros(37, dtype=np.int64)
    # bins: leaves (0,0) -> slot 0 holds 2 vectors, (0,1) -> slot 1 holds 4, (1,0) -> slot 6 holds 3
    off[1:] = 2
    off[2:] += 4
    off[7:] += 3
    ix.offsets = off
    tr = Q.QueryTrace()
    tr.d1 = np.array([[4.0, 1.0, 2.0], [8.0, 10.0, 9.0]])            # w = 2: gaps (4-2)/4 and (10-9)/10
    tr.Ld = np.array([[1.0, 2.0, 5.0, 7.0], [0.5, 1.0, 4.0, 6.0]])
    tr.Lid = np.array([[0, 1, 2, 3], [0, 1, 2, 3]])
    # order by sum: (0,0)=1.5, (0,1)=2.0, (1,0)=2.5, (1,1)=3.0, ...
    tr.tuples = np.array([[0, 0], [0, 1], [1, 0]])
    tr.keys = np.array([1.5, 2.0, 2.5])
    tr.slots = np.array([0, 1, 6])
    tr.cand_ids = np.arange(5)
    tr.scores = np.array([3.0, 1.0, 1.0, 2.0, 8.0])                 # sorted: 1, 1, 2, 3, 8
    m = Q.decision_margins(ix, tr, k=3, w=2, T=3, C=5)
    assert m["select"] == pytest.approx(min((4.0 - 2.0) / 4.0, (10.0 - 9.0) / 10.0))
    assert m["tuples"] == pytest.approx((3.0 - 2.5) / 3.0)           # third key 2.5, the first unexamined 3.0
    # runs 2 + 4 + 3 = 9 > C = 5: the cut falls into the second run (slot 1, key 2.0);
    # its neighbours in the order have keys 1.5 and 2.5
    assert m["budget"] == pytest.approx(min((2.0 - 1.5) / 2.0, (2.5 - 2.0) / 2.5))
    # first k + 1 = 4 scores 1, 1, 2, 3: equal scores are skipped, gaps (2-1)/2 and (3-2)/3
    assert m["topk"] == pytest.approx(1.0 / 3.0)
    assert m["min"] == pytest.approx(0.1)
    # nothing to decide: w = k1, T covers every tuple, budget not reached, one candidate
    tr.scores, tr.cand_ids = np.array([2.0]), np.array([0])
    m = Q.decision_margins(ix, tr, k=3, w=3, T=16, C=50)
    assert m["select"] == np.inf and m["tuples"] == np.inf and m["budget"] == np.inf and m["topk"] == np.inf
