"""GPU parity: the HIP path, called through the C ABI, against the CPU oracle on the same
seeded inputs.  Bit-exact on selected clusters, bin order, proposed slots, candidate lists and
top-k ids (by replaying the oracle's discrete logic on the GPU's fp32 values); fp32 distances
within 1e-4 relative (plus the cancellation floor stated in parity_util)."""
import os
import sys

import numpy as np
import pytest

sys.path.insert(0, os.path.dirname(__file__))
import parity_util as PU  # noqa: E402
from oracle import pqt_build as B  # noqa: E402
from oracle import pqt_index_io as IO  # noqa: E402
from oracle import pqt_query as Q  # noqa: E402

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def pqt():
    import torch
    if not torch.cuda.is_available():
        pytest.fail("GPU tests need a GPU: no silent fallback")
    import paper_1702_05911_amd.binding as binding
    return binding


def _run_debug(pqt, gix, Y, k, w):
    import torch
    yq = torch.from_numpy(np.ascontiguousarray(Y)).cuda()
    names = tuple(n for n in pqt._TAP_FIELDS if n != "lut" or pqt.pqt_index_info(gix)["code_format"] == 0)
    ids, dists, taps = pqt.pqt_query_batch_debug(gix, yq, k, w, taps=names)
    torch.cuda.synchronize()
    ids2, dists2 = pqt.pqt_query_batch(gix, yq, k, w)
    torch.cuda.synchronize()
    assert torch.equal(ids, ids2) and torch.equal(dists.view(torch.int32), dists2.view(torch.int32)), \
        "debug and plain entry points disagree"
    return PU.to_np(ids), PU.to_np(dists), {n: PU.to_np(t) for n, t in taps.items()}


def _stagewise(pqt, ix, path, Y, k, w, T, C, exact=False, must_match_all=False, order="fullsort", truncate_pairs=False):
    gix = pqt.pqt_index_load(path, 0)
    try:
        pqt.pqt_set_budget(gix, T, C)
        if order == "static":
            pqt.pqt_set_bin_order(gix, pqt.PQT_ORDER_STATIC_SLOPES)
        ids, dists, taps = _run_debug(pqt, gix, Y, k, w)
    finally:
        pqt.pqt_index_free(gix)
    same = decided = 0
    for q in range(Y.shape[0]):
        print(f"query {q}", flush=True)
        tr = PU.check_query_stages(ix, Y[q], taps, q, k, w, T, C, ids, dists, exact=exact, order=order,
                                   truncate_pairs=truncate_pairs)
        s, d = PU.end_to_end_agreement(tr, ids[q], dists[q])
        if exact or must_match_all:
            assert s, f"query {q}: ids differ from the float64 oracle"
        if exact:
            assert np.array_equal(dists[q].astype(np.float64), tr.out_dists), f"query {q}: distances not bit-exact"
        if d:
            assert s, f"query {q}: all decision margins > 1e-5 but ids differ from the oracle"
        same += s
        decided += d
    print("tolerance so far: " + PU.STATS.summary(), flush=True)
    return same, decided


def test_tiny_stagewise(pqt, tiny, tmp_path):
    cfg, X, Y, ix = tiny
    path = str(tmp_path / "tiny.pqt")
    IO.write_index(path, ix)
    same, decided = _stagewise(pqt, ix, path, Y, cfg.k, cfg.w, cfg.T, cfg.C)
    print(f"tiny: {same}/{cfg.nq} queries identical to the float64 oracle end to end, {decided} decided by margin")
    assert same >= 0.9 * cfg.nq


def test_tiny_ragged_batches_and_determinism(pqt, tiny, tmp_path):
    import torch
    cfg, X, Y, ix = tiny
    path = str(tmp_path / "tiny.pqt")
    IO.write_index(path, ix)
    gix = pqt.pqt_index_load(path, 0)
    try:
        yq = torch.from_numpy(Y).cuda()
        full_ids, full_d = pqt.pqt_query_batch(gix, yq, cfg.k, cfg.w)
        torch.cuda.synchronize()
        for n in (1, 15, 16, 17, 33):
            ids, d = pqt.pqt_query_batch(gix, yq[:n].contiguous(), cfg.k, cfg.w)
            torch.cuda.synchronize()
            assert torch.equal(ids, full_ids[:n]) and torch.equal(d.view(torch.int32), full_d[:n].view(torch.int32))
        ids0, d0 = pqt.pqt_query_batch(gix, yq[:0].contiguous(), cfg.k, cfg.w)
        assert ids0.shape == (0, cfg.k)
        info = pqt.pqt_index_info(gix)
        assert (info["N"], info["D"], info["P"], info["k1"], info["k2"], info["M"], info["H"]) == \
            (cfg.N, cfg.D, cfg.P, cfg.k1, cfg.k2, cfg.M, cfg.H)
    finally:
        pqt.pqt_index_free(gix)


def test_tiny_exhaustive_visits_everything(pqt, tiny, tmp_path):
    """w = k1, T = K, C >= N: every bin is visited, the candidate list is the whole database."""
    cfg, X, Y, ix = tiny
    path = str(tmp_path / "tiny.pqt")
    IO.write_index(path, ix)
    Ys = Y[:6]
    gix = pqt.pqt_index_load(path, 0)
    try:
        pqt.pqt_set_budget(gix, ix.K, cfg.N)
        ids, dists, taps = _run_debug(pqt, gix, Ys, 10, cfg.k1)
    finally:
        pqt.pqt_index_free(gix)
    for q in range(Ys.shape[0]):
        assert int(taps["n_cand"][q]) == cfg.N
        assert np.array_equal(np.sort(taps["cand_ids"][q]), np.arange(cfg.N))
        PU.check_query_stages(ix, Ys[q], taps, q, 10, cfg.k1, ix.K, cfg.N, ids, dists)


def _exact_arithmetic_index(N=3000, seed=5, k1=4, k2=2, P=2):
    """Integer codebooks, integer data and dyadic lambdas: every fp32 operation of the path is
    exact, so the GPU must equal the float64 oracle bit for bit, distances included."""
    from workloads import small_integer_vectors
    rng = np.random.default_rng(seed)
    D, M = 16, 4
    dp = D // P
    C1 = rng.integers(0, 8, size=(P, k1, dp)).astype(np.float32)
    C2 = np.clip(C1[:, :, None, :] + rng.integers(-1, 2, size=(P, k1, k2, dp)), 0, 7).astype(np.float32)
    lams = [0.0, 0.25, 0.5, 0.75, 1.0, -0.25, 1.25, 0.125]
    ent = [(i, j, lam) for i in range(k1) for j in range(i + 1, k1) for lam in lams]
    ti = np.array([[ent[c % len(ent)][0] for c in range(256)]] * M, np.uint8)
    tj = np.array([[ent[c % len(ent)][1] for c in range(256)]] * M, np.uint8)
    tl = np.array([[ent[c % len(ent)][2] for c in range(256)]] * M, np.float32)
    X = small_integer_vectors(N, D, 0, 8, seed=seed, clusters=40)
    Y = small_integer_vectors(64, D, 0, 8, seed=seed + 1, clusters=40)
    ix = B.build_index(X, P, k1, k2, M, T=64, C=512, codebooks=(C1, C2), line_table=(ti, tj, tl))
    return ix, X, Y


def test_exact_arithmetic_index_is_bit_exact(pqt, tmp_path):
    ix, X, Y = _exact_arithmetic_index()
    path = str(tmp_path / "exact.pqt")
    IO.write_index(path, ix)
    for (k, w, T, C) in ((10, 2, 16, 200), (50, 4, 64, 512), (7, 1, 4, 64)):
        same, _ = _stagewise(pqt, ix, path, Y, k, w, T, C, exact=True)
        assert same == Y.shape[0]


def test_exact_arithmetic_wide_lists_heavily_tied_bin_keys(pqt, tmp_path):
    """Integer level-2 distances over wide lists: thousands of bin keys tie, so the ranking pass must cut
    the ties at the T-th tuple by (r1, r2) exactly (region larger than the sort buffer)."""
    ix, X, Y = _exact_arithmetic_index(N=20000, seed=11, k1=16, k2=8)
    path = str(tmp_path / "exact_wide.pqt")
    IO.write_index(path, ix)
    for (k, w, T, C) in ((20, 8, 1020, 4096), (20, 16, 2040, 2000), (10, 8, 510, 512), (10, 4, 300, 512)):
        same, _ = _stagewise(pqt, ix, path, Y[:24], k, w, T, C, exact=True)
        assert same == 24


def test_duplicate_database_ties_broken_by_id(pqt, tmp_path):
    """All vectors identical: one bin, every score tied -> the k smallest ids."""
    ix, X, Y = _exact_arithmetic_index(N=64)
    Xd = np.repeat(X[:1], 1500, axis=0)
    ixd = B.build_index(Xd, ix.P, ix.k1, ix.k2, ix.M, T=16, C=1000, codebooks=(ix.C1, ix.C2),
                        line_table=(ix.tbl_i, ix.tbl_j, ix.tbl_lam))
    path = str(tmp_path / "dup.pqt")
    IO.write_index(path, ixd)
    same, _ = _stagewise(pqt, ixd, path, np.ascontiguousarray(Xd[:3] + 0), 100, ix.k1, 16, 1000, exact=True)
    assert same == 3
    gix = pqt.pqt_index_load(path, 0)
    try:
        import torch
        ids, d = pqt.pqt_query_batch(gix, torch.from_numpy(Xd[:1].copy()).cuda(), 100, ix.k1)
        assert ids[0].tolist() == list(range(100))
    finally:
        pqt.pqt_index_free(gix)


def test_fewer_candidates_than_k_pads(pqt, tiny, tmp_path):
    cfg, X, Y, ix = tiny
    path = str(tmp_path / "tiny.pqt")
    IO.write_index(path, ix)
    Xs = X[:40]
    ixs = B.build_index(Xs, cfg.P, cfg.k1, cfg.k2, cfg.M, T=4, C=64, codebooks=(ix.C1, ix.C2),
                        line_table=(ix.tbl_i, ix.tbl_j, ix.tbl_lam))
    p2 = str(tmp_path / "small.pqt")
    IO.write_index(p2, ixs)
    gix = pqt.pqt_index_load(p2, 0)
    try:
        ids, dists, taps = _run_debug(pqt, gix, Y[:20], 50, 1)
    finally:
        pqt.pqt_index_free(gix)
    for q in range(20):
        PU.check_query_stages(ixs, Y[q], taps, q, 50, 1, 4, 64, ids, dists)
        nc = int(taps["n_cand"][q])
        assert nc < 50 and np.all(ids[q][nc:] == -1) and np.all(np.isinf(dists[q][nc:]))


def test_large_candidate_budgets_change_the_workgroup_shape(pqt, tiny, tmp_path):
    """The re-rank workgroup grows with the candidate budget (a thread holds at most twenty keys):
    budgets on either side of 5120 and 10240, the largest one reaching every vector of the database."""
    cfg, X, Y, ix = tiny
    path = str(tmp_path / "tiny.pqt")
    IO.write_index(path, ix)
    T = (cfg.k1 * cfg.k2) ** 2                                     # every bin of the tiny tree
    for C in (5120, 5121, 10240, 10241, 16384):
        same, _ = _stagewise(pqt, ix, path, Y[:5], cfg.k, cfg.k1, T, C)
        assert same >= 4
    _stagewise(pqt, ix, path, Y[:3], 1000, cfg.k1, T, 16384)        # k large: the short list holds 2048 keys


def test_more_runs_than_the_workgroup_keeps_in_lds(pqt, tmp_path):
    """Two huge clusters and scattered single vectors: the mean run is long, so the workgroup keeps only
    a short run list in LDS (twice what the budget needs at the mean run length), but a query among the
    scattered vectors gathers from more runs than that and reads the rest of its list from memory."""
    rng = np.random.default_rng(12345)
    P, k1, k2, M, D, T, C = 2, 8, 4, 4, 16, 1024, 3000
    centers = rng.normal(size=(2, D)) * 0.01 + np.array([[4.0] * D, [-4.0] * D])
    big = np.repeat(centers, 4940, axis=0) + rng.normal(size=(9880, D)) * 1e-3
    lone = rng.uniform(-1.5, 1.5, size=(120, D))
    X = np.concatenate([big, lone]).astype(np.float32)
    X = X[rng.permutation(X.shape[0])]
    ix = B.build_index(X, P, k1, k2, M, T=T, C=C, train_n=None, iters=8)
    mean_run = X.shape[0] / np.count_nonzero(np.diff(ix.offsets.astype(np.int64)))
    kept = 64
    while kept < T and kept < 2 * C / mean_run:
        kept *= 2
    Y = (lone[:12] + rng.normal(size=(12, D)) * 0.05).astype(np.float32)
    path = str(tmp_path / "skew.pqt")
    IO.write_index(path, ix)
    gix = pqt.pqt_index_load(path, 0)
    try:
        ids, dists, taps = _run_debug(pqt, gix, Y, 20, k1)
    finally:
        pqt.pqt_index_free(gix)
    assert kept < T and int(taps["n_slots"].max()) > kept, "the case does not reach past the LDS run list"
    for q in range(Y.shape[0]):
        PU.check_query_stages(ix, Y[q], taps, q, 20, k1, T, C, ids, dists)


def test_many_medium_runs_are_walked_by_the_wavefront(pqt, tmp_path):
    """Two huge clusters (so the workgroup keeps only 64 runs in LDS) and a few hundred small groups of
    about twenty near-identical vectors: a query among the groups gathers from well over 64 runs whose
    mean length is above sixteen, so a wavefront walks the run list as one, through several blocks of
    64 runs, the later ones read from memory."""
    rng = np.random.default_rng(4242)
    P, k1, k2, M, D, T, C = 2, 8, 4, 4, 16, 1024, 3000
    centers = rng.normal(size=(2, D)) * 0.01 + np.array([[4.0] * D, [-4.0] * D])
    big = np.repeat(centers, 20000, axis=0) + rng.normal(size=(40000, D)) * 1e-3
    spots = rng.uniform(-1.5, 1.5, size=(300, D))
    groups = np.repeat(spots, 20, axis=0) + rng.normal(size=(6000, D)) * 1e-4
    X = np.concatenate([big, groups]).astype(np.float32)
    X = X[rng.permutation(X.shape[0])]
    # the tree is trained on the groups and a few vectors of the big clusters, so that the groups spread over many bins
    C1, C2 = B.train_tree(np.concatenate([groups, big[::2000]]).astype(np.float32), P, k1, k2, iters=8)
    ix = B.build_index(X, P, k1, k2, M, T=T, C=C, codebooks=(C1, C2))
    mean_run = X.shape[0] / np.count_nonzero(np.diff(ix.offsets.astype(np.int64)))
    kept = 64
    while kept < T and kept < 2 * C / mean_run:
        kept *= 2
    Y = (spots[:12] + rng.normal(size=(12, D)) * 0.05).astype(np.float32)
    path = str(tmp_path / "groups.pqt")
    IO.write_index(path, ix)
    gix = pqt.pqt_index_load(path, 0)
    try:
        ids, dists, taps = _run_debug(pqt, gix, Y, 20, k1)
    finally:
        pqt.pqt_index_free(gix)
    nr, nc = taps["n_slots"].astype(np.int64), taps["n_cand"].astype(np.int64)
    print("runs per query", nr.tolist(), "candidates", nc.tolist(), "runs kept in LDS", kept, flush=True)
    walked = (nr > 2 * 64) & (nc >= 16 * nr)
    assert kept == 64 and walked.any(), "no query with more than two blocks of runs of mean length >= 16"
    for q in range(Y.shape[0]):
        PU.check_query_stages(ix, Y[q], taps, q, 20, k1, T, C, ids, dists)


@pytest.mark.parametrize("seed", range(12))
def test_random_shapes(pqt, tmp_path, seed):
    """Seeded random index shapes and budgets inside the documented limits (tree parts, codebook sizes,
    code bytes and format, hashing, bin order, w, T, C, k): every stage against the oracle."""
    from workloads import tiny_mixture
    rng = np.random.default_rng(1000 + seed)
    P = int(rng.choice([1, 2, 2, 4]))
    dp = int(rng.choice([4, 6, 8, 12]))                        # 6: not a multiple of four -> general level-2 path
    D = P * dp
    k1 = int(rng.choice([2, 3, 5, 8, 12]))
    k2 = int(rng.choice([1, 2, 4, 7]))
    per = [m for m in (1, 2, 4) if dp % m == 0]
    M = P * int(rng.choice(per))
    K = (k1 * k2) ** P
    hashed = bool(rng.integers(0, 2)) and K > 64
    H = int(rng.integers(17, min(K, 4096))) if hashed else K
    if H > (1 << 22):                                          # keep the oracle's pointer array small
        H = 4093
    code_format = int(rng.integers(0, 2)) if k1 >= 2 else 0
    N = int(rng.integers(500, 4000))
    X = tiny_mixture(N, d=D, seed=50 + seed)
    Y = tiny_mixture(10, d=D, seed=90 + seed)
    w = int(rng.integers(1, k1 + 1))
    R = w * k2
    T = int(rng.integers(1, min(R ** P, 3000) + 1))
    C = int(rng.integers(1, 2 * N))
    C = min(C, 16384)
    k = int(rng.integers(1, min(C, 300) + 1))
    ix = B.build_index(X, P, k1, k2, M, H=H, T=T, C=C, iters=3, code_format=code_format)
    path = str(tmp_path / f"rand{seed}.pqt")
    IO.write_index(path, ix)
    order = "static" if (P == 2 and H == K and rng.integers(0, 2)) else "fullsort"
    print(f"seed {seed}: P={P} D={D} k1={k1} k2={k2} M={M} H={H} K={K} N={N} w={w} T={T} C={C} k={k} "
          f"codes={code_format} order={order}", flush=True)
    _stagewise(pqt, ix, path, Y, k, w, T, C, order=order)


def test_hashed_index_dedupes_slots(pqt, tiny, tmp_path):
    cfg, X, Y, ix = tiny
    ixh = B.build_index(X[:3000], cfg.P, cfg.k1, cfg.k2, cfg.M, H=97, T=256, C=1024, codebooks=(ix.C1, ix.C2),
                        line_table=(ix.tbl_i, ix.tbl_j, ix.tbl_lam))
    path = str(tmp_path / "hashed.pqt")
    IO.write_index(path, ixh)
    _stagewise(pqt, ixh, path, Y[:24], 10, 4, 256, 1024)
    _stagewise(pqt, ixh, path, Y[:8], 10, cfg.k1, 1024, 3000)


def test_single_part_index(pqt, tmp_path, rng):
    X = rng.normal(size=(2000, 8)).astype(np.float32)
    Y = rng.normal(size=(20, 8)).astype(np.float32)
    ix1 = B.build_index(X, P=1, k1=8, k2=2, M=2, T=16, C=512, iters=5)
    path = str(tmp_path / "p1.pqt")
    IO.write_index(path, ix1)
    _stagewise(pqt, ix1, path, Y, 10, 3, 16, 512)
    _stagewise(pqt, ix1, path, Y, 10, 8, 3, 100)


def test_wide_selection_two_elements_per_lane(pqt, tmp_path, rng):
    """R = w*k2 = 128 > 64 lanes, k1 = 32 (two MFMA column tiles), ragged last tile."""
    X = rng.random(size=(6000, 24)).astype(np.float32)
    Y = rng.random(size=(19, 24)).astype(np.float32)
    ixw = B.build_index(X, P=2, k1=32, k2=16, M=6, T=300, C=700, iters=4)
    path = str(tmp_path / "wide.pqt")
    IO.write_index(path, ixw)
    _stagewise(pqt, ixw, path, Y, 20, 8, 300, 700)
    # R = 256: four list entries per lane; R = 512: lists sorted in LDS
    _stagewise(pqt, ixw, path, Y[:8], 20, 16, 300, 700)
    _stagewise(pqt, ixw, path, Y[:4], 20, 32, 300, 700)


def test_part_dimension_not_a_multiple_of_four(pqt, tmp_path, rng):
    """D/P = 6: the level-2 codebook keeps its plain layout (no 16-byte pieces)."""
    X = rng.random(size=(3000, 12)).astype(np.float32)
    Y = rng.random(size=(21, 12)).astype(np.float32)
    ix6 = B.build_index(X, P=2, k1=8, k2=4, M=4, T=200, C=500, iters=4)
    path = str(tmp_path / "dp6.pqt")
    IO.write_index(path, ix6)
    _stagewise(pqt, ix6, path, Y, 10, 3, 200, 500)


def test_index_from_arrays_matches_index_from_file(pqt, tiny, tmp_path):
    """pqt_index_from_arrays with host arrays and with device arrays answers exactly like the index
    loaded from the file that holds the same arrays."""
    import torch
    cfg, X, Y, ix = tiny
    path = str(tmp_path / "tiny.pqt")
    IO.write_index(path, ix)
    arrays = dict(N=ix.N, H=ix.H, D=ix.D, P=ix.P, k1=ix.k1, k2=ix.k2, M=ix.M, T=ix.T, C=ix.C,
                  C1=ix.C1, C2=ix.C2, tbl_i=ix.tbl_i, tbl_j=ix.tbl_j, tbl_lam=ix.tbl_lam, cc=ix.cc,
                  offsets=ix.offsets, ids=ix.ids, codes=ix.codes)
    on_dev = dict(arrays)
    on_dev["offsets"] = torch.from_numpy(ix.offsets.astype(np.int64)).cuda()
    on_dev["ids"] = torch.from_numpy(ix.ids.astype(np.int32)).cuda()
    on_dev["codes"] = torch.from_numpy(ix.codes).cuda()
    yq = torch.from_numpy(Y).cuda()
    results = []
    for make in (lambda: pqt.pqt_index_load(path, 0), lambda: pqt.pqt_index_from_arrays(arrays, 0),
                 lambda: pqt.pqt_index_from_arrays(on_dev, 0)):
        gix = make()
        try:
            ids, d = pqt.pqt_query_batch(gix, yq, cfg.k, cfg.w)
            torch.cuda.synchronize()
            results.append((ids.cpu(), d.cpu()))
            info = pqt.pqt_index_info(gix)
            assert (info["N"], info["H"], info["T"], info["C"]) == (ix.N, ix.H, ix.T, ix.C)
        finally:
            pqt.pqt_index_free(gix)
    for ids, d in results[1:]:
        assert torch.equal(ids, results[0][0]) and torch.equal(d.view(torch.int32), results[0][1].view(torch.int32))
    bad = dict(arrays)
    bad["offsets"] = ix.offsets.copy()
    bad["offsets"][3] = bad["offsets"][-1] + 1
    with pytest.raises(pqt.PqtError) as e:
        pqt.pqt_index_from_arrays(bad, 0)
    assert e.value.code == pqt.PQT_EFORMAT


def _check_exact(pqt, gix, ix, X, Y, k_short, k, w, bit_exact):
    """pqt_query_batch_exact against the oracle: the short list is the line-quantisation top-k_short
    (already checked stage by stage elsewhere; taken from the GPU here), its exact re-ranking must be
    the oracle's on the same list."""
    import torch
    yq = torch.from_numpy(np.ascontiguousarray(Y)).cuda()
    short, _ = pqt.pqt_query_batch(gix, yq, k_short, w)
    ids, d = pqt.pqt_query_batch_exact(gix, yq, k_short, k, w)
    ids_all, d_all = pqt.pqt_query_batch_exact(gix, yq, k_short, k_short, w)
    torch.cuda.synchronize()
    short, ids, d, ids_all, d_all = (PU.to_np(t) for t in (short, ids, d, ids_all, d_all))
    for q in range(Y.shape[0]):
        o_ids, o_d = Q.exact_rerank_short_list(Y[q], X, short[q], k_short)
        have = o_ids >= 0
        # every exact distance within tolerance (compare through the id)
        lookup = dict(zip(o_ids[have].tolist(), o_d[have].tolist()))
        assert sorted(ids_all[q][ids_all[q] >= 0].tolist()) == sorted(o_ids[have].tolist()), "id set of the short list"
        got = np.array([lookup[i] for i in ids_all[q][ids_all[q] >= 0].tolist()])
        gd = d_all[q][ids_all[q] >= 0]
        assert PU.close(gd, got), f"query {q}: exact distances"     # sums of squared differences: relative error only
        # the order is the order of the GPU's own distances, ties by id; the first k are the k-result call
        o = np.lexsort((ids_all[q][ids_all[q] >= 0], gd))
        assert np.array_equal(o, np.arange(o.shape[0])), f"query {q}: not sorted by (distance, id)"
        assert np.array_equal(ids[q], ids_all[q][:k]) and np.array_equal(d[q], d_all[q][:k])
        assert np.all(ids_all[q][have.sum():] == -1) and np.all(np.isinf(d_all[q][have.sum():]))
        if bit_exact:
            assert np.array_equal(ids_all[q], o_ids) and np.array_equal(d_all[q].astype(np.float64)[have], o_d[have])


def test_exact_rerank_of_short_list(pqt, tiny, tmp_path):
    import torch
    cfg, X, Y, ix = tiny
    path = str(tmp_path / "tiny.pqt")
    IO.write_index(path, ix)
    gix = pqt.pqt_index_load(path, 0)
    try:
        with pytest.raises(pqt.PqtError) as e:
            pqt.pqt_query_batch_exact(gix, torch.from_numpy(Y).cuda(), 50, 10, cfg.w)
        assert e.value.code == pqt.PQT_EINVAL                      # no vectors attached yet
        pqt.pqt_index_set_vectors(gix, X)                          # host array: copied
        _check_exact(pqt, gix, ix, X, Y[:40], 50, 10, cfg.w, bit_exact=False)
        _check_exact(pqt, gix, ix, X, Y[:10], 256, 100, cfg.k1, bit_exact=False)     # more than the candidates of some queries
        Xd = torch.from_numpy(X).cuda()
        pqt.pqt_index_set_vectors(gix, Xd)                         # device tensor: used in place
        _check_exact(pqt, gix, ix, X, Y[:10], 64, 64, cfg.w, bit_exact=False)
        with pytest.raises(pqt.PqtError) as e:
            pqt.pqt_query_batch_exact(gix, torch.from_numpy(Y).cuda(), 10, 20, cfg.w)   # k > k_short
        assert e.value.code == pqt.PQT_EINVAL
    finally:
        pqt.pqt_index_free(gix)
    # integer data: fp32 and uint8 storage, every operation exact -> equal to the float64 oracle bit for bit
    ixe, Xe, Ye = _exact_arithmetic_index()
    path = str(tmp_path / "exact.pqt")
    IO.write_index(path, ixe)
    gix = pqt.pqt_index_load(path, 0)
    try:
        for stored in (Xe, Xe.astype(np.uint8)):
            pqt.pqt_index_set_vectors(gix, stored)
            _check_exact(pqt, gix, ixe, Xe, Ye[:32], 100, 20, 2, bit_exact=True)
    finally:
        pqt.pqt_index_free(gix)


def test_native_builder(pqt, tiny, tmp_path):
    """pqt_builder_*: vectors streamed in ragged chunks; the saved index satisfies the oracle's
    definitions (bin of every vector, nearest code point, sorted lists) and answers queries exactly as
    the oracle does on that index."""
    import torch
    cfg, X, Y, ix = tiny
    params = dict(N=cfg.N, H=ix.H, D=ix.D, P=ix.P, k1=ix.k1, k2=ix.k2, M=ix.M, T=ix.T, C=ix.C,
                  C1=ix.C1, C2=ix.C2, tbl_i=ix.tbl_i, tbl_j=ix.tbl_j, tbl_lam=ix.tbl_lam, cc=ix.cc)
    Xd = torch.from_numpy(X).cuda()
    b = pqt.pqt_builder_create(params, 0)
    try:
        with pytest.raises(pqt.PqtError) as e:
            pqt.pqt_builder_finish(b)                              # nothing added yet
        assert e.value.code == pqt.PQT_EINVAL
        for lo, hi in ((0, 1), (1, 4097), (4097, 4097), (4097, cfg.N)):
            pqt.pqt_builder_add(b, Xd[lo:hi].contiguous())
        with pytest.raises(pqt.PqtError) as e:
            pqt.pqt_builder_add(b, Xd[:1].contiguous())            # more than N
        assert e.value.code == pqt.PQT_EINVAL
        gix = pqt.pqt_builder_finish(b)
    finally:
        pqt.pqt_builder_free(b)
    path = str(tmp_path / "native.pqt")
    try:
        pqt.pqt_index_save(gix, path)
    finally:
        pqt.pqt_index_free(gix)
    nix = IO.read_index(path)
    off = nix.offsets.astype(np.int64)
    assert off[0] == 0 and off[-1] == cfg.N and np.all(np.diff(off) >= 0)
    assert np.array_equal(np.sort(nix.ids), np.arange(cfg.N, dtype=np.uint32))
    for name in ("C1", "C2", "tbl_i", "tbl_j", "tbl_lam", "cc"):
        assert np.array_equal(getattr(nix, name), getattr(ix, name)), name
    slot_of = np.repeat(np.arange(nix.H), np.diff(off))
    want_slots = B.bin_slots_batch(X, nix.C1, nix.C2, nix.H)
    assert np.mean(slot_of != want_slots[nix.ids]) <= 2e-3       # fp32 vs float64 near-ties only
    for s in np.nonzero(np.diff(off) > 1)[0][:200]:
        assert np.all(np.diff(nix.ids[off[s]:off[s + 1]].astype(np.int64)) > 0)   # ids ascend inside a slot
    # codes: the chosen code point is (within fp32 rounding) as near as the nearest one
    # (the encoder takes the smallest of 256 fp32 values of Eq. 9 on the vector's own level-1 distances:
    # the chosen point may lose to the best one by the rounding of both values)
    ds = nix.D // nix.M
    kenc = (PU.kappa(ds) + 8.0) * PU.U32
    for t in np.random.default_rng(3).integers(0, cfg.N, size=300):
        x = X[nix.ids[t]].astype(np.float64)
        Sl = PU.lut_magnitudes(nix, PU.subpart_magnitudes(nix, x))
        for m in range(nix.M):
            pts = B.code_points(B.subpart_centroids(nix.C1, nix.M, m), nix.tbl_i[m], nix.tbl_j[m], nix.tbl_lam[m])
            d = np.sum((pts - x[m * ds:(m + 1) * ds][None]) ** 2, axis=1)
            got, best = int(nix.codes[t, m]), int(np.argmin(d))
            assert d[got] - d[best] <= kenc * (Sl[m, got] + Sl[m, best]), (t, m, got, best)
    # the index is input data: full stage-wise parity on it
    same, _ = _stagewise(pqt, nix, path, Y[:30], cfg.k, cfg.w, cfg.T, cfg.C)
    assert same >= 27


def _distortion(Xp, cen):
    return float(np.mean(np.min(B.sqdist_matrix(Xp, cen), axis=1)))


def test_training_on_the_gpu(pqt, tiny):
    """pqt_train: after one Lloyd iteration every centroid is the mean of the vectors nearest to the start
    centroids (vectors at evenly spaced places of the sample, of the cell for level 2), checked with the
    oracle's distance routine; after twenty the distortion matches the oracle's own Lloyd training; the
    line table is ordered by (i, j, lambda), shares the 256 code points out in proportion to the votes
    the oracle counts, and places them inside the range of the lambdas voted on each line."""
    import torch
    cfg, X, Y, _ = tiny
    P, k1, k2, M, D = cfg.P, cfg.k1, cfg.k2, cfg.M, cfg.D
    dp, ds, n = D // P, D // M, 6000
    Xd = torch.from_numpy(X[:n]).cuda()
    one = pqt.pqt_train(Xd, P=P, k1=k1, k2=k2, M=M, iters=1, n_table=0)
    again = pqt.pqt_train(Xd, P=P, k1=k1, k2=k2, M=M, iters=1, n_table=0)
    for name in one:
        assert np.array_equal(one[name], again[name]), f"{name}: training is not deterministic"
    for p in range(P):
        Xp = X[:n, p * dp:(p + 1) * dp].astype(np.float64)
        start = Xp[(np.arange(k1) * n) // k1]
        lab = np.argmin(B.sqdist_matrix(Xp, start), axis=1)
        for i in range(k1):
            np.testing.assert_allclose(one["C1"][p, i], Xp[lab == i].mean(axis=0), rtol=1e-5, atol=1e-6)
        # level 2: cells of the finished level-1 quantiser, each trained on its own members
        lab1 = np.argmin(B.sqdist_matrix(Xp, one["C1"][p].astype(np.float64)), axis=1)
        for i in range(k1):
            sub = Xp[lab1 == i]
            if sub.shape[0] <= k2:
                continue
            start2 = sub[(np.arange(k2) * sub.shape[0]) // k2]
            lab2 = np.argmin(B.sqdist_matrix(sub, start2), axis=1)
            for j in range(k2):
                if np.any(lab2 == j):
                    np.testing.assert_allclose(one["C2"][p, i, j], sub[lab2 == j].mean(axis=0), rtol=1e-5, atol=1e-6)
    full = pqt.pqt_train(Xd, P=P, k1=k1, k2=k2, M=M, iters=20, n_table=n)
    oC1, oC2 = B.train_tree(X[:n], P, k1, k2, iters=20)
    for p in range(P):
        Xp = X[:n, p * dp:(p + 1) * dp].astype(np.float64)
        g, o = _distortion(Xp, full["C1"][p].astype(np.float64)), _distortion(Xp, oC1[p].astype(np.float64))
        print(f"part {p}: level-1 distortion GPU {g:.6f} oracle {o:.6f}", flush=True)
        assert abs(g - o) <= 0.01 * o
        g2 = _distortion(Xp, full["C2"][p].reshape(k1 * k2, dp).astype(np.float64))
        o2 = _distortion(Xp, oC2[p].reshape(k1 * k2, dp).astype(np.float64))
        assert g2 <= 1.03 * o2 and g2 < g
    np.testing.assert_allclose(full["cc"], B.pair_table(full["C1"], M), rtol=1e-6, atol=1e-9)
    pairs = Q.centroid_pairs(k1)
    for m in range(M):
        ti, tj, tl = full["tbl_i"][m], full["tbl_j"][m], full["tbl_lam"][m]
        ent = list(zip(ti.tolist(), tj.tolist(), tl.tolist()))
        assert ent == sorted(ent) and all(i < j < k1 for i, j, _ in ent)
        bp, bl, _ = B.best_lines(X[:n, m * ds:(m + 1) * ds].astype(np.float64), B.subpart_centroids(full["C1"], M, m))
        use = np.bincount(bp, minlength=len(pairs))
        got = np.zeros(len(pairs), np.int64)
        for i, j, _ in ent:
            got[pairs.index((i, j))] += 1
        quota = use * 256.0 / use.sum()
        # largest-remainder shares lie within one of the exact quota; an fp32 near-tie may move a vote or two
        assert got.sum() == 256 and np.all(np.abs(got - quota) <= 1.0 + 256.0 * 3 / n), (m, np.max(np.abs(got - quota)))
        for q in np.nonzero(got)[0]:
            lams = bl[bp == q]
            mine = tl[(ti == pairs[q][0]) & (tj == pairs[q][1])]
            assert lams.size and mine.min() >= lams.min() - 1e-3 and mine.max() <= lams.max() + 1e-3
    with pytest.raises(pqt.PqtError) as e:
        pqt.pqt_train(Xd, P=3, k1=k1, k2=k2, M=M)
    assert e.value.code in (pqt.PQT_EINVAL, pqt.PQT_EUNSUPPORTED)


def test_pair_lambda_codes(pqt, tiny_pair, tmp_path):
    """Codes stored as (centroid pair, lambda level): stage-wise parity of the query path on an
    oracle-built index; the lut tap is refused; a pair byte beyond the last pair is a format error."""
    import torch
    cfg, X, Y, ix = tiny_pair
    path = str(tmp_path / "pair.pqt")
    IO.write_index(path, ix)
    same, decided = _stagewise(pqt, ix, path, Y[:40], cfg.k, cfg.w, cfg.T, cfg.C)
    assert same >= 36
    # ragged budgets: few candidates, one tuple
    _stagewise(pqt, ix, path, Y[:8], 5, 1, 1, 7)
    gix = pqt.pqt_index_load(path, 0)
    try:
        inf = pqt.pqt_index_info(gix)
        assert inf["code_format"] == pqt.PQT_CODES_PAIR_LAMBDA and inf["code_bytes"] == 2 * cfg.M
        with pytest.raises(pqt.PqtError) as e:
            pqt.pqt_query_batch_debug(gix, torch.from_numpy(Y[:2]).cuda(), cfg.k, cfg.w, taps=("lut",))
        assert e.value.code == pqt.PQT_EINVAL
        back = pqt.pqt_index_export(gix, ("codes",))["codes"]
        assert np.array_equal(PU.to_np(back), ix.codes)
    finally:
        pqt.pqt_index_free(gix)
    arrays = dict(N=ix.N, H=ix.H, D=ix.D, P=ix.P, k1=ix.k1, k2=ix.k2, M=ix.M, T=ix.T, C=ix.C, C1=ix.C1, C2=ix.C2,
                  cc=ix.cc, offsets=ix.offsets, ids=ix.ids, codes=ix.codes.copy(), code_format=1)
    arrays["codes"][17, 2] = ix.k1 * (ix.k1 - 1) // 2          # one past the last pair
    for on_device in (False, True):
        a = dict(arrays)
        if on_device:
            for n in ("offsets", "ids"):
                a[n] = torch.from_numpy(arrays[n].astype(np.int64)).cuda()
            a["codes"] = torch.from_numpy(arrays["codes"]).cuda()
        with pytest.raises(pqt.PqtError) as e:
            pqt.pqt_index_from_arrays(a, 0)
        assert e.value.code == pqt.PQT_EFORMAT


def test_pair_lambda_native_builder(pqt, tiny_pair, tmp_path):
    """pqt_builder_* with (pair, lambda) codes: every code names a point that is (within fp32 rounding of
    the level-1 distances it is computed from) as near as the nearest code point, with the level nearest
    to the projection on its line; the index answers queries as the oracle does on it."""
    import torch
    cfg, X, Y, ix = tiny_pair
    params = dict(N=cfg.N, H=ix.H, D=ix.D, P=ix.P, k1=ix.k1, k2=ix.k2, M=ix.M, T=ix.T, C=ix.C,
                  C1=ix.C1, C2=ix.C2, cc=ix.cc, code_format=1)
    b = pqt.pqt_builder_create(params, 0)
    try:
        Xd = torch.from_numpy(X).cuda()
        for lo, hi in ((0, 4097), (4097, cfg.N)):
            pqt.pqt_builder_add(b, Xd[lo:hi].contiguous())
        gix = pqt.pqt_builder_finish(b)
    finally:
        pqt.pqt_builder_free(b)
    path = str(tmp_path / "native_pair.pqt")
    try:
        pqt.pqt_index_save(gix, path)
    finally:
        pqt.pqt_index_free(gix)
    nix = IO.read_index(path)
    assert nix.code_format == 1 and nix.codes.shape == (cfg.N, 2 * cfg.M)
    assert np.array_equal(np.sort(nix.ids), np.arange(cfg.N, dtype=np.uint32))
    ds = nix.D // nix.M
    pairs = Q.centroid_pairs(nix.k1)
    same_pair = total = 0
    kenc = (PU.kappa(ds) + 8.0) * PU.U32
    for t in np.random.default_rng(5).integers(0, cfg.N, size=300):
        x = X[nix.ids[t]].astype(np.float64)
        want = B.encode_pair_lambda(X[nix.ids[t]][None], nix.C1, nix.M)[0]
        xr_got, xr_want = Q.reconstruct(nix, nix.codes[t]), Q.reconstruct(nix, want)
        S = PU.subpart_magnitudes(nix, x)
        for m in range(nix.M):
            cen = B.subpart_centroids(nix.C1, nix.M, m)
            xs = x[m * ds:(m + 1) * ds]
            e_got = float(np.sum((xr_got[m * ds:(m + 1) * ds] - xs) ** 2))
            e_want = float(np.sum((xr_want[m * ds:(m + 1) * ds] - xs) ** 2))
            # as near as the nearest code point, up to the rounding of the two fp32 values of Eq. 9 compared
            mags = []
            for code in (nix.codes[t], want):
                ci, cj = pairs[int(code[2 * m])]
                lm = float(Q.lambda_of_level(code[2 * m + 1]))
                mags.append(abs(1 - lm) * S[m, ci] + abs(lm) * S[m, cj] + abs(lm * lm - lm) * float(nix.cc[m, ci, cj]))
            assert e_got - e_want <= kenc * (mags[0] + mags[1]), (t, m, e_got, e_want)
            i, j = pairs[nix.codes[t, 2 * m]]
            lam, _ = B.line_projection(xs, cen[i], cen[j])
            level = int(nix.codes[t, 2 * m + 1])
            if 0 < level < 255:                                               # the level nearest to the projection
                assert abs(float(Q.lambda_of_level(level)) - lam) <= 0.5 / 16 + 1e-4
            else:
                assert lam < -5.96 or lam > 9.9
            same_pair += int(nix.codes[t, 2 * m] == want[2 * m] and level == want[2 * m + 1])
            total += 1
    assert same_pair >= 0.99 * total
    same, _ = _stagewise(pqt, nix, path, Y[:30], cfg.k, cfg.w, cfg.T, cfg.C)
    assert same >= 27


def test_static_slope_order(pqt, tiny, tmp_path, rng):
    """pqt_set_bin_order(PQT_ORDER_STATIC_SLOPES): the tuples are the pre-computed order of the slope the
    oracle picks from the GPU's own lists (bit for bit), everything downstream as usual; switching back
    restores the default answers; unsupported for hashed or four-part indexes."""
    import torch
    cfg, X, Y, ix = tiny
    path = str(tmp_path / "tiny.pqt")
    IO.write_index(path, ix)
    same, _ = _stagewise(pqt, ix, path, Y[:40], cfg.k, cfg.w, cfg.T, cfg.C, order="static")
    assert same >= 36
    for k, w, T, C in ((5, 1, 1, 7), (10, 2, 37, 50), (cfg.k, cfg.k1, cfg.T, cfg.C)):      # ragged tails, R = all leaves
        _stagewise(pqt, ix, path, Y[:6], k, w, T, C, order="static")
    # every slope occurs: scale the second half of the query so that one list rises faster or slower
    slopes = set()
    for f in (0.05, 0.3, 0.6, 0.8, 0.9, 1.0, 1.1, 1.3, 1.7, 3.0, 20.0):
        y = Y[:4].copy()
        y[:, cfg.D // 2:] *= f
        tr = Q.query(ix, y[0], cfg.k, cfg.w, order_method="static")
        slopes.add(Q.choose_slope(tr.Ld[0].astype(np.float32), tr.Ld[1].astype(np.float32)))
        _stagewise(pqt, ix, path, y, cfg.k, cfg.w, cfg.T, cfg.C, order="static")
    assert len(slopes) >= 6, slopes
    gix = pqt.pqt_index_load(path, 0)
    try:
        yq = torch.from_numpy(Y[:50]).cuda()
        ids0, d0 = pqt.pqt_query_batch(gix, yq, cfg.k, cfg.w)
        pqt.pqt_set_bin_order(gix, pqt.PQT_ORDER_STATIC_SLOPES)
        ids1, _ = pqt.pqt_query_batch(gix, yq, cfg.k, cfg.w)
        pqt.pqt_set_bin_order(gix, pqt.PQT_ORDER_SUMMED_DISTANCE)
        ids2, d2 = pqt.pqt_query_batch(gix, yq, cfg.k, cfg.w)
        torch.cuda.synchronize()
        assert torch.equal(ids0, ids2) and torch.equal(d0, d2)
        assert not torch.equal(ids0, ids1)                        # the two orders visit different bins
        with pytest.raises(pqt.PqtError) as e:
            pqt.pqt_set_bin_order(gix, 7)
        assert e.value.code == pqt.PQT_EINVAL
    finally:
        pqt.pqt_index_free(gix)
    hashed = B.build_index(X[:3000], cfg.P, cfg.k1, cfg.k2, cfg.M, H=1009, T=cfg.T, C=cfg.C, iters=3)
    hpath = str(tmp_path / "hashed.pqt")
    IO.write_index(hpath, hashed)
    gix = pqt.pqt_index_load(hpath, 0)
    try:
        with pytest.raises(pqt.PqtError) as e:
            pqt.pqt_set_bin_order(gix, pqt.PQT_ORDER_STATIC_SLOPES)
        assert e.value.code == pqt.PQT_EUNSUPPORTED
    finally:
        pqt.pqt_index_free(gix)


def test_brute_force(pqt, tiny, tmp_path):
    """pqt_brute_force against Eq. 1 written out (the oracle's brute_force): integer data bit for bit
    (fp32 and byte storage, several passes over the database, ragged last pass and tile), real-valued
    data within tolerance with the order replayed on the GPU's own distances."""
    import torch
    ixe, Xe, Ye = _exact_arithmetic_index(N=20000, seed=31)
    path = str(tmp_path / "exact.pqt")
    IO.write_index(path, ixe)
    gix = pqt.pqt_index_load(path, 0)
    try:
        yq = torch.from_numpy(Ye).cuda()
        with pytest.raises(pqt.PqtError) as e:
            pqt.pqt_brute_force(gix, yq, 10)
        assert e.value.code == pqt.PQT_EINVAL                      # no vectors attached
        for stored in (Xe, Xe.astype(np.uint8)):
            pqt.pqt_index_set_vectors(gix, stored)
            for k in (1, 10, 100):
                ids, d = pqt.pqt_brute_force(gix, yq, k)
                torch.cuda.synchronize()
                ids, d = PU.to_np(ids), PU.to_np(d)
                for q in range(0, Ye.shape[0], 7):
                    o_ids, o_d = Q.brute_force(Ye[q], Xe, k)
                    assert np.array_equal(ids[q], o_ids), f"k={k} query {q}"
                    assert np.array_equal(d[q].astype(np.float64), o_d)
    finally:
        pqt.pqt_index_free(gix)
    cfg, X, Y, ix = tiny
    path = str(tmp_path / "tiny.pqt")
    IO.write_index(path, ix)
    gix = pqt.pqt_index_load(path, 0)
    try:
        pqt.pqt_index_set_vectors(gix, X)
        yq = torch.from_numpy(Y).cuda()
        ids, d = pqt.pqt_brute_force(gix, yq, 20)
        ids1, d1 = pqt.pqt_brute_force(gix, yq[:3].contiguous(), 1)
        torch.cuda.synchronize()
        ids, d = PU.to_np(ids), PU.to_np(d)
        assert np.array_equal(PU.to_np(ids1)[:, 0], ids[:3, 0])
        same = 0
        for q in range(cfg.nq):
            o_ids, o_d = Q.brute_force(Y[q], X, 21)
            y64 = Y[q].astype(np.float64)
            xx = np.sum(X[ids[q]].astype(np.float64) ** 2, axis=1)
            exact = np.sum((X[ids[q]].astype(np.float64) - y64[None]) ** 2, axis=1)
            # ||q||^2 + ||x||^2 - 2 q.x accumulated over all D dimensions
            assert PU.close(d[q], exact, np.dot(y64, y64) + xx, PU.kappa(cfg.D)), f"query {q}"
            assert np.array_equal(np.lexsort((ids[q], d[q])), np.arange(20)), "not sorted by (distance, id)"
            gaps = np.diff(o_d) / np.maximum(o_d[1:], 1e-30)
            if np.all(gaps > 1e-4):                                 # no near-ties among the first 21: ids must agree
                assert np.array_equal(ids[q], o_ids[:20]), f"query {q}"
                same += 1
        assert same >= 0.5 * cfg.nq
    finally:
        pqt.pqt_index_free(gix)


def test_four_part_index(pqt, tmp_path):
    """P = 4: parts (1,2) and (3,4) are ranked first, then pairs of positions in those two lists."""
    from workloads import tiny_mixture
    X = tiny_mixture(4000, d=32, seed=3)
    Y = tiny_mixture(24, d=32, seed=4)
    ix4 = B.build_index(X, P=4, k1=4, k2=4, M=8, T=512, C=1024, iters=5)
    path = str(tmp_path / "p4.pqt")
    IO.write_index(path, ix4)
    # (k, w, T, C): R = 8 -> pair lists of 64, final region larger than the sort buffer;
    # R = 16 -> pair lists cut at T; R = 4 -> every combination, T not a power of two; a long T
    for (k, w, T, C) in ((10, 2, 256, 1024), (10, 4, 512, 600), (5, 1, 100, 200), (10, 3, 4096, 4000)):
        _stagewise(pqt, ix4, path, Y, k, w, T, C)
    # hashed slots: bins collide, a slot is proposed once
    ixh = B.build_index(X, P=4, k1=4, k2=4, M=8, H=997, T=512, C=1024, codebooks=(ix4.C1, ix4.C2),
                        line_table=(ix4.tbl_i, ix4.tbl_j, ix4.tbl_lam))
    path = str(tmp_path / "p4h.pqt")
    IO.write_index(path, ixh)
    _stagewise(pqt, ixh, path, Y[:12], 10, 2, 300, 1024)
    # more tuples than the table for repeated slots holds: they are found by sorting (slot, tuple) keys
    _stagewise(pqt, ixh, path, Y[:6], 10, 3, 2500, 4000)


def test_four_part_long_lists(pqt, tmp_path):
    """P = 4 with lists of 128 and 64 children and T = 1024: the pair lists are cut at T, the last ranking's
    region has rows of 1024 entries beside rows of 16, so the kernel that deals out units of a row (not rows)
    to its wavefronts runs, and the keys are placed by histogram bin; hashed and unhashed bins."""
    from workloads import tiny_mixture
    X = tiny_mixture(20000, d=32, seed=5)
    Y = tiny_mixture(12, d=32, seed=6)
    ixh = B.build_index(X, P=4, k1=16, k2=16, M=8, H=65537, T=1024, C=3000, iters=4)
    path = str(tmp_path / "p4_long_hashed.pqt")
    IO.write_index(path, ixh)
    # (the oracle with its pair lists cut at T, which its pin test shows to be the same order: the uncut
    # form sorts R^4 tuples)
    _stagewise(pqt, ixh, path, Y, 10, 8, 1024, 3000, truncate_pairs=True)         # R = 128
    _stagewise(pqt, ixh, path, Y[:6], 10, 4, 700, 1500, truncate_pairs=True)      # R = 64, T not a power of two
    ix = B.build_index(X, P=4, k1=8, k2=8, M=8, T=1024, C=3000, iters=4)
    path = str(tmp_path / "p4_long.pqt")
    IO.write_index(path, ix)
    _stagewise(pqt, ix, path, Y, 10, 8, 1024, 3000, truncate_pairs=True)          # R = 64, 2^24 bins, unhashed


def test_four_part_exact_arithmetic_heavily_tied(pqt, tmp_path):
    """P = 4 on the exact-arithmetic index: integer sums tie by the hundreds in the pair lists and in the
    final ranking, so every tie cut by (position, position) is exercised; results must be bit-exact."""
    ix, X, Y = _exact_arithmetic_index(N=6000, seed=21, k1=8, k2=2, P=4)
    path = str(tmp_path / "exact_p4.pqt")
    IO.write_index(path, ix)
    for (k, w, T, C) in ((10, 8, 600, 2000), (10, 4, 256, 512), (20, 8, 2048, 4096), (10, 2, 30, 300)):
        same, _ = _stagewise(pqt, ix, path, Y[:16], k, w, T, C, exact=True)
        assert same == 16


def test_error_codes(pqt, tiny, tmp_path):
    import torch
    cfg, X, Y, ix = tiny
    path = str(tmp_path / "tiny.pqt")
    IO.write_index(path, ix)
    with pytest.raises(pqt.PqtError) as e:
        pqt.pqt_index_load(str(tmp_path / "missing.pqt"), 0)
    assert e.value.code == pqt.PQT_EIO
    bad = str(tmp_path / "bad.pqt")
    with open(path, "rb") as f:
        blob = f.read()
    with open(bad, "wb") as f:
        f.write(b"NOTANIDX" + blob[8:])
    with pytest.raises(pqt.PqtError) as e:
        pqt.pqt_index_load(bad, 0)
    assert e.value.code == pqt.PQT_EFORMAT
    with open(bad, "wb") as f:
        f.write(blob[:-100])
    with pytest.raises(pqt.PqtError) as e:
        pqt.pqt_index_load(bad, 0)
    assert e.value.code == pqt.PQT_EFORMAT
    broken = IO.read_index(path)
    broken.offsets = broken.offsets.copy()
    broken.offsets[5] = broken.offsets[-1] + 7          # not monotone
    IO.write_index(bad, broken)
    with pytest.raises(pqt.PqtError) as e:
        pqt.pqt_index_load(bad, 0)
    assert e.value.code == pqt.PQT_EFORMAT

    gix = pqt.pqt_index_load(path, 0)
    try:
        yq = torch.from_numpy(Y).cuda()
        for k, w in ((0, 2), (cfg.C + 1, 2), (10, 0), (10, cfg.k1 + 1)):
            with pytest.raises(pqt.PqtError) as e:
                pqt.pqt_query_batch(gix, yq, k, w)
            assert e.value.code == pqt.PQT_EINVAL
        with pytest.raises(pqt.PqtError) as e:
            pqt.pqt_set_budget(gix, 0, 10)
        assert e.value.code == pqt.PQT_EINVAL
        with pytest.raises(pqt.PqtError) as e:
            pqt.pqt_set_budget(gix, 10, 1 << 20)
        assert e.value.code == pqt.PQT_EINVAL
        ids, d = pqt.pqt_query_batch(gix, yq, cfg.k, cfg.w)     # still usable after errors
        torch.cuda.synchronize()
        assert ids.shape == (cfg.nq, cfg.k)
    finally:
        pqt.pqt_index_free(gix)


# ---- full size, in the launch configuration bench.py times -------------------------------------------
@pytest.fixture(scope="module")
def sift_full(pqt, tmp_path_factory):
    """SIFT-shaped 1M x 128 database, 10,000 queries, index trained and built by the library
    (pqt_train, pqt_builder_*; the index is input data for both sides; its validity is checked below)."""
    import torch
    from workloads import CONFIGS, sift_like_tables, sift_like_torch
    from paper_1702_05911_amd import builder
    cfg = CONFIGS["sift"]
    tables = sift_like_tables(cfg.D)
    dev = torch.device("cuda", 0)
    X = sift_like_torch(0, cfg.N, d=cfg.D, seed=cfg.data_seed, tables=tables, device=dev)
    Y = sift_like_torch(0, cfg.nq, d=cfg.D, seed=cfg.query_seed, tables=tables, device=dev)
    path = str(tmp_path_factory.mktemp("sift") / "sift.pqt")
    builder.build_index(path, X, P=cfg.P, k1=cfg.k1, k2=cfg.k2, M=cfg.M, H=cfg.H, T=cfg.T, C=cfg.C,
                        train_n=cfg.train_n, device=0, chunk_rows=1 << 18).close()
    return cfg, X.cpu().numpy(), Y.cpu().numpy(), path, IO.read_index(path)


def test_sift_full_size_index_is_valid(sift_full):
    cfg, X, Y, path, ix = sift_full
    off = ix.offsets.astype(np.int64)
    assert off[0] == 0 and off[-1] == cfg.N and np.all(np.diff(off) >= 0)
    assert np.array_equal(np.sort(ix.ids), np.arange(cfg.N, dtype=np.uint32))
    rng = np.random.default_rng(0)
    mism = 0
    for t in rng.integers(0, cfg.N, size=200):
        slot = int(np.searchsorted(off, t, side="right")) - 1
        x = X[ix.ids[t]]
        mism += slot != B.bin_slot(x, ix.C1, ix.C2, ix.H)
        mism += not np.array_equal(ix.codes[t], B.encode_vector(x, ix.C1, ix.M, ix.tbl_i, ix.tbl_j, ix.tbl_lam))
        if t > 0 and np.searchsorted(off, t - 1, side="right") - 1 == slot:
            assert ix.ids[t - 1] < ix.ids[t]
    assert mism <= 4          # the fp32 builder may settle a near-tie differently from float64


def _full_size_check(pqt, gix, ix, cfg, Y, w, order="fullsort", label="sift"):
    """Properties on every query of the batch bench.py times, and the oracle stage by stage on a sample."""
    ids, dists, taps = _run_debug(pqt, gix, Y, cfg.k, w)
    nc = taps["n_cand"].astype(np.int64)
    assert np.all(nc <= cfg.C) and np.all(nc > 0)
    for q in range(cfg.nq):
        n = int(nc[q])
        sc, cid = taps["scores"][q][:n], taps["cand_ids"][q][:n]
        o = np.lexsort((cid, sc))[:cfg.k]
        assert np.array_equal(ids[q][:len(o)], cid[o]), f"query {q}: top-k is not the k smallest (score, id)"
        assert np.array_equal(dists[q][:len(o)], sc[o])
        assert len(set(cid.tolist())) == n
    same = decided = 0
    sample = list(range(0, cfg.nq, 417))
    for q in sample:
        print(f"{label} w={w} query {q}", flush=True)
        tr = PU.check_query_stages(ix, Y[q], taps, q, cfg.k, w, cfg.T, cfg.C, ids, dists, order=order)
        s, d = PU.end_to_end_agreement(tr, ids[q], dists[q])
        assert s or not d, f"query {q}: margins above threshold but ids differ"
        same += s
        decided += d
    print(f"{label} w={w}: {same}/{len(sample)} sampled queries identical to the float64 oracle, {decided} decided")
    assert same >= 0.8 * len(sample)


@pytest.mark.parametrize("w", [8, 1])
def test_sift_full_size_parity(pqt, sift_full, w):
    cfg, X, Y, path, ix = sift_full
    gix = pqt.pqt_index_load(path, 0)
    try:
        _full_size_check(pqt, gix, ix, cfg, Y, w)
    finally:
        pqt.pqt_index_free(gix)


def test_sift_full_size_static_order(pqt, sift_full):
    cfg, X, Y, path, ix = sift_full
    gix = pqt.pqt_index_load(path, 0)
    try:
        pqt.pqt_set_bin_order(gix, pqt.PQT_ORDER_STATIC_SLOPES)
        _full_size_check(pqt, gix, ix, cfg, Y, cfg.w, order="static", label="sift static order")
    finally:
        pqt.pqt_index_free(gix)


def test_sift_full_size_pair_lambda_codes(pqt, sift_full, tmp_path):
    """The same codebooks and database with (pair, lambda) codes from the library's streaming builder."""
    import torch
    cfg, X, Y, path, ix = sift_full
    params = dict(N=cfg.N, H=ix.H, D=ix.D, P=ix.P, k1=ix.k1, k2=ix.k2, M=ix.M, T=ix.T, C=ix.C,
                  C1=ix.C1, C2=ix.C2, cc=ix.cc, code_format=1)
    b = pqt.pqt_builder_create(params, 0)
    try:
        for lo in range(0, cfg.N, 1 << 18):
            pqt.pqt_builder_add(b, torch.from_numpy(X[lo:lo + (1 << 18)]).cuda())
            torch.cuda.synchronize()
        gix = pqt.pqt_builder_finish(b)
    finally:
        pqt.pqt_builder_free(b)
    ppath = str(tmp_path / "sift_pair.pqt")
    try:
        pqt.pqt_index_save(gix, ppath)
        pix = IO.read_index(ppath)
        off = pix.offsets.astype(np.int64)
        assert pix.code_format == 1 and off[0] == 0 and off[-1] == cfg.N and np.all(np.diff(off) >= 0)
        assert np.array_equal(np.sort(pix.ids), np.arange(cfg.N, dtype=np.uint32))
        # the same bins as the index of the other builder, up to fp32 near-ties
        slot_a = np.empty(cfg.N, np.int64)
        slot_a[pix.ids] = np.repeat(np.arange(pix.H), np.diff(off))
        slot_b = np.empty(cfg.N, np.int64)
        slot_b[ix.ids] = np.repeat(np.arange(ix.H), np.diff(ix.offsets.astype(np.int64)))
        assert np.mean(slot_a != slot_b) <= 2e-3
        _full_size_check(pqt, gix, pix, cfg, Y, cfg.w, label="sift pair codes")
    finally:
        pqt.pqt_index_free(gix)


# ---- the parameter shape of the 100M- and 1B-vector workloads -----------------------------------------
@pytest.mark.parametrize("k1", [32, 64])
def test_large_and_billion_parameter_shape(pqt, tmp_path, k1):
    """D = 128, P = 2, k2 = 16, w = 8 (lists of 128 entries), M = 8, T = 1024, C = 10,000, k = 100, with
    k1 = 32 (the 100M workload) and k1 = 64 (the 1B workload: four MFMA column tiles at level 1), on
    16M SIFT-shaped vectors -- enough for the mean run of a bin to be long, so that the re-rank
    wavefronts walk the run lists as they do at full scale.  Index by the library's streaming builder,
    exported to the oracle through the index file.  4,352 queries in one call (more than a tile per compute
    unit: the launch shapes the benchmark times -- traversal of whole tiles, 512-thread re-rank, head pass +
    in-kernel full ranking) checked stage by stage on a sample; the same queries 64 and 1 per call (the
    small-batch launches: traversal split by tree part, 1024 threads) must return the same bits."""
    import torch
    from workloads import sift_like_tables, sift_like_torch
    from paper_1702_05911_amd import builder
    dev = torch.device("cuda", 0)
    N, D, P, k2, M, w, T, C, k, nq = 1 << 24, 128, 2, 16, 8, 8, 1024, 10_000, 100, 4352
    tables = sift_like_tables(D)

    def chunks(s, n):
        return sift_like_torch(s, n, d=D, seed=0, tables=tables, device=dev, chunk=1 << 19)

    print(f"k1={k1}: building {N:,} vectors", flush=True)
    gix = builder.build_index_native(chunks=chunks, N=N, D=D, P=P, k1=k1, k2=k2, M=M, T=T, C=C,
                                     train_n=200_000, iters=8, device=0, chunk_rows=1 << 20, table_train_n=50_000)
    path = str(tmp_path / f"shape_k1_{k1}.pqt")
    try:
        pqt.pqt_index_save(gix, path)
        ix = IO.read_index(path)
        Yd = sift_like_torch(0, nq, d=D, seed=1, tables=tables, device=dev)
        Y = Yd.cpu().numpy()
        print(f"k1={k1}: one call of {nq} queries, debug and plain entry points", flush=True)
        ids, dists, taps = _run_debug(pqt, gix, Y, k, w)
        nr, nc = taps["n_slots"].astype(np.int64), taps["n_cand"].astype(np.int64)
        print(f"k1={k1}: candidates mean {nc.mean():.0f}, runs mean {nr.mean():.1f}, "
              f"queries whose runs average 8 or more: {np.mean(nr * 8 <= nc):.3f}", flush=True)
        assert np.mean(nc == C) > 0.9 and np.mean(nr * 8 <= nc) > 0.5      # the budget is met, long runs are the rule
        same = decided = 0
        sample = list(range(0, nq, 87))                                      # 51 queries
        for q in sample:
            print(f"k1={k1} query {q}", flush=True)
            tr = PU.check_query_stages(ix, Y[q], taps, q, k, w, T, C, ids, dists)
            s_, d_ = PU.end_to_end_agreement(tr, ids[q], dists[q])
            assert s_ or not d_, f"query {q}: margins above threshold but ids differ"
            same += s_
            decided += d_
        print(f"k1={k1}: {same}/{len(sample)} sampled queries identical to the float64 oracle, {decided} decided; "
              + PU.STATS.summary(), flush=True)
        assert same >= 0.8 * len(sample)
        del taps
        # every query of the batch: the top-k is the k smallest (score, id) of its own candidates is covered by
        # the stage-wise sample; here the small-batch launches against the big one, bit for bit
        ids_t, d_t = torch.from_numpy(ids).cuda(), torch.from_numpy(dists).cuda()
        for B, upto in ((64, 512), (1, 48)):
            print(f"k1={k1}: {B} queries per call", flush=True)
            for o in range(0, upto, B):
                bi, bd = pqt.pqt_query_batch(gix, Yd[o:o + B].contiguous(), k, w)
                assert torch.equal(bi, ids_t[o:o + B]) and torch.equal(bd.view(torch.int32), d_t[o:o + B].view(torch.int32)), \
                    f"batch of {B} at {o}"
        # the small-batch launch stage by stage as well
        ids64, d64, taps64 = _run_debug(pqt, gix, Y[100:164], k, w)
        for q in (0, 31, 63):
            PU.check_query_stages(ix, Y[100 + q], taps64, q, k, w, T, C, ids64, d64)
    finally:
        pqt.pqt_index_free(gix)


@pytest.fixture(scope="module")
def gist_full(pqt, tmp_path_factory):
    """GIST-shaped 1M x 960 database, 1,000 queries, P = 4 with H = K = 2^28 bin slots (the pointer
    array alone is 1 GiB, so its probes are real HBM accesses); index trained and built by the library."""
    import torch
    from workloads import CONFIGS, gist_like_torch
    from paper_1702_05911_amd import builder
    cfg = CONFIGS["gist"]
    dev = torch.device("cuda", 0)
    X = gist_like_torch(0, cfg.N, d=cfg.D, seed=cfg.data_seed, device=dev)
    Y = gist_like_torch(0, cfg.nq, d=cfg.D, seed=cfg.query_seed + 100, device=dev)
    path = str(tmp_path_factory.mktemp("gist") / "gist.pqt")
    builder.build_index(path, X, P=cfg.P, k1=cfg.k1, k2=cfg.k2, M=cfg.M, H=cfg.H, T=cfg.T, C=cfg.C,
                        train_n=cfg.train_n, device=0, chunk_rows=1 << 18).close()
    Xh, Yh = X.cpu().numpy(), Y.cpu().numpy()
    del X, Y
    torch.cuda.empty_cache()
    return cfg, Xh, Yh, path, IO.read_index(path)


def test_gist_full_size_parity(pqt, gist_full):
    cfg, X, Y, path, ix = gist_full
    off = ix.offsets.astype(np.int64)
    assert off[0] == 0 and off[-1] == cfg.N and ix.H == cfg.K
    rng = np.random.default_rng(0)
    mism = 0
    for t in rng.integers(0, cfg.N, size=40):
        slot = int(np.searchsorted(off, t, side="right")) - 1
        mism += slot != B.bin_slot(X[ix.ids[t]], ix.C1, ix.C2, ix.H)
    assert mism <= 2          # the fp32 builder may settle a near-tie differently from float64
    gix = pqt.pqt_index_load(path, 0)
    try:
        ids, dists, taps = _run_debug(pqt, gix, Y, cfg.k, cfg.w)
    finally:
        pqt.pqt_index_free(gix)
    nc = taps["n_cand"].astype(np.int64)
    assert np.all(nc <= cfg.C)
    print(f"gist: candidates per query mean {nc.mean():.1f} min {nc.min()} max {nc.max()}", flush=True)
    for q in range(cfg.nq):
        n = int(nc[q])
        sc, cid = taps["scores"][q][:n], taps["cand_ids"][q][:n]
        o = np.lexsort((cid, sc))[:cfg.k]
        assert np.array_equal(ids[q][:len(o)], cid[o]), f"query {q}: top-k is not the k smallest (score, id)"
        assert np.all(ids[q][len(o):] == -1)
    same = decided = 0
    sample = list(range(0, cfg.nq, 97))
    for q in sample:
        print(f"gist query {q}", flush=True)
        tr = PU.check_query_stages(ix, Y[q], taps, q, cfg.k, cfg.w, cfg.T, cfg.C, ids, dists)
        s, d = PU.end_to_end_agreement(tr, ids[q], dists[q])
        assert s or not d, f"query {q}: margins above threshold but ids differ"
        same += s
        decided += d
    print(f"gist: {same}/{len(sample)} sampled queries identical to the float64 oracle, {decided} decided")
    assert same >= 0.7 * len(sample)
