"""Oracle: a plain offline builder for the Product Quantization Tree index.

TEST INFRASTRUCTURE.  Float64 NumPy, direct squared differences, plain loops;
meant for the small indexes the parity tests use.  It follows Sec. 3.1
("Tree structure - offline phase"), Sec. 3.3 ("Offline computation") and the
data layout of Sec. 4 (sorted id array + pointer array from a histogram and a
prefix sum, modulo hashing of bin numbers).

The functions `leaf_of`, `bin_slot`, `line_projection`, `encode_vector` and
`pair_table` are the *definitions* an index must satisfy; the tests apply them
to indexes produced by any builder.
"""
import numpy as np

from .pqt_query import PQTIndex, linear_bin


# ---------------------------------------------------------------------------
# vector quantiser training (Sec. 2.1: Lloyd iterations; Sec. 3.1 "Training the codebook")
# ---------------------------------------------------------------------------
def sqdist_matrix(X, Cen):
    """|X| x |Cen| squared distances by direct differences."""
    X = np.asarray(X, dtype=np.float64)
    Cen = np.asarray(Cen, dtype=np.float64)
    out = np.empty((X.shape[0], Cen.shape[0]), dtype=np.float64)
    for c in range(Cen.shape[0]):
        diff = X - Cen[c][None, :]
        out[:, c] = np.sum(diff * diff, axis=1)
    return out


def lloyd(X, k, iters=20):
    """k centroids for the rows of X.  Deterministic: the start centroids are k rows at
    evenly spaced indices; an empty cell is re-seeded with the row farthest from its
    centroid.  With fewer than k rows the remaining centroids repeat the mean."""
    X = np.asarray(X, dtype=np.float64)
    n = X.shape[0]
    if n == 0:
        return np.zeros((k, X.shape[1]))
    if n <= k:
        cen = np.repeat(X.mean(axis=0, keepdims=True), k, axis=0)
        cen[:n] = X
        return cen
    cen = X[(np.arange(k) * n) // k].copy()
    for _ in range(iters):
        d = sqdist_matrix(X, cen)
        lab = np.argmin(d, axis=1)
        dmin = d[np.arange(n), lab]
        for c in range(k):
            members = lab == c
            if members.any():
                cen[c] = X[members].mean(axis=0)
            else:
                far = int(np.argmax(dmin))
                cen[c] = X[far]
                dmin[far] = 0.0
    return cen


def train_tree(Xtrain, P, k1, k2, iters=20):
    """Level-1 product quantiser (k1 centroids per part) and, independently for each of its
    cells, a k2-centroid quantiser of the sub-vectors that fall in the cell (Sec. 3.1)."""
    n, D = Xtrain.shape
    dp = D // P
    C1 = np.zeros((P, k1, dp))
    C2 = np.zeros((P, k1, k2, dp))
    for p in range(P):
        Xp = np.asarray(Xtrain[:, p * dp:(p + 1) * dp], dtype=np.float64)
        C1[p] = lloyd(Xp, k1, iters)
        lab = np.argmin(sqdist_matrix(Xp, C1[p]), axis=1)
        for i in range(k1):
            sub = Xp[lab == i]
            C2[p, i] = lloyd(sub, k2, iters) if sub.shape[0] > 0 else np.repeat(C1[p, i][None], k2, axis=0)
    return C1.astype(np.float32), C2.astype(np.float32)


# ---------------------------------------------------------------------------
# the bin map m(x) (Sec. 3.1) and its hashed slot (Sec. 4)
# ---------------------------------------------------------------------------
def leaf_of(x, C1, C2):
    """Per part: nearest level-1 centroid i, then the nearest of ITS k2 children j;
    leaf id i*k2 + j.  Ties go to the smaller index."""
    P, k1, k2, dp = C2.shape
    x = np.asarray(x, dtype=np.float64)
    leaf = []
    for p in range(P):
        xp = x[p * dp:(p + 1) * dp]
        i = int(np.argmin(sqdist_matrix(xp[None], C1[p])[0]))
        j = int(np.argmin(sqdist_matrix(xp[None], C2[p, i])[0]))
        leaf.append(i * k2 + j)
    return leaf


def bin_slot(x, C1, C2, H):
    k1, k2 = C2.shape[1], C2.shape[2]
    return linear_bin(leaf_of(x, C1, C2), k1 * k2) % H


def bin_slots_batch(X, C1, C2, H):
    """bin_slot for every row of X (same arithmetic, vectorised over rows)."""
    P, k1, k2, dp = C2.shape
    n = X.shape[0]
    lin = np.zeros(n, dtype=object)
    for p in range(P):
        Xp = np.asarray(X[:, p * dp:(p + 1) * dp], dtype=np.float64)
        i = np.argmin(sqdist_matrix(Xp, C1[p]), axis=1)
        j = np.zeros(n, dtype=np.int64)
        for c in range(k1):
            rows = np.nonzero(i == c)[0]
            if rows.size:
                j[rows] = np.argmin(sqdist_matrix(Xp[rows], C2[p, c]), axis=1)
        leaf = i * k2 + j
        lin = lin * (k1 * k2) + leaf.astype(object)
    return np.array([int(v) % H for v in lin], dtype=np.int64)


def inverted_lists(slots, H):
    """Sorted id array + pointer array (Sec. 4): histogram of the slots, prefix sum, ids
    ordered by (slot, id)."""
    order = np.argsort(slots, kind="stable")
    hist = np.bincount(slots, minlength=H)
    offsets = np.zeros(H + 1, dtype=np.int64)
    offsets[1:] = np.cumsum(hist)
    return offsets, order.astype(np.int64)


# ---------------------------------------------------------------------------
# line quantisation (Sec. 3.3 "Offline computation", Eq. 7)
# ---------------------------------------------------------------------------
def pair_table(C1, M):
    """cc[m][s][t] = || [c_s]_m - [c_t]_m ||^2 for every sub-part and centroid pair (Sec. 3.3)."""
    P, k1, dp = C1.shape
    ds = (P * dp) // M
    cc = np.zeros((M, k1, k1), dtype=np.float64)
    for m in range(M):
        p = (m * ds) // dp
        lo = m * ds - p * dp
        cen = C1[p, :, lo:lo + ds].astype(np.float64)
        cc[m] = sqdist_matrix(cen, cen)
    return cc


def subpart_centroids(C1, M, m):
    P, k1, dp = C1.shape
    ds = (P * dp) // M
    p = (m * ds) // dp
    lo = m * ds - p * dp
    return C1[p, :, lo:lo + ds].astype(np.float64)


def line_projection(xs, ci, cj):
    """Orthogonal projection of xs onto the line through ci and cj: the lambda with
    projection (1-lambda) ci + lambda cj, and the squared projection error delta."""
    u = cj - ci
    uu = float(np.dot(u, u))
    if uu == 0.0:
        lam = 0.0
    else:
        lam = float(np.dot(xs - ci, u)) / uu
    r = xs - ((1.0 - lam) * ci + lam * cj)
    return lam, float(np.dot(r, r))


def best_lines(Xs, cen):
    """For every row of Xs the centroid pair (i<j) whose line is nearest, its lambda and
    error (ties: first pair in (i, j) lexicographic order)."""
    n = Xs.shape[0]
    k1 = cen.shape[0]
    best_err = np.full(n, np.inf)
    best_pair = np.zeros(n, dtype=np.int64)
    best_lam = np.zeros(n)
    pid = 0
    for i in range(k1):
        for j in range(i + 1, k1):
            u = cen[j] - cen[i]
            uu = float(np.dot(u, u))
            if uu > 0.0:
                lam = ((Xs - cen[i][None]) @ u) / uu
                proj = (1.0 - lam)[:, None] * cen[i][None] + lam[:, None] * cen[j][None]
                r = Xs - proj
                err = np.sum(r * r, axis=1)
                better = err < best_err
                best_err[better] = err[better]
                best_pair[better] = pid
                best_lam[better] = lam[better]
            pid += 1
    return best_pair, best_lam, best_err


def line_codebook(Xs, cen, n_codes=256):
    """256 (i, j, lambda) code points for one sub-part: centroid pairs get code points in
    proportion to how often their line is the nearest one for the training sub-vectors
    (largest-remainder rounding), placed at the quantiles of the lambdas observed on
    that line.  Entries are ordered by (i, j, lambda)."""
    k1 = cen.shape[0]
    pairs = [(i, j) for i in range(k1) for j in range(i + 1, k1)]
    ti = np.zeros(n_codes, dtype=np.uint8)
    tj = np.zeros(n_codes, dtype=np.uint8)
    tl = np.zeros(n_codes, dtype=np.float32)
    if not pairs or Xs.shape[0] == 0:
        return ti, tj, tl
    bp, bl, _ = best_lines(Xs, cen)
    use = np.bincount(bp, minlength=len(pairs)).astype(np.float64)
    quota = use * n_codes / use.sum()
    alloc = np.floor(quota).astype(np.int64)
    rem = quota - alloc
    for q in np.lexsort((np.arange(len(pairs)), -rem))[: n_codes - int(alloc.sum())]:
        alloc[q] += 1
    entries = []
    for q, (i, j) in enumerate(pairs):
        if alloc[q] == 0:
            continue
        lams = np.sort(bl[bp == q])
        for t in range(alloc[q]):
            pos = min(int((t + 0.5) / alloc[q] * lams.shape[0]), lams.shape[0] - 1)
            entries.append((i, j, np.float32(lams[pos])))
    entries.sort(key=lambda e: (e[0], e[1], float(e[2])))
    for c, (i, j, lam) in enumerate(entries[:n_codes]):
        ti[c], tj[c], tl[c] = i, j, lam
    for c in range(len(entries), n_codes):          # fewer samples than codes: repeat the last
        ti[c], tj[c], tl[c] = ti[len(entries) - 1], tj[len(entries) - 1], tl[len(entries) - 1]
    return ti, tj, tl


def code_points(cen, ti, tj, tl):
    """The 256 points (1-lam) c_i + lam c_j of one sub-part."""
    lam = tl.astype(np.float64)[:, None]
    return (1.0 - lam) * cen[ti.astype(np.int64)] + lam * cen[tj.astype(np.int64)]


def encode_vector(x, C1, M, tbl_i, tbl_j, tbl_lam):
    """Code byte per sub-part = index of the nearest code point (ties: smaller index)."""
    ds = x.shape[0] // M
    code = np.zeros(M, dtype=np.uint8)
    for m in range(M):
        pts = code_points(subpart_centroids(C1, M, m), tbl_i[m], tbl_j[m], tbl_lam[m])
        code[m] = np.argmin(sqdist_matrix(np.asarray(x[m * ds:(m + 1) * ds], dtype=np.float64)[None], pts)[0])
    return code


def encode_batch(X, C1, M, tbl_i, tbl_j, tbl_lam):
    n, D = X.shape
    ds = D // M
    codes = np.zeros((n, M), dtype=np.uint8)
    for m in range(M):
        pts = code_points(subpart_centroids(C1, M, m), tbl_i[m], tbl_j[m], tbl_lam[m])
        codes[:, m] = np.argmin(sqdist_matrix(X[:, m * ds:(m + 1) * ds], pts), axis=1)
    return codes


def encode_pair_lambda(X, C1, M):
    """Code format 1 (Eq. 7 stored directly, Sec. 3.3 "Offline computation").  A (pair, level) code
    stands for the point (1-lam) c_i + lam c_j with lam on the level grid, and a sub-vector gets the
    code of the NEAREST such point (ties: smaller pair number).  On one line the
    error is quadratic in lam, so its nearest grid point is the level nearest to the projection's
    lambda (halves go up; clamped to a byte); the pairs are then compared by the error of that point.  (Choosing the
    line by its unclamped projection error instead often picks a line whose projection lies far
    outside what a byte of lambda can express.)  Two bytes per sub-part."""
    from .pqt_query import lambda_of_level, level_of_lambda
    n, D = X.shape
    ds = D // M
    k1 = C1.shape[1]
    codes = np.zeros((n, 2 * M), dtype=np.uint8)
    for m in range(M):
        cen = subpart_centroids(C1, M, m)
        Xs = np.asarray(X[:, m * ds:(m + 1) * ds], dtype=np.float64)
        best_err = np.full(n, np.inf)
        codes[:, 2 * m + 1] = level_of_lambda(0.0)        # no usable pair: pair 0 at lambda = 0
        pid = 0
        for i in range(k1):
            for j in range(i + 1, k1):
                u = cen[j] - cen[i]
                uu = float(np.dot(u, u))
                if uu > 0.0:
                    level = level_of_lambda(((Xs - cen[i][None]) @ u) / uu)
                    lam = lambda_of_level(level)
                    r = Xs - ((1.0 - lam)[:, None] * cen[i][None] + lam[:, None] * cen[j][None])
                    err = np.sum(r * r, axis=1)
                    better = err < best_err
                    best_err[better] = err[better]
                    codes[better, 2 * m] = pid
                    codes[better, 2 * m + 1] = level[better]
                pid += 1
    return codes


# ---------------------------------------------------------------------------
# the whole build
# ---------------------------------------------------------------------------
def build_index(X, P, k1, k2, M, H=None, T=1024, C=4096, train_n=None, iters=20,
                codebooks=None, line_table=None, code_format=0):
    """Train (or take) the tree, sort X into bins, build the inverted lists, the line
    code table and the codes.  `codebooks=(C1, C2)` and `line_table=(tbl_i, tbl_j, tbl_lam)`
    let a test supply hand-made ones.  code_format 1 stores (pair, lambda level) per sub-part
    instead of an entry of the line table (which is then left at zeros)."""
    N, D = X.shape
    assert D % P == 0 and D % M == 0 and M % P == 0 and k1 <= 256
    K = (k1 * k2) ** P
    H = K if H is None else H
    Xt = X[: (train_n or N)]
    if codebooks is None:
        C1, C2 = train_tree(Xt, P, k1, k2, iters)
    else:
        C1, C2 = (np.asarray(c, dtype=np.float32) for c in codebooks)
    if code_format == 1:
        assert 2 <= k1 and k1 * (k1 - 1) // 2 <= 256
        ti, tj, tl = np.zeros((M, 256), np.uint8), np.zeros((M, 256), np.uint8), np.zeros((M, 256), np.float32)
    elif line_table is None:
        ds = D // M
        ti = np.zeros((M, 256), np.uint8)
        tj = np.zeros((M, 256), np.uint8)
        tl = np.zeros((M, 256), np.float32)
        for m in range(M):
            ti[m], tj[m], tl[m] = line_codebook(
                np.asarray(Xt[:, m * ds:(m + 1) * ds], dtype=np.float64), subpart_centroids(C1, M, m))
    else:
        ti, tj, tl = line_table
        ti, tj, tl = np.asarray(ti, np.uint8), np.asarray(tj, np.uint8), np.asarray(tl, np.float32)
    slots = bin_slots_batch(X, C1, C2, H)
    offsets, order = inverted_lists(slots, H)
    codes = (encode_pair_lambda(X, C1, M) if code_format == 1 else encode_batch(X, C1, M, ti, tj, tl))[order]
    return PQTIndex(D=D, P=P, k1=k1, k2=k2, M=M, N=N, H=H, T=T, C=C, C1=C1, C2=C2,
                    tbl_i=ti, tbl_j=tj, tbl_lam=tl, cc=pair_table(C1, M).astype(np.float32),
                    offsets=offsets.astype(np.uint32), ids=order.astype(np.uint32),
                    codes=np.ascontiguousarray(codes), code_format=code_format)
