"""Oracle: the online (query) phase of the Product Quantization Tree.

TEST INFRASTRUCTURE.  Plain float64 NumPy/Python; no blocking, no fusion, no
code shared with the HIP path.  Each function follows one step of Sec. 3.2
("Query - online phase": tree traversal, bin proposal, vector proposal,
re-ranking) or Sec. 3.3 ("Online computation", Eq. 8-9) of the paper.

All distances are squared Euclidean distances (Sec. 1 defines d(.) := ||.||^2).

Readings of the paper taken here (each is listed in the design notes):
  * bins are ranked by the actual sum of their per-part level-2 distances -- the
    order the paper calls optimal (the priority-queue order of [4], Sec. 3.2
    "Bin Proposal Heuristic") and the one it re-sorts by on SIFT1B (Sec. 5.1);
    for P=4 the order is built pairwise: parts (1,2), parts (3,4), then the two
    pair lists;
  * every sort is on (value, id) ascending, smaller id first;
  * level-2 codebooks are quantisers of the sub-vectors themselves (not residuals);
  * a re-rank code byte names one of 256 points (1-lambda)*c_i + lambda*c_j on
    lines through level-1 centroids of that sub-part (Sec. 3.3, Eq. 7);
  * in Eq. 9, b^2 = ||y - c_i||^2 (the lambda=0 end), a^2 = ||y - c_j||^2 (the
    lambda=1 end), c^2 = ||c_i - c_j||^2.
"""
import heapq
from dataclasses import dataclass, field

import numpy as np


@dataclass
class PQTIndex:
    """Read-only index arrays (Sec. 3.1, Sec. 4).  Float arrays are stored fp32."""
    D: int
    P: int
    k1: int
    k2: int
    M: int
    N: int
    H: int
    T: int                     # default number of bin tuples examined
    C: int                     # default candidate budget
    C1: np.ndarray             # (P, k1, D/P)       level-1 centroids per part
    C2: np.ndarray             # (P, k1, k2, D/P)   level-2 centroids, children of each level-1 cell
    tbl_i: np.ndarray          # (M, 256) uint8     line end at lambda = 0
    tbl_j: np.ndarray          # (M, 256) uint8     line end at lambda = 1
    tbl_lam: np.ndarray        # (M, 256) float32   lambda
    cc: np.ndarray             # (M, k1, k1) float32  ||[c_s]_m - [c_t]_m||^2   (Sec. 3.3)
    offsets: np.ndarray        # (H+1,)  start of every bin slot in ids/codes    (Sec. 4)
    ids: np.ndarray            # (N,) uint32, ascending inside a slot
    codes: np.ndarray          # (N, M) uint8, row t belongs to ids[t]; (N, 2M) for code_format 1
    code_format: int = 0       # 0: one byte per sub-part = entry of the (i, j, lambda) table
                               # 1: two bytes per sub-part = (centroid pair, lambda level), Eq. 7 stored directly

    @property
    def dp(self):
        return self.D // self.P

    @property
    def ds(self):
        return self.D // self.M

    @property
    def K(self):
        return (self.k1 * self.k2) ** self.P


# ---------------------------------------------------------------------------
# O1  level-1 distances per sub-part and per part            (Sec. 3.2, Eq. 6; Sec. 3.3 end)
# ---------------------------------------------------------------------------
def level1_subpart_distances(y, C1, M):
    """a[m][i] = || [y]_m - [c1_i]_m ||^2 for every re-rank sub-part m and level-1 centroid i.
    The tree part p is split into M/P equal contiguous sub-parts (Sec. 3.3, last paragraph)."""
    P, k1, dp = C1.shape
    D = P * dp
    ds = D // M
    y = np.asarray(y, dtype=np.float64)
    a = np.zeros((M, k1), dtype=np.float64)
    for m in range(M):
        p = (m * ds) // dp
        lo = m * ds - p * dp
        for i in range(k1):
            diff = y[m * ds:(m + 1) * ds] - C1[p, i, lo:lo + ds].astype(np.float64)
            a[m, i] = np.sum(diff * diff)
    return a


def part_distances(a, P):
    """d1[p][i] = sum over the sub-parts m of part p of a[m][i], added in ascending m,
    in the dtype of `a` (the "aggregating the components" of Sec. 3.3)."""
    M, k1 = a.shape
    per = M // P
    d1 = np.zeros((P, k1), dtype=a.dtype)
    for p in range(P):
        acc = a[p * per].copy()
        for m in range(p * per + 1, (p + 1) * per):
            acc = acc + a[m]
        d1[p] = acc
    return d1


# ---------------------------------------------------------------------------
# O2  keep the w closest level-1 clusters per part                       (Sec. 3.2)
# ---------------------------------------------------------------------------
def order_by_value_then_id(values, ids=None):
    """Indices that sort (value, id) ascending; smaller id first among equal values."""
    values = np.asarray(values)
    if ids is None:
        ids = np.arange(values.shape[0])
    return np.lexsort((np.asarray(ids), values))


def select_clusters(d1, w):
    """sel[p] = ids of the w level-1 centroids closest to [y]_p, closest first."""
    P, k1 = d1.shape
    sel = np.zeros((P, w), dtype=np.int64)
    for p in range(P):
        sel[p] = order_by_value_then_id(d1[p])[:w]
    return sel


# ---------------------------------------------------------------------------
# O3  level-2 refinement inside the selected clusters                    (Sec. 3.2)
# ---------------------------------------------------------------------------
def level2_distances(y, C2, sel):
    """For every part p, selected cluster i and child j: id = i*k2 + j and
    d2 = || [y]_p - c2[p][i][j] ||^2.  Returns (d2, id) arrays of shape (P, w*k2),
    in selection order (not yet sorted)."""
    P, k1, k2, dp = C2.shape
    w = sel.shape[1]
    y = np.asarray(y, dtype=np.float64)
    d2 = np.zeros((P, w * k2), dtype=np.float64)
    ids = np.zeros((P, w * k2), dtype=np.int64)
    for p in range(P):
        yp = y[p * dp:(p + 1) * dp]
        for s in range(w):
            i = int(sel[p, s])
            for j in range(k2):
                diff = yp - C2[p, i, j].astype(np.float64)
                d2[p, s * k2 + j] = np.sum(diff * diff)
                ids[p, s * k2 + j] = i * k2 + j
    return d2, ids


def sort_level2(d2, ids):
    """Per part, sort the (d2, id) pairs ascending -> the ordered lists L_p of Sec. 3.2."""
    Ld = np.empty_like(d2)
    Lid = np.empty_like(ids)
    for p in range(d2.shape[0]):
        o = order_by_value_then_id(d2[p], ids[p])
        Ld[p] = d2[p][o]
        Lid[p] = ids[p][o]
    return Ld, Lid


# ---------------------------------------------------------------------------
# O4  bin order over rank tuples                                (Sec. 2.3, Sec. 3.2)
# ---------------------------------------------------------------------------
def _merge_fullsort(A, B, limit):
    """All (a, b) rank pairs of two ascending lists ordered by (A[a]+B[b], a, b); first `limit`.
    The sum is rounded in the dtype of the inputs.  Returns (sums, a_idx, b_idx)."""
    s = A[:, None] + B[None, :]
    ai, bi = np.meshgrid(np.arange(A.shape[0]), np.arange(B.shape[0]), indexing="ij")
    s, ai, bi = s.ravel(), ai.ravel(), bi.ravel()
    o = np.lexsort((bi, ai, s))[:limit]
    return s[o], ai[o], bi[o]


def _merge_priority_queue(A, B, limit):
    """Same order produced by the multi-sequence walk of [4] (Sec. 2.3): a heap holds the
    frontier; popping (a, b) pushes (a+1, b) and (a, b+1) once their other predecessor
    has been popped."""
    na, nb = A.shape[0], B.shape[0]
    out_s, out_a, out_b = [], [], []
    if na == 0 or nb == 0:
        return np.zeros(0, A.dtype), np.zeros(0, np.int64), np.zeros(0, np.int64)
    done = set()
    heap = [(A[0] + B[0], 0, 0)]
    while heap and len(out_s) < limit:
        s, a, b = heapq.heappop(heap)
        done.add((a, b))
        out_s.append(s)
        out_a.append(a)
        out_b.append(b)
        if a + 1 < na and (b == 0 or (a + 1, b - 1) in done):
            heapq.heappush(heap, (A[a + 1] + B[b], a + 1, b))
        if b + 1 < nb and (a == 0 or (a - 1, b + 1) in done):
            heapq.heappush(heap, (A[a] + B[b + 1], a, b + 1))
    return np.array(out_s, dtype=A.dtype), np.array(out_a, dtype=np.int64), np.array(out_b, dtype=np.int64)


def bin_order(Ld, T, method="fullsort", truncate_pairs=False):
    """The first T rank tuples (r_1..r_P) in the bin order, as an int array (T', P),
    together with their keys.

    P=1: ranks in list order.  P=2: by (L_1[r_1]+L_2[r_2], r_1, r_2).  P=4: rank the pairs
    of parts (1,2) and of parts (3,4) that way, then rank pairs of *positions* in those two
    lists by (s12+s34, pos12, pos34).  With truncate_pairs the two pair lists are cut to
    their first T entries before the final merge (a tuple whose pair position is >= T is
    preceded by at least T tuples, so the result must not change)."""
    merge = {"fullsort": _merge_fullsort, "pq": _merge_priority_queue}[method]
    P = len(Ld)
    if P == 1:
        n = min(T, Ld[0].shape[0])
        return np.arange(n, dtype=np.int64)[:, None], Ld[0][:n].copy()
    if P == 2:
        s, a, b = merge(Ld[0], Ld[1], T)
        return np.stack([a, b], axis=1), s
    if P == 4:
        lim12 = T if truncate_pairs else Ld[0].shape[0] * Ld[1].shape[0]
        lim34 = T if truncate_pairs else Ld[2].shape[0] * Ld[3].shape[0]
        s12, a1, a2 = merge(Ld[0], Ld[1], lim12)
        s34, a3, a4 = merge(Ld[2], Ld[3], lim34)
        s, u, v = merge(s12, s34, T)
        return np.stack([a1[u], a2[u], a3[v], a4[v]], axis=1), s
    raise ValueError("bin order is defined for P in {1, 2, 4}")


# ---------------------------------------------------------------------------
# O4'  the fixed anisotropic traversal order                    (Sec. 3.2 "Bin Proposal Heuristic")
# ---------------------------------------------------------------------------
# The paper replaces the priority-queue order by pre-computed orders of the rank pairs for ten
# slopes 1.08^k, k = -5..4, one of which is used per query.  It prints neither the weighted norm nor
# the rule that picks the slope; the readings below are this build's:
#   * order for slope s: rank pairs v = (v1, v2), counted from 1, ascending by v1^2 + (s v2)^2 --
#     s = 1 is the isotropic order by ||v||_2, a smaller s admits higher ranks in the second part
#     as the paper describes for 1.08^-5 -- ties by (v1, v2);
#   * slope of a query: how far each sorted level-2 list has risen by a reference rank,
#     g_p = L_p[r0] - L_p[0] with r0 = min(R - 1, 8); the list that rises more slowly should be
#     advanced faster, so the slope nearest to g_2 / g_1 in the geometric sense is taken:
#     index = number of j in 1..9 with g_2 > 1.08^(j - 5.5) g_1, compared in the lists' own precision.
N_SLOPES = 10
SLOPE_REFERENCE_RANK = 8


def slopes():
    """1.08^(i - 5), i = 0..9, by repeated multiplication / division (no pow)."""
    up, down = [1.0], [1.0]
    for _ in range(4):
        up.append(up[-1] * 1.08)
    for _ in range(5):
        down.append(down[-1] / 1.08)
    return np.array(down[:0:-1] + up, dtype=np.float64)


def slope_thresholds(dtype=np.float32):
    """1.08^(j - 5.5), j = 1..9: the boundaries between neighbouring slopes."""
    return (slopes()[1:] / np.sqrt(1.08)).astype(dtype)


def choose_slope(L1, L2):
    """Index 0..9 of the slope for one query; arithmetic in the dtype of the lists."""
    dt = L1.dtype.type
    r0 = min(L1.shape[0] - 1, SLOPE_REFERENCE_RANK)
    g1, g2 = dt(L1[r0] - L1[0]), dt(L2[r0] - L2[0])
    return int(sum(1 for t in slope_thresholds(L1.dtype) if g2 > dt(t * g1)))


def static_order(R, T, slope):
    """First min(T, R^2) rank pairs (a, b), counted from 0, ascending by ((a+1)^2 + (slope (b+1))^2, a, b)."""
    a, b = np.meshgrid(np.arange(R), np.arange(R), indexing="ij")
    a, b = a.ravel(), b.ravel()
    key = (a + 1.0) ** 2 + (slope * (b + 1.0)) ** 2
    o = np.lexsort((b, a, key))[:T]
    return np.stack([a[o], b[o]], axis=1).astype(np.int64)


def bin_order_static(Ld, T):
    """Two tree parts: the rank tuples of the pre-computed order for this query's slope, and the
    summed distances of those tuples (they are not what the order is sorted by)."""
    if len(Ld) != 2:
        raise ValueError("the fixed traversal order is defined here for two tree parts")
    k = choose_slope(Ld[0], Ld[1])
    tup = static_order(Ld[0].shape[0], T, slopes()[k])
    return tup, (Ld[0][tup[:, 0]] + Ld[1][tup[:, 1]])


def linear_bin(leaf_ids, k1k2):
    """Multi-index (Eq. 5) -> one unsigned integer, part 1 most significant."""
    lin = 0
    for g in leaf_ids:
        lin = lin * k1k2 + int(g)
    return lin


def propose_bins(tuples, Lid, k1k2, H, offsets):
    """Walk the rank tuples in order; map each to its slot (linear bin id modulo H, Sec. 4:
    collisions are ignored, i.e. colliding bins share one list); keep a slot the first
    time it appears and only if it is not empty (Sec. 4, "All empty bins are removed")."""
    seen = set()
    slots = []
    for t in range(tuples.shape[0]):
        leaf = [Lid[p][tuples[t, p]] for p in range(tuples.shape[1])]
        slot = linear_bin(leaf, k1k2) % H
        if slot in seen:
            continue
        seen.add(slot)
        if int(offsets[slot + 1]) == int(offsets[slot]):
            continue
        slots.append(slot)
    return np.array(slots, dtype=np.int64)


# ---------------------------------------------------------------------------
# O5  vector proposal                                                      (Sec. 4)
# ---------------------------------------------------------------------------
def gather_candidates(slots, offsets, C):
    """Positions (into ids/codes) of the candidates: the runs of the proposed slots in
    visit order, cut after C entries (Table 1 caption: only the first vectors of the
    proposed bins are used)."""
    pos = []
    for slot in slots:
        lo, hi = int(offsets[slot]), int(offsets[slot + 1])
        take = min(hi - lo, C - len(pos))
        pos.extend(range(lo, lo + take))
        if len(pos) >= C:
            break
    return np.array(pos, dtype=np.int64)


# ---------------------------------------------------------------------------
# O6-O7  re-ranking by line quantisation                       (Sec. 3.3, Eq. 8-9)
# ---------------------------------------------------------------------------
def build_lut(a, tbl_i, tbl_j, tbl_lam, cc):
    """LUT[m][c] = b^2 + lam^2 c^2 + lam (a^2 - b^2 - c^2)   (one summand of Eq. 9)
    with (i, j, lam) = table entry c of sub-part m, b^2 = a[m][i], a^2 = a[m][j] looked up
    in the query's level-1 distances, c^2 = cc[m][i][j].  Nothing is clamped."""
    M = a.shape[0]
    lut = np.zeros((M, tbl_i.shape[1]), dtype=np.float64)
    for m in range(M):
        for c in range(tbl_i.shape[1]):
            i, j = int(tbl_i[m, c]), int(tbl_j[m, c])
            lam = float(tbl_lam[m, c])
            b2, a2, c2 = float(a[m, i]), float(a[m, j]), float(cc[m, i, j])
            lut[m, c] = b2 + lam * lam * c2 + lam * (a2 - b2 - c2)
    return lut


# Code format 1 stores the triple of Eq. 7 itself: one byte numbers the centroid pair i < j in
# lexicographic order, one byte is the level of lambda on a fixed grid.  (The paper gives "1+1 bytes"
# but neither the numbering nor the grid; the grid below has 0 and 1 on it and reaches from six
# segment lengths before c_i to nine beyond c_j: on data like the paper's a third of the projections
# fall outside [-0.5, 1.5] and, with short sub-parts, some beyond [-3, 5]; a step of 1/16 moves a point
# by at most 1/32 of the segment, far below the quantisation error itself.)
LAMBDA_ZERO_LEVEL = 96
LAMBDA_LEVELS_PER_UNIT = 16


def lambda_of_level(level):
    return (np.asarray(level, dtype=np.float64) - LAMBDA_ZERO_LEVEL) / LAMBDA_LEVELS_PER_UNIT


def level_of_lambda(lam):
    """Nearest grid level (halves go up), clamped to a byte."""
    return np.clip(np.floor(np.asarray(lam, dtype=np.float64) * LAMBDA_LEVELS_PER_UNIT + LAMBDA_ZERO_LEVEL + 0.5),
                   0, 255).astype(np.uint8)


def centroid_pairs(k1):
    """(i, j) of pair number 0, 1, ...: all i < j in lexicographic order."""
    return [(i, j) for i in range(k1) for j in range(i + 1, k1)]


def score_pair_lambda(a, cc, codes):
    """Eq. 8-9 on codes of format 1: for every sub-part m, in ascending order, the summand
    b^2 + lam^2 c^2 + lam (a^2 - b^2 - c^2) with (i, j) = pair codes[:, 2m], lam = level codes[:, 2m+1],
    b^2 = a[m][i], a^2 = a[m][j], c^2 = cc[m][i][j]."""
    M, k1 = a.shape
    pairs = np.asarray(centroid_pairs(k1), dtype=np.int64).reshape(-1, 2)
    s = np.zeros(codes.shape[0], dtype=np.float64)
    for m in range(M):
        i, j = pairs[codes[:, 2 * m], 0], pairs[codes[:, 2 * m], 1]
        lam = lambda_of_level(codes[:, 2 * m + 1])
        b2, a2, c2 = a[m, i].astype(np.float64), a[m, j].astype(np.float64), cc[m, i, j].astype(np.float64)
        s = s + (b2 + lam * lam * c2 + lam * (a2 - b2 - c2))
    return s


def score_codes(lut, codes):
    """score(x) = sum over m = 0..M-1, in that order, of LUT[m][code_x[m]]   (Eq. 8-9)."""
    n, M = codes.shape
    s = np.zeros(n, dtype=lut.dtype)
    for m in range(M):
        s = s + lut[m, codes[:, m]]
    return s


# ---------------------------------------------------------------------------
# O8  final ordering
# ---------------------------------------------------------------------------
def top_k(scores, ids, k):
    """The k candidates with the smallest (score, id); padded with id -1, distance +inf."""
    o = order_by_value_then_id(scores, ids)[:k]
    out_ids = np.full(k, -1, dtype=np.int64)
    out_d = np.full(k, np.inf, dtype=np.float64)
    out_ids[:o.shape[0]] = np.asarray(ids)[o]
    out_d[:o.shape[0]] = np.asarray(scores)[o]
    return out_ids, out_d


# ---------------------------------------------------------------------------
# O9  oracle-only modes
# ---------------------------------------------------------------------------
def brute_force(y, X, k):
    """Eq. 1 written out: exact squared distances to every database vector."""
    diff = X.astype(np.float64) - np.asarray(y, dtype=np.float64)[None, :]
    d = np.sum(diff * diff, axis=1)
    return top_k(d, np.arange(X.shape[0]), k)


def exact_rerank_short_list(y, X, short_ids, k):
    """Step (3) of the pipelines in Sec. 1 (PQT_2 of Table 1): the entries of a short list (ids, -1 =
    no entry) are re-ranked by their exact squared distance to y; the k best by (distance, id)."""
    ids = np.asarray([i for i in short_ids if i >= 0], dtype=np.int64)
    diff = X[ids].astype(np.float64) - np.asarray(y, dtype=np.float64)[None, :]
    return top_k(np.sum(diff * diff, axis=1), ids, k)


def reconstruct(index, code):
    """The point a code stands for: per sub-part (1-lam)*[c_i]_m + lam*[c_j]_m  (Sec. 3.3)."""
    x = np.zeros(index.D, dtype=np.float64)
    ds, dp = index.ds, index.dp
    pairs = centroid_pairs(index.k1)
    for m in range(index.M):
        p = (m * ds) // dp
        lo = m * ds - p * dp
        if index.code_format == 1:
            i, j = pairs[int(code[2 * m])]
            lam = float(lambda_of_level(code[2 * m + 1]))
        else:
            c = int(code[m])
            i, j, lam = int(index.tbl_i[m, c]), int(index.tbl_j[m, c]), float(index.tbl_lam[m, c])
        ci = index.C1[p, i, lo:lo + ds].astype(np.float64)
        cj = index.C1[p, j, lo:lo + ds].astype(np.float64)
        x[m * ds:(m + 1) * ds] = (1.0 - lam) * ci + lam * cj
    return x


# ---------------------------------------------------------------------------
# the whole query
# ---------------------------------------------------------------------------
@dataclass
class QueryTrace:
    a: np.ndarray = None
    d1: np.ndarray = None
    sel: np.ndarray = None
    Ld: np.ndarray = None
    Lid: np.ndarray = None
    tuples: np.ndarray = None
    keys: np.ndarray = None
    slots: np.ndarray = None
    cand_pos: np.ndarray = None
    cand_ids: np.ndarray = None
    lut: np.ndarray = None
    scores: np.ndarray = None
    out_ids: np.ndarray = None
    out_dists: np.ndarray = None
    margins: dict = field(default_factory=dict)


def _rel_gap(lo, hi):
    scale = max(abs(float(lo)), abs(float(hi)), 1e-300)
    return (float(hi) - float(lo)) / scale


def query(index, y, k, w, T=None, C=None, X=None, exact_rerank=False, order_method="fullsort",
          with_margins=True, truncate_pairs=False):
    # order_method "static": the fixed anisotropic order of O4' instead of the order by summed distance
    # truncate_pairs: bin_order's option (four parts: the pair lists cut at T before the final merge, the
    # same order by construction; lists of 128 are out of reach of the full form)
    """One query through O1..O8.  With exact_rerank (needs the raw vectors X) the scores
    of O6-O7 are replaced by exact squared distances (step (3) of the PQ pipelines in
    Sec. 1; the paper's PQT_2 of Table 1)."""
    T = index.T if T is None else T
    C = index.C if C is None else C
    tr = QueryTrace()
    tr.a = level1_subpart_distances(y, index.C1, index.M)
    tr.d1 = part_distances(tr.a, index.P)
    tr.sel = select_clusters(tr.d1, w)
    d2, ids2 = level2_distances(y, index.C2, tr.sel)
    tr.Ld, tr.Lid = sort_level2(d2, ids2)
    if order_method == "static":
        tr.tuples, tr.keys = bin_order_static([tr.Ld[p] for p in range(index.P)], T)
        with_margins = False           # the margins describe decisions of the order by summed distance
    else:
        tr.tuples, tr.keys = bin_order([tr.Ld[p] for p in range(index.P)], T, method=order_method,
                                       truncate_pairs=truncate_pairs)
    tr.slots = propose_bins(tr.tuples, tr.Lid, index.k1 * index.k2, index.H, index.offsets)
    tr.cand_pos = gather_candidates(tr.slots, index.offsets, C)
    tr.cand_ids = index.ids[tr.cand_pos].astype(np.int64)
    if exact_rerank:
        diff = X[tr.cand_ids].astype(np.float64) - np.asarray(y, dtype=np.float64)[None, :]
        tr.scores = np.sum(diff * diff, axis=1)
    elif index.code_format == 1:
        tr.scores = score_pair_lambda(tr.a, index.cc, index.codes[tr.cand_pos])
    else:
        tr.lut = build_lut(tr.a, index.tbl_i, index.tbl_j, index.tbl_lam, index.cc.astype(np.float64))
        tr.scores = score_codes(tr.lut, index.codes[tr.cand_pos])
    tr.out_ids, tr.out_dists = top_k(tr.scores, tr.cand_ids, k)
    if with_margins:
        tr.margins = decision_margins(index, tr, k, w, T, C, truncate_pairs=truncate_pairs)
    return tr


def decision_margins(index, tr, k, w, T, C, truncate_pairs=False):
    """Relative gaps at the decisions that can change the *set* of returned ids or their
    order: the w-th vs (w+1)-th level-1 distance per part, the last examined vs first
    unexamined bin key, the keys around the run that the candidate budget cuts, and the
    adjacent scores among the first k+1 re-ranked candidates that have different codes."""
    m = {}
    g = np.inf
    if w < index.k1:
        for p in range(index.P):
            s = np.sort(tr.d1[p])
            g = min(g, _rel_gap(s[w - 1], s[w]))
    m["select"] = g
    # T boundary: recompute one more key
    g = np.inf
    total = 1
    for p in range(index.P):
        total *= tr.Ld.shape[1]
    if T < total:
        _, keys = bin_order([tr.Ld[p] for p in range(index.P)], T + 1, truncate_pairs=truncate_pairs)
        g = _rel_gap(keys[T - 1], keys[T])
    m["tuples"] = g
    # C boundary: keys of the emitted slots around the truncated run
    g = np.inf
    lens = (index.offsets[tr.slots + 1].astype(np.int64) - index.offsets[tr.slots].astype(np.int64)) \
        if tr.slots.size else np.zeros(0, np.int64)
    if lens.sum() > C:
        # key of every emitted slot = key of the first tuple that proposed it
        first_key = {}
        for t in range(tr.tuples.shape[0]):
            leaf = [tr.Lid[p][tr.tuples[t, p]] for p in range(index.P)]
            s = linear_bin(leaf, index.k1 * index.k2) % index.H
            first_key.setdefault(s, tr.keys[t])
        ek = np.array([first_key[s] for s in tr.slots])
        e = int(np.searchsorted(np.cumsum(lens), C, side="left"))
        if e > 0:
            g = min(g, _rel_gap(ek[e - 1], ek[e]))
        if e + 1 < ek.shape[0]:
            g = min(g, _rel_gap(ek[e], ek[e + 1]))
    m["budget"] = g
    g = np.inf
    o = order_by_value_then_id(tr.scores, tr.cand_ids)[:k + 1]
    for t in range(len(o) - 1):
        if tr.scores[o[t]] != tr.scores[o[t + 1]]:
            g = min(g, _rel_gap(tr.scores[o[t]], tr.scores[o[t + 1]]))
    m["topk"] = g
    m["min"] = min(m.values())
    return m
