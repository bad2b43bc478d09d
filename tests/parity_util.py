"""Stage-by-stage comparison of the HIP path (through the C ABI's debug taps) with the oracle.

Float stages (level-1 distances, level-2 distances, LUT, scores, output distances) are
compared within a tolerance.  Discrete stages are replayed: the oracle's selection /
sorting / bin ordering / gathering / top-k logic is run ON THE GPU'S OWN fp32 VALUES (in
fp32, the kernel's precision) and must reproduce the GPU's decisions bit for bit.
"""
import numpy as np

from oracle import pqt_query as Q

RTOL = 1e-4            # relative tolerance on fp32 distances (the target the kernels are held to)
U32 = 2.0 ** -24       # unit roundoff of fp32


def kappa(n_terms):
    """Multiple of the unit roundoff allowed as an absolute floor for a value the kernel forms by an
    n-term fp32 accumulation with cancellation (||q||^2 + ||c||^2 - 2 q.c): the worst case of that
    arithmetic is (2 n + 3) u times the magnitude of the terms, its typical size sqrt(n) u; the floor
    takes max(8, n / 4)."""
    return max(8.0, n_terms / 4.0)


class FloorStats:
    """How many compared elements passed only because of the absolute floor, and the largest error
    seen in units of u times the elements' term magnitude."""

    def __init__(self):
        self.reset()

    def reset(self):
        self.compared = 0
        self.needed_floor = 0
        self.max_ratio = 0.0

    def add(self, err, o, mag):
        self.compared += int(err.size)
        self.needed_floor += int(np.count_nonzero(err > RTOL * np.abs(o)))
        if err.size:
            with np.errstate(divide="ignore", invalid="ignore"):
                r = np.where(mag > 0, err / (U32 * mag), 0.0)
            self.max_ratio = max(self.max_ratio, float(np.max(r)))

    def summary(self):
        return (f"{self.compared} float elements compared, {self.needed_floor} needed the absolute floor, "
                f"largest error {self.max_ratio:.2f} u x term magnitude")


STATS = FloorStats()


def close(g, o, mag=None, k=0.0):
    """|g - o| <= 1e-4 |o| + k u mag, element-wise.  mag: magnitude of the terms whose signed sum the
    kernel evaluates for this element (None: no floor, the value is a sum of non-negative terms)."""
    g = np.asarray(g, dtype=np.float64)
    o = np.asarray(o, dtype=np.float64)
    err = np.abs(g - o)
    if mag is None:
        mag = np.zeros_like(o)
    mag = np.broadcast_to(np.asarray(mag, dtype=np.float64), o.shape)
    STATS.add(err, o, mag)
    return bool(np.all(err <= RTOL * np.abs(o) + k * U32 * mag))


def subpart_magnitudes(ix, y):
    """S[m][i] = ||[y]_m||^2 + ||[c_i]_m||^2: the terms of a[m][i] = ||q||^2 + ||c||^2 - 2 q.c."""
    y64 = np.asarray(y, dtype=np.float64)
    ds, dp = ix.D // ix.M, ix.D // ix.P
    S = np.zeros((ix.M, ix.k1))
    for m in range(ix.M):
        p = (m * ds) // dp
        lo = m * ds - p * dp
        c = ix.C1[p, :, lo:lo + ds].astype(np.float64)
        S[m] = np.dot(y64[m * ds:(m + 1) * ds], y64[m * ds:(m + 1) * ds]) + np.sum(c * c, axis=1)
    return S


def lut_magnitudes(ix, S):
    """Term magnitudes of LUT[m][c] = (1 - lam) a[m][i] + lam a[m][j] + (lam^2 - lam) cc[m][i][j]."""
    lam = ix.tbl_lam.astype(np.float64)
    m_idx = np.arange(ix.M)[:, None]
    i, j = ix.tbl_i.astype(np.int64), ix.tbl_j.astype(np.int64)
    return np.abs(1.0 - lam) * S[m_idx, i] + np.abs(lam) * S[m_idx, j] + \
        np.abs(lam * lam - lam) * ix.cc.astype(np.float64)[m_idx, i, j]


def pair_score_magnitudes(ix, S, codes):
    """The same for scores of (pair, lambda level) codes, summed over the sub-parts."""
    pairs = np.asarray(Q.centroid_pairs(ix.k1), dtype=np.int64).reshape(-1, 2)
    out = np.zeros(codes.shape[0])
    for m in range(ix.M):
        i, j = pairs[codes[:, 2 * m], 0], pairs[codes[:, 2 * m], 1]
        lam = Q.lambda_of_level(codes[:, 2 * m + 1])
        out += np.abs(1.0 - lam) * S[m, i] + np.abs(lam) * S[m, j] + np.abs(lam * lam - lam) * ix.cc.astype(np.float64)[m, i, j]
    return out


def to_np(t):
    return t.detach().cpu().numpy()


def check_query_stages(ix, y, taps, q, k, w, T, C, out_ids, out_dists, exact=False, order="fullsort",
                       truncate_pairs=False):
    """ix: oracle PQTIndex (same file the GPU loaded); taps: dict of numpy arrays for the batch;
    q: row in the batch.  Raises AssertionError naming the stage.  Returns the oracle trace of the
    pure float64 run."""
    P, M, k1, k2 = ix.P, ix.M, ix.k1, ix.k2
    R = w * k2
    y64 = np.asarray(y, dtype=np.float64)
    S = subpart_magnitudes(ix, y64)
    ka = kappa(ix.D // M)             # a[m][i]: accumulations over the D / M dimensions of a sub-part
    tr = Q.query(ix, y, k, w, T=T, C=C, order_method=order, truncate_pairs=truncate_pairs)

    # ---- S1 level-1 sub-part distances (float) ---------------------------------------------------
    a_g = taps["a"][q]
    if exact:
        assert np.array_equal(a_g.astype(np.float64), tr.a), "S1 a (exact)"
    assert close(a_g, tr.a, S, ka), f"S1 a: max abs err {np.max(np.abs(a_g - tr.a))}"

    # ---- S2 selection replayed on the GPU's a (fp32 sums, ascending sub-part) -------------------------
    d1_g = Q.part_distances(a_g.astype(np.float32), P)
    sel_r = Q.select_clusters(d1_g, w)
    assert np.array_equal(sel_r, taps["sel"][q]), "S2 sel replay"

    # ---- S3 level-2 lists ---------------------------------------------------------------------------
    Ld_g, Lid_g = taps["L_d"][q], taps["L_id"][q].astype(np.int64)
    d2_o, ids_o = Q.level2_distances(y, ix.C2, sel_r)
    for p in range(P):
        assert sorted(Lid_g[p].tolist()) == sorted(ids_o[p].tolist()), "S3 leaf id set"
        lookup = dict(zip(ids_o[p].tolist(), d2_o[p].tolist()))
        want = np.array([lookup[i] for i in Lid_g[p].tolist()])
        if exact:
            assert np.array_equal(Ld_g[p].astype(np.float64), want), "S3 d2 (exact)"
        assert close(Ld_g[p], want), "S3 d2"        # a sum of squared differences: relative error only
        o = Q.order_by_value_then_id(Ld_g[p], Lid_g[p])
        assert np.array_equal(o, np.arange(R)), "S3 list not sorted by (d2, id)"

    # ---- S4 bin order replayed on the GPU's lists (fp32 sums) ------------------------------------------
    if order == "static":        # the slope is chosen from the GPU's own fp32 lists, the table is fixed
        tup_r, keys_r = Q.bin_order_static([Ld_g[p].astype(np.float32) for p in range(P)], T)
    else:
        tup_r, keys_r = Q.bin_order([Ld_g[p].astype(np.float32) for p in range(P)], T, truncate_pairs=truncate_pairs)
    nt = int(taps["n_tuples"][q])
    assert nt == tup_r.shape[0], "S4 number of tuples"
    assert np.array_equal(taps["tuples"][q][:nt, :P].astype(np.int64), tup_r), "S4 tuple order"
    assert np.array_equal(taps["tuple_keys"][q][:nt], keys_r.astype(np.float32)), "S4 tuple keys"
    slots_r = Q.propose_bins(tup_r, Lid_g, k1 * k2, ix.H, ix.offsets)
    pos_r = Q.gather_candidates(slots_r, ix.offsets, C)
    # slots that contribute at least one candidate before the cut
    lens = ix.offsets[slots_r + 1].astype(np.int64) - ix.offsets[slots_r].astype(np.int64) if slots_r.size else np.zeros(0, np.int64)
    used = int(np.sum(np.cumsum(lens) - lens < C))
    ns = int(taps["n_slots"][q])
    assert ns == used, f"S4 number of proposed slots {ns} vs {used}"
    assert np.array_equal(taps["slots"][q][:ns], slots_r[:ns]), "S4 proposed slots"

    # ---- S5 candidate list ---------------------------------------------------------------------------
    nc = int(taps["n_cand"][q])
    assert nc == pos_r.shape[0], "S5 candidate count"
    cand_r = ix.ids[pos_r].astype(np.int64)
    assert np.array_equal(taps["cand_ids"][q][:nc], cand_r), "S5 candidate ids"

    if ix.code_format == 1:
        # ---- S6-S7 (pair, lambda) codes: Eq. 9 per candidate, no table; float comparison -----------------
        sc_g = taps["scores"][q][:nc]
        sc_o = Q.score_pair_lambda(a_g.astype(np.float64), ix.cc, ix.codes[pos_r])
        mag = pair_score_magnitudes(ix, S, ix.codes[pos_r])
        # evaluated from the GPU's own a: only the rounding of Eq. 9 itself and of the sum over the sub-parts
        assert close(sc_g, sc_o, mag, 8.0 + M), "S7 scores vs oracle formula on the GPU's a"
        tr.parity_mag = dict(zip(cand_r.tolist(), mag.tolist()))
        tr.parity_k = ka + 8.0 + M
        if exact:
            assert np.array_equal(sc_g.astype(np.float64), tr.scores), "S7 scores (exact)"
        ids_r, d_r = Q.top_k(sc_g, cand_r, k)
        assert np.array_equal(out_ids[q], ids_r), "S8 ids replay"
        assert np.array_equal(out_dists[q], d_r.astype(np.float32)), "S8 distances replay"
        return tr

    # ---- S6 LUT (float), S7 scores replayed on the GPU's LUT (fp32, ascending m) ------------------------
    lut_g = taps["lut"][q]
    lut_o = Q.build_lut(a_g.astype(np.float64), ix.tbl_i, ix.tbl_j, ix.tbl_lam, ix.cc.astype(np.float64))
    Sl = lut_magnitudes(ix, S)
    assert close(lut_g, lut_o, Sl, 8.0), "S6 LUT vs oracle formula on the GPU's a"     # rounding of Eq. 9 only
    assert close(lut_g, tr.lut, Sl, ka + 8.0), "S6 LUT vs oracle"                       # plus the error of a
    if exact:
        assert np.array_equal(lut_g.astype(np.float64), tr.lut), "S6 LUT (exact)"
    sc_r = Q.score_codes(lut_g.astype(np.float32), ix.codes[pos_r])
    assert np.array_equal(taps["scores"][q][:nc], sc_r), "S7 scores replay"

    # ---- S8 top-k replayed on the GPU's scores -------------------------------------------------------------
    ids_r, d_r = Q.top_k(sc_r, cand_r, k)
    assert np.array_equal(out_ids[q], ids_r), "S8 ids replay"
    assert np.array_equal(out_dists[q], d_r.astype(np.float32)), "S8 distances replay"
    mag = np.zeros(nc)
    for m in range(M):
        mag += Sl[m, ix.codes[pos_r, m]]
    tr.parity_mag = dict(zip(cand_r.tolist(), mag.tolist()))
    tr.parity_k = ka + 8.0 + M                           # error of a, rounding of Eq. 9, the sum over M sub-parts
    return tr


def end_to_end_agreement(tr, out_ids_q, out_dists_q, margin_thr=1e-5):
    """Compares the final answer with the pure float64 oracle run.  Returns (ids_equal, decided):
    `decided` says whether every set-changing decision of the oracle had a relative margin above
    margin_thr, in which case the ids MUST be equal."""
    same = bool(np.array_equal(out_ids_q, tr.out_ids))
    if same:
        have = tr.out_ids >= 0
        mag = np.array([tr.parity_mag[i] for i in tr.out_ids[have].tolist()])
        assert close(out_dists_q[have], tr.out_dists[have], mag, tr.parity_k), "output distances"
    decided = bool(tr.margins) and tr.margins["min"] > margin_thr
    return same, decided
