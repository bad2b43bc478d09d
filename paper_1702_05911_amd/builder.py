"""Offline phase: builds a PQT index file from database vectors (Sec. 3.1, Sec. 3.3
"Offline computation", Sec. 4 data layout).

Query-independent, so not on the timed path.  Batched fp32 PyTorch on whatever device is
given (GPU when present): Lloyd codebooks per part and per level-1 cell, bin assignment,
inverted lists by a stable sort on the slot number (ids ascending inside a slot), the
256-entry line-code table per sub-part, and the code of every vector stored in the same
order as the ids (bin-major), so that the query kernels read contiguous runs.

The database may be given as an array or as a chunk generator `chunks(start, count)`
(for databases that never exist in memory as raw vectors).
"""
import struct

import numpy as np
import torch

MAGIC = b"PQTIDX1\0"
ALIGN = 256


# ---------------------------------------------------------------------------------------------
def _sqdist(X, Cen):
    """|X| x |Cen| squared distances, ||x||^2 - 2 x.c + ||c||^2 in fp32."""
    return (X * X).sum(1, keepdim=True) - 2.0 * (X @ Cen.t()) + (Cen * Cen).sum(1)[None, :]


def _lloyd(X, k, iters):
    n = X.shape[0]
    if n == 0:
        return torch.zeros((k, X.shape[1]), dtype=X.dtype, device=X.device)
    if n <= k:
        cen = X.mean(0, keepdim=True).repeat(k, 1)
        cen[:n] = X
        return cen
    cen = X[(torch.arange(k, device=X.device) * n) // k].clone()
    for _ in range(iters):
        d = _sqdist(X, cen)
        dmin, lab = d.min(1)
        sums = torch.zeros_like(cen).index_add_(0, lab, X)
        cnt = torch.bincount(lab, minlength=k)
        filled = cnt > 0
        cen[filled] = sums[filled] / cnt[filled, None].to(X.dtype)
        for c in torch.nonzero(~filled).flatten().tolist():     # re-seed an empty cell with the farthest row
            far = int(torch.argmax(dmin))
            cen[c] = X[far]
            dmin[far] = 0.0
    return cen


def train_tree(Xt, P, k1, k2, iters=20):
    """Level-1 product quantiser and, independently per level-1 cell, its level-2 quantiser."""
    D = Xt.shape[1]
    dp = D // P
    C1 = torch.zeros((P, k1, dp), dtype=torch.float32, device=Xt.device)
    C2 = torch.zeros((P, k1, k2, dp), dtype=torch.float32, device=Xt.device)
    for p in range(P):
        Xp = Xt[:, p * dp:(p + 1) * dp].contiguous()
        C1[p] = _lloyd(Xp, k1, iters)
        lab = _sqdist(Xp, C1[p]).argmin(1)
        for i in range(k1):
            sub = Xp[lab == i]
            C2[p, i] = _lloyd(sub, k2, iters) if sub.shape[0] > 0 else C1[p, i][None].repeat(k2, 1)
    return C1, C2


def assign_slots(X, C1, C2, H):
    """Slot (bin number modulo H) of every row of X: nearest level-1 centroid per part, then
    the nearest of its children; bin number with part 1 most significant."""
    P, k1, k2, dp = C2.shape
    n = X.shape[0]
    lin = torch.zeros(n, dtype=torch.int64, device=X.device)
    for p in range(P):
        Xp = X[:, p * dp:(p + 1) * dp]
        i = _sqdist(Xp, C1[p]).argmin(1)
        # distances to the children of the chosen cell only
        child = C2[p][i]                                          # n x k2 x dp
        d2 = ((Xp[:, None, :] - child) ** 2).sum(2)
        j = d2.argmin(1)
        lin = lin * (k1 * k2) + (i * k2 + j)
    return lin % H


def _subpart_centroids(C1, M, m):
    P, k1, dp = C1.shape
    ds = (P * dp) // M
    p = (m * ds) // dp
    lo = m * ds - p * dp
    return C1[p, :, lo:lo + ds]


def line_table(Xt, C1, M, n_codes=256):
    """Per sub-part 256 code points (i, j, lambda) on lines through pairs of level-1 centroids
    (Sec. 3.3): each training sub-vector votes for its nearest line; lines receive code points
    in proportion to their votes (largest-remainder rounding), placed at the quantiles of the
    projection parameters lambda seen on that line; entries ordered by (i, j, lambda)."""
    D = Xt.shape[1]
    ds = D // M
    k1 = C1.shape[1]
    ti = np.zeros((M, n_codes), np.uint8)
    tj = np.zeros((M, n_codes), np.uint8)
    tl = np.zeros((M, n_codes), np.float32)
    pairs = [(i, j) for i in range(k1) for j in range(i + 1, k1)]
    if not pairs or Xt.shape[0] == 0:
        return ti, tj, tl
    pi = torch.tensor([p[0] for p in pairs], device=Xt.device)
    pj = torch.tensor([p[1] for p in pairs], device=Xt.device)
    for m in range(M):
        cen = _subpart_centroids(C1, M, m)
        Xs = Xt[:, m * ds:(m + 1) * ds]
        u = cen[pj] - cen[pi]                                     # npairs x ds
        uu = (u * u).sum(1)
        best_err = torch.full((Xs.shape[0],), float("inf"), device=Xt.device)
        best_pair = torch.zeros(Xs.shape[0], dtype=torch.int64, device=Xt.device)
        best_lam = torch.zeros(Xs.shape[0], device=Xt.device)
        di = _sqdist(Xs, cen)                                     # n x k1
        xu = Xs @ u.t() - (cen[pi] * u).sum(1)[None, :]           # (x - c_i).u   n x npairs
        step = 256
        for q0 in range(0, len(pairs), step):
            sl = slice(q0, min(q0 + step, len(pairs)))
            ok = uu[sl] > 0
            lam = torch.where(ok[None, :], xu[:, sl] / uu[sl].clamp_min(1e-30)[None, :], torch.zeros_like(xu[:, sl]))
            err = di[:, pi[sl]] - lam * lam * uu[sl][None, :]
            err = torch.where(ok[None, :], err, torch.full_like(err, float("inf")))
            e, a = err.min(1)
            better = e < best_err
            best_err = torch.where(better, e, best_err)
            best_pair = torch.where(better, a + q0, best_pair)
            best_lam = torch.where(better, lam.gather(1, a[:, None])[:, 0], best_lam)
        use = torch.bincount(best_pair, minlength=len(pairs)).double().cpu().numpy()
        quota = use * n_codes / use.sum()
        alloc = np.floor(quota).astype(np.int64)
        rem = quota - alloc
        for q in np.lexsort((np.arange(len(pairs)), -rem))[: n_codes - int(alloc.sum())]:
            alloc[q] += 1
        bp = best_pair.cpu().numpy()
        bl = best_lam.cpu().numpy()
        order = np.argsort(bp, kind="stable")
        starts = np.searchsorted(bp[order], np.arange(len(pairs) + 1))
        entries = []
        for q in np.nonzero(alloc)[0]:
            lams = np.sort(bl[order[starts[q]:starts[q + 1]]])
            for t in range(alloc[q]):
                pos = min(int((t + 0.5) / alloc[q] * lams.shape[0]), lams.shape[0] - 1)
                entries.append((pairs[q][0], pairs[q][1], np.float32(lams[pos])))
        entries.sort(key=lambda e: (e[0], e[1], float(e[2])))
        while len(entries) < n_codes:
            entries.append(entries[-1])
        for c, (i, j, lam) in enumerate(entries[:n_codes]):
            ti[m, c], tj[m, c], tl[m, c] = i, j, lam
    return ti, tj, tl


def encode(X, C1, M, ti, tj, tl):
    """Code byte per sub-part: the nearest of the 256 code points (first minimum on ties)."""
    n, D = X.shape
    ds = D // M
    codes = torch.empty((n, M), dtype=torch.uint8, device=X.device)
    for m in range(M):
        cen = _subpart_centroids(C1, M, m)
        lam = torch.from_numpy(tl[m]).to(X.device)[:, None]
        pts = (1.0 - lam) * cen[torch.from_numpy(ti[m].astype(np.int64)).to(X.device)] + \
            lam * cen[torch.from_numpy(tj[m].astype(np.int64)).to(X.device)]
        codes[:, m] = _sqdist(X[:, m * ds:(m + 1) * ds], pts).argmin(1).to(torch.uint8)
    return codes


def pair_table(C1, M):
    P, k1, dp = C1.shape
    cc = torch.zeros((M, k1, k1), dtype=torch.float64)
    for m in range(M):
        cen = _subpart_centroids(C1, M, m).double().cpu()
        cc[m] = ((cen[:, None, :] - cen[None, :, :]) ** 2).sum(2)
    return cc.float().numpy()


# ---------------------------------------------------------------------------------------------
def write_index_file(path, hdr, arrays):
    head = bytearray(ALIGN)
    head[0:8] = MAGIC
    struct.pack_into("<6I", head, 8, 1, hdr["D"], hdr["P"], hdr["k1"], hdr["k2"], hdr["M"])
    struct.pack_into("<2Q", head, 32, hdr["N"], hdr["H"])
    struct.pack_into("<3I", head, 48, hdr["T"], hdr["C"], 32)
    with open(path, "wb") as f:
        f.write(head)
        for name, dt in (("C1", np.float32), ("C2", np.float32), ("tbl_i", np.uint8), ("tbl_j", np.uint8),
                         ("tbl_lam", np.float32), ("cc", np.float32), ("offsets", np.uint32), ("ids", np.uint32),
                         ("codes", np.uint8)):
            f.write(b"\0" * ((-f.tell()) % ALIGN))
            np.ascontiguousarray(arrays[name], dtype=dt).tofile(f)


def build_arrays(X=None, *, chunks=None, N=None, D=None, P, k1, k2, M, H=None, T=1024, C=4096,
                 train_n=None, iters=20, device=None, chunk_rows=1 << 18, table_train_n=100_000,
                 observer=None):
    """Builds the index of X (array, N x D) or of chunks(start, count) -> (count x D) fp32
    tensor/array.  Returns a dict: the header fields, the small arrays (C1, C2, tbl_i, tbl_j,
    tbl_lam, cc) as NumPy arrays, and offsets (int64, H+1), ids (int64, N) and codes (uint8,
    N x M) as tensors on `device`.  observer(start, chunk) is called once per database chunk
    (e.g. to accumulate exact nearest neighbours while the vectors exist)."""
    if device is None:
        device = torch.device("cuda") if torch.cuda.is_available() else torch.device("cpu")
    if X is not None:
        X = torch.as_tensor(np.asarray(X) if not torch.is_tensor(X) else X)
        N, D = X.shape

        def chunks(start, count):                                  # noqa: F811
            return X[start:start + count]
    assert D % P == 0 and D % M == 0 and M % P == 0 and k1 <= 256
    K = (k1 * k2) ** P
    H = K if H is None else H
    train_n = min(train_n or N, N)
    Xt = torch.as_tensor(chunks(0, train_n)).to(device=device, dtype=torch.float32)
    C1, C2 = train_tree(Xt, P, k1, k2, iters)
    ti, tj, tl = line_table(Xt[:table_train_n], C1, M)
    del Xt
    slots = torch.empty(N, dtype=torch.int32 if H < 2 ** 31 else torch.int64, device=device)
    codes = torch.empty((N, M), dtype=torch.uint8, device=device)
    for s in range(0, N, chunk_rows):
        n = min(chunk_rows, N - s)
        Xc = torch.as_tensor(chunks(s, n)).to(device=device, dtype=torch.float32)
        for s2 in range(0, n, 1 << 18):                            # bounds the n x k2 x dp gather below
            sl = slice(s2, min(s2 + (1 << 18), n))
            slots[s + sl.start:s + sl.stop] = assign_slots(Xc[sl], C1, C2, H).to(slots.dtype)
            codes[s + sl.start:s + sl.stop] = encode(Xc[sl], C1, M, ti, tj, tl)
        if observer is not None:
            observer(s, Xc)
        del Xc
    order = torch.sort(slots, stable=True).indices                # ids by (slot, id)
    hist = torch.bincount(slots, minlength=H)
    del slots
    offsets = torch.zeros(H + 1, dtype=torch.int64, device=device)
    offsets[1:] = torch.cumsum(hist, 0)
    del hist
    codes = codes[order]
    return dict(D=D, P=P, k1=k1, k2=k2, M=M, N=N, H=H, T=T, C=C,
                C1=C1.cpu().numpy(), C2=C2.cpu().numpy(), tbl_i=ti, tbl_j=tj, tbl_lam=tl, cc=pair_table(C1, M),
                offsets=offsets, ids=order, codes=codes)


def train(Xt, *, P, k1, k2, M, iters=20, table_train_n=100_000):
    """Everything that is learned from a sample: the two-level codebooks, the line-code table and the
    centroid-pair distances.  Returns NumPy arrays named as the index arrays."""
    C1, C2 = train_tree(Xt, P, k1, k2, iters)
    ti, tj, tl = line_table(Xt[:table_train_n], C1, M)
    return dict(C1=C1.cpu().numpy(), C2=C2.cpu().numpy(), tbl_i=ti, tbl_j=tj, tbl_lam=tl, cc=pair_table(C1, M))


def build_index_native(*, chunks, N, D, P, k1, k2, M, H=None, T=1024, C=4096, train_n=None, iters=20,
                       device=0, chunk_rows=1 << 20, table_train_n=100_000, observer=None, trained_out=None,
                       code_format=0):
    """The same index built by the library's own streaming builder (pqt_builder_*): codebooks and
    table are trained here on the first train_n vectors, every vector is then binned and encoded by
    HIP kernels and the lists are assembled on the GPU.  code_format 1: codes are (centroid pair,
    lambda level) per sub-part instead of table entries.  Returns the binding's Index."""
    from . import binding
    dev = torch.device("cuda", device)
    H = (k1 * k2) ** P if H is None else H
    train_n = min(train_n or N, N)
    Xt = torch.as_tensor(chunks(0, train_n)).to(device=dev, dtype=torch.float32)
    params = train(Xt, P=P, k1=k1, k2=k2, M=M, iters=iters, table_train_n=table_train_n)
    del Xt
    if trained_out is not None:
        trained_out.update(params)                                  # the caller wants the codebooks and table too
    params.update(N=N, H=H, D=D, P=P, k1=k1, k2=k2, M=M, T=T, C=C, code_format=code_format)
    b = binding.pqt_builder_create(params, device)
    try:
        for s in range(0, N, chunk_rows):
            n = min(chunk_rows, N - s)
            Xc = torch.as_tensor(chunks(s, n)).to(device=dev, dtype=torch.float32).contiguous()
            binding.pqt_builder_add(b, Xc)
            if observer is not None:
                observer(s, Xc)
            torch.cuda.synchronize(dev)                             # Xc must outlive the kernels that read it
            del Xc
        return binding.pqt_builder_finish(b)
    finally:
        binding.pqt_builder_free(b)


def build_index(path, X=None, **kw):
    """build_arrays(...) written to the index file `path`; returns the arrays as NumPy arrays."""
    arrays = build_arrays(X, **kw)
    for name, dt in (("offsets", np.uint32), ("ids", np.uint32), ("codes", np.uint8)):
        arrays[name] = arrays[name].cpu().numpy().astype(dt)
    write_index_file(path, arrays, arrays)
    return arrays
