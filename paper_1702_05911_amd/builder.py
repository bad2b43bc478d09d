"""Offline phase: drives the library's training and streaming-builder calls (Sec. 3.1, Sec. 3.3
"Offline computation", Sec. 4 data layout).

Argument marshalling only: the codebooks and the line-code table are trained by pqt_train, every
database vector is binned and encoded by pqt_builder_add, the inverted lists are assembled by
pqt_builder_finish -- all HIP kernels.  PyTorch supplies the device buffers the chunks arrive in.

The database is given as a chunk generator `chunks(start, count)` -> (count, D) float32 tensor or
array (for databases that never exist in memory as raw vectors) or as an array.
"""
import torch


def build_index_native(X=None, *, chunks=None, N=None, D=None, P, k1, k2, M, H=None, T=1024, C=4096, train_n=None,
                       iters=20, device=0, chunk_rows=1 << 20, table_train_n=100_000, observer=None,
                       trained_out=None, code_format=0):
    """Trains on the first train_n vectors (pqt_train), streams all N through pqt_builder_add and
    returns the binding's Index.  code_format 1: codes are (centroid pair, lambda level) per
    sub-part instead of table entries.  observer(start, chunk) is called once per database chunk
    (e.g. to accumulate exact nearest neighbours while the vectors exist); trained_out, a dict,
    receives the trained arrays."""
    from . import binding
    dev = torch.device("cuda", device)
    if X is not None:
        N, D = X.shape

        def chunks(start, count):                                  # noqa: F811
            return X[start:start + count]
    H = (k1 * k2) ** P if H is None else H
    train_n = min(train_n or N, N)
    Xt = torch.as_tensor(chunks(0, train_n)).to(device=dev, dtype=torch.float32).contiguous()
    params = binding.pqt_train(Xt, P=P, k1=k1, k2=k2, M=M, iters=iters,
                               n_table=0 if code_format == 1 else table_train_n)
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
    """build_index_native(...) saved to the index file `path` (pqt_index_save); returns the Index."""
    from . import binding
    index = build_index_native(X, **kw)
    binding.pqt_index_save(index, path)
    return index
