import os
import sys

import numpy as np
import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (runs the HIP library)")


def pytest_terminal_summary(terminalreporter):
    """How many float comparisons of the GPU parity tests passed only through the absolute floor."""
    pu = sys.modules.get("parity_util")
    if pu is not None and pu.STATS.compared:
        terminalreporter.write_line("parity tolerance (1e-4 relative + floor): " + pu.STATS.summary())


@pytest.fixture(scope="session")
def tiny():
    """Tiny workload: vectors, queries and an oracle-built index."""
    from workloads import CONFIGS, tiny_mixture
    from oracle import pqt_build
    cfg = CONFIGS["tiny"]
    X = tiny_mixture(cfg.N, d=cfg.D, seed=cfg.data_seed)
    Y = tiny_mixture(cfg.nq, d=cfg.D, seed=cfg.query_seed)
    ix = pqt_build.build_index(X, cfg.P, cfg.k1, cfg.k2, cfg.M, H=cfg.H, T=cfg.T, C=cfg.C)
    return cfg, X, Y, ix


@pytest.fixture(scope="session")
def tiny_pair(tiny):
    """The tiny index with its codes stored as (centroid pair, lambda level) per sub-part."""
    import dataclasses
    from oracle import pqt_build
    cfg, X, Y, ix = tiny
    codes = pqt_build.encode_pair_lambda(X, ix.C1, ix.M)[ix.ids]
    return cfg, X, Y, dataclasses.replace(ix, codes=np.ascontiguousarray(codes), code_format=1)


@pytest.fixture(scope="session")
def rng():
    return np.random.default_rng(12345)
