import os
import sys

import numpy as np
import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


from paper_2601_07183_amd import datagen, index_build  # noqa: E402


def _small(seed, n=3000, d=16, nlist=16, M=8, integer=False, **kw):
    base = datagen.random_vectors(seed, n, d)
    # a few tight clumps so that large shared cells exist
    g = np.random.Generator(np.random.PCG64(seed + 99))
    centers = g.uniform(-1, 1, size=(8, d)).astype(np.float32)
    base = (centers[g.integers(0, 8, size=n)] + 0.25 * base).astype(np.float32)
    if integer:
        base = np.clip(np.rint(base * 60 + 128), 0, 255).astype(np.float32)
    return base, index_build.build_index(base, nlist, M, seed=seed, coarse_iters=8, pq_iters=8,
                                         **kw)


@pytest.fixture(scope="session")
def small_index():
    """3000 x 16 float vectors, nlist 16, M 8, strict AIR assignment."""
    return _small(11)


@pytest.fixture(scope="session")
def small_index_int():
    """Integer-valued data: every squared distance is exact in fp32."""
    return _small(12, integer=True)


@pytest.fixture(scope="session")
def small_index_nonstrict():
    return _small(13, strict=False, lam=0.5)


@pytest.fixture(scope="session")
def tiny_workload():
    w = datagen.WORKLOADS["tiny"]
    base = datagen.make_base(w)
    hx = index_build.build_index(base, w.nlist, w.M, seed=w.seed)
    return w, base, datagen.make_queries(w), hx


def small_queries(seed, nq, d, integer=False):
    q = datagen.random_vectors(seed + 1000, nq, d)
    if integer:
        q = np.clip(np.rint(q * 60 + 128), 0, 255).astype(np.float32)
    return q
