import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


@pytest.fixture(scope="session")
def tiny_pq():
    """Config-1-shaped PQ at reduced size: d=128, m=16 x 16 centroids, trained by the oracle."""
    import numpy as np
    from oracle import qadc_oracle as O
    from workloads import (MixtureSpec, mixture_vectors, kmeans_init_rows,
                           SEED_TRAIN, SEED_BASE, SEED_QUERY)
    spec = MixtureSpec()
    train = mixture_vectors(spec, SEED_TRAIN, 0, 4000)
    cb = O.pq_train(train, 16, 16, 5, kmeans_init_rows(4000, 16))
    base = mixture_vectors(spec, SEED_BASE, 0, 20000)
    comps = O.pq_encode(base, cb)
    codes = O.pack_nibbles(comps)
    queries = mixture_vectors(spec, SEED_QUERY, 0, 8)
    return dict(spec=spec, train=train, codebooks=cb, base=base, comps=comps, codes=codes,
                queries=queries)
