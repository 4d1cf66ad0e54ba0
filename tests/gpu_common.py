"""Helpers of the GPU parity tests: config-1 data built by the oracle, host<->device copies."""

import functools

import numpy as np


@functools.lru_cache(maxsize=None)
def config1(n=100_000, m=16, d=128, nq=16, train_n=20_000, iters=10):
    """Config 1: mixture data, PQ m x 16 trained by 10 k-means iterations on 20k vectors."""
    from oracle import qadc_oracle as O, cref
    from workloads import (MixtureSpec, mixture_vectors, kmeans_init_rows,
                           SEED_TRAIN, SEED_BASE, SEED_QUERY)
    spec = MixtureSpec(d=d)
    train = mixture_vectors(spec, SEED_TRAIN, 0, train_n)
    cb = O.pq_train(train, m, 16, iters, kmeans_init_rows(train_n, 16))
    base = mixture_vectors(spec, SEED_BASE, 0, n)
    codes = cref.pq_encode(base, cb)
    queries = mixture_vectors(spec, SEED_QUERY, 0, nq)
    return dict(spec=spec, codebooks=cb, base=base, codes=codes, queries=queries)


def to_gpu(a):
    import torch
    return torch.from_numpy(np.ascontiguousarray(a)).to("cuda:0")


def idx_np(t):
    return t.cpu().numpy().view(np.uint32)
