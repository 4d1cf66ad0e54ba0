"""Seeded Gaussian-mixture vectors standing in for the paper's descriptor sets.

The paper evaluates on sets of 8-bit-range image descriptors (128, 256 or 960
dimensions; 1 M to 1 B base vectors; 1000 queries; Section 4.1, datasets
table).  Those sets are not available here, so every input is synthetic: a
mixture of `ncomp` isotropic Gaussians whose samples are clipped to [0, 255]
and kept as float32.  Only shapes and value range are taken from the paper.

Rows are produced in fixed blocks of `BLOCK` rows, each block from its own
counter-seeded generator, so that any row range [start, start+count) has the
same values however the caller chunks its requests.
"""

from __future__ import annotations

from dataclasses import dataclass

import numpy as np

SEED_MIXTURE = 0  # mixture parameters (component means)
SEED_TRAIN = 1    # learning set
SEED_BASE = 2     # base (database) set
SEED_QUERY = 3    # query set

BLOCK = 16384


@dataclass(frozen=True)
class MixtureSpec:
    d: int = 128
    ncomp: int = 64
    mean_mu: float = 48.0
    mean_sigma: float = 32.0
    sigma: float = 24.0
    lo: float = 0.0
    hi: float = 255.0
    seed: int = SEED_MIXTURE


def mixture_params(spec: MixtureSpec) -> np.ndarray:
    """Component means, float32 [ncomp][d], clipped to the value range."""
    rng = np.random.default_rng([spec.seed, spec.d, spec.ncomp])
    mu = rng.normal(spec.mean_mu, spec.mean_sigma, size=(spec.ncomp, spec.d))
    return np.clip(mu, spec.lo, spec.hi).astype(np.float32)


def _block(spec: MixtureSpec, means: np.ndarray, stream_seed: int, b: int):
    rng = np.random.default_rng([spec.seed, stream_seed, b, spec.d])
    labels = rng.integers(0, spec.ncomp, size=BLOCK)
    noise = rng.standard_normal((BLOCK, spec.d), dtype=np.float32)
    x = means[labels] + np.float32(spec.sigma) * noise
    np.clip(x, spec.lo, spec.hi, out=x)
    return x, labels


def mixture_vectors(spec: MixtureSpec, stream_seed: int, start: int, count: int,
                    return_labels: bool = False):
    """Rows [start, start+count) of the stream `stream_seed`, float32 [count][d]."""
    means = mixture_params(spec)
    out = np.empty((count, spec.d), dtype=np.float32)
    lab = np.empty(count, dtype=np.int64)
    pos = 0
    b = start // BLOCK
    off = start - b * BLOCK
    while pos < count:
        x, labels = _block(spec, means, stream_seed, b)
        take = min(BLOCK - off, count - pos)
        out[pos:pos + take] = x[off:off + take]
        lab[pos:pos + take] = labels[off:off + take]
        pos += take
        b += 1
        off = 0
    return (out, lab) if return_labels else out


def kmeans_init_rows(n_train: int, k: int, seed: int = SEED_TRAIN) -> np.ndarray:
    """The k distinct learning-set rows a k-means run starts from (int64 [k])."""
    rng = np.random.default_rng([seed, n_train, k, 0x6B6D])
    return rng.permutation(n_train)[:k].astype(np.int64)


def zipf_list_sizes(n_total: int, n_lists: int, exponent: float = 0.8,
                    seed: int = SEED_BASE) -> np.ndarray:
    """Inverted-list sizes with a Zipf profile, int64 [n_lists], summing to n_total.

    The list of rank r (1-based) gets a share proportional to r**-exponent;
    ranks are assigned to cells by a seeded permutation.  Rounding slack goes
    to the largest list.
    """
    r = np.arange(1, n_lists + 1, dtype=np.float64)
    w = r ** (-exponent)
    sizes = np.floor(n_total * w / w.sum()).astype(np.int64)
    sizes[0] += n_total - sizes.sum()
    rng = np.random.default_rng([seed, n_lists, 0x7A69])
    perm = rng.permutation(n_lists)
    out = np.empty(n_lists, dtype=np.int64)
    out[perm] = sizes
    return out
