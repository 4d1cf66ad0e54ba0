"""Seeded synthetic inputs shaped like the paper's workloads.

This package holds input generators only: raw vectors, queries, random
permutations, inverted-list size profiles.  It contains none of the method's
arithmetic (no quantizer training, no encoding, no distance tables, no scan),
and it imports neither the CPU oracle nor the HIP library.  Both sides of a
parity test draw their inputs from here.
"""

from .mixture import (  # noqa: F401
    MixtureSpec,
    mixture_params,
    mixture_vectors,
    kmeans_init_rows,
    zipf_list_sizes,
    SEED_MIXTURE,
    SEED_TRAIN,
    SEED_BASE,
    SEED_QUERY,
)
