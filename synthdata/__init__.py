"""Seeded synthetic inputs for the IVF-PQ hot-cluster search path.

This module is shared by the tests of the CPU oracle and of the HIP library.
It produces *inputs only*: a clustered vector database, Zipf-skewed queries,
and a trained IVF-PQ index (centroids, codebooks, codes, ids, list offsets).
None of the search arithmetic (coarse probing, lookup tables, ADC sums,
top-k) lives here, and neither the oracle nor the library is imported.
"""
from .workloads import WorkloadSpec, SPECS, get_spec  # noqa: F401
from .generate import (  # noqa: F401
    mixture_centers,
    database_chunk,
    zipf_probabilities,
    zipf_center_choice,
    make_queries,
)
from .index_build import IvfPqIndexData, build_index  # noqa: F401
