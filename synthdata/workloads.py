"""Named workload shapes.

The paper measures on Wiki-All (88M x 768-d) and ORCAS/Wikipedia indexes
(Section 5.1) with heavily skewed cluster access (Section 3.2).  Those
datasets are not available, so seeded Gaussian-mixture embeddings with
Zipf-distributed query-to-cluster choice stand in for them.
"""
from dataclasses import dataclass, replace
from typing import Optional

METRIC_L2 = 0
METRIC_IP = 1


@dataclass(frozen=True)
class WorkloadSpec:
    name: str
    n: int                 # database vectors
    d: int                 # dimensions
    n_centers: int         # mixture components
    nlist: int             # IVF clusters
    m: int                 # PQ sub-quantizers (8-bit codes)
    metric: int            # METRIC_L2 / METRIC_IP
    normalize: bool        # unit-normalise vectors and queries
    nq: int
    nprobe: int
    k: int
    zipf_s: Optional[float]   # None: uniform centre choice for queries
    resident_frac: float      # fraction of clusters (by count) placed on the GPU
    sigma: float = 0.3
    kmeans_iters: int = 10
    seed_data: int = 1234
    seed_kmeans: int = 2345
    seed_pq: int = 3456
    seed_queries: int = 4567
    seed_perm: int = 5678
    seed_calib: int = 6789

    def with_(self, **kw) -> "WorkloadSpec":
        return replace(self, **kw)


SPECS = {
    # tiny L2 config: everything resident
    "C1": WorkloadSpec("C1", 100_000, 128, 1024, 1024, 16, METRIC_L2, False,
                       100, 16, 10, None, 1.0),
    # 1M x 768 IP, hottest 30 % resident
    "C2": WorkloadSpec("C2", 1_000_000, 768, 4096, 4096, 64, METRIC_IP, True,
                       1000, 32, 10, 1.0, 0.30),
    # 10M x 768 IP: the configuration the roofline target is quoted on
    "C3": WorkloadSpec("C3", 10_000_000, 768, 16384, 16384, 96, METRIC_IP, True,
                       1024, 64, 10, 1.0, 1.0),
    # 100M x 768 IP
    "C4": WorkloadSpec("C4", 100_000_000, 768, 65536, 65536, 96, METRIC_IP, True,
                       4096, 128, 100, 1.0, 1.0),
    # scaled-down stand-in for the 100M config's search parameters (nprobe=128, k=100)
    "C4S": WorkloadSpec("C4S", 4_000_000, 768, 4096, 4096, 96, METRIC_IP, True,
                        512, 128, 100, 1.0, 1.0),
    # small shapes for CPU-only tests and smoke runs
    "T_L2": WorkloadSpec("T_L2", 6_000, 32, 48, 48, 16, METRIC_L2, False,
                         24, 6, 10, None, 1.0, kmeans_iters=4),
    "T_IP": WorkloadSpec("T_IP", 8_000, 64, 64, 64, 32, METRIC_IP, True,
                         32, 8, 10, 1.0, 0.3, kmeans_iters=4),
    "T_IP96": WorkloadSpec("T_IP96", 20_000, 192, 96, 96, 96, METRIC_IP, True,
                           40, 12, 10, 1.0, 0.3, kmeans_iters=4),
}


def get_spec(name: str) -> WorkloadSpec:
    return SPECS[name]
