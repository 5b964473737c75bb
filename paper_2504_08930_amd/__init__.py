"""MI355X-native IVF-PQ search over the GPU-resident hot-cluster partition of an
inverted-file index (after VectorLiteRAG, arXiv 2504.08930).

`binding` wraps the C ABI declared in include/ivfpq_hot.h; the functions below
carry the same names as the C entry points and only marshal arguments.
"""
from .binding import (  # noqa: F401
    IVF_METRIC_IP, IVF_METRIC_L2, IvfError, IvfIndex, load_library, LIB_PATH, EXPORTS,
)


def ivf_index_create(data, max_nq, max_nprobe, max_k, **kw):
    return IvfIndex(data, max_nq, max_nprobe, max_k, **kw)


def ivf_index_destroy(index):
    index.close()


def ivf_index_load_partition(index, cluster_ids, stream=None):
    return index.load_partition(cluster_ids, stream)


def ivf_search_batch(index, queries, nprobe, k):
    return index.search_batch(queries, nprobe, k)


def ivf_search_batch_dev(index, queries, nprobe, k, out_ids=None, out_dists=None, stream=None):
    return index.search_batch_dev(queries, nprobe, k, out_ids, out_dists, stream)


def ivf_coarse_probe_dev(index, queries, nprobe, stream=None):
    return index.coarse_probe_dev(queries, nprobe, stream)


def ivf_coarse_probe_dev_noalloc(index, queries, nprobe, out, stream=None):
    return index.coarse_probe_dev_noalloc(queries, nprobe, out, stream)


def ivf_search_batch_probes(index, queries, probe, k):
    return index.search_batch_probes(queries, probe, k)


def ivf_search_batch_async(index, queries, nprobe, k, probe=None, on_done=None):
    return index.search_batch_async(queries, nprobe, k, probe, on_done)


def ivf_search_poll(ticket, cap=None):
    return ticket.poll(cap)


def ivf_search_wait(ticket):
    return ticket.wait()


def ivf_hit_stats(index, reset=False):
    return index.hit_stats(reset)


def ivf_migrate_clusters(index, evict, admit, side_stream=None):
    return index.migrate_clusters(evict, admit, side_stream)


def ivf_hit_rate_moments(index):
    return index.hit_rate_moments()


def ivf_weighted_hit_rate(index):
    return index.weighted_hit_rate()


def ivf_profile_curves(index):
    return index.profile_curves()


def ivf_refresh_hot_set(index, n_hot, reset=True, side_stream=None):
    return index.refresh_hot_set(n_hot, reset, side_stream)


def ivf_migrate_poll(index, wait=False):
    return index.migrate_poll(wait)


def ivf_resident_list(index):
    return index.resident_list()


def ivf_host_scan_form(index):
    return index.host_scan_form()


def ivf_copy_form(index):
    return index.copy_form()
