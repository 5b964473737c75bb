"""Index fixture builder: trains and fills an IVF-PQ index from the synthetic
database (Section 2.1: k-means centroids, one inverted list per centroid,
PQ codes with a trained code-book).

This is input preparation for the search path, not part of it: the oracle
and the HIP library both *consume* the arrays produced here.  torch matmuls
are used freely (CPU or GPU).  Choices the paper leaves open are fixed here:
k-means is initialised from a seeded random sample, trained on the first
64 * nlist vectors (rounded up to a generator chunk), PQ on at most 65536 of
them; an empty cluster keeps its centroid.
"""
from dataclasses import dataclass

import numpy as np
import torch

from .generate import GEN_CHUNK, database_chunk, mixture_centers
from .workloads import METRIC_IP, WorkloadSpec


@dataclass
class IvfPqIndexData:
    d: int
    nlist: int
    m: int
    metric: int
    centroids: np.ndarray      # fp32 [nlist, d]
    codebooks: np.ndarray      # fp32 [m, 2**nbits, d/m]
    list_offsets: np.ndarray   # int64 [nlist+1]
    codes: np.ndarray          # uint8 [n, m * nbits / 8], list-contiguous
    ids: np.ndarray            # int64 [n], database id of each stored code
    n: int
    by_residual: bool = False  # codes encode x - centroid of its list
    nbits: int = 8             # bits per code; 4: two codes per byte, even sub-quantizer low

    @property
    def dsub(self) -> int:
        return self.d // self.m

    def list_len(self, c: int) -> int:
        return int(self.list_offsets[c + 1] - self.list_offsets[c])


def _best_centroid(x, cent, spherical: bool, chunk: int):
    """Index of the best centroid for each row of x (fp32 matmul)."""
    out = torch.empty(x.shape[0], dtype=torch.int64, device=x.device)
    cn = None if spherical else (cent * cent).sum(1)
    for s in range(0, x.shape[0], chunk):
        xs = x[s:s + chunk]
        dots = xs @ cent.t()
        if spherical:
            out[s:s + chunk] = dots.argmax(1)
        else:
            out[s:s + chunk] = (cn[None, :] - 2.0 * dots).argmin(1)
    return out


def _kmeans(x, k, iters, spherical, seed, chunk):
    g = torch.Generator(device="cpu")
    g.manual_seed(seed)
    perm = torch.randperm(x.shape[0], generator=g)[:k].to(x.device)
    cent = x[perm].clone()
    for _ in range(iters):
        a = _best_centroid(x, cent, spherical, chunk)
        # sums in fp64: on a GPU index_add_ adds with atomics in no fixed order, and
        # in fp64 the order no longer shows in the fp32 result (same index every run)
        sums = torch.zeros(cent.shape, dtype=torch.float64, device=x.device)
        for s in range(0, x.shape[0], chunk):
            sums.index_add_(0, a[s:s + chunk], x[s:s + chunk].double())
        cnt = torch.bincount(a, minlength=k).double()
        new = (sums / cnt.clamp_min(1.0)[:, None]).to(x.dtype)
        keep = cnt == 0
        new[keep] = cent[keep]          # an empty cluster keeps its centroid
        if spherical:
            new = new / new.norm(dim=1, keepdim=True).clamp_min(1e-20)
        cent = new
    return cent.contiguous()


def _train_pq(x, m, iters, seed, ksub=256):
    """Per-sub-space k-means, ksub centroids each.  x: [n, d] -> [m, ksub, dsub]."""
    n, d = x.shape
    dsub = d // m
    xs = x.view(n, m, dsub).permute(1, 0, 2).contiguous()      # [m, n, dsub]
    g = torch.Generator(device="cpu")
    g.manual_seed(seed)
    perm = torch.randperm(n, generator=g)[:ksub].to(x.device)
    cb = xs[:, perm, :].clone()                                 # [m, ksub, dsub]
    base = (torch.arange(m, device=x.device) * ksub)[:, None]
    for _ in range(iters):
        dist = (cb * cb).sum(2)[:, None, :] - 2.0 * torch.bmm(xs, cb.transpose(1, 2))
        a = dist.argmin(2)                                      # [m, n]
        flat = (a + base).reshape(-1)
        sums = torch.zeros(m * ksub, dsub, device=x.device, dtype=torch.float64)  # see _kmeans
        sums.index_add_(0, flat, xs.reshape(-1, dsub).double())
        cnt = torch.bincount(flat, minlength=m * ksub).double()
        new = (sums / cnt.clamp_min(1.0)[:, None]).to(x.dtype).view(m, ksub, dsub)
        keep = (cnt == 0).view(m, ksub)
        new[keep] = cb[keep]
        cb = new
    return cb.contiguous()


def _encode(x, cb):
    """Arg-min code per sub-space.  x [b, d], cb [m, ksub, dsub] -> uint8 [b, m], or
    [b, m / 2] when ksub is 16 (two codes per byte, the even sub-quantizer in the low half)."""
    m, ksub, dsub = cb.shape
    xs = x.view(x.shape[0], m, dsub).permute(1, 0, 2)            # [m, b, dsub]
    dist = (cb * cb).sum(2)[:, None, :] - 2.0 * torch.bmm(xs, cb.transpose(1, 2))
    codes = dist.argmin(2).t().contiguous().to(torch.uint8)
    if ksub == 16:
        codes = (codes[:, 0::2] | (codes[:, 1::2] << 4)).contiguous()
    return codes


def build_index(spec: WorkloadSpec, device="cpu", progress=None,
                by_residual: bool = False, nbits: int = 8, m: int = None) -> IvfPqIndexData:
    """Generate the database chunk by chunk, train, assign, encode, and lay the
    codes out list by list.  Returns host (numpy) arrays.  nbits = 4 trains 16
    codewords per sub-quantizer and packs two codes per byte; m overrides the
    spec's number of sub-quantizers."""
    m = spec.m if m is None else m
    assert nbits in (4, 8) and spec.d % m == 0 and (nbits == 8 or m % 2 == 0)
    dev = torch.device(device)
    on_gpu = dev.type == "cuda"
    say = progress if progress is not None else (lambda *_: None)
    centers = mixture_centers(spec, dev)
    spherical = spec.metric == METRIC_IP and spec.normalize

    n_train = min(spec.n, 64 * spec.nlist)
    n_train = -(-n_train // GEN_CHUNK) * GEN_CHUNK if n_train < spec.n else spec.n
    n_train = min(n_train, spec.n)
    train = database_chunk(spec, centers, 0, n_train)
    mm_chunk = 65536 if on_gpu else 8192
    say(f"kmeans nlist={spec.nlist} on {n_train} vectors")
    centroids = _kmeans(train, spec.nlist, spec.kmeans_iters, spherical,
                        spec.seed_kmeans, mm_chunk)
    n_pq = min(n_train, 65536)
    say(f"pq train m={m} x {nbits} bits on {n_pq} vectors")
    pq_train = train[:n_pq].contiguous()
    if by_residual:
        pq_train = pq_train - centroids[_best_centroid(pq_train, centroids, spherical, mm_chunk)]
    codebooks = _train_pq(pq_train, m, spec.kmeans_iters, spec.seed_pq, 1 << nbits)
    del pq_train
    del train

    assign = torch.empty(spec.n, dtype=torch.int32, device=dev)
    codes = torch.empty(spec.n, m * nbits // 8, dtype=torch.uint8, device=dev)
    step = GEN_CHUNK * (4 if on_gpu else 1)
    enc_chunk = 32768 if on_gpu else 2048
    for s in range(0, spec.n, step):
        cnt = min(step, spec.n - s)
        x = database_chunk(spec, centers, s, cnt)
        a = _best_centroid(x, centroids, spherical, mm_chunk)
        assign[s:s + cnt] = a.to(torch.int32)
        if by_residual:
            x = x - centroids[a]
        for e in range(0, cnt, enc_chunk):
            codes[s + e:s + e + enc_chunk] = _encode(x[e:e + enc_chunk], codebooks)
        if (s // step) % 8 == 0:
            say(f"assign+encode {s + cnt}/{spec.n}")
    order = torch.sort(assign.to(torch.int64), stable=True).indices
    counts = torch.bincount(assign.to(torch.int64), minlength=spec.nlist)
    offsets = torch.zeros(spec.nlist + 1, dtype=torch.int64, device=dev)
    offsets[1:] = torch.cumsum(counts, 0)
    codes = codes[order].contiguous()
    return IvfPqIndexData(
        d=spec.d, nlist=spec.nlist, m=m, metric=spec.metric,
        centroids=centroids.cpu().numpy(),
        codebooks=codebooks.cpu().numpy(),
        list_offsets=offsets.cpu().numpy(),
        codes=codes.cpu().numpy(),
        ids=order.cpu().numpy().astype(np.int64),
        n=spec.n,
        by_residual=by_residual,
        nbits=nbits,
    )
