"""The coarse quantizer's entry point that allocates nothing
(ivf_coarse_probe_dev_noalloc, intermediates in the library's file-scope device
array) against ivf_coarse_probe_dev (intermediates in the index's workspace):
the probe lists are integers and must be equal bit for bit."""
import os

import numpy as np
import pytest

from synthdata import SPECS, build_index, make_queries, mixture_centers

pytestmark = pytest.mark.gpu


def _say(msg):
    print(f"[gpu-test] {msg}", flush=True)


@pytest.fixture(scope="module")
def pkg():
    import torch
    assert torch.cuda.is_available(), "these tests need the GPU"
    import paper_2504_08930_amd as p
    assert os.path.exists(p.LIB_PATH), "build the library before running GPU tests"
    p.load_library()
    return p


@pytest.mark.parametrize("name", ["T_IP96", "T_L2"])
def test_noalloc_coarse_probe_equals_the_workspace_one(pkg, name):
    """Two calls in a row through the C ABI, the second with a smaller batch (the array
    keeps the first call's contents), then a third at another nprobe; each compared with
    the existing entry point on the same queries.  A second index on the same GPU shares
    the array: calls alternate between the two."""
    import torch
    spec = SPECS[name]
    ix = build_index(spec, device="cuda")
    centers = mixture_centers(spec, torch.device("cuda"))
    big, _ = make_queries(spec, centers, nq=200, seed=spec.seed_queries + 3)
    index = pkg.IvfIndex(ix, max_nq=256, max_nprobe=ix.nlist, max_k=16)
    other = pkg.IvfIndex(ix, max_nq=256, max_nprobe=ix.nlist, max_k=16)
    for which, nq, nprobe in ((index, 200, spec.nprobe), (index, 37, spec.nprobe),
                              (other, 64, ix.nlist), (index, 5, 1), (other, 200, 3)):
        _say(f"{name}: no-alloc coarse probe nq={nq} nprobe={nprobe}")
        qd = big[:nq].contiguous()
        want = which.coarse_probe_dev(qd, nprobe)
        out = torch.full((nq, nprobe), -7, dtype=torch.int32, device="cuda")
        got = pkg.ivf_coarse_probe_dev_noalloc(which, qd, nprobe, out)
        torch.cuda.synchronize()
        assert got.data_ptr() == out.data_ptr()
        assert np.array_equal(got.cpu().numpy(), want.cpu().numpy()), (nq, nprobe)
    index.close()
    other.close()


def test_noalloc_coarse_probe_rejects_what_does_not_fit(pkg):
    """A batch whose intermediates exceed the array is refused with IVF_EINVAL before
    anything is launched, and the output is left alone; the largest batch that fits
    still works."""
    import torch
    from synthdata.workloads import METRIC_L2, WorkloadSpec
    spec = WorkloadSpec("S20k", 60_000, 16, 512, 20_000, 16, METRIC_L2, False,
                        24, 40, 10, None, 1.0, kmeans_iters=2)
    ix = build_index(spec, device="cuda")
    centers = mixture_centers(spec, torch.device("cuda"))
    index = pkg.IvfIndex(ix, max_nq=512, max_nprobe=64, max_k=16)

    def need(nq):
        r = lambda x: (x + 255) & ~255
        return r(nq * ix.d * 4 + 16384) + r(nq * 4) + r(nq * ix.nlist * 4)
    limit = 32 << 20
    fits = max(n for n in range(1, 600) if need(n) <= limit)
    assert need(fits + 1) > limit and fits < 512
    q, _ = make_queries(spec, centers, nq=fits + 1, seed=spec.seed_queries + 5)
    out = torch.full((fits + 1, spec.nprobe), -7, dtype=torch.int32, device="cuda")
    with pytest.raises(pkg.IvfError) as e:
        pkg.ivf_coarse_probe_dev_noalloc(index, q.contiguous(), spec.nprobe, out)
    assert e.value.code == -1 and "static scratch" in str(e.value)
    torch.cuda.synchronize()
    assert (out == -7).all()
    _say(f"largest batch that fits the array at nlist={ix.nlist}: {fits}")
    qd = q[:fits].contiguous()
    got = pkg.ivf_coarse_probe_dev_noalloc(index, qd, spec.nprobe, out[:fits].contiguous())
    want = index.coarse_probe_dev(qd, spec.nprobe)
    torch.cuda.synchronize()
    assert np.array_equal(got.cpu().numpy(), want.cpu().numpy())
    index.close()
