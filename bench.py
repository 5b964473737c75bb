#!/usr/bin/env python3
"""Benchmark of the IVF-PQ hot path on one MI355X.

A step is one pass of the whole hot path over one query batch that is already
resident in HBM: coarse quantizer (MFMA contraction + per-query top-nprobe),
routing through the mapping table, per-query lookup tables, ADC scan of the
resident inverted lists with in-block top-k, per-query merge.  The workload is
the 10M-vector configuration (N = 10M, D = 768, nlist = 16384, PQ 96 x 8 bit,
inner product, nq = 1024, nprobe = 64, k = 10, Zipf(1.0) query-to-cluster
choice), seeded and synthetic, with every cluster GPU-resident.

Prints ONE JSON line.  `roofline` is for the ADC-scan kernel: algorithmic bytes
(sum over (query, resident probe) pairs of M * list length) per launch over
that kernel's average duration, taken from HIP events recorded on the search
stream inside the timed region.  `cpu_baseline` is the oracle (oracle/) timed on
this machine's host cores on a bounded sample of the same queries.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

METRIC = "search queries/sec at fixed nprobe,k; ADC-scan HBM GB/s as % of peak"
HBM_PEAK_GBS = 8000.0
# HBM-side bytes per k_scan launch from the rocprofv3 --pmc runs (FETCH_SIZE + WRITE_SIZE, scaled
# by the same counters on a plain copy kernel); valid for exactly this workload and launch shape.
MEASURED_TRAFFIC = {
    ("C3", 1024, 1.0): (4.057e9 + 0.164e6, "profiles/c3_nq1024_scan_hbm_traffic.md"),
}


def log(msg):
    print(f"[bench] {msg}", file=sys.stderr, flush=True)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="C3", help="spec name in synthdata.SPECS")
    ap.add_argument("--nq", type=int, default=None)
    ap.add_argument("--slices", type=int, default=0, help="scan blocks per query (0 = auto)")
    ap.add_argument("--resident", type=float, default=1.0,
                    help="fraction of clusters (hottest first) kept on the GPU")
    ap.add_argument("--oracle-sample", type=int, default=256)
    ap.add_argument("--no-oracle", action="store_true")
    ap.add_argument("--calib-copy", action="store_true",
                    help="also launch one 1 GiB streaming copy kernel (counter calibration)")
    ap.add_argument("--no-timing", action="store_true",
                    help="do not record per-kernel HIP events in the timed region")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on exactly one GPU (no sharding, no collectives); "
              "use --gpus 1", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    import paper_2504_08930_amd as pkg
    from synthdata import SPECS, build_index, make_queries, mixture_centers

    if not torch.cuda.is_available():
        print("bench.py needs a GPU", file=sys.stderr)
        sys.exit(1)
    if not os.path.exists(pkg.LIB_PATH):
        from paper_2504_08930_amd.build import build
        build()
    dev = torch.device("cuda:0")
    spec = SPECS[args.workload]
    nq = args.nq or spec.nq

    t0 = time.time()
    ix = build_index(spec, device="cuda:0", progress=log)
    centers = mixture_centers(spec, dev)
    q, _ = make_queries(spec, centers, nq=nq)
    calib, _ = make_queries(spec, centers, nq=max(nq, 1024), seed=spec.seed_calib)
    q = q.contiguous()
    torch.cuda.synchronize()
    log(f"index built in {time.time() - t0:.1f}s: N={ix.n} nlist={ix.nlist} M={ix.m}")

    index = pkg.IvfIndex(ix, max_nq=max(nq, 1024), max_nprobe=spec.nprobe, max_k=spec.k)
    t0 = time.time()
    index.load_partition(np.arange(ix.nlist, dtype=np.int32))
    load_s = time.time() - t0
    log(f"loaded all clusters in {load_s:.2f}s ({index.arena_bytes / 2**30:.2f} GiB arena)")
    resident_frac = 1.0
    if args.resident < 1.0:
        index.hit_stats(reset=True)
        for s in range(0, calib.shape[0], index.max_nq):
            index.search_batch_dev(calib[s:s + index.max_nq].contiguous(), spec.nprobe, 1)
        torch.cuda.synchronize()
        hits = index.hit_stats(reset=True)["per_cluster_hits"].astype(np.int64)
        order = np.lexsort((np.arange(ix.nlist), -hits))
        hot = np.sort(order[: int(round(args.resident * ix.nlist))]).astype(np.int32)
        index.load_partition(hot)
        resident_frac = len(hot) / ix.nlist

    index.set_tuning(scan_slices=args.slices, timing=False)
    out_ids = torch.empty((nq, spec.k), dtype=torch.int64, device=dev)
    out_d = torch.empty((nq, spec.k), dtype=torch.float32, device=dev)
    stream = torch.cuda.current_stream(dev)

    def step():
        index.search_batch_dev(q, spec.nprobe, spec.k, out_ids, out_d, stream)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    index.hit_stats(reset=True)
    index.set_tuning(scan_slices=args.slices, timing=not args.no_timing)
    index.stage_times(reset=True)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    st = index.stage_times(reset=True)
    hs = index.hit_stats()
    index.set_tuning(scan_slices=args.slices, timing=False)

    if args.calib_copy:
        from paper_2504_08930_amd.binding import ivf_calib_copy
        src = torch.ones(1 << 28, dtype=torch.float32, device=dev)      # 1 GiB
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        ivf_calib_copy(src, dst, stream)
        torch.cuda.synchronize()
        del src, dst

    ms_per_step = 1e3 * elapsed / args.steps
    qps = nq * args.steps / elapsed
    roofline = None
    if not args.no_timing and st["launches"]["scan"] > 0:
        n_scan = st["launches"]["scan"]
        scan_ms = st["ms"]["scan"] / n_scan
        bytes_per_launch = st["scan_bytes"] / n_scan
        achieved = bytes_per_launch / (scan_ms * 1e-3) / 1e9
        roofline = {"bound": "hbm", "kernel": "k_scan", "achieved": round(achieved, 1),
                    "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": round(achieved / HBM_PEAK_GBS, 4),
                    "traffic": None, "bytes_per_launch": int(bytes_per_launch),
                    "avg_launch_ms": round(scan_ms, 4)}
        key = (spec.name, nq, round(resident_frac, 4))
        if key in MEASURED_TRAFFIC and args.slices == 0:
            roofline["traffic"], roofline["traffic_source"] = MEASURED_TRAFFIC[key]
    stage_ms = {k: round(v / max(1, st["launches"][k]), 4) for k, v in st["ms"].items()}

    cpu_baseline = None
    parity = None
    if not args.no_oracle:
        from oracle import oracle as orc
        from tests.parity import compare_probes, compare_topk, scale_S
        orc.build()
        ns = min(args.oracle_sample, nq)
        sel = np.linspace(0, nq - 1, ns).astype(np.int64)
        qs = q[torch.from_numpy(sel).to(dev)].cpu().numpy()
        t0 = time.perf_counter()
        probe_ext, score_ext, _ = orc.coarse(ix.metric, ix.centroids, qs, spec.nprobe + 8)
        probe = np.ascontiguousarray(probe_ext[:, :spec.nprobe])
        ref_i, ref_d = orc.scan(ix.metric, ix.codebooks, ix.list_offsets, ix.codes, ix.ids, qs,
                                probe, spec.k + 16)
        cpu_s = time.perf_counter() - t0
        cpu_baseline = {"value": round(ns / cpu_s, 2), "unit": "queries/s",
                        "cores": orc.num_threads(), "kind": "oracle",
                        "sample": f"{ns} of the {nq} queries, same index, nprobe={spec.nprobe}, "
                                  f"k={spec.k}; brute-force coarse + decode-and-distance in fp64"}
        # parity of the timed configuration on the same sample
        got_i = out_ids.cpu().numpy()[sel]
        got_d = out_d.cpu().numpy()[sel]
        got_probe = index.coarse_probe_dev(q, spec.nprobe).cpu().numpy()[sel]
        S = scale_S(ix.metric, qs)
        n_coarse = compare_probes(got_probe, probe_ext, score_ext, spec.nprobe, S)
        if n_coarse:
            ref_i, ref_d = orc.scan(ix.metric, ix.codebooks, ix.list_offsets, ix.codes, ix.ids,
                                    qs, got_probe, spec.k + 16)
        n_amb = compare_topk(got_i, got_d, ref_i, ref_d, spec.k, S)
        parity = {"queries_checked": int(ns), "coarse_ambiguous": int(n_coarse),
                  "id_ambiguous": int(n_amb), "pass": True}

    out = {
        "metric": METRIC,
        "value": round(qps, 1),
        "unit": "queries/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f32 table, i32 accumulate",
        "data": "synthetic",
        "config": {"workload": f"{spec.name}: N={spec.n} D={spec.d} nlist={spec.nlist} "
                               f"PQ{spec.m}x8 IP nq={nq} nprobe={spec.nprobe} k={spec.k} "
                               f"zipf_s={spec.zipf_s}",
                   "resident_fraction": round(resident_frac, 4),
                   "mean_hit_rate": round(hs["mean_hit_rate"], 4),
                   "scan_slices": args.slices, "inputs": "device-resident queries"},
        "roofline": roofline,
        "cpu_baseline": cpu_baseline,
        "stage_ms": stage_ms,
        "parity": parity,
        "index_build_s": None,
        "load_partition_s": round(load_s, 3),
    }
    index.close()
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
