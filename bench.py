#!/usr/bin/env python3
"""Benchmark of the IVF-PQ hot path on one MI355X.

Default mode ("hotpath"): a step is one pass of the whole hot path over one
query batch that is already resident in HBM: coarse quantizer (split-fp16 MFMA
contraction + per-query top-nprobe), routing through the mapping table,
per-query lookup tables, ADC scan of the resident inverted lists with in-block
top-k, per-query merge.  The workload is the 10M-vector configuration (N = 10M,
D = 768, nlist = 16384, PQ 96 x 8 bit, inner product, nq = 1024, nprobe = 64,
k = 10, Zipf(1.0) query-to-cluster choice), seeded and synthetic, with every
cluster GPU-resident.  Prints ONE JSON line.  `roofline` is for the ADC-scan
kernel: algorithmic bytes (sum over (query, resident probe) pairs of M * list
length) per launch over that kernel's average duration, taken from HIP events
recorded on the search stream inside the timed region.  `cpu_baseline` is the
oracle (oracle/) timed on this machine's host cores on a bounded sample of the same
queries.  `other_points` holds short passes over the configuration's other batch
sizes and resident fractions, run after the timed region.

Other modes (each prints one JSON line of its own):
  --mode sweep   nq in {256, 1024, 4096} x resident fraction in {0.1, 0.3, 0.5, 1.0}
  --mode partition  profile the access skew and the CPU tier, pick the partitioning point
                 rho with the latency-bounded model (Eq. 1, Eq. 2, Algorithm 1; synthetic LLM
                 inputs), load it and compare predicted with measured batch latency
  --mode dispatch  dynamic dispatcher on/off (Section 4.2.2): hybrid batches from host memory at
                 several resident fractions; batch latency and mean / p90 per-query hand-off
                 latency of ivf_search_batch_async against the bulk ivf_search_batch
  --mode drift   20 epochs x 10 000 queries, Zipf permutation re-drawn every 5
                 epochs, after every epoch ivf_refresh_hot_set re-ranks the clusters by the
                 router's counters and migrates to the new hot set while searches continue
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
# by the same counters on a plain copy kernel); valid for exactly this workload and launch shape,
# and for the scan kernel's sources as they were when the counters were read: each entry carries
# the hash of those sources (scan_source_hash), and a line measured on other sources reports
# no traffic figure rather than a stale one.
SCAN_SOURCES = ("kernels_scan.hip", "lut_quant.h", "internal.h")
MEASURED_TRAFFIC = {
    ("C3", 1024, 1.0): (3.0220e9 + 0.164e6, "profiles/c3_nq1024_scan_hbm_traffic.md",
                        "6c770ad915d5d1c5"),
    ("C3", 256, 1.0): (739.3e6 + 0.04e6, "profiles/c3_nq256_scan_hbm_traffic.md",
                       "6c770ad915d5d1c5"),
}


def scan_source_hash():
    """First 16 hex digits of the SHA-256 of the sources the scan kernel is built from."""
    import hashlib
    h = hashlib.sha256()
    for name in SCAN_SOURCES:
        with open(os.path.join(ROOT, "paper_2504_08930_amd", "csrc", name), "rb") as f:
            h.update(f.read())
    return h.hexdigest()[:16]


def log(msg):
    print(f"[bench] {msg}", file=sys.stderr, flush=True)


def hottest_clusters(index, calib, nprobe, frac, nlist):
    """Hottest round(frac * nlist) clusters by probe count over calibration queries."""
    import numpy as np
    import torch
    index.hit_stats(reset=True)
    for s in range(0, calib.shape[0], index.max_nq):
        index.search_batch_dev(calib[s:s + index.max_nq].contiguous(), nprobe, 1)
    torch.cuda.synchronize()
    hits = index.hit_stats(reset=True)["per_cluster_hits"].astype(np.int64)
    order = np.lexsort((np.arange(nlist), -hits))
    return np.sort(order[: int(round(frac * nlist))]).astype(np.int32)


def timed_steps(index, q, nprobe, k, steps, warmup, slices, timing=2, n_streams=1):
    """Warm up, then time `steps` searches of the device-resident batch q.  With
    n_streams = 2 consecutive steps go to alternating streams (the library keeps
    one workspace per stream), so one batch's coarse stage can overlap the
    previous batch's scan; every step still does the whole path."""
    import torch
    dev = q.device
    nq = q.shape[0]
    if n_streams <= 1:
        streams = [torch.cuda.current_stream(dev)]
    else:
        streams = [torch.cuda.Stream(device=dev) for _ in range(n_streams)]
    outs = [(torch.empty((nq, k), dtype=torch.int64, device=dev),
             torch.empty((nq, k), dtype=torch.float32, device=dev)) for _ in streams]
    out_ids, out_d = outs[0]
    timing = int(timing)
    index.set_tuning(scan_slices=slices, timing=0)
    torch.cuda.synchronize()
    for i in range(warmup):
        j = i % len(streams)
        index.search_batch_dev(q, nprobe, k, outs[j][0], outs[j][1], streams[j])
    torch.cuda.synchronize()
    index.hit_stats(reset=True)
    index.set_tuning(scan_slices=slices, timing=timing)
    index.stage_times(reset=True)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(steps):
        j = i % len(streams)
        index.search_batch_dev(q, nprobe, k, outs[j][0], outs[j][1], streams[j])
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    st = index.stage_times(reset=True)
    hs = index.hit_stats()
    weighted = index.weighted_hit_rate()[0]
    index.set_tuning(scan_slices=slices, timing=0)
    res = {"elapsed": elapsed, "ms_per_step": 1e3 * elapsed / steps,
           "qps": nq * steps / elapsed, "hit_rate": hs["mean_hit_rate"],
           "min_hit_rate": hs["min_hit_rate"], "bytes_hit_rate": weighted, "stage": st,
           "out_ids": out_ids, "out_d": out_d}
    n_scan = st["launches"]["scan"]
    if timing and n_scan > 0:
        scan_ms = st["ms"]["scan"] / n_scan
        res["scan_ms"] = scan_ms
        res["scan_bytes_per_launch"] = st["scan_bytes"] / n_scan
        res["scan_gbs"] = res["scan_bytes_per_launch"] / (scan_ms * 1e-3) / 1e9
    res["stage_ms"] = {s: round(v / max(1, st["launches"][s]), 4) for s, v in st["ms"].items()
                       if st["launches"][s] > 0}
    return res


def measure_read_ceiling(dev, with_copy=False, launches=100):
    """GB/s of the library's plain streaming-read kernel over a 1 GiB buffer (HIP events on
    the launch stream): `launches` timed launches (about 20 ms of sustained reading, so the
    figure is the rate at the GPU's sustained clock, not at the clock of an idle one) after
    ten untimed ones.  with_copy: also launch the 1 GiB copy kernel once (the launch the
    byte counters are calibrated on when this script runs under rocprofv3 --pmc)."""
    import torch
    from paper_2504_08930_amd.binding import ivf_calib_copy, ivf_calib_read
    src = torch.ones(1 << 28, dtype=torch.float32, device=dev)      # 1 GiB
    sink = torch.empty(1 << 20, dtype=torch.int32, device=dev)
    stream = torch.cuda.current_stream(dev)
    torch.cuda.synchronize()
    if with_copy:
        dst = torch.empty_like(src)
        ivf_calib_copy(src, dst, stream)
        torch.cuda.synchronize()
        del dst
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    for _ in range(10):
        ivf_calib_read(src, sink, stream)
    e0.record(stream)
    for _ in range(launches):
        ivf_calib_read(src, sink, stream)
    e1.record(stream)
    torch.cuda.synchronize()
    return round(launches * (1 << 30) / (e0.elapsed_time(e1) * 1e-3) / 1e9, 1)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=50)
    ap.add_argument("--mode", default="hotpath",
                    choices=["hotpath", "sweep", "drift", "partition", "dispatch"])
    ap.add_argument("--workload", default="C3", help="spec name in synthdata.SPECS")
    ap.add_argument("--nq", type=int, default=None)
    ap.add_argument("--nprobe", type=int, default=0, help="override the workload's nprobe")
    ap.add_argument("--k", type=int, default=0, help="override the workload's k")
    ap.add_argument("--slices", type=int, default=0, help="scan blocks per query (0 = auto)")
    ap.add_argument("--streams", type=int, default=1,
                    help="issue consecutive steps on this many alternating streams (1 or 2)")
    ap.add_argument("--two-streams-pass", action="store_true",
                    help="after the timed region, also time the same steps issued on two "
                         "alternating streams (off by default: the overlapped launches would "
                         "blur the per-kernel times of a profile of this command)")
    ap.add_argument("--nbits", type=int, default=8, choices=[4, 8],
                    help="bits per PQ code (4: two codes per byte)")
    ap.add_argument("--m", type=int, default=0,
                    help="PQ sub-quantizers (default: the workload's; e.g. 192 with --nbits 4 keeps "
                         "C3's 96 bytes per vector)")
    ap.add_argument("--residual", action="store_true",
                    help="index whose PQ codes encode x - centroid (residual encoding)")
    ap.add_argument("--resident", type=float, default=1.0,
                    help="fraction of clusters (hottest first) kept on the GPU")
    ap.add_argument("--oracle-sample", type=int, default=512)
    ap.add_argument("--no-oracle", action="store_true")
    ap.add_argument("--no-other-points", action="store_true",
                    help="default mode: leave out the short passes over the configuration's other "
                         "batch sizes and resident fractions (other_points in the line)")
    ap.add_argument("--calib-copy", action="store_true",
                    help="also launch one 1 GiB streaming copy and a few 1 GiB streaming read "
                         "kernels (counter calibration / read ceiling)")
    ap.add_argument("--no-timing", action="store_true",
                    help="record no HIP events in the timed region (no roofline figure)")
    ap.add_argument("--stage-timing", action="store_true",
                    help="record HIP events around every stage in the timed region instead of "
                         "around the scan only (each event costs a few microseconds per step)")
    ap.add_argument("--nq-list", default="256,1024,4096", help="sweep mode: batch sizes")
    ap.add_argument("--resident-list", default="1.0,0.5,0.3,0.1",
                    help="sweep mode: resident fractions")
    ap.add_argument("--slo-ms", type=float, default=10.0,
                    help="partition mode: search latency target SLO_search in ms")
    ap.add_argument("--epochs", type=int, default=20, help="drift mode: epochs")
    ap.add_argument("--epoch-queries", type=int, default=10000, help="drift mode: queries/epoch")
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
    if args.nprobe or args.k:
        spec = spec.with_(nprobe=args.nprobe or spec.nprobe, k=args.k or spec.k)
    nq = args.nq or spec.nq

    t0 = time.time()
    ix = build_index(spec, device="cuda:0", progress=log, by_residual=args.residual,
                     nbits=args.nbits, m=args.m or None)
    centers = mixture_centers(spec, dev)
    torch.cuda.synchronize()
    build_s = time.time() - t0
    log(f"index built in {build_s:.1f}s: N={ix.n} nlist={ix.nlist} M={ix.m}")
    nq_list = [int(x) for x in args.nq_list.split(",")]
    max_nq = max(nq, max(nq_list) if args.mode == "sweep" else 1024)
    index = pkg.IvfIndex(ix, max_nq=max_nq, max_nprobe=spec.nprobe, max_k=spec.k)
    t0 = time.time()
    all_clusters = np.arange(ix.nlist, dtype=np.int32)
    index.load_partition(all_clusters)
    load_s = time.time() - t0
    log(f"loaded all clusters in {load_s:.2f}s ({index.arena_bytes / 2**30:.2f} GiB arena)")
    calib, _ = make_queries(spec, centers, nq=4096, seed=spec.seed_calib)

    workload = (f"{spec.name}{' (residual-encoded)' if args.residual else ''}: "
                f"N={spec.n} D={spec.d} nlist={spec.nlist} PQ{ix.m}x{ix.nbits} "
                f"{'IP' if spec.metric == 1 else 'L2'} nprobe={spec.nprobe} k={spec.k} "
                f"zipf_s={spec.zipf_s}")

    if args.mode == "sweep":
        rows = []
        for frac in [float(x) for x in args.resident_list.split(",")]:
            if frac < 1.0:
                index.load_partition(all_clusters)
                index.load_partition(hottest_clusters(index, calib, spec.nprobe, frac, ix.nlist))
            for n in nq_list:
                q, _ = make_queries(spec, centers, nq=n)
                steps = min(args.steps, 50) if frac == 1.0 else 3
                r = timed_steps(index, q.contiguous(), spec.nprobe, spec.k, steps,
                                min(args.warmup, 20) if frac == 1.0 else 1, args.slices,
                                timing=1 if args.stage_timing else 2)
                row = {"nq": n, "resident_fraction": frac, "queries_per_s": round(r["qps"], 1),
                       "ms_per_step": round(r["ms_per_step"], 3),
                       "mean_hit_rate": round(r["hit_rate"], 4),
                       "min_hit_rate": round(r["min_hit_rate"], 4),
                       "bytes_hit_rate": round(r["bytes_hit_rate"], 4),
                       "scan_ms": round(r.get("scan_ms", 0.0), 4),
                       "scan_GBs": round(r.get("scan_gbs", 0.0), 1),
                       "scan_frac_of_peak": round(r.get("scan_gbs", 0.0) / HBM_PEAK_GBS, 4),
                       "stage_ms": r["stage_ms"]}
                log(json.dumps(row))
                rows.append(row)
        index.close()
        print(json.dumps({"mode": "sweep", "workload": workload, "unit": "queries/s",
                          "rows": rows}), flush=True)
        return

    if args.mode == "dispatch":
        rows = []
        reps = 5
        for frac in (0.9, 0.5, 0.3):
            index.load_partition(all_clusters)
            index.load_partition(hottest_clusters(index, calib, spec.nprobe, frac, ix.nlist))
            for n in (256, 1024):
                off_ms, on_ms, on_mean, on_p90, min_rate = [], [], [], [], []
                for rep in range(reps + 1):
                    qh = make_queries(spec, centers, nq=n,
                                      seed=spec.seed_queries + 100 + rep)[0].cpu().numpy()
                    index.hit_stats(reset=True)
                    t0 = time.perf_counter()
                    ref_i, ref_d = index.search_batch(qh, spec.nprobe, spec.k)
                    t_off = (time.perf_counter() - t0) * 1e3
                    mr = index.hit_stats(reset=True)["min_hit_rate"]
                    t0 = time.perf_counter()
                    ids, dists, done_ms = index.search_batch_async(qh, spec.nprobe, spec.k).wait()
                    t_on = (time.perf_counter() - t0) * 1e3
                    assert np.array_equal(ids, ref_i) and np.array_equal(dists, ref_d)
                    if rep == 0:
                        continue                      # warm-up pair
                    off_ms.append(t_off)
                    on_ms.append(t_on)
                    on_mean.append(float(done_ms.mean()))
                    on_p90.append(float(np.percentile(done_ms, 90)))
                    min_rate.append(mr)
                row = {"resident_fraction": frac, "nq": n,
                       "min_hit_rate": round(float(np.mean(min_rate)), 4),
                       "bulk_batch_ms": round(float(np.mean(off_ms)), 3),
                       "dispatcher_batch_ms": round(float(np.mean(on_ms)), 3),
                       "dispatcher_mean_query_ms": round(float(np.mean(on_mean)), 3),
                       "dispatcher_p90_query_ms": round(float(np.mean(on_p90)), 3)}
                row["mean_latency_change"] = round(row["dispatcher_mean_query_ms"] /
                                                   row["bulk_batch_ms"] - 1.0, 4)
                log(json.dumps(row))
                rows.append(row)
        index.close()
        print(json.dumps({"mode": "dispatch", "workload": workload, "reps": reps,
                          "note": "bulk: every query of a batch is available at bulk_batch_ms; "
                                  "dispatcher: query i at done_ms[i]; identical results asserted",
                          "rows": rows}), flush=True)
        return

    if args.mode == "partition":
        from paper_2504_08930_amd import binding as B
        nlist = ix.nlist
        # --- access profile from calibration queries (Section 4.1.1) ---
        def run_calibration():
            index.hit_stats(reset=True)
            for s0 in range(0, calib.shape[0], index.max_nq):
                index.search_batch_dev(calib[s0:s0 + index.max_nq].contiguous(), spec.nprobe, 1)
            torch.cuda.synchronize()
        run_calibration()
        # ranking (hottest first), cumulative hit share and cumulative device bytes
        order, hit_cdf, mem_index = index.profile_curves()
        # sigma_max^2, the constant of the variance model (Section 4.1.2), profiled where the mean
        # hit rate is one half: that share of the clusters resident, the same queries again,
        # and the spread of the per-query hit rate the router counted
        i_half = int(np.searchsorted(hit_cdf, 0.5))
        index.load_partition(np.sort(order[:i_half]).astype(np.int32))
        run_calibration()
        sigma_max2 = float(index.hit_rate_moments()["sigma_max2"])
        index.hit_stats(reset=True)
        # --- CPU-tier latency model: knots measured with nothing resident ---
        index.load_partition(np.zeros(0, np.int32))
        knots_b, t_cq, t_lut = [], [], []
        for b in (64, 256, 1024):
            qb, _ = make_queries(spec, centers, nq=b, seed=spec.seed_calib + 17)
            qh = qb.cpu().numpy()
            index.search_batch(qh, spec.nprobe, spec.k)
            index.set_tuning(scan_slices=0, timing=True)
            index.stage_times(reset=True)
            t0 = time.perf_counter()
            reps = 3
            for _ in range(reps):
                index.search_batch(qh, spec.nprobe, spec.k)
            total = (time.perf_counter() - t0) / reps
            st = index.stage_times(reset=True)
            index.set_tuning(scan_slices=0, timing=False)
            cq_s = sum(st["ms"][x] for x in ("coarse_gemm", "coarse_select", "route")) / reps * 1e-3
            knots_b.append(float(b))
            t_cq.append(cq_s)
            t_lut.append(max(total - cq_s, 1e-6))
        model = B.LatencyModel(knots_b, t_cq, t_lut)
        # --- Algorithm 1 with synthetic LLM-side inputs ---
        slo = args.slo_ms * 1e-3
        eps = 1.0
        tau_s = slo / (1 + eps)
        mu0 = 1024.0 / tau_s                     # bare LLM throughput that fills batches of 1024
        kv = 8.0 * mem_index[-1]                 # KV-cache bytes with no index loaded
        rho = B.ivf_model_partition_point(model, hit_cdf, mem_index, sigma_max2, slo, eps, kv, mu0,
                                          1.0 / 512)
        n_hot = int(round(rho * nlist))
        mu = (kv - mem_index[n_hot]) / kv * mu0
        batch = max(1, int(np.floor(tau_s * mu)))
        eta_pred = B.ivf_model_min_hit_rate(float(hit_cdf[n_hot]), sigma_max2, batch)
        lat_pred = B.ivf_model_hybrid_latency(model, batch, eta_pred)
        index.load_partition(np.sort(order[:n_hot]).astype(np.int32))
        lat, min_rates = [], []
        for rep in range(8):
            qb, _ = make_queries(spec, centers, nq=min(batch, index.max_nq),
                                 seed=spec.seed_queries + 50 + rep)
            qh = qb.cpu().numpy()
            index.hit_stats(reset=True)
            t0 = time.perf_counter()
            index.search_batch(qh, spec.nprobe, spec.k)
            lat.append(time.perf_counter() - t0)
            min_rates.append(index.hit_stats(reset=True)["min_hit_rate"])
        index.close()
        print(json.dumps({
            "mode": "partition", "workload": workload, "slo_search_ms": args.slo_ms, "eps": eps,
            "tau_s_ms": round(tau_s * 1e3, 3), "sigma_max2": round(sigma_max2, 5),
            "latency_model_knots": {"batch": knots_b, "t_cq_ms": [round(x * 1e3, 3) for x in t_cq],
                                    "t_lut_ms": [round(x * 1e3, 3) for x in t_lut]},
            "synthetic_llm": {"mu_llm0_per_s": round(mu0, 1), "mem_kvcache_bytes": kv},
            "rho": round(rho, 4), "resident_clusters": n_hot,
            "resident_bytes": float(mem_index[n_hot]), "mean_hit_rate_profile": round(float(hit_cdf[n_hot]), 4),
            "batch": batch, "predicted_min_hit_rate": round(eta_pred, 4),
            "measured_min_hit_rate_mean": round(float(np.mean(min_rates)), 4),
            "predicted_latency_ms": round(lat_pred * 1e3, 3),
            "measured_latency_ms_mean": round(float(np.mean(lat)) * 1e3, 3),
            "measured_latency_ms_max": round(float(np.max(lat)) * 1e3, 3)}), flush=True)
        return

    if args.mode == "drift":
        frac = args.resident if args.resident < 1.0 else 0.30
        batch = 1024
        side = torch.cuda.Stream(device=dev)
        hot = hottest_clusters(index, calib, spec.nprobe, frac, ix.nlist)
        index.load_partition(hot)
        per_epoch = []
        mig_time = 0.0
        total_q = 0
        t_all = time.perf_counter()
        perm_seed = spec.seed_perm
        pending_t0 = None
        for ep in range(args.epochs):
            if ep % 5 == 0:
                perm_seed = spec.seed_perm + ep
            q_ep, _ = make_queries(spec, centers, nq=args.epoch_queries,
                                   seed=spec.seed_queries + 1000 + ep, perm_seed=perm_seed)
            q_host = q_ep.cpu().numpy()
            index.hit_stats(reset=True)
            t_ep = time.perf_counter()
            for s in range(0, args.epoch_queries, batch):
                index.search_batch(q_host[s:s + batch], spec.nprobe, spec.k)
                if pending_t0 is not None and not index.migrate_poll()[0]:
                    mig_time += time.perf_counter() - pending_t0
                    pending_t0 = None
            ep_s = time.perf_counter() - t_ep
            total_q += args.epoch_queries
            st = index.hit_stats()
            if pending_t0 is not None:
                index.migrate_poll(wait=True)
                mig_time += time.perf_counter() - pending_t0
                pending_t0 = None
            # the library ranks this epoch's counters, migrates the difference to the
            # new hot set on the side stream and clears the counters
            t_refresh = time.perf_counter()
            moved = index.refresh_hot_set(len(hot), reset=True, side_stream=side)
            if moved["evicted"] or moved["admitted"]:
                pending_t0 = t_refresh
            row = {"epoch": ep, "queries_per_s": round(args.epoch_queries / ep_s, 1),
                   "mean_hit_rate": round(st["mean_hit_rate"], 4),
                   "min_hit_rate": round(st["min_hit_rate"], 4),
                   "migrated_clusters": moved["admitted"], "deferred_clusters": moved["deferred"]}
            log(json.dumps(row))
            per_epoch.append(row)
        if pending_t0 is not None:
            index.migrate_poll(wait=True)
            mig_time += time.perf_counter() - pending_t0
        total_s = time.perf_counter() - t_all
        _, mig_bytes = index.migrate_poll()
        ms = index.migrate_stats()
        index.close()
        print(json.dumps({
            "mode": "drift", "workload": workload, "resident_fraction": frac,
            "batch": batch, "epochs": args.epochs, "queries": total_q,
            "sustained_queries_per_s": round(total_q / total_s, 1),
            "migration_bytes": int(mig_bytes),
            "migration_bytes_per_s": round(ms["bytes"] / (ms["copy_ms"] * 1e-3), 1)
            if ms["copy_ms"] > 0 else None,
            "migration_copy_ms": round(ms["copy_ms"], 3), "migrations": ms["migrations"],
            "migration_seconds_until_published": round(mig_time, 4),
            "per_epoch": per_epoch}), flush=True)
        return

    # ---------------- default mode: the hot path ----------------
    q, _ = make_queries(spec, centers, nq=nq)
    q = q.contiguous()
    resident_frac = 1.0
    if args.resident < 1.0:
        hot = hottest_clusters(index, calib, spec.nprobe, args.resident, ix.nlist)
        index.load_partition(hot)
        resident_frac = len(hot) / ix.nlist

    # the machine's achievable streaming-read rate, the second denominator of the scan's
    # roofline: the plain read kernel over 1 GiB (it runs right before the warm-up, so the
    # search steps start on a GPU that is already at its sustained clock)
    read_ceiling = measure_read_ceiling(dev, with_copy=args.calib_copy)

    # timed region: HIP events around the scan kernel only (they feed the roofline figure)
    r = timed_steps(index, q, spec.nprobe, spec.k, args.steps, args.warmup, args.slices,
                    timing=0 if args.no_timing else (1 if args.stage_timing else 2),
                    n_streams=args.streams)
    out_ids, out_d = r["out_ids"], r["out_d"]
    out_d_dev = out_d
    stage_ms = r["stage_ms"]
    if not args.stage_timing:
        # per-stage times from a short pass of its own, events around every stage
        stage_ms = timed_steps(index, q, spec.nprobe, spec.k, min(args.steps, 20), 2, args.slices,
                               timing=1, n_streams=1)["stage_ms"]

    # the same steps issued on two alternating streams (the index keeps a workspace per
    # stream, so one batch's coarse stage overlaps the previous batch's scan): what a
    # caller that pipelines its batches gets; per-kernel times mean nothing then, so it
    # is a figure of its own beside `value`, from a short pass of its own
    two_streams = None
    if args.two_streams_pass and args.streams == 1 and resident_frac == 1.0:
        r2s = timed_steps(index, q, spec.nprobe, spec.k, min(args.steps, 100), min(args.warmup, 10),
                          args.slices, timing=0, n_streams=2)
        assert torch.equal(r2s["out_ids"], out_ids) and torch.equal(r2s["out_d"], out_d)
        two_streams = {"queries_per_s": round(r2s["qps"], 1),
                       "ms_per_step": round(r2s["ms_per_step"], 4),
                       "steps": min(args.steps, 100)}

    # the host-pointer entry point on the same batch (PCIe both ways, one call at a
    # time): context for callers that hold their queries on the host, never `value`
    host_ptr = None
    if resident_frac == 1.0 and not args.no_timing:
        index.set_tuning(scan_slices=args.slices, timing=0)
        n_h = min(args.steps, 30)
        host_ptr = {"steps": n_h,
                    "note": "ivf_search_batch: host queries in, host results out, one synchronous "
                            "call at a time (PCIe both ways inside the timed call)"}
        q_pinned = q.cpu().pin_memory()
        for kind, q_host in (("pinned", q_pinned.numpy()), ("pageable", q.cpu().numpy().copy())):
            out_i = torch.empty((nq, spec.k), dtype=torch.int64)
            out_d = torch.empty((nq, spec.k), dtype=torch.float32)
            if kind == "pinned":
                out_i, out_d = out_i.pin_memory(), out_d.pin_memory()
            for _ in range(3):
                index.search_batch(q_host, spec.nprobe, spec.k, out_i.numpy(), out_d.numpy())
            t0 = time.perf_counter()
            for _ in range(n_h):
                index.search_batch(q_host, spec.nprobe, spec.k, out_i.numpy(), out_d.numpy())
            dt = time.perf_counter() - t0
            host_ptr[f"queries_per_s_{kind}"] = round(nq * n_h / dt, 1)
            host_ptr[f"ms_per_call_{kind}"] = round(1e3 * dt / n_h, 4)
            assert torch.equal(out_i, out_ids.cpu()) and torch.equal(out_d, out_d_dev.cpu())
        host_ptr["pinned_over_device_resident"] = round(
            host_ptr["queries_per_s_pinned"] / r["qps"], 4)

    roofline = None
    if "scan_gbs" in r:
        roofline = {"bound": "hbm", "kernel": "k_scan", "achieved": round(r["scan_gbs"], 1),
                    "peak": HBM_PEAK_GBS, "unit": "GB/s",
                    "frac": round(r["scan_gbs"] / HBM_PEAK_GBS, 4), "traffic": None,
                    "bytes_per_launch": int(r["scan_bytes_per_launch"]),
                    "avg_launch_ms": round(r["scan_ms"], 4)}
        key = (spec.name, nq, round(resident_frac, 4))
        roofline["scan_source_hash"] = scan_source_hash()
        if (key in MEASURED_TRAFFIC and args.slices == 0 and not args.residual
                and args.nbits == 8 and not args.m and not args.nprobe and not args.k):
            traffic, source, src_hash = MEASURED_TRAFFIC[key]
            if src_hash == roofline["scan_source_hash"]:
                # bytes that crossed the L2 boundary per launch (rocprofv3 counters, measured
                # once on these sources) over this run's launch time: the counter-based rate
                roofline["traffic"], roofline["traffic_source"] = traffic, source
                roofline["frac_traffic"] = round(
                    traffic / (r["scan_ms"] * 1e-3) / 1e9 / HBM_PEAK_GBS, 4)
            else:
                roofline["traffic_note"] = (f"{source} was measured on other scan sources "
                                            f"({src_hash}); no traffic figure for this build")
        roofline["frac_note"] = ("achieved = algorithmic bytes / time: lists that queries share "
                                 "are counted once per query but can be served from L2, so frac "
                                 "may pass 1; frac_traffic counts the bytes that crossed L2")
        roofline["streaming_read_GBs"] = read_ceiling
        roofline["frac_of_streaming_read"] = round(r["scan_gbs"] / read_ceiling, 4)
        if resident_frac == 1.0:
            # bytes of the distinct lists the batch touches (what a perfect cache would fetch)
            pr = index.coarse_probe_dev(q, spec.nprobe).cpu().numpy()
            lens = np.diff(ix.list_offsets)
            roofline["unique_bytes"] = int(lens[np.unique(pr)].sum()) * int(ix.codes.shape[1])

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
        res_cen = orc.residual_centroids_of(ix)
        ref_i, ref_d = orc.scan(ix.metric, ix.codebooks, ix.list_offsets, ix.codes, ix.ids, qs,
                                probe, spec.k + 16, residual_centroids=res_cen)
        cpu_s = time.perf_counter() - t0
        cpu_baseline = {"value": round(ns / cpu_s, 2), "unit": "queries/s",
                        "cores": orc.num_threads(), "kind": "oracle",
                        "sample": f"{ns} of the {nq} queries, same index, nprobe={spec.nprobe}, "
                                  f"k={spec.k}; brute-force coarse + decode-and-distance in fp64"}
        # the same on one thread, over a sixteenth of the sample
        n1 = max(1, ns // 16)
        all_threads = orc.num_threads()
        orc.set_num_threads(1)
        t1 = time.perf_counter()
        p1, _, _ = orc.coarse(ix.metric, ix.centroids, qs[:n1], spec.nprobe)
        orc.scan(ix.metric, ix.codebooks, ix.list_offsets, ix.codes, ix.ids, qs[:n1],
                 np.ascontiguousarray(p1), spec.k, residual_centroids=res_cen)
        cpu_baseline["value_1_thread"] = round(n1 / (time.perf_counter() - t1), 2)
        cpu_baseline["sample_1_thread"] = f"the first {n1} of those queries"
        try:
            with open("/proc/cpuinfo") as f:
                model = [l.split(":", 1)[1].strip() for l in f if l.startswith("model name")]
            cpu_baseline["host_cpu"] = f"{model[0]} x {len(model)}" if model else None
        except OSError:
            cpu_baseline["host_cpu"] = None
        orc.set_num_threads(all_threads)
        # parity of the timed configuration on the same sample
        got_i = out_ids.cpu().numpy()[sel]
        got_d = out_d.cpu().numpy()[sel]
        got_probe = index.coarse_probe_dev(q, spec.nprobe).cpu().numpy()[sel]
        S = scale_S(ix.metric, qs)
        n_coarse = compare_probes(got_probe, probe_ext, score_ext, spec.nprobe, S)
        if n_coarse:
            ref_i, ref_d = orc.scan(ix.metric, ix.codebooks, ix.list_offsets, ix.codes, ix.ids,
                                    qs, got_probe, spec.k + 16, residual_centroids=res_cen)
        n_amb = compare_topk(got_i, got_d, ref_i, ref_d, spec.k, S)
        parity = {"queries_checked": int(ns), "coarse_ambiguous": int(n_coarse),
                  "id_ambiguous": int(n_amb), "pass": True}

    # The configuration's other named points (batch sizes 256 and 4096, hottest 50 / 30 / 10 %
    # of the clusters resident with the rest scanned by the library's CPU tier), each from a
    # short pass of its own after everything above: context beside `value`, never part of it.
    # Runs under a profiler leave them out (they pass --no-oracle) so that a kernel's
    # statistics cover one launch shape.
    other_points = None
    if (args.workload == "C3" and not args.no_other_points and not args.no_oracle
            and resident_frac == 1.0 and not args.no_timing and args.streams == 1
            and not (args.nq or args.nprobe or args.k or args.residual or args.m)
            and args.nbits == 8):
        index.close()
        index = pkg.IvfIndex(ix, max_nq=4096, max_nprobe=spec.nprobe, max_k=spec.k)
        other_points = []
        for frac in (1.0, 0.5, 0.3, 0.1):
            index.load_partition(all_clusters)
            if frac < 1.0:
                index.load_partition(hottest_clusters(index, calib, spec.nprobe, frac, ix.nlist))
            for n in ((256, 4096) if frac == 1.0 else (1024,)):
                qn = make_queries(spec, centers, nq=n)[0].contiguous()
                rp = timed_steps(index, qn, spec.nprobe, spec.k, 20 if frac == 1.0 else 5,
                                 5 if frac == 1.0 else 2, 0, timing=2)
                row = {"nq": n, "resident_fraction": frac, "queries_per_s": round(rp["qps"], 1),
                       "ms_per_step": round(rp["ms_per_step"], 4),
                       "mean_hit_rate": round(rp["hit_rate"], 4),
                       "min_hit_rate": round(rp["min_hit_rate"], 4),
                       "bytes_hit_rate": round(rp["bytes_hit_rate"], 4)}
                if "scan_gbs" in rp:
                    row["scan_ms"] = round(rp["scan_ms"], 4)
                    row["scan_frac_of_peak"] = round(rp["scan_gbs"] / HBM_PEAK_GBS, 4)
                log(json.dumps(row))
                other_points.append(row)

    out = {
        "metric": METRIC,
        "value": round(r["qps"], 1),
        "unit": "queries/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(r["ms_per_step"], 4),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "i32",
        "dtype_detail": "ADC scan: int32 fixed-point table sums; lookup tables built in f32; coarse "
                        "contraction: two-way f16 split on the matrix cores, f32 accumulate",
        "data": "synthetic",
        "config": {"workload": f"{workload} nq={nq}",
                   "resident_fraction": round(resident_frac, 4),
                   "mean_hit_rate": round(r["hit_rate"], 4),
                   "bytes_hit_rate": round(r["bytes_hit_rate"], 4),
                   "scan_slices": args.slices, "streams": args.streams,
                   "inputs": "queries already in HBM when the timed region starts "
                             "(ivf_search_batch_dev); the host-pointer call is in "
                             "host_pointer_call"},
        "roofline": roofline,
        "cpu_baseline": cpu_baseline,
        "stage_ms": stage_ms,
        "stage_ms_source": "timed region" if args.stage_timing else
                           "separate pass with events around every stage (not in the timed region)",
        "parity": parity,
        "host_pointer_call": host_ptr,
        "two_streams": two_streams,
        "other_points": other_points,
        "other_points_note": "same index, short passes after the timed region: all clusters "
                             "resident at nq = 256 and 4096 (device-resident queries); hottest "
                             "50 / 30 / 10 % resident at nq = 1024, the cold probes scanned by the "
                             "library's CPU tier on the host's threads inside the same call",
        "index_build_s": round(build_s, 2),
        "load_partition_s": round(load_s, 3),
    }
    index.close()
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
