#!/usr/bin/env python3
"""Benchmark of the IVF-PQ search hot path on one MI355X.

One step = one pass of the whole hot path (filtering, thresholded tables, ADC
scan, top-k) over one batch of Q synthetic queries, through the C ABI, with the
index and the queries resident in HBM.  Prints ONE JSON line:

  metric/value  queries per second over the timed steps (whole path)
  roofline      the fused table+scan+top-k kernel against the HBM roofline:
                algorithmic code bytes per launch / its mean duration (HIP events
                recorded on the launch stream inside the timed region)
  cpu_baseline  the CPU oracle timed on this host on a bounded sample of the
                same queries (reported, not a target)

The step issues ivfpq_coarse then ivfpq_scan_topk (the two launches
ivfpq_search makes) so that an event can sit between them.
"""
import argparse
import ctypes
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0   # MI355X HBM3E, published

# HBM bytes per scan-kernel launch from rocprofv3 counter runs of this file (FETCH_SIZE and
# WRITE_SIZE in KiB per dispatch, each scaled by what the same counter reads for an
# elementwise pass over 1 GiB: x2.000 and x1.000).  Commands and raw figures: profiles/.
MEASURED_TRAFFIC_BYTES = {
    ("C2", 0.25): (593718 + 12451) * 1024 * 2.000 + (449093 + 1250) * 1024 * 1.000,
    ("C5", 0.25): (6.63817e6 + 329406) * 1024 * 2.000 + (531216 + 5000) * 1024 * 1.000,
}


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="C2", help="C1..C5, C5_10M (default C2: 1M x 128, nprobe 32)")
    ap.add_argument("--k", type=int, default=0,
                    help="neighbours per query (default: the workload's, 100); above 100 the quality figure is "
                         "R100@k, the share of the true 100 nearest among the k returned (1000: paper Sec. 6.1)")
    ap.add_argument("--metric", choices=["l2", "ip"], default="l2",
                    help="ip: maximum inner product search over the same index (paper Sec. 4.2)")
    ap.add_argument("--keep", type=float, default=0.25, help="fraction of codebook entries inside the radius")
    ap.add_argument("--score-mode", type=int, default=0,
                    help="0 distances (default), 1 hit count, 2 reward/penalty hit count")
    ap.add_argument("--dynamic-radii", action="store_true",
                    help="per-query radii: density map + polynomial fitted offline, looked up by ivfpq_query_radii in every step")
    ap.add_argument("--radius-scale", type=float, default=1.0, help="user scale on the dynamic radii")
    ap.add_argument("--radius-target", choices=["top", "keep"], default="top",
                    help="what the offline polynomial is fitted to: the radius that contains the entries of the true "
                         "top-100 neighbours (the paper's), or the radius that keeps --keep of the entries")
    ap.add_argument("--scan-waves", type=int, default=0)
    ap.add_argument("--scan-loads", type=int, default=0, help="code loads: 0 default (first chunk ahead while pruning), 1 whole blocks, 2 / 3 always first half / first chunk")
    ap.add_argument("--lds-pad", type=int, default=0, help="measurement only: extra LDS bytes per scan workgroup")
    ap.add_argument("--ablate", type=int, default=0, help="measurement only: scan_ablate bit mask (results invalid)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-recall", action="store_true")
    ap.add_argument("--cpu-seconds", type=float, default=12.0)
    ap.add_argument("--calib-copy", action="store_true",
                    help="also launch one elementwise pass over 1 GiB (read 1 GiB, write 1 GiB): the known-size "
                         "kernel that scales the FETCH_SIZE / WRITE_SIZE counters")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on one GPU only (no sharding, no collectives); use --gpus 1")

    import numpy as np
    import torch
    from paper_2312_01712_amd import binding, workloads as wl

    if not torch.cuda.is_available():
        sys.exit("bench.py: no GPU visible; the HIP path has no CPU fallback")
    torch.cuda.set_device(0)
    binding.load_library()
    if args.scan_waves:
        binding.set_option("scan_waves", args.scan_waves)
    if args.scan_loads:
        binding.set_option("scan_loads", args.scan_loads)
    if args.lds_pad:
        binding.set_option("scan_lds_pad", args.lds_pad)
    if args.ablate:
        binding.set_option("scan_ablate", args.ablate)
        if args.ablate & 7:
            args.no_cpu_baseline = args.no_recall = True
    w = wl.WORKLOADS[args.workload]

    t0 = time.time()
    idx, centres = wl.train_index(w, device="cuda", progress=log)
    metric = 1 if args.metric == "ip" else 0
    radii = wl.calibrate_radii(w, idx, centres, args.keep, metric=metric)
    q = wl.queries(w, centres)
    gi = binding.IvfPqIndex.from_index(idx, metric=metric)
    log(f"[{w.name}] index built in {time.time() - t0:.1f}s; code bytes on device {gi.info()['code_bytes']}")

    Q, nprobe, k = w.Q, w.nprobe, (args.k or w.k)
    passes = (k + 127) // 128   # the scan kernel keeps 128 keys per query and launch
    ws = gi.workspace(Q, nprobe, k)
    pid = torch.empty((Q, nprobe), dtype=torch.int32, device="cuda")
    out_ids = torch.empty((Q, k), dtype=torch.int64, device="cuda")
    out_dist = torch.empty((Q, k), dtype=torch.float32, device="cuda")
    lib = binding.load_library()
    stream = torch.cuda.current_stream().cuda_stream
    d_rq = rmodel = None
    if args.dynamic_radii:   # offline: density maps + polynomial (an input); online: ivfpq_query_radii in every step
        model = wl.fit_radius_model(w, idx, centres, args.keep, target=args.radius_target)
        model_arrays = (model["lo"], model["cells_per_unit"], model["map"], model["coef"], model["fallback"])
        rmodel = binding.RadiusModel(gi, *model_arrays)
        d_rq = torch.empty((Q, w.M), dtype=torch.float32, device="cuda")
    rptr, scoring, _keep = binding._scoring(args.score_mode, d_rq, None if args.dynamic_radii else radii, Q, w.M)

    def step(ev=None):
        binding._check(lib.ivfpq_coarse(gi._h, q.data_ptr(), Q, nprobe, pid.data_ptr(), None, ws.data_ptr(),
                                        ws.numel(), stream))
        if rmodel is not None:
            binding._check(lib.ivfpq_query_radii(gi._h, rmodel._h, q.data_ptr(), Q, pid.data_ptr(), nprobe,
                                                 ctypes.c_float(args.radius_scale), d_rq.data_ptr(), stream))
        if ev:
            ev[0].record()
        binding._check(lib.ivfpq_scan_topk_ex(gi._h, q.data_ptr(), Q, nprobe, pid.data_ptr(), k, rptr, scoring,
                                              out_ids.data_ptr(), out_dist.data_ptr(), ws.data_ptr(), ws.numel(),
                                              stream))
        if ev:
            ev[1].record()

    if args.calib_copy:
        src = torch.ones(1 << 28, dtype=torch.float32, device="cuda")
        dst = torch.empty_like(src)
        torch.rsqrt(src, out=dst)   # the only rsqrt in this program: easy to find in the counter output
        torch.cuda.synchronize()
        del src, dst
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    binding.coarse_fallbacks(reset=True)
    events = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(args.steps)]
    start = torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    start.record()
    for i in range(args.steps):
        step(events[i])
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    scan_ms = [a.elapsed_time(b) for a, b in events]
    coarse_ms = [start.elapsed_time(events[0][0])] + [events[i - 1][1].elapsed_time(events[i][0]) for i in range(1, args.steps)]
    scan_avg_ms = float(np.mean(scan_ms))

    # algorithmic bytes of one scan launch: one code byte per (probed point, subspace)
    sizes = torch.from_numpy(np.diff(idx.list_offsets)).cuda()
    scanned_points = int(sizes[pid.long()].sum().item())
    algo_bytes = scanned_points * w.M * passes
    achieved = algo_bytes / (scan_avg_ms * 1e-3) / 1e9

    # the one-call entry point gives the same answer
    ids2, dist2 = gi.search(q, nprobe, k, None if args.dynamic_radii else radii, workspace=ws,
                            mode=args.score_mode, query_radii=d_rq)
    torch.cuda.synchronize()
    assert (args.ablate & 7) or (torch.equal(ids2, out_ids) and torch.equal(dist2, out_dist))

    recall = r1 = None
    if not args.no_recall:
        truth = wl.exact_knn(w, centres, q, min(k, 100), metric=metric)
        recall, r1 = wl.recall_at_k(out_ids.cpu().numpy(), truth)

    result = {
        "metric": "queries/sec at recall@100 (1M x 128, nprobe=32)" if (w.name, k, metric) == ("C2", 100, 0) else f"queries/sec at recall@{k}" if k <= 100 else f"queries/sec at R100@{k}",
        "value": Q * args.steps / elapsed, "unit": "queries/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": elapsed / args.steps * 1e3, "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": f"{w.name}: N={w.N} D={w.D} nlist={w.nlist} M={w.M} Q={Q} nprobe={nprobe} k={k}",
                   "family": w.family, "similarity": args.metric, "keep_fraction": args.keep, "score_mode": args.score_mode,
                   "radii": f"per-query (density map, fitted to {args.radius_target}, scale {args.radius_scale})" if args.dynamic_radii else "per-subspace", "recall_at_k": recall, "recall_truth_k": min(k, 100), "r1_at_k": r1,
                   "coarse_ms": float(np.mean(coarse_ms)), "scan_ms": scan_avg_ms,
                   "coarse_exact_fallbacks_per_step": binding.coarse_fallbacks() / max(1, args.steps + 1)},
        "roofline": {"bound": "hbm", "kernel": "scan_kernel (table + ADC scan + top-k), timed with probe_bound_kernel (list-level bounds, 8 % of it on C2)", "achieved": achieved,
                     "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": achieved / HBM_PEAK_GBS,
                     "traffic": (MEASURED_TRAFFIC_BYTES.get((w.name, args.keep))
                                 if args.score_mode == 0 and not args.dynamic_radii and k == w.k and not metric else None),
                     "algorithmic_bytes_per_launch": algo_bytes // passes, "avg_launch_ms": scan_avg_ms / passes},
    }

    if not args.no_cpu_baseline:
        import oracle
        qh = q.cpu().numpy()
        threads = min(os.cpu_count() or 1, 16)
        t = time.perf_counter()
        probe_n = min(Q, 2 * threads)
        if args.dynamic_radii:   # the oracle's own chain: nearest list, map look-up, polynomial, scale
            o_near, _ = oracle.coarse(qh, idx.centroids, 1)
            o_radii = oracle.query_radii(qh, idx.centroids, o_near[:, 0], *model_arrays, args.radius_scale)
        else:
            o_radii = radii
        osearch = lambda lo, hi, th: oracle.search(qh[lo:hi], idx, nprobe, k,
                                                   o_radii[lo:hi] if args.dynamic_radii else o_radii,
                                                   threads=th, mode=args.score_mode, metric=metric)
        o_ids, o_dist = osearch(0, probe_n, threads)
        per_q = (time.perf_counter() - t) / probe_n          # wall seconds per query with all threads
        n = int(max(probe_n, min(Q, args.cpu_seconds / max(per_q, 1e-9))))
        t = time.perf_counter()
        o_ids, o_dist = osearch(0, n, threads)
        dt = time.perf_counter() - t
        same = bool(np.array_equal(o_ids, out_ids.cpu().numpy()[:n]) and
                    np.array_equal(o_dist.view(np.uint32), out_dist.cpu().numpy()[:n].view(np.uint32)))
        n1 = int(max(1, min(n, 3.0 / max(per_q * threads, 1e-9))))
        t = time.perf_counter()
        osearch(0, n1, 1)
        dt1 = time.perf_counter() - t
        result["cpu_baseline"] = {"value": n / dt, "unit": "queries/s", "cores": threads, "kind": "oracle",
                                  "sample": f"first {n} of {Q} queries, {threads} threads over disjoint query ranges",
                                  "value_1thread": n1 / dt1, "sample_1thread": f"first {n1} queries",
                                  "gpu_matches_oracle_on_sample": same}
    print(json.dumps(result), flush=True)


if __name__ == "__main__":
    main()
