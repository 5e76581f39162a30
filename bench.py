"""Benchmark of the IVFADC+R search path on one MI355X.

A step is one pass of the whole query stage (coarse probe, look-up tables, ADC list scan,
top-k' short-list, re-rank, top-k) over one batch of synthetic queries against an index that
is already resident in HBM.  The index is built on the GPU from the seeded synthetic
generator before the timed region.  Prints one JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--config cfg4]
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0     # MI355X HBM3E peak

# HBM bytes moved per scan launch, from rocprofv3 FETCH_SIZE / WRITE_SIZE counters scaled by a plain copy
# of known size (profiles/search_cfg4_hbm_traffic.txt), stored as a ratio to the algorithmic bytes of the
# launch (m bytes per (query, entry) estimate), for the default run of cfg4; other workloads and settings: null.
#   per-pair scan (sharing mode 0):   101.45 GB read + 0.05 GB written for 101.14 GB of code bytes
#   fp32 units of four (--sharing 1): 24.89 GB read + 0.16 GB written for 96.14 GB (one read serves four queries)
#   fp16 units of eight (default):    11.13 GB read + 0.05 GB written for 92.97 GB (one read serves eight queries,
#                                     and units of one list that run side by side on an XCD share it in L2)
MEASURED_TRAFFIC_RATIO = {("cfg4", "adc_scan_kernel"): 101.500 / 101.141,
                          ("cfg4", "adc_scan_shared_kernel"): 25.051 / 96.142,
                          ("cfg4", "adc_scan_shared8h_kernel"): 11.185 / 92.966}
LDS_PEAK_GBS = 256 * 128 * 2.4    # 256 CUs x 128 B/clk x 2.4 GHz


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def build_index(cfg, dm, n_gt, args):
    """Train, encode and finalize on the GPU; brute-force ground truth of the first n_gt queries
    is accumulated from the same generated chunks (exact: integer data, fp32 products < 2^24)."""
    import torch
    import synthdata as sd
    import paper_1102_3828_amd as pkg

    dev = dm.device
    t0 = time.time()
    ix = pkg.Index(cfg.d, cfg.c, cfg.m, cfg.m_refine)
    train = dm.generate(sd.STREAM_TRAIN, 0, cfg.n_train)
    ix.train(train, iters=args.train_iters, seed=1)
    del train
    torch.cuda.synchronize()
    t_train = time.time() - t0
    log(f"[bench] trained quantizers on {cfg.n_train} vectors in {t_train:.1f}s")

    queries_u8 = dm.generate(sd.STREAM_QUERY, 0, cfg.n_query)
    xq = queries_u8.float().contiguous()
    gt_d = torch.full((n_gt, 1), float("inf"), device=dev)
    gt_i = torch.full((n_gt, 1), -1, dtype=torch.int64, device=dev)
    xg = xq[:n_gt]
    t0 = time.time()
    buf = None
    for j, a in enumerate(range(0, cfg.N, sd.BASE_CHUNK)):
        n = min(sd.BASE_CHUNK, cfg.N - a)
        if buf is None or buf.shape[0] != n:
            buf = torch.empty((n, cfg.d), dtype=torch.uint8, device=dev)
        dm.generate(sd.STREAM_BASE0 + j, 0, n, out=buf)
        ix.add(buf, a)
        if n_gt:
            for s in range(0, n, 1 << 20):
                y = buf[s:s + (1 << 20)].float()
                d2 = (y * y).sum(1)[None, :] - 2.0 * (xg @ y.T)
                dmin, imin = d2.min(dim=1, keepdim=True)
                better = dmin < gt_d
                gt_d = torch.where(better, dmin, gt_d)
                gt_i = torch.where(better, imin + a + s, gt_i)
        if j % 10 == 9 or a + n >= cfg.N:
            torch.cuda.synchronize()
            log(f"[bench] added {a + n} / {cfg.N} vectors ({time.time() - t0:.1f}s)")
    del buf
    ix.finalize()
    torch.cuda.synchronize()
    t_add = time.time() - t0
    log(f"[bench] encoded + finalized {cfg.N} vectors in {t_add:.1f}s")
    return ix, xq, queries_u8, gt_i[:, 0].cpu().numpy(), dict(train_s=t_train, add_s=t_add)


def cpu_baseline(ix, cfg, queries_u8, gpu_ids, budget_s=15.0, max_q=64):
    """The CPU oracle's search on the exported index, timed on this host for a bounded sample."""
    import numpy as np
    from oracle import ivfadcr_oracle as orc
    coarse, pq, rq = ix.get_codebooks()
    t0 = time.time()
    offsets, ids, codes, rcodes = ix.export()
    log(f"[bench] exported index to host in {time.time() - t0:.1f}s")
    index = orc.Index(orc.Codebooks(coarse, pq, rq), offsets, ids, codes, rcodes)
    X = queries_u8[:max_q].cpu().numpy()
    done, same, scanned = 0, 0, 0
    t0 = time.time()
    for qi in range(len(X)):
        o_ids, _, tr = orc.search_one(X[qi], index, cfg.w, cfg.kprime, cfg.k)
        done += 1
        scanned += tr.scanned
        same += int((o_ids == gpu_ids[qi]).sum())
        if time.time() - t0 > budget_s:
            break
    el = time.time() - t0
    return {"value": done / el, "unit": "queries/s", "cores": 1, "kind": "oracle",
            "sample": f"first {done} queries of the same workload, one at a time (numpy float64, single thread)",
            "adc_codes_per_s": scanned / el,
            "ids_identical_to_gpu": same / float(done * cfg.k)}


def sweep(args):
    """Parameter sweeps in the shape of the paper's tables, on the synthetic generator (section 4; the
    absolute recall values belong to this data, not to BIGANN).  One JSON line per setting on stdout.
      table1: ADC / ADC+R (no inverted file) and IVFADC / IVFADC+R, m = 8, m' in {0, 8, 16, 32}
      table2: equal-memory pairs (m, m') without inverted file
      fig3:   recall@10 against the database size, IVFADC+R, m' in {0, 8, 32}"""
    import dataclasses
    import numpy as np
    import torch
    import synthdata as sd
    from synthdata.gpu import DeviceMixture

    base = sd.CONFIGS[args.config]
    if args.batch:
        base = dataclasses.replace(base, batch=args.batch)
    if args.N:
        base = dataclasses.replace(base, N=args.N)
    if args.kprime:
        base = dataclasses.replace(base, kprime=args.kprime)
    if args.k:
        base = dataclasses.replace(base, k=args.k)
    torch.cuda.set_device(0)
    dm = DeviceMixture(base.mixture(), "cuda:0")
    if args.sweep == "table1":
        settings = [dict(c=c, w=w, m_refine=mr) for c, w in ((1, 1), (base.c, base.w)) for mr in (0, 8, 16, 32)]
    elif args.sweep == "table2":
        settings = [dict(c=1, w=1, m=m, m_refine=mr)
                    for m, mr in ((8, 0), (4, 4), (16, 0), (8, 8), (32, 0), (16, 16), (64, 0), (32, 32))]
    else:
        settings = [dict(N=n, m_refine=mr) for n in (10 ** 6, 10 ** 7, 10 ** 8, 10 ** 9) if n <= base.N
                    for mr in (0, 8, 32)]
    gt_cache = {}
    for st in settings:
        cfg = dataclasses.replace(base, **st)
        n_gt = min(args.gt_queries, cfg.n_query)
        have = gt_cache.get(cfg.N)
        ix, xq, _, gt, build_t = build_index(cfg, dm, 0 if have is not None else n_gt, args)
        if have is None:
            gt_cache[cfg.N] = gt
        gt = gt_cache[cfg.N]
        B = min(cfg.batch, cfg.n_query)
        ix.set_tuning(batch=min(B, 65535))
        batches = [xq[i * B:(i + 1) * B].contiguous() for i in range(max(1, cfg.n_query // B))]
        ix.search(batches[-1], cfg.w, cfg.kprime, cfg.k)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        retries = dense = 0
        for s in range(args.steps):
            ix.search(batches[s % len(batches)], cfg.w, cfg.kprime, cfg.k)
            stats = ix.search_stats()
            retries += stats["bound_retries"]
            dense += stats["dense_fallbacks"]
        torch.cuda.synchronize()
        el = time.perf_counter() - t0
        ids, _ = ix.search(batches[0], cfg.w, cfg.kprime, cfg.k)
        ids = ids.cpu().numpy()
        rec = {f"recall@{r}": float((ids[:n_gt, :r] == gt[:n_gt, None]).any(axis=1).mean())
               for r in (1, 10, 100) if r <= cfg.k}
        row = {"sweep": args.sweep, "N": cfg.N, "c": cfg.c, "w": cfg.w, "m": cfg.m, "m_refine": cfg.m_refine,
               "kprime": cfg.kprime, "k": cfg.k, "bytes_per_vector": cfg.m + cfg.m_refine + 4,
               "ms_per_query": 1e3 * el / (args.steps * B), "queries_per_s": args.steps * B / el,
               "bound_retries": retries, "dense_fallbacks": dense, **rec, "build_s": build_t["add_s"]}
        print(json.dumps(row), flush=True)
        ix.close()
        del ix
        torch.cuda.empty_cache()


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--config", default=os.environ.get("IVFR_BENCH_CONFIG", "cfg4"))
    ap.add_argument("--N", type=int, default=0, help="override the database size (debugging)")
    ap.add_argument("--kprime", type=int, default=0)
    ap.add_argument("--k", type=int, default=0, help="override the result length (the paper's Table 1 uses k = 10000, k' = 20000)")
    ap.add_argument("--m-refine", type=int, default=-1)
    ap.add_argument("--c", type=int, default=0, help="override the number of coarse centroids (1 = exhaustive ADC+R)")
    ap.add_argument("--w", type=int, default=0, help="override the number of lists visited")
    ap.add_argument("--batch", type=int, default=0,
                    help="queries per step (default: the workload's 1000); the library's internal batch follows it")
    ap.add_argument("--train-iters", type=int, default=10)
    ap.add_argument("--gt-queries", type=int, default=100)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-whole-set", action="store_true",
                    help="skip the extra calls that hand the workload's whole query set to one search call")
    ap.add_argument("--scan-groups", type=int, default=0)
    ap.add_argument("--per-pair", action="store_true",
                    help="scan every (query, list) pair on its own (no sharing of a list between queries)")
    ap.add_argument("--sharing", type=int, default=2, choices=(0, 1, 2, 3),
                    help="list sharing mode: 0 per pair, 1 fp32 units of four/two, 2 also fp16 units of eight, 3 also matrix-core units of 64")
    ap.add_argument("--sweep-groups", default="",
                    help="comma-separated scan workgroup counts: time a few steps with each (to stderr) before the run")
    ap.add_argument("--sweep", default="", choices=("", "table1", "table2", "fig3"),
                    help="run a parameter sweep in the shape of the paper's Table 1, Table 2 or Figure 3 on the "
                         "synthetic generator (one JSON line per setting) instead of the benchmark")
    ap.add_argument("--calib-copy", action="store_true",
                    help="also run a plain 1 GiB device copy (reads 1 GiB, writes 1 GiB) three times, as the "
                         "known-size reference for scaling rocprofv3's FETCH_SIZE / WRITE_SIZE counters")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build measures one GPU only (the path is not sharded); run with --gpus 1",
              file=sys.stderr)
        sys.exit(2)

    if args.sweep:
        sweep(args)
        return

    import dataclasses
    import numpy as np
    import torch
    import synthdata as sd
    from synthdata.gpu import DeviceMixture

    cfg = sd.CONFIGS[args.config]
    if args.N:
        cfg = dataclasses.replace(cfg, N=args.N)
    if args.kprime:
        cfg = dataclasses.replace(cfg, kprime=args.kprime)
    if args.k:
        cfg = dataclasses.replace(cfg, k=args.k)
    if args.m_refine >= 0:
        cfg = dataclasses.replace(cfg, m_refine=args.m_refine)
    if args.c:
        cfg = dataclasses.replace(cfg, c=args.c)
    if args.w:
        cfg = dataclasses.replace(cfg, w=args.w)
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    dm = DeviceMixture(cfg.mixture(), "cuda:0")
    n_gt = min(args.gt_queries, cfg.n_query)
    ix, xq, queries_u8, gt, build_t = build_index(cfg, dm, n_gt, args)
    if args.scan_groups:
        ix.set_tuning(scan_groups=args.scan_groups)
    if args.per_pair:
        args.sharing = 0
    ix.set_list_sharing(args.sharing)
    if args.batch:
        cfg = dataclasses.replace(cfg, batch=args.batch)

    B = min(cfg.batch, cfg.n_query)
    ix.set_tuning(batch=min(B, 65535))
    n_batches = max(1, cfg.n_query // B)
    batches = [xq[i * B:(i + 1) * B].contiguous() for i in range(n_batches)]

    if args.sweep_groups:
        ix.set_profiling(True)
        for gcount in [int(x) for x in args.sweep_groups.split(",")]:
            ix.set_tuning(scan_groups=gcount)
            acc = {}
            for s in range(4):
                ix.search(batches[s % n_batches], cfg.w, cfg.kprime, cfg.k)
                if s:
                    for name, ms in ix.stage_times().items():
                        acc[name] = acc.get(name, 0.0) + ms / 3.0
            log(f"[bench] scan_groups={gcount}: " + ", ".join(f"{k} {v:.3f}" for k, v in acc.items() if k.startswith("scan") or k == "sample"))
        ix.set_profiling(False)
        ix.set_tuning(scan_groups=args.scan_groups)
    for s in range(args.warmup):
        t0 = time.perf_counter()
        ix.search(batches[s % n_batches], cfg.w, cfg.kprime, cfg.k)
        log(f"[bench] warmup step {s}: {1e3 * (time.perf_counter() - t0):.1f} ms, {ix.search_stats()}")
    # The timed steps record HIP events around the list-scan launches only (the roofline's kernel time);
    # the other stages are timed in three extra steps after the timed region (events around every stage
    # cost the host about 0.1 ms per step).
    ix.set_profiling(1)
    torch.cuda.synchronize()
    codes = 0
    codes_shared = 0
    codes_shared2 = 0
    codes_shared8 = 0
    codes_shared64 = 0
    codes_streamed = 0
    dense_total = 0
    retries_total = 0
    stage_ms = {}
    scan_launches = 0
    t0 = time.perf_counter()
    for s in range(args.steps):
        ix.search(batches[s % n_batches], cfg.w, cfg.kprime, cfg.k)
        st = ix.search_stats()
        pr = ix.stage_times()
        codes += st["codes_scanned"]
        codes_shared += st["codes_scanned_shared"]
        codes_shared2 += st["codes_scanned_shared2"]
        codes_shared8 += st["codes_scanned_shared8"]
        codes_shared64 += st["codes_scanned_shared64"]
        codes_streamed += st["codes_streamed"]
        scan_launches += pr.pop("scan_launches")
        for name, ms in pr.items():
            stage_ms[name] = stage_ms.get(name, 0.0) + ms
        dense_total += st["dense_fallbacks"]
        retries_total += st["bound_retries"]
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    log(f"[bench] timed {args.steps} steps in {elapsed:.3f}s")
    ix.set_profiling(2)
    other_ms = {}
    for s in range(3):
        ix.search(batches[s % n_batches], cfg.w, cfg.kprime, cfg.k)
        pr = ix.stage_times()
        pr.pop("scan_launches")
        for name, ms in pr.items():
            if not name.startswith("scan"):
                other_ms[name] = other_ms.get(name, 0.0) + ms * args.steps / 3.0
    stage_ms.update(other_ms)
    ix.set_profiling(False)

    if args.calib_copy:
        src = torch.empty(1 << 30, dtype=torch.uint8, device="cuda:0").random_(0, 255)
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    # accuracy on the ground-truth subset (first batch holds the first n_gt queries)
    g_ids, g_dist = ix.search(batches[0], cfg.w, cfg.kprime, cfg.k)
    g_ids = g_ids.cpu().numpy()
    recall = {}
    for r in (1, 10, 100):
        if r <= cfg.k and n_gt:
            recall[f"recall@{r}"] = float((g_ids[:n_gt, :r] == gt[:n_gt, None]).any(axis=1).mean())

    qps = args.steps * B / elapsed
    steps = max(args.steps, 1)
    # Dominant kernel: the shared-list scan when it does most of the work, else the per-pair scan.
    # Algorithmic bytes = m bytes per (query, visited entry) estimate the kernel computes.
    kernels = [("adc_scan_kernel", stage_ms.get("scan", 0.0) / steps,
                (codes - codes_shared - codes_shared2 - codes_shared8 - codes_shared64) / steps),
               ("adc_scan_shared_kernel", stage_ms.get("scan_shared", 0.0) / steps, codes_shared / steps),
               ("adc_scan_shared8h_kernel", stage_ms.get("scan_shared8", 0.0) / steps, codes_shared8 / steps),
               ("adc_scan_mfma64_kernel", stage_ms.get("scan_shared64", 0.0) / steps, codes_shared64 / steps)]
    kname, k_ms, k_codes = max(kernels, key=lambda k: k[1])
    code_bytes = cfg.m * k_codes
    lds_b = 2.0 if kname == "adc_scan_shared8h_kernel" else 4.0
    achieved = code_bytes / (k_ms * 1e-3) / 1e9 if k_ms > 0 else 0.0
    traffic_key = (cfg.name, kname)
    plain = not (args.N or args.kprime or args.k or args.m_refine >= 0 or args.c or args.w or args.batch)
    out = {
        "metric": "queries/s", "value": qps, "unit": "queries/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": 1e3 * elapsed / args.steps, "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": f"{cfg.name}: N={cfg.N} d={cfg.d} c={cfg.c} m={cfg.m} m'={cfg.m_refine} "
                               f"w={cfg.w} k'={cfg.kprime} k={cfg.k}, {B} queries per step",
                   "generator": f"uint8 Gaussian mixture G={cfg.G} zipf={cfg.zipf} seed={sd.BASE_SEED}",
                   "list_sharing_mode": args.sharing},
        "adc_codes_per_s": codes / elapsed,
        "codes_scanned_per_step": codes / steps,
        "codes_streamed_per_step": codes_streamed / steps,
        "codes_scanned_shared_per_step": codes_shared / steps,
        "codes_scanned_shared2_per_step": codes_shared2 / steps,
        "codes_scanned_shared8_per_step": codes_shared8 / steps,
        "codes_scanned_shared64_per_step": codes_shared64 / steps,
        "stage_ms_per_step": {name: ms / args.steps for name, ms in stage_ms.items()},
        "dense_fallbacks_total": dense_total,
        "bound_retries_total": retries_total,
        "recall": recall, "recall_queries": n_gt,
        "build_seconds": build_t,
        "roofline": {"bound": "hbm", "kernel": kname, "achieved": achieved,
                     "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": achieved / HBM_PEAK_GBS,
                     "traffic": (code_bytes * MEASURED_TRAFFIC_RATIO[traffic_key]
                                 if traffic_key in MEASURED_TRAFFIC_RATIO and plain else None),
                     "algorithmic_bytes_per_launch": code_bytes,
                     "avg_launch_ms": k_ms,
                     # every estimate is m random LDS reads of 4 bytes (2 with fp16 tables): the scan's other limiter
                     "lds": {"achieved": lds_b * code_bytes / (k_ms * 1e-3) / 1e9 if k_ms > 0 else 0.0,
                             "peak": LDS_PEAK_GBS, "unit": "GB/s",
                             "frac": (lds_b * code_bytes / (k_ms * 1e-3) / 1e9 / LDS_PEAK_GBS) if k_ms > 0 else 0.0}},
    }
    if args.sharing != 0:
        # The same workload with every (query, list) pair scanned on its own (no reuse of a code read between
        # queries): the HBM-bound form of the scan, three steps outside the timed region.
        ix.set_list_sharing(0)
        ix.set_profiling(True)
        ix.search(batches[0], cfg.w, cfg.kprime, cfg.k)
        pp_ms, pp_codes, pp_wall = 0.0, 0, 0.0
        for s in range(3):
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            ix.search(batches[s % n_batches], cfg.w, cfg.kprime, cfg.k)
            torch.cuda.synchronize()
            pp_wall += time.perf_counter() - t0
            pp_ms += ix.stage_times()["scan"]
            pp_codes += ix.search_stats()["codes_scanned"]
        ix.set_profiling(False)
        ix.set_list_sharing(args.sharing)
        pp_bytes = cfg.m * pp_codes / 3.0
        pp_gbs = pp_bytes / (pp_ms / 3.0 * 1e-3) / 1e9 if pp_ms > 0 else 0.0
        key = (cfg.name, "adc_scan_kernel")
        out["roofline_per_pair"] = {"bound": "hbm", "kernel": "adc_scan_kernel", "achieved": pp_gbs, "peak": HBM_PEAK_GBS,
                                    "unit": "GB/s", "frac": pp_gbs / HBM_PEAK_GBS,
                                    "traffic": (pp_bytes * MEASURED_TRAFFIC_RATIO[key]
                                                if key in MEASURED_TRAFFIC_RATIO and plain else None),
                                    "algorithmic_bytes_per_launch": pp_bytes, "avg_launch_ms": pp_ms / 3.0,
                                    "ms_per_step": 1e3 * pp_wall / 3.0, "list_sharing_mode": 0}
    if cfg.n_query > B and not args.batch and not args.no_whole_set:
        # The workload's whole query set in one call (outside the timed region): more queries share every list read.
        ix.set_tuning(batch=min(cfg.n_query, 65535))
        ix.search(xq, cfg.w, cfg.kprime, cfg.k)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(3):
            a_ids, _ = ix.search(xq, cfg.w, cfg.kprime, cfg.k)
        torch.cuda.synchronize()
        el = (time.perf_counter() - t0) / 3.0
        out["whole_query_set_per_call"] = {"queries_per_call": cfg.n_query, "ms_per_call": 1e3 * el,
                                           "queries_per_s": cfg.n_query / el,
                                           "first_batch_ids_identical": bool((a_ids[:B].cpu().numpy() == g_ids).all())}
        ix.set_tuning(batch=min(B, 65535))
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(ix, cfg, queries_u8, g_ids)
    ix.close()
    print(json.dumps(out))


if __name__ == "__main__":
    main()
