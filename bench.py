#!/usr/bin/env python3
"""Benchmark of the GPU embedding-cache hot path on one MI355X.

A step is one pass of the hot path over one batch: one hps_cache_query call (hash, probe,
row gather, miss compaction) on 4096 x 26 = 106,496 Zipf(1.05) keys against the hot cache of
the "query-only hot cache" workload: 2^21 sets x 8 ways, rows of 128 fp32 (8 GiB of rows),
prefilled from ids 2^24-1 .. 0.  All inputs are resident in HBM before the timed region.

Prints one JSON line: Mkeys/s as `value`, the HBM roofline of the query kernel (algorithmic
bytes per launch / measured time per launch / 8 TB/s) and the CPU oracle timed on the host
cores on a bounded sample of the same batches.
"""
import argparse
import ctypes as C
import json
import os
import sys
import threading
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0
METRIC = "cache query Mkeys/s + achieved HBM GB/s (dim 128 fp32, Zipf keys)"


def parse():
    p = argparse.ArgumentParser()
    p.add_argument("--gpus", type=int, default=1)
    p.add_argument("--workload", choices=["query", "refresh", "refresh-host", "stream", "multi", "concurrent", "dedup", "write", "lookup"], default="query",
                   help="query: the headline hot-cache query (default); refresh: dump every cached key, then "
                        "update every cached row (the paper's Table 3); stream: query + miss fill + insert per "
                        "step on a cold cache; multi: 26 tables in one launch; concurrent: queries on one "
                        "stream while updates run on another")
    p.add_argument("--capacity-gb", type=float, default=10.0, help="refresh: bytes of rows in the cache")
    p.add_argument("--policy", choices=["counter", "lru"], default="counter",
                   help="replacement policy of the cache: per-set victim counter (default) or the paper's LRU stamps")
    p.add_argument("--steps", type=int, default=1000)
    p.add_argument("--warmup", type=int, default=50)
    p.add_argument("--log2-sets", type=int, default=21)
    p.add_argument("--ways", type=int, default=8)
    p.add_argument("--dim", type=int, default=128)
    p.add_argument("--samples", type=int, default=4096)
    p.add_argument("--features", type=int, default=26)
    p.add_argument("--alpha", type=float, default=1.05)
    p.add_argument("--key-space", type=int, default=10 ** 8)
    p.add_argument("--keys", choices=["zipf", "uniform-resident"], default="zipf",
                   help="uniform-resident: distinct-ish uniform ids below the prefilled range (diagnostic)")
    p.add_argument("--out-buffers", type=int, default=16)
    p.add_argument("--repeats", type=int, default=5)
    p.add_argument("--coherent", type=int, default=0,
                   help="1: queries validate rows against concurrent writers (not needed for a query-only run)")
    p.add_argument("--graph", type=int, default=0, help="1: replay the timed launches from one HIP graph")
    p.add_argument("--streams", type=int, default=3,
                   help="also time the same batches issued round-robin over this many streams (0: skip)")
    p.add_argument("--threshold", type=float, default=0.8, help="lookup: hit-rate threshold t of Alg. 1")
    p.add_argument("--instances", type=int, default=1,
                   help="lookup: concurrent workers (threads), each with its own lookup object and stream, on one cache")
    p.add_argument("--no-cpu-baseline", action="store_true")
    p.add_argument("--cpu-batches", type=int, default=1000)        # about 10 s of the oracle on one host core
    p.add_argument("--batched", type=int, default=4,
                   help="also time the same batches k per launch (0 or 1: skip)")
    p.add_argument("--no-checked", dest="also_checked", action="store_false",
                   help="skip the extra timing of the checked (library default) query mode")
    p.add_argument("--no-ceiling", dest="ceiling", action="store_false",
                   help="skip the ceiling measurement (row gather with given slots, streaming copy)")
    p.add_argument("--calibrate-copy", action="store_true",
                   help="also run one plain 1 GiB device copy, membench_copy_kernel (reference for the rocprofv3 byte counters)")
    return p.parse_args()


# Paper, Table 3 (A100-80GB, fp32 rows of 128): cache capacity GB -> (update ms, dump ms)
PAPER_REFRESH = {1: (5.152, 0.064), 5: (25.177, 0.184), 10: (50.262, 0.335), 20: (100.530, 0.641),
                 40: (200.345, 1.19)}


def roofline_obj(kernel, alg_bytes, us, traffic=None, **extra):
    """HBM roofline of one kernel: algorithmic bytes per launch / measured time per launch / 8 TB/s."""
    gbs = alg_bytes / (us * 1e-6) / 1e9
    r = {"bound": "hbm", "achieved": round(gbs, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
         "frac": round(gbs / HBM_PEAK_GBS, 4), "traffic": traffic, "kernel": kernel,
         "algorithmic_bytes_per_launch": int(round(alg_bytes)), "us_per_launch": round(us, 3)}
    r.update(extra)
    return r


def query_alg_bytes(np, keys, miss_idx, d):
    """Algorithmic bytes of one query launch over the positions `keys` with the miss positions
    `miss_idx` (indices into keys): 8n + 64 D + 4d D_h + 4d n_h + 12 n_m + 4."""
    n, m = len(keys), len(miss_idx)
    D = np.unique(keys).size
    D_m = np.unique(keys[miss_idx]).size if m else 0
    return 8 * n + 64 * D + 4 * d * (D - D_m) + 4 * d * (n - m) + 12 * m + 4


def event_us(torch, fn, reps, warm=2):
    """Microseconds per call of fn() on the current stream (HIP events around `reps` calls)."""
    for _ in range(warm):
        fn()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    e0.record()
    for _ in range(reps):
        fn()
    e1.record()
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) * 1e3 / reps


def oracle_hot_cache(np, slots, W, d, chunk=1 << 18):
    """The CPU oracle with the hot-cache prefill (ids slots-1 .. 0 in descending chunks)."""
    from oracle import OracleCache
    oc = OracleCache(slots, W, d)
    rng = np.random.Generator(np.random.PCG64(0))
    filler = rng.integers(0, 1 << 32, size=(chunk, d), dtype=np.uint32)     # row content is irrelevant to timing
    for hi in range(slots, 0, -chunk):
        lo = max(0, hi - chunk)
        oc.insert(np.arange(hi - 1, lo - 1, -1, dtype=np.int64), filler[: hi - lo])
    return oc, filler


def refresh(a, np, torch, B):
    """Cache refresh (Sec. 6, steps 2-5; Table 3): Dump all cached keys, then Update every cached
    row from a device-resident key-vector buffer.  A step is one full refresh."""
    W, d = a.ways, a.dim
    slots = int(a.capacity_gb * 1e9 / (4 * d)) // (W * 1024) * (W * 1024)
    S = slots // W
    h = B.hps_cache_create(slots, W, d)
    B.hps_cache_set_concurrent_writers(h, True)
    chunk = 1 << 20
    ids = torch.empty(chunk, dtype=torch.int64, device="cuda")
    rows = torch.empty(chunk, d, dtype=torch.float32, device="cuda")
    for lo in range(0, 2 * slots, chunk):                 # 2x the slots, so that practically every slot fills
        m = min(chunk, 2 * slots - lo)
        ids[:m] = torch.arange(lo, lo + m, dtype=torch.int64, device="cuda")
        B.hps_backing_fetch(ids, m, d, version=0, rows=rows)
        B.hps_cache_insert(h, ids, rows, m)
    torch.cuda.synchronize()
    del ids, rows
    keys = torch.empty(slots, dtype=torch.int64, device="cuda")
    cnt = torch.zeros(1, dtype=torch.int32, device="cuda")
    newrows = torch.empty(slots, d, dtype=torch.float32, device="cuda")
    ev = lambda: torch.cuda.Event(enable_timing=True)
    t_dump, t_upd = [], []
    for it in range(a.warmup + a.steps):
        e0, e1, e2 = ev(), ev(), ev()
        e0.record()
        B.hps_cache_dump(h, 0, slots, keys, cnt)
        e1.record()
        m = int(cnt.item())                                # the host needs the count to size the lookup (Sec. 6 step 3)
        B.hps_backing_fetch(keys, m, d, version=it + 1, rows=newrows)
        torch.cuda.synchronize()
        e1b = ev()
        e1b.record()
        B.hps_cache_update(h, keys, newrows, m)
        e2.record()
        torch.cuda.synchronize()
        if it >= a.warmup:
            t_dump.append(e0.elapsed_time(e1))
            t_upd.append(e1b.elapsed_time(e2))
    # spot check: the cache now returns the rows of the last version
    from paper_2210_08804_amd import inputs
    probe = keys[:: max(1, m // 4096)][:4096].clone()
    out = torch.zeros(len(probe), d, dtype=torch.float32, device="cuda")
    mi = torch.empty(len(probe), dtype=torch.int32, device="cuda")
    mk = torch.empty(len(probe), dtype=torch.int64, device="cuda")
    nm = torch.zeros(1, dtype=torch.int32, device="cuda")
    B.hps_cache_query(h, probe, len(probe), out, mi, mk, nm)
    torch.cuda.synchronize()
    exp = inputs.backing_rows(probe.cpu().numpy(), d, a.warmup + a.steps)
    assert int(nm.item()) == 0 and (out.cpu().numpy().view(np.uint32) == exp.view(np.uint32)).all()
    upd_ms, dump_ms = float(np.median(t_upd)), float(np.median(t_dump))
    cap_gb = m * 4 * d / 1e9
    paper = PAPER_REFRESH.get(int(round(a.capacity_gb))) if abs(a.capacity_gb - round(a.capacity_gb)) < 1e-6 else None
    # per row: key, row in, row out; per set (the dumped keys of a set are adjacent and share them): key line, sequence word
    alg = m * (8 + 4 * d + 4 * d) + S * (8 * W + 8)
    res = {
        "metric": "cache refresh GB/s (cached bytes / Update time, dim 128 fp32)", "value": round(cap_gb / (upd_ms * 1e-3), 1),
        "unit": "GB/s", "n_gpus": 1, "steps": a.steps, "warmup": a.warmup, "ms_per_step": round(upd_ms + dump_ms, 4),
        "higher_is_better": True, "scaling": "weak",
        "vs_baseline": round((cap_gb / (upd_ms * 1e-3)) / (a.capacity_gb / (paper[0] * 1e-3)), 2) if paper else None,
        "dtype": "int64", "data": "synthetic",
        "config": {"workload": f"cache refresh: dump + update of all {m} cached rows ({cap_gb:.2f} GB of rows, {S} sets x {W} ways, dim {d})",
                   "update_ms": round(upd_ms, 4), "dump_ms": round(dump_ms, 4), "occupancy": round(m / slots, 4),
                   "paper_table3_A100": {"update_ms": paper[0], "dump_ms": paper[1]} if paper else None},
        "roofline": {"bound": "hbm", "achieved": round(alg / (upd_ms * 1e-3) / 1e9, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": round(alg / (upd_ms * 1e-3) / 1e9 / HBM_PEAK_GBS, 4), "traffic": None,
                     "kernel": "update_kernel<8>", "algorithmic_bytes_per_launch": alg,
                     "us_per_launch": round(upd_ms * 1e3, 1)},
    }
    if not a.no_cpu_baseline:
        # the oracle's Dump + Update on a bounded sample: a cache of 2^21 slots of the same row width
        from oracle import OracleCache
        cs = 1 << 21
        oc = OracleCache(cs, W, d)
        ids = np.arange(2 * cs, dtype=np.int64)
        filler = np.random.Generator(np.random.PCG64(0)).integers(0, 1 << 32, size=(1 << 18, d), dtype=np.uint32)
        for lo in range(0, 2 * cs, 1 << 18):
            oc.insert(ids[lo:lo + (1 << 18)], filler)
        t0 = time.perf_counter()
        dumped = oc.dump()
        for lo in range(0, len(dumped), 1 << 18):
            oc.update(dumped[lo:lo + (1 << 18)], filler[: len(dumped[lo:lo + (1 << 18)])])
        t1 = time.perf_counter()
        res["cpu_baseline"] = {"value": round(len(dumped) * 4 * d / (t1 - t0) / 1e9, 2), "unit": "GB/s", "cores": 1, "kind": "oracle",
                               "sample": f"dump + update of all {len(dumped)} cached rows of a {cs}-slot cache of the same row width"}
        oc.close()
    torch.cuda.synchronize()
    B.hps_cache_destroy(h)
    print(json.dumps(res))


def _prefill_descending(B, torch, h, n_ids, d, chunk=1 << 20):
    """Insert ids n_ids-1 .. 0 (hottest last) with rows from the device-side backing stand-in."""
    ids = torch.empty(chunk, dtype=torch.int64, device="cuda")
    rows = torch.empty(chunk, d, dtype=torch.float32, device="cuda")
    for hi in range(n_ids, 0, -chunk):
        lo = max(0, hi - chunk)
        m = hi - lo
        ids[:m] = torch.arange(hi - 1, lo - 1, -1, dtype=torch.int64, device="cuda")
        B.hps_backing_fetch(ids, m, d, version=0, rows=rows)
        B.hps_cache_insert(h, ids, rows, m)
    torch.cuda.synchronize()


def stream_fill(a, np, torch, B, inputs):
    """Streaming query + miss fill (Alg. 1, synchronous branch, all on the device): per step query
    16384 x 26 Zipf(1.1) keys, fetch the missing rows from the backing stand-in into `out` and a
    compact buffer, insert them.  Cold start; the hit rate per step shows the warm-up."""
    S, W, d = 1 << 20, 8, a.dim
    n = 16384 * 26
    steps = min(a.steps, 500)
    h = (B.hps_cache_create(S * W, W, d) if a.policy == "counter"
         else B.hps_cache_create_policy(S * W, W, d, B.HPS_POLICY_LRU))
    B.hps_cache_set_concurrent_writers(h, False)
    keys = [torch.from_numpy(inputs.zipf_keys(n, 10 ** 8, 1.1, s + 1)).cuda() for s in range(steps)]
    out = torch.empty(n, d, dtype=torch.float32, device="cuda")
    rows = torch.empty(n, d, dtype=torch.float32, device="cuda")
    mi = torch.empty(n, dtype=torch.int32, device="cuda")
    mk = torch.empty(n, dtype=torch.int64, device="cuda")
    nm = torch.zeros(steps, dtype=torch.int32, device="cuda")
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(steps + 1)]
    evq = [torch.cuda.Event(enable_timing=True) for _ in range(steps)]
    mis = [torch.empty(n, dtype=torch.int32, device="cuda") for _ in range(4)]      # the last steps' miss lists are kept
    torch.cuda.synchronize()
    ev[0].record()
    for s in range(steps):
        mi = mis[s % 4]
        B.hps_cache_query(h, keys[s], n, out, mi, mk, nm[s:s + 1])
        evq[s].record()
        B.hps_backing_fetch(mk, n, d, version=0, rows=rows, n_dev=nm[s:s + 1], scatter_idx=mi, scatter_out=out)
        B.hps_cache_insert_dn(h, mk, rows, n, nm[s:s + 1])
        ev[s + 1].record()
    torch.cuda.synchronize()
    ms = np.array([ev[s].elapsed_time(ev[s + 1]) for s in range(steps)])
    q_us = np.array([ev[s].elapsed_time(evq[s]) for s in range(steps)]) * 1e3
    hit = 1.0 - nm.cpu().numpy() / n
    tail = slice(steps // 2, steps)
    # algorithmic bytes of the query launches of the last four steps (their miss lists are still there)
    algs = []
    for s in range(max(0, steps - 4), steps):
        m = int(nm[s].item())
        algs.append(query_alg_bytes(np, keys[s].cpu().numpy(), mis[s % 4][:m].cpu().numpy().view(np.uint32), d))
    res = {"metric": "streaming lookup Mkeys/s (query + miss fill + insert per step)", "value": round(n / (ms[tail].mean() * 1e-3) / 1e6, 1),
           "unit": "Mkeys/s", "n_gpus": 1, "steps": steps, "warmup": 0, "ms_per_step": round(float(ms[tail].mean()), 4),
           "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "int64", "data": "synthetic",
           "config": {"workload": f"streaming query + miss fill: {S} sets x {W} ways, dim {d}, {n} Zipf(1.1) keys over 1e8 per step, cold start",
                      "replacement_policy": a.policy,
                      "hit_rate_per_step": [round(float(x), 4) for x in hit[: 10]] + ["..."] + [round(float(x), 4) for x in hit[-5:]],
                      "ms_per_step_first10": [round(float(x), 3) for x in ms[:10]],
                      "query_us_per_step_last4": [round(float(x), 1) for x in q_us[-4:]]},
           "roofline": roofline_obj("query_kernel<ways=8, checked=False> (the longest of the step's three kernels)",
                                    float(np.mean(algs)), float(np.mean(q_us[-4:])))}
    if not a.no_cpu_baseline:
        # the oracle running the same steps (query, rows of the missing keys from the generator, insert): first 12 steps
        from oracle import OracleCache
        oc = OracleCache(S * W, W, d, policy=0 if a.policy == "counter" else 1)
        nb = min(12, steps)
        out_cpu = np.empty((n, d), dtype=np.uint32)
        hk = [keys[s].cpu().numpy() for s in range(nb)]
        t0 = time.perf_counter()
        for s in range(nb):
            _, omi, omk = oc.query(hk[s], out_cpu)
            r = inputs.backing_rows(omk, d, 0)
            out_cpu[omi] = r.view(np.uint32)
            oc.insert(omk, r)
        t1 = time.perf_counter()
        res["cpu_baseline"] = {"value": round(nb * n / (t1 - t0) / 1e6, 2), "unit": "Mkeys/s", "cores": 1, "kind": "oracle",
                               "sample": f"the first {nb} steps of the same key stream (cold start, so more misses per step than the stable stage)"}
        oc.close()
    torch.cuda.synchronize()
    B.hps_cache_destroy(h)
    print(json.dumps(res))


def dedup_lookup(a, np, torch, B, inputs):
    """The hot-cache batch looked up two ways: directly (every position answered by the query
    kernel), and as Sec. 2.2 prescribes: Q* = dedup(Q), query Q*, expand to the positions.  Reports
    the time of each stage; `value` is the rate of the deduplicated path."""
    S, W, d = 1 << a.log2_sets, a.ways, a.dim
    n = a.samples * a.features
    steps, warm = min(a.steps, 300), min(a.warmup, 20)
    h = B.hps_cache_create(S * W, W, d)
    _prefill_descending(B, torch, h, S * W, d, chunk=1 << 18)
    B.hps_cache_set_concurrent_writers(h, False)
    dd = B.hps_dedup_create(n)
    keys = [torch.from_numpy(inputs.zipf_keys(n, a.key_space, a.alpha, s + 1)).cuda() for s in range(steps + warm)]
    out = torch.empty(n, d, dtype=torch.float32, device="cuda")
    urows = torch.empty(n, d, dtype=torch.float32, device="cuda")
    uk = torch.empty(n, dtype=torch.int64, device="cuda")
    inv = torch.empty(n, dtype=torch.int32, device="cuda")
    nu = torch.zeros(steps + warm, dtype=torch.int32, device="cuda")
    mi = torch.empty(n, dtype=torch.int32, device="cuda")
    mk = torch.empty(n, dtype=torch.int64, device="cuda")
    nm = torch.zeros(1, dtype=torch.int32, device="cuda")

    def timed(fn):
        for s in range(warm):
            fn(s)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        e0.record()
        for s in range(warm, warm + steps):
            fn(s)
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / steps * 1e3

    t_direct = timed(lambda s: B.hps_cache_query(h, keys[s], n, out, mi, mk, nm))
    t_dedup = timed(lambda s: B.hps_dedup(dd, keys[s], n, uk, inv, nu[s:s + 1]))
    n_u = nu[warm:].cpu().numpy()
    counts = nu.cpu().numpy().tolist()

    def path(s):                                   # no host round trip: the query reads the count on the device
        B.hps_dedup(dd, keys[s], n, uk, inv, nu[s:s + 1])
        B.hps_cache_query_dn(h, uk, n, nu[s:s + 1], urows, mi, mk, nm)
        B.hps_expand_rows(urows, inv, n, d, out)

    t_path = timed(path)
    t_q = timed(lambda s: B.hps_cache_query(h, uk, counts[s], urows, mi, mk, nm))
    t_x = timed(lambda s: B.hps_expand_rows(urows, inv, n, d, out))
    res = {"metric": "deduplicated lookup Mkeys/s (dedup + query of distinct keys + expand)", "value": round(n / t_path, 1),
           "unit": "Mkeys/s", "n_gpus": 1, "steps": steps, "warmup": warm, "ms_per_step": round(t_path * 1e-3, 5),
           "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "int64", "data": "synthetic",
           "config": {"workload": f"dedup in front of the hot-cache query: {S} sets x {W} ways, dim {d}, {n} Zipf({a.alpha}) keys over {a.key_space}",
                      "distinct_fraction": round(float(n_u.mean()) / n, 4),
                      "us": {"direct_query": round(t_direct, 2), "dedup": round(t_dedup, 2), "query_distinct": round(t_q, 2),
                             "expand": round(t_x, 2), "dedup+query+expand": round(t_path, 2)}},
           # expand is the stage that moves the bytes: n rows written, the distinct rows read, 4 bytes of map per position
           "roofline": roofline_obj("expand_rows_kernel", float(n * 4 * d + n_u.mean() * 4 * d + 4 * n), t_x,
                                    note="the dedup kernels themselves move 20 bytes per key and are bound by dependent atomics, not by bytes")}
    if not a.no_cpu_baseline:
        import oracle
        hk = keys[warm].cpu().numpy()
        t0 = time.perf_counter()
        ou, oinv = oracle.dedup(hk)
        t1 = time.perf_counter()
        res["cpu_baseline"] = {"value": round(n / (t1 - t0) / 1e6, 3), "unit": "Mkeys/s", "cores": 1, "kind": "oracle",
                               "sample": "dedup of one batch by the oracle's definition (every key compared with the distinct keys so far)"}
    torch.cuda.synchronize()
    B.hps_dedup_destroy(dd)
    B.hps_cache_destroy(h)
    print(json.dumps(res))


def write_batches(a, np, torch, B, inputs):
    """Insert and update in isolation: batches of `--samples x --features` (default 2^18 when
    --samples is left at 4096: 10082 x 26 is rounded to 2^18) new keys into the hot-cache
    geometry, then updates of the same keys.  A step is one insert call plus one update call."""
    S, W, d = 1 << a.log2_sets, a.ways, a.dim
    n = 1 << 18 if a.samples == 4096 else a.samples * a.features
    steps = min(a.steps, (S * W) // n, 32)
    h = B.hps_cache_create(S * W, W, d)
    rows = torch.empty(n, d, dtype=torch.float32, device="cuda")
    ids = torch.arange(n, dtype=torch.int64, device="cuda")
    B.hps_backing_fetch(ids, n, d, 0, rows=rows)
    ev = lambda: torch.cuda.Event(enable_timing=True)
    t_ins, t_upd = [], []
    for c in range(steps):
        k = ids + c * n
        e0, e1, e2 = ev(), ev(), ev()
        torch.cuda.synchronize()
        e0.record()
        B.hps_cache_insert(h, k, rows, n)
        e1.record()
        B.hps_cache_update(h, k, rows, n)
        e2.record()
        torch.cuda.synchronize()
        t_ins.append(e0.elapsed_time(e1))
        t_upd.append(e1.elapsed_time(e2))
    ins_us, upd_us = float(np.median(t_ins)) * 1e3, float(np.median(t_upd)) * 1e3
    row_b = 4 * d
    alg_ins = n * (8 + 64 + 2 * row_b + 8 + 8)          # key, key line, row read + written, key + counter/word stores
    res = {"metric": "insert + update of one batch, Mrows/s", "value": round(n / (ins_us + upd_us), 1), "unit": "Mrows/s",
           "n_gpus": 1, "steps": steps, "warmup": 0, "ms_per_step": round((ins_us + upd_us) * 1e-3, 5), "higher_is_better": True,
           "scaling": "weak", "vs_baseline": None, "dtype": "int64", "data": "synthetic",
           "config": {"workload": f"insert of {n} new keys, then update of the same keys: {S} sets x {W} ways, dim {d}",
                      "insert_us": round(ins_us, 1), "update_us": round(upd_us, 1),
                      "insert_rows_GBps": round(n * 2 * row_b / ins_us / 1e3, 1), "update_rows_GBps": round(n * 2 * row_b / upd_us / 1e3, 1)},
           "roofline": roofline_obj("insert_kernel<8,16>", alg_ins, ins_us),
           "roofline_update": roofline_obj("update_kernel<8,64>", n * (8 + 64 + 2 * row_b + 8), upd_us)}
    if not a.no_cpu_baseline:
        from oracle import OracleCache
        oc = OracleCache(S * W, W, d)
        hrows = rows.cpu().numpy().view(np.uint32)
        nb = min(steps, 8)
        t_i = t_u = 0.0
        for c in range(nb):
            k = np.arange(c * n, (c + 1) * n, dtype=np.int64)
            t0 = time.perf_counter()
            oc.insert(k, hrows)
            t1 = time.perf_counter()
            oc.update(k, hrows)
            t2 = time.perf_counter()
            t_i += t1 - t0
            t_u += t2 - t1
        res["cpu_baseline"] = {"value": round(nb * n / (t_i + t_u) / 1e6, 2), "unit": "Mrows/s", "cores": 1, "kind": "oracle",
                               "sample": f"the first {nb} batches of the same keys: insert {round(nb * n / t_i / 1e6, 2)} Mrows/s, update {round(nb * n / t_u / 1e6, 2)} Mrows/s"}
        oc.close()
    torch.cuda.synchronize()
    B.hps_cache_destroy(h)
    print(json.dumps(res))


def _lookup_instances(a, np, torch, B, inputs, h, hm, fetch, n, space, S, W, d, steps):
    """Several inference workers on one cache (Sec. 7.2.2): each thread has its own lookup object,
    stream and key stream; `value` is the aggregate rate over the second half of the calls."""
    import threading
    import time as _time
    k = a.instances
    lks = [B.hps_lookup_create(h, n, a.threshold, np.zeros(d, np.float32), fetch, user=hm) for _ in range(k)]
    keys = [[torch.from_numpy(inputs.zipf_keys(n, space, 1.2, 1000 * t + s + 1)).cuda() for s in range(steps)] for t in range(k)]
    outs = [torch.empty(n, d, dtype=torch.float32, device="cuda") for _ in range(k)]
    torch.cuda.synchronize()
    stamps = [[0.0] * (steps + 1) for _ in range(k)]
    rates = [[0.0] * steps for _ in range(k)]
    barrier = threading.Barrier(k)

    def worker(t):
        torch.cuda.set_device(0)
        st = torch.cuda.Stream()
        barrier.wait()
        stamps[t][0] = _time.perf_counter()
        for s in range(steps):
            r, _ = B.hps_lookup(lks[t], keys[t][s], n, outs[t], st)
            st.synchronize()
            stamps[t][s + 1] = _time.perf_counter()
            rates[t][s] = r

    threads = [threading.Thread(target=worker, args=(t,)) for t in range(k)]
    for th in threads:
        th.start()
    for th in threads:
        th.join()
    for lk in lks:
        B.hps_lookup_drain(lk)
    half = steps // 2
    t_begin = min(stamps[t][half] for t in range(k))
    t_end = max(stamps[t][steps] for t in range(k))
    lat = np.array([stamps[t][s + 1] - stamps[t][s] for t in range(k) for s in range(half, steps)]) * 1e3
    value = k * n * (steps - half) / (t_end - t_begin) / 1e6
    res = {"metric": "Alg. 1 lookup Mkeys/s, several workers on one cache (stable stage, aggregate)", "value": round(value, 1),
           "unit": "Mkeys/s", "n_gpus": 1, "steps": steps, "warmup": 0, "ms_per_step": round(float(lat.mean()), 4),
           "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "int64", "data": "synthetic",
           "config": {"workload": f"{k} threads x hps_lookup: {n} Zipf(1.2) keys per call over {space} keys, one cache of {S} sets x {W} ways x dim {d}, "
                                  f"threshold {a.threshold}, lower tier = host map", "replacement_policy": a.policy, "instances": k,
                      "latency_ms_stable": {"mean": round(float(lat.mean()), 4), "p50": round(float(np.median(lat)), 4),
                                            "p99": round(float(np.percentile(lat, 99)), 4)},
                      "hit_rate_stable": round(float(np.mean([rates[t][s] for t in range(k) for s in range(half, steps)])), 4)}}
    for lk in lks:
        B.hps_lookup_destroy(lk)
    torch.cuda.synchronize()
    B.hps_cache_destroy(h)
    B.hps_hostmap_destroy(hm)
    print(json.dumps(res))


def lookup_alg1(a, np, torch, B, inputs):
    """Algorithm 1 end to end: hps_lookup on a cold cache with the library's host map as the lower
    tier (2^22 keys x dim fp32 in host memory), cache = 5 % of the key space, batches of
    1024 x 26 Zipf(1.2) keys (the paper's serving batch, Sec. 7.2).  A step is one hps_lookup call,
    timed on the host (the call returns when `out` is complete); the background insertions of the
    asynchronous mode overlap later calls."""
    import time as _time
    d, W = a.dim, a.ways
    space = 1 << 22
    S = (space // 20) // W
    n = 1024 * a.features
    steps = min(a.steps, 300)
    hm = B.hps_hostmap_create(d, 16, space)
    chunk = 1 << 19
    ids = torch.empty(chunk, dtype=torch.int64, device="cuda")
    rows = torch.empty(chunk, d, dtype=torch.float32, device="cuda")
    for lo in range(0, space, chunk):                     # rows generated on the device, stored on the host
        ids.copy_(torch.arange(lo, lo + chunk, dtype=torch.int64, device="cuda"))
        B.hps_backing_fetch(ids, chunk, d, version=0, rows=rows)
        B.hps_hostmap_put(hm, ids.cpu().numpy(), rows.cpu().numpy())
    del ids, rows
    h = (B.hps_cache_create(S * W, W, d) if a.policy == "counter"
         else B.hps_cache_create_policy(S * W, W, d, B.HPS_POLICY_LRU))
    fetch = B.hps_hostmap_fetch_fn()
    if a.instances > 1:
        return _lookup_instances(a, np, torch, B, inputs, h, hm, fetch, n, space, S, W, d, steps)
    lk = B.hps_lookup_create(h, n, a.threshold, np.zeros(d, np.float32), fetch, user=hm)
    keys = [torch.from_numpy(inputs.zipf_keys(n, space, 1.2, s + 1)).cuda() for s in range(steps)]
    out = torch.empty(n, d, dtype=torch.float32, device="cuda")
    torch.cuda.synchronize()
    lat, rate, mode = [], [], []
    for s in range(steps):
        t0 = _time.perf_counter()
        r, sync = B.hps_lookup(lk, keys[s], n, out)
        torch.cuda.synchronize()
        lat.append((_time.perf_counter() - t0) * 1e3)
        rate.append(r)
        mode.append(sync)
    B.hps_lookup_drain(lk)
    lat = np.array(lat)
    tail = slice(steps // 2, steps)
    first_async = next((i for i, m in enumerate(mode) if not m), None)
    res = {"metric": "Alg. 1 lookup Mkeys/s (hps_lookup with a host-memory lower tier, stable stage)",
           "value": round(n / (lat[tail].mean() * 1e-3) / 1e6, 1), "unit": "Mkeys/s", "n_gpus": 1, "steps": steps, "warmup": 0,
           "ms_per_step": round(float(lat[tail].mean()), 4), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
           "dtype": "int64", "data": "synthetic",
           "config": {"workload": f"hps_lookup: {n} Zipf(1.2) keys per call over {space} keys, cache {S} sets x {W} ways x dim {d} (5 % of the keys), "
                                  f"threshold {a.threshold}, lower tier = host map", "replacement_policy": a.policy,
                      "first_asynchronous_call": first_async,
                      "hit_rate_every_25_calls": [round(float(x), 3) for x in rate[::25]],
                      "latency_ms_first10": [round(float(x), 3) for x in lat[:10]],
                      "latency_ms_stable": {"mean": round(float(lat[tail].mean()), 4), "p50": round(float(np.median(lat[tail])), 4),
                                            "p99": round(float(np.percentile(lat[tail], 99)), 4)},
                      "hit_rate_first10": [round(float(x), 4) for x in rate[:10]],
                      "hit_rate_stable": round(float(np.mean(rate[steps // 2:])), 4)}}
    B.hps_lookup_destroy(lk)
    torch.cuda.synchronize()
    # The call's time is host work (one stream synchronisation, the call sequence, the lower tier);
    # the one kernel that moves rows is the checked query, timed here alone on the last batches
    mi = torch.empty(n, dtype=torch.int32, device="cuda")
    mk = torch.empty(n, dtype=torch.int64, device="cuda")
    nm = torch.zeros(1, dtype=torch.int32, device="cuda")
    cnt = [0]

    def one():
        B.hps_cache_query(h, keys[steps - 1 - cnt[0] % 8], n, out, mi, mk, nm)
        cnt[0] += 1
    q_us = event_us(torch, one, 200, warm=8)
    B.hps_cache_query(h, keys[steps - 1], n, out, mi, mk, nm)
    torch.cuda.synchronize()
    m0 = int(nm.item())
    alg = query_alg_bytes(np, keys[steps - 1].cpu().numpy(), mi[:m0].cpu().numpy().view(np.uint32), d)
    res["roofline"] = roofline_obj("query_kernel<ways=8, checked=True> (the call's row-moving kernel, timed alone)", alg, q_us,
                                   note="a lookup call is bound by host work and the lower tier, not by this kernel")
    if not a.no_cpu_baseline:
        # the oracle's Alg. 1 on the first 40 calls, rows of the lower tier from the generator
        from oracle import OracleCache
        oc = OracleCache(S * W, W, d, policy=0 if a.policy == "counter" else 1)
        nb = min(40, steps)
        hk = [keys[s].cpu().numpy() for s in range(nb)]
        lower = [inputs.backing_rows(k, d, 0) for k in hk]
        t0 = time.perf_counter()
        for s in range(nb):
            oc.lookup(hk[s], lower[s], a.threshold, np.zeros(d, np.float32))
        t1 = time.perf_counter()
        res["cpu_baseline"] = {"value": round(nb * n / (t1 - t0) / 1e6, 2), "unit": "Mkeys/s", "cores": 1, "kind": "oracle",
                               "sample": f"the first {nb} calls of the same key stream (cold start), lower-tier rows prepared beforehand"}
        oc.close()
    B.hps_cache_destroy(h)
    B.hps_hostmap_destroy(hm)
    print(json.dumps(res))


def refresh_from_host(a, np, torch, B, inputs):
    """The whole refresh cycle of Sec. 6 with the lower tier in host memory (hps_cache_refresh):
    dump, copy of the keys to the host, lookup in the host map, upload, Update, in batches of 2^18
    slots, the host lookup of one batch overlapping the upload and Update of the previous one.
    A step is one refresh of a full cache of 2^22 rows (2 GiB at dim 128)."""
    import time as _time
    d, W = a.dim, a.ways
    n_keys = 1 << 22
    S = n_keys // W
    hm = B.hps_hostmap_create(d, 16, n_keys)
    h = B.hps_cache_create(S * W, W, d)
    chunk = 1 << 19
    ids = torch.empty(chunk, dtype=torch.int64, device="cuda")
    rows = torch.empty(chunk, d, dtype=torch.float32, device="cuda")
    for lo in range(0, n_keys, chunk):
        ids.copy_(torch.arange(lo, lo + chunk, dtype=torch.int64, device="cuda"))
        B.hps_backing_fetch(ids, chunk, d, version=0, rows=rows)
        B.hps_cache_insert(h, ids, rows, chunk)
        B.hps_backing_fetch(ids, chunk, d, version=1, rows=rows)
        B.hps_hostmap_put(hm, ids.cpu().numpy(), rows.cpu().numpy())
    torch.cuda.synchronize()
    del ids, rows
    fetch = B.hps_hostmap_fetch_fn()
    steps = max(1, min(a.steps, 5))
    times, n = [], 0
    rs = B.hps_refresh_create(h, 1 << 18)                  # buffers, stream and events allocated once
    for _ in range(steps):
        t0 = _time.perf_counter()
        n = B.hps_refresh_run(rs, fetch, user=hm)
        torch.cuda.synchronize()
        times.append(_time.perf_counter() - t0)
    B.hps_refresh_destroy(rs)
    ms = float(np.median(times)) * 1e3
    gb = n * 4 * d / 1e9
    res = {"metric": "cache refresh from a host-memory lower tier, GB/s of cached rows", "value": round(gb / (ms * 1e-3), 2), "unit": "GB/s",
           "n_gpus": 1, "steps": steps, "warmup": 0, "ms_per_step": round(ms, 2), "higher_is_better": True, "scaling": "weak",
           "vs_baseline": None, "dtype": "int64", "data": "synthetic",
           "config": {"workload": f"hps_cache_refresh: {n} cached rows of dim {d} ({gb:.2f} GB), batches of 262144 slots, lower tier = host map of {n_keys} keys",
                      "Mkeys_per_s": round(n / (ms * 1e-3) / 1e6, 1)}}
    # the cycle is bound by the host map; its row-moving kernel is the Update of one batch of 2^18 slots, timed alone
    m = 1 << 18
    dk = torch.empty(m, dtype=torch.int64, device="cuda")
    cntw = torch.zeros(1, dtype=torch.int32, device="cuda")
    B.hps_cache_dump(h, 0, m, dk, cntw)
    torch.cuda.synchronize()
    mm = int(cntw.item())
    drows = torch.empty(m, d, dtype=torch.float32, device="cuda")
    B.hps_backing_fetch(dk, mm, d, version=1, rows=drows)
    u_us = event_us(torch, lambda: B.hps_cache_update(h, dk, drows, mm), 20, warm=2)
    res["roofline"] = roofline_obj("update_kernel<8,64> (one batch of the cycle, timed alone)",
                                   mm * (8 + 2 * 4 * d) + (m // W) * (8 * W + 8), u_us,
                                   note="the refresh cycle as a whole is bound by the host-memory lower tier")
    if not a.no_cpu_baseline:
        from oracle import OracleCache
        oc = OracleCache(S * W, W, d)
        ids = np.arange(n_keys, dtype=np.int64)
        filler = np.random.Generator(np.random.PCG64(0)).integers(0, 1 << 32, size=(1 << 18, d), dtype=np.uint32)
        for lo in range(0, n_keys, 1 << 18):
            oc.insert(ids[lo:lo + (1 << 18)], filler)
        t0 = _time.perf_counter()
        dumped = oc.dump()
        for lo in range(0, len(dumped), 1 << 18):
            oc.update(dumped[lo:lo + (1 << 18)], filler[: len(dumped[lo:lo + (1 << 18)])])
        t1 = _time.perf_counter()
        res["cpu_baseline"] = {"value": round(len(dumped) * 4 * d / (t1 - t0) / 1e9, 2), "unit": "GB/s", "cores": 1, "kind": "oracle",
                               "sample": f"the oracle's dump + update of all {len(dumped)} cached rows, rows already in memory (no lower-tier lookup)"}
        oc.close()
    torch.cuda.synchronize()
    B.hps_cache_destroy(h)
    B.hps_hostmap_destroy(hm)
    print(json.dumps(res))


def multi_table(a, np, torch, B, inputs):
    """26 independent caches (vocabulary log-uniform in [1e3, 1e8], each cache 20 % of its vocabulary,
    at most 2^22 slots), one Zipf(1.05) key per table and sample, 131072 samples, one launch."""
    W, d, Bn = 8, a.dim, 131072
    vocab = inputs.log_uniform_vocab(26, 1e3, 1e8, 7)
    slots = [int(min(0.2 * v, 1 << 22)) // 8 * 8 for v in vocab]
    hs = []
    for s in slots:
        h = B.hps_cache_create(s, W, d)
        B.hps_cache_set_concurrent_writers(h, False)
        _prefill_descending(B, torch, h, s, d, chunk=1 << 18)
        hs.append(h)
    n = 26 * Bn
    nb = 8
    keys = [torch.from_numpy(np.stack([inputs.zipf_keys(Bn, int(v), 1.05, 7 + 1000 * t + 100000 * b)
                                       for t, v in enumerate(vocab)])).cuda() for b in range(nb)]
    outs = [torch.empty(n, d, dtype=torch.float32, device="cuda") for _ in range(2)]
    mi = torch.empty(n, dtype=torch.int32, device="cuda")
    mk = torch.empty(n, dtype=torch.int64, device="cuda")
    nm = torch.zeros(nb, dtype=torch.int32, device="cuda")
    for b in range(nb):
        B.hps_cache_query_multi(hs, keys[b], Bn, outs[b % 2], mi, mk, nm[b:b + 1])
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    reps = max(1, a.steps // nb)
    e0.record()
    for r in range(reps):
        for b in range(nb):
            B.hps_cache_query_multi(hs, keys[b], Bn, outs[b % 2], mi, mk, nm[b:b + 1])
    e1.record()
    torch.cuda.synchronize()
    ms = e0.elapsed_time(e1) / (reps * nb)
    hit = 1.0 - float(nm.cpu().numpy().mean()) / n
    # algorithmic bytes of one launch, exactly: the query formula per table on the realised batch 0
    B.hps_cache_query_multi(hs, keys[0], Bn, outs[0], mi, mk, nm[0:1])
    torch.cuda.synchronize()
    m0 = int(nm[0].item())
    midx = np.sort(mi[:m0].cpu().numpy().view(np.uint32).astype(np.int64))
    hk = keys[0].cpu().numpy()
    alg = 0
    for t in range(26):
        mt = midx[(midx >= t * Bn) & (midx < (t + 1) * Bn)] - t * Bn
        alg += query_alg_bytes(np, hk[t], mt, d) - 4
    alg += 4
    res = {"metric": "multi-table lookup Mkeys/s (26 tables, one launch)", "value": round(n / (ms * 1e-3) / 1e6, 1),
           "unit": "Mkeys/s", "n_gpus": 1, "steps": reps * nb, "warmup": nb, "ms_per_step": round(ms, 4),
           "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "int64", "data": "synthetic",
           "config": {"workload": f"26 caches, slots {min(slots)}..{max(slots)} (total {sum(slots)}), dim {d}, batch {Bn} samples x 26 keys",
                      "hit_rate": round(hit, 4), "out_write_GBps": round(n * hit * 4 * d / (ms * 1e-3) / 1e9, 1)},
           "roofline": roofline_obj("query_kernel<ways=8, checked=False>, 26 tables in one launch", alg, ms * 1e3)}
    if not a.no_cpu_baseline:
        # the oracle's 26 caches, filled the same way, queried table by table on batch 0
        from oracle import OracleCache
        filler = np.random.Generator(np.random.PCG64(0)).integers(0, 1 << 32, size=(1 << 18, d), dtype=np.uint32)
        ocs = []
        for sl in slots:
            oc = OracleCache(sl, W, d)
            for hi in range(sl, 0, -(1 << 18)):
                lo = max(0, hi - (1 << 18))
                oc.insert(np.arange(hi - 1, lo - 1, -1, dtype=np.int64), filler[: hi - lo])
            ocs.append(oc)
        out_cpu = np.empty((Bn, d), dtype=np.uint32)
        t0 = time.perf_counter()
        for t, oc in enumerate(ocs):
            oc.query(hk[t], out_cpu)
        t1 = time.perf_counter()
        res["cpu_baseline"] = {"value": round(n / (t1 - t0) / 1e6, 2), "unit": "Mkeys/s", "cores": 1, "kind": "oracle",
                               "sample": "one batch of 131072 samples x 26 tables, the oracle's caches prefilled in the same order"}
        for oc in ocs:
            oc.close()
    torch.cuda.synchronize()
    for h in hs:
        B.hps_cache_destroy(h)
    print(json.dumps(res))


def concurrent(a, np, torch, B, inputs):
    """Online update concurrent with query: 2^24 sets x 8 ways x dim (64 GiB at dim 128); queries of
    65536 x 26 Zipf(1.05) keys over 1e9 ids on one stream, updates of 262144 <key, row> pairs (half
    of the keys cached) on a second stream; both rates are reported, alone and overlapped."""
    S, W, d = 1 << 24, 8, a.dim
    n_q, n_u = 65536 * 26, 262144
    h = B.hps_cache_create(S * W, W, d)
    B.hps_cache_set_concurrent_writers(h, True)
    _prefill_descending(B, torch, h, S * W, d)
    nb = 6
    rng = np.random.Generator(np.random.PCG64(5))
    qk = [torch.from_numpy(inputs.zipf_keys(n_q, 10 ** 9, 1.05, 100 + b)).cuda() for b in range(nb)]
    uk = [torch.from_numpy(np.concatenate([rng.integers(0, S * W, n_u // 2), rng.integers(2 * 10 ** 9, 3 * 10 ** 9, n_u // 2)])
                           .astype(np.int64)).cuda() for b in range(nb)]
    urows = torch.empty(n_u, d, dtype=torch.float32, device="cuda")
    B.hps_backing_fetch(uk[0], n_u, d, version=1, rows=urows)
    outs = [torch.empty(n_q, d, dtype=torch.float32, device="cuda") for _ in range(2)]
    mi = torch.empty(n_q, dtype=torch.int32, device="cuda")
    mk = torch.empty(n_q, dtype=torch.int64, device="cuda")
    nm = torch.zeros(nb, dtype=torch.int32, device="cuda")
    qs, us = torch.cuda.Stream(), torch.cuda.Stream()
    torch.cuda.synchronize()

    def run(do_q, do_u, reps):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        e0.record()
        qs.wait_stream(torch.cuda.current_stream())
        us.wait_stream(torch.cuda.current_stream())
        for r in range(reps):
            for b in range(nb):
                if do_q:
                    B.hps_cache_query(h, qk[b], n_q, outs[b % 2], mi, mk, nm[b:b + 1], qs)
                if do_u:
                    for _ in range(2):
                        B.hps_cache_update(h, uk[b], urows, n_u, us)
        torch.cuda.current_stream().wait_stream(qs)
        torch.cuda.current_stream().wait_stream(us)
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / (reps * nb)

    run(True, True, 1)
    reps = max(1, a.steps // nb)
    q_alone, u_alone, both = run(True, False, reps), run(False, True, reps) / 2, run(True, True, reps)
    hit = 1.0 - float(nm.cpu().numpy().mean()) / n_q
    B.hps_cache_query(h, qk[0], n_q, outs[0], mi, mk, nm[0:1], qs)
    torch.cuda.synchronize()
    m0 = int(nm[0].item())
    alg_q = query_alg_bytes(np, qk[0].cpu().numpy(), mi[:m0].cpu().numpy().view(np.uint32), d)
    res = {"metric": "query Mkeys/s while updates run on a second stream", "value": round(n_q / (both * 1e-3) / 1e6, 1),
           "unit": "Mkeys/s", "n_gpus": 1, "steps": reps * nb, "warmup": nb, "ms_per_step": round(both, 4),
           "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "int64", "data": "synthetic",
           "config": {"workload": f"{S} sets x {W} ways, dim {d}; query {n_q} Zipf(1.05) keys over 1e9; 2 update batches of {n_u} pairs per query batch",
                      "hit_rate": round(hit, 4), "query_alone_ms": round(q_alone, 4), "update_batch_alone_ms": round(u_alone, 4),
                      "query_plus_2_updates_overlapped_ms": round(both, 4),
                      "query_alone_Mkeys_s": round(n_q / (q_alone * 1e-3) / 1e6, 1),
                      "update_alone_Mpairs_s": round(n_u / (u_alone * 1e-3) / 1e6, 1)},
           "roofline": roofline_obj("query_kernel<ways=8, checked=True>, alone on its stream", alg_q, q_alone * 1e3),
           "roofline_update": roofline_obj("update_kernel<8,64>, alone on its stream (half of the keys cached)",
                                           n_u * (8 + 64) + (n_u // 2) * (2 * 4 * d + 8), u_alone * 1e3)}
    if not a.no_cpu_baseline:
        # the oracle on a scaled-down geometry (2^21 sets instead of 2^24: the full one needs 64 GiB of host rows),
        # the same query keys folded into its id range, one query batch and one update batch
        oc, filler = oracle_hot_cache(np, (1 << 21) * W, W, d)
        kq = qk[0].cpu().numpy() % (1 << 25)
        ku = uk[0].cpu().numpy() % (1 << 25)
        out_cpu = np.empty((n_q, d), dtype=np.uint32)
        t0 = time.perf_counter()
        oc.query(kq, out_cpu)
        t1 = time.perf_counter()
        oc.update(ku, filler[:n_u] if len(filler) >= n_u else np.resize(filler, (n_u, d)))
        t2 = time.perf_counter()
        res["cpu_baseline"] = {"value": round(n_q / (t1 - t0) / 1e6, 2), "unit": "Mkeys/s", "cores": 1, "kind": "oracle",
                               "sample": (f"one query batch of {n_q} keys against a cache of 2^21 sets (an eighth of the workload's), "
                                          f"then one update batch: {round(n_u / (t2 - t1) / 1e6, 2)} Mpairs/s")}
        oc.close()
    torch.cuda.synchronize()
    B.hps_cache_destroy(h)
    print(json.dumps(res))


def main():
    a = parse()
    if a.gpus != 1:
        print(f"bench.py: this build runs on one GPU only (got --gpus {a.gpus}); "
              "with more GPUs each one would hold its own independent cache", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    from paper_2210_08804_amd import binding as B
    from paper_2210_08804_amd import inputs

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    lib = B.load_library()
    if a.workload == "refresh":
        return refresh(a, np, torch, B)
    if a.workload == "stream":
        return stream_fill(a, np, torch, B, inputs)
    if a.workload == "multi":
        return multi_table(a, np, torch, B, inputs)
    if a.workload == "concurrent":
        return concurrent(a, np, torch, B, inputs)
    if a.workload == "dedup":
        return dedup_lookup(a, np, torch, B, inputs)
    if a.workload == "write":
        return write_batches(a, np, torch, B, inputs)
    if a.workload == "lookup":
        return lookup_alg1(a, np, torch, B, inputs)
    if a.workload == "refresh-host":
        return refresh_from_host(a, np, torch, B, inputs)

    S, W, d = 1 << a.log2_sets, a.ways, a.dim
    slots = S * W
    n = a.samples * a.features
    n_batches = a.steps + a.warmup
    t_setup = time.time()

    # ---- cache + prefill: ids slots-1 .. 0 in descending chunks, rows from the device-side backing stand-in
    h = (B.hps_cache_create(slots, W, d) if a.policy == "counter"
         else B.hps_cache_create_policy(slots, W, d, B.HPS_POLICY_LRU))
    chunk = 1 << 18
    ids = torch.empty(chunk, dtype=torch.int64, device="cuda")
    rows = torch.empty(chunk, d, dtype=torch.float32, device="cuda")
    for hi in range(slots, 0, -chunk):
        lo = max(0, hi - chunk)
        m = hi - lo
        ids[:m] = torch.arange(hi - 1, lo - 1, -1, dtype=torch.int64, device="cuda")
        B.hps_backing_fetch(ids, m, d, version=0, rows=rows)
        B.hps_cache_insert(h, ids, rows, m)
    torch.cuda.synchronize()
    del rows, ids
    B.hps_cache_set_concurrent_writers(h, bool(a.coherent))

    # ---- key batches (seeds 1..), resident in HBM
    host_keys = np.empty((n_batches, n), dtype=np.int64)
    for b in range(n_batches):
        if a.keys == "zipf":
            host_keys[b] = inputs.zipf_keys(n, a.key_space, a.alpha, seed=b + 1)
        else:
            host_keys[b] = inputs.uniform_keys(n, slots, seed=b + 1)
    keys = torch.from_numpy(host_keys).cuda()
    outs = [torch.empty(n, d, dtype=torch.float32, device="cuda") for _ in range(a.out_buffers)]
    mi = torch.empty(n_batches, n, dtype=torch.int32, device="cuda")
    mk = torch.empty(a.out_buffers, n, dtype=torch.int64, device="cuda")
    nm = torch.zeros(n_batches, dtype=torch.int32, device="cuda")
    torch.cuda.synchronize()

    stream = torch.cuda.current_stream()
    sp = stream.cuda_stream
    kp, mip, mkp, nmp = keys.data_ptr(), mi.data_ptr(), mk.data_ptr(), nm.data_ptr()
    outp = [o.data_ptr() for o in outs]
    query = lib.hps_cache_query

    def launch(b):
        r = query(h, kp + b * n * 8, n, outp[b % a.out_buffers], mip + b * n * 4,
                  mkp + (b % a.out_buffers) * n * 8, nmp + b * 4, sp)
        if r != 0:
            raise RuntimeError(B.hps_last_error())

    for b in range(a.warmup):
        launch(b)
    torch.cuda.synchronize()

    graph = None
    if a.graph:
        graph = torch.cuda.CUDAGraph()
        cs = torch.cuda.Stream()
        with torch.cuda.stream(cs):
            sp_saved, sp = sp, cs.cuda_stream
            graph.capture_begin()
            for b in range(a.warmup, n_batches):
                launch(b)
            graph.capture_end()
            sp = sp_saved
        torch.cuda.synchronize()

    times = []
    for rep in range(a.repeats):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        e0.record(stream)
        if graph is not None:
            graph.replay()
        else:
            for b in range(a.warmup, n_batches):
                launch(b)
        e1.record(stream)
        torch.cuda.synchronize()
        times.append(e0.elapsed_time(e1))
    ms_total = float(np.median(times))
    ms_per_step = ms_total / a.steps
    mkeys = n / (ms_per_step * 1e-3) / 1e6

    # ---- the same batches issued round-robin over several streams (concurrent inference workers
    #      sharing one cache, Sec. 4.1): kernels of different batches overlap
    multi = None
    if a.streams > 1:
        ss = [torch.cuda.Stream() for _ in range(a.streams)]
        sps = [x.cuda_stream for x in ss]
        mtimes = []
        for rep in range(a.repeats):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            torch.cuda.synchronize()
            e0.record(stream)
            for x in ss:
                x.wait_stream(stream)
            for b in range(a.warmup, n_batches):
                sp = sps[b % a.streams]
                launch(b)
            for x in ss:
                stream.wait_stream(x)
            e1.record(stream)
            torch.cuda.synchronize()
            mtimes.append(e0.elapsed_time(e1))
        sp = stream.cuda_stream
        m_ms = float(np.median(mtimes)) / a.steps
        multi = {"streams": a.streams, "ms_per_step": round(m_ms, 5),
                 "value": round(n / (m_ms * 1e-3) / 1e6, 1), "unit": "Mkeys/s"}

    # ---- algorithmic bytes per launch (what the method must move), from the realised batches
    n_miss = nm.cpu().numpy()[a.warmup:].astype(np.int64)
    stat_b = list(range(a.warmup, n_batches, max(1, a.steps // 64)))
    alg = []
    distinct_frac = []
    for b in stat_b:
        m = int(nm[b].item())
        midx = mi[b][:m].cpu().numpy().view(np.uint32)
        alg.append(query_alg_bytes(np, host_keys[b], midx, d))
        distinct_frac.append(np.unique(host_keys[b]).size / n)
    alg_bytes = float(np.mean(alg))
    hit_rate = 1.0 - float(n_miss.mean()) / n

    traffic, traffic_source = None, None
    tpath = os.path.join(ROOT, "profiles", "query_c2_traffic.json")
    if a.keys == "zipf" and os.path.exists(tpath) and not a.coherent and n == 106496:
        try:
            traffic = json.load(open(tpath)).get("hbm_bytes_per_launch")
            traffic_source = ("recorded earlier with rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE (profiles/query_c2_traffic.json), "
                              "not measured in this run")
        except Exception:
            traffic = None

    if a.calibrate_copy:
        src = torch.empty(1 << 28, dtype=torch.float32, device="cuda")
        dst = torch.empty_like(src)
        B.hps_membench_copy(src, dst, 1 << 30, False)        # 1 GiB read + 1 GiB written, plain loads and stores
        torch.cuda.synchronize()
        del src, dst

    kernel_name = f"query_kernel<ways={W}, checked={bool(a.coherent)}>"
    result = {
        "metric": METRIC, "value": round(mkeys, 1), "unit": "Mkeys/s", "n_gpus": 1,
        "steps": a.steps, "warmup": a.warmup, "ms_per_step": round(ms_per_step, 5),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "int64", "data": "synthetic",
        "config": {
            "workload": (f"hot-cache query: {S} sets x {W} ways, dim {d} fp32, batch {a.samples}x{a.features}"
                         f" = {n} int64 keys, {a.keys} alpha={a.alpha} over {a.key_space} ids, seeds 1.."),
            "hit_rate": round(hit_rate, 4), "distinct_key_fraction": round(float(np.mean(distinct_frac)), 4),
            "out_buffers_rotated": a.out_buffers, "concurrent_writer_checks": bool(a.coherent),
            "replacement_policy": a.policy,
            "launch": "hip graph" if graph is not None else "eager, one call per batch, one stream",
            "repeat_ms": [round(t, 3) for t in times],
        },
        "roofline": roofline_obj(kernel_name, alg_bytes, ms_per_step * 1e3, traffic, traffic_source=traffic_source),
    }

    if multi is not None:
        multi["achieved_GBps"] = round(alg_bytes / (multi["ms_per_step"] * 1e-3) / 1e9, 1)
        multi["frac_of_peak"] = round(multi["achieved_GBps"] / HBM_PEAK_GBS, 4)
        result["concurrent_streams"] = multi

    # ---- the same batches, several per launch (one launch for k consecutive batches through the
    #      multi-table entry point with the one cache named k times): what a caller with a queue
    #      of batches gets; the launch floor is paid once per k batches
    if a.batched > 1 and not a.coherent and graph is None:
        k = a.batched
        handles = (C.c_void_p * k)(*[h] * k)
        big_outs = [torch.empty(k * n, d, dtype=torch.float32, device="cuda") for _ in range(max(2, 16 // k))]
        bmi = torch.empty(k * n, dtype=torch.int32, device="cuda")
        bmk = torch.empty(k * n, dtype=torch.int64, device="cuda")
        bnm = torch.zeros(n_batches, dtype=torch.int32, device="cuda")
        qm = lib.hps_cache_query_multi
        groups = [b for b in range(a.warmup, n_batches - k + 1, k)]

        def launch_group(gi):
            b = groups[gi % len(groups)]
            r = qm(handles, k, kp + b * n * 8, n, big_outs[gi % len(big_outs)].data_ptr(), bmi.data_ptr(), bmk.data_ptr(),
                   bnm.data_ptr() + b * 4, sp)
            if r != 0:
                raise RuntimeError(B.hps_last_error())

        cnt = [0]

        def one():
            launch_group(cnt[0])
            cnt[0] += 1
        us = event_us(torch, one, len(groups) * 3, warm=len(groups))
        got = int(bnm[groups[0]].item())
        want = int(nm[groups[0]:groups[0] + k].sum().item())
        assert got == want, (got, want)                       # same misses as the k single launches
        result["batched_launch"] = {"batches_per_launch": k, "us_per_batch": round(us / k, 3),
                                    "value": round(n / (us / k) , 1), "unit": "Mkeys/s",
                                    "frac_of_peak": round(alg_bytes / (us / k * 1e-6) / 1e9 / HBM_PEAK_GBS, 4)}
        del big_outs

    # ---- the library's default mode (queries validate rows against concurrent writers), same batches
    if not a.coherent and graph is None and a.also_checked:
        B.hps_cache_set_concurrent_writers(h, True)
        cnt = [0]

        def one_checked():
            launch(a.warmup + cnt[0] % a.steps)
            cnt[0] += 1
        us = event_us(torch, one_checked, a.steps, warm=20)
        B.hps_cache_set_concurrent_writers(h, False)
        result["checked_query"] = {"what": "same batches with hps_cache_set_concurrent_writers(1), the library default",
                                   "us_per_launch": round(us, 3), "value": round(n / us, 1), "unit": "Mkeys/s",
                                   "frac_of_peak": round(alg_bytes / (us * 1e-6) / 1e9 / HBM_PEAK_GBS, 4)}

    # ---- ceiling: the row movement of the same batches with nothing else (slots given, no hash,
    #      no probe, no miss list), and a plain streaming copy of the same number of bytes
    if a.ceiling and graph is None and a.keys == "zipf":
        result["roofline"].update(measure_ceiling(a, np, torch, B, h, host_keys, keys, mi, nm, outs, n, d, S, W, alg_bytes))

    # ---- CPU oracle on the host cores, bounded sample of the same batches
    if not a.no_cpu_baseline:
        oc, _ = oracle_hot_cache(np, slots, W, d, chunk)
        nb = min(a.cpu_batches, a.steps)
        sample = host_keys[a.warmup:a.warmup + nb]
        out_cpu = np.empty((n, d), dtype=np.uint32)
        t0 = time.perf_counter()
        miss_cpu = []
        for b in range(nb):
            _, omi, _ = oc.query(sample[b], out_cpu)
            miss_cpu.append(len(omi))
        t1 = time.perf_counter()
        # The two prefills are independent (the way order of same-chunk arrivals is free on the
        # GPU), so a few rarely used keys differ in residency; the hit rates must still agree closely.
        cpu_hit = 1.0 - float(np.mean(miss_cpu)) / n
        assert abs(cpu_hit - hit_rate) < 0.01, (cpu_hit, hit_rate)
        cpu_mkeys = nb * n / (t1 - t0) / 1e6
        result["cpu_baseline"] = {
            "value": round(cpu_mkeys, 2), "unit": "Mkeys/s", "cores": 1, "kind": "oracle",
            "sample": f"first {nb} timed batches of the same key stream, same cache geometry and prefill order",
            "hit_rate": round(cpu_hit, 4),
        }
        # the same oracle, query positions split statically over host threads (query is read-only)
        nthr = min(16, os.cpu_count() or 1)
        bounds = np.linspace(0, n, nthr + 1).astype(int)
        outs_t = [np.empty((bounds[i + 1] - bounds[i], d), dtype=np.uint32) for i in range(nthr)]

        def work(i):
            for b in range(nb):
                oc.query(sample[b][bounds[i]:bounds[i + 1]], outs_t[i])
        t0 = time.perf_counter()
        th = [threading.Thread(target=work, args=(i,)) for i in range(nthr)]
        [t.start() for t in th]
        [t.join() for t in th]
        t1 = time.perf_counter()
        result["cpu_baseline_all_cores"] = {
            "value": round(nb * n / (t1 - t0) / 1e6, 2), "unit": "Mkeys/s", "cores": nthr, "kind": "oracle",
            "sample": "same sample, positions split statically over threads",
        }
        oc.close()

    torch.cuda.synchronize()
    B.hps_cache_destroy(h)
    result["config"]["setup_seconds"] = round(time.time() - t_setup, 1)
    print(json.dumps(result))


def measure_ceiling(a, np, torch, B, h, host_keys, keys, mi, nm, outs, n, d, S, W, alg_bytes):
    """What the memory system gives for the byte movement of the timed query batches alone.
    The slot of every hit position is looked up on the host in the exported key array; then
    hps_membench_gather moves exactly the rows the query moved (its output is compared with the
    query's), launched the same way on the same rotating `out` buffers."""
    slots = S * W
    nb = min(32, a.steps)
    gk = torch.empty(slots, dtype=torch.int64, device="cuda")
    gc = torch.empty(S, dtype=torch.int32, device="cuda")
    gv = torch.empty(slots, d, dtype=torch.float32, device="cuda")
    B.hps_cache_export(h, gk, gc, gv)
    torch.cuda.synchronize()
    hk = gk.cpu().numpy()
    order = np.argsort(hk, kind="stable")
    sk = hk[order]
    slot_of = np.empty((nb, n), dtype=np.uint32)
    for i in range(nb):
        kb = host_keys[a.warmup + i]
        pos = np.clip(np.searchsorted(sk, kb), 0, slots - 1)
        found = sk[pos] == kb
        slot_of[i] = np.where(found, order[pos], 0xFFFFFFFF).astype(np.uint32)
        m = int(nm[a.warmup + i].item())
        assert int((~found).sum()) == m                   # the same positions miss
    d_slot = torch.from_numpy(slot_of.view(np.int32)).cuda()
    # the gather moves what the query moved: compare one batch bit for bit
    ref = torch.zeros(n, d, dtype=torch.float32, device="cuda")
    got = torch.zeros(n, d, dtype=torch.float32, device="cuda")
    nm1 = torch.zeros(1, dtype=torch.int32, device="cuda")
    mi1 = torch.empty(n, dtype=torch.int32, device="cuda")
    mk1 = torch.empty(n, dtype=torch.int64, device="cuda")
    B.hps_cache_query(h, keys[a.warmup], n, ref, mi1, mk1, nm1)
    B.hps_membench_gather(gv, d_slot[0], n, d, got)
    torch.cuda.synchronize()
    assert torch.equal(ref.view(torch.int32), got.view(torch.int32))
    cnt = [0]

    def one():
        i = cnt[0]
        B.hps_membench_gather(gv, d_slot[i % nb], n, d, outs[i % len(outs)])
        cnt[0] += 1
    us_gather = event_us(torch, one, a.steps, warm=20)
    us_half = {}
    if d == 128:                                 # the two halves of the same movement, each alone
        for name, reads in (("reads_only", True), ("writes_only", False)):
            cnt[0] = 0

            def half_one(reads=reads):
                i = cnt[0]
                B.hps_membench_gather_half(gv, d_slot[i % nb], n, outs[i % len(outs)], reads)
                cnt[0] += 1
            us_half[name] = event_us(torch, half_one, a.steps, warm=20)
        outs[0].view(torch.int32).fill_(0)       # (the write-only pass leaves its pattern in the out buffers)
    # a streaming copy that reads and writes as many bytes as the query's algorithmic figure
    half = int(alg_bytes // 2) // 4096 * 4096
    src = torch.empty(16 * half // 4, dtype=torch.float32, device="cuda")
    dst = torch.empty(16 * half // 4, dtype=torch.float32, device="cuda")
    cnt2 = [0]

    def copy_one():
        o = (cnt2[0] % 16) * (half // 4)
        B.hps_membench_copy(src[o:], dst[o:], half, True)
        cnt2[0] += 1
    us_copy = event_us(torch, copy_one, a.steps, warm=20)
    big = 1 << 30
    bsrc = torch.empty(big // 4, dtype=torch.float32, device="cuda")
    bdst = torch.empty(big // 4, dtype=torch.float32, device="cuda")
    us_big = event_us(torch, lambda: B.hps_membench_copy(bsrc, bdst, big, True), 10, warm=2)
    del gk, gc, gv, src, dst, bsrc, bdst
    return {
        "achievable_frac": round(alg_bytes / (us_gather * 1e-6) / 1e9 / HBM_PEAK_GBS, 4),
        "ceiling": {
            "what": ("hps_membench_gather: out[i] = rows[slot[i]] for the hit positions of the same batches (slots "
                     "precomputed; no hashing, probing or miss list), one launch per batch on the same stream and the same "
                     "rotating out buffers; output equal to the query's"),
            "gather_us_per_launch": round(us_gather, 3),
            **({"gather_reads_only_us_per_launch": round(us_half["reads_only"], 3),
                "gather_writes_only_us_per_launch": round(us_half["writes_only"], 3)} if us_half else {}),
            "streaming_copy_of_the_same_bytes_us_per_launch": round(us_copy, 3),
            "streaming_copy_1GiB_GBps_read_plus_write": round(2 * big / (us_big * 1e-6) / 1e9, 1),
        },
    }


if __name__ == "__main__":
    main()
