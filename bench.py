"""Benchmark: value-driven memory retrieval on one MI355X.

One step = one pass of the whole hot path over one batch: append B new entries (memory growth,
Sec. 3.1), retrieve for B queries (dense recall + value filter, Sec. 3.2), update the Q values of the
B*k2 returned ids (unified value update, Sec. 3.2).  Workload: the clustered bank, N = 1,048,576
entries, d = 1024, bf16 storage, B = 256, k1 = 128, k2 = 16, lambda = 0.5, synthetic and seeded.
Inputs are resident in HBM before the timed region.  Prints one JSON line.
"""
import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0
COUNTER_SUMMARY = os.path.join(ROOT, "profiles", "k_scan_mfma_clustered_hbm_counters.txt")
KERNEL_SOURCES = ("k_scan_mfma.h", "k_scan_gemv.h", "layout.h")      # what the scan kernel is compiled from


def measured_traffic(workload):
    """HBM bytes per launch of the densest scan pass from the committed counter summary, or None when
    it is for another workload or the kernel's sources have changed since the counters were taken."""
    import hashlib
    if workload != "clustered" or not os.path.exists(COUNTER_SUMMARY):
        return None
    h = hashlib.sha256()
    for name in KERNEL_SOURCES:
        h.update(name.encode())
        h.update(open(os.path.join(ROOT, "paper_2603_10846_amd", "csrc", name), "rb").read())
    fields = dict(l.split(": ", 1) for l in open(COUNTER_SUMMARY).read().splitlines() if ": " in l and " " not in l.split(": ")[0])
    if fields.get("kernel_source_sha256") != h.hexdigest():
        return None
    return int(fields["traffic_bytes_per_launch"])


MFMA_PEAK_TFLOPS = 2500.0


def time_calls(torch, fn, reps, warm=10):
    """Average milliseconds of fn() over `reps` calls after `warm` untimed ones (host clock around a synchronised region)."""
    for _ in range(warm):
        fn()
    torch.cuda.synchronize()
    a = time.perf_counter()
    for _ in range(reps):
        fn()
    torch.cuda.synchronize()
    return (time.perf_counter() - a) * 1e3 / reps


def retrieve_figures(torch, bank, q, stage, w, elem, reps=30):
    """Whole-retrieve time and the densest scan pass of a retrieve (the library's HIP events around that
    launch, on the stream it runs on) for one workload shape; the bank is left as it is."""
    B = q.shape[0]
    out = (torch.empty((B, w.k2), dtype=torch.int32, device=q.device),
           torch.empty((B, w.k2), dtype=torch.float32, device=q.device), None, None)
    call = lambda: bank.retrieve(q, stage, w.k1, w.k2, w.lam, out=out)
    ms = time_calls(torch, call, reps)
    bank.profile_read()
    bank.profile_enable(True)
    for _ in range(5):
        call()
    prof = bank.profile_read()
    bank.profile_enable(False)
    max_rows = max(r for _, r in prof)
    dense = [t for t, r in prof if r == max_rows]
    dense_ms = float(np.mean(dense))
    gbps = max_rows * w.d * elem / (dense_ms * 1e-3) / 1e9
    tflops = 2.0 * B * max_rows * w.d / (dense_ms * 1e-3) / 1e12
    return {"B": B, "retrieve_ms": round(ms, 4), "queries_per_s": round(B / (ms * 1e-3), 1),
            "densest_pass_ms": round(dense_ms, 4), "densest_pass_rows": int(max_rows),
            "densest_pass_GBps": round(gbps, 1), "hbm_frac": round(gbps / HBM_PEAK_GBS, 4),
            "mfma_tflops": round(tflops, 1), "mfma_frac": round(tflops / MFMA_PEAK_TFLOPS, 4),
            "whole_retrieve_store_GBps": round(bank.size() * w.d * elem / (ms * 1e-3) / 1e9, 1)}


def read_ceiling(torch, bank, reps=20):
    """GB/s of a read-only pass over the same stored rows (the library's probe kernel)."""
    chk = torch.zeros(1, dtype=torch.int32, device=bank.device)
    nbytes = [0]

    def call():
        nbytes[0] = bank.read_probe(chk)
    ms = time_calls(torch, call, reps, warm=5)
    return {"kernel": "k_read_probe (16-byte loads, every stored byte once)", "bytes": nbytes[0], "ms": round(ms, 4),
            "GBps": round(nbytes[0] / (ms * 1e-3) / 1e9, 1), "frac_of_peak": round(nbytes[0] / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS, 4)}


def other_configs(torch, binding, synth, clustered_bank, clustered_w):
    """Quick figures for the other workload shapes (not part of `value`): the clustered bank at smaller
    batches, the mid bank, the streaming shape at 1M entries (with a 65,536-entry append) and the large
    batched bank.  Rows of the two big banks are seeded normalised Gaussians generated on the device."""
    dev = torch.device("cuda:0")
    todev = lambda a: torch.from_numpy(np.ascontiguousarray(a)).to(dev)
    res = []
    for B in (1, 64):
        w = synth.scaled(clustered_w, B=B)
        r = retrieve_figures(torch, clustered_bank, todev(synth.queries(w)), synth.DRAFT, w, 2)
        res.append({"workload": f"clustered bank, B={B}", **r})
    # the exhaustive retrieve (every entry scored in fp64; the always-exact path for flagged queries): four queries
    w4 = synth.scaled(clustered_w, B=4)
    q4 = todev(synth.queries(w4))
    ex_ms = time_calls(torch, lambda: clustered_bank.retrieve_exact(q4, synth.DRAFT, w4.k1, w4.k2, w4.lam), 5, warm=2)
    res.append({"workload": "clustered bank, mem_retrieve_exact, B=4", "B": 4, "retrieve_ms": round(ex_ms, 3),
                "queries_per_s": round(4 / (ex_ms * 1e-3), 1),
                "store_GBps": round(4 * clustered_bank.size() * w4.d * 2 / (ex_ms * 1e-3) / 1e9, 1),
                "note": "reads the bank once per query"})
    # mid: fp32 rows
    w = synth.MID
    bank = binding.MemoryBank(w.d, w.dtype, w.N, max_B=w.B, max_k1=w.k1)
    qtab = synth.q_tables(w)
    bank.append(todev(synth.bank(w)), todev(qtab[0]), todev(qtab[1]))
    r = retrieve_figures(torch, bank, todev(synth.queries(w)), synth.DRAFT, w, 4, reps=50)
    res.append({"workload": f"mid: N={w.N} d={w.d} f32, B={w.B} k1={w.k1} k2={w.k2}", **r,
                "note": "a pass this short is over-stated by the events' own idle time; see the kernel trace under profiles/"})
    bank.close()
    del bank
    g = torch.Generator(device=dev).manual_seed(synth.SEED + 77)

    def rows(n, d):
        x = torch.randn((n, d), device=dev, generator=g)
        return x / x.norm(dim=1, keepdim=True)
    # stream shape at 1M entries, plus one 65,536-entry append and the update of the returned ids
    w = synth.scaled(synth.STREAM, N=1048576)
    bank = binding.MemoryBank(w.d, w.dtype, w.N + 40 * synth.CHUNK_ROWS, max_B=w.B, max_k1=w.k1)
    for _ in range(w.N // synth.CHUNK_ROWS):
        bank.append(rows(synth.CHUNK_ROWS, w.d))
    r = retrieve_figures(torch, bank, rows(w.B, w.d), synth.REFINE, w, 2, reps=20)
    chunk = rows(synth.CHUNK_ROWS, w.d)
    ap_ms = time_calls(torch, lambda: bank.append(chunk), 30, warm=5)       # the bank grows by 35 chunks here
    ids = torch.randint(0, w.N, (w.B * w.k2,), device=dev, generator=g, dtype=torch.int32)
    rew = (torch.rand(w.B * w.k2, device=dev, generator=g) < 0.2).float()
    up_ms = time_calls(torch, lambda: bank.update_q(ids, synth.REFINE, rew, w.alpha), 50)
    ap_bytes = synth.CHUNK_ROWS * w.d * (4 + 2)
    res.append({"workload": f"stream shape at N={w.N}: d={w.d} f16, B={w.B} k1={w.k1} k2={w.k2}", **r,
                "append_65536_ms": round(ap_ms, 4), "append_GBps": round(ap_bytes / (ap_ms * 1e-3) / 1e9, 1),
                "append_hbm_frac": round(ap_bytes / (ap_ms * 1e-3) / 1e9 / HBM_PEAK_GBS, 4), "update_q_4096_ms": round(up_ms, 4)})
    bank.close()
    del bank, chunk
    torch.cuda.empty_cache()
    # large batched bank
    w = synth.LARGE
    bank = binding.MemoryBank(w.d, w.dtype, w.N, max_B=w.B, max_k1=w.k1)
    for _ in range(w.N // synth.CHUNK_ROWS):
        bank.append(rows(synth.CHUNK_ROWS, w.d))
    r = retrieve_figures(torch, bank, rows(w.B, w.d), synth.REFINE, w, 2, reps=10)
    zipf, rew = (todev(a) for a in synth.zipf_update(w))                     # 16,384 ids, Zipf(1.1): one id about 2,000 times
    up_ms = time_calls(torch, lambda: bank.update_q(zipf, synth.REFINE, rew, w.alpha), 50)
    res.append({"workload": f"large: N={w.N} d={w.d} bf16, B={w.B} k1={w.k1} k2={w.k2}", **r, "update_q_16384_ms": round(up_ms, 4)})
    bank.close()
    return res


def run_stream(torch, binding, synth):
    """The growing bank: starts at 1M entries and grows to 8M by 64K-entry appends (d = 4096, fp16
    store); every step appends a chunk, retrieves for B = 128 fresh queries (k1 = 256, k2 = 32,
    lambda = 0.7, stages alternating) and updates the Q values of the B*k2 returned ids with
    Bernoulli(0.2) rewards.  Rows and queries are seeded normalised Gaussians generated on the device
    (68.7 GB of rows: generating them on the host would take longer than the run).  Every call is
    timed with events on the stream it runs on; one JSON line with samples along the growth."""
    w = synth.STREAM
    dev = torch.device("cuda:0")
    N0, steps, chunk = w.extra["N0"], w.extra["steps"], synth.CHUNK_ROWS
    bank = binding.MemoryBank(w.d, w.dtype, w.N, max_B=w.B, max_k1=w.k1)
    g = torch.Generator(device=dev).manual_seed(synth.SEED + 5)

    def rows(n):
        x = torch.randn((n, w.d), device=dev, generator=g)
        return x / x.norm(dim=1, keepdim=True)
    for _ in range(N0 // chunk):
        bank.append(rows(chunk))
    out = (torch.empty((w.B, w.k2), dtype=torch.int32, device=dev),
           torch.empty((w.B, w.k2), dtype=torch.float32, device=dev), None, None)
    bank.profile_enable(True)
    rec = []
    ev = lambda: torch.cuda.Event(enable_timing=True)
    for t in range(steps):
        new, q = rows(chunk), rows(w.B)
        rewards = (torch.rand(w.B * w.k2, device=dev, generator=g) < 0.2).float()
        e = [ev() for _ in range(4)]
        torch.cuda.synchronize()
        e[0].record(); bank.append(new)
        e[1].record(); ids, _, _, _ = bank.retrieve(q, t % 2, w.k1, w.k2, w.lam, out=out)
        e[2].record(); bank.update_q(ids.view(-1), t % 2, rewards, w.alpha)
        e[3].record(); torch.cuda.synchronize()
        prof = bank.profile_read()
        dense_ms, dense_rows = max(prof, key=lambda p: p[1])
        rec.append({"step": t, "N": bank.size(), "append_ms": e[0].elapsed_time(e[1]), "retrieve_ms": e[1].elapsed_time(e[2]),
                    "update_ms": e[2].elapsed_time(e[3]), "dense_ms": dense_ms, "dense_rows": dense_rows})
        if t % 16 == 0:
            print(f"# step {t} N={bank.size()} retrieve {rec[-1]['retrieve_ms']:.3f} ms", file=sys.stderr, flush=True)
    assert bank.counters() == (0, 0)
    elem = 2
    samples = []
    for t in (0, 27, 55, 83, 111):
        r = rec[t]
        samples.append({"step": t, "N": r["N"], "retrieve_ms": round(r["retrieve_ms"], 3),
                        "queries_per_s": round(w.B / (r["retrieve_ms"] * 1e-3), 1),
                        "store_GBps_whole_retrieve": round(r["N"] * w.d * elem / (r["retrieve_ms"] * 1e-3) / 1e9, 1),
                        "dense_pass_GBps": round(r["dense_rows"] * w.d * elem / (r["dense_ms"] * 1e-3) / 1e9, 1),
                        "append_ms": round(r["append_ms"], 3),
                        "append_GBps": round(chunk * w.d * (4 + elem) / (r["append_ms"] * 1e-3) / 1e9, 1),
                        "update_ms": round(r["update_ms"], 4)})
    total_ms = sum(r["append_ms"] + r["retrieve_ms"] + r["update_ms"] for r in rec)
    last = rec[-1]
    achieved = last["dense_rows"] * w.d * elem / (last["dense_ms"] * 1e-3) / 1e9
    print(json.dumps({
        "metric": "retrieval queries/sec (stream: N 1M -> 8M, d=4096 fp16, B=128)",
        "value": round(w.B * steps / (total_ms * 1e-3), 1), "unit": "queries/s", "n_gpus": 1, "steps": steps, "warmup": 0,
        "ms_per_step": round(total_ms / steps, 4), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f16", "data": "synthetic",
        "config": {"workload": "stream: append 65536 + retrieve B=128 k1=256 k2=32 lambda=0.7 + update_q 4096, 112 steps"},
        "roofline": {"bound": "hbm", "kernel": "k_scan_mfma (densest pass, last step, N=8M)", "achieved": round(achieved, 1),
                     "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": round(achieved / HBM_PEAK_GBS, 4), "traffic": None},
        "cpu_baseline": None, "samples": samples}))
    bank.close()


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    # Defaults: the clocks of the GPU settle only after some tens of milliseconds of continuous load (the
    # densest pass runs 490 us in the first launches, about 600 us from the 7th to the 12th, and levels
    # out near 515 us after some 25), so the untimed warm-up covers that transient.
    ap.add_argument("--steps", type=int, default=100)
    ap.add_argument("--warmup", type=int, default=50)
    ap.add_argument("--workload", default="clustered", choices=["clustered", "tiny", "mid", "large", "stream1m", "stream"])
    ap.add_argument("--batch", type=int, default=0, help="override the workload's query batch size B")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-other-configs", action="store_true", help="skip the quick figures for the other workload shapes")
    ap.add_argument("--cpu-queries", type=int, default=0, help="oracle sample size (0: 16 per thread, at most B)")
    ap.add_argument("--copy-probe", action="store_true",
                    help="only run a plain 1 GiB device-to-device copy five times (reference for HBM counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on one GPU only (no collectives); use --gpus 1")

    import torch

    from paper_2603_10846_amd import binding, synth

    if not torch.cuda.is_available():
        sys.exit("bench.py: needs a GPU (there is no CPU path)")
    if args.copy_probe:
        src = torch.ones(1 << 28, dtype=torch.float32, device="cuda:0")      # 1 GiB
        dst = torch.empty_like(src)
        for _ in range(5):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"copy_probe_bytes_read": src.numel() * 4, "copy_probe_bytes_written": src.numel() * 4}))
        return
    if args.workload == "stream":
        return run_stream(torch, binding, synth)
    w = {"clustered": synth.CLUSTERED, "tiny": synth.TINY, "mid": synth.MID, "large": synth.LARGE,
         "stream1m": synth.scaled(synth.STREAM, N=1048576)}[args.workload]
    if args.batch:
        w = synth.scaled(w, B=args.batch)
    stage = synth.REFINE if args.workload == "large" else synth.DRAFT
    steps, warm = args.steps, args.warmup
    dev = torch.device("cuda:0")
    todev = lambda a: torch.from_numpy(np.ascontiguousarray(a)).to(dev)

    t0 = time.time()
    cap = w.N + (steps + warm + 2) * w.B
    bank = binding.MemoryBank(w.d, w.dtype, cap, max_B=w.B, max_k1=w.k1)
    qtab = synth.q_tables(w)
    need_host_bank = not args.no_cpu_baseline
    host_rows = np.empty((w.N, w.d), np.float32) if need_host_bank else None
    for j in range(synth.n_chunks(w)):
        c = synth.bank_chunk(w, j)
        a = j * synth.CHUNK_ROWS
        bank.append(todev(c), todev(qtab[0, a:a + len(c)]), todev(qtab[1, a:a + len(c)]))
        if need_host_bank:
            host_rows[a:a + len(c)] = c
    print(f"# bank built in {time.time() - t0:.1f}s", file=sys.stderr, flush=True)

    # per-step inputs, resident on the device before timing
    n_total = steps + warm
    q_host = [synth.queries(w, step=s) for s in range(min(n_total, 8))]
    q_dev = [todev(q) for q in q_host]
    new_rows = todev(synth.queries(w, step=1000))                 # entries appended each step
    rewards = [todev(synth.bernoulli_rewards(w, s, w.B * w.k2)) for s in range(min(n_total, 8))]
    out = (torch.empty((w.B, w.k2), dtype=torch.int32, device=dev),
           torch.empty((w.B, w.k2), dtype=torch.float32, device=dev), None, None)

    def step(s):
        bank.append(new_rows)
        ids, _, _, _ = bank.retrieve(q_dev[s % len(q_dev)], stage, w.k1, w.k2, w.lam, out=out)
        bank.update_q(ids.view(-1), stage, rewards[s % len(rewards)], w.alpha)

    # With fewer than 50 warm-up steps the clocks would still be settling inside the timed region (see the
    # note at --steps): read-only retrieve calls, which leave the bank and the Q tables as they are, make
    # up the difference before the warm-up steps.
    bank.profile_enable(True)        # creates the library's timing events now, not inside the timed region
    bank.profile_enable(False)
    settle = max(0, 50 - warm)
    for s in range(settle):
        bank.retrieve(q_dev[s % len(q_dev)], stage, w.k1, w.k2, w.lam, out=out)
    for s in range(warm):
        step(s)
    torch.cuda.synchronize()
    # The library's launch timing (events around every scan launch, on its own stream) is switched on
    # for every tenth timed step only: each event costs about 6 us of idle time on either side of
    # the launch, which would otherwise lengthen every step by ~35 us.
    PROFILE_EVERY = 10
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    for s in range(steps):
        bank.profile_enable(s % PROFILE_EVERY == 0)
        step(warm + s)
    torch.cuda.synchronize()
    t2 = time.perf_counter()
    prof = bank.profile_read()
    bank.profile_enable(False)
    profiled_steps = (steps + PROFILE_EVERY - 1) // PROFILE_EVERY
    ms_per_step = (t2 - t1) * 1e3 / steps
    qps = w.B / (ms_per_step * 1e-3)

    # separate timing of the three calls (not part of `value`)
    def timed(fn, reps=50):
        for _ in range(10):            # back to steady clocks after the idle gap above
            fn()
        torch.cuda.synchronize()
        a = time.perf_counter()
        for _ in range(reps):
            fn()
        torch.cuda.synchronize()
        return (time.perf_counter() - a) * 1e3 / reps
    ids_fixed = out[0].view(-1).clone()
    breakdown = {
        "retrieve_ms": timed(lambda: bank.retrieve(q_dev[0], stage, w.k1, w.k2, w.lam, out=out)),
        "update_q_ms": timed(lambda: bank.update_q(ids_fixed, stage, rewards[0], w.alpha)),
    }

    # roofline of the dominant kernel: the densest scan pass (HBM-bound: it must read its rows once)
    elem = 4 if w.dtype == "f32" else 2
    # (the bank grows by B rows per step, so the densest pass's row count drifts by a tile now and then)
    max_rows = max(r for _, r in prof)
    dense = [(ms, r) for ms, r in prof if r > max_rows // 2]
    avg_ms = float(np.mean([ms for ms, _ in dense]))
    dense_rows = float(np.mean([r for _, r in dense]))
    alg_bytes = dense_rows * w.d * elem
    achieved = alg_bytes / (avg_ms * 1e-3) / 1e9
    roofline = {"bound": "hbm", "kernel": ("k_scan_gemv32" if w.B <= 4 and w.dtype == "f32" else "k_scan_mfma") + " (densest pass)", "achieved": round(achieved, 1),
                "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": round(achieved / HBM_PEAK_GBS, 4), "traffic": None if args.batch else measured_traffic(args.workload),
                "traffic_source": "recorded counters (profiles/k_scan_mfma_clustered_hbm_counters.txt), not measured in this run",
                "avg_launch_ms": round(avg_ms, 4), "launches": len(dense), "rows_per_launch": int(dense_rows),
                "bytes_per_row": w.d * elem, "algorithmic_bytes_per_launch": int(alg_bytes),
                "mfma_tflops": round(2.0 * w.B * dense_rows * w.d / (avg_ms * 1e-3) / 1e12, 1),
                "all_scan_passes_ms_per_step": round(sum(ms for ms, _ in prof) / profiled_steps, 4)}

    cpu = None
    if not args.no_cpu_baseline:
        from oracle import oracle as orc
        threads = min(orc.max_threads(), 16)
        nq = min(w.B, args.cpu_queries or 16 * threads)
        dt = {"f32": 0, "bf16": 1, "f16": 2}[w.dtype]
        rounded = orc.round_to_store(host_rows, dt)
        del host_rows
        qs = orc.round_to_store(q_host[0][:nq], dt)
        a = time.perf_counter()
        res = orc.retrieve(rounded, qs, qtab[stage], w.k1, w.k2, float(np.float32(w.lam)), threads=threads)
        orc.update_q32(qtab[stage], res["ids"].reshape(-1), np.zeros(res["ids"].size, np.float32), w.alpha)
        el = time.perf_counter() - a
        n1 = min(2, nq)
        a = time.perf_counter()
        orc.retrieve(rounded, qs[:n1], qtab[stage], w.k1, w.k2, float(np.float32(w.lam)), threads=1)
        el1 = time.perf_counter() - a
        cpu = {"value": round(nq / el, 3), "unit": "queries/s", "cores": threads, "kind": "oracle",
               "sample": f"{nq} of the {w.B} queries of one step over the full {w.N}-entry bank "
                         f"(recall + value filter + update), {el:.1f} s",
               "single_thread": {"value": round(n1 / el1, 3), "unit": "queries/s", "sample": f"{n1} queries, {el1:.1f} s"},
               "nproc": os.cpu_count(), "openmp_max_threads": orc.max_threads()}
        del rounded

    # the extras below are not part of `value`: a failure in them must not cost the line
    ceiling, configs, extras_error = None, None, None
    try:
        ceiling = read_ceiling(torch, bank)
        if args.workload == "clustered" and not args.batch and not args.no_other_configs:
            configs = other_configs(torch, binding, synth, bank, w)
    except Exception as e:                                      # noqa: BLE001 (reported in the line)
        extras_error = f"{type(e).__name__}: {e}"

    print(json.dumps({
        "metric": "retrieval queries/sec at N=1M,d=1024 + achieved HBM GB/s (% of peak)"
                  if args.workload == "clustered" and not args.batch else f"retrieval queries/sec ({args.workload}, B={w.B})",
        "value": round(qps, 1), "unit": "queries/s", "n_gpus": 1, "steps": steps, "warmup": warm,
        "settle_retrieves_before_warmup": settle, "ms_per_step": round(ms_per_step, 4), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": {"f32": "f32", "bf16": "bf16", "f16": "f16"}[w.dtype], "data": "synthetic",
        "config": {"workload": f"{w.name}: N={w.N} d={w.d} {w.dtype} store / fp32 accumulate, B={w.B} k1={w.k1} "
                               f"k2={w.k2} lambda={w.lam}; step = append B + retrieve B + update_q B*k2 "
                               f"(the bank holds N entries before the first step and grows by B per step)",
                   "N": w.N, "N_after_last_step": w.N + (steps + warm) * w.B, "d": w.d, "B": w.B, "k1": w.k1, "k2": w.k2},
        "roofline": roofline, "cpu_baseline": cpu, "breakdown": breakdown, "read_ceiling": ceiling, "configs": configs,
        "untimed_calls_before_timing": {"steps": warm, "read_only_retrieves": settle}, "extras_error": extras_error,
    }))
    bank.close()


if __name__ == "__main__":
    main()
