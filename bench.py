#!/usr/bin/env python3
"""Headline benchmark: snapshot pack+CRC and restore on a Llama-7B-shaped per-worker shard.

One step = one pass of the whole hot path over the shard, state resident in HBM:
    ff_adam_step_snapshot (when the library provides it)  ->  ff_pack  ->  ff_restore
The shard is one 8-way data-parallel worker's slice of a 7B model: 226 parameters, bf16 weights
plus fp32 master/m/v, 11.79 GB in 904 tensors, 4 MiB chunks (2812 chunks).

Prints ONE JSON line.  `value` is the algorithmic HBM traffic of a step divided by its time
(pack and restore each read and write every payload byte once: 2 B per payload byte; the fused
Adam step moves 42 B per parameter).  `roofline` is the longest-running kernel of the step:
algorithmic bytes per launch over its HIP-event duration against the 8 TB/s HBM peak.
`cpu_baseline` is the plain CPU oracle timed on this machine's host cores on a bounded sample of the
same shard.
"""
import argparse
import hashlib
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0


KERNEL_SOURCES = ("kernels.hip", "kernels.hpp", "fused.hip", "fused.hpp", "fold.h", "fold_taps.h",
                  "gf2.h", "layout.hpp", "xcd_order.h")


def kernel_source_hash():
    """sha256 over the files that define the device code and its tile constants: identifies the
    kernels a counter run belongs to."""
    h = hashlib.sha256()
    for name in KERNEL_SOURCES:
        h.update(name.encode())
        h.update(open(os.path.join(ROOT, "paper_2512_03644_amd", "csrc", name), "rb").read())
    return h.hexdigest()


def measured_traffic(kernel, workload):
    """(HBM bytes per launch of `kernel` on `workload`, where the figure comes from) out of the
    committed rocprofv3 counter runs (profiles/hbm_traffic.json); (None, reason) if the kernel
    sources have changed since the counters were taken or the kernel was not counted."""
    try:
        rec = json.load(open(os.path.join(ROOT, "profiles", "hbm_traffic.json")))
    except (OSError, ValueError):
        return None, "no counter record"
    if rec.get("source_sha256") != kernel_source_hash():
        return None, "kernel sources changed since the counters in profiles/hbm_traffic.json were taken"
    k = rec.get("workloads", {}).get(workload, {}).get(kernel)
    if k is None:
        return None, "kernel not in profiles/hbm_traffic.json for this workload"
    return k["hbm_bytes_per_launch"], (
        "replayed, not measured in this run: rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs of this "
        "command committed in profiles/hbm_traffic.json (same kernel sources by hash), scaled by "
        "the same counters on the library's plain copy kernel; cross-checked there against "
        "TCC_EA0_RDREQ / TCC_EA0_WRREQ")


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-adam", action="store_true", help="leave the fused optimizer step out")
    ap.add_argument("--no-host-staging", action="store_true",
                    help="leave out the snapshot-to-pinned-host-memory timing (it pins a buffer "
                         "as large as the snapshot)")
    ap.add_argument("--tile-log2", type=int, default=0, help="tuning: log2 of the tile size")
    ap.add_argument("--workload", default="llama7b",
                    help="llama7b is the headline shard; llama70b, fragmented and tiny are the "
                         "remaining configurations, timed the same way (fused step where the "
                         "shard has parameter groups and gradients); the names in "
                         "workloads.LAYOUT_VARIANTS (fragmented-16, tensors-32k-gaps, ...) are "
                         "variants of the fragmented shard that take its cost apart")
    return ap.parse_args()


def event_ms(fn, n, torch):
    """Per-call durations of fn in ms, HIP events on the current stream."""
    evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True))
           for _ in range(n)]
    for a, b in evs:
        a.record()
        fn()
        b.record()
    torch.cuda.synchronize()
    return [a.elapsed_time(b) for a, b in evs]


def cpu_oracle_step(shard, n_params, hp, with_adam, cores):
    """One oracle step (AdamW update + pack, pack, restore) on the first n_params parameter groups
    of the shard with `cores` threads: (step bytes, payload bytes, the three wall times)."""
    from concurrent.futures import ThreadPoolExecutor
    import numpy as np
    import oracle
    from paper_2512_03644_amd import workloads as wl
    groups = [[wl.to_numpy_bytes(t) for t in (p.w16, p.master, p.m, p.v)]
              for p in shard.params[:n_params]]
    grads = [wl.to_numpy_bytes(p.grad).view(np.uint16) for p in shard.params[:n_params]] \
        if with_adam else None
    segs = [a for g in groups for a in g]
    nbytes = sum(s.size for s in segs)
    n_el = sum(g[1].size // 4 for g in groups)
    oracle.lib()
    t0 = time.perf_counter()
    if with_adam:
        def upd(i):
            w16, master, m, v = groups[i]
            oracle.adam_f32(grads[i], master.view(np.float32), m.view(np.float32),
                            v.view(np.float32), w16.view(np.uint16), **hp)
        with ThreadPoolExecutor(cores) as ex:
            list(ex.map(upd, range(len(groups))))
        buf, crcs = oracle.pack(segs, shard.chunk_bytes, threads=cores)   # snapshot of the update
    t1 = time.perf_counter()
    buf, crcs = oracle.pack(segs, shard.chunk_bytes, threads=cores)
    t2 = time.perf_counter()
    dst = [np.empty_like(s) for s in segs]
    bad, n_bad = oracle.restore(dst, shard.chunk_bytes, buf, crcs, threads=cores)
    t3 = time.perf_counter()
    assert n_bad == 0
    step_bytes = 4 * nbytes + (42 * n_el if with_adam else 0)
    return step_bytes, nbytes, (t1 - t0, t2 - t1, t3 - t2)


def cpu_baseline(shard, n_params, hp, with_adam, torch):
    """The oracle's step on a bounded sample of the shard: on all host cores available to the
    process (chunk ranges and parameters spread by a thread pool) and, on a smaller sample, on
    one core."""
    # the box gives one GPU's job 16 cores' worth of CPU time whatever the affinity mask shows
    available = len(os.sched_getaffinity(0))
    cores = min(16, available)
    step_bytes, nbytes, t = cpu_oracle_step(shard, n_params, hp, with_adam, cores)
    n_one = max(1, min(n_params, 6))
    one_bytes, one_payload, t_one = cpu_oracle_step(shard, n_one, hp, with_adam, 1)
    what = "oracle %spack, restore; bytes counted as for the GPU step" % (
        "AdamW update + pack (unfused), " if with_adam else "")
    return {"value": round(step_bytes / sum(t) / 1e9, 3), "unit": "GB/s", "cores": cores,
            "cores_in_affinity_mask": available, "kind": "oracle",
            "sample": "first %d of %d parameter groups of the same shard (%.2f GB payload): %s; "
                      "wall %.2f + %.2f + %.2f s" % ((n_params, len(shard.params), nbytes / 1e9,
                                                      what) + t),
            "single_thread": {"value": round(one_bytes / sum(t_one) / 1e9, 3), "unit": "GB/s",
                              "cores": 1,
                              "sample": "first %d parameter groups (%.2f GB payload), same steps; "
                                        "wall %.2f + %.2f + %.2f s"
                                        % ((n_one, one_payload / 1e9) + t_one)}}


def selective_restore(ff, wl, torch, plan, chunks, crcs, bad, n_bad, N):
    """Failover-side variants, timed on the packed buffer with 1 % of its chunks corrupted (one
    flipped bit each, the seeded recipe of the corruption configuration): restore that leaves the
    ranges of bad chunks alone, and restore of just those chunks once they have been fetched
    again.  The buffer is repaired afterwards."""
    C = plan.chunk_bytes
    ff.ff_pack(plan, chunks, crcs)     # a buffer that verifies, whatever ran before
    hits = wl.corrupt_chunks(plan.num_chunks, C)
    for c, off, bit in hits:
        chunks[c * C + off] ^= (1 << bit)
    ts = event_ms(lambda: ff.ff_restore(plan, chunks, crcs, bad, n_bad,
                                        flags=ff.FF_RESTORE_SKIP_BAD), 5, torch)
    found = int(n_bad.item())
    for c, off, bit in hits:
        chunks[c * C + off] ^= (1 << bit)
    ids = [c for c, _, _ in hits]
    ts2 = event_ms(lambda: ff.ff_restore_chunks(plan, chunks, crcs, ids, bad, n_bad), 5, torch)
    assert found == len(hits) and int(n_bad.item()) == 0
    skip_ms, sel_ms = sum(ts) / len(ts), sum(ts2) / len(ts2)
    return {"restore_skip_bad": {"avg_ms": round(skip_ms, 4), "bad_chunks": found,
                                 "bytes": 3 * N, "traffic_GBps": round(3 * N / skip_ms / 1e6, 1)},
            "restore_chunks": {"avg_ms": round(sel_ms, 4), "chunks": len(ids),
                               "payload_GBps": round(len(ids) * C / sel_ms / 1e6, 1)}}


def pack_to_host(ff, torch, plan, chunks, crcs, N):
    """Snapshot into pinned host memory (the paper's device-to-host step): pack, then copy, against
    pack overlapped with the copy slice by slice.  Crosses PCIe: reported beside the step, never
    part of `value`."""
    h_chunks = torch.empty(plan.buffer_bytes, dtype=torch.uint8, pin_memory=True)
    h_crcs = torch.empty(plan.num_chunks, dtype=torch.int32, pin_memory=True)
    s_pack, s_copy = torch.cuda.Stream(), torch.cuda.Stream()

    def serial():
        ff.ff_pack(plan, chunks, crcs)
        h_chunks.copy_(chunks, non_blocking=True)
        h_crcs.copy_(crcs, non_blocking=True)

    def overlapped():
        s_pack.wait_stream(torch.cuda.current_stream())
        ff.ff_pack_to_host(plan, chunks, crcs, h_chunks, h_crcs, 64, s_pack, s_copy)
        torch.cuda.current_stream().wait_stream(s_copy)

    out = {}
    for name, fn in (("pack_then_copy", serial), ("overlapped", overlapped)):
        fn()
        torch.cuda.synchronize()
        walls = []
        for _ in range(3):
            t0 = time.perf_counter()
            fn()
            torch.cuda.synchronize()
            walls.append((time.perf_counter() - t0) * 1e3)
        ms = sorted(walls)[1]  # the median of three: host-side hiccups of tens of ms do occur
        out[name] = {"ms": round(ms, 2), "payload_GBps": round(N / ms / 1e6, 1)}
    out["slice_chunks"] = 64
    del h_chunks, h_crcs
    return out


def main():
    args = parse()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this path runs on one GPU; a worker's snapshot needs no other worker "
              "(--gpus %d is not supported)" % args.gpus, file=sys.stderr)
        sys.exit(2)
    import torch
    from paper_2512_03644_amd import binding as ff
    from paper_2512_03644_amd import workloads as wl

    if not torch.cuda.is_available():
        print("bench.py needs a GPU", file=sys.stderr)
        sys.exit(2)
    dev = "cuda:0"
    torch.cuda.set_device(0)
    ff.lib()

    with_adam = not args.no_adam and args.workload == "llama7b"
    if args.workload == "llama7b":
        shard = wl.config_llama7b(dev, with_grads=with_adam)
    elif args.workload == "llama70b":
        shard = wl.config_llama70b(dev)
    elif args.workload == "fragmented":
        shard = wl.config_fragmented(dev)
    elif args.workload in wl.LAYOUT_VARIANTS:
        shard = wl.config_layout_variant(args.workload, dev)
    elif args.workload == "tiny":
        shard = wl.config_tiny(dev)
    else:
        print("bench.py: unknown workload %r" % args.workload, file=sys.stderr)
        sys.exit(2)
    plan = ff.plan_for_shard(shard, tile_log2=args.tile_log2)
    chunks, crcs, bad, n_bad = ff.alloc_outputs(plan, dev)
    N = plan.payload_bytes
    n_el = sum(p.master.numel() for p in shard.params)
    n_cpu_groups = 48 if args.workload == "llama7b" else 0
    hp = dict(lr=3e-4, beta1=0.9, beta2=0.95, eps=1e-8, weight_decay=0.1, step=1000)
    grads = [p.grad for p in shard.params] if with_adam else None

    def op_adam():
        ff.ff_adam_step_snapshot(plan, grads, hp, chunks, crcs)

    def op_pack():
        ff.ff_pack(plan, chunks, crcs)

    def op_restore():
        ff.ff_restore(plan, chunks, crcs, bad, n_bad)

    ops = [("pack", op_pack, 2 * N), ("restore", op_restore, 2 * N)]
    if with_adam:
        try:
            op_adam()
            torch.cuda.synchronize()
            ops.insert(0, ("adam_snapshot", op_adam, 42 * n_el))
        except ff.FFError as e:
            print("bench.py: fused Adam step unavailable (%s); step = pack + restore" % e,
                  file=sys.stderr)
            with_adam = False
    step_bytes = sum(b for _, _, b in ops)

    def step():
        for _, fn, _ in ops:
            fn()

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    # timed region: K steps; every op is bracketed by HIP events on the stream it is launched on
    evs = {name: [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True))
                  for _ in range(args.steps)] for name, _, _ in ops}
    t0 = time.perf_counter()
    for i in range(args.steps):
        for name, fn, _ in ops:
            a, b = evs[name][i]
            a.record()
            fn()
            b.record()
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    assert int(n_bad.item()) == 0
    ms_per_step = wall / args.steps * 1e3

    detail = {}
    for name, fn, nbytes in ops:
        ts = [a.elapsed_time(b) for a, b in evs[name]]
        avg = sum(ts) / len(ts)
        detail[name] = {"avg_ms": round(avg, 4), "median_ms": round(sorted(ts)[len(ts) // 2], 4),
                        "min_ms": round(min(ts), 4),
                        "traffic_GBps": round(nbytes / avg / 1e6, 1),
                        "frac_of_peak": round(nbytes / avg / 1e6 / HBM_PEAK_GBS, 4)}
    detail["pack"]["payload_GBps"] = round(N / detail["pack"]["avg_ms"] / 1e6, 1)
    detail["restore"]["payload_GBps"] = round(N / detail["restore"]["avg_ms"] / 1e6, 1)
    # the plain-copy ceiling of the same byte count, printed beside the real kernels: the packed
    # buffer itself copied into a scratch buffer (the same bytes the real kernels move; a buffer
    # of zeros copies about 1 % faster)
    n_copy = N // 16 * 16
    scratch = torch.empty(n_copy, dtype=torch.uint8, device=dev)
    ts = event_ms(lambda: ff.ff_copy_ceiling(scratch, chunks, n_copy), 5, torch)
    copy_gbs = 2 * n_copy / (sum(ts) / len(ts)) / 1e6
    del scratch
    for name in detail:
        detail[name]["frac_of_copy_ceiling"] = round(detail[name]["traffic_GBps"] / copy_gbs, 4)

    # the quantity the metric names: pack+CRC and restore together
    pr_ms = detail["pack"]["avg_ms"] + detail["restore"]["avg_ms"]
    pack_restore = {"ms": round(pr_ms, 4), "bytes": 4 * N, "GBps": round(4 * N / pr_ms / 1e6, 1),
                    "frac_of_peak": round(4 * N / pr_ms / 1e6 / HBM_PEAK_GBS, 4)}

    # roofline of the dominant (longest-running) kernel of the step
    kernels = {"adam_snapshot": ("fused_kernel", 42 * n_el), "pack": ("tile_kernel<pack>", 2 * N),
               "restore": ("tile_kernel<restore>", 2 * N)}
    dom = max(detail, key=lambda k: detail[k]["avg_ms"])
    kname, kbytes = kernels[dom]
    achieved = kbytes / detail[dom]["avg_ms"] / 1e6
    traffic, traffic_source = measured_traffic(kname, args.workload)
    roofline = {"bound": "hbm", "kernel": kname, "achieved": round(achieved, 1),
                "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": round(achieved / HBM_PEAK_GBS, 4),
                "traffic": traffic, "traffic_source": traffic_source,
                "algorithmic_bytes_per_launch": kbytes,
                "avg_launch_ms": detail[dom]["avg_ms"],
                "copy_ceiling_GBps": round(copy_gbs, 1)}

    # verify-only (what a receiver runs on arrival): reported beside the step, not part of it; on a
    # buffer that verifies (one in which every chunk is bad takes 8 % longer: every workgroup then
    # adds to the one counter)
    verify = lambda: ff.ff_restore(plan, chunks, crcs, bad, n_bad, flags=ff.FF_RESTORE_VERIFY_ONLY)
    for _ in range(2):  # the first launch of a kernel also loads its code
        verify()
    ts = event_ms(verify, 10, torch)
    verify_ms = sum(ts) / len(ts)
    extra = {"verify_only": {"avg_ms": round(verify_ms, 4), "min_ms": round(min(ts), 4),
                             "payload_GBps": round(N / verify_ms / 1e6, 1),
                             "frac_of_peak": round(N / verify_ms / 1e6 / HBM_PEAK_GBS, 4)}}
    extra.update(selective_restore(ff, wl, torch, plan, chunks, crcs, bad, n_bad, N))
    if not args.no_host_staging:
        extra["pack_to_host"] = pack_to_host(ff, torch, plan, chunks, crcs, N)
    if with_adam:
        # the traffic of the optimizer step alone, in the fastest shape found for this mix of
        # streams (no arithmetic, no CRC): the measured ceiling beside the fused kernel
        ff.ff_pack(plan, chunks, crcs)
        ts = event_ms(lambda: ff.ff_mix_ceiling(plan, grads, None, chunks), 5, torch)
        mix_ms = sum(ts) / len(ts)
        extra["mix_ceiling"] = {"avg_ms": round(mix_ms, 4), "bytes_per_launch": 42 * n_el,
                                "traffic_GBps": round(42 * n_el / mix_ms / 1e6, 1),
                                "frac_of_peak": round(42 * n_el / mix_ms / 1e6 / HBM_PEAK_GBS, 4)}
        detail["adam_snapshot"]["frac_of_mix_ceiling"] = round(
            mix_ms / detail["adam_snapshot"]["avg_ms"], 4)
        roofline["mix_ceiling_GBps"] = extra["mix_ceiling"]["traffic_GBps"]
    if with_adam:
        # The fused step with the optimizer state kept in the two alternating snapshots (reads
        # 14 B and writes 16 B per element): reported beside the step, not part of it.  It runs
        # last, from the step's final snapshot, since it moves the state out of the tensors.
        ff.ff_pack(plan, chunks, crcs)     # a buffer that verifies, whatever ran before
        chunks2 = torch.empty_like(chunks)
        crcs2 = torch.empty_like(crcs)
        pair = [(chunks, crcs), (chunks2, crcs2)]

        def op_chained():
            ff.ff_adam_step_chained(plan, grads, hp, pair[0][0], pair[1][0], pair[1][1])
            pair.reverse()
        ts = event_ms(op_chained, 6, torch)
        chained_ms = sum(ts) / len(ts)
        ff.ff_restore(plan, pair[0][0], pair[0][1], bad, n_bad, flags=ff.FF_RESTORE_VERIFY_ONLY)
        torch.cuda.synchronize()
        assert int(n_bad.item()) == 0
        ts2 = event_ms(lambda: ff.ff_mix_ceiling(plan, grads, pair[0][0], pair[1][0]), 5, torch)
        mixc_ms = sum(ts2) / len(ts2)
        extra["adam_chained"] = {"avg_ms": round(chained_ms, 4), "min_ms": round(min(ts), 4),
                                 "bytes_per_launch": 30 * n_el,
                                 "traffic_GBps": round(30 * n_el / chained_ms / 1e6, 1),
                                 "frac_of_peak": round(30 * n_el / chained_ms / 1e6 / HBM_PEAK_GBS, 4),
                                 "mix_ceiling_ms": round(mixc_ms, 4),
                                 "frac_of_mix_ceiling": round(mixc_ms / chained_ms, 4)}
        del chunks2
    metric = "snapshot pack+CRC and restore GB/s, % of HBM peak, 7B-shaped shard"
    if args.workload != "llama7b":
        metric = "snapshot pack+CRC and restore GB/s, %% of HBM peak, %s shard" % args.workload
    out = {"metric": metric,
           "value": round(step_bytes / (ms_per_step * 1e-3) / 1e9, 1), "unit": "GB/s",
           "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
           "ms_per_step": round(ms_per_step, 4), "higher_is_better": True, "scaling": "weak",
           "vs_baseline": None, "dtype": "f32" if with_adam else "u8", "data": "synthetic",
           "config": {"workload": "%s shard: %d parameter groups, %d B payload, %d segments, "
                                  "%d KiB chunks (%d)"
                                  % (shard.name, len(shard.params), N, plan.num_segments,
                                     plan.chunk_bytes // 1024, plan.num_chunks),
                      "step": " + ".join(n for n, _, _ in ops),
                      "bytes_per_step": step_bytes},
           "pct_of_hbm_peak": round(step_bytes / (ms_per_step * 1e-3) / 1e9 / HBM_PEAK_GBS * 100, 2),
           "pack_restore": pack_restore, "ops": detail, "extra": extra, "roofline": roofline}
    if not args.no_cpu_baseline and n_cpu_groups:
        out["cpu_baseline"] = cpu_baseline(shard, n_cpu_groups, hp, with_adam, torch)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
