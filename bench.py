#!/usr/bin/env python3
"""Benchmark of the snapshot hot path on one MI355X.

A step is one training iteration of the synthetic proxy: a bf16 GEMM phase of fixed length
(forward+backward stand-in), the wait for the immutable window's end, the Adam update over the whole
shard, and, every `ckpt_every` steps, a snapshot request. Everything the checkpoint path does (pack
kernels, device-to-host copies into the pinned ring, file writes) runs in the library, overlapped
with the following steps. Prints ONE JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--config 1..5]
"""
import argparse
import json
import os
import shutil
import statistics
import sys
import tempfile
import time

# More hardware queues than the four HIP uses by default, so that the compute stream, the pack stream
# and the copy streams each get one (must be set before the HIP runtime starts).
if int(os.environ.get("GPU_MAX_HW_QUEUES", "0") or 0) < 8:
    os.environ["GPU_MAX_HW_QUEUES"] = "8"

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--config", type=int, default=2, help="workload 1..5 (default 2: Llama-7B-shaped shard, 94 GB)")
    ap.add_argument("--ckpt-every", type=int, default=0, help="0: the workload's own interval")
    ap.add_argument("--compute-ms", type=float, default=0.0, help="0: the workload's own forward+backward length")
    ap.add_argument("--ring-gib", type=float, default=0.0, help="0: the whole data region, at most 16 GiB")
    ap.add_argument("--staging-gib", type=float, default=0.0, help="0: two super-chunks")
    ap.add_argument("--chunk-mib", type=int, default=256)
    ap.add_argument("--superchunk-mib", type=int, default=1024)
    ap.add_argument("--dma-streams", type=int, default=2)
    ap.add_argument("--io-threads", type=int, default=6)
    ap.add_argument("--policy", choices=["d2h", "pack"], default="d2h")
    ap.add_argument("--io-mode", choices=["auto", "pwrite", "mmap"], default="auto")
    ap.add_argument("--o-direct", type=int, default=0, help="1: checkpoint files are written with O_DIRECT and fsync'ed (a real disk as the sink)")
    ap.add_argument("--fsync", type=int, default=1, help="1: every file is fsync'ed before and its directory after the commit (the library's "
                                                         "default: a file ckpt_flush reports is durable, as far as the sink can be); 0: no fsync")
    ap.add_argument("--keep-last", type=int, default=1, help="checkpoint files kept; older ones are recycled in place (0: keep all)")
    ap.add_argument("--prealloc", type=int, default=2, help="spare files pre-allocated at registration")
    ap.add_argument("--direct-min-mib", type=float, default=0.0,
                    help="hybrid path: tensors of at least this size are copied by the DMA engines straight out of their own "
                         "memory, only smaller ones are packed (0: everything is packed)")
    ap.add_argument("--tier2-dir", default="", help="second, slower storage tier: committed files are copied on to this directory in the background")
    ap.add_argument("--tier2-threads", type=int, default=4)
    ap.add_argument("--tier2-mode", choices=["newest", "every"], default="newest",
                    help="newest: the slow tier takes the newest snapshot whenever it is free; every: no snapshot is skipped, training waits")
    ap.add_argument("--tier2-direct", type=int, default=1, help="1: second-tier files are written with O_DIRECT")
    ap.add_argument("--out-dir", default="")
    ap.add_argument("--baseline-steps", type=int, default=6)
    ap.add_argument("--baseline-discard-s", type=float, default=4.0,
                    help="seconds of steps run and discarded at the start of each no-checkpoint baseline phase")
    ap.add_argument("--oracle-sample-gb", type=float, default=32.0,
                    help="bytes of the workload the CPU oracle serializes for the cpu_baseline figure (about 10 s on one core)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-restore", action="store_true")
    ap.add_argument("--variant-steps", type=int, default=20,
                    help="extra steps measured under window policy PACK with full device staging (0: skip)")
    ap.add_argument("--solo-snapshots", type=int, default=2, help="snapshots taken with no training proxy running, after the timed region (0: off)")
    ap.add_argument("--paired-blocks", type=int, default=3,
                    help="workloads that checkpoint every step: alternate this many blocks of checkpointed and quiet steps "
                         "after the timed region for a stall figure free of thermal drift (0: off)")
    ap.add_argument("--reduce", type=int, default=0,
                    help="1: data reduction (format version 2): every p_bf16 tensor is declared derived from its master weights; "
                         "a snapshot whose pairs hold leaves them out (12 instead of 14 bytes per parameter cross the link)")
    ap.add_argument("--idle-library-steps", type=int, default=6,
                    help="steps run with the library's calls in the loop but no snapshot pending or requested, long after the last "
                         "copy (a third reference for the stall: what the calls themselves cost; 0: off)")
    ap.add_argument("--hbm-victim-gib", type=float, default=0.0,
                    help="G > 0: a heavier victim. After every 16 GEMM launches of the forward/backward stand-in one streaming "
                         "copy kernel moves G GiB through HBM (the memory-bound phases of a real step: normalisation, element-wise "
                         "work, attention softmax), so the snapshot's pack kernel and copies meet HBM traffic as well as MFMA work")
    ap.add_argument("--torch-runtime", type=int, default=1,
                    help="1: before anything else touches the GPU, a child process measures workload 1 with PyTorch owning device "
                         "memory, stream and HIP runtime (paper_2406_10707_amd/torch_runtime_probe.py); its figures go into the "
                         "torch_runtime block of the JSON line. 0: skip")
    ap.add_argument("--pack-only", type=int, default=0,
                    help="N > 0: no snapshot engine, no proxy; N calls of ckpt_pack_image over the whole workload (one launch of the pack "
                         "kernel each) after one 4 GiB launch of the plain copy kernel. For rocprofv3 runs of the pack kernel alone: "
                         "kernel durations and, with --pmc, HBM traffic, the copy kernel being the counters' calibration")
    ap.add_argument("--dump", default="", help="write per-step timings and per-snapshot measurements to this JSON file")
    return ap.parse_args()


def measure_link_peak(B, harness, s, nbytes=1 << 30, reps=10):
    """Best of `reps` single pinned copies of 1 GiB in each direction (GB/s)."""
    d = harness.DevBuf(nbytes)
    h = B.proxy_host_alloc_pinned(nbytes)
    best = {"d2h": 0.0, "h2d": 0.0}
    t_end = time.perf_counter() + 0.5          # half a second of copies first: a card fresh out of idle has been seen at half the rate
    while time.perf_counter() < t_end:
        B.proxy_copy_pinned_async(h, d.ptr, nbytes, True, s.handle)
        s.synchronize()
    for name, to_host in (("d2h", True), ("h2d", False)):
        for _ in range(reps):
            e0, e1 = harness.Event(), harness.Event()
            e0.record(s)
            B.proxy_copy_pinned_async(h if to_host else d.ptr, d.ptr if to_host else h, nbytes, to_host, s.handle)
            e1.record(s)
            e1.synchronize()
            best[name] = max(best[name], nbytes / (e0.elapsed_time(e1) * 1e-3) / 1e9)
    B.proxy_host_free_pinned(h)
    d.free()
    return best


def measure_devcopy(B, harness, s, nbytes=4 << 30, reps=5):
    """Contiguous aligned copy kernel: the practical HBM ceiling for the pack kernel (GB/s read+write)."""
    a, b = harness.DevBuf(nbytes), harness.DevBuf(nbytes)
    B.proxy_device_fill_async(a.ptr, 1, nbytes, s.handle)
    best = 0.0
    for _ in range(reps):
        e0, e1 = harness.Event(), harness.Event()
        e0.record(s)
        B.proxy_devcopy(b.ptr, a.ptr, nbytes, s.handle)
        e1.record(s)
        e1.synchronize()
        best = max(best, 2 * nbytes / (e0.elapsed_time(e1) * 1e-3) / 1e9)
    a.free()
    b.free()
    return best


def cpu_baseline(harness, shard, sample_bytes, out_dir):
    """The oracle as it stands: blocking per-tensor read-back into pageable memory, then the plain C
    serializer writing the same format to the same sink. One host thread."""
    from oracle import oracle, readback
    ks, total = [], 0
    for k, t in enumerate(shard.spec.tensors):
        ks.append(k)
        total += t.nbytes
        if total >= sample_bytes:
            break
    path = os.path.join(out_dir, "oracle_sample.dsl")
    harness.synchronize()
    t0 = time.perf_counter()
    host = [readback.d2h(shard.ptrs[k], shard.spec.tensors[k].nbytes) for k in ks]
    tensors = [(shard.spec.tensors[k].name, shard.spec.tensors[k].dtype, shard.spec.tensors[k].shape, h) for k, h in zip(ks, host)]
    oracle.serialize_file(tensors, 0, path)
    dt = time.perf_counter() - t0
    os.unlink(path)
    return {"value": round(total / dt / 1e9, 3), "unit": "GB/s", "cores": 1, "kind": "oracle",
            "sample": "first %d tensors (%.2f GB) of the workload: blocking read-back + serialize to the same sink, %.1f s; box has %d cores"
                      % (len(ks), total / 1e9, dt, os.cpu_count())}


def traffic_ratio(config):
    """HBM traffic of the pack kernel over its algorithmic bytes on this workload, as measured with rocprofv3
    counters (profiles/snapshot_path_workload<config>_*.txt, part 3); None when the summary is not there."""
    import glob
    for path in glob.glob(os.path.join(ROOT, "profiles", "snapshot_path_workload%d_*.txt" % config)):
        for line in open(path):
            if line.strip().startswith("traffic_over_algorithmic:"):
                return float(line.split(":")[1].split()[0])
    return None


def main():
    args = parse_args()
    if args.gpus != 1:
        print("bench.py: this build measures one GPU; --gpus %d is not supported (each box has one MI355X and the "
              "snapshot path of a shard needs no exchange between GPUs)" % args.gpus, file=sys.stderr)
        sys.exit(2)
    from paper_2406_10707_amd import build as build_lib
    build_lib.ensure_built()           # loads what is built; rebuilds only a missing or outdated library
    from paper_2406_10707_amd import binding as B
    from paper_2406_10707_amd import harness, shards

    args.torch_runtime_result = torch_runtime_probe() if args.torch_runtime and not args.pack_only else None
    spec = shards.make_shard(args.config)
    every = args.ckpt_every or spec.ckpt_every
    compute_ms = args.compute_ms or spec.compute_ms
    base = args.out_dir or ("/dev/shm" if os.path.isdir("/dev/shm") else None)
    out_dir = tempfile.mkdtemp(prefix="dsllm_bench_", dir=base)
    try:
        run(args, B, harness, spec, every, compute_ms, out_dir)
    finally:
        shutil.rmtree(out_dir, ignore_errors=True)


def torch_runtime_probe():
    """The same path in a process of its own where PyTorch owns memory, stream and HIP runtime (this process uses
    neither PyTorch nor its runtime, and has not touched the GPU yet)."""
    import subprocess
    say("child process: workload 1 under PyTorch's HIP runtime")
    try:
        r = subprocess.run([sys.executable, "-m", "paper_2406_10707_amd.torch_runtime_probe"], cwd=ROOT, capture_output=True, text=True,
                           timeout=400)
        lines = [ln for ln in r.stdout.splitlines() if ln.startswith("{")]
        if r.returncode != 0 or not lines:
            return {"error": (r.stderr or r.stdout)[-400:]}
        return json.loads(lines[-1])
    except Exception as e:      # a probe must not take the benchmark down with it
        return {"error": repr(e)[:400]}


def say(msg):
    """Progress line on stderr (stdout carries the one JSON line)."""
    print(f"[bench {time.strftime('%H:%M:%S')}] {msg}", file=sys.stderr, flush=True)


def pack_only(args, B, harness, spec):
    """The pack kernel alone on the workload's real tensor list (ckpt_pack_image), for profiler runs."""
    stream = harness.make_compute_stream()
    shard = harness.DeviceShard(spec)
    shard.fill_device(stream)
    a, b = harness.DevBuf(4 << 30), harness.DevBuf(4 << 30)
    B.proxy_device_fill_async(a.ptr, 1, a.nbytes, stream.handle)
    B.proxy_devcopy(b.ptr, a.ptr, a.nbytes, stream.handle)        # calibration launch: reads 4 GiB, writes 4 GiB
    stream.synchronize()
    a.free()
    b.free()
    descs = shard.descs()
    data = sum(-(-d[4] // 4096) * 4096 for d in descs)
    payload = sum(d[4] for d in descs)
    dst = harness.DevBuf(data)
    wall = []
    for _ in range(args.pack_only):
        t0 = time.perf_counter()
        B.pack_image(descs, dst.ptr, data, stream.cuda_stream)
        wall.append(round((time.perf_counter() - t0) * 1e3, 3))
    print(json.dumps({"mode": "pack_only", "workload": spec.name, "n_tensors": len(descs), "payload_bytes": payload, "data_bytes": data,
                      "algorithmic_bytes_per_launch": payload + data, "calibration_copy_bytes": 4 << 30,
                      "call_wall_ms_including_table_build_alloc_and_sync": wall}), flush=True)


def run(args, B, harness, spec, every, compute_ms, out_dir):
    if args.pack_only > 0:
        return pack_only(args, B, harness, spec)
    info = B.proxy_device_info()
    stream = harness.make_compute_stream()
    say("link peak and copy-kernel ceiling")
    link = measure_link_peak(B, harness, stream)
    devcopy_gbps = measure_devcopy(B, harness, stream)

    shard = harness.DeviceShard(spec)
    say(f"shard {spec.name}: fill on device")
    shard.fill_device(stream)
    stream.synchronize()
    gemm = harness.GemmProxy(8192)
    launches, gemm_ms_per_launch = gemm.calibrate(compute_ms, stream)
    hbm_a = hbm_b = None
    if args.hbm_victim_gib > 0:
        nb = int(args.hbm_victim_gib * (1 << 30)) // 4096 * 4096
        hbm_a, hbm_b = harness.DevBuf(nb), harness.DevBuf(nb)
        B.proxy_device_fill_async(hbm_a.ptr, 1, nb, stream.handle)
        e0, e1 = harness.Event(), harness.Event()
        B.proxy_devcopy(hbm_b.ptr, hbm_a.ptr, nb, stream.handle)
        e0.record(stream)
        B.proxy_devcopy(hbm_b.ptr, hbm_a.ptr, nb, stream.handle)
        e1.record(stream)
        e1.synchronize()
        copy_ms = e0.elapsed_time(e1)
        # keep the phase's length: the copies take their share of it
        launches = max(16, int(round(compute_ms / (gemm_ms_per_launch + copy_ms / 16.0))))

    def forward_backward():
        if hbm_a is None:
            gemm.run(launches, stream)
            return
        done = 0
        while done < launches:
            n = min(16, launches - done)
            gemm.run(n, stream)
            B.proxy_devcopy(hbm_b.ptr, hbm_a.ptr, hbm_a.nbytes, stream.handle)
            done += n

    policy = B.CKPT_WINDOW_PACK if args.policy == "pack" else B.CKPT_WINDOW_D2H
    chunk, sc = args.chunk_mib << 20, args.superchunk_mib << 20
    data_upper = spec.payload_bytes + 4096 * len(spec.tensors)
    # with SDMA copies the ring size does not limit the copy rate; a quarter of the paper's 64 GB host cache is plenty
    ring_bytes = int(args.ring_gib * (1 << 30)) or min(16 << 30, -(-data_upper // chunk) * chunk)
    args.ring_gib = round(ring_bytes / (1 << 30), 2)
    # the variant (update released after the pack, copies drain from device staging) needs staging for the whole
    # data region; under the paper's rule the staging size is not on the critical path
    want_variant = args.variant_steps > 0 and args.policy == "d2h" and args.direct_min_mib == 0
    staging_bytes = int(args.staging_gib * (1 << 30))
    if want_variant and not staging_bytes:
        full = -(-data_upper // sc) * sc
        free = info["free_mem"] - spec.payload_bytes - (8 << 30)
        if full <= free:
            staging_bytes = full
        else:
            want_variant = False
    staging_gib = round((staging_bytes or 2 * sc) / (1 << 30), 2)
    cfg = B.make_config(out_dir=out_dir, host_ring_bytes=ring_bytes, dma_chunk_bytes=chunk, pack_superchunk_bytes=sc,
                        dev_staging_bytes=staging_bytes, n_dma_streams=args.dma_streams, n_io_threads=args.io_threads,
                        window_policy=policy, direct_min_bytes=int(args.direct_min_mib * (1 << 20)),
                        io_mode={"auto": B.CKPT_IO_AUTO, "pwrite": B.CKPT_IO_PWRITE, "mmap": B.CKPT_IO_MMAP}[args.io_mode],
                        o_direct=args.o_direct, fsync_on_commit=1 if args.fsync else -1,
                        keep_last=args.keep_last, prealloc_files=args.prealloc if args.keep_last else 0)
    say("ckpt_init + ckpt_register_tensors (ring pinned and touched, spare files pre-allocated)")
    t0 = time.perf_counter()
    ck = B.Checkpointer(cfg)
    pairs = [(k, k + 1) for k, t in enumerate(spec.tensors) if t.role == "p_bf16"] if args.reduce else []
    if pairs:
        ck.declare_derived(pairs)
    ck.register_tensors(shard.descs())
    tier2_dir = ""
    if args.tier2_dir:
        tier2_dir = tempfile.mkdtemp(prefix="dsllm_tier2_", dir=args.tier2_dir)
        ck.enable_second_tier(tier2_dir, n_threads=args.tier2_threads, o_direct=args.tier2_direct, keep_last=1,
                              mode=B.CKPT_TIER2_EVERY if args.tier2_mode == "every" else B.CKPT_TIER2_NEWEST)
    init_s = time.perf_counter() - t0
    lay = ck.layout()
    # bytes one snapshot moves over the link and into its file: the version-2 data region when derived tensors are declared
    # (and their pairs hold, which the update kernel of the proxy guarantees; every snapshot's own figure is in its stats)
    S = lay["reduced_data_bytes"] if pairs else lay["data_bytes"]
    requested, live_files = [], []
    # the step counter starts so that the last warm-up step requests a snapshot: its copies then run in the
    # first timed steps whatever K and W are (with the defaults, W = 10 and a checkpoint every 10 steps, it starts at 0);
    # without warm-up the first timed step requests one
    state = {"step": (-args.warmup) % every if args.warmup > 0 else every - 1}

    def iteration(step, with_ckpt, marks, snap=True):
        """One step on `stream`; marks gets (start, after-gemm, end) events."""
        e = [harness.Event() for _ in range(3)]
        e[0].record(stream)
        forward_backward()
        e[1].record(stream)
        if with_ckpt:
            ck.wait_immutable_window_end(stream.cuda_stream)
        shard.update(step, stream)
        if with_ckpt and snap and step % every == 0:
            ck.snapshot_async(step, stream.cuda_stream)
            requested.append(step)
            live_files.append(step)
        e[2].record(stream)
        marks.append(e)

    def reap(block=False):
        """Unlink committed checkpoint files except the newest (the sink may be tmpfs, i.e. host memory).
        With keep_last > 0 the library retires old files itself."""
        if args.keep_last:
            return
        for it in live_files[:-1]:
            if block:
                ck.flush(it)
            if ck.stats(it)["committed"]:
                os.unlink(ck.file_name(it))
                live_files.remove(it)

    baseline_trace = []      # per-step times of every no-checkpoint phase, for --dump

    def baseline_phase(n, library_calls=False):
        """Same steps with checkpointing off: (median step ms, median GEMM-phase ms). After an idle period
        the card runs a few per cent faster for some seconds, so the first ~4 s of steps are discarded.
        library_calls: the loop makes the library's calls (window wait) but requests no snapshot."""
        marks = []
        skip = min(max(2, int(args.baseline_discard_s * 1000.0 / max(compute_ms, 1.0)) + 1), 40) if args.baseline_discard_s > 0 else 0
        for i in range(skip + n):
            iteration(1000000 + i, library_calls, marks, snap=False)
        stream.synchronize()
        baseline_trace.append({"library_calls": library_calls, "discarded": skip,
                               "iter_ms": [round(m[0].elapsed_time(m[2]), 3) for m in marks],
                               "gemm_ms": [round(m[0].elapsed_time(m[1]), 3) for m in marks]})
        return (statistics.median(m[0].elapsed_time(m[2]) for m in marks[skip:]),
                statistics.median(m[0].elapsed_time(m[1]) for m in marks[skip:]))

    def region(n_steps):
        """n_steps checkpointed steps bracketed by full synchronisation; returns timings and wall seconds."""
        marks = []
        first = state["step"] + 1
        harness.synchronize()
        t_start = time.perf_counter()
        for _ in range(n_steps):
            state["step"] += 1
            iteration(state["step"], True, marks)
            reap()
        harness.synchronize()
        wall = time.perf_counter() - t_start
        return {"first": first, "last": state["step"], "wall_s": wall,
                "iter_ms": [m[0].elapsed_time(m[2]) for m in marks], "gemm_ms": [m[0].elapsed_time(m[1]) for m in marks]}

    def alternating_phase(blocks, block_len):
        """Blocks of checkpointed steps alternate with blocks of steps that request no snapshot, a few seconds
        each, so both kinds run in the same thermal state of the card (its GEMM speed drifts by a few per cent
        over tens of seconds, which biases a comparison with a separate no-checkpoint phase). Compared are the
        steady steps of each kind: checkpointed steps whose predecessor also requested a snapshot, and quiet
        steps from the third of a block on (the last snapshot's copies are over by then)."""
        marks, kind = [], []
        harness.synchronize()
        for _ in range(blocks):
            for j in range(2 * block_len):
                state["step"] += 1
                iteration(state["step"], True, marks, snap=j < block_len)
                kind.append(("busy" if j >= 1 else None) if j < block_len else ("quiet" if j - block_len >= 2 else None))
                reap()
        harness.synchronize()
        out = {}
        for name in ("busy", "quiet"):
            sel = [m for m, k in zip(marks, kind) if k == name]
            out[name] = (statistics.median(m[0].elapsed_time(m[2]) for m in sel), statistics.median(m[0].elapsed_time(m[1]) for m in sel), len(sel))
        return out

    def gbps(nbytes, ms):
        return nbytes / (ms * 1e-3) / 1e9 if ms and ms > 0 else None

    def stall_report(reg, base_iter_ms, base_gemm_ms, drained_before=False):
        """Stall of a region against BOTH references. The headline figures (stall_ms_per_step, stall_pct,
        stall_ms_per_snapshot) are against the no-checkpoint baseline phases, which is the metric's definition
        (training stall versus no checkpointing). The second reference, the quiet steps of the same region (4 or
        more steps after the latest snapshot request, at least three of them), is given beside it."""
        # snapshots whose copies run inside the region: requested by the step before it (unless everything was
        # drained before the region began) up to the step before its last
        lo = reg["first"] if drained_before else reg["first"] - 1
        in_reg = [it for it in requested if lo <= it < reg["last"]]
        busy, quiet, quiet_iter = [], [], []
        for i, g in enumerate(reg["gemm_ms"]):
            since = min([reg["first"] + i - it for it in requested if it < reg["first"] + i] or [99])
            if since <= 2:
                busy.append(g)
            elif since >= 4:
                quiet.append(g)
                quiet_iter.append(reg["iter_ms"][i])
        n = len(reg["iter_ms"])
        total = sum(reg["iter_ms"]) - base_iter_ms * n
        out = {
            "reference": "no-checkpoint baseline phases (before and after, averaged)",
            "reference_ms_per_step": round(base_iter_ms, 3), "ms_per_step": round(statistics.mean(reg["iter_ms"]), 3),
            "stall_ms_per_step": round(total / n, 3),
            "stall_pct": round(100.0 * total / (base_iter_ms * n), 3),
            "stall_ms_per_snapshot": round(total / max(1, len(in_reg)), 2),
            "gemm_ms_reference": round(base_gemm_ms, 3),
            "gemm_ms_while_copying": round(statistics.median(busy), 3) if busy else None,
            "gemm_slowdown_pct": round(100.0 * (statistics.median(busy) / base_gemm_ms - 1), 3) if busy else None}
        if len(quiet) >= 3:
            q_iter, q_gemm = statistics.median(quiet_iter), statistics.median(quiet)
            q_total = sum(reg["iter_ms"]) - q_iter * n
            out["vs_quiet_steps_of_the_same_region"] = {
                "reference_ms_per_step": round(q_iter, 3), "stall_ms_per_step": round(q_total / n, 3),
                "stall_pct": round(100.0 * q_total / (q_iter * n), 3), "stall_ms_per_snapshot": round(q_total / max(1, len(in_reg)), 2),
                "gemm_ms_reference": round(q_gemm, 3),
                "gemm_slowdown_pct": round(100.0 * (statistics.median(busy) / q_gemm - 1), 3) if busy else None,
                "quiet_steps_slower_than_baseline_pct": round(100.0 * (q_iter / base_iter_ms - 1), 3)}
        return in_reg, out, base_gemm_ms

    # ---- baseline before; warm-up (untimed); the timed region of exactly K steps
    say("baseline phase (no checkpoints)")
    base_before = baseline_phase(args.baseline_steps)
    say(f"warm-up, {args.warmup} steps")
    region(args.warmup)
    say(f"timed region, {args.steps} steps")
    main = region(args.steps)
    say("drain, restore check")
    ms_per_step = main["wall_s"] * 1e3 / args.steps

    # ---- drain (the paper counts pending flushes in end-to-end time; reported, not part of the K steps)
    t0 = time.perf_counter()
    ck.flush()
    drain_s = time.perf_counter() - t0
    reap(block=True)

    # ---- restore of the newest file (its state is the device state only if the last step took a snapshot)
    restore_result = None
    if not args.no_restore and requested:
        last = requested[-1]
        probe = [0, len(shard.ptrs) // 2, len(shard.ptrs) - 1]
        want = {k: shard.readback(k) for k in probe}
        for k in probe:
            B.proxy_device_fill_async(shard.ptrs[k], 0xA5, shard.spec.tensors[k].nbytes, stream.handle)
        harness.synchronize()
        t0 = time.perf_counter()
        ck.restore(ck.file_name(last), stream.cuda_stream)
        stream.synchronize()
        dt = time.perf_counter() - t0
        ok = all((shard.readback(k) == want[k]).all() for k in probe) if last == state["step"] else None
        restore_result = {"gbps": round(S / dt / 1e9, 2), "seconds": round(dt, 2), "probe_tensors_bit_exact": ok if ok is None else bool(ok)}

    # ---- snapshot-only: the same snapshots with nothing else on the card (the interference baseline)
    solo_rows = []
    if args.solo_snapshots > 0:
        say(f"snapshot-only phase, {args.solo_snapshots} snapshots")
        harness.synchronize()
        for j in range(args.solo_snapshots):
            it = 2000000 + j
            ck.snapshot_async(it, stream.cuda_stream)
            ck.wait_immutable_window_end(stream.cuda_stream)
            ck.flush(it)
            solo_rows.append(ck.stats(it))
            if not args.keep_last:
                os.unlink(ck.file_name(it))

    # ---- every-iteration workloads have no quiet steps inside the timed region: paired reference
    paired = None
    if every == 1 and args.paired_blocks > 0:
        ck.flush()
        say("alternating blocks of checkpointed and quiet steps")
        block_len = max(5, min(20, int(1000.0 / max(compute_ms, 1.0) + 0.999)))
        alt = alternating_phase(args.paired_blocks, block_len)
        ck.flush()
        reap(block=True)
        paired = {"checkpointed_ms_per_step": round(alt["busy"][0], 3), "quiet_ms_per_step": round(alt["quiet"][0], 3),
                  "stall_ms_per_step": round(alt["busy"][0] - alt["quiet"][0], 3),
                  "stall_pct": round(100.0 * (alt["busy"][0] / alt["quiet"][0] - 1), 3),
                  "gemm_slowdown_pct": round(100.0 * (alt["busy"][1] / alt["quiet"][1] - 1), 3),
                  "steps_compared": [alt["busy"][2], alt["quiet"][2]], "block_len": block_len,
                  "note": "blocks of checkpointed and of quiet steps alternate, medians of the steady steps of each kind"}

    # ---- variant: window released after the pack (policy PACK, staging holds the whole data region)
    variant = None
    if want_variant:
        say(f"variant: window policy PACK, {args.variant_steps} steps")
        ck.set_window_policy(B.CKPT_WINDOW_PACK)
        if state["step"] % every:                        # start the variant right after a multiple of the interval
            region(every - state["step"] % every)
            ck.flush()
        variant = region(args.variant_steps)
        ck.flush()
        ck.set_window_policy(B.CKPT_WINDOW_D2H)

    # ---- the link peak once more: the first measurement of a process has been seen at half the rate when the previous
    # process on the box had just released a hundred GB of pinned and file memory; the better of the two counts
    link2 = measure_link_peak(B, harness, stream)
    link_first = dict(link)
    link = {k: max(link[k], link2[k]) for k in link}

    # ---- baseline after; GEMM speed drifts a few per cent with temperature, so before and after are averaged
    say("baseline phase (no checkpoints)")
    base_after = baseline_phase(args.baseline_steps)
    base_iter_ms = 0.5 * (base_before[0] + base_after[0])
    base_gemm_ms = 0.5 * (base_before[1] + base_after[1])
    idle_lib = baseline_phase(args.idle_library_steps, library_calls=True) if args.idle_library_steps > 0 else None

    in_region, stall, ref_gemm_ms = stall_report(main, base_iter_ms, base_gemm_ms)
    stats = [ck.stats(it) for it in in_region]
    all_stats = [ck.stats(it) for it in requested]
    if not stats:      # a region too short to hold a snapshot's copies: the figures come from every snapshot of the run
        stats = [s for s in all_stats if s["d2h_done"]]
    snap_gbps = gbps(S * len(stats), sum(s["request_to_d2h_end_ms"] for s in stats)) if stats else None
    link_gbps = gbps(S * len(stats), sum(s["d2h_span_ms"] for s in stats)) if stats else None
    pack_launches = sum(s["pack_launches"] for s in stats)
    pack_ms = sum(s["pack_ms_sum"] for s in stats)
    # algorithmic bytes of the pack kernel: every payload byte read once, every data-region byte written once
    # (tensors copied directly on the hybrid path never pass through the kernel)
    # (nor do the derived tensors a version-2 snapshot leaves out)
    pack_bytes_per_snapshot = (lay["payload_bytes"] - lay["direct_bytes"] + lay["data_bytes"] - lay["direct_data_bytes"] if not pairs else
                               lay["payload_bytes"] - lay["derived_bytes"] + lay["reduced_data_bytes"])
    pack_gbps = gbps(pack_bytes_per_snapshot * len(stats), pack_ms) if stats else None
    # physical floor under the paper's rule: the copies cannot end before D / B_link, the window is the GEMM phase
    stall["floor_ms_per_snapshot"] = round(max(0.0, S / (link["d2h"] * 1e9) * 1e3 - ref_gemm_ms), 2)
    stall["stall_minus_floor_ms_per_snapshot"] = round(stall["stall_ms_per_snapshot"] - stall["floor_ms_per_snapshot"], 2)
    # the paper's own throughput figure: checkpoint size over the time training was blocked by it
    stall["perceived_gbps_paper_definition"] = round(S / (stall["stall_ms_per_snapshot"] * 1e-3) / 1e9, 1) if stall["stall_ms_per_snapshot"] > 0 else None
    if paired:
        paired["stall_minus_floor_ms_per_step"] = round(paired["stall_ms_per_step"] - stall["floor_ms_per_snapshot"], 2)
        stall["paired_alternating_blocks"] = paired
    stall["baseline_before_after_ms"] = [round(base_before[0], 2), round(base_after[0], 2)]
    if idle_lib:
        stall["library_idle_ms_per_step"] = round(idle_lib[0], 3)   # library calls in the loop, nothing pending, long after the last copy
    stall["gemm_tflops"] = round(gemm.flops_per_launch / (gemm_ms_per_launch * 1e-3) / 1e12, 1)

    result = {
        "metric": "snapshot GB/s per GPU (fraction of host-link peak) + training stall ms/iter",
        "value": round(snap_gbps, 3) if snap_gbps else None,
        "unit": "GB/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 3),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "u8", "data": "synthetic",
        "config": {"workload": spec.name, "payload_bytes": lay["payload_bytes"], "n_tensors": lay["n_tensors"],
                   "ckpt_every": every, "compute_ms": compute_ms, "window_policy": args.policy,
                   "ring_gib": args.ring_gib, "dma_chunk_mib": args.chunk_mib, "pack_superchunk_mib": args.superchunk_mib,
                   "staging_gib": staging_gib, "dma_streams": args.dma_streams, "io_threads": args.io_threads,
                   "hw_queues": int(os.environ["GPU_MAX_HW_QUEUES"]), "device": info["name"],
                   "hip_runtime": info["hip_runtime_version"], "io_mode": args.io_mode, "o_direct": args.o_direct, "fsync_on_commit": args.fsync, "keep_last": args.keep_last,
                   "prealloc_files": args.prealloc, "sink": out_dir.rsplit("/", 1)[0],
                   "direct_min_mib": args.direct_min_mib, "direct_tensors": lay["n_direct_tensors"],
                   "direct_bytes": lay["direct_bytes"], "copy_segments": lay["n_segments"],
                   "hbm_victim_gib": args.hbm_victim_gib, "reduce": args.reduce, "derived_tensors": lay["n_derived_tensors"], "link_bytes_per_snapshot": S},
        "roofline": {"bound": "hbm", "kernel": "pack_kernel", "achieved": round(pack_gbps, 1) if pack_gbps else None,
                     "peak": HBM_PEAK_GBPS, "unit": "GB/s", "frac": round(pack_gbps / HBM_PEAK_GBPS, 4) if pack_gbps else None,
                     "traffic": None, "traffic_source": "rocprofv3 FETCH_SIZE+WRITE_SIZE of this kernel on this workload, scaled by a copy kernel of known size (profiles/), as a ratio x algorithmic bytes per launch",
                     "launches": pack_launches,
                     "avg_launch_ms": round(pack_ms / pack_launches, 4) if pack_launches else None,
                     "bytes_per_launch": round(pack_bytes_per_snapshot / (pack_launches / max(1, len(stats)))) if pack_launches else None,
                     "devcopy_ceiling_gbps": round(devcopy_gbps, 1)},
        "snapshot": {"snapshots_in_timed_region": len(in_region), "link_peak_d2h_gbps": round(link["d2h"], 2),
                     "link_peak_h2d_gbps": round(link["h2d"], 2),
                     "link_peak_d2h_measurements_gbps": [round(link_first["d2h"], 2), round(link2["d2h"], 2)],
                     "d2h_gbps": round(link_gbps, 2) if link_gbps else None,
                     "d2h_frac_of_link_peak": round(link_gbps / link["d2h"], 4) if link_gbps else None,
                     "snapshot_gbps_frac_of_link_peak": round(snap_gbps / link["d2h"], 4) if snap_gbps else None,
                     "host_snapshot_call_ms": round(max(s["host_snapshot_call_ms"] for s in all_stats), 3) if all_stats else None,
                     # time inside ckpt_wait_immutable_window_end: in this open loop the host runs steps ahead of the device, and
                     # the call also absorbs that lead; the part the ring causes is the back-pressure time of the submit thread
                     "host_window_wait_ms": round(max(s["host_window_wait_ms"] for s in all_stats), 3) if all_stats else None,
                     "host_backpressure_ms": round(max(s["host_backpressure_ms"] for s in all_stats), 3) if all_stats else None,
                     "format_versions": sorted({s["format_version"] for s in all_stats}),
                     "verify_ms": round(statistics.median(s["verify_ms"] for s in all_stats), 3) if pairs and all_stats else None,
                     "flush_gbps": round(statistics.median(S / (s["host_flush_span_ms"] * 1e-3) / 1e9 for s in all_stats), 2) if all_stats else None,
                     "drain_s": round(drain_s, 2), "init_s": round(init_s, 2), "init_probe_d2h_gbps": round(ck.init_probe(), 2)},
        "stall": stall,
    }
    if solo_rows:
        result["snapshot_only"] = {
            "snapshots": len(solo_rows),
            "d2h_gbps": round(gbps(S * len(solo_rows), sum(s["d2h_span_ms"] for s in solo_rows)), 2),
            "snapshot_gbps": round(gbps(S * len(solo_rows), sum(s["request_to_d2h_end_ms"] for s in solo_rows)), 2),
            "pack_gbps": round(gbps(pack_bytes_per_snapshot * len(solo_rows), sum(s["pack_ms_sum"] for s in solo_rows)), 1),
            "note": "no training proxy running: what the GEMM loop costs the snapshot path is the difference to the timed region"}
    if variant:
        v_in, v_stall, _ = stall_report(variant, base_iter_ms, base_gemm_ms, drained_before=True)
        v_stats = [ck.stats(it) for it in v_in]
        v_stall["steps"] = len(variant["iter_ms"])
        v_stall["snapshots"] = len(v_in)
        v_stall["request_to_pack_end_ms"] = round(statistics.mean(s["request_to_pack_end_ms"] for s in v_stats), 2) if v_stats else None
        v_stall["snapshot_gbps"] = round(gbps(S * len(v_stats), sum(s["request_to_d2h_end_ms"] for s in v_stats)), 2) if v_stats else None
        v_stall["note"] = ("window policy PACK: the update waits for the pack kernels only; copies drain from device staging "
                           "that holds the whole data region (MI355X variant, not the paper's rule)")
        result["variant_pack_policy"] = v_stall

    if args.dump:
        with open(args.dump, "w") as f:
            json.dump({"main": main, "variant": variant, "requested": requested, "snapshots": all_stats,
                       "baseline_iter_ms": base_iter_ms, "baseline_gemm_ms": base_gemm_ms, "baseline_phases": baseline_trace}, f, indent=1)

    # the same kernel without a GEMM competing for the CUs: the snapshot requested by the last timed step
    # (its pack launches run while the host waits for the device at the end of the region)
    tail = [st for st in all_stats if st["iter"] == main["last"] and st["pack_ms_sum"] > 0]
    if tail:
        iso = gbps(pack_bytes_per_snapshot, tail[0]["pack_ms_sum"])
        result["roofline"]["no_gemm_running"] = {"achieved": round(iso, 1), "frac": round(iso / HBM_PEAK_GBPS, 4),
                                                 "avg_launch_ms": round(tail[0]["pack_ms_sum"] / tail[0]["pack_launches"], 4)}
    ratio = traffic_ratio(args.config)
    if ratio and pack_launches:
        result["roofline"]["traffic"] = round(ratio * result["roofline"]["bytes_per_launch"])
    if tier2_dir:
        say("second tier: waiting for the last copy")
        t0 = time.perf_counter()
        ck.wait_second_tier()
        t2_wait = time.perf_counter() - t0
        t2 = [ck.stats(it) for it in requested]
        done = [s for s in t2 if s["tier2_state"] == B.CKPT_TIER2_DONE]
        result["second_tier"] = {
            "dir": args.tier2_dir, "threads": args.tier2_threads, "o_direct": args.tier2_direct, "mode": args.tier2_mode,
            "snapshots": len(t2), "copied": len(done), "superseded": sum(s["tier2_state"] == B.CKPT_TIER2_SKIPPED for s in t2),
            "failed": sum(s["tier2_state"] == B.CKPT_TIER2_FAILED for s in t2),
            "copy_gbps": round(statistics.median(s["file_bytes"] / (s["host_tier2_ms"] * 1e-3) / 1e9 for s in done), 3) if done else None,
            "copy_seconds": round(statistics.median(s["host_tier2_ms"] for s in done) / 1e3, 2) if done else None,
            "wait_after_run_s": round(t2_wait, 2)}
    if restore_result:
        result["restore"] = restore_result
    if args.torch_runtime_result is not None:
        result["torch_runtime"] = args.torch_runtime_result
    ck.destroy()
    if not args.no_cpu_baseline:
        # the library's files go first: the sample's host arrays and its file need the memory (tmpfs is host memory)
        for f in os.listdir(out_dir):
            os.unlink(os.path.join(out_dir, f))
        say("oracle on the host cores (bounded sample)")
        result["cpu_baseline"] = cpu_baseline(harness, shard, int(args.oracle_sample_gb * 1e9), out_dir)
    if tier2_dir:
        shutil.rmtree(tier2_dir, ignore_errors=True)
    print(json.dumps(result), flush=True)


if __name__ == "__main__":
    main()
