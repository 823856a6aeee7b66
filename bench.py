"""Benchmark: decoder-only RTFx of the HIP WFST beam-search decoder on one MI355X.

A step is one wfst_decode_batch call over the whole batch (init, every frame of every
utterance, final choice and traceback) with the log-likelihoods already resident in HBM.
Prints ONE JSON line; see the roofline and cpu_baseline objects in it.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X published HBM3E bandwidth
KERNEL = "wfst_channel_kernel"


def algorithmic_bytes(counters, V):
    """Bytes the method has to move, from the deterministic counters (identical for the
    oracle and the GPU path): per frame one log-likelihood row; per expanded token its queue
    record and one {emitting, epsilon} offset pair; per emitting arc next state + weight +
    ilabel; per epsilon arc next state + weight; per in-beam recombined destination one
    8-byte map read-modify-write; per stored token its queue record and backpointer."""
    tok, earc, xarc, n_in, stored, _, _, frames = [int(x) for x in counters]
    return (frames * V * 4 + tok * (8 + 16) + earc * 12 + xarc * 8 + n_in * 16 + stored * (8 + 8))


def read_traffic(workload):
    """HBM bytes per launch measured with rocprofv3 counters (see profiles/); None if absent."""
    path = os.path.join(ROOT, "profiles", f"wfst_channel_kernel_{workload}_hbm_traffic.md")
    try:
        for ln in open(path):
            if ln.startswith("TRAFFIC_BYTES_PER_LAUNCH="):
                return int(float(ln.split("=", 1)[1]))
    except OSError:
        pass
    return None


def measure_traffic(child_args, timeout_s=180):
    """HBM bytes per launch of the channel kernel, measured now: two child runs of this script (one
    batch in flight, 2 timed steps) under `rocprofv3 --pmc`, FETCH_SIZE then WRITE_SIZE (KiB per
    dispatch), each scaled by what the same counter reads in the same run for the probe's plain copy
    kernel, which reads and writes exactly 1 GiB per launch.  Returns (bytes, detail) or (None, why)."""
    import csv
    import glob
    import shutil
    import subprocess
    import tempfile
    exe = shutil.which("rocprofv3")
    if not exe:
        return None, "rocprofv3 not found"
    if any(k.startswith("ROCPROF") for k in os.environ) or "rocprof" in os.environ.get("LD_PRELOAD", ""):
        return None, "this process is itself being profiled"
    work = tempfile.mkdtemp(prefix="wfst_traffic_")
    env = dict(os.environ, TMPDIR=tempfile.gettempdir(), PYTHONPATH=os.pathsep.join([ROOT, os.environ.get("PYTHONPATH", "")]))
    detail = {}
    try:
        for ctr in ("FETCH_SIZE", "WRITE_SIZE"):
            out = os.path.join(work, ctr.lower())
            cmd = [exe, "--pmc", ctr, "-d", out, "-o", ctr.lower(), "--output-format", "csv", "--",
                   sys.executable, os.path.join(ROOT, "bench.py"), "--pipeline", "1", "--steps", "2", "--warmup", "1",
                   "--no-cpu-baseline", "--no-traffic"] + child_args
            try:
                r = subprocess.run(cmd, cwd=work, env=env, capture_output=True, text=True, timeout=timeout_s)
            except subprocess.TimeoutExpired:
                return None, f"the {ctr} run did not finish in {timeout_s} s"
            if r.returncode != 0:
                return None, f"the {ctr} run ended with status {r.returncode}: {r.stderr[-300:]}"
            kern, copy = [], []
            for f in glob.glob(os.path.join(out, "**", "*counter_collection.csv"), recursive=True):
                for row in csv.DictReader(open(f)):
                    if row.get("Counter_Name") != ctr:
                        continue
                    if "wfst_channel_kernel" in row["Kernel_Name"]:
                        kern.append(float(row["Counter_Value"]))
                    elif "probe_copy" in row["Kernel_Name"]:
                        copy.append(float(row["Counter_Value"]))
            if not kern or not copy or min(copy) <= 0:
                return None, f"no {ctr} values for the kernel or the calibration copy in the profiler's output"
            kern = kern[-2:]                                    # the timed launches (the first one is the warm-up)
            scale = (1 << 20) / (sum(copy) / len(copy))         # the copy moves 2^20 KiB each way
            detail[ctr] = {"kib_per_launch": sum(kern) / len(kern), "copy_kib": sum(copy) / len(copy), "scale": scale}
        total = sum(d["kib_per_launch"] * d["scale"] * 1024.0 for d in detail.values())
        return int(total), detail
    finally:
        shutil.rmtree(work, ignore_errors=True)


def cpu_model():
    try:
        for ln in open("/proc/cpuinfo"):
            if ln.startswith("model name"):
                return ln.split(":", 1)[1].strip()
    except OSError:
        pass
    return "unknown"


def calibrate():
    """Measured ceilings of this GPU (paper_2311_04996_amd/csrc/wfst_probe.hip): a plain device copy,
    random 128-byte line reads and random 64-bit global atomics, each with the whole chip busy."""
    from paper_2311_04996_amd.probe import probe_atomics, probe_copy, probe_random_lines
    return {"copy_gb_per_s": probe_copy(1 << 30, 5),
            "random_128B_lines_per_s": probe_random_lines(1 << 32, 2048, 256),
            "random_64bit_atomics_per_s": probe_atomics(1 << 30, 2048, 64),
            "how": "1 GiB device copy (read + written bytes); 2048 workgroups x 1024 lanes, 8 loads (4 atomics) in "
                   "flight per lane, uniform over 4 GiB (1 GiB)"}


def cpu_baseline(w, threads, budget_s=15.0):
    """The oracle, as it stands, one utterance per thread on a bounded sample of the batch:
    the first N utterances in batch order, N chosen for about budget_s seconds of wall time.
    Also the single-thread rate (on the first 120 frames of one utterance)."""
    from concurrent.futures import ThreadPoolExecutor
    from oracle import Oracle
    o = Oracle(w.graph)

    def dec(b, n):
        return o.decode(w.loglikes[b], length=n, beam=w.beam, max_active=w.max_active,
                        boost=None if w.boosts is None else w.boosts[b],
                        boost_fst=None if w.boost_fsts is None else w.boost_fsts[b])
    probe = int(np.argmax(w.lengths >= min(120, int(w.lengths.max()))))
    t0 = time.perf_counter()
    dec(probe, min(120, int(w.lengths[probe])))
    per_frame = (time.perf_counter() - t0) / min(120, int(w.lengths[probe]))
    frames_budget = budget_s * threads / max(per_frame, 1e-9)
    take, acc = [], 0
    for b in range(len(w.lengths)):
        if len(take) >= threads and acc + int(w.lengths[b]) > frames_budget:
            break
        take.append(b); acc += int(w.lengths[b])
    t0 = time.perf_counter()
    with ThreadPoolExecutor(threads) as ex:
        list(ex.map(lambda b: dec(b, int(w.lengths[b])), take))
    dt = time.perf_counter() - t0
    audio = float(w.lengths[take].sum()) * 0.040
    return {"value": audio / dt, "unit": "audio-s/s", "cores": threads, "kind": "oracle",
            "sample": f"first {len(take)} utterances of the batch ({acc} frames), one per thread, {dt:.1f} s wall",
            "single_thread_value": 0.040 / per_frame, "nproc": os.cpu_count(), "cpu_model": cpu_model()}


def pick_concurrent_streams(torch, n):
    """n streams whose kernels the runtime really runs side by side.  HIP maps streams onto a few
    hardware queues; two streams that share one run their kernels one after the other, and which
    streams share is not visible from the API.  So a short spin kernel is timed alone and on pairs
    of candidate streams; a pair that takes about as long as one kernel is concurrent."""
    if n <= 1:
        return [torch.cuda.Stream() for _ in range(n)]
    cands = [torch.cuda.Stream() for _ in range(8)]
    cycles = 20_000_000                                       # roughly 10 ms

    def timed(streams):
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for st in streams:
            with torch.cuda.stream(st):
                torch.cuda._sleep(cycles)
        torch.cuda.synchronize()
        return time.perf_counter() - t0

    timed(cands)                                              # first use creates the queues
    one = min(timed([cands[0]]) for _ in range(2))
    chosen = [cands[0]]
    for st in cands[1:]:
        if len(chosen) == n:
            break
        if all(min(timed([c, st]) for _ in range(2)) < 1.5 * one for c in chosen):
            chosen.append(st)
    ok = len(chosen) == n
    picked = [cands.index(c) for c in chosen]
    while len(chosen) < n:                                    # none found: take what there is
        chosen.append(cands[len(chosen)])
    print(f"[bench] streams: spin kernel {one * 1e3:.1f} ms alone; "
          f"{'found' if ok else 'did NOT find'} {n} streams that run concurrently (candidates {picked} of 8)",
          file=sys.stderr, flush=True)
    return chosen


def main_streaming(args):
    """Streaming configuration: the c3_large graph, `channels` concurrent audio streams fed
    16-frame (640 ms) chunks with wfst_advance_chunk, partial hypotheses of every channel
    fetched after every chunk.  One JSON line: per-chunk latency and channels sustainable
    at real time."""
    from paper_2311_04996_amd.latency_model import load_table
    import torch
    from paper_2311_04996_amd import Decoder
    from workloads import CONFIGS, ctc_loglikes
    from workloads.configs import make_graph
    C, n_chunks, warm, extra = 16, args.chunks, 5, 10
    n = args.channels
    c = CONFIGS["c3_large"]
    g = make_graph("c3_large")
    T = C * (n_chunks + warm + extra)
    lengths = np.full(n, T, np.int32)
    ll = ctc_loglikes(4, lengths, T, g.num_classes, **c["ll"])                 # seed 4: the streaming config
    # chunk-major copy: [chunk][channel][C][V], the layout a batching server hands over
    chunks = torch.from_numpy(np.ascontiguousarray(
        ll.reshape(n, n_chunks + warm + extra, C, g.num_classes).transpose(1, 0, 2, 3))).cuda()
    # --recycle-window W: every channel's backpointer memory is a ring over W frames, so the streams
    # could go on for any length (a result is flagged if its path joins the previous result's path
    # further back than that; on this graph hypotheses stay apart for hundreds of frames)
    W = args.recycle_window
    dec = Decoder(g, max_channels=n, max_frames=W if W else T, max_words=512, max_active_hint=c["max_active"],
                  outputs_on_host=True, recycle_lattice=bool(W))
    chans = np.arange(n, dtype=np.int32)
    nfr = np.full(n, C, np.int32)
    if args.stream_workgroups:
        dec.set_launch_workgroups(args.stream_workgroups)
    dec.init_channels(chans, float(c["beam"]), int(c["max_active"]))
    torch.cuda.synchronize()
    print(f"[bench] streaming: {n} channels x {n_chunks}+{warm}+{extra} chunks of {C} frames, "
          f"{dec.device_bytes() / 2**30:.1f} GiB on device", file=sys.stderr, flush=True)
    lat, out = [], None
    for k in range(n_chunks + warm):
        t0 = time.perf_counter()
        if args.separate_partials:
            dec.advance_chunk(chans, chunks[k], nfr)
            out = dec.get_partial_batch(chans, finalize=False, out=out)      # host outputs: synchronises
        else:                                                                # both in one launch
            out = dec.advance_chunk_partial(chans, chunks[k], nfr, finalize=False, out=out)
        lat.append(time.perf_counter() - t0)
        assert not (out[3] & (8 | 16)).any(), (f"chunk {k}: a channel overflowed a buffer (flags "
                                               f"{sorted(set(out[3].tolist()))}): the run is invalid")
    assert not (out[3] & (8 | 16)).any(), "a channel overflowed a buffer: the run is invalid"
    # where a chunk's time goes: a few more chunks with a synchronisation between the two calls
    t_adv, t_ker, t_par = [], [], []
    for k in range(n_chunks + warm, n_chunks + warm + extra):
        t0 = time.perf_counter()
        dec.advance_chunk(chans, chunks[k], nfr)
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        t_ker.append(dec.last_kernel_ms())
        out = dec.get_partial_batch(chans, finalize=False, out=out)
        t_adv.append(1e3 * (t1 - t0)); t_par.append(1e3 * (time.perf_counter() - t1))
    assert not (out[3] & (8 | 16)).any(), "a channel overflowed a buffer: the run is invalid"
    device_gib = dec.device_bytes() / 2**30
    lat = np.array(lat[warm:]) * 1e3
    p50, p99 = float(np.percentile(lat, 50)), float(np.percentile(lat, 99))
    chunk_s = C * 0.040
    line = {"metric": "streaming chunk latency p50 (ms), advance 16 frames + partial hypotheses, all channels"
                      + ("" if args.separate_partials else " (one wfst_advance_chunk_partial call)"),
            "value": p50, "unit": "ms", "n_gpus": 1, "steps": n_chunks, "warmup": warm, "ms_per_step": float(lat.mean()),
            "higher_is_better": False, "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
            "config": {"workload": "c4_streaming", "channels": n, "chunk_frames": C, "states": g.num_states,
                       "arcs": g.num_arcs, "beam": c["beam"], "max_active": c["max_active"],
                       "recycled_lattice_window_frames": W or None, "device_gib": round(device_gib, 1)},
            "p50_ms": p50, "p99_ms": p99, "max_ms": float(lat.max()),
            "rtfx": n * chunk_s / (float(lat.mean()) * 1e-3),
            "channels_at_realtime_p99": int(n * chunk_s * 1e3 / p99),
            "channels_at_realtime_p50": int(n * chunk_s * 1e3 / p50),
            "mean_words_per_partial": float(out[1].mean()),
            "breakdown_ms": {"advance_chunk": float(np.median(t_adv)), "advance_chunk_kernel": float(np.median(t_ker)),
                             "get_partial_batch": float(np.median(t_par)),
                             "how": f"medians of {extra} more chunks with a synchronisation between the two calls"},
            # the paper's M/D/1 model (Section "Streaming inference") applied to the measured
            # compute latency: mean queue and total latency of a chunk request against load
            "latency_model": load_table(float(lat.mean()) * 1e-3, chunk_s, n)}
    dec.close()
    print(json.dumps(line), flush=True)


def main_lattice(args):
    """Lattice output on utterances of the c3_large workload: the batch is decoded with token records
    kept, then the lattices of all utterances are generated by one wfst_get_lattice_batch call (and,
    for comparison, by one wfst_get_lattice call per utterance) with the outputs left in device
    memory.  One JSON line: links found per second."""
    import torch
    from paper_2311_04996_amd import Decoder
    from workloads import make_config
    w = make_config(args.workload, batch=args.batch or 8)
    B, T, V = w.loglikes.shape
    dec = Decoder(w.graph, max_channels=B, max_frames=T, max_words=512, max_active_hint=w.max_active,
                  keep_token_records=True)
    ll = torch.from_numpy(w.loglikes).cuda()
    dec.get_counters(reset=True)
    dec.decode_batch(ll, w.lengths, w.beam, w.max_active)
    torch.cuda.synchronize()
    counters = dec.get_counters()
    rows = [ll[b, :int(w.lengths[b])].contiguous() for b in range(B)]
    sizes = []
    for b in range(B):                                # sizes (and warm-up)
        _, _, _, _, nt, nl = dec.get_lattice(b, rows[b], args.lattice_beam, on_device=True)
        sizes.append((nt, nl))
    torch.cuda.synchronize()
    ntok, nlink = sum(s[0] for s in sizes), sum(s[1] for s in sizes)
    t0 = time.perf_counter()
    for _ in range(args.steps):
        for b in range(B):
            dec.get_lattice(b, rows[b], args.lattice_beam, tok_cap=sizes[b][0], link_cap=sizes[b][1], on_device=True)
    torch.cuda.synchronize()
    dt_one = (time.perf_counter() - t0) / args.steps
    # all utterances in one call (wfst_get_lattice_batch): the step that is reported
    chans = np.arange(B, dtype=np.int32)
    out = dec.get_lattice_batch(chans, ll, w.lengths, args.lattice_beam, tok_cap=ntok, link_cap=nlink, on_device=True)
    assert int(out[1][B]) == ntok and int(out[2][B]) == nlink
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        dec.get_lattice_batch(chans, ll, w.lengths, args.lattice_beam, tok_cap=ntok, link_cap=nlink, on_device=True)
    torch.cuda.synchronize()
    dt = (time.perf_counter() - t0) / args.steps
    arcs = int(counters[1] + counters[2])
    frames = int(w.lengths.sum())
    # bytes the method has to move: per frame a log-likelihood row; per token its record when its
    # set is put into the lookup table and again (with the 16-byte header of its state) when its
    # arcs are expanded, state and cost written out; per arc its 16-byte record; per link 32 bytes
    abytes = frames * V * 4 + ntok * (8 + 8 + 16 + 8) + arcs * 16 + nlink * 32
    achieved = abytes / dt / 1e9
    line = {"metric": "lattice links found per second (wfst_get_lattice_batch, outputs on device)", "value": nlink / dt,
            "unit": "links/s", "n_gpus": 1, "steps": args.steps, "warmup": 1, "ms_per_step": 1e3 * dt,
            "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
            "config": {"workload": args.workload, "utterances": B, "frames": frames, "lattice_beam": args.lattice_beam,
                       "tokens": ntok, "links": nlink, "arcs_expanded": arcs, "beam": w.beam, "max_active": w.max_active},
            "ms_per_utterance": 1e3 * dt / B, "audio_s_per_s": w.audio_seconds / dt,
            "one_call_per_utterance": {"ms_per_step": 1e3 * dt_one, "value": nlink / dt_one},
            "timing": "wall clock around the calls (a call launches wfst_lattice_kernel twice and waits for it)",
            "roofline": {"bound": "hbm", "kernel": "wfst_lattice_kernel", "achieved": achieved, "peak": HBM_PEAK_GBS,
                         "unit": "GB/s", "frac": achieved / HBM_PEAK_GBS, "traffic": None,
                         "algorithmic_bytes_per_step": abytes}}
    dec.close()
    print(json.dumps(line), flush=True)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--channels", type=int, default=512, help="streaming mode: concurrent channels")
    ap.add_argument("--separate-partials", action="store_true",
                    help="streaming mode: wfst_advance_chunk and wfst_get_partial_batch as two calls per chunk")
    ap.add_argument("--chunks", type=int, default=50, help="streaming mode: timed chunks")
    ap.add_argument("--recycle-window", type=int, default=0,
                    help="streaming mode: recycle every channel's lattice memory as a ring over this many frames")
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=1)
    ap.add_argument("--workload", default="c3_large")
    ap.add_argument("--batch", type=int, default=None)
    ap.add_argument("--max-active", type=int, default=None, help="override the workload's max-active (a sensitivity run, "
                    "not the configuration the metric is quoted on)")
    ap.add_argument("--beam", type=float, default=None, help="override the workload's beam (likewise)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-traffic", action="store_true",
                    help="do not measure the kernel's HBM traffic with two profiler runs of this script (the figure "
                         "of the committed profile summary is reported instead)")
    ap.add_argument("--calibrate-copy", action="store_true", help="also run one 1 GiB device copy (profiling aid)")
    ap.add_argument("--calibrate", action="store_true",
                    help="only measure this GPU's ceilings (device copy, random 128-byte lines, 64-bit atomics) and "
                         "print them as one JSON line")
    ap.add_argument("--loglike-dtype", default="float32", choices=["float32", "float16", "bfloat16"],
                    help="element type of the log-likelihoods handed to the decoder (costs stay fp32)")
    ap.add_argument("--narrow-arcs", action="store_true",
                    help="8-byte emitting-arc records with binary16 weights (the graph's emitting weights are rounded)")
    ap.add_argument("--lattice-beam", type=float, default=None,
                    help="lattice mode: decode --batch utterances (default 8) with token records kept and time "
                         "wfst_get_lattice with this lattice beam for each of them")
    ap.add_argument("--pipeline", type=int, default=3,
                    help="batch slots of the one decoder (each with its own stream) that take the steps in turn, so "
                         "that the next batch fills the compute units the previous one no longer uses")
    ap.add_argument("--stream-workgroups", type=int, default=256,
                    help="streaming mode: workgroups per launch, which take the channels from a counter on the device "
                         "(one per compute unit; 0: one per channel)")
    ap.add_argument("--launch-workgroups", type=int, default=-1,
                    help="with several batches in flight: workgroups per launch, which take the batch's utterances "
                         "longest first from a counter on the device (wfst_set_launch_workgroups); 0: one per utterance; "
                         "-1: half of the GPU's compute units (two launches hold the chip between them)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build measures one GPU only (utterances are independent; more GPUs "
              "would each take a share of the batch with a replicated graph); run with --gpus 1",
              file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2311_04996_amd import Decoder
    from workloads import make_config
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    if args.calibrate:
        print(json.dumps({"metric": "measured ceilings of this GPU", **calibrate()}), flush=True)
        return
    if args.workload == "c4_streaming":
        return main_streaming(args)
    if args.lattice_beam is not None:
        return main_lattice(args)

    t0 = time.perf_counter()
    w = make_config(args.workload, batch=args.batch)
    if args.max_active is not None:
        w.max_active = int(args.max_active)
    if args.beam is not None:
        w.beam = float(args.beam)
    B, T, V = w.loglikes.shape
    print(f"[bench] {args.workload}: S={w.graph.num_states} A={w.graph.num_arcs} B={B} T={T} V={V} "
          f"audio={w.audio_seconds:.1f}s generated in {time.perf_counter() - t0:.1f}s", file=sys.stderr, flush=True)
    t0 = time.perf_counter()
    # ONE decoder: the batches in flight are its batch slots (shared graph), and a slot's lattice
    # memory is shared out by utterance length, so it is sized for the batch's mean length
    n_slots = max(1, args.pipeline)
    if args.launch_workgroups < 0:
        args.launch_workgroups = torch.cuda.get_device_properties(0).multi_processor_count // 2 // 32 * 32
    mean_frames = float(w.lengths.mean())
    dec = Decoder(w.graph, max_channels=B * n_slots, max_frames=T, max_words=512, max_active_hint=w.max_active,
                  loglike_dtype=args.loglike_dtype, batch_slots=n_slots, lattice_by_length=True,
                  narrow_arcs=args.narrow_arcs,
                  lattice_bytes_per_channel=int(8 * 1.5 * w.max_active * (mean_frames + 2)))
    streams = pick_concurrent_streams(torch, n_slots)
    ll = torch.from_numpy(w.loglikes).cuda().to(getattr(torch, args.loglike_dtype))
    outs = [None] * n_slots
    # the results of every step are copied to (pinned) host memory on the step's own stream, inside the timed region
    host = [[torch.empty((B, 512), dtype=torch.int32, pin_memory=True), torch.empty(B, dtype=torch.int32, pin_memory=True),
             torch.empty(B, dtype=torch.float32, pin_memory=True), torch.empty(B, dtype=torch.int32, pin_memory=True)]
            for _ in range(n_slots)]
    torch.cuda.synchronize()
    print(f"[bench] decoder ready in {time.perf_counter() - t0:.1f}s, {dec.device_bytes() / 2**30:.1f} GiB on device",
          file=sys.stderr, flush=True)

    def run_steps(n_use, nsteps, record_ms):
        """nsteps decode_batch calls taken in turn by the first n_use batch slots (each on its own
        stream); returns the wall time between two device synchronisations."""
        ms = []
        # one batch in flight: a workgroup per utterance, the whole chip for the one launch; several: each
        # launch gets a share of the compute units and its workgroups take the utterances from a queue
        dec.set_launch_workgroups(args.launch_workgroups if n_use > 1 else 0)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(nsteps):
            k = i % n_use
            if n_use > 1 and nsteps % 2 == 1 and i == nsteps - 1:
                dec.set_launch_workgroups(0)          # two launches of 128 workgroups share the chip; an odd last one has it alone
            outs[k] = dec.decode_batch(ll, w.lengths, w.beam, w.max_active, stream=streams[k], out=outs[k],
                                       boosts=w.boosts, boost_fsts=w.boost_fsts, slot=k)
            with torch.cuda.stream(streams[k]):
                for h, o in zip(host[k], outs[k]):
                    h.copy_(o, non_blocking=True)
            if record_ms:
                ms.append(dec.slot_kernel_ms(k))      # HIP events on the launch stream; waits for the kernel
        torch.cuda.synchronize()
        return time.perf_counter() - t0, ms

    for k in range(n_slots):                         # warmup: every slot, every buffer touched
        for _ in range(max(1, args.warmup) if args.warmup else 0):
            outs[k] = dec.decode_batch(ll, w.lengths, w.beam, w.max_active, stream=streams[k], out=outs[k],
                                       boosts=w.boosts, boost_fsts=w.boost_fsts, slot=k)
    torch.cuda.synchronize()
    dec.get_counters(reset=True)
    # one batch in flight: the kernel's own duration (for the roofline) and the unpipelined rate
    wall_one, kernel_ms = run_steps(1, args.steps, True)
    counters = dec.get_counters() // max(1, args.steps)
    # the timed region proper: `pipeline` batches in flight
    wall = run_steps(n_slots, args.steps, False)[0] if n_slots > 1 else wall_one
    # the launches of the timed region itself, by the same HIP events: the last launch of every slot (two of
    # them hold the chip at a time; a third has been waiting in its queue for compute units, which counts)
    kms_at_value = [float(dec.slot_kernel_ms(k)) for k in range(min(n_slots, args.steps))] if n_slots > 1 else None
    # where the workgroups spend their time: one more launch, untimed, with the phase clocks on
    # (they are off in the timed regions: reading the clock at every phase boundary costs about 1 %)
    dec.debug_phase_ticks(reset=True)
    dec.debug_set_phase_timing(True)
    run_steps(1, 1, False)
    dec.debug_set_phase_timing(False)
    ticks = dec.debug_phase_ticks()
    ticks[15] = 0                                   # slot 15 is a count, not a time
    names = ["expand_tail", "select", "tokens", "eps_expand", "eps_round_end", "publish", "trace", "other",
             "tab_clear", "tab_fill", "tab_winners", "eps_table", "eps_new_tokens", "expand_arcs", "eps_meet", "-"]
    print("[bench] phase share of workgroup time (one batch in flight): " +
          ", ".join(f"{n} {100.0 * t / max(1, ticks.sum()):.1f}%" for n, t in zip(names, ticks) if t) +
          f"; mean busy time per workgroup {ticks.sum() / 1e5 / B:.1f} ms",
          file=sys.stderr, flush=True)
    for o in outs:
        if o is not None:
            assert not (o[3].cpu().numpy() & (8 | 16)).any(), "an utterance overflowed a buffer: the run is invalid"
    if args.calibrate_copy:
        # a plain copy of known size in the same process, to scale the profiler's byte counters
        src = torch.empty(1 << 28, dtype=torch.float32, device="cuda").fill_(1.0)
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        dst.copy_(src)
        torch.cuda.synchronize()
        print(f"[bench] calibration copy: {src.numel() * 4} bytes read and written", file=sys.stderr, flush=True)

    ms_per_step = 1e3 * wall / args.steps
    rtfx = w.audio_seconds / (wall / args.steps)
    arcs = int(counters[1] + counters[2])
    kms = float(np.mean(kernel_ms))
    abytes = algorithmic_bytes(counters, V)
    achieved = abytes / (kms * 1e-3) / 1e9
    traffic, traffic_source, traffic_detail = None, None, None
    if not args.no_traffic:
        child = ["--workload", args.workload, "--loglike-dtype", args.loglike_dtype]
        child += ["--batch", str(args.batch)] if args.batch else []
        child += ["--narrow-arcs"] if args.narrow_arcs else []
        child += ["--max-active", str(args.max_active)] if args.max_active is not None else []
        child += ["--beam", str(args.beam)] if args.beam is not None else []
        t0 = time.perf_counter()
        traffic, traffic_detail = measure_traffic(child)
        if traffic is not None:
            traffic_source = ("measured by this run: two child runs of this command with one batch in flight under rocprofv3 "
                              "--pmc FETCH_SIZE / WRITE_SIZE, scaled by the same counters of the 1 GiB probe_copy launches")
            print(f"[bench] HBM traffic per launch measured in {time.perf_counter() - t0:.0f} s: {traffic / 1e9:.1f} GB",
                  file=sys.stderr, flush=True)
        else:
            print(f"[bench] HBM traffic not measured ({traffic_detail}); using the committed profile summary",
                  file=sys.stderr, flush=True)
    if traffic is None:
        why = "" if args.no_traffic else f"; a measurement was tried and failed: {traffic_detail}"
        traffic, traffic_detail = read_traffic(args.workload), None
        traffic_source = ("rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs of this command, summary under profiles/ "
                          "(not measured in this run" + why + ")")
    cal = calibrate()
    achieved_at_value = abytes / (ms_per_step * 1e-3) / 1e9
    line = {
        "metric": f"RTFx (audio-s decoded/s) at batch {B}", "value": rtfx, "unit": "audio-s/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f32",
        "data": "synthetic",
        "config": {"workload": args.workload, "batch": B, "frames": int(w.lengths.sum()),
                   "states": w.graph.num_states, "arcs": w.graph.num_arcs, "classes": V,
                   "beam": w.beam, "max_active": w.max_active, "batches_in_flight": n_slots,
                   "workgroups_per_launch": (min(B, args.launch_workgroups) if args.launch_workgroups > 0 and n_slots > 1 else B),
                   "loglike_dtype": args.loglike_dtype, "decoders": 1, "narrow_arcs": bool(args.narrow_arcs),
                   "device_gib": round(dec.device_bytes() / 2**30, 1)},
        "one_batch_in_flight": {"value": w.audio_seconds / (wall_one / args.steps),
                                "ms_per_step": 1e3 * wall_one / args.steps},
        "arcs_expanded_per_s": arcs / (wall / args.steps),
        "arcs_expanded_per_step": arcs,
        "tokens_per_frame": float(counters[4]) / max(1, int(counters[7])),
        "hbm_frac_of_peak": achieved / HBM_PEAK_GBS,
        "timed_region": "K decode_batch calls (init, all frames, final choice, traceback) plus the copy of their "
                        "results to pinned host memory, between two device synchronisations; log-likelihoods resident",
        "roofline": {"bound": "hbm", "kernel": KERNEL, "achieved": achieved, "peak": HBM_PEAK_GBS,
                     "unit": "GB/s", "frac": achieved / HBM_PEAK_GBS, "traffic": traffic,
                     "traffic_source": traffic_source, "traffic_detail": traffic_detail,
                     "algorithmic_bytes_per_launch": abytes, "kernel_ms": kms,
                     "kernel_ms_of_last_launches_at_value": kms_at_value,
                     "note": "achieved / frac: algorithmic bytes over the kernel's own duration with ONE batch in flight "
                             "(HIP events on the launch stream); *_at_value: over ms_per_step of the timed region, "
                             f"{n_slots} batches in flight",
                     "achieved_at_value": achieved_at_value, "frac_at_value": achieved_at_value / HBM_PEAK_GBS,
                     "peak_measured_copy": cal["copy_gb_per_s"], "frac_of_measured_copy": achieved / cal["copy_gb_per_s"],
                     "frac_of_measured_copy_at_value": achieved_at_value / cal["copy_gb_per_s"],
                     "measured_random_128B_lines_per_s": cal["random_128B_lines_per_s"],
                     "measured_random_64bit_atomics_per_s": cal["random_64bit_atomics_per_s"],
                     "measured_how": cal["how"]},
    }
    if not args.no_cpu_baseline:
        threads = min(16, os.cpu_count() or 1)
        line["cpu_baseline"] = cpu_baseline(w, threads)
    dec.close()
    print(json.dumps(line), flush=True)


if __name__ == "__main__":
    main()
