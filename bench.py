#!/usr/bin/env python3
"""Throughput of the whole JPEG -> normalized tensor path on one MI355X.

One step = the whole path over one batch of a synthetic workload (default: workload 2, 256
images of 300..640 x 250..500 pixels, 4:2:0, quality 90, restart interval 8 MCUs): host
marker parsing, restart-marker scan, entropy decode, RGB reconstruction and
resize/crop/normalize.  Two legs are timed, K steps each: `value` is the leg whose
bitstreams already lie in HBM when the timed region starts (prep_decode_resize_batch_resident),
and the object "host_input" is the leg that starts from pageable host memory
(prep_decode_resize_batch: the copy into pinned memory and the upload are inside its timed
region).  Prints ONE JSON line with images/s, the roofline of the dominant kernel, the other
stages, the host's share of a call, and the CPU oracle (all host threads, and one) and a
third-party CPU library timed on the host cores of the same machine.
"""
import argparse
import json
import os
import sys
import time
from concurrent.futures import ThreadPoolExecutor

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

METRIC = "images/sec JPEG→224² normalized tensor on 1 MI355X; % HBM/VALU roofline"

# chip figures used for the rooflines
HBM_PEAK_GBS = 8000.0
# plain 32-bit integer vector ALU: 256 CUs x 4 SIMDs x 16 lanes x 2.4 GHz
INT_ALU_PEAK_TOPS = 256 * 4 * 16 * 2.4e9 / 1e12
# essential integer operations of decoding one Huffman symbol by the serial definition
# (peek, table lookup, split length/symbol, two buffer shifts, position update, receive
#  bits, two for sign extension, run/zig-zag update, end-of-block test, address, store,
#  refill share)
OPS_PER_SYMBOL = 16

WORKLOAD_NAMES = {
    1: "workload 1: 64 x 256x256 4:2:0 q85, restart per MCU row, crop 224 fp32",
    2: "workload 2: 256 x U[300,640]xU[250,500] 4:2:0 q90, restart interval 8 MCUs, resize 256 crop 224 fp16",
    4: "workload 4: 64 x 1920x1080 4:2:0 q95, restart per MCU row, resize 384 crop 384 fp16",
    5: "workload 5: 512 x 256x256 mixed 4:4:4/4:2:0/gray q50-95, no restart markers, crop 224 fp16",
    3: "workload 3: 7 concurrent streams x batches of 8 from 512 x 256x256 4:2:0 q85, restart per MCU row, crop 224 fp32",
}
N_STREAMS, STREAM_BATCH = 7, 8

# HBM bytes per launch from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE (profiles/all_kernels_workload*_hbm_counters.txt),
# scaled by what the same counters read for a plain 256 MiB copy (FETCH_SIZE x 2, WRITE_SIZE x 1).
# They describe the kernels whose sources hash to MEASURED_SOURCES; for any other sources the
# figure is reported as null.
MEASURED_SOURCES = "e3a24c510a1c23b19a27fbc5bd7d4b7cac41e11943365f9eb83ac318856e23a1"
MEASURED_TRAFFIC = {
    2: {"scan": (5419 * 2 + 1265) * 1024, "decode": (7719 * 2 + 289799) * 1024,
        "reconstruct": (50640 * 2 + 104417) * 1024, "resize": (49121 * 2 + 75264) * 1024},
    4: {"scan": (23814 * 2 + 575) * 1024, "decode": (28211 * 2 + 620821) * 1024,
        "reconstruct": (114438 * 2 + 241160) * 1024, "resize": (91697 * 2 + 55296) * 1024},
}


def sources_hash():
    import glob
    import hashlib
    h = hashlib.sha256()
    for f in sorted(glob.glob(os.path.join(ROOT, "paper_2411_19114_amd", "csrc", "*"))):
        # the image path's sources (the audio path and the batching server have no part in it)
        if f.endswith((".hip", ".cpp", ".h")) and os.path.basename(f) not in ("audio.hip", "batcher.cpp"):
            h.update(os.path.basename(f).encode())
            with open(f, "rb") as fh:
                h.update(fh.read())
    return h.hexdigest()


def measured_traffic(workload, stage):
    if workload not in MEASURED_TRAFFIC or sources_hash() != MEASURED_SOURCES:
        return None
    return MEASURED_TRAFFIC[workload].get(stage)


def cpu_baseline(streams, pr, max_seconds=60.0):
    """The oracle as it stands, on the host cores, over a bounded sample of the batch."""
    import oracle
    cores = min(16, len(os.sched_getaffinity(0)) if hasattr(os, "sched_getaffinity") else os.cpu_count())

    def one(s):
        oracle.decode_preprocess(s, pr["resize_short"], pr["crop_h"], pr["crop_w"], pr["mean"], pr["std"],
                                 bool(pr.get("antialias")))
        return oracle.jpeg_info(s)

    # probe one image to bound the sample to roughly 20 s of CPU work
    t0 = time.perf_counter()
    one(streams[0])
    per = time.perf_counter() - t0
    want = int(max(cores, 20.0 / max(per, 1e-4)))
    if want <= len(streams):
        sample, what = streams[:want], f"first {want} images of the batch"
    else:
        passes = min(-(-want // len(streams)), 64)
        sample, what = streams * passes, f"the batch of {len(streams)} images {passes} times over"
    n = len(sample)
    t0 = time.perf_counter()
    with ThreadPoolExecutor(cores) as ex:
        list(ex.map(one, sample))
    dt = time.perf_counter() - t0
    out = {"value": n / dt, "unit": "images/s", "cores": cores, "kind": "oracle",
           "sample": f"{what}, one image per task, {cores} threads, {dt:.2f} s wall"}
    # the same oracle on one thread, over about 5 s of work
    k = max(1, min(len(streams), int(5.0 / max(per, 1e-4))))
    t0 = time.perf_counter()
    for s_ in streams[:k]:
        one(s_)
    dt1 = time.perf_counter() - t0
    out["one_thread"] = {"value": k / dt1, "unit": "images/s", "cores": 1,
                         "sample": f"first {k} images of the batch, {dt1:.2f} s wall"}
    out["library_context"] = library_context(streams, pr, cores)
    return out


def library_context(streams, pr, cores, seconds=4.0):
    """A tuned third-party CPU library on the same inputs, as context only (it is not the
    oracle and takes no part in any parity check): Pillow decodes (libjpeg-turbo, its own
    upsampling and integer IDCT) and resizes, numpy crops and normalizes."""
    try:
        from PIL import Image
        import io
    except ImportError:
        return None
    mean = np.asarray(pr["mean"], dtype=np.float32).reshape(3, 1, 1)
    std = np.asarray(pr["std"], dtype=np.float32).reshape(3, 1, 1)

    def one(s):
        im = Image.open(io.BytesIO(s)).convert("RGB")
        w, h = im.size
        rs = pr["resize_short"]
        if rs:
            ow, oh = (rs, rs * h // w) if w <= h else (rs * w // h, rs)
            im = im.resize((ow, oh), Image.BILINEAR)
        else:
            ow, oh = w, h
        top, left = (oh - pr["crop_h"]) // 2, (ow - pr["crop_w"]) // 2
        a = np.asarray(im)[top:top + pr["crop_h"], left:left + pr["crop_w"]].transpose(2, 0, 1)
        return ((a.astype(np.float32) / 255.0 - mean) / std).astype(np.float16 if pr["out_dtype"] == "f16" else np.float32)

    t0 = time.perf_counter()
    one(streams[0])
    per = time.perf_counter() - t0
    n = int(max(cores, min(len(streams) * 8, seconds * cores / max(per, 1e-5))))
    sample = [streams[i % len(streams)] for i in range(n)]
    t0 = time.perf_counter()
    with ThreadPoolExecutor(cores) as ex:
        list(ex.map(one, sample))
    dt = time.perf_counter() - t0
    return {"value": n / dt, "unit": "images/s", "cores": cores,
            "kind": "third-party library, context only: Pillow (libjpeg-turbo) decode + its antialiased "
                    "bilinear resize + numpy crop/normalize; not the oracle, no part in parity",
            "sample": f"{n} images drawn in turn from the batch, one per task, {cores} threads, {dt:.2f} s wall"}


def symbols_in(streams, limit=64):
    """Coded symbols per compressed byte, from the oracle's decode statistics on a sample
    (part of the cpu_baseline leg); used to scale the entropy decoder's algorithmic work."""
    import oracle
    sym = byt = 0
    for s in streams[:limit]:
        _, _, info = oracle.decode(s, want_coef=True, want_rgb=False)
        sym += info.symbols
        byt += info.entropy_bytes
    return sym / max(byt, 1)


def algorithmic_bytes(infos, pr):
    """Bytes each HBM-bound stage has to move for these images: what the stage reads and
    writes by its definition, each byte once."""
    esz = 2 if pr["out_dtype"] == "f16" else 4
    n = len(infos)
    out_bytes = n * 3 * pr["crop_h"] * pr["crop_w"] * esz
    entropy_bytes = sum(i.entropy_bytes for i in infos)
    blocks = sum(i.mcu_cols * i.mcu_rows * i.blocks_per_mcu for i in infos)
    # source footprint of the crop: the window of each image that the outputs map back to;
    # reconstruction owes the MCUs that hold the pixels its bilinear taps read
    foot = 0
    recon = 0
    for i in infos:
        s = pr["resize_short"]
        if s:
            ow, oh = (s, s * i.height // i.width) if i.width <= i.height else (s * i.width // i.height, s)
        else:
            ow, oh = i.width, i.height
        foot += int(round(pr["crop_w"] * i.width / ow)) * int(round(pr["crop_h"] * i.height / oh)) * 3
        mcu_px = 16 if i.sampling == 1 else 8
        mcus = 1
        for size, out_size, count in ((i.width, ow, pr["crop_w"]), (i.height, oh, pr["crop_h"])):
            first = (out_size - count) // 2
            # taps floor(s), floor(s) + 1 of the first and last output; 2 s out_size is an integer
            s2_first = (2 * first + 1) * size - out_size
            s2_last = (2 * (first + count - 1) + 1) * size - out_size
            if pr.get("antialias") and size > out_size:
                # the samples strictly inside the first and last output's triangle, half-width
                # size / out_size around the centre s + 1/2: j > s - size/out_size, j < s + size/out_size
                lo = (s2_first - 2 * size) // (2 * out_size) + 1
                hi = -((-(s2_last + 2 * size)) // (2 * out_size)) - 1
            else:
                lo = s2_first // (2 * out_size)
                hi = s2_last // (2 * out_size) + (1 if s2_last % (2 * out_size) else 0)
            lo, hi = min(max(lo, 0), size - 1), min(max(hi, 0), size - 1)
            mcus *= hi // mcu_px - lo // mcu_px + 1
        recon += mcus * (i.blocks_per_mcu * 128 + mcu_px * mcu_px * 3)
    return {
        "scan": entropy_bytes,                          # read the stream once
        "reconstruct": recon,                           # coefficients in, RGB out, MCUs under the crop
        "resize": foot + out_bytes,                     # crop footprint in, tensor out
    }, entropy_bytes


def stage_report(stage_ms, work, entropy_bytes, sym_per_byte, workload=None):
    names = ["scan", "decode", "reconstruct", "resize"]
    kernels = ["scan_restart_markers (+ expanding the Huffman tables)", "decode_entropy", "reconstruct_rgb",
               "resize_crop_normalize"]
    stages = []
    for j, name in enumerate(names):
        ms = float(stage_ms[j])
        if name == "decode":
            if sym_per_byte is None:
                stages.append({"stage": name, "kernel": kernels[j], "ms": ms, "bound": "alu"})
                continue
            ops = sym_per_byte * entropy_bytes * OPS_PER_SYMBOL
            ach = ops / (ms * 1e-3) / 1e12
            stages.append({"stage": name, "kernel": kernels[j], "ms": ms, "bound": "alu",
                           "achieved": ach, "peak": INT_ALU_PEAK_TOPS, "unit": "TOP/s",
                           "frac": ach / INT_ALU_PEAK_TOPS, "traffic": measured_traffic(workload, name),
                           "symbols_per_launch": sym_per_byte * entropy_bytes,
                           "compressed_GB_per_s": entropy_bytes / (ms * 1e-3) / 1e9})
        else:
            b = work[name]
            ach = b / (ms * 1e-3) / 1e9
            stages.append({"stage": name, "kernel": kernels[j], "ms": ms, "bound": "hbm",
                           "achieved": ach, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                           "frac": ach / HBM_PEAK_GBS, "traffic": measured_traffic(workload, name),
                           "algorithmic_bytes": b})
    dominant = max(stages, key=lambda s: s["ms"])
    roofline = {k: dominant.get(k) for k in ("bound", "achieved", "peak", "unit", "frac", "traffic")}
    roofline["kernel"] = dominant["kernel"]
    roofline["avg_launch_ms"] = dominant["ms"]
    return stages, roofline


def run_streams(args, torch, prep, synth, make_params):
    """Workload 3: N_STREAMS host threads, each with its own handle and HIP stream, decode
    batches of STREAM_BATCH images back to back; one step = one batch on every stream.
    Reports whole-job images/s and the distribution of per-batch latency (submit -> done)."""
    import threading
    N_STREAMS = args.streams or globals()["N_STREAMS"]
    STREAM_BATCH = args.stream_batch
    t0 = time.perf_counter()
    streams = synth.make_batch(3)
    gen_s = time.perf_counter() - t0
    blob, offsets = synth.pack(streams)
    pr = synth.params_of(3)
    params = make_params(pr["resize_short"], pr["crop_h"], pr["crop_w"], pr["out_dtype"], pr["mean"], pr["std"])
    infos = prep.parse_headers(blob, offsets)
    assert all(i.status == 0 for i in infos)
    n_batches = len(streams) // STREAM_BATCH
    dev = torch.device("cuda:0")
    dev_bits = torch.from_numpy(blob).to(dev)
    dt = torch.float16 if pr["out_dtype"] == "f16" else torch.float32
    max_w, max_h = max(i.width for i in infos), max(i.height for i in infos)
    max_bytes = max(int(offsets[(b + 1) * STREAM_BATCH] - offsets[b * STREAM_BATCH]) for b in range(n_batches))
    pps, outs, hip_streams = [], [], []
    for _ in range(N_STREAMS):
        pps.append(prep.Preprocessor(device=0, max_batch=STREAM_BATCH, max_width=max_w, max_height=max_h,
                                     max_bitstream_bytes=max_bytes))
        outs.append(torch.empty((STREAM_BATCH, 3, pr["crop_h"], pr["crop_w"]), dtype=dt, device=dev))
        hip_streams.append(torch.cuda.Stream(device=dev))
    torch.cuda.synchronize()
    lat = [[] for _ in range(N_STREAMS)]
    span = [None] * N_STREAMS
    gate = threading.Barrier(N_STREAMS)
    errors = []
    # Open-loop mode: requests (one batch each) arrive as a Poisson process of the given rate,
    # as in the paper's methodology (section 5, input query modeling), and wait in one queue
    # for the next free stream; latency then counts from the arrival, queueing included.
    rate = args.poisson_rate
    n_requests = N_STREAMS * args.steps
    if rate:
        sys.setswitchinterval(1e-4)
        gaps = np.random.default_rng(3000).exponential(1.0 / rate, size=n_requests)
        arrivals = np.cumsum(gaps)
        taken = [0]
        take_lock = threading.Lock()
        epoch = [None]

    def worker(i):
        try:
            pp, out, hs = pps[i], outs[i], hip_streams[i]
            b = i
            for k in range(args.warmup + (0 if rate else args.steps)):
                if k == args.warmup:
                    if i == 0:
                        pp.set_timing(True)
                    gate.wait()
                    span[i] = [time.perf_counter(), None]
                o = offsets[b * STREAM_BATCH:(b + 1) * STREAM_BATCH + 1]
                t = time.perf_counter()
                pp.decode_resize_batch_resident(blob, dev_bits.data_ptr(), o, params, out.data_ptr(), hs.cuda_stream)
                hs.synchronize()
                if k >= args.warmup:
                    lat[i].append(time.perf_counter() - t)
                b = (b + N_STREAMS) % n_batches
            if rate:
                if i == 0:
                    pp.set_timing(True)
                gate.wait()
                if i == 0:
                    epoch[0] = time.perf_counter() + 0.001
                gate.wait()
                span[i] = [epoch[0], None]
                while True:
                    with take_lock:
                        r = taken[0]
                        taken[0] += 1
                    if r >= n_requests:
                        break
                    due = epoch[0] + arrivals[r]
                    wait = due - time.perf_counter()
                    if wait > 3e-4:
                        time.sleep(wait - 2e-4)  # gives the interpreter to the other threads
                    while time.perf_counter() < due:
                        pass
                    b = r % n_batches
                    o = offsets[b * STREAM_BATCH:(b + 1) * STREAM_BATCH + 1]
                    pp.decode_resize_batch_resident(blob, dev_bits.data_ptr(), o, params, out.data_ptr(), hs.cuda_stream)
                    hs.synchronize()
                    lat[i].append(time.perf_counter() - due)
            span[i][1] = time.perf_counter()
            assert pp.get_status(STREAM_BATCH) == [0] * STREAM_BATCH
        except Exception as e:  # surfaced by the main thread
            errors.append(repr(e))
            try:
                gate.abort()
            except Exception:
                pass

    threads = [threading.Thread(target=worker, args=(i,)) for i in range(N_STREAMS)]
    for t in threads:
        t.start()
    for t in threads:
        t.join()
    if errors:
        print("bench.py: " + "; ".join(errors), file=sys.stderr)
        sys.exit(1)
    wall = max(s[1] for s in span) - min(s[0] for s in span)
    images = N_STREAMS * args.steps * STREAM_BATCH
    all_lat = np.sort(np.concatenate([np.array(l) for l in lat])) * 1e3
    k = max(1, min(len(lat[0]), 256))
    stage = np.array([pps[0].stage_ms(i) for i in range(k)]).mean(axis=0)
    pps[0].set_timing(False)
    work, entropy_bytes = algorithmic_bytes(infos[:STREAM_BATCH], pr)
    cpu = sym_per_byte = None
    if not args.no_cpu_baseline:
        cpu = cpu_baseline(streams, pr)
        sym_per_byte = symbols_in(streams)
    stages, roofline = stage_report(stage, work, entropy_bytes, sym_per_byte)
    result = {
        "metric": METRIC, "value": images / wall, "unit": "images/s", "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "ms_per_step": wall / args.steps * 1e3,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "int32 entropy decode, f64 IDCT, f32 resize -> " + pr["out_dtype"] + " output",
        "data": "synthetic",
        "config": {"workload": WORKLOAD_NAMES[3], "streams": N_STREAMS, "batch": STREAM_BATCH,
                   "hw_queues": int(os.environ["GPU_MAX_HW_QUEUES"]), "poisson_rate": rate or None,
                   "input": "resident in HBM", "pool_images": len(streams),
                   "sha256": synth.sha256_of(streams), "input_generation_s": round(gen_s, 2)},
        "latency_ms": {"p50": float(np.percentile(all_lat, 50)), "p95": float(np.percentile(all_lat, 95)),
                       "p99": float(np.percentile(all_lat, 99)), "max": float(all_lat[-1]),
                       "what": (f"one batch of {STREAM_BATCH}: arrival (Poisson, {rate:g} batches/s, one queue) "
                                "until its stream is idle" if rate else
                                f"one batch of {STREAM_BATCH}: call of the entry point until its stream is idle"),
                       "samples": int(all_lat.size)},
        "roofline": roofline,
        "stages": stages,
        "stage_timing": f"stream 0 only, one batch of {STREAM_BATCH} images per launch",
        "gpu_ms_per_step": float(stage.sum()),
        "cpu_baseline": cpu,
    }
    print(json.dumps(result))
    for pp in pps:
        pp.close()


def run_server(args, torch, prep, synth, make_params):
    """Workload 3 through the batching server: single-image requests arrive as a Poisson
    process (the paper's query model, section 5), wait for Batch_max / Time_queue (section 4.3)
    and are served by --streams consumers.  Latency = arrival until the tensor is ready, on
    the library's clock."""
    import threading
    n_consumers = args.streams or N_STREAMS
    streams = synth.make_batch(3)
    pr = synth.params_of(3)
    params = make_params(pr["resize_short"], pr["crop_h"], pr["crop_w"], pr["out_dtype"], pr["mean"], pr["std"])
    blob, offsets = synth.pack(streams)
    infos = prep.parse_headers(blob, offsets)
    max_w, max_h = max(i.width for i in infos), max(i.height for i in infos)
    server = prep.Server(n_consumers=n_consumers, batch_max=args.batch_max, time_queue_us=args.time_queue_us,
                         params=params, max_width=max_w, max_height=max_h,
                         max_request_bytes=max(len(x) for x in streams), queue_capacity=8192)
    rate = args.poisson_rate or 10000.0
    n_req = n_consumers * args.steps * args.batch_max
    # warm-up: every consumer serves a few full batches (the first calls on a stream load code
    # and take milliseconds), all results are read, then the timed arrivals start
    n_warm = max(args.warmup, 4) * n_consumers * args.batch_max
    for k in range(n_warm):
        assert server.submit(streams[k % len(streams)], k) == 0
        if (k + 1) % (n_consumers * args.batch_max) == 0:
            time.sleep(0.03)
    for _ in range(n_warm):
        r = server.next(5000000)
        assert r is not None, "warm-up request lost"
        server.release(r)
    arrivals = np.cumsum(np.random.default_rng(3000).exponential(1.0 / rate, size=n_warm + n_req))
    arrivals[n_warm:] -= arrivals[n_warm]
    results = []
    refused = [0]

    def collect():
        from paper_2411_19114_amd.binding import ServerResult
        buf = (ServerResult * 256)()
        while len(results) + refused[0] < n_req:
            k = server.next_many(buf, 2000000)
            if k == 0:
                break
            for r in buf[:k]:
                results.append((r.tag, r.status, r.batch_size, r.arrival_ns, r.start_ns, r.done_ns))
            server.release_many(buf, k)

    col = threading.Thread(target=collect)
    col.start()
    sys.setswitchinterval(1e-4)
    t0 = time.perf_counter()
    for k in range(n_warm, n_warm + n_req):
        due = t0 + arrivals[k]
        wait = due - time.perf_counter()
        if wait > 3e-4:
            time.sleep(wait - 2e-4)
        while time.perf_counter() < due:
            pass
        if server.submit(streams[k % len(streams)], k) != 0:
            refused[0] += 1
    col.join()
    server.close()
    timed = [r for r in results if r[0] >= n_warm]
    assert timed and all(r[1] == 0 for r in timed), "a request failed"
    lat = np.sort(np.array([(r[5] - r[3]) * 1e-6 for r in timed]))
    wait_q = np.array([(r[4] - r[3]) * 1e-6 for r in timed])
    span = (max(r[5] for r in timed) - min(r[3] for r in timed)) * 1e-9
    batches = {}
    for r in timed:
        batches[(r[4], r[2])] = r[2]
    result = {
        "metric": METRIC, "value": len(timed) / span, "unit": "images/s", "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "ms_per_step": span / max(len(batches), 1) * 1e3,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "int32 entropy decode, f64 IDCT, f32 resize -> " + pr["out_dtype"] + " output",
        "data": "synthetic",
        "config": {"workload": WORKLOAD_NAMES[3] + ", one image per request through the batching server",
                   "consumers": n_consumers, "batch_max": args.batch_max, "time_queue_us": args.time_queue_us,
                   "poisson_rate": rate, "hw_queues": int(os.environ["GPU_MAX_HW_QUEUES"]),
                   "input": "host memory", "refused": refused[0]},
        "latency_ms": {"p50": float(np.percentile(lat, 50)), "p95": float(np.percentile(lat, 95)),
                       "p99": float(np.percentile(lat, 99)), "max": float(lat[-1]),
                       "what": "one request: submission until its tensor is ready", "samples": int(lat.size)},
        "batching": {"batches": len(batches), "mean_batch": float(np.mean(list(batches.values()))),
                     "mean_wait_ms": float(wait_q.mean()), "max_wait_ms": float(wait_q.max())},
        "roofline": None, "cpu_baseline": None,
    }
    print(json.dumps(result))


def audio_batch(n=64, rate=44100, seed=6000):
    """Seeded stand-in for a batch of speech utterances (the paper evaluates on LibriSpeech,
    section 5; its Fig. 13 shows lengths of a few to 35 s with most between 10 and 17 s):
    lengths from a clipped normal (12.3 s, 4 s), each a few drifting harmonics under a slow
    envelope plus low-pass noise, float32, peak 0.5."""
    rng = np.random.default_rng(seed)
    waves = []
    for k in range(n):
        sec = float(np.clip(rng.normal(12.3, 4.0), 1.5, 35.0))
        m = int(rate * sec)
        t = np.arange(m) / rate
        f0 = 110.0 + 60.0 * rng.random() + 20.0 * np.sin(2 * np.pi * (0.7 + rng.random()) * t)
        phase = 2 * np.pi * np.cumsum(f0) / rate
        x = np.zeros(m)
        for h in range(1, 16):
            x += rng.random() / (h ** 0.8) * np.sin(h * phase + rng.random() * 6.28)
        x *= 0.55 + 0.45 * np.sin(2 * np.pi * 3.1 * t + rng.random() * 6.28)
        x += 0.6 * np.convolve(rng.standard_normal(m + 15), np.hanning(16) / 8.0, mode="valid")
        waves.append((0.5 * x / np.abs(x).max()).astype(np.float32))
    return waves


def run_audio(args, torch, prep):
    """The audio path (resample 44.1 kHz -> 16 kHz, log-Mel spectrogram, normalize) on a batch
    of 64 synthetic utterances resident in HBM; one step = the whole batch."""
    rate_in = 44100
    t0 = time.perf_counter()
    waves = audio_batch(64, rate_in)
    gen_s = time.perf_counter() - t0
    offsets = np.zeros(len(waves) + 1, dtype=np.uint64)
    np.cumsum([len(w) for w in waves], out=offsets[1:])
    dev = torch.device("cuda:0")
    x = torch.from_numpy(np.concatenate(waves)).to(dev)
    ap = prep.AudioPreprocessor(max_batch=len(waves), max_total_samples=int(offsets[-1]))
    frames = [ap.frames(len(w), rate_in) for w in waves]
    out = torch.empty(80 * sum(frames), dtype=torch.float32, device=dev)
    stream = torch.cuda.Stream(device=dev)
    for _ in range(args.warmup):
        ap.features(x.data_ptr(), offsets, rate_in, out.data_ptr(), stream.cuda_stream)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        ap.features(x.data_ptr(), offsets, rate_in, out.data_ptr(), stream.cuda_stream)
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    seconds_of_audio = float(offsets[-1]) / rate_in
    # algorithmic work per step: double-precision operations of the definitions' fast forms
    n_frames = sum(frames)
    mid = sum(-(-len(w) * 160 // 441) for w in waves)
    flops = mid * 2 * 34 + n_frames * (9 * 256 * 10 + 512 + 257 * 3 + 2 * 514)
    traffic = int(offsets[-1]) * 4 + mid * 8 * 2 + n_frames * 80 * 4 * 3
    cpu = None
    if not args.no_cpu_baseline:
        from concurrent.futures import ThreadPoolExecutor
        from oracle import audio as oracle_audio
        cores = min(16, len(os.sched_getaffinity(0)))
        sample = sorted(waves, key=len)[:4]  # the shortest: the oracle's resampler is a Python loop
        t1 = time.perf_counter()
        with ThreadPoolExecutor(cores) as ex:
            list(ex.map(lambda w: oracle_audio.preprocess(w.astype(np.float64), rate_in), sample))
        dt = time.perf_counter() - t1
        cpu = {"value": len(sample) / dt, "unit": "utterances/s", "cores": cores, "kind": "oracle",
               "sample": f"the {len(sample)} shortest utterances of the batch "
                         f"({sum(len(w) for w in sample) / rate_in:.0f} s of audio), one per task, {cores} threads, "
                         f"{dt:.1f} s wall", "audio_seconds_per_s": sum(len(w) for w in sample) / rate_in / dt}
    ms = wall / args.steps * 1e3
    result = {
        "metric": "utterances/sec audio -> normalized log-Mel features on 1 MI355X", "value": len(waves) * args.steps / wall,
        "unit": "utterances/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f64 arithmetic, f32 in and out",
        "data": "synthetic",
        "config": {"workload": "audio: 64 utterances of 1.5-35 s (mean 12.3 s) at 44.1 kHz -> 16 kHz, 512-point "
                               "frames of 400 samples every 160, 80 Mel channels, per-feature normalisation",
                   "batch": len(waves), "audio_seconds": seconds_of_audio, "frames": n_frames,
                   "realtime_factor": seconds_of_audio * args.steps / wall, "input": "resident in HBM",
                   "input_generation_s": round(gen_s, 2)},
        "roofline": {"bound": "alu", "achieved": flops / (ms * 1e-3) / 1e12, "peak": 78.6, "unit": "TFLOP/s",
                     "frac": flops / (ms * 1e-3) / 1e12 / 78.6, "traffic": None,
                     "kernel": "whole step (resample_phase_kernel, log_mel_kernel, normalize_kernel)",
                     "algorithmic_bytes": traffic, "hbm_frac_by_algorithmic_bytes": traffic / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS},
        "cpu_baseline": cpu,
    }
    print(json.dumps(result))
    ap.close()


OVERLAP_STREAMS = 3   # handles and streams of the "overlapped" leg


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=None,
                    help="timed steps (default 50; workload 3: 2000 batches per stream, as the workload is stated)")
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--workload", type=int, default=2, choices=[1, 2, 3, 4, 5])
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--streams", type=int, default=None,
                    help="workloads 1, 2, 4, 5: deal the steps in turn to this many handles, each "
                         "with its own HIP stream, so that batches overlap on the GPU (default 1: "
                         "one batch at a time); workload 3: number of host threads (default 7)")
    ap.add_argument("--hw-queues", type=int, default=8,
                    help="workload 3: hardware queues the HIP runtime may use (GPU_MAX_HW_QUEUES; its "
                         "default of 4 makes seven streams share queues and wait for each other)")
    ap.add_argument("--poisson-rate", type=float, default=0.0,
                    help="workload 3: requests (batches) per second arriving as a Poisson process and "
                         "served by the next free stream; 0 = every stream runs back to back")
    ap.add_argument("--audio", action="store_true",
                    help="the audio path (resample, log-Mel spectrogram, normalize) instead of a JPEG workload")
    ap.add_argument("--server", action="store_true",
                    help="workload 3: single-image requests through the batching server (Batch_max, "
                         "Time_queue) with --streams consumers; needs --poisson-rate")
    ap.add_argument("--batch-max", type=int, default=8, help="--server: Batch_max")
    ap.add_argument("--time-queue-us", type=int, default=200, help="--server: Time_queue in microseconds")
    ap.add_argument("--stream-batch", type=int, default=STREAM_BATCH,
                    help="workload 3: images per batch (default 8; 1 = the single-input latency case)")
    ap.add_argument("--antialias", action="store_true",
                    help="resize with the antialiased filter (a variant; the default is the plain "
                         "two-tap bilinear filter of the workloads)")
    ap.add_argument("--copy-probe", action="store_true",
                    help="also run one plain 256 MiB device copy (a reference for HBM counters)")
    ap.add_argument("--host-input", action="store_true",
                    help="make `value` the leg that starts from host memory (prep_decode_resize_batch); "
                         "by default `value` is the HBM-resident leg and the host-memory leg is the "
                         "object \"host_input\" of the same line")
    ap.add_argument("--single-leg", action="store_true",
                    help="time only the leg that `value` reports (for profiler runs)")
    args = ap.parse_args()
    if args.steps is None:
        args.steps = 2000 if args.workload == 3 and not args.server and not args.audio else 50
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (images are independent; a second GPU "
              "would take a share of the batch with no exchange step); use --gpus 1",
              file=sys.stderr)
        sys.exit(2)

    if args.workload == 3:
        # read by the HIP runtime when it starts, so it is set before torch loads it
        os.environ["GPU_MAX_HW_QUEUES"] = str(min(max(args.hw_queues, 1), 32))
    import torch
    import paper_2411_19114_amd as prep
    import synth
    from paper_2411_19114_amd.binding import make_params

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(2)
    if not os.path.exists(prep.lib_path()):
        import __graft_entry__
        __graft_entry__.build()

    if args.audio:
        run_audio(args, torch, prep)
        return
    cfg = args.workload
    if cfg == 3:
        if args.server:
            run_server(args, torch, prep, synth, make_params)
        else:
            run_streams(args, torch, prep, synth, make_params)
        return
    t0 = time.perf_counter()
    streams = synth.make_batch(cfg)
    gen_s = time.perf_counter() - t0
    n = len(streams)
    blob, offsets = synth.pack(streams)
    pr = dict(synth.params_of(cfg), antialias=bool(args.antialias))
    params = make_params(pr["resize_short"], pr["crop_h"], pr["crop_w"], pr["out_dtype"], pr["mean"], pr["std"],
                         prep.FILTER_ANTIALIAS if args.antialias else prep.FILTER_BILINEAR)
    infos = prep.parse_headers(blob, offsets)
    assert all(i.status == 0 for i in infos)
    max_w, max_h = max(i.width for i in infos), max(i.height for i in infos)
    pixels = sum(i.width * i.height for i in infos)
    entropy_bytes = sum(i.entropy_bytes for i in infos)
    blocks = sum(i.mcu_cols * i.mcu_rows * i.blocks_per_mcu for i in infos)

    dev = torch.device("cuda:0")
    n_handles = max(1, args.streams or 1)
    # a further leg deals the steps to OVERLAP_STREAMS handles in turn, each with its own stream
    overlap = OVERLAP_STREAMS if n_handles == 1 and not args.single_leg else 0
    n_made = max(n_handles, overlap)
    pps = [prep.Preprocessor(device=0, max_batch=n, max_width=max_w, max_height=max_h,
                             max_bitstream_bytes=int(offsets[-1]), max_total_pixels=pixels)
           for _ in range(n_made)]
    pp = pps[0]
    dt = torch.float16 if pr["out_dtype"] == "f16" else torch.float32
    outs = [torch.empty((n, 3, pr["crop_h"], pr["crop_w"]), dtype=dt, device=dev) for _ in range(n_made)]
    dev_bits = torch.from_numpy(blob).to(dev)
    hip_streams = [torch.cuda.Stream(device=dev) for _ in range(n_made)]
    turn = [0]
    in_turn = [n_handles]   # handles that the steps are dealt to

    host_s = [0.0]   # time spent inside the entry point (host parse + enqueue), summed

    def step(host_input):
        i = turn[0] % in_turn[0]
        turn[0] += 1
        sp, out = hip_streams[i].cuda_stream, outs[i]
        t = time.perf_counter()
        if host_input:
            pps[i].decode_resize_batch(blob, offsets, params, out.data_ptr(), sp)
        else:
            pps[i].decode_resize_batch_resident(blob, dev_bits.data_ptr(), offsets, params, out.data_ptr(), sp)
        host_s[0] += time.perf_counter() - t

    if args.copy_probe:
        a = torch.empty(256 << 20, dtype=torch.uint8, device=dev)
        b = torch.empty_like(a)
        a.fill_(1)
        b.copy_(a)
        torch.cuda.synchronize()

    def leg(host_input):
        """W untimed steps, then exactly K timed ones between two device synchronisations."""
        for _ in range(args.warmup):
            step(host_input)
        torch.cuda.synchronize()
        for h in pps[:min(in_turn[0], max(args.warmup, 1))]:
            if args.warmup:
                assert h.get_status(n) == [0] * n, "a workload image failed to decode"
        pp.set_timing(True)
        torch.cuda.synchronize()
        host_s[0] = 0.0
        turn[0] = 0   # handle 0, whose stage times are read, takes the first step
        t0 = time.perf_counter()
        for _ in range(args.steps):
            step(host_input)
        torch.cuda.synchronize()
        wall = time.perf_counter() - t0
        k = min((args.steps + in_turn[0] - 1) // in_turn[0], 256)  # timed calls that handle 0 saw
        stage = np.array([pp.stage_ms(i) for i in range(k)]).mean(axis=0)  # ms: scan, decode, recon, resize
        pp.set_timing(False)
        return wall, stage, host_s[0] / args.steps

    # the leg that `value` reports (inputs resident in HBM unless --host-input), then the other
    first_is_host = bool(args.host_input)
    wall, stage, host_per_call = leg(first_is_host)
    other = None
    if not args.single_leg:
        o_wall, o_stage, o_host = leg(not first_is_host)
        other = {"input": "host memory (pageable), copy to pinned memory and upload inside the timed region"
                          if not first_is_host else "resident in HBM",
                 "entry_point": "prep_decode_resize_batch" if not first_is_host else "prep_decode_resize_batch_resident",
                 "value": n * args.steps / o_wall, "unit": "images/s", "steps": args.steps,
                 "ms_per_step": o_wall / args.steps * 1e3,
                 "stages_ms": [float(x) for x in o_stage], "gpu_ms_per_step": float(o_stage.sum()),
                 "host_ms_per_call": o_host * 1e3}

    ms_per_step = wall / args.steps * 1e3
    value = n * args.steps / wall

    # the same steps dealt in turn to several handles, each on a stream of its own: batches are
    # independent, so a server keeps several in flight and the GPU fills the gaps that one
    # batch's kernels leave (the slowest lane of the entropy decoder sets its kernel's time)
    overlapped = None
    if overlap:
        in_turn[0] = overlap
        o_wall, _, _ = leg(False)
        in_turn[0] = n_handles
        overlapped = {"streams": overlap, "input": "resident in HBM", "value": n * args.steps / o_wall,
                      "unit": "images/s", "steps": args.steps, "ms_per_step": o_wall / args.steps * 1e3}
        for h in pps[:overlap]:
            assert h.get_status(n) == [0] * n

    # S1 alone: the time inside the entry point (marker/table parsing, launch planning,
    # enqueueing) with the GPU idle, so that no wait for an earlier call is counted
    s1 = []
    for _ in range(10):
        host_s[0] = 0.0
        step(first_is_host)
        s1.append(host_s[0])
        torch.cuda.synchronize()
    s1_host = float(np.median(s1))

    # ---- algorithmic work per launch ------------------------------------------------------
    work, entropy_bytes = algorithmic_bytes(infos, pr)
    cpu = None
    sym_per_byte = None
    if not args.no_cpu_baseline:
        cpu = cpu_baseline(streams, pr)
        sym_per_byte = symbols_in(streams)
    # counters were taken with the plain filter only
    stages, roofline = stage_report(stage, work, entropy_bytes, sym_per_byte, None if args.antialias else cfg)
    if args.antialias:
        stages[3]["kernel"] = "resize_antialias_crop_normalize"

    result = {
        "metric": METRIC, "value": value, "unit": "images/s", "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "int32 entropy decode, f64 IDCT, f32 resize -> " + pr["out_dtype"] + " output",
        "data": "synthetic",
        "config": {"workload": WORKLOAD_NAMES[cfg], "batch": n, "streams": n_handles,
                   "input": "host memory" if args.host_input else "resident in HBM",
                   "entry_point": "prep_decode_resize_batch" if args.host_input else "prep_decode_resize_batch_resident",
                   "resize_filter": "antialiased bilinear" if args.antialias else "bilinear",
                   "compressed_bytes": int(offsets[-1]), "pixels": int(pixels),
                   "sha256": synth.sha256_of(streams), "input_generation_s": round(gen_s, 2)},
        "roofline": roofline,
        "stages": stages,
        "stage_timing": "one batch at a time" if n_handles == 1 else
                        "stream 0 only, while the other streams' batches share the GPU",
        "gpu_ms_per_step": float(stage.sum()),
        # S1, the host marker/table parser and launch planning: time inside the entry point with
        # the GPU idle (it returns after enqueueing; in the timed region it overlaps the GPU work
        # of the call before, and call_ms_in_timed_region also counts waiting for a free slot)
        "s1_host_ms_per_call": s1_host * 1e3,
        "s1_host_us_per_image": s1_host * 1e6 / n,
        "call_ms_in_timed_region": host_per_call * 1e3,
        ("resident" if first_is_host else "host_input"): other,
        "overlapped": overlapped,
        "cpu_baseline": cpu,
    }
    print(json.dumps(result))
    for h in pps:
        h.close()


if __name__ == "__main__":
    main()
