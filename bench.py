#!/usr/bin/env python3
"""Benchmark of the NeuZip hot path on one MI355X.

Headline workload (config 2 of the baseline): one Llama-style MLP weight, bf16 4096 x 14336,
i.i.d. N(0, 0.02^2), lossless; compressed once, then decompressed K times by the fused
decode kernel into one bf16 scratch buffer.  A "step" is one such decompression: it is
what Alg. 1 runs per layer in every forward and backward pass.  The reported value is
GB/s of bf16 output (2 bytes x elements / time); inputs and outputs are device buffers.

Prints ONE JSON line.  Besides the headline, the default run measures every other baseline
configuration in the same process, so that one line carries all of them:
  sustained   config 2 over 2000 launches after 200 warm-up launches, whatever --steps says
  config4     the lossy 70B-shaped MLP weight (does not fit the last-level cache), k = 7, 3, 1, 0
  config3     the Llama-3-8B-shaped set in forward order into one scratch: tensor by tensor and
              a layer per launch
  config5     the training-step loop on that set: decompress all, synthetic update, compress again
  size_sweep  three matrix sizes of the paper's throughput figure
  cpu_baseline  the CPU oracle on the host cores, all threads and one thread
--extended adds block-wise normalisation, the fused linear layer, binary32/binary16, the weight
step and the 10-step loops; --sweep the full size sweep; --profile-case NAME runs one named
workload a few times and nothing else (the command the rocprofv3 summaries in profiles/ were made with).
"""
import argparse
import json
import math
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0  # MI355X HBM3E, published
CPU_SHARE = 16          # host threads a one-GPU machine grants a job

PROFILE_CASES = ("decode_config2", "decode_config4_k7", "decode_config4_k3", "decode_config4_k1", "decode_config4_k0",
                 "decode_config4_k3_block512",
                 "decode_embedding", "decode_batch_layer",
                 "decode_small_kv", "compress_config2", "recompress_config2", "compress_embedding",
                 "recompress_embedding", "update_config2", "linear_q", "linear_qkv")


def parse_args():
    p = argparse.ArgumentParser()
    p.add_argument("--gpus", type=int, default=1)
    p.add_argument("--steps", type=int, default=2000)
    p.add_argument("--warmup", type=int, default=200)
    p.add_argument("--no-cpu-baseline", action="store_true", help="skip the oracle timing leg")
    p.add_argument("--headline-only", action="store_true", help="config 2 only (skip configs 3, 4, 5 and the sweep)")
    p.add_argument("--extended", action="store_true",
                   help="also time block-wise normalisation, the fused linear layer, the other element types, "
                        "the weight step and the 10-step loops")
    p.add_argument("--sweep", action="store_true",
                   help="time compress/decompress against matrix size, 1e5..1e8 bytes (the axis of the paper's Fig. 4)")
    p.add_argument("--layers", type=int, default=32, help="decoder layers of the Llama-3-8B-shaped set")
    p.add_argument("--profile-case", choices=PROFILE_CASES, default=None,
                   help="run one workload a few times, with a plain device copy of known size beside it, and exit")
    p.add_argument("--profile-launches", type=int, default=20)
    return p.parse_args()


def read_traffic_note():
    """HBM bytes per decode launch measured with rocprofv3 --pmc in a separate run (see profiles/), or None."""
    path = os.path.join(ROOT, "profiles", "decode_config2.txt")
    try:
        with open(path) as fh:
            for line in fh:
                if line.startswith("traffic_bytes_per_launch="):
                    return float(line.split("=", 1)[1])
    except OSError:
        pass
    return None


def timed_region(torch, stream, fn, steps):
    """Runs fn() `steps` times on `stream`; returns (wall seconds, HIP-event milliseconds)."""
    start, stop = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    start.record(stream)
    for _ in range(steps):
        fn()
    stop.record(stream)
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    return wall, start.elapsed_time(stop)


def event_us(torch, stream, fn, launches, warm=3):
    for _ in range(warm):
        fn()
    _, ms = timed_region(torch, stream, fn, launches)
    return ms / launches * 1e3


def wall_us(torch, fn, calls, warm=2):
    """For calls that wait on the host themselves (compress): wall time per call, microseconds."""
    for _ in range(warm):
        fn()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(calls):
        fn()
    torch.cuda.synchronize()
    return (time.perf_counter() - t0) / calls * 1e6


def hbm_frac(nbytes, us):
    return round(nbytes / (us * 1e-6) / 1e9 / HBM_PEAK_GBPS, 4)


def entropy_of(np, counts):
    cnt = counts.astype(np.float64)
    p = cnt[cnt > 0] / cnt.sum()
    return float(-(p * np.log2(p)).sum())


class Model:
    """The Llama-3-8B-shaped set of config 3 / 5, compressed, with one reusable scratch."""

    def __init__(self, torch, nz, inputs, dev, layers):
        names = inputs.llama3_8b_tensors()
        if layers < 32:
            names = names[: 1 + 7 * layers]
        self.blobs, self.total = [], 0
        for i, (_, shp) in enumerate(names):
            t = inputs.gaussian_bf16(shp, inputs.seed_for(3, i), device=dev)
            self.blobs.append(nz.neuzip_compress(t, 7))
            self.total += t.numel()
            del t
        self.comp = sum(b.compressed_bytes for b in self.blobs)
        self.big = torch.empty(max(b.elems for b in self.blobs), dtype=torch.bfloat16, device=dev)
        # layer schedule: the embedding, then the 7 weights of a layer in one launch, each into its own
        # piece of the one scratch
        self.groups = [[0]] + [list(range(1 + 7 * l, 8 + 7 * l)) for l in range((len(self.blobs) - 1) // 7)]
        self.plans = []
        for g in self.groups:
            at, dsts = 0, []
            for i in g:
                dsts.append(self.big[at: at + self.blobs[i].elems])
                at += (self.blobs[i].elems + 127) // 128 * 128
            self.plans.append(([self.blobs[i] for i in g], dsts))
        self.nz = nz

    def tensor_by_tensor(self):
        for b in self.blobs:
            self.nz.neuzip_decompress(b, self.big[: b.elems])

    def sequence(self):
        self.nz.neuzip_decompress_sequence(self.blobs, self.big)

    def layer_by_layer(self):
        for bl, dsts in self.plans:
            self.nz.neuzip_decompress_batch(bl, dsts)


def profile_case(args, torch, nz, inputs, np, dev, stream):
    """One named workload, a few launches, plus a plain device copy of known size (the counters'
    calibration: it reads and writes exactly `copy_bytes`)."""
    case, reps = args.profile_case, args.profile_launches
    info = {"profile_case": case, "launches": reps}
    cal_a = torch.empty(64 << 20, dtype=torch.bfloat16, device=dev)
    cal_b = torch.empty_like(cal_a)
    for _ in range(5):
        cal_b.copy_(cal_a)
    info["copy_bytes_each_way"] = cal_a.numel() * 2

    def run(fn, nbytes, elems):
        us = event_us(torch, stream, fn, reps)
        info.update({"us_per_call": round(us, 2), "algorithmic_bytes": nbytes, "elements": elems,
                     "hbm_frac": hbm_frac(nbytes, us)})

    def run_wall(fn, nbytes, elems):
        us = wall_us(torch, fn, reps)
        info.update({"us_per_call_wall": round(us, 2), "algorithmic_bytes": nbytes, "elements": elems,
                     "hbm_frac": hbm_frac(nbytes, us)})

    if case in ("decode_config2", "compress_config2", "recompress_config2", "update_config2"):
        w = inputs.gaussian_bf16(inputs.MLP_8B, inputs.seed_for(2), device=dev)
    elif case in ("decode_embedding", "compress_embedding", "recompress_embedding"):
        w = inputs.gaussian_bf16((128256, 4096), inputs.seed_for(3, 0), device=dev)
    elif case.startswith("decode_config4"):
        w = inputs.student_t4_bf16(inputs.MLP_70B, inputs.seed_for(4), device=dev)
    elif case == "decode_small_kv":
        w = inputs.gaussian_bf16((1024, 4096), inputs.seed_for(3, 2), device=dev)
    elif case == "linear_q":
        w = inputs.gaussian_bf16((4096, 4096), inputs.seed_for(3, 1), device=dev)
    else:
        w = None

    if case.startswith("decode_") and case != "decode_batch_layer":
        if case.endswith("_block512"):     # the paper's default lossy form: block-wise normalisation (Sec. 2.3)
            k, blob = 3, nz.neuzip_compress_blockwise(w, 3, 512)
        else:
            k = {"_k3": 3, "_k1": 1, "_k0": 0}.get(case[-3:], 7)
            blob = nz.neuzip_compress(w, k)
        out = torch.empty(w.numel(), dtype=torch.bfloat16, device=dev)
        run(lambda: nz.neuzip_decompress(blob, out), blob.compressed_bytes + 2 * w.numel(), w.numel())
        nz.neuzip_check(blob)
    elif case == "decode_batch_layer":
        model = Model(torch, nz, inputs, dev, 1)
        bl, dsts = model.plans[1]
        elems = sum(b.elems for b in bl)
        run(lambda: nz.neuzip_decompress_batch(bl, dsts), sum(b.compressed_bytes for b in bl) + 2 * elems, elems)
    elif case.startswith("compress_"):
        blob = nz.neuzip_compress(w, 7)
        # two reads of the tensor (statistics, then coding), the container written, the run slots
        # written and read once more on their way to their final place
        run_wall(lambda: nz.neuzip_compress(w, 7, blob=blob), 4 * w.numel() + blob.compressed_bytes, w.numel())
    elif case.startswith("recompress_"):
        (blob,) = nz.neuzip_compress_guarded([w], 7, 8)
        new = inputs.synthetic_update(w, inputs.seed_for(5, 1))
        run_wall(lambda: nz.neuzip_recompress([new], [blob]), 2 * w.numel() + blob.compressed_bytes, w.numel())
    elif case == "update_config2":
        (blob,) = nz.neuzip_compress_guarded([w], 7, 8)
        grad = inputs.gaussian_bf16(inputs.MLP_8B, inputs.seed_for(10, 1), std=0.05, device=dev)
        tmp = torch.empty_like(w)
        nz.neuzip_decompress(blob, tmp.view(-1))
        run_wall(lambda: nz.neuzip_update([blob], [grad], [tmp], 1e-3, weights_ready=2),
                 4 * w.numel() + blob.compressed_bytes, w.numel())
    elif case == "linear_qkv":
        outs = (4096, 1024, 1024)
        ws = [inputs.gaussian_bf16((o, 4096), inputs.seed_for(8, 700 + i), device=dev) for i, o in enumerate(outs)]
        blobs = [nz.neuzip_compress(t, 7) for t in ws]
        x = inputs.gaussian_bf16((1, 4096), inputs.seed_for(8, 501), std=1.0, device=dev)
        ys = [torch.empty((1, o), dtype=torch.float32, device=dev) for o in outs]
        run(lambda: nz.neuzip_linear_batch(blobs, outs, 4096, x, None, ys), sum(b.compressed_bytes for b in blobs),
            sum(t.numel() for t in ws))
    elif case == "linear_q":
        blob = nz.neuzip_compress(w, 7)
        x = inputs.gaussian_bf16((1, 4096), inputs.seed_for(8, 501), std=1.0, device=dev)
        y = torch.empty((1, 4096), dtype=torch.float32, device=dev)
        run(lambda: nz.neuzip_linear(blob, 4096, 4096, x, None, y), blob.compressed_bytes, w.numel())
    for _ in range(5):
        cal_b.copy_(cal_a)
    torch.cuda.synchronize()
    print(json.dumps(info), flush=True)


def main():
    args = parse_args()
    if args.gpus != 1:
        print("bench.py measures one GPU: this build has no multi-GPU path (run with --gpus 1)", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    from paper_2410_20650_amd import binding as nz, inputs

    if not torch.cuda.is_available():
        print("bench.py needs a GPU", file=sys.stderr)
        sys.exit(2)
    torch.cuda.set_device(0)
    dev = "cuda:0"
    stream = torch.cuda.current_stream()

    if args.profile_case:
        profile_case(args, torch, nz, inputs, np, dev, stream)
        return

    # ---------------------------------------------------------------- workload: config 2
    shape = inputs.MLP_8B
    w = inputs.gaussian_bf16(shape, inputs.seed_for(2), device=dev)
    n = w.numel()
    blob = nz.neuzip_compress(w, 7)
    scratch = torch.empty(n, dtype=torch.bfloat16, device=dev)

    def step():
        nz.neuzip_decompress(blob, scratch)

    for _ in range(args.warmup):
        step()
    wall, event_ms = timed_region(torch, stream, step, args.steps)
    nz.neuzip_check(blob)
    assert torch.equal(scratch.view(torch.int16), w.reshape(-1).view(torch.int16)), "round trip is not bit exact"

    ms_per_step = wall * 1e3 / args.steps
    out_bytes = 2.0 * n
    value = out_bytes / (wall / args.steps) / 1e9

    # statistics of the tensor and of its container
    entropy = entropy_of(np, nz.neuzip_histogram(blob))
    comp_bytes = blob.compressed_bytes
    bits_per_weight = 8.0 * comp_bytes / n

    # roofline of the decode kernel: algorithmic bytes = container bytes read + bf16 bytes written
    kernel_ms = event_ms / args.steps
    algo_bytes = comp_bytes + out_bytes
    achieved = algo_bytes / (kernel_ms * 1e-3) / 1e9
    roofline = {"bound": "hbm", "achieved": round(achieved, 1), "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                "frac": round(achieved / HBM_PEAK_GBPS, 4), "traffic": read_traffic_note(),
                "traffic_source": "profiles/decode_config2.txt (rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE, a separate run; not measured in this one)",
                "kernel": "decode_kernel<7, false, 0>", "avg_launch_us": round(kernel_ms * 1e3, 2),
                "algorithmic_bytes_per_elem": round(algo_bytes / n, 4),
                "working_set": "196 MB: fits the 256 MB last-level cache, so this figure is cache assisted; "
                               "see roofline_hbm_resident for a tensor that streams through HBM"}

    result = {
        "metric": "bf16 decompress GB/s (output)", "value": round(value, 1), "unit": "GB/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms_per_step, 5),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "u32", "data": "synthetic",
        "config": {"workload": "config 2: bf16 4096x14336 i.i.d. N(0,0.02), lossless, one compress then "
                               "repeated fused decompress into one bf16 scratch", "elements": n,
                   "mantissa_bits": 7, "chunk": 4096, "states_per_chunk": 16, "prob_bits": 12},
        "roofline": roofline,
        "bits_per_weight": round(bits_per_weight, 4), "exponent_entropy_bits": round(entropy, 4),
        "bits_per_weight_over_bound": round(bits_per_weight / (entropy + 8.0), 5),
        "event_ms_per_step": round(kernel_ms, 5),
    }

    # the same launch, sustained: independent of --steps (the first ~100 launches of a process run slower)
    us = event_us(torch, stream, step, 2000, warm=200)
    result["sustained"] = {"launches": 2000, "warmup": 200, "us_per_launch": round(us, 2),
                           "GBps_output": round(out_bytes / us / 1e3, 1), "hbm_frac": hbm_frac(algo_bytes, us)}

    # context: a plain device copy of the same output size
    src = torch.empty_like(scratch)
    us = event_us(torch, stream, lambda: scratch.copy_(src), 50, warm=5)
    result["device_copy_GBps_read_plus_write"] = round(2 * out_bytes / us / 1e3, 1)
    # ... and a kernel that only moves the decoder's bytes (reads the container's size, writes the tensor's)
    probe_in = torch.empty(comp_bytes // 16 * 16, dtype=torch.uint8, device=dev)
    us = event_us(torch, stream, lambda: nz.neuzip_stream_probe(probe_in, src), 50, warm=5)
    result["stream_probe"] = {"config2_GBps": round((probe_in.numel() + out_bytes) / us / 1e3, 1), "config2_us": round(us, 2),
                              "what": "a kernel that only reads the container's bytes and writes the tensor's, in the "
                                      "decoder's launch shape and access pattern (512-lane workgroups owning 32 chunks, "
                                      "the decoder's LDS, field loads and 16-byte stores four turns at a time): the "
                                      "ceiling for a decoder of this shape"}
    del probe_in

    # compress rate (histogram + table + encode + offsets + compaction, incl. the one size read-back)
    us = wall_us(torch, lambda: nz.neuzip_compress(w, 7, blob=blob), 10, warm=3)
    result["compress_GBps_input"] = round(out_bytes / us / 1e3, 1)
    result["compress_us"] = round(us, 1)
    (kept,) = nz.neuzip_compress_guarded([w], 7, 8)
    w_new = inputs.synthetic_update(w, inputs.seed_for(5, 1))
    us = wall_us(torch, lambda: nz.neuzip_recompress([w_new], [kept]), 10, warm=3)
    result["recompress_kept_table_us"] = round(us, 1)
    nz.neuzip_free(kept)
    del w_new

    # ---------------------------------------------------------------- CPU oracle on the host cores
    if not args.no_cpu_baseline:
        from oracle import oracle as O
        affinity = len(os.sched_getaffinity(0))
        cores = min(affinity, CPU_SHARE)
        words = inputs.bits(w)
        container = nz.neuzip_export(blob)
        # about ten seconds of oracle work: repeated whole-tensor passes, the median is reported
        times, spent = [], 0.0
        while len(times) < 3 or (spent < 10.0 and len(times) < 1000):
            t0 = time.perf_counter()
            back = O.decompress(container, n, threads=cores)
            times.append(time.perf_counter() - t0)
            spent += times[-1]
        best = sorted(times)[len(times) // 2]
        assert np.array_equal(back, words), "oracle and GPU disagree"
        t0 = time.perf_counter()
        theirs = O.compress(words, 7, threads=cores)
        enc_s = time.perf_counter() - t0
        assert np.array_equal(theirs, container), "container differs from the oracle's"
        t0 = time.perf_counter()
        O.decompress(container, n, threads=1)
        one_dec = time.perf_counter() - t0
        t0 = time.perf_counter()
        O.compress(words, 7, threads=1)
        one_enc = time.perf_counter() - t0
        result["cpu_baseline"] = {"value": round(out_bytes / best / 1e9, 3), "unit": "GB/s", "cores": cores,
                                  "kind": "oracle",
                                  "sample": "the whole config-2 tensor (58.7M elements), oracle decompress of "
                                            "the GPU-written container, median of %d passes (%.1f s); "
                                            "containers compared byte for byte" % (len(times), spent),
                                  "compress_GBps_input": round(out_bytes / enc_s / 1e9, 3),
                                  "one_thread": {"value": round(out_bytes / one_dec / 1e9, 3),
                                                 "compress_GBps_input": round(out_bytes / one_enc / 1e9, 3),
                                                 "sample": "one pass each over the same tensor"},
                                  "host_affinity_cores": affinity,
                                  "cores_note": "threads = min(cores in the affinity mask, the %d a one-GPU box grants)" % CPU_SHARE}
        del words, container, back, theirs

    del w, scratch, src
    nz.neuzip_free(blob)
    torch.cuda.empty_cache()

    model = None
    if not args.headline_only:
        # ------------------------------------------------------------ config 4: lossy, HBM resident
        t4 = inputs.student_t4_bf16(inputs.MLP_70B, inputs.seed_for(4), device=dev)
        n4 = t4.numel()
        buf = torch.empty(n4, dtype=torch.bfloat16, device=dev)
        c4 = {"elements": n4}
        for k in (7, 3, 1, 0):
            b4 = nz.neuzip_compress(t4, k)
            us = event_us(torch, stream, lambda: nz.neuzip_decompress(b4, buf), 50, warm=5)
            if k == 7:
                c4["exponent_entropy_bits"] = round(entropy_of(np, nz.neuzip_histogram(b4)), 4)
                assert torch.equal(buf.view(torch.int16), t4.reshape(-1).view(torch.int16)), "config 4 round trip"
                result["roofline_hbm_resident"] = {
                    "bound": "hbm", "achieved": round((b4.compressed_bytes + 2.0 * n4) / us / 1e3, 1),
                    "peak": HBM_PEAK_GBPS, "unit": "GB/s", "frac": hbm_frac(b4.compressed_bytes + 2.0 * n4, us),
                    "kernel": "decode_kernel<7, false, 0> (non-temporal stores)", "avg_launch_us": round(us, 2),
                    "workload": "config 4 tensor (bf16 28672x8192, Student-t), lossless: 783 MB per launch, "
                                "beyond the last-level cache", "launches": 50}
            else:
                mask = ~((1 << (7 - k)) - 1)
                assert torch.equal(buf.view(torch.int16), t4.reshape(-1).view(torch.int16) & mask), "config 4 truncation"
            c4[f"k{k}"] = {"GBps_output": round(2.0 * n4 / us / 1e3, 1), "us": round(us, 1),
                           "hbm_frac": hbm_frac(b4.compressed_bytes + 2.0 * n4, us),
                           "bits_per_weight": round(8.0 * b4.compressed_bytes / n4, 4)}
            nz.neuzip_free(b4)
        us = event_us(torch, stream, lambda: buf.copy_(t4.view(-1)), 20, warm=3)
        c4["device_copy_GBps_read_plus_write"] = round(4.0 * n4 / us / 1e3, 1)
        probe_in = torch.empty(int(c4["k7"]["bits_per_weight"] * n4 / 8) // 16 * 16, dtype=torch.uint8, device=dev)
        us = event_us(torch, stream, lambda: nz.neuzip_stream_probe(probe_in, buf), 20, warm=3)
        c4["stream_probe_k7_GBps"] = round((probe_in.numel() + 2.0 * n4) / us / 1e3, 1)
        del probe_in
        result["config4"] = c4
        del t4, buf
        torch.cuda.empty_cache()

        # ------------------------------------------------------------ config 3: forward schedule, one scratch
        model = Model(torch, nz, inputs, dev, args.layers)
        c3 = {"tensors": len(model.blobs), "elements": model.total,
              "bits_per_weight": round(8.0 * model.comp / model.total, 4)}
        for label, fn in (("tensor_by_tensor", model.tensor_by_tensor), ("sequence", model.sequence),
                          ("layer_by_layer", model.layer_by_layer)):
            us = event_us(torch, stream, fn, 5, warm=2)
            c3[label] = {"ms": round(us / 1e3, 4), "GBps_output": round(2.0 * model.total / us / 1e3, 1),
                         "hbm_frac": hbm_frac(model.comp + 2.0 * model.total, us)}
        c3["schedules"] = ("all into ONE scratch of the embedding's size.  tensor_by_tensor: neuzip_decompress per tensor, "
                           "each to the start of the scratch (the small projections cannot fill the chip); sequence: one "
                           "neuzip_decompress_sequence call, neighbours that fit the scratch together share it and a "
                           "launch (8 per launch); layer_by_layer: neuzip_decompress_batch, the 7 weights of a layer "
                           "in one launch into 7 pieces of the scratch")
        result["config3"] = c3

        # ------------------------------------------------------------ config 5: training-step loop
        result["config5"] = training_loop(torch, nz, inputs, stream, model, steps=2, kept_table=False)

        # ------------------------------------------------------------ three sizes of the paper's throughput figure
        result["size_sweep"] = size_sweep(torch, nz, inputs, dev, stream, (1e5, 1e7, 1e8), (7, 3))

    if args.extended:
        if model is None:
            model = Model(torch, nz, inputs, dev, args.layers)
        result["extended"] = extended(args, torch, nz, inputs, np, dev, stream, model)

    if args.sweep:
        result["size_sweep_full"] = size_sweep(torch, nz, inputs, dev, stream,
                                               (1e5, 3e5, 1e6, 3e6, 1e7, 3e7, 1e8), (7, 3, 1, 0), host=True)

    print(json.dumps(result), flush=True)


def training_loop(torch, nz, inputs, stream, model, steps, kept_table):
    """Config 5 on the config-3 set: per step decompress every tensor (a layer per launch), apply the
    synthetic update (torch, not timed), compress again (a layer per call), verify bit by bit.
    kept_table: step 0 builds guarded tables, later steps reuse them (neuzip_recompress)."""
    total = model.total
    upd = torch.empty_like(model.big)
    dec_ms, enc_s, enc_single_s, rebuilt, enc_later_s = 0.0, 0.0, 0.0, 0, 0.0
    for step in range(steps):
        _, ms = timed_region(torch, stream, model.layer_by_layer, 1)
        dec_ms += ms
        for g, (bl, dsts) in zip(model.groups, model.plans):
            nz.neuzip_decompress_batch(bl, dsts)
            news = []
            for i, d in zip(g, dsts):
                at = (d.data_ptr() - model.big.data_ptr()) // 2
                dst = upd[at: at + d.numel()]
                dst.copy_(inputs.synthetic_update(d, inputs.seed_for(5, 1000 * (step + 1) + i + (500 if kept_table else 0))))
                news.append(dst)
            torch.cuda.synchronize()
            if step == 0 and not kept_table:            # reference: one call per tensor
                t0 = time.perf_counter()
                for b, t in zip(bl, news):
                    nz.neuzip_compress(t, 7, blob=b)
                torch.cuda.synchronize()
                enc_single_s += time.perf_counter() - t0
            t0 = time.perf_counter()
            if not kept_table:
                nz.neuzip_compress_batch(news, 7, 0, blobs=bl)
            elif step == 0:
                nz.neuzip_compress_guarded(news, 7, 8, blobs=bl)
            else:
                rebuilt += sum(nz.neuzip_recompress(news, bl))
            torch.cuda.synchronize()
            enc_s += time.perf_counter() - t0
            if step > 0:
                enc_later_s += time.perf_counter() - t0
            nz.neuzip_decompress_batch(bl, dsts)
            for d, t in zip(dsts, news):
                assert torch.equal(d.view(torch.int16), t.view(torch.int16)), "step %d" % step
    out = {"steps": steps, "tensors": len(model.blobs),
           "decompress_GBps_output": round(2.0 * total * steps / (dec_ms * 1e-3) / 1e9, 1),
           "compress_GBps_input": round(2.0 * total * steps / enc_s / 1e9, 1),
           "bitwise_round_trip": "verified for every tensor at every step"}
    if steps > 1:
        out["compress_GBps_input_steps_after_first"] = round(2.0 * total * (steps - 1) / enc_later_s / 1e9, 1)
    if kept_table:
        out.update({"guard": 8, "tensors_rebuilt": rebuilt,
                    "bits_per_weight_after_last_step": round(8.0 * sum(b.compressed_bytes for b in model.blobs) / total, 4)})
    else:
        out["compress_GBps_input_one_call_per_tensor"] = round(2.0 * total / enc_single_s / 1e9, 1)
        out["compress_calls"] = "one neuzip_compress_batch call per layer (7 tensors), fresh statistics every step"
    # what the compress calls hold besides the blobs (encoder run slots, capped by the workspace limit)
    out["compress_workspace_MiB"] = nz.neuzip_workspace_bytes() >> 20
    return out


def size_sweep(torch, nz, inputs, dev, stream, sizes, widths, host=False):
    rows = []
    for nbytes in sizes:
        ne = int(nbytes) // 2 // 8 * 8
        t = inputs.gaussian_bf16(ne, inputs.seed_for(6, int(math.log10(nbytes) * 10)), device=dev)
        o = torch.empty_like(t)
        row = {"bytes": 2 * ne}
        gib = 2.0 * ne / 2 ** 30
        for k in widths:
            bk = nz.neuzip_compress(t, k)
            us = event_us(torch, stream, lambda: nz.neuzip_decompress(bk, o), 50)
            row[f"decompress_k{k}_GiBps"] = round(gib / (us * 1e-6), 1)
            us = wall_us(torch, lambda: nz.neuzip_compress(t, k, blob=bk), 10)
            row[f"compress_k{k}_GiBps"] = round(gib / (us * 1e-6), 1)
            nz.neuzip_free(bk)
        us = event_us(torch, stream, lambda: o.copy_(t), 50)
        row["device_copy_GiBps"] = round(gib / (us * 1e-6), 1)
        if host:
            # the paper's CPU-offloading baseline: the matrix leaves for pinned host memory and comes back
            pinned = torch.empty(ne, dtype=torch.bfloat16, pin_memory=True)
            us_out = event_us(torch, stream, lambda: pinned.copy_(t, non_blocking=True), 10, warm=2)
            us_in = event_us(torch, stream, lambda: o.copy_(pinned, non_blocking=True), 10, warm=2)
            row["offload_to_host_GiBps"] = round(gib / (us_out * 1e-6), 1)
            row["reload_from_host_GiBps"] = round(gib / (us_in * 1e-6), 1)
            del pinned
        rows.append(row)
        del t, o
    return rows


def extended(args, torch, nz, inputs, np, dev, stream, model):
    ext = {}
    # config 4 with block-wise normalisation (Sec. 2.3; block 512 is the paper's default)
    t4 = inputs.student_t4_bf16(inputs.MLP_70B, inputs.seed_for(4), device=dev)
    n4 = t4.numel()
    buf = torch.empty(n4, dtype=torch.bfloat16, device=dev)
    ref = t4.reshape(-1).float()
    for k, blk in ((3, 512), (0, 512), (0, 32)):
        plain = nz.neuzip_compress(t4, k)
        nz.neuzip_decompress(plain, buf)
        err_plain = ((buf.float() - ref).abs().mean() / ref.abs().mean()).item()
        nz.neuzip_free(plain)
        b4 = nz.neuzip_compress_blockwise(t4, k, blk)
        us = event_us(torch, stream, lambda: nz.neuzip_decompress(b4, buf), 50, warm=5)
        err = ((buf.float() - ref).abs().mean() / ref.abs().mean()).item()
        ext[f"config4_k{k}_block{blk}"] = {
            "decompress_GBps_output": round(2.0 * n4 / us / 1e3, 1),
            "hbm_frac": hbm_frac(b4.compressed_bytes + 2.0 * n4, us),
            "bits_per_weight": round(8.0 * b4.compressed_bytes / n4, 4),
            "mean_abs_error_over_mean_abs_weight": round(err, 5),
            "same_without_normalisation": round(err_plain, 5)}
        nz.neuzip_free(b4)
    del t4, buf, ref
    torch.cuda.empty_cache()

    # the compressed forward pass of a linear layer (Sec. 2.2): the fused decode + matrix-core
    # kernel against decompress-into-scratch followed by a dense bf16 product (torch / hipBLASLt),
    # on the projection shapes of a Llama-3-8B layer, decoding batches of 1..16 tokens
    lin = {}
    for label, (out_f, in_f) in (("q_4096x4096", (4096, 4096)), ("up_14336x4096", (14336, 4096)),
                                 ("down_4096x14336", (4096, 14336))):
        wl = inputs.gaussian_bf16((out_f, in_f), inputs.seed_for(8, out_f % 97), device=dev)
        bl_ = nz.neuzip_compress(wl, 7)
        dense = torch.empty_like(wl)
        for tokens in (1, 16):
            xl = inputs.gaussian_bf16((tokens, in_f), inputs.seed_for(8, 500 + tokens), std=1.0, device=dev)
            yl = torch.empty((tokens, out_f), dtype=torch.float32, device=dev)

            def fused():
                nz.neuzip_linear(bl_, out_f, in_f, xl, None, yl)

            def separate():
                nz.neuzip_decompress(bl_, dense.view(-1))
                torch.matmul(xl, dense.t())

            times = {name: event_us(torch, stream, fn, 50, warm=5) for name, fn in (("fused", fused), ("separate", separate))}
            want = xl.float() @ dense.float().t()
            lin[f"{label}_tokens{tokens}"] = {
                "fused_us": round(times["fused"], 1),
                "decompress_then_dense_product_us": round(times["separate"], 1),
                "weights_GBps": round(2.0 * out_f * in_f / times["fused"] / 1e3, 1),
                "max_abs_diff_vs_dense_over_max_abs": round(((yl - want).abs().max() / want.abs().max()).item(), 7)}
        nz.neuzip_free(bl_)
        del wl, dense
    # the q, k and v projections of a Llama-3-8B attention block on the same activations: one fused
    # launch for the three against three fused calls and against decompressing the three (one launch)
    # followed by three dense products
    in_f, outs = 4096, (4096, 1024, 1024)
    wq = [inputs.gaussian_bf16((o, in_f), inputs.seed_for(8, 700 + i), device=dev) for i, o in enumerate(outs)]
    bq = [nz.neuzip_compress(w, 7) for w in wq]
    dq = [torch.empty_like(w) for w in wq]
    for tokens in (1, 16):
        xl = inputs.gaussian_bf16((tokens, in_f), inputs.seed_for(8, 800 + tokens), std=1.0, device=dev)
        yq = [torch.empty((tokens, o), dtype=torch.float32, device=dev) for o in outs]

        def one_launch():
            nz.neuzip_linear_batch(bq, outs, in_f, xl, None, yq)

        def three_calls():
            for b_, o_, y_ in zip(bq, outs, yq):
                nz.neuzip_linear(b_, o_, in_f, xl, None, y_)

        def separate():
            nz.neuzip_decompress_batch(bq, [d.view(-1) for d in dq])
            for d in dq:
                torch.matmul(xl, d.t())

        times = {name: event_us(torch, stream, fn, 50, warm=5)
                 for name, fn in (("one", one_launch), ("three", three_calls), ("separate", separate))}
        one_launch()
        worst = max(((y_ - xl.float() @ d.float().t()).abs().max() / (xl.float() @ d.float().t()).abs().max()).item()
                    for y_, d in zip(yq, dq))
        lin[f"qkv_4096+1024+1024x4096_tokens{tokens}"] = {
            "one_launch_us": round(times["one"], 1), "three_fused_calls_us": round(times["three"], 1),
            "decompress_batch_then_dense_products_us": round(times["separate"], 1),
            "max_abs_diff_vs_dense_over_max_abs": round(worst, 7)}
    for b_ in bq:
        nz.neuzip_free(b_)
    del wq, dq
    ext["linear_forward"] = lin
    torch.cuda.empty_cache()

    # binary32 tensors (beyond the paper's BFloat16): the 8B-shaped MLP weight as float32 --
    # the upper halves take the lossless path, the lower halves ride along as a raw plane
    w32 = inputs.gaussian_f32(inputs.MLP_8B, inputs.seed_for(9), device=dev)
    n32 = w32.numel()
    o32 = torch.empty_like(w32)
    (b32,) = nz.neuzip_compress_guarded([w32], 7, 8)
    u32 = inputs.synthetic_update(w32, inputs.seed_for(9, 1))
    f32 = {"elements": n32, "bits_per_weight": round(8.0 * b32.compressed_bytes / n32, 4)}
    us = event_us(torch, stream, lambda: nz.neuzip_decompress(b32, o32), 20)
    f32["decompress"] = {"us": round(us, 1), "GBps_tensor": round(4.0 * n32 / us / 1e3, 1),
                         "hbm_frac": hbm_frac(b32.compressed_bytes + 4.0 * n32, us)}
    us = wall_us(torch, lambda: nz.neuzip_compress_guarded([w32], 7, 8, blobs=[b32]), 20)
    f32["compress"] = {"us": round(us, 1), "GBps_tensor": round(4.0 * n32 / us / 1e3, 1)}
    us = wall_us(torch, lambda: nz.neuzip_recompress([u32], [b32]), 20)
    f32["recompress_kept_table"] = {"us": round(us, 1), "GBps_tensor": round(4.0 * n32 / us / 1e3, 1)}
    nz.neuzip_decompress(b32, o32)
    assert torch.equal(o32.view(torch.int32), u32.view(torch.int32)), "binary32 round trip"
    f32["bitwise_round_trip"] = "verified"
    ext["binary32_mlp_8b"] = f32
    nz.neuzip_free(b32)
    del w32, o32, u32
    torch.cuda.empty_cache()

    # binary16: the same weight as float16 -- the upper byte of a word is the coded symbol
    w16 = inputs.gaussian_f16(inputs.MLP_8B, inputs.seed_for(11), device=dev)
    o16 = torch.empty_like(w16)
    b16 = nz.neuzip_compress(w16, 7)
    f16 = {"elements": w16.numel(), "bits_per_weight": round(8.0 * b16.compressed_bytes / w16.numel(), 4)}
    us = event_us(torch, stream, lambda: nz.neuzip_decompress(b16, o16), 20)
    f16["decompress"] = {"us": round(us, 1), "GBps_tensor": round(2.0 * w16.numel() / us / 1e3, 1),
                         "hbm_frac": hbm_frac(b16.compressed_bytes + 2.0 * w16.numel(), us)}
    us = wall_us(torch, lambda: nz.neuzip_compress(w16, 7, blob=b16), 20)
    f16["compress"] = {"us": round(us, 1), "GBps_tensor": round(2.0 * w16.numel() / us / 1e3, 1)}
    assert torch.equal(o16.view(torch.int16), w16.view(torch.int16)), "binary16 round trip"
    f16["bitwise_round_trip"] = "verified"
    ext["binary16_mlp_8b"] = f16
    nz.neuzip_free(b16)
    del w16, o16
    torch.cuda.empty_cache()

    # the weight update of the backward loop (Alg. 1): W <- W - lr * grad on the compressed 8B-shaped
    # MLP weight, as one library call (the decoder applies the step, then the kept-table encoder)
    # against decompress, torch's in-place bf16 step, recompress
    wu = inputs.gaussian_bf16(inputs.MLP_8B, inputs.seed_for(10), device=dev)
    gu = inputs.gaussian_bf16(inputs.MLP_8B, inputs.seed_for(10, 1), std=0.05, device=dev)
    su = torch.empty_like(wu)
    (bu,) = nz.neuzip_compress_guarded([wu], 7, 8)
    flags = []

    def update_fused():
        flags.extend(nz.neuzip_update([bu], [gu], [su], 1e-3))

    def update_ready():
        # the backward pass has decompressed the weight anyway (for the input gradient): the
        # library then needs one pass of its encoder over weight and gradient
        nz.neuzip_decompress(bu, su.view(-1))
        flags.extend(nz.neuzip_update([bu], [gu], [su], 1e-3, weights_ready=True))

    def update_ready_discard():
        # ... and nobody needs the new weight uncompressed: it is not written back
        nz.neuzip_decompress(bu, su.view(-1))
        flags.extend(nz.neuzip_update([bu], [gu], [su], 1e-3, weights_ready=2))

    def update_separate():
        nz.neuzip_decompress(bu, su.view(-1))
        su.add_(gu, alpha=-1e-3)
        flags.extend(nz.neuzip_recompress([su], [bu]))

    upd = {"elements": wu.numel(), "lr": 1e-3}
    for name, fn in (("one_call", update_fused), ("decompress_then_one_call_with_weights_ready", update_ready),
                     ("decompress_then_one_call_new_weights_not_kept", update_ready_discard),
                     ("decompress_torch_step_recompress", update_separate)):
        for _ in range(3):
            fn()
        del flags[:]
        us = wall_us(torch, fn, 20, warm=0)
        upd[name] = {"us": round(us, 1), "GBps_weights": round(2.0 * wu.numel() / us / 1e3, 1),
                     "tensors_rebuilt": sum(flags)}
    ext["sgd_update_mlp_8b"] = upd
    nz.neuzip_free(bu)
    del wu, gu, su
    torch.cuda.empty_cache()

    # config 5 at its full length, twice: with a table rebuilt from a fresh histogram at every step, and
    # with the table kept from the step before (guard band 8; rebuilt only for a tensor whose new
    # values it cannot code)
    steps5 = 10 if args.layers >= 32 else 3
    ext["config5_loop"] = training_loop(torch, nz, inputs, stream, model, steps5, False)
    ext["config5_loop_kept_tables"] = training_loop(torch, nz, inputs, stream, model, steps5, True)

    # the backward loop of Alg. 1 at model scale: per layer, decompress the weights (the input
    # gradient needs them), then the weight step on the compressed weights with what is at hand
    # (synthetic gradients; new weights not kept uncompressed).  Checked bitwise against torch's
    # own float32 step on the first and the last group of every step.
    lr5 = 1e-3
    big, total = model.big, model.total
    upd = torch.empty_like(big)
    torch.manual_seed(inputs.seed_for(12))
    upd.normal_(0.0, 0.05)
    steps_u = 3
    dec_ms = upd_s = 0.0
    rebuilt_u = 0
    for step in range(steps_u):
        for gi, (bl, dsts) in enumerate(model.plans):
            _, ms = timed_region(torch, stream, lambda: nz.neuzip_decompress_batch(bl, dsts), 1)
            dec_ms += ms
            grads = [upd[(d.data_ptr() - big.data_ptr()) // 2: (d.data_ptr() - big.data_ptr()) // 2 + d.numel()]
                     for d in dsts]
            check = gi in (0, len(model.plans) - 1)
            if check:
                want = [(d.float() - torch.tensor(lr5, device=dev) * gr.float()).to(torch.bfloat16)
                        for d, gr in zip(dsts, grads)]
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            rebuilt_u += sum(nz.neuzip_update(bl, grads, dsts, lr5, weights_ready=2))
            torch.cuda.synchronize()
            upd_s += time.perf_counter() - t0
            if check:
                nz.neuzip_decompress_batch(bl, dsts)
                for d, t in zip(dsts, want):
                    assert torch.equal(d.view(torch.int16), t.view(torch.int16)), "weight step, step %d" % step
    ext["config5_backward_loop_with_weight_step"] = {
        "steps": steps_u, "tensors": len(model.blobs), "lr": lr5, "tensors_rebuilt": rebuilt_u,
        "decompress_GBps_output": round(2.0 * total * steps_u / (dec_ms * 1e-3) / 1e9, 1),
        "weight_step_GBps_weights": round(2.0 * total * steps_u / upd_s / 1e9, 1),
        "codec_ms_per_step": round((dec_ms * 1e-3 + upd_s) / steps_u * 1e3, 2),
        "bitwise_check": "first and last group of every step against torch's float32 step"}
    return ext


if __name__ == "__main__":
    main()
