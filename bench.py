#!/usr/bin/env python3
"""Benchmark of the NeuZip hot path on one MI355X.

Workload (config 2 of the baseline): one Llama-style MLP weight, bf16 4096 x 14336,
i.i.d. N(0, 0.02^2), lossless; compressed once, then decompressed K times by the fused
decode kernel into one bf16 scratch buffer.  A "step" is one such decompression: it is
what Alg. 1 runs per layer in every forward and backward pass.  The reported value is
GB/s of bf16 output (2 bytes x elements / time) with everything resident in HBM.

Prints ONE JSON line.  Extra keys: the roofline of the decode kernel, the CPU oracle
timed on this machine's host cores, bits/weight against the exponent entropy, the
compress rate, and (with --extended) the lossy 70B-shaped case and a Llama-3-8B-shaped
per-layer sweep.
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


def parse_args():
    p = argparse.ArgumentParser()
    p.add_argument("--gpus", type=int, default=1)
    p.add_argument("--steps", type=int, default=2000)
    p.add_argument("--warmup", type=int, default=200)
    p.add_argument("--no-cpu-baseline", action="store_true", help="skip the oracle timing leg")
    p.add_argument("--extended", action="store_true", help="also time config 4 (lossy) and a config-3 sweep")
    p.add_argument("--sweep", action="store_true",
                   help="also time compress/decompress against matrix size, 1e5..1e8 bytes (the axis of the paper's Fig. 4)")
    p.add_argument("--layers", type=int, default=32, help="decoder layers of the Llama-3-8B-shaped set used with --extended")
    return p.parse_args()


def read_traffic_note():
    """HBM bytes per decode launch measured with rocprofv3 --pmc (see profiles/), or None."""
    path = os.path.join(ROOT, "profiles", "decode_config2_traffic.txt")
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
    cnt = nz.neuzip_histogram(blob).astype(np.float64)
    p = cnt[cnt > 0] / cnt.sum()
    entropy = float(-(p * np.log2(p)).sum())
    comp_bytes = blob.compressed_bytes
    bits_per_weight = 8.0 * comp_bytes / n

    # roofline of the decode kernel: algorithmic bytes = container bytes read + bf16 bytes written
    kernel_ms = event_ms / args.steps
    algo_bytes = comp_bytes + out_bytes
    achieved = algo_bytes / (kernel_ms * 1e-3) / 1e9
    roofline = {"bound": "hbm", "achieved": round(achieved, 1), "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                "frac": round(achieved / HBM_PEAK_GBPS, 4), "traffic": read_traffic_note(),
                "kernel": "decode_kernel<7, false, 0>", "avg_launch_us": round(kernel_ms * 1e3, 2),
                "algorithmic_bytes_per_elem": round(algo_bytes / n, 4)}

    # context: a plain device copy of the same output size
    src = torch.empty_like(scratch)
    for _ in range(5):
        scratch.copy_(src)
    _, copy_ms = timed_region(torch, stream, lambda: scratch.copy_(src), 50)
    copy_gbps = 2 * out_bytes / (copy_ms / 50 * 1e-3) / 1e9

    # compress rate (histogram + table + encode + offsets + compaction, incl. the one size read-back)
    for _ in range(3):
        nz.neuzip_compress(w, 7, blob=blob)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    reps = 10
    for _ in range(reps):
        nz.neuzip_compress(w, 7, blob=blob)
    torch.cuda.synchronize()
    compress_gbps = out_bytes / ((time.perf_counter() - t0) / reps) / 1e9

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
        "compress_GBps_input": round(compress_gbps, 1),
        "device_copy_GBps_read_plus_write": round(copy_gbps, 1),
        "event_ms_per_step": round(kernel_ms, 5),
    }

    # ---------------------------------------------------------------- CPU oracle on the host cores
    if not args.no_cpu_baseline:
        from oracle import oracle as O
        cores = min(len(os.sched_getaffinity(0)), int(os.environ.get("OMP_NUM_THREADS", "16") or 16))
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
        result["cpu_baseline"] = {"value": round(out_bytes / best / 1e9, 3), "unit": "GB/s", "cores": cores,
                                  "kind": "oracle",
                                  "sample": "the whole config-2 tensor (58.7M elements), oracle decompress of "
                                            "the GPU-written container, median of %d passes (%.1f s); "
                                            "containers compared byte for byte" % (len(times), spent),
                                  "compress_GBps_input": round(out_bytes / enc_s / 1e9, 3)}
        del words, container, back, theirs

    # ---------------------------------------------------------------- optional: configs 4, 3 and 5
    if args.extended:
        ext = {}
        del w, scratch, src
        nz.neuzip_free(blob)
        torch.cuda.empty_cache()

        # config 4: lossy inference variant on a 70B-shaped MLP weight, heavy-tailed values
        t4 = inputs.student_t4_bf16(inputs.MLP_70B, inputs.seed_for(4), device=dev)
        n4 = t4.numel()
        buf = torch.empty(n4, dtype=torch.bfloat16, device=dev)
        for k in (7, 3, 1, 0):
            b4 = nz.neuzip_compress(t4, k)
            for _ in range(5):
                nz.neuzip_decompress(b4, buf)
            _, ms = timed_region(torch, stream, lambda: nz.neuzip_decompress(b4, buf), 50)
            ms /= 50
            if k == 7:
                c4 = nz.neuzip_histogram(b4).astype(np.float64)
                p4 = c4[c4 > 0] / c4.sum()
                ext["config4_exponent_entropy_bits"] = round(float(-(p4 * np.log2(p4)).sum()), 4)
            ext[f"config4_k{k}"] = {"decompress_GBps_output": round(2.0 * n4 / (ms * 1e-3) / 1e9, 1),
                                    "hbm_frac": round((b4.compressed_bytes + 2.0 * n4) / (ms * 1e-3) / 1e9 / HBM_PEAK_GBPS, 4),
                                    "bits_per_weight": round(8.0 * b4.compressed_bytes / n4, 4)}
            nz.neuzip_free(b4)
        # the same weight with block-wise normalisation (Sec. 2.3; block 512 is the paper's default)
        ref = t4.reshape(-1).float()
        for k, blk in ((3, 512), (0, 512), (0, 32)):
            plain = nz.neuzip_compress(t4, k)
            nz.neuzip_decompress(plain, buf)
            err_plain = ((buf.float() - ref).abs().mean() / ref.abs().mean()).item()
            nz.neuzip_free(plain)
            b4 = nz.neuzip_compress_blockwise(t4, k, blk)
            for _ in range(5):
                nz.neuzip_decompress(b4, buf)
            _, ms = timed_region(torch, stream, lambda: nz.neuzip_decompress(b4, buf), 50)
            ms /= 50
            err = ((buf.float() - ref).abs().mean() / ref.abs().mean()).item()
            ext[f"config4_k{k}_block{blk}"] = {
                "decompress_GBps_output": round(2.0 * n4 / (ms * 1e-3) / 1e9, 1),
                "hbm_frac": round((b4.compressed_bytes + 2.0 * n4) / (ms * 1e-3) / 1e9 / HBM_PEAK_GBPS, 4),
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

                times = {}
                for name, fn in (("fused", fused), ("separate", separate)):
                    for _ in range(5):
                        fn()
                    _, ms = timed_region(torch, stream, fn, 50)
                    times[name] = ms / 50
                ref = xl.float() @ dense.float().t()
                lin[f"{label}_tokens{tokens}"] = {
                    "fused_us": round(times["fused"] * 1e3, 1),
                    "decompress_then_dense_product_us": round(times["separate"] * 1e3, 1),
                    "weights_GBps": round(2.0 * out_f * in_f / (times["fused"] * 1e-3) / 1e9, 1),
                    "max_abs_diff_vs_dense_over_max_abs": round(((yl - ref).abs().max() / ref.abs().max()).item(), 7)}
            nz.neuzip_free(bl_)
            del wl, dense
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
        for name, fn, nbytes in (("decompress", lambda: nz.neuzip_decompress(b32, o32), b32.compressed_bytes + 4.0 * n32),
                                 ("compress", lambda: nz.neuzip_compress_guarded([w32], 7, 8, blobs=[b32]),
                                  4.0 * n32 * 2 + b32.compressed_bytes),
                                 ("recompress_kept_table", lambda: nz.neuzip_recompress([u32], [b32]),
                                  4.0 * n32 + b32.compressed_bytes)):
            for _ in range(3):
                fn()
            _, ms = timed_region(torch, stream, fn, 20)
            ms /= 20
            f32[name] = {"us": round(ms * 1e3, 1), "GBps_tensor": round(4.0 * n32 / (ms * 1e-3) / 1e9, 1),
                         "hbm_frac": round(nbytes / (ms * 1e-3) / 1e9 / HBM_PEAK_GBPS, 4)}
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
        for name, fn, nbytes in (("decompress", lambda: nz.neuzip_decompress(b16, o16), b16.compressed_bytes + 2.0 * w16.numel()),
                                 ("compress", lambda: nz.neuzip_compress(w16, 7, blob=b16),
                                  4.0 * w16.numel() + b16.compressed_bytes)):
            for _ in range(3):
                fn()
            _, ms = timed_region(torch, stream, fn, 20)
            ms /= 20
            f16[name] = {"us": round(ms * 1e3, 1), "GBps_tensor": round(2.0 * w16.numel() / (ms * 1e-3) / 1e9, 1),
                         "hbm_frac": round(nbytes / (ms * 1e-3) / 1e9 / HBM_PEAK_GBPS, 4)}
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
            _, ms = timed_region(torch, stream, fn, 20)
            ms /= 20
            upd[name] = {"us": round(ms * 1e3, 1), "GBps_weights": round(2.0 * wu.numel() / (ms * 1e-3) / 1e9, 1),
                         "tensors_rebuilt": sum(flags)}
        ext["sgd_update_mlp_8b"] = upd
        nz.neuzip_free(bu)
        del wu, gu, su
        torch.cuda.empty_cache()

        # config 3: every weight of a Llama-3-8B-shaped model, forward order, one reusable scratch
        names = inputs.llama3_8b_tensors()
        if args.layers < 32:
            names = names[: 1 + 7 * args.layers]
        blobs, total = [], 0
        for i, (name, shp) in enumerate(names):
            t = inputs.gaussian_bf16(shp, inputs.seed_for(3, i), device=dev)
            blobs.append(nz.neuzip_compress(t, 7))
            total += t.numel()
            del t
        comp = sum(b.compressed_bytes for b in blobs)
        big = torch.empty(max(b.elems for b in blobs), dtype=torch.bfloat16, device=dev)

        def sweep_tensor_by_tensor():
            nz.neuzip_decompress_sequence(blobs, big)

        # layer schedule: the embedding, then the 7 weights of a layer in one launch into the scratch
        groups = [[0]] + [list(range(1 + 7 * l, 8 + 7 * l)) for l in range((len(blobs) - 1) // 7)]
        plans = []
        for g in groups:
            at, dsts = 0, []
            for i in g:
                dsts.append(big[at: at + blobs[i].elems])
                at += (blobs[i].elems + 127) // 128 * 128
            plans.append(([blobs[i] for i in g], dsts))

        def sweep_layer_by_layer():
            for bl, dsts in plans:
                nz.neuzip_decompress_batch(bl, dsts)

        for label, fn in (("tensor_by_tensor", sweep_tensor_by_tensor), ("layer_by_layer", sweep_layer_by_layer)):
            for _ in range(2):
                fn()
            _, ms = timed_region(torch, stream, fn, 5)
            ms /= 5
            ext[f"config3_{label}"] = {"tensors": len(blobs), "elements": total, "ms": round(ms, 4),
                                       "decompress_GBps_output": round(2.0 * total / (ms * 1e-3) / 1e9, 1),
                                       "hbm_frac": round((comp + 2.0 * total) / (ms * 1e-3) / 1e9 / HBM_PEAK_GBPS, 4),
                                       "bits_per_weight": round(8.0 * comp / total, 4)}

        # config 5: training-step loop on the same blobs: decompress all, synthetic update,
        # compress again (a layer's weights per call), bitwise check, 10 steps.  Twice: with a table
        # rebuilt from a fresh histogram at every step, and with the table kept from the step
        # before (guard band 8; rebuilt only for a tensor whose new values it cannot code).
        steps5 = 10 if args.layers >= 32 else 3
        upd = torch.empty_like(big)

        def training_loop(kept_table):
            dec_ms, enc_s, enc_single_s, rebuilt, enc_later_s = 0.0, 0.0, 0.0, 0, 0.0
            for step in range(steps5):
                _, ms = timed_region(torch, stream, sweep_layer_by_layer, 1)
                dec_ms += ms
                for g, (bl, dsts) in zip(groups, plans):
                    nz.neuzip_decompress_batch(bl, dsts)
                    news = []
                    for i, d in zip(g, dsts):
                        at = d.data_ptr() - big.data_ptr()
                        dst = upd[at // 2: at // 2 + d.numel()]
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
            return dec_ms, enc_s, enc_single_s, rebuilt, enc_later_s

        dec_ms, enc_s, enc_single_s, _, enc_later_s = training_loop(False)
        ext["config5_loop"] = {"steps": steps5, "tensors": len(blobs),
                               "decompress_GBps_output": round(2.0 * total * steps5 / (dec_ms * 1e-3) / 1e9, 1),
                               "compress_GBps_input": round(2.0 * total * steps5 / enc_s / 1e9, 1),
                               "compress_GBps_input_steps_after_first": round(2.0 * total * (steps5 - 1) / enc_later_s / 1e9, 1),
                               "compress_GBps_input_one_call_per_tensor": round(2.0 * total / enc_single_s / 1e9, 1),
                               "bitwise_round_trip": "verified for every tensor at every step"}
        dec_ms, enc_s, _, rebuilt, enc_later_s = training_loop(True)
        ext["config5_loop_kept_tables"] = {
            "steps": steps5, "guard": 8, "tensors_rebuilt": rebuilt,
            "compress_GBps_input": round(2.0 * total * steps5 / enc_s / 1e9, 1),
            "compress_GBps_input_steps_after_first": round(2.0 * total * (steps5 - 1) / enc_later_s / 1e9, 1),
            "decompress_GBps_output": round(2.0 * total * steps5 / (dec_ms * 1e-3) / 1e9, 1),
            "bits_per_weight_after_last_step": round(8.0 * sum(b.compressed_bytes for b in blobs) / total, 4),
            "bitwise_round_trip": "verified for every tensor at every step"}
        # the backward loop of Alg. 1 at model scale: per layer, decompress the weights (the input
        # gradient needs them), then the weight step on the compressed weights with what is at hand
        # (synthetic gradients; new weights not kept uncompressed).  Checked bitwise against torch's
        # own float32 step on the first and the last group of every step.
        lr5 = 1e-3
        torch.manual_seed(inputs.seed_for(12))
        upd.normal_(0.0, 0.05)
        steps_u = 3
        dec_ms = upd_s = 0.0
        rebuilt_u = 0
        for step in range(steps_u):
            for gi, (g, (bl, dsts)) in enumerate(zip(groups, plans)):
                _, ms = timed_region(torch, stream, lambda: nz.neuzip_decompress_batch(bl, dsts), 1)
                dec_ms += ms
                grads = [upd[(d.data_ptr() - big.data_ptr()) // 2: (d.data_ptr() - big.data_ptr()) // 2 + d.numel()]
                         for d in dsts]
                check = gi in (0, len(groups) - 1)
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
            "steps": steps_u, "tensors": len(blobs), "lr": lr5, "tensors_rebuilt": rebuilt_u,
            "decompress_GBps_output": round(2.0 * total * steps_u / (dec_ms * 1e-3) / 1e9, 1),
            "weight_step_GBps_weights": round(2.0 * total * steps_u / upd_s / 1e9, 1),
            "codec_ms_per_step": round((dec_ms * 1e-3 + upd_s) / steps_u * 1e3, 2),
            "bitwise_check": "first and last group of every step against torch's float32 step"}
        result["extended"] = ext

    # ---------------------------------------------------------------- optional: size sweep (Fig. 4's axis)
    if args.sweep:
        rows = []
        for nbytes in (1e5, 3e5, 1e6, 3e6, 1e7, 3e7, 1e8):
            ne = int(nbytes) // 2 // 8 * 8
            t = inputs.gaussian_bf16(ne, inputs.seed_for(6, int(math.log10(nbytes) * 10)), device=dev)
            o = torch.empty_like(t)
            row = {"bytes": 2 * ne}
            gib = 2.0 * ne / 2 ** 30
            for k in (7, 3):
                bk = nz.neuzip_compress(t, k)
                for _ in range(3):
                    nz.neuzip_decompress(bk, o)
                _, ms = timed_region(torch, stream, lambda: nz.neuzip_decompress(bk, o), 50)
                row[f"decompress_k{k}_GiBps"] = round(gib / (ms / 50 * 1e-3), 1)
                for _ in range(2):
                    nz.neuzip_compress(t, k, blob=bk)
                torch.cuda.synchronize()
                t0 = time.perf_counter()
                for _ in range(10):
                    nz.neuzip_compress(t, k, blob=bk)
                torch.cuda.synchronize()
                row[f"compress_k{k}_GiBps"] = round(gib / ((time.perf_counter() - t0) / 10), 1)
                nz.neuzip_free(bk)
            _, ms = timed_region(torch, stream, lambda: o.copy_(t), 50)
            row["device_copy_GiBps"] = round(gib / (ms / 50 * 1e-3), 1)
            # the paper's CPU-offloading baseline: the matrix leaves for pinned host memory and comes back
            host = torch.empty(ne, dtype=torch.bfloat16, pin_memory=True)
            for _ in range(2):
                host.copy_(t, non_blocking=True)
                o.copy_(host, non_blocking=True)
            _, ms_out = timed_region(torch, stream, lambda: host.copy_(t, non_blocking=True), 10)
            _, ms_in = timed_region(torch, stream, lambda: o.copy_(host, non_blocking=True), 10)
            row["offload_to_host_GiBps"] = round(gib / (ms_out / 10 * 1e-3), 1)
            row["reload_from_host_GiBps"] = round(gib / (ms_in / 10 * 1e-3), 1)
            rows.append(row)
            del t, o, host
        result["size_sweep"] = rows

    print(json.dumps(result), flush=True)


if __name__ == "__main__":
    main()
