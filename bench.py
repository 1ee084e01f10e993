#!/usr/bin/env python3
"""Benchmark of the NUQSGD compression hot path on one MI355X.

A step is one pass of the whole path over one batch of synthetic gradients: fused
norms + quantize + ENCODE of each of the K workers' gradients, then DECODE + average of the K
messages.  The default workload is the benchmark's configs[2] (ResNet-50-shaped, 25.6 M fp32
parameters, K = 8, bucket 8192, s = 3), the configuration the >= 50 % HBM target is quoted on.

Prints one JSON line:
  value      = fp32-in GB/s of the whole step: 4*d*K bytes of gradients pushed through
               encode and decode+average, inputs resident in HBM, per wall second of the step
  roofline   = the fused quantize+encode kernel (dominant by time), algorithmic bytes per launch
               over its mean launch duration from HIP events recorded on its stream
  cpu_baseline = the CPU oracle timed on a bounded sample of the same workload on this host: its buckets dealt out
               to all cores (value, cores), and on one thread (one_thread)
  per_config = the other four workloads of the benchmark spec measured in the same process (default run only)
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

HBM_PEAK_GBS = 8000.0   # MI355X HBM3E, published


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--config", type=int, default=3, help="workload 1..5 (BASELINE.json configs, 1-based)")
    ap.add_argument("--sync-stride", type=int, default=None,
                    help="decoder index stride in coordinates (0 = none); default 256, or 128 for buckets below 1024")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also launch one plain 1 GiB device copy before the timed region (a known-size reference "
                         "for hardware-counter runs)")
    ap.add_argument("--levels", default="nuq",
                    help="level sequence: nuq (the paper's main scheme, levels 2^(j-1-s): the default path), "
                         "uniform (QSGD's grid) or exp:P (0, P^s, ..., P, 1); anything but nuq runs the level-table "
                         "entry points")
    ap.add_argument("--fixed-bits", type=int, default=0,
                    help="b in 3..8: fixed-width coding (sign and level index in b bits per coordinate, the paper's "
                         "\"4-bit\"/\"8-bit\" variants) instead of the ERC bit strings; with --levels / --norm: QSGD and QSGDinf at fixed width")
    ap.add_argument("--huffman", action="store_true",
                    help="Huffman-coded levels (the paper's \"encoded\" variant) instead of the ERC bit strings: per "
                         "fused norms + quantizer + Huffman coding; decode to level bytes and one averaging kernel; "
                         "the code is built once from worker 0's level histogram; main scheme's levels only")
    ap.add_argument("--huffman-two-kernels", action="store_true",
                    help="with --huffman: decode to level bytes, then average them (two launches and K x d bytes in "
                         "between) instead of the fused decoder")
    ap.add_argument("--update", default="none", choices=["none", "sgd", "momentum", "momentum-unfused"],
                    help="what the receiver does with the average: none (write it out: the default path), sgd "
                         "(Alg. 1's aggregate step: the decoder adds -alpha/K times the sum onto the parameters in the "
                         "same launch), momentum (the decoder applies the momentum rule of Sec. 4.2 to the parameters and "
                         "y^l in the same launch) or momentum-unfused (the average, then the rule in one more kernel); "
                         "main scheme and ERC coding only")
    ap.add_argument("--norm", default="l2", choices=["l2", "linf"],
                    help="bucket norm for a level table: Euclidean, or maximum (QSGDinf with --levels uniform)")
    ap.add_argument("--reference-kernels", action="store_true",
                    help="also time PyTorch's own sum, copy and fill over a tensor of the step's input size and add "
                         "them to the line as `reference` (what library streaming kernels reach on this GPU: context "
                         "for the roofline fractions, not a target)")
    ap.add_argument("--graph", action="store_true",
                    help="capture one step into a HIP graph and time replays of it (the step's launches without the "
                         "host's launch gaps); the per-kernel HIP-event brackets then come from eager steps after the "
                         "timed region, since events cannot be read back from inside a graph")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-per-config", action="store_true",
                    help="only the workload --config names (the default run also measures the other four workloads of "
                         "BASELINE.json, with fewer steps, and attaches them as per_config)")
    ap.add_argument("--per-worker-calls", action="store_true",
                    help="encode with K nuq_quantize_encode calls instead of one nuq_quantize_encode_batch")
    return ap.parse_args()


def main():
    args = parse_args()
    if args.gpus != 1:
        print("bench.py measures one GPU: this build has no multi-GPU path (run with --gpus 1)", file=sys.stderr)
        sys.exit(2)
    import torch
    if not torch.cuda.is_available():
        print("bench.py needs a GPU", file=sys.stderr)
        sys.exit(2)
    result = measure(args, args.config, args.steps, args.warmup, None if args.no_cpu_baseline else 300_000_000)
    plain = (args.levels == "nuq" and args.norm == "l2" and not args.fixed_bits and not args.huffman
             and args.update == "none" and not args.graph and not args.per_worker_calls)
    if plain and not args.no_per_config:
        # the other four workloads of the benchmark spec in the same process (fewer steps, a smaller oracle sample), and
        # what a launch costs at the least: the floor under the small one-worker workloads
        result["launch_floor_ms"] = launch_floor(torch)
        result["per_config"] = {}
        for cfg in (1, 2, 3, 4, 5):
            if cfg == args.config:
                continue
            torch.cuda.empty_cache()
            r = measure(args, cfg, max(3, min(args.steps, 10)), min(args.warmup, 2),
                        None if args.no_cpu_baseline else 60_000_000)
            result["per_config"]["config%d" % cfg] = {k: r[k] for k in ("config", "value", "unit", "steps", "ms_per_step",
                                                                        "phases", "bits_per_coord", "roofline",
                                                                        "roofline_decode", "cpu_baseline") if k in r}
    print(json.dumps(result))


def launch_floor(torch):
    """Milliseconds per launch of the library's smallest kernel (norm of one coordinate), 200 back to back."""
    import paper_1908_06077_amd as nuq
    dev = torch.device("cuda:0")
    v = torch.ones(1, dtype=torch.float32, device=dev)
    out = torch.empty(1, dtype=torch.float32, device=dev)
    for _ in range(10):
        nuq.nuq_bucket_norms(v, 1, out)
    a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    a.record()
    for _ in range(200):
        nuq.nuq_bucket_norms(v, 1, out)
    b.record()
    torch.cuda.synchronize()
    return round(a.elapsed_time(b) / 200, 5)


def measure(args, config, steps, warmup, cpu_budget):
    """One workload: `warmup` untimed steps, `steps` timed ones, phase split, rooflines; the result as a dict."""
    import numpy as np
    import torch

    import paper_1908_06077_amd as nuq
    import workloads

    dev = torch.device("cuda:0")
    w = workloads.workload(config)
    d, n, s, K = w.d, w.bucket, w.s, w.K
    S = args.sync_stride if args.sync_stride is not None else workloads.sync_stride(w)
    if n <= S:
        S = 0
    B = nuq.nuq_num_buckets(d, n)
    nsync = nuq.nuq_huffman_num_sync(n, S) if args.huffman else nuq.nuq_num_sync(n, S)

    grads = [workloads.generate(w, k, dev) for k in range(K)]
    ws = torch.empty(nuq.nuq_encode_workspace_bytes(K, d, n, s), dtype=torch.uint8, device=dev)
    seeds = [w.quant_seed(k) for k in range(K)]
    # size the word buffers from a first encode into 16-word buffers (the capacity flag is expected; offsets are
    # complete); worst-case capacity would be ~1 B/coord per worker
    def new_msg(nwords):
        return nuq.Message(torch.empty(B, dtype=torch.float32, device=dev),
                           torch.empty(B + 1, dtype=torch.int64, device=dev),
                           torch.zeros(nwords, dtype=torch.int32, device=dev),
                           torch.empty(max(1, B * nsync), dtype=torch.int32, device=dev))
    # a level table only when one is asked for: the default is the main scheme's own entry points
    lev = None
    if args.levels != "nuq" or args.norm != "l2":
        kind, _, pstr = args.levels.partition(":")
        lev = workloads.level_table("exp" if kind in ("nuq", "exp") else kind, s, float(pstr) if pstr else 0.5)
    norm_kind = nuq.NORM_LINF if args.norm == "linf" else nuq.NORM_L2

    def encode_batch(messages):
        if lev is not None:
            nuq.nuq_quantize_encode_table_batch(grads, n, lev, norm_kind, seeds, S, messages, ws)
        else:
            nuq.nuq_quantize_encode_batch(grads, n, s, seeds, S, messages, ws)

    fb = args.fixed_bits
    huff = args.huffman
    if huff:
        if lev is not None or fb:
            print("--huffman goes with the main scheme's levels and no other coding", file=sys.stderr)
            sys.exit(2)
        hq = [torch.empty(d, dtype=torch.uint8, device=dev) for _ in range(K)]          # quantizer output
        hback = ([torch.empty(d, dtype=torch.uint8, device=dev) for _ in range(K)]      # decoder output
                 if args.huffman_two_kernels else None)
        hnorms = [torch.empty(B, dtype=torch.float32, device=dev) for _ in range(K)]
        hws = torch.empty(nuq.nuq_encode_huffman_batch_workspace_bytes(K, d, n, s), dtype=torch.uint8, device=dev)
        nuq.nuq_bucket_norms(grads[0], n, hnorms[0])
        nuq.nuq_quantize(grads[0], n, s, seeds[0], hnorms[0], hq[0])
        hhist = torch.empty(16, dtype=torch.int64, device=dev)
        nuq.nuq_level_histogram(hq[0], hhist)
        hlen = nuq.nuq_huffman_lengths([int(x) for x in hhist.cpu().numpy()[: s + 2]], s)
        msgs = [new_msg(nuq.nuq_huffman_max_words(d, n) // 4) for _ in range(K)]       # 4 bits/coord of room
    elif fb:
        wpb = (n * fb + 31) // 32
        fnorms = [torch.empty(B, dtype=torch.float32, device=dev) for _ in range(K)]
        fpacked = [torch.empty(nuq.nuq_fixed_words(d, n, fb), dtype=torch.int32, device=dev) for _ in range(K)]
        msgs = []
    else:
        probes = [new_msg(16) for _ in range(K)]
        encode_batch(probes)
        nuq.nuq_last_error_flags()
        msgs = [new_msg((int(p.bit_off[-1].item()) + 31) // 32 + 64) for p in probes]
        del probes
    out = torch.empty(d, dtype=torch.float32, device=dev)
    plain_decoder = lev is None and not fb and not huff and args.update == "none"
    upd = args.update
    if upd != "none":
        if huff or fb or lev is not None:
            print("--update goes with the main scheme and the ERC coding", file=sys.stderr)
            sys.exit(2)
        alpha, mu, nesterov_l = 0.1, 0.9, 1.0
        params = torch.empty(d, dtype=torch.float32, device=dev).normal_()
        yl = params.clone()

    def encode_all():
        if huff:
            nuq.nuq_quantize_encode_huffman_batch(grads, n, s, seeds, S, hlen, msgs, hws)
        elif fb and lev is not None:
            nuq.nuq_quantize_pack_fixed_table_batch(grads, n, lev, norm_kind, fb, seeds, fnorms, fpacked)
        elif fb:
            nuq.nuq_quantize_pack_fixed_batch(grads, n, s, fb, seeds, fnorms, fpacked)
        elif lev is not None:
            encode_batch(msgs)
        elif args.per_worker_calls:
            for k in range(K):
                m = msgs[k]
                nuq.nuq_quantize_encode(grads[k], n, s, seeds[k], S, m.norms, m.bit_off, m.words, m.sync, ws)
        else:
            nuq.nuq_quantize_encode_batch(grads, n, s, seeds, S, msgs, ws)

    def decode_all():
        if huff and hback is not None:
            nuq.nuq_decode_huffman_batch(msgs, d, n, s, S, hlen, hback)
            nuq.nuq_average_levels([m.norms for m in msgs], hback, d, n, s, 1.0 / K, False, out)
        elif huff:
            nuq.nuq_decode_accumulate_huffman(msgs, d, n, s, S, hlen, 1.0 / K, False, out)
        elif fb and lev is not None:
            nuq.nuq_unpack_accumulate_fixed_table(fnorms, fpacked, d, n, lev, fb, 1.0 / K, False, out)
        elif fb:
            nuq.nuq_unpack_accumulate_fixed(fnorms, fpacked, d, n, s, fb, 1.0 / K, False, out)
        elif lev is not None:
            nuq.nuq_decode_accumulate_table(msgs, d, n, lev, S, 1.0 / K, False, out)
        elif upd == "sgd":
            nuq.nuq_decode_accumulate(msgs, d, n, s, S, -alpha / K, True, params)
        elif upd == "momentum":
            nuq.nuq_decode_momentum_step(msgs, d, n, s, S, 1.0 / K, alpha, mu, nesterov_l, params, yl)
        else:
            nuq.nuq_decode_accumulate(msgs, d, n, s, S, 1.0 / K, False, out)
            if upd == "momentum-unfused":
                nuq.nuq_momentum_step(params, yl, out, alpha, mu, nesterov_l)

    def step():
        encode_all()
        decode_all()

    if args.calibrate_copy:
        src = torch.empty(1 << 28, dtype=torch.float32, device=dev).normal_()
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
    for _ in range(warmup):
        step()
    torch.cuda.synchronize()
    assert nuq.nuq_last_error_flags() == 0, "device error flags raised during warmup"

    # the timed region: K steps, with the library's per-launch HIP-event brackets (on its launch stream) switched on
    if args.graph:
        graph = torch.cuda.CUDAGraph()
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            with torch.cuda.graph(graph, stream=side):
                step()
        torch.cuda.current_stream().wait_stream(side)
        graph.replay()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(steps):
            graph.replay()
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        nuq.nuq_timing_begin(min(4096, steps * (4 * K + 2)))
        for i in range(steps):
            step()
        torch.cuda.synchronize()
    else:
        nuq.nuq_timing_begin(min(4096, steps * (4 * K + 2)))
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(steps):
            step()
        torch.cuda.synchronize()
        t1 = time.perf_counter()
    launches = nuq.nuq_timing_collect()
    assert nuq.nuq_last_error_flags() == 0, "device error flags raised during the timed region"

    # phase split, outside the timed region: events around the two library calls of a few more steps
    ev = [[torch.cuda.Event(enable_timing=True) for _ in range(3)] for _ in range(min(steps, 10))]
    for e in ev:
        e[0].record()
        encode_all()
        e[1].record()
        decode_all()
        e[2].record()
    torch.cuda.synchronize()

    ms_step = (t1 - t0) * 1e3 / steps
    ms_enc = float(np.median([e[0].elapsed_time(e[1]) for e in ev]))
    ms_dec = float(np.median([e[1].elapsed_time(e[2]) for e in ev]))
    in_bytes = 4.0 * d * K
    value = in_bytes / (ms_step * 1e-3) / 1e9

    # message sizes -> bits per coordinate and algorithmic bytes
    if fb:
        W = [B * wpb] * K
        paper_bits = (32.0 * B + float(fb) * d) / d
        wire_bits = (32.0 * B + 32.0 * B * wpb) / d
        enc_alg = [4.0 * d + 4 * B + 4 * Wk for Wk in W]                                    # per worker
        dec_alg = sum(4.0 * Wk + 4 * B for Wk in W) + 4.0 * d                               # per launch
    else:
        total_bits = [int(m.bit_off[-1].item()) for m in msgs]
        starts = [(m.bit_off[:-1] + 31) // 32 * 32 for m in msgs]
        payload_bits = [int((m.bit_off[1:] - st).sum().item()) for m, st in zip(msgs, starts)]
        W = [(tb + 31) // 32 for tb in total_bits]
        paper_bits = float(np.mean([(32 * B + pb) / d for pb in payload_bits]))
        wire_bits = float(np.mean([(32 * Wk + 32 * B + 64 * (B + 1) + 32 * B * nsync) / d for Wk in W]))
        enc_alg = [4.0 * d + 4 * B + 8 * (B + 1) + 4 * Wk + 4 * B * nsync for Wk in W]      # per worker
        dec_alg = sum(4.0 * Wk + 12 * B + 4 * B * nsync for Wk in W) + 4.0 * d               # per launch
    if huff:
        enc_ms = [t for e, t in launches if e == nuq.T_QUANTIZE_ENCODE]
        dec_ms = [t for e, t in launches if e == nuq.T_DECODE]
    else:
        enc_ms = [t for e, t in launches if e == nuq.T_QUANTIZE_ENCODE]
        dec_ms = [t for e, t in launches if e == nuq.T_DECODE]
    enc_kernel_ms = float(np.mean(enc_ms))
    dec_kernel_ms = float(np.mean(dec_ms))
    enc_launch_bytes = float(np.mean(enc_alg)) if args.per_worker_calls else float(sum(enc_alg))
    enc_gbs = enc_launch_bytes / (enc_kernel_ms * 1e-3) / 1e9
    dec_gbs = dec_alg / (dec_kernel_ms * 1e-3) / 1e9

    result = {
        "metric": "quantize+encode and decode+avg GB/s (fp32 in) + % HBM peak; bits/coord",
        "value": round(value, 2),
        "unit": "GB/s",
        "n_gpus": 1,
        "steps": steps,
        "warmup": warmup,
        "ms_per_step": round(ms_step, 4),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f32",
        "data": "synthetic",
        "config": {"workload": "configs[%d] %s: d=%d fp32, bucket=%d, s=%d, K=%d workers, sync_stride=%d%s"
                               % (config - 1, w.name, d, n, s, K, S,
                                  ", Huffman-coded levels, lengths %s" % hlen if huff else
                                  (", fixed-width %d bits" % fb + ("" if lev is None else ", level table %s, %s norm"
                                                                    % (args.levels, args.norm))) if fb else
                                  "" if lev is None else ", level table %s, %s norm" % (args.levels, args.norm))},
        "phases": {
            "quantize_encode": {"ms": round(ms_enc, 4), "fp32_in_GBps": round(in_bytes / (ms_enc * 1e-3) / 1e9, 2),
                                "hbm_frac": round(sum(enc_alg) / (ms_enc * 1e-3) / 1e9 / HBM_PEAK_GBS, 4)},
            "decode_average": {"ms": round(ms_dec, 4), "fp32_GBps": round(in_bytes / (ms_dec * 1e-3) / 1e9, 2),
                               "hbm_frac": round(dec_alg / (ms_dec * 1e-3) / 1e9 / HBM_PEAK_GBS, 4)},
        },
        "bits_per_coord": {"paper": round(paper_bits, 4), "wire": round(wire_bits, 4)},
        "roofline": {"kernel": ("k_huffman_fused (norms+quantize+Huffman coding), one launch per step (all K workers)"
                                if huff else
                                "k_pack_fixed (fused norms+quantize+b-bit packing), one launch per step (all K workers)"
                                if fb else "k_encode (fused norms+quantize+ENCODE), one launch per %s"
                                % ("worker" if args.per_worker_calls else "step (all K workers)")),
                     "bound": "hbm", "achieved": round(enc_gbs, 2), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": round(enc_gbs / HBM_PEAK_GBS, 4),
                     "traffic": None if lev is not None or fb or huff else measured_traffic("k_encode", config, S),
                     "bytes_per_launch": round(enc_launch_bytes), "launch_ms": round(enc_kernel_ms, 5),
                     "launches": len(enc_ms)},
        "roofline_decode": {"kernel": ("k_huffman_decode_direct, all K messages in one launch (k_average_levels follows)"
                                       if huff and args.huffman_two_kernels else
                                       "k_decode_wave_huffman (decode + average of K Huffman-coded messages)" if huff else
                                       "k_unpack_accumulate_fixed (unpack + average of K messages)" if fb else
                                       "tile decoder k_decode_wave, or k_decode_single for one message (DECODE + average of K messages)"),
                            "bound": "hbm", "achieved": round(dec_gbs, 2), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                            "frac": round(dec_gbs / HBM_PEAK_GBS, 4),
                            "traffic": None if lev is not None or fb or huff or upd in ("sgd", "momentum")
                            else measured_traffic("k_decode_accumulate", config, S),
                            "bytes_per_launch": round(dec_alg), "launch_ms": round(dec_kernel_ms, 5),
                            "launches": len(dec_ms)},
    }

    if plain_decoder:
        # The decoder is bound by vector instruction issue, not memory: the same launch time against the chip's issue
        # rate (1024 SIMDs, a wave instruction per 4 clocks at 2.4 GHz), with the instruction count of the counter runs.
        insts = measured_traffic("k_decode_accumulate", config, S, "valu_insts")
        if insts:
            peak = 1024 * 2.4e9 / 4 / 1e9
            rate = insts / (dec_kernel_ms * 1e-3) / 1e9
            result["roofline_decode"]["issue"] = {"bound": "alu", "achieved": round(rate, 1), "peak": round(peak, 1),
                                                  "unit": "G wave-instructions/s", "frac": round(rate / peak, 4),
                                                  "instructions_per_launch": insts}
    if args.graph:
        result["config"]["launch"] = "one HIP graph replay per step; kernel brackets from eager steps after the timed region"
    if upd != "none":
        result["config"]["workload"] += ", parameter update: %s" % (
            "plain step inside the decoder" if upd == "sgd" else
            "momentum rule, mu=%g l=%g, %s" % (mu, nesterov_l, "inside the decoder" if upd == "momentum"
                                               else "in a kernel of its own"))
        if upd in ("sgd", "momentum"):
            # the decoder also reads the parameters (sgd), or reads and writes parameters and y^l instead of
            # writing the average (momentum)
            dec_upd = dec_alg + (4.0 if upd == "sgd" else 12.0) * d
            result["roofline_decode"].update(bytes_per_launch=round(dec_upd),
                                             achieved=round(dec_upd / (dec_kernel_ms * 1e-3) / 1e9, 2),
                                             frac=round(dec_upd / (dec_kernel_ms * 1e-3) / 1e9 / HBM_PEAK_GBS, 4))
        else:
            a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            a.record()
            for _ in range(20):
                nuq.nuq_momentum_step(params, yl, out, alpha, mu, nesterov_l)
            b.record()
            torch.cuda.synchronize()
            ms_mom = a.elapsed_time(b) / 20
            result["update"] = {"kernel": "k_momentum_step (reads w, y^l, average; writes w, y^l)", "bound": "hbm",
                                "ms": round(ms_mom, 5), "bytes_per_launch": 20 * d,
                                "achieved": round(20.0 * d / (ms_mom * 1e-3) / 1e9, 2), "peak": HBM_PEAK_GBS,
                                "unit": "GB/s", "frac": round(20.0 * d / (ms_mom * 1e-3) / 1e9 / HBM_PEAK_GBS, 4)}
    if args.reference_kernels:
        result["reference"] = reference_kernels(torch, d * K, dev)
    if cpu_budget:
        result["cpu_baseline"] = cpu_baseline(w, grads, S, lev, args.norm, fb, hlen if huff else None, cpu_budget)
    return result


def reference_kernels(torch, numel, dev):
    """PyTorch's own streaming kernels over `numel` floats (the step's input size): achieved HBM TB/s."""
    x = torch.empty(numel, dtype=torch.float32, device=dev).normal_()
    y = torch.empty_like(x)

    def timed(f, reps=20):
        f()
        torch.cuda.synchronize()
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        for _ in range(reps):
            f()
        b.record()
        torch.cuda.synchronize()
        return a.elapsed_time(b) / reps

    nbytes = 4.0 * numel
    out = {}
    for name, f, traffic in (("sum", lambda: x.sum(), nbytes), ("copy", lambda: y.copy_(x), 2 * nbytes),
                             ("fill", lambda: y.zero_(), nbytes)):
        ms = timed(f)
        out[name] = {"ms": round(ms, 4), "TBps": round(traffic / (ms * 1e-3) / 1e12, 2)}
    return out


def measured_traffic(kernel, config, S, field="bytes_per_launch"):
    """HBM bytes per launch of `kernel` from the hardware-counter runs recorded in profiles/hbm_traffic.json
    (rocprofv3 FETCH_SIZE and WRITE_SIZE, scaled by a plain copy of known size), or None if that file has no
    entry for this workload.  The counters cannot be read from inside this process."""
    path = os.path.join(ROOT, "profiles", "hbm_traffic.json")
    try:
        with open(path) as f:
            table = json.load(f)
    except (OSError, ValueError):
        return None
    entry = table.get("config%d_stride%d" % (config, S), {}).get(kernel)
    return None if entry is None else entry.get(field)


def cpu_baseline(w, grads, S, lev=None, norm="l2", fb=0, hlen=None, budget_coords=300_000_000):
    """The CPU oracle as it stands on a bounded sample of the same workload: once on one thread, once with the sample's
    buckets dealt out to all of the host's cores (buckets are independent: every thread runs the same sequential
    oracle calls on its own run of buckets of every worker; ctypes releases the interpreter lock during a call)."""
    import numpy as np
    import oracle
    from concurrent.futures import ThreadPoolExecutor

    d, n, s, K = w.d, w.bucket, w.s, w.K
    d_s = d if d * K <= budget_coords else max(n, (budget_coords // K) // n * n)
    host = [g[:d_s].cpu().numpy() for g in grads]
    nb = (d_s + n - 1) // n
    nproc = os.cpu_count() or 1
    # the GPU machines give a job 16 cores whatever the machine has
    threads = max(1, min(nproc, int(os.environ.get("OMP_NUM_THREADS", "16")), 16))

    def chunk(b_lo, b_hi):
        """Whole step on buckets [b_lo, b_hi): encode of each worker, then decode + average of the K messages."""
        c_lo, c_hi = b_lo * n, min(d_s, b_hi * n)
        t0 = time.perf_counter()
        parts = []
        for k in range(K):
            v = host[k][c_lo:c_hi]
            norms = (oracle.bucket_norms_linf if norm == "linf" else oracle.bucket_norms)(v, n).astype(np.float32)
            if lev is None:
                q = oracle.quantize(v, n, s, w.quant_seed(k), norms, b_lo)
            else:
                q = oracle.quantize_table(v, n, lev, w.quant_seed(k), norms, b_lo)
            if fb:
                parts.append((norms, oracle.pack_fixed(q, n, s, fb), None))
            elif hlen is not None:
                bo, words, _ = oracle.encode_huffman(q, n, s, hlen, S)
                parts.append((norms, bo, words))
            else:
                bo, words, _ = oracle.encode(q, n, s, S)
                parts.append((norms, bo, words))
        t1 = time.perf_counter()
        m = c_hi - c_lo
        if hlen is not None:
            acc = np.zeros(m)
            for norms, bo, words in parts:
                acc += oracle.dequantize(oracle.decode_huffman(bo, words, m, n, s, hlen), n, s, norms)
            acc *= 1.0 / K
        elif fb and lev is not None:
            acc = np.zeros(m)
            for norms, packed, _ in parts:
                acc += oracle.dequantize_table(oracle.unpack_fixed(packed, m, n, s, fb), n, lev, norms)
            acc *= 1.0 / K
        elif fb:
            oracle.unpack_average_fixed([p[0] for p in parts], [p[1] for p in parts], m, n, s, fb, 1.0 / K)
        elif lev is None:
            oracle.decode_average([p[0] for p in parts], [p[1] for p in parts], [p[2] for p in parts], m, n, s, 1.0 / K)
        else:
            oracle.decode_average_table([p[0] for p in parts], [p[1] for p in parts], [p[2] for p in parts], m, n, lev,
                                        1.0 / K)
        return t1 - t0, time.perf_counter() - t1

    # runs of buckets: a few per thread, so that the threads finish together
    nchunks = max(1, min(nb, 4 * threads))
    edges = [nb * i // nchunks for i in range(nchunks + 1)]
    runs = [(edges[i], edges[i + 1]) for i in range(nchunks) if edges[i + 1] > edges[i]]
    in_bytes = 4.0 * d_s * K
    t0 = time.perf_counter()
    split = [chunk(lo, hi) for lo, hi in runs]
    t_one = time.perf_counter() - t0
    with ThreadPoolExecutor(max_workers=threads) as pool:
        t0 = time.perf_counter()
        list(pool.map(lambda r: chunk(*r), runs))
        t_all = time.perf_counter() - t0
    return {"value": round(in_bytes / t_all / 1e9, 4), "unit": "GB/s", "cores": threads, "kind": "oracle",
            "nproc": nproc,
            "one_thread": {"value": round(in_bytes / t_one / 1e9, 4), "unit": "GB/s", "cores": 1,
                           "encode_s": round(sum(x[0] for x in split), 2),
                           "decode_average_s": round(sum(x[1] for x in split), 2)},
            "sample": "same workload, first %d of %d coordinates of each of the %d workers, whole step (encode, then "
                      "decode + average), in %d runs of buckets: %.2f s on one thread, %.2f s on %d threads"
                      % (d_s, d, K, len(runs), t_one, t_all, threads)}


if __name__ == "__main__":
    main()
