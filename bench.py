#!/usr/bin/env python3
"""Benchmark of the OCTOPUS hot path on one MI355X.

One step = one pass of the whole hot path over one batch of synthetic input resident in HBM:
prefill-time encode of every cached token (octopus_encode) followed by one decode-attention step
over the compressed cache (octopus_attn_decode: query rotation, fused split-K kernel, merge).

Headline workload: the Llama-3-8B-shaped GQA decode configuration (batch 16, 32 query heads over 8 KV
heads, head_dim 128, 32768 cached tokens per sequence, bf16 keys / values / queries, 3 bits per
coordinate).

Prints ONE JSON line.  `value` is the effective HBM rate of the decode-attention call: algorithmic
bytes (per key: the 58-byte canonical record + the 256-byte bf16 value row; plus queries and outputs)
divided by the call's average duration over the timed steps, measured with events on the launch stream.
`roofline` is the same byte count over the fused kernel's own duration (events recorded by the library
around its launch), against the published 8 TB/s.  `workloads` holds the other named configurations
(30 warm-up + 50 timed calls, median: the protocol of the paper's kernel table), `variants_on_llama3_8b_decode` the
optional pieces (QJL residual, quantised values, window, paged cache) on the headline shape, `encode_roofline` the
encoder against the fp32 vector issue rate, `cpu_baseline` the oracle on the host cores.
"""
import argparse
import ctypes
import hashlib
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X published HBM3E bandwidth
KERNEL_EVENT_STRIDE = 4        # every 4th timed step carries the event pair around the dominant kernel
FP32_VALU_PEAK_TFLOPS = 157.3  # MI355X published fp32 vector peak (packed fp32; 2 flops per lane-op)
# fp32 lane-operations per second without packed math (this library builds with packed fp32 off):
# 256 compute units x 4 SIMDs x 16 lanes x 2.4 GHz = a quarter of the published flop rate
FP32_LANE_OPS_PER_S = FP32_VALU_PEAK_TFLOPS * 1e12 / 4.0
BF16_MFMA_PEAK_TFLOPS = 2500.0 # MI355X published dense bf16 matrix peak
PROTOCOL_WARMUP, PROTOCOL_TIMED = 30, 50   # App. G: 30 warm-up + 50 timed iterations, median


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="llama3_8b_decode")
    ap.add_argument("--bits", type=float, default=None,
                    help="bits per coordinate (1, 1.5, 2, 2.5, 3, 4) instead of the workload's own")
    ap.add_argument("--pair", default="",
                    help="BD:BN - an explicit (b_dir, b_nrm) pair of the bit-allocation sweep of App. D instead of a nominal "
                         "bit width (octopus_build_codebooks_pair); workloads of head_dim 128, plain variant")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-extras", action="store_true",
                    help="skip the `workloads` block (the other named configurations) and the `variants_on_...` block")
    ap.add_argument("--seed", type=int, default=0)
    ap.add_argument("--rounding", type=int, default=1,
                    help="encoder rounding mode (App. E): 0 seed only, 1 local 3x3 (default), 2 full grid, "
                         "3 independent rounds, 4 local 2x2; the decoder is the same")
    ap.add_argument("--vq", default="",
                    help="BITS:GROUP, e.g. 3:32 - quantise the values per group (octopus_encode_values in the encode "
                         "phase) and decode over them (octopus_attn_decode_vq); single-query workloads only")
    ap.add_argument("--window", type=int, default=0,
                    help="hybrid cache: keep the last WINDOW tokens of every sequence at native precision "
                         "(octopus_attn_decode_hybrid); single-query workloads, plain variant only")
    ap.add_argument("--qjl", action="store_true",
                    help="time the variant with the 1-bit QJL residual (octopus_encode_qjl + octopus_attn_decode_qjl); "
                         "single-query workloads only")
    ap.add_argument("--paged", action="store_true",
                    help="paged cache: 64-token pages handed out in a random order from pools (octopus_encode_paged + "
                         "octopus_attn_decode_paged); single-query bf16 workloads, plain variant or with --vq "
                         "(octopus_encode_values_paged + octopus_attn_decode_paged_vq)")
    ap.add_argument("--read-probe", action="store_true",
                    help="instead of the benchmark: time a plain streaming read of 1.25 GiB (octopus_probe_read), with and "
                         "without the non-temporal hint, and print the rates: the read rate this machine reaches with "
                         "nothing else to do, to set beside the published peak")
    ap.add_argument("--calibration-copy", action="store_true",
                    help="also run a plain 1 GiB device-to-device copy (torch) three times, so that a rocprofv3 "
                         "--pmc run of this command can scale FETCH_SIZE / WRITE_SIZE by a kernel of known size")
    return ap.parse_args()


def encode_lane_ops_per_key(head_dim):
    """Algorithmic fp32 lane-operations of Alg. 1 per key: the Walsh-Hadamard butterflies (d log2 d add / sub), norm,
    scale and sign flip (3 d), and per triplet the octahedral map with the two seed searches (14), nine candidate
    evaluations of 3 multiply-adds + compare + select + index (9 x 6) and the norm index + packing (8)."""
    n_tri = (head_dim + 2) // 3
    return head_dim * (head_dim.bit_length() - 1) + 3 * head_dim + n_tri * (14 + 9 * 6 + 8)


def set_omp_threads(n):
    try:
        ctypes.CDLL("libgomp.so.1").omp_set_num_threads(int(n))
        return True
    except OSError:
        return False


def cpu_baseline(wl, keys, vals, q, signs, scale, record_bytes, budget_s=12.0, signs2=None, mode=1, vq=None, pair=None):
    """The oracle as it stands, timed on this machine's host cores on a bounded sample of the workload:
    whole sequences (all KV heads, all cached tokens; encode, then attention of each KV head's group of
    query heads over its tokens), one sequence after another until about `budget_s` seconds are spent;
    then one (sequence, KV head) pair once more on a single thread."""
    import numpy as np

    import oracle

    plan = oracle.make_plan_pair(wl.head_dim, *pair) if pair else oracle.make_plan(wl.head_dim, wl.bits)
    g = wl.n_q_heads // wl.n_kv_heads
    n_tok = wl.n_tokens
    oracle.encode(plan, np.zeros((64, wl.head_dim)), signs[0])               # load the library
    enc_s = dec_s = 0.0
    n_seq_done = 0
    for s in range(wl.n_seq):
        k_host = keys[s, :n_tok].float().cpu().numpy().astype(np.float64)    # [n_tok, n_kv, d]
        v_host = vals[s].float().cpu().numpy().astype(np.float64)            # [n_kv, n_tok, d]
        nq_s = min(wl.n_q, 4)                                                # a few queries of a chunk
        q_host = q[s, :nq_s].float().cpu().numpy().astype(np.float64)        # [nq_s, n_qh, d]
        k_heads = [np.ascontiguousarray(k_host[:, h]) for h in range(wl.n_kv_heads)]
        t0 = time.perf_counter()
        recs = [oracle.encode(plan, k_heads[h], signs[h], mode=mode) for h in range(wl.n_kv_heads)]   # same numbering
        if vq is not None:      # quantise and dequantise the values as the value codec does
            v_host = [oracle.vq_decode(oracle.vq_encode(v_host[h][:n_tok], vq[0], vq[1]), wl.head_dim, vq[0], vq[1])
                      for h in range(wl.n_kv_heads)]
        if signs2 is not None:
            side = [oracle.qjl_encode(plan, k_heads[h], signs[h], signs2[h], recs[h]) for h in range(wl.n_kv_heads)]
        t1 = time.perf_counter()
        for h in range(wl.n_kv_heads):
            qq = q_host[:, h * g:(h + 1) * g].reshape(-1, wl.head_dim)
            if signs2 is not None:
                oracle.attention_qjl(plan, recs[h], signs[h], signs2[h], side[h][0], side[h][1], qq, v_host[h][:n_tok],
                                     scale)
            else:
                oracle.attention(plan, recs[h], signs[h], qq, v_host[h][:n_tok], scale)
        t2 = time.perf_counter()
        enc_s += t1 - t0
        dec_s += t2 - t1
        n_seq_done += 1
        if enc_s + dec_s >= budget_s:
            break
    n_keys = n_seq_done * n_tok * wl.n_kv_heads
    elt = 2 if wl.dtype == "bf16" else 4
    v_bytes = oracle.vq_row_bytes(wl.head_dim, vq[0], vq[1]) if vq is not None else wl.head_dim * elt
    key_bytes = record_bytes + v_bytes + (wl.head_dim // 8 + 2 if signs2 is not None else 0)
    dec_bytes = n_keys * key_bytes
    threads = int(os.environ.get("OMP_NUM_THREADS", os.cpu_count() or 1))
    result = {
        "value": round(dec_bytes / dec_s / 1e9, 4),
        "unit": "GB/s",
        "cores": min(threads, os.cpu_count() or threads),
        "kind": "oracle",
        "sample": f"{n_seq_done} of {wl.n_seq} sequences of the workload, each {wl.n_kv_heads} KV heads x {n_tok} "
                  f"tokens ({n_keys} keys in all), {g} query heads per KV head"
                  + (f", {min(wl.n_q, 4)} of the {wl.n_q} queries" if wl.n_q > 1 else "")
                  + "; fp64 oracle, OpenMP over keys",
        "decode_seconds": round(dec_s, 3),
        "encode_seconds": round(enc_s, 3),
        "encode_mtokens_per_s": round(n_seq_done * n_tok / enc_s / 1e6, 4),
    }
    # the same code on ONE thread, on one (sequence, KV head) pair of the sample (plain variant)
    if signs2 is None and vq is None and set_omp_threads(1):
        n1 = min(n_tok, 32768)
        t0 = time.perf_counter()
        rec1 = oracle.encode(plan, k_heads[0][:n1], signs[0], mode=mode)
        t1 = time.perf_counter()
        oracle.attention(plan, rec1, signs[0], q_host[:, :g].reshape(-1, wl.head_dim), v_host[0][:n1], scale)
        t2 = time.perf_counter()
        set_omp_threads(threads)
        result["one_thread"] = {
            "sample": f"one (sequence, KV head) pair, {n1} keys, {g} query heads" + (f" x {nq_s} queries" if wl.n_q > 1 else ""),
            "encode_seconds": round(t1 - t0, 3), "decode_seconds": round(t2 - t1, 3),
            "decode_gb_per_s": round(n1 * key_bytes / (t2 - t1) / 1e9, 4),
            "encode_mkeys_per_s": round(n1 / (t1 - t0) / 1e6, 4),
            # the whole workload on one thread at this rate (keys scale linearly)
            "whole_workload_seconds_extrapolated": round((t2 - t0) * (wl.n_seq * wl.n_kv_heads * n_tok / n1), 1),
        }
    return result


def kernel_source_digest(kernel="decode_kernel_mfma"):
    """First 16 hex digits of the SHA-256 of the sources of a decode kernel: what a traffic summary under
    profiles/ records, so that a summary measured on other code is not reported as this build's."""
    names = ["octopus_decode.hpp", "octopus_decode_mq.hpp", "octopus_device.hpp"]
    if kernel == "decode_kernel_vq_mfma":
        names.append("octopus_decode_vq.hpp")
    h = hashlib.sha256()
    for name in names:
        with open(os.path.join(ROOT, "paper_2605_21226_amd", "csrc", name), "rb") as f:
            h.update(f.read())
    return h.hexdigest()[:16]


def measured_traffic(workload, kernel="decode_kernel_mfma", profiles_dir=None):
    """HBM bytes per launch of the dominant decode kernel as measured with rocprofv3 --pmc FETCH_SIZE /
    WRITE_SIZE (scaled by a plain copy of known size); read from the committed profile summary of this
    kernel and workload.  -> (bytes or None, note).  None when there is no summary or when it was taken on
    other kernel sources than the ones in this tree (KERNEL_SOURCE_SHA in the summary)."""
    path = os.path.join(profiles_dir or os.path.join(ROOT, "profiles"), f"{kernel}_{workload}_traffic.txt")
    try:
        vals = {}
        with open(path) as f:
            for line in f:
                if "=" in line and not line.startswith("#"):
                    k, v = line.split("=", 1)
                    vals[k.strip()] = v.strip()
        total = int(float(vals["FETCH_BYTES_PER_LAUNCH"]) + float(vals["WRITE_BYTES_PER_LAUNCH"]))
    except (OSError, KeyError, ValueError):
        return None, "no traffic summary under profiles/ for this kernel and workload"
    sha, commit = vals.get("KERNEL_SOURCE_SHA"), vals.get("MEASURED_AT_COMMIT", "unknown")
    if sha != kernel_source_digest(kernel):
        return None, f"the traffic summary (commit {commit}) was taken on other kernel sources than this tree's"
    return total, f"rocprofv3 --pmc FETCH_SIZE + WRITE_SIZE, measured at commit {commit} on these kernel sources"


class Run:
    """One workload resident in device memory, with closures for its encode and decode calls."""

    def __init__(self, wl, args, dev, variants=True):
        import numpy as np
        import torch

        from paper_2605_21226_amd import binding, synth
        from paper_2605_21226_amd.synth_device import device_inputs

        self.wl, self.args, self.dev = wl, args, dev
        self.qjl = bool(args.qjl) and variants
        self.paged = bool(args.paged) and variants
        self.window = args.window if variants else 0
        self.rounding = args.rounding if variants else 1
        self.v_bits, self.v_group = ((int(x) for x in args.vq.split(":")) if (args.vq and variants) else (0, 0))
        self.many_rows = wl.n_q > 1
        self.pair = tuple(int(x) for x in args.pair.split(":")) if (args.pair and variants) else None
        self.cb = cb = (binding.octopus_build_codebooks_pair(wl.head_dim, *self.pair) if self.pair
                        else binding.octopus_build_codebooks(wl.head_dim, wl.bits))
        self.keys, self.vals, self.q, self.signs, lens = device_inputs(wl, args.seed, dev)
        self.cap = cap = -(-wl.n_tokens // 64) * 64
        if cap != wl.n_tokens:                      # the values need t_capacity rows
            padded = torch.zeros((wl.n_seq, wl.n_kv_heads, cap, wl.head_dim), dtype=self.vals.dtype, device=dev)
            padded[:, :, :wl.n_tokens] = self.vals
            self.vals = padded
        self.sbits = torch.from_numpy(synth.sign_bits(self.signs)).to(dev)
        self.cache = torch.zeros(binding.octopus_cache_bytes(cb, wl.n_seq, wl.n_kv_heads, cap), dtype=torch.uint8,
                                 device=dev)
        self.k_win = self.win_dev = None
        if self.window:
            # the last `window` tokens of every sequence stay uncompressed; the compressed part shrinks by as much
            win = np.minimum(lens, self.window).astype(np.int32)
            self.k_win = torch.zeros((wl.n_seq, wl.n_kv_heads, self.window, wl.head_dim), dtype=self.keys.dtype,
                                     device=dev)
            for s_i in range(wl.n_seq):
                a, b = int(lens[s_i] - win[s_i]), int(lens[s_i])
                self.k_win[s_i, :, :b - a] = self.keys[s_i, a:b].permute(1, 0, 2)
            lens = (lens - win).astype(np.int32)
            self.win_dev = torch.from_numpy(win).to(dev)
        self.lens = lens
        self.max_len = int(lens.max())
        self.ws = torch.empty(binding.octopus_attn_decode_workspace(cb, wl.n_seq, wl.n_q_heads, wl.n_kv_heads, wl.n_q,
                                                                    self.max_len), dtype=torch.uint8, device=dev)
        self.out = torch.zeros((wl.n_seq, wl.n_q, wl.n_q_heads, wl.head_dim), dtype=torch.float32, device=dev)
        self.lens_dev = torch.from_numpy(lens).to(dev)
        self.scale = 1.0 / float(np.sqrt(wl.head_dim))
        # single-query workloads: prefill-time encode of the whole cache; a chunk workload: the cache is
        # filled up to the chunk once, and a step encodes the chunk's tokens at their position
        self.n_new = wl.n_new if self.many_rows else wl.n_tokens
        self.first = wl.n_tokens - self.n_new
        self.start_dev = None
        if self.first > 0:
            binding.octopus_encode(cb, self.keys[:, :self.first], self.sbits, self.cache, cap)
            self.start_dev = torch.full((wl.n_seq,), self.first, dtype=torch.int32, device=dev)
        self.signs2 = self.s2bits = self.side = None
        if self.qjl:
            self.signs2 = synth.sign_vectors(args.seed + 1, wl.n_kv_heads, wl.head_dim)
            self.s2bits = torch.from_numpy(synth.sign_bits(self.signs2)).to(dev)
            self.side = torch.zeros(binding.octopus_qjl_bytes(cb, wl.n_seq, wl.n_kv_heads, cap), dtype=torch.uint8,
                                    device=dev)
        self.vq = self.vals_tok = None
        if self.v_bits:
            self.vq = torch.zeros(binding.octopus_vq_bytes(wl.head_dim, self.v_bits, self.v_group, wl.n_seq,
                                                           wl.n_kv_heads, cap), dtype=torch.uint8, device=dev)
            self.vals_tok = self.vals.permute(0, 2, 1, 3)[:, :wl.n_tokens]      # [n_seq, n_tokens, n_kv_heads, d] view
        self.table = self.k_pool = self.v_pool = None
        if self.paged:
            tiles = cap // 64
            self.n_pages = n_pages = wl.n_seq * tiles + 7
            gen = torch.Generator(device="cpu").manual_seed(args.seed + 5)
            self.table = (torch.randperm(n_pages, generator=gen)[:wl.n_seq * tiles].to(torch.int32)
                          .reshape(wl.n_seq, tiles).to(dev))
            self.k_pool = torch.zeros(binding.octopus_paged_pool_bytes(cb, n_pages, wl.n_kv_heads), dtype=torch.uint8,
                                      device=dev)
            self.v_pool = torch.zeros((n_pages, wl.n_kv_heads, 64, wl.head_dim), dtype=self.vals.dtype, device=dev)
            self.v_pool[self.table.reshape(-1).long()] = (
                self.vals.reshape(wl.n_seq, wl.n_kv_heads, tiles, 64, wl.head_dim).permute(0, 2, 1, 3, 4)
                .reshape(-1, wl.n_kv_heads, 64, wl.head_dim))
            if self.v_bits:   # quantised value pages instead (written by the encode phase)
                self.v_pool = None
                self.vq = torch.zeros(binding.octopus_vq_bytes(wl.head_dim, self.v_bits, self.v_group, n_pages,
                                                               wl.n_kv_heads, 64), dtype=torch.uint8, device=dev)

    def encode(self):
        from paper_2605_21226_amd import binding
        cb, cap = self.cb, self.cap
        if self.v_bits and self.paged:
            binding.octopus_encode_values_paged(self.vals_tok, self.v_bits, self.v_group, self.vq, self.wl.n_kv_heads,
                                                self.table)
        elif self.v_bits:
            binding.octopus_encode_values(self.vals_tok, self.v_bits, self.v_group, self.vq, cap)
        if self.qjl:
            binding.octopus_encode_qjl(cb, self.keys[:, self.first:], self.sbits, self.s2bits, self.cache, self.side, cap,
                                       self.start_dev)
        elif self.paged:
            binding.octopus_encode_paged(cb, self.keys, self.sbits, self.k_pool, self.n_pages, self.table)
        elif self.rounding != 1:
            binding.octopus_encode_rounding(cb, self.keys[:, self.first:], self.sbits, self.cache, cap, self.rounding,
                                            self.start_dev)
        else:
            binding.octopus_encode(cb, self.keys[:, self.first:], self.sbits, self.cache, cap, self.start_dev)

    def decode(self):
        from paper_2605_21226_amd import binding
        cb, cap, wl = self.cb, self.cap, self.wl
        if self.qjl:
            binding.octopus_attn_decode_qjl(cb, self.q, self.sbits, self.s2bits, self.cache, self.side, cap, self.vals,
                                            self.lens_dev, self.max_len, self.scale, self.out, self.ws)
        elif self.window:
            binding.octopus_attn_decode_hybrid(cb, self.q, self.sbits, self.cache, cap, self.vals, self.lens_dev,
                                               self.max_len, self.k_win, self.win_dev, self.scale, self.out, self.ws)
        elif self.v_bits and self.paged:
            binding.octopus_attn_decode_paged_vq(cb, self.q, self.sbits, self.k_pool, self.vq, self.v_bits, self.v_group,
                                                 wl.n_kv_heads, self.table, self.lens_dev, self.max_len, self.scale,
                                                 self.out, self.ws)
        elif self.v_bits:
            binding.octopus_attn_decode_vq(cb, self.q, self.sbits, self.cache, cap, self.vq, self.v_bits, self.v_group,
                                           wl.n_kv_heads, self.lens_dev, self.max_len, self.scale, self.out, self.ws)
        elif self.paged:
            binding.octopus_attn_decode_paged(cb, self.q, self.sbits, self.k_pool, self.v_pool, self.table, self.lens_dev,
                                              self.max_len, self.scale, self.out, self.ws)
        else:
            binding.octopus_attn_decode(cb, self.q, self.sbits, self.cache, cap, self.vals, self.lens_dev, self.max_len,
                                        self.scale, self.out, self.ws)

    # ---- byte and flop counts -----------------------------------------------------------------------
    def decode_bytes(self):
        from paper_2605_21226_amd import binding
        import numpy as np
        wl = self.wl
        elt = 2 if wl.dtype == "bf16" else 4
        n_keys = int(self.lens.astype(np.int64).sum()) * wl.n_kv_heads
        q_out = wl.n_seq * wl.n_q * wl.n_q_heads * wl.head_dim * (elt + 4)
        side = wl.head_dim // 8 + 2 if self.qjl else 0     # sign bits + fp16 residual norm per key
        v_row = binding.octopus_vq_row_bytes(wl.head_dim, self.v_bits, self.v_group) if self.v_bits else wl.head_dim * elt
        total = n_keys * (self.cb.plan.record_bytes + side + v_row) + q_out
        if self.window:       # window tokens: native key and value rows
            total += int(self.win_dev.sum().item()) * wl.n_kv_heads * 2 * wl.head_dim * elt
        return total, n_keys, side, v_row

    def uses_mq(self):
        wl = self.wl
        return (self.many_rows and wl.head_dim <= 128 and wl.n_q * (wl.n_q_heads // wl.n_kv_heads) >= 32 and
                wl.dtype == "bf16")

    def dominant_kernel(self):
        if self.v_bits:     # quantised values: the matrix-core kernel where one is built for the shape
            from paper_2605_21226_amd import binding
            wl = self.wl
            on_mfma = binding.octopus_vq_on_matrix_cores(self.cb, wl.n_q_heads, wl.n_kv_heads, wl.n_q, self.v_bits, self.v_group)
            return "decode_kernel_vq_mfma" if on_mfma else "decode_kernel_valu"
        return "decode_kernel_mq" if self.uses_mq() else "decode_kernel_mfma"

    def dense_flops(self):
        import numpy as np
        wl = self.wl
        return 4.0 * wl.head_dim * wl.n_q * wl.n_q_heads * float(self.lens.astype(np.int64).sum())


def timed_calls(fn, warmup, timed):
    """ms per call of `fn` (device time between events on the launch stream), after `warmup` untimed calls."""
    import numpy as np
    import torch
    for _ in range(warmup):
        fn()
    ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(timed)]
    for a, b in ev:
        a.record()
        fn()
        b.record()
    torch.cuda.synchronize()
    return np.array([a.elapsed_time(b) for a, b in ev])


def kernel_times(run, calls):
    """ms of the fused kernel alone inside `calls` decode calls (events recorded by the library around its launch)."""
    import numpy as np
    import torch
    from paper_2605_21226_amd import binding
    ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(calls)]
    for a, b in ev:          # a first record creates the HIP handles the library records into
        a.record()
        b.record()
    torch.cuda.synchronize()
    for a, b in ev:
        binding.octopus_profile_events(a, b)
        run.decode()
    torch.cuda.synchronize()
    return np.array([a.elapsed_time(b) for a, b in ev])


def roofline_of(run, ker_s, dec_bytes):
    """The roofline entry of the run's dominant decode kernel for a kernel time of ker_s seconds."""
    wl = run.wl
    kernel = run.dominant_kernel()
    if run.uses_mq():
        # hundreds of query rows per key: a dense contraction on the matrix cores, 4 d flops per (query row, key)
        flops = run.dense_flops()
        tf = flops / ker_s / 1e12
        return {"kernel": kernel, "bound": "mfma", "achieved": round(tf, 2), "peak": BF16_MFMA_PEAK_TFLOPS,
                "unit": "TFLOP/s", "frac": round(tf / BF16_MFMA_PEAK_TFLOPS, 4), "dense_flops_per_launch": flops,
                "note": "achieved counts the flops of dense attention on the reconstructed keys (2 d for q.k and 2 d "
                        "for p.v per query row and key); the kernel issues 2.5 times as many bf16 matrix flops, because "
                        "scores and probabilities go through the bf16 units as hi + lo pairs to keep fp32 accuracy"}
    gbs = dec_bytes / ker_s / 1e9
    return {"kernel": kernel, "bound": "hbm", "achieved": round(gbs, 2), "peak": HBM_PEAK_GBS, "unit": "GB/s",
            "frac": round(gbs / HBM_PEAK_GBS, 4)}


def measure_extra(run, encode_calls=8):
    """One of the other named workloads under the 30 + 50 median protocol: back-to-back decode calls on a cache
    encoded once, the fused kernel alone, and the encode call."""
    import numpy as np
    import torch
    wl = run.wl
    enc_ms = timed_calls(run.encode, 2, encode_calls)
    dec_ms = timed_calls(run.decode, PROTOCOL_WARMUP, PROTOCOL_TIMED)
    ker_ms = kernel_times(run, 20)
    assert bool(torch.isfinite(run.out).all())
    dec_bytes, n_keys, _, _ = run.decode_bytes()
    med, ker = float(np.median(dec_ms)), float(np.median(ker_ms))
    res = {
        "bits": wl.bits, "record_bytes": run.cb.plan.record_bytes, "keys": n_keys,
        "decode_ms": round(med, 4), "decode_ms_min": round(float(dec_ms.min()), 4),
        "effective_gb_per_s": round(dec_bytes / (med * 1e-3) / 1e9, 1),
        "pct_of_hbm_peak": round(100.0 * dec_bytes / (med * 1e-3) / 1e9 / HBM_PEAK_GBS, 2),
        "kernel_ms": round(ker, 4),
        "roofline": roofline_of(run, ker * 1e-3, dec_bytes),
        "encode_ms": round(float(np.median(enc_ms)), 4),
        "encode_tokens": wl.n_seq * run.n_new,
        "encode_mtokens_per_s": round(wl.n_seq * run.n_new / (float(np.median(enc_ms)) * 1e-3) / 1e6, 3),
    }
    return res


def streaming_append(run):
    """Config 3's encode side: ONE new token per sequence per call, appended at the end of a full cache (the cache
    holds n_tokens - 1 tokens; the call writes the last slot of every sequence).  us per call, 30 + 50 median."""
    import numpy as np
    import torch
    from paper_2605_21226_amd import binding
    wl = run.wl
    pos = torch.full((wl.n_seq,), wl.n_tokens - 1, dtype=torch.int32, device=run.dev)
    last = run.keys[:, wl.n_tokens - 1:wl.n_tokens]
    ms = timed_calls(lambda: binding.octopus_encode(run.cb, last, run.sbits, run.cache, run.cap, pos), PROTOCOL_WARMUP,
                     PROTOCOL_TIMED)
    return {"tokens_per_call": wl.n_seq, "keys_per_call": wl.n_seq * wl.n_kv_heads,
            "us_per_call": round(float(np.median(ms)) * 1e3, 2), "us_per_call_min": round(float(ms.min()) * 1e3, 2)}


def read_probe(dev):
    """Plain streaming reads of 1.25 GiB (about the bytes of one decode call of the headline workload)."""
    import numpy as np
    import torch
    from paper_2605_21226_amd import binding
    data = torch.zeros(1342177280, dtype=torch.uint8, device=dev)
    sink = torch.zeros(4, dtype=torch.uint8, device=dev)
    rows = []
    for nt in (0, 1):
        for n_wg in (1024, 2048, 4096, 8192):
            ms = timed_calls(lambda: binding.octopus_probe_read(data, nt, n_wg, sink), 5, 30)
            rows.append({"nontemporal": bool(nt), "workgroups": n_wg, "ms_median": round(float(np.median(ms)), 4),
                         "gb_per_s": round(data.numel() / (float(np.median(ms)) * 1e-3) / 1e9, 1),
                         "frac_of_8_tb_per_s": round(data.numel() / (float(np.median(ms)) * 1e-3) / 1e9 / HBM_PEAK_GBS, 4)})
    return {"probe": "plain streaming read, 16 bytes per lane, 256 threads per workgroup", "bytes": data.numel(),
            "protocol": "5 warm-up + 30 timed launches, median", "results": rows}


def extras(args, dev):
    """The other configurations of the contract, each generated, measured and released in turn."""
    import dataclasses
    import torch
    from paper_2605_21226_amd import synth
    out = {}
    plan = [("tiny", None), ("long_context_2bit", None), ("causal_video", None)] + \
           [("ragged_d256", b) for b in (1.5, 2.0, 2.5, 3.0, 4.0)]
    for name, bits in plan:
        wl = synth.WORKLOADS[name]
        if bits is not None:
            wl = dataclasses.replace(wl, bits=bits)
        try:
            run = Run(wl, args, dev, variants=False)
            res = measure_extra(run, encode_calls=4 if name == "ragged_d256" else 8)
            if name == "tiny":
                res["note"] = "2.3 MB working set, resident in cache: a latency figure, not a bandwidth one"
            if name == "long_context_2bit":
                res["streaming_append"] = streaming_append(run)
            out[name if bits is None else f"{name}@{bits:g}"] = res
        except Exception as exc:    # a failing extra must not take the headline line with it
            out[name if bits is None else f"{name}@{bits:g}"] = {"error": f"{type(exc).__name__}: {exc}"}
        run = None
        torch.cuda.empty_cache()
    return out


def variant_block(args, dev):
    """The optional pieces on the headline workload (same protocol as `workloads`): the QJL residual, quantised
    values, the native-precision window and the paged cache, each through its own entry points."""
    import torch
    from paper_2605_21226_amd import synth
    wl = synth.WORKLOADS["llama3_8b_decode"]
    out = {}
    plan = [("qjl", {"qjl": True}), ("vq3g32", {"vq": "3:32"}), ("vq3g16", {"vq": "3:16"}), ("window32", {"window": 32}),
            ("paged", {"paged": True}), ("paged_vq3g32", {"paged": True, "vq": "3:32"})]
    for name, flags in plan:
        try:
            run = Run(wl, argparse.Namespace(**{**vars(args), **flags}), dev, variants=True)
            res = measure_extra(run, encode_calls=8)
            res["kernel"] = run.dominant_kernel()
            res["value_row_bytes"] = run.decode_bytes()[3]
            out[name] = res
        except Exception as exc:    # a failing variant must not take the headline line with it
            out[name] = {"error": f"{type(exc).__name__}: {exc}"}
        run = None
        torch.cuda.empty_cache()
    return out


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (one process, no collectives); --gpus must be 1. "
              "Over several GPUs the path would shard by sequence or KV head without any exchange; one long "
              "sequence splits by tokens, with one all-gather of the (m, l, acc) partials before the merge.",
              file=sys.stderr)
        sys.exit(2)

    import dataclasses

    import numpy as np
    import torch

    from paper_2605_21226_amd import binding, synth

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)
    dev = "cuda:0"
    torch.cuda.set_device(0)
    if args.read_probe:
        print(json.dumps(read_probe(dev)))
        return
    wl = synth.WORKLOADS[args.workload]
    if args.bits is not None:
        wl = dataclasses.replace(wl, bits=float(args.bits))
    many_rows = wl.n_q > 1
    if args.vq and (many_rows or args.qjl):
        print("bench.py: --vq times single-query workloads without --qjl", file=sys.stderr)
        sys.exit(2)
    if args.window and (many_rows or args.qjl or args.vq):
        print("bench.py: --window times single-query workloads of the plain variant", file=sys.stderr)
        sys.exit(2)
    if args.paged and (many_rows or args.qjl or args.window or args.rounding != 1 or wl.dtype != "bf16"):
        print("bench.py: --paged times single-query bf16 workloads of the plain variant or with --vq", file=sys.stderr)
        sys.exit(2)
    if args.qjl and args.rounding != 1:
        print("bench.py: --qjl goes with the default rounding", file=sys.stderr)
        sys.exit(2)
    if args.qjl and many_rows:
        print("bench.py: --qjl times single-query workloads only", file=sys.stderr)
        sys.exit(2)
    if args.pair and (args.qjl or args.vq or args.paged or args.rounding != 1 or args.bits is not None or wl.head_dim != 128):
        print("bench.py: --pair goes with the plain variant of a head_dim 128 workload, without --bits", file=sys.stderr)
        sys.exit(2)
    variant = bool(args.qjl or args.vq or args.window or args.paged or args.rounding != 1 or args.pair)

    run = Run(wl, args, dev)
    cb = run.cb

    def step(ev=None, kernel_events=False):
        if ev:
            ev[0].record()
        run.encode()
        if ev:
            ev[1].record()
            if kernel_events:
                binding.octopus_profile_events(ev[3], ev[4])  # around the fused kernel inside the next call
        run.decode()
        if ev:
            ev[2].record()

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    events = [[torch.cuda.Event(enable_timing=True) for _ in range(5)] for _ in range(args.steps)]
    for ev in events:          # a first record creates the HIP handles the library records into
        ev[3].record()
        ev[4].record()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    # The pair of events around the kernel sits between the call's launches and costs the call about 7 us
    # (measured: 0.2658 ms with it on every step, 0.2584 ms without).  Every KERNEL_EVENT_STRIDE-th step of the
    # timed region carries it; the call time is taken over the other steps (over all of them when there are
    # no others), the kernel time over those that carry it.
    with_kernel_events = np.array([i % KERNEL_EVENT_STRIDE == 0 for i in range(args.steps)])
    for i in range(args.steps):
        step(events[i], bool(with_kernel_events[i]))
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    enc_ms = np.array([e[0].elapsed_time(e[1]) for e in events])
    dec_ms_all = np.array([e[1].elapsed_time(e[2]) for e in events])
    dec_ms = dec_ms_all[~with_kernel_events] if (~with_kernel_events).any() else dec_ms_all
    ker_ms = np.array([e[3].elapsed_time(e[4]) for e, k in zip(events, with_kernel_events) if k])
    assert bool(torch.isfinite(run.out).all())

    dec_bytes, n_keys_dec, side_bytes, v_row_bytes = run.decode_bytes()
    n_new = run.n_new
    n_keys_enc = wl.n_seq * n_new * wl.n_kv_heads
    rec_bytes = cb.plan.record_bytes
    dec_s = float(dec_ms.mean()) * 1e-3
    enc_s = float(enc_ms.mean()) * 1e-3
    gbs = dec_bytes / dec_s / 1e9
    ker_s = float(ker_ms.mean()) * 1e-3

    # after the timed region: the same decode call back to back on the cache as it stands (no re-encode between
    # calls), under the 30 + 50 median protocol, and the fused kernel alone in that setting
    b2b_ms = timed_calls(run.decode, PROTOCOL_WARMUP, PROTOCOL_TIMED)
    b2b_ker_ms = kernel_times(run, 20)

    result = {
        "metric": "fused decode-attn effective HBM GB/s (% of peak); encode Mtokens/s",
        "value": round(gbs, 2),
        "unit": "GB/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(wall / args.steps * 1e3, 4),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "bf16",
        "data": "synthetic",
        "config": {
            "workload": f"{wl.name}{' + QJL residual' if args.qjl else ''}"
                        f"{f' + values quantised to {run.v_bits} bits in groups of {run.v_group}' if args.vq else ''}"
                        f"{' + paged cache (64-token pages in random order)' if args.paged else ''}: batch {wl.n_seq}, {wl.n_q_heads} query / {wl.n_kv_heads} KV heads, head_dim "
                        f"{wl.head_dim}, {wl.n_tokens} cached tokens, {wl.dtype} K/V/Q, "
                        f"{'an explicit pair of the App. D sweep' if args.pair else f'{wl.bits:g} bits/coordinate'} "
                        f"(b_dir {cb.plan.b_dir[0]}, b_nrm {cb.plan.b_nrm[0]}); step = encode of "
                        f"{wl.n_seq * n_new} tokens + one decode-attention call"
                        + (f" of {wl.n_q} queries per sequence" if many_rows else ""),
            "record_bytes": rec_bytes,
            "qjl_sidecar_bytes": side_bytes,
            "encoder_rounding": args.rounding,
            "value_row_bytes": v_row_bytes,
            "window_tokens": args.window,
            "encode_phase_includes_value_quantisation": bool(args.vq),
            "keys": n_keys_dec,
            "arithmetic": "inputs bf16 (fp32 for the tiny workload); scores and P.V on the bf16 matrix cores with hi + lo "
                          "operand pairs and fp32 accumulation (relative error below 2^-16), softmax in fp32",
        },
        "pct_of_hbm_peak": round(100.0 * gbs / HBM_PEAK_GBS, 2),
        "decode_ms": round(dec_s * 1e3, 4),
        "decode_ms_median": round(float(np.median(dec_ms)), 4),
        "decode_ms_steps_with_kernel_events": round(float(dec_ms_all[with_kernel_events].mean()), 4),
        "kernel_event_steps": int(with_kernel_events.sum()),
        "decode_back_to_back": {
            "what": f"{PROTOCOL_TIMED} decode calls in a row after {PROTOCOL_WARMUP} warm-up calls, no encode between them "
                    "(the timed steps above re-encode the whole cache before every decode call)",
            "decode_ms_median": round(float(np.median(b2b_ms)), 4),
            "decode_ms_min": round(float(b2b_ms.min()), 4),
            "kernel_ms_median": round(float(np.median(b2b_ker_ms)), 4),
            "pct_of_hbm_peak_call": round(100.0 * dec_bytes / (float(np.median(b2b_ms)) * 1e-3) / 1e9 / HBM_PEAK_GBS, 2),
            "frac_kernel": round(dec_bytes / (float(np.median(b2b_ker_ms)) * 1e-3) / 1e9 / HBM_PEAK_GBS, 4),
        },
        "encode_ms": round(enc_s * 1e3, 4),
        "encode_mtokens_per_s": round(wl.n_seq * n_new / enc_s / 1e6, 3),
        "encode_mkeys_per_s": round(n_keys_enc / enc_s / 1e6, 3),
    }
    roof = roofline_of(run, ker_s, dec_bytes)
    roof["kernel"] = (f"{roof['kernel']} (the fused decode kernel inside the decode call), timed with HIP events recorded by "
                      f"the library around its launch on the launch stream, on every {KERNEL_EVENT_STRIDE}th step of the "
                      "timed region")
    roof["algorithmic_bytes_per_launch"] = dec_bytes
    roof["kernel_ms"] = round(ker_s * 1e3, 4)
    if args.window or args.paged:
        roof["traffic"], roof["traffic_source"] = None, "not measured for this variant"
    else:
        roof["traffic"], roof["traffic_source"] = measured_traffic(
            wl.name + ("_qjl" if args.qjl else "") + (f"_vq{run.v_bits}g{run.v_group}" if args.vq else ""),
            run.dominant_kernel())
    result["roofline"] = roof
    # the encoder against the fp32 vector units (its bound: plain ALU work, not HBM, not the matrix cores)
    ops = encode_lane_ops_per_key(wl.head_dim)
    result["encode_roofline"] = {
        "kernel": "encode_kernel", "bound": "alu",
        "achieved": round(ops * n_keys_enc / enc_s / 1e12, 3), "peak": round(FP32_LANE_OPS_PER_S / 1e12, 3),
        "unit": "T lane-ops/s", "frac": round(ops * n_keys_enc / enc_s / FP32_LANE_OPS_PER_S, 4),
        "algorithmic_lane_ops_per_key": ops,
        "note": "peak = fp32 lane-operations per second without packed math (256 CUs x 64 lanes x 2.4 GHz = the "
                "published 157.3 TFLOP/s / 4); algorithmic operations per key as counted in "
                "bench.encode_lane_ops_per_key",
        "hbm_frac": round((n_keys_enc * (wl.head_dim * (2 if wl.dtype == "bf16" else 4) + cb.plan.granules * 16)) /
                          enc_s / 1e9 / HBM_PEAK_GBS, 4),
    }
    if args.calibration_copy:
        src = torch.zeros(1 << 30, dtype=torch.uint8, device=dev)
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
    if not args.no_cpu_baseline and not args.window:      # (the baseline leg times the plain variants)
        result["cpu_baseline"] = cpu_baseline(wl, run.keys, run.vals, run.q, run.signs, run.scale, rec_bytes,
                                              signs2=run.signs2, mode=args.rounding,
                                              vq=(run.v_bits, run.v_group) if args.vq else None, pair=run.pair)
    if not args.no_extras and not variant and args.workload == "llama3_8b_decode" and args.bits is None:
        run = None
        torch.cuda.empty_cache()
        result["protocol_of_workloads"] = (f"{PROTOCOL_WARMUP} warm-up + {PROTOCOL_TIMED} timed decode calls back to back on a "
                                           "cache encoded once, median; kernel_ms: the fused kernel alone, median of 20")
        result["workloads"] = extras(args, dev)
        result["variants_on_llama3_8b_decode"] = variant_block(args, dev)
    print(json.dumps(result))


if __name__ == "__main__":
    main()
