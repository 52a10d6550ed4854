#!/usr/bin/env python3
"""Benchmark of the OCTOPUS hot path on one MI355X.

One step = one pass of the whole hot path over one batch of synthetic input resident in HBM:
prefill-time encode of every cached token (octopus_encode) followed by one decode-attention step
over the compressed cache (octopus_attn_decode: query rotation, fused split-K kernel, merge).

Workload: the Llama-3-8B-shaped GQA decode configuration (batch 16, 32 query heads over 8 KV heads,
head_dim 128, 32768 cached tokens per sequence, bf16 keys / values / queries, 3 bits per coordinate).

Prints ONE JSON line.  `value` is the effective HBM rate of the decode-attention call: algorithmic
bytes (per key: the 58-byte canonical record + the 256-byte bf16 value row; plus queries and outputs)
divided by the call's average duration, measured with events on the launch stream.  `roofline`
is the same byte count over the fused kernel's own duration (events recorded by the library around
its launch), against the published 8 TB/s.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X published HBM3E bandwidth
KERNEL_EVENT_STRIDE = 4        # every 4th timed step carries the event pair around the dominant kernel
FP32_VALU_PEAK_TFLOPS = 157.3  # MI355X published fp32 vector peak
BF16_MFMA_PEAK_TFLOPS = 2500.0 # MI355X published dense bf16 matrix peak


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="llama3_8b_decode")
    ap.add_argument("--no-cpu-baseline", action="store_true")
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
                         "octopus_attn_decode_paged); single-query bf16 workloads, plain variant only")
    ap.add_argument("--calibration-copy", action="store_true",
                    help="also run a plain 1 GiB device-to-device copy (torch) three times, so that a rocprofv3 "
                         "--pmc run of this command can scale FETCH_SIZE / WRITE_SIZE by a kernel of known size")
    return ap.parse_args()


def cpu_baseline(wl, keys, vals, q, signs, scale, record_bytes, budget_s=12.0, signs2=None, mode=1, vq=None):
    """The oracle as it stands, timed on this machine's host cores on a bounded sample of the workload:
    whole sequences (all KV heads, all cached tokens; encode, then attention of each KV head's group of
    query heads over its tokens), one sequence after another until about `budget_s` seconds are spent."""
    import numpy as np

    import oracle

    plan = oracle.make_plan(wl.head_dim, wl.bits)
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
    dec_bytes = n_keys * (record_bytes + v_bytes + (wl.head_dim // 8 + 2 if signs2 is not None else 0))
    threads = int(os.environ.get("OMP_NUM_THREADS", os.cpu_count() or 1))
    return {
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


def measured_traffic(workload, kernel="decode_kernel_mfma"):
    """HBM bytes per launch of the dominant decode kernel as measured with rocprofv3 --pmc FETCH_SIZE /
    WRITE_SIZE (scaled by a plain copy of known size); read from the committed profile summary of this
    kernel and workload, None if there is none."""
    path = os.path.join(ROOT, "profiles", f"{kernel}_{workload}_traffic.txt")
    try:
        vals = {}
        with open(path) as f:
            for line in f:
                if "=" in line and not line.startswith("#"):
                    k, v = line.split("=", 1)
                    vals[k.strip()] = v.strip()
        return int(float(vals["FETCH_BYTES_PER_LAUNCH"]) + float(vals["WRITE_BYTES_PER_LAUNCH"]))
    except (OSError, KeyError, ValueError):
        return None


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (one process, no collectives); --gpus must be 1. "
              "Over several GPUs the path would shard by sequence or KV head without any exchange; one long "
              "sequence splits by tokens, with one all-gather of the (m, l, acc) partials before the merge.",
              file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch

    from paper_2605_21226_amd import binding, synth
    from paper_2605_21226_amd.synth_device import device_inputs

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)
    dev = "cuda:0"
    torch.cuda.set_device(0)
    wl = synth.WORKLOADS[args.workload]
    many_rows = wl.n_q > 1
    v_bits, v_group = (int(x) for x in args.vq.split(":")) if args.vq else (0, 0)
    if args.vq and (many_rows or args.qjl):
        print("bench.py: --vq times single-query workloads without --qjl", file=sys.stderr)
        sys.exit(2)
    if args.window and (many_rows or args.qjl or args.vq):
        print("bench.py: --window times single-query workloads of the plain variant", file=sys.stderr)
        sys.exit(2)
    if args.paged and (many_rows or args.qjl or args.vq or args.window or args.rounding != 1 or wl.dtype != "bf16"):
        print("bench.py: --paged times single-query bf16 workloads of the plain variant", file=sys.stderr)
        sys.exit(2)
    if args.qjl and args.rounding != 1:
        print("bench.py: --qjl goes with the default rounding", file=sys.stderr)
        sys.exit(2)
    if args.qjl and many_rows:
        print("bench.py: --qjl times single-query workloads only", file=sys.stderr)
        sys.exit(2)

    cb = binding.octopus_build_codebooks(wl.head_dim, wl.bits)
    keys, vals, q, signs, lens = device_inputs(wl, args.seed, dev)
    cap = -(-wl.n_tokens // 64) * 64
    if cap != wl.n_tokens:                      # the values need t_capacity rows
        padded = torch.zeros((wl.n_seq, wl.n_kv_heads, cap, wl.head_dim), dtype=vals.dtype, device=dev)
        padded[:, :, :wl.n_tokens] = vals
        vals = padded
    sbits = torch.from_numpy(synth.sign_bits(signs)).to(dev)
    cache = torch.zeros(binding.octopus_cache_bytes(cb, wl.n_seq, wl.n_kv_heads, cap), dtype=torch.uint8, device=dev)
    k_win = win_dev = None
    if args.window:
        # the last `window` tokens of every sequence stay uncompressed; the compressed part shrinks by as much
        win = np.minimum(lens, args.window).astype(np.int32)
        k_win = torch.zeros((wl.n_seq, wl.n_kv_heads, args.window, wl.head_dim), dtype=keys.dtype, device=dev)
        for s_i in range(wl.n_seq):
            a, b = int(lens[s_i] - win[s_i]), int(lens[s_i])
            k_win[s_i, :, :b - a] = keys[s_i, a:b].permute(1, 0, 2)
        lens = (lens - win).astype(np.int32)
        win_dev = torch.from_numpy(win).to(dev)
    max_len = int(lens.max())
    ws = torch.empty(binding.octopus_attn_decode_workspace(cb, wl.n_seq, wl.n_q_heads, wl.n_kv_heads, wl.n_q, max_len),
                     dtype=torch.uint8, device=dev)
    out = torch.zeros((wl.n_seq, wl.n_q, wl.n_q_heads, wl.head_dim), dtype=torch.float32, device=dev)
    lens_dev = torch.from_numpy(lens).to(dev)
    scale = 1.0 / float(np.sqrt(wl.head_dim))
    # single-query workloads: prefill-time encode of the whole cache; a chunk workload: the cache is
    # filled up to the chunk once, and a step encodes the chunk's tokens at their position
    n_new = wl.n_new if many_rows else wl.n_tokens
    first = wl.n_tokens - n_new
    start_dev = None
    if first > 0:
        binding.octopus_encode(cb, keys[:, :first], sbits, cache, cap)
        start_dev = torch.full((wl.n_seq,), first, dtype=torch.int32, device=dev)

    signs2 = s2bits = side = None
    if args.qjl:
        signs2 = synth.sign_vectors(args.seed + 1, wl.n_kv_heads, wl.head_dim)
        s2bits = torch.from_numpy(synth.sign_bits(signs2)).to(dev)
        side = torch.zeros(binding.octopus_qjl_bytes(cb, wl.n_seq, wl.n_kv_heads, cap), dtype=torch.uint8, device=dev)

    vq = vals_tok = None
    if args.vq:
        vq = torch.zeros(binding.octopus_vq_bytes(wl.head_dim, v_bits, v_group, wl.n_seq, wl.n_kv_heads, cap),
                         dtype=torch.uint8, device=dev)
        vals_tok = vals.permute(0, 2, 1, 3)[:, :wl.n_tokens]      # [n_seq, n_tokens, n_kv_heads, d] view

    table = k_pool = v_pool = None
    if args.paged:
        tiles = cap // 64
        n_pages = wl.n_seq * tiles + 7
        gen = torch.Generator(device="cpu").manual_seed(args.seed + 5)
        table = torch.randperm(n_pages, generator=gen)[:wl.n_seq * tiles].to(torch.int32).reshape(wl.n_seq, tiles).to(dev)
        k_pool = torch.zeros(binding.octopus_paged_pool_bytes(cb, n_pages, wl.n_kv_heads), dtype=torch.uint8, device=dev)
        v_pool = torch.zeros((n_pages, wl.n_kv_heads, 64, wl.head_dim), dtype=vals.dtype, device=dev)
        v_pool[table.reshape(-1).long()] = (vals.reshape(wl.n_seq, wl.n_kv_heads, tiles, 64, wl.head_dim)
                                            .permute(0, 2, 1, 3, 4).reshape(-1, wl.n_kv_heads, 64, wl.head_dim))

    def step(ev=None, kernel_events=False):
        if ev:
            ev[0].record()
        if args.vq:
            binding.octopus_encode_values(vals_tok, v_bits, v_group, vq, cap)
        if args.qjl:
            binding.octopus_encode_qjl(cb, keys[:, first:], sbits, s2bits, cache, side, cap, start_dev)
        elif args.paged:
            binding.octopus_encode_paged(cb, keys, sbits, k_pool, n_pages, table)
        elif args.rounding != 1:
            binding.octopus_encode_rounding(cb, keys[:, first:], sbits, cache, cap, args.rounding, start_dev)
        else:
            binding.octopus_encode(cb, keys[:, first:], sbits, cache, cap, start_dev)
        if ev:
            ev[1].record()
            if kernel_events:
                binding.octopus_profile_events(ev[3], ev[4])  # around the fused kernel inside the next call
        if args.qjl:
            binding.octopus_attn_decode_qjl(cb, q, sbits, s2bits, cache, side, cap, vals, lens_dev, max_len, scale, out, ws)
        elif args.window:
            binding.octopus_attn_decode_hybrid(cb, q, sbits, cache, cap, vals, lens_dev, max_len, k_win, win_dev, scale,
                                               out, ws)
        elif args.vq:
            binding.octopus_attn_decode_vq(cb, q, sbits, cache, cap, vq, v_bits, v_group, wl.n_kv_heads, lens_dev, max_len,
                                           scale, out, ws)
        elif args.paged:
            binding.octopus_attn_decode_paged(cb, q, sbits, k_pool, v_pool, table, lens_dev, max_len, scale, out, ws)
        else:
            binding.octopus_attn_decode(cb, q, sbits, cache, cap, vals, lens_dev, max_len, scale, out, ws)
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
    assert bool(torch.isfinite(out).all())

    elt = 2 if wl.dtype == "bf16" else 4
    n_keys_dec = int(lens.astype(np.int64).sum()) * wl.n_kv_heads
    n_keys_enc = wl.n_seq * n_new * wl.n_kv_heads
    rec_bytes = cb.plan.record_bytes
    q_out_bytes = wl.n_seq * wl.n_q * wl.n_q_heads * wl.head_dim * (elt + 4)
    side_bytes = wl.head_dim // 8 + 2 if args.qjl else 0     # sign bits + fp16 residual norm per key
    v_row_bytes = binding.octopus_vq_row_bytes(wl.head_dim, v_bits, v_group) if args.vq else wl.head_dim * elt
    dec_bytes = n_keys_dec * (rec_bytes + side_bytes + v_row_bytes) + q_out_bytes
    n_keys_win = int(win_dev.sum().item()) * wl.n_kv_heads if args.window else 0
    dec_bytes += n_keys_win * 2 * wl.head_dim * elt          # window tokens: native key and value rows
    dec_s = float(dec_ms.mean()) * 1e-3
    enc_s = float(enc_ms.mean()) * 1e-3
    gbs = dec_bytes / dec_s / 1e9
    ker_s = float(ker_ms.mean()) * 1e-3
    ker_gbs = dec_bytes / ker_s / 1e9

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
        "dtype": "f32",
        "data": "synthetic",
        "config": {
            "workload": f"{wl.name}{' + QJL residual' if args.qjl else ''}"
                        f"{f' + values quantised to {v_bits} bits in groups of {v_group}' if args.vq else ''}"
                        f"{' + paged cache (64-token pages in random order)' if args.paged else ''}: batch {wl.n_seq}, {wl.n_q_heads} query / {wl.n_kv_heads} KV heads, head_dim "
                        f"{wl.head_dim}, {wl.n_tokens} cached tokens, {wl.dtype} K/V/Q, {wl.bits:g} bits/coordinate "
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
        },
        "pct_of_hbm_peak": round(100.0 * gbs / HBM_PEAK_GBS, 2),
        "decode_ms": round(dec_s * 1e3, 4),
        "decode_ms_median": round(float(np.median(dec_ms)), 4),
        "decode_ms_steps_with_kernel_events": round(float(dec_ms_all[with_kernel_events].mean()), 4),
        "kernel_event_steps": int(with_kernel_events.sum()),
        "encode_ms": round(enc_s * 1e3, 4),
        "encode_mtokens_per_s": round(wl.n_seq * n_new / enc_s / 1e6, 3),
        "encode_mkeys_per_s": round(n_keys_enc / enc_s / 1e6, 3),
        "roofline": {
            "kernel": "decode_kernel_mfma (the fused split-K decode kernel inside octopus_attn_decode), timed "
                      "with HIP events recorded by the library around its launch on the launch stream, on every "
                      f"{KERNEL_EVENT_STRIDE}th step of the timed region",
            "bound": "hbm",
            "achieved": round(ker_gbs, 2),
            "peak": HBM_PEAK_GBS,
            "unit": "GB/s",
            "frac": round(ker_gbs / HBM_PEAK_GBS, 4),
            "traffic": None,
            "algorithmic_bytes_per_launch": dec_bytes,
            "kernel_ms": round(ker_s * 1e3, 4),
        },
    }
    uses_mq = (many_rows and wl.head_dim <= 128 and wl.n_q * (wl.n_q_heads // wl.n_kv_heads) >= 32 and
               wl.dtype == "bf16")
    dominant = "decode_kernel_valu" if args.vq else ("decode_kernel_mq" if uses_mq else "decode_kernel_mfma")
    result["roofline"]["traffic"] = None if (args.window or args.paged) else measured_traffic(
        wl.name + ("_qjl" if args.qjl else "") + (f"_vq{v_bits}g{v_group}" if args.vq else ""), dominant)
    if args.vq:
        result["roofline"]["kernel"] = result["roofline"]["kernel"].replace("decode_kernel_mfma", "decode_kernel_valu")
    if uses_mq:
        # hundreds of query rows per key: a dense contraction on the matrix cores, 4 d flops per (query row, key)
        flops = 4.0 * wl.head_dim * wl.n_q * wl.n_q_heads * float(lens.astype(np.int64).sum())
        tf = flops / ker_s / 1e12
        result["roofline"].update({
            "kernel": "decode_kernel_mq (decode attention for many query rows on the matrix cores), timed with HIP "
                      "events recorded by the library around its launch on the launch stream",
            "bound": "mfma", "achieved": round(tf, 2), "peak": BF16_MFMA_PEAK_TFLOPS, "unit": "TFLOP/s",
            "frac": round(tf / BF16_MFMA_PEAK_TFLOPS, 4), "dense_flops_per_launch": flops,
            "note": "achieved counts the flops of dense attention on the reconstructed keys (2 d for q.k and 2 d for "
                    "p.v per query row and key); the kernel issues 2.5 times as many bf16 matrix flops, because "
                    "scores and probabilities go through the bf16 units as hi + lo pairs to keep fp32 accuracy"})
    if args.calibration_copy:
        src = torch.zeros(1 << 30, dtype=torch.uint8, device=dev)
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
    if not args.no_cpu_baseline and not args.window:      # (the baseline leg times the plain variants)
        result["cpu_baseline"] = cpu_baseline(wl, keys, vals, q, signs, scale, rec_bytes, signs2=signs2, mode=args.rounding,
                                              vq=(v_bits, v_group) if args.vq else None)
    print(json.dumps(result))


if __name__ == "__main__":
    main()
