"""Benchmark of the KVComp hot path on one MI355X.

One step = one pass of the whole path over a seeded synthetic workload: histogram + codebook, compress the prompt's
KV cache, then `decode_steps` decode steps, each appending one new token per sequence and running the fused
decode attention over the compressed blocks plus the fp16 buffer.  The metric is the fused decode-attention
throughput on COMPRESSED bytes (GB/s, also as a fraction of the HBM peak), next to the compression ratio, the same-GPU
uncompressed fp16 decode attention, and the CPU oracle timed on the host cores.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload c4]

The headline workload is c4 (8 sequences x 8 KV heads x 64 query heads, 16384 prompt tokens, 512 decode steps with
eight flushes of the fp16 buffer): the largest single-GPU configuration and the only one whose decode loop runs every
step of the path.  The other configurations (c0..c3, c2 at each error bound of its sweep) are measured in the same run
with a few steps each and reported under "configs".  Prints one JSON line.
"""
from __future__ import annotations

import argparse
import json
import os
import pathlib
import re
import sys
import time

import numpy as np

ROOT = pathlib.Path(__file__).resolve().parent
HBM_PEAK_GBPS = 8000.0  # MI355X HBM3E, published
# wave64 VALU instructions per second: the published 157.3 TFLOP/s of fp32 vector FMA = 256 CUs x 4 SIMDs x 2.4 GHz
# x 32 lanes x 2 flops, i.e. one wave64 instruction per SIMD every 2 cycles
VALU_ISSUE_PER_S = 157.3e12 / 2 / 64


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=5)
    ap.add_argument("--warmup", type=int, default=1)
    ap.add_argument("--workload", default="c4", choices=["c0", "c1", "c2", "c3", "c4"],
                    help="the headline workload (the timed region and `value`)")
    ap.add_argument("--no-configs", action="store_true",
                    help="measure the headline workload only (profiling runs); by default the other configurations "
                         "follow with a few steps each")
    ap.add_argument("--rel-eb", type=float, default=None, help="override the workload's relative error bound")
    ap.add_argument("--rel-eb-v", type=float, default=None,
                    help="relative error bound of V if it differs from K's (the paper's operating points quantize V "
                         "more coarsely than K)")
    ap.add_argument("--no-graph", action="store_true", help="launch the decode loop eagerly instead of replaying a HIP graph")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--n-splits", type=int, default=0)
    ap.add_argument("--stage-bytes", type=int, default=0)
    ap.add_argument("--max-code-len", type=int, default=0,
                    help="longest Huffman code word; 0 = the width of a fixed-length code of the quantization levels, at "
                         "least 6 bits (6 for the error bounds 1e-2 and 2e-2 of the workloads, 7 for 5e-3): with code "
                         "words of up to 6 bits the fused kernel decodes two symbols per table lookup")
    ap.add_argument("--k-mode", type=int, default=0, choices=[0, 1],
                    help="0: K quantized channel-wise inside a block (the workloads' definition); 1: one range per K "
                         "block (BlockQuant)")
    ap.add_argument("--buffer-tokens", type=int, default=64,
                    help="capacity of the fp16 buffer of new tokens (multiple of 64): the newest tokens stay "
                         "uncompressed, the oldest block of a full buffer is compressed; 64 = the workloads' definition")
    ap.add_argument("--separate-append", action="store_true",
                    help="run every decode step as kvcomp_append_token + kvcomp_attn_decode (two launches) instead of "
                         "kvcomp_append_attn_decode")
    ap.add_argument("--three-pass-store", action="store_true",
                    help="store the prompt with kvcomp_build_codebook + kvcomp_compress_blocks (three quantization "
                         "passes) instead of kvcomp_prefill (one)")
    ap.add_argument("--no-cold", action="store_true",
                    help="skip the cold timings (a 512 MiB copy before every launch scrubs the last-level cache): a "
                         "profile of such a run then sees warm launches only")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also launch a 256 MiB device-to-device copy (reference for rocprofv3 FETCH_SIZE/WRITE_SIZE)")
    return ap.parse_args()


def profile_figures(workload):
    """Counter-derived figures of the fused kernel for one workload, read from the tracked rocprofv3 summary
    profiles/fused_attn_kernel_<workload>.md: lines of the form `key: value` inside its "figures" block (HBM bytes per
    launch from FETCH_SIZE / WRITE_SIZE, vector instructions per decoded wave-symbol, LDS-busy share, the commit the
    profile was taken at).  Missing file or key -> None: nothing is assumed."""
    path = ROOT / "profiles" / f"fused_attn_kernel_{workload}.md"
    out = {}
    if path.exists():
        for m in re.finditer(r"^\s*(traffic_bytes_per_launch|valu_instr_per_wave_symbol|valu_issue_slots_per_wave_symbol|"
                             r"lds_busy_frac|commit|rel_eb|max_code_len)\s*:\s*(\S+)\s*$", path.read_text(), re.M):
            out[m.group(1)] = m.group(2)
    return out


_INPUTS = {}   # the host tensors of the workload measured last


class Scrub:
    """A 512 MiB copy: twice the 256 MiB last-level cache, so whatever a kernel left there is gone afterwards."""

    def __init__(self, torch):
        self.src = torch.empty(512 << 20, dtype=torch.uint8, device="cuda").fill_(1)
        self.dst = torch.empty_like(self.src)

    def __call__(self):
        self.dst.copy_(self.src)


def measure(torch, args, name, rel_eb, rel_eb_v, steps, warmup, headline):
    """Store + decode loop of one workload, `steps` timed passes; then the fused kernel alone (warm, cold), the fp16
    comparison kernel (warm, cold) and the streaming-read bound.  headline: also the multi-kernel pipeline."""
    import workloads as W
    from paper_2509_00579_amd import binding

    w = W.CONFIGS[name]
    B, H, Hq, S, T = w.batch, w.n_kv_heads, w.n_q_heads, w.seq, w.decode_steps
    scale = 1.0 / np.sqrt(128.0)
    max_code_len = args.max_code_len
    if max_code_len == 0:
        levels = int(np.rint(1.0 / (2.0 * np.float32(min(rel_eb, rel_eb_v))))) + 1
        max_code_len = max(6, int(np.ceil(np.log2(levels))))

    # ---- inputs: generated on the host from the seed, resident in HBM before any timed region ----
    if _INPUTS.get("name") != name:   # the error-bound sweep of c2 reuses the tensors of its first run
        _INPUTS.clear()
        _INPUTS.update(name=name, kv=W.make_kv(B, H, S, w.seed), q=W.make_queries(B, Hq, T, w.seed),
                       new=W.make_new_tokens(B, H, T, w.seed))
    (Kx, Vx), qs, (kn, vn) = _INPUTS["kv"], _INPUTS["q"], _INPUTS["new"]
    dK, dV = torch.from_numpy(Kx).cuda(), torch.from_numpy(Vx).cuda()
    dq, dkn, dvn = torch.from_numpy(qs).cuda(), torch.from_numpy(kn).cuda(), torch.from_numpy(vn).cuda()
    out = torch.empty((B, Hq, 128), dtype=torch.float32, device="cuda")
    max_seq = (S + T + 63) // 64 * 64
    cache = binding.KVCompCache(B, H, Hq, max_seq, rel_eb, rel_eb_v, k_mode=args.k_mode, max_code_len=max_code_len,
                                buffer_tokens=args.buffer_tokens)
    cache.set_tuning(args.n_splits, args.stage_bytes)

    prefill_ws = None if args.three_pass_store else torch.empty(cache.prefill_workspace_bytes(S), dtype=torch.uint8,
                                                                device="cuda")

    def store():
        cache.reset(keep_codebook=False)
        if prefill_ws is None:   # the two calls: every pass of the encoder quantizes the input again
            cache.build_codebook(dK, dV)
            cache.compress_blocks(dK, dV)
        else:                    # one quantization pass, codes kept in a workspace
            cache.prefill(dK, dV, prefill_ws)

    def decode_loop():
        for i in range(T):
            if args.separate_append:
                cache.append_token(dkn[i], dvn[i])
                cache.attn_decode(dq[i], scale, out)
            else:   # the same step as one call (one launch unless the token completes a block)
                cache.append_attn_decode(dkn[i], dvn[i], dq[i], scale, out)

    ev = [torch.cuda.Event(enable_timing=True) for _ in range(4)]

    # ---- warm-up (eager; also sizes the kernel's LDS) ----
    for _ in range(max(warmup, 1)):
        store()
        decode_loop()
    torch.cuda.synchronize()
    stats_end = cache.stats()

    # algorithmic bytes of each decode step i (token i appended before it): records + offsets + fp16 buffer
    # + q + out + split partials (written once, read once) + the two lookup tables
    def decode_bytes(n_blocks, n_res, n_splits_est):
        blocks = B * H * n_blocks
        rec = rec0 + (n_blocks - nb0) * flush_bytes
        return (rec + 2 * blocks * 8 + 2 * B * H * n_res * 128 * 2 + B * Hq * 128 * 2 + B * Hq * 128 * 4
                + 2 * n_splits_est * B * Hq * 130 * 4 + 2 * 4096 * 2)

    store()
    stats0 = cache.stats()
    torch.cuda.synchronize()
    nb0 = stats0["n_blocks"]
    rec0 = stats0["record_bytes_k"] + stats0["record_bytes_v"]
    n_flush = stats_end["n_blocks"] - nb0
    flush_bytes = ((stats_end["record_bytes_k"] + stats_end["record_bytes_v"] - rec0) / n_flush) if n_flush else 0.0
    if args.n_splits:
        n_splits_est = args.n_splits
    else:  # mirrors the library's split heuristic (only used to count the bytes of the split partials)
        ns = max(1, min(max(1, 256 // (B * H)), -(-nb0 // 4)))
        bps = -(-nb0 // ns)
        n_splits_est = max(1, min(128, -(-nb0 // bps))) if bps else 1

    def blocks_of(tokens):  # compressed blocks after `tokens` tokens: the buffer keeps the newest ones
        return 0 if tokens < args.buffer_tokens else (tokens - args.buffer_tokens) // 64 + 1

    step_bytes = []
    for i in range(T):
        tokens = S + i + 1
        step_bytes.append(decode_bytes(blocks_of(tokens), tokens - 64 * blocks_of(tokens), n_splits_est))
    loop_bytes = float(sum(step_bytes))

    # ---- capture the decode loop (launch-bound at the small sizes) in a HIP graph ----
    graph = None
    if not args.no_graph:
        try:
            g = torch.cuda.CUDAGraph()
            with torch.cuda.graph(g):
                decode_loop()
            graph = g
        except Exception as e:  # noqa: BLE001
            print(f"bench.py: graph capture failed ({e}); running the decode loop eagerly", file=sys.stderr)
            graph = None
        torch.cuda.synchronize()

    def run_decode():
        if graph is not None:
            graph.replay()
        else:
            decode_loop()

    # ---- timed region: exactly `steps` steps ----
    torch.cuda.synchronize()
    store_ms, decode_ms = [], []
    t0 = time.perf_counter()
    for _ in range(steps):
        ev[0].record()
        store()              # synchronises (histogram and sizes cross to the host)
        ev[1].record()
        run_decode()
        ev[2].record()
        ev[2].synchronize()
        store_ms.append(ev[0].elapsed_time(ev[1]))
        decode_ms.append(ev[1].elapsed_time(ev[2]))
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_per_step = (t1 - t0) * 1e3 / steps
    dec_ms = float(np.mean(decode_ms))
    value = loop_bytes / (dec_ms * 1e-3) / 1e9
    assert torch.isfinite(out).all()

    # ---- dominant kernel: HIP events around every fused-kernel launch (eager pass, same process) ----
    pair_ms = None
    if headline:
        cache.set_profiling(True)
        store()
        decode_loop()
        launches, total_ms = cache.get_profile()
        cache.set_profiling(False)
        pair_ms = total_ms / max(launches, 1)   # an event pair per launch also sees the gap to the previous kernel
    # ... and back to back, like the fp16 kernel below: launches of the fused kernel on the cache as the loop left it
    # (a graph replay, or eager launches), one event pair around all of them
    krep = 64   # per replay; two warm-up replays, then three timed ones: the first hundred launches after the store and
    # the host-side work around it run a few per cent slower than the steady state
    kgraph = None
    if not args.no_graph:
        try:
            kg = torch.cuda.CUDAGraph()
            with torch.cuda.graph(kg):
                for i in range(krep):
                    cache.attn_decode(dq[i % T], scale, out)
            kgraph = kg
        except Exception:  # noqa: BLE001
            kgraph = None
        torch.cuda.synchronize()
    for r in range(5):   # the first two rounds are a warm-up
        if r == 2:
            ev[0].record()
        if kgraph is not None:
            kgraph.replay()
        else:
            for i in range(krep):
                cache.attn_decode(dq[i % T], scale, out)
    ev[1].record()
    ev[1].synchronize()
    kern_ms = ev[0].elapsed_time(ev[1]) / (3 * krep)
    launches = 3 * krep
    tokens_end = S + T
    kern_bytes = float(decode_bytes(blocks_of(tokens_end), tokens_end - 64 * blocks_of(tokens_end), n_splits_est)
                       - B * Hq * 128 * 4 - n_splits_est * B * Hq * 130 * 4)   # no out, partials once
    achieved = kern_bytes / (kern_ms * 1e-3) / 1e9
    symbols_per_launch = 2.0 * B * H * blocks_of(tokens_end) * 8192

    # ---- the same launches with the caches scrubbed in between (the compressed cache of every workload fits the
    # 256 MiB last-level cache; a 512 MiB copy before every launch evicts it): the regime of a model with many
    # layers, where a layer's cache is touched once per decode step ----
    cold_kern_ms = None
    scrub = None
    if not args.no_cold:
        scrub = Scrub(torch)
        cache.set_profiling(True)
        for i in range(8):
            scrub()
            cache.attn_decode(dq[i % T], scale, out)
        cold_launches, cold_total_ms = cache.get_profile()
        cache.set_profiling(False)
        cold_kern_ms = cold_total_ms / max(cold_launches, 1)

    if args.calibrate_copy and headline:  # a plain copy of known size: scales the HBM byte counters of a --pmc run
        src = torch.empty(256 << 20, dtype=torch.uint8, device="cuda").fill_(1)
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    # ---- same-GPU uncompressed fp16 decode attention on the prompt ----
    base = binding.BaselineFp16Attention(B, H, Hq)
    for i in range(3):
        base(dK, dV, dq[i % T], scale, out)
    torch.cuda.synchronize()
    nrep = 64   # as for the fused kernel: two warm-up replays, three timed ones
    bgraph = None
    if not args.no_graph:
        try:
            bg = torch.cuda.CUDAGraph()
            with torch.cuda.graph(bg):
                for i in range(nrep):
                    base(dK, dV, dq[i % T], scale, out)
            bgraph = bg
        except Exception:  # noqa: BLE001
            bgraph = None
    for r in range(5):
        if r == 2:
            ev[0].record()
        if bgraph is not None:
            bgraph.replay()
        else:
            for i in range(nrep):
                base(dK, dV, dq[i % T], scale, out)
    ev[1].record()
    ev[1].synchronize()
    base_ms = ev[0].elapsed_time(ev[1]) / (3 * nrep)
    base_bytes = 2 * B * H * S * 128 * 2 + B * Hq * 128 * (2 + 4)
    # what a plain streaming read of the same two tensors takes (warm, like the kernels): the bound for any fp16 kernel
    sink = torch.zeros(4, dtype=torch.uint8, device="cuda")
    k8, v8 = dK.view(torch.uint8).reshape(-1), dV.view(torch.uint8).reshape(-1)
    stream_bytes = 0
    for r in range(11):   # the first round is a warm-up
        if r == 1:
            ev[2].record()
        stream_bytes = binding.probe_read_stream(k8, sink) + binding.probe_read_stream(v8, sink)
    ev[3].record()
    ev[3].synchronize()
    stream_ms = ev[2].elapsed_time(ev[3]) / 10
    stream_GBps = stream_bytes / (stream_ms * 1e-3) / 1e9 if stream_bytes else None
    # the fp16 kernel with the caches scrubbed before every launch, like the fused kernel above
    base_cold_ms = None
    if scrub is not None:
        cold = []
        for i in range(8):
            scrub()
            ev[2].record()
            base(dK, dV, dq[i % T], scale, out)
            ev[3].record()
            ev[3].synchronize()
            cold.append(ev[2].elapsed_time(ev[3]))
        base_cold_ms = float(np.mean(cold))
    del scrub

    raw_bytes = 2 * B * H * S * 128 * 2
    res = {
        "workload": name,
        "shape": {"batch": B, "kv_heads": H, "q_heads": Hq, "prompt_tokens": S, "decode_steps": T},
        "rel_eb": rel_eb, "rel_eb_v": rel_eb_v, "max_code_len": max_code_len,
        "steps": steps, "warmup": warmup,
        "value_GBps": value, "pct_hbm_peak": 100.0 * value / HBM_PEAK_GBPS,
        "ms_per_step": ms_per_step, "decode_ms_per_token": dec_ms / T, "tokens_per_s": B * T / (dec_ms * 1e-3),
        "compression_ratio": stats0["compression_ratio"],
        "bits_per_symbol": {"k": stats0["payload_bits_k"] / (B * H * nb0 * 8192.0),
                            "v": stats0["payload_bits_v"] / (B * H * nb0 * 8192.0)},
        "equivalent_fp16_GBps": raw_bytes * T / (dec_ms * 1e-3) / 1e9,
        "store_ms": float(np.mean(store_ms)),
        "store_GBps_fp16_in": raw_bytes / (float(np.mean(store_ms)) * 1e-3) / 1e9,
        "fused_kernel": {"ms_warm": kern_ms, "ms_cold": cold_kern_ms, "bytes_per_launch": kern_bytes,
                         "GBps_warm": achieved, "frac_hbm_peak_warm": achieved / HBM_PEAK_GBPS,
                         "GBps_cold": (kern_bytes / (cold_kern_ms * 1e-3) / 1e9) if cold_kern_ms else None,
                         "frac_hbm_peak_cold": (kern_bytes / (cold_kern_ms * 1e-3) / 1e9 / HBM_PEAK_GBPS)
                         if cold_kern_ms else None,
                         "symbols_per_launch": symbols_per_launch, "launches_timed": launches,
                         "ms_event_pair_each": pair_ms},
        "fp16_kernel": {"ms_warm": base_ms, "ms_cold": base_cold_ms, "GBps_warm": base_bytes / (base_ms * 1e-3) / 1e9,
                        "pct_hbm_peak_warm": 100.0 * base_bytes / (base_ms * 1e-3) / 1e9 / HBM_PEAK_GBPS,
                        # a plain streaming read of the same K and V tensors (two launches, warm): no fp16 attention
                        # kernel can be faster than this
                        "stream_read": {"ms": stream_ms, "GBps": stream_GBps, "bytes": stream_bytes}},
        "fused_vs_fp16": {"kernel_speedup_warm": base_ms / kern_ms,   # kernel against kernel, both HIP-event timed
                          "kernel_speedup_cold": (base_cold_ms / cold_kern_ms) if cold_kern_ms else None,
                          "step_speedup_warm": base_ms / (dec_ms / T),  # the fused side also appends a token
                          "fused_vs_stream_read": stream_ms / kern_ms},
        "decode_loop": "hip graph replay" if graph is not None else "eager launches",
        "store": "kvcomp_build_codebook + kvcomp_compress_blocks" if args.three_pass_store
                 else "kvcomp_prefill (one quantization pass, codes kept in a workspace)",
    }

    # ---- the multi-kernel pipeline (decompress K, decompress V to fp16 in HBM, then the fp16 attention kernel) ----
    if headline:
        st_now = cache.stats()
        tokens_now = st_now["n_blocks"] * 64 + st_now["n_res"]
        decK = torch.empty((B, tokens_now, H, 128), dtype=torch.float16, device="cuda")
        decV = torch.empty_like(decK)
        for _ in range(2):
            cache.decompress(0, tokens_now, decK)
            cache.decompress(1, tokens_now, decV)
            base(decK, decV, dq[0], scale, out)
        torch.cuda.synchronize()
        mk = []
        for i in range(5):
            ev[0].record()
            cache.decompress(0, tokens_now, decK)
            cache.decompress(1, tokens_now, decV)
            ev[1].record()
            base(decK, decV, dq[i % T], scale, out)
            ev[2].record()
            ev[2].synchronize()
            mk.append((ev[0].elapsed_time(ev[1]), ev[1].elapsed_time(ev[2])))
        dec_only_ms = float(np.mean([m[0] for m in mk]))
        mk_attn_ms = float(np.mean([m[1] for m in mk]))
        tw = []  # the same decompression with the paper's bit-serial tree-walk decoder (Section 3.3.1)
        for i in range(3):
            ev[0].record()
            cache.decompress(0, tokens_now, decK, tree_walk=True)
            cache.decompress(1, tokens_now, decV, tree_walk=True)
            ev[1].record()
            ev[1].synchronize()
            tw.append(ev[0].elapsed_time(ev[1]))
        dec_tree_ms = float(np.mean(tw[1:]))
        del decK, decV
        # Section 4.3's comparison: decompress to fp16 in HBM (two launches, each synchronising once), then attention
        res["multi_kernel"] = {"decompress_ms": dec_only_ms, "decompress_tree_walk_ms": dec_tree_ms,
                               "attention_ms": mk_attn_ms,
                               "decompress_GBps_fp16_out": 2 * B * H * tokens_now * 128 * 2 / (dec_only_ms * 1e-3) / 1e9,
                               "fused_speedup": (dec_only_ms + mk_attn_ms) / kern_ms}
    cache.close()
    del cache, base, dK, dV, dq, dkn, dvn, out, graph, kgraph, bgraph, prefill_ws
    torch.cuda.empty_cache()
    return res, (Kx, Vx, qs, kn, vn, max_seq, max_code_len)


def cpu_baseline(args, name, rel_eb, rel_eb_v, inputs):
    """The CPU oracle as it stands on the host cores: a bounded sample of the same workload (about 10 s of CPU work)."""
    import workloads as W
    from oracle import kvcomp_oracle as oracle
    w = W.CONFIGS[name]
    B, H, Hq, S, T = w.batch, w.n_kv_heads, w.n_q_heads, w.seq, w.decode_steps
    Kx, Vx, qs, kn, vn, max_seq, max_code_len = inputs
    scale = 1.0 / np.sqrt(128.0)
    ob = 1                                          # bounded sample: one sequence of the batch ...
    oh = max(1, min(H, (4 * 16384) // S))           # ... and as many KV heads as keep it near 64K tokens
    G = Hq // H
    oc = oracle.OracleCache(ob, oh, oh * G, max_seq, rel_eb, rel_eb_v, k_mode=args.k_mode, max_code_len=max_code_len,
                            buffer_tokens=args.buffer_tokens)
    Ks, Vs = np.ascontiguousarray(Kx[:ob, :, :oh]), np.ascontiguousarray(Vx[:ob, :, :oh])
    oc.build_codebook(Ks, Vs)
    oc.compress_blocks(Ks, Vs)
    # about 10 s of CPU work: repeat decode steps (fresh query each) until the clock says so, at most 30 s
    obytes, osteps = 0.0, 0
    tc0 = time.perf_counter()
    while True:
        i = osteps % T
        if osteps < T:
            oc.append_token(np.ascontiguousarray(kn[i][:ob, :oh]), np.ascontiguousarray(vn[i][:ob, :oh]))
        oc.attn_decode(np.ascontiguousarray(qs[i][:ob, : oh * G]), scale)
        obytes += oc.stats()["stored_bytes"] + ob * oh * G * 128 * 6
        osteps += 1
        elapsed = time.perf_counter() - tc0
        if elapsed >= 10.0 or (osteps >= 2 and elapsed * (osteps + 1) / osteps > 30.0):
            break
    tc1 = time.perf_counter()
    # the same step on one core (a few steps only)
    all_threads = oracle.num_threads()
    oracle.set_num_threads(1)
    ts0 = time.perf_counter()
    sbytes, ssteps = 0.0, 0
    while ssteps < 2 or (time.perf_counter() - ts0 < 3.0 and ssteps < 64):
        oc.attn_decode(np.ascontiguousarray(qs[ssteps % T][:ob, : oh * G]), scale)
        sbytes += oc.stats()["stored_bytes"] + ob * oh * G * 128 * 6
        ssteps += 1
    ts1 = time.perf_counter()
    oracle.set_num_threads(all_threads)
    return {"value": obytes / (tc1 - tc0) / 1e9, "unit": "GB/s", "cores": all_threads, "kind": "oracle",
            "value_one_core": sbytes / (ts1 - ts0) / 1e9,
            "sample": f"{osteps} decode steps (append + attention over the compressed cache) of {name} "
                      f"restricted to batch {ob} x {oh} kv heads ({oh * G} query heads), prompt {S} tokens",
            "seconds": tc1 - tc0}


def main():
    args = parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        sys.exit("bench.py: this build runs on ONE GPU (the path would shard by batch and KV head, with no exchange per step); "
                 "--gpus N with N > 1 is not supported")

    import torch

    import workloads as W

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    name = args.workload
    w = W.CONFIGS[name]
    rel_eb = args.rel_eb if args.rel_eb is not None else w.rel_eb
    rel_eb_v = args.rel_eb_v if args.rel_eb_v is not None else rel_eb

    head, inputs = measure(torch, args, name, rel_eb, rel_eb_v, args.steps, args.warmup, headline=True)
    cpu = None if args.no_cpu_baseline else cpu_baseline(args, name, rel_eb, rel_eb_v, inputs)
    del inputs

    # ---- the other configurations, a few steps each: c0, c1, c2 at every error bound of its sweep, c3 (and c4 when
    # another workload is the headline) ----
    configs = []
    if not args.no_configs:
        todo = []
        for other in ("c0", "c1", "c2", "c3", "c4"):
            if other == name:
                continue
            if other == "c2":
                todo += [("c2", eb) for eb in W.C2_REL_EB_SWEEP]
            else:
                todo.append((other, W.CONFIGS[other].rel_eb))
        for other, eb in todo:
            r, _ = measure(torch, args, other, eb, eb, steps=min(args.steps, 3), warmup=1, headline=False)
            configs.append(r)

    fig = profile_figures(name)
    G = head["shape"]["q_heads"] // head["shape"]["kv_heads"]
    fk, bk = head["fused_kernel"], head["fp16_kernel"]

    def num(key):
        return float(fig[key]) if key in fig else None

    # the figures of a profile apply only to the workload, error bound and code word limit it was taken with
    if fig and (abs(float(fig.get("rel_eb", rel_eb)) - rel_eb) > 1e-12 or
                int(fig.get("max_code_len", head["max_code_len"])) != head["max_code_len"] or rel_eb_v != rel_eb or
                args.k_mode or args.buffer_tokens != 64):
        fig = {}
    valu_slots = num("valu_issue_slots_per_wave_symbol")
    sym_rate = fk["symbols_per_launch"] / (fk["ms_warm"] * 1e-3)
    T = head["shape"]["decode_steps"]
    result = {
        "metric": "fused decode-attention GB/s (compressed) & % HBM peak; compression ratio",
        "value": head["value_GBps"],
        "unit": "GB/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": head["ms_per_step"],
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f32",
        "data": "synthetic",
        "config": {"workload": f"{name}: batch {w.batch}, {w.n_kv_heads} kv heads / {w.n_q_heads} q heads x 128, prompt "
                               f"{w.seq} tokens, {T} decode steps (append one token, flush full 64-token blocks, then "
                               f"fused decode attention), block 64, rel_eb {rel_eb}"
                               + (f" (V: {rel_eb_v})" if rel_eb_v != rel_eb else "")
                               + f", max code word {head['max_code_len']} bits" + (", K BlockQuant" if args.k_mode else "")
                               + (f", fp16 buffer of {args.buffer_tokens} tokens" if args.buffer_tokens != 64 else ""),
                   "decode_loop": head["decode_loop"],
                   "decode_step": "kvcomp_append_token + kvcomp_attn_decode" if args.separate_append
                                  else "kvcomp_append_attn_decode (append fused into the attention launch)"},
        "pct_hbm_peak": head["pct_hbm_peak"],
        "compression_ratio": head["compression_ratio"],
        "bits_per_symbol": head["bits_per_symbol"],
        "decode_ms_per_token": head["decode_ms_per_token"],
        "tokens_per_s": head["tokens_per_s"],
        "equivalent_fp16_GBps": head["equivalent_fp16_GBps"],
        "store_ms": head["store_ms"],
        "store_GBps_fp16_in": head["store_GBps_fp16_in"],
        "fp16_baseline": {"ms": bk["ms_warm"], "ms_cold": bk["ms_cold"], "GBps": bk["GBps_warm"],
                          "pct_hbm_peak": bk["pct_hbm_peak_warm"], "stream_read": bk["stream_read"],
                          "fused_kernel_speedup": head["fused_vs_fp16"]["kernel_speedup_warm"],
                          "fused_kernel_speedup_cold": head["fused_vs_fp16"]["kernel_speedup_cold"],
                          "fused_step_speedup": head["fused_vs_fp16"]["step_speedup_warm"]},
        "multi_kernel": head.get("multi_kernel"),
        "roofline": {"bound": "hbm", "kernel": f"fused_attn_kernel, groups of {G} query heads per KV head",
                     "achieved": fk["GBps_warm"], "peak": HBM_PEAK_GBPS,
                     "unit": "GB/s", "frac": fk["frac_hbm_peak_warm"],
                     "traffic": num("traffic_bytes_per_launch"), "traffic_profile_commit": fig.get("commit"),
                     "bytes_per_launch": fk["bytes_per_launch"], "avg_launch_ms": fk["ms_warm"],
                     "launches_timed": fk["launches_timed"],
                     "avg_launch_ms_cold": fk["ms_cold"],  # every launch preceded by a 512 MiB copy (caches scrubbed)
                     "frac_cold": fk["frac_hbm_peak_cold"],
                     "avg_launch_ms_event_pair_each": fk["ms_event_pair_each"],
                     "timing": f"one HIP event pair around 3 x {fk['launches_timed'] // 3} back-to-back launches of the "
                               "fused kernel on the cache as the decode loop left it (graph replay unless --no-graph; two "
                               "replays of warm-up before them), on the launch stream, right after the timed region; avg_launch_ms_event_pair_each: an "
                               "event pair around every launch of one eager pass of the decode loop, which also sees "
                               "the gap to the previous kernel; avg_launch_ms_cold: an event pair per launch with a "
                               "512 MiB copy before it"},
        # The kernel is not bound by HBM: per decoded symbol it spends one LDS table lookup and several VALU
        # instructions.  Symbols decoded per second against what the vector ALUs could issue at that cost per
        # symbol (instruction counts from the tracked rocprofv3 summary of this workload; null without one).
        "roofline_alu": {"bound": "alu", "achieved": sym_rate / 1e12,
                         "peak": (VALU_ISSUE_PER_S * 64 / valu_slots / 1e12) if valu_slots else None,
                         "unit": "Tsymbol/s",
                         "frac": (sym_rate / (VALU_ISSUE_PER_S * 64 / valu_slots)) if valu_slots else None,
                         "valu_instr_per_symbol": num("valu_instr_per_wave_symbol"),
                         "valu_issue_slots_per_symbol": valu_slots,
                         "lds_busy_frac": num("lds_busy_frac"), "profile_commit": fig.get("commit")},
        "cpu_baseline": cpu,
        "configs": configs,
    }
    print(json.dumps(result))


if __name__ == "__main__":
    main()
