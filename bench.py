#!/usr/bin/env python3
"""Benchmark of the LoRC hot path on one MI355X: decode over a rank-r latent KV cache.

Workload (config.workload): LLaMA-3-8B-shaped single layer, d_model 4096, 32 query / 8 KV heads, head_dim
128, W_k/W_v 4096x1024 with a power-law spectrum, rank 512 for K and V, batch 16, context 4096, bf16 latent
cache, RoPE base 500000.  One step = the whole run-time path for one decode token per sequence:
lorc_append_latent (16 new tokens) + lorc_decode_attention (split and merge kernels).  All inputs are in
HBM before the timed region; the step cycles over several copies of the cache so that the 134 MB of latents
cannot be served from the 256 MB last-level cache.

Prints ONE JSON line: metric/value/unit (decode tok/s of the step above), ms_per_step, `roofline` (the dominant
kernel, decode_split_kernel: achieved TFLOP/s against the bf16 matrix-core peak from HIP events recorded around it
on the launch stream on every fifth step of the timed region, plus its latent stream in GB/s, the profiled HBM bytes per launch, and the HBM read rate
and matrix-core rate this machine sustains by the library's two probes), `cpu_baseline` (the
fp64 oracle timed on the host cores on a bounded sample of the same workload), `prefill` (down-projection and
causal attention of 4 x 8192 tokens), `absorbed` (the same cache and step for a model without positional rotation:
absorbed-query decode, HBM-bound, with its own roofline object and a long-context measurement) and `setup`.
"""
from __future__ import annotations

import argparse
import ctypes
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0       # MI355X HBM3E, published
MFMA_BF16_PEAK_TFLOPS = 2500.0  # MI355X dense bf16 matrix cores, published
# HBM bytes per launch of the dominant decode kernel on the default workload, from rocprofv3 FETCH_SIZE + WRITE_SIZE
# runs of this script scaled by a plain 1 GiB copy (profiles/bench_kernels_hbm_traffic.md): 143.6 MB read + 2.1 MB written.
# Not measurable from inside the process; reported only when the run uses the profiled workload and cache pools.
SPLIT_TRAFFIC_BYTES_PROFILED = 145.7e6
EVENT_STRIDE = 5  # steps between two event-bracketed launches of the dominant kernel
ABSORBED_TRAFFIC_BYTES_PROFILED = 155.7e6  # same source: 138.8 MB read + 16.9 MB written per decode_absorbed_kernel launch


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--pools", type=int, default=8, help="distinct copies of the latent cache cycled through")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-events", action="store_true", help="do not record per-kernel events in the timed loop")
    ap.add_argument("--no-prefill", action="store_true", help="skip the prefill (configs[3]) measurement")
    ap.add_argument("--no-absorbed", action="store_true",
                    help="skip the leg for models without positional rotation (absorbed-query decode)")
    ap.add_argument("--no-stack", action="store_true", help="skip the configs[2] leg (32-layer stack, progressive ranks)")
    ap.add_argument("--no-share", action="store_true", help="skip the configs[4] leg (70B-shaped 8-layer share)")
    ap.add_argument("--no-wide", action="store_true", help="skip the 13B-shaped (rank 2048) and the uncompressed-layer legs")
    ap.add_argument("--copy-probe", action="store_true",
                    help="also run three plain 1 GiB device-to-device copies (reference for scaling hardware "
                         "traffic counters when this command runs under a profiler)")
    ap.add_argument("--zero-data", action="store_true",
                    help="power probe, not a measurement of the workload: the decode and prefill legs run the same "
                         "launches on all-zero caches, tokens and queries (no switching activity in the operands); "
                         "the other legs and the CPU baseline are skipped and the line says data = zeros")
    args = ap.parse_args()
    if args.zero_data:
        args.no_cpu_baseline = args.no_absorbed = args.no_stack = args.no_share = args.no_wide = True
    if args.gpus != 1:
        print("bench.py: this build is single-GPU by design (no sharding or collectives); run with --gpus 1",
              file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    import lorc_inputs as gen
    import paper_2410_03111_amd as L

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    dev = torch.device("cuda:0")
    hip = ctypes.CDLL("libamdhip64.so.7")  # resolves to the runtime already loaded by torch
    hip.hipEventCreate.argtypes = [ctypes.POINTER(ctypes.c_void_p)]
    hip.hipEventElapsedTime.argtypes = [ctypes.POINTER(ctypes.c_float), ctypes.c_void_p, ctypes.c_void_p]
    hip.hipEventDestroy.argtypes = [ctypes.c_void_p]
    hip.hipEventRecord.argtypes = [ctypes.c_void_p, ctypes.c_void_p]

    c = gen.CONFIGS[1]
    D, h_q, h_kv, d, r = c["d_model"], c["n_q_heads"], c["n_kv_heads"], c["head_dim"], c["rank"]
    b, N, base, seed = c["batch"], c["context"], c["rope_base"], c["seed"]
    n = h_kv * d
    desc = L.layer_desc(D, h_q, h_kv, d, r, r, base)
    t_setup = time.perf_counter()

    # ---- offline: weights, factorisation (library, host), packing
    W_k, _ = gen.power_law_weight(D, n, seed=1000 + 2 * seed)
    W_v, _ = gen.power_law_weight(D, n, seed=1001 + 2 * seed)
    t0 = time.perf_counter()
    A_k, B_k, _, eps_k = L.factorize(W_k, r)
    A_v, B_v, _, eps_v = L.factorize(W_v, r)
    t_factorize = time.perf_counter() - t0
    bf = lambda a: torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).to(dev).to(torch.bfloat16).contiguous()
    packed = L.pack_factors(desc, bf(A_k), bf(A_v), bf(B_k), bf(B_v))

    # ---- cache pools, filled by the real append kernel from seeded hidden states
    pages_per_seq = N // L.PAGE_TOKENS
    n_pages = b * pages_per_seq + 5
    page_bytes = L.page_bytes(desc)
    bt_np = gen.block_table(b, pages_per_seq, n_pages, seed=seed)
    bt = torch.from_numpy(bt_np).to(dev)
    pools = [torch.zeros(n_pages * page_bytes, dtype=torch.uint8, device=dev)]
    X_host = []
    for s in range(b):
        x = gen.hidden_states(N, D, seed=50000 + 97 * seed + s)
        X_host.append(x)
        L.append_latent(desc, torch.from_numpy(x).to(dev).to(torch.bfloat16), packed,
                        torch.full((N,), s, dtype=torch.int32, device=dev),
                        torch.arange(N, dtype=torch.int32, device=dev), bt, pools[0])
    torch.cuda.synchronize()
    for _ in range(1, args.pools):
        pools.append(pools[0].clone())

    # ---- per-step inputs: the newest token of every sequence (position N-1) and its query
    x_new = torch.from_numpy(np.stack([X_host[s][N - 1] for s in range(b)])).to(dev).to(torch.bfloat16).contiguous()
    q_np = gen.queries(b, h_q, d, seed=90000 + seed)
    q = torch.from_numpy(q_np).to(dev).to(torch.bfloat16).contiguous()
    slot_seq = torch.arange(b, dtype=torch.int32, device=dev)
    slot_pos = torch.full((b,), N - 1, dtype=torch.int32, device=dev)
    q_pos = torch.full((b,), N - 1, dtype=torch.int32, device=dev)
    ctx_len = torch.full((b,), N, dtype=torch.int32, device=dev)
    out = torch.empty_like(q)
    ws = torch.empty(L.decode_workspace_bytes(desc, b, N), dtype=torch.uint8, device=dev)
    if args.zero_data:
        for tns in pools + [x_new, q]:
            tns.zero_()
    t_setup = time.perf_counter() - t_setup

    def make_events(k):
        evs = []
        for _ in range(k):
            pair = []
            for _ in range(2):
                e = ctypes.c_void_p()
                assert hip.hipEventCreate(ctypes.byref(e)) == 0
                pair.append(e.value)
            evs.append(pair)
        return evs

    def step(i, events=None):
        pool = pools[i % len(pools)]
        L.append_latent(desc, x_new, packed, slot_seq, slot_pos, bt, pool)
        L.decode_attention(desc, q, q_pos, ctx_len, N, packed, pool, bt, out=out, workspace=ws, events=events)

    for i in range(args.warmup):
        step(i)
    torch.cuda.synchronize()
    # the dominant kernel is bracketed by events on every EVENT_STRIDE-th step of the timed region (a pair of
    # event records costs 4-5 us of a 0.12 ms step; the stride is odd, so the sampled steps cycle through the pools)
    sampled = [i for i in range(args.steps) if i % EVENT_STRIDE == 0]
    evs = None if args.no_events else dict(zip(sampled, make_events(len(sampled))))
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        step(i, None if evs is None else evs.get(i))
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    ms_per_step = elapsed / args.steps * 1e3

    def event_times_ms(pairs):
        """Elapsed milliseconds of every (begin, end) pair; the events are destroyed."""
        out_ms = []
        for a, e in pairs:
            ms = ctypes.c_float()
            assert hip.hipEventElapsedTime(ctypes.byref(ms), a, e) == 0
            out_ms.append(ms.value)
            hip.hipEventDestroy(a)
            hip.hipEventDestroy(e)
        return out_ms

    split_kernel_name, plan_ns, plan_tps = L.decode_plan_info(desc, b, N)
    split_ms = split_stats = None
    if evs is not None:
        ts = event_times_ms(evs.values())
        split_ms = sum(ts) / len(ts)
        split_stats = {"samples": len(ts), "mean_us": round(split_ms * 1e3, 2), "median_us": round(float(np.median(ts)) * 1e3, 2),
                       "min_us": round(min(ts) * 1e3, 2)}

    # ---- practical HBM read ceiling of this machine: the library's streaming-read probe over 2 GiB (far beyond the
    # 256 MB last-level cache), best of five launches
    probe_buf = torch.empty(1 << 31, dtype=torch.uint8, device=dev).random_(0, 255)
    probe_sink = torch.zeros(1, dtype=torch.int32, device=dev)
    L.stream_read_probe(probe_buf, probe_sink)
    torch.cuda.synchronize()
    pe = [[torch.cuda.Event(enable_timing=True) for _ in range(2)] for _ in range(5)]
    for a, e in pe:
        a.record()
        L.stream_read_probe(probe_buf, probe_sink)
        e.record()
    torch.cuda.synchronize()
    stream_ceiling_gbps = probe_buf.numel() / (min(a.elapsed_time(e) for a, e in pe) * 1e-3) / 1e9
    del probe_buf

    # ---- matrix-core rate this machine sustains: the library's MFMA probe (register operands, no memory traffic), on
    # pseudo-random operands and on zeros; the gap is what power management takes from the nominal peak
    mfma_ceiling = {}
    probe_wgs, probe_iters = 256, 20000
    probe_out = torch.empty(256 * probe_wgs, dtype=torch.float32, device=dev)
    for name_, mode_ in (("random_operands", 0), ("zero_operands", 1)):
        L.mfma_rate_probe(probe_out, probe_wgs, probe_iters, mode_)
        torch.cuda.synchronize()
        pe = [[torch.cuda.Event(enable_timing=True) for _ in range(2)] for _ in range(3)]
        for a, e in pe:
            a.record()
            L.mfma_rate_probe(probe_out, probe_wgs, probe_iters, mode_)
            e.record()
        torch.cuda.synchronize()
        mfma_ceiling[name_] = round(4.0 * probe_wgs * probe_iters * 8 * 32768 / (min(a.elapsed_time(e) for a, e in pe) * 1e-3) / 1e12, 1)
    del probe_out

    if args.copy_probe:
        src = torch.zeros(1 << 30, dtype=torch.uint8, device=dev)
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    # ---- roofline of the dominant kernel (decode split): algorithmic work per launch
    positions = b * N
    latent_bytes = positions * 2 * (r + r)                                    # bf16 K and V latents read once
    flops = positions * (2 * r * n + 2 * h_q * d + 2 * h_q * r)               # rebuild K, scores, latent-space PV
    roof = None
    if split_ms:
        t = split_ms * 1e-3
        tflops = flops / t / 1e12
        gbps = latent_bytes / t / 1e9
        roof = {"kernel": split_kernel_name, "n_splits": plan_ns, "tiles_per_split": plan_tps, "bound": "mfma", "achieved": round(tflops, 2),
                "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s", "frac": round(tflops / MFMA_BF16_PEAK_TFLOPS, 4),
                "traffic": SPLIT_TRAFFIC_BYTES_PROFILED if args.pools == 8 else None, "traffic_unit": "bytes/launch",
                "avg_launch_us": round(split_ms * 1e3, 2), "launch_us": split_stats, "flops_per_launch": flops,
                "hbm_bytes_per_launch": latent_bytes, "hbm_achieved_gbps": round(gbps, 1),
                "hbm_peak_gbps": HBM_PEAK_GBPS, "hbm_frac": round(gbps / HBM_PEAK_GBPS, 4),
                "hbm_stream_ceiling_gbps": round(stream_ceiling_gbps, 1),
                "mfma_sustained_tflops": mfma_ceiling}

    # ---- absorbed-query leg: the same cache, shapes and step, for a model without positional rotation (the key
    # factor folded into the query): nothing is rebuilt, the step is one stream over the latents -> HBM roofline
    absorbed = None
    out_abs = None
    if not args.no_absorbed:
        q_lat_np = np.stack([np.stack([B_k[:, (h // (h_q // h_kv)) * d:(h // (h_q // h_kv) + 1) * d] @ q_np[s, h].astype(np.float64)
                                       for h in range(h_q)]) for s in range(b)])
        q_lat = bf(q_lat_np)
        out_abs = torch.empty_like(q)
        ws_abs = torch.empty(L.decode_absorbed_workspace_bytes(desc, b, N), dtype=torch.uint8, device=dev)

        def step_abs(i, events=None):
            pool = pools[i % len(pools)]
            L.append_latent(desc, x_new, packed, slot_seq, slot_pos, bt, pool)
            L.decode_attention_absorbed(desc, q_lat, ctx_len, N, packed, pool, bt, out=out_abs, workspace=ws_abs, events=events)

        for i in range(args.warmup):
            step_abs(i)
        torch.cuda.synchronize()
        evs_a = None if args.no_events else dict(zip(sampled, make_events(len(sampled))))
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(args.steps):
            step_abs(i, None if evs_a is None else evs_a.get(i))
        torch.cuda.synchronize()
        ms_abs = (time.perf_counter() - t0) / args.steps * 1e3
        absorbed = {"workload": "configs[1] shapes and cache, no positional rotation, q_lat = B_k q (Section 4.1, Eq. 7)",
                    "step": "lorc_append_latent(16 tokens) + lorc_decode_attention_absorbed",
                    "ms_per_step": round(ms_abs, 5), "tok_per_s": round(b / (ms_abs * 1e-3), 1)}
        if evs_a is not None:
            ts_a = event_times_ms(evs_a.values())
            t_k = sum(ts_a) / len(ts_a) * 1e-3
            absorbed["roofline"] = {"kernel": "decode_absorbed_kernel", "bound": "hbm",
                                    "achieved": round(latent_bytes / t_k / 1e9, 1), "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                                    "frac": round(latent_bytes / t_k / 1e9 / HBM_PEAK_GBPS, 4),
                                    "traffic": ABSORBED_TRAFFIC_BYTES_PROFILED if args.pools == 8 else None,
                                    "traffic_unit": "bytes/launch",
                                    "avg_launch_us": round(t_k * 1e6, 2),
                                    "launch_us": {"samples": len(ts_a), "median_us": round(float(np.median(ts_a)) * 1e3, 2), "min_us": round(min(ts_a) * 1e3, 2)},
                                    "hbm_stream_ceiling_gbps": round(stream_ceiling_gbps, 1), "hbm_bytes_per_launch": latent_bytes,
                                    "flops_per_launch": positions * (2 * h_q * r + 2 * h_q * r)}

        # the same kernel on a context long enough to amortise its fixed costs: 16 x 65536 positions (2.1 GB of
        # latents, sampled directly as N(0, 1) bf16 -- the step never looks at how a latent was produced)
        if not args.no_events:
            NL = 65536
            pages_l = NL // L.PAGE_TOKENS
            n_pages_l = b * pages_l + 3
            bt_l = torch.from_numpy(gen.block_table(b, pages_l, n_pages_l, seed=seed + 1)).to(dev)
            cache_l = torch.empty(n_pages_l * page_bytes // 2, dtype=torch.bfloat16, device=dev).normal_().view(torch.uint8)
            ctx_l = torch.full((b,), NL, dtype=torch.int32, device=dev)
            ws_l = torch.empty(L.decode_absorbed_workspace_bytes(desc, b, NL), dtype=torch.uint8, device=dev)
            reps_l = 20
            for _ in range(3):
                L.decode_attention_absorbed(desc, q_lat, ctx_l, NL, packed, cache_l, bt_l, out=out_abs, workspace=ws_l)
            evs_l = make_events(reps_l)
            torch.cuda.synchronize()
            for i in range(reps_l):
                L.decode_attention_absorbed(desc, q_lat, ctx_l, NL, packed, cache_l, bt_l, out=out_abs, workspace=ws_l, events=evs_l[i])
            torch.cuda.synchronize()
            t_l = sum(event_times_ms(evs_l)) / reps_l * 1e-3
            bytes_l = b * NL * 2 * (r + r)
            absorbed["long_context"] = {"context": NL, "batch": b, "kernel": "decode_absorbed_kernel", "avg_launch_us": round(t_l * 1e6, 1),
                                        "hbm_bytes_per_launch": bytes_l, "achieved_gbps": round(bytes_l / t_l / 1e9, 1),
                                        "frac_of_hbm_peak": round(bytes_l / t_l / 1e9 / HBM_PEAK_GBPS, 4)}
            del cache_l, ws_l
            # restore the configs[1] result for the cross-check below
            step_abs(0)
            torch.cuda.synchronize()

    # ---- prefill leg (configs[3]): down-projection of 4 x 8192 tokens into the paged cache + causal attention
    prefill = None
    if not args.no_prefill:
        c3 = gen.CONFIGS[3]
        pb3, N3 = c3["batch"], c3["context"]
        T3 = pb3 * N3
        pages3 = N3 // L.PAGE_TOKENS
        n_pages3 = pb3 * pages3 + 3
        bt3 = torch.from_numpy(gen.block_table(pb3, pages3, n_pages3, seed=c3["seed"])).to(dev)
        cache3 = torch.zeros(n_pages3 * page_bytes, dtype=torch.uint8, device=dev)
        x3 = torch.cat([torch.from_numpy(gen.hidden_states(N3, D, seed=70000 + s)).to(dev).to(torch.bfloat16) for s in range(pb3)])
        q3 = torch.cat([torch.from_numpy(gen.queries(N3, h_q, d, seed=71000 + s)).to(dev).to(torch.bfloat16) for s in range(pb3)])
        seq3 = torch.arange(pb3, dtype=torch.int32, device=dev).repeat_interleave(N3).contiguous()
        pos3 = torch.arange(N3, dtype=torch.int32, device=dev).repeat(pb3).contiguous()
        cu3 = torch.arange(0, T3 + 1, N3, dtype=torch.int32, device=dev)
        ws3 = torch.empty(L.prefill_workspace_bytes(desc, pb3, N3), dtype=torch.uint8, device=dev)
        out3 = torch.empty_like(q3)
        if args.zero_data:
            x3.zero_()
            q3.zero_()
        reps = 5
        # all iterations are queued before the first one is waited for: an iteration that starts on an idle GPU would
        # count the host's launch latency into its first kernel
        ev = [[torch.cuda.Event(enable_timing=True) for _ in range(3)] for _ in range(reps + 1)]
        for it in range(reps + 1):
            ev[it][0].record()
            L.append_latent(desc, x3, packed, seq3, pos3, bt3, cache3)
            ev[it][1].record()
            L.prefill_attention(desc, q3, cu3, N3, packed, cache3, bt3, out=out3, workspace=ws3)
            ev[it][2].record()
        torch.cuda.synchronize()
        t_ap = sum(ev[it][0].elapsed_time(ev[it][1]) for it in range(1, reps + 1)) / reps
        t_at = sum(ev[it][1].elapsed_time(ev[it][2]) for it in range(1, reps + 1)) / reps
        f_ap = 2.0 * T3 * D * (2 * r)
        f_at = pb3 * (2.0 * N3 * n * (2 * r) + 2.0 * 2.0 * h_q * d * N3 * (N3 + 1) / 2)   # rebuild K,V + causal QK^T, PV
        prefill = {"workload": "configs[3]: batch 4 x 8192 tokens, rank 512/512, paged cache",
                   "down_projection_ms": round(t_ap, 4), "down_projection_tflops": round(f_ap / t_ap / 1e9, 1),
                   "down_projection_mfma_frac": round(f_ap / t_ap / 1e9 / MFMA_BF16_PEAK_TFLOPS, 4),
                   "attention_ms": round(t_at, 4), "attention_tflops": round(f_at / t_at / 1e9, 1),
                   "attention_mfma_frac": round(f_at / t_at / 1e9 / MFMA_BF16_PEAK_TFLOPS, 4),
                   "prefill_tok_per_s": round(T3 / ((t_ap + t_at) * 1e-3), 1)}
        del x3, q3, cache3, ws3, out3

    # ---- decode legs at the other benchmark configurations.  Their hidden states would be 2 .. 34 GB per layer, so
    # the caches are filled directly with latents c_j ~ N(0, sigma_j^2) (the law of x U_r Sigma_r for x ~ N(0, I),
    # drawn on the device in the page tiling), and the factors are drawn too: B with orthonormal rows, A with
    # column norms sigma_j.  The kernels do not look at how a latent was produced; parity for these layer shapes is
    # in tests/.  One step = every layer's lorc_append_latent (one token per sequence) + lorc_decode_attention.
    def decode_stack_leg(tag, D2, hq2, hkv2, ranks, b2, N2, base2, steps2, seed2, plain=False):
        """plain: uncompressed layers (rank = n, keys and values cached themselves, lorc_decode_attention_plain)."""
        n2 = hkv2 * d
        sigma = gen.power_law_spectrum(n2)
        gcpu = torch.Generator(device="cpu").manual_seed(seed2)
        gdev = torch.Generator(device=dev).manual_seed(seed2)
        pages2 = N2 // L.PAGE_TOKENS
        n_pages2 = b2 * pages2 + 3
        bt2 = torch.from_numpy(gen.block_table(b2, pages2, n_pages2, seed=seed2)).to(dev)
        slot = np.arange(L.PAGE_TOKENS)[:, None]
        layers = []
        by_rank = {}
        for r2 in ranks:
            desc2 = L.layer_desc(D2, hq2, hkv2, d, r2, r2, base2)
            if r2 not in by_rank:   # layers of equal rank share their factors (same synthetic spectrum)
                qmat, _ = torch.linalg.qr(torch.randn(n2, r2, generator=gcpu, dtype=torch.float32))
                Bf = None if plain else qmat.t().contiguous().to(dev).to(torch.bfloat16)   # [r, n], orthonormal rows
                Af = (torch.randn(D2, r2, generator=gcpu, dtype=torch.float32) * torch.from_numpy(sigma[:r2] / np.sqrt(D2)).float()).to(dev).to(torch.bfloat16)
                packed2 = L.pack_factors(desc2, Af, Af, Bf, Bf)
                # per-element standard deviation of a page: sigma_j at the tiled position of latent j
                idx_k = ((slot // 32 * (r2 // 16) + np.arange(r2)[None, :] // 16) * 64 + slot % 32 + 32 * ((np.arange(r2)[None, :] % 16) // 8)) * 8 + np.arange(r2)[None, :] % 8
                idx_v = 64 * r2 + (((np.arange(r2)[None, :] // 32) * 4 + slot // 16) * 64 + np.arange(r2)[None, :] % 32 + 32 * ((slot % 16) // 8)) * 8 + slot % 8
                scale = np.empty(64 * 2 * r2, np.float32)
                scale[idx_k.reshape(-1)] = np.broadcast_to(sigma[:r2].astype(np.float32), (64, r2)).reshape(-1)
                scale[idx_v.reshape(-1)] = np.broadcast_to(sigma[:r2].astype(np.float32), (64, r2)).reshape(-1)
                by_rank[r2] = (packed2, torch.from_numpy(scale).to(dev))
            packed2, scale_d = by_rank[r2]
            cache2 = torch.empty(n_pages2, 64 * 2 * r2, dtype=torch.bfloat16, device=dev)
            cache2.normal_(generator=gdev)
            cache2.mul_(scale_d.to(torch.bfloat16))
            layers.append((desc2, packed2, cache2.view(-1).view(torch.uint8)))
        x2 = torch.randn(b2, D2, generator=gdev, device=dev, dtype=torch.float32).to(torch.bfloat16)
        q2 = torch.randn(b2, hq2, d, generator=gdev, device=dev, dtype=torch.float32).to(torch.bfloat16)
        sseq = torch.arange(b2, dtype=torch.int32, device=dev)
        spos = torch.full((b2,), N2 - 1, dtype=torch.int32, device=dev)
        ctx2 = torch.full((b2,), N2, dtype=torch.int32, device=dev)
        out2 = torch.empty_like(q2)
        ws_bytes = L.decode_plain_workspace_bytes if plain else L.decode_workspace_bytes
        ws2 = torch.empty(max(ws_bytes(ds, b2, N2) for ds, _, _ in layers), dtype=torch.uint8, device=dev)

        def stack_step(events=None):
            for li, (ds, pk, ch) in enumerate(layers):
                L.append_latent(ds, x2, pk, sseq, spos, bt2, ch)
                if plain:   # no event-bracketed variant: the whole call (two streaming launches + merge) is timed
                    if events is not None:
                        assert hip.hipEventRecord(ctypes.c_void_p(events[li][0]), ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)) == 0
                    L.decode_attention_plain(ds, q2, spos, ctx2, N2, pk, ch, bt2, out=out2, workspace=ws2)
                    if events is not None:
                        assert hip.hipEventRecord(ctypes.c_void_p(events[li][1]), ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)) == 0
                else:
                    L.decode_attention(ds, q2, spos, ctx2, N2, pk, ch, bt2, out=out2, workspace=ws2,
                                       events=None if events is None else events[li])

        for _ in range(2):
            stack_step()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps2):
            stack_step()
        torch.cuda.synchronize()
        ms_step = (time.perf_counter() - t0) / steps2 * 1e3
        evl = make_events(len(layers))
        stack_step(evl)
        torch.cuda.synchronize()
        per_layer_ms = event_times_ms(evl)
        assert bool(torch.isfinite(out2.float()).all())
        pos2 = b2 * N2
        lat_bytes = sum(pos2 * 4 * r2 for r2 in ranks)
        fl = sum(pos2 * ((0 if plain else 2 * r2 * n2) + 2 * hq2 * d + 2 * hq2 * (d if plain else r2)) for r2 in ranks)
        t_split = sum(per_layer_ms) * 1e-3
        kname = "plain_scores_kernel + latent_pv_kernel + decode_merge_kernel" if plain else sorted({L.decode_plan_info(ds, b2, N2)[0] for ds, _, _ in layers})
        rec2 = {"workload": tag, "layers": len(ranks), "batch": b2, "context": N2, "ranks": sorted(set(ranks), reverse=True), "kernels": kname,
                "cache_fill": "latents sampled directly, N(0, sigma_j^2); factors sampled (orthonormal B)",
                "ms_per_step": round(ms_step, 4), "tok_per_s": round(b2 / (ms_step * 1e-3), 1),
                "latent_gb_per_step": round(lat_bytes / 1e9, 2), "achieved_hbm_gbps_whole_step": round(lat_bytes / (ms_step * 1e-3) / 1e9, 1),
                "split_kernel": {"sum_ms": round(sum(per_layer_ms), 4),
                                 "per_layer_ms": {"first": round(per_layer_ms[0], 4), "median": round(float(np.median(per_layer_ms)), 4), "last": round(per_layer_ms[-1], 4)},
                                 "tflops": round(fl / t_split / 1e12, 1), "mfma_frac": round(fl / t_split / 1e12 / MFMA_BF16_PEAK_TFLOPS, 4),
                                 "hbm_gbps": round(lat_bytes / t_split / 1e9, 1), "hbm_frac": round(lat_bytes / t_split / 1e9 / HBM_PEAK_GBPS, 4)}}
        del layers, by_rank
        torch.cuda.empty_cache()
        return rec2

    stack = share = wide13 = plain8 = None
    if not args.no_wide:
        # Table 2's LLaMA-2-13B row (40 MHA heads, n = D = 5120, rank 2048): one layer, batch 16, context 4096; and the 8B
        # layer shape left uncompressed (Algorithm 1's threshold): keys and values themselves in the cache, batch 16, context 4096
        wide13 = decode_stack_leg("LLaMA-2-13B layer shape: MHA 40 heads, D 5120, rank 2048, batch 16, context 4096 (three-launch path)",
                                  5120, 40, 40, [2048], 16, 4096, 10000.0, 5, 13)
        plain8 = decode_stack_leg("8B layer shape, uncompressed (rank = n = 1024): batch 16, context 4096", D, h_q, h_kv, [n], b, N, base, 20, 8, plain=True)
    if not args.no_stack:
        c2 = gen.CONFIGS[2]
        stack = decode_stack_leg("configs[2]: 32-layer 8B-shaped stack, ranks 768 -> 384 (gen.rank_ramp), batch 32, context 8192",
                                 c2["d_model"], c2["n_q_heads"], c2["n_kv_heads"], gen.rank_ramp(c2["layers"], c2["rank_first"], c2["rank_last"]),
                                 c2["batch"], c2["context"], c2["rope_base"], 5, c2["seed"])
    if not args.no_share:
        c4 = gen.CONFIGS[4]
        share = decode_stack_leg("configs[4]: 70B-shaped 8-layer share, D 8192, 64q/8kv heads, rank 512, batch 64, context 32768",
                                 c4["d_model"], c4["n_q_heads"], c4["n_kv_heads"], [c4["rank"]] * c4["layers"], c4["batch"], c4["context"],
                                 c4["rope_base"], 5, c4["seed"])

    # ---- CPU baseline: the fp64 oracle, as it stands, on a bounded sample of the same workload
    cpu = None
    if not args.no_cpu_baseline:
        from oracle import lorc_oracle as orc
        t0 = time.perf_counter()
        Wt_k, _ = orc.low_rank_weight(W_k, r)
        Wt_v, _ = orc.low_rank_weight(W_v, r)
        t_svd = time.perf_counter() - t0
        done, t_or, errs = 0, 0.0, []
        got = out.float().cpu().numpy().astype(np.float64)
        while done < b and (done < 2 or t_or < 12.0):
            s = done
            t0 = time.perf_counter()
            X = X_host[s].astype(np.float64)
            K = orc.split_heads(X @ Wt_k, h_kv, d)
            V = orc.split_heads(X @ Wt_v, h_kv, d)
            ref = orc.attention_decode(q_np[s].astype(np.float64), N - 1, K, V, np.arange(N), base)
            t_or += time.perf_counter() - t0
            errs.append(float(np.max(np.abs(got[s] - ref)) / np.max(np.abs(ref))))
            if s == 0 and out_abs is not None:  # the absorbed leg's output against the oracle without rotation
                ref_p = orc.attention_decode_plain(q_np[s].astype(np.float64), K, V)
                got_p = out_abs[s].float().cpu().numpy().astype(np.float64)
                absorbed["max_rel_err_vs_oracle_seq0"] = round(float(np.max(np.abs(got_p - ref_p)) / np.max(np.abs(ref_p))), 5)
            done += 1
        cores = len(os.sched_getaffinity(0))
        cpu = {"value": round(done / t_or, 3), "unit": "tok/s", "cores": cores, "kind": "oracle",
               "sample": f"{done} of {b} sequences of the same workload (materialise K~,V~ for {N} positions + "
                         f"attention, fp64 numpy); offline SVD of W_k,W_v timed apart: {t_svd:.2f} s",
               "max_rel_err_vs_gpu": round(max(errs), 5)}

    rec = {
        "metric": "decode tok/s + achieved HBM GB/s, low-rank KV attention (8B-shaped)",
        "value": round(b / (ms_per_step * 1e-3), 1), "unit": "tok/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": round(ms_per_step, 5), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "bf16",
        "data": "zeros (power probe: the same launches without switching activity in the operands; not a measurement of the workload)" if args.zero_data else "synthetic",
        "config": {"workload": "configs[1]: LLaMA-3-8B-shaped single layer decode, D=4096, 32q/8kv heads, d=128, "
                               "rank 512/512 of 1024, batch 16, context 4096, RoPE base 500000, page 64",
                   "step": "lorc_append_latent(16 tokens) + lorc_decode_attention", "cache_pools": len(pools),
                   "per_layer": True},
        "achieved_hbm_gbps_whole_step": round(latent_bytes / (ms_per_step * 1e-3) / 1e9, 1),
        "roofline": roof, "cpu_baseline": cpu, "prefill": prefill, "absorbed": absorbed,
        "stack_configs2": stack, "share_configs4": share, "wide_13b": wide13, "uncompressed_8b": plain8,
        "setup": {"factorize_s": round(t_factorize, 2), "rel_frob_err_k": round(eps_k, 4), "rel_frob_err_v": round(eps_v, 4),
                  "setup_s": round(t_setup, 1)},
    }
    print(json.dumps(rec))


if __name__ == "__main__":
    main()
