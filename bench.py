#!/usr/bin/env python3
"""Benchmark of the fused CCD compression step (ccd_compress) on one MI355X.

A step is one ccd_compress call over one full pot of the headline configuration (32 layers x 8 KV heads
x 128, 32 query heads, pot 4096 -> 2048, 64 CaP query tokens, T = 1024 NuC slots, max-pool window 7, bf16,
synthetic seeded data).  Every call of a pass gets a pot (K, V) that has not been compressed before (as many
pots as warm-up + timed steps are resident in HBM, 0.5 GiB each; they are refilled with fresh seeded data between
the passes), and the calls cycle over 4 catalyst-query sets and 5 novelty vectors.  No call finds its cache
warm, and the kept set is spread over the whole pot, as in steady-state streaming where half of the pot is new
context: nearly every kept row moves.  (Re-compressing the same few pots over and over instead lets copies of
the best-scoring rows pile up in them, and after some dozens of calls a growing prefix of every pot stays put.)
Prints one JSON line.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

HBM_PEAK_GBPS = 8000.0          # MI355X HBM3E
MFMA_BF16_PEAK_TFLOPS = 2500.0  # dense bf16
VALU_FP32_PEAK_TFLOPS = 157.3
# HBM bytes per launch on the headline config from the committed rocprofv3 counter runs
# (profiles/ccd_compress_c3_hbm_traffic.md: FETCH_SIZE x 2.00 + WRITE_SIZE x 1.00, the factors a plain copy of known
# size gives; equal to read requests x 128 B + write requests x 64 B)
MEASURED_TRAFFIC_C3 = {"score_stats": 286_600_000, "score_prob": 290_700_000, "select_compact": 543_300_000,
                       "score_unit": 525_400_000}
TRAFFIC_SOURCE = "profiles/ccd_compress_c3_hbm_traffic.md (a committed counter run, not this run)"


def algorithmic_bytes(cfg) -> dict:
    """Bytes the method has to move per call, by stage and for the whole call: K and Q_cat read once per score pass,
    kept K and V rows read and written once, the score row, novelty and keep_idx."""
    e = 4 if cfg.dtype == "fp32" else 2
    u, N, k, d, GP = cfg.units, cfg.N, cfg.k, cfg.d, cfg.G * cfg.P
    kbytes, qbytes = u * N * d * e, u * GP * d * e
    rows = u * k * d * e
    return {
        "score_stats": kbytes + qbytes,
        "score_merge": 0,
        "score_prob": kbytes + qbytes + u * N * 4,
        "score_unit": 2 * kbytes + qbytes + u * N * 4,      # both passes in one kernel: K twice
        "select": u * N * 4 + cfg.B * N * 4 + u * k * 4,
        "compact": 4 * rows + u * k * 4,
        # selection and compaction in one kernel: keep_idx is written once and never read back
        "select_compact": u * N * 4 + cfg.B * N * 4 + u * k * 4 + 4 * rows,
        # causal variant (--kcat): Q_cat and the CaP keys read, one (max, sum) pair per query written
        "cap_block": qbytes + u * cfg.P * d * e + u * GP * 8,
        # sliding window (--window): both head kernels read Q_cat and the hidden rows of K (at most P + 31 per unit)
        "window_head": 2 * (qbytes + u * (cfg.P + 31) * d * e),
        # whole call: K read once, Q_cat once, kept V rows read once, K' and V' written once, keep_idx, novelty
        "call": kbytes + qbytes + rows + 2 * rows + u * k * 4 + cfg.B * N * 4,
    }


def algorithmic_flops(cfg) -> float:
    return 2.0 * cfg.units * cfg.G * cfg.P * cfg.N * cfg.d


def stream_measure(reps, dev, torch, ip, synth):
    """Streaming use of the step (Sec. 3.2): a 131072-token context of a 32-layer, 8-KV-head, d 128 model is fed into a
    pot of 4096 in 2048-token chunks (seeded synthetic K, V, novelty already resident in HBM); whenever the next chunk
    does not fit, the pot is distilled to 2048 first: 62 calls.  Returns (best seconds per context, calls, all times,
    algorithmic bytes per context: the 62 calls plus reading and writing every appended chunk)."""
    from paper_2410_01518_amd.pot import MemoryPot
    cfg = synth.CONFIGS["c3"]
    context, chunk = 131072, 2048
    g = torch.Generator(device=dev).manual_seed(99)
    kv_shape = (cfg.B, cfg.L, cfg.Hkv, chunk, cfg.d)
    chunks = [(torch.empty(kv_shape, dtype=torch.bfloat16, device=dev).normal_(generator=g),
               torch.empty(kv_shape, dtype=torch.bfloat16, device=dev).normal_(generator=g),
               torch.rand((cfg.B, chunk), generator=g, device=dev, dtype=torch.float32)) for _ in range(8)]
    qsets = [torch.empty((cfg.B, cfg.L, cfg.Hq, cfg.P, cfg.d), dtype=torch.bfloat16, device=dev).normal_(generator=g)
             for _ in range(4)]

    def run():
        pot = MemoryPot(cfg.B, cfg.L, cfg.Hkv, cfg.d, cfg.N, cfg.k, cfg.T, pool_w=cfg.w)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for c in range(context // chunk):
            if pot.room < chunk:
                rc = pot.distill(qsets[c % len(qsets)])
                assert rc == ip.CCD_OK, rc
            Kc, Vc, nv = chunks[c % len(chunks)]
            pot.append(Kc, Vc, nv)
        torch.cuda.synchronize()
        return time.perf_counter() - t0, pot.calls

    run()                                         # warm-up: allocations, first launches
    times = [run() for _ in range(reps)]
    dt, calls = min(t for t, _ in times), times[0][1]
    chunk_bytes = 2 * cfg.units * chunk * cfg.d * 2                  # K and V of a chunk
    nbytes = calls * algorithmic_bytes(cfg)["call"] + (context // chunk) * 2 * chunk_bytes
    return dt, calls, [t for t, _ in times], nbytes, context


def stream_bench(args, dev, torch, ip, synth) -> int:
    reps = max(1, min(args.steps, 5))
    dt, calls, times, nbytes, context = stream_measure(reps, dev, torch, ip, synth)
    gbps = nbytes / dt / 1e9
    print(json.dumps({"metric": "streaming CCD cache maintenance tokens/s (32L x 8KV x 128d, pot 4096 -> 2048, 2048-token chunks)",
                      "value": context / dt, "unit": "tokens/s", "n_gpus": 1, "steps": reps, "warmup": 1,
                      "ms_per_step": dt * 1e3, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
                      "dtype": "bf16", "data": "synthetic",
                      "config": {"workload": f"131072-token context, {calls} ccd_compress calls, per-head novelty",
                                 "ms_per_context": dt * 1e3, "all_repetitions_ms": [t * 1e3 for t in times]},
                      "roofline": {"kernel": "whole context (calls + appends)", "bound": "hbm", "achieved": gbps,
                                   "peak": HBM_PEAK_GBPS, "unit": "GB/s", "frac": gbps / HBM_PEAK_GBPS, "traffic": None},
                      "cpu_baseline": None}))
    return 0


def small_config_latency(cfg, dev, torch, ip, synth, calls=40):
    """Microseconds per ccd_compress call (HIP events around `calls` back-to-back calls, each on its own copy of the pot)
    of a configuration that is far too small to fill the chip."""
    host = synth.make_inputs(cfg)

    def upload(a):
        if a.dtype == np.uint16:
            return torch.from_numpy(a.view(np.int16)).view(torch.bfloat16).to(dev)
        return torch.from_numpy(a).to(dev)

    d0 = {k: upload(v) for k, v in host.items()}
    pots = [(d0["K"].clone(), d0["V"].clone()) for _ in range(calls + 4)]
    shape = ip.make_shape(d0["Q_cat"], pots[0][0], d0["novelty"], k=cfg.k, T=cfg.T, pool_w=cfg.w, pool_mode=ip.CCD_POOL_MAX)
    ws = ip.alloc_workspace(shape)
    keep = torch.empty((cfg.B, cfg.L, cfg.Hkv, cfg.k), dtype=torch.int32, device=dev)
    for K, V in pots[calls:]:
        assert ip.ccd_compress(shape, d0["Q_cat"], K, V, d0["novelty"], keep, ws) == ip.CCD_OK
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for K, V in pots[:calls]:
        ip.ccd_compress(shape, d0["Q_cat"], K, V, d0["novelty"], keep, ws)
    e1.record()
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) * 1e3 / calls


def other_configs(dev, torch, ip, synth) -> list:
    """The benchmark's other single-GPU configurations next to the headline one, a few seconds in all: the tiny fp32
    call (c1), the single GQA layer (c2) and the streaming use (c4).  (The large-pot configuration needs 43 GB per pot:
    `--aux stress`.)"""
    out = []
    for name in ("c1", "c2"):
        cfg = synth.CONFIGS[name]
        us = small_config_latency(cfg, dev, torch, ip, synth)
        gbps = algorithmic_bytes(cfg)["call"] / (us * 1e-6) / 1e9
        out.append({"workload": f"{name}: L{cfg.L} Hq{cfg.Hq} Hkv{cfg.Hkv} d{cfg.d} {cfg.dtype} N{cfg.N}->k{cfg.k} P{cfg.P} pool{cfg.w}",
                    "value": us, "unit": "us per ccd_compress call", "bound": "launch latency (a few workgroups)",
                    "achieved_GBps": gbps, "frac_of_hbm_peak": gbps / HBM_PEAK_GBPS})
    dt, calls, times, nbytes, context = stream_measure(2, dev, torch, ip, synth)
    gbps = nbytes / dt / 1e9
    out.append({"workload": f"c4: 131072-token context in 2048-token chunks through a pot of 4096, {calls} ccd_compress calls",
                "value": context / dt, "unit": "tokens/s", "bound": "hbm", "achieved_GBps": gbps,
                "frac_of_hbm_peak": gbps / HBM_PEAK_GBPS, "ms_per_context": dt * 1e3})
    return out


def stress_bench(args, dev, torch, ip, synth) -> int:
    """The large-pot configuration at full size: 4 sequences x 80 layers x 8 KV heads (2560 units), 64 query heads,
    pot 32768 -> 4096, 128 CaP tokens, bf16; keys N(0,1) x sqrt(min(z_t, 64)), z_t ~ Zipf(1.1) per (sequence, token).
    A pot is 43 GB, so the inputs are drawn on the device, and every call (1 warm-up, up to 3 timed, then as many
    again with an event after every kernel) gets a pot that has not been compressed before."""
    cfg = synth.CONFIGS["c5"]
    g = torch.Generator(device=dev).manual_seed(5005)
    rng = np.random.default_rng(5005)
    z = np.minimum(rng.zipf(1.1, size=(cfg.B, cfg.N)), 64).astype(np.float32)
    gain = torch.from_numpy(np.sqrt(z)).to(dev)[:, None, None, :, None]
    kv_shape = (cfg.B, cfg.L, cfg.Hkv, cfg.N, cfg.d)
    pot_bytes = 2 * cfg.units * cfg.N * cfg.d * 2
    n_pots = min(4, int(0.85 * torch.cuda.mem_get_info()[0]) // pot_bytes)
    if n_pots < 2:
        print("bench.py: --aux stress needs room for two 43 GB pots", file=sys.stderr)
        return 2
    steps = max(1, min(args.steps, n_pots - 1))

    def draw(K, V):
        for b in range(cfg.B):
            K[b] = (torch.randn(K[b].shape, generator=g, device=dev, dtype=torch.float32) * gain[b]).to(torch.bfloat16)
        V.normal_(generator=g)

    pots = [(torch.empty(kv_shape, dtype=torch.bfloat16, device=dev), torch.empty(kv_shape, dtype=torch.bfloat16, device=dev))
            for _ in range(n_pots)]
    for K, V in pots:
        draw(K, V)
    Q = torch.randn((cfg.B, cfg.L, cfg.Hq, cfg.P, cfg.d), generator=g, device=dev, dtype=torch.float32).to(torch.bfloat16)
    nov = torch.rand((cfg.B, cfg.N), generator=g, device=dev, dtype=torch.float32)
    shape = ip.make_shape(Q, pots[0][0], nov, k=cfg.k, T=cfg.T, pool_w=cfg.w, pool_mode=ip.CCD_POOL_MAX)
    ws = ip.alloc_workspace(shape)
    keep = torch.empty((cfg.B, cfg.L, cfg.Hkv, cfg.k), dtype=torch.int32, device=dev)
    stream = torch.cuda.current_stream()

    def step(i):
        K, V = pots[i]
        rc = ip.ccd_compress(shape, Q, K, V, nov, keep, ws, stream=stream)
        assert rc == ip.CCD_OK, rc

    step(n_pots - 1)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(steps):
        step(i)
    torch.cuda.synchronize()
    ms = (time.perf_counter() - t0) * 1e3 / steps
    for K, V in pots[:steps]:
        draw(K, V)
    torch.cuda.synchronize()
    ip.ccd_profile_enable(True)
    for i in range(steps):
        step(i)
    stage_ms, calls = ip.ccd_profile_collect()
    ip.ccd_profile_enable(False)
    stage_us = {k: 1e3 * v / max(calls, 1) for k, v in stage_ms.items() if v > 0}
    ab = algorithmic_bytes(cfg)
    dom = max(stage_us, key=stage_us.get)
    t = stage_us[dom] * 1e-6
    if dom in ("score_stats", "score_prob", "score_unit"):
        roof = {"kernel": dom, "bound": "mfma", "achieved": algorithmic_flops(cfg) * (2 if dom == "score_unit" else 1) / t / 1e12, "peak": MFMA_BF16_PEAK_TFLOPS,
                "unit": "TFLOP/s"}
    else:
        roof = {"kernel": dom, "bound": "hbm", "achieved": ab[dom] / t / 1e9, "peak": HBM_PEAK_GBPS, "unit": "GB/s"}
    roof["frac"] = roof["achieved"] / roof["peak"]
    roof["traffic"] = None
    print(json.dumps({"metric": "ccd_compress calls/s (large pot: 4 x 80L x 8KV x 128d, 64 query heads, pot 32768 -> 4096, 128 CaP tokens)",
                      "value": 1e3 / ms, "unit": "calls/s", "n_gpus": 1, "steps": steps, "warmup": 1, "ms_per_step": ms,
                      "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
                      "config": {"workload": f"{cfg.name}: B{cfg.B} L{cfg.L} Hq{cfg.Hq} Hkv{cfg.Hkv} d{cfg.d} N{cfg.N}->k{cfg.k} "
                                             f"P{cfg.P} T{cfg.T} pool{cfg.w}", "pots": n_pots, "pot_GB": pot_bytes / 1e9},
                      "call_hbm": {"algorithmic_bytes": ab["call"], "achieved_GBps": ab["call"] / (ms * 1e-3) / 1e9},
                      "stage_avg_us": stage_us, "roofline": roof, "cpu_baseline": None}))
    return 0


def aux_bench(args, cfg, dev, torch, ip, synth) -> int:
    """Stand-alone companion kernels (HBM-bound): HIP-event time over `steps` calls on rotating cold buffers."""
    g = torch.Generator(device=dev).manual_seed(77)
    steps, warmup = min(args.steps, 80), min(args.warmup, 8)
    if args.aux == "nuc":
        rows, V = 4096, 128256
        bufs = [torch.empty((rows, V), dtype=torch.bfloat16, device=dev).normal_(generator=g) for _ in range(4)]
        labels = torch.randint(0, V, (rows,), generator=g, device=dev, dtype=torch.int32)
        nov = torch.empty(rows, dtype=torch.float32, device=dev)
        call = lambda i: ip.ccd_nuc_from_logits(bufs[i % 4], labels, nov)
        nbytes, work = rows * V * 2 + rows * 8, f"{rows} x {V} bf16 logits"
        metric = "ccd_nuc_from_logits calls/s (per-token cross entropy, Eq. 3)"
    else:
        Ks = [torch.empty((cfg.B, cfg.L, cfg.Hkv, cfg.N, cfg.d), dtype=torch.bfloat16, device=dev).normal_(generator=g)
              for _ in range(8)]
        Q = torch.empty((cfg.B, cfg.L, cfg.Hq, cfg.P, cfg.d), dtype=torch.bfloat16, device=dev)
        k_rot = torch.empty_like(Ks[0])
        c, s = synth.rope_tables(cfg.k, cfg.d)
        c, s = torch.from_numpy(c).to(dev), torch.from_numpy(s).to(dev)
        shape = ip.make_shape(Q, Ks[0], None, k=cfg.k)
        call = lambda i: ip.ccd_cr_rope(shape, Ks[i % 8], c, s, cfg.k, k_rot)
        nbytes, work = 2 * cfg.units * cfg.k * cfg.d * 2, f"{cfg.name}: first {cfg.k} rows of {cfg.units} units, bf16 d{cfg.d}"
        metric = "ccd_cr_rope calls/s (CR-RoPE of the kept keys, Sec. 3.5)"
    for i in range(warmup):
        call(i)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for i in range(steps):
        call(i)
    e1.record()
    torch.cuda.synchronize()
    ms = e0.elapsed_time(e1) / steps
    gbps = nbytes / (ms * 1e-3) / 1e9
    cpu = None
    if not args.no_cpu_baseline:
        from oracle import ccd_oracle as O   # CPU baseline leg only
        c0 = time.perf_counter()
        if args.aux == "nuc":
            n_s = 256
            O.nuc_from_logits(bufs[0][:n_s].view(torch.int16).cpu().numpy().view(np.uint16), labels[:n_s].cpu().numpy())
            frac, sample = n_s / rows, f"{n_s} of {rows} rows"
        else:
            n_s = 16
            Kh = Ks[0].view(torch.int16).cpu().numpy().view(np.uint16).reshape(cfg.units, cfg.N, cfg.d)
            ch, sh_ = synth.rope_tables(cfg.k, cfg.d)
            for u in range(n_s):
                O.cr_rope(Kh[u, :cfg.k], ch, sh_)
            frac, sample = n_s / cfg.units, f"{n_s} of {cfg.units} units"
        dt = time.perf_counter() - c0
        cpu = {"value": frac / dt, "unit": "calls/s", "cores": 1, "kind": "oracle",
               "sample": f"{sample} in {dt:.2f} s, scaled to a whole call"}
    print(json.dumps({"cpu_baseline": cpu, "metric": metric, "value": 1e3 / ms, "unit": "calls/s", "n_gpus": 1, "steps": steps, "warmup": warmup,
                      "ms_per_step": ms, "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16",
                      "data": "synthetic", "config": {"workload": work},
                      "roofline": {"bound": "hbm", "achieved": gbps, "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                                   "frac": gbps / HBM_PEAK_GBPS, "traffic": None}}))
    return 0


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--ring", type=int, default=0,
                    help="pots cycled through (0: one fresh pot per call of a pass, as far as 60 %% of free HBM allows)")
    ap.add_argument("--config", default="c3")
    ap.add_argument("--score-path", type=int, default=0,
                    help="kernels for Eq. 2: 0 automatic, 1 vector ALUs, 2 matrix cores with a workgroup per token slice, "
                         "3 matrix cores with a workgroup per unit")
    ap.add_argument("--rope", action="store_true",
                    help="time ccd_compress_rope (CR-RoPE of the kept keys written on the side) instead of ccd_compress")
    ap.add_argument("--kcat", action="store_true",
                    help="the causal variant of Eq. 2: the CaP tokens' own keys join the softmax (ccd_compress_kcat, or "
                         "ccd_compress_rope with K_cap when combined with --rope)")
    ap.add_argument("--lse", action="store_true",
                    help="time ccd_compress_lse: the log-sum-exp of every CaP query row is handed in (as the attention "
                         "kernel of the model returns it), so the statistics pass over K is not run; the normalisers of "
                         "every pot are computed with torch outside the timed region")
    ap.add_argument("--per-head-novelty", action="store_true",
                    help="novelty carried per (layer, KV head) as in the cycles after the first one: [B, L, Hkv, N] "
                         "instead of [B, N]; it is compacted in place with K and V")
    ap.add_argument("--streams", type=int, default=1,
                    help="issue the timed calls round-robin over this many HIP streams (default priority), each with its "
                         "own workspace: how a server drives the step for several independent sequences; the per-kernel "
                         "pass stays on one stream")
    ap.add_argument("--window", type=int, default=0,
                    help="sliding attention window in tokens (0 = none), e.g. 4096 for a window as long as the pot")
    ap.add_argument("--aux", choices=["nuc", "cr_rope", "stream", "stress"], default=None,
                    help="time something else than the headline call: nuc = ccd_nuc_from_logits on 4096 x 128256 bf16 "
                         "logits, cr_rope = ccd_cr_rope on the kept half of a headline pot, stream = a 131072-token "
                         "context streamed through a pot of 4096 in 2048-token chunks (62 distillations), stress = the "
                         "large-pot configuration at full size (2560 units, pot 32768 -> 4096, 43 GB per pot)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-other-configs", action="store_true",
                    help="leave the other configurations (tiny call, single layer, streaming) out of the JSON line")
    ap.add_argument("--clock-warmup-ms", type=float, default=300.0,
                    help="before the W warm-up steps, keep calling on the warm-up pots for this long, so that the timed "
                         "steps of a short run do not fall into the clock ramp of an idle GPU (reported in the line)")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run a plain 256 MiB device copy a few times (reference for scaling rocprofv3's "
                         "FETCH_SIZE / WRITE_SIZE counters)")
    ap.add_argument("--cpu-units", type=int, default=0, help="units the CPU oracle is timed on (0 = the whole call)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (the units of a call are independent and would shard without "
              "communication); "
              f"--gpus {args.gpus} is not supported", file=sys.stderr)
        return 2

    import torch
    from paper_2410_01518_amd import infinipot as ip
    from paper_2410_01518_amd import synth

    cfg = synth.CONFIGS[args.config]
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    ip.lib()
    if args.aux == "stream":
        return stream_bench(args, dev, torch, ip, synth)
    if args.aux == "stress":
        return stress_bench(args, dev, torch, ip, synth)
    if args.aux is not None:
        return aux_bench(args, cfg, dev, torch, ip, synth)

    def upload(a):
        if a.dtype == np.uint16:
            return torch.from_numpy(a.view(np.int16)).view(torch.bfloat16).to(dev)
        return torch.from_numpy(a).to(dev)

    host0 = synth.make_inputs(cfg)                       # set 0: host-generated, also feeds the CPU baseline
    dev0 = {k: upload(v) for k, v in host0.items()}
    tdt = torch.float32 if cfg.dtype == "fp32" else torch.bfloat16
    g = torch.Generator(device=dev).manual_seed(1000 * cfg.seed)

    def randn(*shape):                                   # further sets: same recipe drawn on the device
        return torch.randn(shape, generator=g, device=dev, dtype=torch.float32).to(tdt)

    pot_bytes = 2 * dev0["K"].numel() * dev0["K"].element_size()
    n_pots = args.ring if args.ring > 0 else args.steps + args.warmup
    n_pots = max(1, min(n_pots, int(0.6 * torch.cuda.mem_get_info()[0]) // pot_bytes))

    def fresh(t):                                        # same recipe as synth: N(0,1) rounded to the storage dtype
        return t.normal_(generator=g)

    def refill():                                        # pot 0 from the host copy, the others drawn anew
        pots[0][0].copy_(upload(host0["K"]))
        pots[0][1].copy_(upload(host0["V"]))
        for K, V in pots[1:]:
            fresh(K)
            fresh(V)
        if args.per_head_novelty:
            for nv in novs:
                nv.uniform_(generator=g)

    pots = [(dev0["K"], dev0["V"])] + [(fresh(torch.empty_like(dev0["K"])), fresh(torch.empty_like(dev0["V"])))
                                       for _ in range(1, n_pots)]
    qsets = [dev0["Q_cat"]] + [randn(cfg.B, cfg.L, cfg.Hq, cfg.P, cfg.d) for _ in range(3)]
    nov_shape = (cfg.B, cfg.L, cfg.Hkv, cfg.N) if args.per_head_novelty else (cfg.B, cfg.N)
    novs = [dev0["novelty"]] + [torch.rand(nov_shape, generator=g, device=dev, dtype=torch.float32) for _ in range(4)]
    if args.per_head_novelty:
        # carried novelty is compacted with the pot it belongs to: one array per pot, redrawn whenever the pot is
        novs = [torch.rand(nov_shape, generator=g, device=dev, dtype=torch.float32) for _ in range(n_pots)]
    shape = ip.make_shape(qsets[0], pots[0][0], novs[0], k=cfg.k, T=cfg.T, pool_w=cfg.w, pool_mode=ip.CCD_POOL_MAX,
                          window=args.window, score_path=args.score_path)
    ws = ip.alloc_workspace(shape)
    keep = torch.empty((cfg.B, cfg.L, cfg.Hkv, cfg.k), dtype=torch.int32, device=dev)
    stream = torch.cuda.current_stream()
    n_streams = max(1, args.streams)
    lanes = [(stream, ws, keep)] + [(torch.cuda.Stream(), ip.alloc_workspace(shape), torch.empty_like(keep))
                                    for _ in range(n_streams - 1)]

    if args.calibrate_copy:
        src = torch.empty(256 << 20, dtype=torch.uint8, device=dev).random_(0, 255)
        dst = torch.empty_like(src)
        for _ in range(5):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    if args.rope:
        cos_h, sin_h = synth.rope_tables(cfg.k, cfg.d)
        rope_cos, rope_sin = torch.from_numpy(cos_h).to(dev), torch.from_numpy(sin_h).to(dev)
        k_rot = torch.empty_like(dev0["K"])

    lses = None

    def row_lse(i):
        """fp32 [B, L, Hq, P]: natural-log-sum-exp of the CaP rows of pot i under its query set (torch, fp32)."""
        K = pots[i % len(pots)][0].float()                                   # [B, L, Hkv, N, d]
        Q = qsets[i % len(qsets)].float().reshape(cfg.B, cfg.L, cfg.Hkv, cfg.G * cfg.P, cfg.d)
        logits = torch.matmul(Q, K.transpose(-1, -2)) * (1.0 / float(np.sqrt(cfg.d)))
        return torch.logsumexp(logits, dim=-1).reshape(cfg.B, cfg.L, cfg.Hq, cfg.P).contiguous()

    def prepare_lse():
        nonlocal lses
        if args.lse:
            lses = [row_lse(i) for i in range(len(pots))]
            torch.cuda.synchronize()

    prepare_lse()
    k_cap_h = synth.cap_keys(cfg) if args.kcat else None
    k_cap = upload(k_cap_h) if args.kcat else None

    def step(i, lane=0, keep_out=None):
        K, V = pots[i % len(pots)]
        stream, ws, keep = lanes[lane]
        if keep_out is not None:
            keep = keep_out
        if args.rope:
            p = i % len(pots)
            rc = ip.ccd_compress_rope(shape, qsets[p % len(qsets) if args.lse else i % len(qsets)], K, V, novs[i % len(novs)],
                                      keep, rope_cos, rope_sin, k_rot, ws, K_cap=k_cap, lse=lses[p] if args.lse else None,
                                      stream=stream)
        elif args.lse:
            p = i % len(pots)                     # the normalisers belong to (pot p, query set p mod 4)
            rc = ip.ccd_compress_lse(shape, qsets[p % len(qsets)], K, V, lses[p], novs[i % len(novs)], keep, ws, stream=stream)
        elif args.kcat:
            rc = ip.ccd_compress_kcat(shape, qsets[i % len(qsets)], K, V, k_cap, novs[i % len(novs)], keep, ws, stream=stream)
        else:
            rc = ip.ccd_compress(shape, qsets[i % len(qsets)], K, V, novs[i % len(novs)], keep, ws, stream=stream)
        assert rc == ip.CCD_OK, rc

    torch.cuda.synchronize()                             # the inputs were drawn on the default stream

    def warm_up():
        """Clock warm-up (untimed, on the pots behind the timed ones, which it compresses over and over): an idle GPU
        needs some hundred milliseconds of load to reach its working clocks, and a run of 25 calls is over after 7 ms.
        Then the W warm-up steps proper, on full pots again.  Returns (calls, seconds) of the clock warm-up."""
        calls, t_start = 0, time.perf_counter()
        while (args.warmup > 0 and len(pots) >= args.steps + args.warmup
               and (time.perf_counter() - t_start) * 1e3 < args.clock_warmup_ms):
            for i in range(args.warmup):
                step(args.steps + i, i % n_streams)
            calls += args.warmup
            torch.cuda.synchronize()
        seconds = time.perf_counter() - t_start
        if calls:
            for K, V in pots[args.steps:args.steps + args.warmup]:
                fresh(K)
                fresh(V)
            if args.per_head_novelty:
                for nv in novs[args.steps:args.steps + args.warmup]:
                    nv.uniform_(generator=g)
            prepare_lse()
            torch.cuda.synchronize()
        for i in range(args.warmup):
            step(args.steps + i, i % n_streams)          # the warm-up calls use the pots behind the timed ones
        torch.cuda.synchronize()
        return calls, seconds

    cw_calls, cw_seconds = warm_up()
    t0 = time.perf_counter()
    for i in range(args.steps):
        step(i, i % n_streams)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_per_step = (t1 - t0) * 1e3 / args.steps

    # The same K steps again, back to back as in the timed region, every kernel launched with a pair of events that take
    # its own begin and end time stamps: per-kernel average durations.  (Kept out of the timed region: the completion
    # signal that every kernel then carries costs 3 - 4 us per kernel between launches.)  Each call writes its keep_idx
    # to a buffer of its own, from which the fraction of kept rows that really moved is taken afterwards.
    refill()
    prepare_lse()
    keeps = [torch.empty_like(keep) for _ in range(args.steps)]
    warm_up()                                            # as before the timed region
    ip.ccd_profile_enable(True)
    for i in range(args.steps):
        step(i, keep_out=keeps[i])
    torch.cuda.synchronize()
    stage_ms, calls = ip.ccd_profile_collect()
    ip.ccd_profile_enable(False)
    stage_avg_us = {k: 1e3 * v / max(calls, 1) for k, v in stage_ms.items()}

    # how much of the cache a call actually moves (rows with keep_idx[j] != j), mean over the profiled calls
    ar = torch.arange(cfg.k, device=dev)
    moved = float(sum((kp.to(torch.int64) != ar).float().mean().item() for kp in keeps)) / max(args.steps, 1)
    del keeps

    ab = algorithmic_bytes(cfg)
    keep_bytes = cfg.units * cfg.k * 4
    row_bytes = ab["compact"] - keep_bytes                                        # K and V rows read and written
    ab["call"] -= int((1.0 - moved) * 0.75 * row_bytes)                          # only moved rows travel
    ab["compact"] -= int((1.0 - moved) * row_bytes)
    ab["select_compact"] -= int((1.0 - moved) * row_bytes)
    if args.kcat:
        ab["call"] += cfg.units * cfg.P * cfg.d * (4 if cfg.dtype == "fp32" else 2)
    if args.rope:                                # every kept K row is read (moved or not) and K_rot is written
        extra = int((1.0 - moved) * row_bytes / 4) + row_bytes // 4
        ab["select_compact"] += extra
        ab["call"] += extra
    def roofline_of(stage):
        t = stage_avg_us[stage] * 1e-6
        if stage in ("score_stats", "score_prob", "score_unit"):
            flops = algorithmic_flops(cfg) * (2 if stage == "score_unit" and not args.lse else 1)   # both passes in one kernel
            if stage == "score_unit" and cfg.dtype == "fp32":
                # an fp32 product runs as three bf16 products on the matrix cores: executed flops against the bf16 peak
                r = {"kernel": stage, "bound": "mfma", "achieved": 3 * flops / t / 1e12, "peak": MFMA_BF16_PEAK_TFLOPS,
                     "unit": "TFLOP/s", "note": "fp32 values as hi + lo bf16: three bf16 products per fp32 product, counted as executed"}
            elif args.score_path == 1 or cfg.dtype == "fp32":
                r = {"kernel": stage, "bound": "alu", "achieved": flops / t / 1e12, "peak": VALU_FP32_PEAK_TFLOPS, "unit": "TFLOP/s"}
            else:
                r = {"kernel": stage, "bound": "mfma", "achieved": flops / t / 1e12, "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s"}
        else:
            r = {"kernel": stage, "bound": "hbm", "achieved": ab[stage] / t / 1e9, "peak": HBM_PEAK_GBPS, "unit": "GB/s"}
        r["frac"] = r["achieved"] / r["peak"]
        plain = cfg.name == "c3" and args.score_path == 0 and not (args.rope or args.kcat or args.window or args.lse)
        r["traffic"] = MEASURED_TRAFFIC_C3.get(stage) if plain else None
        r["traffic_source"] = TRAFFIC_SOURCE if r["traffic"] else None
        r["avg_us"] = stage_avg_us[stage]
        return r

    dom = max(stage_avg_us, key=stage_avg_us.get)
    roof = roofline_of(dom)
    by_kernel = [roofline_of(st) for st in stage_avg_us if stage_avg_us[st] > 0 and st != dom]

    call_gbps = ab["call"] / (ms_per_step * 1e-3) / 1e9
    out = {
        "metric": ("ccd_compress_rope calls/s (fused score+select+compact+CR-RoPE, 32L x 8KV x 128d pot 4096->2048)"
                   if args.rope else
                   "ccd_compress_kcat calls/s (causal Eq. 2: CaP keys in the softmax; 32L x 8KV x 128d pot 4096->2048)"
                   if args.kcat else
                   "ccd_compress_lse calls/s (row normalisers handed in: one pass over K; 32L x 8KV x 128d pot 4096->2048)"
                   if args.lse else
                   "ccd_compress calls/s (fused score+select+compact, 32L x 8KV x 128d pot 4096->2048)"),
        "value": 1e3 / ms_per_step, "unit": "calls/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": cfg.dtype, "data": "synthetic",
        "config": {"workload": f"{cfg.name}: B{cfg.B} L{cfg.L} Hq{cfg.Hq} Hkv{cfg.Hkv} d{cfg.d} N{cfg.N}->k{cfg.k} "
                               f"P{cfg.P} T{cfg.T} pool{cfg.w}", "ring": [len(pots), len(qsets), len(novs)], "score_path": args.score_path,
                   "cap_keys_in_softmax": bool(args.kcat), "window": args.window,
                   "per_head_novelty": bool(args.per_head_novelty), "lse_given": bool(args.lse), "streams": n_streams},
        # the figure the target is stated on: the whole call's algorithmic bytes against the HBM peak
        "roofline_call": {"kernel": "whole call", "bound": "hbm", "achieved": call_gbps, "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                          "frac": call_gbps / HBM_PEAK_GBPS, "algorithmic_bytes": ab["call"], "target_frac": 0.70},
        "call_hbm": {"algorithmic_bytes": ab["call"], "achieved_GBps": call_gbps, "frac_of_peak": call_gbps / HBM_PEAK_GBPS},
        "stage_avg_us": stage_avg_us, "moved_row_fraction": moved,
        # the kernel with the largest average duration (HIP events around every kernel, second pass over the same steps)
        "roofline": roof, "roofline_other_kernels": by_kernel,
        "clock_warmup": {"seconds": cw_seconds, "calls": cw_calls},
    }
    plain_headline = cfg.name == "c3" and not (args.rope or args.kcat or args.window or args.lse or args.per_head_novelty)
    if plain_headline and not args.no_other_configs:
        del pots, lanes                                   # make room: the streaming leg holds 3 GiB of its own
        torch.cuda.empty_cache()
        out["other_configs"] = other_configs(dev, torch, ip, synth)

    if not args.no_cpu_baseline:
        from oracle import ccd_oracle as O   # CPU baseline leg only
        try:
            from threadpoolctl import threadpool_info
            threads = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
        except Exception:
            threads = os.cpu_count() or 1
        n_units = cfg.units if args.cpu_units <= 0 else min(args.cpu_units, cfg.units)
        sample = [(u // (cfg.L * cfg.Hkv), (u // cfg.Hkv) % cfg.L, u % cfg.Hkv)
                  for u in np.linspace(0, cfg.units - 1, n_units).astype(int)]
        c0 = time.perf_counter()
        rope_kw = dict(rope_cos=cos_h, rope_sin=sin_h) if args.rope else {}
        if args.kcat:
            rope_kw["K_cap"] = k_cap_h
        if args.window:
            rope_kw["window"] = args.window
        if args.lse:
            rope_kw["lse"] = row_lse(0).cpu().numpy()
        O.compress(host0["Q_cat"], host0["K"], host0["V"], host0["novelty"], k=cfg.k, T=cfg.T, pool_w=cfg.w,
                   pool_mode=O.POOL_MAX, units=sample, **rope_kw)
        c1 = time.perf_counter()
        per_call = (c1 - c0) * cfg.units / n_units
        out["cpu_baseline"] = {"value": 1.0 / per_call, "unit": "calls/s", "cores": threads, "kind": "oracle",
                               "sample": f"{n_units} of {cfg.units} units of pot 0 in {c1 - c0:.2f} s, scaled to a whole call"}
    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
