#!/usr/bin/env python3
"""Benchmark of the PolyKV pool hot path on one MI355X.

One step = one pass of the whole path over the Llama-3-8B-shaped pool (32 layers x 8 KV heads x
head_dim 128, 4096 tokens, 15 agents x 32 query heads): pool_encode -> pool_decode -> pool_attend.
Inputs are synthetic and already resident in HBM when timing starts.  Prints ONE JSON line:
`value` is the decode-attention rate in pool GB/s (packed pool + Q + out bytes over the duration of
the pool attention kernel, taken from HIP events that the runtime stamps at the kernel's begin and
end); encode tokens/s and the other kernels' rates ride along as extra keys;
`roofline` describes the attention kernel against HBM peak and `cpu_baseline` times the CPU oracle
on the same workload, layer by layer.  After the timed region (unless --no-extras) the same process adds context:
a plain device copy (what this GPU sustains for read + write traffic), pool_attend launched back to back over the
rotated pools (the steady-state read loop of a write-once / read-many pool), and `other_configs`: attention on the
SmolLM2-shaped pool, the 7,194-token pool with 64-token private tails and the 1,024-row stress shape.
All durations are medians over the timed calls.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

HBM_PEAK_GBPS = 8000.0


def cpu_baseline(cfg, W, layers=None):
    """The oracle, as it stands, on the same workload, one layer at a time (all KV heads, all tokens, all
    agents): about 10-30 s of CPU work for the whole Llama-shaped pool."""
    from oracle import polykv_oracle as O
    try:
        from threadpoolctl import threadpool_info
        threads = max([i.get("num_threads", 1) for i in threadpool_info()] or [1])
    except Exception:
        threads = 1
    layers = cfg.layers if layers is None else min(layers, cfg.layers)
    Q = W.queries(cfg)
    t_enc = t_dec = t_att = 0.0
    for l in range(layers):
        Kl, Vl = W.kv_layer(cfg, l)
        t0 = time.perf_counter()
        ref = O.pool_encode(Kl[None], Vl[None])
        t1 = time.perf_counter()
        Kh, Vh = O.pool_decode(ref)
        t2 = time.perf_counter()
        O.pool_attend(Kh, Vh, Q[l:l + 1])
        t3 = time.perf_counter()
        t_enc, t_dec, t_att = t_enc + (t1 - t0), t_dec + (t2 - t1), t_att + (t3 - t2)
    b = O.stored_bytes(layers, cfg.kv_heads, cfg.tokens, cfg.head_dim)
    q_part = Q[:layers]
    attend_bytes = b["packed"] + q_part.size * 2 + q_part.size * 4
    return {
        "value": attend_bytes / t_att / 1e9, "unit": "GB/s", "cores": threads, "kind": "oracle",
        "sample": "%d of %d layers of the same workload (all %d KV heads x %d tokens, %d agents), layer by layer; "
                  "encode %.2f s, decode %.2f s, attend %.2f s" % (layers, cfg.layers, cfg.kv_heads, cfg.tokens,
                                                                   cfg.agents, t_enc, t_dec, t_att),
        # one token = one position across ALL layers and heads of the full pool
        "encode_tokens_per_s": cfg.tokens / (t_enc * cfg.layers / layers),
    }


def attend_back_to_back(pk, pools, Q, out, ws, tails, kprec, n=None):
    """pool_attend in a row over the rotated pools, in steady state: the launches run for about 60 ms before the
    timed ones start (the shader clock takes tens of milliseconds to settle after a burst begins) and n launches
    (default: about 100 ms worth, at least 20) are timed.  Returns (median stream-level time per call, median
    duration of the call's main kernel), seconds."""
    import torch

    def launch(i):
        pools[i % len(pools)].attend(Q, out, workspace=ws, tails=tails, key_precision=kprec)
    a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    for i in range(3):
        launch(i)
    a.record()
    for i in range(5):
        launch(i)
    b.record()
    torch.cuda.synchronize()
    est = max(a.elapsed_time(b) * 1e-3 / 5, 1e-6)             # seconds per call, roughly
    warm = int(min(max(0.06 / est, 3), 5000))
    n = int(min(max(0.1 / est, 20), 3000)) if n is None else n
    evs = [[torch.cuda.Event(enable_timing=True) for _ in range(4)] for _ in range(n)]
    for e in evs:
        for x in e:
            x.record()
    torch.cuda.synchronize()
    for i in range(warm):
        launch(i)
    for i, e in enumerate(evs):
        e[0].record()
        pk.time_next_kernel(e[2], e[3])
        launch(warm + i)
        e[1].record()
    torch.cuda.synchronize()
    call = float(np.median([e[0].elapsed_time(e[1]) for e in evs])) * 1e-3
    kern = float(np.median([e[2].elapsed_time(e[3]) for e in evs])) * 1e-3
    return call, kern


def other_config(pk, W, n, kprec):
    """Attention on another of the paper-shaped configurations, back to back over two or three rotated pools.
    The tensors are drawn on the GPU (seeded torch generator) with the recipe of workloads.py: throughput does
    not depend on the values."""
    import torch
    cfg = W.CONFIGS[n]
    L, H, d, T = cfg.layers, cfg.kv_heads, cfg.head_dim, cfg.tokens
    g = torch.Generator(device="cuda")
    g.manual_seed(1000 * n)

    def draw(shape, scale=None):
        x = torch.randn(shape, device="cuda", generator=g, dtype=torch.float32)
        return (x * scale if scale is not None else x).to(torch.float16)
    gain = torch.exp(0.5 * torch.randn((L, H, 1, d), device="cuda", generator=g))
    gain = torch.where(torch.rand((L, H, 1, d), device="cuda", generator=g) < 0.01, gain * 8.0, gain)
    K = draw((L, H, T, d), gain)
    V = draw((L, H, T, d), torch.exp(0.3 * torch.randn((L, H, T, 1), device="cuda", generator=g)))
    Q = draw((L, cfg.agents, cfg.q_per_agent, cfg.q_heads, d))
    out = torch.empty(Q.shape, dtype=torch.float32, device="cuda")
    units = L * H
    packed = units * T * (d + d // 16 + 3 * d // 8)
    copies = 3 if 2 * packed < (256 << 20) else 2          # more than the 256 MB last-level cache in rotation
    pools = [pk.Pool(L, H, d, T).bind() for _ in range(copies)]
    for p in pools:
        p.encode(K, V)
    tails, tail_len = None, 0
    if cfg.max_tail:                                        # every agent carries max_tail private tokens
        tail_len = cfg.max_tail
        tails = pk.Tails(pools[0], [(draw((L, H, tail_len, d)), draw((L, H, tail_len, d))) for _ in range(cfg.agents)],
                         [tail_len] * cfg.agents)
    del K, V
    ws = torch.empty(max(pools[0].attend_workspace_bytes(Q, tails=tails), 256), dtype=torch.uint8, device="cuda")
    call, kern = attend_back_to_back(pk, pools, Q, out, ws, tails, kprec)
    tail_bytes = cfg.agents * tail_len * units * 4 * d
    nbytes = packed + Q.numel() * 2 + out.numel() * 4 + tail_bytes
    R = cfg.rows_per_kv_head
    nt = 1 if R <= 32 else 2
    t = call if tails is not None else kern                 # with tails a call is three kernels: stream-level time
    res = {"workload": cfg.name, "rows_per_kv_head": R, "tokens": T, "pool_bytes": packed, "tail_len": tail_len,
           "tail_bytes": tail_bytes, "algorithmic_bytes": nbytes, "pool_copies_rotated": copies,
           "kernel": "attend_mfma_kernel<%d,%d,0,0>" % (d, nt), "kernel_ms": kern * 1e3, "call_ms": call * 1e3,
           "timed": "pool_attend back to back; " + ("call (tail kernel + pool kernel + merge kernel, stream events)"
                                                    if tails is not None else "the pool kernel's own events"),
           "GB_per_s": nbytes / t / 1e9, "frac_of_hbm_peak": nbytes / t / 1e9 / HBM_PEAK_GBPS}
    if R >= 256:                                            # matrix-bound shape: useful attention arithmetic
        flops = 4.0 * R * d * T * units
        res["useful_TFLOP_per_s"] = flops / kern / 1e12
        res["frac_of_f16_matrix_peak"] = flops / kern / 1e12 / 2500.0
    for p in pools:
        p.close()
    return res


# name -> (codec id of the C ABI, bits per value code, per-vector scale stored)
VALUE_CODECS = {"tq3": (0, 3, False), "tq3-scaled": (1, 3, True), "int8": (2, 8, True), "tq2": (3, 2, False),
                "tq2-scaled": (4, 2, True), "tq4": (5, 4, False), "tq4-scaled": (6, 4, True)}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    # The defaults measure the steady state: after a burst of work begins the shader clock needs tens of
    # milliseconds to settle (steps 8 to 30 run up to 40 % slower), so the run settles for 80 ms (below), 100 steps
    # warm up and 500 are timed.
    ap.add_argument("--steps", type=int, default=500)
    ap.add_argument("--warmup", type=int, default=100)
    ap.add_argument("--config", type=int, default=3, help="workload configuration (default: Llama-3-8B shape)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--pools", type=int, default=3, help="distinct pool copies rotated between steps")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run a plain device copy of known size (for scaling rocprofv3 FETCH_SIZE / WRITE_SIZE)")
    ap.add_argument("--tail-len", type=int, default=0,
                    help="private uncompressed tokens per agent attended together with the pool (the decode step "
                         "number of the tails configuration); their bytes count as attention traffic")
    ap.add_argument("--per-layer", action="store_true",
                    help="attention as the decode loop issues it: one pool_attend per layer (32 calls per step) instead "
                         "of all layers in one call; the attention time is then the stream-level time of the 32 calls")
    ap.add_argument("--no-extras", action="store_true",
                    help="skip what runs after the timed region (device copy, back-to-back attention, other "
                         "configurations): for profiles that should hold the timed steps only")
    ap.add_argument("--extras", action="store_true", help="(default; kept for older command lines)")
    ap.add_argument("--value-codec", choices=tuple(VALUE_CODECS), default="tq3",
                    help="value codec: tq3 = the paper's (headline configuration); tqB-scaled = with a per-vector fp16 "
                    "scale; tq2 / tq4 = 2 / 4 bits per coordinate; int8 = uniform int8 without rotation (the paper's "
                    "proposed ablation)")
    ap.add_argument("--key-codec", choices=("block32", "tensor"), default="block32",
                    help="key codec: block32 = q8_0 blocks of 32 (headline configuration); tensor = one scale per layer "
                    "tensor, the key formula as the paper prints it (two passes over K at encode)")
    ap.add_argument("--bf16", action="store_true",
                    help="dense tensors (K, V, Q, decode output, tails) in bfloat16 instead of fp16: the dtype of the "
                    "paper's Llama-3-8B cache; the headline configuration is stated in fp16")
    ap.add_argument("--key-precision", choices=("exact", "fp16"), default="exact",
                    help="exact = scores over code * scale exactly (headline); fp16 = over the dequantized keys rounded "
                    "to fp16, the precision of the dense cache the paper's read path attends over")
    ap.add_argument("--no-settle", action="store_true",
                    help="skip the 80 ms of untimed steps before the warm-up (for counter runs that want few launches)")
    ap.add_argument("--phases", default="eda", help="the phases of a step, in the order given: e(ncode) d(ecode) "
                    "a(ttend); a subset is for profiling one kernel and is marked partial")
    args = ap.parse_args()
    if not args.phases or len(set(args.phases)) != len(args.phases) or not set(args.phases) <= set("eda"):
        ap.error("--phases takes each of e, d, a at most once")
    args.extras = not args.no_extras and len(args.phases) == 3 and not args.per_layer
    if args.gpus != 1:
        print("bench.py: this build runs on exactly one GPU (--gpus 1); the pool path shards by layer / KV head "
              "with no exchange between GPUs", file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2604_24971_amd import polykv as pk          # fails loudly if the library is not built
    from paper_2604_24971_amd import workloads as W

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)
    torch.cuda.set_device(0)
    cfg = W.CONFIGS[args.config]
    L, H, d, T = cfg.layers, cfg.kv_heads, cfg.head_dim, cfg.tokens

    Kn, Vn = W.kv_pool(cfg)
    K = torch.from_numpy(Kn).cuda()
    V = torch.from_numpy(Vn).cuda()
    del Kn, Vn
    Q = torch.from_numpy(W.queries(cfg)).cuda()
    io_dtype = torch.bfloat16 if args.bf16 else torch.float16
    K, V, Q = K.to(io_dtype), V.to(io_dtype), Q.to(io_dtype)
    out = torch.empty(Q.shape, dtype=torch.float32, device="cuda")
    Kd = torch.empty_like(K)
    Vd = torch.empty_like(V)
    codec = VALUE_CODECS[args.value_codec][0]
    kcodec = pk.KEYS_Q8_TENSOR if args.key_codec == "tensor" else pk.KEYS_Q8_BLOCK32
    kprec = pk.KEY_PRECISION_FP16 if args.key_precision == "fp16" else pk.KEY_PRECISION_EXACT
    pools = [pk.Pool(L, H, d, T, value_codec=codec, key_codec=kcodec).bind() for _ in range(max(1, args.pools))]
    tails = None
    if args.tail_len > 0:        # every agent has produced tail_len private tokens (fp16, uncompressed)
        cap = max(args.tail_len, cfg.max_tail)
        tails = pk.Tails(pools[0], [(torch.from_numpy(kt).cuda().to(io_dtype), torch.from_numpy(vt).cuda().to(io_dtype))
                                    for kt, vt in W.tails(cfg, [cap] * cfg.agents)], [args.tail_len] * cfg.agents)
    ws = torch.empty(max(pools[0].attend_workspace_bytes(Q, tails=tails), 256), dtype=torch.uint8, device="cuda")
    if args.per_layer:
        Ql = [Q[l:l + 1].contiguous() for l in range(L)]
        outl = [out[l:l + 1] for l in range(L)]
        ws = torch.empty(max(pools[0].attend_workspace_bytes(Ql[0], tails=tails, layer_begin=0, layer_end=1), 256),
                         dtype=torch.uint8, device="cuda")

    if args.phases[0] != "e":
        for p in pools:
            p.encode(K, V)

    def step(i, ev=None, kev=None):
        # The phases run in the order --phases names them.  ev: per phase a (before, after) pair of events
        # recorded on the stream around the call (stream-level phase times, launch gaps included); kev: three
        # (start, stop) pairs stamped by the runtime at the begin / end of each call's main kernel (kernel
        # durations, what rocprofv3 --kernel-trace reports).  Index 0 = encode, 1 = decode, 2 = attend.
        p = pools[i % len(pools)]
        for ph in args.phases:
            idx = "eda".index(ph)
            if ev:
                ev[2 * idx].record()
            if ph == "e":
                if kev:
                    pk.time_next_kernel(*kev[0])
                p.encode(K, V)
            elif ph == "d":
                if kev:
                    pk.time_next_kernel(*kev[1])
                p.decode(io_dtype, Kd, Vd)
            elif args.per_layer:
                for l in range(L):
                    p.attend(Ql[l], outl[l], layer_begin=l, layer_end=l + 1, workspace=ws, tails=tails, key_precision=kprec)
            else:
                if kev:
                    pk.time_next_kernel(*kev[2])
                p.attend(Q, out, workspace=ws, tails=tails, key_precision=kprec)
            if ev:
                ev[2 * idx + 1].record()

    if args.calibrate_copy:      # elementwise copy kernel: reads and writes K.numel()*2 bytes
        for _ in range(3):
            Kd.copy_(K)
    events = [[torch.cuda.Event(enable_timing=True) for _ in range(6)] for _ in range(args.steps)]
    for e in events:                 # (a phase that is left out keeps its pair: recorded here, zero apart)
        for x in e:
            x.record()
    kevents = [[(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(3)]
               for _ in range(args.steps)]
    for trio in kevents:             # torch creates an event's handle at its first record()
        for a, b in trio:
            a.record()
            b.record()
    # Settling: whatever --warmup says, the GPU has run steps for at least 80 ms before the timed ones begin.
    # After an idle period the first few steps run at the boost clock, the next twenty to thirty up to 40 % slower
    # (step 12 is the worst), and only after some 30 ms of continuous work are the durations steady; a bare
    # synchronize between steps does not start that over.  Untimed, like the warm-up steps that follow.
    # The untimed steps are launched exactly as the timed ones (same events around and inside the calls, here into a
    # spare set): a change in the launch pattern changes the GPU's duty cycle and starts a transient of its own.
    spare_ev = [torch.cuda.Event(enable_timing=True) for _ in range(6)]
    spare_kev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(3)]
    g0, g1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    g0.record()
    for i in range(3):
        step(i, spare_ev, spare_kev)
    g1.record()
    torch.cuda.synchronize()
    t_est = max(g0.elapsed_time(g1) * 1e-3 / 3, 1e-6)          # seconds of GPU time per step
    for i in range(0 if args.no_settle else max(0, int(0.08 / t_est) - args.warmup)):
        step(i, spare_ev, spare_kev)
    for i in range(args.warmup):
        step(i, spare_ev, spare_kev)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        step(i, events[i], kevents[i])
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0

    # Context for the numbers above, outside the timed region: a plain device copy of the dense K tensor
    # (what this GPU sustains for read + write traffic) and pool_attend launched back to back on its own
    # (the attention kernel is issue-bound, so its duration follows the shader clock, which the power
    # management keeps lower while memory-bound kernels run in between).
    t_copy = t_att_iso = k_att_iso = k_att_zero = append_rate = None
    other = None
    if args.extras:
        def timed(fn, n):
            evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(n)]
            for a, b in evs:
                a.record()
                fn()
                b.record()
            torch.cuda.synchronize()
            return float(np.median([a.elapsed_time(b) for a, b in evs])) * 1e-3
        t_copy = timed(lambda: Kd.copy_(K), 10)
        t_att_iso, k_att_iso = attend_back_to_back(pk, pools, Q, out, ws, tails, kprec)
        # The same launches over all-zero contents (zero K, V and Q: the same kernel, instruction stream and
        # bytes).  The power management lowers the shader clock by how much the operands make the matrix cores
        # and vector ALUs switch; with nothing switching the kernel shows what its instruction stream alone
        # takes at the full clock.
        if tails is None and not args.per_layer:
            zK, zV, zQ = torch.zeros_like(K), torch.zeros_like(V), torch.zeros_like(Q)
            for p in pools:
                p.encode(zK, zV)
            k_att_zero = attend_back_to_back(pk, pools, zQ, out, ws, None, kprec)[1]
            del zK, zV, zQ
            for p in pools:
                p.encode(K, V)
        # incremental fill: the same tensors appended 64 tokens at a time into a pool of the same capacity
        chunk = 64
        Kc = [K[:, :, i:i + chunk].contiguous() for i in range(0, T - chunk + 1, chunk)]
        Vc = [V[:, :, i:i + chunk].contiguous() for i in range(0, T - chunk + 1, chunk)]
        spare = pools[0]

        def fill():
            spare.bind(spare.storage)                      # empties the pool
            for kc, vc in zip(Kc, Vc):
                spare.append(kc, vc)
        if args.key_codec == "block32":                    # (a per-tensor key scale cannot be appended to)
            fill()
            t_fill = timed(fill, 3)
            append_rate = len(Kc) * chunk / t_fill
            spare.encode(K, V)
        del Kc, Vc
        if args.config == 3 and args.value_codec == "tq3" and args.key_codec == "block32" and not args.bf16:
            del pools[1:]
            other = [other_config(pk, W, n, kprec) for n in (2, 4, 5)]

    enc = np.array([e[0].elapsed_time(e[1]) for e in events]) * 1e-3
    dec = np.array([e[2].elapsed_time(e[3]) for e in events]) * 1e-3
    att = np.array([e[4].elapsed_time(e[5]) for e in events]) * 1e-3
    t_enc, t_dec, t_att = (max(float(np.median(x)), 1e-9) for x in (enc, dec, att))    # stream-level, with launch gaps

    def kernel_time(idx, phase, fallback):
        if phase not in args.phases:
            return fallback
        return max(float(np.median([k[idx][0].elapsed_time(k[idx][1]) for k in kevents])) * 1e-3, 1e-9)
    k_enc, k_dec, k_att = kernel_time(0, "e", t_enc), kernel_time(1, "d", t_dec), kernel_time(2, "a", t_att)
    if args.key_codec == "tensor":            # encode is three kernels (zero, max|k|, encode): the stream time covers them
        k_enc = t_enc

    units = L * H
    v_bits, v_scaled = VALUE_CODECS[args.value_codec][1:]
    v_bytes = v_bits * d // 8 + (2 if v_scaled else 0)
    k_bytes = d + (d // 16 if args.key_codec == "block32" else 0)
    packed = units * T * (k_bytes + v_bytes)                         # algorithmic pool bytes
    enc_bytes = units * T * 4 * d + packed
    dec_bytes = packed + units * T * 4 * d
    tail_bytes = cfg.agents * args.tail_len * units * 4 * d                    # fp16 K and V of every agent's tail
    att_bytes = packed + Q.numel() * 2 + out.numel() * 4 + tail_bytes
    if tails is not None or args.per_layer:   # several kernels per step: only the stream-level time covers them
        k_att = t_att
    att_gbps = att_bytes / k_att / 1e9

    def roof(gbps, kernel):
        return {"bound": "hbm", "achieved": gbps, "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                "frac": gbps / HBM_PEAK_GBPS, "traffic": None, "kernel": kernel}

    how = ("; duration = the kernel's own begin/end HIP events (hipExtLaunchKernel start/stop events on the launch "
           "stream), median over the timed steps; traffic = the stored rocprofv3 FETCH_SIZE + WRITE_SIZE figure of "
           "profiles/ (copy-scaled), not measured in this run")
    vc = codec                                                          # the kernels' value-codec template argument
    nt = 1 if (cfg.rows_per_kv_head <= 32 or d == 256 or (vc in (2, 6) and d == 128)) else 2
    kc = 1 if args.key_codec == "tensor" else 0
    attend_roof = roof(att_gbps, "attend_mfma_kernel<%d,%d,%d,%d,%s> (pool_attend)" % (d, nt, vc, kc, "true" if args.key_precision == "fp16" else "false") + how +
                       "; achieved = algorithmic bytes (packed pool + Q + out) / duration")
    traffic_file = os.path.join(os.path.dirname(os.path.abspath(__file__)), "profiles",
                                "attend_hbm_traffic_%s.txt" % cfg.name)
    if os.path.exists(traffic_file) and args.value_codec == "tq3" and args.key_codec == "block32":     # rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE, scaled by a copy kernel
        vals = dict(line.split()[:2] for line in open(traffic_file) if line.strip() and not line.startswith("#"))
        attend_roof["traffic"] = float(vals["hbm_bytes_per_launch"])
    else:
        vals = {}
    result = {
        "metric": "decode_attention_pool_GB_per_s", "value": att_gbps, "unit": "GB/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": wall / args.steps * 1e3, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "f16 operands, f32 accumulate", "data": "synthetic",
        "config": {"workload": cfg.name, "layers": L, "kv_heads": H, "q_heads": cfg.q_heads, "head_dim": d,
                   "tokens": T, "agents": cfg.agents, "q_per_agent": cfg.q_per_agent,
                   "rows_per_kv_head": cfg.rows_per_kv_head, "pool_bytes": packed, "pool_copies_rotated": len(pools),
                   "value_codec": args.value_codec, "key_codec": args.key_codec, "key_precision": args.key_precision, "dense_dtype": "bf16" if args.bf16 else "f16",
                   "tail_len": args.tail_len, "tail_bytes": tail_bytes,
                   "attend_calls_per_step": L if args.per_layer else 1},
        "step": " -> ".join({"e": "pool_encode", "d": "pool_decode(fp16)", "a": "pool_attend"}[ph] for ph in args.phases) + ", all layers",
        "encode_tokens_per_s": T / k_enc, "encode_GB_per_s": enc_bytes / k_enc / 1e9,
        "decode_GB_per_s": dec_bytes / k_dec / 1e9,
        "kernel_ms": {"attend": k_att * 1e3, "encode": k_enc * 1e3, "decode": k_dec * 1e3},
        "stream_ms": {"attend": t_att * 1e3, "encode": t_enc * 1e3, "decode": t_dec * 1e3,
                      "note": "events recorded on the stream around each call: kernel + launch gaps"},
        "attend_ms": k_att * 1e3, "encode_ms": k_enc * 1e3, "decode_ms": k_dec * 1e3,
        "attend_algorithmic_bytes": att_bytes,
        "attend_back_to_back_ms": k_att_iso and k_att_iso * 1e3,
        "attend_back_to_back_GB_per_s": k_att_iso and att_bytes / k_att_iso / 1e9,
        "attend_back_to_back_frac_of_hbm_peak": k_att_iso and att_bytes / k_att_iso / 1e9 / HBM_PEAK_GBPS,
        "attend_back_to_back_call_ms": t_att_iso and t_att_iso * 1e3,
        "attend_back_to_back_note": "pool_attend launched back to back over the rotated pools, outside the timed "
                                    "region: kernel duration from the kernel's own events; call_ms = stream events "
                                    "around each call (kernel + launch gap)",
        "attend_zero_data_back_to_back_ms": k_att_zero and k_att_zero * 1e3,
        "attend_zero_data_frac_of_hbm_peak": k_att_zero and att_bytes / k_att_zero / 1e9 / HBM_PEAK_GBPS,
        "attend_zero_data_note": "the same back-to-back launches with K = V = Q = 0 (same kernel, same bytes): the "
                                 "duration of the instruction stream at the full shader clock; with random data the "
                                 "power management lowers the clock (2.4 -> about 1.4 GHz), which is the gap to the "
                                 "figure above",
        "other_configs": other,
        "device_copy_GB_per_s": t_copy and 2 * K.numel() * 2 / t_copy / 1e9,
        "append_64_tokens_per_s": append_rate,
        "roofline": attend_roof,
        "roofline_encode": roof(enc_bytes / k_enc / 1e9, "encode_kernel<%d,%d,%s,%d> (pool_encode); dense 16-bit K,V in + packed out" % (d, vc, "true" if args.bf16 else "false", kc)),
        "roofline_decode": roof(dec_bytes / k_dec / 1e9, "decode_kernel<%d,%d,%s,%d> (pool_decode); packed in + dense 16-bit out" % (d, vc, "bf16" if args.bf16 else "half", kc)),
    }
    for key, name in (("roofline_encode", "encode_hbm_bytes_per_launch"), ("roofline_decode", "decode_hbm_bytes_per_launch")):
        if name in vals:
            result[key]["traffic"] = float(vals[name])
    if len(args.phases) != 3:
        result["partial"] = "phases=%s: not a full step" % args.phases
    if not args.no_cpu_baseline:
        result["cpu_baseline"] = cpu_baseline(cfg, W)
    else:
        result["cpu_baseline"] = None
    print(json.dumps(result))


if __name__ == "__main__":
    main()
