#!/usr/bin/env python3
"""Benchmark of the PPD decode path on one MI355X.

A step is one PPD round (`ppd_step`): main token to the exit layer when the previous round
missed, early LM head + top-k, d-dbar pipelined steps (main row at layer dbar+j and k candidate
rows at layer j in the same launches), final head, verification, adoption.  One round emits
one token.  Inputs (synthetic weights and prompt) are resident in HBM before the timed region.

Prints one JSON line: PPD tokens/s as `value`, plain greedy on the same kernels next to it;
`roofline`: the dominant kernel of a pipelined step, the two-group FFN-in GEMM (main row on one
layer's gate/up matrices, the k candidate rows on another's), timed live with HIP events, with the
one-row launch of the solo phase / plain steps beside it; `pipelined_step`: the unit the 70 % target
is stated on, against both byte counts (bf16 KV as the hot-path table counts it, fp32 KV as built);
per-kernel bytes / time / fraction for both launch shapes; a two-term time model (bytes / rate +
launches x fixed cost) for plain tokens and for rounds after a miss and after a hit; the measured
match rate and layer-row counts against Theorem 4.1; the CPU oracle timed on the host cores.

`--sweep-exit` instead sweeps the exit layer and the controlled-match-rate variants (Theorem 4.1's
(d - dbar) factor, the layer axis of the paper's match-rate table) and prints one JSON line with the table.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0   # MI355X HBM3E, published
# HBM bytes per launch of the roofline kernel (the two-group FFN-in GEMM) from rocprofv3 FETCH_SIZE / WRITE_SIZE, scaled
# by a copy kernel of known size, keyed by (configuration, k); collected with the counter probe on the C ABI
# (paper_2307_05908_amd/ppd_pmc_probe), see profiles/.  A property of the kernel source it was collected on.
MEASURED_TRAFFIC = {("llama7b", 3): 361.75e6}
# sha1 of csrc/ppd_kernels.h when the counters were collected: a changed kernel source voids the figure (null is printed)
TRAFFIC_KERNELS_SHA1 = "009930545f1fa5ba9fbe0077f60eaffaf9e4f03d"
TRAFFIC_SOURCE = "profiles/llama7b_ppd_k3_traffic.txt"


def measured_traffic(cfg_name, k):
    import hashlib
    try:
        h = hashlib.sha1(open(os.path.join(ROOT, "paper_2307_05908_amd", "csrc", "ppd_kernels.h"), "rb").read()).hexdigest()
    except OSError:
        return None, None
    v = MEASURED_TRAFFIC.get((cfg_name, k))
    if v is None or h != TRAFFIC_KERNELS_SHA1:
        return None, None
    return v, TRAFFIC_SOURCE


def kernel_bytes(cfg, pi, ctx, k):
    """Algorithmic bytes one launch must move, per kernel class and launch shape (g1: one row group; g2: the
    two-group launch of a pipelined step).  Attention: keys and values as cached (fp32)."""
    dm, F, wb = cfg.d_model, cfg.d_ff, cfg.wbytes
    n_in = 2 if cfg.act == pi.ACT_SWIGLU else 1
    one = {"gemm_qkv": 3 * dm * dm * wb, "gemm_o": dm * dm * wb, "gemm_ffn_in": n_in * dm * F * wb,
           "gemm_ffn_out": dm * F * wb, "head": cfg.vocab * dm * wb, "attn": ctx * cfg.kv_bytes_per_pos_layer()}
    out = {}
    for n, b in one.items():
        out[n + ".g1"] = b
        if n != "head":
            out[n + ".g2"] = 2 * b
    return out


def prefill_report(cfg, pi, rows, secs, first_secs):
    """The prompt pass against the MFMA roofline: multiply-adds of the linear layers (2 x rows x weights) and of
    causal attention; bf16 models run every product twice (the rows as two bf16 terms), priced at the dense bf16 peak."""
    lin = 2.0 * rows * (cfg.layer_weight_bytes() / cfg.wbytes) * cfg.n_layers
    att = 4.0 * cfg.d_model * (rows * (rows + 1) / 2) * cfg.n_layers
    out = {"positions": rows, "ms": round(secs * 1e3, 2), "first_call_ms": round(first_secs * 1e3, 2),
           "positions_per_s": round(rows / secs, 1), "useful_TFLOPs": round((lin + att) / secs / 1e12, 1)}
    if cfg.wdtype == pi.WD_BF16 and rows >= 32:
        out["roofline"] = {"bound": "mfma", "achieved": round(2 * lin / secs / 1e12, 1), "peak": 2500.0, "unit": "TFLOP/s",
                           "frac": round(2 * lin / secs / 1e12 / 2500.0, 4),
                           "what": "bf16 MFMA work of the linear layers (two products per weight and row: rows = hi + lo) over the whole "
                                   "prompt pass, attention (the same MFMA, three products per operand pair) and packing included in the time"}
    return out


def fit_two_term(points):
    """Least squares t_us = t_fixed + bytes / rate over (bytes, us) points.  Returns (t_fixed_us, rate GB/s)."""
    import numpy as np
    x = np.array([p[0] for p in points], dtype=np.float64)
    y = np.array([p[1] for p in points], dtype=np.float64)
    A = np.stack([np.ones_like(x), x], axis=1)
    (t0, slope), *_ = np.linalg.lstsq(A, y, rcond=None)
    return float(t0), float(1.0 / slope / 1e3)


def sweep(args):
    import numpy as np
    import torch
    import ppd_inputs as pi
    from paper_2307_05908_amd import binding, tradeoff
    rows = []
    base = pi.CONFIGS[args.config]
    d = base.n_layers
    if args.sweep_k:     # the number of candidates at the middle exit layer
        cases = [(k, args.exit_layer or d // 2) for k in (1, 3, 5)]
        alphas = (1.0, 0.1, 0.02)
    else:                # the exit layer at one k
        cases = [(args.k or base.k, e) for e in (d // 2, 5 * d // 8, 3 * d // 4, 7 * d // 8) if d // 2 <= e <= d - 1]
        alphas = (1.0, 0.1)
    K, W = args.steps, args.warmup
    for alpha in alphas:
        # one model per alpha (the blocks after layer d/2 damped by alpha, as in the controlled-match-rate
        # configuration), every exit layer on that same model
        cfg = base.replace(alpha=alpha, seed_p=2005)
        model = pi.make_model(cfg)
        prompt = pi.make_prompt(cfg, args.prompt or cfg.n_prompt)
        dev = binding.upload_model(model, "cuda:0")
        for k, e in cases:
            P = binding.PPD(cfg, dev, k=k, exit_layer=e)
            P.ppd_prefill(prompt)
            for _ in range(W):
                P.ppd_step(want_info=False)
            torch.cuda.synchronize()
            st0 = P.ppd_get_stats()
            t = time.perf_counter()
            for _ in range(K):
                P.ppd_step(want_info=False)
            wall = time.perf_counter() - t
            st = P.ppd_get_stats()
            ell = st["rounds"] - st0["rounds"]
            p_hat = (st["matches"] - st0["matches"]) / ell
            main = (st["main_layer_rows"] - st0["main_layer_rows"]) / ell
            t = time.perf_counter()
            for _ in range(K // 4):
                P.plain_greedy_step()
            plain = (time.perf_counter() - t) / (K // 4)
            rows.append({"alpha": alpha, "k": k, "exit_layer": e, "p_correct": round(p_hat, 4),
                         "main_layer_rows_per_token": round(main, 3),
                         "theorem_4_1_per_token": round((d * ell - (d - e) * ell * p_hat) / ell, 3),
                         "layer_rows_per_token": round((st["main_layer_rows"] - st0["main_layer_rows"] +
                                                        st["branch_layer_rows"] - st0["branch_layer_rows"]) / ell, 3),
                         "ms_per_round": round(wall / K * 1e3, 4), "plain_ms_per_token": round(plain * 1e3, 4)})
            print("sweep", rows[-1], file=sys.stderr, flush=True)
            P.close()
            del P
        del dev, model
        torch.cuda.empty_cache()
    print(json.dumps({"metric": "%s sweep, PPD decode on %s shape" % ("k" if args.sweep_k else "exit-layer", base.name),
                      "n_gpus": 1, "steps": K, "warmup": W, "data": "synthetic", "sweep": rows}))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=240)
    ap.add_argument("--warmup", type=int, default=16)
    ap.add_argument("--config", default="llama7b")
    ap.add_argument("--k", type=int, default=None)
    ap.add_argument("--exit-layer", type=int, default=None)
    ap.add_argument("--prompt", type=int, default=None)
    ap.add_argument("--sampling", choices=["greedy", "topk", "topp"], default="greedy",
                    help="final prediction: arg max (the headline), top-k sampling (3 kept) or top-p sampling (0.95), Appendix B")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--profile-rounds", type=int, default=32)
    ap.add_argument("--sweep-exit", action="store_true",
                    help="sweep the exit layer (d/2 .. 7d/8) on the alpha = 1 and alpha = 0.1 models instead of the benchmark")
    ap.add_argument("--sweep-k", action="store_true",
                    help="instead of the benchmark line: k = 1, 3, 5 at the exit layer, on alpha = 1, 0.1 and 0.02 models")
    ap.add_argument("--copy-probe", action="store_true",
                    help="also run one 1 GiB device-to-device copy (a kernel of known traffic, to scale rocprofv3 byte counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (the pipelined decode step of one sequence "
              "lives on one device); --gpus must be 1", file=sys.stderr)
        sys.exit(2)
    if args.sweep_exit or args.sweep_k:
        sweep(args)
        return

    import numpy as np
    import torch
    import ppd_inputs as pi
    from paper_2307_05908_amd import binding, tradeoff

    cfg = pi.CONFIGS[args.config]
    k = args.k or cfg.k
    e = args.exit_layer or cfg.exit_layer
    n_prompt = args.prompt or cfg.n_prompt
    K, W = args.steps, args.warmup
    assert n_prompt + W + K + 1 <= cfg.max_ctx, "prompt + steps exceed the context window"

    t0 = time.time()
    model = pi.make_model(cfg)
    prompt = pi.make_prompt(cfg, n_prompt)
    t_gen = time.time() - t0
    dev = binding.upload_model(model, "cuda:0")
    torch.cuda.synchronize()

    def timed(P, step_fn, warm, steps):
        P.ppd_prefill(prompt)
        for _ in range(warm):
            step_fn()
        torch.cuda.synchronize()
        t = time.perf_counter()
        for _ in range(steps):
            step_fn()
        torch.cuda.synchronize()
        return time.perf_counter() - t

    if args.copy_probe:
        src = torch.empty(1 << 28, dtype=torch.float32, device="cuda:0").normal_()
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    # ---- what a plain streaming read reaches on this GPU (1 GiB, the library's probe kernel)
    probe_buf = torch.empty(1 << 30, dtype=torch.uint8, device="cuda:0")
    probe_buf.zero_()
    torch.cuda.synchronize()
    stream_gbs = binding.ppd_stream_read_probe(probe_buf, iters=8)
    del probe_buf

    # ---- PPD rounds (each call returns when the round's record is on the host: the host clock around a call is the round's latency)
    P = binding.PPD(cfg, dev, k=k, exit_layer=e)
    if args.sampling != "greedy":
        P.ppd_set_sampling(1 if args.sampling == "topk" else 2, 3, 0.95, 1234)
    round_ms, round_hit = [], []

    def ppd_round():
        t = time.perf_counter()
        _, info = P.ppd_step(want_info=True)
        round_ms.append((time.perf_counter() - t) * 1e3)
        round_hit.append(bool(info.matched))

    t = time.perf_counter()
    P.ppd_prefill(prompt)                  # (synchronous) the prompt, all but its last token, fills the KV cache
    prefill_first_s = time.perf_counter() - t      # (includes making the prompt pass's buffers)
    t = time.perf_counter()
    P.ppd_prefill(prompt)
    prefill_s = time.perf_counter() - t
    wall_ppd = timed(P, ppd_round, W, K)
    round_ms, round_hit = np.array(round_ms[W:]), np.array(round_hit[W:])
    # a round's length is set by how it starts: after a hit it resumes mid-stack (no solo phase when dbar = d/2)
    after_hit = np.concatenate([[False], round_hit[:-1]])
    st = P.ppd_get_stats()
    ell = st["rounds"]
    p_hat = st["matches"] / ell
    # ---- plain greedy on the same kernels, same context
    wall_plain = timed(P, P.plain_greedy_step, W, K)

    # ---- timing with HIP events on the library's own stream, separate short passes
    # (a) every kernel bracketed, plain greedy steps and PPD rounds: per-kernel durations of both launch shapes
    # (b) only the phases bracketed, PPD rounds: the parallel phase as it runs in normal operation
    # (c) the roofline kernel alone: bursts of FFN-in GEMMs (other layers' weights in every launch) between two events
    kt, ph = {}, {}
    burst1_ms = burst2_ms = None
    R = args.profile_rounds
    if R > 0:
        P.ppd_prefill(prompt)
        for _ in range(W):
            P.plain_greedy_step()
        P.ppd_set_profiling(2)
        for _ in range(R):
            P.plain_greedy_step()
        kt = P.ppd_get_kernel_time()
        P.ppd_set_profiling(0)
        P.ppd_prefill(prompt)
        for _ in range(W):
            P.ppd_step(want_info=False)
        P.ppd_set_profiling(2)
        for _ in range(R):
            P.ppd_step(want_info=False)
        kt2 = P.ppd_get_kernel_time()
        for n, v in kt2.items():
            if n.endswith(".g2"):
                kt[n] = v
        P.ppd_set_profiling(0)
        P.ppd_prefill(prompt)
        for _ in range(W):
            P.ppd_step(want_info=False)
        P.ppd_set_profiling(1)
        for _ in range(R):
            P.ppd_step(want_info=False)
        ph = P.ppd_get_kernel_time()
        P.ppd_set_profiling(0)
        P.ppd_prefill(prompt)
        burst1_ms = P.ppd_time_ffn_in(4 * cfg.n_layers, groups=1)
        P.ppd_prefill(prompt)
        burst2_ms = P.ppd_time_ffn_in(2 * cfg.n_layers, groups=2)
    ctx_mid = n_prompt + W + R // 2
    wl = cfg.layer_weight_bytes()
    n_in = 2 if cfg.act == pi.ACT_SWIGLU else 1
    ffn_in_bytes = n_in * cfg.d_model * cfg.d_ff * cfg.wbytes
    kb = kernel_bytes(cfg, pi, ctx_mid, k)
    kernels = {}
    for n, v in kt.items():
        us = v["ms"] / v["launches"] * 1e3
        ent = {"avg_us": round(us, 2), "launches": v["launches"]}
        if n in kb:
            ent["bytes"] = kb[n]
            ent["hbm_frac"] = round(kb[n] / (us * 1e-6) / 1e9 / HBM_PEAK_GBS, 4)
        kernels[n] = ent

    roof = None
    if burst1_ms and burst2_ms:
        if cfg.wdtype != pi.WD_BF16:
            kname = "gemm_kernel<float, 1, %d, %s, WR> (norm + first FFN matrix + activation)" % (k, "true" if n_in == 2 else "false")
        else:
            kname = "gemm_mfma_kernel<%s, false> (norm + FFN-in matrices + activation)" % ("true" if n_in == 2 else "false")
        ach2 = 2 * ffn_in_bytes / (burst2_ms * 1e-3) / 1e9
        ach1 = ffn_in_bytes / (burst1_ms * 1e-3) / 1e9
        roof = {"bound": "hbm",
                "kernel": kname + ", the two-group launch of a pipelined step: main row on one layer's matrices, the %d candidate rows on another's" % k,
                "achieved": round(ach2, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": round(ach2 / HBM_PEAK_GBS, 4),
                "traffic": measured_traffic(cfg.name, k)[0], "traffic_source": measured_traffic(cfg.name, k)[1],
                "bytes_per_launch": 2 * ffn_in_bytes, "avg_launch_us": round(burst2_ms * 1e3, 2),
                "timing": "HIP events around a burst of %d back-to-back launches on the library's stream, other layers' weights in every launch" % (2 * cfg.n_layers),
                "stream_read_GBps": round(stream_gbs, 1), "frac_of_stream_read": round(ach2 / stream_gbs, 4),
                "one_row_launch": {"what": "the same kernel with the main row alone (solo phase, plain steps)",
                                   "bytes_per_launch": ffn_in_bytes, "avg_launch_us": round(burst1_ms * 1e3, 2),
                                   "achieved": round(ach1, 1), "frac": round(ach1 / HBM_PEAK_GBS, 4)}}
    pp = ph.get("phase.g2")
    pipe = None
    if pp:
        nb = cfg.n_layers - e
        kv_built = ctx_mid * cfg.kv_bytes_per_pos_layer()           # fp32 keys and values, as cached
        kv_table = kv_built // 2                                     # bf16, as the hot-path scope table counts them
        step_s = pp["ms"] / pp["launches"] / nb / 1e3
        b_built, b_table = 2 * wl + 2 * kv_built, 2 * wl + 2 * kv_table
        pipe = {"us_per_step": round(step_s * 1e6, 2),
                "bytes_per_step": b_table, "GBps": round(b_table / step_s / 1e9, 1),
                "hbm_frac": round(b_table / step_s / 1e9 / HBM_PEAK_GBS, 4),
                "bytes_basis": "two layers' weights + two layers' keys and values at 2 bytes each (the hot-path table's count)",
                "bytes_per_step_fp32_kv": b_built, "hbm_frac_fp32_kv": round(b_built / step_s / 1e9 / HBM_PEAK_GBS, 4),
                "frac_of_stream_read": round(b_table / step_s / 1e9 / stream_gbs, 4), "context": ctx_mid,
                "target_hbm_frac": 0.70}

    # ---- two-term time model: t = bytes / rate + launches * t_fixed, fitted on the bracketed GEMM launches of both shapes
    model_fit = None
    gemms = [n for n in kernels if n.startswith("gemm_") or n.startswith("head")]
    if len(gemms) >= 4:
        t_fixed, rate = fit_two_term([(kernels[n]["bytes"], kernels[n]["avg_us"]) for n in gemms if "bytes" in kernels[n]])
        d, nb = cfg.n_layers, cfg.n_layers - e
        head_b = cfg.head_weight_bytes()

        def us(n):
            return kernels[n]["avg_us"] if n in kernels else 0.0

        lat1 = us("attn.g1") + us("attn_merge.g1")               # latency-bound kernels of a layer, one group
        lat2 = us("attn.g2") + us("attn_merge.g2")
        small = us("select.g1")

        def est(layers1, layers2, heads, embeds):
            bytes_ = (layers1 + 2 * layers2) * wl + heads * head_b
            launches = 4 * (layers1 + layers2) + heads
            stream_ms = bytes_ / (rate * 1e9) * 1e3
            fixed_ms = (launches * t_fixed + layers1 * lat1 + layers2 * lat2 + heads * small + embeds * us("embed.g1")) / 1e3
            return bytes_, launches, stream_ms, fixed_ms

        solo_after_hit = e - nb
        spec = 2 * e == d and cfg.wdtype == pi.WD_BF16
        cases = {"plain_token": (est(d, 0, 1, 1), wall_plain / K * 1e3),
                 "ppd_round_after_miss": (est(e, nb, 2, 1), float(round_ms[~after_hit].mean()) if (~after_hit).any() else None),
                 "ppd_round_after_hit": (est(solo_after_hit, nb, 1 if spec else 2, 0), float(round_ms[after_hit].mean()) if after_hit.any() else None)}
        # The event pair around every bracketed launch is part of the bracketed durations: what it adds per launch is
        # read off the roofline kernel (bracketed single launches against the burst between two events), and taken
        # out of every launch of a case (6 per layer step, 2 per head pass, the embedding).
        bracket_us = 0.0
        if burst1_ms and "gemm_ffn_in.g1" in kernels:
            bracket_us = max(0.0, kernels["gemm_ffn_in.g1"]["avg_us"] - burst1_ms * 1e3)
        n_launch = {"plain_token": 6 * d + 3, "ppd_round_after_miss": 6 * (e + nb) + 5,
                    "ppd_round_after_hit": 6 * (solo_after_hit + nb) + (2 if spec else 4)}
        cases = {n: ((m[0], m[1], m[2], m[3] - n_launch[n] * bracket_us / 1e3), meas) for n, (m, meas) in cases.items()}
        model_fit = {"form": "t = bytes / rate + launches * t_fixed (GEMM launches) + latency-bound kernels (attention, merge, selection) as measured",
                     "rate_GBps": round(rate, 1), "t_fixed_us_per_gemm_launch": round(t_fixed, 2),
                     "fitted_on": "bracketed durations (an event pair around every launch) of %d GEMM launch shapes" % len(gemms),
                     "bracket_overhead_us_per_launch": round(bracket_us, 2),
                     "note": "fixed_ms is net of the bracketing; measured_ms minus model_ms is what a round costs outside its kernels (graph launch, host wait)",
                     "cases": {n: {"weight_bytes": m[0], "gemm_launches": m[1], "stream_ms": round(m[2], 4), "fixed_ms": round(m[3], 4),
                                   "model_ms": round(m[2] + m[3], 4), "measured_ms": None if meas is None else round(meas, 4)}
                               for n, (m, meas) in cases.items()}}

    # ---- CPU oracle on the host cores (bounded sample)
    cpu = None
    if not args.no_cpu_baseline:
        import oracle
        o = oracle.Oracle(model, ctx_cap=64)
        sp, sg = 8, 8
        small_prompt = pi.make_prompt(cfg, sp)
        t = time.perf_counter()
        o.plain_greedy(small_prompt, sg)
        dt = time.perf_counter() - t
        fwd = sp - 1 + sg
        cpu = {"value": round(fwd / dt, 3), "unit": "tokens/s", "cores": int(os.environ.get("OMP_NUM_THREADS", os.cpu_count())),
               "kind": "oracle", "sample": f"plain greedy, fp64, {sp}-token prompt + {sg} generated tokens "
               f"({fwd} full-model token passes, context <= {sp + sg}, against context {n_prompt}+ on the GPU: the oracle's "
               "attention share is smaller than the GPU run's); same weights as the GPU run"}
        o.close()

    d = cfg.n_layers
    out = {
        "metric": "tokens/s, PPD decode (k=%d, exit layer %d) on %s shape" % (k, e, cfg.name),
        "value": round(K / wall_ppd, 2), "unit": "tokens/s", "n_gpus": 1, "steps": K, "warmup": W,
        "ms_per_step": round(wall_ppd / K * 1e3, 4), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "bf16" if cfg.wdtype == pi.WD_BF16 else "f32", "data": "synthetic",
        "config": {"workload": f"{cfg.name}: {d} layers, d_model {cfg.d_model}, d_ff {cfg.d_ff}, vocab {cfg.vocab}, "
                               f"batch 1, prompt {n_prompt} uniform-random ids, random-init N(0,0.02) weights",
                   "k": k, "exit_layer": e, "alpha": cfg.alpha,
                   "final_prediction": {"greedy": "arg max", "topk": "top-k sampling, 3 kept", "topp": "top-p sampling, p = 0.95"}[args.sampling]},
        "round_ms": {"mean": round(float(round_ms.mean()), 4), "p50": round(float(np.percentile(round_ms, 50)), 4),
                     "p95": round(float(np.percentile(round_ms, 95)), 4),
                     "after_hit_mean": round(float(round_ms[after_hit].mean()), 4) if after_hit.any() else None,
                     "after_miss_mean": round(float(round_ms[~after_hit].mean()), 4) if (~after_hit).any() else None},
        "plain_greedy": {"tokens_per_s": round(K / wall_plain, 2), "ms_per_token": round(wall_plain / K * 1e3, 4)},
        "ppd_vs_plain_speed": round(wall_plain / wall_ppd, 4),
        "p_correct": round(p_hat, 4),
        "lm_head_passes_per_round": round((st["weight_bytes"] - (st["main_layer_rows"] + (cfg.n_layers - e) * ell) * wl)
                                          / (cfg.vocab * cfg.d_model * cfg.wbytes) / ell, 4),
        "layer_rows_per_token": {"measured_main": st["main_layer_rows"] / ell,
                                 "measured_total": (st["main_layer_rows"] + st["branch_layer_rows"]) / ell,
                                 "theorem_latency": tradeoff.expected_latency(d, e, ell, p_hat) / ell,
                                 "theorem_compute": tradeoff.expected_compute(d, e, ell, k, p_hat) / ell},
        "prefill": prefill_report(cfg, pi, n_prompt - 1, prefill_s, prefill_first_s),
        "roofline": roof, "pipelined_step": pipe, "kernels": kernels, "time_model": model_fit, "cpu_baseline": cpu,
        "setup_s": {"generate_weights": round(t_gen, 1)},
    }
    print(json.dumps(out))


if __name__ == "__main__":
    main()
