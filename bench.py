#!/usr/bin/env python3
"""Benchmark of the PPD decode path on one MI355X.

A step is one PPD round (`ppd_step`): main token to the exit layer when the previous round
missed, early LM head + top-k, d-dbar pipelined steps (main row at layer dbar+j and k candidate
rows at layer j in the same launches), final head, verification, adoption.  One round emits
one token.  Inputs (synthetic weights and prompt) are resident in HBM before the timed region.

Prints one JSON line: PPD tokens/s as `value`, plain greedy on the same kernels next to it,
the roofline of the dominant kernel (the two-group FFN-in GEMM), the HBM fraction of the whole
pipelined phase, the measured match rate and layer-row counts against Theorem 4.1, and the
CPU oracle timed on the host cores.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0   # MI355X HBM3E, published
# HBM bytes per launch of the roofline kernel from rocprofv3 FETCH_SIZE / WRITE_SIZE, scaled by a copy kernel of
# known size (profiles/llama7b_ppd_k3_kernels.txt); only valid for the configuration it was collected on
MEASURED_TRAFFIC = {"llama7b": 180.80e6}


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
    ap.add_argument("--copy-probe", action="store_true",
                    help="also run one 1 GiB device-to-device copy (a kernel of known traffic, to scale rocprofv3 byte counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (the pipelined decode step of one sequence "
              "lives on one device); --gpus must be 1", file=sys.stderr)
        sys.exit(2)

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
    stream = torch.cuda.current_stream()

    def timed(P, step_fn, warm, steps):
        P.ppd_prefill(prompt)
        for _ in range(warm):
            step_fn()
        torch.cuda.synchronize()
        ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        t = time.perf_counter()
        ev0.record(stream)
        for _ in range(steps):
            step_fn()
        ev1.record(stream)
        torch.cuda.synchronize()
        wall = time.perf_counter() - t
        return wall, ev0.elapsed_time(ev1) / 1e3

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

    # ---- PPD rounds (each call is synchronous: the host clock around a call is the round's latency)
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
    P.ppd_prefill(prompt)                  # (synchronous) the prompt in chunks of 8 positions through the decode kernels
    prefill_s = time.perf_counter() - t
    wall_ppd, _ = timed(P, ppd_round, W, K)
    round_ms, round_hit = np.array(round_ms[W:]), np.array(round_hit[W:])
    # a round's length is set by how it starts: after a hit it resumes mid-stack (no solo phase when dbar = d/2)
    after_hit = np.concatenate([[False], round_hit[:-1]])
    st = P.ppd_get_stats()
    ell = st["rounds"]
    p_hat = st["matches"] / ell
    # ---- plain greedy on the same kernels, same context
    wall_plain, _ = timed(P, P.plain_greedy_step, W, K)

    # ---- timing with HIP events on the library's own streams, separate short passes
    # (a) every kernel bracketed, plain greedy steps: the kernels run alone on the machine, as rocprofv3 sees them
    # (b) only the phases bracketed, PPD rounds: the parallel phase as it runs in normal operation
    kt, ph = {}, {}
    if args.profile_rounds > 0:
        P.ppd_prefill(prompt)
        for _ in range(W):
            P.plain_greedy_step()
        P.ppd_set_profiling(2)
        for _ in range(args.profile_rounds):
            P.plain_greedy_step()
        kt = P.ppd_get_kernel_time()
        P.ppd_set_profiling(0)
        P.ppd_prefill(prompt)
        for _ in range(W):
            P.ppd_step(want_info=False)
        P.ppd_set_profiling(1)
        for _ in range(args.profile_rounds):
            P.ppd_step(want_info=False)
        ph = P.ppd_get_kernel_time()
        P.ppd_set_profiling(0)
    # (c) the roofline kernel alone: a burst of FFN-in GEMMs (one per layer, cold weights each) between two events
    burst_ms = None
    if args.profile_rounds > 0:
        P.ppd_prefill(prompt)
        burst_ms = P.ppd_time_ffn_in(4 * cfg.n_layers)
    ctx_mid = n_prompt + W + args.profile_rounds // 2
    wl = cfg.layer_weight_bytes()
    n_in = 2 if cfg.act == pi.ACT_SWIGLU else 1
    ffn_in_bytes = n_in * cfg.d_model * cfg.d_ff * cfg.wbytes
    dom = kt.get("gemm_ffn_in.g1")
    roof = None
    if dom and burst_ms:
        avg_s = burst_ms / 1e3
        ach = ffn_in_bytes / avg_s / 1e9
        if cfg.wdtype != pi.WD_BF16:
            kname = "gemm_kernel<float, 1, 0, %s, WR> (norm + first FFN matrix + activation), one row" % ("true" if n_in == 2 else "false")
        elif n_in == 2:
            kname = "gemm_mfma_kernel<true, false> (norm + FFN-in gate and up matrices + SwiGLU), one row"
        else:
            kname = "gemm_mfma_kernel<false, false> (norm + first FFN matrix + activation), one row"
        roof = {"bound": "hbm", "kernel": kname, "achieved": round(ach, 1),
                "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": round(ach / HBM_PEAK_GBS, 4),
                "traffic": MEASURED_TRAFFIC.get(cfg.name) if cfg.name.startswith("llama7b") else None,
                "bytes_per_launch": ffn_in_bytes, "avg_launch_us": round(avg_s * 1e6, 2),
                "timing": "HIP events around a burst of %d back-to-back launches on the library's stream" % (4 * cfg.n_layers),
                "avg_launch_us_single_bracketed": round(dom["ms"] / dom["launches"] * 1e3, 2),
                "stream_read_GBps": round(stream_gbs, 1), "frac_of_stream_read": round(ach / stream_gbs, 4)}
    pp = ph.get("phase.g2")
    pipe = None
    if pp:
        nb = cfg.n_layers - e
        kv = ctx_mid * cfg.kv_bytes_per_pos_layer()
        step_bytes = 2 * wl + 2 * kv
        step_s = pp["ms"] / pp["launches"] / nb / 1e3
        pipe = {"bytes_per_step": step_bytes, "us_per_step": round(step_s * 1e6, 2),
                "GBps": round(step_bytes / step_s / 1e9, 1), "hbm_frac": round(step_bytes / step_s / 1e9 / HBM_PEAK_GBS, 4),
                "frac_of_stream_read": round(step_bytes / step_s / 1e9 / stream_gbs, 4)}
    kernels = {n: {"avg_us": round(v["ms"] / v["launches"] * 1e3, 2), "launches": v["launches"]} for n, v in kt.items()}

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
               f"({fwd} full-model token passes, context <= {sp + sg}); same weights as the GPU run"}
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
        "prefill": {"positions": n_prompt - 1, "ms": round(prefill_s * 1e3, 2),
                    "positions_per_s": round((n_prompt - 1) / prefill_s, 1)},
        "roofline": roof, "pipelined_step": pipe, "kernels": kernels, "cpu_baseline": cpu,
        "setup_s": {"generate_weights": round(t_gen, 1)},
    }
    print(json.dumps(out))


if __name__ == "__main__":
    main()
