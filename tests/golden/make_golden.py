#!/usr/bin/env python3
"""Writes the stored oracle outputs for the full-size configurations.

Calls only the CPU oracle and the input generator (never the HIP library).  One file per
configuration, tests/golden/<config>.npz, holding the oracle's greedy tokens and, for every
generated position, its final-layer and early-exit logits at a fixed sample of vocabulary ids
plus its top-8 (ids and values).  The early-exit logits and the tokens do not depend on k, so the
oracle's PPD loop is run with k = 1 (Algorithm 2; exit layer of the configuration).

With --full, writes tests/golden/<config>_full.npz instead: every logit of the vocabulary (final and early) at the
first, the middle and the last generated position, from the same oracle run.

Usage: python tests/golden/make_golden.py [--full] llama7b [llama7b_a0p1 ...]
"""
import os
import sys
import time

import numpy as np

HERE = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, os.path.dirname(os.path.dirname(HERE)))

import oracle  # noqa: E402
import ppd_inputs as pi  # noqa: E402

N_SAMPLE, N_TOP = 256, 8


def sample_ids(cfg):
    rng = np.random.default_rng(12345)
    return np.sort(rng.choice(cfg.vocab, N_SAMPLE, replace=False)).astype(np.int32)


def top(z):
    order = np.lexsort((np.arange(z.shape[-1]), -z))[:N_TOP]
    return order.astype(np.int32), z[order]


def make(name, n_gen=None, full=False):
    cfg = pi.CONFIGS[name]
    ell = n_gen or cfg.n_gen
    t0 = time.time()
    m = pi.make_model(cfg)
    prompt = pi.make_prompt(cfg)
    o = oracle.Oracle(m, ctx_cap=cfg.n_prompt + ell + 1)
    print(name, "weights ready", round(time.time() - t0, 1), "s", flush=True)
    r = o.ppd(prompt, ell, 1, cfg.exit_layer, want_logits=True)
    if full:
        pos = np.array(sorted({0, ell // 2, ell - 1}), dtype=np.int32)
        np.savez_compressed(
            os.path.join(HERE, name + "_full.npz"),
            config=name, n_prompt=cfg.n_prompt, n_gen=ell, exit_layer=cfg.exit_layer,
            weights_checksum=np.uint64(m.checksum()), tokens=r["tokens"], positions=pos,
            final_logits=r["final_logits"][pos].astype(np.float32),
            early_logits=r["early_logits"][pos].astype(np.float32))
        print(name, "full logits done in", round(time.time() - t0, 1), "s", flush=True)
        return
    ids = sample_ids(cfg)
    ft = [top(z) for z in r["final_logits"]]
    et = [top(z) for z in r["early_logits"]]
    np.savez_compressed(
        os.path.join(HERE, name + ".npz"),
        config=name, n_prompt=cfg.n_prompt, n_gen=ell, exit_layer=cfg.exit_layer,
        weights_checksum=np.uint64(m.checksum()), prompt=prompt, tokens=r["tokens"], sample_ids=ids,
        final_samples=r["final_logits"][:, ids].astype(np.float32),
        early_samples=r["early_logits"][:, ids].astype(np.float32),
        final_top_ids=np.stack([a for a, _ in ft]), final_top_vals=np.stack([b for _, b in ft]).astype(np.float32),
        early_top_ids=np.stack([a for a, _ in et]), early_top_vals=np.stack([b for _, b in et]).astype(np.float32))
    print(name, "done in", round(time.time() - t0, 1), "s", flush=True)


if __name__ == "__main__":
    args = sys.argv[1:]
    full = "--full" in args
    for arg in (a for a in args if a != "--full"):
        n, _, g = arg.partition(":")
        make(n, int(g) if g else None, full)
