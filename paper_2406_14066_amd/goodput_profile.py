"""Offline profiler for the speculation controller (Section 5.2 of the paper, "Offline
Profiler and Online Adaptor"): times the verification step of this library on a grid of
batch sizes, context lengths and proposed lengths, fits Eq. 3 to the measurements, and
prints the fitted model together with the proposed length the search of Section 4.2
picks for a range of batch sizes and acceptance rates.

    python -m paper_2406_14066_amd.goodput_profile [--draft-fraction 0.1]

What is timed is the verification step only (attention over the paged KV cache and the
acceptance stage): the dense layers of a model are not part of this library, so the
fitted constant is far smaller than a real model's.  The draft model is a stand-in: one
draft pass is taken to cost `--draft-fraction` of a one-token target pass.
"""
from __future__ import annotations

import argparse
import json
import sys

import numpy as np


def time_step(w, sv, DeviceStep, torch, steps=30):
    import time
    ds = DeviceStep(w, kv_layout=sv.KV_MFMA, with_debug=False)
    # a serving system runs this step once per layer on that layer's own KV: time it on inputs
    # that are not in the caches (copies at different addresses in turn, about 2 GB in all)
    pairs = ds.rotated(int(min(16, max(2, -(-2_000_000_000 // max(ds.input_bytes(), 1))))))
    # the GPU clocks down while the host prepares the next workload: run for a while before timing
    t0 = time.perf_counter()
    while time.perf_counter() - t0 < 0.05:
        for i in range(20):
            sv.spec_verify_step(*pairs[i % len(pairs)], ds.workspace)
        torch.cuda.synchronize()
    sv.spec_profile_begin(steps)
    for i in range(steps):
        sv.spec_verify_step(*pairs[i % len(pairs)], ds.workspace)
    torch.cuda.synchronize()
    ms, n = sv.spec_profile_end()["step"]
    return ms / n * 1e-3


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--draft-fraction", type=float, default=0.1)
    ap.add_argument("--batch", type=int, nargs="*", default=[4, 16, 64])
    ap.add_argument("--context", type=int, nargs="*", default=[512, 1024, 2048])
    ap.add_argument("--k", type=int, nargs="*", default=[0, 2, 4, 8])
    args = ap.parse_args()

    import torch
    from . import spec_verify as sv
    from . import workloads as W
    from .harness import DeviceStep
    if not torch.cuda.is_available():
        print("goodput_profile: no GPU visible", file=sys.stderr)
        sys.exit(2)

    rows = []
    for B in args.batch:
        for L in args.context:
            for k in args.k:
                w = W.make_workload("grid", B=B, Hq=32, Hkv=32, d=128, V=32000, dtype="bf16", kv_len=[L] * B,
                                    k=[k] * B, draft_std=3.0, sigma=0.77, data_seed=B * 100003 + L * 11 + k,
                                    philox_seed=1, philox_step=0)
                t = time_step(w, sv, DeviceStep, torch)
                rows.append((B * L, B * (k + 1), t))
                print("B=%d L=%d k=%d: N_context=%d N_batched=%d step %.1f us" % (B, L, k, B * L, B * (k + 1), t * 1e6),
                      flush=True)
    nc, nb, t = (np.array(c, dtype=np.float64) for c in zip(*rows))
    target = sv.fit_latency(nc, nb, t)
    pred = np.array([sv.predict_latency(target, a, b) for a, b in zip(nc, nb)])
    rel = np.abs(pred - t) / t
    draft = sv.LatencyModel(target.c_context * args.draft_fraction, target.c_batched * args.draft_fraction,
                            target.c_fixed * args.draft_fraction)
    table = {}
    for B in (1, 4, 16, 64, 256):
        for alpha in (0.3, 0.5, 0.7, 0.9):
            k, _ = sv.argmax_goodput([1024] * B, alpha, sv.K_MAX, target, draft)
            table["B=%d,alpha=%.1f" % (B, alpha)] = k
    print(json.dumps({
        "eq3_fit_seconds": {"per_context_token": target.c_context, "per_batched_token": target.c_batched,
                            "fixed": target.c_fixed},
        "fit_points": len(rows),
        "fit_rel_error_mean": float(rel.mean()), "fit_rel_error_max": float(rel.max()),
        "draft_fraction": args.draft_fraction,
        "best_k_at_context_1024": table,
    }))


if __name__ == "__main__":
    main()
