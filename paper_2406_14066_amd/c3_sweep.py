"""The c3 sweep (B=32, L=1024, 7B-shaped heads): for every proposed length k = 0..8 and
acceptance level 0.5 / 0.7 / 0.9 run the verification step and report its time, the verified
positions per second, the accepted and emitted token counts, and Eq. 4's prediction of the
emitted tokens at the measured per-token acceptance rate.

    python -m paper_2406_14066_amd.c3_sweep [--steps 50] [--k 0 1 2 ...] [--alpha 0.5 0.7 0.9]

One JSON object per line.
"""
from __future__ import annotations

import argparse
import json
import sys


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--k", type=int, nargs="*", default=list(range(9)))
    ap.add_argument("--alpha", type=float, nargs="*", default=[0.5, 0.7, 0.9])
    args = ap.parse_args()

    import torch
    from . import spec_verify as sv
    from . import workloads as W
    from .harness import DeviceStep
    if not torch.cuda.is_available():
        print("c3_sweep: no GPU visible", file=sys.stderr)
        sys.exit(2)

    for k in args.k:
        for alpha in args.alpha:
            w = W.config("c3", k=k, alpha=alpha)
            ds = DeviceStep(w, kv_layout=sv.KV_MFMA, with_debug=False)
            # four copies of the big inputs in turn (2.3 GB in all), so that consecutive launches read
            # different addresses and the 256 MB last-level cache cannot serve them
            pairs = ds.rotated(4)
            for i in range(10):
                sv.spec_verify_step(*pairs[i % len(pairs)], ds.workspace)
            torch.cuda.synchronize()
            ds.counters.zero_()
            sv.spec_profile_begin(args.steps)
            for i in range(args.steps):
                sv.spec_verify_step(*pairs[i % len(pairs)], ds.workspace)
            torch.cuda.synchronize()
            ms, n = sv.spec_profile_end()["step"]
            us = ms / n * 1e3
            c = ds.counters.cpu().numpy() // args.steps
            proposed, accepted, attempted, emitted = (int(x) for x in c[:4])
            rate = accepted / attempted if attempted else None
            predicted = w.B * sv.expected_generated_len(rate, k) if rate is not None else float(w.B)
            step_bytes = w.attn_algorithmic_bytes() + w.reject_algorithmic_bytes()
            print(json.dumps({
                "k": k, "alpha_target": alpha, "step_us": round(us, 1),
                "verified_tokens_per_s": round(w.verified_tokens() / (us * 1e-6)),
                "emitted_tokens_per_s": round(emitted / (us * 1e-6)),
                "accepted": accepted, "emitted": emitted, "proposed": proposed,
                "acceptance_rate_measured": None if rate is None else round(rate, 4),
                "emitted_predicted_eq4": round(predicted, 2),
                "algorithmic_TBps": round(step_bytes / (us * 1e-6) / 1e12, 3),
            }), flush=True)
            del ds, pairs
            torch.cuda.empty_cache()


if __name__ == "__main__":
    main()
