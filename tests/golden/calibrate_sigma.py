"""Calibrate the target-vs-draft noise level of the synthetic logits.

Writes nothing by itself: prints, for each (vocab, draft_std, alpha) of the named
workloads, the sigma at which the mean per-token acceptance probability
sum_v min(p_v, q_v) -- evaluated by the CPU oracle only -- reaches alpha on rows
drawn the way ``workloads.make_logits`` draws them.  The printed values are the
ones stored in ``workloads.SIGMA_FOR_ALPHA``.

Run from the repository root:  python tests/golden/calibrate_sigma.py
"""
import os
import sys

import numpy as np

sys.path.insert(0, os.path.join(os.path.dirname(__file__), "..", ".."))
import oracle  # noqa: E402


def mean_alpha(V, draft_std, sigma, rows=24, seed=1234):
    rng = np.random.default_rng(seed)
    draft = rng.standard_normal((rows, V), dtype=np.float32) * np.float32(draft_std)
    noise = rng.standard_normal((rows, V), dtype=np.float32)
    target = draft + noise * np.float32(sigma)
    return float(np.mean([oracle.accept_probability(target[r], draft[r]) for r in range(rows)]))


def solve(V, draft_std, alpha, lo=0.05, hi=3.0, iters=18):
    for _ in range(iters):
        mid = 0.5 * (lo + hi)
        if mean_alpha(V, draft_std, mid) > alpha:
            lo = mid
        else:
            hi = mid
    return 0.5 * (lo + hi)


if __name__ == "__main__":
    for V, s, alphas in [(1024, 2.0, [0.61]), (32000, 3.0, [0.5, 0.6, 0.7, 0.9]), (128256, 3.0, [0.75])]:
        for a in alphas:
            sg = solve(V, s, a)
            print("V=%d draft_std=%.1f alpha=%.2f -> sigma=%.3f (check %.4f)" % (V, s, a, sg, mean_alpha(V, s, sg, seed=99)))
