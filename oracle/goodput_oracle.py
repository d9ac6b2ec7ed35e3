"""Plain reference for the host-side speculation control of arXiv 2406.14066 (Section 4.1,
Eq. 1-4, and the search of Section 4.2's listing "Finding k to maximize goodput").

TEST INFRASTRUCTURE ONLY: the tests compare the library's host entry points with these
functions.  Written from the equations, in their notation; numpy's least squares solver is
the one library step.  Where the listing is silent or garbled the reading is:
  * k = 0 (no speculation, one token per request) is a candidate of the search: the prose
    of Section 4.2 has the system disable speculation when the proposed length comes out as 0;
  * the listing's proposed-token count depends on k (it is printed without it);
  * T_draft = k passes of the draft model over the batch (Section 4.1), or a constant for
    proposers whose cost does not depend on k; a step with k = 0 runs no proposer.
"""
import numpy as np


def expected_generated_len(alpha, k):
    """Eq. 4: (1 - alpha^(k+1)) / (1 - alpha), bonus token included."""
    if alpha == 1.0:
        return float(k + 1)
    return (1.0 - alpha ** (k + 1)) / (1.0 - alpha)


def predict_latency(model, n_context, n_batched):
    """Eq. 3 with model = (per context token, per batched token, constant)."""
    return model[0] * n_context + model[1] * n_batched + model[2]


def fit_latency(n_context, n_batched, seconds):
    """Eq. 3's coefficients by linear regression."""
    X = np.stack([np.asarray(n_context, float), np.asarray(n_batched, float), np.ones(len(seconds))], axis=1)
    coef, *_ = np.linalg.lstsq(X, np.asarray(seconds, float), rcond=None)
    return tuple(float(c) for c in coef)


def acceptance_rate(history, decay, prior):
    """Weighted average of past steps; history = [(accepted, attempted), ...], oldest first."""
    num = den = 0.0
    n = len(history)
    for age, (acc, att) in zip(range(n - 1, -1, -1), history):
        num += decay ** age * acc
        den += decay ** age * att
    return num / den if den > 0 else prior


def goodput_curve(context_len, alphas, max_k, target, draft=None, draft_fixed=0.0, free_kv_tokens=None):
    """Eq. 1 for k = 0..max_k (None where the batch would not fit)."""
    B = len(context_len)
    n_context = float(sum(context_len))
    if len(alphas) == 1:
        alphas = list(alphas) * B
    out = []
    for k in range(max_k + 1):
        proposed = B * (k + 1)
        if free_kv_tokens is not None and proposed > free_kv_tokens:
            out.append(None)
            continue
        generated = sum(expected_generated_len(a, k) for a in alphas)
        t = predict_latency(target, n_context, proposed)                  # Eq. 2: T_target
        if k > 0:                                                         #        + T_draft
            t += k * predict_latency(draft, n_context, B) if draft is not None else draft_fixed
        out.append(generated / t)
    return out


def argmax_goodput(*args, **kw):
    curve = goodput_curve(*args, **kw)
    best_k, best = -1, -1.0
    for k, g in enumerate(curve):
        if g is not None and g > best:
            best_k, best = k, g
    return best_k
