"""Host-side speculation control (Section 4.1 / 4.2 of the paper): pins of the plain
reference, and the library's host entry points against it.  No GPU needed."""
import ctypes as C
import math

import numpy as np
import pytest

from oracle import goodput_oracle as G
from paper_2406_14066_amd import spec_verify as sv


# --------------------------------------------------------------------------- pins of the reference
def test_generated_length_values_the_paper_states():
    # Section 4.1 (3): acceptance 0.7 -> first token 0.7, first two 0.49; with k = 2 that is 1 + 0.7 + 0.49
    assert abs(G.expected_generated_len(0.7, 2) - 2.19) < 1e-12
    assert G.expected_generated_len(0.7, 0) == 1.0               # minimum of one token (Section 2.2)
    assert G.expected_generated_len(1.0, 5) == 6.0               # maximum of k + 1 tokens
    assert G.expected_generated_len(0.0, 7) == 1.0
    for a in (0.1, 0.5, 0.9, 0.999):
        for k in range(9):
            geometric = sum(a ** j for j in range(k + 1))
            assert abs(G.expected_generated_len(a, k) - geometric) < 1e-9 * geometric


def test_fit_recovers_planted_coefficients_and_is_orthogonal():
    rng = np.random.default_rng(0)
    nc = rng.integers(1000, 200000, size=60).astype(float)
    nb = rng.integers(1, 600, size=60).astype(float)
    true = (3.1e-10, 4.0e-8, 2.5e-5)
    t = true[0] * nc + true[1] * nb + true[2]
    fit = G.fit_latency(nc, nb, t)
    np.testing.assert_allclose(fit, true, rtol=1e-6)
    # with noise: the residual is orthogonal to every regressor (normal equations)
    tn = t * (1 + 0.05 * rng.standard_normal(60))
    f = G.fit_latency(nc, nb, tn)
    r = tn - (f[0] * nc + f[1] * nb + f[2])
    scale = np.abs(tn).sum()
    assert abs((r * nc).sum()) < 1e-8 * scale * nc.max()
    assert abs((r * nb).sum()) < 1e-8 * scale * nb.max()
    assert abs(r.sum()) < 1e-8 * scale


def test_acceptance_rate_weighted_average():
    assert G.acceptance_rate([], 0.9, 0.6) == 0.6
    assert abs(G.acceptance_rate([(7, 10)], 0.5, 0.0) - 0.7) < 1e-15
    # decay 1: plain ratio of totals; decay 0.5: the newest step counts double the one before
    h = [(1, 10), (9, 10)]
    assert abs(G.acceptance_rate(h, 1.0, 0) - 0.5) < 1e-15
    assert abs(G.acceptance_rate(h, 0.5, 0) - (0.5 * 1 + 9) / (0.5 * 10 + 10)) < 1e-15


def test_search_limits_by_hand():
    ctx = [1000] * 4
    target = (0.0, 0.0, 1.0)          # a pass costs one second whatever it scores
    # free, perfect draft: every extra proposed token is a free generated token
    assert G.argmax_goodput(ctx, [1.0], 8, target, draft=(0, 0, 0.0)) == 8
    # nothing is ever accepted: speculation only costs
    assert G.argmax_goodput(ctx, [0.0], 8, target, draft=(0, 0, 0.1)) == 0
    # alpha = 0.5, draft pass = 0.25 target passes: goodput(k) = (2 - 0.5^k) / (1 + 0.25 k); k = 1: 1.2, k = 2: 1.1667
    curve = G.goodput_curve(ctx, [0.5], 3, target, draft=(0, 0, 0.25))
    np.testing.assert_allclose(curve, [4 * 1.0, 4 * 1.5 / 1.25, 4 * 1.75 / 1.5, 4 * 1.875 / 1.75], rtol=1e-12)
    assert G.argmax_goodput(ctx, [0.5], 3, target, draft=(0, 0, 0.25)) == 1
    # memory: k = 2 needs 4 * 3 = 12 new slots
    assert G.argmax_goodput(ctx, [1.0], 8, target, draft=(0, 0, 0.0), free_kv_tokens=12) == 2
    assert G.argmax_goodput(ctx, [1.0], 8, target, draft=(0, 0, 0.0), free_kv_tokens=3) == -1


def test_search_follows_the_trends_of_section_4_1():
    """Propose more for small batches and for accurate drafts, less for large or inaccurate ones."""
    target = (2e-10, 2.5e-7, 3e-5)    # per batched token cost matters once batches are large
    draft = (2e-11, 1e-8, 3e-6)
    best_by_B = [G.argmax_goodput([1024] * B, [0.7], 8, target, draft) for B in (1, 4, 16, 64, 256)]
    assert best_by_B == sorted(best_by_B, reverse=True) and best_by_B[0] > best_by_B[-1]
    best_by_a = [G.argmax_goodput([1024] * 16, [a], 8, target, draft) for a in (0.3, 0.5, 0.7, 0.9)]
    assert best_by_a == sorted(best_by_a) and best_by_a[0] < best_by_a[-1]


# --------------------------------------------------------------------------- the library against the reference
class LatencyModel(C.Structure):
    _fields_ = [("c_context", C.c_double), ("c_batched", C.c_double), ("c_fixed", C.c_double)]


class Tracker(C.Structure):
    _fields_ = [("accepted_weighted", C.c_double), ("attempted_weighted", C.c_double)]


class GoodputArgs(C.Structure):
    _fields_ = [("B", C.c_int32), ("max_k", C.c_int32), ("context_len", C.c_void_p), ("alpha", C.c_void_p),
                ("alpha_per_request", C.c_int32), ("target", LatencyModel), ("draft_is_model", C.c_int32),
                ("draft", LatencyModel), ("draft_fixed_seconds", C.c_double), ("free_kv_tokens", C.c_int64)]


@pytest.fixture(scope="module")
def lib():
    l = sv.lib()
    l.spec_expected_generated_len.restype = C.c_double
    l.spec_expected_generated_len.argtypes = [C.c_double, C.c_int32]
    l.spec_predict_latency.restype = C.c_double
    l.spec_predict_latency.argtypes = [C.c_void_p, C.c_double, C.c_double]
    l.spec_fit_latency.restype = C.c_int
    l.spec_fit_latency.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_int32, C.c_void_p]
    l.spec_acceptance_update.restype = None
    l.spec_acceptance_update.argtypes = [C.c_void_p, C.c_int64, C.c_int64, C.c_double]
    l.spec_acceptance_rate.restype = C.c_double
    l.spec_acceptance_rate.argtypes = [C.c_void_p, C.c_double]
    l.spec_argmax_goodput.restype = C.c_int32
    l.spec_argmax_goodput.argtypes = [C.c_void_p, C.c_void_p]
    return l


def test_library_generated_length(lib):
    for a in (0.0, 0.3, 0.7, 0.95, 0.999999, 1.0):
        for k in range(9):
            assert abs(lib.spec_expected_generated_len(a, k) - G.expected_generated_len(a, k)) < 1e-9
    assert math.isnan(lib.spec_expected_generated_len(1.2, 3))
    assert math.isnan(lib.spec_expected_generated_len(0.5, -1))


def test_library_fit_matches_reference(lib):
    rng = np.random.default_rng(3)
    nc = rng.integers(1000, 300000, size=40).astype(np.float64)
    nb = rng.integers(1, 2000, size=40).astype(np.float64)
    t = (2.2e-10 * nc + 6e-8 * nb + 4e-5) * (1 + 0.03 * rng.standard_normal(40))
    m = LatencyModel()
    assert lib.spec_fit_latency(nc.ctypes.data, nb.ctypes.data, t.ctypes.data, 40, C.addressof(m)) == sv.SPEC_OK
    ref = G.fit_latency(nc, nb, t)
    np.testing.assert_allclose([m.c_context, m.c_batched, m.c_fixed], ref, rtol=1e-8)
    assert abs(lib.spec_predict_latency(C.addressof(m), 5000.0, 40.0) - G.predict_latency(ref, 5000.0, 40.0)) < 1e-12
    # dependent columns (every pass scores the same number of tokens) are refused
    same = np.full(40, 32.0)
    assert lib.spec_fit_latency(nc.ctypes.data, same.ctypes.data, t.ctypes.data, 40, C.addressof(m)) == sv.SPEC_EINVAL
    assert lib.spec_fit_latency(nc.ctypes.data, nb.ctypes.data, t.ctypes.data, 2, C.addressof(m)) == sv.SPEC_EINVAL


def test_library_acceptance_tracker(lib):
    rng = np.random.default_rng(4)
    hist = []
    tr = Tracker()
    assert lib.spec_acceptance_rate(C.addressof(tr), 0.55) == 0.55
    for _ in range(30):
        att = int(rng.integers(0, 200))
        acc = int(rng.integers(0, att + 1))
        lib.spec_acceptance_update(C.addressof(tr), acc, att, 0.8)
        if att > 0:
            hist.append((acc, att))
        assert abs(lib.spec_acceptance_rate(C.addressof(tr), 0.55) - G.acceptance_rate(hist, 0.8, 0.55)) < 1e-12


def _call_search(lib, ctx, alphas, max_k, target, draft=None, draft_fixed=0.0, free=None):
    ctx = np.asarray(ctx, dtype=np.int32)
    al = np.asarray(alphas, dtype=np.float64)
    a = GoodputArgs()
    a.B, a.max_k = len(ctx), max_k
    a.context_len, a.alpha = ctx.ctypes.data, al.ctypes.data
    a.alpha_per_request = 1 if len(al) == len(ctx) and len(al) > 1 else 0
    a.target = LatencyModel(*target)
    a.draft_is_model = 1 if draft is not None else 0
    if draft is not None:
        a.draft = LatencyModel(*draft)
    a.draft_fixed_seconds = draft_fixed
    a.free_kv_tokens = -1 if free is None else free
    curve = np.zeros(max_k + 1, dtype=np.float64)
    k = lib.spec_argmax_goodput(C.addressof(a), curve.ctypes.data)
    return k, curve


def test_library_search_matches_reference(lib):
    rng = np.random.default_rng(6)
    for case in range(200):
        B = int(rng.integers(1, 80))
        ctx = rng.integers(0, 4000, size=B)
        per_req = case % 2 == 0 and B > 1
        alphas = rng.random(B) if per_req else [float(rng.random())]
        max_k = int(rng.integers(0, 9))
        target = (rng.random() * 1e-9, rng.random() * 1e-6, 1e-6 + rng.random() * 1e-4)
        use_model = case % 3 != 0
        draft = (rng.random() * 1e-10, rng.random() * 1e-7, rng.random() * 1e-5) if use_model else None
        fixed = float(rng.random() * 1e-4)
        free = None if case % 5 else int(rng.integers(0, B * 10))
        k, curve = _call_search(lib, ctx, alphas, max_k, target, draft, fixed, free)
        ref_curve = G.goodput_curve(list(ctx), list(alphas), max_k, target, draft, fixed, free)
        assert k == G.argmax_goodput(list(ctx), list(alphas), max_k, target, draft, fixed, free)
        for got, want in zip(curve, ref_curve):
            if want is None:
                assert math.isnan(got)
            else:
                assert abs(got - want) <= 1e-9 * want


def test_library_search_rejects_bad_arguments(lib):
    assert lib.spec_argmax_goodput(None, None) == -1
    k, _ = _call_search(lib, [10, 20], [1.5], 4, (0, 0, 1.0))
    assert k == -1
    k, _ = _call_search(lib, [10, -1], [0.5], 4, (0, 0, 1.0))
    assert k == -1
    a = GoodputArgs()
    a.B, a.max_k = 1, 9    # beyond SPEC_K_MAX
    assert lib.spec_argmax_goodput(C.addressof(a), None) == -1
