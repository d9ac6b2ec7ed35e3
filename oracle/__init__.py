"""ctypes wrapper of the CPU oracle (``spec_oracle.c``).

Test infrastructure only: the tests, the smoke check and the benchmark's
CPU-baseline leg import this; the product package never does.  The wrapper
only marshals numpy arrays; all arithmetic is in the C file.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from dataclasses import dataclass

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "spec_oracle.c")
_LIB = os.path.join(_HERE, "libspec_oracle.so")

K_MAX = 8
NEAR_TIE = 1e-6


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (strict IEEE: no fast-math, no FMA contraction)."""
    stale = (not os.path.exists(_LIB)) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC)
    if force or stale:
        tmp = _LIB + ".tmp.%d" % os.getpid()
        subprocess.run(
            ["gcc", "-O2", "-std=c99", "-fPIC", "-shared", "-ffp-contract=off",
             "-fno-fast-math", "-Wall", "-o", tmp, _SRC, "-lm"],
            check=True,
        )
        os.replace(tmp, _LIB)
    return _LIB


_lib = None


def _load():
    global _lib
    if _lib is None:
        lib = ctypes.CDLL(build())
        c = ctypes
        lib.oracle_philox4x32_10.argtypes = [c.c_void_p, c.c_void_p, c.c_void_p]
        lib.oracle_philox4x32_10.restype = None
        lib.oracle_u_accept.argtypes = [c.c_uint64, c.c_uint64, c.c_int32, c.c_int32]
        lib.oracle_u_accept.restype = c.c_double
        lib.oracle_u_race.argtypes = [c.c_uint64, c.c_uint64, c.c_int32, c.c_int32]
        lib.oracle_u_race.restype = c.c_double
        lib.oracle_verify_attn.argtypes = [c.c_int32] * 8 + [c.c_void_p] * 6 + [c.c_double, c.c_void_p]
        lib.oracle_verify_attn.restype = c.c_int
        lib.oracle_softmax_row.argtypes = [c.c_void_p, c.c_int32, c.c_void_p]
        lib.oracle_softmax_row.restype = None
        lib.oracle_accept_probability.argtypes = [c.c_void_p, c.c_void_p, c.c_int32]
        lib.oracle_accept_probability.restype = c.c_double
        lib.oracle_reject_sample.argtypes = (
            [c.c_int32, c.c_int32] + [c.c_void_p] * 4 + [c.c_uint64, c.c_uint64] + [c.c_void_p] * 7
        )
        lib.oracle_reject_sample.restype = c.c_int
        lib.oracle_reject_greedy.argtypes = [c.c_int32, c.c_int32] + [c.c_void_p] * 7
        lib.oracle_reject_greedy.restype = c.c_int
        lib.oracle_reject_onehot.argtypes = (
            [c.c_int32, c.c_int32] + [c.c_void_p] * 3 + [c.c_uint64, c.c_uint64] + [c.c_void_p] * 7)
        lib.oracle_reject_onehot.restype = c.c_int
        lib.oracle_kv_append.argtypes = [c.c_int32] * 8 + [c.c_void_p] * 7
        lib.oracle_kv_append.restype = c.c_int
        lib.oracle_kv_after_accept.argtypes = [c.c_int32] + [c.c_void_p] * 5
        lib.oracle_kv_after_accept.restype = None
        lib.oracle_expected_generated_len.argtypes = [c.c_double, c.c_int32]
        lib.oracle_expected_generated_len.restype = c.c_double
        _lib = lib
    return _lib


def _ptr(a):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def _carr(a, dtype):
    a = np.ascontiguousarray(a, dtype=dtype)
    return a


def philox4x32_10(ctr, key):
    c = _carr(ctr, np.uint32)
    k = _carr(key, np.uint32)
    assert c.shape == (4,) and k.shape == (2,)
    out = np.zeros(4, dtype=np.uint32)
    _load().oracle_philox4x32_10(_ptr(c), _ptr(k), _ptr(out))
    return out


def u_accept(seed, step, b, i):
    return float(_load().oracle_u_accept(seed, step, b, i))


def u_race(seed, step, b, v):
    return float(_load().oracle_u_race(seed, step, b, v))


def softmax_row(logits):
    x = _carr(logits, np.float32)
    out = np.empty(x.shape[0], dtype=np.float64)
    _load().oracle_softmax_row(_ptr(x), x.shape[0], _ptr(out))
    return out


def accept_probability(target_row, draft_row):
    t = _carr(target_row, np.float32)
    d = _carr(draft_row, np.float32)
    assert t.shape == d.shape and t.ndim == 1
    return float(_load().oracle_accept_probability(_ptr(t), _ptr(d), t.shape[0]))


def expected_generated_len(alpha, k):
    return float(_load().oracle_expected_generated_len(float(alpha), int(k)))


def verify_attn(q, k_pages, v_pages, block_table, kv_len, cu_q_len, scale=0.0):
    """Lookahead attention.  q [T,Hq,d]; pages [nb,Hkv,bs,d] token-major; fp32
    arrays, or uint16 arrays holding bfloat16 bit patterns.  Returns fp32 [T,Hq,d]."""
    if q.dtype == np.float32:
        dtype = 0
    elif q.dtype == np.uint16:
        dtype = 1
    else:
        raise TypeError("q must be float32 or uint16 (bf16 bits)")
    assert k_pages.dtype == q.dtype and v_pages.dtype == q.dtype
    q = np.ascontiguousarray(q)
    k_pages = np.ascontiguousarray(k_pages)
    v_pages = np.ascontiguousarray(v_pages)
    block_table = _carr(block_table, np.int32)
    kv_len = _carr(kv_len, np.int32)
    cu_q_len = _carr(cu_q_len, np.int32)
    T, Hq, d = q.shape
    nb, Hkv, bs, d2 = k_pages.shape
    assert d2 == d and v_pages.shape == k_pages.shape
    B = kv_len.shape[0]
    assert cu_q_len.shape == (B + 1,) and int(cu_q_len[-1]) == T
    assert block_table.ndim == 2 and block_table.shape[0] == B
    out = np.zeros((T, Hq, d), dtype=np.float32)
    rc = _load().oracle_verify_attn(
        B, Hq, Hkv, d, bs, nb, block_table.shape[1], dtype,
        _ptr(q), _ptr(k_pages), _ptr(v_pages), _ptr(block_table), _ptr(kv_len), _ptr(cu_q_len),
        float(scale), _ptr(out))
    if rc != 0:
        raise ValueError("oracle_verify_attn: malformed arguments")
    return out


@dataclass
class RejectResult:
    accepted_len: np.ndarray      # [B] int32
    next_token: np.ndarray        # [B] int32
    out_tokens: np.ndarray        # [B, K_MAX+1] int32, -1 padded
    counters: np.ndarray          # [8] int64
    dec_u: np.ndarray             # [T-B] float64, NaN where not evaluated
    dec_ratio: np.ndarray         # [T-B] float64
    race_margin: np.ndarray       # [B] float64


def reject_sample(target_logits, draft_logits, draft_tokens, cu_q_len, seed, step, counters=None):
    t = _carr(target_logits, np.float32)
    cu = _carr(cu_q_len, np.int32)
    B = cu.shape[0] - 1
    T, V = t.shape
    assert int(cu[-1]) == T
    d = _carr(draft_logits, np.float32).reshape(T - B, V)
    x = _carr(draft_tokens, np.int32)
    assert x.shape == (T - B,)
    acc = np.zeros(B, dtype=np.int32)
    nxt = np.zeros(B, dtype=np.int32)
    out_tokens = np.zeros((B, K_MAX + 1), dtype=np.int32)
    cnt = np.zeros(8, dtype=np.int64) if counters is None else _carr(counters, np.int64).copy()
    dec_u = np.full(max(T - B, 1), np.nan, dtype=np.float64)
    dec_ratio = np.full(max(T - B, 1), np.nan, dtype=np.float64)
    margin = np.zeros(B, dtype=np.float64)
    rc = _load().oracle_reject_sample(
        B, V, _ptr(t), _ptr(d), _ptr(x), _ptr(cu), int(seed), int(step),
        _ptr(acc), _ptr(nxt), _ptr(out_tokens), _ptr(cnt), _ptr(dec_u), _ptr(dec_ratio), _ptr(margin))
    if rc != 0:
        raise ValueError("oracle_reject_sample: malformed arguments")
    return RejectResult(acc, nxt, out_tokens, cnt, dec_u[: T - B], dec_ratio[: T - B], margin)


def reject_greedy(target_logits, draft_tokens, cu_q_len, counters=None):
    """Greedy acceptance; no random numbers.  dec_u / dec_ratio / race_margin of the result are empty."""
    t = _carr(target_logits, np.float32)
    cu = _carr(cu_q_len, np.int32)
    B = cu.shape[0] - 1
    T, V = t.shape
    assert int(cu[-1]) == T
    x = _carr(draft_tokens, np.int32)
    assert x.shape == (T - B,)
    acc = np.zeros(B, dtype=np.int32)
    nxt = np.zeros(B, dtype=np.int32)
    out_tokens = np.zeros((B, K_MAX + 1), dtype=np.int32)
    cnt = np.zeros(8, dtype=np.int64) if counters is None else _carr(counters, np.int64).copy()
    rc = _load().oracle_reject_greedy(B, V, _ptr(t), _ptr(x), _ptr(cu), _ptr(acc), _ptr(nxt), _ptr(out_tokens), _ptr(cnt))
    if rc != 0:
        raise ValueError("oracle_reject_greedy: malformed arguments")
    empty = np.zeros(0, dtype=np.float64)
    return RejectResult(acc, nxt, out_tokens, cnt, empty, empty, np.full(B, np.inf))


def reject_onehot(target_logits, draft_tokens, cu_q_len, seed, step, counters=None):
    """Stochastic acceptance against a point-mass draft distribution (proposer without logits)."""
    t = _carr(target_logits, np.float32)
    cu = _carr(cu_q_len, np.int32)
    B = cu.shape[0] - 1
    T, V = t.shape
    assert int(cu[-1]) == T
    x = _carr(draft_tokens, np.int32)
    assert x.shape == (T - B,)
    acc = np.zeros(B, dtype=np.int32)
    nxt = np.zeros(B, dtype=np.int32)
    out_tokens = np.zeros((B, K_MAX + 1), dtype=np.int32)
    cnt = np.zeros(8, dtype=np.int64) if counters is None else _carr(counters, np.int64).copy()
    dec_u = np.full(max(T - B, 1), np.nan, dtype=np.float64)
    dec_ratio = np.full(max(T - B, 1), np.nan, dtype=np.float64)
    margin = np.zeros(B, dtype=np.float64)
    rc = _load().oracle_reject_onehot(
        B, V, _ptr(t), _ptr(x), _ptr(cu), int(seed), int(step),
        _ptr(acc), _ptr(nxt), _ptr(out_tokens), _ptr(cnt), _ptr(dec_u), _ptr(dec_ratio), _ptr(margin))
    if rc != 0:
        raise ValueError("oracle_reject_onehot: malformed arguments")
    return RejectResult(acc, nxt, out_tokens, cnt, dec_u[: T - B], dec_ratio[: T - B], margin)


def kv_append(new_k, new_v, k_cache, v_cache, block_table, kv_len, cu_q_len, layout=0):
    """Writes the step's new K/V rows [T,Hkv,d] into COPIES of the caches (flat or
    [nb,Hkv,bs,d] arrays of nb*Hkv*bs*d elements; layout 0 token-major, 1 matrix-operand
    tiles) and returns the copies."""
    new_k = np.ascontiguousarray(new_k)
    new_v = np.ascontiguousarray(new_v)
    T, Hkv, d = new_k.shape
    dtype = 0 if new_k.dtype == np.float32 else 1
    kc = np.array(k_cache, copy=True, order="C")
    vc = np.array(v_cache, copy=True, order="C")
    assert kc.dtype == new_k.dtype and vc.dtype == new_k.dtype
    bs = 16
    nb = kc.size // (Hkv * bs * d)
    bt = _carr(block_table, np.int32)
    kl = _carr(kv_len, np.int32)
    cu = _carr(cu_q_len, np.int32)
    rc = _load().oracle_kv_append(kl.shape[0], Hkv, d, bs, nb, bt.shape[1], dtype, layout, _ptr(new_k), _ptr(new_v),
                                  _ptr(kc), _ptr(vc), _ptr(bt), _ptr(kl), _ptr(cu))
    if rc != 0:
        raise ValueError("oracle_kv_append: malformed arguments")
    return kc, vc


def kv_after_accept(kv_len, cu_q_len, accepted_len):
    kl = _carr(kv_len, np.int32)
    cu = _carr(cu_q_len, np.int32)
    acc = _carr(accepted_len, np.int32)
    new_len = np.zeros_like(kl)
    draft_next = np.zeros_like(kl)
    _load().oracle_kv_after_accept(kl.shape[0], _ptr(kl), _ptr(cu), _ptr(acc), _ptr(new_len), _ptr(draft_next))
    return new_len, draft_next
