"""Pins of the CPU oracle against things other than itself.

Each test checks an oracle function against a published known-answer vector, a
number the paper prints, a closed form, an independent brute-force formulation
or a library routine, so that a dropped term, a wrong sign or index, or a
transposed operand in ``oracle/spec_oracle.c`` fails at least one of them.
"""
import math
import os

import numpy as np
import pytest
import scipy.stats

import oracle
from paper_2406_14066_amd import workloads as W

K_MAX = oracle.K_MAX


# --------------------------------------------------------------------------
# Philox4x32-10
# --------------------------------------------------------------------------
def _py_philox(ctr, key):
    """Independent big-int implementation of the published round function."""
    c = [int(x) for x in ctr]
    k = [int(x) for x in key]
    for _ in range(10):
        lo0 = (0xD2511F53 * c[0]) & 0xFFFFFFFF
        hi0 = (0xD2511F53 * c[0]) >> 32
        lo1 = (0xCD9E8D57 * c[2]) & 0xFFFFFFFF
        hi1 = (0xCD9E8D57 * c[2]) >> 32
        c = [hi1 ^ c[1] ^ k[0], lo1, hi0 ^ c[3] ^ k[1], lo0]
        k = [(k[0] + 0x9E3779B9) & 0xFFFFFFFF, (k[1] + 0xBB67AE85) & 0xFFFFFFFF]
    return c


def test_philox_known_answers(golden_dir):
    rows = [l.split() for l in open(os.path.join(golden_dir, "philox4x32_10_kat.txt"))
            if l.strip() and not l.startswith("#")]
    assert len(rows) == 3
    for r in rows:
        vals = [int(x, 16) for x in r]
        got = oracle.philox4x32_10(vals[0:4], vals[4:6]).tolist()
        assert got == vals[6:10]
        assert _py_philox(vals[0:4], vals[4:6]) == vals[6:10]


def test_philox_matches_independent_implementation():
    rng = np.random.default_rng(7)
    for _ in range(200):
        ctr = rng.integers(0, 2**32, size=4, dtype=np.uint64)
        key = rng.integers(0, 2**32, size=2, dtype=np.uint64)
        assert oracle.philox4x32_10(ctr, key).tolist() == _py_philox(ctr, key)


def test_uniform_counter_mapping():
    seed = 0x1234_5678_9ABC_DEF0
    step = (0xABCDEF << 32) | 0x13572468
    key = [seed & 0xFFFFFFFF, seed >> 32]
    for b, i in [(0, 0), (3, 7), (255, 1)]:
        w = _py_philox([i, b, step & 0xFFFFFFFF, (((step >> 32) & 0xFFFFFF) << 8) | 0], key)
        assert oracle.u_accept(seed, step, b, i) == (w[0] >> 8) / 2.0**24
    for b, v in [(0, 0), (2, 5), (9, 128255), (1, 31999)]:
        w = _py_philox([v >> 2, b, step & 0xFFFFFFFF, (((step >> 32) & 0xFFFFFF) << 8) | 1], key)
        assert oracle.u_race(seed, step, b, v) == ((w[v & 3] >> 8) + 1) / 2.0**24


def test_uniform_ranges_and_moments():
    ua = np.array([oracle.u_accept(11, 5, b, i) for b in range(500) for i in range(8)])
    ur = np.array([oracle.u_race(11, 5, 0, v) for v in range(4000)])
    assert ua.min() >= 0.0 and ua.max() < 1.0
    assert ur.min() > 0.0 and ur.max() <= 1.0
    assert abs(ua.mean() - 0.5) < 4 * math.sqrt(1 / 12 / ua.size)
    assert abs(ur.mean() - 0.5) < 4 * math.sqrt(1 / 12 / ur.size)
    # distinct streams: the two families must not coincide
    assert oracle.u_accept(11, 5, 0, 0) != oracle.u_race(11, 5, 0, 0) - 2.0**-24


# --------------------------------------------------------------------------
# Attention
# --------------------------------------------------------------------------
def _decode(a):
    return W.bf16_bits_to_f32(a).astype(np.float64) if a.dtype == np.uint16 else a.astype(np.float64)


def _dense_attention(w):
    """Brute force: gather each request's K/V into dense [L,Hkv,d] arrays, build the
    explicit [q,L] visibility matrix, and evaluate softmax(QK^T/sqrt(d)+mask)V with
    whole-matrix numpy operations in float64."""
    out = np.zeros((w.T, w.Hq, w.d))
    G = w.Hq // w.Hkv
    kp, vp, qq = _decode(w.k_pages), _decode(w.v_pages), _decode(w.q)
    for b in range(w.B):
        L, ql = int(w.kv_len[b]), int(w.q_len[b])
        nblk = (L + w.block_size - 1) // w.block_size
        pages = w.block_table[b, :nblk]
        Kd = kp[pages].transpose(0, 2, 1, 3).reshape(nblk * w.block_size, w.Hkv, w.d)[:L]
        Vd = vp[pages].transpose(0, 2, 1, 3).reshape(nblk * w.block_size, w.Hkv, w.d)[:L]
        mask = np.full((ql, L), -np.inf)
        for j in range(ql):
            mask[j, : L - ql + j + 1] = 0.0
        Qb = qq[w.cu_q_len[b]: w.cu_q_len[b + 1]]                      # [ql,Hq,d]
        Kh = np.repeat(Kd, G, axis=1)                                   # [L,Hq,d]
        Vh = np.repeat(Vd, G, axis=1)
        S = np.einsum("jhc,thc->hjt", Qb, Kh) / math.sqrt(w.d) + mask[None]
        P = np.exp(S - S.max(axis=2, keepdims=True))
        P /= P.sum(axis=2, keepdims=True)
        out[w.cu_q_len[b]: w.cu_q_len[b + 1]] = np.einsum("hjt,thc->jhc", P, Vh)
    return out


def _small(dtype, B=3, Hq=4, Hkv=2, d=8, kv_len=(37, 16, 5), k=(3, 0, 4), seed=11):
    return W.make_workload("t", B=B, Hq=Hq, Hkv=Hkv, d=d, V=8, dtype=dtype, kv_len=kv_len, k=k,
                           draft_std=1.0, sigma=0.5, data_seed=seed, philox_seed=1)


def _attn(w, **kw):
    return oracle.verify_attn(w.q, w.k_pages, w.v_pages, w.block_table, w.kv_len, w.cu_q_len, **kw)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_attention_vs_dense_bruteforce(dtype):
    w = _small(dtype)
    np.testing.assert_allclose(_attn(w), _dense_attention(w), rtol=0, atol=2e-7)
    # a second shape: MHA, ragged tails, long enough to cross several pages
    w2 = _small(dtype, B=2, Hq=3, Hkv=3, d=16, kv_len=(70, 33), k=(8, 1), seed=5)
    np.testing.assert_allclose(_attn(w2), _dense_attention(w2), rtol=0, atol=2e-7)


def test_attention_k0_is_plain_decode():
    w = _small("f32", B=2, Hq=2, Hkv=2, d=8, kv_len=(21, 40), k=(0, 0))
    out = _attn(w)
    kp, vp = w.k_pages.astype(np.float64), w.v_pages.astype(np.float64)
    for b in range(2):
        L = int(w.kv_len[b])
        for h in range(2):
            keys = np.stack([kp[w.block_table[b, t // 16], h, t % 16] for t in range(L)])
            vals = np.stack([vp[w.block_table[b, t // 16], h, t % 16] for t in range(L)])
            s = keys @ w.q[b, h].astype(np.float64) / math.sqrt(8)
            p = np.exp(s - s.max())
            p /= p.sum()
            np.testing.assert_allclose(out[b, h], p @ vals, atol=2e-7)


def test_attention_block_table_permutation_invariance():
    w = _small("bf16")
    base = _attn(w)
    perm = np.random.default_rng(3).permutation(w.num_blocks)
    inv = np.argsort(perm)
    # page i moves to slot inv[i]; the table must follow
    k2 = w.k_pages[perm]
    v2 = w.v_pages[perm]
    bt2 = inv[w.block_table].astype(np.int32)
    out = oracle.verify_attn(w.q, k2, v2, bt2, w.kv_len, w.cu_q_len)
    np.testing.assert_array_equal(out, base)


def test_attention_causality_rows_equal_truncated_decode():
    w = _small("f32", B=1, Hq=4, Hkv=2, d=8, kv_len=(45,), k=(4,))
    full = _attn(w)
    for j in range(5):
        cu = np.array([0, 1], dtype=np.int32)
        out = oracle.verify_attn(w.q[j: j + 1], w.k_pages, w.v_pages, w.block_table,
                                 np.array([45 - 5 + j + 1], dtype=np.int32), cu)
        np.testing.assert_array_equal(out[0], full[j])


def test_attention_equal_keys_gives_mean_of_visible_values():
    w = _small("f32", B=1, Hq=2, Hkv=1, d=8, kv_len=(30,), k=(2,))
    w.k_pages[...] = 0.25
    out = _attn(w)
    vals = np.stack([w.v_pages[w.block_table[0, t // 16], 0, t % 16] for t in range(30)]).astype(np.float64)
    for j in range(3):
        mean = vals[: 30 - 3 + j + 1].mean(axis=0)
        for h in range(2):
            np.testing.assert_allclose(out[j, h], mean, atol=2e-7)


def test_attention_gqa_equals_mha_with_duplicated_kv_heads():
    w = _small("bf16", B=2, Hq=6, Hkv=2, d=8, kv_len=(19, 50), k=(1, 5))
    out = _attn(w)
    k_dup = np.repeat(w.k_pages, 3, axis=1)
    v_dup = np.repeat(w.v_pages, 3, axis=1)
    out2 = oracle.verify_attn(w.q, k_dup, v_dup, w.block_table, w.kv_len, w.cu_q_len)
    np.testing.assert_array_equal(out, out2)


def test_attention_scale_argument_and_tail_filler_ignored():
    w = _small("f32", B=1, Hq=2, Hkv=2, d=8, kv_len=(21,), k=(1,))
    a = _attn(w)
    b = _attn(w, scale=1 / math.sqrt(8))
    np.testing.assert_array_equal(a, b)
    c = _attn(w, scale=0.5)
    assert np.abs(a - c).max() > 1e-3
    # tail slots hold the filler; changing them must not matter
    w.k_pages[w.block_table[0, 1], :, 5:, :] = -777.0
    w.v_pages[w.block_table[0, 1], :, 5:, :] = 555.0
    np.testing.assert_array_equal(_attn(w), a)


def test_attention_c1_vs_torch_sdpa():
    torch = pytest.importorskip("torch")
    w = W.config("c1", with_logits=False)
    out = _attn(w)
    L, ql = 128, 5
    K = torch.from_numpy(w.k_pages.transpose(1, 0, 2, 3).reshape(8, 128, 64).copy()).double()
    Vv = torch.from_numpy(w.v_pages.transpose(1, 0, 2, 3).reshape(8, 128, 64).copy()).double()
    Q = torch.from_numpy(w.q.transpose(1, 0, 2).copy()).double()             # [H, ql, d]
    mask = torch.zeros(ql, L, dtype=torch.bool)
    for j in range(ql):
        mask[j, : L - ql + j + 1] = True
    ref = torch.nn.functional.scaled_dot_product_attention(Q[None], K[None], Vv[None], attn_mask=mask)[0]
    np.testing.assert_allclose(out, ref.permute(1, 0, 2).numpy(), atol=2e-7)


def test_attention_rejects_malformed():
    w = _small("f32")
    bad = w.block_table.copy()
    bad[0, 0] = w.num_blocks
    with pytest.raises(ValueError):
        oracle.verify_attn(w.q, w.k_pages, w.v_pages, bad, w.kv_len, w.cu_q_len)


# --------------------------------------------------------------------------
# Rejection sampling
# --------------------------------------------------------------------------
def _logits_of(prob):
    """fp32 logits whose softmax is `prob` (zero probability -> a logit so low that
    exp underflows to exactly 0 in double)."""
    prob = np.asarray(prob, dtype=np.float64)
    with np.errstate(divide="ignore"):
        lg = np.where(prob > 0, np.log(np.maximum(prob, 1e-300)), -1.0e4)
    return lg.astype(np.float32)


def _batch(p_rows, q_rows, tokens, k, B):
    """B identical requests: target rows p_rows [k+1,V], draft rows q_rows [k,V]."""
    V = len(p_rows[0])
    tl = np.tile(np.stack([_logits_of(p) for p in p_rows]), (B, 1))
    dl = np.tile(np.stack([_logits_of(q) for q in q_rows]), (B, 1)) if k else np.zeros((0, V), np.float32)
    cu = (np.arange(B + 1) * (k + 1)).astype(np.int32)
    return tl, dl, np.asarray(tokens, dtype=np.int32), cu


def test_softmax_row_matches_scipy():
    x = (np.random.default_rng(0).standard_normal(1000) * 5).astype(np.float32)
    np.testing.assert_allclose(oracle.softmax_row(x), scipy.special.softmax(x.astype(np.float64)), rtol=1e-13)
    assert abs(oracle.softmax_row(x).sum() - 1) < 1e-13


def test_accept_probability_closed_form():
    p = np.array([0.5, 0.2, 0.2, 0.1])
    q = np.array([0.1, 0.6, 0.2, 0.1])
    assert abs(oracle.accept_probability(_logits_of(p), _logits_of(q)) - 0.6) < 1e-7


def test_identical_draft_and_target_accepts_everything():
    w = W.make_workload("t", B=40, Hq=1, Hkv=1, d=8, V=50, dtype="f32", kv_len=[16] * 40,
                        k=list(np.arange(40) % (K_MAX + 1)), draft_std=2.0, sigma=0.0, data_seed=3,
                        philox_seed=9, with_kv=False)
    r = oracle.reject_sample(w.target_logits, w.draft_logits, w.draft_tokens, w.cu_q_len, 9, 0)
    np.testing.assert_array_equal(r.accepted_len, w.k)
    ev = ~np.isnan(r.dec_ratio)
    assert ev.all() and np.allclose(r.dec_ratio, 1.0, atol=1e-12)
    assert r.counters[0] == r.counters[1] == r.counters[2] == w.k.sum()
    assert r.counters[3] == w.k.sum() + 40 and r.counters[5] == 40
    for b in range(40):
        kb = int(w.k[b])
        row = r.out_tokens[b]
        d0 = int(w.cu_q_len[b]) - b
        assert row[:kb].tolist() == w.draft_tokens[d0: d0 + kb].tolist()
        assert row[kb] == r.next_token[b] and (row[kb + 1:] == -1).all()


def test_worked_example_probabilities(golden_dir):
    g = dict(l.split() for l in open(os.path.join(golden_dir, "worked_example_sec3.txt"))
             if l.strip() and not l.startswith("#"))
    alpha, k = float(g["alpha"]), int(g["k"])
    want = [float(g["prob_emitted_%d" % n]) for n in (1, 2, 3)]
    lat = [float(g["latency_ms_%d" % n]) for n in (1, 2, 3)]
    # the paper's own arithmetic
    assert abs(sum(p * t for p, t in zip(want, lat)) - float(g["expected_latency_ms"])) < 0.005
    assert abs(oracle.expected_generated_len(alpha, k) - float(g["expected_generated_len"])) < 1e-12
    # a draft that always proposes token 0 against a target with p(0) = alpha:
    # each accept test passes with probability exactly alpha
    B = 60000
    tl, dl, tok, cu = _batch([[alpha, 1 - alpha]] * (k + 1), [[1.0, 0.0]] * k, [0] * (k * B), k, B)
    r = oracle.reject_sample(tl, dl, tok, cu, 2024, 1)
    freq = np.bincount(r.accepted_len, minlength=k + 1) / B
    for f, p in zip(freq, want):
        assert abs(f - p) < 4.5 * math.sqrt(p * (1 - p) / B)
    assert abs(r.counters[3] / B - float(g["expected_generated_len"])) < 4.5 * 0.87 / math.sqrt(B)


@pytest.mark.parametrize("alpha", [0.5, 0.7, 0.9])
def test_mean_generated_length_matches_eq4(alpha):
    B = 20000
    for k in range(0, K_MAX + 1):
        tl, dl, tok, cu = _batch([[alpha, 1 - alpha]] * (k + 1), [[1.0, 0.0]] * k, [0] * (k * B), k, B)
        r = oracle.reject_sample(tl, dl, tok, cu, 77, k)
        closed = sum(alpha ** j for j in range(k + 1))
        assert abs(oracle.expected_generated_len(alpha, k) - closed) < 1e-12
        sd = math.sqrt(max(np.var(r.accepted_len), 1e-12))
        assert abs(r.counters[3] / B - closed) < 4.5 * sd / math.sqrt(B) + 1e-12
        assert (r.accepted_len >= 0).all() and (r.accepted_len <= k).all()


def test_non_iid_generated_length():
    # per-position acceptance probabilities 0.9, 0.5, 0.2: E[emitted] = 1 + 0.9 + 0.45 + 0.09
    alphas = [0.9, 0.5, 0.2]
    B = 50000
    tl, dl, tok, cu = _batch([[a, 1 - a] for a in alphas] + [[0.5, 0.5]], [[1.0, 0.0]] * 3, [0] * (3 * B), 3, B)
    r = oracle.reject_sample(tl, dl, tok, cu, 5, 0)
    want = 1 + 0.9 + 0.45 + 0.09
    assert abs(r.counters[3] / B - want) < 4.5 * math.sqrt(np.var(r.accepted_len) / B)


def test_accept_frequency_matches_sum_min_p_q():
    p = np.array([0.05, 0.30, 0.10, 0.25, 0.05, 0.25])
    q = np.array([0.30, 0.05, 0.20, 0.25, 0.15, 0.05])
    alpha = np.minimum(p, q).sum()
    B = 80000
    tokens = np.random.default_rng(8).choice(6, size=B, p=q)
    tl, dl, _, cu = _batch([p, p], [q], [], 1, B)
    r = oracle.reject_sample(tl, dl, tokens.astype(np.int32), cu, 31, 2)
    assert abs(r.accepted_len.mean() - alpha) < 4.5 * math.sqrt(alpha * (1 - alpha) / B)
    assert abs(oracle.accept_probability(_logits_of(p), _logits_of(q)) - alpha) < 1e-7
    # per-token: P(accept | x) = min(1, p_x/q_x)
    for x in range(6):
        sel = tokens == x
        want = min(1.0, p[x] / q[x])
        assert abs(r.accepted_len[sel].mean() - want) < 4.5 * math.sqrt(max(want * (1 - want), 1e-4) / sel.sum())


def test_first_emitted_token_is_distributed_as_target():
    """Losslessness (Section 2.2): with x ~ q, the first emitted token ~ p exactly."""
    p = np.array([0.02, 0.30, 0.10, 0.20, 0.05, 0.25, 0.08, 0.0])
    q = np.array([0.25, 0.05, 0.20, 0.20, 0.15, 0.05, 0.0, 0.10])
    B = 200000
    tokens = np.random.default_rng(12).choice(8, size=B, p=q)
    tl, dl, _, cu = _batch([p, [0.125] * 8], [q], [], 1, B)
    r = oracle.reject_sample(tl, dl, tokens.astype(np.int32), cu, 99, 3)
    first = r.out_tokens[:, 0]
    counts = np.bincount(first, minlength=8)
    assert counts[7] == 0                      # zero-probability token never emitted
    chi = scipy.stats.chisquare(counts[:7], B * p[:7])
    assert chi.pvalue > 1e-3
    # correction token, conditioned on rejection, ~ normalised max(0, p - q)
    rej = r.accepted_len == 0
    res = np.maximum(p - q, 0)
    res /= res.sum()
    cc = np.bincount(r.next_token[rej], minlength=8)
    assert (cc[res == 0] == 0).all()
    chi2 = scipy.stats.chisquare(cc[res > 0], rej.sum() * res[res > 0])
    assert chi2.pvalue > 1e-3
    # bonus token after full acceptance ~ last target row (uniform here)
    acc = ~rej
    cb = np.bincount(r.next_token[acc], minlength=8)
    chi3 = scipy.stats.chisquare(cb, acc.sum() * np.full(8, 0.125))
    assert chi3.pvalue > 1e-3


def test_k0_samples_from_target_row():
    p = np.array([0.4, 0.1, 0.0, 0.2, 0.3])
    B = 100000
    tl, dl, tok, cu = _batch([p], [], [], 0, B)
    r = oracle.reject_sample(tl, dl, tok, cu, 4, 4)
    assert (r.accepted_len == 0).all()
    counts = np.bincount(r.next_token, minlength=5)
    assert counts[2] == 0
    assert scipy.stats.chisquare(counts[[0, 1, 3, 4]], B * p[[0, 1, 3, 4]]).pvalue > 1e-3
    assert r.counters[:4].tolist() == [0, 0, 0, B]


def test_one_hot_target_reduces_to_argmax():
    V = 16
    for hot in (0, 7, 15):
        p = np.zeros(V)
        p[hot] = 1.0
        q = np.full(V, 1 / V)
        B = 64
        tokens = (np.arange(B) % V).astype(np.int32)
        tl, dl, _, cu = _batch([p, p], [q], [], 1, B)
        r = oracle.reject_sample(tl, dl, tokens, cu, 1, 0)
        # accepted iff the draft token is the arg-max; the first emitted token is always the arg-max
        np.testing.assert_array_equal(r.accepted_len, (tokens == hot).astype(np.int32))
        assert (r.out_tokens[:, 0] == hot).all()
        assert (r.next_token == hot).all()


def test_decision_follows_recorded_u_and_ratio():
    w = W.make_workload("t", B=64, Hq=1, Hkv=1, d=8, V=200, dtype="f32", kv_len=[16] * 64,
                        k=[5] * 64, draft_std=2.0, sigma=1.0, data_seed=21, philox_seed=6, with_kv=False)
    r = oracle.reject_sample(w.target_logits, w.draft_logits, w.draft_tokens, w.cu_q_len, 6, 11)
    for b in range(64):
        m = int(r.accepted_len[b])
        u = r.dec_u[b * 5: b * 5 + 5]
        ratio = r.dec_ratio[b * 5: b * 5 + 5]
        assert (u[:m] < ratio[:m]).all()
        if m < 5:
            assert u[m] >= ratio[m]
            assert np.isnan(u[m + 1:]).all()
        for i in range(min(m + 1, 5)):
            assert u[i] == oracle.u_accept(6, 11, b, i)
            x = int(w.draft_tokens[b * 5 + i])
            pt = scipy.special.softmax(w.target_logits[b * 6 + i].astype(np.float64))
            qd = scipy.special.softmax(w.draft_logits[b * 5 + i].astype(np.float64))
            assert abs(ratio[i] - pt[x] / qd[x]) <= 1e-12 * ratio[i]
    c = r.counters
    assert c[3] == c[1] + 64 and c[1] <= c[2] <= c[0] == 64 * 5
    assert c[1] == r.accepted_len.sum()
    assert c[2] == np.minimum(r.accepted_len + 1, 5).sum()


def test_race_winner_recomputed_in_python():
    """The next token is arg max r_v / (-log U'_v); recompute it from the definition."""
    w = W.make_workload("t", B=12, Hq=1, Hkv=1, d=8, V=300, dtype="f32", kv_len=[16] * 12,
                        k=[2] * 12, draft_std=2.0, sigma=1.0, data_seed=33, philox_seed=8, with_kv=False)
    r = oracle.reject_sample(w.target_logits, w.draft_logits, w.draft_tokens, w.cu_q_len, 8, 2)
    for b in range(12):
        m = int(r.accepted_len[b])
        p = scipy.special.softmax(w.target_logits[b * 3 + m].astype(np.float64))
        if m < 2:
            qd = scipy.special.softmax(w.draft_logits[b * 2 + m].astype(np.float64))
            wgt = np.maximum(p - qd, 0)
        else:
            wgt = p
        e = np.array([-math.log(oracle.u_race(8, 2, b, v)) for v in range(300)])
        score = wgt / e
        assert int(np.argmax(score)) == r.next_token[b]
        srt = np.sort(score)
        assert r.race_margin[b] > 0
        # the margin is a lower bound of the plain relative gap between best and runner-up
        assert r.race_margin[b] <= (srt[-1] - srt[-2]) / srt[-1] + 1e-15


def _race_e(seed, step, b, V):
    return np.array([-math.log(oracle.u_race(seed, step, b, v)) for v in range(V)])


@pytest.mark.parametrize("delta", [1e-3, 2e-5, 0.25])
def test_race_margin_equals_a_constructed_relative_gap(delta):
    """Bonus row (k = 0, weights r = p): logits are built so that the two best race scores are
    proportional to 1 + delta and 1 - delta and every other score is a tenth of that.  The margin
    (smallest relative perturbation of the weights that can change the winner) is then delta by
    construction: (s_a - s_b) / (s_a + s_b) = delta, every other pair being far apart."""
    V, seed, step = 8, 77, 5
    for b in range(3):
        e = _race_e(seed, step, b, V)
        want = np.full(V, 0.1)
        a, c = (2 + b) % V, (5 + b) % V
        want[a], want[c] = 1.0 + delta, 1.0 - delta
        logits = np.log(want * e).astype(np.float32)[None, :]         # p_v / e_v proportional to want_v
        tl = np.tile(logits, (b + 1, 1))                              # B = b + 1 requests of one bonus row each
        cu = np.arange(b + 2, dtype=np.int32)
        r = oracle.reject_sample(tl, np.zeros((0, V), np.float32), np.zeros(0, np.int32), cu, seed, step)
        assert r.next_token[b] == a
        # fp32 logits move each score by a relative 1e-7 at most
        assert abs(r.race_margin[b] - delta) < 4e-7, (r.race_margin[b], delta)


def test_race_margin_is_the_flipping_threshold_of_a_correction_row():
    """Correction row (weights max(0, p - q)): perturb every p and q by a relative eps in the
    direction that hurts the winner most (winner: p down, q up; challenger: p up, q down).
    Just below the reported margin the winner must survive against every id, just above it some
    id must overtake: that is what "smallest relative perturbation that can change the winner"
    means, recomputed here by brute force from scipy's softmax."""
    V, seed, step = 40, 91, 3
    rng = np.random.default_rng(5)
    checked = 0
    for trial in range(30):
        tl = (rng.standard_normal((2, V)) * 2).astype(np.float32)
        dl = (rng.standard_normal((1, V)) * 2).astype(np.float32)
        x = int(np.argmin(tl[0] - dl[0]))            # the token the target likes least relative to the draft
        tl[0, x] -= 30.0                             # p(x)/q(x) ~ e^-30: rejected whatever u is
        r = oracle.reject_sample(tl, dl, np.array([x], np.int32), np.array([0, 2], np.int32), seed, step + trial)
        assert r.accepted_len[0] == 0
        p = scipy.special.softmax(tl[0].astype(np.float64))
        q = scipy.special.softmax(dl[0].astype(np.float64))
        e = _race_e(seed, step + trial, 0, V)
        best = int(r.next_token[0])
        mg = float(r.race_margin[0])
        assert mg > 0

        def winner_survives(eps):
            s_best = (p[best] * (1 - eps) - q[best] * (1 + eps)) / e[best]
            others = (p * (1 + eps) - q * (1 - eps)) / e
            others[best] = -np.inf
            return bool((others < s_best).all())

        assert winner_survives(mg * (1 - 1e-6))
        assert not winner_survives(mg * (1 + 1e-6))
        checked += 1
    assert checked == 30


def _near_tie_case(eps, seed=12, step=(3 << 32) + 9, b=2, i=1, V=8):
    """B = b + 1 requests with k = i + 1 draft tokens each; every accept test but (b, i) has
    p/q = 1 + something large (always accepted); test (b, i) has p(x)/q(x) = u + eps where u is
    the uniform that test will draw.  Draft rows are flat (q = 1/V); the target row of the
    constructed test has logit t at x and 0 elsewhere: p(x) = e^t / (e^t + V - 1)."""
    B, k = b + 1, i + 1
    u = oracle.u_accept(seed, step, b, i)
    tl = np.zeros((B * (k + 1), V), np.float32)
    dl = np.zeros((B * k, V), np.float32)
    tok = np.full(B * k, 3, np.int32)
    tl[:, 3] = 4.0                                    # p(3) > 1/V: ratio > 1, always accepted
    ratio = u + eps
    t = math.log((V - 1) * ratio / (V - ratio))       # V e^t / (e^t + V - 1) = ratio
    row = b * (k + 1) + i
    tl[row, :] = 0.0
    tl[row, 3] = np.float32(t)
    cu = (np.arange(B + 1) * (k + 1)).astype(np.int32)
    return tl, dl, tok, cu, seed, step, u, B, k


@pytest.mark.parametrize("eps,accepted,near", [(4e-7, True, 1), (-4e-7, False, 1), (5e-6, True, 0), (-5e-6, False, 0)])
def test_near_tie_counter_on_a_constructed_accept_test(eps, accepted, near):
    """counters[4] counts the evaluated accept tests with |u - p/q| < 1e-6.  One test is built to
    sit eps away from its uniform (the uniform comes from the pinned Philox mapping); the counter
    must be 1 inside the window and 0 outside, and the decision must follow the sign of eps."""
    tl, dl, tok, cu, seed, step, u, B, k = _near_tie_case(eps)
    assert 1e-3 < u < 1 - 1e-3      # the constructed ratio is a valid probability ratio below 1
    r = oracle.reject_sample(tl, dl, tok, cu, seed, step)
    b, i = B - 1, k - 1
    assert r.counters[4] == near
    assert r.accepted_len[b] == (k if accepted else i)
    assert (r.accepted_len[:b] == k).all()
    got_ratio = r.dec_ratio[b * k + i]
    assert abs(got_ratio - (u + eps)) < 5e-8          # fp32 rounding of the one logit
    assert r.dec_u[b * k + i] == u


def test_counters_accumulate():
    w = W.make_workload("t", B=8, Hq=1, Hkv=1, d=8, V=64, dtype="f32", kv_len=[16] * 8,
                        k=[3] * 8, draft_std=2.0, sigma=1.0, data_seed=2, philox_seed=1, with_kv=False)
    r1 = oracle.reject_sample(w.target_logits, w.draft_logits, w.draft_tokens, w.cu_q_len, 1, 0)
    r2 = oracle.reject_sample(w.target_logits, w.draft_logits, w.draft_tokens, w.cu_q_len, 1, 0, counters=r1.counters)
    np.testing.assert_array_equal(r2.counters, 2 * r1.counters)


def test_synthetic_acceptance_levels_hit_their_targets():
    """The stored noise levels give the acceptance rates the named workloads ask for."""
    for (V, s), table in W.SIGMA_FOR_ALPHA.items():
        if V > 40000:
            continue
        for alpha, sigma in table.items():
            rng = np.random.default_rng(4321)
            d = rng.standard_normal((6, V), dtype=np.float32) * np.float32(s)
            t = d + rng.standard_normal((6, V), dtype=np.float32) * np.float32(sigma)
            got = np.mean([oracle.accept_probability(t[i], d[i]) for i in range(6)])
            assert abs(got - alpha) < 0.04


# ---------------------------------------------------------------------------
# Greedy acceptance and acceptance against a point-mass draft (proposers that
# give tokens but no distribution): Section 2.2 and Section 7 of the paper.
# ---------------------------------------------------------------------------
def _ragged_logits(seed, B, V, ks):
    rng = np.random.default_rng(seed)
    cu = np.concatenate([[0], np.cumsum(np.asarray(ks) + 1)]).astype(np.int32)
    tl = (rng.standard_normal((int(cu[-1]), V)) * 3).astype(np.float32)
    return rng, tl, cu


def test_greedy_matches_numpy_argmax_walk():
    """Brute force: leading run of draft tokens equal to the row arg-max, then that row's arg-max."""
    B, V = 200, 37
    ks = np.arange(B) % (K_MAX + 1)
    rng, tl, cu = _ragged_logits(21, B, V, ks)
    am = tl.argmax(axis=1)
    toks = []
    for b in range(B):
        row0 = cu[b]
        for i in range(ks[b]):
            # mostly the arg-max (so that runs of several accepts occur), sometimes another token
            toks.append(am[row0 + i] if rng.random() < 0.7 else rng.integers(V))
    toks = np.asarray(toks, dtype=np.int32)
    r = oracle.reject_greedy(tl, toks, cu)
    for b in range(B):
        row0, d0 = cu[b], cu[b] - b
        m = 0
        while m < ks[b] and toks[d0 + m] == am[row0 + m]:
            m += 1
        assert r.accepted_len[b] == m
        assert r.next_token[b] == am[row0 + m]
        want = list(toks[d0:d0 + m]) + [am[row0 + m]] + [-1] * (K_MAX - m)
        assert r.out_tokens[b].tolist() == want
    assert r.counters[0] == ks.sum() and r.counters[1] == r.accepted_len.sum()
    assert r.counters[3] == r.accepted_len.sum() + B and r.counters[5] == B and r.counters[4] == 0


def test_greedy_ties_take_the_lowest_id():
    tl = np.zeros((2, 8), dtype=np.float32)
    tl[0, [3, 5]] = 2.0        # two equal maxima: id 3 is the maximiser
    tl[1, [6, 1]] = 1.0
    cu = np.array([0, 2], dtype=np.int32)
    r = oracle.reject_greedy(tl, np.array([5], dtype=np.int32), cu)
    assert r.accepted_len[0] == 0 and r.next_token[0] == 3
    r = oracle.reject_greedy(tl, np.array([3], dtype=np.int32), cu)
    assert r.accepted_len[0] == 1 and r.next_token[0] == 1


def test_greedy_equals_stochastic_rule_on_one_hot_target():
    """A one-hot target makes the stochastic rule deterministic: the two rules agree."""
    B, V, k = 50, 12, 3
    rng = np.random.default_rng(5)
    hot = rng.integers(V, size=B * (k + 1))
    p = np.zeros((B * (k + 1), V))
    p[np.arange(B * (k + 1)), hot] = 1.0
    tl = np.stack([_logits_of(row) for row in p])
    q = np.full(V, 1.0 / V)
    dl = np.tile(_logits_of(q), (B * k, 1))
    cu = (np.arange(B + 1) * (k + 1)).astype(np.int32)
    toks = np.where(rng.random(B * k) < 0.6, hot.reshape(B, k + 1)[:, :k].reshape(-1), rng.integers(V, size=B * k)).astype(np.int32)
    g = oracle.reject_greedy(tl, toks, cu)
    s = oracle.reject_sample(tl, dl, toks, cu, 3, 1)
    np.testing.assert_array_equal(g.accepted_len, s.accepted_len)
    np.testing.assert_array_equal(g.next_token, s.next_token)
    np.testing.assert_array_equal(g.out_tokens, s.out_tokens)


def test_onehot_draft_equals_general_rule_with_point_mass_logits():
    """The general rule fed draft logits that ARE a point mass gives the same decisions and tokens."""
    B, V = 120, 40
    ks = np.arange(B) % (K_MAX + 1)
    rng, tl, cu = _ragged_logits(33, B, V, ks)
    T = int(cu[-1])
    toks = rng.integers(V, size=T - B).astype(np.int32)
    dl = np.full((T - B, V), -1.0e4, dtype=np.float32)     # exp underflows to exactly 0 in double
    dl[np.arange(T - B), toks] = 0.0
    a = oracle.reject_onehot(tl, toks, cu, 77, 5)
    b = oracle.reject_sample(tl, dl, toks, cu, 77, 5)
    np.testing.assert_array_equal(a.accepted_len, b.accepted_len)
    np.testing.assert_array_equal(a.next_token, b.next_token)
    np.testing.assert_array_equal(a.out_tokens, b.out_tokens)
    np.testing.assert_array_equal(a.counters, b.counters)
    ev = ~np.isnan(a.dec_u)
    np.testing.assert_array_equal(ev, ~np.isnan(b.dec_u))
    np.testing.assert_allclose(a.dec_ratio[ev], b.dec_ratio[ev], rtol=1e-12)


def test_onehot_draft_is_lossless_and_accepts_with_probability_p_x():
    """Any fixed proposal x: P(accept) = p(x), and the first emitted token ~ p exactly."""
    p = np.array([0.05, 0.35, 0.10, 0.20, 0.0, 0.30])
    B = 150000
    x = 3
    tl, _, _, cu = _batch([p, [1 / 6] * 6], [p], [], 1, B)
    toks = np.full(B, x, dtype=np.int32)
    r = oracle.reject_onehot(tl, toks, cu, 1234, 0)
    acc = r.accepted_len.mean()
    assert abs(acc - p[x]) < 4.5 * math.sqrt(p[x] * (1 - p[x]) / B)
    counts = np.bincount(r.out_tokens[:, 0], minlength=6)
    assert counts[4] == 0
    keep = p > 0
    assert scipy.stats.chisquare(counts[keep], B * p[keep]).pvalue > 1e-3
    # the correction never repeats the rejected token and is ~ p without x
    rej = r.accepted_len == 0
    cc = np.bincount(r.next_token[rej], minlength=6)
    assert cc[x] == 0
    res = p.copy(); res[x] = 0; res /= res.sum()
    assert scipy.stats.chisquare(cc[res > 0], rej.sum() * res[res > 0]).pvalue > 1e-3


# ---------------------------------------------------------------------------
# KV append and the bookkeeping after acceptance (Section 5.1 of the paper).
# ---------------------------------------------------------------------------
def _append_case(dtype):
    return W.make_workload("app", B=4, Hq=4, Hkv=2, d=64 if dtype == "f32" else 128, V=8, dtype=dtype,
                           kv_len=[37, 16, 300, 5], k=[3, 0, 8, 4], draft_std=1.0, sigma=1.0, data_seed=77,
                           philox_seed=1, with_logits=False)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_kv_append_token_major_restores_erased_rows(dtype):
    """Erase the last q_len tokens of every request from the pools, append them again from a
    packed [T,Hkv,d] array: the pools, and the attention output, are what they were."""
    w = _append_case(dtype)
    T = w.T
    new_k = np.zeros((T, w.Hkv, w.d), dtype=w.k_pages.dtype)
    new_v = np.zeros_like(new_k)
    kc, vc = w.k_pages.copy(), w.v_pages.copy()
    for b in range(w.B):
        for j in range(int(w.q_len[b])):
            pos = int(w.kv_len[b]) - int(w.q_len[b]) + j
            page, slot = int(w.block_table[b, pos // 16]), pos % 16
            new_k[w.cu_q_len[b] + j] = kc[page, :, slot, :]
            new_v[w.cu_q_len[b] + j] = vc[page, :, slot, :]
            kc[page, :, slot, :] = 0
            vc[page, :, slot, :] = 0
    assert not np.array_equal(kc, w.k_pages)
    k2, v2 = oracle.kv_append(new_k, new_v, kc, vc, w.block_table, w.kv_len, w.cu_q_len, layout=0)
    np.testing.assert_array_equal(k2, w.k_pages)
    np.testing.assert_array_equal(v2, w.v_pages)
    np.testing.assert_array_equal(kc[kc != 0], kc[kc != 0])     # inputs were copied, not written
    a = oracle.verify_attn(w.q, k2, v2, w.block_table, w.kv_len, w.cu_q_len)
    b = oracle.verify_attn(w.q, w.k_pages, w.v_pages, w.block_table, w.kv_len, w.cu_q_len)
    np.testing.assert_array_equal(a, b)


def test_kv_append_tiled_layout_offsets():
    """The matrix-operand layout, checked against offsets worked out by hand from its definition
    (K: [d/8][16 tokens][8 dims]; V: [d/32][4 token groups][16 dims][2 dim halves][4 tokens])."""
    B, Hkv, d = 1, 1, 128
    cu = np.array([0, 1], dtype=np.int32)
    bt = np.array([[0]], dtype=np.int32)
    seen_k, seen_v = set(), set()
    hand = {  # (slot, dim) -> (K offset, V offset)
        (0, 0): (0, 0),
        (3, 9): (1 * 128 + 3 * 8 + 1, (((0 * 4 + 0) * 16 + 9) * 2 + 0) * 4 + 3),
        (7, 16): (2 * 128 + 7 * 8 + 0, (((0 * 4 + 1) * 16 + 0) * 2 + 1) * 4 + 3),
        (15, 127): (15 * 128 + 15 * 8 + 7, (((3 * 4 + 3) * 16 + 15) * 2 + 1) * 4 + 3),
        (5, 40): (5 * 128 + 5 * 8 + 0, (((1 * 4 + 1) * 16 + 8) * 2 + 0) * 4 + 1),
    }
    for slot in range(16):
        row_k = (np.arange(d) + 1 + 200 * slot).astype(np.uint16)       # distinct non-zero values
        row_v = (np.arange(d) + 1 + 200 * slot + 5000).astype(np.uint16)
        kc = np.zeros(16 * d, dtype=np.uint16)
        vc = np.zeros(16 * d, dtype=np.uint16)
        k2, v2 = oracle.kv_append(row_k.reshape(1, 1, d), row_v.reshape(1, 1, d), kc, vc, bt,
                                  np.array([slot + 1], dtype=np.int32), cu, layout=1)
        assert np.count_nonzero(k2) == d and np.count_nonzero(v2) == d
        for c in range(d):
            ok = int(np.nonzero(k2 == row_k[c])[0][0])
            ov = int(np.nonzero(v2 == row_v[c])[0][0])
            seen_k.add(ok)
            seen_v.add(ov)
            if (slot, c) in hand:
                assert (ok, ov) == hand[(slot, c)], (slot, c, ok, ov)
    assert seen_k == set(range(16 * d)) and seen_v == set(range(16 * d))     # a bijection onto the 4 KB


def test_kv_bookkeeping_after_accept():
    kv = np.array([100, 50, 33, 20], dtype=np.int32)
    cu = np.array([0, 3, 6, 7, 12], dtype=np.int32)     # k = 2, 2, 0, 4
    acc = np.array([2, 0, 0, 3], dtype=np.int32)
    new_len, draft_next = oracle.kv_after_accept(kv, cu, acc)
    # Section 5.1's example (k = 2): all accepted -> nothing dropped, the draft model is two tokens
    # behind; a rejection -> the rejected tail is dropped and it is one behind
    assert new_len.tolist() == [100, 48, 33, 19]
    assert draft_next.tolist() == [2, 1, 1, 1]
