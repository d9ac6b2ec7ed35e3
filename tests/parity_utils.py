"""Comparison of the HIP library's results with the CPU oracle on the same inputs."""
import numpy as np

import oracle

ATTN_TOL = {"f32": 1e-5, "bf16": 2e-3}      # max abs error of the attention output
ACCEPT_NEAR_TIE = 1e-6                      # |u - p/q| below this: either decision is legitimate
RACE_NEAR_TIE = 1e-5                        # oracle race margin below this: either winner is legitimate


def oracle_attn(w, requests=None):
    """Oracle attention for all requests, or for the listed ones (rows returned packed in that order)."""
    if requests is None:
        return oracle.verify_attn(w.q, w.k_pages, w.v_pages, w.block_table, w.kv_len, w.cu_q_len), np.arange(w.T)
    rows = np.concatenate([np.arange(w.cu_q_len[b], w.cu_q_len[b + 1]) for b in requests])
    q_len = np.array([w.q_len[b] for b in requests], dtype=np.int32)
    cu = np.concatenate([[0], np.cumsum(q_len)]).astype(np.int32)
    out = oracle.verify_attn(np.ascontiguousarray(w.q[rows]), w.k_pages, w.v_pages,
                             np.ascontiguousarray(w.block_table[requests]),
                             np.ascontiguousarray(w.kv_len[requests]), cu)
    return out, rows


def check_attn(w, got, requests=None):
    ref, rows = oracle_attn(w, requests)
    err = float(np.abs(got[rows].astype(np.float64) - ref.astype(np.float64)).max())
    assert np.isfinite(got).all()
    assert err <= ATTN_TOL[w.dtype], "attention max abs error %.3e > %.1e" % (err, ATTN_TOL[w.dtype])
    return err


def oracle_reject(w):
    return oracle.reject_sample(w.target_logits, w.draft_logits, w.draft_tokens, w.cu_q_len,
                                w.philox_seed, w.philox_step)


def check_reject(w, res, ref=None, max_excluded=0, input_errors=0):
    """Bit-exact accepted lengths and tokens for every request whose decisions are not
    near-ties.  A request is excluded from the bit-exact comparison if one of its evaluated
    accept tests has |u - p/q| < 1e-6 (the benchmark spec's category) or if the oracle's race
    margin is below 1e-5 (this build's category for the next-token draw); excluded requests must
    still hold a valid outcome.  At most ``max_excluded`` requests may be excluded (0 unless a
    test says otherwise), so the comparison cannot become vacuous; the counts are returned."""
    ref = ref or oracle_reject(w)
    B = w.B
    near_accept = np.zeros(B, dtype=bool)
    near_race = np.zeros(B, dtype=bool)
    for b in range(B):
        d0 = int(w.cu_q_len[b]) - b
        kb = int(w.q_len[b]) - 1
        u, ratio = ref.dec_u[d0: d0 + kb], ref.dec_ratio[d0: d0 + kb]
        ev = ~np.isnan(u)
        near_accept[b] = bool(np.any(np.abs(u[ev] - ratio[ev]) < ACCEPT_NEAR_TIE))
        near_race[b] = bool(ref.race_margin[b] < RACE_NEAR_TIE)
    near = near_accept | near_race
    assert int(near.sum()) <= max_excluded, (
        "%d requests excluded from the bit-exact comparison (accept near ties %d, race near ties %d), allowed %d"
        % (near.sum(), near_accept.sum(), near_race.sum(), max_excluded))
    ok = ~near
    np.testing.assert_array_equal(res["accepted_len"][ok], ref.accepted_len[ok])
    np.testing.assert_array_equal(res["next_token"][ok], ref.next_token[ok])
    np.testing.assert_array_equal(res["out_tokens"][ok], ref.out_tokens[ok])
    # whatever was decided must be a valid outcome
    assert (res["accepted_len"] >= 0).all() and (res["accepted_len"] <= w.q_len - 1).all()
    assert (res["next_token"] >= 0).all() and (res["next_token"] < w.V).all()
    c = res["counters"]
    assert c[0] == ref.counters[0] and c[5] == ref.counters[5]
    assert c[1] == res["accepted_len"].sum() and c[3] == c[1] + B
    assert c[2] == np.minimum(res["accepted_len"] + 1, w.q_len - 1).sum()
    assert c[6] == input_errors and c[7] == 0, c   # findings of the device-side input checks, abandoned requests
    if not near.any():
        np.testing.assert_array_equal(c[:4], ref.counters[:4])
    # the recorded u and p/q of every evaluated accept test
    if res.get("debug") is not None and w.T > w.B:
        gu, gr = res["debug"][:, 0], res["debug"][:, 1]
        rows_ok = np.concatenate([np.arange(int(w.cu_q_len[b]) - b, int(w.cu_q_len[b + 1]) - b - 1)
                                  for b in range(B) if ok[b]] or [np.zeros(0, dtype=np.int64)]).astype(np.int64)
        ev = ~np.isnan(ref.dec_u[rows_ok])
        assert (np.isnan(gu[rows_ok]) == ~ev).all()
        np.testing.assert_array_equal(gu[rows_ok][ev], ref.dec_u[rows_ok][ev])
        rr = ref.dec_ratio[rows_ok][ev]
        fin = np.isfinite(rr) & (rr > 0)
        rel = np.abs(gr[rows_ok][ev][fin] - rr[fin]) / rr[fin]
        assert rel.size == 0 or rel.max() < 1e-6, "p/q relative error %.3e" % rel.max()
    # the library's own near-tie counter (evaluated accept tests within 1e-6 of their uniform)
    if not near_accept.any():
        assert c[4] == ref.counters[4] == 0
    return dict(near_ties=int(near.sum()), near_accept=int(near_accept.sum()), near_race=int(near_race.sum()),
                excluded=int(near.sum()), min_race_margin=float(ref.race_margin.min()), ref=ref)
