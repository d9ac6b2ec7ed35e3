"""The closed loop of the paper's listing "Generate": propose k -> append -> verify -> counters ->
acceptance estimate -> search for the next k, run for consecutive steps on the GPU.  At every step the
controller's choice is compared with the plain reference of the control equations
(oracle/goodput_oracle.py) fed the same counters, the step's decisions with the rejection-sampling
oracle on the step's own inputs, and the cache bookkeeping with the oracle's."""
import numpy as np
import pytest

import oracle
from oracle import goodput_oracle as G
from paper_2406_14066_amd import spec_verify as sv

pytestmark = pytest.mark.gpu


def _run(sigma, steps, target, draft, B=8, seed=5):
    import torch
    from paper_2406_14066_amd.control_loop import ControlLoop
    loop = ControlLoop(B, 100, Hq=8, Hkv=2, d=128, V=4096, sigma=sigma, max_kv_len=512, target=target, draft=draft,
                       decay=0.8, prior=0.6, seed=seed)
    t_tuple = (target.c_context, target.c_batched, target.c_fixed)
    d_tuple = (draft.c_context, draft.c_batched, draft.c_fixed)
    history = []
    kept = np.full(B, 100, dtype=np.int32)
    ks = []
    # the first choice: the prior
    assert loop.k == G.argmax_goodput(kept.tolist(), [0.6], sv.K_MAX, t_tuple, d_tuple)
    for step in range(steps):
        k = loop.k
        ks.append(k)
        rec = loop.run_step()
        assert rec["k"] == k and rec["input_errors"] == 0 and rec["abandoned"] == 0
        T = B * (k + 1)
        cu = (np.arange(B + 1) * (k + 1)).astype(np.int32)
        # the step's decisions against the oracle on the step's own inputs
        tl = loop.target_logits[:T].cpu().numpy()
        dl = loop.draft_logits[: T - B].cpu().numpy() if k else np.zeros((0, loop.V), np.float32)
        tok = loop.draft_tokens[: T - B].cpu().numpy() if k else np.zeros(0, np.int32)
        ref = oracle.reject_sample(tl, dl, tok, cu, loop.seed, step)
        with np.errstate(invalid="ignore"):
            assert ref.race_margin.min() > 1e-5 and not np.any(np.abs(ref.dec_u - ref.dec_ratio) < 1e-6)
        np.testing.assert_array_equal(loop.accepted_len.cpu().numpy(), ref.accepted_len)
        np.testing.assert_array_equal(loop.next_token.cpu().numpy(), ref.next_token)
        assert (rec["accepted"], rec["attempted"], rec["emitted"]) == tuple(int(x) for x in ref.counters[1:4])
        # the cache keeps the first query position and the accepted tokens
        new_len, _ = oracle.kv_after_accept(kept + (k + 1), cu, ref.accepted_len)
        np.testing.assert_array_equal(loop.kept, new_len)
        kept = new_len
        # Eq. 1 as reported
        assert rec["goodput_tokens_per_s"] == pytest.approx(
            rec["emitted"] / (rec["verify_seconds"] + k * G.predict_latency(d_tuple, float(rec["context_tokens"]), B)))
        # the acceptance estimate and the next k from the reference equations, fed the same counters
        history.append((rec["accepted"], rec["attempted"]))
        alpha = G.acceptance_rate(history, 0.8, 0.6)
        assert rec["alpha_estimate"] == pytest.approx(alpha, rel=1e-12)
        assert rec["next_k"] == G.argmax_goodput(kept.tolist(), [alpha], sv.K_MAX, t_tuple, d_tuple)
    return ks, loop.acceptance_estimate()


def test_controller_in_the_loop_follows_the_reference_equations():
    import torch
    assert torch.cuda.is_available()
    print("case control loop", flush=True)
    # a latency model in which batched tokens are not free (a whole model's, not this step's alone):
    # the search then has an interior optimum that moves with the acceptance rate
    target = sv.LatencyModel(2.0e-9, 4.0e-6, 2.0e-4)
    draft = sv.LatencyModel(0.2e-9, 0.4e-6, 0.2e-4)
    ks_low, a_low = _run(1.6, 10, target, draft)       # target and draft far apart: few acceptances
    ks_high, a_high = _run(0.15, 10, target, draft)    # close together: most draft tokens pass
    print("low acceptance: k", ks_low, "estimate %.2f; high acceptance: k" % a_low, ks_high, "estimate %.2f" % a_high)
    assert a_low < 0.55 < 0.85 < a_high
    # Section 4.1: the better the proposals, the more of them pay off
    assert np.mean(ks_high[3:]) > np.mean(ks_low[3:])
