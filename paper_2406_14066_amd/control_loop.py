"""Closed-loop speculation control around the verification step (arXiv 2406.14066, the
listing "Generate" of Section 4 and the listing "Finding k to maximize goodput" of Section 4.2).

Every step of the loop: the controller's proposed length k -> the step's K/V rows enter the
paged cache (`spec_kv_append`) -> lookahead attention and rejection sampling
(`spec_verify_step`) -> the step's counters (accepted, attempted, emitted) update the running
acceptance rate (`spec_acceptance_update`, Section 4.1) -> `spec_argmax_goodput` (Eq. 1-4 with
the latency model of Eq. 3) picks the next k.  Goodput of a step is Eq. 1: generated tokens over
the step's time (the measured verification time plus the proposer's modelled time).

There is no model around the step here, so the inputs of each step are synthetic: Gaussian
queries, keys and values; draft logits N(0, 3^2); target logits = draft logits + N(0, sigma^2)
noise (sigma sets the acceptance level); draft tokens drawn from softmax(draft row) by the
Gumbel-max trick -- drawn on the device from a seeded generator.  The proposer is a stand-in
too: one draft pass over the batch costs a fixed fraction of a one-token target pass.

    python -m paper_2406_14066_amd.control_loop [--steps 24] [--draft-fraction 0.1]

prints one JSON line per (acceptance level, batch size): the k chosen at every step, the
acceptance estimate, measured goodput, and the same batch decoded without speculation.
This module only generates inputs, marshals arguments and calls the library's entry points.
"""
from __future__ import annotations

import argparse
import json
import sys

import numpy as np

from . import spec_verify as sv
from .workloads import SIGMA_FOR_ALPHA


class ControlLoop:
    """B synthetic requests that decode together, one verification step at a time."""

    def __init__(self, B, context_len, *, Hq=32, Hkv=8, d=128, V=32000, sigma=0.773, max_kv_len=None, max_k=sv.K_MAX,
                 target: sv.LatencyModel, draft: sv.LatencyModel, decay=0.9, prior=0.7, seed=1, device="cuda"):
        import torch
        self.torch = torch
        self.B, self.Hq, self.Hkv, self.d, self.V = B, Hq, Hkv, d, V
        self.sigma, self.max_k, self.decay, self.prior = float(sigma), int(max_k), float(decay), float(prior)
        self.target, self.draft = target, draft
        self.device = device
        self.seed = seed
        self.kept = np.full(B, context_len, dtype=np.int32)       # cached tokens each request keeps (host copy)
        self.max_kv_len = int(max_kv_len or (context_len + 64 * (max_k + 1) + 15) // 16 * 16)
        self.gen = torch.Generator(device=device)
        self.gen.manual_seed(seed)
        max_blocks = (self.max_kv_len + 15) // 16
        num_blocks = B * max_blocks + 3
        perm = np.random.default_rng(seed).permutation(num_blocks)[: B * max_blocks]
        self.block_table = torch.from_numpy(perm.reshape(B, max_blocks).astype(np.int32)).to(device)
        self.num_blocks = num_blocks
        # the pools hold random keys and values everywhere (matrix-operand page layout: any bytes are valid pages)
        shape = (num_blocks, Hkv, sv.BLOCK_SIZE, d)
        self.k_cache = torch.randn(shape, generator=self.gen, device=device, dtype=torch.float32).to(torch.bfloat16)
        self.v_cache = torch.randn(shape, generator=self.gen, device=device, dtype=torch.float32).to(torch.bfloat16)
        t_max = B * (max_k + 1)
        self.q = torch.zeros((t_max, Hq, d), dtype=torch.bfloat16, device=device)
        self.new_k = torch.zeros((t_max, Hkv, d), dtype=torch.bfloat16, device=device)
        self.new_v = torch.zeros((t_max, Hkv, d), dtype=torch.bfloat16, device=device)
        self.out = torch.zeros((t_max, Hq, d), dtype=torch.float32, device=device)
        self.target_logits = torch.zeros((t_max, V), dtype=torch.float32, device=device)
        self.draft_logits = torch.zeros((max(t_max - B, 1), V), dtype=torch.float32, device=device)
        self.draft_tokens = torch.zeros(max(t_max - B, 1), dtype=torch.int32, device=device)
        self.kv_len = torch.zeros(B, dtype=torch.int32, device=device)
        self.cu_q_len = torch.zeros(B + 1, dtype=torch.int32, device=device)
        self.accepted_len = torch.zeros(B, dtype=torch.int32, device=device)
        self.next_token = torch.zeros(B, dtype=torch.int32, device=device)
        self.new_kv_len = torch.zeros(B, dtype=torch.int32, device=device)
        self.draft_next_len = torch.zeros(B, dtype=torch.int32, device=device)
        self.counters = torch.zeros(sv.NUM_COUNTERS, dtype=torch.int64, device=device)
        self.append_errors = torch.zeros(1, dtype=torch.int64, device=device)
        self.workspace = None
        self.tracker = sv.AcceptanceTracker()
        self.step_index = 0
        self.k = self.choose_k()

    # -- the controller ---------------------------------------------------------------------
    def acceptance_estimate(self) -> float:
        return self.tracker.rate(self.prior)

    def choose_k(self) -> int:
        """The search of Section 4.2 at the current acceptance estimate, within the cache capacity."""
        room = int(self.max_kv_len - self.kept.max())                 # every request gets k + 1 new slots
        max_k = min(self.max_k, room - 1)
        if max_k < 0:
            raise RuntimeError("the requests have outgrown max_kv_len")
        k, self.last_curve = sv.argmax_goodput(self.kept, self.acceptance_estimate(), max_k, self.target, self.draft)
        return k

    def draft_seconds(self, k: int) -> float:
        """Eq. 2's T_draft for the stand-in proposer: k passes of the draft model over the batch."""
        return k * sv.predict_latency(self.draft, float(self.kept.sum()), float(self.B)) if k > 0 else 0.0

    # -- one step -----------------------------------------------------------------------------
    def _fill_inputs(self, k: int):
        torch, B, V = self.torch, self.B, self.V
        T = B * (k + 1)
        for buf in (self.q, self.new_k, self.new_v):
            buf[:T].copy_(torch.randn(buf[:T].shape, generator=self.gen, device=self.device).to(torch.bfloat16))
        # every request gets k + 1 draft rows; the last one only seeds the extra target row
        draft_full = torch.randn((T, V), generator=self.gen, device=self.device) * 3.0
        self.target_logits[:T].copy_(draft_full + torch.randn((T, V), generator=self.gen, device=self.device) * self.sigma)
        if k > 0:
            keep = torch.ones(T, dtype=torch.bool, device=self.device)
            keep[torch.arange(B, device=self.device) * (k + 1) + k] = False
            draft = draft_full[keep]
            self.draft_logits[: T - B].copy_(draft)
            u = torch.rand((T - B, V), generator=self.gen, device=self.device).clamp_(1e-12, 1.0)
            gumbel = -torch.log(-torch.log(u).clamp_(min=1e-30))
            self.draft_tokens[: T - B].copy_(torch.argmax(draft + gumbel, dim=1).to(torch.int32))
        return T

    def run_step(self, k: int | None = None, advance: bool = True) -> dict:
        """One verification step with k draft tokens per request (default: the controller's choice)."""
        torch, B = self.torch, self.B
        k = self.k if k is None else int(k)
        T = self._fill_inputs(k)
        host_len = (self.kept + (k + 1)).astype(np.int32)
        host_cu = (np.arange(B + 1) * (k + 1)).astype(np.int32)
        self.kv_len.copy_(torch.from_numpy(host_len))
        self.cu_q_len.copy_(torch.from_numpy(host_cu))
        attn, keep_a = sv.make_attn_args(self.q[:T], self.k_cache, self.v_cache, self.block_table, self.kv_len,
                                         self.cu_q_len, self.out[:T], host_len, host_cu, Hkv=self.Hkv,
                                         kv_layout=sv.KV_MFMA, max_kv_len=self.max_kv_len)
        rej, keep_r = sv.make_reject_args(self.target_logits[:T], self.draft_logits[: T - B] if k else None,
                                          self.draft_tokens[: T - B] if k else None, self.cu_q_len, host_cu,
                                          self.accepted_len, self.next_token, self.counters, philox_seed=self.seed,
                                          philox_step=self.step_index, kv_len=self.kv_len, new_kv_len=self.new_kv_len,
                                          draft_next_len=self.draft_next_len)
        need = sv.spec_verify_workspace_bytes(attn, rej)
        if self.workspace is None or self.workspace.numel() < need:
            self.workspace = sv.alloc_workspace(need, self.device)
        before = self.counters.cpu().numpy().copy()
        start, stop = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        append, _keep_append = sv.make_kv_append_args(self.new_k[:T], self.new_v[:T], self.k_cache, self.v_cache,
                                                      self.block_table, self.kv_len, self.cu_q_len, host_len, host_cu,
                                                      kv_layout=sv.KV_MFMA, error_count=self.append_errors)
        start.record()
        sv.spec_kv_append_args(append)
        sv.spec_verify_step(attn, rej, self.workspace)
        stop.record()
        torch.cuda.synchronize()
        seconds = start.elapsed_time(stop) * 1e-3
        delta = self.counters.cpu().numpy() - before
        accepted, attempted, emitted = int(delta[1]), int(delta[2]), int(delta[3])
        rec = dict(step=self.step_index, k=k, context_tokens=int(self.kept.sum()), accepted=accepted, attempted=attempted,
                   emitted=emitted, verify_seconds=seconds, draft_seconds=self.draft_seconds(k),
                   input_errors=int(delta[6]) + int(self.append_errors.item()), abandoned=int(delta[7]))
        rec["goodput_tokens_per_s"] = emitted / (seconds + rec["draft_seconds"])      # Eq. 1
        if advance:
            # the cache keeps the first query position and the accepted draft tokens (Section 5.1)
            self.kept = self.new_kv_len.cpu().numpy().astype(np.int32)
            self.tracker.update(accepted, attempted, self.decay)
            self.step_index += 1
            rec["alpha_estimate"] = self.acceptance_estimate()
            self.k = self.choose_k()
            rec["next_k"] = self.k
        return rec

    def time_step(self, k: int, context_len: int, reps: int = 8) -> float:
        """Mean time of the verification step at a given k and context length, without advancing the loop."""
        saved = self.kept.copy()
        self.kept[:] = context_len
        for _ in range(3):
            self.run_step(k, advance=False)
        t = float(np.mean([self.run_step(k, advance=False)["verify_seconds"] for _ in range(reps)]))
        self.kept = saved
        return t


def fit_latency_on_this_device(B, context_len, *, draft_fraction=0.1, **shape):
    """The offline profiler of Section 5.2 in small: Eq. 3 fitted to the verification step timed on this
    device at two context lengths and four proposed lengths; the draft model is a stand-in that costs
    `draft_fraction` of the target's pass."""
    unit = sv.LatencyModel(1e-9, 1e-9, 1e-6)
    loop = ControlLoop(B, context_len, target=unit, draft=unit, max_kv_len=2 * context_len + 64 * (sv.K_MAX + 1), **shape)
    nc, nb, t = [], [], []
    for L in (context_len, 2 * context_len):
        for k in (0, 2, 4, 8):
            nc.append(B * L)
            nb.append(B * (k + 1))
            t.append(loop.time_step(k, L))
    target = sv.fit_latency(nc, nb, t)
    draft = sv.LatencyModel(target.c_context * draft_fraction, target.c_batched * draft_fraction,
                            target.c_fixed * draft_fraction)
    no_spec = t[0]
    del loop
    return target, draft, no_spec


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--steps", type=int, default=24)
    ap.add_argument("--draft-fraction", type=float, default=0.1)
    ap.add_argument("--context", type=int, default=512)
    ap.add_argument("--batch", type=int, nargs="*", default=[8, 32, 256])
    ap.add_argument("--alpha", type=float, nargs="*", default=[0.5, 0.7, 0.9])
    args = ap.parse_args()
    import torch
    if not torch.cuda.is_available():
        print("control_loop: no GPU visible", file=sys.stderr)
        sys.exit(2)
    sv.lib()
    shape = dict(Hq=32, Hkv=8, d=128, V=32000)
    for B in args.batch:
        target, draft, no_spec_seconds = fit_latency_on_this_device(B, args.context, draft_fraction=args.draft_fraction, **shape)
        torch.cuda.empty_cache()
        for alpha in args.alpha:
            sigma = SIGMA_FOR_ALPHA[(32000, 3.0)][alpha]
            loop = ControlLoop(B, args.context, sigma=sigma, target=target, draft=draft, seed=7 + B, **shape)
            recs = [loop.run_step() for _ in range(args.steps)]
            tail = recs[len(recs) // 2:]
            print(json.dumps({
                "B": B, "alpha_of_inputs": alpha, "context_len_start": args.context, "steps": args.steps,
                "eq3_fit_seconds": {"per_context_token": target.c_context, "per_batched_token": target.c_batched,
                                    "fixed": target.c_fixed},
                "draft_fraction": args.draft_fraction,
                "k_per_step": [r["k"] for r in recs],
                "alpha_estimate_final": recs[-1]["alpha_estimate"],
                "emitted_per_step_second_half": float(np.mean([r["emitted"] for r in tail])),
                "verify_us_second_half": 1e6 * float(np.mean([r["verify_seconds"] for r in tail])),
                "goodput_tokens_per_s_second_half": float(np.mean([r["goodput_tokens_per_s"] for r in tail])),
                "no_speculation_tokens_per_s": B / no_spec_seconds,
                "input_errors": sum(r["input_errors"] for r in recs), "abandoned": sum(r["abandoned"] for r in recs),
            }), flush=True)
            del loop
            torch.cuda.empty_cache()


if __name__ == "__main__":
    main()
