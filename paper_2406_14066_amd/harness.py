"""Device-side plumbing shared by the tests, the smoke check and the benchmark:
uploads a ``workloads.VerifyWorkload`` into torch device tensors, builds the C
argument structs and runs the library.  No arithmetic of the method lives here."""
from __future__ import annotations

import numpy as np
import torch

from . import spec_verify as sv
from .workloads import VerifyWorkload


def _to_device_kv(a: np.ndarray, device):
    if a.dtype == np.uint16:
        return torch.from_numpy(a.view(np.int16)).to(device).view(torch.bfloat16)
    return torch.from_numpy(a).to(device)


class DeviceStep:
    """One verification step resident on the GPU."""

    def __init__(self, w: VerifyWorkload, kv_layout: int = sv.KV_TOKEN_MAJOR, device="cuda",
                 with_debug: bool = True, accept_mode: int = sv.ACCEPT_SAMPLE, max_kv_len: int = 0):
        self.w = w
        self.device = device
        self.kv_layout = kv_layout
        self.accept_mode = accept_mode
        self.max_kv_len = max_kv_len
        self.q = _to_device_kv(w.q, device)
        k_tm = _to_device_kv(w.k_pages, device)
        v_tm = _to_device_kv(w.v_pages, device)
        if kv_layout == sv.KV_MFMA:
            self.k_cache = torch.empty_like(k_tm)
            self.v_cache = torch.empty_like(v_tm)
            sv.spec_kv_repack_mfma(k_tm, v_tm, self.k_cache, self.v_cache)
            torch.cuda.synchronize()
            del k_tm, v_tm
        else:
            self.k_cache, self.v_cache = k_tm, v_tm
        self.block_table = torch.from_numpy(w.block_table).to(device)
        self.kv_len = torch.from_numpy(w.kv_len).to(device)
        self.cu_q_len = torch.from_numpy(w.cu_q_len).to(device)
        self.out = torch.zeros((w.T, w.Hq, w.d), dtype=torch.float32, device=device)
        self.target_logits = torch.from_numpy(w.target_logits).to(device)
        self.draft_logits = (torch.from_numpy(w.draft_logits).to(device)
                             if (w.T > w.B and accept_mode == sv.ACCEPT_SAMPLE) else None)
        self.draft_tokens = torch.from_numpy(w.draft_tokens).to(device) if w.T > w.B else None
        self.accepted_len = torch.full((w.B,), -7, dtype=torch.int32, device=device)
        self.next_token = torch.full((w.B,), -7, dtype=torch.int32, device=device)
        self.out_tokens = torch.full((w.B, sv.K_MAX + 1), -7, dtype=torch.int32, device=device)
        self.counters = torch.zeros(sv.NUM_COUNTERS, dtype=torch.int64, device=device)
        self.debug = (torch.full((max(w.T - w.B, 1), 2), float("nan"), dtype=torch.float64, device=device)
                      if with_debug else None)
        self.attn_args, self._keep_a = sv.make_attn_args(
            self.q, self.k_cache, self.v_cache, self.block_table, self.kv_len, self.cu_q_len, self.out,
            w.kv_len, w.cu_q_len, Hkv=w.Hkv, kv_layout=kv_layout, max_kv_len=max_kv_len)
        self.reject_args, self._keep_r = sv.make_reject_args(
            self.target_logits, self.draft_logits, self.draft_tokens, self.cu_q_len, w.cu_q_len,
            self.accepted_len, self.next_token, self.counters, philox_seed=w.philox_seed,
            philox_step=w.philox_step, out_tokens=self.out_tokens, debug_u_ratio=self.debug,
            accept_mode=accept_mode)
        self.workspace = sv.alloc_workspace(sv.spec_verify_workspace_bytes(self.attn_args, self.reject_args), device)

    def rotated(self, copies: int):
        """``copies`` argument pairs for the same step whose KV pools and logits live at different
        addresses (the first pair is this object's own), for timing loops that must not find their
        inputs in the 256 MB last-level cache.  The copies stay alive with this object."""
        pairs = [(self.attn_args, self.reject_args)]
        self._rotated_keep = []
        w = self.w
        for _ in range(max(copies, 1) - 1):
            kc, vc = self.k_cache.clone(), self.v_cache.clone()
            tl = self.target_logits.clone()
            dl = self.draft_logits.clone() if self.draft_logits is not None else None
            a, keep_a = sv.make_attn_args(self.q, kc, vc, self.block_table, self.kv_len, self.cu_q_len, self.out,
                                          w.kv_len, w.cu_q_len, Hkv=w.Hkv, kv_layout=self.kv_layout,
                                          max_kv_len=self.max_kv_len)
            r, keep_r = sv.make_reject_args(tl, dl, self.draft_tokens, self.cu_q_len, w.cu_q_len, self.accepted_len,
                                            self.next_token, self.counters, philox_seed=w.philox_seed,
                                            philox_step=w.philox_step, out_tokens=self.out_tokens,
                                            debug_u_ratio=self.debug, accept_mode=self.accept_mode)
            pairs.append((a, r))
            self._rotated_keep.append((kc, vc, tl, dl, keep_a, keep_r))
        return pairs

    def plan(self) -> dict:
        """How the library runs this step (attention path, split, launches)."""
        return sv.spec_verify_plan(self.attn_args, self.reject_args)

    def input_bytes(self) -> int:
        """Bytes of the big inputs (K and V pools, logits) of one copy."""
        n = 2 * self.k_cache.numel() * self.k_cache.element_size()
        n += self.target_logits.numel() * 4
        if self.draft_logits is not None:
            n += self.draft_logits.numel() * 4
        return n

    def run_attn(self, stream=None):
        sv.spec_verify_attn(self.attn_args, self.workspace, stream)

    def run_reject(self, stream=None):
        sv.spec_reject_sample(self.reject_args, self.workspace, stream)

    def run_step(self, stream=None):
        sv.spec_verify_step(self.attn_args, self.reject_args, self.workspace, stream)

    def results(self):
        torch.cuda.synchronize()
        return dict(
            out=self.out.cpu().numpy(),
            accepted_len=self.accepted_len.cpu().numpy(),
            next_token=self.next_token.cpu().numpy(),
            out_tokens=self.out_tokens.cpu().numpy(),
            counters=self.counters.cpu().numpy(),
            debug=None if self.debug is None else self.debug.cpu().numpy()[: max(self.w.T - self.w.B, 0)],
        )
